// Host-side index tables (see geometry.hpp).
#include "geometry.hpp"

#include <cmath>

namespace httm {

int check_geom(const httm_geom_t& g) {
  if (g.S <= 0 || g.Hp <= 0 || g.Wp <= 0 || g.n_special < 0 || g.H <= 0 || g.b <= 0 || g.T <= 0)
    return HTTM_E_INVALID_ARG;
  if (!(g.rho_q >= 0.0 && g.rho_q <= 1.0) || !(g.rho_kv >= 0.0 && g.rho_kv <= 1.0))
    return HTTM_E_INVALID_ARG;
  if (g.variant != HTTM_VARIANT_HEADWISE && g.variant != HTTM_VARIANT_UNIFORM &&
      g.variant != HTTM_VARIANT_NONE)
    return HTTM_E_INVALID_ARG;
  if (g.flags & ~(HTTM_FLAG_ANCHOR_FIRST_FRAME | HTTM_FLAG_CHUNKED_BLOCKS | HTTM_FLAG_LOG2_KEYS))
    return HTTM_E_INVALID_ARG;
  if (!(g.outlier_frac >= 0.0 && g.outlier_frac <= HTTM_MAX_OUTLIER_FRAC)) return HTTM_E_INVALID_ARG;
  if (!(g.dst_frac >= 0.0 && g.dst_frac <= 1.0)) return HTTM_E_INVALID_ARG;
  if (g.d_head != 64 || g.H > HTTM_MAX_HEADS) return HTTM_E_UNSUPPORTED;
  const int64_t tpf = (int64_t)g.n_special + (int64_t)g.Hp * g.Wp;
  const int64_t N = tpf * g.S;
  if (N >= (int64_t)1 << 25) return HTTM_E_UNSUPPORTED;  // per-head byte offsets (N*128) stay below 2^32
  const int64_t bh = g.b < g.Hp ? g.b : g.Hp, bw = g.b < g.Wp ? g.b : g.Wp, bt = g.T < g.S ? g.T : g.S;
  const int64_t P = (int64_t)g.Hp * g.Wp;
  const int64_t ns = (g.flags & HTTM_FLAG_CHUNKED_BLOCKS) ? (g.b < P ? g.b : P) : bh * bw;
  if (ns * bt > HTTM_MAX_BLOCK) return HTTM_E_UNSUPPORTED;
  return HTTM_OK;
}

int32_t clusters_kept(int32_t n, double rho, int32_t n0, double dst_frac, int32_t* kd_out) {
  // Sec. 3.2: r tokens are merged away, M = N - r remain; in Sec. 4.1 a ratio rho leaves the share
  // 1 - rho.  Applied per block with the count rounded down; at least one cluster survives,
  // and every anchored token (App. C.2) is one.
  const int32_t r = (int32_t)std::floor(rho * (double)n + 1e-9);
  int32_t k, kd;
  if (dst_frac > 0.0) {
    // general rule: a fixed share of dst tokens, only src tokens can be merged away
    kd = (int32_t)std::floor(dst_frac * (double)n + 1e-9);
    if (kd < 1) kd = 1;
    if (kd < n0) kd = n0;
    const int32_t n_src = n - kd;
    k = n - (r < n_src ? r : n_src);
  } else {
    k = n - r;
    if (k < 1) k = 1;
    if (k < n0) k = n0;
    kd = k;
  }
  if (kd_out) *kd_out = kd;
  return k;
}

int64_t outlier_budget(const httm_geom_t& g, int64_t N) {
  // Sec. 3.4 step 3: the share d of the tokens of all heads together, rounded down
  if (g.variant == HTTM_VARIANT_NONE || !(g.outlier_frac > 0.0)) return 0;
  return (int64_t)std::floor(g.outlier_frac * (double)g.H * (double)N + 1e-9);
}

int build_tables(const httm_geom_t& g, bool with_pi, HostTables* out) {
  const int rc = check_geom(g);
  if (rc != HTTM_OK) return rc;
  HostTables& t = *out;
  const double rho_q = g.variant == HTTM_VARIANT_NONE ? 0.0 : g.rho_q;
  const double rho_k = g.variant == HTTM_VARIANT_NONE ? 0.0 : g.rho_kv;
  const int32_t tpf = g.n_special + g.Hp * g.Wp;
  t.N = (int64_t)tpf * g.S;
  t.n_prefix = (int64_t)g.S * g.n_special;
  const int32_t groups = (g.S + g.T - 1) / g.T;
  // Spatial blocks of a frame: b x b windows of the patch grid (row-major over windows), or runs of
  // b consecutive patch tokens (Sec. 4.1) - then a "window" is one row of slots [x0, x1).
  const bool chunked = (g.flags & HTTM_FLAG_CHUNKED_BLOCKS) != 0;
  const int32_t P = g.Hp * g.Wp;
  const int32_t wy = chunked ? 1 : (g.Hp + g.b - 1) / g.b;
  const int32_t wx = chunked ? (P + g.b - 1) / g.b : (g.Wp + g.b - 1) / g.b;
  const int32_t row_len = chunked ? P : g.Wp;    // slots per "row" of the loops below
  const int32_t n_rows = chunked ? 1 : g.Hp;
  t.n_blocks = (int64_t)groups * wy * wx;
  t.block_start.resize(t.n_blocks);
  t.block_n.resize(t.n_blocks);
  t.block_kq.resize(t.n_blocks);
  t.block_kk.resize(t.n_blocks);
  t.block_offq.resize(t.n_blocks);
  t.block_offk.resize(t.n_blocks);
  if (with_pi) {
    t.pi.resize(t.N);
    t.block_src0.resize(t.n_blocks);
    t.block_dims.resize(t.n_blocks);
  }

  // Special tokens first, frame-major.
  int64_t pos = 0;
  if (with_pi)
    for (int32_t f = 0; f < g.S; ++f)
      for (int32_t s = 0; s < g.n_special; ++s) t.pi[pos++] = f * tpf + s;
  pos = t.n_prefix;

  // Pseudo-blocks over the prefix: identity clusters.
  t.items_q.clear();
  t.items_k.clear();
  for (int64_t p = 0; p < t.n_prefix; p += kPrefixChunk) {
    const int32_t n = (int32_t)((t.n_prefix - p) < kPrefixChunk ? (t.n_prefix - p) : kPrefixChunk);
    t.items_q.push_back({(int32_t)p, n, n, (int32_t)p, 0, n, 0, 0});
    t.items_k.push_back({(int32_t)p, n, n, (int32_t)p, 0, n, 0, 0});
  }

  int64_t mq = t.n_prefix, mk = t.n_prefix;
  t.max_block = 0;
  int64_t bi = 0;
  for (int32_t grp = 0; grp < groups; ++grp) {
    const int32_t f0 = grp * g.T, f1 = (f0 + g.T < g.S) ? f0 + g.T : g.S;
    for (int32_t by = 0; by < wy; ++by) {
      const int32_t y0 = chunked ? 0 : by * g.b;
      const int32_t y1 = chunked ? 1 : ((y0 + g.b < n_rows) ? y0 + g.b : n_rows);
      for (int32_t bx = 0; bx < wx; ++bx, ++bi) {
        const int32_t x0 = bx * g.b, x1 = (x0 + g.b < row_len) ? x0 + g.b : row_len;
        const int32_t n = (f1 - f0) * (y1 - y0) * (x1 - x0);
        t.block_start[bi] = (int32_t)pos;
        t.block_n[bi] = n;
        if (n > t.max_block) t.max_block = n;
        if (with_pi) {
          int64_t w = pos;
          for (int32_t f = f0; f < f1; ++f)
            for (int32_t y = y0; y < y1; ++y) {
              const int32_t row = f * tpf + g.n_special + y * row_len;
              for (int32_t x = x0; x < x1; ++x) t.pi[w++] = row + x;
            }
        }
        // first-frame anchoring: blocks are frame-major, so the frame-0 tokens of a block of the
        // first temporal group are its first (rows x cols) positions
        const bool anchor = (g.flags & HTTM_FLAG_ANCHOR_FIRST_FRAME) && grp == 0;
        const int32_t n0 = anchor ? (y1 - y0) * (x1 - x0) : 0;
        const double df = g.variant == HTTM_VARIANT_NONE ? 0.0 : g.dst_frac;
        int32_t kdq = 0, kdk = 0;
        const int32_t kq = clusters_kept(n, rho_q, n0, df, &kdq), kk = clusters_kept(n, rho_k, n0, df, &kdk);
        t.block_kq[bi] = kq;
        t.block_kk[bi] = kk;
        t.block_offq[bi] = (int32_t)mq;
        t.block_offk[bi] = (int32_t)mk;
        const int32_t nx = x1 - x0, plane = (y1 - y0) * nx;
        const int32_t src0 = f0 * tpf + g.n_special + y0 * row_len + x0;
        int32_t dims = plane < 32768 ? (nx | (plane << 16)) : 0;
        if (with_pi && dims) {
          // the closed form is evaluated here the way the kernels evaluate it (fp32 quotients) and
          // kept only if it reproduces the table
          const float r_plane = 1.0f / (float)plane, r_nx = 1.0f / (float)nx;
          for (int32_t r = 0; r < n && dims; ++r) {
            const int32_t f = (int32_t)(((float)r + 0.5f) * r_plane);
            const int32_t rem = r - f * plane;
            const int32_t y = (int32_t)(((float)rem + 0.5f) * r_nx);
            if (src0 + f * tpf + y * row_len + (rem - y * nx) != t.pi[pos + r]) dims = 0;
          }
        }
        if (with_pi) {
          t.block_src0[bi] = src0;
          t.block_dims[bi] = dims;
        }
        t.items_q.push_back({(int32_t)pos, n, kq, (int32_t)mq, n0, kdq, src0, dims});
        t.items_k.push_back({(int32_t)pos, n, kk, (int32_t)mk, n0, kdk, src0, dims});
        mq += kq;
        mk += kk;
        pos += n;
      }
    }
  }
  t.M_q = mq;
  t.M_k = mk;
  return HTTM_OK;
}

int workspace_layout(const httm_geom_t& g, const HostTables& t, httm_workspace_layout_t* out) {
  const int64_t row = (int64_t)g.d_head * 2;
  int64_t off = 0;
  out->q_m = off;      off = align_up(off + (int64_t)g.H * t.M_q * row, 256);
  out->k_m = off;      off = align_up(off + (int64_t)g.H * t.M_k * row, 256);
  out->v_m = off;      off = align_up(off + (int64_t)g.H * t.M_k * row, 256);
  out->o_m = off;      off = align_up(off + (int64_t)g.H * t.M_q * row, 256);
  out->assign_q = off; off = align_up(off + (int64_t)g.H * t.N * 4, 256);
  out->assign_k = off; off = align_up(off + (int64_t)g.H * t.N * 4, 256);
  const int64_t cap = outlier_budget(g, t.N);
  out->eps_q = off;    off = align_up(off + (cap ? (int64_t)g.H * t.N * 4 : 0), 256);
  out->q_out = off;    off = align_up(off + cap * row, 256);
  out->o_out = off;    off = align_up(off + cap * row, 256);
  out->attn_split = off; off = align_up(off + attention_scratch_bytes(g.H), 256);
  out->total = off;
  return HTTM_OK;
}

}  // namespace httm
