// C-ABI layer of libhttm: argument checks, the plan object, and the stage sequencing of
// httm_layer_forward.  See include/httm.h for the contract of every entry point.
#include <hip/hip_runtime.h>

#include <cstring>
#include <new>

#include "../../include/httm.h"
#include "attention_split.hpp"
#include "geometry.hpp"
#include "kernels.hpp"

using namespace httm;

struct httm_plan {
  httm_geom_t geom;
  httm_sizes_t sizes;
  httm_workspace_layout_t ws;
  int device = -1;
  int32_t* d_pi = nullptr;
  WorkItem* d_items_q = nullptr;
  WorkItem* d_items_k = nullptr;
  int32_t n_items = 0;
  int32_t max_k = 0;   // most clusters any work item keeps (Q or K)
  // head-uniform variant only
  float* d_mean = nullptr;    // [2][N][64] fp32: head-averaged Q then K
  int32_t* d_slot = nullptr;  // [2][N] shared cluster slot of every reordered token
  float* d_uscore = nullptr;  // [2][N]
  // general rule (dst_frac > 0) on blocks of more than 512 tokens: the similarities the selection of
  // the merging src tokens needs, when the caller asks for none
  float* d_score = nullptr;   // [2][H][N]
  // outlier filtering only
  int64_t outlier_cap = 0;
  OutlierBuffers ob = {};
};

namespace {

thread_local int g_last_hip_error = 0;

int hip_fail(hipError_t e) {
  g_last_hip_error = (int)e;
  return HTTM_E_HIP;
}

#define HTTM_HIP(call)                         \
  do {                                         \
    hipError_t e_ = (call);                    \
    if (e_ != hipSuccess) return hip_fail(e_); \
  } while (0)

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// build_tables() fills std::vectors; nothing may throw across the C boundary.
int build_tables_nothrow(const httm_geom_t& g, bool with_pi, HostTables* t) {
  try {
    return build_tables(g, with_pi, t);
  } catch (const std::bad_alloc&) {
    return HTTM_E_OUT_OF_MEMORY;
  } catch (...) {
    return HTTM_E_INVALID_ARG;
  }
}

void fill_sizes(const httm_geom_t& g, const HostTables& t, httm_sizes_t* s,
                httm_workspace_layout_t* ws) {
  s->N = t.N;
  s->n_prefix = t.n_prefix;
  s->n_blocks = t.n_blocks;
  s->max_block = t.max_block;
  s->M_q = t.M_q;
  s->M_k = t.M_k;
  httm_workspace_layout_t l;
  workspace_layout(g, t, &l);
  s->workspace_bytes = l.total;
  s->outlier_cap = outlier_budget(g, t.N);
  if (ws) *ws = l;
}

template <typename T>
int upload(const std::vector<T>& host, T** dev) {
  *dev = nullptr;
  if (host.empty()) return HTTM_OK;
  HTTM_HIP(hipMalloc((void**)dev, host.size() * sizeof(T)));
  HTTM_HIP(hipMemcpy(*dev, host.data(), host.size() * sizeof(T), hipMemcpyHostToDevice));
  return HTTM_OK;
}

bool log2_keys(const httm_plan_t* p) { return (p->geom.flags & HTTM_FLAG_LOG2_KEYS) != 0; }

// Matching + aggregation on `q,k,v`, which are in input order when `pi` is given and in
// reordered order when it is nullptr.
int run_match_merge(const httm_plan_t* p, const int32_t* pi, const void* q, const void* k,
                    const void* v, void* q_m, void* k_m, void* v_m, int32_t* assign_q,
                    int32_t* assign_k, float* score_q, float* score_k, hipStream_t st,
                    float* eps_q = nullptr) {
  const httm_geom_t& g = p->geom;
  MatchMergeArgs a;
  std::memset(&a, 0, sizeof(a));
  a.n_streams = 2;
  a.pi = pi;
  a.tpf = g.n_special + g.Hp * g.Wp;
  a.row_len = (g.flags & HTTM_FLAG_CHUNKED_BLOCKS) ? g.Hp * g.Wp : g.Wp;
  a.N = p->sizes.N;
  a.H = g.H;
  a.max_block = (int32_t)(p->sizes.max_block < kPrefixChunk ? kPrefixChunk : p->sizes.max_block);
  a.max_k = p->max_k;
  a.top_r = p->geom.dst_frac > 0.0 && p->geom.variant != HTTM_VARIANT_NONE;
  if (p->d_score) {
    if (!score_q) score_q = p->d_score;
    if (!score_k) score_k = p->d_score + (int64_t)g.H * p->sizes.N;
  }
  a.s[0] = {q, nullptr, q_m, nullptr, assign_q, score_q, p->d_items_q, p->n_items, p->sizes.M_q,
            nullptr, nullptr, eps_q, 1.0f};
  a.s[1] = {k, v, k_m, v_m, assign_k, score_k, p->d_items_k, p->n_items, p->sizes.M_k, nullptr,
            nullptr, nullptr, log2_keys(p) ? kLog2KeyScale : 1.0f};
  if (g.variant == HTTM_VARIANT_UNIFORM) {
    const int64_t N = p->sizes.N;
    const void* src[2] = {q, k};
    const WorkItem* items[2] = {p->d_items_q, p->d_items_k};
    for (int t = 0; t < 2; ++t) {
      float* mean = p->d_mean + (int64_t)t * N * 64;
      HTTM_HIP(launch_head_mean(src[t], mean, g.H, N, st));
      HTTM_HIP(launch_match_f32(mean, pi, items[t], p->n_items, a.max_block, p->d_slot + t * N,
                                p->d_uscore + t * N, st));
      a.s[t].preset = p->d_slot + t * N;
      a.s[t].preset_score = p->d_uscore + t * N;
    }
    if (a.top_r) {
      // general rule of Sec. 3.2 on the shared topology: which src tokens merge
      TopRArgs tr = {};
      tr.n_streams = 2;
      for (int t = 0; t < 2; ++t) tr.s[t] = {p->d_slot + t * N, p->d_uscore + t * N, items[t], p->n_items, N};
      HTTM_HIP(launch_top_r_select(tr, 1, st));
    }
  }
  HTTM_HIP(launch_match_merge(a, st));
  return HTTM_OK;
}

// Stage 2 with the outlier filter (Sec. 3.4): matching + aggregation with the deviations written
// out, the device-wide threshold, then the un-merging of the outliers.
int run_match_merge_filtered(const httm_plan_t* p, const void* q, const void* k, const void* v,
                             void* q_m, void* k_m, void* v_m, int32_t* assign_q, int32_t* assign_k,
                             float* eps_q, void* q_out, hipStream_t st) {
  int rc = run_match_merge(p, p->d_pi, q, k, v, q_m, k_m, v_m, assign_q, assign_k, nullptr, nullptr,
                           st, eps_q);
  if (rc != HTTM_OK) return rc;
  HTTM_HIP(launch_outlier_select(eps_q, p->geom.H, p->sizes.N, p->outlier_cap, p->d_items_q,
                                 p->n_items, (int)p->sizes.max_block, p->ob, kAttnDevTileRows, st));
  RefineArgs r;
  std::memset(&r, 0, sizeof(r));
  r.x = q;
  r.xm = q_m;
  r.assign = assign_q;
  r.eps = eps_q;
  r.q_out = q_out;
  r.items = p->d_items_q;
  r.n_items = p->n_items;
  r.M = p->sizes.M_q;
  r.pi = p->d_pi;
  r.tpf = p->geom.n_special + p->geom.Hp * p->geom.Wp;
  r.row_len = (p->geom.flags & HTTM_FLAG_CHUNKED_BLOCKS) ? p->geom.Hp * p->geom.Wp : p->geom.Wp;
  r.N = p->sizes.N;
  r.H = p->geom.H;
  r.max_block = (int32_t)(p->sizes.max_block < kPrefixChunk ? kPrefixChunk : p->sizes.max_block);
  r.eager = (double)p->outlier_cap * (double)p->sizes.max_block >= (double)p->geom.H * (double)p->sizes.N;
  r.b = p->ob;
  if (r.max_block > kSmallBlockMax)
    HTTM_HIP(launch_outlier_refine_big(r, p->max_k, st));
  else
    HTTM_HIP(launch_outlier_refine(r, st));
  return HTTM_OK;
}

int run_attention_outliers(const httm_plan_t* p, const void* q_out, const void* k_m, const void* v_m,
                           void* o_out, hipStream_t st) {
  int64_t k_off[HTTM_MAX_HEADS + 1];
  for (int h = 0; h <= p->geom.H; ++h) k_off[h] = (int64_t)h * p->sizes.M_k;
  HTTM_HIP(launch_attention_dev_tiles(q_out, k_m, v_m, o_out, p->ob.offsets, p->ob.tiles,
                                      p->ob.max_tiles, k_off, p->geom.H, 0.125f, log2_keys(p), st));
  return HTTM_OK;
}

}  // namespace

extern "C" {

int httm_version(void) { return HTTM_VERSION; }

const char* httm_strerror(int code) {
  switch (code) {
    case HTTM_OK: return "success";
    case HTTM_E_INVALID_ARG: return "invalid argument (null or misaligned pointer, bad size or enum)";
    case HTTM_E_UNSUPPORTED: return "unsupported configuration (d_head != 64, block too large, too many heads)";
    case HTTM_E_WORKSPACE_TOO_SMALL: return "workspace too small";
    case HTTM_E_HIP: return "HIP runtime error (see httm_last_hip_error)";
    case HTTM_E_NO_DEVICE: return "no usable GPU";
    case HTTM_E_OUT_OF_MEMORY: return "out of host memory while building the index tables";
    default: return "unknown error code";
  }
}

int httm_last_hip_error(void) { return g_last_hip_error; }

int httm_geom_sizes(const httm_geom_t* g, httm_sizes_t* out) {
  if (!g || !out) return HTTM_E_INVALID_ARG;
  HostTables t;
  const int rc = build_tables_nothrow(*g, false, &t);
  if (rc != HTTM_OK) return rc;
  fill_sizes(*g, t, out, nullptr);
  return HTTM_OK;
}

int httm_workspace_layout(const httm_geom_t* g, httm_workspace_layout_t* out) {
  if (!g || !out) return HTTM_E_INVALID_ARG;
  HostTables t;
  const int rc = build_tables_nothrow(*g, false, &t);
  if (rc != HTTM_OK) return rc;
  return workspace_layout(*g, t, out);
}

int httm_geom_tables(const httm_geom_t* g, int32_t* pi, int32_t* block_start, int32_t* block_n,
                     int32_t* block_kq, int32_t* block_kk, int32_t* block_offq, int32_t* block_offk) {
  if (!g) return HTTM_E_INVALID_ARG;
  HostTables t;
  const int rc = build_tables_nothrow(*g, pi != nullptr, &t);
  if (rc != HTTM_OK) return rc;
  const size_t nb = (size_t)t.n_blocks * sizeof(int32_t);
  if (pi) std::memcpy(pi, t.pi.data(), (size_t)t.N * sizeof(int32_t));
  if (block_start) std::memcpy(block_start, t.block_start.data(), nb);
  if (block_n) std::memcpy(block_n, t.block_n.data(), nb);
  if (block_kq) std::memcpy(block_kq, t.block_kq.data(), nb);
  if (block_kk) std::memcpy(block_kk, t.block_kk.data(), nb);
  if (block_offq) std::memcpy(block_offq, t.block_offq.data(), nb);
  if (block_offk) std::memcpy(block_offk, t.block_offk.data(), nb);
  return HTTM_OK;
}

int httm_geom_block_forms(const httm_geom_t* g, int32_t* block_src0, int32_t* block_dims) {
  if (!g || !block_src0 || !block_dims) return HTTM_E_INVALID_ARG;
  HostTables t;
  const int rc = build_tables_nothrow(*g, true, &t);
  if (rc != HTTM_OK) return rc;
  const size_t nb = (size_t)t.n_blocks * sizeof(int32_t);
  std::memcpy(block_src0, t.block_src0.data(), nb);
  std::memcpy(block_dims, t.block_dims.data(), nb);
  return HTTM_OK;
}

int httm_plan_create(const httm_geom_t* g, httm_plan_t** out) {
  if (!g || !out) return HTTM_E_INVALID_ARG;
  *out = nullptr;
  HostTables t;
  int rc = build_tables_nothrow(*g, true, &t);
  if (rc != HTTM_OK) return rc;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev == 0) return HTTM_E_NO_DEVICE;
  httm_plan_t* p = new (std::nothrow) httm_plan_t();
  if (!p) return HTTM_E_OUT_OF_MEMORY;
  p->geom = *g;
  fill_sizes(*g, t, &p->sizes, &p->ws);
  p->n_items = (int32_t)t.items_q.size();
  for (const WorkItem& w : t.items_q) p->max_k = w.k > p->max_k ? w.k : p->max_k;
  for (const WorkItem& w : t.items_k) p->max_k = w.k > p->max_k ? w.k : p->max_k;
  hipError_t e = hipGetDevice(&p->device);
  if (e != hipSuccess) {
    delete p;
    return hip_fail(e);
  }
  rc = upload(t.pi, &p->d_pi);
  if (rc == HTTM_OK) rc = upload(t.items_q, &p->d_items_q);
  if (rc == HTTM_OK) rc = upload(t.items_k, &p->d_items_k);
  if (rc == HTTM_OK && g->variant == HTTM_VARIANT_UNIFORM) {
    e = hipMalloc((void**)&p->d_mean, (size_t)2 * t.N * 64 * sizeof(float));
    if (e == hipSuccess) e = hipMalloc((void**)&p->d_slot, (size_t)2 * t.N * sizeof(int32_t));
    if (e == hipSuccess) e = hipMalloc((void**)&p->d_uscore, (size_t)2 * t.N * sizeof(float));
    if (e != hipSuccess) rc = hip_fail(e);
  }
  if (rc == HTTM_OK && g->dst_frac > 0.0 && g->variant == HTTM_VARIANT_HEADWISE && t.max_block > kSmallBlockMax) {
    e = hipMalloc((void**)&p->d_score, (size_t)2 * g->H * t.N * sizeof(float));
    if (e != hipSuccess) rc = hip_fail(e);
  }
  p->outlier_cap = p->sizes.outlier_cap;
  if (rc == HTTM_OK && p->outlier_cap > 0) {
    OutlierBuffers& b = p->ob;
    b.max_tiles = (int32_t)(p->outlier_cap / kAttnDevTileRows + g->H);
    const size_t words = sizeof(SelectState) / 4 + 3 * 2048 + (size_t)g->H * 2 + 1 +
                         2 * (size_t)g->H * p->n_items + (size_t)g->H * (p->n_items / kOutlierCountItemsMin + 1) + 1 +
                         2 * (size_t)b.max_tiles;
    uint32_t* base = nullptr;
    e = hipMalloc((void**)&base, words * 4);
    if (e == hipSuccess) e = hipMemset(base, 0, words * 4);
    if (e != hipSuccess) {
      rc = hip_fail(e);
    } else {
      b.state = (SelectState*)base;
      b.hist = base + sizeof(SelectState) / 4;
      b.counts = (int32_t*)(b.hist + 3 * 2048);
      b.offsets = b.counts + g->H;
      b.item_cnt = b.offsets + g->H + 1;
      b.item_base = b.item_cnt + (size_t)g->H * p->n_items;
      b.wg_cnt = b.item_base + (size_t)g->H * p->n_items;
      b.tiles = b.wg_cnt + (size_t)g->H * (p->n_items / kOutlierCountItemsMin + 1);
    }
  }
  // "Synchronous": the copies and the memset above are complete before a kernel on any stream
  // (blocking or not) can read the tables.
  if (rc == HTTM_OK) {
    e = hipDeviceSynchronize();
    if (e != hipSuccess) rc = hip_fail(e);
  }
  if (rc != HTTM_OK) {
    httm_plan_destroy(p);
    return rc;
  }
  *out = p;
  return HTTM_OK;
}

int httm_plan_clone(const httm_plan_t* p, httm_plan_t** out) {
  if (!p || !out) return HTTM_E_INVALID_ARG;
  return httm_plan_create(&p->geom, out);
}

int httm_plan_destroy(httm_plan_t* p) {
  if (!p) return HTTM_OK;
  void* ptrs[] = {p->d_pi, p->d_items_q, p->d_items_k, p->d_mean, p->d_slot, p->d_uscore, p->d_score, p->ob.state};
  for (void* q : ptrs)
    if (q) (void)hipFree(q);
  delete p;
  return HTTM_OK;
}

int httm_plan_query(const httm_plan_t* p, httm_sizes_t* out) {
  if (!p || !out) return HTTM_E_INVALID_ARG;
  *out = p->sizes;
  return HTTM_OK;
}

int httm_reorder(const httm_plan_t* p, const void* src, void* dst, int direction, void* stream) {
  if (!p || !src || !dst || src == dst || (direction != 0 && direction != 1)) return HTTM_E_INVALID_ARG;
  if (!aligned16(src) || !aligned16(dst)) return HTTM_E_INVALID_ARG;
  HTTM_HIP(launch_reorder(src, dst, p->d_pi, p->geom.H, p->sizes.N, direction, (hipStream_t)stream));
  return HTTM_OK;
}

int httm_match_merge(const httm_plan_t* p, const void* q_r, const void* k_r, const void* v_r,
                     void* q_m, void* k_m, void* v_m, int32_t* assign_q, int32_t* assign_k,
                     float* score_q, float* score_k, void* stream) {
  if (!p || !q_r || !k_r || !v_r || !q_m || !k_m || !v_m || !assign_q || !assign_k)
    return HTTM_E_INVALID_ARG;
  const void* ptrs[] = {q_r, k_r, v_r, q_m, k_m, v_m, assign_q, assign_k};
  for (const void* q : ptrs)
    if (!aligned16(q)) return HTTM_E_INVALID_ARG;
  return run_match_merge(p, nullptr, q_r, k_r, v_r, q_m, k_m, v_m, assign_q, assign_k, score_q,
                         score_k, (hipStream_t)stream);
}

int httm_reorder_match_merge(const httm_plan_t* p, const void* q, const void* k, const void* v,
                             void* q_m, void* k_m, void* v_m, int32_t* assign_q, int32_t* assign_k,
                             float* score_q, float* score_k, void* stream) {
  if (!p || !q || !k || !v || !q_m || !k_m || !v_m || !assign_q || !assign_k)
    return HTTM_E_INVALID_ARG;
  const void* ptrs[] = {q, k, v, q_m, k_m, v_m, assign_q, assign_k};
  for (const void* x : ptrs)
    if (!aligned16(x)) return HTTM_E_INVALID_ARG;
  return run_match_merge(p, p->d_pi, q, k, v, q_m, k_m, v_m, assign_q, assign_k, score_q, score_k,
                         (hipStream_t)stream);
}

int httm_global_match(const void* x, int64_t N, int H, int d_head, double dst_frac, int32_t* best_dst,
                      float* sim, void* stream) {
  if (!x || !best_dst || N <= 0 || H <= 0 || !(dst_frac > 0.0 && dst_frac <= 1.0)) return HTTM_E_INVALID_ARG;
  if (d_head != 64 || H > HTTM_MAX_HEADS || N >= ((int64_t)1 << 24)) return HTTM_E_UNSUPPORTED;
  if (!aligned16(x) || !aligned16(best_dst)) return HTTM_E_INVALID_ARG;
  int64_t kd = (int64_t)(dst_frac * (double)N + 1e-9);
  if (kd < 1) kd = 1;
  HTTM_HIP(launch_global_match(x, N, H, (int32_t)kd, best_dst, sim, (hipStream_t)stream));
  return HTTM_OK;
}

}  // extern "C"

namespace {

// Stage 3 behind its six entry points: argument checks, then the launch.  `scratch` may be nullptr
// (every tile runs whole) or any 16-byte aligned room; the launch uses it only if its partial
// results fit.
int run_attention(const void* q_m, const void* k_m, const void* v_m, void* o_m, const int64_t* q_offsets,
                  const int64_t* k_offsets, int H, int d_head, float scale, bool log2_keys_in, void* scratch,
                  int64_t scratch_bytes, void* stream) {
  if (!q_offsets || !k_offsets || H <= 0 || !(scale > 0.0f)) return HTTM_E_INVALID_ARG;
  if (scratch && (!aligned16(scratch) || scratch_bytes < 0)) return HTTM_E_INVALID_ARG;
  if (d_head != 64 || H > HTTM_MAX_HEADS) return HTTM_E_UNSUPPORTED;
  for (int h = 0; h < H; ++h)
    if (q_offsets[h + 1] < q_offsets[h] || k_offsets[h + 1] < k_offsets[h] ||
        q_offsets[h + 1] - q_offsets[h] >= ((int64_t)1 << 24) ||
        k_offsets[h + 1] - k_offsets[h] >= ((int64_t)1 << 24))
      return HTTM_E_INVALID_ARG;
  if (q_offsets[0] < 0 || k_offsets[0] < 0) return HTTM_E_INVALID_ARG;
  const bool any_q = q_offsets[H] > q_offsets[0], any_k = k_offsets[H] > k_offsets[0];
  if (any_q && (!q_m || !o_m)) return HTTM_E_INVALID_ARG;
  if (any_q && any_k && (!k_m || !v_m)) return HTTM_E_INVALID_ARG;
  if (!aligned16(q_m) || !aligned16(k_m) || !aligned16(v_m) || !aligned16(o_m)) return HTTM_E_INVALID_ARG;
  HTTM_HIP(launch_attention(q_m, k_m, v_m, o_m, q_offsets, k_offsets, H, log2_keys_in ? 1.0f : scale, log2_keys_in,
                            (hipStream_t)stream, scratch, scratch ? scratch_bytes : 0));
  return HTTM_OK;
}

}  // namespace

extern "C" {

int httm_attention_scratch(const void* q_m, const void* k_m, const void* v_m, void* o_m,
                           const int64_t* q_offsets, const int64_t* k_offsets, int H, int d_head,
                           float scale, void* scratch, int64_t scratch_bytes, void* stream) {
  if (scratch && H > 0 && H <= HTTM_MAX_HEADS && scratch_bytes < attention_scratch_bytes(H)) return HTTM_E_INVALID_ARG;
  return run_attention(q_m, k_m, v_m, o_m, q_offsets, k_offsets, H, d_head, scale, false, scratch, scratch_bytes, stream);
}

int httm_attention(const void* q_m, const void* k_m, const void* v_m, void* o_m,
                   const int64_t* q_offsets, const int64_t* k_offsets, int H, int d_head,
                   float scale, void* stream) {
  return run_attention(q_m, k_m, v_m, o_m, q_offsets, k_offsets, H, d_head, scale, false, nullptr, 0, stream);
}

int httm_attention_log2_scratch(const void* q_m, const void* k_log2, const void* v_m, void* o_m,
                                const int64_t* q_offsets, const int64_t* k_offsets, int H, int d_head,
                                void* scratch, int64_t scratch_bytes, void* stream) {
  if (scratch && H > 0 && H <= HTTM_MAX_HEADS && scratch_bytes < attention_scratch_bytes(H)) return HTTM_E_INVALID_ARG;
  return run_attention(q_m, k_log2, v_m, o_m, q_offsets, k_offsets, H, d_head, 1.0f, true, scratch, scratch_bytes, stream);
}

int httm_attention_log2(const void* q_m, const void* k_log2, const void* v_m, void* o_m,
                        const int64_t* q_offsets, const int64_t* k_offsets, int H, int d_head,
                        void* stream) {
  return run_attention(q_m, k_log2, v_m, o_m, q_offsets, k_offsets, H, d_head, 1.0f, true, nullptr, 0, stream);
}

int httm_attention_log2_static(const void* q_m, const void* k_log2, const void* v_m, void* o_m,
                               const int64_t* q_offsets, const int64_t* k_offsets, int H, int d_head,
                               void* stream) {
  if (!q_offsets || !k_offsets || H <= 0) return HTTM_E_INVALID_ARG;
  if (d_head != 64 || H > HTTM_MAX_HEADS) return HTTM_E_UNSUPPORTED;
  for (int h = 0; h < H; ++h)
    if (q_offsets[h + 1] < q_offsets[h] || k_offsets[h + 1] < k_offsets[h]) return HTTM_E_INVALID_ARG;
  // the partial results of this launch must fit the library's array; nothing is launched otherwise
  if (attention_scratch_need(q_offsets, k_offsets, H) > kAttnStaticScratchBytes) return HTTM_E_WORKSPACE_TOO_SMALL;
  void* lib_scratch = nullptr;
  HTTM_HIP(attention_static_scratch(&lib_scratch));
  return run_attention(q_m, k_log2, v_m, o_m, q_offsets, k_offsets, H, d_head, 1.0f, true, lib_scratch,
                       kAttnStaticScratchBytes, stream);
}

int httm_attention_split_plan(const int64_t* q_offsets, const int64_t* k_offsets, int H, int compute_units,
                              int32_t* summary, int32_t* segments, int64_t max_segments, int32_t* tiles,
                              int64_t max_tiles) {
  if (!q_offsets || !k_offsets || !summary || H <= 0 || compute_units <= 0) return HTTM_E_INVALID_ARG;
  if (H > HTTM_MAX_HEADS) return HTTM_E_UNSUPPORTED;
  for (int h = 0; h < H; ++h)
    if (q_offsets[h + 1] < q_offsets[h] || k_offsets[h + 1] < k_offsets[h]) return HTTM_E_INVALID_ARG;
  SplitPlan sp;
  int64_t kept_full = 0;
  int split_ragged = 0;
  plan_attention_split(q_offsets, k_offsets, H, compute_units, &sp, &kept_full, &split_ragged);
  const int64_t n_slots = split_slots(sp);
  summary[0] = sp.n_tiles;
  summary[1] = sp.shares;
  summary[2] = sp.share_units;
  summary[3] = sp.span;
  summary[4] = (int32_t)n_slots;
  summary[5] = sp.units;
  summary[6] = (int32_t)kept_full;
  summary[7] = split_ragged;
  if (segments) {
    if (max_segments < n_slots) return HTTM_E_WORKSPACE_TOO_SMALL;
    for (int64_t b = 0; b < n_slots; ++b) {
      const int32_t unused[5] = {0, 0, 0, 0, (int32_t)b};
      std::memcpy(segments + 5 * b, unused, sizeof(unused));
    }
    for (int s = 0; s < sp.shares; ++s) {       // as a workgroup walks its share
      int first = 0, count = 0;
      split_share_tiles(sp, s, &first, &count);
      for (int e = first; e < first + count; ++e) {
        const SplitSegment g = split_segment(sp, s, e);
        const int32_t row[5] = {g.head, g.q0, g.t0, g.t1, g.slot};
        if (g.slot < 0 || g.slot >= n_slots) return HTTM_E_INVALID_ARG;
        std::memcpy(segments + 5 * (int64_t)g.slot, row, sizeof(row));
      }
    }
  }
  if (tiles) {
    if (max_tiles < sp.n_tiles) return HTTM_E_WORKSPACE_TOO_SMALL;
    for (int e = 0; e < sp.n_tiles; ++e) {
      const SplitTile t = split_tile(sp, e);
      const int32_t row[4] = {t.head, t.q0, t.first_share, t.last_share};
      std::memcpy(tiles + 4 * e, row, sizeof(row));
    }
  }
  return HTTM_OK;
}

int64_t httm_attention_scratch_bytes(int H) { return H > 0 && H <= HTTM_MAX_HEADS ? attention_scratch_bytes(H) : 0; }

int httm_unmerge(const httm_plan_t* p, const void* o_m, const int32_t* assign_q, void* out,
                 int fuse_inverse_reorder, void* stream) {
  if (!p || !o_m || !assign_q || !out || o_m == out) return HTTM_E_INVALID_ARG;
  // The assignment a plan with the outlier filter writes holds negative entries (rows of o_out),
  // which this call has no tensor for: such plans go through httm_unmerge_filtered.
  if (p->outlier_cap > 0) return HTTM_E_INVALID_ARG;
  if (!aligned16(o_m) || !aligned16(out) || !aligned16(assign_q)) return HTTM_E_INVALID_ARG;
  HTTM_HIP(launch_unmerge(o_m, assign_q, p->d_pi, out, p->geom.H, p->sizes.N, p->sizes.M_q,
                          fuse_inverse_reorder ? 1 : 0, (hipStream_t)stream));
  return HTTM_OK;
}

int httm_layer_forward(const httm_plan_t* p, const void* q, const void* k, const void* v, void* out,
                       void* workspace, size_t workspace_bytes, void* stream) {
  if (!p || !q || !k || !v || !out || !workspace) return HTTM_E_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out)) return HTTM_E_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return HTTM_E_INVALID_ARG;
  if ((int64_t)workspace_bytes < p->ws.total) return HTTM_E_WORKSPACE_TOO_SMALL;
  hipStream_t st = (hipStream_t)stream;
  char* ws = (char*)workspace;
  void* q_m = ws + p->ws.q_m;
  void* k_m = ws + p->ws.k_m;
  void* v_m = ws + p->ws.v_m;
  void* o_m = ws + p->ws.o_m;
  int32_t* assign_q = (int32_t*)(ws + p->ws.assign_q);
  int32_t* assign_k = (int32_t*)(ws + p->ws.assign_k);
  const bool filtered = p->outlier_cap > 0;
  float* eps_q = (float*)(ws + p->ws.eps_q);
  void* q_out = ws + p->ws.q_out;
  void* o_out = ws + p->ws.o_out;
  // Stages 1+2 fused: the matching kernel gathers its rows through pi.
  int rc = filtered ? run_match_merge_filtered(p, q, k, v, q_m, k_m, v_m, assign_q, assign_k, eps_q,
                                               q_out, st)
                    : run_match_merge(p, p->d_pi, q, k, v, q_m, k_m, v_m, assign_q, assign_k, nullptr,
                                      nullptr, st);
  if (rc != HTTM_OK) return rc;
  // Stage 3.
  const int H = p->geom.H;
  int64_t q_off[HTTM_MAX_HEADS + 1], k_off[HTTM_MAX_HEADS + 1];
  for (int h = 0; h <= H; ++h) {
    q_off[h] = (int64_t)h * p->sizes.M_q;
    k_off[h] = (int64_t)h * p->sizes.M_k;
  }
  if (filtered) {
    // Alg. 1: the outlier queries attend on their own - same launch, workgroups appended to the grid
    HTTM_HIP(launch_attention_both(q_m, k_m, v_m, o_m, q_off, k_off, H, 0.125f, q_out, o_out, p->ob.offsets,
                                   p->ob.tiles, p->ob.max_tiles, log2_keys(p), st, ws + p->ws.attn_split,
                                   attention_scratch_bytes(H)));
  } else {
    HTTM_HIP(launch_attention(q_m, k_m, v_m, o_m, q_off, k_off, H, 0.125f, log2_keys(p), st, ws + p->ws.attn_split,
                              attention_scratch_bytes(H)));
  }
  // Stage 4 with the inverse reorder fused.
  HTTM_HIP(launch_unmerge(o_m, assign_q, p->d_pi, out, H, p->sizes.N, p->sizes.M_q, 1, st,
                          filtered ? o_out : nullptr));
  return HTTM_OK;
}

int httm_reorder_match_merge_filtered(const httm_plan_t* p, const void* q, const void* k, const void* v,
                                      void* q_m, void* k_m, void* v_m, int32_t* assign_q,
                                      int32_t* assign_k, float* eps_q, void* q_out, void* stream) {
  if (!p || !q || !k || !v || !q_m || !k_m || !v_m || !assign_q || !assign_k || !eps_q || !q_out)
    return HTTM_E_INVALID_ARG;
  if (p->outlier_cap <= 0) return HTTM_E_INVALID_ARG;
  const void* ptrs[] = {q, k, v, q_m, k_m, v_m, assign_q, assign_k, eps_q, q_out};
  for (const void* x : ptrs)
    if (!aligned16(x)) return HTTM_E_INVALID_ARG;
  return run_match_merge_filtered(p, q, k, v, q_m, k_m, v_m, assign_q, assign_k, eps_q, q_out,
                                  (hipStream_t)stream);
}

int httm_attention_outliers(const httm_plan_t* p, const void* q_out, const void* k_m, const void* v_m,
                            void* o_out, void* stream) {
  if (!p || !q_out || !k_m || !v_m || !o_out) return HTTM_E_INVALID_ARG;
  if (p->outlier_cap <= 0) return HTTM_E_INVALID_ARG;
  if (!aligned16(q_out) || !aligned16(k_m) || !aligned16(v_m) || !aligned16(o_out)) return HTTM_E_INVALID_ARG;
  return run_attention_outliers(p, q_out, k_m, v_m, o_out, (hipStream_t)stream);
}

int httm_unmerge_filtered(const httm_plan_t* p, const void* o_m, const void* o_out,
                          const int32_t* assign_q, void* out, void* stream) {
  if (!p || !o_m || !o_out || !assign_q || !out || o_m == out) return HTTM_E_INVALID_ARG;
  if (p->outlier_cap <= 0) return HTTM_E_INVALID_ARG;
  if (!aligned16(o_m) || !aligned16(o_out) || !aligned16(out) || !aligned16(assign_q)) return HTTM_E_INVALID_ARG;
  HTTM_HIP(launch_unmerge(o_m, assign_q, p->d_pi, out, p->geom.H, p->sizes.N, p->sizes.M_q, 1,
                          (hipStream_t)stream, o_out));
  return HTTM_OK;
}

int httm_outlier_stats(const httm_plan_t* p, float* tau, int32_t* counts, void* stream) {
  if (!p || !tau || !counts) return HTTM_E_INVALID_ARG;
  if (p->outlier_cap <= 0) return HTTM_E_INVALID_ARG;
  HTTM_HIP(hipStreamSynchronize((hipStream_t)stream));
  SelectState st;
  HTTM_HIP(hipMemcpy(&st, p->ob.state, sizeof(st), hipMemcpyDeviceToHost));
  *tau = st.tau;
  int32_t off[HTTM_MAX_HEADS + 1];
  HTTM_HIP(hipMemcpy(off, p->ob.offsets, (size_t)(p->geom.H + 1) * 4, hipMemcpyDeviceToHost));
  for (int h = 0; h < p->geom.H; ++h) counts[h] = off[h + 1] - off[h];
  return HTTM_OK;
}

}  // extern "C"
