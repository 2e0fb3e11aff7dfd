// C-ABI entry points of libckv: argument validation on the host, then kernel launches.
// Nothing here allocates or synchronises; every entry point either enqueues all of its kernels on
// the caller's stream or returns an error before the first launch.
#include <math.h>

#include <mutex>

#include "ckv_internal.h"

namespace ckv {

static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

ckv_status validate(const ckv_params *p) {
  if (!p) return CKV_EINVAL;
  if (p->batch < 1 || p->n_kv_heads < 1 || p->n_q_heads < 1) return CKV_EINVAL;
  if (p->n_q_heads % p->n_kv_heads) return CKV_EINVAL;
  if (p->seq_len < 1 || p->window < 1 || p->window > p->seq_len) return CKV_EINVAL;
  if (p->n_layers < 1 || p->layer < 0 || p->layer >= p->n_layers) return CKV_EINVAL;
  if (p->dtype != CKV_F32 && p->dtype != CKV_BF16) return CKV_EINVAL;
  if (!(p->softmax_scale >= 0.0f) || isinf(p->softmax_scale)) return CKV_EINVAL;
  if (p->pool != CKV_POOL_NONE && p->pool != CKV_POOL_AVG && p->pool != CKV_POOL_MAX) return CKV_EINVAL;
  if (p->pool != CKV_POOL_NONE && (p->pool_kernel < 1 || p->pool_kernel > 63 || p->pool_kernel % 2 == 0))
    return CKV_EINVAL;
  if (p->budget_per_kv_head < p->window) return CKV_EINVAL;
  if (p->flags & ~(uint32_t)(CKV_FLAG_VALUE_NORM | CKV_FLAG_GROUP_MASS)) return CKV_EINVAL;
  if (p->head_dim < 1) return CKV_EINVAL;
  const int64_t b_tot = (int64_t)p->budget_per_kv_head * p->n_kv_heads;
  int64_t need = b_tot - (int64_t)(p->n_kv_heads - 1) * p->window;
  if (need > p->seq_len) need = p->seq_len;
  if (p->cap < need) return CKV_EINVAL;
  for (int i = 0; i < 3; ++i)
    if (p->q_stride[i] < 0 || p->k_stride[i] < 0 || p->v_stride[i] < 0) return CKV_EINVAL;
  // rows must hold head_dim contiguous elements and start 16-byte aligned for the 128-bit loads
  const int64_t per16 = p->dtype == CKV_BF16 ? 8 : 4;
  if (p->q_stride[2] < p->head_dim || p->k_stride[2] < p->head_dim || p->v_stride[2] < p->head_dim)
    return CKV_EINVAL;
  for (int i = 0; i < 3; ++i)
    if (p->q_stride[i] % per16 || p->k_stride[i] % per16 || p->v_stride[i] % per16) return CKV_EINVAL;
  if (p->head_dim != 64 && p->head_dim != 128) return CKV_EUNSUPPORTED;
  if (p->window > kMaxWindowTiles * kTile) return CKV_EUNSUPPORTED;
  if ((int64_t)p->batch * p->n_kv_heads > 65535) return CKV_EUNSUPPORTED;  // grid.y
  if (p->seq_len > (1 << 24)) return CKV_EUNSUPPORTED;
  // the staged scan addresses the 32 rows of a key tile with 32-bit offsets
  if (p->k_stride[2] * (int64_t)(p->dtype == CKV_BF16 ? 2 : 4) * kTile >= ((int64_t)1 << 31)) return CKV_EUNSUPPORTED;
  if ((int64_t)p->n_q_heads * p->seq_len >= (1 << 29)) return CKV_EUNSUPPORTED;  // scores of one batch element: < 2 GiB
  return CKV_OK;
}

void derive(const ckv_params *p, Shape *s) {
  s->Bz = p->batch;
  s->Hq = p->n_q_heads;
  s->Hkv = p->n_kv_heads;
  s->G = s->Hq / s->Hkv;
  s->d = p->head_dim;
  s->T = p->seq_len;
  s->W = p->window;
  s->P = s->T - s->W;
  s->esize = p->dtype == CKV_BF16 ? 2 : 4;
  s->WT = (s->W + kTile - 1) / kTile;
  s->n_tiles = s->G * s->WT;
  // Tiles a wave keeps in registers, whole heads only: eight for bf16 (a wave alone on its SIMD has 512
  // registers, and the matrix cores read operands from either half), four for f32 rows of 256 bytes,
  // one head's tiles for f32 rows of 512 bytes.
  const int budget_tiles = p->dtype == CKV_BF16 ? kMaxQTiles : s->d * s->esize <= 256 ? kMaxQTilesF32 : 1;
  const int per_wave_max = budget_tiles >= s->WT ? (budget_tiles / s->WT) * s->WT : s->WT;
  s->n_groups = (s->n_tiles + per_wave_max - 1) / per_wave_max;
  int nq = (s->n_tiles + s->n_groups - 1) / s->n_groups;
  nq = (nq + s->WT - 1) / s->WT * s->WT;
  s->NQ = nq;
  s->n_groups = (s->n_tiles + nq - 1) / nq;
  // Split the key axis. The bf16 kernels keep one workgroup per CU busy for the whole launch (their
  // set-up is not overlapped with anything, so there is one workgroup per CU and its waves sweep long
  // ranges, a whole number of four-tile pipeline rounds); the f32 kernels run two workgroups per CU
  // and like a few thousand of them.
  const int64_t units = (int64_t)s->Bz * s->Hkv * s->n_groups;
  const int64_t target_wgs = p->dtype == CKV_BF16 ? kComputeUnits : 2048;
  int64_t kpw = ((int64_t)s->T * units + kScoreWaves * target_wgs - 1) / (kScoreWaves * target_wgs);
  const int64_t quantum = p->dtype == CKV_BF16 && kpw > 4 * kTile ? 4 * kTile : kTile;
  kpw = (kpw + quantum - 1) / quantum * quantum;
  if (kpw < 2 * kTile) kpw = 2 * kTile;
  if (kpw > 4096) kpw = 4096;
  s->keys_per_wave = (int)kpw;
  s->n_chunks = (int)((s->T + kScoreWaves * kpw - 1) / (kScoreWaves * kpw));
  s->scale = p->softmax_scale > 0.0f ? p->softmax_scale : 1.0f / sqrtf((float)s->d);
}

int vnorm_blocks_per_unit(const Shape &s) {
  const int rows_per_block = 1024;
  return (s.T + rows_per_block - 1) / rows_per_block;
}

void layout(const ckv_params *p, const Shape &s, Workspace *w) {
  const size_t units = (size_t)s.Bz * s.Hkv;
  size_t off = 0;
  w->part_off = off;
  w->part_bytes = units * (size_t)s.n_groups * s.NQ * kTile * s.n_chunks * sizeof(float2);
  off = align256(off + w->part_bytes);
  w->lse_off = off;
  w->lse_bytes = (size_t)s.Bz * s.Hq * s.W * sizeof(float);
  off = align256(off + w->lse_bytes);
  w->vsum_off = off;
  w->vsum_bytes = (p->flags & CKV_FLAG_VALUE_NORM) ? units * vnorm_blocks_per_unit(s) * sizeof(float) : 0;
  off = align256(off + w->vsum_bytes);
  w->select_off = off;
  w->select_bytes = select_workspace_bytes(s);
  off = align256(off + w->select_bytes);
  w->total = off;
}

static ckv_status workspace_ok(const Workspace &w, const void *ws, size_t bytes) {
  if (!ws || ((uintptr_t)ws & 255) || bytes < w.total) return CKV_EWORKSPACE;
  return CKV_OK;
}

}  // namespace ckv

using namespace ckv;

extern "C" size_t ckv_workspace_bytes(const ckv_params *params) {
  if (validate(params) != CKV_OK) return 0;
  Shape s;
  Workspace w;
  derive(params, &s);
  layout(params, s, &w);
  return w.total;
}

extern "C" ckv_status ckv_window_scores(const ckv_params *params, const void *q_win, const void *k,
                                        const void *v, const float *lse, float *scores,
                                        float *vnorm_ratio, void *workspace, size_t workspace_bytes,
                                        void *hip_stream) {
  ckv_status st = validate(params);
  if (st != CKV_OK) return st;
  if (!q_win || !k || !scores) return CKV_EINVAL;
  const bool vn = params->flags & CKV_FLAG_VALUE_NORM;
  if (vn && (!v || !vnorm_ratio)) return CKV_EINVAL;
  Shape s;
  Workspace w;
  derive(params, &s);
  layout(params, s, &w);
  st = workspace_ok(w, workspace, workspace_bytes);
  if (st != CKV_OK) return st;
  // the group-mass output exists where one wave holds all query heads of a KV head, one tile each
  if ((params->flags & CKV_FLAG_GROUP_MASS) && !(params->dtype == CKV_BF16 && s.n_groups == 1 && s.WT == 1 && s.NQ <= 4))
    return CKV_EUNSUPPORTED;
  hipStream_t stream = (hipStream_t)hip_stream;
  if (launch_window_scores(params, s, w, q_win, k, lse, nullptr, scores, (char *)workspace, stream) != hipSuccess)
    return CKV_EHIP;
  if (vn && launch_value_norm(params, s, w, v, vnorm_ratio, (char *)workspace, stream) != hipSuccess)
    return CKV_EHIP;
  return CKV_OK;
}

extern "C" ckv_status ckv_window_lse(const ckv_params *params, const void *q_win, const void *k,
                                     float *lse, void *workspace, size_t workspace_bytes,
                                     void *hip_stream) {
  ckv_status st = validate(params);
  if (st != CKV_OK) return st;
  if (!q_win || !k || !lse) return CKV_EINVAL;
  Shape s;
  Workspace w;
  derive(params, &s);
  layout(params, s, &w);
  st = workspace_ok(w, workspace, workspace_bytes);
  if (st != CKV_OK) return st;
  if (launch_window_scores(params, s, w, q_win, k, nullptr, lse, nullptr, (char *)workspace,
                           (hipStream_t)hip_stream) != hipSuccess)
    return CKV_EHIP;
  return CKV_OK;
}

// ---------------------------------------------------------------------------------------------
// ckv_window_lse for callers that cannot allocate: the row partials of the scan's first pass live in a
// device array of the library instead of a caller's workspace. Host code never passes the array's name
// to a kernel (on the host it is only a stand-in for the symbol): the device address is looked up once
// per device, with that device current, and kept.
// ---------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[CKV_STATIC_SCRATCH_BYTES];
static constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device, once known

static hipError_t static_scratch(void **out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

extern "C" size_t ckv_window_lse_static_bytes(const ckv_params *params) {
  if (validate(params) != CKV_OK) return 0;
  Shape s;
  Workspace w;
  derive(params, &s);
  layout(params, s, &w);
  return w.part_bytes;
}

extern "C" ckv_status ckv_window_lse_static(const ckv_params *params, const void *q_win, const void *k, float *lse,
                                            void *hip_stream) {
  ckv_status st = validate(params);
  if (st != CKV_OK) return st;
  if (!q_win || !k || !lse) return CKV_EINVAL;
  Shape s;
  Workspace w;
  derive(params, &s);
  layout(params, s, &w);
  // only the row partials are scratch here (they sit first in the layout); LSE goes to the caller's buffer
  if (w.part_off != 0 || w.part_bytes > (size_t)CKV_STATIC_SCRATCH_BYTES) return CKV_EWORKSPACE;
  void *ptr = nullptr;
  if (static_scratch(&ptr) != hipSuccess) return CKV_EHIP;
  if (launch_window_scores(params, s, w, q_win, k, nullptr, lse, nullptr, (char *)ptr, (hipStream_t)hip_stream) !=
      hipSuccess)
    return CKV_EHIP;
  return CKV_OK;
}

extern "C" ckv_status ckv_apply_tables(const ckv_params *params, const float *scores,
                                       const float *vnorm_ratio, const float *w_head,
                                       const float *head_share, const float *t_gate, int32_t n_ent,
                                       int32_t n_ppl, const int32_t *risk_bins, float *utility,
                                       int32_t *budget, float *tau, void *hip_stream) {
  ckv_status st = validate(params);
  if (st != CKV_OK) return st;
  if (!scores || !w_head || !utility || !budget || !tau) return CKV_EINVAL;
  if (params->flags & CKV_FLAG_GROUP_MASS) return CKV_EINVAL;  // needs per-head masses
  if ((params->flags & CKV_FLAG_VALUE_NORM) && !vnorm_ratio) return CKV_EINVAL;
  if (t_gate && (n_ent < 1 || n_ppl < 1 || !risk_bins)) return CKV_EINVAL;
  Shape s;
  derive(params, &s);
  if (launch_apply_tables(params, s, scores, vnorm_ratio, w_head, head_share, t_gate, n_ent, n_ppl,
                          risk_bins, utility, budget, tau, (hipStream_t)hip_stream) != hipSuccess)
    return CKV_EHIP;
  return CKV_OK;
}

// Whether ckv_window_utility can run its fused second pass for this call (else it runs the two
// unfused steps through the scratch buffer): the pipelined bf16 kernels with at most two 32-row tiles per
// head and all query tiles of a group in one wave (at most eight), pooling kernels of at most 7 taps, rows that keep the
// 128-bit and 64-bit accesses aligned. With the value-norm flag the ratio, which is common to a group's
// heads and non-negative, multiplies the group maximum afterwards (in the value-norm scaling pass).
static bool utility_fast_path(const ckv_params *p, const Shape &s, const float *scratch, const float *utility) {
  const int kernel = p->pool == CKV_POOL_NONE ? 1 : p->pool_kernel;
  return p->dtype == CKV_BF16 && s.n_groups == 1 && s.WT <= 2 && kernel / 2 <= 3 && s.T % 4 == 0 && s.P % 4 == 0 && s.P > 0 && (uintptr_t)scratch % 16 == 0 &&
         (uintptr_t)utility % 16 == 0 && (int64_t)s.Hkv * s.P < (1 << 29);
}

extern "C" ckv_status ckv_window_utility(const ckv_params *params, const void *q_win, const void *k,
                                         const void *v, const float *lse, const float *w_head,
                                         const float *head_share, const float *t_gate, int32_t n_ent,
                                         int32_t n_ppl, const int32_t *risk_bins, float *scores_scratch,
                                         float *vnorm_ratio, float *utility, int32_t *budget, float *tau,
                                         void *workspace, size_t workspace_bytes, void *hip_stream) {
  ckv_status st = validate(params);
  if (st != CKV_OK) return st;
  if (!q_win || !k || !scores_scratch || !w_head || !utility || !budget || !tau) return CKV_EINVAL;
  if (params->flags & CKV_FLAG_GROUP_MASS) return CKV_EINVAL;  // needs per-head masses
  const bool vn = params->flags & CKV_FLAG_VALUE_NORM;
  if (vn && (!v || !vnorm_ratio)) return CKV_EINVAL;
  if (t_gate && (n_ent < 1 || n_ppl < 1 || !risk_bins)) return CKV_EINVAL;
  Shape s;
  Workspace w;
  derive(params, &s);
  layout(params, s, &w);
  st = workspace_ok(w, workspace, workspace_bytes);
  if (st != CKV_OK) return st;
  hipStream_t stream = (hipStream_t)hip_stream;
  if (utility_fast_path(params, s, scores_scratch, utility)) {
    UtilityFusion fuse;
    fuse.w_row = w_head + (size_t)params->layer * s.Hq;
    fuse.utility = utility;
    fuse.pool = params->pool;
    const int kernel = params->pool == CKV_POOL_NONE ? 1 : params->pool_kernel;
    fuse.radius = kernel / 2;
    fuse.inv_kernel = 1.0f / (float)kernel;
    if (launch_window_scores(params, s, w, q_win, k, lse, nullptr, scores_scratch, (char *)workspace, stream,
                             &fuse) != hipSuccess)
      return CKV_EHIP;
    if (launch_utility_fixup(params, s, scores_scratch, w_head, head_share, t_gate, n_ent, n_ppl, risk_bins,
                             utility, budget, tau, stream) != hipSuccess)
      return CKV_EHIP;
    if (vn && launch_value_norm(params, s, w, v, vnorm_ratio, (char *)workspace, stream, utility) != hipSuccess)
      return CKV_EHIP;
    return CKV_OK;
  }
  if (launch_window_scores(params, s, w, q_win, k, lse, nullptr, scores_scratch, (char *)workspace, stream) !=
      hipSuccess)
    return CKV_EHIP;
  if (vn && launch_value_norm(params, s, w, v, vnorm_ratio, (char *)workspace, stream) != hipSuccess) return CKV_EHIP;
  if (launch_apply_tables(params, s, scores_scratch, vnorm_ratio, w_head, head_share, t_gate, n_ent, n_ppl,
                          risk_bins, utility, budget, tau, stream) != hipSuccess)
    return CKV_EHIP;
  return CKV_OK;
}

extern "C" ckv_status ckv_select_topk(const ckv_params *params, const float *utility,
                                      const int32_t *budget, const float *tau, int32_t *idx,
                                      int32_t *count, void *workspace, size_t workspace_bytes,
                                      void *hip_stream) {
  ckv_status st = validate(params);
  if (st != CKV_OK) return st;
  if (!utility || !budget || !tau || !idx || !count) return CKV_EINVAL;
  Shape s;
  derive(params, &s);
  // Optional: short prefixes are selected by one workgroup per unit, everything on chip; for long ones a
  // workspace lets the selection split a unit over several workgroups.
  Workspace w;
  layout(params, s, &w);
  const bool split = workspace && w.select_bytes > 0;
  if (split && workspace_ok(w, workspace, workspace_bytes) != CKV_OK) return CKV_EWORKSPACE;
  if (launch_select(params, s, utility, budget, tau, idx, count, split ? (char *)workspace + w.select_off : nullptr,
                    (hipStream_t)hip_stream) != hipSuccess)
    return CKV_EHIP;
  return CKV_OK;
}

extern "C" ckv_status ckv_compact_kv(const ckv_params *params, const void *k, const void *v,
                                     const int32_t *idx, const int32_t *count, void *k_out,
                                     void *v_out, void *hip_stream) {
  ckv_status st = validate(params);
  if (st != CKV_OK) return st;
  if (!k || !v || !idx || !count || !k_out || !v_out) return CKV_EINVAL;
  Shape s;
  derive(params, &s);
  if (launch_gather(params, s, k, v, idx, count, k_out, v_out, (hipStream_t)hip_stream) != hipSuccess)
    return CKV_EHIP;
  return CKV_OK;
}

extern "C" ckv_status ckv_alpha_accumulate(const ckv_params *params, const float *scores, float weight,
                                           float *alpha, void *hip_stream) {
  ckv_status st = validate(params);
  if (st != CKV_OK) return st;
  if (!scores || !alpha || !isfinite(weight)) return CKV_EINVAL;
  Shape s;
  derive(params, &s);
  const int rows = (params->flags & CKV_FLAG_GROUP_MASS) ? s.Hkv : s.Hq;  // rows of scores per batch element
  if (launch_alpha_accumulate(s, rows, scores, weight, alpha, (hipStream_t)hip_stream) != hipSuccess) return CKV_EHIP;
  return CKV_OK;
}

extern "C" ckv_status ckv_risk_struct(const ckv_params *params, const float *alpha, const float *ent_edges,
                                      int32_t n_edges, float *risk, int32_t *bin, void *hip_stream) {
  ckv_status st = validate(params);
  if (st != CKV_OK) return st;
  if (!alpha || !risk || n_edges < 0 || (bin && n_edges > 0 && !ent_edges)) return CKV_EINVAL;
  Shape s;
  derive(params, &s);
  if (launch_risk_struct(s, alpha, ent_edges, n_edges, risk, bin, (hipStream_t)hip_stream) != hipSuccess)
    return CKV_EHIP;
  return CKV_OK;
}

extern "C" ckv_status ckv_shared_utility(const ckv_params *params, const float *alpha, const float *vnorm_ratio,
                                         const float *w_head, const float *t_gate, int32_t n_ent, int32_t n_ppl,
                                         const int32_t *risk_bins, float *utility, float *tau, void *hip_stream) {
  ckv_status st = validate(params);
  if (st != CKV_OK) return st;
  if (!alpha || !vnorm_ratio || !w_head || !utility || !tau) return CKV_EINVAL;
  if (t_gate && (n_ent < 1 || n_ppl < 1 || !risk_bins)) return CKV_EINVAL;
  Shape s;
  derive(params, &s);
  if (launch_shared_utility(params, s, alpha, vnorm_ratio, w_head, t_gate, n_ent, n_ppl, risk_bins, utility, tau,
                            (hipStream_t)hip_stream) != hipSuccess)
    return CKV_EHIP;
  return CKV_OK;
}

extern "C" ckv_status ckv_compact_kv_shared(const ckv_params *params, const void *k, const void *v,
                                            const int32_t *idx, const int32_t *count, void *k_out, void *v_out,
                                            void *hip_stream) {
  ckv_status st = validate(params);
  if (st != CKV_OK) return st;
  if (!k || !v || !idx || !count || !k_out || !v_out) return CKV_EINVAL;
  Shape s;
  derive(params, &s);
  if (launch_gather(params, s, k, v, idx, count, k_out, v_out, (hipStream_t)hip_stream, true) != hipSuccess)
    return CKV_EHIP;
  return CKV_OK;
}

extern "C" ckv_status ckv_map_table_depth(const float *table, int32_t n_layers_src, int32_t row_elems, float *mapped,
                                          int32_t n_layers_dst, void *hip_stream) {
  if (!table || !mapped || n_layers_src < 1 || n_layers_dst < 1 || row_elems < 1) return CKV_EINVAL;
  if ((int64_t)n_layers_dst * row_elems > (1 << 30)) return CKV_EUNSUPPORTED;
  if (launch_map_depth(table, n_layers_src, row_elems, mapped, n_layers_dst, (hipStream_t)hip_stream) != hipSuccess)
    return CKV_EHIP;
  return CKV_OK;
}

static ckv_status decode_args_ok(const ckv_params *p, int32_t n_q, int32_t n_rows, const int64_t *k_stride,
                                 const int64_t *v_stride) {
  if (n_q < 1 || n_rows < 1 || !k_stride || !v_stride) return CKV_EINVAL;
  const int64_t per16 = p->dtype == CKV_BF16 ? 8 : 4;
  for (int i = 0; i < 3; ++i)
    if (k_stride[i] < 0 || v_stride[i] < 0 || k_stride[i] % per16 || v_stride[i] % per16) return CKV_EINVAL;
  if (k_stride[2] < p->head_dim || v_stride[2] < p->head_dim) return CKV_EINVAL;
  if (n_rows > (1 << 24)) return CKV_EUNSUPPORTED;
  return CKV_OK;
}

extern "C" size_t ckv_decode_workspace_bytes(const ckv_params *params, int32_t n_q, int32_t n_rows) {
  if (validate(params) != CKV_OK || n_q < 1 || n_rows < 1) return 0;
  Shape s;
  derive(params, &s);
  const DecodePlan plan = plan_decode(s, n_q, n_rows);
  if (plan.grid_y > 65535) return 0;
  return align256(plan.workspace_bytes);
}

extern "C" ckv_status ckv_decode_attention(const ckv_params *params, const void *q_dec, int32_t n_q,
                                           const void *k_rows, const void *v_rows, const int64_t *k_stride,
                                           const int64_t *v_stride, int32_t n_rows, const int32_t *count,
                                           float *out, float *lse, void *workspace, size_t workspace_bytes,
                                           void *hip_stream) {
  ckv_status st = validate(params);
  if (st != CKV_OK) return st;
  if (!q_dec || !k_rows || !v_rows || !out || !lse) return CKV_EINVAL;
  st = decode_args_ok(params, n_q, n_rows, k_stride, v_stride);
  if (st != CKV_OK) return st;
  if (((uintptr_t)q_dec | (uintptr_t)k_rows | (uintptr_t)v_rows) & 15) return CKV_EINVAL;
  Shape s;
  derive(params, &s);
  const DecodePlan plan = plan_decode(s, n_q, n_rows);
  if (plan.grid_y > 65535) return CKV_EUNSUPPORTED;  // grid.y
  if (plan.workspace_bytes > 0 &&
      (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < plan.workspace_bytes))
    return CKV_EWORKSPACE;
  if (launch_decode_attention(params, s, q_dec, n_q, k_rows, v_rows, k_stride, v_stride, n_rows, count, out, lse,
                              (char *)workspace, (hipStream_t)hip_stream) != hipSuccess)
    return CKV_EHIP;
  return CKV_OK;
}

extern "C" ckv_status ckv_discarded_mass(const ckv_params *params, int32_t n_q, const float *lse_full,
                                         const float *lse_kept, float *mass, float *eps_tail, void *hip_stream) {
  ckv_status st = validate(params);
  if (st != CKV_OK) return st;
  if (n_q < 1 || !lse_full || !lse_kept || !mass) return CKV_EINVAL;
  Shape s;
  derive(params, &s);
  if (launch_discarded_mass(s, n_q, lse_full, lse_kept, mass, eps_tail, (hipStream_t)hip_stream) != hipSuccess)
    return CKV_EHIP;
  return CKV_OK;
}

extern "C" const char *ckv_status_string(ckv_status status) {
  switch (status) {
    case CKV_OK: return "ok";
    case CKV_EINVAL: return "invalid argument";
    case CKV_EUNSUPPORTED: return "unsupported configuration";
    case CKV_EWORKSPACE: return "workspace missing, misaligned or too small";
    case CKV_EHIP: return "HIP launch failed";
  }
  return "unknown status";
}
