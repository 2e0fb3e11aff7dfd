// Pooling + compiled-table application (paper Eq. 4 u = alpha * rho, Eq. 6 weighted max over heads,
// Sec. 4.3 gate lookup; 1-D pooling and the per-head budget split are workload definitions).
//
// One workgroup owns one tile of kTablesTile prefix positions of one (batch, KV head). For each query
// head of the group it stages the tile plus a halo of pool_kernel/2 positions in LDS, pools, multiplies
// by rho and by the head's weight, and keeps the running maximum in registers, so the window mass
// is read from HBM once and the utility written once.
#include "ckv_tables.h"

namespace ckv {

__global__ void __launch_bounds__(kTablesThreads) tables_kernel(TablesArgs a) {
  __shared__ float sm[kTablesTile + 2 * kMaxHalo];
  const int unit = blockIdx.y, tile = blockIdx.x;
  const int b = unit / a.Hkv, g = unit % a.Hkv;
  const int t0 = tile * kTablesTile;

  if (tile == 0 && g == 0 && threadIdx.x == 0) write_tau_and_budgets(a, b);
  if (a.P == 0) return;

  float best[kTablesPerThread];
  float rho[kTablesPerThread];
#pragma unroll
  for (int e = 0; e < kTablesPerThread; ++e) {
    best[e] = -INFINITY;
    const int t = t0 + threadIdx.x + e * kTablesThreads;
    rho[e] = (a.rho && t < a.P) ? a.rho[(size_t)unit * a.T + t] : 1.0f;
  }
  const int span = kTablesTile + 2 * a.radius;
  const float pad = a.pool == CKV_POOL_MAX ? -INFINITY : 0.0f;
  for (int hg = 0; hg < a.G; ++hg) {
    const int h = g * a.G + hg;
    const float *row = a.scores + ((size_t)b * a.Hq + h) * a.T;
    __syncthreads();  // previous head's tile fully consumed
    for (int i = threadIdx.x; i < span; i += kTablesThreads) {
      const int t = t0 - a.radius + i;
      sm[i] = (t >= 0 && t < a.P) ? row[t] : pad;  // pooling sees the prefix only
    }
    __syncthreads();
    const float wgt = a.w_row[h];
#pragma unroll
    for (int e = 0; e < kTablesPerThread; ++e) {
      const int i = threadIdx.x + e * kTablesThreads + a.radius;  // centre in sm
      float c;
      if (a.pool == CKV_POOL_AVG) {
        c = 0.0f;
        for (int dt = -a.radius; dt <= a.radius; ++dt) c += sm[i + dt];
        c = c / (float)a.kernel;
      } else if (a.pool == CKV_POOL_MAX) {
        c = -INFINITY;
        for (int dt = -a.radius; dt <= a.radius; ++dt) c = fmaxf(c, sm[i + dt]);
      } else {
        c = sm[i];
      }
      best[e] = fmaxf(best[e], wgt * (c * rho[e]));
    }
  }
#pragma unroll
  for (int e = 0; e < kTablesPerThread; ++e) {
    const int t = t0 + threadIdx.x + e * kTablesThreads;
    if (t < a.P) a.utility[(size_t)unit * a.P + t] = best[e];
  }
}

template <int POOL, int R>
__global__ void __launch_bounds__(kTablesThreads) tables_window_kernel(TablesArgs a) {
  const int unit = blockIdx.y;
  const int t = (blockIdx.x * kTablesThreads + threadIdx.x) * 4;  // first of this thread's positions
  if (blockIdx.x == 0 && unit % a.Hkv == 0 && threadIdx.x == 0) write_tau_and_budgets(a, unit / a.Hkv);
  if (t >= a.P) return;
  pool_four<POOL, R>(a, unit, t);
}

// Companion of the fused utility form of the scan's second pass (see fixup_range): one workgroup of 64
// threads per (wave range, unit) finishes what that pass leaves out; also writes tau and the budgets.
constexpr int kFixupThreads = 64;

template <int POOL, int R>
__global__ void __launch_bounds__(kFixupThreads) tables_fixup_kernel(TablesArgs a, FixupArgs f) {
  const int unit = blockIdx.y, range = blockIdx.x;
  if (range == 0 && unit % a.Hkv == 0 && threadIdx.x == 0) write_tau_and_budgets(a, unit / a.Hkv);
  fixup_range<POOL, R>(a, f, unit, range, threadIdx.x, kFixupThreads);
}

template <int POOL>
static bool launch_window_pool(const TablesArgs &a, dim3 grid, hipStream_t stream) {
  const dim3 block(kTablesThreads);
  switch (a.radius) {
    case 0: hipLaunchKernelGGL((tables_window_kernel<POOL, 0>), grid, block, 0, stream, a); return true;
    case 1: hipLaunchKernelGGL((tables_window_kernel<POOL, 1>), grid, block, 0, stream, a); return true;
    case 2: hipLaunchKernelGGL((tables_window_kernel<POOL, 2>), grid, block, 0, stream, a); return true;
    case 3: hipLaunchKernelGGL((tables_window_kernel<POOL, 3>), grid, block, 0, stream, a); return true;
    case 4: hipLaunchKernelGGL((tables_window_kernel<POOL, 4>), grid, block, 0, stream, a); return true;
  }
  return false;
}

hipError_t launch_apply_tables(const ckv_params *p, const Shape &s, const float *scores,
                               const float *vnorm_ratio, const float *w_head, const float *head_share,
                               const float *t_gate, int n_ent, int n_ppl, const int32_t *risk_bins,
                               float *utility, int32_t *budget, float *tau, hipStream_t stream) {
  const TablesArgs a = tables_args(p, s, scores, vnorm_ratio, w_head, head_share, t_gate, n_ent, n_ppl, risk_bins,
                                   utility, budget, tau);
  const dim3 grid(a.n_tiles, s.Bz * s.Hkv), block(kTablesThreads);
  const bool aligned = s.T % 4 == 0 && ((uintptr_t)scores % 16 == 0) && ((uintptr_t)utility % 16 == 0) &&
                       (!a.rho || (uintptr_t)a.rho % 16 == 0);
  bool done = false;
  if (aligned && s.P > 0 && a.radius <= 4)
    done = p->pool == CKV_POOL_MAX ? launch_window_pool<CKV_POOL_MAX>(a, grid, stream)
                                   : launch_window_pool<CKV_POOL_AVG>(a, grid, stream);
  if (!done) hipLaunchKernelGGL(tables_kernel, grid, block, 0, stream, a);
  return hipGetLastError();
}

template <int POOL>
static void launch_fixup_pool(const TablesArgs &a, const FixupArgs &f, dim3 grid, hipStream_t stream) {
  const dim3 block(kFixupThreads);
  switch (a.radius) {
    case 0: hipLaunchKernelGGL((tables_fixup_kernel<POOL, 0>), grid, block, 0, stream, a, f); break;
    case 1: hipLaunchKernelGGL((tables_fixup_kernel<POOL, 1>), grid, block, 0, stream, a, f); break;
    case 2: hipLaunchKernelGGL((tables_fixup_kernel<POOL, 2>), grid, block, 0, stream, a, f); break;
    default: hipLaunchKernelGGL((tables_fixup_kernel<POOL, 3>), grid, block, 0, stream, a, f); break;
  }
}

// The caller has checked utility_fast_path(): no value norm, radius <= 3, T and P multiples of four,
// 16-byte aligned scores and utility.
hipError_t launch_utility_fixup(const ckv_params *p, const Shape &s, const float *sparse_scores,
                                const float *w_head, const float *head_share, const float *t_gate, int n_ent,
                                int n_ppl, const int32_t *risk_bins, float *utility, int32_t *budget, float *tau,
                                hipStream_t stream) {
  const TablesArgs a = tables_args(p, s, sparse_scores, nullptr, w_head, head_share, t_gate, n_ent, n_ppl,
                                   risk_bins, utility, budget, tau);
  FixupArgs f;
  f.keys_per_wave = s.keys_per_wave;
  f.n_ranges = s.n_chunks * kScoreWaves;
  const dim3 grid(f.n_ranges, s.Bz * s.Hkv);
  if (p->pool == CKV_POOL_MAX) launch_fixup_pool<CKV_POOL_MAX>(a, f, grid, stream);
  else launch_fixup_pool<CKV_POOL_AVG>(a, f, grid, stream);
  return hipGetLastError();
}

}  // namespace ckv
