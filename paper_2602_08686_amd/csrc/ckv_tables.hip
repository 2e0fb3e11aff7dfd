// Pooling + compiled-table application (paper Eq. 4 u = alpha * rho, Eq. 6 weighted max over heads,
// Sec. 4.3 gate lookup; 1-D pooling and the per-head budget split are workload definitions).
//
// One workgroup owns one tile of kTablesTile prefix positions of one (batch, KV head). For each query
// head of the group it stages the tile plus a halo of pool_kernel/2 positions in LDS, pools, multiplies
// by rho and by the head's weight, and keeps the running maximum in registers, so the window mass
// is read from HBM once and the utility written once.
#include "ckv_internal.h"

namespace ckv {

constexpr int kTablesThreads = 256;
constexpr int kTablesPerThread = 4;
constexpr int kTablesTile = kTablesThreads * kTablesPerThread;  // 1024 positions
constexpr int kMaxHalo = 31;                                    // pool_kernel <= 63
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

struct TablesArgs {
  const float *scores;  // [Bz][Hq][T]
  const float *rho;     // [Bz][Hkv][T] or null
  const float *w_row;   // w_head + layer*Hq
  const float *share_row;  // head_share + layer*Hkv or null
  const float *gate_layer; // t_gate + layer*n_ent*n_ppl or null
  const int32_t *risk_bins;
  int n_ent, n_ppl;
  float *utility;  // [Bz][Hkv][P]
  int32_t *budget;
  float *tau;
  int Bz, Hq, Hkv, G, T, W, P;
  int pool, radius, kernel;
  int B;  // nominal budget per KV head
  int n_tiles;
};

// Per-head budgets of one batch element (same rule for every b; written per b for the ABI's layout).
__device__ void write_budgets(const TablesArgs &a, int b) {
  int32_t *out = a.budget + (size_t)b * a.Hkv;
  if (!a.share_row) {
    for (int g = 0; g < a.Hkv; ++g) out[g] = min(a.B, a.T);
    return;
  }
  const long long b_tot = (long long)a.B * a.Hkv;
  long long total = 0;
  for (int g = 0; g < a.Hkv; ++g) {
    double want = floor((double)a.share_row[g] * (double)b_tot);
    if (!(want >= (double)a.W)) want = (double)a.W;
    if (want > (double)a.T) want = (double)a.T;
    out[g] = (int32_t)want;
    total += out[g];
  }
  // "While the sum exceeds B_tot, the largest budget above W (lowest head on ties) loses one", done
  // a level at a time: the n1 leaders drop together to the runner-up's value (never below W), or,
  // when the excess runs out first, share it evenly with the remainder going to the lowest heads.
  long long excess = total - b_tot;
  while (excess > 0) {
    int v1 = a.W, v2 = a.W, n1 = 0;
    for (int g = 0; g < a.Hkv; ++g) v1 = max(v1, out[g]);
    if (v1 <= a.W) break;
    for (int g = 0; g < a.Hkv; ++g) {
      if (out[g] == v1) ++n1;
      else v2 = max(v2, out[g]);
    }
    const long long drop = v1 - v2;
    if ((long long)n1 * drop <= excess) {
      for (int g = 0; g < a.Hkv; ++g)
        if (out[g] == v1) out[g] = v2;
      excess -= (long long)n1 * drop;
    } else {
      const int each = (int)(excess / n1);
      int extra = (int)(excess % n1);
      for (int g = 0; g < a.Hkv; ++g)
        if (out[g] == v1) {
          out[g] = v1 - each - (extra > 0 ? 1 : 0);
          if (extra > 0) --extra;
        }
      excess = 0;
    }
  }
}

__device__ __forceinline__ void write_tau_and_budgets(const TablesArgs &a, int b) {
  float tau = 0.0f;
  if (a.gate_layer) {
    const int be = min(max(a.risk_bins[2 * b], 0), a.n_ent - 1);
    const int bp = min(max(a.risk_bins[2 * b + 1], 0), a.n_ppl - 1);
    tau = a.gate_layer[be * a.n_ppl + bp];
  }
  a.tau[b] = tau;
  write_budgets(a, b);
}

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

// Fast path for pooling kernels of at most 9 taps on 16-byte aligned rows (T % 4 == 0): a thread owns
// four consecutive positions and reads them plus the four on either side as three 128-bit loads per
// head (the neighbours' loads hit L1), pools from registers with the taps unrolled, and writes one
// 128-bit store (or scalars where P is not a multiple of four). No LDS and no barriers.
// Utilities of the four positions t .. t + 3 (t a multiple of four, t < P) of one (batch, KV head).
template <int POOL, int R>
__device__ __forceinline__ void pool_four(const TablesArgs &a, int unit, int t) {
  const int b = unit / a.Hkv, g = unit % a.Hkv;
  const float pad = POOL == CKV_POOL_MAX ? -INFINITY : 0.0f;
  float rho[4] = {1.0f, 1.0f, 1.0f, 1.0f};
  if (a.rho) {
    const f32x4_t r4 = *reinterpret_cast<const f32x4_t *>(a.rho + (size_t)unit * a.T + t);
#pragma unroll
    for (int e = 0; e < 4; ++e) rho[e] = r4[e];
  }
  float best[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
  for (int hg = 0; hg < a.G; ++hg) {
    const int h = g * a.G + hg;
    const float *row = a.scores + ((size_t)b * a.Hq + h) * a.T;
    // w[0..11] = positions t-4 .. t+7; everything outside [0, P) counts as padding. Rows hold T >= P + 1
    // floats and T % 4 == 0, so the three loads stay inside the row whenever their first index is < T.
    float w[12];
    const f32x4_t mid = *reinterpret_cast<const f32x4_t *>(row + t);
    f32x4_t lo = {pad, pad, pad, pad}, hi = {pad, pad, pad, pad};
    if (R > 0 && t >= 4) lo = *reinterpret_cast<const f32x4_t *>(row + t - 4);
    if (R > 0 && t + 4 < a.T) hi = *reinterpret_cast<const f32x4_t *>(row + t + 4);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      w[e] = lo[e];
      w[4 + e] = (t + e < a.P) ? mid[e] : pad;
      w[8 + e] = (t + 4 + e < a.P) ? hi[e] : pad;
    }
    const float wgt = a.w_row[h];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float c = w[4 + e - R];
#pragma unroll
      for (int d = 1 - R; d <= R; ++d) c = POOL == CKV_POOL_MAX ? fmaxf(c, w[4 + e + d]) : c + w[4 + e + d];
      if (POOL == CKV_POOL_AVG) c = c / (float)(2 * R + 1);
      best[e] = fmaxf(best[e], wgt * (c * rho[e]));
    }
  }
  float *out = a.utility + (size_t)unit * a.P + t;
  if (a.P % 4 == 0) {
    *reinterpret_cast<f32x4_t *>(out) = f32x4_t{best[0], best[1], best[2], best[3]};
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (t + e < a.P) out[e] = best[e];
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

// Companion of the fused utility form of the scan's second pass. That pass writes the utilities of
// the keys its pipeline takes (whole 128-key rounds at the front of every wave's key range) except
// the first four and the last kScanTrail of them (its output windows trail the rounds by that much so
// that its stores stay 128-byte aligned), and stores raw column sums only around those two places and
// for the tail of the range. This kernel computes what is missing from the raw sums: per wave range
// the four-key group at the front, the last kScanTrail / 4 groups of the pipelined part, and every
// group of the tail. One workgroup of 64 threads per (wave range, unit); also writes tau and the
// budgets.
struct FixupArgs {
  int keys_per_wave, n_ranges;  // the scan's split of the key axis
};
constexpr int kFixupThreads = 64;
constexpr int kScanBlockKeys = kRing * kTile;  // keys per pipeline round of the scan
constexpr int kScanTrail = kUtilShift;         // pipelined keys at the end of a range that the scan leaves to this kernel

template <int POOL, int R>
__global__ void __launch_bounds__(kFixupThreads) tables_fixup_kernel(TablesArgs a, FixupArgs f) {
  const int unit = blockIdx.y, range = blockIdx.x;
  if (range == 0 && unit % a.Hkv == 0 && threadIdx.x == 0) write_tau_and_budgets(a, unit / a.Hkv);
  const int t_begin = range * f.keys_per_wave;
  if (t_begin >= a.T) return;
  const int t_end = min(t_begin + f.keys_per_wave, a.T);
  const int n_full = max(0, (min(t_end, a.P) - t_begin) / kTile);   // tiles wholly inside the prefix
  const int n_blocks = n_full / kRing;                               // pipeline rounds
  const int tail0 = t_begin + n_blocks * kScanBlockKeys, tail1 = min(t_end, a.P);
  const int n_tail = tail1 > tail0 ? (tail1 - tail0 + 3) / 4 : 0;
  const int n_edge = n_blocks > 0 ? 1 + kScanTrail / 4 : 0;
  for (int i = threadIdx.x; i < n_edge + n_tail; i += kFixupThreads) {
    const int t = i < n_edge ? (i == 0 ? t_begin : tail0 - kScanTrail + (i - 1) * 4) : tail0 + (i - n_edge) * 4;
    pool_four<POOL, R>(a, unit, t);
  }
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

static TablesArgs tables_args(const ckv_params *p, const Shape &s, const float *scores,
                              const float *vnorm_ratio, const float *w_head, const float *head_share,
                              const float *t_gate, int n_ent, int n_ppl, const int32_t *risk_bins,
                              float *utility, int32_t *budget, float *tau) {
  TablesArgs a;
  a.scores = scores;
  a.rho = (p->flags & CKV_FLAG_VALUE_NORM) ? vnorm_ratio : nullptr;
  a.w_row = w_head + (size_t)p->layer * s.Hq;
  a.share_row = head_share ? head_share + (size_t)p->layer * s.Hkv : nullptr;
  a.gate_layer = t_gate ? t_gate + (size_t)p->layer * n_ent * n_ppl : nullptr;
  a.risk_bins = risk_bins;
  a.n_ent = n_ent;
  a.n_ppl = n_ppl;
  a.utility = utility;
  a.budget = budget;
  a.tau = tau;
  a.Bz = s.Bz; a.Hq = s.Hq; a.Hkv = s.Hkv; a.G = s.G; a.T = s.T; a.W = s.W; a.P = s.P;
  a.pool = p->pool;
  a.kernel = p->pool == CKV_POOL_NONE ? 1 : p->pool_kernel;
  a.radius = a.kernel / 2;
  a.B = p->budget_per_kv_head;
  a.n_tiles = s.P > 0 ? (s.P + kTablesTile - 1) / kTablesTile : 1;
  return a;
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
