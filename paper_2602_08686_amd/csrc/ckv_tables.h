// Device code of the tables kernels (ckv_tables.hip): the argument block, the budget rule and the gate
// lookup (paper Sec. 4.3), the four-position pooling + weighted group maximum (paper Eq. 6), and the
// enumeration of the positions that the fused utility form of the scan's second pass (ckv_scan.h) leaves
// to be finished from raw column sums -- the geometry constants both sides use are in ckv_internal.h.
#ifndef CKV_TABLES_H_
#define CKV_TABLES_H_
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
__device__ inline void write_budgets(const TablesArgs &a, int b) {
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

// What the fused utility form of the scan's second pass leaves out. That pass writes the utilities of the
// keys its pipeline takes (whole rounds of kRing * kTile keys at the front of every wave's key range)
// except the first four and the last kUtilShift of them (its output windows trail the rounds by that
// much so that its stores stay 128-byte aligned), and stores raw column sums only around those two
// places and for the tail of the range. fixup_range computes what is missing from the raw sums, for
// one wave range of one (batch, KV head): the four-key group at the front, the last kUtilShift / 4
// groups of the pipelined part, and every group of the tail. Thread tid of n_threads takes every
// n_threads-th group.
struct FixupArgs {
  int keys_per_wave, n_ranges;  // the scan's split of the key axis
};
// Groups of four positions that the fix-up computes in wave range `range`: n_edge at the edges of the
// pipelined part, then n_tail in the tail; group i starts at position group_start(i).
struct FixupRange {
  int t_begin, tail0, n_edge, n_tail;
  __device__ __forceinline__ FixupRange(const TablesArgs &a, const FixupArgs &f, int range) {
    constexpr int kBlockKeys = kRing * kTile;  // keys per pipeline round of the scan
    t_begin = range * f.keys_per_wave;
    const int t_end = min(t_begin + f.keys_per_wave, a.T);
    const int n_full = max(0, (min(t_end, a.P) - t_begin) / kTile);   // tiles wholly inside the prefix
    const int n_blocks = n_full / kRing;                               // pipeline rounds
    tail0 = t_begin + n_blocks * kBlockKeys;
    const int tail1 = min(t_end, a.P);
    n_tail = t_begin < a.T && tail1 > tail0 ? (tail1 - tail0 + 3) / 4 : 0;
    n_edge = t_begin < a.T && n_blocks > 0 ? 1 + kUtilShift / 4 : 0;
  }
  __device__ __forceinline__ int groups() const { return n_edge + n_tail; }
  __device__ __forceinline__ int group_start(int i) const {
    return i < n_edge ? (i == 0 ? t_begin : tail0 - kUtilShift + (i - 1) * 4) : tail0 + (i - n_edge) * 4;
  }
};

// One wave range, thread tid of n_threads taking every n_threads-th group.
template <int POOL, int R>
__device__ __forceinline__ void fixup_range(const TablesArgs &a, const FixupArgs &f, int unit, int range, int tid,
                                            int n_threads) {
  const FixupRange fr(a, f, range);
  for (int i = tid; i < fr.groups(); i += n_threads) pool_four<POOL, R>(a, unit, fr.group_start(i));
}

// Host side: the argument block for one call.
inline TablesArgs tables_args(const ckv_params *p, const Shape &s, const float *scores,
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

}  // namespace ckv
#endif
