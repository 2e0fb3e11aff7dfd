// Elastic candidate pool with budget clamp (paper Eq. 8, Alg. 1 Select) as a radix select.
//
// One 1024-thread workgroup per (batch, KV head). Utilities are non-negative floats, so their bit
// patterns order like unsigned integers. The kp-th largest candidate key is found MSB-first with an
// LDS histogram per pass (integer LDS atomics: the counts, and so the result, do not depend on
// scheduling). The final pass emits the kept positions in ascending order with ranks from prefix
// counts in position order. Equal keys at the threshold are taken lowest position first, which is
// exactly "utility descending, position ascending".
//
// Two kernels. select_reg_kernel (prefixes of up to 65536 positions, rows 16-byte aligned) reads the
// utilities once, with 128-bit loads, and keeps them in registers for all passes: digits of 11, 10
// and 10 bits, so the first one already splits the mantissa and same-address atomics stay rare.
// select_kernel streams the utilities from L2 in every pass (any length): digits of 8 bits.
#include "ckv_internal.h"

namespace ckv {

struct SelectArgs {
  const float *utility;   // [units][P]
  const int32_t *budget;  // [units]
  const float *tau;       // [Bz]
  int32_t *idx;           // [units][cap]
  int32_t *count;         // [units]
  int Hkv, T, W, P, cap;
};

__device__ __forceinline__ uint32_t key_of(float u) {
  const uint32_t bits = __builtin_bit_cast(uint32_t, u);
  return (bits & 0x80000000u) ? 0u : bits;  // -0.0 orders like +0.0
}

// Adds one count per active lane to hist[digit]. Utilities cluster in a few exponent bins, so plain
// per-lane LDS atomics would serialise on one address: the wave first elects up to three leaders
// whose digit is shared by many lanes and adds a popcount for each; stragglers use their own atomic.
// Every lane of the wave must call this (it uses ballots).
__device__ __forceinline__ void hist_add(int *hist, bool active, int digit, int lane) {
  unsigned long long rem = __ballot(active);
#pragma unroll
  for (int it = 0; it < 3; ++it) {
    if (rem == 0) break;
    const int leader = __ffsll((long long)rem) - 1;
    const int d = __shfl(digit, leader);
    const unsigned long long same = __ballot(active && digit == d);
    if (lane == leader) atomicAdd(&hist[d], __popcll(same));
    active = active && digit != d;
    rem &= ~same;
  }
  if (active) atomicAdd(&hist[digit], 1);
}

// Executed by wave 0. Scans hist[NB-1..0]; returns the bin where the running count first reaches k
// (1-based) and the count strictly above that bin, plus the grand total.
struct BinResult {
  int bin, above, total;
};
template <int NB>
__device__ __forceinline__ BinResult find_bin(const int *hist, int k, int lane) {
  constexpr int PER = NB / kWave;  // lane i owns bins NB-1-PER*i .. NB-PER*(i+1) (descending)
  int c[PER], sum = 0;
#pragma unroll
  for (int e = 0; e < PER; ++e) {
    c[e] = hist[NB - 1 - PER * lane - e];
    sum += c[e];
  }
  int incl = sum;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int up = __shfl_up(incl, o);
    if (lane >= o) incl += up;
  }
  BinResult r;
  r.total = __shfl(incl, 63);
  const int excl = incl - sum;
  const bool mine = excl < k && k <= incl;
  int bin = -1, above = 0;
  if (mine) {
    int run = excl;
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      if (bin < 0 && run + c[e] >= k) {
        bin = NB - 1 - PER * lane - e;
        above = run;
      }
      run += c[e];
    }
  }
  const unsigned long long who = __ballot(mine);
  const int src = who ? __ffsll((long long)who) - 1 : 0;
  r.bin = __shfl(bin, src);
  r.above = __shfl(above, src);
  if (!who) r.bin = -1;
  return r;
}

// ---------------------------------------------------------------------------------------------
// Register-resident select: thread tid holds positions 4 * (j * 1024 + tid) + e, j < NV, e < 4, as
// keys k' = candidate ? bits + 1 : 0 (so "not a candidate" sorts below every candidate).
// ---------------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(4))) float f32x4_sel;

// AGGREGATE: lanes that share a digit are counted with one atomic (hist_add). With digits this fine
// the plain atomics measured faster even in the first pass, where every candidate takes part.
template <int NV, int SHIFT, int BITS, bool AGGREGATE>
__device__ __forceinline__ void digit_histogram(int *hist, const uint32_t (&key)[NV][4], uint32_t prefix_hi,
                                                int lane) {
#pragma unroll
  for (int j = 0; j < NV; ++j) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t k = key[j][e];
      const bool active = k != 0u && (k >> (SHIFT + BITS)) == prefix_hi;
      const int digit = (int)((k >> SHIFT) & ((1u << BITS) - 1u));
      if (AGGREGATE) hist_add(hist, active, digit, lane);
      else if (active) atomicAdd(&hist[digit], 1);
    }
  }
}

// Scratch of ranked_write, in LDS.
template <int NV>
struct RankScratch {
  static constexpr int N = NV * (kSelectThreads / kWave);
  int wave_tot[N];             // per (block of 4096 positions, wave): kept-above count | equal count << 16
  int pre_gt[N + 1], pre_eq[N + 1];  // their exclusive prefixes, unpacked, then the totals
};
struct BlockTotals {
  int gt, eq;  // keys above / equal to the threshold among the workgroup's positions
};

// Writes the kept positions of the workgroup's NV * 4096 positions (thread tid holds positions
// t_base + 4 * (j * 1024 + tid) + e) in ascending order: every key above thr, and the first need_eq keys
// equal to it, at the rank they have among all kept positions. base_gt / base_eq count the keys above /
// equal that lie before t_base; ranks at or beyond kp are dropped. All threads of the workgroup call it.
template <int NV>
__device__ __forceinline__ BlockTotals ranked_write(const uint32_t (&key)[NV][4], uint32_t thr, int need_eq, int kp,
                                                    int base_gt, int base_eq, int t_base, int32_t *out,
                                                    RankScratch<NV> &rs, int tid, int lane, int wave) {
  constexpr int NW = kSelectThreads / kWave;
  int *wave_tot = rs.wave_tot, *pre_gt = rs.pre_gt, *pre_eq = rs.pre_eq;
  // Ranks in position order: block j, then wave, then lane, then element. A wave's counts come from the
  // lane masks of the comparisons themselves (population counts on the scalar unit, no cross-lane traffic);
  // they travel packed as (above | equal << 16): a wave covers 256 positions, so neither half overflows.
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    int c = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e)
      c += __popcll(__ballot(key[j][e] > thr)) + (__popcll(__ballot(key[j][e] == thr)) << 16);
    if (lane == 0) wave_tot[j * NW + wave] = c;
  }
  __syncthreads();
  // exclusive prefix over the (block, wave) totals in position order, by wave 0; the grand totals
  // end up behind the last entry
  if (wave == 0) {
    constexpr int PER = (NV * NW + kWave - 1) / kWave;
    int g[PER], q[PER], sg = 0, sq = 0;
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      const int i = lane * PER + e;
      const int c = i < NV * NW ? wave_tot[i] : 0;
      g[e] = c & 0xffff;
      q[e] = c >> 16;
      sg += g[e];
      sq += q[e];
    }
    int ig = sg, iq = sq;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int ug = __shfl_up(ig, o), uq = __shfl_up(iq, o);
      if (lane >= o) {
        ig += ug;
        iq += uq;
      }
    }
    int rg = ig - sg, rq = iq - sq;
#pragma unroll
    for (int e = 0; e < PER; ++e) {
      const int i = lane * PER + e;
      if (i < NV * NW) {
        pre_gt[i] = rg;
        pre_eq[i] = rq;
      }
      rg += g[e];
      rq += q[e];
    }
    if (lane == 63) {
      pre_gt[NV * NW] = ig;
      pre_eq[NV * NW] = iq;
    }
  }
  __syncthreads();
  const int tot_gt = pre_gt[NV * NW], tot_eq = pre_eq[NV * NW];
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    // kept keys above / equal in front of this lane's four: the blocks and waves before, then the lower
    // lanes of this wave (bits of the comparison masks below the lane, counted per element)
    uint32_t gt_before = (uint32_t)(base_gt + pre_gt[j * NW + wave]);
    uint32_t eq_before = (uint32_t)(base_eq + pre_eq[j * NW + wave]);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const unsigned long long mg = __ballot(key[j][e] > thr), me = __ballot(key[j][e] == thr);
      gt_before = __builtin_amdgcn_mbcnt_hi((uint32_t)(mg >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mg, gt_before));
      eq_before = __builtin_amdgcn_mbcnt_hi((uint32_t)(me >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)me, eq_before));
    }
    const int t = 4 * (j * kSelectThreads + tid);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const bool gt = key[j][e] > thr, eq = key[j][e] == thr;
      if (gt || (eq && (int)eq_before < need_eq)) {
        const int pos = (int)gt_before + min((int)eq_before, need_eq);
        if (pos < kp) out[pos] = t_base + t + e;
      }
      gt_before += gt;
      eq_before += eq;
    }
  }
  return BlockTotals{tot_gt, tot_eq};
}

template <int NV>
__global__ void __launch_bounds__(kSelectThreads) select_reg_kernel(SelectArgs a) {
  __shared__ int hist[2048 + 1024 + 1024];  // one histogram per digit, all cleared up front
  __shared__ RankScratch<NV> ranks;
  __shared__ uint32_t s_prefix;
  __shared__ int s_k, s_state;  // s_state: 0 = keep all candidates, 1 = select, 2 = keep none

  const int unit = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int P = a.P, W = a.W;
  const float *u = a.utility + (size_t)unit * P;
  const float tau = a.tau[unit / a.Hkv];
  int bud = a.budget[unit];
  bud = max(W, min(bud, min(a.cap, a.T)));
  const int kp = bud - W;

  uint32_t key[NV][4];
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const int t = 4 * (j * kSelectThreads + tid);
    f32x4_sel x = {-1.0f, -1.0f, -1.0f, -1.0f};
    if (t < P) x = *reinterpret_cast<const f32x4_sel *>(u + t);  // P % 4 == 0: whole vectors only
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float xe = x[e];
      key[j][e] = (t < P && xe >= tau) ? key_of(xe) + 1u : 0u;
    }
  }

  for (int i = tid; i < 4096; i += kSelectThreads) hist[i] = 0;
  __syncthreads();
  digit_histogram<NV, 20, 11, false>(hist, key, 0u, lane);
  __syncthreads();
  if (wave == 0) {
    const BinResult r = find_bin<2048>(hist, max(kp, 1), lane);
    if (lane == 0) {
      if (r.total <= kp) s_state = 0;
      else if (kp == 0) s_state = 2;
      else {
        s_state = 1;
        s_prefix = (uint32_t)r.bin;  // bits 30..20 of the threshold
        s_k = kp - r.above;          // still needed from inside the chosen bin
      }
    }
  }
  __syncthreads();
  const int state = s_state;
  uint32_t thr = 0u;  // keep-all: every candidate has k' > 0
  int need_eq = 0;    // how many keys equal to thr are kept
  if (state == 2) {
    thr = 0xffffffffu;
  } else if (state == 1) {
    {
      const uint32_t prefix = s_prefix;
      const int k = s_k;
      digit_histogram<NV, 10, 10, false>(hist + 2048, key, prefix, lane);
      __syncthreads();
      if (wave == 0) {
        const BinResult r = find_bin<1024>(hist + 2048, k, lane);
        if (lane == 0) {
          s_prefix = (prefix << 10) | (uint32_t)r.bin;
          s_k = k - r.above;
        }
      }
      __syncthreads();
    }
    {
      const uint32_t prefix = s_prefix;
      const int k = s_k;
      digit_histogram<NV, 0, 10, false>(hist + 3072, key, prefix, lane);
      __syncthreads();
      if (wave == 0) {
        const BinResult r = find_bin<1024>(hist + 3072, k, lane);
        if (lane == 0) {
          s_prefix = (prefix << 10) | (uint32_t)r.bin;
          s_k = k - r.above;
        }
      }
      __syncthreads();
    }
    thr = s_prefix;
    need_eq = s_k;
  }

  int32_t *out = a.idx + (size_t)unit * a.cap;
  const BlockTotals tot = ranked_write<NV>(key, thr, need_eq, kp, 0, 0, 0, out, ranks, tid, lane, wave);
  const int tot_gt = tot.gt, tot_eq = tot.eq;
  const int kept = min(tot_gt + min(tot_eq, need_eq), kp);
  for (int j = tid; j < W; j += kSelectThreads) out[kept + j] = P + j;
  if (tid == 0) a.count[unit] = kept + W;
}

// ---------------------------------------------------------------------------------------------
// Split select: prefixes beyond 32768 positions, when the caller passes a workspace. A unit's positions are cut into slices of 8192, one workgroup each, so that long contexts
// with few (batch, head) units still fill the chip. Five launches walk the same steps as the register
// kernel: three digit histograms (slices merge theirs into the unit's histogram in global memory with
// integer atomics: order-independent, so the result is deterministic), the slices' counts of keys above
// / equal to the threshold, and the ranked write. Every workgroup derives the threshold digits from
// the merged histograms itself (4096 integers per unit), which saves the launches in between.
// ---------------------------------------------------------------------------------------------
constexpr int kSplitNV = 2;
constexpr int kSplitSlice = kSplitNV * 4 * kSelectThreads;  // positions per workgroup
constexpr int kSplitHist = 2048 + 1024 + 1024;              // merged histogram words per unit

struct SplitArgs {
  SelectArgs a;
  int *hist;       // [units][kSplitHist], zero before the first phase
  int *slice_cnt;  // [units][S] keys above | equal << 16 of each slice
  int *thr;        // [units][4 phases][4] digits found so far, keys still needed, state
  int S;           // slices per unit
};

__global__ void __launch_bounds__(kSelectThreads) select_split_zero_kernel(int *words, int n) {
  const int i = blockIdx.x * kSelectThreads + threadIdx.x;
  if (i < n) words[i] = 0;
}

// PHASE 0..2: histogram of digit PHASE (11, 10, 10 bits from the top) among the keys that match the
// digits found so far. PHASE 3: per-slice counts and the unit's threshold. PHASE 4: ranked write.
template <int PHASE>
__global__ void __launch_bounds__(kSelectThreads) select_split_kernel(SplitArgs sa) {
  __shared__ int hist[2048];
  __shared__ RankScratch<kSplitNV> ranks;
  __shared__ uint32_t s_prefix;
  __shared__ int s_k, s_state;  // s_state: 0 = keep all candidates, 1 = select, 2 = keep none
  __shared__ int s_red[kSelectThreads / kWave];

  const SelectArgs &a = sa.a;
  const int unit = blockIdx.x / sa.S, slice = blockIdx.x % sa.S;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int P = a.P, W = a.W;
  const float *u = a.utility + (size_t)unit * P;
  const float tau = a.tau[unit / a.Hkv];
  int bud = a.budget[unit];
  bud = max(W, min(bud, min(a.cap, a.T)));
  const int kp = bud - W;
  const int t_base = slice * kSplitSlice;
  int *gh = sa.hist + (size_t)unit * kSplitHist;

  uint32_t key[kSplitNV][4];
#pragma unroll
  for (int j = 0; j < kSplitNV; ++j) {
    const int t = t_base + 4 * (j * kSelectThreads + tid);
    f32x4_sel x = {-1.0f, -1.0f, -1.0f, -1.0f};
    if (t < P) x = *reinterpret_cast<const f32x4_sel *>(u + t);  // P % 4 == 0: whole vectors only
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float xe = x[e];
      key[j][e] = (t < P && xe >= tau) ? key_of(xe) + 1u : 0u;
    }
  }

  // Threshold digits: phase p finds digit p - 1 from the histogram that phase p - 1 merged (the same
  // arithmetic in every workgroup of the unit) and takes the digits before it from the record that
  // the previous phase's first slice left; records are per phase, so no workgroup reads one that is
  // being written in its own launch.
  int state = 1, k = max(kp, 1);
  uint32_t prefix = 0u;
  int *rec = sa.thr + (size_t)unit * 16;  // [phase][prefix, k, state, -]
  if constexpr (PHASE >= 2) {
    prefix = (uint32_t)rec[4 * (PHASE - 1) + 0];
    k = rec[4 * (PHASE - 1) + 1];
    state = rec[4 * (PHASE - 1) + 2];
  }
  if constexpr (PHASE == 1) {
    for (int i = tid; i < 2048; i += kSelectThreads) hist[i] = gh[i];
    __syncthreads();
    if (wave == 0) {
      const BinResult r = find_bin<2048>(hist, max(kp, 1), lane);
      if (lane == 0) {
        s_prefix = (uint32_t)max(r.bin, 0);
        s_k = kp - r.above;
        s_state = r.total <= kp ? 0 : (kp == 0 ? 2 : 1);
      }
    }
    __syncthreads();
    state = s_state;
    prefix = s_prefix;
    k = s_k;
  }
  if constexpr (PHASE == 2 || PHASE == 3) {
    if (state == 1) {
      hist[tid] = gh[2048 + 1024 * (PHASE - 2) + tid];
      __syncthreads();
      if (wave == 0) {
        const BinResult r = find_bin<1024>(hist, k, lane);
        if (lane == 0) {
          s_prefix = (prefix << 10) | (uint32_t)r.bin;
          s_k = k - r.above;
        }
      }
      __syncthreads();
      prefix = s_prefix;
      k = s_k;
    }
  }
  if constexpr (PHASE >= 1 && PHASE <= 3) {
    if (slice == 0 && tid == 0) {
      rec[4 * PHASE + 0] = (int)prefix;
      rec[4 * PHASE + 1] = k;
      rec[4 * PHASE + 2] = state;
    }
  }

  if constexpr (PHASE <= 2) {
    if (PHASE > 0 && state != 1) return;
    constexpr int NB = PHASE == 0 ? 2048 : 1024;
    __syncthreads();
    for (int i = tid; i < NB; i += kSelectThreads) hist[i] = 0;
    __syncthreads();
    digit_histogram<kSplitNV, 20 - 10 * PHASE, PHASE == 0 ? 11 : 10, false>(hist, key, prefix, lane);
    __syncthreads();
    int *g = gh + (PHASE == 0 ? 0 : 2048 + 1024 * (PHASE - 1));
    for (int i = tid; i < NB; i += kSelectThreads) {
      const int h = hist[i];
      if (h) atomicAdd(&g[i], h);
    }
    return;
  }

  if constexpr (PHASE == 3) {
    uint32_t thr = 0u;  // keep-all: every candidate has k' > 0
    if (state == 2) thr = 0xffffffffu;
    else if (state == 1) thr = prefix;
    int c = 0;
#pragma unroll
    for (int j = 0; j < kSplitNV; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) c += (key[j][e] > thr ? 1 : 0) + (key[j][e] == thr ? 0x10000 : 0);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) c += __shfl_xor(c, o);  // 256 positions a wave: neither half overflows
    if (lane == 0) s_red[wave] = c;
    __syncthreads();
    if (tid == 0) {
      int tot = 0;  // 8192 positions a slice: neither half overflows
      for (int w = 0; w < kSelectThreads / kWave; ++w) tot += s_red[w];
      sa.slice_cnt[(size_t)unit * sa.S + slice] = tot;
    }
    return;
  }

  if constexpr (PHASE == 4) {
    uint32_t thr = 0u;  // as in phase 3, from its record
    int need_eq = 0;
    if (state == 2) thr = 0xffffffffu;
    else if (state == 1) {
      thr = prefix;
      need_eq = k;
    }
    int base_gt = 0, base_eq = 0, all_gt = 0, all_eq = 0;
    for (int i = 0; i < sa.S; ++i) {  // same address in every lane: one broadcast load each
      const int c = sa.slice_cnt[(size_t)unit * sa.S + i];
      if (i < slice) {
        base_gt += c & 0xffff;
        base_eq += c >> 16;
      }
      all_gt += c & 0xffff;
      all_eq += c >> 16;
    }
    int32_t *out = a.idx + (size_t)unit * a.cap;
    ranked_write<kSplitNV>(key, thr, need_eq, kp, base_gt, base_eq, t_base, out, ranks, tid, lane, wave);
    if (slice == 0) {
      const int kept = min(all_gt + min(all_eq, need_eq), kp);
      for (int j = tid; j < W; j += kSelectThreads) out[kept + j] = P + j;
      if (tid == 0) a.count[unit] = kept + W;
    }
  }
}

size_t select_workspace_bytes(const Shape &s) {
  // up to 32768 positions the register kernel (one workgroup per unit, one launch) is the faster one
  if (s.P <= 8 * 4 * kSelectThreads || s.P % 4 != 0) return 0;
  const size_t units = (size_t)s.Bz * s.Hkv, S = (s.P + kSplitSlice - 1) / kSplitSlice;
  return units * (kSplitHist + S + 16) * sizeof(int);
}

// ---------------------------------------------------------------------------------------------
// Streaming select: any length.
// ---------------------------------------------------------------------------------------------
constexpr int kUnroll = 8;

__global__ void __launch_bounds__(kSelectThreads) select_kernel(SelectArgs a) {
  __shared__ int hist[256];
  __shared__ int wave_gt[kSelectThreads / kWave], wave_eq[kSelectThreads / kWave];
  __shared__ uint32_t s_prefix;
  __shared__ int s_k, s_state;  // s_state: 0 = keep all candidates, 1 = select, 2 = keep none

  const int unit = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int P = a.P, W = a.W;
  const float *u = a.utility + (size_t)unit * P;
  const float tau = a.tau[unit / a.Hkv];
  int bud = a.budget[unit];
  bud = max(W, min(bud, min(a.cap, a.T)));
  const int kp = bud - W;

  // pass 0: histogram of the top byte over the candidates (also counts them)
  if (tid < 256) hist[tid] = 0;
  __syncthreads();
  // eight loads in flight per thread: the pass is bound by L2 latency, not by arithmetic
  for (int t0 = 0; t0 < P; t0 += kUnroll * kSelectThreads) {
    float x[kUnroll];
#pragma unroll
    for (int e = 0; e < kUnroll; ++e) {
      const int t = t0 + e * kSelectThreads + tid;
      x[e] = t < P ? u[t] : -INFINITY;  // never a candidate
    }
#pragma unroll
    for (int e = 0; e < kUnroll; ++e) hist_add(hist, x[e] >= tau, (int)(key_of(x[e]) >> 24), lane);
  }
  __syncthreads();
  if (wave == 0) {
    const BinResult r = find_bin<256>(hist, max(kp, 1), lane);
    if (lane == 0) {
      if (r.total <= kp) s_state = 0;
      else if (kp == 0) s_state = 2;
      else {
        s_state = 1;
        s_prefix = (uint32_t)r.bin << 24;
        s_k = kp - r.above;  // still needed from inside the chosen bin
      }
    }
  }
  __syncthreads();
  const int state = s_state;

  uint32_t thr = 0u;   // keep-all: every candidate has key > 0 or ties at 0 with unlimited quota
  int need_eq = 0x7fffffff;
  if (state == 2) {
    thr = 0xffffffffu;
    need_eq = 0;
  } else if (state == 1) {
    for (int shift = 16; shift >= 0; shift -= 8) {
      const uint32_t prefix = s_prefix;
      const int k = s_k;
      if (tid < 256) hist[tid] = 0;
      __syncthreads();
      const uint32_t hi_mask = 0xffffffffu << (shift + 8);
      for (int t0 = 0; t0 < P; t0 += kUnroll * kSelectThreads) {
        float x[kUnroll];
#pragma unroll
        for (int e = 0; e < kUnroll; ++e) {
          const int t = t0 + e * kSelectThreads + tid;
          x[e] = t < P ? u[t] : -INFINITY;
        }
#pragma unroll
        for (int e = 0; e < kUnroll; ++e) {
          const uint32_t key = key_of(x[e]);
          hist_add(hist, x[e] >= tau && (key & hi_mask) == prefix, (int)((key >> shift) & 255u), lane);
        }
      }
      __syncthreads();
      if (wave == 0) {
        const BinResult r = find_bin<256>(hist, k, lane);
        if (lane == 0) {
          s_prefix = prefix | ((uint32_t)r.bin << shift);
          s_k = k - r.above;
        }
      }
      __syncthreads();
    }
    thr = s_prefix;
    need_eq = s_k;  // how many keys equal to thr are kept (>= 1)
  }

  // Final pass. Wave w owns positions [w*seg, (w+1)*seg); seg is a multiple of 64.
  const int n_waves = kSelectThreads / kWave;
  const int seg = ((P + n_waves - 1) / n_waves + kWave - 1) / kWave * kWave;
  const int lo = wave * seg, hi = min(lo + seg, P);
  int n_gt = 0, n_eq = 0;
  for (int t0 = lo; t0 < hi; t0 += kUnroll * kWave) {
    float x[kUnroll];
#pragma unroll
    for (int e = 0; e < kUnroll; ++e) {
      const int t = t0 + e * kWave + lane;
      x[e] = t < hi ? u[t] : -INFINITY;
    }
#pragma unroll
    for (int e = 0; e < kUnroll; ++e) {
      const uint32_t key = key_of(x[e]);
      const bool cand = x[e] >= tau;
      n_gt += __popcll(__ballot(cand && key > thr));
      n_eq += __popcll(__ballot(cand && key == thr));
    }
  }
  if (lane == 0) {
    wave_gt[wave] = n_gt;
    wave_eq[wave] = n_eq;
  }
  __syncthreads();
  int base_gt = 0, base_eq = 0;
  for (int w = 0; w < wave; ++w) {
    base_gt += wave_gt[w];
    base_eq += wave_eq[w];
  }
  int32_t *out = a.idx + (size_t)unit * a.cap;
  const unsigned long long below = (1ull << lane) - 1ull;
  for (int t0 = lo; t0 < hi; t0 += kUnroll * kWave) {
    float x[kUnroll];
#pragma unroll
    for (int e = 0; e < kUnroll; ++e) {
      const int t = t0 + e * kWave + lane;
      x[e] = t < hi ? u[t] : -INFINITY;
    }
#pragma unroll
    for (int e = 0; e < kUnroll; ++e) {
      const uint32_t key = key_of(x[e]);
      const bool cand = x[e] >= tau;
      const bool gt = cand && key > thr, eq = cand && key == thr;
      const unsigned long long bg = __ballot(gt), be = __ballot(eq);
      const int gt_before = base_gt + __popcll(bg & below);
      const int eq_before = base_eq + __popcll(be & below);
      if (gt || (eq && eq_before < need_eq)) {
        const int pos = gt_before + min(eq_before, need_eq);
        if (pos < kp) out[pos] = t0 + e * kWave + lane;
      }
      base_gt += __popcll(bg);
      base_eq += __popcll(be);
    }
  }
  // kept prefix tokens, then the window
  __syncthreads();
  int tot_gt = 0, tot_eq = 0;
  for (int w = 0; w < n_waves; ++w) {
    tot_gt += wave_gt[w];
    tot_eq += wave_eq[w];
  }
  const int kept = min(tot_gt + min(tot_eq, need_eq), kp);
  for (int j = tid; j < W; j += kSelectThreads) out[kept + j] = P + j;
  if (tid == 0) a.count[unit] = kept + W;
}

hipError_t launch_select(const ckv_params *p, const Shape &s, const float *utility,
                         const int32_t *budget, const float *tau, int32_t *idx, int32_t *count,
                         char *ws, hipStream_t stream) {
  SelectArgs a;
  a.utility = utility;
  a.budget = budget;
  a.tau = tau;
  a.idx = idx;
  a.count = count;
  a.Hkv = s.Hkv; a.T = s.T; a.W = s.W; a.P = s.P;
  a.cap = p->cap;
  const dim3 grid(s.Bz * s.Hkv), block(kSelectThreads);
  const int vectors = (s.P + 4 * kSelectThreads - 1) / (4 * kSelectThreads);  // 128-bit loads per thread
  const bool aligned = s.P % 4 == 0 && (uintptr_t)utility % 16 == 0 && s.P > 0;
  const bool split = aligned && ws && select_workspace_bytes(s) > 0;
  if (split) {
    SplitArgs sa;
    sa.a = a;
    sa.S = (s.P + kSplitSlice - 1) / kSplitSlice;
    const size_t units = (size_t)s.Bz * s.Hkv;
    sa.hist = reinterpret_cast<int *>(ws);
    sa.slice_cnt = sa.hist + units * kSplitHist;
    sa.thr = sa.slice_cnt + units * sa.S;
    const int n_zero = (int)(units * kSplitHist);
    const dim3 split_grid((unsigned)(units * sa.S));
    hipLaunchKernelGGL(select_split_zero_kernel, dim3((n_zero + kSelectThreads - 1) / kSelectThreads), block, 0,
                       stream, sa.hist, n_zero);
    hipLaunchKernelGGL(select_split_kernel<0>, split_grid, block, 0, stream, sa);
    hipLaunchKernelGGL(select_split_kernel<1>, split_grid, block, 0, stream, sa);
    hipLaunchKernelGGL(select_split_kernel<2>, split_grid, block, 0, stream, sa);
    hipLaunchKernelGGL(select_split_kernel<3>, split_grid, block, 0, stream, sa);
    hipLaunchKernelGGL(select_split_kernel<4>, split_grid, block, 0, stream, sa);
  } else if (aligned && vectors <= 1) hipLaunchKernelGGL(select_reg_kernel<1>, grid, block, 0, stream, a);
  else if (aligned && vectors <= 2) hipLaunchKernelGGL(select_reg_kernel<2>, grid, block, 0, stream, a);
  else if (aligned && vectors <= 4) hipLaunchKernelGGL(select_reg_kernel<4>, grid, block, 0, stream, a);
  else if (aligned && vectors <= 8) hipLaunchKernelGGL(select_reg_kernel<8>, grid, block, 0, stream, a);
  else if (aligned && vectors <= 16) hipLaunchKernelGGL(select_reg_kernel<16>, grid, block, 0, stream, a);
  else hipLaunchKernelGGL(select_kernel, grid, block, 0, stream, a);
  return hipGetLastError();
}

}  // namespace ckv
