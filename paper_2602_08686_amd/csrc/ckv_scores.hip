// Observation-window scan (paper Sec. 3 attention definition, Eq. 3, Eq. 4's alpha per query head):
//   pass 1  rowstats kernels : stream K, QK^T on the matrix cores, online (max, sum) per window row
//           lse_kernel       : merge the per-chunk partials into LSE_j
//   pass 2  colsum kernels   : stream K again, recompute QK^T, exp(z - LSE_j), sum over window rows
// plus the value-norm ratio rho of Eq. 4 (two small kernels).
//
// Work decomposition. A "unit" is one (batch, KV head): its G*W window query rows all contract with
// the same K. Rows are cut into 32-row tiles (one MFMA 32x32 edge), whole heads only; a wave keeps up
// to four tiles of Q in registers for its lifetime and streams 32-key tiles of K straight from
// global memory into MFMA operand layout: lane (m, hh) = (lane % 32, lane / 32) owns row m of a tile
// and the 16-byte chunks 2c+hh of that row. The contraction index may be permuted freely as long as
// both operands use the same permutation, so whole 16-byte chunks become MFMA k-groups and no LDS
// transpose is needed. The four waves of a workgroup sweep four adjacent key ranges.
//
// The two passes use opposite operand orders on purpose:
//   pass 1: D = K Q^T, lane <-> query row: the running (max, sum) of a row never leaves its lane;
//   pass 2: D = Q K^T, lane <-> key: the sum over window rows is 16 in-lane adds and one half swap.
//
// Two families of kernels: plain ones for every shape (two waves per SIMD, one accumulator set), and
// software-pipelined ones for bf16 with an even number of query tiles per wave (the GQA shapes).
#include "ckv_internal.h"

namespace ckv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t chunk_t;  // 16 bytes of one Q or K row

struct ScoreArgs {
  const char *q, *k;
  int64_t qs_b, qs_h, qs_w;  // byte strides
  int64_t ks_b, ks_h, ks_t;
  int Hq, Hkv, G, T, W, P;
  int WT, n_tiles, n_groups, keys_per_wave, n_chunks;
  float c2;     // softmax scale * log2(e): logits are kept in the log2 domain
  float norm;   // T / W
  float2 *part;      // [unit][group][NQ*32][n_chunks] (max, sum) in the log2 domain
  const float *lse;  // [Bz][Hq][W] natural log
  float *lse_out;
  float *scores;     // [Bz][Hq][T]
};

template <int DT> struct Mma;
template <> struct Mma<CKV_BF16> {
  static __device__ __forceinline__ void step(f32x16 &acc, const chunk_t &a, const chunk_t &b) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                  __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
  }
};
template <> struct Mma<CKV_F32> {
  static __device__ __forceinline__ void step(f32x16 &acc, const chunk_t &a, const chunk_t &b) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      // copy the lanes out first: a bit_cast applied directly to a vector element reads element 0
      const uint32_t ua = a[e], ub = b[e];
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(ua), __uint_as_float(ub), acc, 0, 0, 0);
    }
  }
};

// acc = sum over the row's chunks of a[c] . b[c]  (a: the 32 rows of D, b: the 32 columns of D)
template <int DT, int NCH>
__device__ __forceinline__ void mma_chain(f32x16 &acc, const chunk_t (&a)[NCH], const chunk_t (&b)[NCH]) {
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
#pragma unroll
  for (int c = 0; c < NCH; ++c) Mma<DT>::step(acc, a[c], b[c]);
}

// Row of the 32x32 accumulator that element r of lane (m, hh) holds; its column is m.
__device__ __forceinline__ int acc_row(int r, int hh) { return 8 * (r >> 2) + 4 * hh + (r & 3); }

__device__ __forceinline__ void merge_stats(float &m, float &l, float om, float ol) {
  const float mn = fmaxf(m, om);
  l = l * __builtin_amdgcn_exp2f(m - mn) + ol * __builtin_amdgcn_exp2f(om - mn);
  m = mn;
}

template <int NCH>
__device__ __forceinline__ void load_row(chunk_t (&f)[NCH], const char *row, int hh) {
#pragma unroll
  for (int c = 0; c < NCH; ++c) f[c] = *reinterpret_cast<const chunk_t *>(row + (2 * c + hh) * 16);
}

struct BlockCoord {
  int chunk, grp, unit, b, g;
};
__device__ __forceinline__ BlockCoord decode_block(const ScoreArgs &a) {
  BlockCoord c;
  int bid = blockIdx.x;
  c.chunk = bid % a.n_chunks;
  bid /= a.n_chunks;
  c.grp = bid % a.n_groups;
  c.unit = bid / a.n_groups;
  c.b = c.unit / a.Hkv;
  c.g = c.unit % a.Hkv;
  return c;
}

// Loads this lane's rows of the group's NQ query tiles; jrow[i] = window row index of tile i, row m
// (or -1 where the tile or the row is padding).
template <int NCH, int NQ>
__device__ __forceinline__ void load_q_tiles(const ScoreArgs &a, const BlockCoord &bc, int m, int hh,
                                             chunk_t (&qf)[NQ][NCH], int (&jrow)[NQ]) {
#pragma unroll
  for (int i = 0; i < NQ; ++i) {
    const int tile = bc.grp * NQ + i;
    const int j = (tile % a.WT) * kTile + m;
    const bool valid = tile < a.n_tiles && j < a.W;
    jrow[i] = valid ? j : -1;
    if (valid) {
      const int h = bc.g * a.G + tile / a.WT;
      load_row<NCH>(qf[i], a.q + bc.b * a.qs_b + h * a.qs_h + j * a.qs_w, hh);
    } else {
#pragma unroll
      for (int c = 0; c < NCH; ++c) qf[i][c] = chunk_t{0u, 0u, 0u, 0u};
    }
  }
}

// Pass 1, vector part: online (max, sum) update of this lane's query row with the 16 logits it holds
// of one tile. The maximum is taken on the raw dot products (the scale is positive); scale and
// subtraction are one FMA per element.
template <bool EDGE>
__device__ __forceinline__ void rowstats_update(const f32x16 &acc, float c2, int t0, int hh, int limit,
                                                float &rm, float &rl) {
  float v[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) v[r] = acc[r];
  if (EDGE) {
#pragma unroll
    for (int r = 0; r < 16; ++r)
      if (t0 + acc_row(r, hh) > limit) v[r] = -INFINITY;
  }
  float t[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) t[e] = fmaxf(fmaxf(v[4 * e], v[4 * e + 1]), fmaxf(v[4 * e + 2], v[4 * e + 3]));
  const float tmax = fmaxf(fmaxf(t[0], t[1]), fmaxf(t[2], t[3]));
  const float mn = fmaxf(rm, tmax * c2);
  float s[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
  for (int r = 0; r < 16; ++r) s[r & 3] += __builtin_amdgcn_exp2f(fmaf(v[r], c2, -mn));
  rl = fmaf(rl, __builtin_amdgcn_exp2f(rm - mn), (s[0] + s[1]) + (s[2] + s[3]));
  rm = mn;
}

// Merges the (max, sum) pairs of the two half-waves and of the workgroup's waves, one partial per chunk.
template <int NQ>
__device__ __forceinline__ void store_row_partials(const ScoreArgs &a, const BlockCoord &bc, int wave, int m,
                                                   int hh, float (&rm)[NQ], float (&rl)[NQ]) {
  __shared__ float2 sm[kScoreWaves][NQ * kTile];
#pragma unroll
  for (int i = 0; i < NQ; ++i) {
    const float om = __shfl_xor(rm[i], 32), ol = __shfl_xor(rl[i], 32);
    merge_stats(rm[i], rl[i], om, ol);
    if (hh == 0) sm[wave][i * kTile + m] = make_float2(rm[i], rl[i]);
  }
  __syncthreads();
  if (threadIdx.x < NQ * kTile) {
    float2 s = sm[0][threadIdx.x];
#pragma unroll
    for (int w = 1; w < kScoreWaves; ++w) merge_stats(s.x, s.y, sm[w][threadIdx.x].x, sm[w][threadIdx.x].y);
    const size_t row = ((size_t)bc.unit * a.n_groups + bc.grp) * (NQ * kTile) + threadIdx.x;
    a.part[row * a.n_chunks + bc.chunk] = s;
  }
}

// ---------------------------------------------------------------------------------------------
// Plain kernels: every dtype / tile count. Two waves per SIMD, K double-buffered in registers.
// ---------------------------------------------------------------------------------------------
template <int DT, int DH, int NQ>
__global__ void __launch_bounds__(kScoreWaves *kWave, 2) rowstats_kernel(ScoreArgs a) {
  constexpr int NCH = DH * (DT == CKV_BF16 ? 2 : 4) / 32;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, m = lane & 31, hh = lane >> 5;
  const BlockCoord bc = decode_block(a);

  chunk_t qf[NQ][NCH];
  int jrow[NQ], limit[NQ];
  load_q_tiles<NCH, NQ>(a, bc, m, hh, qf, jrow);
  float rm[NQ], rl[NQ];
#pragma unroll
  for (int i = 0; i < NQ; ++i) {
    limit[i] = jrow[i] < 0 ? -1 : a.P + jrow[i];  // last key this row may see (causal)
    rm[i] = -1e30f;
    rl[i] = 0.0f;
  }

  const char *kbase = a.k + bc.b * a.ks_b + bc.g * a.ks_h;
  const int t_begin = (bc.chunk * kScoreWaves + wave) * a.keys_per_wave;
  const int t_end = min(t_begin + a.keys_per_wave, a.T);
  auto tile_body = [&](const chunk_t (&kf)[NCH], int t0) {
    f32x16 acc;
    if (t0 + kTile > a.P) {  // the tile touches the window (causal mask) or the end of the keys
#pragma unroll
      for (int i = 0; i < NQ; ++i) {
        mma_chain<DT, NCH>(acc, kf, qf[i]);  // rows: keys, cols: query rows
        rowstats_update<true>(acc, a.c2, t0, hh, limit[i], rm[i], rl[i]);
      }
    } else {
#pragma unroll
      for (int i = 0; i < NQ; ++i) {
        mma_chain<DT, NCH>(acc, kf, qf[i]);
        rowstats_update<false>(acc, a.c2, t0, hh, limit[i], rm[i], rl[i]);
      }
    }
  };
  // two K tiles in registers, used alternately: one is computed on while the other is in flight
  chunk_t ka[NCH], kb[NCH];
  if (t_begin < t_end) load_row<NCH>(ka, kbase + (int64_t)min(t_begin + m, a.T - 1) * a.ks_t, hh);
  for (int t0 = t_begin; t0 < t_end; t0 += 2 * kTile) {
    load_row<NCH>(kb, kbase + (int64_t)min(t0 + kTile + m, a.T - 1) * a.ks_t, hh);
    tile_body(ka, t0);
    if (t0 + kTile >= t_end) break;
    load_row<NCH>(ka, kbase + (int64_t)min(t0 + 2 * kTile + m, a.T - 1) * a.ks_t, hh);
    tile_body(kb, t0 + kTile);
  }
  store_row_partials<NQ>(a, bc, wave, m, hh, rm, rl);
}

// One thread per (unit, group, tile row): LSE_j = ln2 * (M + log2 sum_c l_c 2^(m_c - M)).
__global__ void lse_kernel(ScoreArgs a, int NQ, int n_rows_total) {
  const int row = blockIdx.x * blockDim.x + threadIdx.x;
  if (row >= n_rows_total) return;
  const int per_group = NQ * kTile;
  const int in_group = row % per_group;
  const int grp = (row / per_group) % a.n_groups;
  const int unit = row / (per_group * a.n_groups);
  const int tile = grp * NQ + in_group / kTile;
  const int j = (tile % a.WT) * kTile + in_group % kTile;
  if (tile >= a.n_tiles || j >= a.W) return;
  const float2 *p = a.part + (size_t)row * a.n_chunks;
  float M = -1e30f;
  for (int c = 0; c < a.n_chunks; ++c) M = fmaxf(M, p[c].x);
  float L = 0.0f;
  for (int c = 0; c < a.n_chunks; ++c) L += p[c].y * __builtin_amdgcn_exp2f(p[c].x - M);
  const int b = unit / a.Hkv, g = unit % a.Hkv, h = g * a.G + tile / a.WT;
  a.lse_out[((size_t)b * a.Hq + h) * a.W + j] = (M + __log2f(L)) * kLn2;
}

// One 32-row x 32-key tile of pass 2 for the plain kernel. The accumulator starts at -LSE_row / scale
// (read from LDS before the MFMA chain, so the LDS latency hides behind it), the chain adds <q, k>, and
// the weight is exp2(c2 * acc) = exp(z - LSE). Returns this lane's sum over its 16 rows.
template <int DT, int NCH, bool EDGE>
__device__ __forceinline__ float colsum_tile(const chunk_t (&qf)[NCH], const chunk_t (&kf)[NCH], float c2,
                                             const float *init_tile, int hh, int first_masked_row) {
  f32x16 acc;
#pragma unroll
  for (int q4 = 0; q4 < 4; ++q4) {
    const f32x4 ini = *reinterpret_cast<const f32x4 *>(init_tile + 8 * q4 + 4 * hh);
#pragma unroll
    for (int e = 0; e < 4; ++e) acc[4 * q4 + e] = ini[e];
  }
#pragma unroll
  for (int c = 0; c < NCH; ++c) Mma<DT>::step(acc, qf[c], kf[c]);  // rows: query rows, cols: keys
  float s[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    float pr = __builtin_amdgcn_exp2f(acc[r] * c2);
    // causal: key kt is visible to window row j iff kt <= P + j, i.e. tile row >= kt - P - j0
    if (EDGE && acc_row(r, hh) < first_masked_row) pr = 0.0f;
    s[r & 3] += pr;
  }
  return (s[0] + s[1]) + (s[2] + s[3]);
}

template <int DT, int DH, int NQ>
__global__ void __launch_bounds__(kScoreWaves *kWave, 2) colsum_kernel(ScoreArgs a) {
  constexpr int NCH = DH * (DT == CKV_BF16 ? 2 : 4) / 32;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, m = lane & 31, hh = lane >> 5;
  const BlockCoord bc = decode_block(a);

  // accumulator start value -LSE / scale of every row of the group's tiles; -inf on padding rows so
  // that their weights come out as exp2(-inf) = 0
  __shared__ __attribute__((aligned(16))) float s_init[NQ * kTile];
  if (threadIdx.x < NQ * kTile) {
    const int tile = bc.grp * NQ + threadIdx.x / kTile;
    const int j = (tile % a.WT) * kTile + threadIdx.x % kTile;
    const int h = bc.g * a.G + tile / a.WT;
    const bool valid = tile < a.n_tiles && j < a.W;
    s_init[threadIdx.x] = valid ? -a.lse[((size_t)bc.b * a.Hq + h) * a.W + j] * (kLog2e / a.c2) : -INFINITY;
  }
  chunk_t qf[NQ][NCH];
  int jrow[NQ];
  load_q_tiles<NCH, NQ>(a, bc, m, hh, qf, jrow);
  __syncthreads();

  const char *kbase = a.k + bc.b * a.ks_b + bc.g * a.ks_h;
  const int t_begin = (bc.chunk * kScoreWaves + wave) * a.keys_per_wave;
  const int t_end = min(t_begin + a.keys_per_wave, a.T);

  auto tile_body = [&](const chunk_t (&kf)[NCH], int t0) {
    const int kt = t0 + m;  // this lane's key
    float cs[NQ];
    if (t0 + kTile > a.P) {
#pragma unroll
      for (int i = 0; i < NQ; ++i) {
        const int j0 = ((bc.grp * NQ + i) % a.WT) * kTile;
        cs[i] = colsum_tile<DT, NCH, true>(qf[i], kf, a.c2, s_init + i * kTile, hh, kt - a.P - j0);
      }
    } else {
#pragma unroll
      for (int i = 0; i < NQ; ++i) cs[i] = colsum_tile<DT, NCH, false>(qf[i], kf, a.c2, s_init + i * kTile, hh, 0);
    }
    // the other half-wave holds the other 16 rows of each tile: swap and add (all swaps in flight together)
    float other[NQ];
#pragma unroll
    for (int i = 0; i < NQ; ++i) other[i] = __shfl_xor(cs[i], 32);
#pragma unroll
    for (int i = 0; i < NQ; ++i) cs[i] += other[i];
    // one output per head: add the tiles of a head (WT of them), scale by T/W, lanes 0..31 store
#pragma unroll
    for (int i = 0; i < NQ; ++i) {
      if (i % a.WT) continue;
      float v = cs[i];
#pragma unroll
      for (int e = 1; e < kMaxQTiles; ++e)
        if (e < a.WT && i + e < NQ) v += cs[(i + e) < NQ ? (i + e) : i];
      const int tile = bc.grp * NQ + i;
      if (tile < a.n_tiles && hh == 0 && kt < a.T) {
        const int h = bc.g * a.G + tile / a.WT;
        a.scores[((size_t)bc.b * a.Hq + h) * a.T + kt] = v * a.norm;
      }
    }
  };

  chunk_t ka[NCH], kb[NCH];
  if (t_begin < t_end) load_row<NCH>(ka, kbase + (int64_t)min(t_begin + m, a.T - 1) * a.ks_t, hh);
  for (int t0 = t_begin; t0 < t_end; t0 += 2 * kTile) {
    load_row<NCH>(kb, kbase + (int64_t)min(t0 + kTile + m, a.T - 1) * a.ks_t, hh);
    tile_body(ka, t0);
    if (t0 + kTile >= t_end) break;
    load_row<NCH>(ka, kbase + (int64_t)min(t0 + 2 * kTile + m, a.T - 1) * a.ks_t, hh);
    tile_body(kb, t0 + kTile);
  }
}

// ---------------------------------------------------------------------------------------------
// Software-pipelined kernels (bf16, even tile count NQ, WT tiles per head). One wave per SIMD runs a
// two-stage pipeline over (key tile, query tile) pairs: the MFMA chain of pair p+1 is issued in
// between the vector instructions that consume pair p's logits (two accumulator sets; scheduling
// hints place one MFMA in front of every few vector instructions), and K is prefetched D-1 tiles
// ahead. Tiles that touch the window or the end of the keys are handled after the pipeline, masked.
// ---------------------------------------------------------------------------------------------
constexpr int kPrefetchTiles = 4;

template <int N_MFMA, int VALU_PER>
__device__ __forceinline__ void interleave_hint() {
#pragma unroll
  for (int u = 0; u < N_MFMA; ++u) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);         // one MFMA
    __builtin_amdgcn_sched_group_barrier(0x002, VALU_PER, 0);  // then a few vector instructions
  }
}

// Geometry shared by both pipelined kernels: wave-uniform values live in scalar registers.
struct WaveRange {
  int wave, t_begin, t_end, n_full;
};
__device__ __forceinline__ WaveRange wave_range(const ScoreArgs &a, const BlockCoord &bc) {
  WaveRange r;
  r.wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  r.t_begin = (bc.chunk * kScoreWaves + r.wave) * a.keys_per_wave;
  r.t_end = min(r.t_begin + a.keys_per_wave, a.T);
  r.n_full = max(0, (min(r.t_end, a.P) - r.t_begin) / kTile);  // tiles wholly inside the prefix
  return r;
}

template <int DT, int DH, int NQ>
__global__ void __launch_bounds__(kScoreWaves *kWave) rowstats_pipe_kernel(ScoreArgs a) {
  static_assert(NQ % 2 == 0, "accumulator parity is static only for an even tile count");
  constexpr int NCH = DH * (DT == CKV_BF16 ? 2 : 4) / 32;
  constexpr int N_MFMA = NCH * (DT == CKV_BF16 ? 1 : 4);
  constexpr int D = kPrefetchTiles;
  const int lane = threadIdx.x & 63, m = lane & 31, hh = lane >> 5;
  const BlockCoord bc = decode_block(a);
  const WaveRange wr = wave_range(a, bc);

  const char *kbase = a.k + bc.b * a.ks_b + bc.g * a.ks_h;
  const char *klane = kbase + (int64_t)(wr.t_begin + m) * a.ks_t;  // this lane's row of the wave's tile 0
  const int64_t tile_stride = (int64_t)kTile * a.ks_t;
  const int last_full = max(wr.n_full - 1, 0);
  chunk_t kbuf[D][NCH];
  if (wr.n_full > 0) {
#pragma unroll
    for (int d = 0; d < D - 1; ++d) load_row<NCH>(kbuf[d], klane + min(d, last_full) * tile_stride, hh);
  }

  chunk_t qf[NQ][NCH];
  int jrow[NQ], limit[NQ];
  load_q_tiles<NCH, NQ>(a, bc, m, hh, qf, jrow);
  float rm[NQ], rl[NQ];
#pragma unroll
  for (int i = 0; i < NQ; ++i) {
    limit[i] = jrow[i] < 0 ? -1 : a.P + jrow[i];
    rm[i] = -1e30f;
    rl[i] = 0.0f;
  }

  f32x16 acc[2];
  if (wr.n_full > 0) mma_chain<DT, NCH>(acc[0], kbuf[0], qf[0]);
  for (int kt0 = 0; kt0 < wr.n_full; kt0 += D) {
#pragma unroll
    for (int u = 0; u < D; ++u) {
      const int k = kt0 + u;
      if (k >= wr.n_full) break;
      // D-1 tiles ahead; past the last full tile the last one is fetched again (in bounds, unused)
      load_row<NCH>(kbuf[(u + D - 1) % D], klane + min(k + D - 1, last_full) * tile_stride, hh);
#pragma unroll
      for (int i = 0; i < NQ; ++i) {
        // logits of the next pair; the last pair of a key tile already starts the next key tile
        if (i + 1 < NQ) mma_chain<DT, NCH>(acc[(i + 1) & 1], kbuf[u], qf[i + 1]);
        else mma_chain<DT, NCH>(acc[0], kbuf[(u + 1) % D], qf[0]);
        rowstats_update<false>(acc[i & 1], a.c2, 0, hh, 0, rm[i], rl[i]);
        interleave_hint<N_MFMA, 8>();
      }
    }
  }
  for (int t0 = wr.t_begin + wr.n_full * kTile; t0 < wr.t_end; t0 += kTile) {
    load_row<NCH>(kbuf[0], kbase + (int64_t)min(t0 + m, a.T - 1) * a.ks_t, hh);
#pragma unroll
    for (int i = 0; i < NQ; ++i) {
      mma_chain<DT, NCH>(acc[0], kbuf[0], qf[i]);
      rowstats_update<true>(acc[0], a.c2, t0, hh, limit[i], rm[i], rl[i]);
    }
  }
  store_row_partials<NQ>(a, bc, wr.wave, m, hh, rm, rl);
}

template <bool EDGE>
__device__ __forceinline__ float colsum_weights(const f32x16 &acc, const float (&nl2)[16], float c2, int hh,
                                                int first_masked_row) {
  float s[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    float pr = __builtin_amdgcn_exp2f(fmaf(acc[r], c2, nl2[r]));
    if (EDGE && acc_row(r, hh) < first_masked_row) pr = 0.0f;
    s[r & 3] += pr;
  }
  return (s[0] + s[1]) + (s[2] + s[3]);
}

// Adds the two half-waves' row sums and stores one value per (head, key). Heads are taken in pairs:
// v_permlane32_swap turns (x, y) into ([x.lo, y.lo], [x.hi, y.hi]), so one add leaves head x's
// totals in lanes 0..31 and head y's in lanes 32..63, and all 64 lanes store.
template <int NQ, int WT>
__device__ __forceinline__ void store_column_sums(const ScoreArgs &a, const BlockCoord &bc, const float (&cs)[NQ],
                                                  int kt, int hh) {
  constexpr int NH = NQ / WT;  // heads in this group
  float hv[NH];
#pragma unroll
  for (int h = 0; h < NH; ++h) {
    hv[h] = cs[h * WT];
#pragma unroll
    for (int e = 1; e < WT; ++e) hv[h] += cs[h * WT + e];
  }
  const int head0 = bc.g * a.G + (bc.grp * NQ) / WT;       // first head of the group
  const int heads_left = a.G - (bc.grp * NQ) / WT;         // heads of the KV group from there on
#pragma unroll
  for (int h = 0; h < NH; h += 2) {
    const float x = hv[h], y = hv[(h + 1 < NH) ? h + 1 : h];
    const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(y), false, false);
    const float tot = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
    const int mine = h + hh;  // lanes 32..63 carry the second head of the pair
    if (mine < NH && mine < heads_left && kt < a.T)
      a.scores[((size_t)bc.b * a.Hq + head0 + mine) * a.T + kt] = tot * a.norm;
  }
}

template <int DT, int DH, int NQ, int WT>
__global__ void __launch_bounds__(kScoreWaves *kWave) colsum_pipe_kernel(ScoreArgs a) {
  static_assert(NQ % 2 == 0 && NQ % WT == 0, "whole heads, even tile count");
  constexpr int NCH = DH * (DT == CKV_BF16 ? 2 : 4) / 32;
  constexpr int N_MFMA = NCH * (DT == CKV_BF16 ? 1 : 4);
  constexpr int D = kPrefetchTiles;
  const int lane = threadIdx.x & 63, m = lane & 31, hh = lane >> 5;
  const BlockCoord bc = decode_block(a);
  const WaveRange wr = wave_range(a, bc);

  const char *kbase = a.k + bc.b * a.ks_b + bc.g * a.ks_h;
  const char *klane = kbase + (int64_t)(wr.t_begin + m) * a.ks_t;
  const int64_t tile_stride = (int64_t)kTile * a.ks_t;
  const int last_full = max(wr.n_full - 1, 0);
  chunk_t kbuf[D][NCH];
  if (wr.n_full > 0) {
#pragma unroll
    for (int d = 0; d < D - 1; ++d) load_row<NCH>(kbuf[d], klane + min(d, last_full) * tile_stride, hh);
  }

  // -LSE (log2 domain) of the accumulator rows this lane holds; -inf on padding rows. Staged through
  // LDS so that the global read is one coalesced load per row instead of 16 dependent ones per lane.
  __shared__ __attribute__((aligned(16))) float s_nl2[NQ * kTile];
  if (threadIdx.x < NQ * kTile) {
    const int tile = bc.grp * NQ + threadIdx.x / kTile;
    const int j = (tile % WT) * kTile + threadIdx.x % kTile;
    const int h = bc.g * a.G + tile / WT;
    const bool valid = tile < a.n_tiles && j < a.W;
    s_nl2[threadIdx.x] = valid ? -a.lse[((size_t)bc.b * a.Hq + h) * a.W + j] * kLog2e : -INFINITY;
  }
  chunk_t qf[NQ][NCH];
  int jrow[NQ];
  load_q_tiles<NCH, NQ>(a, bc, m, hh, qf, jrow);
  __syncthreads();
  float nl2[NQ][16];
#pragma unroll
  for (int i = 0; i < NQ; ++i) {
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const f32x4 v = *reinterpret_cast<const f32x4 *>(s_nl2 + i * kTile + 8 * q4 + 4 * hh);
#pragma unroll
      for (int e = 0; e < 4; ++e) nl2[i][4 * q4 + e] = v[e];
    }
  }

  f32x16 acc[2];
  if (wr.n_full > 0) mma_chain<DT, NCH>(acc[0], qf[0], kbuf[0]);
  for (int kt0 = 0; kt0 < wr.n_full; kt0 += D) {
#pragma unroll
    for (int u = 0; u < D; ++u) {
      const int k = kt0 + u;
      if (k >= wr.n_full) break;
      load_row<NCH>(kbuf[(u + D - 1) % D], klane + min(k + D - 1, last_full) * tile_stride, hh);
      float cs[NQ];
#pragma unroll
      for (int i = 0; i < NQ; ++i) {
        if (i + 1 < NQ) mma_chain<DT, NCH>(acc[(i + 1) & 1], qf[i + 1], kbuf[u]);
        else mma_chain<DT, NCH>(acc[0], qf[0], kbuf[(u + 1) % D]);
        cs[i] = colsum_weights<false>(acc[i & 1], nl2[i], a.c2, hh, 0);
        interleave_hint<N_MFMA, 6>();
      }
      store_column_sums<NQ, WT>(a, bc, cs, wr.t_begin + k * kTile + m, hh);
    }
  }
  for (int t0 = wr.t_begin + wr.n_full * kTile; t0 < wr.t_end; t0 += kTile) {
    load_row<NCH>(kbuf[0], kbase + (int64_t)min(t0 + m, a.T - 1) * a.ks_t, hh);
    const int kt = t0 + m;
    float cs[NQ];
#pragma unroll
    for (int i = 0; i < NQ; ++i) {
      const int j0 = ((bc.grp * NQ + i) % WT) * kTile;
      mma_chain<DT, NCH>(acc[0], qf[i], kbuf[0]);
      cs[i] = colsum_weights<true>(acc[0], nl2[i], a.c2, hh, kt - a.P - j0);
    }
    store_column_sums<NQ, WT>(a, bc, cs, kt, hh);
  }
}

// ---------------------------------------------------------------------------------------------
// Launch
// ---------------------------------------------------------------------------------------------
template <int DT, int DH, int NQ>
static void launch_rowstats(const Shape &s, const ScoreArgs &a, dim3 grid, dim3 block, hipStream_t stream) {
  if constexpr (DT == CKV_BF16 && NQ % 2 == 0)
    hipLaunchKernelGGL((rowstats_pipe_kernel<DT, DH, NQ>), grid, block, 0, stream, a);
  else
    hipLaunchKernelGGL((rowstats_kernel<DT, DH, NQ>), grid, block, 0, stream, a);
  const int rows = s.Bz * s.Hkv * s.n_groups * NQ * kTile;
  hipLaunchKernelGGL(lse_kernel, dim3((rows + 255) / 256), dim3(256), 0, stream, a, NQ, rows);
}

template <int DT, int DH, int NQ>
static void launch_colsum(const Shape &s, const ScoreArgs &a, dim3 grid, dim3 block, hipStream_t stream) {
  if constexpr (DT == CKV_BF16 && NQ % 2 == 0) {
    if (s.WT == 1) {
      hipLaunchKernelGGL((colsum_pipe_kernel<DT, DH, NQ, 1>), grid, block, 0, stream, a);
      return;
    }
    if (s.WT == 2) {
      hipLaunchKernelGGL((colsum_pipe_kernel<DT, DH, NQ, 2>), grid, block, 0, stream, a);
      return;
    }
    if constexpr (NQ == 4) {
      if (s.WT == 4) {
        hipLaunchKernelGGL((colsum_pipe_kernel<DT, DH, NQ, 4>), grid, block, 0, stream, a);
        return;
      }
    }
  }
  hipLaunchKernelGGL((colsum_kernel<DT, DH, NQ>), grid, block, 0, stream, a);
}

template <int DT, int DH>
static hipError_t launch_scores_t(const Shape &s, ScoreArgs &a, bool need_lse, bool need_scores,
                                  hipStream_t stream) {
  const int units = s.Bz * s.Hkv;
  const dim3 grid((unsigned)((size_t)units * s.n_groups * s.n_chunks)), block(kScoreWaves * kWave);
#define CKV_LAUNCH_NQ(NQ)                                                        \
  case NQ:                                                                       \
    if (need_lse) launch_rowstats<DT, DH, NQ>(s, a, grid, block, stream);        \
    if (need_scores) launch_colsum<DT, DH, NQ>(s, a, grid, block, stream);       \
    break;
  switch (s.NQ) {
    CKV_LAUNCH_NQ(1)
    CKV_LAUNCH_NQ(2)
    CKV_LAUNCH_NQ(3)
    CKV_LAUNCH_NQ(4)
    default: return hipErrorInvalidValue;
  }
#undef CKV_LAUNCH_NQ
  return hipGetLastError();
}

hipError_t launch_window_scores(const ckv_params *p, const Shape &s, const Workspace &w, const void *q,
                                const void *k, const float *lse_in, float *lse_out, float *scores,
                                char *ws, hipStream_t stream) {
  ScoreArgs a;
  a.q = (const char *)q;
  a.k = (const char *)k;
  a.qs_b = p->q_stride[0] * s.esize;
  a.qs_h = p->q_stride[1] * s.esize;
  a.qs_w = p->q_stride[2] * s.esize;
  a.ks_b = p->k_stride[0] * s.esize;
  a.ks_h = p->k_stride[1] * s.esize;
  a.ks_t = p->k_stride[2] * s.esize;
  a.Hq = s.Hq; a.Hkv = s.Hkv; a.G = s.G; a.T = s.T; a.W = s.W; a.P = s.P;
  a.WT = s.WT; a.n_tiles = s.n_tiles; a.n_groups = s.n_groups;
  a.keys_per_wave = s.keys_per_wave; a.n_chunks = s.n_chunks;
  a.c2 = s.scale * kLog2e;
  a.norm = (float)s.T / (float)s.W;
  a.part = (float2 *)(ws + w.part_off);
  a.lse_out = lse_out ? lse_out : (float *)(ws + w.lse_off);
  a.lse = lse_in ? lse_in : a.lse_out;
  a.scores = scores;
  const bool need_lse = lse_in == nullptr, need_scores = scores != nullptr;
  if (p->dtype == CKV_BF16) {
    if (s.d == 128) return launch_scores_t<CKV_BF16, 128>(s, a, need_lse, need_scores, stream);
    return launch_scores_t<CKV_BF16, 64>(s, a, need_lse, need_scores, stream);
  }
  if (s.d == 128) return launch_scores_t<CKV_F32, 128>(s, a, need_lse, need_scores, stream);
  return launch_scores_t<CKV_F32, 64>(s, a, need_lse, need_scores, stream);
}

// ---------------------------------------------------------------------------------------------
// Value-norm ratio (paper Eq. 4, Alg. 1 Stage 1): r_t = ||v_t||_2, rho_t = r_t / (mean_t r_t + eps).
// Kernel 1 writes r_t and one partial sum per 1024-row block; kernel 2 adds the partials in a fixed
// order (no float atomics: results are bit-stable from run to run) and divides.
// ---------------------------------------------------------------------------------------------
struct VnormArgs {
  const char *v;
  int64_t vs_b, vs_h, vs_t;  // bytes
  int Hkv, T, n_blocks;
  float *ratio;  // [units][T]
  float *vsum;   // [units][n_blocks]
};
constexpr int kVnormRows = 1024;

template <int DT, int DH>
__global__ void __launch_bounds__(256) vnorm_rows_kernel(VnormArgs a) {
  constexpr int LPR = DH * (DT == CKV_BF16 ? 2 : 4) / 16;  // lanes per row, 8..32
  const int unit = blockIdx.y, blk = blockIdx.x;
  const int b = unit / a.Hkv, g = unit % a.Hkv;
  const char *base = a.v + b * a.vs_b + g * a.vs_h;
  const int sub = threadIdx.x % LPR, rloc = threadIdx.x / LPR;
  float local = 0.0f;
  for (int r = rloc; r < kVnormRows; r += 256 / LPR) {
    const int t = blk * kVnormRows + r;
    float sq = 0.0f;
    if (t < a.T) {
      const chunk_t c = *reinterpret_cast<const chunk_t *>(base + (int64_t)t * a.vs_t + sub * 16);
      if (DT == CKV_BF16) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const uint32_t pair = c[e];
          const float lo = __uint_as_float(pair << 16);
          const float hi = __uint_as_float(pair & 0xffff0000u);
          sq = fmaf(lo, lo, sq);
          sq = fmaf(hi, hi, sq);
        }
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const uint32_t word = c[e];
          const float x = __uint_as_float(word);
          sq = fmaf(x, x, sq);
        }
      }
    }
#pragma unroll
    for (int o = LPR / 2; o > 0; o >>= 1) sq += __shfl_xor(sq, o);
    if (sub == 0 && t < a.T) {
      const float nrm = sqrtf(sq);
      a.ratio[(size_t)unit * a.T + t] = nrm;
      local += nrm;
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) local += __shfl_xor(local, o);
  __shared__ float sm[4];
  if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = local;
  __syncthreads();
  if (threadIdx.x == 0) a.vsum[(size_t)unit * a.n_blocks + blk] = (sm[0] + sm[1]) + (sm[2] + sm[3]);
}

__global__ void __launch_bounds__(256) vnorm_scale_kernel(VnormArgs a) {
  const int unit = blockIdx.y, blk = blockIdx.x;
  float total = 0.0f;
  for (int i = 0; i < a.n_blocks; ++i) total += a.vsum[(size_t)unit * a.n_blocks + i];
  const float inv = 1.0f / (total / (float)a.T + kValueNormEps);
  for (int r = threadIdx.x; r < kVnormRows; r += 256) {
    const int t = blk * kVnormRows + r;
    if (t < a.T) a.ratio[(size_t)unit * a.T + t] *= inv;
  }
}

hipError_t launch_value_norm(const ckv_params *p, const Shape &s, const Workspace &w, const void *v,
                             float *ratio, char *ws, hipStream_t stream) {
  VnormArgs a;
  a.v = (const char *)v;
  a.vs_b = p->v_stride[0] * s.esize;
  a.vs_h = p->v_stride[1] * s.esize;
  a.vs_t = p->v_stride[2] * s.esize;
  a.Hkv = s.Hkv;
  a.T = s.T;
  a.n_blocks = vnorm_blocks_per_unit(s);
  a.ratio = ratio;
  a.vsum = (float *)(ws + w.vsum_off);
  const dim3 grid(a.n_blocks, s.Bz * s.Hkv), block(256);
  if (p->dtype == CKV_BF16) {
    if (s.d == 128) hipLaunchKernelGGL((vnorm_rows_kernel<CKV_BF16, 128>), grid, block, 0, stream, a);
    else hipLaunchKernelGGL((vnorm_rows_kernel<CKV_BF16, 64>), grid, block, 0, stream, a);
  } else {
    if (s.d == 128) hipLaunchKernelGGL((vnorm_rows_kernel<CKV_F32, 128>), grid, block, 0, stream, a);
    else hipLaunchKernelGGL((vnorm_rows_kernel<CKV_F32, 64>), grid, block, 0, stream, a);
  }
  hipLaunchKernelGGL(vnorm_scale_kernel, grid, block, 0, stream, a);
  return hipGetLastError();
}

}  // namespace ckv
