// Kernel templates of the observation-window scan (paper Sec. 3 attention definition, Eq. 3, Eq. 4's alpha per query head):
//   pass 1  rowstats kernels : stream K, QK^T on the matrix cores, online (max, sum) per window row
//           lse_kernel       : merge the per-chunk partials into LSE_j
//   pass 2  colsum kernels   : stream K again, recompute QK^T, exp(z - LSE_j), sum over window rows;
//                              in the fused form also the pooling, head weights and group maximum of
//                              Eq. 6 (Alg. 1 Stage 3), so that the per-head mass is never written
//
// Work decomposition. A "unit" is one (batch, KV head): its G*W window query rows all contract with
// the same K. Rows are cut into 32-row tiles (one MFMA 32x32 edge), whole heads only; a wave keeps its
// tiles of Q (up to eight for bf16, four for f32) in registers for its lifetime and takes 32-key tiles of
// K in MFMA operand layout: lane (m, hh) = (lane % 32, lane / 32) owns row m of a tile and the 16-byte
// chunks 2c+hh of that row. The contraction index may be permuted freely as long as both operands use
// the same permutation, so whole 16-byte chunks become MFMA k-groups and no transpose is needed. The
// four waves of a workgroup sweep four adjacent key ranges.
//
// The two passes use opposite operand orders on purpose:
//   pass 1: D = K Q^T, lane <-> query row: the running (max, sum) of a row never leaves its lane;
//   pass 2: D = Q K^T, lane <-> key: the sum over window rows is 16 in-lane adds and one half swap.
//
// Two families of kernels: plain ones that load every operand straight from global memory (f32,
// whose workloads are small), and LDS-staged, software-pipelined ones for bf16.
#ifndef CKV_SCAN_H_
#define CKV_SCAN_H_
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
  int lse_from_part; // pass 2 merges the row partials of pass 1 itself (no lse_kernel in between)
  float *lse_out;
  float *scores;     // [Bz][Hq][T]; with group_sum: [Bz][Hkv][T], the sum over each KV head's query heads
  int group_sum;
  // fused utility form of pass 2 only
  const float *w_row;  // w_head + layer * Hq
  float *utility;      // [Bz][Hkv][P]
  int pool, radius;    // pooling mode and radius (kernel / 2, at most kUtilMaxRadius)
  float inv_kernel;    // 1 / pool_kernel
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
  // wave-uniform by construction; the divisions run on the vector ALU, so say it (addresses derived from
  // these feed scalar operands)
  c.chunk = __builtin_amdgcn_readfirstlane(c.chunk);
  c.grp = __builtin_amdgcn_readfirstlane(c.grp);
  c.unit = __builtin_amdgcn_readfirstlane(c.unit);
  c.b = __builtin_amdgcn_readfirstlane(c.b);
  c.g = __builtin_amdgcn_readfirstlane(c.g);
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

// LSE_j = ln2 * (M + log2 sum_c l_c 2^(m_c - M)) from the n_chunks partials of one row, in chunk order.
__device__ __forceinline__ float merge_row_partials(const float2 *p, int n_chunks) {
  float M = -1e30f;
  for (int c = 0; c < n_chunks; ++c) M = fmaxf(M, p[c].x);
  float L = 0.0f;
  for (int c = 0; c < n_chunks; ++c) L += p[c].y * __builtin_amdgcn_exp2f(p[c].x - M);
  return (M + __log2f(L)) * kLn2;
}

// One thread per (unit, group, tile row).
template <int NQ>
__global__ void lse_kernel(ScoreArgs a, int n_rows_total) {
  const int row = blockIdx.x * blockDim.x + threadIdx.x;
  if (row >= n_rows_total) return;
  const int per_group = NQ * kTile;
  const int in_group = row % per_group;
  const int grp = (row / per_group) % a.n_groups;
  const int unit = row / (per_group * a.n_groups);
  const int tile = grp * NQ + in_group / kTile;
  const int j = (tile % a.WT) * kTile + in_group % kTile;
  if (tile >= a.n_tiles || j >= a.W) return;
  const int b = unit / a.Hkv, g = unit % a.Hkv, h = g * a.G + tile / a.WT;
  a.lse_out[((size_t)b * a.Hq + h) * a.W + j] = merge_row_partials(a.part + (size_t)row * a.n_chunks, a.n_chunks);
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
      for (int e = 1; e < kMaxWindowTiles; ++e)
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
// LDS-staged kernels for bf16 (rows of 128 or 256 bytes).
//
// A load instruction in which every lane addresses a different row touches 32 cache lines and keeps
// the texture-address unit busy several times longer than a contiguous one; with four waves per CU
// the scan then runs at the address unit's pace. These kernels therefore move K (and once per
// workgroup, Q) with global -> LDS loads in which the 64 lanes of one instruction read 1 KiB of whole
// rows, and pick the MFMA operand layout up from LDS with 128-bit reads. Each wave owns a ring of
// four tile images. The image of a 32-row tile holds chunk kappa of row r at
// r * ROW + ((kappa ^ (r & SW)) * 16) so that the operand reads (32 lanes, same chunk, consecutive
// rows) spread over all banks; the load writes lane l's 16 bytes at image offset 16 * (64 * i + l),
// so the swizzle is applied to the source address instead.
//
// One wave per SIMD runs a two-stage software pipeline over (key tile, query tile) pairs: the MFMA
// chain of the next pair is issued in between the vector instructions that consume the current
// pair's logits (two accumulator sets). A lone wave issues one instruction at a time, so everything
// that is not vector arithmetic is kept out of the loop: the loop is unrolled over the ring (image
// addresses become immediates), key tiles are addressed by a running scalar pointer, and the loads
// use the scalar-base form with one M0 write per four instructions (their immediate offset moves the
// global and the LDS address alike, which the per-lane offsets compensate). In pass 2 the -LSE of the
// accumulator rows is folded into the contraction as one more MFMA step whose Q-side operand holds
// -LSE / scale split into three bf16 terms (exact to 2^-24) and whose K-side operand is ones.
// Tiles that touch the window or the end of the keys are handled after the pipeline, masked.
// ---------------------------------------------------------------------------------------------
typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(1))) const void glb_void_t;

// Cache policy of the pipeline's output stores (column sums, group sums, utilities): sc1. The outputs
// are consumed by a later kernel, never by this one; with the default policy the stores, although a
// few percent of the pass's bytes, cost it 6-8 us more (measured on the 32k / batch-16 shape).
#ifndef CKV_OUT_STORE_AUX
#define CKV_OUT_STORE_AUX 16
#endif
constexpr int kOutStoreAux = CKV_OUT_STORE_AUX;

template <int DT, int DH>
struct Geom {
  static constexpr int ROW = DH * (DT == CKV_BF16 ? 2 : 4);  // bytes per row
  static constexpr int CH = ROW / 16;                        // 16-byte chunks per row
  static constexpr int NCH = CH / 2;                         // chunks per lane (the other half-wave holds the rest)
  static constexpr int TILE = kTile * ROW;                   // bytes per 32-row tile image
  static constexpr int NDMA = TILE / 1024;                   // load instructions per tile
  static constexpr int SW = (CH < 16 ? CH : 16) - 1;         // swizzle mask
  static_assert(ROW == 128 || ROW == 256, "row size");
};

// Row and chunk of a tile that lane `lane` moves in load instruction i (the lane's 16 bytes land at
// image offset 16 * (64 * i + lane)).
template <class G>
__device__ __forceinline__ void dma_source(int i, int lane, int &r, int &kappa) {
  const int s = i * 64 + lane;
  r = s / G::CH;
  kappa = (s % G::CH) ^ (r & G::SW);
}

template <class G>
__device__ __forceinline__ int image_offset(int r, int kappa) {
  return r * G::ROW + ((kappa ^ (r & G::SW)) << 4);
}

// Waits until at most N of this wave's vector memory operations are still in flight (they complete
// in issue order); also keeps the compiler from moving LDS accesses across the wait.
template <int N>
__device__ __forceinline__ void wait_vm() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
  asm volatile("" ::: "memory");
}

// A wave-uniform pointer as a scalar register pair. The compiler may form uniform 64-bit address
// arithmetic on the vector ALU; operands of the scalar-base loads below must be told apart from that.
__device__ __forceinline__ const char *uniform_ptr(const char *p) {
  const uint64_t v = (uint64_t)(uintptr_t)p;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return (const char *)(uintptr_t)(((uint64_t)hi << 32) | lo);
}

// Four loads with one M0 write: instruction j reads 16 bytes per lane at sbase + voff_j + 1024 * j
// and writes them at LDS address lds + 1024 * j + 16 * lane. K is read once per pass and never again
// before everything else has gone through the caches: the loads are marked non-temporal (streaming),
// which measurably raises the rate at which HBM delivers them and leaves L2 and the memory-side cache
// to the data that is reused (Q, the column sums on their way to the next kernel).
__device__ __forceinline__ void dma_quad(const char *sbase, uint32_t lds, uint32_t v0, uint32_t v1, uint32_t v2,
                                         uint32_t v3) {
  asm volatile(
      "s_mov_b32 m0, %0\n\ts_nop 0\n\t"
      "global_load_lds_dwordx4 %2, %1 offset:0 nt\n\t"
      "global_load_lds_dwordx4 %3, %1 offset:1024 nt\n\t"
      "global_load_lds_dwordx4 %4, %1 offset:2048 nt\n\t"
      "global_load_lds_dwordx4 %5, %1 offset:3072 nt"
      :
      : "s"(lds), "s"(sbase), "v"(v0), "v"(v1), "v"(v2), "v"(v3)
      : "memory");
}

// One whole tile whose first row starts at tile_base. voff[i] already holds the lane's source offset
// minus the immediate of its instruction plus kDmaBias, so the scalar base is tile_base - kDmaBias.
constexpr int kDmaBias = 3072;
template <class G>
__device__ __forceinline__ void dma_tile(const char *tile_base, const uint32_t (&voff)[G::NDMA], uint32_t lds_image) {
#pragma unroll
  for (int q = 0; q < G::NDMA / 4; ++q)
    dma_quad(tile_base - kDmaBias, lds_image + q * 4096, voff[4 * q] + q * 4096, voff[4 * q + 1] + q * 4096,
             voff[4 * q + 2] + q * 4096, voff[4 * q + 3] + q * 4096);
}

// A tile whose rows may run past the last key: row indices are clamped (the logits of the clamped
// rows are masked by the caller). Outside the pipeline, so the plain form will do.
template <class G>
__device__ __forceinline__ void dma_tile_clamped(const char *kbase, int64_t ks_t, int t0, int T, int lane,
                                                 char *image) {
#pragma unroll
  for (int i = 0; i < G::NDMA; ++i) {
    int r, kappa;
    dma_source<G>(i, lane, r, kappa);
    const char *src = kbase + (int64_t)min(t0 + r, T - 1) * ks_t + kappa * 16;
    __builtin_amdgcn_global_load_lds((glb_void_t *)src, (lds_void_t *)(uintptr_t)(image + i * 1024), 16, 0, 0);
  }
}

template <class G>
__device__ __forceinline__ void read_image(chunk_t (&f)[G::NCH], const char *image, const int (&roff)[G::NCH]) {
#pragma unroll
  for (int c = 0; c < G::NCH; ++c) f[c] = *reinterpret_cast<const chunk_t *>(image + roff[c]);
}

// Scheduling hint for one pipeline step: N_MFMA groups of one MFMA, (where the step also picks up the
// next key tile) one LDS read, and a few vector instructions.
template <int N_MFMA, int VALU_PER, int N_DS>
__device__ __forceinline__ void interleave_hint() {
#pragma unroll
  for (int u = 0; u < N_MFMA; ++u) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                 // one MFMA
    if (u < N_DS) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read
    __builtin_amdgcn_sched_group_barrier(0x002, VALU_PER, 0);          // then a few vector instructions
  }
}

// Key tiles per unrolled body of the pipelines. Up to four query tiles per wave the body is a whole ring
// cycle (every ring image address is an immediate). Beyond that a body of four tiles holds so many
// scheduling-hint groups that the compiler's solver for them needs minutes per kernel; half a cycle
// keeps it at seconds, and the ring image of a body's first tile becomes a run-time (scalar) value.
__host__ __device__ constexpr int unroll_tiles(int nq) { return nq > 4 ? 2 : kRing; }
static_assert(kRing % 2 == 0, "half a ring cycle starts at an even image");

// Vector instructions that the hint places behind each MFMA of the next pair's chain. Fewer than an even
// spread (pass 1 has ~63 per 8 MFMAs, pass 2 ~52 per 9): the chain is then issued early, and what is left
// of the current pair's vector work runs after its last MFMA -- the 18 wait states between an MFMA and the
// first read of its result are filled with work instead of s_nop (one `s_nop 11` per pair with an even
// spread). Measured in cycles per pair where memory does not limit (T = 128k, W = 64, eight tiles per
// wave): pass 1 492 (8 per MFMA), 426 (6), 439 (5); pass 2 517 (6), 492 (5), 428 (4), 443 (3). With
// four tiles per wave on the 32k / batch-16 shape, which sits at the memory ceiling, pass 1 gains 3 us with
// 6 and pass 2 is best left at 6 (5 and 4: 2-3 us slower).
__host__ __device__ constexpr int vector_per_mfma_pass1(int nq) { return 6; }
__host__ __device__ constexpr int vector_per_mfma_pass2(int nq) { return nq > 4 ? 4 : 6; }

// Geometry of a wave's key range: wave-uniform values live in scalar registers.
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

// Everything the two staged kernels share: the ring, the per-lane offsets, Q in registers.
#ifndef CKV_PIN_Q_ABOVE
#define CKV_PIN_Q_ABOVE 4
#endif
template <int DT, int DH, int NQ>
struct Staged {
  using G = Geom<DT, DH>;
  static constexpr int NCH = G::NCH;
  typedef char Ring[kScoreWaves][kRing][G::TILE];
  uint32_t voff[G::NDMA];  // lane's biased source offset inside a K tile, per load instruction
  int roff[NCH];           // lane's operand chunks inside a tile image
  const char *kbase;       // first key row of the unit
  const char *kcur;        // first row of the key tile the pipeline is working on
  const char *klast;       // first row of the wave's last full tile
  int64_t tile_stride;
  uint32_t lds_ring;       // LDS address of this wave's first image

  // Starts the loads of Q (wave w moves query tiles w and w + 4 into the last images of its ring) and of the
  // first key tiles, then hands every wave all NQ query tiles in registers; on return the wave's first
  // three key tiles are in flight, in order. jrow[i] = window row of tile i, row m, or -1 on padding.
  static constexpr int QI = (NQ + kScoreWaves - 1) / kScoreWaves;  // ring images per wave that first hold Q
  static_assert(QI >= 1 && QI <= kRing - 2, "query tiles pass through the ring's last images");
  __device__ __forceinline__ void start(const ScoreArgs &a, const BlockCoord &bc, const WaveRange &wr, Ring &ring,
                                        int lane, int m, int hh, chunk_t (&qf)[NQ][NCH], int (&jrow)[NQ]) {
#pragma unroll
    for (int i = 0; i < G::NDMA; ++i) {
      int r, kappa;
      dma_source<G>(i, lane, r, kappa);
      voff[i] = (uint32_t)(r * a.ks_t + kappa * 16 + kDmaBias - (i % 4) * 1024 - (i / 4) * 4096);
    }
#pragma unroll
    for (int c = 0; c < NCH; ++c) roff[c] = image_offset<G>(m, c + NCH * hh);
    kbase = uniform_ptr(a.k + bc.b * a.ks_b + bc.g * a.ks_h);
    kcur = uniform_ptr(kbase + (int64_t)wr.t_begin * a.ks_t);
    tile_stride = (int64_t)kTile * a.ks_t;
    klast = uniform_ptr(kcur + max(wr.n_full - 1, 0) * tile_stride);
    lds_ring = (uint32_t)(uintptr_t)&ring[wr.wave][0][0];

#pragma unroll
    for (int qi = 0; qi < QI; ++qi) {
      if (wr.wave + qi * kScoreWaves < NQ) {
        const int tile = min(bc.grp * NQ + wr.wave + qi * kScoreWaves, a.n_tiles - 1);
        const char *qhead = a.q + bc.b * a.qs_b + (bc.g * a.G + tile / a.WT) * a.qs_h;
        const int j0 = (tile % a.WT) * kTile;
#pragma unroll
        for (int i = 0; i < G::NDMA; ++i) {
          int r, kappa;
          dma_source<G>(i, lane, r, kappa);
          const char *src = qhead + (int64_t)min(j0 + r, a.W - 1) * a.qs_w + kappa * 16;
          __builtin_amdgcn_global_load_lds((glb_void_t *)src,
                                           (lds_void_t *)(uintptr_t)(ring[wr.wave][kRing - 1 - qi] + i * 1024), 16, 0, 0);
        }
      }
    }
    constexpr int N_PRE = kRing - QI;  // key tiles whose images are free while Q passes through
    if (wr.n_full > 0) {
#pragma unroll
      for (int d = 0; d < N_PRE; ++d)
        dma_tile<G>(d < wr.n_full ? kcur + d * tile_stride : klast, voff, lds_ring + d * G::TILE);
      wait_vm<N_PRE * G::NDMA>();  // Q has landed, the key tiles may still be on their way
    } else {
      wait_vm<0>();
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NQ; ++i) {
      const int tile = bc.grp * NQ + i;
      const int j = (tile % a.WT) * kTile + m;
      const bool valid = tile < a.n_tiles && j < a.W;
      jrow[i] = valid ? j : -1;
      read_image<G>(qf[i], ring[i % kScoreWaves][kRing - 1 - i / kScoreWaves], roff);
      if (!valid) {
#pragma unroll
        for (int c = 0; c < NCH; ++c) qf[i][c] = chunk_t{0u, 0u, 0u, 0u};
      }
      // With more than four query tiles the ordinary vector registers are what runs out (the logits, the key
      // tile and the vector work's temporaries must live there), while the matrix cores take their operands
      // from accumulation registers just as well: say where Q is to live, or the allocator keeps a tile of it
      // in vector registers and serialises the exponentials through one temporary.
      if constexpr (NQ > CKV_PIN_Q_ABOVE) {
#pragma unroll
        for (int c = 0; c < NCH; ++c) asm volatile("" : "+a"(qf[i][c]));
      }
    }
    __syncthreads();  // the images that held Q are free for key tiles from here on
    if (wr.n_full > 0) {
#pragma unroll
      for (int d = N_PRE; d < kRing - 1; ++d)
        dma_tile<G>(d < wr.n_full ? kcur + d * tile_stride : klast, voff, lds_ring + d * G::TILE);
    }
  }

  // Load of the tile three ahead of the one at kcur (tile index t + 3) into ring image `slot`; past
  // the last full tile the last one is fetched again (in bounds, unused).
  __device__ __forceinline__ void prefetch(int t, int n_full, int slot) {
    dma_tile<G>(t + 3 < n_full ? kcur + 3 * tile_stride : klast, voff, lds_ring + slot * G::TILE);
  }
};

template <int DT, int DH, int NQ>
__global__ void __launch_bounds__(kScoreWaves *kWave) rowstats_lds_kernel(ScoreArgs a) {
  using G = Geom<DT, DH>;
  constexpr int NCH = G::NCH;
  constexpr int N_MFMA = NCH * (DT == CKV_BF16 ? 1 : 4);
  constexpr int READ_AT = NQ >= 2 ? NQ - 2 : 0;  // query tile during which the next key tile is picked up
  __shared__ __attribute__((aligned(1024))) typename Staged<DT, DH, NQ>::Ring ring;
  const int lane = threadIdx.x & 63, m = lane & 31, hh = lane >> 5;
  const BlockCoord bc = decode_block(a);
  const WaveRange wr = wave_range(a, bc);

  Staged<DT, DH, NQ> st;
  chunk_t qf[NQ][NCH];
  int jrow[NQ], limit[NQ];
  st.start(a, bc, wr, ring, lane, m, hh, qf, jrow);
  float rm[NQ], rl[NQ];
#pragma unroll
  for (int i = 0; i < NQ; ++i) {
    limit[i] = jrow[i] < 0 ? -1 : a.P + jrow[i];  // last key this row may see (causal)
    rm[i] = -1e30f;
    rl[i] = 0.0f;
  }

  chunk_t kreg[2][NCH];
  f32x16 acc[2];
  const int n_piped = wr.n_full / kRing * kRing;  // the pipeline takes key tiles one ring at a time
  if (n_piped > 0) {
    wait_vm<(kRing - 2) * G::NDMA>();
    read_image<G>(kreg[0], ring[wr.wave][0], st.roff);
    mma_chain<DT, NCH>(acc[0], kreg[0], qf[0]);
  }
  constexpr int UR = unroll_tiles(NQ);
  for (int t0 = 0; t0 < n_piped; t0 += UR) {
    const int slot0 = UR == kRing ? 0 : (t0 & (kRing - 1));  // ring image of tile t0
#pragma unroll
    for (int v = 0; v < UR; ++v) {  // tile t0 + v lives in image u and in kreg[v & 1]
      const int u = slot0 + v;
      st.prefetch(t0 + v, wr.n_full, (u + kRing - 1) % kRing);
#pragma unroll
      for (int i = 0; i < NQ; ++i) {
        const int cur = (v * NQ + i) & 1;  // accumulator set holding this pair's logits
        if (i == READ_AT) {
          wait_vm<(kRing - 2) * G::NDMA>();  // tile t0 + v + 1 has landed
          read_image<G>(kreg[(v + 1) & 1], ring[wr.wave][(u + 1) % kRing], st.roff);
        }
        // logits of the next pair; the last pair of a key tile already starts the next key tile
        if (i + 1 < NQ) mma_chain<DT, NCH>(acc[cur ^ 1], kreg[v & 1], qf[i + 1]);
        else mma_chain<DT, NCH>(acc[cur ^ 1], kreg[(v + 1) & 1], qf[0]);
        rowstats_update<false>(acc[cur], a.c2, 0, hh, 0, rm[i], rl[i]);
        if (i == READ_AT) interleave_hint<N_MFMA, vector_per_mfma_pass1(NQ), NCH>();
        else interleave_hint<N_MFMA, vector_per_mfma_pass1(NQ), 0>();
      }
      st.kcur += st.tile_stride;
    }
  }
  // What the pipeline left: up to a ring of whole tiles and the masked ones. Their loads go out a ring at
  // a time, so the memory latency is paid once per ring and not once per tile.
  wait_vm<0>();
  for (int r0 = wr.t_begin + n_piped * kTile; r0 < wr.t_end; r0 += kRing * kTile) {
#pragma unroll
    for (int j = 0; j < kRing; ++j)
      if (r0 + j * kTile < wr.t_end) dma_tile_clamped<G>(st.kbase, a.ks_t, r0 + j * kTile, a.T, lane, ring[wr.wave][j]);
    wait_vm<0>();
    for (int j = 0; j < kRing && r0 + j * kTile < wr.t_end; ++j) {
      const int t0 = r0 + j * kTile;
      read_image<G>(kreg[0], ring[wr.wave][j], st.roff);
#pragma unroll
      for (int i = 0; i < NQ; ++i) {
        mma_chain<DT, NCH>(acc[0], kreg[0], qf[i]);
        rowstats_update<true>(acc[0], a.c2, t0, hh, limit[i], rm[i], rl[i]);
      }
    }
  }
  store_row_partials<NQ>(a, bc, wr.wave, m, hh, rm, rl);
}

// The extra contraction step of pass 2 that adds bias_j = -LSE_j / scale to every logit of query row
// j. bf16: the bias as hi + mid + lo bf16 terms in the first three slots of the Q-side operand of the
// lanes with hh = 0, ones in the same slots on the K side. f32: one 32x32x2 step with (bias, 1).
__device__ __forceinline__ uint32_t bf16_bits(float x) {  // round to nearest even; x is finite
  const uint32_t u = __float_as_uint(x);
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
template <int DT>
struct Bias;
template <>
struct Bias<CKV_BF16> {
  chunk_t q;
  __device__ __forceinline__ void set(float bias, int hh) {
    const uint32_t hi = bf16_bits(bias);
    const float r1 = bias - __uint_as_float(hi << 16);
    const uint32_t mid = bf16_bits(r1);
    const float r2 = r1 - __uint_as_float(mid << 16);
    const uint32_t lo = bf16_bits(r2);
    q = hh == 0 ? chunk_t{hi | (mid << 16), lo, 0u, 0u} : chunk_t{0u, 0u, 0u, 0u};
  }
  static __device__ __forceinline__ chunk_t ones(int hh) {
    return hh == 0 ? chunk_t{0x3f803f80u, 0x3f80u, 0u, 0u} : chunk_t{0u, 0u, 0u, 0u};
  }
  __device__ __forceinline__ void add(f32x16 &acc, const chunk_t &one) const { Mma<CKV_BF16>::step(acc, q, one); }
};
template <>
struct Bias<CKV_F32> {
  float q;
  __device__ __forceinline__ void set(float bias, int hh) { q = hh == 0 ? bias : 0.0f; }
  static __device__ __forceinline__ chunk_t ones(int hh) {
    return chunk_t{hh == 0 ? 0x3f800000u : 0u, 0u, 0u, 0u};
  }
  __device__ __forceinline__ void add(f32x16 &acc, const chunk_t &one) const {
    const uint32_t o = one[0];
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(q, __uint_as_float(o), acc, 0, 0, 0);
  }
};

// Weights exp(z - LSE) of one tile from acc = <q, k> - LSE / scale, summed over this lane's 16 rows.
template <bool EDGE>
__device__ __forceinline__ float colsum_weights(const f32x16 &acc, float c2, int hh, int first_masked_row) {
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

// Adds the two half-waves' row sums and stores one value per (head, key). Heads are taken in pairs:
// v_permlane32_swap turns (x, y) into ([x.lo, y.lo], [x.hi, y.hi]), so one add leaves head x's
// totals in lanes 0..31 and head y's in lanes 32..63, and all 64 lanes store.
template <int NQ>
__device__ __forceinline__ void store_column_sums(const ScoreArgs &a, const BlockCoord &bc, const float (&cs)[NQ],
                                                  int WT, int kt, int hh) {
  float hv[NQ];  // per head of the group (NQ / WT of them), the sum over its tiles
  int nh = 0;
#pragma unroll
  for (int i = 0; i < NQ; ++i) {
    if (i % WT == 0) hv[nh++] = cs[i];
    else hv[nh - 1] += cs[i];
  }
  const int head0 = bc.g * a.G + (bc.grp * NQ) / WT;  // first head of the group
  const int heads_left = a.G - (bc.grp * NQ) / WT;    // heads of the KV group from there on
#pragma unroll
  for (int h = 0; h < NQ; h += 2) {
    if (h >= nh) break;
    const float x = hv[h], y = hv[(h + 1 < nh) ? h + 1 : h];
    const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(y), false, false);
    const float tot = (__uint_as_float(sw[0]) + __uint_as_float(sw[1])) * a.norm;
    const int mine = h + hh;  // lanes 32..63 carry the second head of the pair
    if (mine < nh && mine < heads_left && kt < a.T) a.scores[((size_t)bc.b * a.Hq + head0 + mine) * a.T + kt] = tot;
  }
}

// Group-sum form of the same: one value per key, the sum over the group's heads.
template <int NQ>
__device__ __forceinline__ void store_group_sum(const ScoreArgs &a, const BlockCoord &bc, const float (&cs)[NQ], int kt,
                                                int hh) {
  float x = cs[0];  // padding heads have zero query rows and bias -1000: their weights are exactly 0
#pragma unroll
  for (int i = 1; i < NQ; ++i) x += cs[i];
  const float tot = (x + __shfl_xor(x, 32)) * a.norm;
  if (hh == 0 && kt < a.T) a.scores[((size_t)bc.b * a.Hkv + bc.g) * a.T + kt] = tot;
}

// Pipeline form of the same: the totals of one key tile go to a per-wave LDS stage
// [head of the group][key of the ring cycle], and once per ring cycle (4 tiles, 128 keys) every lane
// stores four consecutive keys of one head with one 128-bit buffer store per pair of heads.
template <int NQ, int WT, int ROW = kRing * kTile>
__device__ __forceinline__ void stage_column_sums(const float (&cs)[NQ], float norm, float *stage, int u, int m,
                                                  int hh) {
  constexpr int NH = NQ / WT;
  float hv[NH];
#pragma unroll
  for (int h = 0; h < NH; ++h) {
    hv[h] = cs[h * WT];
#pragma unroll
    for (int e = 1; e < WT; ++e) hv[h] += cs[h * WT + e];
  }
#pragma unroll
  for (int h = 0; h < NH; h += 2) {
    const float x = hv[h], y = hv[(h + 1 < NH) ? h + 1 : h];
    const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(y), false, false);
    const float tot = (__uint_as_float(sw[0]) + __uint_as_float(sw[1])) * norm;
    if (h + hh < NH) stage[(h + hh) * ROW + u * kTile + m] = tot;
  }
}

// The stage is written by one set of lanes and read by another of the same wave. The hardware keeps a
// wave's LDS operations in order, but the compiler, reasoning per lane, sees a store and a load that can
// never touch the same word and may swap them: this keeps every memory access on its side of the line.
__device__ __forceinline__ void stage_fence() { asm volatile("" ::: "memory"); }

template <int NQ, int WT>
__device__ __forceinline__ void flush_column_sums(const ScoreArgs &a, const BlockCoord &bc, const float *stage,
                                                  int t_first, int lane, __amdgpu_buffer_rsrc_t rsrc) {
  constexpr int NH = NQ / WT;
  const int head0 = bc.g * a.G + (bc.grp * NQ) / WT;
  const int heads_left = a.G - (bc.grp * NQ) / WT;
#pragma unroll
  for (int h = 0; h < NH; h += 2) {
    const int mine = h + (lane >> 5), key4 = 4 * (lane & 31);
    const bool valid = mine < NH && mine < heads_left;
    const f32x4 v = *reinterpret_cast<const f32x4 *>(stage + (valid ? mine : 0) * (kRing * kTile) + key4);
    const uint32_t off = valid ? (uint32_t)(((head0 + mine) * a.T + t_first + key4) * 4) : 0x80000000u;
    typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4_t, v), rsrc, off, 0, kOutStoreAux);
  }
}

// Group-sum form of the flush (layer-shared mode: the prompt's alpha is a mean over heads, so only the
// sum over a KV head's query heads is needed): lanes 0..31 add the even heads of the stage, lanes
// 32..63 the odd ones, four consecutive keys each; the halves are added and lanes 0..31 store one
// 128-bit piece of the single output row -- a quarter of the per-head form's bytes for groups of four.
template <int NQ>
__device__ __forceinline__ void flush_group_sums(const ScoreArgs &a, const BlockCoord &bc, const float *stage,
                                                 int t_first, int lane, __amdgpu_buffer_rsrc_t rsrc_g) {
  const int half = lane >> 5, key4 = 4 * (lane & 31);
  const int heads_left = a.G - bc.grp * NQ;
  f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
  for (int h = 0; h < NQ; h += 2) {
    const int mine = h + half;
    if (mine < NQ && mine < heads_left) acc += *reinterpret_cast<const f32x4 *>(stage + mine * (kRing * kTile) + key4);
  }
#pragma unroll
  for (int e = 0; e < 4; ++e) acc[e] += __shfl_xor(acc[e], 32);
  const uint32_t off = half == 0 ? (uint32_t)((bc.g * a.T + t_first + key4) * 4) : 0x80000000u;
  typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
  __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4_t, acc), rsrc_g, off, 0, kOutStoreAux);
}

// Fused form of the flush (ckv_window_utility): instead of the column sums, the wave writes the
// UTILITY -- pooled along the keys, weighted per head, maximum over the group's heads (paper Eq. 6) --
// straight from the stage. A stage row holds, in front of the block's 128 values, the last 40 of the
// previous block, and each flush covers the 128 keys that END 32 keys before the block does: every
// pooling window (radius <= 3) lies inside the row and every store covers whole 128-byte lines
// (partial lines proved expensive). What this leaves out per wave range -- the first four keys, the
// last 32 keys of the pipelined part, and the tail tiles -- a small kernel computes afterwards from
// raw column sums, which the first block (its first eight keys), the last block (its last 40 keys)
// and the tail tiles store. Lanes 0..31 take the even heads of the group, lanes 32..63 the odd ones,
// four consecutive keys each (three 128-bit reads per head); the halves then swap so that each lane
// ends up with the group maximum of two adjacent keys and stores them with one 64-bit store. The taps
// are combined left to right, as the stand-alone tables kernel does.
constexpr int kUtilRow = kUtilCarry + kRing * kTile;
// win[hp]: the twelve values around this lane's four keys (win[hp][4 .. 7]) of head 2 hp + half.
template <int NH, int POOL, int R>
__device__ __forceinline__ void pooled_group_max(const ScoreArgs &a, const float (&win)[(NH + 1) / 2][12], int lane,
                                                 int heads_left, const float (&wgt)[NH], float (&best)[4]) {
  const int half = lane >> 5;
#pragma unroll
  for (int e = 0; e < 4; ++e) best[e] = -INFINITY;
#pragma unroll
  for (int hp = 0; hp < (NH + 1) / 2; ++hp) {
    const int h = 2 * hp + half;
    const bool live = h < NH && h < heads_left;
    float wg = 0.0f;
#pragma unroll
    for (int x = 0; x < NH; ++x) wg = (x == h) ? wgt[x] : wg;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float c = win[hp][4 + e - R];
#pragma unroll
      for (int d = 1 - R; d <= R; ++d) c = POOL == CKV_POOL_MAX ? fmaxf(c, win[hp][4 + e + d]) : c + win[hp][4 + e + d];
      if (POOL == CKV_POOL_AVG) c *= a.inv_kernel;
      // a select, not a branch: heads that do not exist leave the maximum alone
      best[e] = fmaxf(best[e], live ? wg * c : -INFINITY);
    }
  }
}

// rows: the wave's stage rows (carry included); t_first: first key of the block just staged. Every LDS
// read of the flush is issued before anything waits for one (the wave is alone on its SIMD: a read's
// latency is otherwise paid once per dependent step).
template <int NQ, int WT>
__device__ __forceinline__ void flush_utility(const ScoreArgs &a, const BlockCoord &bc, float *rows, int t_first,
                                              bool first_block, bool last_block, int lane,
                                              __amdgpu_buffer_rsrc_t rsrc, __amdgpu_buffer_rsrc_t rsrc_u,
                                              const float (&wgt)[NQ / WT]) {
  constexpr int NH = NQ / WT;
  constexpr int NP = (NH + 1) / 2;  // pairs of heads: lanes 0..31 take the even head, lanes 32..63 the odd one
  constexpr int BLK = kRing * kTile;
  const int head0 = bc.g * a.G + (bc.grp * NQ) / WT;
  const int heads_left = a.G - (bc.grp * NQ) / WT;
  const int half = lane >> 5, grp = lane & 31, key4 = 4 * grp;
  typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
  typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;
  typedef __attribute__((ext_vector_type(2))) float f32x2;
  // -- reads: raw sums of this lane's keys, the pooling windows, the pieces of the carry
  f32x4 raw[NP];
  float win[NP][12];
#pragma unroll
  for (int hp = 0; hp < NP; ++hp) {
    const int mine = 2 * hp + half;
    const float *row = rows + (mine < NH ? mine : 0) * kUtilRow;
    raw[hp] = *reinterpret_cast<const f32x4 *>(row + kUtilCarry + key4);
    const float *w0 = row + (kUtilCarry - kUtilShift - 4) + key4;  // w0[4 .. 7]: keys 4 grp - 32 .. of the block
#pragma unroll
    for (int q = 0; q < 3; ++q) {
      const f32x4 v = *reinterpret_cast<const f32x4 *>(w0 + 4 * q);
#pragma unroll
      for (int e = 0; e < 4; ++e) win[hp][4 * q + e] = v[e];
    }
  }
  constexpr int PER = kUtilCarry / 4;  // 128-bit pieces of the carry per head
  constexpr int NC = (PER * NH + kWave - 1) / kWave;
  static_assert(NC <= 2, "at most two pieces per lane");
  f32x4 carry[NC];
#pragma unroll
  for (int i = 0; i < NC; ++i) {
    const int piece = lane + i * kWave;
    const int pc = piece < PER * NH ? piece : 0;
    carry[i] = *reinterpret_cast<const f32x4 *>(rows + (pc / PER) * kUtilRow + BLK + 4 * (pc % PER));
  }
  // -- carry: the block's last kUtilCarry values move in front of the rows for the next block (LDS operations
  // of a wave complete in order: the windows above were read before these writes land)
  stage_fence();
#pragma unroll
  for (int i = 0; i < NC; ++i) {
    const int piece = lane + i * kWave;
    if (piece < PER * NH) *reinterpret_cast<f32x4 *>(rows + (piece / PER) * kUtilRow + 4 * (piece % PER)) = carry[i];
  }
  // -- raw column sums for the fix-up kernel: the first block's first eight keys, the last block's last 40
#pragma unroll
  for (int hp = 0; hp < NP; ++hp) {
    const int mine = 2 * hp + half;
    const bool valid = mine < NH && mine < heads_left &&
                       ((first_block && key4 < kUtilHead) || (last_block && key4 >= BLK - kUtilCarry));
    const uint32_t off = valid ? (uint32_t)(((head0 + mine) * a.T + t_first + key4) * 4) : 0x80000000u;
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4_t, raw[hp]), rsrc, off, 0, kOutStoreAux);
  }
  float best[4];
  if (a.pool == CKV_POOL_MAX) {
    switch (a.radius) {
      case 1: pooled_group_max<NH, CKV_POOL_MAX, 1>(a, win, lane, heads_left, wgt, best); break;
      case 2: pooled_group_max<NH, CKV_POOL_MAX, 2>(a, win, lane, heads_left, wgt, best); break;
      case 3: pooled_group_max<NH, CKV_POOL_MAX, 3>(a, win, lane, heads_left, wgt, best); break;
      default: pooled_group_max<NH, CKV_POOL_MAX, 0>(a, win, lane, heads_left, wgt, best); break;
    }
  } else {
    switch (a.radius) {
      case 1: pooled_group_max<NH, CKV_POOL_AVG, 1>(a, win, lane, heads_left, wgt, best); break;
      case 2: pooled_group_max<NH, CKV_POOL_AVG, 2>(a, win, lane, heads_left, wgt, best); break;
      case 3: pooled_group_max<NH, CKV_POOL_AVG, 3>(a, win, lane, heads_left, wgt, best); break;
      default: pooled_group_max<NH, CKV_POOL_AVG, 0>(a, win, lane, heads_left, wgt, best); break;
    }
  }
  // (x, y) -> ([x.lo, y.lo], [x.hi, y.hi]): lanes 0..31 get both halves' values of keys 0 and 1 of their
  // group, lanes 32..63 those of keys 2 and 3
  const auto s02 = __builtin_amdgcn_permlane32_swap(__float_as_uint(best[0]), __float_as_uint(best[2]), false, false);
  const auto s13 = __builtin_amdgcn_permlane32_swap(__float_as_uint(best[1]), __float_as_uint(best[3]), false, false);
  const f32x2 out = {fmaxf(__uint_as_float(s02[0]), __uint_as_float(s02[1])),
                     fmaxf(__uint_as_float(s13[0]), __uint_as_float(s13[1]))};
  // groups 0..7 lie in front of the block; in the range's first block they and group 8 (the range's
  // first four keys, whose windows reach in front of the range) are left to the fix-up kernel
  const bool emit = grp >= kUtilShift / 4 + 1 || !first_block;
  const uint32_t off_u =
      emit ? (uint32_t)((bc.g * a.P + t_first - kUtilShift + 4 * grp + 2 * half) * 4) : 0x80000000u;
  __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2_t, out), rsrc_u, off_u, 0, kOutStoreAux);
}

template <int DT, int DH, int NQ, int WT, bool UTIL = false, bool GSUM = false>
__global__ void __launch_bounds__(kScoreWaves *kWave) colsum_lds_kernel(ScoreArgs a) {
  static_assert(!(UTIL && GSUM) && (!GSUM || WT == 1), "one epilogue at a time; group sums take one tile per head");
  static_assert(NQ % WT == 0, "whole heads");
  using G = Geom<DT, DH>;
  constexpr int NCH = G::NCH;
  constexpr int N_MFMA = NCH * (DT == CKV_BF16 ? 1 : 4) + 1;
  constexpr int READ_AT = NQ >= 2 ? NQ - 2 : 0;
  __shared__ __attribute__((aligned(1024))) typename Staged<DT, DH, NQ>::Ring ring;
  const int lane = threadIdx.x & 63, m = lane & 31, hh = lane >> 5;
  const BlockCoord bc = decode_block(a);
  const WaveRange wr = wave_range(a, bc);

  Staged<DT, DH, NQ> st;
  chunk_t qf[NQ][NCH];
  int jrow[NQ];
  st.start(a, bc, wr, ring, lane, m, hh, qf, jrow);
  // bias of this lane's query row in every tile; padding rows (q = 0) get exp2(-1000) = 0 as weight
  Bias<DT> bias[NQ];
  const float to_raw = -kLog2e / a.c2;  // LSE (natural log) -> units of the raw dot product, negated
#pragma unroll
  for (int i = 0; i < NQ; ++i) {
    const int h = bc.g * a.G + (bc.grp * NQ + i) / WT;
    float lse_j = 0.0f;
    if (jrow[i] >= 0) {
      // same arithmetic as lse_kernel, which this saves when both passes run in one call
      if (a.lse_from_part)
        lse_j = merge_row_partials(
            a.part + (((size_t)bc.unit * a.n_groups + bc.grp) * (NQ * kTile) + i * kTile + m) * a.n_chunks, a.n_chunks);
      else lse_j = a.lse[((size_t)bc.b * a.Hq + h) * a.W + jrow[i]];
    }
    bias[i].set(jrow[i] >= 0 ? lse_j * to_raw : -1000.0f / a.c2, hh);
  }
  const chunk_t ones = Bias<DT>::ones(hh);
  // Descriptor over scores[b]: Hq * T floats (the host checks that this stays below 2 GiB). Lanes with
  // nothing to store present an offset outside it, which the hardware drops: no branch splits the
  // pipeline's code, and every flush issues exactly N_STORES store instructions.
  const int score_rows = GSUM ? a.Hkv : a.Hq;  // rows of a batch element in the output
  const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void *)(a.scores + (size_t)bc.b * score_rows * a.T), 0, score_rows * a.T * 4, 0x00020000);
  // Vector memory operations complete in issue order, stores included. When tile t + 1 is picked up,
  // the loads of tiles t + 2 and t + 3 were issued after its own, and so were the stores of the
  // previous ring cycle if t is the cycle's first or second tile; that many operations may still be
  // in flight. The first cycle has no such stores behind it: dropped stores (offset outside the
  // descriptor) issued after the first loads stand in.
  // per flush; the fused form adds the utility store, the group-sum form has a single store
  constexpr int N_STORES = GSUM ? 1 : (NQ / WT + 1) / 2 + (UTIL ? 1 : 0);
  __shared__ __attribute__((aligned(16))) float s_stage[kScoreWaves][(NQ / WT) * (UTIL ? kUtilRow : kRing * kTile)];
  // fused form: descriptor over utility[b] (Hkv * P floats) and the weights of this group's heads
  const __amdgpu_buffer_rsrc_t rsrc_u = __builtin_amdgcn_make_buffer_rsrc(
      (void *)(UTIL ? a.utility + (size_t)bc.b * a.Hkv * a.P : a.scores), 0, UTIL ? a.Hkv * a.P * 4 : 0, 0x00020000);
  float wgt[NQ / WT];
#pragma unroll
  for (int h = 0; h < NQ / WT; ++h) {
    const int head = bc.g * a.G + (bc.grp * NQ) / WT + h;
    wgt[h] = UTIL && head < a.Hq ? a.w_row[head] : 0.0f;
  }
  float *stage = s_stage[wr.wave];
  const int n_piped = wr.n_full / kRing * kRing;
  // (distinct offsets, all outside the descriptor: identical stores could be merged into one)
#pragma unroll
  for (int i = 0; i < N_STORES; ++i) __builtin_amdgcn_raw_buffer_store_b32(0u, rsrc, 0x80000000u + 64u * i, 0, 0);

  chunk_t kreg[2][NCH];
  f32x16 acc[2];
  if (n_piped > 0) {
    wait_vm<(kRing - 2) * G::NDMA>();
    read_image<G>(kreg[0], ring[wr.wave][0], st.roff);
    mma_chain<DT, NCH>(acc[0], qf[0], kreg[0]);
    bias[0].add(acc[0], ones);
  }
  constexpr int UR = unroll_tiles(NQ);
  for (int t0 = 0; t0 < n_piped; t0 += UR) {
    const int slot0 = UR == kRing ? 0 : (t0 & (kRing - 1));  // ring image of tile t0
#pragma unroll
    for (int v = 0; v < UR; ++v) {
      const int u = slot0 + v;
      st.prefetch(t0 + v, wr.n_full, (u + kRing - 1) % kRing);
      float cs[NQ];
#pragma unroll
      for (int i = 0; i < NQ; ++i) {
        const int cur = (v * NQ + i) & 1;
        if (i == READ_AT) {
          // tile t0 + v + 1 has landed. In the first half of a ring cycle the previous cycle's stores were
          // issued after its load and may still be in flight; where the half is only known at run time the
          // wait does not allow for them (stricter, never wrong).
          if (UR == kRing && v < 2) wait_vm<(kRing - 2) * G::NDMA + N_STORES>();
          else wait_vm<(kRing - 2) * G::NDMA>();
          read_image<G>(kreg[(v + 1) & 1], ring[wr.wave][(u + 1) % kRing], st.roff);
        }
        if (i + 1 < NQ) {
          mma_chain<DT, NCH>(acc[cur ^ 1], qf[i + 1], kreg[v & 1]);  // rows: query rows, cols: keys
          bias[i + 1].add(acc[cur ^ 1], ones);
        } else {
          mma_chain<DT, NCH>(acc[cur ^ 1], qf[0], kreg[(v + 1) & 1]);
          bias[0].add(acc[cur ^ 1], ones);
        }
        cs[i] = colsum_weights<false>(acc[cur], a.c2, hh, 0);
        if (i == READ_AT) interleave_hint<N_MFMA, vector_per_mfma_pass2(NQ), NCH>();
        else interleave_hint<N_MFMA, vector_per_mfma_pass2(NQ), 0>();
      }
      if constexpr (UTIL) stage_column_sums<NQ, WT, kUtilRow>(cs, a.norm, stage + kUtilCarry, u, m, hh);
      else stage_column_sums<NQ, WT>(cs, a.norm, stage, u, m, hh);
      st.kcur += st.tile_stride;
    }
    if (UR == kRing || slot0 + UR == kRing) {  // a ring cycle is complete
      const int c0 = t0 + UR - kRing;          // its first tile
      stage_fence();  // the tiles' sums are staged
      if constexpr (UTIL)
        flush_utility<NQ, WT>(a, bc, stage, wr.t_begin + c0 * kTile, c0 == 0, c0 + kRing >= n_piped, lane, rsrc, rsrc_u, wgt);
      else if constexpr (GSUM) flush_group_sums<NQ>(a, bc, stage, wr.t_begin + c0 * kTile, lane, rsrc);
      else flush_column_sums<NQ, WT>(a, bc, stage, wr.t_begin + c0 * kTile, lane, rsrc);
      stage_fence();  // and read, before the next cycle's overwrite them
    }
  }
  wait_vm<0>();
  for (int r0 = wr.t_begin + n_piped * kTile; r0 < wr.t_end; r0 += kRing * kTile) {  // loads a ring at a time
#pragma unroll
    for (int j = 0; j < kRing; ++j)
      if (r0 + j * kTile < wr.t_end) dma_tile_clamped<G>(st.kbase, a.ks_t, r0 + j * kTile, a.T, lane, ring[wr.wave][j]);
    wait_vm<0>();
    for (int j = 0; j < kRing && r0 + j * kTile < wr.t_end; ++j) {
      const int t0 = r0 + j * kTile;
      read_image<G>(kreg[0], ring[wr.wave][j], st.roff);
      const int kt = t0 + m;
      float cs[NQ];
#pragma unroll
      for (int i = 0; i < NQ; ++i) {
        const int j0 = ((bc.grp * NQ + i) % WT) * kTile;
        mma_chain<DT, NCH>(acc[0], qf[i], kreg[0]);
        bias[i].add(acc[0], ones);
        cs[i] = colsum_weights<true>(acc[0], a.c2, hh, kt - a.P - j0);
      }
      if constexpr (GSUM) store_group_sum<NQ>(a, bc, cs, kt, hh);
      else store_column_sums<NQ>(a, bc, cs, WT, kt, hh);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Launch
// ---------------------------------------------------------------------------------------------
template <int DT, int DH, int NQ>
static void launch_rowstats(const Shape &s, const ScoreArgs &a, dim3 grid, dim3 block, hipStream_t stream) {
  if constexpr (DT == CKV_BF16)
    hipLaunchKernelGGL((rowstats_lds_kernel<DT, DH, NQ>), grid, block, 0, stream, a);
  else
    hipLaunchKernelGGL((rowstats_kernel<DT, DH, NQ>), grid, block, 0, stream, a);
  if (a.lse_from_part) return;  // the second pass of the same call merges the partials itself
  const int rows = s.Bz * s.Hkv * s.n_groups * NQ * kTile;
  hipLaunchKernelGGL(lse_kernel<NQ>, dim3((rows + 255) / 256), dim3(256), 0, stream, a, rows);
}

// Whether launch_colsum takes the LDS-staged kernel (the one that can merge the row partials itself).
template <int DT, int NQ>
static bool colsum_is_staged(const Shape &s) {
  if (DT != CKV_BF16) return false;
  return s.WT >= 1 && s.WT <= kMaxWindowTiles && NQ % s.WT == 0;
}

template <int DT, int DH, int NQ>
static void launch_colsum(const Shape &s, const ScoreArgs &a, dim3 grid, dim3 block, hipStream_t stream) {
  if constexpr (DT == CKV_BF16) {
    // NQ is a multiple of WT (whole heads per wave)
    if (s.WT == 1) {
      if (a.utility) hipLaunchKernelGGL((colsum_lds_kernel<DT, DH, NQ, 1, true>), grid, block, 0, stream, a);
      else if (a.group_sum) {
        if constexpr (NQ <= 4) hipLaunchKernelGGL((colsum_lds_kernel<DT, DH, NQ, 1, false, true>), grid, block, 0, stream, a);
      } else hipLaunchKernelGGL((colsum_lds_kernel<DT, DH, NQ, 1>), grid, block, 0, stream, a);
      return;
    }
    if constexpr (NQ % 2 == 0) {
      if (s.WT == 2) {
        if (a.utility) hipLaunchKernelGGL((colsum_lds_kernel<DT, DH, NQ, 2, true>), grid, block, 0, stream, a);
        else hipLaunchKernelGGL((colsum_lds_kernel<DT, DH, NQ, 2>), grid, block, 0, stream, a);
        return;
      }
    }
    if constexpr (NQ % 3 == 0) {
      if (s.WT == 3) {
        hipLaunchKernelGGL((colsum_lds_kernel<DT, DH, NQ, 3>), grid, block, 0, stream, a);
        return;
      }
    }
    if constexpr (NQ % 4 == 0) {
      if (s.WT == 4) {
        hipLaunchKernelGGL((colsum_lds_kernel<DT, DH, NQ, 4>), grid, block, 0, stream, a);
        return;
      }
    }
  }
  hipLaunchKernelGGL((colsum_kernel<DT, DH, NQ>), grid, block, 0, stream, a);
}

// Where a lane has at most this many row partials to merge (query tiles per wave x workgroups along the key
// axis), the second pass merges the first pass's partials in its own prologue: every workgroup of a unit
// repeats the merge, which is cheaper than a launch while the partials are few. Beyond it the small merge
// kernel runs in between (measured at 8 tiles x 32 workgroups, T = 128k with 8 units: 26 us of prologue
// against 11 us for the kernel; at 4 x 8 the kernel still wins, at 4 x 2 and 1 x 8 the prologue does).
constexpr int kMergeInPassTwo = 16;

// Launches for the query-tile counts NQ_LO..NQ_HI (the instantiations are spread over several translation
// units, each covering a range, to keep compile times apart).
template <int DT, int DH, int NQ_LO, int NQ_HI>
static hipError_t launch_scores_t(const Shape &s, ScoreArgs &a, bool need_lse, bool need_scores, hipStream_t stream) {
  const int units = s.Bz * s.Hkv;
  const dim3 grid((unsigned)((size_t)units * s.n_groups * s.n_chunks)), block(kScoreWaves * kWave);
#define CKV_LAUNCH_NQ(NQ)                                                          \
  case NQ:                                                                         \
    if constexpr (NQ >= NQ_LO && NQ <= NQ_HI) {                                    \
      a.lse_from_part = need_lse && need_scores && colsum_is_staged<DT, NQ>(s) && \
                        NQ * s.n_chunks <= kMergeInPassTwo;                         \
      if (need_lse) launch_rowstats<DT, DH, NQ>(s, a, grid, block, stream);        \
      if (need_scores) launch_colsum<DT, DH, NQ>(s, a, grid, block, stream);       \
      break;                                                                       \
    }                                                                              \
    return hipErrorInvalidValue;
  switch (s.NQ) {
    CKV_LAUNCH_NQ(1)
    CKV_LAUNCH_NQ(2)
    CKV_LAUNCH_NQ(3)
    CKV_LAUNCH_NQ(4)
    CKV_LAUNCH_NQ(5)
    CKV_LAUNCH_NQ(6)
    CKV_LAUNCH_NQ(7)
    CKV_LAUNCH_NQ(8)
    default: return hipErrorInvalidValue;
  }
#undef CKV_LAUNCH_NQ
  return hipGetLastError();
}


// One definition per (element type, head size, range of query-tile counts), each in a translation unit of
// its own.
#define CKV_DECLARE_SCAN(name) \
  hipError_t name(const Shape &s, ScoreArgs &a, bool need_lse, bool need_scores, hipStream_t stream)
CKV_DECLARE_SCAN(launch_scores_bf16_d128);       // 1..4 query tiles per wave
CKV_DECLARE_SCAN(launch_scores_bf16_d128_nq56);
CKV_DECLARE_SCAN(launch_scores_bf16_d128_nq78);
CKV_DECLARE_SCAN(launch_scores_bf16_d64);
CKV_DECLARE_SCAN(launch_scores_bf16_d64_nq56);
CKV_DECLARE_SCAN(launch_scores_bf16_d64_nq78);
CKV_DECLARE_SCAN(launch_scores_f32_d128);
CKV_DECLARE_SCAN(launch_scores_f32_d64);

}  // namespace ckv
#endif
