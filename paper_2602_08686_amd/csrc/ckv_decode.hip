// Decode-side consumer of the compact cache (paper Sec. 4.5, Proposition 1 and its proof in App. A).
// A decoding query sits after the prompt, so it sees every row of a KV set; over the retained set its
// attention row is the full row restricted to S and renormalised (p~ of the Proposition), and the mass
// the full row had outside S is m = 1 - exp(lse_S - lse_full).
//
// decode_partial_kernel: attention of one decoding query per (batch, query head) over a ragged KV set
// (the first count[b,g] rows of each (batch, KV head)), the query heads of a GQA group sharing each K/V
// row they read. HBM-bound (every valid K and V row once, 2 * rows * d * e bytes per unit); the
// arithmetic is 4 * G * d flops per row pair, far below the vector rate needed to keep up, so the
// products run on the vector ALUs in fp32 -- with one to eight query rows per K row there is no
// matrix-core tile to fill. A 16-byte piece of a row per lane (d * e / 16 lanes per row, several rows
// per wave step, whole rows coalesced), four row steps in flight, online softmax in the log2 domain;
// the key axis is cut into chunks over workgroups and decode_merge_kernel combines the partial
// (max, sum, weighted V) triples in a fixed order (bit-stable).
#include "ckv_internal.h"

namespace ckv {

struct DecodeArgs {
  const void *q;         // [Bz][Hq][n_q][d]
  const void *k, *v;     // rows of (batch, kv head) through the strides below
  const int32_t *count;  // [Bz*Hkv] valid rows, or null: all n_rows
  int64_t ks[3], vs[3];  // element strides over (batch, kv head, row)
  float *part;           // [grid.y][n_chunks][RQ][d + 2]: weighted V sum, running max (log2), sum
  float *out;            // [Bz][Hq][n_q][d]
  float *lse;            // [Bz][Hq][n_q] natural log
  int Hq, Hkv, G, n_q, n_rows, rows_per_chunk, n_chunks, head_chunks;
  float scale2;          // softmax scale * log2(e)
};

constexpr int kXcds = 8;  // accelerator dies of the part; workgroup i of a launch runs on die i % 8
constexpr int kDecodeThreads = 256;
constexpr int kDecodeWaves = kDecodeThreads / kWave;

template <int DT>
struct Piece;  // a 16-byte piece of a row as floats
template <>
struct Piece<CKV_BF16> {
  static constexpr int E = 8;
  __device__ static __forceinline__ void to_float(const uint4 &raw, float (&f)[8]) {
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __uint_as_float(w[i] << 16);
      f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
};
template <>
struct Piece<CKV_F32> {
  static constexpr int E = 4;
  __device__ static __forceinline__ void to_float(const uint4 &raw, float (&f)[4]) {
    f[0] = __uint_as_float(raw.x);
    f[1] = __uint_as_float(raw.y);
    f[2] = __uint_as_float(raw.z);
    f[3] = __uint_as_float(raw.w);
  }
};

// exp2(a - b) with the conventions of an online softmax: a = -inf gives 0 also when b was reset to 0
__device__ __forceinline__ float exp2_diff(float a, float b) { return exp2f(a - b); }

// NW waves per workgroup, U row steps whose loads are in flight together (PIPE: of the next block too). With one chunk per
// (unit, query) the workgroup writes the final result itself and no merge kernel follows.
template <int DT, int DH, int RQ, int NW, int U, bool PIPE>
__global__ void __launch_bounds__(NW *kWave) decode_partial_kernel(DecodeArgs a) {
  constexpr int E = Piece<DT>::E;
  constexpr int ESIZE = 16 / E;
  constexpr int LPR = DH / E;        // lanes per row
  constexpr int KPW = kWave / LPR;   // rows per wave step
  constexpr int ROW = DH + 2;
  constexpr bool STREAM = NW == kDecodeWaves;  // the chunked form sweeps long caches once: streaming loads
  __shared__ float sm[NW][RQ][ROW];

  const int chunk = blockIdx.x;
  int y = blockIdx.y;
  // One launch over a short KV set: the workgroups that read the same rows (the head chunks of a unit) are
  // consecutive in y, and consecutive workgroups go to different XCDs, each with an L2 of its own -- the
  // rows would come from HBM once per head chunk. Within groups of 8 * head_chunks workgroups the index is
  // transposed, so that a unit's head chunks are 8 apart: same XCD, the second reader hits its L2.
  if (PIPE && a.head_chunks > 1) {
    const int span = kXcds * a.head_chunks, base = y / span * span;
    if (base + span <= (int)gridDim.y) {
      const int j = y - base;
      y = base + (j % kXcds) * a.head_chunks + j / kXcds;
    }
  }
  const int hc = y % a.head_chunks;
  y /= a.head_chunks;
  const int qi = y % a.n_q, unit = y / a.n_q;
  const int b = unit / a.Hkv, g = unit % a.Hkv;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int sub = lane % LPR, slot = lane / LPR;
  int n_valid = a.n_rows;
  if (a.count) n_valid = min(max(a.count[unit], 0), a.n_rows);
  const int r0 = chunk * a.rows_per_chunk, r1 = min(r0 + a.rows_per_chunk, n_valid);
  const bool single = a.n_chunks == 1;
  if (r0 >= r1 && !single) return;  // the merge reads the chunks below n_valid only

  float qv[RQ][E];
#pragma unroll
  for (int r = 0; r < RQ; ++r) {
    const int hg = hc * RQ + r;
    uint4 raw = make_uint4(0u, 0u, 0u, 0u);
    if (hg < a.G) {
      const size_t row = ((size_t)b * a.Hq + (size_t)g * a.G + hg) * a.n_q + qi;
      raw = *reinterpret_cast<const uint4 *>(static_cast<const char *>(a.q) + (row * DH + sub * E) * ESIZE);
    }
    Piece<DT>::to_float(raw, qv[r]);
#pragma unroll
    for (int e = 0; e < E; ++e) qv[r][e] *= a.scale2;
  }

  float m[RQ], l[RQ], acc[RQ][E];
#pragma unroll
  for (int r = 0; r < RQ; ++r) {
    m[r] = -INFINITY;
    l[r] = 0.0f;
#pragma unroll
    for (int e = 0; e < E; ++e) acc[r][e] = 0.0f;
  }

  const char *kb = static_cast<const char *>(a.k) + ((size_t)b * a.ks[0] + (size_t)g * a.ks[1]) * ESIZE;
  const char *vb = static_cast<const char *>(a.v) + ((size_t)b * a.vs[0] + (size_t)g * a.vs[1]) * ESIZE;
  // a wave takes KPW * U consecutive rows at a time; the workgroup's waves interleave such blocks
  // The loads of the wave's next block are issued before the current block is worked on: a short KV set
  // is a handful of dependent round trips otherwise.
  auto load_block = [&](int base, uint4 (&kraw)[U], uint4 (&vraw)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int row = base + u * KPW + slot;
      kraw[u] = make_uint4(0u, 0u, 0u, 0u);
      vraw[u] = make_uint4(0u, 0u, 0u, 0u);
      if (row < r1) {
        kraw[u] = load_piece<STREAM>(kb + ((size_t)row * a.ks[2] + sub * E) * ESIZE);
        vraw[u] = load_piece<STREAM>(vb + ((size_t)row * a.vs[2] + sub * E) * ESIZE);
      }
    }
  };
  uint4 kraw[U], vraw[U];
  const int base0 = r0 + wave * KPW * U;
  if (base0 < r1) load_block(base0, kraw, vraw);
  for (int base = base0; base < r1; base += NW * KPW * U) {
    uint4 knext[U], vnext[U];
    if (PIPE) load_block(base + NW * KPW * U, knext, vnext);  // rows at and beyond r1 are not read
    float s[U][RQ], vf[U][E];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float kf[E];
      Piece<DT>::to_float(kraw[u], kf);
      Piece<DT>::to_float(vraw[u], vf[u]);
      const bool ok = base + u * KPW + slot < r1;
#pragma unroll
      for (int r = 0; r < RQ; ++r) {
        float dot = 0.0f;
#pragma unroll
        for (int e = 0; e < E; ++e) dot = fmaf(qv[r][e], kf[e], dot);
        dot = row_sum<LPR>(dot);  // the row's lanes all end with the sum
        s[u][r] = ok ? dot : -INFINITY;
      }
    }
#pragma unroll
    for (int r = 0; r < RQ; ++r) {
      float mx = s[0][r];
#pragma unroll
      for (int u = 1; u < U; ++u) mx = fmaxf(mx, s[u][r]);
      const float m_new = fmaxf(m[r], mx);
      const float ref = m_new == -INFINITY ? 0.0f : m_new;
      const float keep = exp2_diff(m[r], ref);
      l[r] *= keep;
#pragma unroll
      for (int e = 0; e < E; ++e) acc[r][e] *= keep;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const float p = exp2_diff(s[u][r], ref);
        l[r] += p;
#pragma unroll
        for (int e = 0; e < E; ++e) acc[r][e] = fmaf(p, vf[u][e], acc[r][e]);
      }
      m[r] = m_new;
    }
    if (PIPE) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        kraw[u] = knext[u];
        vraw[u] = vnext[u];
      }
    } else if (base + NW * KPW * U < r1) {
      load_block(base + NW * KPW * U, kraw, vraw);
    }
  }

  // the wave's row slots, in a fixed butterfly order
#pragma unroll
  for (int o = LPR; o < kWave; o <<= 1) {
#pragma unroll
    for (int r = 0; r < RQ; ++r) {
      const float m_o = __shfl_xor(m[r], o), l_o = __shfl_xor(l[r], o);
      const float m_new = fmaxf(m[r], m_o);
      const float ref = m_new == -INFINITY ? 0.0f : m_new;
      // both partners must add in the same order for identical results: lower lane's value first
      const bool low = (lane & o) == 0;
      const float f_self = exp2_diff(m[r], ref), f_other = exp2_diff(m_o, ref);
      l[r] = low ? fmaf(l[r], f_self, l_o * f_other) : fmaf(l_o, f_other, l[r] * f_self);
#pragma unroll
      for (int e = 0; e < E; ++e) {
        const float a_o = __shfl_xor(acc[r][e], o);
        acc[r][e] = low ? fmaf(acc[r][e], f_self, a_o * f_other) : fmaf(a_o, f_other, acc[r][e] * f_self);
      }
      m[r] = m_new;
    }
  }
  if (slot == 0) {
#pragma unroll
    for (int r = 0; r < RQ; ++r) {
#pragma unroll
      for (int e = 0; e < E; ++e) sm[wave][r][sub * E + e] = acc[r][e];
      if (sub == 0) {
        sm[wave][r][DH] = m[r];
        sm[wave][r][DH + 1] = l[r];
      }
    }
  }
  __syncthreads();
  if (single) {
    for (int i = tid; i < RQ * DH; i += NW * kWave) {
      const int r = i / DH, c = i % DH;
      const int hg = hc * RQ + r;
      if (hg >= a.G) continue;
      float top = sm[0][r][DH];
#pragma unroll
      for (int w = 1; w < NW; ++w) top = fmaxf(top, sm[w][r][DH]);
      const float ref = top == -INFINITY ? 0.0f : top;
      float num = 0.0f, den = 0.0f;
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        const float f = exp2_diff(sm[w][r][DH], ref);
        num = fmaf(sm[w][r][c], f, num);
        den = fmaf(sm[w][r][DH + 1], f, den);
      }
      const size_t row = ((size_t)b * a.Hq + (size_t)g * a.G + hg) * a.n_q + qi;
      a.out[row * DH + c] = den > 0.0f ? num / den : 0.0f;
      if (c == 0) a.lse[row] = den > 0.0f ? (top + log2f(den)) * kLn2 : -INFINITY;
    }
    return;
  }
  float *part = a.part + ((size_t)blockIdx.y * a.n_chunks + chunk) * RQ * ROW;
  for (int i = tid; i < RQ * ROW; i += NW * kWave) {
    const int r = i / ROW, c = i % ROW;
    float top = sm[0][r][DH];
#pragma unroll
    for (int w = 1; w < NW; ++w) top = fmaxf(top, sm[w][r][DH]);
    const float ref = top == -INFINITY ? 0.0f : top;
    float val;
    if (c == DH) val = top;
    else {
      const int src = c < DH ? c : DH + 1;  // a V component, or the sum
      val = 0.0f;
#pragma unroll
      for (int w = 0; w < NW; ++w) val = fmaf(sm[w][r][src], exp2_diff(sm[w][r][DH], ref), val);
    }
    part[i] = val;
  }
}

constexpr int kMergeBatch = 16;  // chunks whose partials are loaded together

template <int DH, int RQ>
__global__ void __launch_bounds__(kDecodeThreads) decode_merge_kernel(DecodeArgs a) {
  constexpr int ROW = DH + 2;
  int y = blockIdx.x;
  const int hc = y % a.head_chunks;
  y /= a.head_chunks;
  const int qi = y % a.n_q, unit = y / a.n_q;
  const int b = unit / a.Hkv, g = unit % a.Hkv;
  int n_valid = a.n_rows;
  if (a.count) n_valid = min(max(a.count[unit], 0), a.n_rows);
  const int n_chunks = (n_valid + a.rows_per_chunk - 1) / a.rows_per_chunk;  // the chunks that were written
  const float *part = a.part + (size_t)blockIdx.x * a.n_chunks * RQ * ROW;
  for (int i = threadIdx.x; i < RQ * DH; i += kDecodeThreads) {
    const int r = i / DH, c = i % DH;
    const int hg = hc * RQ + r;
    if (hg >= a.G) continue;
    // online merge in chunk order, a batch of independent loads at a time
    float top = -INFINITY, num = 0.0f, den = 0.0f;
    for (int c0 = 0; c0 < n_chunks; c0 += kMergeBatch) {
      float pm[kMergeBatch], pl[kMergeBatch], pa[kMergeBatch];
#pragma unroll
      for (int j = 0; j < kMergeBatch; ++j) {
        const bool ok = c0 + j < n_chunks;
        const float *p = part + ((size_t)(ok ? c0 + j : 0) * RQ + r) * ROW;
        pm[j] = ok ? p[DH] : -INFINITY;
        pl[j] = ok ? p[DH + 1] : 0.0f;
        pa[j] = ok ? p[c] : 0.0f;
      }
      float mx = pm[0];
#pragma unroll
      for (int j = 1; j < kMergeBatch; ++j) mx = fmaxf(mx, pm[j]);
      const float m_new = fmaxf(top, mx);
      const float ref = m_new == -INFINITY ? 0.0f : m_new;
      const float keep = exp2_diff(top, ref);
      num *= keep;
      den *= keep;
#pragma unroll
      for (int j = 0; j < kMergeBatch; ++j) {
        const float f = exp2_diff(pm[j], ref);
        num = fmaf(pa[j], f, num);
        den = fmaf(pl[j], f, den);
      }
      top = m_new;
    }
    const size_t row = ((size_t)b * a.Hq + (size_t)g * a.G + hg) * a.n_q + qi;
    a.out[row * DH + c] = den > 0.0f ? num / den : 0.0f;
    if (c == 0) a.lse[row] = den > 0.0f ? (top + log2f(den)) * kLn2 : -INFINITY;
  }
}

// ---------------------------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------------------------
static int query_rows_per_pass(int G) { return G >= 8 ? 8 : G > 2 ? 4 : G; }  // 1, 2, 4, 8 (G = 3 pads to 4)

DecodePlan plan_decode(const Shape &s, int n_q, int n_rows) {
  DecodePlan p;
  p.rq = query_rows_per_pass(s.G);
  p.head_chunks = (s.G + p.rq - 1) / p.rq;
  p.grid_y = (int64_t)s.Bz * s.Hkv * n_q * p.head_chunks;
  // Short KV sets (a compact cache): one large workgroup per (unit, query, pair of heads) finishes the job
  // in one launch -- a decoding step is a chain of dependent layers, so a second launch costs more than
  // reading the few rows once per pair of heads, and two heads per workgroup leave registers for sixteen
  // waves with the loads of two blocks of rows in flight each.
  if (n_rows <= 4096 || (p.grid_y >= 1024 && n_rows <= 16384)) {
    p.rq = s.G >= 2 ? 2 : 1;
    p.head_chunks = (s.G + p.rq - 1) / p.rq;
    p.grid_y = (int64_t)s.Bz * s.Hkv * n_q * p.head_chunks;
    p.rows_per_chunk = (n_rows + 63) / 64 * 64;
    p.n_chunks = 1;
    p.workspace_bytes = 0;
    return p;
  }
  // enough workgroups to fill the chip several times, chunks of at least 64 rows (one step of a
  // workgroup's four waves), at most 64 chunks
  const int64_t want = (4096 + p.grid_y - 1) / p.grid_y;
  int64_t chunks = (n_rows + 63) / 64;
  if (chunks > want) chunks = want;
  if (chunks > 64) chunks = 64;
  if (chunks < 1) chunks = 1;
  int64_t rows = (n_rows + chunks - 1) / chunks;
  rows = (rows + 63) / 64 * 64;
  p.rows_per_chunk = (int)rows;
  p.n_chunks = (int)((n_rows + rows - 1) / rows);
  p.workspace_bytes = (size_t)p.grid_y * p.n_chunks * p.rq * (s.d + 2) * sizeof(float);
  return p;
}

template <int DT, int DH, int RQ>
static void launch_decode_t(const DecodeArgs &a, const DecodePlan &p, hipStream_t stream) {
  if (p.n_chunks == 1) {
    if constexpr (RQ <= 2)
      hipLaunchKernelGGL((decode_partial_kernel<DT, DH, RQ, 16, 2, true>), dim3(1, (unsigned)p.grid_y),
                         dim3(16 * kWave), 0, stream, a);
    return;
  }
  hipLaunchKernelGGL((decode_partial_kernel<DT, DH, RQ, kDecodeWaves, 4, false>), dim3(p.n_chunks, (unsigned)p.grid_y),
                     dim3(kDecodeThreads), 0, stream, a);
  hipLaunchKernelGGL((decode_merge_kernel<DH, RQ>), dim3((unsigned)p.grid_y), dim3(kDecodeThreads), 0, stream, a);
}

template <int DT, int DH>
static void launch_decode_rq(const DecodeArgs &a, const DecodePlan &p, hipStream_t stream) {
  switch (p.rq) {
    case 1: launch_decode_t<DT, DH, 1>(a, p, stream); break;
    case 2: launch_decode_t<DT, DH, 2>(a, p, stream); break;
    case 4: launch_decode_t<DT, DH, 4>(a, p, stream); break;
    default: launch_decode_t<DT, DH, 8>(a, p, stream); break;
  }
}

hipError_t launch_decode_attention(const ckv_params *p, const Shape &s, const void *q_dec, int n_q, const void *k_rows,
                                   const void *v_rows, const int64_t *k_stride, const int64_t *v_stride, int n_rows,
                                   const int32_t *count, float *out, float *lse, char *ws, hipStream_t stream) {
  const DecodePlan plan = plan_decode(s, n_q, n_rows);
  DecodeArgs a;
  a.q = q_dec;
  a.k = k_rows;
  a.v = v_rows;
  a.count = count;
  for (int i = 0; i < 3; ++i) {
    a.ks[i] = k_stride[i];
    a.vs[i] = v_stride[i];
  }
  a.part = reinterpret_cast<float *>(ws);
  a.out = out;
  a.lse = lse;
  a.Hq = s.Hq; a.Hkv = s.Hkv; a.G = s.G;
  a.n_q = n_q;
  a.n_rows = n_rows;
  a.rows_per_chunk = plan.rows_per_chunk;
  a.n_chunks = plan.n_chunks;
  a.head_chunks = plan.head_chunks;
  a.scale2 = s.scale * kLog2e;
  if (p->dtype == CKV_BF16) {
    if (s.d == 128) launch_decode_rq<CKV_BF16, 128>(a, plan, stream);
    else launch_decode_rq<CKV_BF16, 64>(a, plan, stream);
  } else {
    if (s.d == 128) launch_decode_rq<CKV_F32, 128>(a, plan, stream);
    else launch_decode_rq<CKV_F32, 64>(a, plan, stream);
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Discarded mass and tail epsilon from the two normalisers
// ---------------------------------------------------------------------------------------------
struct MassArgs {
  const float *lse_full, *lse_kept;  // [rows][n_q]
  float *mass;                       // [rows][n_q]
  float *eps;                        // [rows] or null
  int rows, n_q;
};

__global__ void __launch_bounds__(256) discarded_mass_kernel(MassArgs a) {
  const int row = blockIdx.x * 256 + threadIdx.x;
  if (row >= a.rows) return;
  float sq = 0.0f;
  for (int i = 0; i < a.n_q; ++i) {
    const size_t j = (size_t)row * a.n_q + i;
    // retained mass exp(lse_S - lse) <= 1; expm1 keeps small discarded masses accurate
    float m = -expm1f(a.lse_kept[j] - a.lse_full[j]);
    m = fminf(fmaxf(m, 0.0f), 1.0f);
    a.mass[j] = m;
    sq = fmaf(m, m, sq);
  }
  if (a.eps) a.eps[row] = sqrtf(sq / (float)a.n_q);
}

hipError_t launch_discarded_mass(const Shape &s, int n_q, const float *lse_full, const float *lse_kept, float *mass,
                                 float *eps, hipStream_t stream) {
  MassArgs a;
  a.lse_full = lse_full;
  a.lse_kept = lse_kept;
  a.mass = mass;
  a.eps = eps;
  a.rows = s.Bz * s.Hq;
  a.n_q = n_q;
  hipLaunchKernelGGL(discarded_mass_kernel, dim3((a.rows + 255) / 256), dim3(256), 0, stream, a);
  return hipGetLastError();
}

}  // namespace ckv
