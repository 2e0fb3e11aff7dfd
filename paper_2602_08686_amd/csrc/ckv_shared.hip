// Layer-shared mode: the paper's Alg. 1 as printed. One window mass alpha per prompt, the mean of the
// per-head masses over all layers and heads (Eq. 4, Alg. 1 (A)); the structural risk coordinate
// R_struct = H(alpha / ||alpha||_1) and its bin (Eq. 7, Alg. 1 (A)); per layer one utility vector
// u_hat = max over ALL heads of W_head[l,h] * alpha * rho^(l,h) (Eq. 4, Eq. 6, Alg. 1 (B)-(C)). The
// selection reuses the per-head kernels with one "head" per batch element; the gather of the shared
// index set is a mode of the gather kernel. All of it is a few passes over [Bz,T] vectors: HBM-bound,
// small next to the scan that produces the per-head masses.
#include "ckv_internal.h"

namespace ckv {

typedef __attribute__((ext_vector_type(4))) float f32x4_s;

struct AlphaArgs {
  const float *scores;  // [Bz][Hq][T] (Hq = rows per batch element: query heads, or KV heads of group masses)
  float *alpha;         // [Bz][T], read and written
  float weight;
  int Hq, T;
};

// One thread per four (or one) positions: alpha += weight * sum over heads, heads added in order.
template <bool VEC>
__global__ void __launch_bounds__(256) alpha_accumulate_kernel(AlphaArgs a) {
  const int b = blockIdx.y;
  const float *s = a.scores + (size_t)b * a.Hq * a.T;
  float *al = a.alpha + (size_t)b * a.T;
  if (VEC) {
    const int t = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (t >= a.T) return;
    f32x4_s acc = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int h = 0; h < a.Hq; ++h) acc += *reinterpret_cast<const f32x4_s *>(s + (size_t)h * a.T + t);
    f32x4_s cur = *reinterpret_cast<const f32x4_s *>(al + t);
#pragma unroll
    for (int e = 0; e < 4; ++e) cur[e] = fmaf(a.weight, acc[e], cur[e]);
    *reinterpret_cast<f32x4_s *>(al + t) = cur;
  } else {
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= a.T) return;
    float acc = 0.0f;
    for (int h = 0; h < a.Hq; ++h) acc += s[(size_t)h * a.T + t];
    al[t] = fmaf(a.weight, acc, al[t]);
  }
}

struct RiskArgs {
  const float *alpha;  // [Bz][T]
  const float *edges;  // ascending, or null
  int n_edges, T;
  float *risk;         // [Bz]
  int32_t *bin;        // [Bz] or null
};
constexpr int kRiskThreads = 1024;

// One workgroup per prompt. With S = sum alpha: H = ln S - (sum alpha ln alpha) / S. Sums in double,
// thread-strided partials combined by a fixed tree: bit-stable from run to run.
__global__ void __launch_bounds__(kRiskThreads) risk_struct_kernel(RiskArgs a) {
  __shared__ double s1[kRiskThreads], s2[kRiskThreads];
  const int b = blockIdx.x, tid = threadIdx.x;
  const float *al = a.alpha + (size_t)b * a.T;
  double p1 = 0.0, p2 = 0.0;
  for (int t = tid; t < a.T; t += kRiskThreads) {
    const double x = (double)al[t];
    if (x > 0.0) {
      p1 += x;
      p2 += x * log(x);
    }
  }
  s1[tid] = p1;
  s2[tid] = p2;
  __syncthreads();
  for (int o = kRiskThreads / 2; o > 0; o >>= 1) {
    if (tid < o) {
      s1[tid] += s1[tid + o];
      s2[tid] += s2[tid + o];
    }
    __syncthreads();
  }
  if (tid == 0) {
    const double S = s1[0];
    const float h = S > 0.0 ? (float)(log(S) - s2[0] / S) : 0.0f;
    a.risk[b] = h;
    if (a.bin) {
      int n = 0;
      for (int i = 0; i < a.n_edges; ++i) n += a.edges[i] <= h ? 1 : 0;
      a.bin[b] = n;
    }
  }
}

struct SharedUtilArgs {
  const float *alpha;  // [Bz][T]
  const float *rho;    // [Bz][Hkv][T]
  const float *w_row;  // [Hq]
  const float *gate_layer;
  const int32_t *risk_bins;
  int n_ent, n_ppl;
  float *utility;      // [Bz][P]
  float *tau;          // [Bz]
  int Hkv, G, T, P;
};

__global__ void __launch_bounds__(256) shared_utility_kernel(SharedUtilArgs a) {
  const int b = blockIdx.y, t = blockIdx.x * 256 + threadIdx.x;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    float tau = 0.0f;
    if (a.gate_layer) {
      const int be = min(max(a.risk_bins[2 * b], 0), a.n_ent - 1);
      const int bp = min(max(a.risk_bins[2 * b + 1], 0), a.n_ppl - 1);
      tau = a.gate_layer[be * a.n_ppl + bp];
    }
    a.tau[b] = tau;
  }
  if (t >= a.P) return;
  const float al = a.alpha[(size_t)b * a.T + t];
  float best = -INFINITY;
  for (int g = 0; g < a.Hkv; ++g) {
    const float u = al * a.rho[((size_t)b * a.Hkv + g) * a.T + t];  // u^(l,h) of every head of the group
    for (int hg = 0; hg < a.G; ++hg) best = fmaxf(best, a.w_row[g * a.G + hg] * u);
  }
  a.utility[(size_t)b * a.P + t] = best;
}

hipError_t launch_alpha_accumulate(const Shape &s, int rows, const float *scores, float weight, float *alpha,
                                   hipStream_t stream) {
  AlphaArgs a;
  a.scores = scores;
  a.alpha = alpha;
  a.weight = weight;
  a.Hq = rows;
  a.T = s.T;
  const bool vec = s.T % 4 == 0 && (uintptr_t)scores % 16 == 0 && (uintptr_t)alpha % 16 == 0;
  if (vec) hipLaunchKernelGGL(alpha_accumulate_kernel<true>, dim3((s.T / 4 + 255) / 256, s.Bz), dim3(256), 0, stream, a);
  else hipLaunchKernelGGL(alpha_accumulate_kernel<false>, dim3((s.T + 255) / 256, s.Bz), dim3(256), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_risk_struct(const Shape &s, const float *alpha, const float *edges, int n_edges, float *risk,
                              int32_t *bin, hipStream_t stream) {
  RiskArgs a;
  a.alpha = alpha;
  a.edges = edges;
  a.n_edges = edges ? n_edges : 0;
  a.T = s.T;
  a.risk = risk;
  a.bin = bin;
  hipLaunchKernelGGL(risk_struct_kernel, dim3(s.Bz), dim3(kRiskThreads), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_shared_utility(const ckv_params *p, const Shape &s, const float *alpha, const float *rho,
                                 const float *w_head, const float *t_gate, int n_ent, int n_ppl,
                                 const int32_t *risk_bins, float *utility, float *tau, hipStream_t stream) {
  SharedUtilArgs a;
  a.alpha = alpha;
  a.rho = rho;
  a.w_row = w_head + (size_t)p->layer * s.Hq;
  a.gate_layer = t_gate ? t_gate + (size_t)p->layer * n_ent * n_ppl : nullptr;
  a.risk_bins = risk_bins;
  a.n_ent = n_ent;
  a.n_ppl = n_ppl;
  a.utility = utility;
  a.tau = tau;
  a.Hkv = s.Hkv;
  a.G = s.G;
  a.T = s.T;
  a.P = s.P;
  const int blocks = s.P > 0 ? (s.P + 255) / 256 : 1;
  hipLaunchKernelGGL(shared_utility_kernel, dim3(blocks, s.Bz), dim3(256), 0, stream, a);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Depth mapping of a compiled table (paper App., "Model choice and cross-architecture applicability"):
// relative-depth linear interpolation of the rows of a table compiled on n_src layers to n_dst layers.
// Table preparation, not part of the per-layer path: one thread per output element.
// ---------------------------------------------------------------------------------------------
struct DepthArgs {
  const float *src;  // [n_src][row]
  float *dst;        // [n_dst][row]
  int n_src, n_dst, row;
};

__global__ void __launch_bounds__(256) map_depth_kernel(DepthArgs a) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= a.n_dst * a.row) return;
  const int l = i / a.row, c = i % a.row;
  // x = l (n_src - 1) / (n_dst - 1) in double: the row index and the weight are exact for the table sizes in use
  const double x = a.n_dst == 1 ? 0.0 : (double)l * (double)(a.n_src - 1) / (double)(a.n_dst - 1);
  const int lo = min((int)floor(x), a.n_src - 1), hi = min(lo + 1, a.n_src - 1);
  const double f = x - (double)lo;
  a.dst[i] = (float)((1.0 - f) * (double)a.src[(size_t)lo * a.row + c] + f * (double)a.src[(size_t)hi * a.row + c]);
}

hipError_t launch_map_depth(const float *src, int n_src, int row, float *dst, int n_dst, hipStream_t stream) {
  DepthArgs a;
  a.src = src;
  a.dst = dst;
  a.n_src = n_src;
  a.n_dst = n_dst;
  a.row = row;
  const int n = n_dst * row;
  hipLaunchKernelGGL(map_depth_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, a);
  return hipGetLastError();
}

}  // namespace ckv
