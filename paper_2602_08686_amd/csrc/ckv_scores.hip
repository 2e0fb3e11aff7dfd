// Observation-window scan, host side: fills the kernel arguments and dispatches on element type and
// head size; each (type, size) pair is compiled in a translation unit of its own (ckv_scan_*.hip) from
// the templates in ckv_scan.h. Also the value-norm ratio rho of Eq. 4 (two small kernels).
#include "ckv_scan.h"

namespace ckv {

hipError_t launch_window_scores(const ckv_params *p, const Shape &s, const Workspace &w, const void *q,
                                const void *k, const float *lse_in, float *lse_out, float *scores,
                                char *ws, hipStream_t stream, const UtilityFusion *fuse) {
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
  a.lse_from_part = 0;
  a.group_sum = (p->flags & CKV_FLAG_GROUP_MASS) && !fuse ? 1 : 0;
  a.w_row = fuse ? fuse->w_row : nullptr;
  a.utility = fuse ? fuse->utility : nullptr;
  a.pool = fuse ? fuse->pool : CKV_POOL_NONE;
  a.radius = fuse ? fuse->radius : 0;
  a.inv_kernel = fuse ? fuse->inv_kernel : 1.0f;
  const bool need_lse = lse_in == nullptr, need_scores = scores != nullptr;
  if (p->dtype == CKV_BF16) {
    if (s.d == 128) {
      if (s.NQ <= 4) return launch_scores_bf16_d128(s, a, need_lse, need_scores, stream);
      if (s.NQ <= 6) return launch_scores_bf16_d128_nq56(s, a, need_lse, need_scores, stream);
      return launch_scores_bf16_d128_nq78(s, a, need_lse, need_scores, stream);
    }
    if (s.NQ <= 4) return launch_scores_bf16_d64(s, a, need_lse, need_scores, stream);
    if (s.NQ <= 6) return launch_scores_bf16_d64_nq56(s, a, need_lse, need_scores, stream);
    return launch_scores_bf16_d64_nq78(s, a, need_lse, need_scores, stream);
  }
  if (s.d == 128) return launch_scores_f32_d128(s, a, need_lse, need_scores, stream);
  return launch_scores_f32_d64(s, a, need_lse, need_scores, stream);
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
  float *utility;  // [units][P] multiplied by the ratio in the scaling pass, or null
  int P;
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
  constexpr int RPI = 256 / LPR;  // rows per step of the workgroup
  constexpr int U = 8;            // steps whose loads are in flight together
  typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_v;
  for (int r0 = rloc; r0 < kVnormRows; r0 += U * RPI) {
    u32x4_v c[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int t = blk * kVnormRows + r0 + u * RPI;
      c[u] = u32x4_v{0u, 0u, 0u, 0u};
      // V is read once: streaming (non-temporal) loads
      if (r0 + u * RPI < kVnormRows && t < a.T)
        c[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_v *>(base + (int64_t)t * a.vs_t + sub * 16));
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int t = blk * kVnormRows + r0 + u * RPI;
      float sq = 0.0f;
      if (DT == CKV_BF16) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const uint32_t pair = c[u][e];
          const float lo = __uint_as_float(pair << 16);
          const float hi = __uint_as_float(pair & 0xffff0000u);
          sq = fmaf(lo, lo, sq);
          sq = fmaf(hi, hi, sq);
        }
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const uint32_t word = c[u][e];
          const float x = __uint_as_float(word);
          sq = fmaf(x, x, sq);
        }
      }
      sq = row_sum<LPR>(sq);
      if (sub == 0 && r0 + u * RPI < kVnormRows && t < a.T) {
        const float nrm = sqrtf(sq);
        a.ratio[(size_t)unit * a.T + t] = nrm;
        local += nrm;
      }
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
    if (t < a.T) {
      const float rho = a.ratio[(size_t)unit * a.T + t] * inv;
      a.ratio[(size_t)unit * a.T + t] = rho;
      if (a.utility && t < a.P) a.utility[(size_t)unit * a.P + t] *= rho;
    }
  }
}

hipError_t launch_value_norm(const ckv_params *p, const Shape &s, const Workspace &w, const void *v,
                             float *ratio, char *ws, hipStream_t stream, float *utility_scaled) {
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
  a.utility = utility_scaled;
  a.P = s.P;
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
