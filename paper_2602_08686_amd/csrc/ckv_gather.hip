// Token-axis gather (paper Sec. 3: K~ = K[S], V~ = V[S]; Alg. 1 Gather_tok): bit copies of rows.
// A row of head_dim elements is moved as 16-byte pieces, one per lane, so a wave copies 64/LPR whole
// rows per instruction with 128-bit loads and stores; K and V rows travel in the same thread.
#include "ckv_internal.h"

namespace ckv {

typedef __attribute__((ext_vector_type(4))) uint32_t piece_t;

struct GatherArgs {
  const char *k, *v;
  char *k_out, *v_out;
  const int32_t *idx, *count;
  int64_t ks_b, ks_h, ks_t, vs_b, vs_h, vs_t;  // bytes
  int Hkv, T, cap;
  int lpr;        // lanes (16-byte pieces) per row
  int shared;     // idx [Bz][cap] and count [Bz]: one index list for all KV heads of a batch element
  int row_bytes;
};

constexpr int kGatherThreads = 256;

__global__ void __launch_bounds__(kGatherThreads) gather_kernel(GatherArgs a) {
  const int unit = blockIdx.y;
  const int b = unit / a.Hkv, g = unit % a.Hkv;
  const int list = a.shared ? b : unit;  // whose index list this unit follows
  const int n = min(a.count[list], a.cap);
  const int rows_per_block = kGatherThreads / a.lpr;
  const int piece = (threadIdx.x % a.lpr) * 16;
  const char *kb = a.k + b * a.ks_b + g * a.ks_h + piece, *vb = a.v + b * a.vs_b + g * a.vs_h + piece;
  // a few workgroups per unit stride over its kept rows (the count is far below cap in practice)
  for (int r = blockIdx.x * rows_per_block + threadIdx.x / a.lpr; r < n; r += gridDim.x * rows_per_block) {
    const int t = a.idx[(size_t)list * a.cap + r];
    if (t < 0 || t >= a.T) continue;
    const piece_t kk = *reinterpret_cast<const piece_t *>(kb + (int64_t)t * a.ks_t);
    const piece_t vv = *reinterpret_cast<const piece_t *>(vb + (int64_t)t * a.vs_t);
    const size_t o = ((size_t)unit * a.cap + r) * a.row_bytes + piece;
    *reinterpret_cast<piece_t *>(a.k_out + o) = kk;
    *reinterpret_cast<piece_t *>(a.v_out + o) = vv;
  }
}

hipError_t launch_gather(const ckv_params *p, const Shape &s, const void *k, const void *v,
                         const int32_t *idx, const int32_t *count, void *k_out, void *v_out,
                         hipStream_t stream, bool shared_list) {
  GatherArgs a;
  a.k = (const char *)k;
  a.v = (const char *)v;
  a.k_out = (char *)k_out;
  a.v_out = (char *)v_out;
  a.idx = idx;
  a.count = count;
  a.ks_b = p->k_stride[0] * s.esize; a.ks_h = p->k_stride[1] * s.esize; a.ks_t = p->k_stride[2] * s.esize;
  a.vs_b = p->v_stride[0] * s.esize; a.vs_h = p->v_stride[1] * s.esize; a.vs_t = p->v_stride[2] * s.esize;
  a.Hkv = s.Hkv;
  a.T = s.T;
  a.cap = p->cap;
  a.row_bytes = s.d * s.esize;
  a.lpr = a.row_bytes / 16;
  a.shared = shared_list ? 1 : 0;
  const int rows_per_block = kGatherThreads / a.lpr;
  // enough workgroups to fill the chip, at most what cap rows need
  const int units = s.Bz * s.Hkv;
  int per_unit = (4096 + units - 1) / units;
  per_unit = max(1, min(per_unit, (p->cap + rows_per_block - 1) / rows_per_block));
  const dim3 grid(per_unit, units), block(kGatherThreads);
  hipLaunchKernelGGL(gather_kernel, grid, block, 0, stream, a);
  return hipGetLastError();
}

}  // namespace ckv
