// Private declarations shared by the HIP translation units of libckv (not part of the ABI).
#ifndef CKV_INTERNAL_H_
#define CKV_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "ckv.h"

namespace ckv {

constexpr int kWave = 64;          // CDNA wavefront width
constexpr int kTile = 32;          // MFMA 32x32 tile edge: query rows and keys per tile
constexpr int kMaxQTiles = 8;      // query-row tiles a wave keeps in registers (bf16; f32 kernels: kMaxQTilesF32)
constexpr int kMaxQTilesF32 = 4;
constexpr int kMaxWindowTiles = 4; // 32-row tiles per query head: W <= 128
constexpr int kScoreWaves = 4;     // waves per workgroup in the scan kernels
// Compute units of the build target (gfx950: MI355X, 256). A constant on purpose, not a device query: the
// split of the key axis, and with it the workspace layout, must be the same for ckv_workspace_bytes
// (which may run where no device is visible) and for the calls that use the workspace.
constexpr int kComputeUnits = 256;
constexpr int kSelectThreads = 1024;
// Geometry of the fused utility form of the scan's second pass, shared by that pass (ckv_scan.h) and by
// the kernel that finishes what it leaves out (ckv_tables.hip). The pass works in rounds of
// kRing * kTile keys per wave; each round writes the utilities of the kRing * kTile keys that end
// kUtilShift keys before the round does, keeps its last kUtilCarry column sums in front of the next
// round's, and stores raw column sums for the first kUtilHead and the last kUtilCarry keys of a wave's
// pipelined range; the first four keys of a range, its last kUtilShift pipelined keys and its tail tiles
// are finished by the other kernel.
constexpr int kRing = 4;           // key-tile images per wave, and tiles per pipeline round
constexpr int kUtilShift = 32;
constexpr int kUtilCarry = 40;
constexpr int kUtilHead = 8;
constexpr int kUtilMaxRadius = 3;  // pooling kernels of up to 7 taps
static_assert(kUtilShift % 4 == 0 && kUtilCarry % 4 == 0 && kUtilHead % 4 == 0, "128-bit pieces");
static_assert(kUtilCarry >= kUtilShift + 4 + kUtilMaxRadius, "a round's first output window reaches this far back");
static_assert(kUtilHead >= 4 + kUtilMaxRadius, "the range's first four keys need their right neighbours");
static_assert(kUtilShift >= kUtilMaxRadius, "a round's last output window stays inside the round");
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kValueNormEps = 1e-6f;

// Derived quantities every entry point needs; filled by derive() after validation.
struct Shape {
  int Bz, Hq, Hkv, G, d, T, W, P;
  int esize;        // bytes per element of Q/K/V
  int WT;           // 32-row tiles per query head = ceil(W / 32)
  int n_tiles;      // G * WT, query-row tiles per KV head
  int NQ;           // tiles per wave (multiple of WT, <= kMaxQTiles)
  int n_groups;     // ceil(n_tiles / NQ): how often K is swept for one KV head
  int keys_per_wave;
  int n_chunks;     // workgroups along the key axis per (unit, group)
  float scale;      // softmax scale
};

// A 16-byte piece of a row; STREAM marks data that is used once (non-temporal: it should not displace
// what the caches hold).
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_d;
template <bool STREAM>
__device__ __forceinline__ uint4 load_piece(const char *p) {
  if (STREAM) {
    const u32x4_d v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_d *>(p));
    return make_uint4(v[0], v[1], v[2], v[3]);
  }
  return *reinterpret_cast<const uint4 *>(p);
}

// Sum over the LPR (8, 16 or 32) consecutive lanes that hold one row; every lane ends with the total.
// Lane exchanges inside a row of 16 lanes are DPP operands of the add (quad permutes give the xor-1 and
// xor-2 partners; once quads agree, mirroring a half row or a row pairs each lane with its xor-4 /
// xor-8 partner's value); only 32-lane rows need one exchange through the LDS crossbar.
template <int CTRL>
__device__ __forceinline__ float dpp_add(float x) {
  const int y = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, false);
  return x + __int_as_float(y);
}
template <int LPR>
__device__ __forceinline__ float row_sum(float x) {
  x = dpp_add<0xB1>(x);                  // quad_perm [1,0,3,2]
  x = dpp_add<0x4E>(x);                  // quad_perm [2,3,0,1]
  x = dpp_add<0x141>(x);                 // row_half_mirror
  if (LPR >= 16) x = dpp_add<0x140>(x);  // row_mirror
  if (LPR >= 32) x += __shfl_xor(x, 16);
  return x;
}

ckv_status validate(const ckv_params *p);
void derive(const ckv_params *p, Shape *s);

// Workspace layout (bytes, 256-aligned sections), all sized from Shape.
struct Workspace {
  size_t part_off, part_bytes;   // float2 [units][n_tiles*32][n_chunks] row-stat partials
  size_t lse_off, lse_bytes;     // float  [Bz][Hq][W]
  size_t vsum_off, vsum_bytes;   // float  [units][vnorm blocks] partial sums of value norms
  size_t select_off, select_bytes;  // int: the split selection's merged histograms, slice counts, thresholds
  size_t total;
};
void layout(const ckv_params *p, const Shape &s, Workspace *w);
int vnorm_blocks_per_unit(const Shape &s);

// Kernel launchers (each returns hipGetLastError() after its launches).
// lse_in == nullptr: pass 1 first, LSE into lse_out (or the workspace). scores == nullptr: pass 1 only.
// Fused utility form of pass 2 (see ckv_window_utility): where `fuse` is given, the second pass writes
// utilities of block-interior keys to fuse->utility and raw column sums only where the fix-up kernel
// needs them (into `scores`).
struct UtilityFusion {
  const float *w_row;  // w_head + layer * Hq
  float *utility;      // [Bz][Hkv][P]
  int pool, radius;
  float inv_kernel;
};
hipError_t launch_window_scores(const ckv_params *p, const Shape &s, const Workspace &w, const void *q,
                                const void *k, const float *lse_in, float *lse_out, float *scores,
                                char *ws, hipStream_t stream, const UtilityFusion *fuse = nullptr);
hipError_t launch_utility_fixup(const ckv_params *p, const Shape &s, const float *sparse_scores,
                                const float *w_head, const float *head_share, const float *t_gate, int n_ent,
                                int n_ppl, const int32_t *risk_bins, float *utility, int32_t *budget, float *tau,
                                hipStream_t stream);
// utility_scaled: if given, [units][P] utilities that the scaling pass multiplies by the ratio
hipError_t launch_value_norm(const ckv_params *p, const Shape &s, const Workspace &w, const void *v,
                             float *ratio, char *ws, hipStream_t stream, float *utility_scaled = nullptr);
hipError_t launch_apply_tables(const ckv_params *p, const Shape &s, const float *scores,
                               const float *vnorm_ratio, const float *w_head, const float *head_share,
                               const float *t_gate, int n_ent, int n_ppl, const int32_t *risk_bins,
                               float *utility, int32_t *budget, float *tau, hipStream_t stream);
// ws: nullptr, or select_workspace_bytes(s) bytes (256-byte aligned) that let long prefixes be split
// over several workgroups per unit; the result is the same either way.
size_t select_workspace_bytes(const Shape &s);
hipError_t launch_select(const ckv_params *p, const Shape &s, const float *utility,
                         const int32_t *budget, const float *tau, int32_t *idx, int32_t *count,
                         char *ws, hipStream_t stream);
hipError_t launch_gather(const ckv_params *p, const Shape &s, const void *k, const void *v,
                         const int32_t *idx, const int32_t *count, void *k_out, void *v_out,
                         hipStream_t stream, bool shared_list = false);
// layer-shared mode (Alg. 1 as printed)
hipError_t launch_alpha_accumulate(const Shape &s, int rows, const float *scores, float weight, float *alpha,
                                   hipStream_t stream);
hipError_t launch_risk_struct(const Shape &s, const float *alpha, const float *edges, int n_edges, float *risk,
                              int32_t *bin, hipStream_t stream);
hipError_t launch_shared_utility(const ckv_params *p, const Shape &s, const float *alpha, const float *rho,
                                 const float *w_head, const float *t_gate, int n_ent, int n_ppl,
                                 const int32_t *risk_bins, float *utility, float *tau, hipStream_t stream);

hipError_t launch_map_depth(const float *src, int n_src, int row, float *dst, int n_dst, hipStream_t stream);
// decode-side consumer (Proposition 1): attention over a ragged KV set, discarded mass
struct DecodePlan {
  int rq;              // query heads of a group that share one sweep over the rows (1, 2, 4 or 8)
  int head_chunks;     // ceil(G / rq)
  int rows_per_chunk, n_chunks;
  int64_t grid_y;      // Bz * Hkv * n_q * head_chunks
  size_t workspace_bytes;
};
DecodePlan plan_decode(const Shape &s, int n_q, int n_rows);
hipError_t launch_decode_attention(const ckv_params *p, const Shape &s, const void *q_dec, int n_q, const void *k_rows,
                                   const void *v_rows, const int64_t *k_stride, const int64_t *v_stride, int n_rows,
                                   const int32_t *count, float *out, float *lse, char *ws, hipStream_t stream);
hipError_t launch_discarded_mass(const Shape &s, int n_q, const float *lse_full, const float *lse_kept, float *mass,
                                 float *eps, hipStream_t stream);

}  // namespace ckv
#endif
