// Read-bandwidth probe with the scan's load pattern (global_load_lds_dwordx4: the 64 lanes of one instruction
// move 1 KiB of contiguous bytes into LDS; a ring of four 8 KiB images per wave, three in flight): what the
// memory system delivers to kernels shaped like the scan, independent of their arithmetic.
//   1. one region re-read many times, for footprints from 32 MiB (fits the eight L2 caches) through
//      64-192 MiB (fits the memory-side cache) to 1 GiB (HBM), with default and non-temporal loads;
//   2. a 2 GiB stream read once (HBM);
//   3. half of the workgroups streaming 1 GiB from HBM while the other half re-reads a cache-sized region
//      (the same number of bytes): whether cache hits add to the HBM rate or share one ceiling with it.
// Build: python -m paper_2602_08686_amd.build probes      Run: paper_2602_08686_amd/probes/read_bandwidth
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#define CHECK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("err %s line %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void glb_void;

template <int AUX>
__device__ __forceinline__ void tile_load(const char* g, char* image, int lane) {
#pragma unroll
  for (int i = 0; i < 8; ++i)
    __builtin_amdgcn_global_load_lds((glb_void*)(g + i * 1024 + lane * 16), (lds_void*)(uintptr_t)(image + i * 1024), 16, 0, AUX);
}
template <int N> __device__ __forceinline__ void wait_vm() {
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// role 0: wave streams `tiles` tiles starting at its own offset, `sweeps` times.
// blocks >= split take region B (base_b, tiles_b, sweeps_b), others region A.
template <int AUX_A, int AUX_B>
__global__ void __launch_bounds__(256) rd(const char* base_a, long tiles_a, int sweeps_a, const char* base_b, long tiles_b,
                                          int sweeps_b, int split, unsigned* out) {
  __shared__ __attribute__((aligned(1024))) char ring[4][4][8192];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const bool isb = (int)blockIdx.x >= split;
  const long nw = isb ? (long)(gridDim.x - split) * 4 : (long)split * 4;
  const long wid = (isb ? (long)(blockIdx.x - split) : (long)blockIdx.x) * 4 + wave;
  const long per = (isb ? tiles_b : tiles_a) / nw;
  const char* p = (isb ? base_b : base_a) + wid * per * 8192;
  const int sweeps = isb ? sweeps_b : sweeps_a;
  for (int s = 0; s < sweeps; ++s) {
    for (long t = 0; t < per; t += 4) {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const char* g = p + (t + u < per ? t + u : per - 1) * 8192;
        if (isb) tile_load<AUX_B>(g, ring[wave][u], lane); else tile_load<AUX_A>(g, ring[wave][u], lane);
        wait_vm<24>();
      }
    }
  }
  wait_vm<0>();
  if (ring[wave][0][lane] == 0x7f && ring[wave][3][lane * 3] == 0x11) out[0] = 1;
}

template <int AUX_A, int AUX_B>
float run(int blocks, int split, const char* a, size_t bytes_a, int sw_a, const char* b, size_t bytes_b, int sw_b, unsigned* out) {
  hipEvent_t e0, e1; CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
  float best = 1e9;
  for (int rep = 0; rep < 3; ++rep) {
    CHECK(hipEventRecord(e0));
    hipLaunchKernelGGL((rd<AUX_A, AUX_B>), dim3(blocks), dim3(256), 0, 0, a, (long)(bytes_a / 8192), sw_a, b, (long)(bytes_b / 8192), sw_b, split, out);
    CHECK(hipEventRecord(e1)); CHECK(hipEventSynchronize(e1));
    float ms; CHECK(hipEventElapsedTime(&ms, e0, e1));
    if (ms < best) best = ms;
  }
  return best;
}

int main() {
  char* buf; unsigned* out;
  const size_t cap = 3ull << 30;
  CHECK(hipMalloc(&buf, cap)); CHECK(hipMalloc(&out, 4));
  CHECK(hipMemset(buf, 1, cap));
  const char* hbm = buf; const char* small = buf + (2ull << 30);
  for (int blocks : {256, 512}) {
    printf("--- %d workgroups of 4 waves\n", blocks);
    // 1. pure streams / re-reads
    for (size_t mb : {32, 64, 128, 192, 1024}) {
      size_t bytes = mb << 20; int sw = (int)((4ull << 30) / bytes);
      float ms = run<0, 0>(blocks, blocks, small - (mb > 1024 ? 0 : 0), bytes, sw, small, bytes, 0, out);
      printf("re-read %5zu MiB x %3d default : %.3f ms %6.0f GB/s\n", mb, sw, ms, (double)bytes * sw / ms / 1e6);
      ms = run<2, 2>(blocks, blocks, small, bytes, sw, small, bytes, 0, out);
      printf("re-read %5zu MiB x %3d nt      : %.3f ms %6.0f GB/s\n", mb, sw, ms, (double)bytes * sw / ms / 1e6);
    }
    {
      float ms = run<0, 0>(blocks, blocks, hbm, 2ull << 30, 1, small, 0, 0, out);
      printf("stream 2 GiB default : %.3f ms %6.0f GB/s\n", ms, (double)(2ull << 30) / ms / 1e6);
      ms = run<2, 2>(blocks, blocks, hbm, 2ull << 30, 1, small, 0, 0, out);
      printf("stream 2 GiB nt      : %.3f ms %6.0f GB/s\n", ms, (double)(2ull << 30) / ms / 1e6);
    }
    // 2. half the workgroups stream 1 GiB from HBM, the other half re-read a resident region (same bytes)
    for (size_t mb : {64, 128}) {
      size_t bytes = mb << 20; int sw = (int)((1ull << 30) / bytes);
      float ms = run<2, 0>(blocks, blocks / 2, hbm, 1ull << 30, 1, small, bytes, sw, out);
      printf("mixed: 1 GiB nt stream + %3zu MiB x %2d default re-read : %.3f ms total %6.0f GB/s\n", mb, sw, ms, 2.0 * (1ull << 30) / ms / 1e6);
      ms = run<0, 0>(blocks, blocks / 2, hbm, 1ull << 30, 1, small, bytes, sw, out);
      printf("mixed: 1 GiB default stream + %3zu MiB x %2d default re-read : %.3f ms total %6.0f GB/s\n", mb, sw, ms, 2.0 * (1ull << 30) / ms / 1e6);
      ms = run<2, 2>(blocks, blocks / 2, hbm, 1ull << 30, 1, small, bytes, sw, out);
      printf("mixed: 1 GiB nt stream + %3zu MiB x %2d nt re-read : %.3f ms total %6.0f GB/s\n", mb, sw, ms, 2.0 * (1ull << 30) / ms / 1e6);
    }
  }
  return 0;
}
