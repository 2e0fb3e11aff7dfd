// Single-read observation-window scan: both passes of the scan in ONE persistent kernel that reads K
// from HBM once (paper Sec. 3 attention definition, Eq. 3, Eq. 4's alpha per query head). Included by
// ckv_scan.h; bf16 only, all query tiles of a KV head in one group (n_groups == 1), W <= 64.
//
// Why. The column sums need every row's softmax normaliser, so the two-kernel scan streams K twice
// and is bound by twice the K bytes. Here a (batch, KV head) unit is handed to ONE XCD: its 32
// workgroups (one per CU, one wave per SIMD) split the unit's keys, and every wave keeps its key tiles
// on chip after their first use: up to kFusedRes tiles of 32 keys sit in the accumulation registers
// (they are only ever MFMA operands, which the matrix cores read from either register file; the
// ordinary vector registers stay free for Q and the arithmetic). The XCD's workgroups exchange their
// partial (max, sum) row statistics through memory and pass 2 recomputes QK^T from the resident
// tiles. Tiles outside the pipelines (window / end-of-keys tiles, left-overs of a four-tile round,
// keys beyond the register capacity) are fetched again where they are needed.
//
// Phases. The query tiles of a unit are taken QPH at a time (Q stays in LDS for the whole unit and a
// phase loads its tiles into registers): statistics of phase 0 (K streamed from HBM through a ring of
// LDS images and parked in registers), statistics of phases 1.. (K from registers), then the column
// sums phase by phase. The team exchange of a phase is therefore hidden behind the work of the
// other phases.
//
// Synchronisation. Workgroups find their XCD from the XCC_ID hardware register and number themselves
// with one atomic per XCD; a grid-wide start barrier fixes the team sizes (the kernel is launched
// cooperatively, so all workgroups are resident). Per unit and phase, a team's workgroups publish
// their row partials with device-scope write-through stores, wait for them to be acknowledged, bump
// the team's arrival counter of that phase and later poll it; then every workgroup merges the team's
// partials itself, in rank order (bit-stable results, no float atomics). Partial buffers alternate
// with the unit's parity: a workgroup can only publish unit k + 2 after every team mate has published
// all of unit k + 1, i.e. has finished reading unit k. Every wait is bounded: after kSpinLimit polls
// a workgroup records a status word and goes on (results are then invalid, but every wave exits).
#ifndef CKV_SCAN_FUSED_H_
#define CKV_SCAN_FUSED_H_

namespace ckv {

constexpr int kFusedRes = 8;   // key tiles a wave keeps in registers between the passes
constexpr int kFusedRing = 3;  // LDS tile images per wave
constexpr int kFusedGroup = 4; // key tiles per store group (128 keys per head and flush)
constexpr int kFusedMaxPhases = 4;
// sync words: [0] workgroups started, [1] status, [8 + x] team size, [16 + 4 x + phase] arrivals
constexpr int kFusedSyncWords = kFusedSyncBytes / 4;
constexpr int kSpinLimit = 1 << 21;

struct FusedArgs {
  uint32_t *sync;  // kFusedSyncWords words, zero when the kernel starts
  float2 *fpart;   // [2][phases][gridDim.x][QPH * 32] row partials (max, sum), log2 domain
  int units;       // Bz * Hkv
};

namespace {  // one copy per translation unit that includes this header
__global__ void __attribute__((unused)) fused_init_kernel(uint32_t *sync) {
  if (threadIdx.x < kFusedSyncWords) sync[threadIdx.x] = 0u;
}
}  // namespace

__device__ __forceinline__ uint32_t load_dev(const uint32_t *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Polls *p until it reaches target or the sync area reports a failure. Returns false on time-out.
__device__ __forceinline__ bool spin_until(const uint32_t *p, uint32_t target, uint32_t *status) {
  for (int it = 0; it < kSpinLimit; ++it) {
    if (load_dev(p) >= target) return true;
    if ((it & 255) == 255 && load_dev(status) != 0u) return false;
    __builtin_amdgcn_s_sleep(1);
  }
  __hip_atomic_store(status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return false;
}

template <int N>
__device__ __forceinline__ void wait_vm_upto(int n) {  // waits until <= min(n, N) rounded down to 8 ops are in flight
  if constexpr (N == 0) {
    wait_vm<0>();
  } else {
    if (n >= N) wait_vm<N>();
    else wait_vm_upto<(N > 8 ? N - 8 : 0)>(n);
  }
}

// LDS reads that target accumulation registers directly. The compiler does not track such reads, so
// the reads of one tile and the wait for them are ONE statement: when the compiler sees the values
// (it may copy them between registers at once) they have arrived. LDS operations return in order, so
// the compiler's own counted waits stay conservative.
template <int NCH, int IMAGE_OFFSET>
__device__ __forceinline__ void lds_to_acc_regs(chunk_t (&f)[NCH], const uint32_t (&vaddr)[NCH]) {
  if constexpr (NCH == 8) {
    asm volatile(
        "ds_read_b128 %0, %8 offset:%16\n\tds_read_b128 %1, %9 offset:%16\n\t"
        "ds_read_b128 %2, %10 offset:%16\n\tds_read_b128 %3, %11 offset:%16\n\t"
        "ds_read_b128 %4, %12 offset:%16\n\tds_read_b128 %5, %13 offset:%16\n\t"
        "ds_read_b128 %6, %14 offset:%16\n\tds_read_b128 %7, %15 offset:%16\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&a"(f[0]), "=&a"(f[1]), "=&a"(f[2]), "=&a"(f[3]), "=&a"(f[4]), "=&a"(f[5]), "=&a"(f[6]), "=&a"(f[7])
        : "v"(vaddr[0]), "v"(vaddr[1]), "v"(vaddr[2]), "v"(vaddr[3]), "v"(vaddr[4]), "v"(vaddr[5]), "v"(vaddr[6]),
          "v"(vaddr[7]), "n"(IMAGE_OFFSET)
        : "memory");
  } else {
    static_assert(NCH == 4, "chunks per lane");
    asm volatile(
        "ds_read_b128 %0, %4 offset:%8\n\tds_read_b128 %1, %5 offset:%8\n\t"
        "ds_read_b128 %2, %6 offset:%8\n\tds_read_b128 %3, %7 offset:%8\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&a"(f[0]), "=&a"(f[1]), "=&a"(f[2]), "=&a"(f[3])
        : "v"(vaddr[0]), "v"(vaddr[1]), "v"(vaddr[2]), "v"(vaddr[3]), "n"(IMAGE_OFFSET)
        : "memory");
  }
}
template <int NCH, int TILE_BYTES>
__device__ __forceinline__ void lds_slot_to_acc_regs(chunk_t (&f)[NCH], const uint32_t (&vaddr)[NCH], int slot) {
  static_assert(kFusedRing == 3, "slots");
  if (slot == 0) lds_to_acc_regs<NCH, 0>(f, vaddr);
  else if (slot == 1) lds_to_acc_regs<NCH, TILE_BYTES>(f, vaddr);
  else lds_to_acc_regs<NCH, 2 * TILE_BYTES>(f, vaddr);
}
// A copy of x the compiler cannot see through: what is computed from it is computed where it is used
// instead of being hoisted out of the unit loop into long-lived registers.
__device__ __forceinline__ int opaque(int x) {
  asm volatile("" : "+v"(x));
  return x;
}
// Ordinary (compiler-tracked) read of this lane's operand chunks from the image `delta` bytes past
// image 0 of the wave's ring.
template <int NCH>
__device__ __forceinline__ void read_lds(chunk_t (&f)[NCH], const uint32_t (&vaddr)[NCH], int delta) {
#pragma unroll
  for (int c = 0; c < NCH; ++c)
    f[c] = *(const __attribute__((address_space(3))) chunk_t *)(uintptr_t)(vaddr[c] + (uint32_t)delta);
}

template <int DT, int DH, int NQ, int WT, int QPH>
__global__ void __launch_bounds__(kScoreWaves *kWave) fused_scan_kernel(ScoreArgs a, FusedArgs f) {
  static_assert(DT == CKV_BF16, "bf16 only");
  static_assert(NQ <= kScoreWaves, "one query tile per loading wave");
  static_assert(NQ % QPH == 0 && QPH % WT == 0, "whole heads per phase");
  using G = Geom<DT, DH>;
  constexpr int NCH = G::NCH;
  constexpr int NDMA = G::NDMA;
  constexpr int N_MFMA = NCH;
  constexpr int NPH = NQ / QPH;       // phases
  constexpr int RP = QPH * kTile;     // query rows per phase
  constexpr int NSPLIT = (kScoreWaves * kWave) / RP;  // thread groups that share the merge of one row
  constexpr int READ_AT = QPH >= 2 ? QPH - 2 : 0;
  static_assert(NPH <= kFusedMaxPhases, "phases");

  __shared__ __attribute__((aligned(1024))) char ring[kScoreWaves][kFusedRing][G::TILE];
  __shared__ __attribute__((aligned(1024))) char qarea[NQ][G::TILE];  // the unit's query tiles, tile images
  __shared__ __attribute__((aligned(16))) float s_stage[kScoreWaves][(QPH / WT) * kFusedGroup * kTile];
  __shared__ __attribute__((aligned(16))) chunk_t s_bias[QPH][kWave];  // per (query tile, lane): the bias operand of pass 2
  __shared__ float2 s_part[kScoreWaves][RP];
  __shared__ float2 s_mrg[NSPLIT][RP];
  __shared__ int s_team[6];

  const int tid = threadIdx.x, lane = tid & 63, m = lane & 31, hh = lane >> 5, lane_id = lane;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grid = gridDim.x;
  uint32_t *const status = f.sync + 1;

  // ---- teams: one per XCD that received workgroups --------------------------------------------
  if (tid == 0) {
    const uint32_t xcc = __builtin_amdgcn_s_getreg((3 << 11) | 20) & 7u;  // XCC_ID, bits 3:0
    const uint32_t rank = __hip_atomic_fetch_add(&f.sync[8 + xcc], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the team counter is updated before "started"
    __hip_atomic_fetch_add(&f.sync[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    spin_until(&f.sync[0], (uint32_t)grid, status);
    int base = 0, n_active = 0, aidx = 0, nx = 1;
    for (uint32_t x = 0; x < 8; ++x) {
      const int c = (int)load_dev(&f.sync[8 + x]);
      if (x < xcc) base += c;
      if (x == xcc) { aidx = n_active; nx = c > 0 ? c : 1; }
      if (c > 0) ++n_active;
    }
    s_team[0] = (int)xcc;
    s_team[1] = (int)rank;
    s_team[2] = nx;
    s_team[3] = base;
    s_team[4] = aidx;
    s_team[5] = n_active > 0 ? n_active : 1;
  }
  __syncthreads();
  // LDS reads land in vector registers: readfirstlane tells the compiler that these are wave-uniform,
  // so everything derived from them stays in scalar registers
  const int xcc = __builtin_amdgcn_readfirstlane(s_team[0]), rank = __builtin_amdgcn_readfirstlane(s_team[1]),
            nx = __builtin_amdgcn_readfirstlane(s_team[2]), slot0 = __builtin_amdgcn_readfirstlane(s_team[3]),
            aidx = __builtin_amdgcn_readfirstlane(s_team[4]), n_active = __builtin_amdgcn_readfirstlane(s_team[5]);

  // ---- this wave's share of a unit's keys (the same for every unit) ----------------------------
  const int n_key_tiles = (a.T + kTile - 1) / kTile;
  const int NTW = (n_key_tiles + kScoreWaves * nx - 1) / (kScoreWaves * nx);  // key tiles per wave
  const int tile0 = (rank * kScoreWaves + wave) * NTW;
  const int ntw = max(0, min(n_key_tiles - tile0, NTW));
  const int t_begin = tile0 * kTile;
  const int n_prefix = max(0, (min(t_begin + ntw * kTile, a.P) - t_begin) / kTile);  // tiles wholly inside the prefix
  const int n_fast = min(n_prefix, kFusedRes) / kFusedGroup * kFusedGroup;  // tiles the pipelines take (0, 4 or 8)
  // Tiles outside the pipelines are not kept: every phase fetches them again through ring image 0, so
  // a wave that has any starts the next unit's key loads only after its last phase.
  const bool early_k = ntw == n_fast;

  uint32_t voff[NDMA];
#pragma unroll
  for (int i = 0; i < NDMA; ++i) {
    int r, kappa;
    dma_source<G>(i, lane, r, kappa);
    voff[i] = (uint32_t)(r * a.ks_t + kappa * 16 + kDmaBias - (i % 4) * 1024 - (i / 4) * 4096);
  }
  const int64_t tile_stride = (int64_t)kTile * a.ks_t;
  const uint32_t lds_ring = (uint32_t)(uintptr_t)&ring[wave][0][0];
  const int q_delta = (int)((uint32_t)(uintptr_t)&qarea[0][0] - lds_ring);  // query tile 0 relative to ring image 0
  uint32_t vaddr[NCH];  // this lane's operand chunks in image 0 of the wave's ring
#pragma unroll
  for (int c = 0; c < NCH; ++c) vaddr[c] = lds_ring + (uint32_t)image_offset<G>(m, c + NCH * hh);
  float *stage = s_stage[wave];
  const chunk_t ones = Bias<DT>::ones(hh);

  // Starts the loads of a unit's query tiles (wave w moves tile w into the Q area) / of this wave's
  // first three pipeline tiles (ring images 0..2).
  auto prefetch_q = [&](int unit) {
    const int b = unit / a.Hkv, g = unit % a.Hkv;
    if (wave < NQ) {
      const int lane = opaque(lane_id);  // per-lane addresses are recomputed here, not kept across the unit
      const int tile = min(wave, a.n_tiles - 1);
      const char *qhead = a.q + b * a.qs_b + (g * a.G + tile / WT) * a.qs_h;
      const int j0 = (tile % WT) * kTile;
#pragma unroll
      for (int i = 0; i < NDMA; ++i) {
        int r, kappa;
        dma_source<G>(i, lane, r, kappa);
        const char *src = qhead + (int64_t)min(j0 + r, a.W - 1) * a.qs_w + kappa * 16;
        __builtin_amdgcn_global_load_lds((glb_void_t *)src, (lds_void_t *)(uintptr_t)(qarea[wave] + i * 1024), 16, 0, 0);
      }
    }
  };
  auto prefetch_k = [&](int unit) {
    if (n_fast > 0) {
      const int b = unit / a.Hkv, g = unit % a.Hkv;
      const char *kwave = a.k + b * a.ks_b + g * a.ks_h + (int64_t)t_begin * a.ks_t;
#pragma unroll
      for (int d = 0; d < kFusedRing; ++d) dma_tile<G>(kwave + d * tile_stride, voff, lds_ring + d * G::TILE);
    }
  };

  int unit = aidx;
  if (unit < f.units) {
    prefetch_q(unit);
    prefetch_k(unit);
  }

  for (int k = 0; unit < f.units; ++k, unit += n_active) {
    const int b = unit / a.Hkv, g = unit % a.Hkv;
    const char *kbase = a.k + b * a.ks_b + g * a.ks_h;
    const char *kwave = kbase + (int64_t)t_begin * a.ks_t;
    const int next_unit = unit + n_active;
    float2 *const part = f.fpart + (size_t)(k & 1) * NPH * grid * RP;
    wait_vm<0>();
    __syncthreads();  // Q of this unit is in the Q area, the first key tiles are in the ring

    chunk_t qf[QPH][NCH];
    chunk_t kres[kFusedRes][NCH];
    f32x16 acc[2];

    // This phase's query tiles into registers; rows past W and tiles past n_tiles are zero.
    auto load_q = [&](int ph) {
#pragma unroll
      for (int i = 0; i < QPH; ++i) {
        const int tile = ph * QPH + i;
        read_lds<NCH>(qf[i], vaddr, q_delta + tile * G::TILE);
        if (!(tile < a.n_tiles && (tile % WT) * kTile + m < a.W)) {
#pragma unroll
          for (int c = 0; c < NCH; ++c) qf[i][c] = chunk_t{0u, 0u, 0u, 0u};
        }
      }
    };

    // Counts this workgroup in for a phase whose partials it has stored: every storing wave waits for
    // the acknowledgement of its write-through stores (vector memory operations complete in order, so
    // this is a wait for everything it has in flight), then one thread bumps the team's counter.
    auto arrive = [&](int ph) {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
      if (tid == 0)
        __hip_atomic_fetch_add(&f.sync[16 + kFusedMaxPhases * xcc + ph], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    };

    // ======================= pass 1: row statistics, phase by phase ==========================
#pragma unroll
    for (int ph = 0; ph < NPH; ++ph) {
      load_q(ph);
      float rm[QPH], rl[QPH];
#pragma unroll
      for (int i = 0; i < QPH; ++i) {
        rm[i] = -1e30f;
        rl[i] = 0.0f;
      }
      if (n_fast > 0) {
        if (ph == 0) {
          lds_to_acc_regs<NCH, 0>(kres[0], vaddr);
        }
        mma_chain<DT, NCH>(acc[0], kres[0], qf[0]);
#pragma unroll
        for (int t = 0; t < kFusedRes; ++t) {
          if (t == kFusedGroup && n_fast <= kFusedGroup) break;
          // the pipeline goes on to tile t + 1
          const bool has_next = t + 1 < kFusedRes && (t + 1 != kFusedGroup || n_fast > kFusedGroup);
          if (ph == 0 && t + 3 < kFusedRes) {
            // tile t's image was emptied into registers during tile t - 1: tile t + 3 goes there
            if (t + 3 < kFusedGroup || n_fast > kFusedGroup)
              dma_tile<G>(kwave + (t + 3) * tile_stride, voff, lds_ring + (t % kFusedRing) * G::TILE);
          }
#pragma unroll
          for (int i = 0; i < QPH; ++i) {
            const int cur = (t * QPH + i) & 1;
            if (ph == 0 && i == READ_AT && has_next) {
              // loads issued after tile t + 1's own: tiles t + 2 and t + 3 where the pipeline has them
              wait_vm_upto<2 * NDMA>(max(0, min(n_fast - 2 - t, 2)) * NDMA);
              lds_slot_to_acc_regs<NCH, G::TILE>(kres[(t + 1) % kFusedRes], vaddr, (t + 1) % kFusedRing);
            }
            if (i + 1 < QPH) {
              mma_chain<DT, NCH>(acc[cur ^ 1], kres[t], qf[i + 1]);
            } else if (has_next) {
              mma_chain<DT, NCH>(acc[cur ^ 1], kres[(t + 1) % kFusedRes], qf[0]);
            }
            rowstats_update<false>(acc[cur], a.c2, 0, hh, 0, rm[i], rl[i]);
            interleave_hint<N_MFMA, 8, 0>();
          }
        }
        if (ph == 0) wait_vm<0>();
      }
      for (int t = n_fast; t < ntw; ++t) {  // tiles outside the pipeline, masked
        const int t0 = t_begin + t * kTile;
        chunk_t kreg[NCH];
        dma_tile_clamped<G>(kbase, a.ks_t, t0, a.T, opaque(lane_id), ring[wave][0]);
        wait_vm<0>();
        read_lds<NCH>(kreg, vaddr, 0);
#pragma unroll
        for (int i = 0; i < QPH; ++i) {
          const int tile = ph * QPH + i, j = (tile % WT) * kTile + m;
          const int limit = tile < a.n_tiles && j < a.W ? a.P + j : -1;  // last key this row may see (causal)
          mma_chain<DT, NCH>(acc[0], kreg, qf[i]);
          rowstats_update<true>(acc[0], a.c2, t0, hh, limit, rm[i], rl[i]);
        }
      }
      // The previous phase's partials have had a whole phase to reach memory: count this workgroup in.
      if (ph > 0) arrive(ph - 1);
      // publish this workgroup's row partials of the phase (its arrival is counted later)
#pragma unroll
      for (int i = 0; i < QPH; ++i) {
        const float om = __shfl_xor(rm[i], 32), ol = __shfl_xor(rl[i], 32);
        merge_stats(rm[i], rl[i], om, ol);
        if (hh == 0) s_part[wave][i * kTile + m] = make_float2(rm[i], rl[i]);
      }
      __syncthreads();
      if (tid < RP) {
        float2 s = s_part[0][tid];
#pragma unroll
        for (int w = 1; w < kScoreWaves; ++w) merge_stats(s.x, s.y, s_part[w][tid].x, s_part[w][tid].y);
        unsigned long long bits;
        __builtin_memcpy(&bits, &s, 8);
        __hip_atomic_store((unsigned long long *)&part[((size_t)ph * grid + slot0 + rank) * RP + tid], bits,
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    // ======================= pass 2: column sums, phase by phase ==============================
#pragma unroll
    for (int ph = 0; ph < NPH; ++ph) {
      if (NPH > 1) load_q(ph);  // a single phase still holds its tiles
      if (NPH == 1) arrive(0);
      // wait for the team, merge its partials of this phase
      if (tid == 0)
        spin_until(&f.sync[16 + kFusedMaxPhases * xcc + ph], (uint32_t)(k + 1) * (uint32_t)nx, status);
      __syncthreads();
      {
        const int grp = tid / RP, row = tid % RP;
        const int per = (nx + NSPLIT - 1) / NSPLIT;
        const int s_end = min(nx, (grp + 1) * per);
        float M = -1e30f, L = 0.0f;
        for (int s0 = grp * per; s0 < s_end; s0 += 8) {
          unsigned long long v[8];
#pragma unroll
          for (int e = 0; e < 8; ++e)
            v[e] = __hip_atomic_load(
                (const unsigned long long *)&part[((size_t)ph * grid + slot0 + min(s0 + e, s_end - 1)) * RP + row],
                __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            float2 p;
            __builtin_memcpy(&p, &v[e], 8);
            if (s0 + e < s_end) merge_stats(M, L, p.x, p.y);
          }
        }
        s_mrg[grp][row] = make_float2(M, L);
      }
      if (ph == 0) {
        // the last phase's partials went out before this merge: count this workgroup in for it, then
        // (the ring is idle until the next unit) start the next unit's key loads
        if (NPH > 1) arrive(NPH - 1);
        else __syncthreads();
        if (early_k && next_unit < f.units) prefetch_k(next_unit);
      } else {
        __syncthreads();
      }
      // Wave w < QPH finishes the rows of the phase's query tile w (both half-waves alike) and leaves,
      // per lane, the MFMA operand that adds -LSE / scale to that tile's logits; padding rows (q = 0)
      // get a bias that makes their weights exp2(-1000) = 0.
      if (wave < QPH) {
        const int row = wave * kTile + m, tile = ph * QPH + wave;
        float2 s = s_mrg[0][row];
#pragma unroll
        for (int p = 1; p < NSPLIT; ++p) merge_stats(s.x, s.y, s_mrg[p][row].x, s_mrg[p][row].y);
        const float lse2 = s.x + __log2f(s.y);
        const int j = (tile % WT) * kTile + m;
        const bool valid = tile < a.n_tiles && j < a.W;
        if (rank == 0 && valid && hh == 0) a.lse_out[((size_t)b * a.Hq + g * a.G + tile / WT) * a.W + j] = lse2 * kLn2;
        Bias<DT> bs;
        bs.set(valid ? -lse2 / a.c2 : -1000.0f / a.c2, hh);
        s_bias[wave][lane] = bs.q;
      }
      __syncthreads();
      // From here on nobody reads this unit's Q area again (the last phase has its tiles in registers).
      if (ph == NPH - 1 && next_unit < f.units) prefetch_q(next_unit);

      BlockCoord bc;
      bc.chunk = 0; bc.grp = ph; bc.unit = unit; bc.b = b; bc.g = g;
      auto add_bias = [&](f32x16 &d, int i) {
        Bias<DT> bs;
        bs.q = s_bias[i][lane];
        bs.add(d, ones);
      };
      const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
          (void *)(a.scores + (size_t)b * a.Hq * a.T), 0, a.Hq * a.T * 4, 0x00020000);
      if (n_fast > 0) {
        mma_chain<DT, NCH>(acc[0], qf[0], kres[0]);
        add_bias(acc[0], 0);
#pragma unroll
        for (int t = 0; t < kFusedRes; ++t) {
          if (t == kFusedGroup && n_fast <= kFusedGroup) break;
          const int u = t % kFusedGroup;
          const bool has_next = t + 1 < kFusedRes && (t + 1 != kFusedGroup || n_fast > kFusedGroup);
          float cs[QPH];
#pragma unroll
          for (int i = 0; i < QPH; ++i) {
            const int cur = (t * QPH + i) & 1;
            if (i + 1 < QPH) {
              mma_chain<DT, NCH>(acc[cur ^ 1], qf[i + 1], kres[t]);  // rows: query rows, cols: keys
              add_bias(acc[cur ^ 1], i + 1);
            } else if (has_next) {
              mma_chain<DT, NCH>(acc[cur ^ 1], qf[0], kres[(t + 1) % kFusedRes]);
              add_bias(acc[cur ^ 1], 0);
            }
            cs[i] = colsum_weights<false>(acc[cur], a.c2, hh, 0);
            interleave_hint<N_MFMA + 1, 6, 0>();
          }
          stage_column_sums<QPH, WT>(cs, a.norm, stage, u, m, hh);
          if (u == kFusedGroup - 1)
            flush_column_sums<QPH, WT>(a, bc, stage, t_begin + (t - (kFusedGroup - 1)) * kTile, lane, rsrc);
        }
      }
      for (int t = n_fast; t < ntw; ++t) {
        const int t0 = t_begin + t * kTile, kt = t0 + m;
        chunk_t kreg[NCH];
        dma_tile_clamped<G>(kbase, a.ks_t, t0, a.T, opaque(lane_id), ring[wave][0]);
        wait_vm<0>();
        read_lds<NCH>(kreg, vaddr, 0);
        float cs[QPH];
#pragma unroll
        for (int i = 0; i < QPH; ++i) {
          const int j0 = ((ph * QPH + i) % WT) * kTile;
          mma_chain<DT, NCH>(acc[0], qf[i], kreg);
          add_bias(acc[0], i);
          cs[i] = colsum_weights<true>(acc[0], a.c2, hh, kt - a.P - j0);
        }
        store_column_sums<QPH>(a, bc, cs, WT, kt, hh);
      }
    }
    if (!early_k && next_unit < f.units) {
      wait_vm<0>();
      prefetch_k(next_unit);
    }
  }
}

}  // namespace ckv
#endif
