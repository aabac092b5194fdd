// bf16 main loop tuned for gfx950: 256 x 256 tile, 256 threads = 4 wavefronts (one per
// SIMD) arranged 2 x 2, each owning a 128 x 128 sub-tile (4 x 4 blocks of the
// 32x32x16 MFMA, 256 fp32 accumulators per lane).
//
//   * Operand tiles go from global memory straight into LDS (buffer_load ... lds,
//     16 bytes per lane), four stages of 32 bf16 of K deep, so a tile is requested
//     two to three K steps before it is read.  Rows past the end of a
//     tensor are zero-filled by the buffer's range check.
//   * LDS tile layout [256 rows][64 bytes]; the 16-byte chunk index is XOR-ed with
//     (row / 4) % 4, which spreads the 16 consecutive rows that a quarter wavefront
//     reads in one cycle over all 64 banks.  The DMA writes LDS linearly, so the
//     swizzle is applied to the global address each lane fetches from.
//   * Fragments are double buffered in registers and the single barrier per K step
//     sits between the two MFMA groups of the step: LDS latency and the barrier wait
//     are both covered by 16 independent MFMAs.
//   * The instruction order inside a K step is written out by hand (one LDS read or
//     one global request between consecutive MFMAs, pinned with scheduling barriers):
//     with one wavefront per SIMD a burst of memory instructions stalls the MFMA
//     stream, and the 8 requests of a tile are spread over the whole step.
//
// Requires K * 2 bytes to be a multiple of 64 and row pitches below 2^23 bytes; the
// generic loop in tile_mma.h covers everything else.
#pragma once
#include "tile_mma.h"

namespace flce {
namespace fast {

constexpr int THREADS = 256;
constexpr int WM = 4, WN = 4;
constexpr int BKB = 64;                   // bytes of K per stage and row
constexpr int NS = 4;                     // stages
constexpr int OPER = TILE * BKB;          // 16 KiB per operand per stage
constexpr int STAGE = 2 * OPER;
constexpr int LDS_BYTES = NS * STAGE;     // 128 KiB
constexpr int LOADS_PER_TILE = 8;         // buffer_load...lds instructions per wavefront per stage

typedef __attribute__((address_space(3))) void lds_void;

struct Src {
  const char* base;     // first byte of row 0 of the tensor (K offset already applied)
  int64_t ld_bytes;     // row pitch
  int row0;             // first row of this tile
  int rows;             // valid rows in the tensor
};

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const Src& s, int k_bytes) {
  int vr = min(TILE, s.rows - s.row0);
  if (vr < 0) vr = 0;
  // bytes from the tile's first row to the end of its last valid row
  const uint32_t n = vr > 0 ? (uint32_t)((int64_t)(vr - 1) * s.ld_bytes + k_bytes) : 0u;
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(s.base) + (int64_t)s.row0 * s.ld_bytes, 0, (int)n,
                                           0x00020000);
}

__device__ __forceinline__ int tile_m(int i, int r) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  return (wave >> 1) * 128 + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
}
__device__ __forceinline__ int tile_n(int j) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  return (wave & 1) * 128 + j * 32 + (lane & 31);
}
__device__ __forceinline__ int slot_of_lane() {      // which of the 4 lanes sharing a token column this is
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  return (wave >> 1) * 2 + (lane >> 5);
}

// s_waitcnt with vmcnt <= N and lgkmcnt == 0 (all of this wavefront's LDS reads returned).
// gfx9 encoding: vmcnt in bits [3:0] and [15:14], expcnt [6:4], lgkmcnt [11:8].
template <int N>
__device__ __forceinline__ void wait_vm_and_lds() {
  constexpr int lo = N & 15, hi = (N >> 4) & 3;
  __builtin_amdgcn_s_waitcnt((hi << 14) | (0x0 << 8) | (0x7 << 4) | lo);
}

struct Loader {
  __amdgpu_buffer_rsrc_t ra, rb;
  int va[4], vb[4];       // per-lane byte offsets of the 4 requests of each operand
  int lds_wave;           // LDS byte offset of this wavefront's first destination row
  __device__ __forceinline__ void init(const Src& A, const Src& B, int k_bytes) {
    ra = make_rsrc(A, k_bytes);
    rb = make_rsrc(B, k_bytes);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    lds_wave = wave * 64 * BKB;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = wave * 64 + i * 16 + (lane >> 2);
      const int chunk = (lane & 3) ^ ((row >> 2) & 3);
      va[i] = (int)(row * A.ld_bytes) + chunk * 16;
      vb[i] = (int)(row * B.ld_bytes) + chunk * 16;
    }
  }
  __device__ __forceinline__ void issue(char* lds, int stage, int k0_bytes) const {
    char* dst = lds + stage * STAGE + lds_wave;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, (lds_void*)(dst + i * 16 * BKB), 16, va[i], k0_bytes, 0, 0);
#pragma unroll
    for (int i = 0; i < 4; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rb, (lds_void*)(dst + OPER + i * 16 * BKB), 16, vb[i], k0_bytes, 0, 0);
  }
};

struct Frags {
  bf16x8 a[WM], b[WN];
};

// acc = A_tile . B_tile^T over k_bytes of K.  On return all wavefronts have passed a
// barrier after their last LDS read, so the caller may reuse `lds`.
__device__ __forceinline__ void mainloop(const Src& A, const Src& B, int k_bytes, char* lds, f32x16 (&acc)[WM][WN]) {
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int KT = k_bytes / BKB;
  Loader ld;
  ld.init(A, B, k_bytes);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int l32 = lane & 31, half = lane >> 5;
  const int sw = (l32 >> 2) & 3;
  // byte offsets of this lane's fragment inside an operand tile for the two MFMA K steps of a stage
  int offA[2], offB[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    const int c = ((ks * 2 + half) ^ sw) << 4;
    offA[ks] = ((wave >> 1) * 128 + l32) * BKB + c;
    offB[ks] = ((wave & 1) * 128 + l32) * BKB + c;
  }

  // prologue: tiles 0..2 requested, tile 0 landed
#pragma unroll
  for (int s = 0; s < NS - 1; ++s)
    if (s < KT) ld.issue(lds, s, s * BKB);
  if (KT > 2) wait_vm_and_lds<2 * LOADS_PER_TILE>();
  else if (KT > 1) wait_vm_and_lds<LOADS_PER_TILE>();
  else wait_vm_and_lds<0>();
  __builtin_amdgcn_s_barrier();
  Frags f0, f1;
#pragma unroll
  for (int i = 0; i < WM; ++i) f0.a[i] = *reinterpret_cast<const bf16x8*>(lds + offA[0] + i * 32 * BKB);
#pragma unroll
  for (int j = 0; j < WN; ++j) f0.b[j] = *reinterpret_cast<const bf16x8*>(lds + OPER + offB[0] + j * 32 * BKB);

#define FLCE_SB __builtin_amdgcn_sched_barrier(0);
#define FLCE_MF(F, i, j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(F.a[i], F.b[j], acc[i][j], 0, 0, 0);
#define FLCE_RA(F, i, st, ks) F.a[i] = *reinterpret_cast<const bf16x8*>((st) + offA[ks] + (i) * 32 * BKB);
#define FLCE_RB(F, j, st, ks) F.b[j] = *reinterpret_cast<const bf16x8*>((st) + OPER + offB[ks] + (j) * 32 * BKB);
#define FLCE_LA(i) \
  __builtin_amdgcn_raw_ptr_buffer_load_lds(ld.ra, (lds_void*)(dstn + (i) * 16 * BKB), 16, ld.va[i], k0n, 0, 0);
#define FLCE_LB(i) \
  __builtin_amdgcn_raw_ptr_buffer_load_lds(ld.rb, (lds_void*)(dstn + OPER + (i) * 16 * BKB), 16, ld.vb[i], k0n, 0, 0);
// One half of a K step: the 16 MFMAs of fragment set FM, with the 8 LDS reads that fill
// fragment set FR (from stage ST, MFMA K step KS) and 4 global requests (LX) in between.
#define FLCE_HALF(FM, FR, ST, KS, LX)                               \
  FLCE_MF(FM, 0, 0) FLCE_RA(FR, 0, ST, KS) FLCE_SB                  \
  FLCE_MF(FM, 0, 1) FLCE_RA(FR, 1, ST, KS) FLCE_SB                  \
  FLCE_MF(FM, 0, 2) LX(0) FLCE_SB                                   \
  FLCE_MF(FM, 0, 3) FLCE_SB                                         \
  FLCE_MF(FM, 1, 0) FLCE_RA(FR, 2, ST, KS) FLCE_SB                  \
  FLCE_MF(FM, 1, 1) FLCE_RA(FR, 3, ST, KS) FLCE_SB                  \
  FLCE_MF(FM, 1, 2) LX(1) FLCE_SB                                   \
  FLCE_MF(FM, 1, 3) FLCE_SB                                         \
  FLCE_MF(FM, 2, 0) FLCE_RB(FR, 0, ST, KS) FLCE_SB                  \
  FLCE_MF(FM, 2, 1) FLCE_RB(FR, 1, ST, KS) FLCE_SB                  \
  FLCE_MF(FM, 2, 2) LX(2) FLCE_SB                                   \
  FLCE_MF(FM, 2, 3) FLCE_SB                                         \
  FLCE_MF(FM, 3, 0) FLCE_RB(FR, 2, ST, KS) FLCE_SB                  \
  FLCE_MF(FM, 3, 1) FLCE_RB(FR, 3, ST, KS) FLCE_SB                  \
  FLCE_MF(FM, 3, 2) LX(3) FLCE_SB                                   \
  FLCE_MF(FM, 3, 3) FLCE_SB
#define FLCE_NOLOAD(i)

  // Steady state: K step kt computes tile kt and requests tile kt+3 into the stage that
  // was freed by the barrier of step kt-1.
  int kt = 0;
  for (; kt + NS - 1 < KT; ++kt) {
    const char* cur = lds + (kt & (NS - 1)) * STAGE;
    const char* nxt = lds + ((kt + 1) & (NS - 1)) * STAGE;
    char* dstn = lds + ((kt + NS - 1) & (NS - 1)) * STAGE + ld.lds_wave;
    const int k0n = (kt + NS - 1) * BKB;
    FLCE_SB
    FLCE_HALF(f0, f1, cur, 1, FLCE_LA)
    // tile kt+1 has landed once only tile kt+2 and the first half of tile kt+3 are in flight;
    // lgkmcnt(0): this wavefront holds all its fragments of tile kt
    wait_vm_and_lds<LOADS_PER_TILE + LOADS_PER_TILE / 2>();
    __builtin_amdgcn_s_barrier();
    FLCE_SB
    FLCE_HALF(f1, f0, nxt, 0, FLCE_LB)
  }
  // Drain: the last (up to NS-1) tiles, nothing left to request.
  for (; kt < KT; ++kt) {
    const char* cur = lds + (kt & (NS - 1)) * STAGE;
    const char* nxt = lds + ((kt + 1) & (NS - 1)) * STAGE;   // past the last tile: stale data, never used
    FLCE_SB
    FLCE_HALF(f0, f1, cur, 1, FLCE_NOLOAD)
    if (kt + 2 < KT) wait_vm_and_lds<LOADS_PER_TILE>();
    else wait_vm_and_lds<0>();
    __builtin_amdgcn_s_barrier();
    FLCE_SB
    FLCE_HALF(f1, f0, nxt, 0, FLCE_NOLOAD)
  }
  wait_vm_and_lds<0>();
  __builtin_amdgcn_s_barrier();
#undef FLCE_SB
#undef FLCE_MF
#undef FLCE_RA
#undef FLCE_RB
#undef FLCE_LA
#undef FLCE_LB
#undef FLCE_HALF
#undef FLCE_NOLOAD
}

}  // namespace fast
}  // namespace flce
