// bf16 main loop tuned for gfx950: 256 x 256 tile, 256 threads = 4 wavefronts (one per
// SIMD) arranged 2 x 2, each owning a 128 x 128 sub-tile (4 x 4 blocks of the
// 32x32x16 MFMA, 256 fp32 accumulators per lane).
//
//   * Operand tiles go from global memory straight into LDS (buffer_load ... lds,
//     16 bytes per lane), four stages of 32 bf16 of K deep, so a tile is requested
//     two to three K steps before it is read.  Rows past the end of a tensor are
//     zero-filled by the buffer's range check.
//   * Each operand may be stored either way round in memory:
//       KC ("K contiguous"): 256 tile rows, each with its 32 K values adjacent (64 bytes).
//           LDS tile [256][64 B]; fragments are plain 128-bit LDS reads.
//       KR ("K rows"): the 32 K values of a tile row lie in 32 different memory rows, and
//           one memory row holds the 256 tile rows' values side by side (512 bytes).
//           LDS tile [32][512 B]; fragments come from the transposing LDS read
//           (ds_read_b64_tr_b16: 16 lanes hand in four K rows of 4 x 8 bytes and each
//           lane gets back 4 consecutive K values of one tile row).
//     This lets dH = G.W and dW = G^T.H read G, W and H where they are, with no
//     transposed copies.
//       PK ("packed"): the operand has been copied into the order of its LDS tiles beforehand:
//           per 256-row block and K step one 16 KiB image of the KC tile (swizzle included),
//           images of a block one after the other.  Every request is then 1 KiB of consecutive
//           bytes (KC: 16 pieces of 64 bytes) and the fragments are KC's.  Worth a copy for an
//           operand that is small and read many times (the hidden states in the forward and the
//           recompute: +2 % on the whole loop).
//   * LDS swizzles (applied on the global side, because the DMA writes LDS linearly):
//     KC: 16-byte chunk index ^ (row / 4) % 4; KR: 64-byte chunk index ^ (k % 4).  Both
//     spread what one LDS instruction touches in a cycle over all 64 banks.
//   * Fragments are double buffered in registers and the single barrier per K step
//     sits between the two MFMA groups of the step: LDS latency and the barrier wait
//     are both covered by 16 independent MFMAs.
//   * The instruction order inside a K step is pinned by hand (LDS reads and global
//     requests spread between consecutive MFMAs, fenced with scheduling barriers):
//     with one wavefront per SIMD a burst of memory instructions stalls the MFMA
//     stream.
//
// Requires the K extent to be a multiple of 32 elements and offsets inside one tile's
// address window within 2^32 bytes (unsigned 32-bit buffer offsets); the generic loop in tile_mma.h covers everything else.
#pragma once
#include <type_traits>

#include "tile_mma.h"

namespace flce {
namespace fast {

constexpr int THREADS = 256;
constexpr int WM = 4, WN = 4;
constexpr int BK = 32;                    // K elements per stage
#ifndef FLCE_STAGES
#define FLCE_STAGES 4
#endif
constexpr int NS = FLCE_STAGES;           // stages
constexpr int OPER = TILE * BK * 2;       // 16 KiB per operand per stage (either layout)
constexpr int STAGE = 2 * OPER;
constexpr int LDS_BYTES = NS * STAGE;     // 128 KiB with 4 stages

enum : int { KC = 0, KR = 1, PK = 2, KB = 3, RB = 4 };
// KB and RB read a matrix that is stored in blocks of 16 rows x 32 columns (1 KiB, row-major inside), the blocks of a
// group of 16 rows one after the other along the columns and the row groups `ld_bytes` apart ("blocked"): both of its
// readers then fetch whole blocks, 1 KiB of consecutive bytes per request.
//   KB: K runs along the columns (32 columns = one block per 16 tile rows and K step); the LDS tile and the fragment
//       reads are KC's.  Operand: base = the block of the tile's first row and first K column, ld_bytes = bytes
//       from one row group to the next.
//   RB: K runs over the rows (two row groups per K step), the 256 tile rows are 256 consecutive columns (8 blocks);
//       the LDS tile holds the 16 blocks as they are, [2][8][16 rows][64 B], and the fragments come from the
//       transposing LDS read (rows of a block lie 64 bytes apart: every bank once without a swizzle).  Operand:
//       base = the block of the first K row and the tile's first column, ld_bytes as for KB.
constexpr bool kc_like(int layout) { return layout == KC || layout == PK || layout == KB; }

typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

// One operand of the contraction.
//   KC: base = first byte of row 0 of the tensor at the first K element; row0 = first tile
//       row; rows = valid rows of the tensor; width_bytes unused.
//   KR: base = first byte of K row 0 at the tile's first column; rows = valid K rows from
//       there; width_bytes = valid bytes of the tile's 512-byte column window (columns
//       beyond it may read as the next row's data: the caller masks what they produce).
struct Operand {
  const char* base;
  int64_t ld_bytes;
  int row0;
  int rows;
  int width_bytes;
};

// The global -> LDS request is issued through inline assembly: as an intrinsic the compiler
// treats it as a store that may alias every later LDS read it cannot disambiguate (the
// transposing reads among them) and waits for vmcnt(0) before each, which serialises the
// pipeline.  Here the only consumers are separated from the DMA by the explicit vmcnt
// wait + barrier of the main loop.  M0 carries the LDS destination of the wavefront.
__device__ __forceinline__ void dma16(u32x4 rsrc, uint32_t lds_addr, uint32_t voffset, uint32_t soffset) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :
               : "s"(lds_addr), "v"(voffset), "s"(rsrc), "s"(soffset)
               : "memory", "m0");
}

__device__ __forceinline__ uint32_t lds_address(const char* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)p;
}

template <int LAYOUT, int TILE_ROWS = TILE>
__device__ __forceinline__ u32x4 make_rsrc(const Operand& s, int k_elems) {
  uint32_t n = 0;
  const char* b = s.base;
  if (LAYOUT == PK) {
    n = (uint32_t)(k_elems / BK) * OPER;
  } else if (LAYOUT == KB) {         // 16 row groups, the last one up to the end of the K extent
    n = (uint32_t)(15 * s.ld_bytes + (int64_t)(k_elems / BK) * 1024);
  } else if (LAYOUT == RB) {         // k_elems / 16 row groups, 8 blocks of the last one
    if (k_elems > 0) n = (uint32_t)((int64_t)(k_elems / 16 - 1) * s.ld_bytes + 8 * 1024);
  } else if (LAYOUT == KC) {
    int vr = min(TILE_ROWS, s.rows - s.row0);
    if (vr > 0) n = (uint32_t)((int64_t)(vr - 1) * s.ld_bytes + k_elems * 2);
    b += (int64_t)s.row0 * s.ld_bytes;
  } else {
    const int kr = min(s.rows, k_elems);
    if (kr > 0 && s.width_bytes > 0) n = (uint32_t)((int64_t)(kr - 1) * s.ld_bytes + s.width_bytes);
  }
  // raw buffer descriptor: 48-bit base, stride 0, num_records in bytes, untyped 32-bit data format
  const uint64_t addr = (uint64_t)(uintptr_t)b;
  u32x4 r = {(uint32_t)addr, (uint32_t)(addr >> 32) & 0xFFFFu, n, 0x00020000u};
  r[0] = __builtin_amdgcn_readfirstlane(r[0]);
  r[1] = __builtin_amdgcn_readfirstlane(r[1]);
  r[2] = __builtin_amdgcn_readfirstlane(r[2]);
  return r;
}

__device__ __forceinline__ int tile_m(int i, int r) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  return (wave >> 1) * 128 + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
}
__device__ __forceinline__ int tile_n(int j) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  return (wave & 1) * 128 + j * 32 + (lane & 31);
}
__device__ __forceinline__ int slot_of_lane() {      // which of the 4 lanes sharing an N column this is
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

// Global -> LDS requests of one operand: REQS per wavefront per stage (4 for a 256-row tile; a K-contiguous tile
// may also be 128 rows high: 2), 1 KiB each, written linearly into this wavefront's slice of the operand tile.
template <int LAYOUT, int REQS = 4>
struct Loader {
  static_assert(REQS == 4 || (LAYOUT == KC && REQS == 2), "a half-height tile exists in the K-contiguous layout only");
  u32x4 rs;
  uint32_t v[REQS];       // per-lane byte offsets of the requests (K tile 0); unsigned: a window may reach 2^32 bytes
  uint32_t k_step;        // KC: bytes of K per stage (scalar offset); KR: bytes of 32 K rows (added per lane)
  __device__ __forceinline__ void init(const Operand& s, int k_elems) {
    rs = make_rsrc<LAYOUT, 64 * REQS>(s, k_elems);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
    for (int i = 0; i < REQS; ++i) {
      if (LAYOUT == PK) {
        v[i] = (uint32_t)(wave * 4096 + i * 1024 + lane * 16);
      } else if (LAYOUT == KB) {     // request = row group wave * 4 + i of the tile: one block, KC's chunk order
        const int chunk = (lane & 3) ^ ((lane >> 4) & 3);
        v[i] = (uint32_t)((wave * 4 + i) * s.ld_bytes) + (lane >> 2) * 64 + chunk * 16;
      } else if (LAYOUT == RB) {     // request = block (row group, column block) = ((wave * 4 + i) / 8, % 8), as it is
        const int b = wave * 4 + i;
        v[i] = (uint32_t)((b >> 3) * s.ld_bytes) + (b & 7) * 1024 + lane * 16;
      } else if (LAYOUT == KC) {
        const int row = wave * (16 * REQS) + i * 16 + (lane >> 2);
        const int chunk = (lane & 3) ^ ((row >> 2) & 3);
        v[i] = (uint32_t)(row * s.ld_bytes) + chunk * 16;
      } else {
        const int krow = wave * 8 + i * 2 + (lane >> 5);
        const int off = ((lane & 31) * 16) ^ ((krow & 3) << 6);
        v[i] = (uint32_t)(krow * s.ld_bytes) + off;
      }
    }
    k_step = LAYOUT == PK ? OPER : LAYOUT == KC ? BK * 2 : LAYOUT == KB ? 1024 : LAYOUT == RB ? (uint32_t)(2 * s.ld_bytes)
                                                                                      : (uint32_t)(BK * s.ld_bytes);
  }
  // request i of K tile kt into `dst` (this wavefront's slice of the operand tile of some stage)
  __device__ __forceinline__ void issue(int i, char* dst, int kt) const {
    if (kc_like(LAYOUT))
      dma16(rs, lds_address(dst + i * 1024), v[i], (uint32_t)kt * k_step);
    else   // the K advance moves to other rows: keep it in the per-lane offset, which the range check covers
      dma16(rs, lds_address(dst + i * 1024), v[i] + (uint32_t)kt * k_step, 0);
  }
};

// Per-lane LDS byte offsets of the fragment reads of one operand; wsub = which half of the tile's rows this
// wavefront works on (BLOCKS 32-row blocks each: 4 for a 256-row tile, 2 for a 128-row one).
template <int LAYOUT, int BLOCKS = 4>
struct FragAddr {
  static_assert(BLOCKS == 4 || (LAYOUT == KC && BLOCKS == 2), "a half-height tile exists in the K-contiguous layout only");
  int o[4];   // KC: o[ks] for the two MFMA K steps (o[2], o[3] unused); KR: o[i] for the 4 blocks
  __device__ __forceinline__ void init(int wsub) {
    const int lane = threadIdx.x & 63;
    if (kc_like(LAYOUT)) {
      const int l32 = lane & 31, half = lane >> 5, sw = (l32 >> 2) & 3;
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) o[ks] = (wsub * 32 * BLOCKS + l32) * 64 + (((ks * 2 + half) ^ sw) << 4);
      o[2] = o[3] = 0;
    } else {
      const int e = (lane >> 2) & 3, q = lane & 3, mg = (lane >> 4) & 1, kh = lane >> 5;
#pragma unroll
      for (int i = 0; i < 4; ++i)
        o[i] = LAYOUT == RB ? (wsub * 4 + i) * 1024 + (8 * kh + e) * 64 + 32 * mg + 8 * q
                            : (8 * kh + e) * 512 + wsub * 256 + 64 * (i ^ e) + 32 * mg + 8 * q;
    }
  }
  static constexpr int READS = kc_like(LAYOUT) ? BLOCKS : 8;   // LDS reads per MFMA K step
};

struct Frags {
  bf16x8 a[WM], b[WN];
};

// Read number t (0 .. READS-1) of the fragments of one operand for MFMA K step ks of a stage.
template <int LAYOUT, int BLOCKS>
__device__ __forceinline__ void read_frag(bf16x8 (&f)[4], const FragAddr<LAYOUT, BLOCKS>& fa, const char* tile, int ks, int t) {
  if (kc_like(LAYOUT)) {
    f[t] = *reinterpret_cast<const bf16x8*>(tile + fa.o[ks] + t * 32 * 64);
  } else {
    const int i = t >> 1, r = t & 1;
    // K rows 16 ks + 4 r + (0..3, +8 for the upper lanes): KR has them 512 bytes apart; RB has the 16 rows of MFMA
    // K step ks in row group ks of the tile (8 blocks of 1 KiB), 64 bytes apart
    const int koff = LAYOUT == RB ? ks * 8192 + r * 256 : (16 * ks + 4 * r) * 512;
    const s16x4 h = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(tile + fa.o[i] + koff));
    const bf16x4 hb = __builtin_bit_cast(bf16x4, h);
    if (r == 0) { f[i][0] = hb[0]; f[i][1] = hb[1]; f[i][2] = hb[2]; f[i][3] = hb[3]; }
    else        { f[i][4] = hb[0]; f[i][5] = hb[1]; f[i][6] = hb[2]; f[i][7] = hb[3]; }
  }
}

// The contraction of one tile, split in two calls so that a kernel that works on several
// tiles can request the first stages of the next tile before it post-processes the
// accumulators of the current one:
//   start(A, B, k_elems, lds): requests K tiles 0..2 into stages 0..2 (all stages must be free:
//                              every wavefront has passed the final barrier of the previous run);
//   run(lds, acc):             acc = A_tile . B_tile^T over k_elems of K (a multiple of 32).  On
//                              return all wavefronts have passed a barrier after their last LDS
//                              read, so the caller may reuse `lds` or call start() again.
//
// WITH_MFMA = false leaves the matrix instructions out (everything else, i.e. the global -> LDS requests, the LDS
// fragment reads, the waits and barriers, stays): only the measurement probe uses it, to time the data path alone.
//
// AM = 32-row blocks of A per wavefront: 4 is the 256 x 256 tile above; 2 halves the A tile (128 rows, K-contiguous
// only), i.e. a 128 x 256 tile with 128 accumulators per lane, which lets two workgroups share a CU (with NSTAGES = 3
// a workgroup then needs 72 KiB of LDS).  `acc` has AM x 4 blocks.
template <int LA, int LB, bool WITH_MFMA = true, int AM = WM, int NSTAGES = NS>
struct Pipe {
  static_assert(AM == 4 || (AM == 2 && LA == KC), "a half-height A tile exists in the K-contiguous layout only");
  static constexpr int REQS_A = AM;                    // requests per wavefront per stage, A (1 KiB each)
  static constexpr int OPER_A = AM * 4096;             // bytes of the A tile of one stage
  static constexpr int STAGE_BYTES = OPER_A + OPER;    // A tile, then B tile
  static constexpr int LDS_TOTAL = NSTAGES * STAGE_BYTES;
  static constexpr int LOADS = REQS_A + 4;             // requests per wavefront per K tile
  static constexpr int NM = AM * WN;                   // MFMAs per half step
  Loader<LA, REQS_A> la;
  Loader<LB> lb;
  FragAddr<LA, AM> fa;
  FragAddr<LB> fb;
  int KT, lds_wave;

  __device__ __forceinline__ void start(const Operand& A, const Operand& B, int k_elems, char* lds) {
    KT = k_elems / BK;
    la.init(A, k_elems);
    lb.init(B, k_elems);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    fa.init(wave >> 1);
    fb.init(wave & 1);
    lds_wave = wave * 4096;      // this wavefront's slice of a 256-row operand tile (of a shorter A tile: pro rata)
    // Opaque to the optimiser: in a kernel that walks several tiles these two are loop invariant, and everything
    // derived from them (a dozen comparisons of the K count, the LDS address of every request of every stage)
    // would be precomputed once and kept alive in scalar registers across the whole tile loop, which overflows them.
    asm volatile("" : "+s"(KT), "+s"(lds_wave));
#pragma unroll
    for (int s = 0; s < NSTAGES - 1; ++s)
      if (s < KT) {
#pragma unroll
        for (int i = 0; i < REQS_A; ++i) la.issue(i, lds + s * STAGE_BYTES + lds_wave * REQS_A / 4, s);
#pragma unroll
        for (int i = 0; i < 4; ++i) lb.issue(i, lds + s * STAGE_BYTES + OPER_A + lds_wave, s);
      }
  }

  // waits until at most n whole K tiles of this wavefront's requests are outstanding (and its LDS reads returned)
  static __device__ __forceinline__ void wait_tiles_in_flight(int n) {
    static_assert(NSTAGES >= 3 && NSTAGES <= 6, "the switch below covers up to NSTAGES - 2 tiles in flight");
    switch (n) {
      case 0: wait_vm_and_lds<0>(); break;
      case 1: wait_vm_and_lds<LOADS>(); break;
      case 2: wait_vm_and_lds<2 * LOADS>(); break;
      case 3: wait_vm_and_lds<3 * LOADS>(); break;
      default: wait_vm_and_lds<4 * LOADS>(); break;
    }
  }

  __device__ __forceinline__ void run(char* lds, f32x16 (&acc)[AM][WN]) {
    constexpr int RA = FragAddr<LA, AM>::READS, RB = FragAddr<LB>::READS, RT = RA + RB;
    if (KT <= 0) {          // an empty K extent (no counted row, or a K slice past the end): the tile is zero
#pragma unroll
      for (int i = 0; i < AM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
      __builtin_amdgcn_s_barrier();
      return;
    }

    // tile 0 has landed once only the other tiles requested by start() are in flight
    wait_tiles_in_flight(min(KT, NSTAGES - 1) - 1);
    __builtin_amdgcn_s_barrier();
    Frags f0, f1;
#pragma unroll
    for (int t = 0; t < RA; ++t) read_frag<LA>(f0.a, fa, lds, 0, t);
#pragma unroll
    for (int t = 0; t < RB; ++t) read_frag<LB>(f0.b, fb, lds + OPER_A, 0, t);

    // One half of a K step: the NM (16) MFMAs of fragment set FM; between them the LDS reads that
    // fill fragment set FR (stage `st`, MFMA K step ks) and, if load_kt >= 0, the global
    // requests of operand `which` (0 = A, 1 = B) of K tile load_kt into stage `lst`.
    // `first`: the very first half step of a tile starts every accumulator block from zero (the
    // matrix instruction takes the constant as its addend: no pass over the 256 registers to clear them).
    auto half_step = [&](auto first, const Frags& FM, Frags& FR, const char* st, int ks, int which, int load_kt,
                         char* lst) {
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int s = 0; s < NM; ++s) {
        const int mi = s >> 2, mj = s & 3;
        if constexpr (WITH_MFMA) {
          if constexpr (decltype(first)::value) {
            const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            acc[mi][mj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(FM.a[mi], FM.b[mj], zero, 0, 0, 0);
          } else {
            acc[mi][mj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(FM.a[mi], FM.b[mj], acc[mi][mj], 0, 0, 0);
          }
        } else {
          // keep the fragment reads alive without arithmetic on them
          asm volatile("" ::"v"(FM.a[mi]), "v"(FM.b[mj]));
        }
        // reads t with t * NM / RT == s: spread evenly over the MFMA slots
#pragma unroll
        for (int t = 0; t < RT; ++t)
          if (t * NM / RT == s) {
            if (t < RA) read_frag<LA>(FR.a, fa, st, ks, t);
            else read_frag<LB>(FR.b, fb, st + OPER_A, ks, t - RA);
          }
        // the requests of one operand, evenly spread too: one in the middle of every NM / requests slots
        constexpr int PER_A = NM / REQS_A, PER_B = NM / 4;
        if (load_kt >= 0) {
          if (which == 0) {
            if (s % PER_A == PER_A / 2) la.issue(s / PER_A, lst + lds_wave * REQS_A / 4, load_kt);
          } else {
            if (s % PER_B == PER_B / 2) lb.issue(s / PER_B, lst + OPER_A + lds_wave, load_kt);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    constexpr std::true_type FIRST{};
    constexpr std::false_type LATER{};

    // Steady state: K step kt computes tile kt (stage sc) and requests tile kt+NSTAGES-1 into the stage that
    // was freed by the barrier of step kt-1 (the one before sc in the ring).
    auto stage_at = [&](int idx) { return lds + idx * STAGE_BYTES; };
    auto after = [](int idx) { return idx + 1 == NSTAGES ? 0 : idx + 1; };
    auto before = [](int idx) { return idx == 0 ? NSTAGES - 1 : idx - 1; };
    auto steady_step = [&](auto first, int kt, int sc) {
      char* lst = stage_at(before(sc));
      half_step(first, f0, f1, stage_at(sc), 1, 0, kt + NSTAGES - 1, lst);
      // tile kt+1 has landed once only tiles kt+2 .. kt+NSTAGES-2 and A's requests of tile kt+NSTAGES-1 are in
      // flight; lgkmcnt(0): this wavefront holds all its fragments of tile kt
      wait_vm_and_lds<(NSTAGES - 3) * LOADS + REQS_A>();
      __builtin_amdgcn_s_barrier();
      half_step(LATER, f1, f0, stage_at(after(sc)), 0, 1, kt + NSTAGES - 1, lst);
    };
    // Drain: the last (up to NS-1) tiles, nothing left to request.
    auto drain_step = [&](auto first, int kt, int sc) {
      half_step(first, f0, f1, stage_at(sc), 1, 0, -1, nullptr);
      wait_tiles_in_flight(max(0, KT - kt - 2));            // tile kt+1 landed; the later ones may be in flight
      __builtin_amdgcn_s_barrier();
      half_step(LATER, f1, f0, stage_at(after(sc)), 0, 1, -1, nullptr);   // past the last tile: stale data, never used
    };
    int kt = 1, sc = 1 % NSTAGES;
    if (NSTAGES - 1 < KT) {
      steady_step(FIRST, 0, 0);
      for (; kt + NSTAGES - 1 < KT; ++kt, sc = after(sc)) steady_step(LATER, kt, sc);
    } else {
      drain_step(FIRST, 0, 0);
    }
    for (; kt < KT; ++kt, sc = after(sc)) drain_step(LATER, kt, sc);
    wait_vm_and_lds<0>();
    __builtin_amdgcn_s_barrier();
  }
};

template <int LA, int LB>
__device__ __forceinline__ void mainloop(const Operand& A, const Operand& B, int k_elems, char* lds,
                                         f32x16 (&acc)[WM][WN]) {
  Pipe<LA, LB> pipe;
  pipe.start(A, B, k_elems, lds);
  pipe.run(lds, acc);
}

}  // namespace fast
}  // namespace flce
