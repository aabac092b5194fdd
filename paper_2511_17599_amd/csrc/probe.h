// Measurement probe (not part of the computation): what the pieces of the tuned main loop sustain on their own on
// this chip, so that a kernel's rate can be read against the rate of the matrix pipe alone and of the bare loop
// rather than against the nominal peak only.  One workgroup per CU-sized slot, 4 wavefronts, as in the real kernels.
//   PROBE_MFMA     : the 32x32x16 bf16 MFMA issued back to back from registers (fragments loaded once): the rate
//                    the matrix pipe sustains under the chip's power limit with this data.
//   PROBE_LOOP_KR  : the complete main loop with A K-contiguous and B read across memory rows,
//                    tile after tile with no post-processing of the accumulators.
//   PROBE_LOOP_PK  : the same with B pre-tiled (its bytes taken as the LDS tile images of its K steps, whatever they
//                    hold): the main loop of the forward / recompute.
//   PROBE_LOOP_KC  : the same with both operands K-contiguous.
//   PROBE_DATA_KR / PROBE_DATA_KC : those loops with the matrix instructions left out (global -> LDS requests, LDS
//                    fragment reads, waits, barriers only): the data path alone.
//   PROBE_FREE_RUN : the matrix instructions from registers AND the forward layout's global -> LDS requests and LDS
//                    fragment reads of every K step, issued side by side with no wait or barrier between them (the
//                    fragments read are discarded): what the two streams reach when nothing makes one wait for the
//                    other, i.e. how much of the complete loop's loss is synchronisation.
//   PROBE_LOOP_KR_SOFTMAX : PROBE_LOOP_KR plus, after every tile, the plain-ALU work of the forward's tile
//                    post-processing (per lane and column: a maximum over the column's accumulators, then the sum
//                    of exp2 of their distances to it), with no overlap with the next tile's matrix work: one
//                    wavefront per SIMD does both in turn.
//   PROBE_HALF_KR / PROBE_HALF_KR_SOFTMAX : the same two on a 128 x 256 tile (A tile of half the height, 128
//                    accumulators per lane, three stages, 72 KiB of LDS) with TWO workgroups per CU, so that one
//                    workgroup's post-processing can overlap the other's matrix work.  Launch twice the workgroups
//                    for the same total work.
//   PROBE_LOOP_KR_COLD : PROBE_LOOP_KR with every group of workgroups walking its own contiguous run of A tiles, so
//                    that no A tile is read twice in a launch (the other modes walk overlapping runs: what one group
//                    reads, its neighbour read one tile earlier and the caches still hold it).  This is how the
//                    forward reads W: every tile comes from HBM.
//   PROBE_MFMA_16X16 : PROBE_MFMA with the 16x16x32 bf16 MFMA instead (8 x 8 blocks of 4 accumulators per wavefront:
//                    the same 128 x 128 sub-tile, the same flops per fragment, a quarter of the accumulator
//                    registers read and written per instruction).
//   PROBE_PAIR_*   : the complete main loop for other pairs of operand layouts (A / B): KR / KR is the dW
//                    contraction, KR / KC the dH contraction; PK in a pair shows what a pre-tiled copy of that
//                    operand would give.  Timing only: an operand's bytes are taken from A, B or BT as that layout,
//                    whatever they hold.
#pragma once
#include "mainloop_fast.h"

namespace flce {

enum : int {
  PROBE_MFMA = 0, PROBE_LOOP_KR = 1, PROBE_LOOP_KC = 2, PROBE_DATA_KR = 3, PROBE_DATA_KC = 4, PROBE_FREE_RUN = 5,
  PROBE_LOOP_KR_SOFTMAX = 6, PROBE_HALF_KR = 7, PROBE_HALF_KR_SOFTMAX = 8, PROBE_LOOP_KR_COLD = 9, PROBE_MFMA_16X16 = 10, PROBE_LOOP_PK = 11,
  PROBE_PAIR_KR_KR = 12, PROBE_PAIR_PK_KR = 13, PROBE_PAIR_KR_KC = 14, PROBE_PAIR_KR_PK = 15, PROBE_PAIR_PK_PK = 16
};

struct ProbeArgs {
  const bf16_t* A;      // [a_rows][k_elems], K-contiguous (plays W)
  const bf16_t* B;      // [b_rows][k_elems], K-contiguous (plays H)
  const bf16_t* BT;     // [k_elems][b_rows] (plays H transposed)
  int a_rows, b_rows, k_elems;
  int tiles_per_wg;     // tiles each workgroup walks along A (wrapping around a_rows)
  float* sink;          // [gridDim.x * 256] one float per thread, so that nothing is optimised away
};

// The arithmetic of one tile's softmax statistics on the accumulators as they lie in the registers (each lane holds,
// per block column j, AM x 16 entries of one output column): the same instruction mix as the forward's tile
// post-processing, minus its bookkeeping.
template <int AM>
__device__ __forceinline__ float softmax_work(f32x16 (&acc)[AM][fast::WN]) {
  constexpr float LOG2E = 1.4426950408889634f;
  float out = 0.f;
#pragma unroll
  for (int j = 0; j < fast::WN; ++j) {
    float m = -INFINITY;
#pragma unroll
    for (int i = 0; i < AM; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float v;
        asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(acc[i][j][r]));
        m = fmaxf(m, v);
      }
    const float mc = m * LOG2E;
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < AM; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float v;
        asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(acc[i][j][r]));
        sum += __builtin_amdgcn_exp2f(fmaf(v, LOG2E, -mc));
      }
    out += sum + m;
  }
  return out;
}

typedef __attribute__((ext_vector_type(4))) float f32x4_probe;

template <int UNUSED = 0>
__global__ __launch_bounds__(fast::THREADS) void probe_mfma16_kernel(ProbeArgs p) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int b0 = (blockIdx.x % (p.b_rows / TILE)) * TILE;
  bf16x8 fa[8], fb[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
    fa[i] = *reinterpret_cast<const bf16x8*>(p.A + (int64_t)((wave * 8 + i) * 64 + lane) % p.a_rows * p.k_elems);
#pragma unroll
  for (int j = 0; j < 8; ++j)
    fb[j] = *reinterpret_cast<const bf16x8*>(p.B + (int64_t)(b0 + (wave * 8 + j) * 64 % TILE + lane) % p.b_rows * p.k_elems);
  f32x4_probe acc[8][8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[i][j] = f32x4_probe{0.f, 0.f, 0.f, 0.f};
  const int steps = p.tiles_per_wg * (p.k_elems / 32);       // MFMA K steps (32 deep) of all tiles
  for (int s = 0; s < steps; ++s) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
  }
  float keep = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float v;
      asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(acc[i][j][0]));
      keep += v;
    }
  p.sink[(int64_t)blockIdx.x * fast::THREADS + threadIdx.x] = keep;
}

// One operand of a layout pair, tile index `tile`, taken from the probe's buffers (timing only).
template <int LAYOUT>
__device__ __forceinline__ fast::Operand probe_operand(const ProbeArgs& p, int tile, bool is_a) {
  const bf16_t* M = is_a ? p.A : p.B;                 // [rows][k_elems]
  const int rows = is_a ? p.a_rows : p.b_rows;
  const int64_t ld = (int64_t)p.k_elems * 2;
  const int row0 = (tile * TILE) % rows;
  if (LAYOUT == fast::KC) return fast::Operand{reinterpret_cast<const char*>(M), ld, row0, rows, 0};
  if (LAYOUT == fast::PK) return fast::Operand{reinterpret_cast<const char*>(M) + (int64_t)row0 * ld, 0, 0, 0, 0};
  // KR: K over the rows of BT [k_elems][b_rows], a window of 256 columns
  const int col0 = (tile * TILE) % p.b_rows;
  return fast::Operand{reinterpret_cast<const char*>(p.BT) + (int64_t)col0 * 2, (int64_t)p.b_rows * 2, 0, p.k_elems,
                       TILE * 2};
}

template <int LA, int LB>
__global__ __launch_bounds__(fast::THREADS) void probe_pair_kernel(ProbeArgs p) {
  extern __shared__ __align__(16) char lds[];
  f32x16 acc[fast::WM][fast::WN];
  const int n_bt = p.b_rows / TILE;
  float keep = 0.f;
  fast::Pipe<LA, LB> pipe;
  for (int t = 0; t < p.tiles_per_wg; ++t) {
    pipe.start(probe_operand<LA>(p, blockIdx.x / n_bt + t, true), probe_operand<LB>(p, blockIdx.x % n_bt, false),
               p.k_elems, lds);
    pipe.run(lds, acc);
#pragma unroll
    for (int i = 0; i < fast::WM; ++i)
#pragma unroll
      for (int j = 0; j < fast::WN; ++j) {
        float v;
        asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(acc[i][j][(i * 4 + j) & 15]));
        keep += v;
      }
  }
  p.sink[(int64_t)blockIdx.x * fast::THREADS + threadIdx.x] = keep;
}

// 128 x 256 tiles, two workgroups per CU (at most 256 registers per lane, 72 KiB of LDS per workgroup).
template <bool SOFTMAX>
__global__ __launch_bounds__(fast::THREADS, 2) void probe_half_kernel(ProbeArgs p) {
  extern __shared__ __align__(16) char lds[];
  using HalfPipe = fast::Pipe<fast::KC, fast::KR, true, 2, 3>;
  constexpr int AROWS = 128;
  f32x16 acc[2][fast::WN];
  const int n_at = p.a_rows / AROWS, n_bt = p.b_rows / TILE;
  const int b0 = (blockIdx.x % n_bt) * TILE;
  float keep = 0.f;
  HalfPipe pipe;
  const int64_t ld = (int64_t)p.k_elems * 2;
  for (int t = 0; t < p.tiles_per_wg; ++t) {
    const int a0 = ((blockIdx.x / n_bt + t) % n_at) * AROWS;
    const fast::Operand As{reinterpret_cast<const char*>(p.A), ld, a0, p.a_rows, 0};
    const fast::Operand Bs{reinterpret_cast<const char*>(p.BT) + (int64_t)b0 * 2, (int64_t)p.b_rows * 2, 0, p.k_elems,
                           TILE * 2};
    pipe.start(As, Bs, p.k_elems, lds);
    pipe.run(lds, acc);
    if constexpr (SOFTMAX) {
      keep += softmax_work<2>(acc);
    } else {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < fast::WN; ++j) {
          float v;
          asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(acc[i][j][(i * 4 + j) & 15]));
          keep += v;
        }
    }
  }
  p.sink[(int64_t)blockIdx.x * fast::THREADS + threadIdx.x] = keep;
}
constexpr int PROBE_HALF_LDS = fast::Pipe<fast::KC, fast::KR, true, 2, 3>::LDS_TOTAL;

template <int MODE>
__global__ __launch_bounds__(fast::THREADS) void probe_kernel(ProbeArgs p) {
  extern __shared__ __align__(16) char lds[];
  f32x16 acc[fast::WM][fast::WN];
  const int n_at = p.a_rows / TILE, n_bt = p.b_rows / TILE;
  const int b0 = (blockIdx.x % n_bt) * TILE;
  float keep = 0.f;
  if constexpr (MODE == PROBE_MFMA) {
    // fragments: 16 bytes per lane straight from global memory, then registers only
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    bf16x8 fa[fast::WM], fb[fast::WN];
#pragma unroll
    for (int i = 0; i < fast::WM; ++i)
      fa[i] = *reinterpret_cast<const bf16x8*>(p.A + (int64_t)((wave * 4 + i) * 64 + lane) % p.a_rows * p.k_elems);
#pragma unroll
    for (int j = 0; j < fast::WN; ++j)
      fb[j] = *reinterpret_cast<const bf16x8*>(p.B + (int64_t)(b0 + (wave * 4 + j) * 64 % TILE + lane) % p.b_rows * p.k_elems);
#pragma unroll
    for (int i = 0; i < fast::WM; ++i)
#pragma unroll
      for (int j = 0; j < fast::WN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    const int steps = p.tiles_per_wg * (p.k_elems / 16);       // MFMA K steps of all tiles
    for (int s = 0; s < steps; ++s) {
#pragma unroll
      for (int i = 0; i < fast::WM; ++i)
#pragma unroll
        for (int j = 0; j < fast::WN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
  } else if constexpr (MODE == PROBE_FREE_RUN) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    bf16x8 fa[fast::WM], fb[fast::WN];
#pragma unroll
    for (int i = 0; i < fast::WM; ++i)
      fa[i] = *reinterpret_cast<const bf16x8*>(p.A + (int64_t)((wave * 4 + i) * 64 + lane) % p.a_rows * p.k_elems);
#pragma unroll
    for (int j = 0; j < fast::WN; ++j)
      fb[j] = *reinterpret_cast<const bf16x8*>(p.B + (int64_t)(b0 + (wave * 4 + j) * 64 % TILE + lane) % p.b_rows * p.k_elems);
#pragma unroll
    for (int i = 0; i < fast::WM; ++i)
#pragma unroll
      for (int j = 0; j < fast::WN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    fast::Loader<fast::KC> la;
    fast::Loader<fast::KR> lb;
    fast::FragAddr<fast::KC> fra;
    fast::FragAddr<fast::KR> frb;
    fra.init(wave >> 1);
    frb.init(wave & 1);
    const int lds_wave = __builtin_amdgcn_readfirstlane(wave) * 4096;
    const int64_t ld = (int64_t)p.k_elems * 2;
    const int KT = p.k_elems / fast::BK;
    for (int t = 0; t < p.tiles_per_wg; ++t) {
      const int a0 = ((blockIdx.x / n_bt + t) % n_at) * TILE;
      const fast::Operand As{reinterpret_cast<const char*>(p.A), ld, a0, p.a_rows, 0};
      const fast::Operand Bs{reinterpret_cast<const char*>(p.BT) + (int64_t)b0 * 2, (int64_t)p.b_rows * 2, 0, p.k_elems,
                             TILE * 2};
      la.init(As, p.k_elems);
      lb.init(Bs, p.k_elems);
      for (int kt = 0; kt < KT; ++kt) {
        char* st = lds + (kt & (fast::NS - 1)) * fast::STAGE;
        fast::Frags junk;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
#pragma unroll
          for (int s16 = 0; s16 < 16; ++s16) {
            const int mi = s16 >> 2, mj = s16 & 3;
            acc[mi][mj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[mi], fb[mj], acc[mi][mj], 0, 0, 0);
            // the forward layout's 12 fragment reads per half step, results never waited for
            if (s16 < 12) {
              if (s16 < 4) fast::read_frag<fast::KC>(junk.a, fra, st, h, s16);
              else fast::read_frag<fast::KR>(junk.b, frb, st + fast::OPER, h, s16 - 4);
            }
            if ((s16 & 3) == 2) {
              if (h == 0) la.issue(s16 >> 2, st + lds_wave, kt);
              else lb.issue(s16 >> 2, st + fast::OPER + lds_wave, kt);
            }
            __builtin_amdgcn_sched_barrier(0);
          }
        }
        asm volatile("" ::"v"(junk.a[0]), "v"(junk.a[1]), "v"(junk.a[2]), "v"(junk.a[3]), "v"(junk.b[0]), "v"(junk.b[1]),
                     "v"(junk.b[2]), "v"(junk.b[3]));
      }
    }
    fast::wait_vm_and_lds<0>();
    __builtin_amdgcn_s_barrier();
  } else {
    constexpr int LB = (MODE == PROBE_LOOP_KR || MODE == PROBE_DATA_KR || MODE == PROBE_LOOP_KR_SOFTMAX || MODE == PROBE_LOOP_KR_COLD) ? fast::KR
                       : MODE == PROBE_LOOP_PK ? fast::PK : fast::KC;
    constexpr bool MF = MODE == PROBE_LOOP_KR || MODE == PROBE_LOOP_KC || MODE == PROBE_LOOP_KR_SOFTMAX || MODE == PROBE_LOOP_KR_COLD || MODE == PROBE_LOOP_PK;
    fast::Pipe<fast::KC, LB, MF> pipe;
    const int64_t ld = (int64_t)p.k_elems * 2;
    for (int t = 0; t < p.tiles_per_wg; ++t) {
      const int a0 = (MODE == PROBE_LOOP_KR_COLD ? (blockIdx.x / n_bt * p.tiles_per_wg + t) % n_at
                                                 : (blockIdx.x / n_bt + t) % n_at) * TILE;
      const fast::Operand As{reinterpret_cast<const char*>(p.A), ld, a0, p.a_rows, 0};
      if constexpr (LB == fast::KR) {
        const fast::Operand Bs{reinterpret_cast<const char*>(p.BT) + (int64_t)b0 * 2, (int64_t)p.b_rows * 2, 0,
                               p.k_elems, TILE * 2};
        pipe.start(As, Bs, p.k_elems, lds);
      } else if constexpr (LB == fast::PK) {
        // the B tile's bytes taken as a pre-tiled image: K tile kt of the tile is the 16 KiB at kt * 16 KiB
        const fast::Operand Bs{reinterpret_cast<const char*>(p.B) + (int64_t)b0 * ld, 0, 0, 0, 0};
        pipe.start(As, Bs, p.k_elems, lds);
      } else {
        const fast::Operand Bs{reinterpret_cast<const char*>(p.B), ld, b0, p.b_rows, 0};
        pipe.start(As, Bs, p.k_elems, lds);
      }
      pipe.run(lds, acc);
      if constexpr (MODE == PROBE_LOOP_KR_SOFTMAX) {
        keep += softmax_work<fast::WM>(acc);
      } else if constexpr (MF) {
#pragma unroll
        for (int i = 0; i < fast::WM; ++i)
#pragma unroll
          for (int j = 0; j < fast::WN; ++j) {
            float v;
            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(acc[i][j][(i * 4 + j) & 15]));
            keep += v;
          }
      }
    }
  }
  if constexpr (MODE == PROBE_MFMA || MODE == PROBE_FREE_RUN) {
    // one element of every accumulator block keeps every MFMA chain alive
#pragma unroll
    for (int i = 0; i < fast::WM; ++i)
#pragma unroll
      for (int j = 0; j < fast::WN; ++j) {
        float v;
        asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(acc[i][j][0]));
        keep += v;
      }
  }
  p.sink[(int64_t)blockIdx.x * fast::THREADS + threadIdx.x] = keep;
}

}  // namespace flce
