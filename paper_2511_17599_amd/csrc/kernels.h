// Device kernels of the fused projection + cross-entropy path.
//
//   forward : fwd_tiles_kernel  (logit tiles on MFMA, online max / sum-exp and target
//             gather per lane: Alg. 1 in tile form; one workgroup per row block x
//             vocabulary window: Section 3.2.1)
//             merge_rows_kernel + finalize_loss_kernel (the merging epilogue of
//             Section 3.2.1, lse = m + ln a, per-row loss, fixed-order sums)
//   backward: compact_targets_kernel + prep_rows_kernel (n_valid, range flag, and the
//             rows that count packed together: ignored rows have a zero row of G; a second
//             copy of them transposed (generic loop) or pre-tiled (tuned loop))
//             pack_rows_kernel (the forward's pre-tiled copy of H for the tuned loop);
//             transpose_pad_kernel (generic loop: the K-contiguous copy of W that the dH
//             contraction needs)
//             recompute_kernel (Alg. 2: z recomputed, g = p - onehot, staged once in a
//             fixed-size buffer; the generic loop also stages the transpose)
//             contract_kernel (Eq. 4 and Eq. 5 as output-stationary MFMA
//             contractions with a fixed chunk order; Gamma applied at the flush)
//             splitk_reduce_kernel (fixed-order sum of K slices when a contraction
//             launch would otherwise leave most CUs idle)
//   Alg. 3/4: the forward and the backward above with Gamma = 1, then scale_kernel
//   per row : merge_rows_kernel writes one loss per row (label smoothing: colsum_* and
//             mean_logit_kernel give mean_v Z_iv), recompute_kernel<.., PER_ROW> scales each
//             row of G by that row's upstream gradient
//   slices  : the same kernels on rows [v_begin, v_begin + V) of the vocabulary
//             (classify_target_in_slice); merge_rows_partial_kernel hands out (m, a, z_target)
#pragma once
#include <type_traits>

#include "mainloop_fast.h"
#include "tile_mma.h"

namespace flce {

// Byte offset of row block rb in a pre-tiled copy of a matrix with d columns: the block's d / 32 images of 16 KiB
// plus a skew, so that the blocks do not start a power of two apart (the workgroups resident at one time stream
// several dozen blocks side by side, and blocks exactly 2^k bytes apart land on the same DRAM banks).
#ifndef FLCE_PACK_SKEW
#define FLCE_PACK_SKEW 17408
#endif
__host__ __device__ __forceinline__ int64_t packed_block_offset(int rb, int d) {
  return (int64_t)rb * ((int64_t)d * (TILE * 2) + FLCE_PACK_SKEW);
}
// The same for the transposed pre-tiled copy of a matrix with `rows` rows (a multiple of 256): byte offset of the
// block of column tile q (256 columns), which holds rows / 32 images.
__host__ __device__ __forceinline__ int64_t packed_cols_offset(int q, int rows) {
  return (int64_t)q * ((int64_t)rows * (TILE * 2) + FLCE_PACK_SKEW);
}

// Main-loop policies.  A kernel is written once against this interface:
//   THREADS, WM x WN (32x32 accumulator blocks per wavefront), LDS (dynamic LDS bytes),
//   tile_m(i, r) / tile_n(j): position of acc[i][j][r] inside the 256 x 256 tile,
//   slot(): which of the 4 lanes that share an N column this lane is,
//   run(): acc = A_tile . B_tile^T, ending with a barrier after the last LDS read.
template <typename T>
struct GenericLoop {      // any dtype, any K that is a multiple of 16 bytes; 8 wavefronts 2 x 4
  static constexpr int THREADS = flce::THREADS, WM = flce::WM, WN = flce::WN, LDS = LDS_BYTES;
  static constexpr bool TRANSPOSING = false;  // needs K-contiguous copies of every operand
  static __device__ __forceinline__ int tile_m(int i, int r) { return flce::tile_m(i, r); }
  static __device__ __forceinline__ int tile_n(int j) { return flce::tile_n(j); }
  static __device__ __forceinline__ int slot() {
    return ((threadIdx.x >> 6) >> 2) * 2 + ((threadIdx.x & 63) >> 5);
  }
  // element r of an accumulator block, for the code that post-processes a finished tile
  static __device__ __forceinline__ float acc_get(const f32x16& blk, int r) { return blk[r]; }
  // A sequence of tiles A[a_row0 ..][:] x B[b_row0 ..][:] over K = k_elems; start() names the next tile, run() computes
  // it.  This loop has nothing to request ahead: start() only records the operands.
  template <bool BT>
  struct Stream {
    TileSrc As, Bs;
    int k_bytes;
    __device__ __forceinline__ void start(const T* A, int64_t lda_bytes, int a_row0, int a_rows, const T* B, const T*,
                                          int64_t ldb_bytes, int b_row0, int b_rows, int k_elems, char*) {
      As = TileSrc{reinterpret_cast<const char*>(A), lda_bytes, a_row0, a_rows};
      Bs = TileSrc{reinterpret_cast<const char*>(B), ldb_bytes, b_row0, b_rows};
      k_bytes = k_elems * (int)sizeof(T);
    }
    __device__ __forceinline__ void run(char* lds, f32x16 (&acc)[WM][WN]) { tile_mainloop<T>(As, Bs, k_bytes, lds, acc); }
  };
  static __device__ __forceinline__ void run(const void* A, int64_t lda_bytes, int a_row0, int a_rows, const void* B,
                                             int64_t ldb_bytes, int b_row0, int b_rows, int k_bytes, char* lds,
                                             f32x16 (&acc)[WM][WN]) {
    const TileSrc As{static_cast<const char*>(A), lda_bytes, a_row0, a_rows};
    const TileSrc Bs{static_cast<const char*>(B), ldb_bytes, b_row0, b_rows};
    tile_mainloop<T>(As, Bs, k_bytes, lds, acc);
  }
};

struct FastLoop {         // bf16, K a multiple of 32 elements; 4 wavefronts 2 x 2, global -> LDS DMA
  static constexpr int THREADS = fast::THREADS, WM = fast::WM, WN = fast::WN, LDS = fast::LDS_BYTES;
  static constexpr bool TRANSPOSING = true;   // can take an operand whose K index runs over memory rows
  // LDS that post-processing may use while the next tile's first three K stages are being filled: the fourth stage
  static constexpr int FREE_LDS_OFFSET = (fast::NS - 1) * fast::STAGE, FREE_LDS_BYTES = fast::STAGE;
  static __device__ __forceinline__ int tile_m(int i, int r) { return fast::tile_m(i, r); }
  static __device__ __forceinline__ int tile_n(int j) { return fast::tile_n(j); }
  static __device__ __forceinline__ int slot() { return fast::slot_of_lane(); }
  // The 256 accumulators of a wavefront live in the accumulation registers.  Post-processing reads them one
  // block at a time where it uses them; left to itself the compiler copies most of a tile into vector
  // registers in one sweep at the end of the main loop, which overflows the register file into scratch memory.
  // A sequence of tiles with the same B operand: start() requests the first K stages of a tile (all LDS stages must
  // be free: every wavefront is past the previous run()), run() computes it.  BP: B is also given pre-tiled (Bp:
  // per 256-row block and K step the 16 KiB image of its LDS tile, see pack_rows_kernel), and that copy is read.
  template <bool BP>
  struct Stream {
    fast::Pipe<fast::KC, BP ? fast::PK : fast::KC> pipe;
    __device__ __forceinline__ void start(const bf16_t* A, int64_t lda_bytes, int a_row0, int a_rows, const bf16_t* B,
                                          const bf16_t* Bp, int64_t ldb_bytes, int b_row0, int b_rows, int k_elems,
                                          char* lds) {
      const fast::Operand As{reinterpret_cast<const char*>(A), lda_bytes, a_row0, a_rows, 0};
      if constexpr (BP) {
        // b_row0 is a multiple of 256: the block's images follow each other, one per K step
        const fast::Operand Bs{reinterpret_cast<const char*>(Bp) + packed_block_offset(b_row0 / TILE, k_elems), 0, 0, 0, 0};
        pipe.start(As, Bs, k_elems, lds);
      } else {
        const fast::Operand Bs{reinterpret_cast<const char*>(B), ldb_bytes, b_row0, b_rows, 0};
        pipe.start(As, Bs, k_elems, lds);
      }
    }
    __device__ __forceinline__ void run(char* lds, f32x16 (&acc)[WM][WN]) { pipe.run(lds, acc); }
  };
  static __device__ __forceinline__ float acc_get(const f32x16& blk, int r) {   // r: a constant after unrolling
    float v;
    asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(blk[r]));
    return v;
  }
  static __device__ __forceinline__ void run(const void* A, int64_t lda_bytes, int a_row0, int a_rows, const void* B,
                                             int64_t ldb_bytes, int b_row0, int b_rows, int k_bytes, char* lds,
                                             f32x16 (&acc)[WM][WN]) {
    const fast::Operand As{static_cast<const char*>(A), lda_bytes, a_row0, a_rows, 0};
    const fast::Operand Bs{static_cast<const char*>(B), ldb_bytes, b_row0, b_rows, 0};
    fast::mainloop<fast::KC, fast::KC>(As, Bs, k_bytes / 2, lds, acc);
  }
};

#ifndef FLCE_FWD_GROUP
#define FLCE_FWD_GROUP 8     // row blocks per raster patch of the forward (x 32 / this many windows per XCD)
#endif
constexpr float LOG2E = 1.4426950408889634f;
constexpr float NEG_INF = -__builtin_inff();

// First 256 bytes of every workspace.
struct Header {
  int32_t status;      // 0 or FLCE_ERR_TARGET_RANGE
  int32_t pad0;
  int64_t n_valid;     // number of counted rows
  float loss_sum;      // un-normalised sum of per-row losses (forward only)
  float pad1;
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Four consecutive elements of the storage type <-> four floats.
template <typename T> struct Pack4;
template <> struct Pack4<float> {
  static __device__ __forceinline__ void store(float* p, float a, float b, float c, float d) {
    *reinterpret_cast<f32x4*>(p) = f32x4{a, b, c, d};
  }
  static __device__ __forceinline__ void load(const float* p, float (&v)[4]) {
    const f32x4 x = *reinterpret_cast<const f32x4*>(p);
    v[0] = x[0]; v[1] = x[1]; v[2] = x[2]; v[3] = x[3];
  }
  static __device__ __forceinline__ float one(float v) { return v; }
};
template <> struct Pack4<bf16_t> {
  static __device__ __forceinline__ void store(bf16_t* p, float a, float b, float c, float d) {
    uint2 v;
    v.x = f32x2_to_bf16x2_bits(a, b);
    v.y = f32x2_to_bf16x2_bits(c, d);
    *reinterpret_cast<uint2*>(p) = v;
  }
  static __device__ __forceinline__ void load(const bf16_t* p, float (&v)[4]) {
    const uint2 x = *reinterpret_cast<const uint2*>(p);
    v[0] = __uint_as_float(x.x << 16); v[1] = __uint_as_float(x.x & 0xFFFF0000u);
    v[2] = __uint_as_float(x.y << 16); v[3] = __uint_as_float(x.y & 0xFFFF0000u);
  }
  static __device__ __forceinline__ bf16_t one(float v) { return bf16_t{f32_to_bf16_bits(v)}; }
};


// Whether a row counts towards the loss: its target is not the ignore index and lies in
// [0, V_total); a target outside that range that is not the ignore index is reported through `oor`.
__device__ __forceinline__ bool target_counts(int64_t y, int64_t ignore_index, int64_t V_total, bool& oor) {
  oor = false;
  if (y == ignore_index) return false;
  if (y < 0 || y >= V_total) { oor = true; return false; }
  return true;
}

// A counted target as a column of the vocabulary slice [v_begin, v_begin + Vs) that a call works
// on: its column inside the slice, or `outside` when it lies in another slice; -1 for rows that do
// not count.  The whole vocabulary as the slice is v_begin = 0, Vs = V_total.
__device__ __forceinline__ int classify_target_in_slice(int64_t y, int64_t ignore_index, int64_t V_total,
                                                        int64_t v_begin, int Vs, int outside, bool& oor) {
  if (!target_counts(y, ignore_index, V_total, oor)) return -1;
  const int64_t c = y - v_begin;
  return (c >= 0 && c < (int64_t)Vs) ? (int)c : outside;
}

// Merge of safe-softmax partials (m_k, a_k) in slot order; slots with a == 0 are
// the identity.  Returns (M, A) with A relative to M.
template <int S>
__device__ __forceinline__ void merge_fixed(const float (&m)[S], const float (&a)[S], float& M, float& A) {
  M = NEG_INF;
#pragma unroll
  for (int s = 0; s < S; ++s) if (a[s] > 0.f) M = fmaxf(M, m[s]);
  A = 0.f;
#pragma unroll
  for (int s = 0; s < S; ++s) if (a[s] > 0.f) A += a[s] * fast_exp2((m[s] - M) * LOG2E);
}

// ------------------------------------------------------------------------------------
// Forward tiles.  A = W tile (M = vocabulary, inside a lane), B = H tile (N = tokens,
// across lanes): each lane streams the logits of its own token columns and keeps
// (m, a, z_target) in registers across the vocabulary tiles of its window.
// part = [3][n_win][n_rb * 256] floats: m, a, z_target per (window, row).
// ------------------------------------------------------------------------------------
// HKR: the hidden states are also given pre-tiled (HT: pack_rows_kernel's copy, zero padded to whole row
// blocks), and the main loop reads that copy: every global -> LDS request is then 1 KiB of consecutive
// bytes, where the rows of H themselves give it 64 bytes at a time.
template <typename T, typename L, bool HKR>
__global__ __launch_bounds__(L::THREADS) void fwd_tiles_kernel(
    const T* __restrict__ H, const T* __restrict__ HT, const T* __restrict__ W, const int64_t* __restrict__ y,
    int N, int d, int V, int64_t ignore_index, int64_t V_total, int64_t v_begin, int n_rb, int n_win, int n_vt,
    float* __restrict__ part, int item_begin) {
  extern __shared__ __align__(16) char lds[];
  // One workgroup per item (row block x window); a launch covers the items item_begin .. item_begin + gridDim.x - 1
  // of the raster (the host launches at most one round of workgroups at a time: all of them start together, and the
  // workgroups of an XCD stay close enough to each other to share the operands of their raster patch in its L2).
  const int id = item_begin + xcd_contiguous_id(blockIdx.x, gridDim.x);
  int rb, win;
  grouped_raster(id, n_rb, n_win, FLCE_FWD_GROUP, rb, win);
  const int vt_begin = (int)((int64_t)win * n_vt / n_win);
  const int vt_end = (int)((int64_t)(win + 1) * n_vt / n_win);
  const int n0 = rb * TILE;
  const int64_t ld_bytes = (int64_t)d * sizeof(T);

  int tgt[L::WN];
  float m[L::WN], a[L::WN], zt[L::WN];
#pragma unroll
  for (int j = 0; j < L::WN; ++j) {
    const int n = n0 + L::tile_n(j);
    bool oor;
    // W holds the V vocabulary rows [v_begin, v_begin + V) of V_total; a target in another slice matches no column
    tgt[j] = (n < N) ? classify_target_in_slice(y[n], ignore_index, V_total, v_begin, V, -1, oor) : -1;
    m[j] = NEG_INF; a[j] = 0.f; zt[j] = 0.f;
  }

  f32x16 acc[L::WM][L::WN];
  // The tuned loop's first K stages of tile t+1 are requested before the softmax update of tile t (which touches
  // no memory), so the update hides their latency: it matters when the K loop is short (small d).
  typename L::template Stream<HKR> stream;
  if (vt_begin < vt_end) stream.start(W, ld_bytes, vt_begin * TILE, V, H, HT, ld_bytes, n0, N, d, lds);
  for (int vt = vt_begin; vt < vt_end; ++vt) {
    const int v0 = vt * TILE;
    stream.run(lds, acc);
    if (vt + 1 < vt_end) stream.start(W, ld_bytes, v0 + TILE, V, H, HT, ld_bytes, n0, N, d, lds);

    // Online update of (m, a) and the target gather, one 32 x 32 accumulator block at a time
    // (16 logits of one token per lane).  All 32 rows of a block belong to one wavefront, so
    // "entirely behind the vocabulary's end" and "straddles the end" are wave-uniform tests;
    // padded rows count as logits of -inf.
#pragma unroll
    for (int j = 0; j < L::WN; ++j) {
#pragma unroll
      for (int i = 0; i < L::WM; ++i) {
        const int blk0 = v0 + __builtin_amdgcn_readfirstlane(L::tile_m(i, 0) & ~31);   // first row of the block
        if (blk0 >= V) continue;
        float z[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) z[r] = L::acc_get(acc[i][j], r);
        // Row of register r inside its 32-row block: 8 * (r / 4) + (r % 4), a constant, plus 4 for the upper
        // half of the lanes (the 32x32 MFMA's accumulator layout); comparisons are written against the constant.
        const int half4 = L::tile_m(i, 0) & 4;
        if (blk0 + 32 > V) {
          const int live = V - blk0 - half4;                // rows of this block below the vocabulary's end, per lane half
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if ((r >> 2) * 8 + (r & 3) >= live) z[r] = NEG_INF;
        }
        float bmax = z[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) bmax = fmaxf(bmax, z[r]);
        const float mn = fmaxf(m[j], bmax);
        const float ms = (mn == NEG_INF) ? 0.f : mn;     // nothing but padding so far: keep exp arguments finite
        const float msl = -ms * LOG2E;                   // exp(z - ms) = 2^(z * log2e - ms * log2e): one fma per logit
        float sum = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) sum += fast_exp2(fmaf(z[r], LOG2E, msl));
        a[j] = a[j] * fast_exp2((m[j] - ms) * LOG2E) + sum;
        m[j] = mn;

        const int rel = tgt[j] - blk0;                    // target row inside this block, if any
        const bool mine = (unsigned)rel < 32u && tgt[j] >= 0;
        if (__ballot(mine) != 0ull) {
          const int relh = rel - half4;
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (mine && (r >> 2) * 8 + (r & 3) == relh) zt[j] = z[r];
        }
        // one block at a time in VGPRs
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }

  // Four lanes hold partial state of each token (2 M-wavefronts x 2 lane halves):
  // merge them in fixed slot order through LDS (free after the main loop's barrier).
  float* sm = reinterpret_cast<float*>(lds);
  float* sa = sm + 4 * TILE;
  float* sz = sa + 4 * TILE;
  {
    const int slot = L::slot();
#pragma unroll
    for (int j = 0; j < L::WN; ++j) {
      const int tok = L::tile_n(j);
      sm[slot * TILE + tok] = m[j];
      sa[slot * TILE + tok] = a[j];
      sz[slot * TILE + tok] = zt[j];
    }
  }
  __syncthreads();
  if (threadIdx.x < TILE) {
    const int tok = threadIdx.x;
    float pm[4], pa[4];
    float z = 0.f;
#pragma unroll
    for (int s = 0; s < 4; ++s) { pm[s] = sm[s * TILE + tok]; pa[s] = sa[s * TILE + tok]; z += sz[s * TILE + tok]; }
    float M, A;
    merge_fixed<4>(pm, pa, M, A);
    const int64_t npad = (int64_t)n_rb * TILE;
    const int64_t o = (int64_t)win * npad + n0 + tok;
    part[o] = M;
    part[(int64_t)n_win * npad + o] = A;
    part[2 * (int64_t)n_win * npad + o] = z;
  }
}

// Deterministic block sum of 256 values (fixed tree).
__device__ __forceinline__ float block_sum_256(float v, float* sh) {
  sh[threadIdx.x] = v;
  __syncthreads();
#pragma unroll
  for (int s = 128; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) sh[threadIdx.x] += sh[threadIdx.x + s];
    __syncthreads();
  }
  float r = sh[0];
  __syncthreads();
  return r;
}

// One thread per row: merge the partials (m, a, z_target) of `n_parts` windows or vocabulary
// slices in their order (part k of row n at pm[k * stride + n], likewise pa, pz).
__device__ __forceinline__ void merge_parts_of_row(const float* __restrict__ pm, const float* __restrict__ pa,
                                                   const float* __restrict__ pz, int n_parts, int64_t stride, int n,
                                                   float& M, float& A, float& z) {
  // The parts are taken eight at a time with all their loads issued before the first use (a part past the end
  // re-reads the last one and is not used): the parts of one row lie in different memory rows, and a load per loop
  // trip would make the merge wait for memory once per part.  The arithmetic and its order are those of the plain loop.
  constexpr int U = 8;
  M = NEG_INF;
  for (int w0 = 0; w0 < n_parts; w0 += U) {
    float mw[U], aw[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t o = (int64_t)min(w0 + u, n_parts - 1) * stride + n;
      mw[u] = pm[o]; aw[u] = pa[o];
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (w0 + u < n_parts && aw[u] > 0.f) M = fmaxf(M, mw[u]);
  }
  A = 0.f; z = 0.f;
  for (int w0 = 0; w0 < n_parts; w0 += U) {
    float mw[U], aw[U], zw[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t o = (int64_t)min(w0 + u, n_parts - 1) * stride + n;
      mw[u] = pm[o]; aw[u] = pa[o]; zw[u] = pz[o];
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (w0 + u < n_parts) {
        if (aw[u] > 0.f) A += aw[u] * fast_exp2((mw[u] - M) * LOG2E);
        z += zw[u];
      }
  }
}

// lse = M + ln A, loss_i = lse - z_target for counted rows (optionally label-smoothed and written out
// per row); per-block sums in a fixed tree.
__global__ __launch_bounds__(256) void merge_rows_kernel(
    const float* __restrict__ pm, const float* __restrict__ pa, const float* __restrict__ pz, int n_parts,
    int64_t stride, const int64_t* __restrict__ y, int N, int64_t V_total, int64_t ignore_index,
    float* __restrict__ lse_out, float* __restrict__ blk_loss, int* __restrict__ blk_cnt, int* __restrict__ blk_oor,
    float* __restrict__ loss_rows_out, const float* __restrict__ zbar, float eps) {
  __shared__ float sh[256];
  const int n = blockIdx.x * 256 + threadIdx.x;
  float loss = 0.f, cnt = 0.f, bad = 0.f;
  if (n < N) {
    float M, A, z;
    merge_parts_of_row(pm, pa, pz, n_parts, stride, n, M, A, z);
    const float lse = M + logf(A);
    lse_out[n] = lse;
    bool oor;
    if (target_counts(y[n], ignore_index, V_total, oor)) {
      loss = lse - z;
      // label smoothing: the target distribution keeps 1 - eps on y_i and spreads eps evenly, so
      // the row's loss mixes in eps * (lse - mean_v Z_iv)
      if (zbar) loss = (1.f - eps) * loss + eps * (lse - zbar[n]);
      cnt = 1.f;
    }
    if (oor) bad = 1.f;
    if (loss_rows_out) loss_rows_out[n] = loss;
  }
  const float bl = block_sum_256(loss, sh);
  const float bc = block_sum_256(cnt, sh);     // <= 256: exact in fp32
  const float bb = block_sum_256(bad, sh);
  if (threadIdx.x == 0) {
    blk_loss[blockIdx.x] = bl;
    blk_cnt[blockIdx.x] = (int)bc;
    blk_oor[blockIdx.x] = bb > 0.f ? 1 : 0;
  }
}

// mean_v Z_iv = H_i . (sum_v W_v) / V, for label smoothing: the column sums of W in two fixed-order
// steps (1024-row chunks, then the chunks in order), then one dot product per row.
template <typename T>
__global__ __launch_bounds__(256) void colsum_chunks_kernel(const T* __restrict__ W, int V, int d,
                                                            float* __restrict__ wpart) {
  const int r0 = blockIdx.x * 1024, r1 = min(V, r0 + 1024);
  for (int m = threadIdx.x * 4; m < d; m += 1024) {
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int r = r0; r < r1; ++r) {
      float v[4];
      Pack4<T>::load(W + (int64_t)r * d + m, v);
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[e] += v[e];
    }
    *reinterpret_cast<f32x4*>(wpart + (int64_t)blockIdx.x * d + m) = f32x4{acc[0], acc[1], acc[2], acc[3]};
  }
}

__global__ __launch_bounds__(256) void colsum_finish_kernel(const float* __restrict__ wpart, int n_chunks, int d,
                                                            float* __restrict__ wsum) {
  const int m = blockIdx.x * 256 + threadIdx.x;
  if (m >= d) return;
  float acc = 0.f;
  for (int c = 0; c < n_chunks; ++c) acc += wpart[(int64_t)c * d + m];
  wsum[m] = acc;
}

template <typename T>
__global__ __launch_bounds__(256) void mean_logit_kernel(const T* __restrict__ H, const float* __restrict__ wsum,
                                                         int d, float inv_V, float* __restrict__ zbar) {
  __shared__ float sh[256];
  const int n = blockIdx.x;
  float acc = 0.f;
  for (int m = threadIdx.x * 4; m < d; m += 1024) {
    float v[4];
    Pack4<T>::load(H + (int64_t)n * d + m, v);
    const f32x4 w = *reinterpret_cast<const f32x4*>(wsum + m);
    acc += v[0] * w[0] + v[1] * w[1] + v[2] * w[2] + v[3] * w[3];
  }
  const float tot = block_sum_256(acc, sh);
  if (threadIdx.x == 0) zbar[n] = tot * inv_V;
}

// The window merge of a call that covers one vocabulary slice: the slice's (m, a, z_target) per row,
// to be merged with the other slices' later (Section 3.2, "Model Parallelism": tensor parallelism).
__global__ __launch_bounds__(256) void merge_rows_partial_kernel(const float* __restrict__ part, int n_win,
                                                                 int64_t npad, int N, float* __restrict__ m_out,
                                                                 float* __restrict__ a_out,
                                                                 float* __restrict__ zt_out) {
  const int n = blockIdx.x * 256 + threadIdx.x;
  if (n >= N) return;
  float M, A, z;
  merge_parts_of_row(part, part + (int64_t)n_win * npad, part + 2 * (int64_t)n_win * npad, n_win, npad, n, M, A, z);
  m_out[n] = M; a_out[n] = A; zt_out[n] = z;
}

// One block: fixed-order fp64 sum of the per-block partials, normalisation, header.
__global__ __launch_bounds__(256) void finalize_loss_kernel(
    const float* __restrict__ blk_loss, const int* __restrict__ blk_cnt, const int* __restrict__ blk_oor, int n_blk,
    int mean, Header* __restrict__ hdr, float* __restrict__ loss_out) {
  __shared__ double sl[256];
  __shared__ long long sc[256];
  __shared__ int so[256];
  double l = 0.0; long long c = 0; int o = 0;
  for (int b = threadIdx.x; b < n_blk; b += 256) { l += (double)blk_loss[b]; c += blk_cnt[b]; o |= blk_oor[b]; }
  sl[threadIdx.x] = l; sc[threadIdx.x] = c; so[threadIdx.x] = o;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) {
      sl[threadIdx.x] += sl[threadIdx.x + s];
      sc[threadIdx.x] += sc[threadIdx.x + s];
      so[threadIdx.x] |= so[threadIdx.x + s];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const double total = sl[0];
    const long long nv = sc[0];
    double loss = total;
    if (mean) loss = nv > 0 ? total / (double)nv : 0.0;
    hdr->status = so[0] ? 4 : 0;
    hdr->pad0 = 0;
    hdr->n_valid = nv;
    hdr->loss_sum = (float)total;
    hdr->pad1 = 0.f;
    *loss_out = (float)loss;
  }
}

// Backward's integer pass over the targets (exact): n_valid, the range flag, and the
// compaction map.  Rows that do not count have an all-zero row of G, so the three
// backward contractions run on the counted rows only, packed in ascending row order:
//   rowmap[c] = original row of compact row c   (c < n_valid),  -1 for c >= n_valid
//   tgt_c[c]  = its target's column in the vocabulary slice W holds (2^31 - 1, which matches no column,
//               when the target lies in another slice),           -1 for c >= n_valid
// One block; every thread owns a contiguous range of rows, an exclusive scan of the
// per-thread counts gives each range its first compact index.
__global__ __launch_bounds__(1024) void compact_targets_kernel(const int64_t* __restrict__ y, int N, int V,
                                                               int64_t V_total, int64_t v_begin,
                                                               int64_t ignore_index, int npad,
                                                               int* __restrict__ rowmap, int* __restrict__ tgt_c,
                                                               Header* __restrict__ hdr) {
  __shared__ int sc[1024];
  __shared__ int so[1024];
  const int t = threadIdx.x;
  const int per = (N + 1023) / 1024;
  const int r0 = min(N, t * per), r1 = min(N, r0 + per);
  int c = 0, o = 0;
  for (int n = r0; n < r1; ++n) {
    bool oor;
    if (classify_target_in_slice(y[n], ignore_index, V_total, v_begin, V, 0x7FFFFFFF, oor) >= 0) ++c;
    o |= oor ? 1 : 0;
  }
  sc[t] = c; so[t] = o;
  __syncthreads();
  for (int off = 1; off < 1024; off <<= 1) {          // inclusive scan (Hillis-Steele)
    const int v = (t >= off) ? sc[t - off] : 0;
    const int w = (t >= off) ? so[t - off] : 0;
    __syncthreads();
    sc[t] += v; so[t] |= w;
    __syncthreads();
  }
  const int total = sc[1023];
  int pos = sc[t] - c;                                 // exclusive prefix
  for (int n = r0; n < r1; ++n) {
    bool oor;
    const int tg = classify_target_in_slice(y[n], ignore_index, V_total, v_begin, V, 0x7FFFFFFF, oor);
    if (tg >= 0) { rowmap[pos] = n; tgt_c[pos] = tg; ++pos; }
  }
  for (int cidx = total + t; cidx < npad; cidx += 1024) { rowmap[cidx] = -1; tgt_c[cidx] = -1; }
  if (t == 0) {
    hdr->status = so[1023] ? 4 : 0;
    hdr->pad0 = 0;
    hdr->n_valid = total;
    hdr->loss_sum = 0.f;
    hdr->pad1 = 0.f;
  }
}

// The backward's row preparation, one launch, 64 compact rows x 64 hidden positions per block:
//   Hc[c][:]  = H[rowmap[c]][:], zero for the padding rows behind the last counted row;
//   HcT[:][c] = the same transposed, when a main loop reads that copy (HcT != nullptr; ld_t elements per row);
//   lse_c[c], gam_c[c] = the row's log-sum-exp and (per-row variant) upstream gradient, 0 for padding rows;
//   dH[n][:]  = exactly +0 for every token n that does not count (the contractions write the counted rows only).
// U is an unsigned integer type of the element's width (pure data movement).
template <typename U>
__global__ __launch_bounds__(256) void prep_rows_kernel(const U* __restrict__ H, int d, const int* __restrict__ rowmap,
                                                        U* __restrict__ Hc, U* __restrict__ HcT, int64_t ld_t,
                                                        const float* __restrict__ lse, float* __restrict__ lse_c,
                                                        const float* __restrict__ grad_rows, float* __restrict__ gam_c,
                                                        const int64_t* __restrict__ y, int N, int64_t V_total,
                                                        int64_t ignore_index, U* __restrict__ dH) {
  __shared__ U tile[64][65];
  __shared__ int src_row[64];
  __shared__ int dead[64];
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int rb = blockIdx.x * 64, cb = blockIdx.y * 64;
  if (threadIdx.x < 64) {
    const int r = rb + (int)threadIdx.x;               // a compact row, and also token r of the original order
    const int n = rowmap[r];
    src_row[threadIdx.x] = n;
    bool oor;
    dead[threadIdx.x] = (r < N && !target_counts(y[r], ignore_index, V_total, oor)) ? 1 : 0;
    if (blockIdx.y == 0) {
      lse_c[r] = (n >= 0) ? lse[n] : 0.f;
      if (grad_rows) gam_c[r] = (n >= 0) ? grad_rows[n] : 0.f;
    }
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < 16; ++k) {
    const int rr = ty + 4 * k, r = rb + rr, c = cb + tx;
    const int n = src_row[rr];
    U v = 0;
    if (c < d) {
      if (n >= 0) v = H[(int64_t)n * d + c];
      Hc[(int64_t)r * d + c] = v;
      if (dead[rr]) dH[(int64_t)r * d + c] = 0;
    }
    tile[rr][tx] = v;
  }
  if (HcT == nullptr) return;
  __syncthreads();
#pragma unroll
  for (int k = 0; k < 16; ++k) {
    const int c = cb + ty + 4 * k, r = rb + tx;
    if (c < d) HcT[(int64_t)c * ld_t + r] = tile[tx][ty + 4 * k];
  }
}

// The pre-tiled copy of a row-major bf16 matrix X[rows][d] (d a multiple of 32) that the tuned main loop reads as
// its B operand: for every block of 256 rows and every K step of 32 elements, the 16 KiB image of that step's LDS
// tile, images of one row block following each other in K order:
//   P[(rb * d / 32 + kt) * 16 KiB + r * 64 + 16 * pos] = the 16 bytes X[rb * 256 + r][kt * 32 + 8 * (pos ^ (r / 4) % 4) ...]
// (the main loop's K-contiguous LDS tile, 256 rows of 64 bytes with its chunk swizzle), rows past the end as zeros.
// pack_rows_store: one thread's part, the 64 bytes of row r of row block rb at K step kt.
__device__ __forceinline__ void pack_rows_store(const u32x4 (&chunk)[4], char* __restrict__ P, int rb, int kt, int d, int r) {
  u32x4* dst = reinterpret_cast<u32x4*>(P + packed_block_offset(rb, d) + (int64_t)kt * fast::OPER + r * 64);
  const int sw = (r >> 2) & 3;
#pragma unroll
  for (int c = 0; c < 4; ++c) dst[c ^ sw] = chunk[c];
}

// grid (rows_pad / 64, ceil(d / 128)), 256 threads: thread t copies the 64 bytes of row 64 * blockIdx.x + t / 4 at
// K step 4 * blockIdx.y + t % 4, so that a wavefront reads 16 rows x 256 consecutive bytes and writes 1 KiB runs.
__global__ __launch_bounds__(256) void pack_rows_kernel(const char* __restrict__ X, int rows, int d,
                                                        char* __restrict__ P) {
  const int row = blockIdx.x * 64 + (threadIdx.x >> 2), kt = blockIdx.y * 4 + (threadIdx.x & 3);
  const int KT = d / fast::BK;
  if (kt >= KT) return;
  u32x4 chunk[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) chunk[c] = u32x4{0u, 0u, 0u, 0u};
  if (row < rows) {
    const u32x4* src = reinterpret_cast<const u32x4*>(X + ((int64_t)row * d + kt * fast::BK) * 2);
#pragma unroll
    for (int c = 0; c < 4; ++c) chunk[c] = src[c];
  }
  pack_rows_store(chunk, P, row / TILE, kt, d, row % TILE);
}

// The backward's row preparation for the tuned loop, one launch; block (kt, q) handles the 32 compact rows of K step
// kt of the dW contraction and the 256 hidden columns of tile q (grid: rows_pad / 32 x ceil(d / 256), 256 threads):
//   HcP  = the counted rows of H, packed together (zero behind the last one), pre-tiled as pack_rows_kernel does: the
//          recompute's second operand (nullptr: not wanted);
//   HcTP = the same rows pre-tiled the other way round, for the dW contraction, whose K index runs over the rows: per
//          hidden tile q and K step kt the 16 KiB LDS image [256 hidden positions][32 rows] (chunk swizzle included),
//          the images of one q following each other, block q at packed_cols_offset(q, rows_pad); hidden positions
//          past d are zeros;
//   lse_c / gam_c gathered likewise; dH rows of tokens that do not count set to exactly +0.
__global__ __launch_bounds__(256) void prep_rows_tiled_kernel(const char* __restrict__ H, int d,
                                                              const int* __restrict__ rowmap, int rows_pad,
                                                              char* __restrict__ HcP, char* __restrict__ HcTP,
                                                              const float* __restrict__ lse, float* __restrict__ lse_c,
                                                              const float* __restrict__ grad_rows,
                                                              float* __restrict__ gam_c,
                                                              const int64_t* __restrict__ y, int N, int64_t V_total,
                                                              int64_t ignore_index, char* __restrict__ dH) {
  __shared__ __align__(16) uint16_t tile[32][TILE + 8];     // 528-byte rows: a column read touches every bank once
  const int kt = blockIdx.x, q = blockIdx.y;
  const int rr = threadIdx.x >> 3, g = threadIdx.x & 7;    // row of the K step, group of 32 hidden positions
  const int c = kt * 32 + rr;                               // compact row c, and also token c of the original order
  const int col0 = q * TILE + g * 32;
  const int n = rowmap[c];
  if (q == 0 && g == 0) {
    lse_c[c] = (n >= 0) ? lse[n] : 0.f;
    if (grad_rows) gam_c[c] = (n >= 0) ? grad_rows[n] : 0.f;
  }
  u32x4 chunk[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) chunk[i] = u32x4{0u, 0u, 0u, 0u};
  if (col0 < d) {                                           // d is a multiple of 32: a group is inside or outside
    if (n >= 0) {
      const u32x4* src = reinterpret_cast<const u32x4*>(H + ((int64_t)n * d + col0) * 2);
#pragma unroll
      for (int i = 0; i < 4; ++i) chunk[i] = src[i];
    }
    if (HcP) pack_rows_store(chunk, HcP, c / TILE, col0 / fast::BK, d, c % TILE);
    bool oor;
    if (c < N && !target_counts(y[c], ignore_index, V_total, oor)) {
      u32x4* z = reinterpret_cast<u32x4*>(dH + ((int64_t)c * d + col0) * 2);
#pragma unroll
      for (int i = 0; i < 4; ++i) z[i] = u32x4{0u, 0u, 0u, 0u};
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4*>(&tile[rr][g * 32 + i * 8]) = chunk[i];
  __syncthreads();
  // thread m: the 32 rows' values at hidden position q * 256 + m, as the 64 bytes of row m of the image
  const int m = threadIdx.x, sw = (m >> 2) & 3;
  u32x4* dst = reinterpret_cast<u32x4*>(HcTP + packed_cols_offset(q, rows_pad) + (int64_t)kt * fast::OPER + m * 64);
#pragma unroll
  for (int ch = 0; ch < 4; ++ch) {
    u32x4 v;
#pragma unroll
    for (int e = 0; e < 4; ++e)
      v[e] = (uint32_t)tile[ch * 8 + 2 * e][m] | ((uint32_t)tile[ch * 8 + 2 * e + 1][m] << 16);
    dst[ch ^ sw] = v;
  }
}

// dst[c][r] = src[r0 + r][c]  for c < cols, r < rows_pad; zero where r0 + r >= rows_total.
// U is an unsigned integer type of the element's width (pure data movement).
template <typename U>
__global__ __launch_bounds__(256) void transpose_pad_kernel(const U* __restrict__ src, int64_t ld_src, int rows_total,
                                                            int r0, int cols, U* __restrict__ dst, int64_t ld_dst,
                                                            int rows_pad) {
  __shared__ U tile[64][65];
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int rb = blockIdx.x * 64, cb = blockIdx.y * 64;
#pragma unroll
  for (int k = 0; k < 16; ++k) {
    const int r = rb + ty + 4 * k, c = cb + tx;
    U v = 0;
    if (r < rows_pad && r0 + r < rows_total && c < cols) v = src[(int64_t)(r0 + r) * ld_src + c];
    tile[ty + 4 * k][tx] = v;
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < 16; ++k) {
    const int c = cb + ty + 4 * k, r = rb + tx;
    if (c < cols && r < rows_pad) dst[(int64_t)c * ld_dst + r] = tile[tx][ty + 4 * k];
  }
}

// ------------------------------------------------------------------------------------
// Backward, step 1 (on the compacted rows): logit tile recomputed exactly as in the
// forward, then
//   g = exp(z - lse_row) - [v == y_row]            (unscaled; Gamma comes later)
// rounded to T and written to the staging tile
//   G [row - chunk_n0][vocab - chunk_v0]   (ldG  elements per row; with the tuned loop in blocks of 16 rows x 32
//                                           positions of 1 KiB, ldG = BYTES from one group of 16 rows to the next)
// and, for main loops that need K-contiguous operands, also transposed:
//   GT[vocab - chunk_v0][row - chunk_n0]   (ldGT elements per row)
// Padded vocabulary columns and the padding rows behind the last counted row are 0.
// Tiles that lie entirely behind the last counted row return at once; the
// contractions never read them.
// ------------------------------------------------------------------------------------
template <typename T>
struct RecomputeArgs {
  const T* Hc; const T* HcT; const T* W; const int* tgt_c; const float* lse_c; const Header* hdr;
  int npad, d, V, nt0, n_nt, vt0, n_vt;
  T* G; int64_t ldG; T* GT; int64_t ldGT;
  // per-row variant only: upstream gradient of each compact row, label-smoothing constants
  const float* gam_c; float onehot_weight; float uniform_part;   // 1 - eps, eps / V
};

// Per-row inputs of a recompute tile, one set per token column a lane owns.
template <typename L>
struct RowMeta {
  int tgt[L::WN];       // target column inside the slice, -1 for a padding row
  float lse[L::WN];
  float gam[L::WN];     // per-row variant only
};

// The recompute step.  The launch has min(tiles, 256) workgroups; workgroup b takes tiles b, b + gridDim.x, ... of
// the chunk.  With the tuned loop the first K stages of a workgroup's next tile (and that tile's per-row inputs) are
// requested before the current tile's G is formed and stored, so the latency of a tile's first operands hides behind
// the previous tile's post-processing: it matters when the K loop is short (small d).
// PER_ROW: g = Gamma_row * (p - (1 - eps) [v == y_row] - eps / V), the upstream gradient applied here because
// it differs from row to row (Alg. 2 with a per-position Gamma); otherwise g = p - [v == y_row] and the
// scalar Gamma is applied when the contractions write out.
template <typename T, typename L, bool HKR, bool PER_ROW = false>
__global__ __launch_bounds__(L::THREADS) void recompute_kernel(RecomputeArgs<T> a) {
  extern __shared__ __align__(16) char lds[];
  const T* __restrict__ Hc = a.Hc; const T* __restrict__ HcT = a.HcT; const T* __restrict__ W = a.W;
  const int npad = a.npad, d = a.d, V = a.V;
  T* __restrict__ G = a.G; T* __restrict__ GT = a.GT; const int64_t ldG = a.ldG, ldGT = a.ldGT;
  // Only the row tiles that hold counted rows are rastered (their number is known on the device
  // alone), so the XCDs share the work evenly however many rows are ignored; workgroups beyond the
  // useful tiles of a launch sized for N rows leave at once.
  const int n_nt = max(0, min(a.n_nt, ((int)a.hdr->n_valid - a.nt0 * TILE + TILE - 1) / TILE));
  const int useful = n_nt * a.n_vt;
  int t = blockIdx.x;
  if (t >= useful) return;
  const int64_t ld_bytes = (int64_t)d * sizeof(T);
  auto place = [&](int tile, int& p, int& q) {     // row tile, vocabulary tile inside the chunk
    grouped_raster(xcd_contiguous_id(tile, useful), n_nt, a.n_vt, 8, p, q);
  };
  auto load_meta = [&](int n0, RowMeta<L>& m) {
#pragma unroll
    for (int j = 0; j < L::WN; ++j) {
      const int n = n0 + L::tile_n(j);
      m.tgt[j] = a.tgt_c[n];
      m.lse[j] = a.lse_c[n];
      if constexpr (PER_ROW) m.gam[j] = a.gam_c[n];
    }
  };
  // Marks the point where a tile's per-row inputs must have arrived: the compiler's wait for them lands here (it
  // cannot see the main loop's own requests, so a wait placed later would also wait for the next tile's operands).
  auto need_meta = [&](RowMeta<L>& m) {
#pragma unroll
    for (int j = 0; j < L::WN; ++j) {
      asm volatile("" : "+v"(m.tgt[j]), "+v"(m.lse[j]));
      if constexpr (PER_ROW) asm volatile("" : "+v"(m.gam[j]));
    }
  };
  typename L::template Stream<HKR> stream;
  int p, q;
  place(t, p, q);
  RowMeta<L> meta;
  if constexpr (L::TRANSPOSING) load_meta((a.nt0 + p) * TILE, meta);
  stream.start(W, ld_bytes, (a.vt0 + q) * TILE, V, Hc, HcT, ld_bytes, (a.nt0 + p) * TILE, npad, d, lds);
  f32x16 acc[L::WM][L::WN];
  for (;;) {
    stream.run(lds, acc);
    const int t_next = t + gridDim.x;
    // (a main loop with nothing to request ahead gets one tile per workgroup)
    const bool more = L::TRANSPOSING && t_next < useful;
    int p_next = 0, q_next = 0;
    RowMeta<L> meta_next;
    if constexpr (!L::TRANSPOSING) load_meta((a.nt0 + p) * TILE, meta);   // no registers to spare across that main loop
    need_meta(meta);
    if (more) {
      place(t_next, p_next, q_next);
      load_meta((a.nt0 + p_next) * TILE, meta_next);
      stream.start(W, ld_bytes, (a.vt0 + q_next) * TILE, V, Hc, HcT, ld_bytes, (a.nt0 + p_next) * TILE, npad, d, lds);
    }

    const int v0 = (a.vt0 + q) * TILE;
    if constexpr (L::TRANSPOSING) {
      // Tuned loop.  A lane holds, of 32 token rows x 128 vocabulary positions per j, scattered 8-byte pieces of one
      // row; stored as they lie, every store instruction would touch 64 different memory rows.  Each wavefront
      // therefore passes its 32 x 128 piece (8 KiB of bf16) through its own slice of the free LDS stage and writes
      // whole 256-byte runs: 16 lanes per row, 4 rows per instruction.  LDS row = 256 bytes = 32 slots of 8 bytes,
      // slot index XOR-ed with the row number: the 32 rows that one 8-byte write instruction touches land in 32
      // different slots (all 64 banks once), and a 16-byte read finds its two slots side by side, in swapped order
      // on odd rows.
      static_assert(sizeof(T) == 2 && L::WM == 4 && L::WN == 4, "tuned epilogue is laid out for bf16 128 x 128 wave tiles");
      const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
      char* stage = lds + L::FREE_LDS_OFFSET + wave * 8192;
      const int wrow = lane & 31, whalf = lane >> 5;              // writer: token row of the piece, lane half
      const int rrow = lane >> 4, rchunk = lane & 15;             // reader: row within a group of 4, 16-byte chunk
      const int vbase = v0 + (wave >> 1) * 128;                   // first vocabulary position of the piece
#pragma unroll
      for (int j = 0; j < L::WN; ++j) {
        const int tgt = meta.tgt[j];
        // exp(z - lse) = 2^(z * log2e - lse * log2e); a padding row (tgt < 0) gets lse = +inf here, so its p is
        // exactly 0, and no column equals its target: its row of G is 0 without a mask
        const float ll = tgt >= 0 ? -meta.lse[j] * LOG2E : NEG_INF;
        float gam = 1.f;
        if constexpr (PER_ROW) gam = tgt >= 0 ? meta.gam[j] : 0.f;
        const float unif = tgt >= 0 ? a.uniform_part : 0.f;
#pragma unroll
        for (int i = 0; i < L::WM; ++i) {
          const int blk0 = vbase + i * 32;                        // wave-uniform
          const bool whole = blk0 + 32 <= V;
          // Does any token column of this wavefront have its target among the block's 32 vocabulary positions?
          // Almost never (32 of V positions), and then the one-hot term costs nothing: a wave-uniform branch.
          const bool hit = __ballot((unsigned)(tgt - blk0) < 32u) != 0ull;
#pragma unroll
          for (int rq = 0; rq < 4; ++rq) {
            const int vpos = blk0 + rq * 8 + whalf * 4;           // first of this lane's 4 consecutive positions
            float g[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) g[e] = fast_exp2(fmaf(L::acc_get(acc[i][j], rq * 4 + e), LOG2E, ll));
            if (hit) {
#pragma unroll
              for (int e = 0; e < 4; ++e)
                if (vpos + e == tgt) g[e] -= PER_ROW ? a.onehot_weight : 1.f;
            }
            if constexpr (PER_ROW) {
#pragma unroll
              for (int e = 0; e < 4; ++e) g[e] = gam * (g[e] - unif);
            }
            if (!whole) {
#pragma unroll
              for (int e = 0; e < 4; ++e)
                if (vpos + e >= V) g[e] = 0.f;
            }
            uint2 packed;
            packed.x = f32x2_to_bf16x2_bits(g[0], g[1]);
            packed.y = f32x2_to_bf16x2_bits(g[2], g[3]);
            const int slot = ((i * 4 + rq) * 2 + whalf) ^ wrow;
            *reinterpret_cast<uint2*>(stage + wrow * 256 + slot * 8) = packed;
          }
          __builtin_amdgcn_sched_barrier(0);   // one 32x32 block at a time in VGPRs
        }
        // the piece is complete in LDS (a wavefront's LDS operations complete in order): write it out, four rows of
        // 256 bytes per instruction.  G is stored in blocks of 16 rows x 32 positions (1 KiB; the blocks of a row
        // group along the vocabulary, row groups ldG BYTES apart), so that both contractions fetch whole blocks:
        // a row's 16 bytes at position chunk c lie in block c / 4 at (row % 16) * 64 + (c % 4) * 16.
        const int row0 = p * TILE + (wave & 1) * 128 + j * 32;                  // a multiple of 32: two row groups
        const int cchunk = q * 32 + (wave >> 1) * 16 + rchunk;                  // 8-position chunk inside the chunk's row
        char* __restrict__ gdst = reinterpret_cast<char*>(G) + (int64_t)(row0 >> 4) * ldG + (int64_t)(cchunk >> 2) * 1024 +
                                  rrow * 64 + (cchunk & 3) * 16;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const int r = k * 4 + rrow;
          u32x4 vq = *reinterpret_cast<const u32x4*>(stage + r * 256 + ((rchunk ^ (r >> 1)) * 16));
          if (rrow & 1) vq = u32x4{vq[2], vq[3], vq[0], vq[1]};      // r is odd exactly when rrow is
          *reinterpret_cast<u32x4*>(gdst + (int64_t)(k >> 2) * ldG + (k & 3) * 256) = vq;
        }
      }
    } else {
    // Blocks in (i, j) order, i outermost: what depends on the vocabulary position only (the padding masks of a
    // block that straddles the vocabulary's end) is then shared by the four j of one i and dies with it.
#pragma unroll
    for (int i = 0; i < L::WM; ++i) {
      // All 32 vocabulary positions of a block belong to one wavefront: "behind the vocabulary's end" and
      // "straddles the end" are wave-uniform tests, and only a straddling block masks single elements.
      const int blk0 = v0 + __builtin_amdgcn_readfirstlane(L::tile_m(i, 0) & ~31);
      const bool whole = blk0 + 32 <= V;
#pragma unroll
      for (int j = 0; j < L::WN; ++j) {
        const int nl = p * TILE + L::tile_n(j);       // row inside the staging tile
        // this lane's first position in the row; block (i, rq) lies a constant 32 i + 8 rq further on
        T* __restrict__ grow = G + (int64_t)nl * ldG + q * TILE + L::tile_m(0, 0);
        const int tgt = meta.tgt[j];
        // exp(z - lse) = 2^(z * log2e - lse * log2e); a padding row (tgt < 0) gets lse = +inf here, so its p is
        // exactly 0, and no column equals its target: its row of G is 0 without a mask
        const float ll = tgt >= 0 ? -meta.lse[j] * LOG2E : NEG_INF;
        float gam = 1.f;
        if constexpr (PER_ROW) gam = tgt >= 0 ? meta.gam[j] : 0.f;
        const float unif = tgt >= 0 ? a.uniform_part : 0.f;
        // Does any token column of this wavefront have its target among the block's 32 vocabulary positions?
        // Almost never (32 of V positions), and then the one-hot term costs nothing: a wave-uniform branch.
        const bool hit = __ballot((unsigned)(tgt - blk0) < 32u) != 0ull;
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
          const int mloc = L::tile_m(i, rq * 4);    // first of 4 consecutive vocabulary positions
          float g[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) g[e] = fast_exp2(fmaf(L::acc_get(acc[i][j], rq * 4 + e), LOG2E, ll));
          if (hit) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (v0 + mloc + e == tgt) g[e] -= PER_ROW ? a.onehot_weight : 1.f;
          }
          if constexpr (PER_ROW) {
#pragma unroll
            for (int e = 0; e < 4; ++e) g[e] = gam * (g[e] - unif);
          }
          if (!whole) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (v0 + mloc + e >= V) g[e] = 0.f;
          }
          const int vl = q * TILE + mloc;
          Pack4<T>::store(grow + (i * 32 + rq * 8), g[0], g[1], g[2], g[3]);
          if (!L::TRANSPOSING) {
#pragma unroll
            for (int e = 0; e < 4; ++e) GT[(int64_t)(vl + e) * ldGT + nl] = Pack4<T>::one(g[e]);
          }
        }
        __builtin_amdgcn_sched_barrier(0);   // one 32x32 block at a time in VGPRs
      }
    }
    }
    if (!more) break;
    need_meta(meta_next);
    t = t_next; p = p_next; q = q_next;
    meta = meta_next;
  }
}

// ------------------------------------------------------------------------------------
// Backward, step 2: out[n][m] (+)= sum_k A[m][k] * B[n][k]
//   dH: A = W^T chunk [d][Vc], B = G  [rows][Vc]   (contraction over the vocabulary chunk)
//   dW: A = Hc^T      [d][Nc], B = GT [vocab][Nc]  (contraction over the compact-row chunk)
// M = hidden index, so each lane owns 4 consecutive output elements of one row.
// Chunks are accumulated in fp32 in a fixed order: READ_ACC adds the running sum,
// WRITE_ACC stores it back, WRITE_OUT multiplies by Gamma and rounds to T.
// ROWS_COMPACT (dH): output rows are compact rows; tiles behind the last counted row
// return at once and row c is written to out[rowmap[c]].
// K_COMPACT (dW): the contraction runs over compact rows k_start .. k_start + k_elems and
// stops at the last counted row (rounded up to a whole tile; that padding is zero).
// ------------------------------------------------------------------------------------
//
// OPS selects how the operands lie in memory:
//   OPS_KC    : A[m][k], B[n][k] both K-contiguous (the transposed copies W^T, Hc^T, GT)
//   OPS_DH_TR : A = W rows of the vocabulary chunk [k][m] (K over memory rows), B = G of the chunk, stored in blocks
//               of 16 rows x 32 positions (recompute_kernel; ldb = BYTES from one group of 16 rows to the next)
//   OPS_DW_TR : A = the transposed pre-tiled copy of Hc (prep_rows_tiled_kernel; lda = its padded row count, the
//               K steps of the row chunk start at image k_start / 32), B = the same blocked G, K over its rows
enum : int { READ_ACC = 1, WRITE_ACC = 2, WRITE_OUT = 4, ROWS_COMPACT = 8, K_COMPACT = 16 };
enum : int { OPS_KC = 0, OPS_DH_TR = 1, OPS_DW_TR = 2 };

template <typename T>
struct ContractArgs {
  const T* A; int64_t lda; int a_krows, d;
  const T* B; int64_t ldb; int b_rows, k_elems, k_start, n_mt, n_nt;
  float* accbuf; int acc_row0;
  T* out; int out_row0, out_rows, flags;
  const Header* hdr; const int* rowmap; float grad_loss; int mean;
  // split-K (n_split > 1): the launch has n_split x tiles workgroups; slice z contracts K elements
  // [z * k_split, (z + 1) * k_split) and stores its fp32 tile into partial + z * partial_stride (indexed like
  // accbuf); splitk_reduce_kernel then adds the slices in slice order and does the READ/WRITE part of `flags`.
  int n_split, k_split; float* partial; int64_t partial_stride;
};

// With the tuned loop a launch has at most 256 workgroups; workgroup b takes work items b, b + gridDim.x, ... (an
// item = one output tile of one K slice) and requests the first K stages of its next item before it writes out the
// current one, as the recompute step does.
template <typename T, typename L, int OPS>
__global__ __launch_bounds__(L::THREADS) void contract_kernel(ContractArgs<T> a) {
  extern __shared__ __align__(16) char lds[];
  const T* __restrict__ A = a.A; const T* __restrict__ B = a.B;
  const int64_t lda = a.lda, ldb = a.ldb;
  const int d = a.d;
  T* __restrict__ out = a.out;
  const int nv = (int)a.hdr->n_valid;
  // With compacted output rows only the row tiles that hold counted rows are rastered, so the
  // XCDs share the work evenly; surplus workgroups of the launch leave at once.
  int n_nt = a.n_nt;
  if (a.flags & ROWS_COMPACT) n_nt = max(0, min(n_nt, (nv - a.out_row0 + TILE - 1) / TILE));
  const int tiles = n_nt * a.n_mt;
  const int n_split = max(1, a.n_split);
  const int total = tiles * n_split;
  int b = blockIdx.x;
  if (b >= total) return;
  int k_all = a.k_elems;
  if (a.flags & K_COMPACT) k_all = max(0, min(k_all, (nv - a.k_start + TILE - 1) / TILE * TILE));
  float scale = a.grad_loss;
  if (a.mean) scale = nv > 0 ? a.grad_loss / (float)nv : 0.f;

  // item -> K slice z, output-row tile p, hidden tile q; K range [k0, k0 + k_elems) of the slice
  auto place = [&](int item, int& z, int& p, int& q, int& k0, int& k_elems) {
    z = item / tiles;
    grouped_raster(xcd_contiguous_id(item - z * tiles, tiles), n_nt, a.n_mt, 8, p, q);
    k0 = 0; k_elems = k_all;
    if (a.n_split > 1) { k0 = z * a.k_split; k_elems = max(0, min(a.k_split, k_all - k0)); }
  };
  // output rows of the lane's token columns: the original row of a compact row, -1 = nothing to write
  auto load_rows = [&](int p, int64_t (&orow)[L::WN]) {
#pragma unroll
    for (int j = 0; j < L::WN; ++j) {
      const int n = a.out_row0 + p * TILE + L::tile_n(j);
      orow[j] = -1;
      if (n < a.out_rows) orow[j] = (a.flags & ROWS_COMPACT) ? (int64_t)a.rowmap[n] : (int64_t)n;
    }
  };
  auto need_rows = [&](int64_t (&orow)[L::WN]) {     // the compiler's wait for the loads above lands here
#pragma unroll
    for (int j = 0; j < L::WN; ++j) asm volatile("" : "+v"(orow[j]));
  };
  // Running sum / Gamma / rounding of one finished tile.
  auto flush = [&](f32x16 (&acc)[L::WM][L::WN], int z, int p, int q, const int64_t (&orow)[L::WN]) {
    int flags = a.flags;
    float* __restrict__ accbuf = a.accbuf;
    if (a.n_split > 1) {
      accbuf = a.partial + (int64_t)z * a.partial_stride;
      flags = (flags & ROWS_COMPACT) | WRITE_ACC;
    }
#pragma unroll
    for (int j = 0; j < L::WN; ++j) {
      if (orow[j] < 0) continue;
      const int n = a.out_row0 + p * TILE + L::tile_n(j);
      // this lane's first hidden position; block (i, rq) lies a constant 32 i + 8 rq further on
      const int m0 = q * TILE + L::tile_m(0, 0);
      float* __restrict__ arow = accbuf + (int64_t)(n - a.acc_row0) * d + m0;
      T* __restrict__ orowp = out + orow[j] * d + m0;
#pragma unroll
      for (int i = 0; i < L::WM; ++i)
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
          const int c = i * 32 + rq * 8;
          if (m0 + c >= d) continue;
          f32x4 v = {L::acc_get(acc[i][j], rq * 4), L::acc_get(acc[i][j], rq * 4 + 1), L::acc_get(acc[i][j], rq * 4 + 2),
                     L::acc_get(acc[i][j], rq * 4 + 3)};
          float* ap = arow + c;
          if (flags & READ_ACC) v += *reinterpret_cast<const f32x4*>(ap);
          if (flags & WRITE_ACC) *reinterpret_cast<f32x4*>(ap) = v;
          if (flags & WRITE_OUT) {
            // "+ 0.f" turns a -0 product into +0
            Pack4<T>::store(orowp + c, v[0] * scale + 0.f, v[1] * scale + 0.f, v[2] * scale + 0.f,
                            v[3] * scale + 0.f);
          }
          if (rq == 3) __builtin_amdgcn_sched_barrier(0);   // one 32x32 block at a time in VGPRs
        }
    }
  };

  f32x16 acc[L::WM][L::WN];
  int z, p, q, k0, k_elems;
  place(b, z, p, q, k0, k_elems);
  int64_t orow[L::WN];
  if constexpr (OPS == OPS_KC) {
    // one item per workgroup: this main loop has nothing to request ahead
    L::run(A + k0, lda * (int64_t)sizeof(T), q * TILE, d, B + k0, ldb * (int64_t)sizeof(T), p * TILE, a.b_rows,
           k_elems * (int)sizeof(T), lds, acc);
    load_rows(p, orow);
    flush(acc, z, p, q, orow);
  } else {
    fast::Pipe<OPS == OPS_DH_TR ? fast::KR : fast::PK, OPS == OPS_DH_TR ? fast::KB : fast::RB> pipe;
    auto start = [&](int p, int q, int k0, int k_elems) {
      if constexpr (OPS == OPS_DH_TR) {
        // A: K rows start at A (a_krows valid from there), window of 256 hidden columns at q
        const int width = max(0, min(TILE, d - q * TILE)) * 2;
        const fast::Operand As{reinterpret_cast<const char*>(A + (int64_t)k0 * lda) + (int64_t)q * TILE * 2, lda * 2, 0,
                               a.a_krows - k0, width};
        // B: G blocked (ldb = bytes from one group of 16 rows to the next), rows p * 256 ..., K from position k0
        const fast::Operand Bs{reinterpret_cast<const char*>(B) + (int64_t)(p * (TILE / 16)) * ldb + (int64_t)(k0 / 32) * 1024,
                               ldb, 0, 0, 0};
        pipe.start(As, Bs, k_elems, lds);
      } else {
        // A: the images of hidden tile q, from K step (k_start + k0) / 32 on
        const fast::Operand As{reinterpret_cast<const char*>(A) + packed_cols_offset(q, (int)lda) +
                                   (int64_t)((a.k_start + k0) / fast::BK) * fast::OPER, 0, 0, 0, 0};
        // B: G blocked, K over its rows from row k0, the tile's 256 vocabulary positions from p * 256
        const fast::Operand Bs{reinterpret_cast<const char*>(B) + (int64_t)(k0 / 16) * ldb + (int64_t)(p * (TILE / 32)) * 1024,
                               ldb, 0, 0, 0};
        pipe.start(As, Bs, k_elems, lds);
      }
    };
    load_rows(p, orow);
    start(p, q, k0, k_elems);
    for (;;) {
      pipe.run(lds, acc);
      const int b_next = b + gridDim.x;
      const bool more = b_next < total;
      int z_next = 0, p_next = 0, q_next = 0, k0_next = 0, k_next = 0;
      int64_t orow_next[L::WN];
      need_rows(orow);
      if (more) {
        place(b_next, z_next, p_next, q_next, k0_next, k_next);
        load_rows(p_next, orow_next);
        start(p_next, q_next, k0_next, k_next);
      }
      flush(acc, z, p, q, orow);
      if (!more) break;
      need_rows(orow_next);
      b = b_next; z = z_next; p = p_next; q = q_next;
#pragma unroll
      for (int j = 0; j < L::WN; ++j) orow[j] = orow_next[j];
    }
  }
}

// Second half of a split-K contraction: one block per output row of the launch; adds the K
// slices in slice order (fixed), then the running sum / Gamma / rounding exactly as the
// unsplit epilogue would.
template <typename T>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(ContractArgs<T> a) {
  const int n = a.out_row0 + blockIdx.x;
  if (n >= a.out_rows) return;
  const int nv = (int)a.hdr->n_valid;
  int64_t orow = n;
  if (a.flags & ROWS_COMPACT) {
    if (n >= nv) return;
    orow = a.rowmap[n];
    if (orow < 0) return;
  }
  float scale = a.grad_loss;
  if (a.mean) scale = nv > 0 ? a.grad_loss / (float)nv : 0.f;
  const int d = a.d;
  for (int m = threadIdx.x * 4; m < d; m += 256 * 4) {
    const int64_t off = (int64_t)(n - a.acc_row0) * d + m;
    f32x4 v = *reinterpret_cast<const f32x4*>(a.partial + off);
    for (int z = 1; z < a.n_split; ++z) v += *reinterpret_cast<const f32x4*>(a.partial + z * a.partial_stride + off);
    float* ap = a.accbuf + off;
    if (a.flags & READ_ACC) v += *reinterpret_cast<const f32x4*>(ap);
    if (a.flags & WRITE_ACC) *reinterpret_cast<f32x4*>(ap) = v;
    if (a.flags & WRITE_OUT)
      Pack4<T>::store(a.out + orow * d + m, v[0] * scale + 0.f, v[1] * scale + 0.f, v[2] * scale + 0.f,
                      v[3] * scale + 0.f);
  }
}

// Alg. 4, scalar branch: out = Gamma * in, elementwise, Gamma from the header's n_valid.
template <typename T>
__global__ __launch_bounds__(256) void scale_kernel(const T* __restrict__ in, T* __restrict__ out, int64_t n4,
                                                    const Header* __restrict__ hdr, float grad_loss, int mean) {
  const int nv = (int)hdr->n_valid;
  float scale = grad_loss;
  if (mean) scale = nv > 0 ? grad_loss / (float)nv : 0.f;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (int64_t)gridDim.x * 256) {
    float v[4];
    Pack4<T>::load(in + i * 4, v);
    Pack4<T>::store(out + i * 4, v[0] * scale + 0.f, v[1] * scale + 0.f, v[2] * scale + 0.f, v[3] * scale + 0.f);
  }
}

}  // namespace flce
