// 256 x 256 output tile of an "NT" contraction  D[m][n] = sum_k A[m][k] * B[n][k]
// on the gfx950 matrix cores, both operands K-contiguous in memory.
//
// One workgroup = 512 threads = 8 wavefronts arranged 2 (M) x 4 (N); each
// wavefront owns a 128 x 64 sub-tile = 4 x 2 blocks of one 32 x 32 MFMA.
// Accumulator layout of a 32 x 32 block (fp32, 16 registers per lane):
//     n = lane % 32,   m = 8 * (r / 4) + 4 * (lane / 32) + (r % 4),   r = 0..15
// so the M index runs inside a lane (4 consecutive values per register quad)
// and the N index runs across lanes.  Every kernel of the path picks which
// tensor plays A so that the dimension it reduces over, or stores
// contiguously, is M.
//
// Operand tiles are staged through LDS as [256 rows][128 bytes of K] with the
// 16-byte chunk index XOR-ed with (row % 8), which makes the 128-bit fragment
// reads conflict-free; two stages are kept so one barrier per K step is enough.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace flce {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int TILE = 256;            // BM = BN
constexpr int KB = 128;              // bytes of K per stage and row
constexpr int THREADS = 512;
constexpr int WM = 4, WN = 2;        // 32x32 blocks per wavefront along M, N
constexpr int STAGE_BYTES = 2 * TILE * KB;       // A tile + B tile
constexpr int LDS_BYTES = 2 * STAGE_BYTES;       // double buffered: 128 KiB

struct bf16_t { uint16_t bits; };

// fp32 -> bf16, round to nearest even: gfx950 converts in hardware (v_cvt_pk_bf16_f32), two values per
// instruction.
typedef __bf16 hw_bf16x2 __attribute__((ext_vector_type(2)));
typedef float hw_f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t f32x2_to_bf16x2_bits(float lo, float hi) {
  const hw_bf16x2 b = __builtin_convertvector(hw_f32x2{lo, hi}, hw_bf16x2);
  return __builtin_bit_cast(uint32_t, b);
}
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  return __builtin_bit_cast(uint16_t, (__bf16)f);
}

__device__ __forceinline__ int lds_off(int row, int chunk) {
  return row * KB + ((chunk ^ (row & 7)) << 4);
}

template <typename T> struct Mma;

template <> struct Mma<bf16_t> {
  static constexpr int KSTEPS = 4;   // 16 bf16 = 32 bytes of K per MFMA, 128 bytes per stage
  typedef bf16x8 frag;
  static __device__ __forceinline__ frag load(const char* tile, int row, int ks, int half) {
    return *reinterpret_cast<const bf16x8*>(tile + lds_off(row, ks * 2 + half));
  }
  static __device__ __forceinline__ f32x16 mma(frag a, frag b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
  }
};

template <> struct Mma<float> {
  static constexpr int KSTEPS = 16;  // 2 floats = 8 bytes of K per MFMA
  typedef float frag;
  static __device__ __forceinline__ frag load(const char* tile, int row, int ks, int half) {
    int k = ks * 2 + half;           // element index inside the 32-float stage
    return *reinterpret_cast<const float*>(tile + lds_off(row, k >> 2) + ((k & 3) << 2));
  }
  static __device__ __forceinline__ f32x16 mma(frag a, frag b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
  }
};

// Global -> register staging of one operand tile slice: 4 chunks of 16 bytes per thread.
struct Stage {
  u32x4 a[4], b[4];
};

// Rows beyond the limit are clamped to the last valid row (always in bounds; the
// callers mask what those rows produce).  K beyond k_bytes reads as zero.
struct TileSrc {
  const char* base;   // first byte of row 0
  int64_t ld_bytes;   // row pitch
  int row0;           // first row of this tile
  int rows;           // number of valid rows in the tensor (>= 1)
};

__device__ __forceinline__ void load_stage(Stage& s, const TileSrc& A, const TileSrc& B, int k0_bytes, int k_bytes) {
  const int t = threadIdx.x;
  const int chunk = t & 7;
  const int kb = k0_bytes + chunk * 16;
  const bool k_ok = kb < k_bytes;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    int r = (t >> 3) + 64 * j;
    int ra = min(A.row0 + r, A.rows - 1);
    int rb = min(B.row0 + r, B.rows - 1);
    u32x4 z = {0u, 0u, 0u, 0u};
    s.a[j] = k_ok ? *reinterpret_cast<const u32x4*>(A.base + (int64_t)ra * A.ld_bytes + kb) : z;
    s.b[j] = k_ok ? *reinterpret_cast<const u32x4*>(B.base + (int64_t)rb * B.ld_bytes + kb) : z;
  }
}

__device__ __forceinline__ void store_stage(const Stage& s, char* lds_stage) {
  const int t = threadIdx.x;
  const int chunk = t & 7;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    int r = (t >> 3) + 64 * j;
    *reinterpret_cast<u32x4*>(lds_stage + lds_off(r, chunk)) = s.a[j];
    *reinterpret_cast<u32x4*>(lds_stage + TILE * KB + lds_off(r, chunk)) = s.b[j];
  }
}

template <typename T>
__device__ __forceinline__ void compute_stage(const char* lds_stage, f32x16 (&acc)[WM][WN]) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int wm = wave >> 2, wn = wave & 3;
  const int l32 = lane & 31, half = lane >> 5;
  const char* At = lds_stage;
  const char* Bt = lds_stage + TILE * KB;
#pragma unroll
  for (int ks = 0; ks < Mma<T>::KSTEPS; ++ks) {
    typename Mma<T>::frag a[WM], b[WN];
#pragma unroll
    for (int i = 0; i < WM; ++i) a[i] = Mma<T>::load(At, wm * 128 + i * 32 + l32, ks, half);
#pragma unroll
    for (int j = 0; j < WN; ++j) b[j] = Mma<T>::load(Bt, wn * 64 + j * 32 + l32, ks, half);
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
      for (int j = 0; j < WN; ++j) acc[i][j] = Mma<T>::mma(a[i], b[j], acc[i][j]);
  }
}

// acc = A_tile . B_tile^T over the whole K extent.  `lds` is LDS_BYTES of dynamic
// shared memory.  On return every wavefront has passed a barrier after its last
// LDS read, so the caller may reuse `lds`.
template <typename T>
__device__ __forceinline__ void tile_mainloop(const TileSrc& A, const TileSrc& B, int k_bytes, char* lds,
                                              f32x16 (&acc)[WM][WN]) {
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int kt_n = (k_bytes + KB - 1) / KB;
  Stage s;
  load_stage(s, A, B, 0, k_bytes);
  store_stage(s, lds);
  __syncthreads();
  for (int kt = 0; kt < kt_n; ++kt) {
    const bool more = kt + 1 < kt_n;
    if (more) load_stage(s, A, B, (kt + 1) * KB, k_bytes);
    compute_stage<T>(lds + (kt & 1) * STAGE_BYTES, acc);
    if (more) store_stage(s, lds + ((kt + 1) & 1) * STAGE_BYTES);
    __syncthreads();
  }
}

// Position of this lane's accumulator entries inside the 256 x 256 tile.
__device__ __forceinline__ int tile_m(int i, int r) {   // M index of acc[i][*][r]
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  return (wave >> 2) * 128 + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
}
__device__ __forceinline__ int tile_n(int j) {          // N index of acc[*][j][*]
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  return (wave & 3) * 64 + j * 32 + (lane & 31);
}

// Workgroups are handed to the 8 XCDs round-robin by linear id.  This returns a
// logical id such that each XCD works on one contiguous range of logical ids,
// so that tiles sharing operands share that XCD's L2.
__device__ __forceinline__ int xcd_contiguous_id(int bid, int grid) {
  const int x = bid & 7, q = bid >> 3;
  const int per = grid >> 3, rem = grid & 7;
  return x * per + min(x, rem) + q;
}

// Grouped raster: logical id -> (p, q) on a P x Q grid, walking `group` values of
// p for each q before moving on, so neighbouring ids share both operands.
__device__ __forceinline__ void grouped_raster(int id, int P, int Q, int group, int& p, int& q) {
  const int per_group = group * Q;
  const int g = id / per_group;
  const int first = g * group;
  const int size = min(group, P - first);
  const int in = id - g * per_group;
  p = first + in % size;
  q = in / size;
}

}  // namespace flce
