// C-ABI entry points of libflce (see include/flce.h): argument checks, the launch
// plan (windows, chunks, workspace layout) and the launch sequences.  Host code
// only; every step of the path runs in the kernels of kernels.h.
#include "../../include/flce.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <mutex>
#include <vector>

#include "kernels.h"
#include "probe.h"

// Workspace of flce_forward_static, the forward for callers that cannot allocate: a file-scope device array.
// Every GPU the library is loaded on holds its own copy, at its own address, until the process ends.  In host
// code this name is only a handle for hipGetSymbolAddress; kernels are given the address that call returns.
static __device__ __align__(256) unsigned char scratch[FLCE_STATIC_SCRATCH_BYTES];

namespace flce {
namespace {

constexpr int64_t ALIGN = 256;
constexpr int NUM_CU = 256;   // MI355X; the plan must not depend on a device query

int64_t align_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }
int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

int env_int(const char* name, int dflt, int lo, int hi) {
  const char* s = std::getenv(name);
  if (!s || !*s) return dflt;
  long v = std::strtol(s, nullptr, 10);
  if (v < lo) v = lo;
  if (v > hi) v = hi;
  return (int)v;
}

// The tuning knobs of the launch plan.  Read from the environment once, when the first call needs them, and
// fixed for the process from then on (flce_tuning_reload reads them again): a plan never changes between the
// sizing of a workspace and its use, and no call touches the environment afterwards.
struct Tuning {
  int windows, vc_tiles, nc_tiles, splitk_dh, splitk_dw, generic;
};
std::mutex g_tuning_mu;
bool g_tuning_loaded = false;
Tuning g_tuning;

Tuning read_tuning_from_env() {
  Tuning t;
  t.windows = env_int("FLCE_WINDOWS", 0, 0, 1 << 16);
  t.vc_tiles = env_int("FLCE_VC_TILES", 0, 0, 4096);
  t.nc_tiles = env_int("FLCE_NC_TILES", 128, 1, 4096);
  t.splitk_dh = env_int("FLCE_SPLITK_DH", 0, 0, 16);
  t.splitk_dw = env_int("FLCE_SPLITK_DW", 0, 0, 16);
  t.generic = env_int("FLCE_GENERIC", 0, 0, 1);
  return t;
}

Tuning tuning() {
  std::lock_guard<std::mutex> lk(g_tuning_mu);
  if (!g_tuning_loaded) { g_tuning = read_tuning_from_env(); g_tuning_loaded = true; }
  return g_tuning;
}

struct Plan {
  int64_t N, d, V;
  int esize;
  int n_rb, n_vt;          // 256-row tiles of tokens / vocabulary
  int64_t npad;
  // forward
  int n_win;
  int64_t off_part, off_blk_loss, off_blk_cnt, off_blk_oor, off_wpart, off_wsum, off_zbar, off_fHT, fwd_bytes;
  // backward
  int n_vch, n_nch;        // chunks along vocabulary / tokens
  int vc_tiles, nc_tiles;  // largest chunk, in tiles
  int64_t ld_v, ld_n;      // elements per row of the buffers whose rows run over a vocabulary / row chunk: the
                           // chunk's extent plus 64, so that rows never lie a power of two apart
  bool fast;               // tuned bf16 loop: W, Hc and G read in place by the contractions
  bool hkr;                // forward / recompute read a pre-tiled copy of H (tuned loop, unless the caller rules the copy out)
  int split_dh, split_dw;  // K slices of the dH / dW contraction launches (1 = unsplit)
  int64_t off_Hc, off_rowmap, off_tgt, off_lsec, off_gamc, off_HT, off_WT, off_G, off_GT, off_dHacc, off_dWacc, off_partial, bwd_bytes;
};

// A contraction launch of more than one round of workgroups whose last round would be mostly empty: the output-row
// tiles of that last round ("tail") are launched on their own with their K extent cut into `slices` slices (summed
// in slice order by splitk_reduce_kernel, like any split-K launch), so that the tail takes 1 / slices of a round.
// rows = 0: no tail (one round or less; more than four rounds, where the last one matters little and the partial
// sums would cost workspace for it; a last round that is more than half full; a launch that is split anyway).
struct TailSplit { int rows, slices; };
TailSplit tail_split(int64_t out_row_tiles, int64_t n_mt, int n_split, int64_t k_tiles) {
  if (n_split != 1) return {0, 1};
  const int64_t tiles = out_row_tiles * n_mt;
  if (tiles <= NUM_CU || tiles > 4 * NUM_CU) return {0, 1};
  const int64_t body_rows = tiles / NUM_CU * NUM_CU / n_mt;
  const int64_t rows = out_row_tiles - body_rows;
  if (rows <= 0 || body_rows <= 0) return {0, 1};
  // whole slices of at least two 256-element K tiles each, at most 8
  const int64_t slices = std::min<int64_t>(std::min<int64_t>(NUM_CU / (rows * n_mt), 8), k_tiles / 2);
  if (slices < 2) return {0, 1};
  return {(int)rows, (int)slices};
}

// The tuned bf16 loop needs K extents that are multiples of 32 elements and every tile's address
// window within reach of a buffer descriptor: offsets and the record count are unsigned 32-bit, and
// the zero-filled overshoot of a last K stage (up to 32 rows) must not wrap 2^32.
// The `generic` knob forces the generic loop everywhere.
bool window_ok(int64_t k_rows, int64_t ld_bytes) { return (k_rows + 32) * ld_bytes < ((int64_t)1 << 32); }
bool fast_loop_ok(const Plan& p, const Tuning& tn) {
  if (p.esize != 2 || tn.generic) return false;
  const int64_t vc = (int64_t)p.vc_tiles * TILE, nc = (int64_t)p.nc_tiles * TILE;
  const int64_t ld_hw = p.d * 2, ld_g = p.ld_v * 2;
  return p.d % 32 == 0 && window_ok(257, ld_hw) && window_ok(257, ld_g) &&      // K-contiguous tiles
         window_ok(vc, ld_hw) && window_ok(nc, ld_hw) && window_ok(nc, ld_g);   // K over memory rows
}

bool make_plan(int64_t N, int64_t d, int64_t V, flce_dtype dt, Plan& p, bool allow_h_copy = true) {
  if (N <= 0 || d <= 0 || V <= 0 || (d % 8) != 0) return false;
  if (N > 0x7FFFFF00ll || V > 0x7FFFFF00ll || d > (1 << 24)) return false;
  if (dt != FLCE_DTYPE_BF16 && dt != FLCE_DTYPE_F32) return false;
  p.N = N; p.d = d; p.V = V;
  p.esize = dt == FLCE_DTYPE_BF16 ? 2 : 4;
  p.n_rb = (int)ceil_div(N, TILE);
  p.n_vt = (int)ceil_div(V, TILE);
  p.npad = (int64_t)p.n_rb * TILE;

  // Windows (Section 3.2.1): enough (row block, window) workgroups to cover the CUs.
  // At least 4, so that the 32 workgroups resident on one XCD are 8 row blocks x 4 windows and
  // share both operands through that XCD's L2 (one window would stream every H block from HBM).
  const Tuning tn = tuning();
  int win = tn.windows;
  if (win == 0) win = (int)std::max<int64_t>(4, ceil_div(NUM_CU, p.n_rb));
  if (win > p.n_vt) win = p.n_vt;
  p.n_win = win;
  int64_t o = ALIGN;                                  // header
  p.off_part = o;       o = align_up(o + 3ll * win * p.npad * 4, ALIGN);
  p.off_blk_loss = o;   o = align_up(o + (int64_t)p.n_rb * 4, ALIGN);
  p.off_blk_cnt = o;    o = align_up(o + (int64_t)p.n_rb * 4, ALIGN);
  p.off_blk_oor = o;    o = align_up(o + (int64_t)p.n_rb * 4, ALIGN);
  // label smoothing (per-row forward): column sums of W by 1024-row chunks, their sum, mean logit per row
  p.off_wpart = o;      o = align_up(o + ceil_div(V, 1024) * d * 4, ALIGN);
  p.off_wsum = o;       o = align_up(o + d * 4, ALIGN);
  p.off_zbar = o;       o = align_up(o + N * 4, ALIGN);
  p.off_fHT = o;        // sized below, once the loop flavour is known
  const int64_t fwd_fixed = o;

  // Backward staging: a fixed-size G tile of at most vc x nc 256-tiles.
  const int nc_max = tn.nc_tiles;
  // Automatic vocabulary chunk: 128 tiles; with few token rows the same staging bytes reach further along the
  // vocabulary (at most 128 x 32 tiles of G, 512 MiB in bf16, up to 512 vocabulary tiles), which saves whole
  // launches and the fp32 running sum of dH on short-sequence shapes.  Kept within a buffer descriptor's reach.
  int vc_max = tn.vc_tiles;
  if (vc_max == 0) {
    const int64_t nct = std::min<int64_t>(p.n_rb, nc_max);
    vc_max = (int)std::max<int64_t>(128, std::min<int64_t>(512, 4096 / nct));
    const int64_t reach = (((int64_t)1 << 32) / (d * p.esize) - 64) / TILE;
    if (vc_max > 128 && reach < vc_max) vc_max = (int)std::max<int64_t>(128, reach);
  }
  // Chunks of the full size plus a remainder, so that launches of full chunks come out in whole rounds of 256
  // workgroups (128 tiles times any even tile count); an even split only when the remainder would be a sliver.
  auto chunking = [](int tiles, int cmax, int& n_chunks, int& chunk) {
    n_chunks = (int)ceil_div(tiles, cmax);
    const int rem = tiles - (n_chunks - 1) * cmax;
    chunk = (n_chunks == 1 || rem * 4 >= cmax) ? std::min(tiles, cmax) : (int)ceil_div(tiles, n_chunks);
  };
  chunking(p.n_vt, vc_max, p.n_vch, p.vc_tiles);
  chunking(p.n_rb, nc_max, p.n_nch, p.nc_tiles);
  const int64_t vc_pad = (int64_t)p.vc_tiles * TILE, nc_pad = (int64_t)p.nc_tiles * TILE;
  p.ld_v = vc_pad + 64;
  p.ld_n = nc_pad + 64;
  p.fast = fast_loop_ok(p, tn);
  p.hkr = allow_h_copy && p.fast;
  p.fwd_bytes = fwd_fixed + (p.hkr ? align_up(packed_block_offset(p.n_rb, (int)d), ALIGN) : 0);
  o = ALIGN;
  // the counted rows of H: as they are (generic loop), or pre-tiled for the dW contraction (tuned loop)
  p.off_Hc = o;     o = align_up(o + (p.fast ? packed_cols_offset((int)ceil_div(d, TILE), (int)p.npad) : d * p.npad * p.esize), ALIGN);
  p.off_rowmap = o; o = align_up(o + p.npad * 4, ALIGN);
  p.off_tgt = o;    o = align_up(o + p.npad * 4, ALIGN);
  p.off_lsec = o;   o = align_up(o + p.npad * 4, ALIGN);
  p.off_gamc = o;   o = align_up(o + p.npad * 4, ALIGN);
  p.off_G = o;      o = align_up(o + nc_pad * p.ld_v * p.esize, ALIGN);
  // K-contiguous copies, only for main loops that cannot read an operand across memory rows
  p.off_HT = o;     if (!p.fast) o = align_up(o + d * p.npad * p.esize, ALIGN);
                    else if (p.hkr) o = align_up(o + packed_block_offset(p.n_rb, (int)d), ALIGN);
  p.off_WT = o;     if (!p.fast) o = align_up(o + d * p.ld_v * p.esize, ALIGN);
  p.off_GT = o;     if (!p.fast) o = align_up(o + vc_pad * p.ld_n * p.esize, ALIGN);
  p.off_dHacc = o;  if (p.n_vch > 1) o = align_up(o + N * d * 4, ALIGN);
  p.off_dWacc = o;  if (p.n_nch > 1) o = align_up(o + vc_pad * d * 4, ALIGN);
  // Split-K for launches with too few output tiles to occupy the CUs (small N or small d): the K
  // extent is cut into slices whose fp32 tiles are summed in slice order by a second kernel.
  const int64_t n_mt = ceil_div(d, TILE);
  auto auto_split = [&](int64_t tiles, int64_t k_tiles) -> int {
    // How full the rounds of workgroups are, discounted for the partial-sum traffic of each extra
    // slice (about 30 % of a tile's time when K is 16 tiles, less in proportion for longer K); a
    // split has to win by 5 %.
    int best = 1;
    double best_score = 0.0;
    for (int sp = 1; sp <= 8 && (sp == 1 || k_tiles / sp >= 2); ++sp) {
      const int64_t wg = tiles * sp;
      const double fill = (double)wg / (double)(ceil_div(wg, NUM_CU) * NUM_CU);
      const double score = fill / (1.0 + (4.8 / (double)k_tiles) * (sp - 1));
      if (score > best_score * (sp == 1 ? 1.0 : 1.05)) { best_score = score; best = sp; }
    }
    return best;
  };
  p.split_dh = tn.splitk_dh;
  p.split_dw = tn.splitk_dw;
  if (p.split_dh == 0) p.split_dh = auto_split(p.nc_tiles * n_mt, p.vc_tiles);
  if (p.split_dw == 0) p.split_dw = auto_split(p.vc_tiles * n_mt, p.nc_tiles);
  p.split_dh = (int)std::min<int64_t>(p.split_dh, p.vc_tiles);
  p.split_dw = (int)std::min<int64_t>(p.split_dw, p.nc_tiles);
  p.off_partial = o;
  {
    int64_t bytes = 0;
    if (p.split_dh > 1) bytes = std::max(bytes, (int64_t)p.split_dh * nc_pad * d * 4);
    if (p.split_dw > 1) bytes = std::max(bytes, (int64_t)p.split_dw * vc_pad * d * 4);
    if (p.fast) {
      // tails of the launches that occur: full chunks and the last (shorter) chunk of either direction
      const int64_t v_last = p.n_vt - (int64_t)(p.n_vch - 1) * p.vc_tiles, n_last = p.n_rb - (int64_t)(p.n_nch - 1) * p.nc_tiles;
      for (const int64_t vt : {(int64_t)p.vc_tiles, v_last})
        for (const int64_t nt : {(int64_t)p.nc_tiles, n_last}) {
          const TailSplit tw = tail_split(vt, n_mt, p.split_dw, nt), th = tail_split(nt, n_mt, p.split_dh, vt);
          if (tw.rows) bytes = std::max(bytes, (int64_t)tw.slices * tw.rows * TILE * d * 4);
          if (th.rows) bytes = std::max(bytes, (int64_t)th.slices * th.rows * TILE * d * 4);
        }
    }
    o = align_up(o + bytes, ALIGN);
  }
  p.bwd_bytes = o;
  return true;
}

// Optional per-launch event timing (flce_profile_*).
struct ProfRec { int cls; hipEvent_t a, b; };
struct Prof {
  std::mutex mu;
  bool on = false;
  std::vector<hipEvent_t> pool;
  std::vector<ProfRec> recs;
  hipEvent_t get() {
    if (!pool.empty()) { hipEvent_t e = pool.back(); pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
  }
};
Prof g_prof;

struct ProfScope {
  hipStream_t st;
  hipEvent_t b = nullptr;
  ProfScope(int cls, hipStream_t s) : st(s) {
    if (!g_prof.on) return;
    std::lock_guard<std::mutex> lk(g_prof.mu);
    hipEvent_t a = g_prof.get();
    b = g_prof.get();
    if (!a || !b) { b = nullptr; return; }
    (void)hipEventRecord(a, st);
    g_prof.recs.push_back(ProfRec{cls, a, b});
  }
  ~ProfScope() { if (b) (void)hipEventRecord(b, st); }
};

template <typename K>
hipError_t allow_big_lds(K kernel, int bytes) {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

// The kernels of one (storage type, main loop) pair need the large dynamic LDS allowance; it is a property of
// the loaded code object on a device, so it is set once per device and pair, not per call.
constexpr int MAX_DEVICES = 64;

template <typename T, typename L>
hipError_t set_lds_allowances() {
  hipError_t e;
  if ((e = allow_big_lds(fwd_tiles_kernel<T, L, false>, L::LDS)) != hipSuccess) return e;
  if ((e = allow_big_lds(recompute_kernel<T, L, false>, L::LDS)) != hipSuccess) return e;
  if ((e = allow_big_lds(recompute_kernel<T, L, false, true>, L::LDS)) != hipSuccess) return e;
  if constexpr (L::TRANSPOSING) {
    if ((e = allow_big_lds(fwd_tiles_kernel<T, L, true>, L::LDS)) != hipSuccess) return e;
    if ((e = allow_big_lds(recompute_kernel<T, L, true>, L::LDS)) != hipSuccess) return e;
    if ((e = allow_big_lds(recompute_kernel<T, L, true, true>, L::LDS)) != hipSuccess) return e;
    if ((e = allow_big_lds(contract_kernel<T, L, OPS_DH_TR>, L::LDS)) != hipSuccess) return e;
    if ((e = allow_big_lds(contract_kernel<T, L, OPS_DW_TR>, L::LDS)) != hipSuccess) return e;
  } else {
    if ((e = allow_big_lds(contract_kernel<T, L, OPS_KC>, L::LDS)) != hipSuccess) return e;
  }
  return hipSuccess;
}

template <typename T, typename L>
hipError_t prepare_kernels() {
  static std::mutex mu;
  static bool done[MAX_DEVICES] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lk(mu);
  if (done[dev]) return hipSuccess;
  if ((e = set_lds_allowances<T, L>()) != hipSuccess) return e;
  done[dev] = true;
  return hipSuccess;
}

// W holds the p.V vocabulary rows [slice.v_begin, slice.v_begin + p.V) of slice.V_total.  With m_out set the
// call stops after the window merge and hands out the slice's (m, a, z_target) per row.
struct Slice { int64_t V_total, v_begin; };
// Per-row variant: the forward writes one loss per row (label-smoothed by eps), the backward takes one
// upstream gradient per row (device arrays of N floats).
struct PerRow { float* loss_rows_out; const float* grad_rows; float eps; };

template <typename T, typename U, typename L>
flce_status forward_t(const Plan& p, const void* H, const void* W, const int64_t* y, int64_t ignore_index,
                      int mean, float* loss_out, float* lse_out, char* ws, hipStream_t st, Slice slice,
                      float* m_out = nullptr, float* a_out = nullptr, float* zt_out = nullptr,
                      PerRow rows = PerRow{nullptr, nullptr, 0.f}) {
  if (prepare_kernels<T, L>() != hipSuccess) return FLCE_ERR_HIP;
  Header* hdr = reinterpret_cast<Header*>(ws);
  float* part = reinterpret_cast<float*>(ws + p.off_part);
  float* blk_loss = reinterpret_cast<float*>(ws + p.off_blk_loss);
  int* blk_cnt = reinterpret_cast<int*>(ws + p.off_blk_cnt);
  int* blk_oor = reinterpret_cast<int*>(ws + p.off_blk_oor);
  // One workgroup per item (row block x window).  With the tuned loop a launch takes at most one round of workgroups
  // (256 items, whole raster groups of 8 row blocks when the window count divides 32): a larger grid's later rounds
  // drift apart over the ~100 tiles of an item and stop sharing their operands in the L2 (measured at 512 row blocks:
  // 361 GB of fabric traffic per forward against 192 GB that the raster should need).
  const int items = p.n_rb * p.n_win;
  const int per_launch = L::TRANSPOSING ? NUM_CU : items;
  bool hkr = false;
  if constexpr (L::TRANSPOSING) hkr = p.hkr;
  T* HT = nullptr;
  if (hkr) {
    if constexpr (L::TRANSPOSING) {
      HT = reinterpret_cast<T*>(ws + p.off_fHT);
      // the pre-tiled copy of H, zero padded to whole row blocks: the forward's second operand
      ProfScope ps(FLCE_PROF_FWD_EPILOGUE, st);
      pack_rows_kernel<<<dim3((unsigned)(p.npad / 64), (unsigned)ceil_div(p.d, 128)), 256, 0, st>>>(
          static_cast<const char*>(H), (int)p.N, (int)p.d, reinterpret_cast<char*>(HT));
    }
  }
  {
    ProfScope ps(FLCE_PROF_FWD_TILES, st);
    for (int item0 = 0; item0 < items; item0 += per_launch) {
      const int grid = std::min(per_launch, items - item0);
      if (hkr) {
        if constexpr (L::TRANSPOSING)
          fwd_tiles_kernel<T, L, true><<<grid, L::THREADS, L::LDS, st>>>(
              static_cast<const T*>(H), HT, static_cast<const T*>(W), y, (int)p.N, (int)p.d, (int)p.V, ignore_index,
              slice.V_total, slice.v_begin, p.n_rb, p.n_win, p.n_vt, part, item0);
      } else {
        fwd_tiles_kernel<T, L, false><<<grid, L::THREADS, L::LDS, st>>>(
            static_cast<const T*>(H), nullptr, static_cast<const T*>(W), y, (int)p.N, (int)p.d, (int)p.V, ignore_index,
            slice.V_total, slice.v_begin, p.n_rb, p.n_win, p.n_vt, part, item0);
      }
    }
  }
  {
    ProfScope ps(FLCE_PROF_FWD_EPILOGUE, st);
    if (m_out) {
      merge_rows_partial_kernel<<<p.n_rb, 256, 0, st>>>(part, p.n_win, p.npad, (int)p.N, m_out, a_out, zt_out);
    } else {
      const int64_t plane = (int64_t)p.n_win * p.npad;
      const float* zbar = nullptr;
      if (rows.loss_rows_out && rows.eps != 0.f) {
        float* wpart = reinterpret_cast<float*>(ws + p.off_wpart);
        float* wsum = reinterpret_cast<float*>(ws + p.off_wsum);
        float* zb = reinterpret_cast<float*>(ws + p.off_zbar);
        const int n_chunks = (int)ceil_div(p.V, 1024);
        colsum_chunks_kernel<T><<<n_chunks, 256, 0, st>>>(static_cast<const T*>(W), (int)p.V, (int)p.d, wpart);
        colsum_finish_kernel<<<(unsigned)ceil_div(p.d, 256), 256, 0, st>>>(wpart, n_chunks, (int)p.d, wsum);
        mean_logit_kernel<T><<<(unsigned)p.N, 256, 0, st>>>(static_cast<const T*>(H), wsum, (int)p.d,
                                                            1.0f / (float)p.V, zb);
        zbar = zb;
      }
      merge_rows_kernel<<<p.n_rb, 256, 0, st>>>(part, part + plane, part + 2 * plane, p.n_win, p.npad, y, (int)p.N,
                                                slice.V_total, ignore_index, lse_out, blk_loss, blk_cnt, blk_oor,
                                                rows.loss_rows_out, zbar, rows.eps);
      // the per-row call has no scalar loss to hand out: the sum goes to a spare word of the header block
      float* scalar = loss_out ? loss_out : reinterpret_cast<float*>(ws + 64);
      finalize_loss_kernel<<<1, 256, 0, st>>>(blk_loss, blk_cnt, blk_oor, p.n_rb, mean, hdr, scalar);
    }
  }
  return hipGetLastError() == hipSuccess ? FLCE_OK : FLCE_ERR_HIP;
}

template <typename T, typename U, typename L>
flce_status backward_t(const Plan& p, const void* H, const void* W, const int64_t* y, const float* lse,
                       int64_t ignore_index, int mean, float grad_loss, void* dH, void* dW, char* ws,
                       hipStream_t st, Slice slice, PerRow rows = PerRow{nullptr, nullptr, 0.f}) {
  if (prepare_kernels<T, L>() != hipSuccess) return FLCE_ERR_HIP;
  if (L::TRANSPOSING && !p.hkr) return FLCE_ERR_UNSUPPORTED;   // (no caller plans a backward without the copies of H)
  const int N = (int)p.N, d = (int)p.d, V = (int)p.V;
  Header* hdr = reinterpret_cast<Header*>(ws);
  T* Hc = reinterpret_cast<T*>(ws + p.off_Hc);
  int* rowmap = reinterpret_cast<int*>(ws + p.off_rowmap);
  int* tgt_c = reinterpret_cast<int*>(ws + p.off_tgt);
  float* lse_c = reinterpret_cast<float*>(ws + p.off_lsec);
  float* gam_c = reinterpret_cast<float*>(ws + p.off_gamc);
  T* HT = reinterpret_cast<T*>(ws + p.off_HT);
  T* WT = reinterpret_cast<T*>(ws + p.off_WT);
  T* G = reinterpret_cast<T*>(ws + p.off_G);
  T* GT = reinterpret_cast<T*>(ws + p.off_GT);
  float* dHacc = reinterpret_cast<float*>(ws + p.off_dHacc);
  float* dWacc = reinterpret_cast<float*>(ws + p.off_dWacc);
  const int64_t vc_pad = (int64_t)p.vc_tiles * TILE, nc_pad = (int64_t)p.nc_tiles * TILE;
  const int n_mt = (int)ceil_div(d, TILE);
  const int npad = (int)p.npad;

  {
    ProfScope ps(FLCE_PROF_BWD_PREP, st);
    compact_targets_kernel<<<1, 1024, 0, st>>>(y, N, V, slice.V_total, slice.v_begin, ignore_index, npad, rowmap,
                                               tgt_c, hdr);
    // lse and Gamma per compact row, zero rows of dH, and the counted rows of H packed together, twice: with the
    // generic loop as they are (Hc) and transposed [d][npad] (the dW contraction's K-contiguous operand); with the
    // tuned loop pre-tiled for the recompute (in HT's place) and pre-tiled the other way round for dW (in Hc's place)
    if constexpr (L::TRANSPOSING)
      prep_rows_tiled_kernel<<<dim3((unsigned)(p.npad / 32), (unsigned)n_mt), 256, 0, st>>>(
          static_cast<const char*>(H), d, rowmap, npad, reinterpret_cast<char*>(HT), reinterpret_cast<char*>(Hc), lse,
          lse_c, rows.grad_rows, gam_c, y, N, slice.V_total, ignore_index, static_cast<char*>(dH));
    else
      prep_rows_kernel<U><<<dim3((unsigned)(p.npad / 64), (unsigned)ceil_div(d, 64)), 256, 0, st>>>(
          static_cast<const U*>(H), d, rowmap, reinterpret_cast<U*>(Hc), reinterpret_cast<U*>(HT), p.npad, lse, lse_c,
          rows.grad_rows, gam_c, y, N, slice.V_total, ignore_index, static_cast<U*>(dH));
  }

  // With the tuned loop G is staged in blocks of 16 rows x 32 positions (1 KiB), the blocks of a row group one after
  // the other plus one block of skew, so that row groups do not lie a power of two apart; this fits the row-major
  // size the plan reserves (16 rows of ld_v = vc_pad + 64 elements are one block more per group).
  const int64_t g_group_bytes = (vc_pad / 32 + 1) * 1024;
  float* partial = reinterpret_cast<float*>(ws + p.off_partial);
  // K elements per split-K slice: whole 256-element tiles
  auto slice_len = [](int k_elems, int n_split) { return (int)ceil_div(ceil_div(k_elems, TILE), n_split) * TILE; };
  // argument blocks of the three steps of chunk (vc, nc); `Gb` is the staging buffer of that chunk
  auto chunk_vt = [&](int vc, int& vt0, int& n_vt) {
    vt0 = vc * p.vc_tiles;
    n_vt = std::min(p.vc_tiles, p.n_vt - vt0);
  };
  auto chunk_nt = [&](int nc, int& nt0, int& n_nt) {
    nt0 = nc * p.nc_tiles;
    n_nt = std::min(p.nc_tiles, p.n_rb - nt0);
  };
  auto recompute_args = [&](int vc, int nc, T* Gb) {
    int vt0, n_vt, nt0, n_nt;
    chunk_vt(vc, vt0, n_vt);
    chunk_nt(nc, nt0, n_nt);
    return RecomputeArgs<T>{Hc, HT, static_cast<const T*>(W), tgt_c, lse_c, hdr, npad, d, V, nt0, n_nt, vt0, n_vt,
                            Gb, L::TRANSPOSING ? g_group_bytes : p.ld_v, GT, p.ld_n, gam_c, 1.f - rows.eps,
                            rows.eps / (float)slice.V_total};
  };
  // dW[vocab chunk] += G^T . Hc[row chunk]   (contraction over the compact rows of the chunk)
  auto dw_args = [&](int vc, int nc, const T* Gb) {
    int vt0, n_vt, nt0, n_nt;
    chunk_vt(vc, vt0, n_vt);
    chunk_nt(nc, nt0, n_nt);
    int flags = K_COMPACT;
    if (nc > 0) flags |= READ_ACC;
    flags |= (nc + 1 < p.n_nch) ? WRITE_ACC : WRITE_OUT;
    if constexpr (L::TRANSPOSING)
      return ContractArgs<T>{Hc, npad, 0, d, Gb, g_group_bytes, n_nt * TILE,
                             n_nt * TILE, nt0 * TILE, n_mt, n_vt, dWacc, vt0 * TILE, static_cast<T*>(dW), vt0 * TILE,
                             V, flags, hdr, rowmap, grad_loss, mean, p.split_dw,
                             slice_len(n_nt * TILE, p.split_dw), partial, vc_pad * d};
    else
      return ContractArgs<T>{HT + (int64_t)nt0 * TILE, p.npad, 0, d, GT, p.ld_n, n_vt * TILE, n_nt * TILE,
                             nt0 * TILE, n_mt, n_vt, dWacc, vt0 * TILE, static_cast<T*>(dW), vt0 * TILE, V, flags,
                             hdr, rowmap, grad_loss, mean, p.split_dw, slice_len(n_nt * TILE, p.split_dw), partial,
                             vc_pad * d};
  };
  // dH[row chunk] += G . W[vocab chunk]      (contraction over the vocabulary chunk)
  auto dh_args = [&](int vc, int nc, const T* Gb) {
    int vt0, n_vt, nt0, n_nt;
    chunk_vt(vc, vt0, n_vt);
    chunk_nt(nc, nt0, n_nt);
    int flags = ROWS_COMPACT;
    if (vc > 0) flags |= READ_ACC;
    flags |= (vc + 1 < p.n_vch) ? WRITE_ACC : WRITE_OUT;
    if constexpr (L::TRANSPOSING)
      return ContractArgs<T>{static_cast<const T*>(W) + (int64_t)vt0 * TILE * d, d, V - vt0 * TILE, d, Gb, g_group_bytes,
                             n_nt * TILE, n_vt * TILE, 0, n_mt, n_nt, dHacc, 0, static_cast<T*>(dH), nt0 * TILE, npad,
                             flags, hdr, rowmap, grad_loss, mean, p.split_dh, slice_len(n_vt * TILE, p.split_dh),
                             partial - (int64_t)nt0 * TILE * d, nc_pad * d};
    else
      return ContractArgs<T>{WT, p.ld_v, 0, d, Gb, p.ld_v, n_nt * TILE, n_vt * TILE, 0, n_mt, n_nt, dHacc, 0,
                             static_cast<T*>(dH), nt0 * TILE, npad, flags, hdr, rowmap, grad_loss, mean, p.split_dh,
                             slice_len(n_vt * TILE, p.split_dh), partial - (int64_t)nt0 * TILE * d, nc_pad * d};
  };

  // One contraction (dW or dH) of a chunk: the launch, its split-K sum if it has one, and with the tuned loop a
  // separately launched, K-split tail when the last round of workgroups would be mostly empty (tail_split).
  auto contract = [&](const ContractArgs<T>& a, bool is_dw) {
    auto launch = [&](const ContractArgs<T>& x) {
      if constexpr (L::TRANSPOSING) {
        const int grid = std::min(x.n_nt * x.n_mt * x.n_split, NUM_CU);
        if (is_dw) contract_kernel<T, L, OPS_DW_TR><<<grid, L::THREADS, L::LDS, st>>>(x);
        else contract_kernel<T, L, OPS_DH_TR><<<grid, L::THREADS, L::LDS, st>>>(x);
      } else {
        contract_kernel<T, L, OPS_KC><<<x.n_nt * x.n_mt * x.n_split, L::THREADS, L::LDS, st>>>(x);
      }
      if (x.n_split > 1) splitk_reduce_kernel<T><<<x.n_nt * TILE, 256, 0, st>>>(x);
    };
    TailSplit ts{0, 1};
    if constexpr (L::TRANSPOSING) ts = tail_split(a.n_nt, a.n_mt, a.n_split, a.k_elems / TILE);
    if (!ts.rows) { launch(a); return; }
    ContractArgs<T> body = a, tail = a;
    body.n_nt = a.n_nt - ts.rows;
    const int64_t first = (int64_t)body.n_nt * TILE;     // the tail's first output row, relative to the launch's
    tail.n_nt = ts.rows;
    tail.out_row0 = a.out_row0 + (int)first;
    // G (blocked, ldb = bytes per group of 16 rows) is the B operand of both: its columns are dW's output rows (32
    // per block of 1 KiB), its rows are dH's
    const char* g = reinterpret_cast<const char*>(a.B);
    if (is_dw) { tail.B = reinterpret_cast<const T*>(g + first / 32 * 1024); }
    else { tail.B = reinterpret_cast<const T*>(g + first / 16 * a.ldb); tail.b_rows = a.b_rows - (int)first; }
    tail.n_split = ts.slices;
    tail.k_split = slice_len(a.k_elems, ts.slices);
    tail.partial = a.partial - first * a.d;                // indexed like accbuf: by output row from the launch's first
    tail.partial_stride = (int64_t)ts.rows * TILE * a.d;
    launch(body);
    launch(tail);
  };

  for (int vc = 0; vc < p.n_vch; ++vc) {
    int vt0, n_vt;
    chunk_vt(vc, vt0, n_vt);
    if constexpr (!L::TRANSPOSING) {
      // W^T chunk [d][ld_v]: K-contiguous operand of the dH contraction
      ProfScope ps(FLCE_PROF_BWD_PREP, st);
      transpose_pad_kernel<U><<<dim3((unsigned)(n_vt * TILE / 64), (unsigned)ceil_div(d, 64)), 256, 0, st>>>(
          static_cast<const U*>(W), d, V, vt0 * TILE, d, reinterpret_cast<U*>(WT), p.ld_v, n_vt * TILE);
    }
    for (int nc = 0; nc < p.n_nch; ++nc) {
      {
        const RecomputeArgs<T> rc = recompute_args(vc, nc, G);
        ProfScope ps(FLCE_PROF_RECOMPUTE, st);
        // at most one workgroup per CU: each walks its share of the chunk's tiles
        const int grid = L::TRANSPOSING ? std::min(rc.n_nt * rc.n_vt, NUM_CU) : rc.n_nt * rc.n_vt;
        if constexpr (L::TRANSPOSING) {     // the tuned loop's backward always has the pre-tiled copies
          if (rows.grad_rows) recompute_kernel<T, L, true, true><<<grid, L::THREADS, L::LDS, st>>>(rc);
          else recompute_kernel<T, L, true><<<grid, L::THREADS, L::LDS, st>>>(rc);
        } else {
          if (rows.grad_rows) recompute_kernel<T, L, false, true><<<grid, L::THREADS, L::LDS, st>>>(rc);
          else recompute_kernel<T, L, false><<<grid, L::THREADS, L::LDS, st>>>(rc);
        }
      }
      {
        ProfScope ps(FLCE_PROF_CONTRACT_DW, st);
        contract(dw_args(vc, nc, G), true);
      }
      {
        ProfScope ps(FLCE_PROF_CONTRACT_DH, st);
        contract(dh_args(vc, nc, G), false);
      }
    }
  }
  return hipGetLastError() == hipSuccess ? FLCE_OK : FLCE_ERR_HIP;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

constexpr size_t STATIC_SCRATCH_BYTES = FLCE_STATIC_SCRATCH_BYTES;

std::mutex g_scratch_mu;
void* g_scratch_ptr[MAX_DEVICES] = {};

// Device address of `scratch` on the current device (looked up once per device), or nullptr.
hipError_t static_scratch(void** out) {
  *out = nullptr;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(::scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

// Hands the status header of a finished forward to the caller's own device words (either may be null).
__global__ void export_header_kernel(const Header* __restrict__ hdr, int32_t* __restrict__ status_out,
                                     int64_t* __restrict__ n_valid_out) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    if (status_out) *status_out = hdr->status;
    if (n_valid_out) *n_valid_out = hdr->n_valid;
  }
}

}  // namespace
}  // namespace flce

extern "C" {

const char* flce_version(void) { return "0.2.0"; }

void flce_tuning_reload(void) {
  std::lock_guard<std::mutex> lk(flce::g_tuning_mu);
  flce::g_tuning = flce::read_tuning_from_env();
  flce::g_tuning_loaded = true;
}

const char* flce_status_string(flce_status s) {
  switch (s) {
    case FLCE_OK: return "ok";
    case FLCE_ERR_BAD_ARG: return "bad argument";
    case FLCE_ERR_BAD_SHAPE: return "bad shape";
    case FLCE_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case FLCE_ERR_TARGET_RANGE: return "target outside [0, V)";
    case FLCE_ERR_UNSUPPORTED: return "unsupported";
    case FLCE_ERR_HIP: return "HIP runtime error";
  }
  return "unknown status";
}

int flce_plan_describe(int64_t N, int64_t d, int64_t V, flce_dtype dt, char* buf, size_t buf_bytes) {
  flce::Plan p;
  if (!buf || buf_bytes == 0 || !flce::make_plan(N, d, V, dt, p)) return -1;
  // K-split tails of the contraction launches of a full chunk (output-row tiles x slices; 0x1 = none)
  const int64_t n_mt = (d + flce::TILE - 1) / flce::TILE;
  flce::TailSplit th{0, 1}, tw{0, 1};
  if (p.fast) {
    th = flce::tail_split(p.nc_tiles, n_mt, p.split_dh, p.vc_tiles);
    tw = flce::tail_split(p.vc_tiles, n_mt, p.split_dw, p.nc_tiles);
  }
  return std::snprintf(buf, buf_bytes,
                       "flce %s loop=%s h_copy=%d windows=%d vocab_chunks=%dx%d row_chunks=%dx%d splitk_dH=%d splitk_dW=%d "
                       "tail_dH=%dx%d tail_dW=%dx%d staging_bytes=%lld fwd_ws=%lld bwd_ws=%lld",
                       flce_version(), p.fast ? "tuned" : "generic", p.hkr ? 1 : 0, p.n_win, p.n_vch, p.vc_tiles, p.n_nch,
                       p.nc_tiles, p.split_dh, p.split_dw, th.rows, th.slices, tw.rows, tw.slices,
                       (long long)((int64_t)p.nc_tiles * flce::TILE * p.ld_v * p.esize), (long long)p.fwd_bytes,
                       (long long)p.bwd_bytes);
}

size_t flce_workspace_bytes(int64_t N, int64_t d, int64_t V, flce_dtype dt, int for_backward) {
  flce::Plan p;
  if (!flce::make_plan(N, d, V, dt, p)) return 0;
  return (size_t)(for_backward ? p.bwd_bytes : p.fwd_bytes);
}

static flce_status forward_impl(const void* H, const void* W, const int64_t* targets, int64_t N, int64_t d,
                                int64_t V, int64_t ignore_index, flce_reduction reduction, flce_dtype dt,
                                float* loss_out, float* lse_out, void* workspace, size_t workspace_bytes,
                                void* hip_stream, flce::Slice slice, float* m_out, float* a_out, float* zt_out,
                                flce::PerRow rows = flce::PerRow{nullptr, nullptr, 0.f}, bool allow_h_copy = true) {
  const bool partial = m_out || a_out || zt_out;
  if (!H || !W || !targets) return FLCE_ERR_BAD_ARG;
  if (partial ? (!m_out || !a_out || !zt_out) : ((!loss_out && !rows.loss_rows_out) || !lse_out))
    return FLCE_ERR_BAD_ARG;
  if (!(rows.eps >= 0.f && rows.eps < 1.f)) return FLCE_ERR_BAD_ARG;
  if (reduction != FLCE_REDUCE_MEAN && reduction != FLCE_REDUCE_SUM) return FLCE_ERR_BAD_ARG;
  if (dt != FLCE_DTYPE_BF16 && dt != FLCE_DTYPE_F32) return FLCE_ERR_BAD_ARG;
  flce::Plan p;
  if (!flce::make_plan(N, d, V, dt, p, allow_h_copy)) return FLCE_ERR_BAD_SHAPE;
  if (slice.v_begin < 0 || slice.v_begin + V > slice.V_total) return FLCE_ERR_BAD_SHAPE;
  if (!flce::aligned16(H) || !flce::aligned16(W)) return FLCE_ERR_BAD_ARG;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < (size_t)p.fwd_bytes)
    return FLCE_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int mean = reduction == FLCE_REDUCE_MEAN;
  char* ws = static_cast<char*>(workspace);
  if (dt == FLCE_DTYPE_BF16) {
    if (p.fast)
      return flce::forward_t<flce::bf16_t, uint16_t, flce::FastLoop>(p, H, W, targets, ignore_index, mean, loss_out,
                                                                     lse_out, ws, st, slice, m_out, a_out, zt_out,
                                                                     rows);
    return flce::forward_t<flce::bf16_t, uint16_t, flce::GenericLoop<flce::bf16_t>>(
        p, H, W, targets, ignore_index, mean, loss_out, lse_out, ws, st, slice, m_out, a_out, zt_out, rows);
  }
  return flce::forward_t<float, uint32_t, flce::GenericLoop<float>>(p, H, W, targets, ignore_index, mean, loss_out,
                                                                    lse_out, ws, st, slice, m_out, a_out, zt_out,
                                                                    rows);
}

static flce_status backward_impl(const void* H, const void* W, const int64_t* targets, const float* lse, int64_t N,
                                 int64_t d, int64_t V, int64_t ignore_index, flce_reduction reduction, flce_dtype dt,
                                 float grad_loss, void* dH_out, void* dW_out, void* workspace, size_t workspace_bytes,
                                 void* hip_stream, flce::Slice slice,
                                 flce::PerRow rows = flce::PerRow{nullptr, nullptr, 0.f}) {
  if (!H || !W || !targets || !lse || !dH_out || !dW_out) return FLCE_ERR_BAD_ARG;
  if (!(rows.eps >= 0.f && rows.eps < 1.f)) return FLCE_ERR_BAD_ARG;
  if (reduction != FLCE_REDUCE_MEAN && reduction != FLCE_REDUCE_SUM) return FLCE_ERR_BAD_ARG;
  if (dt != FLCE_DTYPE_BF16 && dt != FLCE_DTYPE_F32) return FLCE_ERR_BAD_ARG;
  flce::Plan p;
  if (!flce::make_plan(N, d, V, dt, p)) return FLCE_ERR_BAD_SHAPE;
  if (slice.v_begin < 0 || slice.v_begin + V > slice.V_total) return FLCE_ERR_BAD_SHAPE;
  if (!flce::aligned16(H) || !flce::aligned16(W) || !flce::aligned16(dH_out) || !flce::aligned16(dW_out))
    return FLCE_ERR_BAD_ARG;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < (size_t)p.bwd_bytes)
    return FLCE_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int mean = reduction == FLCE_REDUCE_MEAN;
  char* ws = static_cast<char*>(workspace);
  if (dt == FLCE_DTYPE_BF16) {
    if (p.fast)
      return flce::backward_t<flce::bf16_t, uint16_t, flce::FastLoop>(p, H, W, targets, lse, ignore_index, mean,
                                                                      grad_loss, dH_out, dW_out, ws, st, slice,
                                                                      rows);
    return flce::backward_t<flce::bf16_t, uint16_t, flce::GenericLoop<flce::bf16_t>>(
        p, H, W, targets, lse, ignore_index, mean, grad_loss, dH_out, dW_out, ws, st, slice, rows);
  }
  return flce::backward_t<float, uint32_t, flce::GenericLoop<float>>(p, H, W, targets, lse, ignore_index, mean,
                                                                     grad_loss, dH_out, dW_out, ws, st, slice, rows);
}

flce_status flce_forward(const void* H, const void* W, const int64_t* targets, int64_t N, int64_t d, int64_t V,
                         int64_t ignore_index, flce_reduction reduction, flce_dtype dt, float* loss_out,
                         float* lse_out, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return forward_impl(H, W, targets, N, d, V, ignore_index, reduction, dt, loss_out, lse_out, workspace,
                      workspace_bytes, hip_stream, flce::Slice{V, 0}, nullptr, nullptr, nullptr);
}

flce_status flce_backward(const void* H, const void* W, const int64_t* targets, const float* lse, int64_t N,
                          int64_t d, int64_t V, int64_t ignore_index, flce_reduction reduction, flce_dtype dt,
                          float grad_loss, void* dH_out, void* dW_out, void* workspace, size_t workspace_bytes,
                          void* hip_stream) {
  return backward_impl(H, W, targets, lse, N, d, V, ignore_index, reduction, dt, grad_loss, dH_out, dW_out,
                       workspace, workspace_bytes, hip_stream, flce::Slice{V, 0});
}

flce_status flce_forward_static(const void* H, const void* W, const int64_t* targets, int64_t N, int64_t d, int64_t V,
                                int64_t ignore_index, flce_reduction reduction, flce_dtype dt, float* loss_out,
                                float* lse_out, int32_t* status_out, int64_t* n_valid_out, void* hip_stream) {
  // The plan without the pre-tiled copy of H (its size grows with N*d): what is left of the forward
  // workspace is the per-window partials and per-block sums, O(N) words.
  if (!H || !W || !targets || !loss_out || !lse_out) return FLCE_ERR_BAD_ARG;
  if (reduction != FLCE_REDUCE_MEAN && reduction != FLCE_REDUCE_SUM) return FLCE_ERR_BAD_ARG;
  if (dt != FLCE_DTYPE_BF16 && dt != FLCE_DTYPE_F32) return FLCE_ERR_BAD_ARG;
  flce::Plan p;
  if (!flce::make_plan(N, d, V, dt, p, /*allow_h_copy=*/false)) return FLCE_ERR_BAD_SHAPE;
  if ((size_t)p.fwd_bytes > flce::STATIC_SCRATCH_BYTES) return FLCE_ERR_WORKSPACE;
  void* ws = nullptr;
  if (flce::static_scratch(&ws) != hipSuccess) return FLCE_ERR_HIP;
  const flce_status st = forward_impl(H, W, targets, N, d, V, ignore_index, reduction, dt, loss_out, lse_out, ws,
                                      flce::STATIC_SCRATCH_BYTES, hip_stream, flce::Slice{V, 0}, nullptr, nullptr,
                                      nullptr, flce::PerRow{nullptr, nullptr, 0.f}, /*allow_h_copy=*/false);
  if (st != FLCE_OK) return st;
  if (status_out || n_valid_out) {
    flce::export_header_kernel<<<1, 64, 0, static_cast<hipStream_t>(hip_stream)>>>(
        static_cast<const flce::Header*>(ws), status_out, n_valid_out);
    if (hipGetLastError() != hipSuccess) return FLCE_ERR_HIP;
  }
  return FLCE_OK;
}

flce_status flce_forward_rows(const void* H, const void* W, const int64_t* targets, int64_t N, int64_t d, int64_t V,
                              int64_t ignore_index, float label_smoothing, flce_dtype dt, float* loss_rows_out,
                              float* lse_out, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!loss_rows_out) return FLCE_ERR_BAD_ARG;
  return forward_impl(H, W, targets, N, d, V, ignore_index, FLCE_REDUCE_SUM, dt, nullptr, lse_out, workspace,
                      workspace_bytes, hip_stream, flce::Slice{V, 0}, nullptr, nullptr, nullptr,
                      flce::PerRow{loss_rows_out, nullptr, label_smoothing});
}

flce_status flce_backward_rows(const void* H, const void* W, const int64_t* targets, const float* lse,
                               const float* grad_rows, int64_t N, int64_t d, int64_t V, int64_t ignore_index,
                               float label_smoothing, flce_dtype dt, void* dH_out, void* dW_out, void* workspace,
                               size_t workspace_bytes, void* hip_stream) {
  if (!grad_rows) return FLCE_ERR_BAD_ARG;
  return backward_impl(H, W, targets, lse, N, d, V, ignore_index, FLCE_REDUCE_SUM, dt, 1.0f, dH_out, dW_out,
                       workspace, workspace_bytes, hip_stream, flce::Slice{V, 0},
                       flce::PerRow{nullptr, grad_rows, label_smoothing});
}

flce_status flce_forward_partial(const void* H, const void* W_slice, const int64_t* targets, int64_t N, int64_t d,
                                 int64_t V_slice, int64_t v_begin, int64_t V_total, int64_t ignore_index,
                                 flce_dtype dt, float* m_out, float* a_out, float* zt_out, void* workspace,
                                 size_t workspace_bytes, void* hip_stream) {
  if (!m_out || !a_out || !zt_out) return FLCE_ERR_BAD_ARG;
  return forward_impl(H, W_slice, targets, N, d, V_slice, ignore_index, FLCE_REDUCE_SUM, dt, nullptr, nullptr,
                      workspace, workspace_bytes, hip_stream, flce::Slice{V_total, v_begin}, m_out, a_out, zt_out);
}

size_t flce_merge_workspace_bytes(int64_t N) {
  if (N <= 0 || N > 0x7FFFFF00ll) return 0;
  const int64_t n_rb = flce::ceil_div(N, flce::TILE);
  return (size_t)(flce::ALIGN + 3 * flce::align_up(n_rb * 4, flce::ALIGN));
}

flce_status flce_merge_partials(const float* m_parts, const float* a_parts, const float* zt_parts, int n_parts,
                                const int64_t* targets, int64_t N, int64_t V_total, int64_t ignore_index,
                                flce_reduction reduction, float* loss_out, float* lse_out, void* workspace,
                                size_t workspace_bytes, void* hip_stream) {
  if (!m_parts || !a_parts || !zt_parts || !targets || !loss_out || !lse_out || n_parts < 1) return FLCE_ERR_BAD_ARG;
  if (reduction != FLCE_REDUCE_MEAN && reduction != FLCE_REDUCE_SUM) return FLCE_ERR_BAD_ARG;
  const size_t need = flce_merge_workspace_bytes(N);
  if (need == 0 || V_total <= 0) return FLCE_ERR_BAD_SHAPE;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < need)
    return FLCE_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  char* ws = static_cast<char*>(workspace);
  const int n_rb = (int)flce::ceil_div(N, flce::TILE);
  const int64_t blk = flce::align_up((int64_t)n_rb * 4, flce::ALIGN);
  flce::Header* hdr = reinterpret_cast<flce::Header*>(ws);
  float* blk_loss = reinterpret_cast<float*>(ws + flce::ALIGN);
  int* blk_cnt = reinterpret_cast<int*>(ws + flce::ALIGN + blk);
  int* blk_oor = reinterpret_cast<int*>(ws + flce::ALIGN + 2 * blk);
  flce::ProfScope ps(FLCE_PROF_FWD_EPILOGUE, st);
  flce::merge_rows_kernel<<<n_rb, 256, 0, st>>>(m_parts, a_parts, zt_parts, n_parts, N, targets, (int)N, V_total,
                                                ignore_index, lse_out, blk_loss, blk_cnt, blk_oor, nullptr, nullptr,
                                                0.f);
  flce::finalize_loss_kernel<<<1, 256, 0, st>>>(blk_loss, blk_cnt, blk_oor, n_rb, reduction == FLCE_REDUCE_MEAN, hdr,
                                                loss_out);
  return hipGetLastError() == hipSuccess ? FLCE_OK : FLCE_ERR_HIP;
}

flce_status flce_backward_partial(const void* H, const void* W_slice, const int64_t* targets, const float* lse,
                                  int64_t N, int64_t d, int64_t V_slice, int64_t v_begin, int64_t V_total,
                                  int64_t ignore_index, flce_reduction reduction, flce_dtype dt, float grad_loss,
                                  void* dH_partial_out, void* dW_slice_out, void* workspace,
                                  size_t workspace_bytes, void* hip_stream) {
  return backward_impl(H, W_slice, targets, lse, N, d, V_slice, ignore_index, reduction, dt, grad_loss,
                       dH_partial_out, dW_slice_out, workspace, workspace_bytes, hip_stream,
                       flce::Slice{V_total, v_begin});
}

flce_status flce_forward_with_grads(const void* H, const void* W, const int64_t* targets, int64_t N, int64_t d,
                                    int64_t V, int64_t ignore_index, flce_reduction reduction, flce_dtype dt,
                                    float* loss_out, float* lse_out, void* dH_partial, void* dW_partial,
                                    void* workspace, size_t workspace_bytes, void* hip_stream) {
  // Alg. 3 = Alg. 1 followed by the gradient sweep with the upstream gradient left out: the forward,
  // then the backward with Gamma = 1 (sum semantics, grad_loss 1), on the same stream and workspace.
  flce::Plan p;
  if (!flce::make_plan(N, d, V, dt, p)) return FLCE_ERR_BAD_SHAPE;
  if (workspace_bytes < (size_t)std::max(p.fwd_bytes, p.bwd_bytes)) return FLCE_ERR_WORKSPACE;
  if (!dH_partial || !dW_partial) return FLCE_ERR_BAD_ARG;
  const flce_status st = flce_forward(H, W, targets, N, d, V, ignore_index, reduction, dt, loss_out, lse_out,
                                      workspace, workspace_bytes, hip_stream);
  if (st != FLCE_OK) return st;
  return flce_backward(H, W, targets, lse_out, N, d, V, ignore_index, FLCE_REDUCE_SUM, dt, 1.0f, dH_partial,
                       dW_partial, workspace, workspace_bytes, hip_stream);
}

flce_status flce_scale(const void* dH_partial, const void* dW_partial, int64_t N, int64_t d, int64_t V,
                       flce_reduction reduction, flce_dtype dt, float grad_loss, const void* workspace,
                       void* dH_out, void* dW_out, void* hip_stream) {
  if (!dH_partial || !dW_partial || !dH_out || !dW_out || !workspace) return FLCE_ERR_BAD_ARG;
  if (reduction != FLCE_REDUCE_MEAN && reduction != FLCE_REDUCE_SUM) return FLCE_ERR_BAD_ARG;
  flce::Plan p;
  if (!flce::make_plan(N, d, V, dt, p)) return FLCE_ERR_BAD_SHAPE;
  if (!flce::aligned16(dH_partial) || !flce::aligned16(dW_partial) || !flce::aligned16(dH_out) ||
      !flce::aligned16(dW_out))
    return FLCE_ERR_BAD_ARG;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const flce::Header* hdr = static_cast<const flce::Header*>(workspace);
  const int mean = reduction == FLCE_REDUCE_MEAN;
  auto run = [&](auto tag) {
    using T = decltype(tag);
    flce::ProfScope ps(FLCE_PROF_SCALE, st);
    const int64_t nh = N * d / 4, nw = V * d / 4;
    const unsigned gh = (unsigned)std::min<int64_t>(flce::ceil_div(nh, 256), 16384);
    const unsigned gw = (unsigned)std::min<int64_t>(flce::ceil_div(nw, 256), 16384);
    flce::scale_kernel<T><<<gh, 256, 0, st>>>(static_cast<const T*>(dH_partial), static_cast<T*>(dH_out), nh, hdr,
                                              grad_loss, mean);
    flce::scale_kernel<T><<<gw, 256, 0, st>>>(static_cast<const T*>(dW_partial), static_cast<T*>(dW_out), nw, hdr,
                                              grad_loss, mean);
  };
  if (dt == FLCE_DTYPE_BF16) run(flce::bf16_t{});
  else run(float{});
  return hipGetLastError() == hipSuccess ? FLCE_OK : FLCE_ERR_HIP;
}

flce_status flce_last_device_status(const void* workspace, void* hip_stream, int64_t* n_valid_out) {
  if (!workspace) return FLCE_ERR_BAD_ARG;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  flce::Header h;
  if (hipStreamSynchronize(st) != hipSuccess) return FLCE_ERR_HIP;
  if (hipMemcpy(&h, workspace, sizeof(h), hipMemcpyDeviceToHost) != hipSuccess) return FLCE_ERR_HIP;
  if (n_valid_out) *n_valid_out = h.n_valid;
  return h.status == 0 ? FLCE_OK : FLCE_ERR_TARGET_RANGE;
}

flce_status flce_probe(int mode, const void* A, const void* B, const void* BT, int64_t a_rows, int64_t b_rows,
                       int64_t k_elems, int workgroups, int tiles_per_workgroup, float* sink, void* hip_stream) {
  if (!A || !B || !BT || !sink) return FLCE_ERR_BAD_ARG;
  if (mode < flce::PROBE_MFMA || mode > flce::PROBE_PAIR_PK_PK) return FLCE_ERR_BAD_ARG;
  if (a_rows <= 0 || b_rows <= 0 || (a_rows % flce::TILE) || (b_rows % flce::TILE) || k_elems < 32 || (k_elems % 32) ||
      workgroups <= 0 || tiles_per_workgroup <= 0)
    return FLCE_ERR_BAD_SHAPE;
  if (!flce::window_ok(257, k_elems * 2) || !flce::window_ok(k_elems, b_rows * 2)) return FLCE_ERR_BAD_SHAPE;
  if (!flce::aligned16(A) || !flce::aligned16(B) || !flce::aligned16(BT)) return FLCE_ERR_BAD_ARG;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const flce::ProbeArgs pa{static_cast<const flce::bf16_t*>(A), static_cast<const flce::bf16_t*>(B),
                           static_cast<const flce::bf16_t*>(BT), (int)a_rows, (int)b_rows, (int)k_elems,
                           tiles_per_workgroup, sink};
  auto launch = [&](auto kernel, int lds_bytes = flce::fast::LDS_BYTES) -> flce_status {
    if (flce::allow_big_lds(kernel, lds_bytes) != hipSuccess) return FLCE_ERR_HIP;
    kernel<<<workgroups, flce::fast::THREADS, lds_bytes, st>>>(pa);
    return hipGetLastError() == hipSuccess ? FLCE_OK : FLCE_ERR_HIP;
  };
  switch (mode) {
    case flce::PROBE_MFMA: return launch(flce::probe_kernel<flce::PROBE_MFMA>);
    case flce::PROBE_LOOP_KR: return launch(flce::probe_kernel<flce::PROBE_LOOP_KR>);
    case flce::PROBE_LOOP_KC: return launch(flce::probe_kernel<flce::PROBE_LOOP_KC>);
    case flce::PROBE_DATA_KR: return launch(flce::probe_kernel<flce::PROBE_DATA_KR>);
    case flce::PROBE_DATA_KC: return launch(flce::probe_kernel<flce::PROBE_DATA_KC>);
    case flce::PROBE_FREE_RUN: return launch(flce::probe_kernel<flce::PROBE_FREE_RUN>);
    case flce::PROBE_LOOP_KR_SOFTMAX: return launch(flce::probe_kernel<flce::PROBE_LOOP_KR_SOFTMAX>);
    case flce::PROBE_HALF_KR: return launch(flce::probe_half_kernel<false>, flce::PROBE_HALF_LDS);
    case flce::PROBE_HALF_KR_SOFTMAX: return launch(flce::probe_half_kernel<true>, flce::PROBE_HALF_LDS);
    case flce::PROBE_LOOP_KR_COLD: return launch(flce::probe_kernel<flce::PROBE_LOOP_KR_COLD>);
    case flce::PROBE_MFMA_16X16: return launch(flce::probe_mfma16_kernel<0>);
    case flce::PROBE_LOOP_PK: return launch(flce::probe_kernel<flce::PROBE_LOOP_PK>);
    case flce::PROBE_PAIR_KR_KR: return launch(flce::probe_pair_kernel<flce::fast::KR, flce::fast::KR>);
    case flce::PROBE_PAIR_PK_KR: return launch(flce::probe_pair_kernel<flce::fast::PK, flce::fast::KR>);
    case flce::PROBE_PAIR_KR_KC: return launch(flce::probe_pair_kernel<flce::fast::KR, flce::fast::KC>);
    case flce::PROBE_PAIR_KR_PK: return launch(flce::probe_pair_kernel<flce::fast::KR, flce::fast::PK>);
    case flce::PROBE_PAIR_PK_PK: return launch(flce::probe_pair_kernel<flce::fast::PK, flce::fast::PK>);
  }
  return FLCE_ERR_BAD_ARG;
}

flce_status flce_profile_enable(int on) {
  std::lock_guard<std::mutex> lk(flce::g_prof.mu);
  for (auto& r : flce::g_prof.recs) { flce::g_prof.pool.push_back(r.a); flce::g_prof.pool.push_back(r.b); }
  flce::g_prof.recs.clear();
  flce::g_prof.on = on != 0;
  return FLCE_OK;
}

flce_status flce_profile_collect(double* ms_by_class, int64_t* launches_by_class) {
  std::lock_guard<std::mutex> lk(flce::g_prof.mu);
  flce_status rc = FLCE_OK;
  for (auto& r : flce::g_prof.recs) {
    float ms = 0.f;
    if (hipEventSynchronize(r.b) != hipSuccess || hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) rc = FLCE_ERR_HIP;
    if (r.cls >= 0 && r.cls < FLCE_PROF_CLASSES) {
      if (ms_by_class) ms_by_class[r.cls] += (double)ms;
      if (launches_by_class) launches_by_class[r.cls] += 1;
    }
    flce::g_prof.pool.push_back(r.a);
    flce::g_prof.pool.push_back(r.b);
  }
  flce::g_prof.recs.clear();
  return rc;
}

}  // extern "C"
