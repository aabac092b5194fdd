/*
 * flce - fused lm_head projection + cross-entropy loss for AMD MI355X (gfx950).
 *
 * C ABI.  Computes, from hidden states H[N,d], vocabulary weights W[V,d] and
 * integer targets y[N], the cross-entropy loss of the logits Z = H.W^T and its
 * gradients dH, dW, without ever storing the N x V logits (the paper's
 * Section 3.2: the direct loss of Eq. 3, the streaming forward of Alg. 1, the
 * recompute backward of Alg. 2 / Eq. 4 / Eq. 5, and the window strategy with
 * its merging epilogue of Section 3.2.1).  Further entry points cover the
 * partial-gradient variant (Alg. 3 / Alg. 4), a per-row loss with per-row
 * upstream gradients and label smoothing, and vocabulary-sliced calls for
 * tensor / sequence parallel layouts.
 *
 * Conventions common to every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller, row-major and
 *     contiguous: H[N][d], W[V][d], dH[N][d], dW[V][d]; 16-byte aligned.
 *   - Element type of H, W, dH, dW is `dt`: bf16 (2 bytes) or fp32.  Logits,
 *     softmax statistics and all accumulations are fp32; loss and lse are fp32.
 *   - targets are int64, 0-based, in [0, V).  A row whose target equals
 *     `ignore_index` (any int64 value; compared first) does not count: its loss
 *     is 0, its dH row is all +0, it adds nothing to dW and it is left out of
 *     the mean's denominator.  A counted target outside [0, V) is an input
 *     error: the row is treated as ignored and FLCE_ERR_TARGET_RANGE is latched
 *     in the workspace (read it with flce_last_device_status).
 *   - The library never allocates device memory.  Scratch comes from the
 *     caller's `workspace` (size from flce_workspace_bytes; 256-byte aligned).
 *     The forward's is O(N + d) words plus one pre-tiled copy of H; the
 *     backward's is copies of H, fp32 running sums of the outputs where a
 *     launch is chunked, and ONE staging tile for G of a capped size (see
 *     flce_workspace_bytes): a problem smaller than the cap stages its whole
 *     G there (in the storage type, half the bytes of fp32 logits for bf16),
 *     a larger one never more than the cap.  The workspace contents are
 *     undefined on entry and between calls; forward and backward may use
 *     the same buffer.
 *   - All work is enqueued on `hip_stream` (a hipStream_t, NULL = the default
 *     stream) and the calls return without synchronising.  Outputs are fully
 *     overwritten.  Results are bit-identical from run to run for the same
 *     inputs, shapes and tuning environment: no floating-point atomics, every
 *     sum has a fixed order.  Only kernels are enqueued (no allocation, memset or
 *     synchronisation), so a sequence of calls can be captured into a HIP graph.
 *   - Host-detectable errors (null pointer, non-positive size, d not a multiple
 *     of 8, workspace too small, unknown enum) return a status and launch
 *     nothing.  A failing HIP runtime call returns FLCE_ERR_HIP.  Nothing is
 *     printed, nothing throws.
 *   - All state of a computation lives in the caller's workspace; concurrent calls must use
 *     distinct workspaces.  Process-wide state is limited to: the tuning knobs below (read once),
 *     a per-device "kernel attributes set" flag, and the optional launch profiler
 *     (flce_profile_*); all three are guarded by mutexes.
 *   - n_valid == 0 gives loss 0 and zero gradients (both reductions).
 *
 * Tuning environment.  Read ONCE per process, by the first call that needs a launch plan
 * (flce_workspace_bytes included), and fixed from then on, so the plan a workspace was sized
 * for is the plan that runs; flce_tuning_reload() reads it again (tests use it; do not call it
 * between sizing a workspace and using it, or while another thread is inside the library).
 * Defaults suit MI355X; results stay within the tolerances for any setting but their
 * rounding, and the bit pattern, depend on it:
 *   FLCE_WINDOWS    vocabulary windows of the forward (Section 3.2.1); 0 / unset = automatic
 *                   (at least 4, enough row block x window workgroups to cover 256 CUs).
 *   FLCE_VC_TILES   largest vocabulary chunk of the backward, in 256-row tiles; 0 / unset = automatic
 *                   (128; up to 512 when there are fewer than 32 token tiles, same staging bytes).
 *   FLCE_NC_TILES   largest token chunk of the backward, in 256-row tiles (default 128).
 *                   The staging buffer for G holds one chunk pair: at most VC x NC tiles.
 *   FLCE_SPLITK_DH, FLCE_SPLITK_DW
 *                   K slices of the dH / dW contraction launches; 0 / unset = automatic
 *                   (split only when a launch has too few output tiles for the CUs).
 *   FLCE_GENERIC    1 = use the generic main loop also where the tuned bf16 loop applies.
 */
#ifndef FLCE_H_
#define FLCE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  FLCE_OK = 0,
  FLCE_ERR_BAD_ARG = 1,      /* null pointer, unknown enum value */
  FLCE_ERR_BAD_SHAPE = 2,    /* N, d or V <= 0, d % 8 != 0, sizes beyond 2^31-1 rows */
  FLCE_ERR_WORKSPACE = 3,    /* workspace null, misaligned or smaller than required */
  FLCE_ERR_TARGET_RANGE = 4, /* a counted target was outside [0, V) (device-detected) */
  FLCE_ERR_UNSUPPORTED = 5,  /* reserved */
  FLCE_ERR_HIP = 6           /* a HIP runtime call failed */
} flce_status;

typedef enum { FLCE_DTYPE_BF16 = 0, FLCE_DTYPE_F32 = 1 } flce_dtype;

/* mean: divide by the number of counted rows (Eq. 2 / Alg. 1's last step, with
 * B*T replaced by n_valid); sum: no division. */
typedef enum { FLCE_REDUCE_MEAN = 0, FLCE_REDUCE_SUM = 1 } flce_reduction;

/* Library version, "major.minor.patch". Host call. */
const char* flce_version(void);

/* Reads the FLCE_* tuning variables again (see the top of this file). Host call. */
void flce_tuning_reload(void);

/* Static, human-readable name of a status code. Host call. */
const char* flce_status_string(flce_status s);

/*
 * Bytes of device workspace needed by flce_forward (for_backward == 0) or
 * flce_backward (for_backward != 0) at this shape.  Returns 0 for an invalid
 * shape or dtype.  Host call, touches no device.
 *   forward : 12 * windows * Npad + 4 * ceil(V/1024) * d + 4 * N + O(N/256) bytes, plus Npad * d elements (and 17 KiB
 *             per 256 rows) for the pre-tiled copy of H that the tuned bf16 loop reads.  Npad = N rounded up to 256.
 *   backward: 2 * Npad * d elements (the counted rows of H packed together, in two copies: pre-tiled for the two
 *             kernels that read them, or plain and transposed with the generic loop; d rounded up to 256 in one) + 16 * Npad bytes
 *             + the staging tile for G: Nc x (Vc + 64) elements with Nc = min(Npad, 32768) and
 *               Vc = min(Vpad, 256 * vc) where vc = 128 tiles, or up to 512 when Nc < 8192 rows (so that
 *               Nc * Vc stays within 2^25 elements there): at most 2 GiB + 4 MiB in bf16 whatever N and V,
 *               512 MiB at N = 8192; below the cap this IS Npad x Vpad, the whole G in the storage type;
 *             + fp32 running sums N * d (more than one vocabulary chunk) and Vc * d (more than one row chunk)
 *             + fp32 K-slice tiles when a contraction launch is split (small N or small d), or when the output-row
 *               tiles of its last, mostly empty round are launched on their own with K in slices (at most 64 MiB);
 *             the generic loop (fp32, or bf16 with d % 32 != 0) adds transposed copies of a W chunk and of G.
 *   Beyond the cap the size grows like c1 * (N + V) * d + c2 * N + c3: no N * V term.  flce_plan_describe
 *   prints the staging bytes of a shape.
 */
size_t flce_workspace_bytes(int64_t N, int64_t d, int64_t V, flce_dtype dt, int for_backward);

/*
 * Writes a one-line description of the launch plan at this shape (library version, main loop, windows,
 * chunk counts x largest chunk in 256-row tiles, K slices, K-split tails of a full chunk's dH / dW launch as
 * output-row tiles x slices, staging and workspace bytes) into `buf`; returns
 * the length it needs (as snprintf) or -1 for an invalid shape.  Reports and profile summaries carry it, so
 * that a measurement can be matched to the plan it was taken on.  Host call.
 */
int flce_plan_describe(int64_t N, int64_t d, int64_t V, flce_dtype dt, char* buf, size_t buf_bytes);

/*
 * Forward (Alg. 1 over tiles, Section 3.2.1 windows + merging epilogue).
 *   H, W, targets : device, read-only.
 *   loss_out      : device, 1 float.  mean or sum of (lse_i - z_{i,y_i}) over counted rows.
 *   lse_out       : device, N floats. lse_i = log sum_v exp(Z_iv) for EVERY row,
 *                   ignored ones included (this is m + ln a of Alg. 1; it is what
 *                   flce_backward takes back in place of the pair (m, a)).
 * Returns FLCE_OK once the work is enqueued.
 */
flce_status flce_forward(const void* H, const void* W, const int64_t* targets,
                         int64_t N, int64_t d, int64_t V, int64_t ignore_index,
                         flce_reduction reduction, flce_dtype dt,
                         float* loss_out, float* lse_out,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Backward (Alg. 2: logits recomputed tile by tile, G = p - onehot formed from
 * the saved lse, then Eq. 4 dH = G.W and Eq. 5 dW = G^T.H as MFMA contractions).
 *   lse        : device, N floats, as written by flce_forward for the same inputs.
 *   grad_loss  : upstream gradient of the scalar loss (host value).  Every
 *                counted row gets Gamma = grad_loss / n_valid (mean) or grad_loss (sum).
 *   dH_out     : device, N*d elements of type dt.
 *   dW_out     : device, V*d elements of type dt.
 * G is rounded to `dt` before the two contractions (unscaled, |G| <= 1); Gamma
 * is applied in fp32 when the fp32 sums are written out.
 */
flce_status flce_backward(const void* H, const void* W, const int64_t* targets, const float* lse,
                          int64_t N, int64_t d, int64_t V, int64_t ignore_index,
                          flce_reduction reduction, flce_dtype dt, float grad_loss,
                          void* dH_out, void* dW_out,
                          void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * flce_forward for callers that cannot allocate device memory or pass a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc).  Same computation and outputs as
 * flce_forward; the scratch (per-window softmax partials, per-block sums, status header) lives in a device
 * array inside the library, FLCE_STATIC_SCRATCH_BYTES large, that each GPU holds from the moment the library
 * is loaded on it until the process ends.  The call allocates nothing and frees nothing: it looks up the
 * array's address once per device, then only launches kernels on `hip_stream`.
 *   Limit    : shapes whose forward scratch exceeds the array return FLCE_ERR_WORKSPACE and launch nothing.
 *              The scratch is 12 * windows * ceil(N/256)*256 + 4 * ceil(V/1024) * d + 4 * N bytes + ~2 KiB
 *              (windows = max(4, ceil(256 / ceil(N/256))) unless FLCE_WINDOWS says otherwise): N up to about
 *              250 000 rows at d = 4096, V = 128256.  H is read in place (flce_forward's pre-tiled copy of
 *              H is what does not fit a fixed array), which costs up to a tenth of the forward's speed.
 *   status_out, n_valid_out : device, one int32 / one int64, either may be NULL: the range flag (0 or
 *              FLCE_ERR_TARGET_RANGE) and the number of counted rows of THIS call, written on the stream
 *              (flce_last_device_status cannot be pointed at the internal array).
 *   Sharing  : every call on a GPU uses that GPU's one array.  Nothing in it needs to start at zero (each
 *              call overwrites what it reads), so calls in sequence on one stream, or ordered by events, are
 *              fine whatever their shapes; calls that OVERLAP on one GPU (two streams, two threads) race on
 *              it and give undefined results.
 */
#define FLCE_STATIC_SCRATCH_BYTES (16u << 20)
flce_status flce_forward_static(const void* H, const void* W, const int64_t* targets,
                                int64_t N, int64_t d, int64_t V, int64_t ignore_index,
                                flce_reduction reduction, flce_dtype dt,
                                float* loss_out, float* lse_out,
                                int32_t* status_out, int64_t* n_valid_out, void* hip_stream);

/*
 * Forward with partial gradient accumulation (Alg. 3): the loss and lse of flce_forward
 * plus the gradients not yet scaled by the upstream gradient,
 *   dH_partial[i] = sum_v (P_iv - 1[v = y_i]) W_v,   dW_partial[v] = sum_i (P_iv - 1[v = y_i]) H_i,
 * over the counted rows (rows that do not count get a zero row of dH_partial and add nothing
 * to dW_partial).  Only meaningful when the upstream gradient is a scalar, i.e. for the mean
 * and sum reductions this library has (Section "Backward", remark before Alg. 3).
 *   dH_partial : device, N*d elements of type dt.   dW_partial : device, V*d elements of type dt.
 *   workspace  : device, at least max(flce_workspace_bytes(.., 0), flce_workspace_bytes(.., 1))
 *                bytes; its header afterwards holds n_valid for flce_scale.
 * The partial sums are rounded once to `dt` here and once more by flce_scale; flce_forward +
 * flce_backward round once (Gamma is applied to the fp32 sums) and are the cheaper pair on
 * this implementation: the second sweep of Alg. 3 recomputes the logits either way.
 */
flce_status flce_forward_with_grads(const void* H, const void* W, const int64_t* targets,
                                    int64_t N, int64_t d, int64_t V, int64_t ignore_index,
                                    flce_reduction reduction, flce_dtype dt,
                                    float* loss_out, float* lse_out,
                                    void* dH_partial, void* dW_partial,
                                    void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Backward scaling (Alg. 4, scalar branch): dH_out = Gamma * dH_partial, dW_out = Gamma * dW_partial
 * with Gamma = grad_loss / n_valid (mean; 0 when no row counts) or grad_loss (sum), n_valid read
 * on the device from the header of the workspace flce_forward_with_grads used.
 *   grad_loss : upstream gradient of the scalar loss (host value).
 *   dH_out, dW_out : device; may be the partial buffers themselves (in place).
 * Elementwise: reads and writes each element once.
 */
flce_status flce_scale(const void* dH_partial, const void* dW_partial,
                       int64_t N, int64_t d, int64_t V,
                       flce_reduction reduction, flce_dtype dt, float grad_loss,
                       const void* workspace, void* dH_out, void* dW_out, void* hip_stream);

/*
 * Per-row variant (no reduction): one loss per row out of the forward, one upstream gradient per row
 * into the backward (Alg. 2's Gamma given per position), optionally with label smoothing (the loss
 * variant the Discussion names; reading taken: target distribution (1 - eps) onehot + eps / V, so
 *   loss_i = (1 - eps) (lse_i - Z_{i,y_i}) + eps (lse_i - mean_v Z_iv),   dloss_i/dZ_iv = P_iv - q_v).
 *   label_smoothing : eps in [0, 1); 0 gives the plain loss.
 *   loss_rows_out   : device, N floats; 0 for rows that do not count.   lse_out as in flce_forward.
 *   grad_rows       : device, N floats, d(total)/d(loss_i); ignored for rows that do not count.
 *   dH_out = sum_v G_iv W_v, dW_out = sum_i G_iv H_i with G_iv = grad_rows[i] * (P_iv - q_v), G rounded to
 *   `dt` after the scaling (the gradient differs per row, so it cannot wait for the output flush).
 * mean_v Z_iv is computed as H_i . (sum_v W_v) / V (one pass over W, fixed summation order).
 * Workspaces as for flce_forward / flce_backward; the header reports n_valid and the range flag.
 */
flce_status flce_forward_rows(const void* H, const void* W, const int64_t* targets,
                              int64_t N, int64_t d, int64_t V, int64_t ignore_index,
                              float label_smoothing, flce_dtype dt,
                              float* loss_rows_out, float* lse_out,
                              void* workspace, size_t workspace_bytes, void* hip_stream);
flce_status flce_backward_rows(const void* H, const void* W, const int64_t* targets, const float* lse,
                               const float* grad_rows,
                               int64_t N, int64_t d, int64_t V, int64_t ignore_index,
                               float label_smoothing, flce_dtype dt,
                               void* dH_out, void* dW_out,
                               void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Vocabulary-sliced calls (Section "Model Parallelism", tensor parallelism: the outer loop restricted to
 * the local weight slice, partial results aggregated afterwards).  A slice is the V_slice vocabulary
 * rows [v_begin, v_begin + V_slice) of V_total, given as W_slice[V_slice][d]; targets stay global ids.
 * One GPU can run the slices one after another; across GPUs the (m, a, z_target) arrays and the partial
 * dH are what the ranks exchange (this library does not communicate).
 *
 * flce_forward_partial: per row i, over the slice only,
 *     m_out[i] = max_v Z_iv,  a_out[i] = sum_v exp(Z_iv - m_out[i]),
 *     zt_out[i] = Z_{i,y_i} if y_i lies in the slice and the row counts, else 0.
 *   (Alg. 1's state after the slice's part of the vocabulary loop; N floats each, device.)
 *   workspace: flce_workspace_bytes(N, d, V_slice, dt, 0).  Writes no status header.
 *
 * flce_merge_partials: merges n_parts such triples in part order (part k of row i at index k*N + i of
 *   each array) into lse_out[N] and the mean or sum loss over the counted rows, exactly as the
 *   forward's own epilogue merges its windows (Section "Window-based Strategy").  Counted = target
 *   not ignore_index and inside [0, V_total); the workspace (flce_merge_workspace_bytes(N) bytes,
 *   256-byte aligned) receives the status header read by flce_last_device_status.
 *
 * flce_backward_partial: Alg. 2 restricted to the slice, with the GLOBAL lse:
 *     dW_slice_out[V_slice][d] = the rows [v_begin, v_begin + V_slice) of dW, complete;
 *     dH_partial_out[N][d]     = sum over the slice's v of G_iv W_v; dH is the sum of these over all slices
 *                                (rounded to dt per slice; rows that do not count are +0).
 *   Gamma = grad_loss / n_valid (mean) or grad_loss (sum), n_valid counted over all rows as above.
 *   workspace: flce_workspace_bytes(N, d, V_slice, dt, 1).
 * Errors as for flce_forward / flce_backward; FLCE_ERR_BAD_SHAPE also when the slice is not inside [0, V_total).
 */
flce_status flce_forward_partial(const void* H, const void* W_slice, const int64_t* targets,
                                 int64_t N, int64_t d, int64_t V_slice, int64_t v_begin, int64_t V_total,
                                 int64_t ignore_index, flce_dtype dt,
                                 float* m_out, float* a_out, float* zt_out,
                                 void* workspace, size_t workspace_bytes, void* hip_stream);
size_t flce_merge_workspace_bytes(int64_t N);
flce_status flce_merge_partials(const float* m_parts, const float* a_parts, const float* zt_parts, int n_parts,
                                const int64_t* targets, int64_t N, int64_t V_total, int64_t ignore_index,
                                flce_reduction reduction, float* loss_out, float* lse_out,
                                void* workspace, size_t workspace_bytes, void* hip_stream);
flce_status flce_backward_partial(const void* H, const void* W_slice, const int64_t* targets, const float* lse,
                                  int64_t N, int64_t d, int64_t V_slice, int64_t v_begin, int64_t V_total,
                                  int64_t ignore_index, flce_reduction reduction, flce_dtype dt, float grad_loss,
                                  void* dH_partial_out, void* dW_slice_out,
                                  void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Synchronises `hip_stream`, then reports what the last flce_forward or
 * flce_backward that used `workspace` latched on the device: FLCE_OK or
 * FLCE_ERR_TARGET_RANGE (FLCE_ERR_HIP if the synchronisation or copy fails).
 * If n_valid_out is not NULL it receives the number of counted rows (host).
 */
flce_status flce_last_device_status(const void* workspace, void* hip_stream, int64_t* n_valid_out);

/*
 * Measurement aid (not part of the computation; the paper's evaluation, Section 4,
 * reports end-to-end latency only).  While enabled, every kernel launch of
 * flce_forward / flce_backward is bracketed by a pair of HIP events recorded on the
 * caller's stream, grouped into the classes below.  Process-wide, off by default,
 * not meant to be toggled while another thread is inside the library.
 *   flce_profile_enable(on) : on != 0 starts a fresh recording, 0 stops and discards.
 *   flce_profile_collect    : waits for the recorded events, adds the elapsed
 *                             milliseconds and launch counts per class into the two
 *                             host arrays of FLCE_PROF_CLASSES entries (either may be
 *                             NULL), then clears the recording (profiling stays on).
 */
enum {
  FLCE_PROF_FWD_TILES = 0,   /* forward logit tiles + online softmax */
  FLCE_PROF_FWD_EPILOGUE = 1,/* window merge, per-row loss, scalar reduction */
  FLCE_PROF_BWD_PREP = 2,    /* target scan and K-contiguous operand copies */
  FLCE_PROF_RECOMPUTE = 3,   /* backward logit recompute + G */
  FLCE_PROF_CONTRACT_DW = 4, /* dW = G^T.H */
  FLCE_PROF_CONTRACT_DH = 5, /* dH = G.W */
  FLCE_PROF_SCALE = 6,       /* Alg. 4 scaling pass */
  FLCE_PROF_CLASSES = 7
};
flce_status flce_profile_enable(int on);
flce_status flce_profile_collect(double* ms_by_class, int64_t* launches_by_class);

/*
 * Second measurement aid (not part of the computation): runs a piece of the tuned bf16 main loop on its own, so
 * that a kernel's rate can be compared with what the matrix pipe and the bare loop sustain on this chip, not
 * only with the nominal peak.  `workgroups` workgroups of 4 wavefronts each walk `tiles_per_workgroup` tiles
 * of 256 x 256 outputs over K = k_elems.
 *   mode 0 : the 32x32x16 bf16 MFMA back to back from registers (no memory traffic in the loop)
 *   mode 1 : the complete main loop, A K-contiguous and B read across memory rows (the contractions' layouts)
 *   mode 2 : the complete main loop, both operands K-contiguous
 *   mode 3, 4 : modes 1, 2 with the matrix instructions left out (global -> LDS requests, LDS reads, waits and
 *            barriers only): the data path alone
 *   mode 5 : mode 0's MFMAs and mode 1's requests and LDS reads issued side by side with no wait or barrier between
 *            them (what is read is discarded): the two streams when neither waits for the other
 *   mode 6 : mode 1 plus, after every tile, the plain-ALU work of the forward's tile post-processing (a maximum and
 *            a sum of exponentials over the accumulators), done by the same wavefronts, nothing overlapped
 *   mode 7, 8 : modes 1 and 6 on tiles of 128 x 256 outputs (128 accumulators per lane, three stages) so that two
 *            workgroups share a CU and one's post-processing overlaps the other's matrix work; a tile is half
 *            the work, so these modes execute half the flops stated below per workgroup
 *   mode 9 : mode 1 with every group of workgroups that shares an A tile walking a run of A tiles of its own, so
 *            that each A tile is read once per launch, from HBM (the forward's access to W); in the other modes a
 *            group reads what its neighbour read one tile earlier
 *   mode 10 : mode 0 with the 16x16x32 bf16 MFMA (64 blocks of 4 accumulators per wavefront instead of 16 of 16)
 *   mode 11 : the complete main loop, A K-contiguous and B pre-tiled, i.e. B's bytes taken as the 16 KiB LDS tile
 *            images of its K steps one after the other (the forward / recompute layout: W and the pre-tiled copy of H)
 *   mode 12 .. 16 : the complete main loop for the operand layout pairs (A / B) rows / rows (the dW contraction),
 *            pre-tiled / rows, rows / K-contiguous (the dH contraction), rows / pre-tiled, pre-tiled / pre-tiled;
 *            "rows" = read across memory rows.  Timing only: the operands' bytes are taken from the buffers as they are.
 *   A  : device, bf16 [a_rows][k_elems];  B : device, bf16 [b_rows][k_elems];  BT : device, bf16 [k_elems][b_rows]
 *        (a_rows, b_rows multiples of 256, k_elems a multiple of 32); contents are the caller's choice of data.
 *   sink : device, workgroups * 256 floats, written once per thread.
 * Every mode executes 2 * 256 * 256 * k_elems * tiles_per_workgroup * workgroups nominal flops (modes 3, 4 move
 * the bytes of as many tiles).  Enqueues one kernel on `hip_stream`; the caller times it.
 */
flce_status flce_probe(int mode, const void* A, const void* B, const void* BT,
                       int64_t a_rows, int64_t b_rows, int64_t k_elems,
                       int workgroups, int tiles_per_workgroup, float* sink, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* FLCE_H_ */
