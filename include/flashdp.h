/*
 * flashdp.h - C ABI of the MI355X (gfx950) per-layer DP weight-gradient library.
 *
 * One call computes, for a linear layer Y = X W^T with activations X[B][T][d_in] and
 * output gradients dY[B][T][d_out] (row-major, last index contiguous), the clipped and
 * noised weight gradient of per-layer DP-SGD:
 *
 *     G_i      = dY_i^T X_i                      per-sample gradient, [d_out][d_in]
 *     n_i      = ||G_i||_F                       per-sample, per-layer norm
 *     c_i      = 1 / max(1, n_i / C)             clip factor
 *     out_grad = sum_i c_i G_i + sigma * C * z   z ~ N(0, I), counter-based
 *
 * Paper: Algorithm 1 "FlashDP with Block-wise All-Reduce" (tile contraction, intra/inter
 * block norm reduction, synchronisation, clip, noise + batch aggregation, store) and
 * Appendix B.2 (the explicit four-stage flow it is equivalent to).  The batch is summed,
 * not averaged (Algorithm 1, aggregation step); the caller divides by B if it wants the
 * mean of Appendix A.1.
 *
 * Noise: the paper names no generator.  z is a stateless field
 *     z[e] = BoxMuller(Philox4x32-10(key = (seed & 0xffffffff, seed >> 32),
 *                                    counter = (g & 0xffffffff, g >> 32, layer, 0)))[e & 3],
 *     e = d * d_in + p,  g = e >> 2,
 * uniforms u(r) = ((r >> 8) + 0.5) * 2^-24, pairs (r0,r1) -> (z0,z1) = rho*(cos,sin)(2 pi u(r1)),
 * rho = sqrt(-2 ln u(r0)), and (r2,r3) -> (z2,z3) likewise.  Same (seed, layer) => same noise:
 * the caller must fold the training step into seed, or noise repeats across steps.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers (HIP, current device) owned by the caller.
 *     flashdp_layer_t arrays and scalar arguments are HOST memory.
 *   - Calls enqueue work on a HIP stream and return without synchronising it.  Device
 *     faults surface at the caller's next synchronisation.  With a caller-owned workspace a call
 *     only launches kernels (plus event records/waits between its two streams in the overlapped
 *     schedule), so it can be captured into a HIP graph once each kernel has been launched eagerly.
 *   - out_grad and out_norms are overwritten, never accumulated into.
 *   - Inputs are read-only.  X pointers of different layers may alias.
 *   - dtype: FLASHDP_BF16 / FLASHDP_F16 / FLASHDP_F32 is the storage type of X and dY; products are
 *     accumulated in fp32; out_grad and out_norms are fp32.
 *   - Pointers must be 16-byte aligned.  Any positive B, T, d_in, d_out is accepted; the
 *     matrix-core path needs d_in and d_out to be multiples of 8 (16-bit types), other shapes
 *     take a slower generic kernel.
 *   - NaN/Inf in the inputs propagate to out_norms / out_grad: a sample with a NaN norm gets a NaN clip
 *     factor and so turns the whole of out_grad into NaN (it is never let through unclipped).
 *     A per-sample gradient that overflows fp32 (infinite norm) poisons out_grad with NaN/Inf under every
 *     schedule.  TWOPASS and GHOST rescale the running sum by c_i / c_(i+1) at sample boundaries; two
 *     consecutive clip factors further apart than about 1e38 (a norm beyond 1e38 * C) overflow that ratio and
 *     give Inf/NaN as well, where SCRATCH / OVERLAP / EXPLICIT still give the finite result.
 *   - Return value: FLASHDP_OK (0) or a negative flashdp_status.  Argument errors (everything but
 *     FLASHDP_HIP_ERROR) are found before anything is enqueued; a FLASHDP_HIP_ERROR comes from the runtime
 *     while enqueuing, and kernels of earlier layers or stages of the same call may then already be enqueued:
 *     treat the outputs of that call as undefined.
 *
 * Environment overrides (measurement aids, not needed in normal use), read once per process at the first call;
 * with FLASHDP_DEBUG_ENV=1 set at that moment they are read again at every call:
 *   FLASHDP_SCHEDULE = twopass | scratch | overlap | explicit | ghost | fused   replaces the schedule argument;
 *   FLASHDP_TILE = 2 | 3 | 4 | 6 | 7 | 8 forces the matrix-core kernel (256x256 with 64-deep k-tiles, 128x128,
 *                                256x256 with 32-deep k-tiles - these three stage tiles through registers -,
 *                                256x256, 384x192, 192x384 with 32-deep k-tiles loaded straight into LDS);
 *                                -1 sends fp32 inputs to the generic kernel;
 *   FLASHDP_OVERLAP_GRID = n     workgroups of the aggregation kernel in the overlapped schedule (default: one per
 *                                compute unit).
 */
#ifndef FLASHDP_H
#define FLASHDP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum flashdp_status {
  FLASHDP_OK = 0,
  FLASHDP_INVALID_ARGUMENT = -1,   /* null pointer, dim <= 0, C <= 0 or not finite, sigma < 0 or not finite, bad enum */
  FLASHDP_MISALIGNED = -2,         /* a data pointer or the workspace is not 16-byte aligned */
  FLASHDP_UNSUPPORTED_SHAPE = -3,  /* a dimension or byte count exceeds what the kernels index (2^31 elements per sample tensor) */
  FLASHDP_WORKSPACE_TOO_SMALL = -4,
  FLASHDP_NO_DEVICE = -5,          /* no HIP device visible */
  FLASHDP_HIP_ERROR = -6           /* allocation or launch failure reported by the runtime */
} flashdp_status;

enum { FLASHDP_BF16 = 0, FLASHDP_F32 = 1, FLASHDP_F16 = 2 };

/* How the grid-wide dependency of Algorithm 1 (the clip factor needs every tile of G_i;
 * Section 4.2 "Adaptive Kernel Implementation") is resolved:
 *   TWOPASS  norm pass, then a second contraction that accumulates c_i G_i (each G_i computed twice;
 *            workspace: a few KB);
 *   SCRATCH  each G_i tile is computed once, its square-sum taken from the fp32 accumulators, the tile
 *            parked in a per-layer scratch (bfloat16 for both 16-bit input types - fp16's range could
 *            overflow on an unclipped gradient -, fp32 for fp32 inputs), and a
 *            streaming kernel forms sum_i c_i G_i + noise (workspace: B * d_out * d_in elements);
 *   EXPLICIT the explicit four-stage flow of Appendix B.2, one kernel per stage, the fp32 per-sample
 *            gradients written to and re-read from HBM between stages (workspace: 4 * B * d_out * d_in
 *            bytes).  Never chosen by AUTO: it exists to be measured against;
 *   OVERLAP  SCRATCH for a block of two or more layers with the streaming kernel of layer l running on a
 *            second, library-owned stream (default priority) beside the contraction of layer l+1
 *            (workspace: two scratch slots).  Same arithmetic, bit-identical results.  The caller's
 *            stream is made to wait for the side stream before the call's work counts as complete, so
 *            stream-order semantics are unchanged.  Falls back to SCRATCH for a single layer, fp32 inputs
 *            or small shapes;
 *   GHOST    the norms come from the ghost-clipping identity the paper cites among the implicit methods
 *            (Section 2): n_i^2 = <X_i X_i^T, dY_i dY_i^T>_F, two T x T Gram matrices per sample that are
 *            never stored, then the clipped accumulation of TWOPASS (workspace: a few KB to MB of partial
 *            sums).  Costs T^2 (d_in + d_out) extra FLOPs per sample instead of a second 2 T d_in d_out.
 *            Never chosen by AUTO: it exists to be measured against;
 *   FUSED    Algorithm 1 in one launch with its block-wise synchronisation as a barrier across the grid (the
 *            "ideal single-kernel solution" of Section 4.2): one workgroup owns one 256 x 256 output tile for all
 *            samples, parks all but the last sample's tile (bfloat16), meets the other workgroups at a barrier in
 *            memory once every squared-norm partial is written, and forms the clipped, noised sum of its tile from
 *            its own parked tiles and the accumulators it still holds.  For layers whose tiles all fit on the chip
 *            at once (d_out/256 * d_in/256 <= compute units, 16-bit inputs, B <= 16; e.g. 4096 x 4096); other
 *            layers of the call take SCRATCH.  Workspace: (B - 1) * d_out * d_in * 2 bytes + partials.  The barrier
 *            wait is bounded: if the workgroups are not co-resident (chip shared with long-running work) the call
 *            still terminates, after about two seconds, with out_grad all NaN and an error flag in the workspace.
 *   AUTO     OVERLAP when it applies and the workspace holds two slots, else SCRATCH when it holds one.  When a
 *            caller's workspace holds fewer parked samples than the batch has, AUTO goes through the batch in
 *            chunks of as many samples as fit (two slots of a smaller chunk where OVERLAP applies: chunk k's
 *            streaming kernel then runs beside chunk k+1's contraction), every chunk's clipped sum added to
 *            out_grad and the noise added with the last: memory bounded by the workspace whatever B is, each
 *            G_i still computed once (flashdp_workspace_bytes_chunked sizes such a workspace).  Only a
 *            workspace too small for a single sample falls back to TWOPASS.                              */
enum { FLASHDP_SCHEDULE_AUTO = 0, FLASHDP_SCHEDULE_TWOPASS = 1, FLASHDP_SCHEDULE_SCRATCH = 2, FLASHDP_SCHEDULE_EXPLICIT = 3,
       FLASHDP_SCHEDULE_OVERLAP = 4, FLASHDP_SCHEDULE_GHOST = 5, FLASHDP_SCHEDULE_FUSED = 6 };

/* One linear layer of a block (Appendix A.1, "Per-Layer Gradient Processing": every layer is clipped
 * by its own norm with its own C and sigma). */
typedef struct flashdp_layer {
  const void* X;      /* device, [B][T][d_in],  dtype */
  const void* dY;     /* device, [B][T][d_out], dtype */
  int64_t d_in;       /* P */
  int64_t d_out;      /* D */
  float C;            /* clipping threshold, > 0 */
  float sigma;        /* noise multiplier, >= 0; 0 adds no noise and generates none */
  uint64_t seed;      /* Philox key */
  uint32_t layer;     /* Philox counter word 2 */
  float* out_grad;    /* device, [d_out][d_in] fp32, overwritten */
  float* out_norms;   /* device, [B] fp32, pre-clip n_i, overwritten; may be NULL */
} flashdp_layer_t;

/* Algorithm 1 for one layer with the calling thread's context (stream, dtype, layer index, schedule,
 * workspace; see the setters below; defaults: null stream, bf16, layer 0, AUTO, library-owned workspace).
 * When no workspace has been set the library allocates one with hipMalloc on first use and keeps it
 * (grow-only, per device, grown by at least half at a time) until flashdp_release(); growing it synchronises
 * the device, frees and allocates: a caller that must not stall in a step sets a workspace of
 * flashdp_workspace_bytes() itself, or uses flashdp_linear_dp_grad_static. */
int flashdp_linear_dp_grad(const void* X, const void* dY, int64_t B, int64_t T, int64_t d_in, int64_t d_out,
                           float C, float sigma, uint64_t seed, float* out_grad, float* out_norms);

/* Per-block multi-layer variant: Algorithm 1 for each of n_layers layers (same B and T), enqueued in
 * order on `stream` (a hipStream_t, may be NULL).  `workspace` is caller-owned device memory of at least
 * flashdp_workspace_bytes(...) bytes, reused layer after layer; with workspace == NULL the library-owned
 * workspace is used as above (sized for the schedule asked for).  Calls that share a workspace must be
 * ordered on one stream; the library-owned workspace is one per device, so this holds for all calls on a
 * device that pass no workspace of their own, from whichever thread they come. */
int flashdp_block_dp_grad(const flashdp_layer_t* layers, int n_layers, int64_t B, int64_t T, int dtype,
                          int schedule, void* workspace, size_t workspace_bytes, void* stream);

/* Micro-batch form of flashdp_block_dp_grad for gradient accumulation (the paper's micro-batch experiment,
 * Appendix D.1: several micro-batches per optimizer step).  Per-sample clipping does not depend on how
 * the batch is split, so calling this once per micro-batch with
 *     accumulate = 0 on the first micro-batch (out_grad overwritten), 1 on the later ones (added to), and
 *     add_noise  = 1 on the last micro-batch only (sigma*C*z added once per accumulated batch)
 * gives the result of one flashdp_block_dp_grad call on the concatenated batch, up to fp32 summation
 * order.  out_norms receives the norms of this micro-batch's samples.  accumulate = 0, add_noise = 1 is
 * flashdp_block_dp_grad itself. */
int flashdp_block_dp_grad_micro(const flashdp_layer_t* layers, int n_layers, int64_t B, int64_t T, int dtype,
                                int schedule, void* workspace, size_t workspace_bytes, void* stream,
                                int accumulate, int add_noise);

/* For callers that cannot allocate device memory: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  flashdp_block_dp_grad for ONE layer under the SCRATCH schedule (same kernels, same
 * arithmetic, bit-identical results), with the schedule's workspace - clip factors, per-workgroup norm partials and
 * the parked per-sample tiles - kept in a fixed array of flashdp_static_scratch_bytes() (64 MiB) of device memory
 * that is part of the library's code object: each GPU the library runs on holds that array from the first use of
 * the library on it until the process ends.  The call allocates and frees nothing (no hipMalloc / hipFree, no
 * library-owned workspace, no side stream); the caller passes inputs and outputs as usual, dtype and layer as
 * arguments instead of thread context, and `stream` (a hipStream_t, may be NULL) to enqueue on.
 * Limit: flashdp_workspace_bytes(layer, 1, B, T, dtype, FLASHDP_SCHEDULE_SCRATCH) must not exceed
 * flashdp_static_scratch_bytes(), i.e. roughly B * d_out * d_in * (2 or, for fp32 inputs, 4) bytes <= 64 MiB
 * (the GPT-2 up-projection at B = 8 takes 36 MiB); larger problems return FLASHDP_WORKSPACE_TOO_SMALL with nothing
 * enqueued.  All calls on one GPU share that GPU's array: calls that can overlap in time on one GPU (different
 * streams, different threads) race on it and must be ordered by the caller.  The array keeps the last call's
 * contents; nothing in it needs clearing between calls, because a call reads only what it has itself written. */
int flashdp_linear_dp_grad_static(const void* X, const void* dY, int64_t B, int64_t T, int64_t d_in, int64_t d_out,
                                  int dtype, float C, float sigma, uint64_t seed, uint32_t layer, float* out_grad,
                                  float* out_norms, void* stream);
size_t flashdp_static_scratch_bytes(void);

/* Bytes of workspace the given schedule needs for these layers (the maximum over layers).  Returns 0 on
 * invalid arguments. */
size_t flashdp_workspace_bytes(const flashdp_layer_t* layers, int n_layers, int64_t B, int64_t T, int dtype,
                               int schedule);

/* Bytes of workspace with which AUTO parks chunk_samples (1..B) samples at a time, in one slot (slots = 1,
 * scratch schedule over chunks) or two (slots = 2, overlapped schedule over chunks).  With the 16-bit types that is
 * about slots * chunk_samples * d_out * d_in * 2 bytes for the largest layer: slots = 2, chunk_samples = 1 costs as
 * much memory as out_grad itself (4 * d_out * d_in bytes), independent of B.  Returns 0 on invalid arguments. */
size_t flashdp_workspace_bytes_chunked(const flashdp_layer_t* layers, int n_layers, int64_t B, int64_t T, int dtype,
                                       int64_t chunk_samples, int slots);

/* Number of samples the last block call on this thread parked at a time (B when the batch was not chunked). */
int64_t flashdp_last_chunk(void);

/* Non-private weight gradient out_grad = sum_i dY_i^T X_i (Appendix B.1, Eq. "batched-grad") computed by
 * the same contraction kernel with the norm, clip and noise steps switched off: the comparator the DP
 * path is timed against, and the C -> infinity, sigma = 0 special case. */
int flashdp_plain_grad(const void* X, const void* dY, int64_t B, int64_t T, int64_t d_in, int64_t d_out,
                       int dtype, float* out_grad, void* stream);

/* The same non-private gradient with the work balanced over the chip whatever the tile count: the output is cut into
 * blocks of 32 tiles of 256 x 256, the eight XCDs are each dealt an equal, contiguous share of (block, k-tile) units,
 * blocks at the edge of a share are cut along the reduction index (all samples' tokens, one sample after the other)
 * and their fp32 pieces added by a second kernel in a fixed order (bit-repeatable, no atomics).  This is the
 * comparator the DP path's ratio is quoted against: flashdp_plain_grad runs one workgroup per tile, and e.g. the 400
 * tiles of a 5120 x 5120 layer leave its second round of 256 workgroups half empty.
 * `workspace`: device memory of at least flashdp_plain_grad_balanced_workspace_bytes() (128 MiB, for the pieces of cut
 * tiles), or NULL to use the library-owned workspace (allocated on first use, shared with the DP entry points: order
 * such calls on one stream).  16-bit inputs with d_in and d_out multiples of 8; other problems are passed on to
 * flashdp_plain_grad. */
int flashdp_plain_grad_balanced(const void* X, const void* dY, int64_t B, int64_t T, int64_t d_in, int64_t d_out,
                                int dtype, float* out_grad, void* workspace, size_t workspace_bytes, void* stream);
size_t flashdp_plain_grad_balanced_workspace_bytes(void);

/* Fills z[0..n) (device, fp32) with the noise field of (seed, layer): the field that out_grad receives
 * scaled by sigma*C.  For checking the generator on its own. */
int flashdp_noise_field(uint64_t seed, uint32_t layer, int64_t n, float* z, void* stream);

/* z[4g + j] = j-th normal made from words[4g .. 4g+3] by the Box-Muller map above (device pointers,
 * n_groups groups of four 32-bit words).  For checking the uniform -> normal map at words a keyed field
 * reaches only by chance (extreme uniforms, quadrant boundaries). */
int flashdp_box_muller(const uint32_t* words, int64_t n_groups, float* z, void* stream);

/* Thread-local context used by flashdp_linear_dp_grad. */
int flashdp_set_stream(void* hip_stream);
int flashdp_set_workspace(void* device_ptr, size_t bytes);   /* NULL, 0: back to the library-owned one */
int flashdp_set_dtype(int dtype);
int flashdp_set_layer(uint32_t layer);
int flashdp_set_schedule(int schedule);

/* Measurement aid, not a step of the method: runs the matrix-core instruction mix of the contraction kernel's
 * inner loop (bf16, 32x32x16, eight accumulators per wave) on register-resident operands - no memory, no LDS,
 * no barrier - so that a benchmark can quote the rate this part actually sustains next to the nominal peak.
 * pattern 0 = all-zero operands, 1 = pseudo-random operands, both held in registers; 2 and 3 = the same two
 * with the operand fragments re-read from LDS every k-step through the contraction kernel's transposed reads
 * (matrix cores + LDS traffic, still no memory loads and no barrier); 4 = the random operands of 1 with consecutive
 * instructions of a wave sharing one operand fragment, 5 = with one and the same operand pair for every instruction,
 * 6 = random operands with eight different exponents instead of two (4-6: does the rate on random data depend on how
 * operands are delivered, or on the values themselves?); 7 = the random operands of 1 through the 16x16x32
 * instruction, two per 32x32x16 one (the same FLOPs), 8 = the same with the LDS fragment reads of 3, 9 = 16x16x32 on
 * zeros, 10 / 11 = 16x16x32 on random operands with the accumulators updated in place, in accumulation registers /
 * in ordinary vector registers, 12 = pattern 8 with a third fewer fragment reads (what 128 x 128 per wave would
 * save).  `workgroups` workgroups of 8 waves, each wave issuing 16 * iters instructions of
 * 32768 FLOP (32 * iters of 16384 for the 16x16x32 patterns); sink (device, 4 bytes) is never written in practice.
 * INVALID_ARGUMENT for other patterns, iters or workgroups <= 0 or absurdly large, or a null sink. */
int flashdp_mfma_probe(int pattern, int iters, int workgroups, float* sink, void* stream);

/* Measurement aid: one launch of the per-sample contraction kernel for large shapes (bf16, tiles loaded straight into
 * LDS; park = 0: norm only, 1: norm + the bfloat16 tile parked in the workspace) in an instantiation that also records,
 * per workgroup, where its time went.  trace[8 * w + k] (device, 64-bit words, zero them beforehand) for workgroup w:
 *   k = 0..4  constant-rate timestamps, 10 ns units: start; first k-tile landed; end of the main loop; stores issued;
 *             stores acknowledged
 *   k = 5     XCD id << 32 | hardware id register (CU: bits 8..15)
 *   k = 6     shader-clock cycles of the main loop (ceil(T / 32) k-tiles; 1024 per k-tile = matrix cores never idle)
 *   k = 7     1 if the workgroup had a work item (grid slots beyond the last item write nothing).
 * Returns the number of workgroups launched (trace_entries must be at least that: B * ceil(tiles / 32) * 32 rounded up
 * to a multiple of 256), or a negative status.  `workspace` as for the scratch schedule of this layer.  d_in, d_out
 * multiples of 8.  Results of the contraction itself are discarded. */
int64_t flashdp_contraction_timeline(const void* X, const void* dY, int64_t B, int64_t T, int64_t d_in, int64_t d_out,
                                     int park, void* workspace, size_t workspace_bytes, uint64_t* trace, int64_t trace_entries,
                                     void* stream);

/* Measurement aid: which stages of Algorithm 1 the following calls on this thread enqueue (default: all).
 * With a partial mask the outputs are not meaningful; the stages left out read whatever the workspace
 * holds from an earlier full call.  CONTRACT = per-sample contraction + intra-block norm (the dominant
 * kernel), CLIP = inter-block reduce and clip factors, AGGREGATE = clipped batch sum + noise. */
enum { FLASHDP_STAGE_CONTRACT = 1, FLASHDP_STAGE_CLIP = 2, FLASHDP_STAGE_AGGREGATE = 4, FLASHDP_STAGE_ALL = 7 };
int flashdp_set_stages(int mask);

/* Frees the library-owned workspaces, side streams and events (synchronises the device first). */
int flashdp_release(void);

/* Name of the schedule the last call on this thread used: "twopass", "scratch", "overlap", "explicit", "ghost" or "fused" ("none" before any). */
const char* flashdp_last_schedule(void);

/* Name of the contraction kernel the last layer enqueued on this thread took (the per-sample pass of Algorithm 1):
 * "gemm_mfma_dma_kernel" (16-bit inputs, tiles loaded straight into LDS), "gemm_mfma_kernel" (16-bit, register-staged,
 * small shapes), "gemm_mfma_f32_kernel" (fp32 inputs), "gemm_simple_kernel" (any shape); "none" before any call. */
const char* flashdp_last_kernel(void);

const char* flashdp_status_string(int status);
int flashdp_version(void);   /* major*10000 + minor*100 + patch */

#ifdef __cplusplus
}
#endif
#endif /* FLASHDP_H */
