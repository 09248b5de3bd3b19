/*
 * lstm.h -- C ABI of the MI355X (gfx950) stacked-LSTM library.
 *
 * The library computes the forward pass and full back-propagation through time
 * of the network that Section 2 of Appleyard, Kocisky & Blunsom, "Optimizing
 * Performance of Recurrent Neural Networks on GPUs" (arXiv 1604.01946) studies:
 * a standard four-gate LSTM without peepholes,
 *
 *     i_t = sigma(W_i x_t + R_i h_{t-1} + b_i)      f_t = sigma(W_f x_t + R_f h_{t-1} + b_f)
 *     o_t = sigma(W_o x_t + R_o h_{t-1} + b_o)      c'_t = tanh(W_c x_t + R_c h_{t-1} + b_c)
 *     c_t = f_t o c_{t-1} + i_t o c'_t              h_t = o_t o tanh(c_t)
 *
 * stacked as Section 2.4 describes (layer l at step t reads h of layer l-1 at
 * step t).  The two subscript misprints of the printed equations are read the
 * standard way (x_t in the first line, previous cell state c_{t-1} in the fifth).
 *
 * Conventions common to every call
 *   - all tensors are fp32, contiguous, row-major (last index fastest);
 *   - every pointer is a DEVICE pointer owned by the caller and 16-byte aligned;
 *     the library never allocates or frees device memory in lstm_forward /
 *     lstm_backward (helper streams and events are created on first use and
 *     released by lstm_shutdown);
 *   - gate order along every 4H axis (W, R, b, dW, dR, db): i, f, o, c' -- the order
 *     in which Section 2 lists the equations;
 *   - one bias vector per gate, as printed;
 *   - W is the concatenation of layer 0's [4H][I] matrix and the [4H][H] matrices of
 *     layers 1..L-1; R is [L][4H][H]; b is [L][4H];
 *   - calls are asynchronous on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream); internal helper streams fork from it and join back to it, and
 *     no call synchronises the host;
 *   - calls on different streams, also from different host threads, may overlap when
 *     each has its own `reserve` and `workspace`; two calls must never share a
 *     workspace or a reserve while either is in flight.  The library's own helper
 *     streams and events are shared by the process: calls that use them take turns
 *     while they enqueue (a mutex), their GPU work overlaps as the streams allow;
 *   - the persistent kernels (Section 4's idea: weights on chip, workgroups that wait
 *     on each other) need all their workgroups resident at once.  Those of one process
 *     are chained through an event and never share the device, so their results do not
 *     depend on the process's other work.  Nothing orders them against OTHER processes
 *     or against long kernels of the caller that hold compute units for longer than
 *     the kernels' bounded waits (about a second): LSTM_COOP_LAUNCH=1 in the
 *     environment selects cooperative launches, which give the device-wide guarantee
 *     at a small cost per launch;
 *   - a persistent kernel whose bounded wait expires stops waiting, finishes and raises
 *     a host-visible word.  The call that launched it has returned LSTM_OK long before
 *     and ITS OUTPUTS ARE INVALID; the next lstm_* / rnn_* forward or backward call on
 *     any path returns LSTM_INTERNAL without launching anything and clears the word,
 *     the call after that runs normally (lstm_shutdown clears it too).  A caller that
 *     needs certainty about one call synchronises its stream and makes a second call;
 *   - return value: LSTM_OK or an LSTM_* error code.  Arguments are validated before
 *     any GPU work; on error nothing has been launched except for LSTM_HIP_ERROR,
 *     which can surface after partial execution;
 *   - diagnostic settings come from environment variables (LSTM_NO_PAD, LSTM_COOP_LAUNCH,
 *     ...); they are read once, at the first call that needs one, and again after
 *     lstm_shutdown(), never in between.
 */
#ifndef LSTM_MI355X_H
#define LSTM_MI355X_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- status codes ---------------------------------------------------------------- */
#define LSTM_OK                0
#define LSTM_INVALID_ARG       1 /* non-positive dimension, required pointer NULL, misaligned pointer, bad flags */
#define LSTM_BUFFER_TOO_SMALL  2 /* workspace_bytes below lstm_workspace_bytes() */
#define LSTM_HIP_ERROR         3 /* a HIP runtime call or kernel launch failed */
#define LSTM_INTERNAL          4 /* a bounded wait of a persistent kernel of an EARLIER call expired; reported once */
#define LSTM_UNSUPPORTED       5 /* the forced path cannot run this shape on this device */

/* ---- flags: bits 0..3 select the execution path ---------------------------------------
 * The paths are the rungs of the paper's optimisation ladder (Table 1) rebuilt for
 * gfx950, plus the on-chip-weights variant that Section 4 names as future work.  */
#define LSTM_PATH_AUTO        0u /* persistent when the shape fits, else wavefront */
#define LSTM_PATH_NAIVE       1u /* Section 2.1 starting point: one kernel per operation, eight per-gate GEMMs per cell */
#define LSTM_PATH_GROUPED     2u /* + the four gates stacked into one GEMM per operand (optimisation 1) */
#define LSTM_PATH_FUSED       3u /* + one fused point-wise kernel per cell (optimisation 3) */
#define LSTM_PATH_STEP        4u /* + time-batched input GEMM per layer and a fused recurrent-GEMM+point-wise
                                    step kernel, layers one after the other (optimisations 4, 5) */
#define LSTM_PATH_WAVEFRONT   5u /* + layers overlapped on HIP streams in diagonal order (optimisations 2, 6) */
#define LSTM_PATH_PERSISTENT  6u /* one kernel for the whole recurrence, all workgroups resident: weights in
                                    registers, steps ordered by flags in device memory (Section 4) */
#define LSTM_PATH_MASK        0xFu

/* Bytes of the opaque `reserve` buffer that lstm_forward fills for lstm_backward.
 * Returns 0 if any dimension is non-positive.
 *
 * Hidden sizes below 512 other than 128 and 256 (with more than a few steps of one layer; above
 * 512 rows not the sizes from 257 to 415) are computed at the next of 128, 256, 512, and sizes between 512 and 1024 at 1024
 * (with up to 64 rows; up to 128 rows from 608, up to 256 from 640, up to 768 from 832), sizes from 1472 (up to
 * 32 rows) or 1664 (up to 64 rows) to 2047 at 2048: the library copies W, R, b, the initial states
 * and, backward, the upstream gradients into zero-padded buffers inside the workspace, runs the
 * padded network on the chosen path and copies the results back.  The result is that of the
 * given network: a hidden unit whose weights, bias and initial state are zero stays at h = c = 0
 * at every step and receives zero gradients.  The persistent kernels (Section 4) exist for those
 * sizes, and the padded run is faster than the per-step paths at the given size (three to
 * five times with four layers).  Reserve and workspace sizes are those of the padded network, and
 * the copies are part of the weight re-layout that Section 2.3 redoes every pass.  The smallest
 * networks (H = 8, 16 or 32 with I <= 64, B <= 8 and L (3 + B) <= 20) are not padded either: one
 * workgroup runs a whole pass of theirs as given, steps looped inside one launch (the low end of
 * Section 3.1's range, where a launch costs more than a step); LSTM_MICRO=0 in the environment
 * switches that off.  LSTM_NO_PAD=1 in the
 * environment runs every shape as given; both size queries return the larger of the padded and the
 * as-given requirement, so a buffer sized under one setting is never too small under the other (the
 * reserve's layout still differs: forward and backward of one reserve must run under one setting of both variables, which
 * holds by itself because settings are only read again after lstm_shutdown). */
size_t lstm_reserve_bytes(int L, int T, int B, int I, int H);

/* Bytes of scratch that lstm_forward / lstm_backward need (the maximum over both and
 * over all paths).  Contents need not survive between calls.  Returns 0 on invalid
 * dimensions. */
size_t lstm_workspace_bytes(int L, int T, int B, int I, int H);

/*
 * Forward pass (Section 2 equations; execution per Sections 2.2-2.4 and 4).
 *   x   [T][B][I]  input sequence, time-major
 *   h0  [L][B][H]  initial hidden state, NULL = zeros
 *   c0  [L][B][H]  initial cell state,   NULL = zeros
 *   W, R, b        parameters, layouts above
 *   y   [T][B][H]  out: hidden state of the top layer at every step
 *   hT  [L][B][H]  out: hidden state of every layer after the last step, NULL = not written
 *   cT  [L][B][H]  out: cell state of every layer after the last step,   NULL = not written
 *   reserve        out: lstm_reserve_bytes() bytes kept for lstm_backward; NULL = inference
 *                  (the same data then lives in the workspace and is discarded)
 *   workspace      scratch of at least lstm_workspace_bytes() bytes
 */
int lstm_forward(int L, int T, int B, int I, int H,
                 const float* x, const float* h0, const float* c0,
                 const float* W, const float* R, const float* b,
                 float* y, float* hT, float* cT,
                 void* reserve, void* workspace, size_t workspace_bytes,
                 void* stream, unsigned flags);

/*
 * One-time set-up for the current device, for callers that want nothing created inside their calls:
 * resolves the address of the library's static scratch array on this device and creates what the
 * persistent path otherwise creates on first use (the host-visible watchdog word, pinned host memory,
 * and the event that chains persistent launches).  Optional: every entry point does its own set-up on
 * first use.  Call it again after lstm_shutdown().  Returns LSTM_OK or LSTM_HIP_ERROR.
 */
int lstm_init(void);

/*
 * lstm_forward for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and results as
 * lstm_forward without `workspace` / `workspace_bytes`: the scratch is a static array in device memory,
 * LSTM_NOALLOC_SCRATCH_BYTES (64 MiB) per GPU, held from library load until the process ends.
 *   - shapes whose lstm_workspace_bytes() exceeds that size are rejected with LSTM_BUFFER_TOO_SMALL
 *     (lstm_last_error() gives both numbers) before anything is launched;
 *   - the call allocates and frees nothing and creates no stream or event once lstm_init() has run on
 *     the device (without it the first call on a device performs that set-up itself);
 *   - LSTM_PATH_WAVEFRONT is refused (LSTM_UNSUPPORTED), and where LSTM_PATH_AUTO would choose it the
 *     step path runs instead: the wavefront's helper streams are created to the size of the shape;
 *   - every call on a GPU uses that GPU's one array: calls that overlap in time on one GPU (two
 *     streams, two threads) race on it and must be ordered by the caller.  Nothing is assumed about
 *     what the previous call left there: counters that must start at zero are cleared by a fill kernel
 *     inside the call (no memset node, so a captured call replays correctly).
 */
#define LSTM_NOALLOC_SCRATCH_BYTES ((size_t)64 << 20)
int lstm_forward_noalloc(int L, int T, int B, int I, int H,
                         const float* x, const float* h0, const float* c0,
                         const float* W, const float* R, const float* b,
                         float* y, float* hT, float* cT,
                         void* reserve, void* stream, unsigned flags);

/*
 * Backward pass: gradients of  <dy,y> + <dhT,hT> + <dcT,cT>  with respect to every input
 * of lstm_forward.  The paper gives no backward equations; this is the chain rule through
 * the Section 2 equations, with the data-gradient products grouped over the four gates
 * (Section 2.1) and the weight gradients formed as one large product per matrix after all
 * propagation is complete (Section 2.6).
 *   x, h0, c0, W, R  the arguments given to lstm_forward (h0/c0 may be NULL again)
 *   reserve          as written by lstm_forward with the same dimensions
 *   dy   [T][B][H]   gradient with respect to y
 *   dhT, dcT [L][B][H] gradients with respect to hT, cT; NULL = zeros
 *   dx   [T][B][I]   out, NULL = skipped
 *   dh0, dc0 [L][B][H] out, NULL = skipped
 *   dW, dR, db       out, shaped like W, R, b; OVERWRITTEN (not accumulated into)
 */
int lstm_backward(int L, int T, int B, int I, int H,
                  const float* x, const float* h0, const float* c0,
                  const float* W, const float* R, const void* reserve,
                  const float* dy, const float* dhT, const float* dcT,
                  float* dx, float* dh0, float* dc0,
                  float* dW, float* dR, float* db,
                  void* workspace, size_t workspace_bytes,
                  void* stream, unsigned flags);

/*
 * C[M][N] (row stride ldc) = A * B, or += when accumulate != 0, on the fp32 matrix cores.
 * This is the time-batched product of Section 2.3 (input projections of many steps in one
 * call) and of Section 2.6 (weight gradients); the LSTM calls use it internally and it is
 * exported so that tests can check it alone.  Element (m,k) of A is A[m*sAm + k*sAk],
 * element (k,n) of B is B[k*sBk + n*sBn]; one stride of each operand must be 1.
 */
int lstm_gemm_f32(int M, int N, int K,
                  const float* A, long sAm, long sAk,
                  const float* B, long sBk, long sBn,
                  float* C, long ldc, int accumulate, void* stream);

/*
 * The same product with a scratch buffer (device memory, 16-byte aligned, scratch_bytes long, NULL: none; it must
 * stay untouched until the stream has passed the call).  A product whose 128 x 128 tiles do not fill the chip evenly --
 * fewer tiles than the chip holds workgroups, or a last round with few tiles -- has the tile rows of that round cut
 * along K into as many slices as fill the chip once more; the slices' partial tiles go to the scratch buffer and are
 * added in a fixed order, so the result is repeatable and differs from lstm_gemm_f32's only by the order of the
 * additions.  Too small a buffer means fewer slices or none (never an error).  This is how the LSTM calls run the
 * time-batched products of Section 2.3 at large hidden sizes (M = T*B = 1600 rows leave 832 tiles for 768 places).
 */
int lstm_gemm_f32_ws(int M, int N, int K,
                  const float* A, long sAm, long sAk,
                  const float* B, long sBk, long sBn,
                  float* C, long ldc, int accumulate, void* scratch, size_t scratch_bytes, void* stream);

/* Which path LSTM_PATH_AUTO resolves to for this shape on the current device
 * (returns an LSTM_PATH_* value; LSTM_PATH_AUTO on invalid dimensions). */
unsigned lstm_auto_path(int L, int T, int B, int I, int H, int backward);

/*
 * Overrides what LSTM_PATH_AUTO resolves to for one shape and direction (Sections 2.3 and 3.2: whether
 * a strategy pays depends on the hidden size, the minibatch and the number of layers, and choosing is
 * "not trivial"; a caller, or the bundled autotuner, can measure and pin the choice).  `path` is an
 * LSTM_PATH_* value; LSTM_PATH_AUTO removes the override.  Host-side table, thread-safe, emptied by
 * lstm_shutdown.  Returns LSTM_OK, LSTM_INVALID_ARG (non-positive dimension, unknown path) or
 * LSTM_UNSUPPORTED (the path does not take this shape on the current device).
 */
int lstm_set_path(int L, int T, int B, int I, int H, int backward, unsigned path);

/*
 * Number of chunks the stream-wavefront path cuts the sequence into for one shape (both directions).
 * Section 2.3: batching the input products of s steps makes them more efficient but makes the layer
 * above wait longer, and the best s depends on the hardware and the shape; the default is about 2L
 * chunks.  `chunks` = 0 removes the setting; values above T or 64 are clamped.  Host-side table,
 * thread-safe, emptied by lstm_shutdown.  Returns LSTM_OK or LSTM_INVALID_ARG (non-positive
 * dimension, negative count).  The bundled autotuner measures a few counts and pins the best.
 */
int lstm_set_wavefront_chunks(int L, int T, int B, int I, int H, int chunks);

/*
 * Phase timing for measurement (Section 2.5 reports time per optimisation stage; this is the
 * same breakdown taken live).  While enabled, lstm_forward / lstm_backward record HIP events
 * on the stream each phase is launched on, at the phase's first and last launch.
 * lstm_profile_read waits for the recorded events, adds the elapsed milliseconds of every
 * recorded interval to ms[phase], the interval count to count[phase] and, when `flops` is not
 * NULL, the algorithmic FLOPs (2*M*N*K of every matrix product launched inside the interval,
 * whichever kernel carried it: a product folded into a persistent kernel counts in that
 * kernel's phase) to flops[phase] (arrays of LSTM_PHASE_COUNT entries, host memory,
 * overwritten), and forgets the events.  lstm_profile_kernel names the kernel that carried the
 * matrix products of a phase in the most recent profiled call ("" if none; static storage).
 * Returns LSTM_OK or LSTM_HIP_ERROR.  Not thread-safe; intended for benchmarks.
 */
#define LSTM_PHASE_FWD_PACK        0 /* weight re-layout / exchange set-up, forward */
#define LSTM_PHASE_FWD_INPUT_GEMM  1 /* time-batched input projection(s) */
#define LSTM_PHASE_FWD_RECURRENCE  2 /* per-step recurrent work (step kernels or the persistent kernel) */
#define LSTM_PHASE_BWD_PACK        3 /* weight re-layout, backward */
#define LSTM_PHASE_BWD_RECURRENCE  4 /* backward per-step work */
#define LSTM_PHASE_BWD_INPUT_GEMM  5 /* batched input-gradient product(s) */
#define LSTM_PHASE_WEIGHT_GRAD     6 /* dW, dR products */
#define LSTM_PHASE_BIAS_GRAD       7 /* db reductions */
#define LSTM_PHASE_COUNT           8
void lstm_profile_enable(int on);
int lstm_profile_read(float* ms, int* count, double* flops);
const char* lstm_profile_kernel(int phase);
const char* lstm_phase_name(int phase);

/*
 * Diagnostic hook for the persistent path: while a buffer is set, the workgroup with index
 * `block` of every persistent launch writes a wall-clock time stamp (100 MHz ticks, int64) at
 * up to 8 points of each step into device_buf[step*8 + point].  The buffer must hold T*8 int64
 * values for the launches it is used with (smaller buffers are ignored); NULL turns it off.
 */
void lstm_debug_set_trace(void* device_buf, size_t bytes, int block);

/* Human-readable text for a status code (static storage, never NULL). */
const char* lstm_status_string(int status);

/* Text of the last HIP error seen by this thread's most recent failing call ("" if none). */
const char* lstm_last_error(void);

/* Destroys the helper streams and events the library created, empties the per-shape tables, clears a
 * pending watchdog report and forgets the settings read from the environment.  Safe to call
 * repeatedly (not while a call is in flight); the next call re-creates what it needs. */
void lstm_shutdown(void);

#ifdef __cplusplus
}
#endif
#endif /* LSTM_MI355X_H */
