/*
 * qadam.h -- C boundary of the MI355X (gfx950) library for the optimizer step of
 * Quantized Adam with error feedback (arXiv 2004.14180).
 *
 * The step, per parameter (notation of the paper: x iterate, m and v moments, e error-feedback
 * term, alpha_t step size, beta momentum, theta_t averaging parameter, N workers):
 *
 *   worker i :  p = g_i + e_i                         error-feedback add   (Alg. 1 update step, Alg. 3 send step)
 *               s_il = ||p||_inf over layer l        scale of Q_g         (Sec. 5.1)
 *               q = Q_g(p) = s * nearest point of G  G = {0, +-2^-k_g, ..., +-1/2, +-1}   (Sec. 5.1)
 *               e_i <- p - q                          residual             (Alg. 1 / Alg. 3 residual step)
 *   server   :  gbar = (1/N) sum_i q_i               mean of the messages (Alg. 2 gather step)
 *               v <- theta_t v + (1-theta_t) gbar^2   (Alg. 1 second-moment step)
 *               m <- beta m + (1-beta) gbar           (Alg. 1 first-moment step)
 *               x <- x - alpha_t m / sqrt(v + eps)    (Alg. 1 update step without the quantizer)
 *               x^ = Q_x(x [+ e^x]),  e^x <- (x [+ e^x]) - x^      (Sec. 5.1; Alg. 2 broadcast and output steps)
 *
 * This is "variant S": the workers quantize gradients and the server owns the moments.  The
 * paper's Algorithms 2-3 keep the moments on the workers and quantize the Adam update instead
 * ("variant W"); the entry points ending in _w implement that placement with the same kernels.
 *
 * All arithmetic is IEEE binary32, one rounding per operation (no fused multiply-add), subnormals
 * kept, division and square root correctly rounded; integer codes are therefore reproducible bit
 * for bit by a plain CPU implementation of the same formulas.
 *
 * Conventions
 *   - Every pointer named *_dev (and every element of the pointer arrays) is DEVICE memory on the
 *     current HIP device, 16-byte aligned, owned by the caller and alive until the stream has
 *     passed the call.  Pointer arrays themselves and seg_offsets are HOST memory, read during
 *     the call only.
 *   - `stream` is a hipStream_t passed as void*.  Compute calls only enqueue work on it; they do
 *     not synchronise.  Calls on one handle that touch the same worker, or the server state, must
 *     be ordered by the caller (one stream, or events).  qadam_worker_quantize / qadam_worker_step_w
 *     calls for DIFFERENT workers may run concurrently on different streams: the handle keeps
 *     separate scratch rows per worker, and the status word is only ever OR-ed into.  The whole-step
 *     calls and qadam_layer_sumsq use scratch of all workers, so they must not overlap anything else
 *     on the same handle.
 *   - The parameter vector is flat, P = seg_offsets[L] elements, split into L layer segments
 *     [seg_offsets[l], seg_offsets[l+1]); empty segments are allowed.  Any offsets are accepted; a
 *     segment that starts on a multiple of 4 elements is moved with 16-byte-aligned accesses, the others
 *     with 4-byte-aligned ones, which costs about 8 % of the step on this GPU.  A caller who lays the
 *     vector out can pad each layer with zeros (in every buffer) to a multiple of 4 elements: a zero
 *     element stays zero in every buffer and changes no scale, so the other results are the same.
 *   - `step` is the 1-based iteration t.
 *   - Return value: QADAM_OK or a negative error code.  QADAM_EINVAL, QADAM_EALIGN and QADAM_ERANGE come from
 *     checks made before anything is enqueued: the buffers are untouched.  QADAM_EHIP means a kernel launch
 *     was refused by the runtime part way through the call: launches accepted before it still run, so the
 *     buffers of the call are then in an intermediate state (variant S: scales written, state not yet
 *     advanced; variant W: m_i, v_i already advanced and the error buffers holding the parked
 *     alpha_t m_i / sqrt(v_i + eps) + e_i instead of e_i) and the step cannot be repeated on them.
 *     Non-finite scales (NaN/Inf in g + e) are data errors: they set a bit in the status word that
 *     qadam_get_status reads; the outputs of that layer are then unspecified (codes stay in range).
 *   - HIP graphs: the compute calls may be recorded into a graph (stream capture).  A replay repeats the
 *     call with the arguments it was recorded with: the same pointers, and the same step, lr and beta2.
 *     With nearest rounding and the paper's Adam (adam_flavor = 0) the step number enters no kernel, so a
 *     replay stands for any iteration with that lr and beta2.  The calls return QADAM_EINVAL when asked to
 *     record what a replay cannot follow: rounding = 1 (the random stream is keyed on the step) and
 *     adam_flavor = 1 (bias corrections depend on the step).  A recorded call always uses the full scale
 *     pass, whatever qadam_trust_error_buffers says, and a handle whose graph is being replayed should
 *     not also run eager steps with that option on (replays rewrite the handle's residual bounds).
 *   - The library allocates only in qadam_init (tables proportional to P/4096 plus the segment
 *     table) and frees in qadam_destroy.
 *
 * Packed gradient codes (one buffer per worker, qadam_grad_code_bytes bytes): a code is
 * (sign << w) | mu with mu in 0..k_g+1 the grid level (0 = zero, mu >= 1 = 2^(mu-1-k_g)),
 * w = ceil(log2(k_g+2)), b = 1 + w bits (k_g=0: 2 bits; k_g=1,2: 3 bits; k_g=3..6: 4 bits).
 * Per segment, in segment order: groups of 32 consecutive elements, each group stored as b
 * consecutive uint32 words where word k holds bit k of the 32 codes and bit n of a word belongs to
 * element 32*group + n; a ragged last group is zero padded, and each segment is padded with zero
 * words to a multiple of 16 bytes.  Exactly b bits per element (Tables 1-2: 3/32 and 2/32 of fp32).
 * Weight codes: one signed integer j per element, x^ = j * 2^-(k_x+1), |j| <= 2^k_x, stored as int8
 * when k_x <= 6 and int16 otherwise (Tables 1-2: 1/4 and 1/2 of fp32).
 */
#ifndef QADAM_H
#define QADAM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define QADAM_OK        0
#define QADAM_EINVAL   -1   /* bad argument (null pointer, worker out of range, bad config, bad segments) */
#define QADAM_EALIGN   -2   /* a device pointer is not 16-byte aligned */
#define QADAM_ERANGE   -3   /* size beyond what the library supports */
#define QADAM_EHIP     -4   /* a HIP runtime call failed (see qadam_last_error) */

#define QADAM_MAX_WORKERS 32

/* k_g or k_x = QADAM_IDENTITY: that quantizer is the identity.  These are the settings of the paper's
 * Theorem 1 (Q_x = id: gradient quantization with error feedback, full-precision weights) and Theorem 2
 * (Q_g = id: full-precision messages, quantized weights), and of the corresponding rows of Tables 1-2;
 * both = plain (distributed) generic Adam.  Only the whole-step calls run in these modes:
 *   Q_g = id, qadam_step_fused:   the message of worker i is g_i itself; errs, codes and scales are not
 *                                 used (the arrays may be NULL); qadam_grad_code_bytes is 0;
 *   Q_g = id, qadam_step_fused_w: the message is alpha_t m_i / sqrt(v_i + eps) + e_i and e_i <- 0 (the
 *                                 error buffers are still needed as working space); codes, scales unused;
 *   Q_x = id:                     no weight codes and no weight residual are produced (werr_dev and
 *                                 wcodes_dev may be NULL); qadam_weight_code_bytes is 0.
 * The single-purpose calls of a quantizer that is switched off return QADAM_EINVAL. */
#define QADAM_IDENTITY (-1)

/* status word bits */
#define QADAM_STATUS_NONFINITE_SCALE 1u   /* some ||g+e||_inf was NaN or Inf */
#define QADAM_STATUS_ERR_BOUND_VIOLATED 2u /* qadam_trust_error_buffers(h, 3): an error buffer was not what the
                                             previous step left (some |e| beyond the recorded bound) */

typedef struct qadam_ctx* qadam_handle_t;

typedef struct {
    uint32_t struct_size;   /* = sizeof(qadam_config_t) */
    int32_t  k_g;           /* Q_g grid exponent count, 0..6 (0 = ternary), or QADAM_IDENTITY    Sec. 5.1 */
    int32_t  k_x;           /* Q_x grid: multiples of 2^-(k_x+1) on [-1/2, 1/2], 0..14,
                               or QADAM_IDENTITY                                                 Sec. 5.1 */
    int32_t  rounding;      /* 0 = nearest, a midpoint goes to the larger magnitude (the paper's arg-min);
                               1 = unbiased stochastic rounding driven by Philox4x32-10 keyed on
                               (seed; element index, step, worker, stream) */
    int32_t  weight_ef;     /* 0 = e^x written (x - x^) but not fed back (the server keeps full-precision x,
                               Alg. 2); 1 = Q_x sees x + e^x and e^x accumulates */
    int32_t  adam_flavor;   /* 0 = the paper's generic Adam (eps inside the root, no bias correction);
                               1 = bias-corrected moments and eps outside the root */
    float    beta1;         /* beta */
    float    eps;           /* epsilon */
    uint64_t seed;          /* key of the random stream (rounding = 1) */
} qadam_config_t;

typedef struct {
    uint32_t flags;         /* OR of QADAM_STATUS_* since init or the last reset */
    uint32_t reserved;
} qadam_status_t;

/* Create a handle for one flat parameter vector x in R^d (Sec. 3, problem statement; state of Alg. 1 and
 * of Alg. 2-3), split into the layers over which the norm of Q_g (Sec. 5.1) is taken.  seg_offsets: L+1
 * non-decreasing HOST values with seg_offsets[0] = 0; num_workers = N of Alg. 2-3, in 1..QADAM_MAX_WORKERS.
 * Allocates the handle's device tables on the current device. */
int qadam_init(qadam_handle_t* out, const qadam_config_t* cfg,
               const int64_t* seg_offsets, int32_t num_segments, int32_t num_workers);
int qadam_destroy(qadam_handle_t h);

/* Bytes of one worker's packed gradient codes for the whole vector (including segment padding), and of the
 * weight codes: the message and model sizes of Tables 1-2 (b bits and 8 or 16 bits per element). */
size_t qadam_grad_code_bytes(qadam_handle_t h);
size_t qadam_weight_code_bytes(qadam_handle_t h);
int64_t qadam_num_params(qadam_handle_t h);

/* Worker side: the send and residual steps of Alg. 3 (update and residual steps of Alg. 1) applied to the
 * gradient, with Q_g of Sec. 5.1 -- p = g + e, s = ||p||_inf per layer, codes of Q_g(p), e <- p - Q_g(p):
 *   grad_dev   [P] in        stochastic gradient g_i
 *   err_dev    [P] in/out    e_i -> p - Q_g(p)
 *   codes_dev  out           packed codes, qadam_grad_code_bytes bytes
 *   scales_dev [L] out       per-layer scales s_il (fp32)
 * worker in [0, num_workers). */
int qadam_worker_quantize(qadam_handle_t h, int32_t worker, int64_t step,
                          const float* grad_dev, float* err_dev,
                          void* codes_dev, float* scales_dev, void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): qadam_worker_quantize for ONE layer segment without a handle and without
 * any allocation, here or in any routine it calls.  Same results, bit for bit, as qadam_worker_quantize on a
 * handle with the single segment [0, n), nearest rounding (rounding = 0) and this k_g:
 *   grad_dev [n] in; err_dev [n] in/out; codes_dev out, ((n+31)/32 * b words rounded up to 4 words) * 4 bytes with
 *   b = 2, 3, 4 bits for k_g = 0, 1..2, 3..6; scale_dev [1] out (device), ||g+e||_inf.
 * The per-tile maxima, the reciprocal scale and a status word that the handle keeps in allocated tables live
 * in a static device array of (QADAM_NOALLOC_MAX_ELEMS / 4096 + 64) * 4 bytes = 256.25 KiB, which each GPU the
 * library runs on holds until the process ends; n > QADAM_NOALLOC_MAX_ELEMS returns QADAM_ERANGE.  The array's
 * address on the current device is looked up once per device: by qadam_init, else by the first call of this
 * function on that device (only that first call should stay outside a graph capture).
 * ALL calls on one GPU share the array: two calls that may overlap on one GPU (different streams without an
 * ordering event, or two host threads on different streams) race and give wrong results; calls on one stream
 * are ordered and need nothing.  Nothing in the array has to be cleared between calls (every word is written
 * before it is read).  A non-finite ||g+e||_inf is visible in scale_dev (codes are then all zero); there is no
 * status word to read for this call.  Enqueues three kernels on `stream`; does not synchronise. */
#define QADAM_NOALLOC_MAX_ELEMS (1 << 28)
int qadam_quantize_segment_noalloc(int32_t k_g, int64_t n, const float* grad_dev, float* err_dev,
                                   void* codes_dev, float* scale_dev, void* stream);

/* Server side: the gather step of Alg. 2 (mean of the dequantized messages, in worker order), then the
 * moment recursions and the update step of Alg. 1 on that mean (no quantizer in the update: Q_g acted on
 * the worker):
 *   codes[i], scales[i]: worker i's outputs of qadam_worker_quantize, i = 0..N-1 (HOST arrays of
 *   device pointers);  x, m, v [P] in/out.  lr = alpha_t, beta2 = theta_t. */
int qadam_server_step(qadam_handle_t h, int64_t step, float lr, float beta2,
                      const void* const* codes, const float* const* scales,
                      float* x_dev, float* m_dev, float* v_dev, void* stream);

/* Weight quantizer Q_x of Sec. 5.1 with its residual; what the broadcast and output steps of Alg. 2 emit,
 * Q_x(x_t), while the server keeps x_t:
 *   x_dev [P] in;  werr_dev [P]: in/out when weight_ef = 1, out only when 0 (may then be NULL);
 *   wcodes_dev out, qadam_weight_code_bytes bytes. */
int qadam_weight_quantize(qadam_handle_t h, int64_t step, const float* x_dev,
                          float* werr_dev, void* wcodes_dev, void* stream);

/* The whole step in one call (Alg. 3 send/residual steps for every worker, Alg. 2 gather step, Alg. 1
 * moment and update steps, Q_x of Sec. 5.1): identical results, bit for bit, to qadam_worker_quantize for
 * i = 0..N-1, then qadam_server_step, then qadam_weight_quantize, but each buffer makes one trip
 * through memory in the main kernel (the scales need one earlier read of g and e).
 * grads, errs, codes, scales: HOST arrays of N device pointers. */
int qadam_step_fused(qadam_handle_t h, int64_t step, float lr, float beta2,
                     const float* const* grads, float* const* errs,
                     void* const* codes, float* const* scales,
                     float* x_dev, float* m_dev, float* v_dev,
                     float* werr_dev, void* wcodes_dev, void* stream);

/* Variant W (Algorithms 2-3 as printed; Alg. 1 for N = 1): the worker owns m_i, v_i (moment steps of
 * Alg. 3) and quantizes its update (send step of Alg. 3); the server applies x <- x - mean (update step of
 * Alg. 2, with the sign of Alg. 1).  The worker quantizes
 * alpha_t m_i / sqrt(v_i + eps) + e_i; the server subtracts the mean of the messages.
 *   qadam_worker_step_w: grad [P] in; mw, vw [P] in/out; err [P] in/out; codes, scales out.
 *   qadam_server_apply_w: x [P] in/out from the N messages. */
int qadam_worker_step_w(qadam_handle_t h, int32_t worker, int64_t step, float lr, float beta2,
                        const float* grad_dev, float* mw_dev, float* vw_dev, float* err_dev,
                        void* codes_dev, float* scales_dev, void* stream);
int qadam_server_apply_w(qadam_handle_t h, int64_t step,
                         const void* const* codes, const float* const* scales,
                         float* x_dev, void* stream);

/* Variant W, the whole step in one call: identical results, bit for bit, to qadam_worker_step_w for
 * i = 0..N-1, then qadam_server_apply_w, then qadam_weight_quantize.  grads, mw, vw, errs, codes,
 * scales: HOST arrays of N device pointers. */
int qadam_step_fused_w(qadam_handle_t h, int64_t step, float lr, float beta2,
                       const float* const* grads, float* const* mw, float* const* vw,
                       float* const* errs, void* const* codes, float* const* scales,
                       float* x_dev, float* werr_dev, void* wcodes_dev, void* stream);

/* Dequantize weight codes (the receive step of Alg. 3: what a worker does with the broadcast of Alg. 2;
 * grid X of Sec. 5.1): x^ = j * 2^-(k_x+1).
 *   qadam_weight_dequantize      xhat_dev [P] fp32, exact.
 *   qadam_weight_dequantize_f16  xhat_dev [P] IEEE binary16 (2 bytes per element, 16-byte aligned), for
 *                                a consumer that computes in half precision; exact for k_x <= 10,
 *                                round-to-nearest-even of the fp32 value beyond (|j| needs more than
 *                                11 significand bits). */
int qadam_weight_dequantize(qadam_handle_t h, const void* wcodes_dev, float* xhat_dev, void* stream);
int qadam_weight_dequantize_f16(qadam_handle_t h, const void* wcodes_dev, void* xhat_dev, void* stream);

/* Opt-in: let qadam_step_fused and qadam_worker_quantize skip most of the first read of the error buffers.
 * The per-layer scale ||g_i + e_i||_inf normally costs one full read of g_i and e_i before the main pass.
 * The quantizer bounds the residual it leaves (|e| <= s/4 per element for k_g >= 1 with nearest rounding,
 * s/2 for the ternary grid, twice that with stochastic rounding), so when e_i is exactly what the previous
 * step of this handle wrote, an element whose |g| lies more than that bound below a known lower bound of the
 * scale cannot be the maximum.  With the option on the scale pass takes the exact maxima of a sample of tiles as
 * that lower bound and then reads e only where |g| is large enough to matter; the scales (and so every
 * output) are the same bits as without the option.  On Gaussian-like gradients this halves the scale
 * pass; on heavy-tailed ones it falls back to reading everything, layer by layer.
 * CONTRACT with the option on: between two step calls the caller must not change the contents of errs[i] (or
 * must call this function again, which makes the next step read everything).  Passing ANOTHER buffer for a
 * worker than the one its bound was recorded for is noticed (the pointer is remembered) and gets the full pass.  The first step after qadam_init, or after
 * this call, always reads everything.  Violating the contract gives scales that are too small.
 * on = 1 uses the filtered pass only where it pays (it adds two small launches: from about
 * 10^8 worker-elements per call on); on = 2 uses it always; on = 0 (the default) never.
 * on = 3 is a bring-up aid: the scale pass reads everything as with 0, and in addition every error buffer is
 * checked against the bound recorded by the previous step; a violation sets QADAM_STATUS_ERR_BOUND_VIOLATED
 * in the status word.  An integration that runs clean with 3 honours the contract of 1 and 2. */
int qadam_trust_error_buffers(qadam_handle_t h, int32_t on);

/* Placement of a handle's buffers inside ONE caller-allocated block (host arithmetic only; nothing is
 * allocated, no HIP call is made).  Why: the main pass of qadam_step_fused reads 2N+4 and writes N+5 streams at
 * once, and on MI355X its speed depends on where those streams lie in physical memory: with the buffers
 * packed closely one after the other (what a process gets when it allocates them in turn on a freshly booted
 * GPU) the pass runs 8-14 % slower than with the streams spread widely over the device's memory.  A block
 * obtained with one hipMalloc on an otherwise empty device is physically contiguous, so offsets inside it
 * decide the placement: the layout deals the buffers of each kind alternately to the first half of the block
 * and to its second half.  The block should therefore be much larger than the buffers (ideally most of the
 * device's memory; the space between the two groups stays free for the caller's other data).  Results never
 * depend on placement, only speed does.
 *   arena_bytes   size of the caller's block; its base must be 256-byte aligned
 *   with_worker_moments  non-zero: also place mw[i], vw[i] (variant W)
 *   out           byte offsets from the block's base, each a multiple of 256: x, m, v, werr [4P bytes each],
 *                 wcodes [qadam_weight_code_bytes], and per worker i < N: grads[i], errs[i], mw[i], vw[i]
 *                 [4P], codes[i] [qadam_grad_code_bytes], scales[i] [4L]; bytes_needed = the smallest block
 *                 this layout fits in when packed (arena_bytes below it: QADAM_ERANGE).
 * Entries of unused buffers (mw, vw without with_worker_moments; workers >= N) are SIZE_MAX. */
typedef struct {
    size_t x, m, v, werr, wcodes;
    size_t grads[QADAM_MAX_WORKERS], errs[QADAM_MAX_WORKERS], codes[QADAM_MAX_WORKERS], scales[QADAM_MAX_WORKERS];
    size_t mw[QADAM_MAX_WORKERS], vw[QADAM_MAX_WORKERS];
    size_t bytes_needed;
} qadam_arena_t;
int qadam_arena_layout(qadam_handle_t h, size_t arena_bytes, int32_t with_worker_moments, qadam_arena_t* out);

/* Diagnostic: per-layer squared Euclidean norms  out[l] = sum_{j in layer l} (a_j + b_j)^2, with the sum
 * a_j + b_j taken in fp32 (as the step forms g + e) and squares and sums in fp64 in a fixed order, so the
 * result is the same bits on every run.  b_dev may be NULL (then a alone).  out_dev: L doubles (device).
 * Called with (g_i, e_i) before a step and with (e_i, NULL) after it, the ratio of the two is the
 * empirical ||p - Q_g(p)||^2 / ||p||^2 of Assumption 2 (must stay below 1). */
int qadam_layer_sumsq(qadam_handle_t h, const float* a_dev, const float* b_dev, double* out_dev, void* stream);

/* Read (and optionally clear) the status word.  The read and the clear are enqueued on `stream` and the call
 * waits for that stream, so they are ordered against this stream's kernels; if the handle has work on other
 * streams (per-worker calls), wait for those streams first, or a bit set there concurrently can be lost by
 * the clear. */
int qadam_get_status(qadam_handle_t h, qadam_status_t* out, int32_t clear, void* stream);

/* Kernel timing for measurements.  When enabled, qadam_step_fused (and qadam_step_fused_w) bracket their two passes with HIP
 * events on the caller's stream; qadam_profile_read waits for the last bracketed call and returns
 * the durations in milliseconds: scale_pass_ms (the read of g and e that produces the per-layer
 * scales) and main_pass_ms (the fused worker + server + weight-quantize kernel). */
typedef struct {
    float scale_pass_ms;
    float main_pass_ms;
} qadam_profile_t;
int qadam_profile_enable(qadam_handle_t h, int32_t on);
int qadam_profile_read(qadam_handle_t h, qadam_profile_t* out);

/* Text of the last HIP error seen by this thread's calls (static storage). */
const char* qadam_last_error(void);

#ifdef __cplusplus
}
#endif
#endif
