/*
 * CPU oracle for the Quantized-Adam-with-error-feedback optimizer step.
 *
 * TEST INFRASTRUCTURE ONLY.  This is the slow, single-threaded, plainly
 * written checker that the GPU library is compared against.  Nothing on the
 * product path may call it, and it shares no code with the HIP kernels.
 *
 * What it follows (arXiv 2004.14180):
 *   - Sec. 5.1 "Implementation Details": the gradient quantizer Q_g
 *     (infinity-norm scale times the nearest point of the power-of-two grid
 *     G = {0, +-2^-k_g, ..., +-1/2, +-1}) and the weight quantizer Q_x
 *     (half of the nearest point of the uniform grid with spacing 2^-k_x on
 *     [-1, 1]).
 *   - Algorithm 1 and Algorithm 3 (moment, update and residual steps): moment updates
 *     v = theta*v + (1-theta)*g^2, m = beta*m + (1-beta)*g, the step
 *     alpha*m/sqrt(v+eps) (eps inside the root, no bias correction) and the
 *     error-feedback residual e' = (value + e) - Q_g(value + e).
 *   - Algorithm 2 (broadcast, gather, update and output steps): the server averages the N worker
 *     messages, keeps the full-precision iterate and emits Q_x of it.
 *
 * Two placements of the moments are implemented:
 *   variant S ("server moments"): workers quantize g+e; the server averages
 *     the dequantized gradients and runs the Adam update.
 *   variant W ("worker moments"): Algorithms 2-3 as printed; each worker owns
 *     m, v and quantizes alpha*m/sqrt(v+eps)+e; the server subtracts the mean.
 *
 * Arithmetic: every floating-point operation is a separate IEEE-754 binary32
 * operation, round-to-nearest-even, no fused multiply-add, subnormals kept
 * (compile with -ffp-contract=off and without -ffast-math).  The paper is
 * written over the reals; this precision is the reading fixed for the build
 * so that integer codes can be compared bit for bit.
 *
 * Pins (tests/test_oracle_*.py): identity quantizers reduce to generic Adam
 * with a closed form for constant gradients; exact residual q + e' == p;
 * codes in range; Assumption 2 / Assumption 3 inequalities; error-feedback
 * telescoping (Notation 1 / Notation 3); hand-worked vectors; brute-force
 * arg-min in fp64; a library Adam for the bias-corrected flavour; Philox
 * published known-answer vectors.
 * Parity unpinned: the values of k_g and k_x the authors actually ran (the
 * paper never states them; only bits per element follow from Tables 1-2).
 */
#ifndef QADAM_ORACLE_H
#define QADAM_ORACLE_H

#include <stdint.h>
#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t k_g;          /* Q_g grid: levels 2^-k_g .. 1 (k_g = 0 is ternary), 0 <= k_g <= 6 */
    int32_t k_x;          /* Q_x grid: spacing 2^-(k_x+1) on [-1/2, 1/2], 0 <= k_x <= 14 */
    int32_t rounding;     /* 0 nearest (ties to the larger magnitude), 1 stochastic (Philox) */
    int32_t weight_ef;    /* 0: residual x - Q_x(x) reported only; 1: fed back (y = x + e^x) */
    int32_t adam_flavor;  /* 0: paper (eps inside sqrt, no bias correction); 1: bias-corrected, eps outside */
    int32_t identity_g;   /* oracle-only: Q_g(p) = p */
    int32_t identity_x;   /* oracle-only: Q_x(y) = y */
    float   beta1;
    float   eps;
    uint64_t seed;        /* Philox key */
} oq_config;

/* status bits returned by the step functions */
#define OQ_NONFINITE_SCALE 1   /* some layer scale was NaN or Inf */

/* ---- counter-based random numbers (Salmon et al., SC'11, Philox4x32-10) ---- */
void oq_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);
/* uniform in [0,1) with 24 bits for element j of (step, worker, stream) */
float oq_uniform24(uint64_t seed, int64_t j, int64_t step, int32_t worker, int32_t stream);

/* ---- sizes of the packed code layouts ---- */
int32_t oq_grad_code_bits(int32_t k_g);                 /* bits per gradient code: 1 + ceil(log2(k_g+2)) */
int64_t oq_grad_code_words_segment(int32_t k_g, int64_t n); /* uint32 words of one segment, padded to 16 B */
int64_t oq_grad_code_words(int32_t k_g, const int64_t* seg_off, int32_t L);
int32_t oq_weight_code_bytes_per_elem(int32_t k_x);     /* 1 (k_x <= 6) or 2 */

/* ---- quantizers on one layer ---- */
/* Q_g, Sec. 5.1.  p[n] -> scale s = max|p|, per-element code (sign << w | mu),
 * dequantized value q, and tie flag (pre-rounding ratio within one ulp of a
 * decision threshold).  j0 = global flat index of p[0] (for the random
 * stream).  Returns OQ_NONFINITE_SCALE if s is not finite (outputs then
 * unspecified but in range). */
int oq_qg_layer(const oq_config* cfg, const float* p, int64_t n, int64_t j0,
                int64_t step, int32_t worker,
                float* s_out, uint8_t* code, float* q, uint8_t* tie);

/* the element-wise part of Q_g on a window of a layer whose scale s was
 * obtained separately (layers too large to run whole are checked on windows) */
void oq_qg_window(const oq_config* cfg, const float* p, int64_t n, int64_t j0,
                  int64_t step, int32_t worker, float s,
                  uint8_t* code, float* q, uint8_t* tie);
void oq_worker_quantize_window(const oq_config* cfg, int64_t n, int64_t j0,
                               int32_t worker, int64_t step, float s,
                               const float* grad, float* err,
                               uint8_t* code, uint8_t* tie, float* q_out);

/* value of one gradient code */
float oq_qg_decode(int32_t k_g, float s, uint8_t code);

/* Q_x, Sec. 5.1.  y[n] -> integer grid index j in [-2^k_x, 2^k_x], value
 * xhat = j * 2^-(k_x+1), tie flag. */
void oq_qx(const oq_config* cfg, const float* y, int64_t n, int64_t j0, int64_t step,
           int32_t* jcode, float* xhat, uint8_t* tie);

/* pack / unpack the bit-plane layout: per segment, groups of 32 consecutive
 * elements; a group is b consecutive uint32 words, word k carries bit k of
 * the 32 codes, bit n of a word belongs to element 32*group + n. */
void oq_pack_codes(int32_t bits, const uint8_t* code, int64_t n, uint32_t* words);
void oq_unpack_codes(int32_t bits, const uint32_t* words, int64_t n, uint8_t* code);

/* ---- Adam core (moment and update steps of Algorithm 1 without the quantizer) ---- */
/* updates m, v in place and writes the step u = alpha*m/sqrt(v+eps) (flavour 0)
 * so that the caller forms x - u or Q_g(u + e). */
void oq_adam_update(const oq_config* cfg, float lr, float beta2, int64_t step,
                    const float* g, float* m, float* v, float* u, int64_t n);

/* ---- the three calls of the hot path, variant S ---- */
/* worker side: p = g + e; per segment Q_g; e <- p - q.  Outputs: packed codes
 * (words), per-element codes (code_unpacked, may be NULL), scales[L],
 * tie[P] (may be NULL), q[P] dequantized values (may be NULL). */
int oq_worker_quantize(const oq_config* cfg, const int64_t* seg_off, int32_t L,
                       int64_t index_base, int32_t worker, int64_t step,
                       const float* grad, float* err,
                       uint32_t* words, uint8_t* code_unpacked, float* scales,
                       uint8_t* tie, float* q_out);

/* server side: gbar = (sum_i q_i) / N in worker order from the packed codes
 * and scales, then the Adam update of m, v, x. */
void oq_server_step(const oq_config* cfg, const int64_t* seg_off, int32_t L,
                    int32_t N, int64_t step, float lr, float beta2,
                    const uint32_t* const* words, const float* const* scales,
                    float* x, float* m, float* v);

/* weight quantize: y = x (+ werr if weight_ef); code; werr <- y - xhat.
 * wcodes is int8 (k_x <= 6) or int16; xhat/tie may be NULL. */
void oq_weight_quantize(const oq_config* cfg, int64_t P, int64_t index_base, int64_t step,
                        const float* x, float* werr, void* wcodes, float* xhat, uint8_t* tie);

/* one whole step of variant S = the three calls above; honours identity_g /
 * identity_x.  Returns status bits.  ties_g[N] / ties_x count flagged
 * elements (may be NULL). */
int oq_step_s(const oq_config* cfg, const int64_t* seg_off, int32_t L, int32_t N,
              int64_t index_base, int64_t step, float lr, float beta2,
              const float* const* grads, float* const* errs,
              uint32_t* const* words, float* const* scales,
              float* x, float* m, float* v, float* werr, void* wcodes,
              uint8_t* const* tie_g, uint8_t* tie_x);

/* the same step on a window of ONE layer with the workers' layer scales given */
int oq_step_s_window(const oq_config* cfg, int64_t n, int64_t j0, int32_t N,
                     int64_t step, float lr, float beta2, const float* s,
                     const float* const* grads, float* const* errs,
                     float* x, float* m, float* v, float* werr,
                     uint8_t* const* codes, void* wcodes,
                     uint8_t* const* tie_g, uint8_t* tie_x);

/* one whole step of variant W (Algorithms 2-3): per-worker m_i, v_i. */
int oq_step_w(const oq_config* cfg, const int64_t* seg_off, int32_t L, int32_t N,
              int64_t index_base, int64_t step, float lr, float beta2,
              const float* const* grads, float* const* errs,
              float* const* mw, float* const* vw,
              uint32_t* const* words, float* const* scales,
              float* x, float* werr, void* wcodes,
              uint8_t* const* tie_g, uint8_t* tie_x);

#ifdef __cplusplus
}
#endif
#endif
