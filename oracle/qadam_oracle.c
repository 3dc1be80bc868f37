/*
 * CPU oracle for the Quantized-Adam-with-error-feedback optimizer step.
 * TEST INFRASTRUCTURE ONLY -- see qadam_oracle.h for what it follows, the
 * arithmetic it fixes and how it is pinned.  Plain C, one thread, no
 * blocking, no fusion: every function is the formula of the paper written
 * as a loop.
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fno-fast-math -shared -fPIC
 */
#include "qadam_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------ */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as  */
/* easy as 1, 2, 3", SC'11).  One round maps (c0,c1,c2,c3) with key (k0,k1) */
/* to (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1, lo(M0*c0)); the key is  */
/* advanced by the Weyl constants between rounds; ten rounds.               */
/* ------------------------------------------------------------------------ */
void oq_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)M0 * c0;
        uint64_t p1 = (uint64_t)M1 * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += W0; k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Random stream of the optional stochastic rounding: key = the 64-bit seed,
 * counter = (floor(j/4) low, floor(j/4) high, step, worker + (stream << 16)),
 * element j takes output word j mod 4; its top 24 bits make U in [0,1). */
float oq_uniform24(uint64_t seed, int64_t j, int64_t step, int32_t worker, int32_t stream)
{
    uint64_t blk = (uint64_t)j >> 2;
    uint32_t ctr[4] = { (uint32_t)blk, (uint32_t)(blk >> 32), (uint32_t)step,
                        (uint32_t)worker + ((uint32_t)stream << 16) };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    oq_philox4x32_10(ctr, key, out);
    return (float)(out[j & 3] >> 8) * 0x1p-24f;
}

/* ------------------------------------------------------------------------ */
/* sizes                                                                     */
/* ------------------------------------------------------------------------ */
static int32_t mu_bits(int32_t k_g)
{
    /* mu ranges over 0 .. k_g+1, i.e. k_g+2 values */
    int32_t w = 0;
    while ((1 << w) < k_g + 2) ++w;
    return w;
}

int32_t oq_grad_code_bits(int32_t k_g) { return 1 + mu_bits(k_g); }

int64_t oq_grad_code_words_segment(int32_t k_g, int64_t n)
{
    int64_t groups = (n + 31) / 32;
    int64_t words = groups * oq_grad_code_bits(k_g);
    return (words + 3) / 4 * 4;          /* next segment starts 16-byte aligned */
}

int64_t oq_grad_code_words(int32_t k_g, const int64_t* seg_off, int32_t L)
{
    int64_t total = 0;
    for (int32_t l = 0; l < L; ++l)
        total += oq_grad_code_words_segment(k_g, seg_off[l + 1] - seg_off[l]);
    return total;
}

int32_t oq_weight_code_bytes_per_elem(int32_t k_x) { return k_x <= 6 ? 1 : 2; }

/* ------------------------------------------------------------------------ */
/* Q_g (Sec. 5.1)                                                            */
/* ------------------------------------------------------------------------ */
/* level mu of the grid G: l_0 = 0, l_mu = 2^(mu-1-k_g) for mu = 1..k_g+1 */
static float level(int32_t k_g, int32_t mu)
{
    return mu == 0 ? 0.0f : ldexpf(1.0f, mu - 1 - k_g);
}

static float ulp_above(float a) { return nextafterf(a, INFINITY) - a; }

float oq_qg_decode(int32_t k_g, float s, uint8_t code)
{
    int32_t w = mu_bits(k_g);
    int32_t mu = code & ((1 << w) - 1);
    int32_t neg = (code >> w) & 1;
    if (mu == 0) return 0.0f;
    float q = s * level(k_g, mu);          /* ||p||_inf times the grid point; exact unless it underflows */
    return neg ? -q : q;
}

/* element-wise part of Q_g once the scale s (finite, > 0) is known */
static void qg_elements(const oq_config* cfg, const float* p, int64_t n, int64_t j0,
                        int64_t step, int32_t worker, float s,
                        uint8_t* code, float* q, uint8_t* tie)
{
    const int32_t k_g = cfg->k_g;
    const int32_t top = k_g + 1;
    const int32_t w = mu_bits(k_g);
    float lv[16], mid[16];                 /* lv[c] = level c; mid[c] = midpoint of levels c-1 and c (exact) */
    for (int32_t c = 0; c <= top + 1; ++c) lv[c] = level(k_g, c <= top ? c : top);
    for (int32_t c = 1; c <= top; ++c) mid[c] = 0.5f * (lv[c - 1] + lv[c]);
    for (int64_t j = 0; j < n; ++j) {
        float r = p[j] / s;                /* g / ||g||_inf */
        float a = fabsf(r);                /* in [0, 1] */
        int32_t mu = 0;
        uint8_t flagged = 0;
        if (cfg->rounding == 0) {
            /* nearest point of G: the largest level whose lower midpoint is <= a
             * (a value on a midpoint goes to the level of larger magnitude) */
            for (int32_t c = top; c >= 1; --c)
                if (a >= mid[c]) { mu = c; break; }
            if (tie) {
                double ulp = (double)ulp_above(a);
                for (int32_t c = 1; c <= top; ++c)
                    if (fabs((double)a - (double)mid[c]) <= ulp) flagged = 1;
            }
        } else {
            /* unbiased rounding between the two neighbours lo <= a < hi */
            if (a >= 1.0f) {
                mu = top;
            } else {
                int32_t below = 0;
                for (int32_t c = top; c >= 1; --c)
                    if (a >= lv[c]) { below = c; break; }
                float lo = lv[below], hi = lv[below + 1];
                float frac = (a - lo) / (hi - lo);
                float U = oq_uniform24(cfg->seed, j0 + j, step, worker, 0);
                mu = below + (U < frac ? 1 : 0);
            }
        }
        int32_t neg = (p[j] < 0.0f) && (mu > 0);
        uint8_t c8 = (uint8_t)((neg << w) | mu);
        if (code) code[j] = c8;
        if (q) {
            float qa = (mu == 0) ? 0.0f : s * lv[mu];
            q[j] = neg ? -qa : qa;
        }
        if (tie) tie[j] = flagged;
    }
}

int oq_qg_layer(const oq_config* cfg, const float* p, int64_t n, int64_t j0,
                int64_t step, int32_t worker,
                float* s_out, uint8_t* code, float* q, uint8_t* tie)
{
    /* s = ||p||_inf */
    float s = 0.0f;
    int saw_nan = 0;
    for (int64_t j = 0; j < n; ++j) {
        float a = fabsf(p[j]);
        if (isnan(a)) saw_nan = 1;
        else if (a > s) s = a;
    }
    if (saw_nan) s = NAN;
    if (s_out) *s_out = s;
    if (!isfinite(s) || s == 0.0f) {
        /* zero layer: every code 0 (so e' = p); non-finite: flagged, same filler */
        for (int64_t j = 0; j < n; ++j) {
            if (code) code[j] = 0;
            if (q) q[j] = 0.0f;
            if (tie) tie[j] = 0;
        }
        return isfinite(s) ? 0 : OQ_NONFINITE_SCALE;
    }
    qg_elements(cfg, p, n, j0, step, worker, s, code, q, tie);
    return 0;
}

/* Q_g on a window of a layer whose scale was obtained separately (used to
 * check sampled windows of layers too large to run whole). */
void oq_qg_window(const oq_config* cfg, const float* p, int64_t n, int64_t j0,
                  int64_t step, int32_t worker, float s,
                  uint8_t* code, float* q, uint8_t* tie)
{
    if (!isfinite(s) || s == 0.0f) {
        for (int64_t j = 0; j < n; ++j) {
            if (code) code[j] = 0;
            if (q) q[j] = 0.0f;
            if (tie) tie[j] = 0;
        }
        return;
    }
    qg_elements(cfg, p, n, j0, step, worker, s, code, q, tie);
}

/* worker side on a window of one layer, the layer's scale s = ||g+e||_inf
 * given: p = g + e, codes of Q_g(p), e <- p - q. */
void oq_worker_quantize_window(const oq_config* cfg, int64_t n, int64_t j0,
                               int32_t worker, int64_t step, float s,
                               const float* grad, float* err,
                               uint8_t* code, uint8_t* tie, float* q_out)
{
    float* p = (float*)calloc((size_t)(n > 0 ? n : 1), sizeof(float));
    float* q = (float*)malloc(sizeof(float) * (size_t)(n > 0 ? n : 1));
    for (int64_t j = 0; j < n; ++j) p[j] = grad[j] + err[j];
    oq_qg_window(cfg, p, n, j0, step, worker, s, code, q, tie);
    for (int64_t j = 0; j < n; ++j) err[j] = p[j] - q[j];
    if (q_out) memcpy(q_out, q, sizeof(float) * (size_t)n);
    free(p); free(q);
}

/* ------------------------------------------------------------------------ */
/* Q_x (Sec. 5.1): 0.5 * nearest point to 2x of {-1, ..., -2^-k_x, 0, 2^-k_x, ..., 1} */
/* i.e. the nearest multiple of 2^-(k_x+1) to x, saturated to [-1/2, 1/2].   */
/* ------------------------------------------------------------------------ */
void oq_qx(const oq_config* cfg, const float* y, int64_t n, int64_t j0, int64_t step,
           int32_t* jcode, float* xhat, uint8_t* tie)
{
    const int32_t k_x = cfg->k_x;
    const float jmax = ldexpf(1.0f, k_x);
    const float per_unit = ldexpf(1.0f, k_x + 1);     /* 1 / grid spacing of Q_x, a power of two */
    const float spacing = ldexpf(1.0f, -(k_x + 1));
    for (int64_t i = 0; i < n; ++i) {
        float u = y[i] * per_unit;         /* 2x in units of the spacing of X; exact scaling */
        float jf;
        uint8_t flagged = 0;
        if (isnan(u)) {
            jf = 0.0f;
        } else {
            if (cfg->rounding == 0) {
                jf = roundf(u);            /* nearest, halves away from zero */
                if (tie && fabsf(u) < 0x1p23f) {
                    double h = floor((double)u) + 0.5;
                    if (fabs((double)u - h) <= (double)ulp_above(fabsf(u))) flagged = 1;
                }
            } else {
                float U = oq_uniform24(cfg->seed, j0 + i, step, 0, 1);
                jf = floorf(u + U);
            }
            if (jf > jmax) jf = jmax;      /* outside [-1/2, 1/2]: saturate */
            if (jf < -jmax) jf = -jmax;
        }
        if (jcode) jcode[i] = (int32_t)jf;
        if (xhat) xhat[i] = jf * spacing;
        if (tie) tie[i] = flagged;
    }
}

/* ------------------------------------------------------------------------ */
/* packed layout of gradient codes                                           */
/* ------------------------------------------------------------------------ */
void oq_pack_codes(int32_t bits, const uint8_t* code, int64_t n, uint32_t* words)
{
    int64_t groups = (n + 31) / 32;
    for (int64_t gidx = 0; gidx < groups; ++gidx) {
        for (int32_t k = 0; k < bits; ++k) {
            uint32_t wv = 0;
            for (int32_t b = 0; b < 32; ++b) {
                int64_t j = gidx * 32 + b;
                if (j < n && ((code[j] >> k) & 1)) wv |= (uint32_t)1 << b;
            }
            words[gidx * bits + k] = wv;
        }
    }
    int64_t used = groups * bits, padded = (used + 3) / 4 * 4;
    for (int64_t t = used; t < padded; ++t) words[t] = 0;
}

void oq_unpack_codes(int32_t bits, const uint32_t* words, int64_t n, uint8_t* code)
{
    for (int64_t j = 0; j < n; ++j) {
        int64_t gidx = j / 32;
        int32_t b = (int32_t)(j % 32);
        uint8_t c = 0;
        for (int32_t k = 0; k < bits; ++k)
            c |= (uint8_t)(((words[gidx * bits + k] >> b) & 1u) << k);
        code[j] = c;
    }
}

/* ------------------------------------------------------------------------ */
/* Adam core: moment recursions and step of Algorithm 1 (= Algorithm 3)      */
/* ------------------------------------------------------------------------ */
void oq_adam_update(const oq_config* cfg, float lr, float beta2, int64_t step,
                    const float* g, float* m, float* v, float* u, int64_t n)
{
    const float beta1 = cfg->beta1, eps = cfg->eps;
    const float omb1 = 1.0f - beta1;
    const float omb2 = 1.0f - beta2;
    float bc1 = 1.0f, sbc2 = 1.0f, lr1 = lr;
    if (cfg->adam_flavor == 1) {
        /* textbook Adam: bias-corrected moments, eps outside the root */
        bc1 = (float)(1.0 - pow((double)beta1, (double)step));
        sbc2 = (float)sqrt(1.0 - pow((double)beta2, (double)step));
        lr1 = lr / bc1;
    }
    for (int64_t j = 0; j < n; ++j) {
        float gj = g[j];
        float g2 = gj * gj;
        float vj = (beta2 * v[j]) + (omb2 * g2);       /* v_t = theta v_{t-1} + (1-theta) g^2 */
        float mj = (beta1 * m[j]) + (omb1 * gj);       /* m_t = beta m_{t-1} + (1-beta) g   */
        v[j] = vj;
        m[j] = mj;
        if (cfg->adam_flavor == 0) {
            float den = sqrtf(vj + eps);               /* sqrt(v_t + eps) */
            u[j] = (lr * mj) / den;                    /* alpha m_t / sqrt(v_t + eps) */
        } else {
            float den = (sqrtf(vj) / sbc2) + eps;
            u[j] = (lr1 * mj) / den;
        }
    }
}

/* ------------------------------------------------------------------------ */
/* the three calls, variant S                                                */
/* ------------------------------------------------------------------------ */
int oq_worker_quantize(const oq_config* cfg, const int64_t* seg_off, int32_t L,
                       int64_t index_base, int32_t worker, int64_t step,
                       const float* grad, float* err,
                       uint32_t* words, uint8_t* code_unpacked, float* scales,
                       uint8_t* tie, float* q_out)
{
    int status = 0;
    const int32_t bits = oq_grad_code_bits(cfg->k_g);
    int64_t word_off = 0;
    for (int32_t l = 0; l < L; ++l) {
        const int64_t a = seg_off[l], n = seg_off[l + 1] - seg_off[l];
        float* p = (float*)calloc((size_t)(n > 0 ? n : 1), sizeof(float));
        float* q = (float*)malloc(sizeof(float) * (size_t)(n > 0 ? n : 1));
        uint8_t* c = (uint8_t*)malloc((size_t)(n > 0 ? n : 1));
        for (int64_t j = 0; j < n; ++j) p[j] = grad[a + j] + err[a + j];     /* g + e */
        float s;
        status |= oq_qg_layer(cfg, p, n, index_base + a, step, worker, &s, c, q,
                              tie ? tie + a : NULL);
        for (int64_t j = 0; j < n; ++j) err[a + j] = p[j] - q[j];            /* e' = p - Q_g(p) */
        if (scales) scales[l] = s;
        if (words) oq_pack_codes(bits, c, n, words + word_off);
        if (code_unpacked) memcpy(code_unpacked + a, c, (size_t)n);
        if (q_out) memcpy(q_out + a, q, sizeof(float) * (size_t)n);
        word_off += oq_grad_code_words_segment(cfg->k_g, n);
        free(p); free(q); free(c);
    }
    return status;
}

/* gbar_j = (sum over workers, in worker order, of q_ij) / N */
static void mean_of_workers(float* acc, int32_t N, int64_t n)
{
    for (int64_t j = 0; j < n; ++j) acc[j] = acc[j] / (float)N;
}

void oq_server_step(const oq_config* cfg, const int64_t* seg_off, int32_t L,
                    int32_t N, int64_t step, float lr, float beta2,
                    const uint32_t* const* words, const float* const* scales,
                    float* x, float* m, float* v)
{
    const int32_t bits = oq_grad_code_bits(cfg->k_g);
    int64_t word_off = 0;
    for (int32_t l = 0; l < L; ++l) {
        const int64_t a = seg_off[l], n = seg_off[l + 1] - seg_off[l];
        float* acc = (float*)calloc((size_t)(n > 0 ? n : 1), sizeof(float));
        float* u = (float*)malloc(sizeof(float) * (size_t)(n > 0 ? n : 1));
        uint8_t* c = (uint8_t*)malloc((size_t)(n > 0 ? n : 1));
        for (int32_t i = 0; i < N; ++i) {
            oq_unpack_codes(bits, words[i] + word_off, n, c);
            float s = scales[i][l];
            for (int64_t j = 0; j < n; ++j) acc[j] = acc[j] + oq_qg_decode(cfg->k_g, s, c[j]);
        }
        mean_of_workers(acc, N, n);
        oq_adam_update(cfg, lr, beta2, step, acc, m + a, v + a, u, n);
        for (int64_t j = 0; j < n; ++j) x[a + j] = x[a + j] - u[j];          /* x - alpha m / sqrt(v+eps) */
        word_off += oq_grad_code_words_segment(cfg->k_g, n);
        free(acc); free(u); free(c);
    }
}

void oq_weight_quantize(const oq_config* cfg, int64_t P, int64_t index_base, int64_t step,
                        const float* x, float* werr, void* wcodes, float* xhat, uint8_t* tie)
{
    float* y = (float*)calloc((size_t)(P > 0 ? P : 1), sizeof(float));
    float* xh = (float*)malloc(sizeof(float) * (size_t)(P > 0 ? P : 1));
    int32_t* jc = (int32_t*)malloc(sizeof(int32_t) * (size_t)(P > 0 ? P : 1));
    for (int64_t j = 0; j < P; ++j)
        y[j] = (cfg->weight_ef && werr) ? x[j] + werr[j] : x[j];
    if (cfg->identity_x) {
        for (int64_t j = 0; j < P; ++j) { xh[j] = y[j]; jc[j] = 0; if (tie) tie[j] = 0; }
    } else {
        oq_qx(cfg, y, P, index_base, step, jc, xh, tie);
    }
    for (int64_t j = 0; j < P; ++j) {
        if (werr) werr[j] = y[j] - xh[j];
        if (xhat) xhat[j] = xh[j];
        if (wcodes && !cfg->identity_x) {
            if (oq_weight_code_bytes_per_elem(cfg->k_x) == 1) ((int8_t*)wcodes)[j] = (int8_t)jc[j];
            else ((int16_t*)wcodes)[j] = (int16_t)jc[j];
        }
    }
    free(y); free(xh); free(jc);
}

/* ------------------------------------------------------------------------ */
/* whole steps                                                               */
/* ------------------------------------------------------------------------ */
/* worker message for one worker: either Q_g with error feedback or, with the
 * oracle-only identity quantizer, the value itself (then e' = 0). */
static int worker_message(const oq_config* cfg, const int64_t* seg_off, int32_t L,
                          int64_t index_base, int32_t worker, int64_t step,
                          const float* value, float* err, uint32_t* words, float* scales,
                          uint8_t* tie, float* q)
{
    const int64_t P = seg_off[L];
    if (cfg->identity_g) {
        for (int64_t j = 0; j < P; ++j) { q[j] = value[j] + err[j]; err[j] = 0.0f; }
        if (tie) memset(tie, 0, (size_t)P);
        return 0;
    }
    return oq_worker_quantize(cfg, seg_off, L, index_base, worker, step, value, err,
                              words, NULL, scales, tie, q);
}

int oq_step_s(const oq_config* cfg, const int64_t* seg_off, int32_t L, int32_t N,
              int64_t index_base, int64_t step, float lr, float beta2,
              const float* const* grads, float* const* errs,
              uint32_t* const* words, float* const* scales,
              float* x, float* m, float* v, float* werr, void* wcodes,
              uint8_t* const* tie_g, uint8_t* tie_x)
{
    const int64_t P = seg_off[L];
    int status = 0;
    float* acc = (float*)calloc((size_t)(P > 0 ? P : 1), sizeof(float));
    float* q = (float*)malloc(sizeof(float) * (size_t)(P > 0 ? P : 1));
    float* u = (float*)malloc(sizeof(float) * (size_t)(P > 0 ? P : 1));
    for (int32_t i = 0; i < N; ++i) {
        status |= worker_message(cfg, seg_off, L, index_base, i, step, grads[i], errs[i],
                                 words ? words[i] : NULL, scales ? scales[i] : NULL,
                                 tie_g ? tie_g[i] : NULL, q);
        for (int64_t j = 0; j < P; ++j) acc[j] = acc[j] + q[j];
    }
    mean_of_workers(acc, N, P);
    oq_adam_update(cfg, lr, beta2, step, acc, m, v, u, P);
    for (int64_t j = 0; j < P; ++j) x[j] = x[j] - u[j];
    oq_weight_quantize(cfg, P, index_base, step, x, werr, wcodes, NULL, tie_x);
    free(acc); free(q); free(u);
    return status;
}

/* The same step on a window of ONE layer, the workers' layer scales s[i] = ||g_i + e_i||_inf given
 * (everything but the scale is element-wise).  codes[i][n]: per-element codes. */
int oq_step_s_window(const oq_config* cfg, int64_t n, int64_t j0, int32_t N,
                     int64_t step, float lr, float beta2, const float* s,
                     const float* const* grads, float* const* errs,
                     float* x, float* m, float* v, float* werr,
                     uint8_t* const* codes, void* wcodes,
                     uint8_t* const* tie_g, uint8_t* tie_x)
{
    float* acc = (float*)calloc((size_t)(n > 0 ? n : 1), sizeof(float));
    float* q = (float*)malloc(sizeof(float) * (size_t)(n > 0 ? n : 1));
    float* u = (float*)malloc(sizeof(float) * (size_t)(n > 0 ? n : 1));
    int status = 0;
    for (int32_t i = 0; i < N; ++i) {
        if (!isfinite(s[i])) status |= OQ_NONFINITE_SCALE;
        oq_worker_quantize_window(cfg, n, j0, i, step, s[i], grads[i], errs[i],
                                  codes ? codes[i] : NULL, tie_g ? tie_g[i] : NULL, q);
        for (int64_t j = 0; j < n; ++j) acc[j] = acc[j] + q[j];
    }
    mean_of_workers(acc, N, n);
    oq_adam_update(cfg, lr, beta2, step, acc, m, v, u, n);
    for (int64_t j = 0; j < n; ++j) x[j] = x[j] - u[j];
    oq_weight_quantize(cfg, n, j0, step, x, werr, wcodes, NULL, tie_x);
    free(acc); free(q); free(u);
    return status;
}

int oq_step_w(const oq_config* cfg, const int64_t* seg_off, int32_t L, int32_t N,
              int64_t index_base, int64_t step, float lr, float beta2,
              const float* const* grads, float* const* errs,
              float* const* mw, float* const* vw,
              uint32_t* const* words, float* const* scales,
              float* x, float* werr, void* wcodes,
              uint8_t* const* tie_g, uint8_t* tie_x)
{
    const int64_t P = seg_off[L];
    int status = 0;
    float* acc = (float*)calloc((size_t)(P > 0 ? P : 1), sizeof(float));
    float* q = (float*)malloc(sizeof(float) * (size_t)(P > 0 ? P : 1));
    float* u = (float*)malloc(sizeof(float) * (size_t)(P > 0 ? P : 1));
    for (int32_t i = 0; i < N; ++i) {
        /* Algorithm 3: local moments, then delta = Q_g(u + e) and e' = u + e - delta */
        oq_adam_update(cfg, lr, beta2, step, grads[i], mw[i], vw[i], u, P);
        status |= worker_message(cfg, seg_off, L, index_base, i, step, u, errs[i],
                                 words ? words[i] : NULL, scales ? scales[i] : NULL,
                                 tie_g ? tie_g[i] : NULL, q);
        for (int64_t j = 0; j < P; ++j) acc[j] = acc[j] + q[j];
    }
    /* Algorithm 2: mean of the messages, then the update, with the descent sign of Algorithm 1 */
    mean_of_workers(acc, N, P);
    for (int64_t j = 0; j < P; ++j) x[j] = x[j] - acc[j];
    oq_weight_quantize(cfg, P, index_base, step, x, werr, wcodes, NULL, tie_x);
    free(acc); free(q); free(u);
    return status;
}
