/*
 * Memory-safety self-test of the CPU oracle (test infrastructure only).
 * Built together with qadam_oracle.c under -fsanitize=address,undefined and run by
 * tests/test_oracle_sanitizers.py: every entry point is driven with ragged segment lists
 * (empty segments, sizes around the 32-element code groups and the 16-byte segment padding),
 * with every buffer allocated at its exact size so that an out-of-bounds access, a misuse of
 * the packed layout's padding or an undefined shift or conversion aborts the run.
 * It checks no values; the pins in tests/test_oracle_*.py do that.
 */
#include "qadam_oracle.h"

#include <stdio.h>
#include <stdlib.h>
#include <string.h>

static uint32_t rng_state = 12345u;
static float rnd(void)
{
    rng_state = rng_state * 1664525u + 1013904223u;
    return ((float)(rng_state >> 8) * 0x1p-24f - 0.5f) * 0.02f;
}

static float* vec(int64_t n, int random)
{
    float* p = (float*)malloc(sizeof(float) * (size_t)(n > 0 ? n : 1));
    for (int64_t j = 0; j < n; ++j) p[j] = random ? rnd() : 0.0f;
    return p;
}

int main(void)
{
    const int64_t sizes[] = { 1, 3, 31, 32, 33, 0, 63, 64, 65, 127, 129, 0, 1000, 4097, 7 };
    const int32_t L = (int32_t)(sizeof sizes / sizeof sizes[0]);
    int64_t seg[sizeof sizes / sizeof sizes[0] + 1];
    seg[0] = 0;
    for (int32_t l = 0; l < L; ++l) seg[l + 1] = seg[l] + sizes[l];
    const int64_t P = seg[L];
    enum { N = 3 };
    int runs = 0;
    for (int32_t k_g = 0; k_g <= 6; ++k_g)
    for (int32_t k_x = 0; k_x <= 14; k_x += 7)
    for (int32_t rounding = 0; rounding <= 1; ++rounding)
    for (int32_t weight_ef = 0; weight_ef <= 1; ++weight_ef) {
        oq_config cfg;
        memset(&cfg, 0, sizeof cfg);
        cfg.k_g = k_g; cfg.k_x = k_x; cfg.rounding = rounding; cfg.weight_ef = weight_ef;
        cfg.adam_flavor = (k_g & 1); cfg.beta1 = 0.9f; cfg.eps = 1e-8f; cfg.seed = 0x123456789abcdefull;
        const int64_t nwords = oq_grad_code_words(k_g, seg, L);
        float *grads[N], *errs[N], *mw[N], *vw[N], *scales[N];
        uint32_t* words[N];
        uint8_t* ties[N];
        for (int i = 0; i < N; ++i) {
            grads[i] = vec(P, 1); errs[i] = vec(P, 1); mw[i] = vec(P, 0); vw[i] = vec(P, 0);
            scales[i] = vec(L, 0);
            words[i] = (uint32_t*)malloc(sizeof(uint32_t) * (size_t)(nwords > 0 ? nwords : 1));
            ties[i] = (uint8_t*)malloc((size_t)P);
        }
        float *x = vec(P, 1), *m = vec(P, 0), *v = vec(P, 0), *werr = vec(P, 0);
        void* wcodes = malloc((size_t)P * (size_t)oq_weight_code_bytes_per_elem(k_x));
        uint8_t* tie_x = (uint8_t*)malloc((size_t)P);
        uint8_t* codes = (uint8_t*)malloc((size_t)P);
        for (int64_t step = 1; step <= 2; ++step) {
            /* the three calls */
            for (int i = 0; i < N; ++i)
                oq_worker_quantize(&cfg, seg, L, 0, i, step, grads[i], errs[i], words[i], codes, scales[i], ties[i], NULL);
            oq_server_step(&cfg, seg, L, N, step, 1e-3f, 0.999f, (const uint32_t* const*)words,
                           (const float* const*)scales, x, m, v);
            oq_weight_quantize(&cfg, P, 0, step, x, werr, wcodes, NULL, tie_x);
            /* whole steps, both variants */
            oq_step_s(&cfg, seg, L, N, 0, step, 1e-3f, 0.999f, (const float* const*)grads, errs, words, scales,
                      x, m, v, werr, wcodes, ties, tie_x);
            oq_step_w(&cfg, seg, L, N, 0, step, 1e-3f, 0.999f, (const float* const*)grads, errs, mw, vw, words,
                      scales, x, werr, wcodes, ties, tie_x);
        }
        /* a window of the largest layer with given scales */
        {
            const int64_t a = seg[13] + 32, n = 1000;
            float s[N];
            const float* gw[N]; float* ew[N]; uint8_t* cw[N]; uint8_t* tw[N];
            for (int i = 0; i < N; ++i) {
                s[i] = 0.01f; gw[i] = grads[i] + a; ew[i] = errs[i] + a;
                cw[i] = (uint8_t*)malloc((size_t)n); tw[i] = (uint8_t*)malloc((size_t)n);
            }
            oq_step_s_window(&cfg, n, a, N, 3, 1e-3f, 0.999f, s, gw, ew, x + a, m + a, v + a, werr + a, cw,
                             (char*)wcodes + a * oq_weight_code_bytes_per_elem(k_x), tw, tie_x + a);
            for (int i = 0; i < N; ++i) { free(cw[i]); free(tw[i]); }
        }
        /* pack / unpack at every ragged length */
        for (int64_t n = 0; n <= 70; ++n) {
            const int32_t bits = oq_grad_code_bits(k_g);
            const int64_t nw = oq_grad_code_words_segment(k_g, n);
            uint8_t* c = (uint8_t*)malloc((size_t)(n > 0 ? n : 1));
            uint8_t* d = (uint8_t*)malloc((size_t)(n > 0 ? n : 1));
            uint32_t* w = (uint32_t*)malloc(sizeof(uint32_t) * (size_t)(nw > 0 ? nw : 1));
            for (int64_t j = 0; j < n; ++j) c[j] = (uint8_t)((j * 7 + 3) & ((1 << bits) - 1));
            oq_pack_codes(bits, c, n, w);
            oq_unpack_codes(bits, w, n, d);
            if (n > 0 && memcmp(c, d, (size_t)n) != 0) { fprintf(stderr, "pack/unpack mismatch at n=%lld\n", (long long)n); return 2; }
            free(c); free(d); free(w);
        }
        for (int i = 0; i < N; ++i) {
            free(grads[i]); free(errs[i]); free(mw[i]); free(vw[i]); free(scales[i]); free(words[i]); free(ties[i]);
        }
        free(x); free(m); free(v); free(werr); free(wcodes); free(tie_x); free(codes);
        ++runs;
    }
    printf("oracle sanitizer self-test: %d configurations, no findings\n", runs);
    return 0;
}
