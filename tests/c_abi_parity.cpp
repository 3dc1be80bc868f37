// Parity of the C boundary WITHOUT Python or torch: a plain host program that allocates with
// hipMalloc, calls the library through include/qadam.h on the default stream and compares every
// output byte with the CPU oracle (liboracle_qadam.so, linked in: this is a test).
// Built and run by tests/test_gpu_c_abi.py.  It also shows the library working against the
// system's HIP runtime alone.  Exit status 0 = all equal.
#include <hip/hip_runtime_api.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "qadam.h"
#include "qadam_oracle.h"

#define HIPCHECK(call)                                                                        \
    do {                                                                                      \
        hipError_t e_ = (call);                                                               \
        if (e_ != hipSuccess) { std::printf("HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__); return 3; } \
    } while (0)
#define QCHECK(call)                                                                          \
    do {                                                                                      \
        int rc_ = (call);                                                                     \
        if (rc_ != QADAM_OK) { std::printf("qadam error %d (%s) at line %d\n", rc_, qadam_last_error(), __LINE__); return 4; } \
    } while (0)

static uint32_t lcg_state = 2463534242u;
static float gauss_like()          // sum of four uniforms, centred: good enough as synthetic input
{
    float s = 0.0f;
    for (int k = 0; k < 4; ++k) {
        lcg_state = lcg_state * 1664525u + 1013904223u;
        s += (float)(lcg_state >> 8) * 0x1p-24f;
    }
    return (s - 2.0f) * 1.7320508f;
}

template <typename T>
static int differs(const char* name, const T* dev, const T* host, size_t n, std::vector<T>& tmp)
{
    tmp.resize(n);
    if (hipMemcpy(tmp.data(), dev, n * sizeof(T), hipMemcpyDeviceToHost) != hipSuccess) return 1;
    if (std::memcmp(tmp.data(), host, n * sizeof(T)) != 0) {
        size_t j = 0;
        while (j < n && std::memcmp(&tmp[j], &host[j], sizeof(T)) == 0) ++j;
        std::printf("MISMATCH in %s at element %zu of %zu\n", name, j, n);
        return 1;
    }
    return 0;
}

int main()
{
    const int64_t sizes[] = { 9408, 64, 7, 36864, 1000, 0, 4097, 300000 };
    const int32_t L = (int32_t)(sizeof sizes / sizeof sizes[0]);
    enum { N = 4 };
    std::vector<int64_t> seg(L + 1, 0);
    for (int l = 0; l < L; ++l) seg[l + 1] = seg[l] + sizes[l];
    const int64_t P = seg[L];

    qadam_config_t cfg;
    std::memset(&cfg, 0, sizeof cfg);
    cfg.struct_size = sizeof cfg; cfg.k_g = 2; cfg.k_x = 6; cfg.rounding = 0; cfg.weight_ef = 1;
    cfg.adam_flavor = 0; cfg.beta1 = 0.9f; cfg.eps = 1e-8f; cfg.seed = 0;
    oq_config ocfg;
    std::memset(&ocfg, 0, sizeof ocfg);
    ocfg.k_g = 2; ocfg.k_x = 6; ocfg.weight_ef = 1; ocfg.beta1 = 0.9f; ocfg.eps = 1e-8f;

    qadam_handle_t h = nullptr;
    QCHECK(qadam_init(&h, &cfg, seg.data(), L, N));
    QCHECK(qadam_trust_error_buffers(h, 2));
    const size_t code_bytes = qadam_grad_code_bytes(h);
    if (code_bytes != (size_t)oq_grad_code_words(2, seg.data(), L) * 4u) { std::printf("code size differs\n"); return 5; }

    // host state (oracle) and device state
    std::vector<float> hx(P), hm(P, 0.f), hv(P, 0.f), hw(P, 0.f);
    std::vector<std::vector<float>> hg(N, std::vector<float>(P)), he(N, std::vector<float>(P, 0.f));
    std::vector<std::vector<uint32_t>> hwords(N, std::vector<uint32_t>(code_bytes / 4));
    std::vector<std::vector<float>> hscales(N, std::vector<float>(L));
    std::vector<int8_t> hwc(P);
    for (int64_t j = 0; j < P; ++j) hx[j] = 0.02f * gauss_like();

    float *dx, *dm, *dv, *dw, *dg[N], *de[N], *dsc[N];
    void* dcodes[N];
    int8_t* dwc;
    HIPCHECK(hipMalloc((void**)&dx, P * 4)); HIPCHECK(hipMalloc((void**)&dm, P * 4));
    HIPCHECK(hipMalloc((void**)&dv, P * 4)); HIPCHECK(hipMalloc((void**)&dw, P * 4));
    HIPCHECK(hipMalloc((void**)&dwc, P));
    HIPCHECK(hipMemcpy(dx, hx.data(), P * 4, hipMemcpyHostToDevice));
    HIPCHECK(hipMemset(dm, 0, P * 4)); HIPCHECK(hipMemset(dv, 0, P * 4)); HIPCHECK(hipMemset(dw, 0, P * 4));
    for (int i = 0; i < N; ++i) {
        HIPCHECK(hipMalloc((void**)&dg[i], P * 4)); HIPCHECK(hipMalloc((void**)&de[i], P * 4));
        HIPCHECK(hipMalloc((void**)&dsc[i], L * 4)); HIPCHECK(hipMalloc(&dcodes[i], code_bytes));
        HIPCHECK(hipMemset(de[i], 0, P * 4));
    }

    std::vector<float> tmpf; std::vector<uint32_t> tmpu; std::vector<int8_t> tmpb;
    int bad = 0;
    for (int64_t step = 1; step <= 4 && !bad; ++step) {
        const float lr = 1e-3f / (float)step, beta2 = 0.999f;
        for (int i = 0; i < N; ++i) {
            for (int64_t j = 0; j < P; ++j) hg[i][j] = (step == 3 ? 1e-4f : 1e-2f) * gauss_like();
            HIPCHECK(hipMemcpy(dg[i], hg[i].data(), P * 4, hipMemcpyHostToDevice));
        }
        const float* grads[N]; float* errs[N]; float* scales[N]; void* codes[N];
        const float* ograds[N]; float* oerrs[N]; uint32_t* owords[N]; float* oscales[N];
        for (int i = 0; i < N; ++i) {
            grads[i] = dg[i]; errs[i] = de[i]; scales[i] = dsc[i]; codes[i] = dcodes[i];
            ograds[i] = hg[i].data(); oerrs[i] = he[i].data(); owords[i] = hwords[i].data(); oscales[i] = hscales[i].data();
        }
        QCHECK(qadam_step_fused(h, step, lr, beta2, grads, errs, codes, scales, dx, dm, dv, dw, dwc, nullptr));
        qadam_status_t st;
        QCHECK(qadam_get_status(h, &st, 0, nullptr));          // synchronises the default stream
        const int ost = oq_step_s(&ocfg, seg.data(), L, N, 0, step, lr, beta2, ograds, oerrs, owords, oscales,
                                  hx.data(), hm.data(), hv.data(), hw.data(), hwc.data(), nullptr, nullptr);
        if (st.flags != 0 || ost != 0) { std::printf("unexpected status %u / %d\n", st.flags, ost); return 6; }
        bad |= differs("x", dx, hx.data(), P, tmpf) | differs("m", dm, hm.data(), P, tmpf) |
               differs("v", dv, hv.data(), P, tmpf) | differs("werr", dw, hw.data(), P, tmpf) |
               differs("wcodes", dwc, hwc.data(), P, tmpb);
        for (int i = 0; i < N; ++i)
            bad |= differs("err", de[i], he[i].data(), P, tmpf) | differs("scales", dsc[i], hscales[i].data(), L, tmpf) |
                   differs("codes", (const uint32_t*)dcodes[i], hwords[i].data(), code_bytes / 4, tmpu);
        std::printf("step %lld: %s\n", (long long)step, bad ? "MISMATCH" : "all outputs equal the oracle's");
        std::fflush(stdout);
    }
    QCHECK(qadam_destroy(h));
    return bad ? 1 : 0;
}
