// Host side of the C boundary declared in include/qadam.h: argument checks, the handle with its
// device-resident tile table, and the sequencing of kernel launches for each call.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "qadam_internal.h"

using namespace qadam;

struct qadam_ctx {
    qadam_config_t cfg;
    int32_t num_workers;
    int32_t num_segments;
    int64_t num_params;
    int32_t mu_bits, code_bits, wcode_bytes;
    int64_t code_words;         // uint32 words of one worker's packed codes
    int32_t tile_elems;
    int     device;
    Tile*     d_tiles;
    int32_t   num_tiles;
    uint32_t* d_status;
    float*    d_inv_scales;     // [num_workers][num_segments]
    uint32_t* d_tile_max;       // [num_workers][num_tiles]
    int32_t*  d_seg_tile_begin; // [num_segments + 1]
    double*   d_tile_sum;       // [num_tiles]
    float*    d_err_bound;      // [num_workers][num_segments]
    uint32_t* d_thr;            // [num_workers][num_segments]
    int32_t*  d_sample_tiles;   // indices of the sampled tiles
    int32_t   num_sample_tiles;
    int       trust_errs;                       // qadam_trust_error_buffers: 0 off, 1 when it pays, 2 always, 3 verify
    bool      bound_valid[QADAM_MAX_WORKERS];   // d_err_bound row i describes what errs[i] now holds
    bool       profile;
    bool       profile_valid;
    hipEvent_t ev[3];
};

namespace {

thread_local char g_last_error[256] = "";

int hip_fail(hipError_t e, const char* what)
{
    std::snprintf(g_last_error, sizeof g_last_error, "%s: %s", what, hipGetErrorString(e));
    return QADAM_EHIP;
}

#define QADAM_HIP(call)                                      \
    do {                                                     \
        hipError_t e_ = (call);                              \
        if (e_ != hipSuccess) return hip_fail(e_, #call);    \
    } while (0)

int fail(int code, const char* msg)
{
    std::snprintf(g_last_error, sizeof g_last_error, "%s", msg);
    return code;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int mu_bits_for(int k_g)
{
    int w = 0;
    while ((1 << w) < k_g + 2) ++w;
    return w;
}

int64_t segment_code_words(int code_bits, int64_t n)
{
    const int64_t words = (n + 31) / 32 * code_bits;
    return (words + 3) / 4 * 4;
}

int tile_elems_from_env()
{
    // tuning knob for experiments; the default is what the library is measured with
    const char* s = std::getenv("QADAM_TILE_ELEMS");
    if (s) {
        const long v = std::strtol(s, nullptr, 10);
        if (v >= 256 && v <= (1 << 20) && v % 256 == 0) return (int)v;
    }
    return 4096;
}

StepScalars make_scalars(const qadam_ctx* h, int64_t step, float lr, float beta2)
{
    StepScalars S;
    std::memset(&S, 0, sizeof S);
    S.num_workers = h->num_workers;
    S.k_g = h->cfg.k_g; S.mu_bits = h->mu_bits; S.code_bits = h->code_bits;
    S.k_x = h->cfg.k_x; S.wcode_bytes = h->wcode_bytes;
    S.rounding = h->cfg.rounding; S.weight_ef = h->cfg.weight_ef; S.adam_flavor = h->cfg.adam_flavor;
    S.key0 = (uint32_t)h->cfg.seed; S.key1 = (uint32_t)(h->cfg.seed >> 32);
    S.step = (uint32_t)step;
    S.lr = lr; S.beta1 = h->cfg.beta1; S.beta2 = beta2; S.eps = h->cfg.eps;
    S.omb1 = 1.0f - h->cfg.beta1;
    S.omb2 = 1.0f - beta2;
    S.lr1 = lr; S.sbc2 = 1.0f;
    if (h->cfg.adam_flavor == 1) {
        const float bc1 = (float)(1.0 - std::pow((double)h->cfg.beta1, (double)step));
        S.sbc2 = (float)std::sqrt(1.0 - std::pow((double)beta2, (double)step));
        S.lr1 = lr / bc1;
    }
    S.n_workers_f = (float)h->num_workers;
    S.n_is_pow2 = (h->num_workers & (h->num_workers - 1)) == 0;
    S.inv_n = 1.0f / (float)h->num_workers;
    return S;
}

Launch make_launch(const qadam_ctx* h, void* stream)
{
    Launch L;
    L.tiles = h->d_tiles; L.inv_scales = h->d_inv_scales;
    L.tile_max = h->d_tile_max; L.seg_tile_begin = h->d_seg_tile_begin; L.tile_sum = h->d_tile_sum;
    L.err_bound = h->d_err_bound; L.thr = h->d_thr;
    L.sample_tiles = h->d_sample_tiles; L.num_sample_tiles = h->num_sample_tiles;
    L.num_tiles = h->num_tiles; L.num_segments = h->num_segments;
    L.num_params = h->num_params; L.status = h->d_status; L.stream = static_cast<hipStream_t>(stream);
    return L;
}

int check_handle(const qadam_ctx* h)
{
    if (!h) return fail(QADAM_EINVAL, "null handle");
    int dev = -1;
    QADAM_HIP(hipGetDevice(&dev));
    if (dev != h->device) return fail(QADAM_EINVAL, "handle belongs to another device");
    return QADAM_OK;
}

int check_ptr(const void* p, const char* name, bool required = true)
{
    if (!p) return required ? fail(QADAM_EINVAL, name) : QADAM_OK;
    if (!aligned16(p)) return fail(QADAM_EALIGN, name);
    return QADAM_OK;
}

#define QADAM_CHECK(expr)                 \
    do {                                  \
        const int rc_ = (expr);           \
        if (rc_ != QADAM_OK) return rc_;  \
    } while (0)

// Record of whether d_err_bound describes the error buffers: cleared for the workers a call is about
// to rewrite, set again only when every launch of the call was accepted (a call that fails half way
// leaves the record cleared, so the next step reads everything).
struct BoundRecord {
    qadam_ctx* h;
    int first, num;
    bool complete;
    BoundRecord(qadam_ctx* h_, int first_, int num_) : h(h_), first(first_), num(num_), complete(false)
    {
        for (int i = first; i < first + num; ++i) h->bound_valid[i] = false;
    }
    ~BoundRecord()
    {
        for (int i = first; i < first + num; ++i) h->bound_valid[i] = complete;
    }
};

bool identity_g(const qadam_ctx* h) { return h->cfg.k_g == QADAM_IDENTITY; }
bool identity_x(const qadam_ctx* h) { return h->cfg.k_x == QADAM_IDENTITY; }

int fill_worker_tables(const qadam_ctx* h, WorkerPtrs& W, const float* const* grads, float* const* errs,
                       void* const* codes, float* const* scales, bool need_grad, bool need_err, bool need_codes)
{
    std::memset(&W, 0, sizeof W);
    if ((need_codes && (!codes || !scales)) || (need_grad && !grads) || (need_err && !errs))
        return fail(QADAM_EINVAL, "null pointer array");
    const bool empty = h->num_params == 0;
    for (int i = 0; i < h->num_workers; ++i) {
        if (need_grad) {
            QADAM_CHECK(check_ptr(grads[i], "grads[i]", !empty));
            W.grad[i] = grads[i];
        }
        if (need_err) {
            QADAM_CHECK(check_ptr(errs[i], "errs[i]", !empty));
            W.err[i] = errs[i];
        }
        if (need_codes) {
            QADAM_CHECK(check_ptr(codes[i], "codes[i]", !empty));
            QADAM_CHECK(check_ptr(scales[i], "scales[i]", h->num_segments > 0));
            W.codes[i] = static_cast<uint32_t*>(codes[i]);
            W.scales[i] = scales[i];
        }
    }
    return QADAM_OK;
}

}  // namespace

extern "C" {

const char* qadam_last_error(void) { return g_last_error; }

int qadam_init(qadam_handle_t* out, const qadam_config_t* cfg, const int64_t* seg_offsets,
               int32_t num_segments, int32_t num_workers)
{
    if (!out || !cfg || !seg_offsets) return fail(QADAM_EINVAL, "null argument");
    *out = nullptr;
    if (cfg->struct_size != sizeof(qadam_config_t)) return fail(QADAM_EINVAL, "config struct_size mismatch");
    if (cfg->k_g != QADAM_IDENTITY && (cfg->k_g < 0 || cfg->k_g > 6))
        return fail(QADAM_EINVAL, "k_g outside 0..6 (or QADAM_IDENTITY)");
    if (cfg->k_x != QADAM_IDENTITY && (cfg->k_x < 0 || cfg->k_x > 14))
        return fail(QADAM_EINVAL, "k_x outside 0..14 (or QADAM_IDENTITY)");
    if ((cfg->rounding | 1) != 1 || (cfg->weight_ef | 1) != 1 || (cfg->adam_flavor | 1) != 1)
        return fail(QADAM_EINVAL, "rounding, weight_ef and adam_flavor are 0 or 1");
    if (!(cfg->beta1 >= 0.0f && cfg->beta1 < 1.0f)) return fail(QADAM_EINVAL, "beta1 outside [0,1)");
    if (!(cfg->eps >= 0.0f)) return fail(QADAM_EINVAL, "eps negative or NaN");
    if (num_workers < 1) return fail(QADAM_EINVAL, "num_workers < 1");
    if (num_workers > QADAM_MAX_WORKERS) return fail(QADAM_ERANGE, "num_workers > QADAM_MAX_WORKERS");
    if (num_segments < 0) return fail(QADAM_EINVAL, "num_segments < 0");
    if (seg_offsets[0] != 0) return fail(QADAM_EINVAL, "seg_offsets[0] != 0");
    for (int l = 0; l < num_segments; ++l)
        if (seg_offsets[l + 1] < seg_offsets[l]) return fail(QADAM_EINVAL, "seg_offsets decreasing");
    const int64_t P = seg_offsets[num_segments];
    if (P > ((int64_t)1 << 40)) return fail(QADAM_ERANGE, "more than 2^40 parameters");

    qadam_ctx* h = new (std::nothrow) qadam_ctx;
    if (!h) return fail(QADAM_EINVAL, "out of host memory");
    std::memset(h, 0, sizeof *h);
    h->cfg = *cfg;
    h->num_workers = num_workers;
    h->num_segments = num_segments;
    h->num_params = P;
    h->mu_bits = cfg->k_g == QADAM_IDENTITY ? 0 : mu_bits_for(cfg->k_g);
    h->code_bits = cfg->k_g == QADAM_IDENTITY ? 0 : 1 + h->mu_bits;       /* 0: no codes are stored */
    h->wcode_bytes = cfg->k_x == QADAM_IDENTITY ? 0 : (cfg->k_x <= 6 ? 1 : 2);
    h->tile_elems = tile_elems_from_env();

    // one workgroup per tile: a launch needs tiles * threads per workgroup below 2^32
    int64_t tile_count = 0;
    for (int l = 0; l < num_segments; ++l)
        tile_count += (seg_offsets[l + 1] - seg_offsets[l] + h->tile_elems - 1) / h->tile_elems;
    if (tile_count >= ((int64_t)1 << 32) / kBlockThreads) {
        delete h;
        return fail(QADAM_ERANGE, "too many tiles for one launch (about parameters / 4096 must stay below 2^24)");
    }

    // tile table: segments cut into runs of tile_elems elements
    std::vector<Tile> tiles;
    tiles.reserve((size_t)tile_count);
    std::vector<int32_t> sample_tiles;
    std::vector<int32_t> seg_tile_begin(num_segments + 1, 0);
    int64_t word_off = 0;
    for (int l = 0; l < num_segments; ++l) {
        seg_tile_begin[l] = (int32_t)tiles.size();
        const int64_t a = seg_offsets[l], n = seg_offsets[l + 1] - a;
        const int64_t seg_words = segment_code_words(h->code_bits, n);
        const int64_t used_words = (n + 31) / 32 * h->code_bits;
        for (int64_t o = 0; o < n; o += h->tile_elems) {
            Tile t;
            t.start = a + o;
            t.code_word = word_off + o / 32 * h->code_bits;
            t.len = (int32_t)((n - o) < h->tile_elems ? (n - o) : h->tile_elems);
            t.seg = l;
            t.flags = (a % 4 != 0) ? kTileUnaligned : 0;
            if (o + h->tile_elems >= n) t.flags |= (int32_t)(seg_words - used_words) << 8;
            if ((o / h->tile_elems) % kSampleStride == 0) {
                t.flags |= kTileSampled;
                sample_tiles.push_back((int32_t)tiles.size());
            }
            t.reserved = 0;
            tiles.push_back(t);
        }
        word_off += seg_words;
    }
    h->code_words = word_off;

    seg_tile_begin[num_segments] = (int32_t)tiles.size();
    h->num_tiles = (int32_t)tiles.size();
    h->num_sample_tiles = (int32_t)sample_tiles.size();

    hipError_t e = hipGetDevice(&h->device);
    // set-up of the allocation-free entry point for this device (address of its static array), so that
    // a caller who created any handle never meets that lookup inside a region that must not allocate
    if (e == hipSuccess) e = noalloc_prepare();
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&h->d_status), 256);
    if (e == hipSuccess) e = hipMemset(h->d_status, 0, 256);
    if (e == hipSuccess && num_segments > 0)
        e = hipMalloc(reinterpret_cast<void**>(&h->d_inv_scales), sizeof(float) * (size_t)num_segments * num_workers);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&h->d_seg_tile_begin), sizeof(int32_t) * (num_segments + 1));
    if (e == hipSuccess)
        e = hipMemcpy(h->d_seg_tile_begin, seg_tile_begin.data(), sizeof(int32_t) * (num_segments + 1), hipMemcpyHostToDevice);
    if (e == hipSuccess && h->num_tiles > 0)
        e = hipMalloc(reinterpret_cast<void**>(&h->d_tile_max), sizeof(uint32_t) * (size_t)h->num_tiles * num_workers);
    if (e == hipSuccess && h->num_tiles > 0)
        e = hipMalloc(reinterpret_cast<void**>(&h->d_tile_sum), sizeof(double) * (size_t)h->num_tiles);
    if (e == hipSuccess && num_segments > 0)
        e = hipMalloc(reinterpret_cast<void**>(&h->d_err_bound), sizeof(float) * (size_t)num_segments * num_workers);
    if (e == hipSuccess && num_segments > 0)
        e = hipMalloc(reinterpret_cast<void**>(&h->d_thr), sizeof(uint32_t) * (size_t)num_segments * num_workers);
    if (e == hipSuccess && h->num_sample_tiles > 0) {
        e = hipMalloc(reinterpret_cast<void**>(&h->d_sample_tiles), sizeof(int32_t) * sample_tiles.size());
        if (e == hipSuccess)
            e = hipMemcpy(h->d_sample_tiles, sample_tiles.data(), sizeof(int32_t) * sample_tiles.size(),
                          hipMemcpyHostToDevice);
    }
    if (e == hipSuccess && h->num_tiles > 0) {
        e = hipMalloc(reinterpret_cast<void**>(&h->d_tiles), sizeof(Tile) * tiles.size());
        if (e == hipSuccess)
            e = hipMemcpy(h->d_tiles, tiles.data(), sizeof(Tile) * tiles.size(), hipMemcpyHostToDevice);
    }
    if (e != hipSuccess) {
        if (h->d_tiles) (void)hipFree(h->d_tiles);
        if (h->d_status) (void)hipFree(h->d_status);
        if (h->d_inv_scales) (void)hipFree(h->d_inv_scales);
        if (h->d_tile_max) (void)hipFree(h->d_tile_max);
        if (h->d_seg_tile_begin) (void)hipFree(h->d_seg_tile_begin);
        if (h->d_tile_sum) (void)hipFree(h->d_tile_sum);
        if (h->d_err_bound) (void)hipFree(h->d_err_bound);
        if (h->d_thr) (void)hipFree(h->d_thr);
        if (h->d_sample_tiles) (void)hipFree(h->d_sample_tiles);
        delete h;
        return hip_fail(e, "qadam_init device tables");
    }
    *out = h;
    return QADAM_OK;
}

int qadam_destroy(qadam_handle_t h)
{
    if (!h) return QADAM_OK;
    for (hipEvent_t& e : h->ev)
        if (e) (void)hipEventDestroy(e);
    if (h->d_tiles) (void)hipFree(h->d_tiles);
    if (h->d_status) (void)hipFree(h->d_status);
    if (h->d_inv_scales) (void)hipFree(h->d_inv_scales);
    if (h->d_tile_max) (void)hipFree(h->d_tile_max);
    if (h->d_seg_tile_begin) (void)hipFree(h->d_seg_tile_begin);
    if (h->d_tile_sum) (void)hipFree(h->d_tile_sum);
    if (h->d_err_bound) (void)hipFree(h->d_err_bound);
    if (h->d_thr) (void)hipFree(h->d_thr);
    if (h->d_sample_tiles) (void)hipFree(h->d_sample_tiles);
    delete h;
    return QADAM_OK;
}

size_t qadam_grad_code_bytes(qadam_handle_t h) { return h ? (size_t)h->code_words * 4u : 0; }
size_t qadam_weight_code_bytes(qadam_handle_t h) { return h ? (size_t)h->num_params * (size_t)h->wcode_bytes : 0; }
int64_t qadam_num_params(qadam_handle_t h) { return h ? h->num_params : 0; }

int qadam_worker_quantize(qadam_handle_t h, int32_t worker, int64_t step, const float* grad_dev,
                          float* err_dev, void* codes_dev, float* scales_dev, void* stream)
{
    QADAM_CHECK(check_handle(h));
    if (identity_g(h)) return fail(QADAM_EINVAL, "the handle has no gradient quantizer (k_g = QADAM_IDENTITY)");
    if (worker < 0 || worker >= h->num_workers) return fail(QADAM_EINVAL, "worker out of range");
    if (step < 1) return fail(QADAM_EINVAL, "step < 1");
    const bool empty = h->num_params == 0;
    QADAM_CHECK(check_ptr(grad_dev, "grad_dev", !empty));
    QADAM_CHECK(check_ptr(err_dev, "err_dev", !empty));
    QADAM_CHECK(check_ptr(codes_dev, "codes_dev", !empty));
    QADAM_CHECK(check_ptr(scales_dev, "scales_dev", h->num_segments > 0));
    WorkerPtrs W;
    std::memset(&W, 0, sizeof W);
    W.grad[worker] = grad_dev; W.err[worker] = err_dev;
    W.codes[worker] = static_cast<uint32_t*>(codes_dev); W.scales[worker] = scales_dev;
    const StepScalars S = make_scalars(h, step, 0.0f, 0.0f);
    const Launch L = make_launch(h, stream);
    const bool filtered = h->bound_valid[worker] &&
                          (h->trust_errs == 2 || (h->trust_errs == 1 && h->num_tiles >= 4096));
    if (h->trust_errs == 3 && h->bound_valid[worker]) QADAM_HIP(launch_check_error_bounds(L, W, worker, 1));
    BoundRecord record(h, worker, 1);
    if (filtered) QADAM_HIP(launch_amax_filtered(L, S, W, worker, 1));
    else QADAM_HIP(launch_amax(L, S, W, worker, 1));
    QADAM_HIP(launch_reduce_scales(L, S, W, worker, 1));
    QADAM_HIP(launch_worker_quantize(L, S, W, worker));
    record.complete = true;
    return QADAM_OK;
}

int qadam_quantize_segment_noalloc(int32_t k_g, int64_t n, const float* grad_dev, float* err_dev,
                                   void* codes_dev, float* scale_dev, void* stream)
{
    if (k_g < 0 || k_g > 6) return fail(QADAM_EINVAL, "k_g outside 0..6");
    if (n < 0) return fail(QADAM_EINVAL, "n < 0");
    if (n > kNoallocMaxElems)
        return fail(QADAM_ERANGE, "segment longer than QADAM_NOALLOC_MAX_ELEMS: use a handle (qadam_worker_quantize)");
    QADAM_CHECK(check_ptr(grad_dev, "grad_dev", n > 0));
    QADAM_CHECK(check_ptr(err_dev, "err_dev", n > 0));
    QADAM_CHECK(check_ptr(codes_dev, "codes_dev", n > 0));
    QADAM_CHECK(check_ptr(scale_dev, "scale_dev", true));
    StepScalars S;
    std::memset(&S, 0, sizeof S);
    S.num_workers = 1;
    S.k_g = k_g; S.mu_bits = mu_bits_for(k_g); S.code_bits = 1 + S.mu_bits;
    S.step = 1;
    S.n_workers_f = 1.0f; S.inv_n = 1.0f; S.n_is_pow2 = 1;
    QADAM_HIP(noalloc_quantize_segment(S, n, grad_dev, err_dev, static_cast<uint32_t*>(codes_dev), scale_dev,
                                       static_cast<hipStream_t>(stream)));
    return QADAM_OK;
}

int qadam_server_step(qadam_handle_t h, int64_t step, float lr, float beta2, const void* const* codes,
                      const float* const* scales, float* x_dev, float* m_dev, float* v_dev, void* stream)
{
    QADAM_CHECK(check_handle(h));
    if (identity_g(h)) return fail(QADAM_EINVAL, "the handle has no gradient quantizer (k_g = QADAM_IDENTITY)");
    if (step < 1) return fail(QADAM_EINVAL, "step < 1");
    const bool empty = h->num_params == 0;
    WorkerPtrs W;
    QADAM_CHECK(fill_worker_tables(h, W, nullptr, nullptr, const_cast<void* const*>(codes),
                                   const_cast<float* const*>(scales), false, false, true));
    QADAM_CHECK(check_ptr(x_dev, "x_dev", !empty));
    QADAM_CHECK(check_ptr(m_dev, "m_dev", !empty));
    QADAM_CHECK(check_ptr(v_dev, "v_dev", !empty));
    ServerPtrs sp;
    sp.x = x_dev; sp.m = m_dev; sp.v = v_dev; sp.werr = nullptr; sp.wcodes = nullptr;
    const StepScalars S = make_scalars(h, step, lr, beta2);
    QADAM_HIP(launch_server_step(make_launch(h, stream), S, W, sp));
    return QADAM_OK;
}

int qadam_weight_quantize(qadam_handle_t h, int64_t step, const float* x_dev, float* werr_dev,
                          void* wcodes_dev, void* stream)
{
    QADAM_CHECK(check_handle(h));
    if (identity_x(h)) return fail(QADAM_EINVAL, "the handle has no weight quantizer (k_x = QADAM_IDENTITY)");
    if (step < 1) return fail(QADAM_EINVAL, "step < 1");
    const bool empty = h->num_params == 0;
    QADAM_CHECK(check_ptr(x_dev, "x_dev", !empty));
    QADAM_CHECK(check_ptr(werr_dev, "werr_dev", !empty && h->cfg.weight_ef == 1));
    QADAM_CHECK(check_ptr(wcodes_dev, "wcodes_dev", !empty));
    const StepScalars S = make_scalars(h, step, 0.0f, 0.0f);
    QADAM_HIP(launch_weight_quantize(make_launch(h, stream), S, x_dev, werr_dev, wcodes_dev));
    return QADAM_OK;
}

int qadam_weight_dequantize(qadam_handle_t h, const void* wcodes_dev, float* xhat_dev, void* stream)
{
    QADAM_CHECK(check_handle(h));
    if (identity_x(h)) return fail(QADAM_EINVAL, "the handle has no weight quantizer (k_x = QADAM_IDENTITY)");
    const bool empty = h->num_params == 0;
    QADAM_CHECK(check_ptr(wcodes_dev, "wcodes_dev", !empty));
    QADAM_CHECK(check_ptr(xhat_dev, "xhat_dev", !empty));
    const StepScalars S = make_scalars(h, 1, 0.0f, 0.0f);
    QADAM_HIP(launch_weight_dequantize(make_launch(h, stream), S, wcodes_dev, xhat_dev, false));
    return QADAM_OK;
}

int qadam_weight_dequantize_f16(qadam_handle_t h, const void* wcodes_dev, void* xhat_dev, void* stream)
{
    QADAM_CHECK(check_handle(h));
    if (identity_x(h)) return fail(QADAM_EINVAL, "the handle has no weight quantizer (k_x = QADAM_IDENTITY)");
    const bool empty = h->num_params == 0;
    QADAM_CHECK(check_ptr(wcodes_dev, "wcodes_dev", !empty));
    QADAM_CHECK(check_ptr(xhat_dev, "xhat_dev", !empty));
    const StepScalars S = make_scalars(h, 1, 0.0f, 0.0f);
    QADAM_HIP(launch_weight_dequantize(make_launch(h, stream), S, wcodes_dev, xhat_dev, true));
    return QADAM_OK;
}

int qadam_step_fused(qadam_handle_t h, int64_t step, float lr, float beta2, const float* const* grads,
                     float* const* errs, void* const* codes, float* const* scales, float* x_dev,
                     float* m_dev, float* v_dev, float* werr_dev, void* wcodes_dev, void* stream)
{
    QADAM_CHECK(check_handle(h));
    if (step < 1) return fail(QADAM_EINVAL, "step < 1");
    const bool empty = h->num_params == 0;
    WorkerPtrs W;
    const bool idg = identity_g(h), idx = identity_x(h);
    QADAM_CHECK(fill_worker_tables(h, W, grads, errs, codes, scales, true, !idg, !idg));
    QADAM_CHECK(check_ptr(x_dev, "x_dev", !empty));
    QADAM_CHECK(check_ptr(m_dev, "m_dev", !empty));
    QADAM_CHECK(check_ptr(v_dev, "v_dev", !empty));
    QADAM_CHECK(check_ptr(werr_dev, "werr_dev", !empty && !idx && h->cfg.weight_ef == 1));
    QADAM_CHECK(check_ptr(wcodes_dev, "wcodes_dev", !empty && !idx));
    ServerPtrs sp;
    sp.x = x_dev; sp.m = m_dev; sp.v = v_dev;
    sp.werr = idx ? nullptr : werr_dev; sp.wcodes = idx ? nullptr : wcodes_dev;
    const StepScalars S = make_scalars(h, step, lr, beta2);
    const Launch L = make_launch(h, stream);
    if (h->profile) QADAM_HIP(hipEventRecord(h->ev[0], L.stream));
    if (idg) {
        // the error buffers are not touched: whatever is recorded about them stays true
        if (h->profile) QADAM_HIP(hipEventRecord(h->ev[1], L.stream));
        QADAM_HIP(launch_plain_messages(L, S, W, sp, false));
    } else {
        // the filtered pass costs two more (small) launches: only worth it beyond a few million worker-elements
        bool filtered = h->trust_errs == 2 ||
                        (h->trust_errs == 1 && (int64_t)h->num_tiles * h->num_workers >= 4096);
        bool all_recorded = true;
        for (int i = 0; i < h->num_workers; ++i) all_recorded = all_recorded && h->bound_valid[i];
        filtered = filtered && all_recorded;
        if (h->trust_errs == 3 && all_recorded) QADAM_HIP(launch_check_error_bounds(L, W, 0, h->num_workers));
        BoundRecord record(h, 0, h->num_workers);
        if (filtered) QADAM_HIP(launch_amax_filtered(L, S, W, 0, h->num_workers));
        else QADAM_HIP(launch_amax(L, S, W, 0, h->num_workers));
        QADAM_HIP(launch_reduce_scales(L, S, W, 0, h->num_workers));
        if (h->profile) QADAM_HIP(hipEventRecord(h->ev[1], L.stream));
        QADAM_HIP(launch_fused(L, S, W, sp));
        record.complete = true;
    }
    if (h->profile) {
        QADAM_HIP(hipEventRecord(h->ev[2], L.stream));
        h->profile_valid = true;
    }
    return QADAM_OK;
}

int qadam_worker_step_w(qadam_handle_t h, int32_t worker, int64_t step, float lr, float beta2,
                        const float* grad_dev, float* mw_dev, float* vw_dev, float* err_dev,
                        void* codes_dev, float* scales_dev, void* stream)
{
    QADAM_CHECK(check_handle(h));
    if (identity_g(h)) return fail(QADAM_EINVAL, "the handle has no gradient quantizer (k_g = QADAM_IDENTITY)");
    if (worker < 0 || worker >= h->num_workers) return fail(QADAM_EINVAL, "worker out of range");
    if (step < 1) return fail(QADAM_EINVAL, "step < 1");
    const bool empty = h->num_params == 0;
    QADAM_CHECK(check_ptr(grad_dev, "grad_dev", !empty));
    QADAM_CHECK(check_ptr(mw_dev, "mw_dev", !empty));
    QADAM_CHECK(check_ptr(vw_dev, "vw_dev", !empty));
    QADAM_CHECK(check_ptr(err_dev, "err_dev", !empty));
    QADAM_CHECK(check_ptr(codes_dev, "codes_dev", !empty));
    QADAM_CHECK(check_ptr(scales_dev, "scales_dev", h->num_segments > 0));
    WorkerPtrs W;
    std::memset(&W, 0, sizeof W);
    W.grad[worker] = grad_dev; W.err[worker] = err_dev; W.mw[worker] = mw_dev; W.vw[worker] = vw_dev;
    W.codes[worker] = static_cast<uint32_t*>(codes_dev); W.scales[worker] = scales_dev;
    const StepScalars S = make_scalars(h, step, lr, beta2);
    const Launch L = make_launch(h, stream);
    // pass 1: local moments, p = alpha m / sqrt(v + eps) + e parked in the error buffer, tile maxima
    BoundRecord record(h, worker, 1);
    QADAM_HIP(launch_worker_moments_w(L, S, W, worker, 1));
    QADAM_HIP(launch_reduce_scales(L, S, W, worker, 1));
    // pass 2: quantize the parked p
    W.grad[worker] = nullptr;
    QADAM_HIP(launch_worker_quantize(L, S, W, worker));
    record.complete = true;
    return QADAM_OK;
}

int qadam_step_fused_w(qadam_handle_t h, int64_t step, float lr, float beta2, const float* const* grads,
                       float* const* mw, float* const* vw, float* const* errs, void* const* codes,
                       float* const* scales, float* x_dev, float* werr_dev, void* wcodes_dev, void* stream)
{
    QADAM_CHECK(check_handle(h));
    if (step < 1) return fail(QADAM_EINVAL, "step < 1");
    if (!mw || !vw) return fail(QADAM_EINVAL, "null pointer array");
    const bool empty = h->num_params == 0;
    WorkerPtrs W;
    const bool idg = identity_g(h), idx = identity_x(h);
    QADAM_CHECK(fill_worker_tables(h, W, grads, errs, codes, scales, true, true, !idg));
    for (int i = 0; i < h->num_workers; ++i) {
        QADAM_CHECK(check_ptr(mw[i], "mw[i]", !empty));
        QADAM_CHECK(check_ptr(vw[i], "vw[i]", !empty));
        W.mw[i] = mw[i]; W.vw[i] = vw[i];
    }
    QADAM_CHECK(check_ptr(x_dev, "x_dev", !empty));
    QADAM_CHECK(check_ptr(werr_dev, "werr_dev", !empty && !idx && h->cfg.weight_ef == 1));
    QADAM_CHECK(check_ptr(wcodes_dev, "wcodes_dev", !empty && !idx));
    ServerPtrs sp;
    sp.x = x_dev; sp.m = nullptr; sp.v = nullptr;
    sp.werr = idx ? nullptr : werr_dev; sp.wcodes = idx ? nullptr : wcodes_dev;
    const StepScalars S = make_scalars(h, step, lr, beta2);
    const Launch L = make_launch(h, stream);
    if (h->profile) QADAM_HIP(hipEventRecord(h->ev[0], L.stream));
    // pass 1 (all workers): local moments, p parked in the error buffers, tile maxima; then scales
    BoundRecord record(h, 0, h->num_workers);
    QADAM_HIP(launch_worker_moments_w(L, S, W, 0, h->num_workers));
    if (!idg) QADAM_HIP(launch_reduce_scales(L, S, W, 0, h->num_workers));
    if (h->profile) QADAM_HIP(hipEventRecord(h->ev[1], L.stream));
    // pass 2: quantize every worker's parked p, subtract the mean message, Q_x
    if (idg) QADAM_HIP(launch_plain_messages(L, S, W, sp, true));
    else QADAM_HIP(launch_fused_w(L, S, W, sp));
    record.complete = !idg;     // with the identity quantizer no scale, hence no bound, was produced
    if (h->profile) {
        QADAM_HIP(hipEventRecord(h->ev[2], L.stream));
        h->profile_valid = true;
    }
    return QADAM_OK;
}

int qadam_server_apply_w(qadam_handle_t h, int64_t step, const void* const* codes,
                         const float* const* scales, float* x_dev, void* stream)
{
    QADAM_CHECK(check_handle(h));
    if (identity_g(h)) return fail(QADAM_EINVAL, "the handle has no gradient quantizer (k_g = QADAM_IDENTITY)");
    if (step < 1) return fail(QADAM_EINVAL, "step < 1");
    WorkerPtrs W;
    QADAM_CHECK(fill_worker_tables(h, W, nullptr, nullptr, const_cast<void* const*>(codes),
                                   const_cast<float* const*>(scales), false, false, true));
    QADAM_CHECK(check_ptr(x_dev, "x_dev", h->num_params != 0));
    const StepScalars S = make_scalars(h, step, 0.0f, 0.0f);
    QADAM_HIP(launch_server_apply_w(make_launch(h, stream), S, W, x_dev));
    return QADAM_OK;
}

int qadam_layer_sumsq(qadam_handle_t h, const float* a_dev, const float* b_dev, double* out_dev, void* stream)
{
    QADAM_CHECK(check_handle(h));
    QADAM_CHECK(check_ptr(a_dev, "a_dev", h->num_params != 0));
    QADAM_CHECK(check_ptr(b_dev, "b_dev", false));
    QADAM_CHECK(check_ptr(out_dev, "out_dev", h->num_segments > 0));
    QADAM_HIP(launch_layer_sumsq(make_launch(h, stream), a_dev, b_dev, out_dev));
    return QADAM_OK;
}

int qadam_trust_error_buffers(qadam_handle_t h, int32_t on)
{
    QADAM_CHECK(check_handle(h));
    if (on < 0 || on > 3) return fail(QADAM_EINVAL, "on must be 0, 1, 2 or 3");
    h->trust_errs = on;
    for (bool& b : h->bound_valid) b = false;     // the next step reads everything and starts the record
    return QADAM_OK;
}

int qadam_profile_enable(qadam_handle_t h, int32_t on)
{
    QADAM_CHECK(check_handle(h));
    if (on) {
        for (hipEvent_t& e : h->ev)
            if (!e) QADAM_HIP(hipEventCreate(&e));
    }
    h->profile = on != 0;
    h->profile_valid = false;
    return QADAM_OK;
}

int qadam_profile_read(qadam_handle_t h, qadam_profile_t* out)
{
    QADAM_CHECK(check_handle(h));
    if (!out) return fail(QADAM_EINVAL, "null profile");
    if (!h->profile || !h->profile_valid) return fail(QADAM_EINVAL, "no profiled call to read");
    QADAM_HIP(hipEventSynchronize(h->ev[2]));
    QADAM_HIP(hipEventElapsedTime(&out->scale_pass_ms, h->ev[0], h->ev[1]));
    QADAM_HIP(hipEventElapsedTime(&out->main_pass_ms, h->ev[1], h->ev[2]));
    return QADAM_OK;
}

int qadam_get_status(qadam_handle_t h, qadam_status_t* out, int32_t clear, void* stream)
{
    QADAM_CHECK(check_handle(h));
    if (!out) return fail(QADAM_EINVAL, "null status");
    hipStream_t s = static_cast<hipStream_t>(stream);
    QADAM_HIP(hipStreamSynchronize(s));
    uint32_t word = 0;
    QADAM_HIP(hipMemcpy(&word, h->d_status, sizeof word, hipMemcpyDeviceToHost));
    out->flags = word;
    out->reserved = 0;
    if (clear) QADAM_HIP(hipMemset(h->d_status, 0, sizeof word));
    return QADAM_OK;
}

}  // extern "C"
