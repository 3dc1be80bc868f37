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
    bool      need_amax, need_reduce;   // which launches of the scale pass this layer list needs at all
    int       trust_errs;                       // qadam_trust_error_buffers: 0 off, 1 when it pays, 2 always, 3 verify
    bool      bound_valid[QADAM_MAX_WORKERS];   // d_err_bound row i describes what bound_err[i] now holds
    const float* bound_err[QADAM_MAX_WORKERS];  // the error buffer that row was recorded for
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

// qadam_trust_error_buffers(h, 1): smallest number of (tile, worker) pairs of a call for which the filtered
// scale pass, with its two extra launches, is faster than the full one (measured: slower on a 4-worker,
// 11.7 M-parameter vector, 6 % faster on an 8-worker, 124 M-parameter one)
constexpr int64_t kFilterMinTiles = 32768;

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
    L.need_amax = h->need_amax; L.need_reduce = h->need_reduce;
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
    BoundRecord(qadam_ctx* h_, int first_, int num_, const WorkerPtrs& W) : h(h_), first(first_), num(num_), complete(false)
    {
        for (int i = first; i < first + num; ++i) {
            h->bound_valid[i] = false;
            h->bound_err[i] = W.err[i];
        }
    }
    ~BoundRecord()
    {
        for (int i = first; i < first + num; ++i) h->bound_valid[i] = complete;
    }
};

// The recorded bound of worker i can be used for this call: it is valid and was recorded for the very
// buffer the caller passes now (another buffer, e.g. a restored checkpoint, gets the full scale pass).
bool bound_usable(const qadam_ctx* h, int i, const float* err) { return h->bound_valid[i] && h->bound_err[i] == err; }

// Is the stream recording a HIP graph?  A captured call is replayed later with the kernel arguments
// it was recorded with, so what depends on the step number must not be captured.
int stream_capturing(void* stream, bool* capturing)
{
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    QADAM_HIP(hipStreamIsCapturing(static_cast<hipStream_t>(stream), &st));
    *capturing = st != hipStreamCaptureStatusNone;
    return QADAM_OK;
}

// Refuses to record a call whose kernel arguments change from step to step in a way a replay cannot
// follow: the Philox counter (rounding = 1) and the bias corrections (adam_flavor = 1).
int check_capture(const qadam_ctx* h, void* stream, bool* capturing)
{
    QADAM_CHECK(stream_capturing(stream, capturing));
    if (*capturing && (h->cfg.rounding == 1 || h->cfg.adam_flavor == 1))
        return fail(QADAM_EINVAL, "stream is capturing a graph: a replay would reuse this step's random stream "
                                  "(rounding = 1) or bias correction (adam_flavor = 1)");
    return QADAM_OK;
}

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
    h->tile_elems = kDefaultTileElems;

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
    bool need_amax = false, need_reduce = false;
    for (int l = 0; l < num_segments; ++l) {
        seg_tile_begin[l] = (int32_t)tiles.size();
        const int64_t a = seg_offsets[l], n = seg_offsets[l + 1] - a;
        const int64_t seg_words = segment_code_words(h->code_bits, n);
        const int64_t used_words = (n + 31) / 32 * h->code_bits;
        const int64_t layer_tiles = (n + h->tile_elems - 1) / h->tile_elems;
        if (n == 0 || layer_tiles > kMediumLayerTiles) need_reduce = true;   // an empty layer's scale (0) comes from there too
        if (n > kSmallLayerElems) need_amax = true;
        for (int64_t o = 0; o < n; o += h->tile_elems) {
            Tile t;
            t.start = a + o;
            t.code_word = word_off + o / 32 * h->code_bits;
            t.len = (int32_t)((n - o) < h->tile_elems ? (n - o) : h->tile_elems);
            t.seg = l;
            t.flags = (a % 4 != 0) ? kTileUnaligned : 0;
            if (o + h->tile_elems >= n) t.flags |= (int32_t)(seg_words - used_words) << 8;
            t.layer_len = 0;
            if (layer_tiles <= kMediumLayerTiles) t.flags |= kTileMedium;
            if (n <= kSmallLayerElems) {
                // one workgroup (that of the first tile) handles the whole layer; never a sampled tile
                t.flags |= o == 0 ? kTileSmallHead : kTileSmallBody;
                if (o == 0) t.layer_len = (int32_t)n;
            } else {
                if ((o / h->tile_elems) % kSampleStride == 0) {
                    t.flags |= kTileSampled;
                    sample_tiles.push_back((int32_t)tiles.size());
                }
            }
            tiles.push_back(t);
        }
        word_off += seg_words;
    }
    h->code_words = word_off;

    seg_tile_begin[num_segments] = (int32_t)tiles.size();
    h->num_tiles = (int32_t)tiles.size();
    h->num_sample_tiles = (int32_t)sample_tiles.size();
    h->need_amax = need_amax;
    h->need_reduce = need_reduce;

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
    bool capturing = false;
    QADAM_CHECK(check_capture(h, stream, &capturing));
    // a recorded call always takes the full scale pass: a replay must not depend on what ran before it
    const bool recorded = !capturing && bound_usable(h, worker, err_dev);
    const bool filtered = recorded && (h->trust_errs == 2 || (h->trust_errs == 1 && h->num_tiles >= kFilterMinTiles));
    if (h->trust_errs == 3 && recorded) QADAM_HIP(launch_check_error_bounds(L, W, worker, 1));
    BoundRecord record(h, worker, 1, W);
    if (filtered) QADAM_HIP(launch_amax_filtered(L, S, W, worker, 1));
    else QADAM_HIP(launch_amax(L, S, W, worker, 1));
    QADAM_HIP(launch_reduce_scales(L, S, W, worker, 1));
    QADAM_HIP(launch_worker_quantize(L, S, W, worker));
    record.complete = !capturing;       // nothing has run yet when the call was only recorded
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
    bool capturing = false;
    QADAM_CHECK(check_capture(h, stream, &capturing));
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
    bool capturing = false;
    QADAM_CHECK(check_capture(h, stream, &capturing));
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
    bool capturing = false;
    QADAM_CHECK(check_capture(h, stream, &capturing));
    if (h->profile && !capturing) QADAM_HIP(hipEventRecord(h->ev[0], L.stream));
    if (idg) {
        // the error buffers are not touched: whatever is recorded about them stays true
        if (h->profile && !capturing) QADAM_HIP(hipEventRecord(h->ev[1], L.stream));
        QADAM_HIP(launch_plain_messages(L, S, W, sp, false));
    } else {
        // the filtered pass costs two more (small) launches: only worth it from about 10^8 worker-elements on
        bool filtered = h->trust_errs == 2 ||
                        (h->trust_errs == 1 && (int64_t)h->num_tiles * h->num_workers >= kFilterMinTiles);
        bool all_recorded = true;
        for (int i = 0; i < h->num_workers; ++i) all_recorded = all_recorded && bound_usable(h, i, W.err[i]);
        all_recorded = all_recorded && !capturing;     // a recorded call always takes the full scale pass
        filtered = filtered && all_recorded;
        if (h->trust_errs == 3 && all_recorded) QADAM_HIP(launch_check_error_bounds(L, W, 0, h->num_workers));
        BoundRecord record(h, 0, h->num_workers, W);
        if (filtered) QADAM_HIP(launch_amax_filtered(L, S, W, 0, h->num_workers));
        else QADAM_HIP(launch_amax(L, S, W, 0, h->num_workers));
        QADAM_HIP(launch_reduce_scales(L, S, W, 0, h->num_workers));
        if (h->profile && !capturing) QADAM_HIP(hipEventRecord(h->ev[1], L.stream));
        QADAM_HIP(launch_fused(L, S, W, sp));
        record.complete = !capturing;
    }
    if (h->profile && !capturing) {
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
    bool capturing = false;
    QADAM_CHECK(check_capture(h, stream, &capturing));
    // pass 1: local moments, p = alpha m / sqrt(v + eps) + e parked in the error buffer, tile maxima
    BoundRecord record(h, worker, 1, W);
    QADAM_HIP(launch_worker_moments_w(L, S, W, worker, 1));
    QADAM_HIP(launch_reduce_scales(L, S, W, worker, 1));
    // pass 2: quantize the parked p
    W.grad[worker] = nullptr;
    QADAM_HIP(launch_worker_quantize(L, S, W, worker));
    record.complete = !capturing;
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
    bool capturing = false;
    QADAM_CHECK(check_capture(h, stream, &capturing));
    if (h->profile && !capturing) QADAM_HIP(hipEventRecord(h->ev[0], L.stream));
    // pass 1 (all workers): local moments, p parked in the error buffers, tile maxima; then scales
    BoundRecord record(h, 0, h->num_workers, W);
    QADAM_HIP(launch_worker_moments_w(L, S, W, 0, h->num_workers));
    if (!idg) QADAM_HIP(launch_reduce_scales(L, S, W, 0, h->num_workers));
    if (h->profile && !capturing) QADAM_HIP(hipEventRecord(h->ev[1], L.stream));
    // pass 2: quantize every worker's parked p, subtract the mean message, Q_x
    if (idg) QADAM_HIP(launch_plain_messages(L, S, W, sp, true));
    else QADAM_HIP(launch_fused_w(L, S, W, sp));
    record.complete = !idg && !capturing;   // with the identity quantizer no scale, hence no bound, was produced
    if (h->profile && !capturing) {
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

int qadam_arena_layout(qadam_handle_t h, size_t arena_bytes, int32_t with_worker_moments, qadam_arena_t* out)
{
    if (!h) return fail(QADAM_EINVAL, "null handle");
    if (!out) return fail(QADAM_EINVAL, "null layout");
    std::memset(out, 0xff, sizeof *out);            // every entry SIZE_MAX until placed
    const int N = h->num_workers;
    constexpr size_t align = 2u << 20;              // buffers start on 2 MiB boundaries (the driver's large pages)
    auto rup = [](size_t n) { return (n + align - 1) / align * align; };
    const size_t big = rup((size_t)h->num_params * 4u);
    const size_t code = rup(qadam_grad_code_bytes(h));
    const size_t wcode = rup(qadam_weight_code_bytes(h));
    const size_t scale = rup((size_t)h->num_segments * 4u);
    // the buffers in the order they are dealt to the two groups: the read+write streams first, then the
    // read-only gradients, then the small write-only ones
    struct Item { size_t* where; size_t bytes; };
    std::vector<Item> items;
    items.push_back({&out->x, big}); items.push_back({&out->m, big});
    items.push_back({&out->v, big}); items.push_back({&out->werr, big});
    for (int i = 0; i < N; ++i) items.push_back({&out->errs[i], big});
    if (with_worker_moments)
        for (int i = 0; i < N; ++i) { items.push_back({&out->mw[i], big}); items.push_back({&out->vw[i], big}); }
    for (int i = 0; i < N; ++i) items.push_back({&out->grads[i], big});
    for (int i = 0; i < N; ++i) items.push_back({&out->codes[i], code});
    items.push_back({&out->wcodes, wcode});
    for (int i = 0; i < N; ++i) items.push_back({&out->scales[i], scale});
    size_t fill[2] = {0, 0};
    for (size_t k = 0; k < items.size(); ++k) {
        const int grp = (int)(k & 1);
        *items[k].where = fill[grp];                // offset inside the group for now
        fill[grp] += items[k].bytes;
    }
    out->bytes_needed = fill[0] + fill[1];
    if (arena_bytes < out->bytes_needed) return fail(QADAM_ERANGE, "the block is smaller than the buffers");
    // group 1 starts in the middle of the block, or right behind group 0 when the block is that tight
    size_t second = (arena_bytes / 2) / align * align;
    if (second < fill[0]) second = fill[0];
    if (second + fill[1] > arena_bytes) second = fill[0];
    for (size_t k = 1; k < items.size(); k += 2) *items[k].where += second;
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
    // read and clear in stream order, so that they are ordered against the kernels of this stream that
    // OR into the word; work of the handle on OTHER streams must be idle (see the header)
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint32_t word = 0;
    QADAM_HIP(hipMemcpyAsync(&word, h->d_status, sizeof word, hipMemcpyDeviceToHost, s));
    if (clear) QADAM_HIP(hipMemsetAsync(h->d_status, 0, sizeof word, s));
    QADAM_HIP(hipStreamSynchronize(s));
    out->flags = word;
    out->reserved = 0;
    return QADAM_OK;
}

}  // extern "C"
