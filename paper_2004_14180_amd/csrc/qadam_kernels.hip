// gfx950 (MI355X, CDNA4) kernels of the Quantized-Adam-with-error-feedback step
// (arXiv 2004.14180: Sec. 5.1 for the quantizers Q_g and Q_x, Algorithm 1 for the
// moments / step / residual, Algorithm 2 (gather step) for the mean over workers).
//
// Everything here is a streaming pass bound by HBM bandwidth: no contraction, no MFMA.  The design
// rules are the ones that matter for that regime on CDNA4:
//   * 64-wide wavefronts, 256-thread workgroups; a lane owns 4 consecutive fp32 values so every
//     global access is a 128-bit load/store and a wavefront touches 1 KiB of contiguous memory;
//     all buffers are touched once per pass, so loads and stores carry the non-temporal hint;
//   * a workgroup owns one tile (<= 4096 elements of one layer), so all per-layer quantities
//     (scales, code offsets) are wave-uniform and live in scalar registers;
//   * the loads of a group of workers are issued together before any arithmetic, so a wavefront
//     keeps 16-20 KiB in flight and few wavefronts per SIMD suffice to cover HBM latency;
//   * the per-layer scale is a max over |g+e|: lanes reduce with integer max on the bit pattern
//     (non-negative floats order like integers; NaN/Inf sort above every finite value and so
//     surface in the scale), wavefront reduction by cross-lane shuffles, LDS across the four
//     wavefronts, one plain store of the tile's maximum; the tile maxima of a layer are folded by a
//     second small kernel (layers of more than 640 tiles) or by the quantizing workgroups themselves
//     (smaller layers: the few maxima sit in L2, and the launch is saved).  No atomics: thousands of
//     workgroups hitting one freshly zeroed word at the start of every layer cost more than the whole pass;
//   * a layer of at most 16384 elements is done by ONE workgroup, scale included: g and e are read
//     once from memory (the quantizing phase finds them in cache), no scale pass is needed for it;
//   * a segment that starts off the 16-byte grid keeps the same lane-to-element mapping (the codes are
//     anchored at the segment start) and moves its data with dword-aligned 128-bit accesses;
//   * when the error buffers are what the previous step wrote, |e| <= s/4 (half the widest gap of
//     the grid), so an element whose |g| lies that far below a known lower bound of the scale
//     cannot be the maximum: the filtered scale pass takes the exact maxima of every 64th tile as
//     that lower bound and then reads g alone, and e only for the few elements that can matter;
//   * codes are stored as bit planes of 32-element groups; a lane's four codes are combined with
//     the other seven lanes of its group by three DPP OR steps per plane, so packing costs no
//     LDS traffic and no scatter;
//   * fp32 arithmetic is kept bit-reproducible: one rounding per operation (built with
//     -ffp-contract=off), IEEE division and square root, subnormals kept.  The quotient p/s that
//     selects the grid level is taken as p * (1/s) and redone with the IEEE division only when it
//     lands within 8 ulp of a decision threshold, which cannot change any decision (the product
//     is within 2.5 ulp of the correctly rounded quotient).
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include <cstring>
#include <mutex>

#include "qadam_internal.h"

namespace qadam {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef short s4 __attribute__((ext_vector_type(4)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));
typedef uint32_t u2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t f2u(float f) { return __float_as_uint(f); }
__device__ __forceinline__ float u2f(uint32_t u) { return __uint_as_float(u); }

// ------------------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11): counter (c0..c3), key (k0,k1) -> four 32-bit words.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&out)[4])
{
    constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(M0, c0), lo0 = M0 * c0;
        const uint32_t hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
        c0 = hi1 ^ c1 ^ k0;
        c1 = lo1;
        c2 = hi0 ^ c3 ^ k1;
        c3 = lo0;
        k0 += W0;
        k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Uniforms in [0,1) with 24 bits for the V consecutive elements starting at global index gi.
// Counter = (gi/4 low, gi/4 high, step, worker + (stream << 16)); element j takes word j mod 4.
template <int V>
__device__ __forceinline__ void uniforms(const StepScalars& S, int64_t gi, uint32_t worker, uint32_t stream,
                                         float (&U)[V])
{
    const uint64_t blk = (uint64_t)gi >> 2;
    uint32_t out[4];
    philox4x32_10((uint32_t)blk, (uint32_t)(blk >> 32), S.step, worker + (stream << 16), S.key0, S.key1, out);
    if constexpr (V == 4) {
#pragma unroll
        for (int j = 0; j < 4; ++j) U[j] = (float)(out[j] >> 8) * 0x1p-24f;
    } else {
        const int wsel = (int)(gi & 3);
        const uint32_t w = wsel == 0 ? out[0] : wsel == 1 ? out[1] : wsel == 2 ? out[2] : out[3];
        U[0] = (float)(w >> 8) * 0x1p-24f;
    }
}

// ------------------------------------------------------------------------------------------------
// Q_g on one value (Sec. 5.1).  r = p / s lies in [-1, 1]; the grid is {0} and 2^(mu-1-k_g),
// mu = 1..k_g+1.  Nearest point: the midpoint below level 2^-j is 0.75 * 2^-j, i.e. mantissa
// 0x400000 one exponent lower, so adding 0x400000 to the bit pattern of |r| and keeping the
// exponent field rounds |r| to the nearest power of two with midpoints going up.  Below the first
// level 2^-k_g the only midpoint is 2^(-k_g-1) (halfway to zero).
// ------------------------------------------------------------------------------------------------
struct QgConst {
    int ebias;             // 126 - k_g: exponent field of level mu is mu + ebias
    uint32_t half_l1_bits; // bit pattern of 2^(-k_g-1)
    uint32_t l1_bits;      // bit pattern of 2^-k_g
};

__device__ __forceinline__ QgConst make_qg(int k_g)
{
    QgConst c;
    c.ebias = 126 - k_g;
    c.half_l1_bits = (uint32_t)(126 - k_g) << 23;
    c.l1_bits = (uint32_t)(127 - k_g) << 23;
    return c;
}

// bit pattern of the grid point nearest to |r| (0 for the zero level); `zero_below` is
// half_l1_bits, or 0xffffffff to force every level to zero (invalid scale)
__device__ __forceinline__ uint32_t qg_nearest_bits(uint32_t ab, const QgConst& c, uint32_t zero_below)
{
    uint32_t lvl = (ab + 0x00400000u) & 0x7f800000u;
    lvl = lvl > c.l1_bits ? lvl : c.l1_bits;
    lvl = lvl < 0x3f800000u ? lvl : 0x3f800000u;
    return ab >= zero_below ? lvl : 0u;
}

// unbiased choice between the neighbours lo <= |r| < hi: up with probability (|r|-lo)/(hi-lo)
__device__ __forceinline__ uint32_t qg_stochastic_bits(uint32_t ab, const QgConst& c, float U, bool valid)
{
    if (ab >= 0x3f800000u) return valid ? 0x3f800000u : 0u;
    uint32_t lo = ab & 0x7f800000u;                         // largest power of two <= |r|
    lo = lo >= c.l1_bits ? lo : 0u;                         // below the first level the lower neighbour is 0
    const uint32_t width = lo ? lo : c.l1_bits;             // hi - lo, a power of two
    const float inv_width = u2f((254u << 23) - width);      // exact reciprocal
    const float frac = (u2f(ab) - u2f(lo)) * inv_width;
    const uint32_t hi = lo ? lo + (1u << 23) : c.l1_bits;
    const uint32_t lvl = U < frac ? hi : lo;
    return valid ? lvl : 0u;
}

// One worker's share of one lane: p = g + e, level, dequantized value q, residual p - q, and the
// V codes (4 bits each) of the lane.  s is the layer scale, inv_s its reciprocal or 0 when the
// fast quotient must not be used (tiny, huge, zero or non-finite scale).
template <int V, int ROUNDING>
__device__ __forceinline__ void worker_lane(const float (&g)[V], const float (&e)[V], float s, float inv_s,
                                            const QgConst& c, int mu_bits, const float (&U)[V],
                                            float (&q)[V], float (&enew)[V], uint32_t& codes)
{
    float p[V], r[V];
#pragma unroll
    for (int j = 0; j < V; ++j) p[j] = g[j] + e[j];
    const bool valid = s > 0.0f && s < __builtin_inff();
    if (ROUNDING == 0 && inv_s != 0.0f) {
        uint32_t near = 0;
#pragma unroll
        for (int j = 0; j < V; ++j) {
            r[j] = p[j] * inv_s;
            // within 8 ulp of a power of two or of 0.75 times one?
            const uint32_t t = (f2u(r[j]) & 0x7fffffffu) + 0x00400000u;
            near |= (((t + 8u) & 0x003fffffu) < 16u) ? 1u : 0u;
        }
        if (near) {
#pragma unroll
            for (int j = 0; j < V; ++j) r[j] = p[j] / s;
        }
    } else {
#pragma unroll
        for (int j = 0; j < V; ++j) r[j] = p[j] / s;
    }
    const uint32_t zero_below = valid ? c.half_l1_bits : 0xffffffffu;
    const float s_mul = valid ? s : 0.0f;               // an invalid scale quantizes everything to 0
    const int sign_shift = 31 - mu_bits;
    codes = 0;
#pragma unroll
    for (int j = 0; j < V; ++j) {
        const uint32_t ab = f2u(r[j]) & 0x7fffffffu;
        uint32_t lvl;
        if constexpr (ROUNDING == 0) lvl = qg_nearest_bits(ab, c, zero_below);
        else lvl = qg_stochastic_bits(ab, c, U[j], valid);
        const float qa = s_mul * u2f(lvl);                // s * 2^(mu-1-k_g); 0 when lvl == 0
        const uint32_t sign = f2u(p[j]) & 0x80000000u;
        const float qv = u2f(f2u(qa) | sign);
        q[j] = qv;
        enew[j] = p[j] - qv;
        const int mu = max((int)(lvl >> 23) - c.ebias, 0);
        const uint32_t code = mu > 0 ? ((uint32_t)mu | (sign >> sign_shift)) : 0u;
        codes |= code << (4 * j);
    }
}

// Value of the code stored at bit `pos` of a 32-element group's plane words w[0..MU_BITS]
// (planes 0..MU_BITS-1 hold the level index mu, plane MU_BITS the sign), with layer scale s:
// +-s * 2^(mu-1-k_g), or 0 for mu == 0.  The bits are taken straight from the words, so no
// per-element code has to be assembled first.
template <int MU_BITS>
__device__ __forceinline__ float qg_decode_planes(const uint32_t (&w)[4], uint32_t pos, float s, const QgConst& c)
{
    uint32_t mu = __builtin_amdgcn_ubfe(w[0], pos, 1u);
#pragma unroll
    for (int k = 1; k < MU_BITS; ++k) mu |= __builtin_amdgcn_ubfe(w[k], pos, 1u) << k;
    const uint32_t sign = (w[MU_BITS] << (31u - pos)) & 0x80000000u;
    const float lvl = u2f((mu + (uint32_t)c.ebias) << 23);
    float qa = s * lvl;
    qa = mu > 0u ? qa : 0.0f;
    return u2f(f2u(qa) | sign);
}

// ------------------------------------------------------------------------------------------------
// Bit-plane packing.  A lane holds the codes of elements 4*lane..4*lane+3 of a 256-element
// wave chunk as four nibbles of `codes`; the 8 lanes 8G..8G+7 form 32-element group G.  For plane k
// every lane gathers its 4 plane bits (a multiply moves bits 0,4,8,12 to bits 9..12), shifts them
// to position 4*(lane%8) and the group ORs them with three DPP steps (swap within pairs, swap
// pairs within quads, mirror the two quads of a half row).  Lane 8G+k keeps word k.  Must be
// called with all 64 lanes active.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t dpp_or8(uint32_t w)
{
    w |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w, 0xB1, 0xF, 0xF, false);   // quad_perm [1,0,3,2]
    w |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w, 0x4E, 0xF, 0xF, false);   // quad_perm [2,3,0,1]
    w |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w, 0x141, 0xF, 0xF, false);  // row_half_mirror
    return w;
}

template <int V>
__device__ __forceinline__ uint32_t pack_planes(uint32_t codes, int code_bits, int lane, int& word_slot,
                                                bool& writes)
{
    uint32_t sel = 0;
    if constexpr (V == 4) {
        const int sub = lane & 7;
        const int sh = sub * 4;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (k < code_bits) {
                const uint32_t t = codes & (0x1111u << k);
                const uint32_t nib = ((t * 0x249u) >> (9 + k)) & 0xFu;
                const uint32_t w = dpp_or8(nib << sh);
                sel = sub == k ? w : sel;
            }
        }
        word_slot = (lane >> 3) * code_bits + sub;     // word within the wave chunk's 8 groups
        writes = sub < code_bits;
    }
    return sel;
}

// plane words of the 32-element group that holds this lane's V elements, and the bit position of
// the lane's first element in them (inverse of pack_planes)
template <int V, int MU_BITS>
__device__ __forceinline__ uint32_t load_planes(const uint32_t* __restrict__ chunk_words, int lane, uint32_t (&w)[4])
{
    constexpr int CODE_BITS = MU_BITS + 1;
    static_assert(V == 4, "a lane owns four consecutive elements");
    const uint32_t* gw = chunk_words + (lane >> 3) * CODE_BITS;
#pragma unroll
    for (int k = 0; k < 4; ++k) w[k] = k < CODE_BITS ? gw[k] : 0u;
    return (uint32_t)(lane & 7) * 4u;
}

// ------------------------------------------------------------------------------------------------
// guarded vector access: one 128-bit non-temporal access when the lane's V=4 elements are all
// inside the tile (every buffer is streamed exactly once per pass)
// ------------------------------------------------------------------------------------------------
template <int V, bool STREAMING = true>
__device__ __forceinline__ void load_v(const float* __restrict__ p, int nvalid, float (&out)[V])
{
    if constexpr (V == 4) {
        if (nvalid == 4) {
            // STREAMING = false: the data is read again shortly (small layers), so no non-temporal hint
            const f4 t = STREAMING ? __builtin_nontemporal_load(reinterpret_cast<const f4*>(p))
                                   : *reinterpret_cast<const f4*>(p);
            out[0] = t.x; out[1] = t.y; out[2] = t.z; out[3] = t.w;
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) out[j] = j < nvalid ? p[j] : 0.0f;
        }
    } else {
        out[0] = nvalid > 0 ? p[0] : 0.0f;
    }
}

template <int V>
__device__ __forceinline__ void store_v(float* __restrict__ p, int nvalid, const float (&in)[V])
{
    if constexpr (V == 4) {
        if (nvalid == 4) {
            f4 t;
            t.x = in[0]; t.y = in[1]; t.z = in[2]; t.w = in[3];
            __builtin_nontemporal_store(t, reinterpret_cast<f4*>(p));
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) if (j < nvalid) p[j] = in[j];
        }
    } else {
        if (nvalid > 0) p[0] = in[0];
    }
}

template <int V>
__device__ __forceinline__ void store_wcodes(void* __restrict__ base, int wcode_bytes, int64_t gi, int nvalid,
                                             const int (&j)[V])
{
    if (wcode_bytes == 1) {
        int8_t* p = static_cast<int8_t*>(base) + gi;
        if constexpr (V == 4) {
            if (nvalid == 4) {
                const uint32_t packed = ((uint32_t)j[0] & 0xFFu) | (((uint32_t)j[1] & 0xFFu) << 8) |
                                        (((uint32_t)j[2] & 0xFFu) << 16) | ((uint32_t)j[3] << 24);
                __builtin_nontemporal_store(packed, reinterpret_cast<uint32_t*>(p));
                return;
            }
        }
#pragma unroll
        for (int t = 0; t < V; ++t) if (t < nvalid) p[t] = (int8_t)j[t];
    } else {
        int16_t* p = static_cast<int16_t*>(base) + gi;
        if constexpr (V == 4) {
            if (nvalid == 4) {
                s4 t;
                t.x = (short)j[0]; t.y = (short)j[1]; t.z = (short)j[2]; t.w = (short)j[3];
                __builtin_nontemporal_store(t, reinterpret_cast<s4*>(p));
                return;
            }
        }
#pragma unroll
        for (int t = 0; t < V; ++t) if (t < nvalid) p[t] = (int16_t)j[t];
    }
}

// ------------------------------------------------------------------------------------------------
// Tiles of a segment that does not start on a 16-byte boundary.  The packed codes are anchored at the
// segment start (a lane's four elements are four consecutive bits of a plane word), so a lane's four
// values lie r = (flat start mod 4) floats off the 16-byte grid of memory.  The lane still moves them
// with ONE 128-bit access: the vector type below carries 4-byte alignment, for which the compiler emits
// the same global_load/store_dwordx4 (the memory unit of this target accepts dword-aligned wide
// accesses); a wavefront's access is still one contiguous 1 KiB run, it merely touches nine 128-byte
// lines instead of eight.  The weight codes (four int8 or int16) are stored likewise through types of
// element alignment.  What differs besides is the random stream of stochastic rounding, which is
// indexed by the flat element number (below).
// ------------------------------------------------------------------------------------------------
typedef f4 f4_a4 __attribute__((aligned(4)));
typedef uint32_t u32_a1 __attribute__((aligned(1)));
typedef s4 s4_a2 __attribute__((aligned(2)));

struct Shift {
    int r;              // flat index of the tile's first element mod 4 (1..3 when used)
};

__device__ __forceinline__ Shift make_shift(const Tile& t)
{
    Shift sf;
    sf.r = (int)(t.start & 3);
    return sf;
}

__device__ __forceinline__ void load_shifted(const float* __restrict__ p, int nvalid, float (&out)[4])
{
    if (nvalid == 4) {
        const f4 t = *reinterpret_cast<const f4_a4*>(p);
        out[0] = t.x; out[1] = t.y; out[2] = t.z; out[3] = t.w;
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) out[j] = j < nvalid ? p[j] : 0.0f;
    }
}

__device__ __forceinline__ void store_shifted(float* __restrict__ p, int nvalid, const float (&in)[4])
{
    if (nvalid == 4) {
        f4 t;
        t.x = in[0]; t.y = in[1]; t.z = in[2]; t.w = in[3];
        __builtin_nontemporal_store(t, reinterpret_cast<f4_a4*>(p));
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) if (j < nvalid) p[j] = in[j];
    }
}

// weight codes of the lane's four elements at element index gi (not a multiple of 4)
__device__ __forceinline__ void store_wcodes_shifted(void* __restrict__ base, int wcode_bytes, int64_t gi, int nvalid,
                                                     const int (&j)[4])
{
    if (wcode_bytes == 1) {
        int8_t* p = static_cast<int8_t*>(base) + gi;
        if (nvalid == 4) {
            const uint32_t packed = ((uint32_t)j[0] & 0xFFu) | (((uint32_t)j[1] & 0xFFu) << 8) |
                                    (((uint32_t)j[2] & 0xFFu) << 16) | ((uint32_t)j[3] << 24);
            __builtin_nontemporal_store(packed, reinterpret_cast<u32_a1*>(p));
            return;
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) if (t < nvalid) p[t] = (int8_t)j[t];
    } else {
        int16_t* p = static_cast<int16_t*>(base) + gi;
        if (nvalid == 4) {
            s4 t;
            t.x = (short)j[0]; t.y = (short)j[1]; t.z = (short)j[2]; t.w = (short)j[3];
            __builtin_nontemporal_store(t, reinterpret_cast<s4_a2*>(p));
            return;
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) if (t < nvalid) p[t] = (int16_t)j[t];
    }
}

// uniforms of four consecutive elements that start r into a Philox block: words r..3 of the block
// of gi and words 0..r-1 of the next one
__device__ __forceinline__ void uniforms_shifted(const StepScalars& S, int64_t gi, uint32_t worker, uint32_t stream,
                                                 int r, float (&U)[4])
{
    float lo[4], hi[4];
    uniforms<4>(S, gi - r, worker, stream, lo);
    uniforms<4>(S, gi - r + 4, worker, stream, hi);
    const bool r1 = r == 1, r2 = r == 2;
    U[0] = r1 ? lo[1] : (r2 ? lo[2] : lo[3]);
    U[1] = r1 ? lo[2] : (r2 ? lo[3] : hi[0]);
    U[2] = r1 ? lo[3] : (r2 ? hi[0] : hi[1]);
    U[3] = r1 ? hi[0] : (r2 ? hi[1] : hi[2]);
}

// the accessors of the tile loops: SH selects the shifted forms
template <int V, bool SH>
__device__ __forceinline__ void ld(const float* __restrict__ buf, int64_t gi, int nvalid, const Shift& sf, float (&out)[V])
{
    if constexpr (SH) load_shifted(buf + gi, nvalid, out);
    else load_v<V>(buf + gi, nvalid, out);
}

template <int V, bool SH>
__device__ __forceinline__ void st(float* __restrict__ buf, int64_t gi, int nvalid, const Shift& sf, const float (&in)[V])
{
    if constexpr (SH) store_shifted(buf + gi, nvalid, in);
    else store_v<V>(buf + gi, nvalid, in);
}

template <int V, bool SH>
__device__ __forceinline__ void stw(void* __restrict__ base, int wcode_bytes, int64_t gi, int nvalid, const Shift& sf,
                                    const int (&j)[V])
{
    if constexpr (SH) store_wcodes_shifted(base, wcode_bytes, gi, nvalid, j);
    else store_wcodes<V>(base, wcode_bytes, gi, nvalid, j);
}

template <int V, bool SH>
__device__ __forceinline__ void unif(const StepScalars& S, int64_t gi, uint32_t worker, uint32_t stream, const Shift& sf,
                                     float (&U)[V])
{
    if constexpr (SH) uniforms_shifted(S, gi, worker, stream, sf.r, U);
    else uniforms<V>(S, gi, worker, stream, U);
}

// ------------------------------------------------------------------------------------------------
// Server arithmetic on one lane: moments (Alg. 1, moment recursions) and the step alpha m / sqrt(v + eps).
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ float adam_step(const StepScalars& S, float gbar, float& m, float& v)
{
    const float g2 = gbar * gbar;
    const float vn = (S.beta2 * v) + (S.omb2 * g2);
    const float mn = (S.beta1 * m) + (S.omb1 * gbar);
    v = vn;
    m = mn;
    if (S.adam_flavor == 0) {
        const float den = sqrtf(vn + S.eps);
        return (S.lr * mn) / den;
    } else {
        const float den = (sqrtf(vn) / S.sbc2) + S.eps;
        return (S.lr1 * mn) / den;
    }
}

__device__ __forceinline__ float mean_over_workers(const StepScalars& S, float acc)
{
    // N a power of two: multiplying by the exact 1/N rounds exactly like dividing by N
    return S.n_is_pow2 ? acc * S.inv_n : acc / S.n_workers_f;
}

// Q_x on one value (Sec. 5.1): nearest multiple of 2^-(k_x+1), saturated to [-1/2, 1/2].
template <int ROUNDING>
__device__ __forceinline__ void qx_value(float y, float two_kx1, float inv_two_kx1, float jmax, float U,
                                         int& j, float& xhat)
{
    const float u = y * two_kx1;
    float jf;
    if constexpr (ROUNDING == 0) {
        const float t = truncf(u);
        const float d = fabsf(u - t);                   // exact
        jf = d >= 0.5f ? t + copysignf(1.0f, u) : t;     // halves away from zero
    } else {
        jf = floorf(u + U);
    }
    jf = fminf(fmaxf(jf, -jmax), jmax);
    jf = (u != u) ? 0.0f : jf;
    j = (int)jf;
    xhat = jf * inv_two_kx1;
}

template <int V, int ROUNDING, bool SH = false>
__device__ __forceinline__ void weight_lane(const StepScalars& S, const float (&x)[V], const float (&werr_in)[V],
                                            int64_t gi, const Shift& sf, float (&werr_out)[V], int (&j)[V])
{
    const float two_kx1 = u2f((uint32_t)(127 + S.k_x + 1) << 23);
    const float inv = u2f((uint32_t)(127 - S.k_x - 1) << 23);
    const float jmax = u2f((uint32_t)(127 + S.k_x) << 23);
    float U[V];
#pragma unroll
    for (int t = 0; t < V; ++t) U[t] = 0.0f;
    if constexpr (ROUNDING == 1) unif<V, SH>(S, gi, 0u, 1u, sf, U);
#pragma unroll
    for (int t = 0; t < V; ++t) {
        const float y = S.weight_ef ? x[t] + werr_in[t] : x[t];
        float xh;
        qx_value<ROUNDING>(y, two_kx1, inv, jmax, U[t], j[t], xh);
        werr_out[t] = y - xh;
    }
}

// ------------------------------------------------------------------------------------------------
// kernel argument blocks
// ------------------------------------------------------------------------------------------------
struct AmaxArgs {
    const Tile* tiles;
    int num_tiles;
    const float* grad[QADAM_MAX_WORKERS];
    const float* err[QADAM_MAX_WORKERS];
    uint32_t* tile_max;     // [N][num_tiles]
    int first_worker;
    const int32_t* tile_list;   // null: workgroup b takes tile b; else tile tile_list[b] (the sampled tiles)
    const uint32_t* thr;        // filtered pass only: [N][L] thresholds on |g| as bit patterns (0: read everything)
    int num_segments;
    const float* err_bound;     // verification only: [N][L] bounds the error buffers must respect
    uint32_t* status;
    int64_t seg_len;            // tiles == null only: length of the single segment
    int skip_small;             // non-zero: tiles of small layers are left to the quantizing kernel
};

struct FusedArgs {
    const Tile* tiles;
    int num_tiles;
    uint32_t* status;
    float* inv_scales;            // [N][L]
    float* err_bound;             // [N][L], written for small and medium layers (the scale kernel writes the others)
    float bound_factor;
    const uint32_t* tile_max;     // [N][num_tiles]
    const int32_t* seg_tile_begin;
    int num_segments;
    StepScalars S;
    ServerPtrs sp;
    const float* grad[QADAM_MAX_WORKERS];
    float* err[QADAM_MAX_WORKERS];
    uint32_t* codes[QADAM_MAX_WORKERS];
    float* scales[QADAM_MAX_WORKERS];
};

struct WorkerArgs {        // one worker
    const Tile* tiles;
    int num_tiles;
    uint32_t* status;
    StepScalars S;
    const float* grad;     // variant S: g;  variant W second pass: null (p was parked in err)
    float* err;
    uint32_t* codes;
    float* scales;
    float* inv_scales;         // this worker's row
    float* err_bound;          // this worker's row, written for small and medium layers
    float bound_factor;
    const uint32_t* tile_max;  // this worker's row
    const int32_t* seg_tile_begin;
    int worker;
    int64_t seg_len;           // tiles == null only: length of the single segment
};

// Tile record of workgroup `ti`: from the handle's table, or, for the handle-free single-segment
// call (tiles == null), computed from the segment length: tile ti covers elements
// [ti * kDefaultTileElems, ...) of a segment that starts 16-byte aligned at element 0.
__device__ __forceinline__ Tile tile_at(const Tile* __restrict__ tiles, int ti, int64_t seg_len, int code_bits)
{
    if (tiles) return tiles[ti];
    Tile t;
    t.start = (int64_t)ti * kDefaultTileElems;
    t.code_word = (int64_t)ti * (kDefaultTileElems / 32) * code_bits;
    const int64_t left = seg_len - t.start;
    t.len = (int32_t)(left < kDefaultTileElems ? left : kDefaultTileElems);
    t.seg = 0;
    t.flags = 0;
    if (left <= kDefaultTileElems) {
        const int64_t used = (seg_len + 31) / 32 * code_bits;
        t.flags = (int32_t)((used + 3) / 4 * 4 - used) << 8;     // zero words up to a multiple of 16 bytes
    }
    t.layer_len = 0;
    return t;
}

struct ScaleArgs {
    float* scales[QADAM_MAX_WORKERS];
    float* inv_scales;
    const uint32_t* tile_max;
    const int32_t* seg_tile_begin;
    int first_worker, num_segments, num_tiles;
    float* err_bound;       // [N][L]: bound on |e'| after the step that uses these scales
    uint32_t* thr;          // [N][L]: thresholds of the filtered pass (written by k_reduce_lower_bounds)
    float bound_factor;     // |e'| <= bound_factor * s for this quantizer and rounding mode
    int sample_stride;      // every sample_stride-th tile of a layer is a sampled tile
    const Tile* tiles;      // to recognise the layers whose scales the quantizing kernel folds itself (null: none)
};

// ------------------------------------------------------------------------------------------------
// scales: per-tile max |g + e| (k_amax), then per (worker, layer) the max over the layer's tiles
// and its reciprocal for the fast quotient (k_reduce_scales)
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const uint32_t o = (uint32_t)__shfl_xor((int)v, d, 64);
        v = o > v ? o : v;
    }
    return v;
}

// block-wide max of the lanes' values; thread 0 gets the result
__device__ __forceinline__ uint32_t block_max(uint32_t local)
{
    __shared__ uint32_t wave_part[kBlockThreads / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t wm = wave_max_u32(local);
    if (lane == 0) wave_part[wave] = wm;
    __syncthreads();
    uint32_t bm = wave_part[0];
#pragma unroll
    for (int w = 1; w < kBlockThreads / 64; ++w) bm = wave_part[w] > bm ? wave_part[w] : bm;
    return bm;
}

// max |g + e| (g == null: max |e|) over the flat range [start, start + len) wherever it begins: a
// maximum does not care which lane sees which element, so the range is walked as the aligned quads of
// memory it contains plus at most three single elements at either end.  thr != 0: e is read only for
// quads (elements) whose |g| reaches thr (filtered scale pass).
template <bool STREAMING>
__device__ __forceinline__ uint32_t amax_range(const float* __restrict__ g, const float* __restrict__ e,
                                               int64_t start, int len, uint32_t thr)
{
    const int64_t end = start + len;
    int64_t a0 = (start + 3) & ~(int64_t)3;
    a0 = a0 < end ? a0 : end;
    int64_t a1 = end & ~(int64_t)3;
    a1 = a1 > a0 ? a1 : a0;
    uint32_t local = 0;
    const int head = (int)(a0 - start), tail = (int)(end - a1);
    if ((int)threadIdx.x < head + tail) {
        const int64_t idx = (int)threadIdx.x < head ? start + threadIdx.x : a1 + ((int)threadIdx.x - head);
        const float gv = g ? g[idx] : 0.0f;
        if (thr == 0u || (f2u(gv) & 0x7fffffffu) >= thr) {
            const uint32_t ab = f2u(gv + e[idx]) & 0x7fffffffu;
            local = ab;
        }
    }
    // four quads per lane per trip, their loads issued together (a tile holds at most 1024 quads)
    for (int64_t q0 = a0 + (int64_t)threadIdx.x * 4; q0 < a1; q0 += kBlockThreads * 16) {
        float gv[4][4], ev[4][4];
        bool live[4], cand[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int64_t q = q0 + (int64_t)k * kBlockThreads * 4;
            live[k] = q < a1;
#pragma unroll
            for (int j = 0; j < 4; ++j) { gv[k][j] = 0.0f; ev[k][j] = 0.0f; }
            if (live[k] && g) load_v<4, STREAMING>(g + q, 4, gv[k]);
            if (live[k] && thr == 0u) load_v<4, STREAMING>(e + q, 4, ev[k]);
        }
        if (thr != 0u) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                uint32_t top = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t ab = f2u(gv[k][j]) & 0x7fffffffu;
                    top = ab > top ? ab : top;
                }
                cand[k] = live[k] && top >= thr;
                if (cand[k]) load_v<4, STREAMING>(e + q0 + (int64_t)k * kBlockThreads * 4, 4, ev[k]);
            }
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (thr == 0u ? live[k] : cand[k]) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t ab = f2u(gv[k][j] + ev[k][j]) & 0x7fffffffu;
                    local = ab > local ? ab : local;
                }
            }
        }
    }
    return local;
}

// ---- small layers: the scales are taken by the quantizing workgroup itself -----------------------
struct SmallLayerShared {
    uint32_t part[QADAM_MAX_WORKERS][kBlockThreads / 64];
    float scale[QADAM_MAX_WORKERS];
    float inv[QADAM_MAX_WORKERS];
};

// max |g + e| over the n elements of a layer that start at flat index `start`, over this wavefront's
// share; the loads carry no streaming hint because the quantizing phase reads the same lines again
template <int V>
__device__ __forceinline__ uint32_t small_layer_wave_max(const float* __restrict__ g, const float* __restrict__ e,
                                                         int64_t start, int n)
{
    uint32_t local = 0;
    for (int off = threadIdx.x * V; off < n; off += kBlockThreads * V) {
        const int nvalid = min(n - off, V);
        float gv[V], ev[V];
        load_v<V, false>(g + start + off, nvalid, gv);
        load_v<V, false>(e + start + off, nvalid, ev);
#pragma unroll
        for (int j = 0; j < V; ++j) {
            const uint32_t ab = f2u(gv[j] + ev[j]) & 0x7fffffffu;
            local = ab > local ? ab : local;
        }
    }
    return wave_max_u32(local);
}

// After every wavefront has stored its part for workers first..first+count-1: thread k folds the parts of
// worker first+k into the scale and its reciprocal (the same two operations k_reduce_scales performs),
// keeps them in LDS for the workgroup and writes scale, reciprocal and residual bound to global memory.
__device__ __forceinline__ void small_layer_finish(SmallLayerShared& sh, int first, int count, int seg, int num_segments,
                                                   float* const* scales, float* inv_scales, float* err_bound,
                                                   float bound_factor, bool per_worker_rows, bool write_global = true)
{
    __syncthreads();
    if ((int)threadIdx.x < count) {
        const int i = first + (int)threadIdx.x;
        uint32_t bm = sh.part[i][0];
#pragma unroll
        for (int w = 1; w < kBlockThreads / 64; ++w) bm = sh.part[i][w] > bm ? sh.part[i][w] : bm;
        const float s = u2f(bm);
        const bool ok = s >= 0x1p-100f && s <= 0x1p100f;
        const float inv = ok ? 1.0f / s : 0.0f;
        sh.scale[i] = s;
        sh.inv[i] = inv;
        if (write_global) {
            // per_worker_rows: the table pointers address worker i's row; else row i of an [N][L] table
            const size_t row = per_worker_rows ? 0 : (size_t)i * num_segments;
            scales[per_worker_rows ? 0 : i][seg] = s;
            inv_scales[row + seg] = inv;
            err_bound[row + seg] = s * bound_factor + 0x1p-140f;
        }
    }
    __syncthreads();
}

// this wavefront's share of the max over the tile maxima [t0, t1) of one worker (medium layers)
__device__ __forceinline__ uint32_t medium_layer_wave_max(const uint32_t* __restrict__ tile_max_row, int t0, int t1)
{
    uint32_t local = 0;
    for (int t = t0 + (int)threadIdx.x; t < t1; t += kBlockThreads) {
        const uint32_t v = tile_max_row[t];
        local = v > local ? v : local;
    }
    return wave_max_u32(local);
}

// grid: (layers, workers).  One workgroup folds the tile maxima of its (worker, layer).
__global__ void __launch_bounds__(kBlockThreads) k_reduce_scales(ScaleArgs A)
{
    const int l = blockIdx.x, w = A.first_worker + blockIdx.y;
    // no table: a single segment that owns every tile
    const int t0 = A.seg_tile_begin ? A.seg_tile_begin[l] : 0;
    const int t1 = A.seg_tile_begin ? A.seg_tile_begin[l + 1] : A.num_tiles;
    if (A.tiles && t1 > t0 && (A.tiles[t0].flags & kTileMedium)) return;
    const uint32_t* part = A.tile_max + (size_t)w * A.num_tiles;
    uint32_t local = 0;
    for (int t = t0 + threadIdx.x; t < t1; t += kBlockThreads) {
        const uint32_t v = part[t];
        local = v > local ? v : local;
    }
    const uint32_t bm = block_max(local);
    if (threadIdx.x == 0) {
        const float s = u2f(bm);
        A.scales[w][l] = s;
        // 1/s must be a normal number with full precision for the error bound of the fast quotient
        const bool ok = s >= 0x1p-100f && s <= 0x1p100f;
        A.inv_scales[(size_t)w * A.num_segments + l] = ok ? 1.0f / s : 0.0f;
        // what the residual p - Q_g(p) of this step can reach (a non-finite scale gives a non-finite
        // bound, which switches the next step's filter off)
        // bound on the next |e|; the added 2^-140 covers scales so small that s * level itself is rounded
        A.err_bound[(size_t)w * A.num_segments + l] = s * A.bound_factor + 0x1p-140f;
    }
}

// Filtered scale pass, stage 2 of 4.  grid: (layers, workers).  The sampled tiles (every
// sample_stride-th of a layer) have their exact maxima: their max is a lower bound LB of the
// layer's scale.  With |e_j| <= B (the bound left by the previous step), an element with
// |g_j| < LB - B has |g_j + e_j| < LB and cannot be the maximum, so the next stage reads e only
// where |g_j| >= thr = (LB - B) minus a safety margin that covers the rounding of g + e.
__global__ void __launch_bounds__(kBlockThreads) k_reduce_lower_bounds(ScaleArgs A)
{
    const int l = blockIdx.x, w = A.first_worker + blockIdx.y;
    const int t0 = A.seg_tile_begin[l], t1 = A.seg_tile_begin[l + 1];
    if (t1 > t0 && (A.tiles[t0].flags & kTileSmallHead)) return;
    const uint32_t* part = A.tile_max + (size_t)w * A.num_tiles;
    uint32_t local = 0;
    for (int t = t0 + (int)threadIdx.x * A.sample_stride; t < t1; t += kBlockThreads * A.sample_stride) {
        const uint32_t v = part[t];
        local = v > local ? v : local;
    }
    const uint32_t bm = block_max(local);
    if (threadIdx.x == 0) {
        const float lb = u2f(bm);
        const float bound = A.err_bound[(size_t)w * A.num_segments + l];
        const float thr = (lb - bound * 1.001f) * 0.999f;
        const bool usable = thr > 0.0f && thr < __builtin_inff() && lb < __builtin_inff();
        A.thr[(size_t)w * A.num_segments + l] = usable ? f2u(thr) : 0u;
    }
}

template <int V>
__device__ __forceinline__ uint32_t amax_tile(const float* __restrict__ g, const float* __restrict__ e, const Tile& t)
{
    constexpr int BLOCK_ELEMS = kBlockThreads * V;
    uint32_t local = 0;
    if constexpr (V == 4) {
        if (t.len == 4 * BLOCK_ELEMS) {
            // full 4096-element tile: all eight loads of the lane in flight at once
            float gv[4][4], ev[4][4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                load_v<4>(g + t.start + k * BLOCK_ELEMS + threadIdx.x * 4, 4, gv[k]);
                load_v<4>(e + t.start + k * BLOCK_ELEMS + threadIdx.x * 4, 4, ev[k]);
            }
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t ab = f2u(gv[k][j] + ev[k][j]) & 0x7fffffffu;
                    local = ab > local ? ab : local;
                }
            return local;
        }
    }
    for (int off = threadIdx.x * V; off < t.len; off += BLOCK_ELEMS) {
        const int nvalid = min(t.len - off, V);
        float gv[V], ev[V];
        load_v<V>(g + t.start + off, nvalid, gv);
        load_v<V>(e + t.start + off, nvalid, ev);
#pragma unroll
        for (int j = 0; j < V; ++j) {
            const uint32_t ab = f2u(gv[j] + ev[j]) & 0x7fffffffu;
            local = ab > local ? ab : local;
        }
    }
    return local;
}

// grid: (tiles, workers)
__global__ void __launch_bounds__(kBlockThreads) k_amax(AmaxArgs A)
{
    const int ti = A.tile_list ? A.tile_list[blockIdx.x] : (int)blockIdx.x;
    const Tile t = tile_at(A.tiles, ti, A.seg_len, 0);
    if (A.skip_small && (t.flags & (kTileSmallHead | kTileSmallBody))) return;
    const int w = A.first_worker + blockIdx.y;
    const float* g = A.grad[w];
    const float* e = A.err[w];
    uint32_t local;
    if (t.flags & kTileUnaligned) local = amax_range<true>(g, e, t.start, t.len, 0u);
    else local = amax_tile<4>(g, e, t);
    const uint32_t bm = block_max(local);
    if (threadIdx.x == 0) A.tile_max[(size_t)w * A.num_tiles + ti] = bm;
}

// Filtered scale pass, stage 3 of 4: max |g + e| over the elements of a tile that can still be the
// layer's maximum, i.e. those with |g| >= thr; e is read for those only.  Comparing bit patterns
// makes a NaN or Inf in g a candidate, so it still surfaces in the scale.
template <int V>
__device__ __forceinline__ uint32_t amax_tile_filtered(const float* __restrict__ g, const float* __restrict__ e,
                                                       const Tile& t, uint32_t thr)
{
    constexpr int BLOCK_ELEMS = kBlockThreads * V;
    uint32_t local = 0;
    if constexpr (V == 4) {
        if (t.len == 4 * BLOCK_ELEMS) {
            float gv[4][4];
#pragma unroll
            for (int k = 0; k < 4; ++k) load_v<4>(g + t.start + k * BLOCK_ELEMS + threadIdx.x * 4, 4, gv[k]);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                uint32_t top = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t ab = f2u(gv[k][j]) & 0x7fffffffu;
                    top = ab > top ? ab : top;
                }
                if (top >= thr) {
                    float ev[4];
                    load_v<4>(e + t.start + k * BLOCK_ELEMS + threadIdx.x * 4, 4, ev);
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const uint32_t ab = f2u(gv[k][j] + ev[j]) & 0x7fffffffu;
                        local = ab > local ? ab : local;
                    }
                }
            }
            return local;
        }
    }
    for (int off = threadIdx.x * V; off < t.len; off += BLOCK_ELEMS) {
        const int nvalid = min(t.len - off, V);
        float gv[V], ev[V];
        load_v<V>(g + t.start + off, nvalid, gv);
        uint32_t top = 0;
#pragma unroll
        for (int j = 0; j < V; ++j) {
            const uint32_t ab = f2u(gv[j]) & 0x7fffffffu;
            top = ab > top ? ab : top;
        }
        if (top >= thr) {
            load_v<V>(e + t.start + off, nvalid, ev);
#pragma unroll
            for (int j = 0; j < V; ++j) {
                const uint32_t ab = f2u(gv[j] + ev[j]) & 0x7fffffffu;
                local = ab > local ? ab : local;
            }
        }
    }
    return local;
}

// grid: (tiles, workers).  Sampled tiles keep the exact maximum stage 1 stored for them.
__global__ void __launch_bounds__(kBlockThreads) k_amax_filtered(AmaxArgs A)
{
    const int ti = blockIdx.x;
    const Tile t = A.tiles[ti];
    if (t.flags & kTileSampled) return;
    if (A.skip_small && (t.flags & (kTileSmallHead | kTileSmallBody))) return;
    const int w = A.first_worker + blockIdx.y;
    const float* g = A.grad[w];
    const float* e = A.err[w];
    const uint32_t thr = A.thr[(size_t)w * A.num_segments + t.seg];
    uint32_t local;
    if (t.flags & kTileUnaligned) local = amax_range<true>(g, e, t.start, t.len, thr);
    else if (thr == 0u) local = amax_tile<4>(g, e, t);
    else local = amax_tile_filtered<4>(g, e, t, thr);
    const uint32_t bm = block_max(local);
    if (threadIdx.x == 0) A.tile_max[(size_t)w * A.num_tiles + ti] = bm;
}

// max |e| over a tile
template <int V>
__device__ __forceinline__ uint32_t emax_tile(const float* __restrict__ e, const Tile& t)
{
    uint32_t local = 0;
    for (int off = threadIdx.x * V; off < t.len; off += kBlockThreads * V) {
        const int nvalid = min(t.len - off, V);
        float ev[V];
        load_v<V>(e + t.start + off, nvalid, ev);
#pragma unroll
        for (int j = 0; j < V; ++j) {
            const uint32_t ab = f2u(ev[j]) & 0x7fffffffu;
            local = ab > local ? ab : local;
        }
    }
    return local;
}

// Verification of the contract behind the filtered pass (bring-up aid): every |e_j| must be within
// the bound the previous step recorded for its layer.  grid: (tiles, workers); reads e only.
__global__ void __launch_bounds__(kBlockThreads) k_check_error_bounds(AmaxArgs A)
{
    const int ti = blockIdx.x;
    const Tile t = A.tiles[ti];
    const int w = A.first_worker + blockIdx.y;
    const float* e = A.err[w];
    const uint32_t local = (t.flags & kTileUnaligned) ? amax_range<true>(nullptr, e, t.start, t.len, 0u) : emax_tile<4>(e, t);
    const uint32_t bm = block_max(local);
    if (threadIdx.x == 0) {
        const float bound = A.err_bound[(size_t)w * A.num_segments + t.seg];
        // a NaN or Inf in e, or a magnitude beyond a finite bound, breaks the contract
        const bool finite_bound = bound < __builtin_inff();
        if (finite_bound && !(u2f(bm) <= bound)) atomicOr(A.status, QADAM_STATUS_ERR_BOUND_VIOLATED);
    }
}

// ------------------------------------------------------------------------------------------------
// common tile walk: every wave of the block takes 64*V elements per iteration; the trip count is
// wave-uniform so the cross-lane packing always runs with all lanes active.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ void write_pad_words(uint32_t* codes, const Tile& t, int code_bits)
{
    const int pad = (t.flags >> 8) & 3;
    if ((int)threadIdx.x < pad) {
        const int64_t groups = (t.len + 31) / 32;
        codes[t.code_word + groups * code_bits + threadIdx.x] = 0u;
    }
}

__device__ __forceinline__ void store_chunk_words(uint32_t* __restrict__ codes, const Tile& t, int base,
                                                  int code_bits, uint32_t word, int word_slot, bool writes)
{
    // first element of the group this lane's word belongs to
    const int grp = word_slot / code_bits;
    const bool group_live = base + grp * 32 < t.len;
    if (writes && group_live) {
        const int64_t cw = t.code_word + (int64_t)(base >> 5) * code_bits;
        __builtin_nontemporal_store(word, codes + cw + word_slot);
    }
}

// ---- worker side alone (qadam_worker_quantize, second pass of variant W) -------------------------
template <int V, int ROUNDING, bool PARKED, bool INLINE = false, bool SH = false>
__device__ __forceinline__ void worker_tile(const WorkerArgs& A, const Tile& t, const SmallLayerShared* sh = nullptr)
{
    constexpr int WAVE_ELEMS = 64 * V, BLOCK_ELEMS = (kBlockThreads / 64) * WAVE_ELEMS;
    const StepScalars& S = A.S;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const QgConst c = make_qg(S.k_g);
    const float s = INLINE ? sh->scale[0] : A.scales[t.seg];
    const float inv_s = INLINE ? sh->inv[0] : A.inv_scales[t.seg];
    if (!(s >= 0.0f && s < __builtin_inff()) && threadIdx.x == 0) atomicOr(A.status, QADAM_STATUS_NONFINITE_SCALE);
    const Shift sf = make_shift(t);
    for (int base = wave * WAVE_ELEMS; base < t.len; base += BLOCK_ELEMS) {
        const int off = base + lane * V;
        const int nvalid = min(max(t.len - off, 0), V);
        const int64_t gi = t.start + off;
        float g[V], e[V], q[V], en[V], U[V];
#pragma unroll
        for (int j = 0; j < V; ++j) U[j] = 0.0f;
        if constexpr (PARKED) {
            // the first pass left p = u + e in the error buffer; p + 0 reproduces it
            ld<V, SH>(A.err, gi, nvalid, sf, g);
#pragma unroll
            for (int j = 0; j < V; ++j) e[j] = 0.0f;
        } else {
            ld<V, SH>(A.grad, gi, nvalid, sf, g);
            ld<V, SH>(A.err, gi, nvalid, sf, e);
        }
        if constexpr (ROUNDING == 1) unif<V, SH>(S, gi, (uint32_t)A.worker, 0u, sf, U);
        uint32_t codes;
        worker_lane<V, ROUNDING>(g, e, s, inv_s, c, S.mu_bits, U, q, en, codes);
        st<V, SH>(A.err, gi, nvalid, sf, en);
        int slot; bool writes;
        const uint32_t word = pack_planes<V>(codes, S.code_bits, lane, slot, writes);
        store_chunk_words(A.codes, t, base, S.code_bits, word, slot, writes);
    }
    write_pad_words(A.codes, t, S.code_bits);
}

// the tiles of a small layer, one after the other, with the flags each would carry in the table
__device__ __forceinline__ Tile small_layer_tile(const Tile& head, int o, int code_bits)
{
    const int n = head.layer_len;
    Tile t = head;
    t.start = head.start + o;
    t.code_word = head.code_word + (int64_t)(o / 32) * code_bits;
    t.len = min(n - o, kDefaultTileElems);
    t.flags = head.flags & kTileUnaligned;
    if (o + kDefaultTileElems >= n) {
        const int used = (n + 31) / 32 * code_bits;
        t.flags |= ((used + 3) / 4 * 4 - used) << 8;
    }
    return t;
}

template <int ROUNDING>
__device__ __forceinline__ void worker_small_layer(const WorkerArgs& A, const Tile& head)
{
    __shared__ SmallLayerShared sh;
    const int n = head.layer_len;
    const bool unaligned = head.flags & kTileUnaligned;
    const uint32_t wm = unaligned ? wave_max_u32(amax_range<false>(A.grad, A.err, head.start, n, 0u))
                                  : small_layer_wave_max<4>(A.grad, A.err, head.start, n);
    if ((threadIdx.x & 63) == 0) sh.part[0][threadIdx.x >> 6] = wm;
    float* scales_row[1] = {A.scales};
    small_layer_finish(sh, 0, 1, head.seg, 1, scales_row, A.inv_scales, A.err_bound, A.bound_factor, true);
    for (int o = 0; o < n; o += kDefaultTileElems) {
        const Tile t = small_layer_tile(head, o, A.S.code_bits);
        if (unaligned) worker_tile<4, ROUNDING, false, true, true>(A, t, &sh);
        else worker_tile<4, ROUNDING, false, true, false>(A, t, &sh);
    }
}

template <int ROUNDING, bool PARKED>
__global__ void __launch_bounds__(kBlockThreads) k_worker_quantize(WorkerArgs A)
{
    const int ti = blockIdx.x;
    const Tile t = tile_at(A.tiles, ti, A.seg_len, A.S.code_bits);
    if constexpr (!PARKED) {
        // small layers: the workgroup of the first tile does the whole layer, scale included
        if (t.flags & kTileSmallBody) return;
        if (t.flags & kTileSmallHead) {
            worker_small_layer<ROUNDING>(A, t);
            return;
        }
    }
    if (t.flags & kTileMedium) {
        // the layer has few tiles: fold their maxima here instead of in a launch of its own
        __shared__ SmallLayerShared sh;
        const int t0 = A.seg_tile_begin[t.seg], t1 = A.seg_tile_begin[t.seg + 1];
        const uint32_t wm = medium_layer_wave_max(A.tile_max, t0, t1);
        if ((threadIdx.x & 63) == 0) sh.part[0][threadIdx.x >> 6] = wm;
        float* scales_row[1] = {A.scales};
        small_layer_finish(sh, 0, 1, t.seg, 1, scales_row, A.inv_scales, A.err_bound, A.bound_factor, true, ti == t0);
        if (t.flags & kTileUnaligned) worker_tile<4, ROUNDING, PARKED, true, true>(A, t, &sh);
        else worker_tile<4, ROUNDING, PARKED, true, false>(A, t, &sh);
        return;
    }
    if (t.flags & kTileUnaligned) worker_tile<4, ROUNDING, PARKED, false, true>(A, t);
    else worker_tile<4, ROUNDING, PARKED, false, false>(A, t);
}

// ---- server side alone (qadam_server_step) -------------------------------------------------------
struct ServerArgs {
    const Tile* tiles;
    int num_tiles;
    StepScalars S;
    float* x; float* m; float* v;
    const uint32_t* codes[QADAM_MAX_WORKERS];
    const float* scales[QADAM_MAX_WORKERS];
    int apply_only;         // variant W: x <- x - mean_i q_i, no moments
};

// U = number of workers whose code words are loaded together (N must be a multiple of U);
// MU_BITS = bits of the level index (code bits minus the sign)
template <int V, int U, int MU_BITS, bool SH = false>
__device__ __forceinline__ void server_tile(const ServerArgs& A, const Tile& t)
{
    constexpr int WAVE_ELEMS = 64 * V, BLOCK_ELEMS = (kBlockThreads / 64) * WAVE_ELEMS;
    const StepScalars& S = A.S;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const QgConst c = make_qg(S.k_g);
    const Shift sf = make_shift(t);
    for (int base = wave * WAVE_ELEMS; base < t.len; base += BLOCK_ELEMS) {
        const int off = base + lane * V;
        const int nvalid = min(max(t.len - off, 0), V);
        if (nvalid == 0) continue;
        const int64_t gi = t.start + off;
        const int64_t cw = t.code_word + (int64_t)(base >> 5) * S.code_bits;
        // server state first: its latency hides behind the decoding
        float xv[V], mv[V], vv[V];
        ld<V, SH>(A.x, gi, nvalid, sf, xv);
        if (!A.apply_only) {
            ld<V, SH>(A.m, gi, nvalid, sf, mv);
            ld<V, SH>(A.v, gi, nvalid, sf, vv);
        }
        float acc[V];
#pragma unroll
        for (int j = 0; j < V; ++j) acc[j] = 0.0f;
        for (int i0 = 0; i0 < S.num_workers; i0 += U) {
            uint32_t w[U][4];
            uint32_t pos = 0;
#pragma unroll
            for (int u = 0; u < U; ++u) pos = load_planes<V, MU_BITS>(A.codes[i0 + u] + cw, lane, w[u]);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const float s = A.scales[i0 + u][t.seg];
#pragma unroll
                for (int j = 0; j < V; ++j)
                    acc[j] = acc[j] + qg_decode_planes<MU_BITS>(w[u], pos + (uint32_t)j, s, c);
            }
        }
        if (A.apply_only) {
#pragma unroll
            for (int j = 0; j < V; ++j) xv[j] = xv[j] - mean_over_workers(S, acc[j]);
        } else {
#pragma unroll
            for (int j = 0; j < V; ++j) {
                const float u = adam_step(S, mean_over_workers(S, acc[j]), mv[j], vv[j]);
                xv[j] = xv[j] - u;
            }
            st<V, SH>(A.m, gi, nvalid, sf, mv);
            st<V, SH>(A.v, gi, nvalid, sf, vv);
        }
        st<V, SH>(A.x, gi, nvalid, sf, xv);
    }
}

template <int U, int MU_BITS>
__global__ void __launch_bounds__(kBlockThreads) k_server_step(ServerArgs A)
{
    const int ti = blockIdx.x;
    const Tile t = A.tiles[ti];
    if (t.flags & kTileUnaligned) server_tile<4, U, MU_BITS, true>(A, t);
    else server_tile<4, U, MU_BITS, false>(A, t);
}

// ---- weight quantizer alone (qadam_weight_quantize) ----------------------------------------------
struct WeightArgs {
    StepScalars S;
    const float* x;
    float* werr;
    void* wcodes;
    int64_t n;
};

// One workgroup per 4096 consecutive elements; a lane owns four quads, quad k being elements
// 4 * (lane + 256 k) .. + 3, and issues the loads of all four before any arithmetic.
template <int ROUNDING>
__global__ void __launch_bounds__(kBlockThreads) k_weight_quantize(WeightArgs A)
{
    const StepScalars& S = A.S;
    const int64_t base = (int64_t)blockIdx.x * (kBlockThreads * 16);
    float xv[4][4], wi[4][4];
    int nvalid[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int64_t gi = base + 4 * ((int64_t)threadIdx.x + kBlockThreads * k);
        nvalid[k] = (int)max((int64_t)0, min((int64_t)4, A.n - gi));
#pragma unroll
        for (int t = 0; t < 4; ++t) wi[k][t] = 0.0f;
        if (nvalid[k] > 0) {
            load_v<4>(A.x + gi, nvalid[k], xv[k]);
            if (S.weight_ef) load_v<4>(A.werr + gi, nvalid[k], wi[k]);
        }
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        if (nvalid[k] == 0) continue;
        const int64_t gi = base + 4 * ((int64_t)threadIdx.x + kBlockThreads * k);
        float wo[4];
        int j[4];
        weight_lane<4, ROUNDING>(S, xv[k], wi[k], gi, Shift{}, wo, j);
        if (A.werr) store_v<4>(A.werr + gi, nvalid[k], wo);
        store_wcodes<4>(A.wcodes, S.wcode_bytes, gi, nvalid[k], j);
    }
}

struct DequantArgs {
    const void* wcodes;
    void* xhat;             // float or __half, per the kernel's template argument
    int64_t n;
    int wcode_bytes;
    float inv_two_kx1;
};

// A lane owns four pieces of E consecutive codes (E = 4 for fp32 output, 8 for binary16, so that an output
// store is always 128 bits), piece k being elements E * (lane + 256 k) .. of the workgroup's 1024 E codes:
// every store of a wavefront is one contiguous 1 KiB run and the four code loads are issued together.
template <bool HALF, int CODE_BYTES>
__global__ void __launch_bounds__(kBlockThreads) k_weight_dequantize(DequantArgs A)
{
    constexpr int E = HALF ? 8 : 4;
    constexpr int WORDS = E * CODE_BYTES / 4;           // code words per piece: 1, 2 or 4
    const int64_t base = (int64_t)blockIdx.x * (kBlockThreads * E * 4);
    uint32_t w[4][WORDS];
    bool full[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int64_t i = base + E * ((int64_t)threadIdx.x + kBlockThreads * k);
        full[k] = i + E <= A.n;
#pragma unroll
        for (int t = 0; t < WORDS; ++t) w[k][t] = 0u;
        const char* src = static_cast<const char*>(A.wcodes) + i * CODE_BYTES;
        if (full[k]) {
            if constexpr (WORDS == 1) {
                w[k][0] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(src));
            } else if constexpr (WORDS == 2) {
                const u2 v = __builtin_nontemporal_load(reinterpret_cast<const u2*>(src));
                w[k][0] = v.x; w[k][1] = v.y;
            } else {
                const u4 v = __builtin_nontemporal_load(reinterpret_cast<const u4*>(src));
                w[k][0] = v.x; w[k][1] = v.y; w[k][2] = v.z; w[k][3] = v.w;
            }
        } else {
            // ragged end of the vector: code by code
#pragma unroll
            for (int t = 0; t < E; ++t) {
                if (i + t < A.n) {
                    const uint32_t c = CODE_BYTES == 1 ? (uint32_t)(uint8_t)src[t]
                                                       : (uint32_t)reinterpret_cast<const uint16_t*>(src)[t];
                    w[k][t * CODE_BYTES / 4] |= c << (8 * ((t * CODE_BYTES) & 3));
                }
            }
        }
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int64_t i = base + E * ((int64_t)threadIdx.x + kBlockThreads * k);
        float xh[E];
#pragma unroll
        for (int t = 0; t < E; ++t) {
            const uint32_t c = w[k][t * CODE_BYTES / 4] >> (8 * ((t * CODE_BYTES) & 3));
            const int j = CODE_BYTES == 1 ? (int)(int8_t)c : (int)(int16_t)c;
            xh[t] = (float)j * A.inv_two_kx1;
        }
        if constexpr (HALF) {
            __half* out = static_cast<__half*>(A.xhat) + i;
            if (full[k]) {
                u4 v;
                v.x = (uint32_t)__half_as_ushort(__float2half_rn(xh[0])) | ((uint32_t)__half_as_ushort(__float2half_rn(xh[1])) << 16);
                v.y = (uint32_t)__half_as_ushort(__float2half_rn(xh[2])) | ((uint32_t)__half_as_ushort(__float2half_rn(xh[3])) << 16);
                v.z = (uint32_t)__half_as_ushort(__float2half_rn(xh[4])) | ((uint32_t)__half_as_ushort(__float2half_rn(xh[5])) << 16);
                v.w = (uint32_t)__half_as_ushort(__float2half_rn(xh[6])) | ((uint32_t)__half_as_ushort(__float2half_rn(xh[7])) << 16);
                __builtin_nontemporal_store(v, reinterpret_cast<u4*>(out));
            } else {
#pragma unroll
                for (int t = 0; t < E; ++t) if (i + t < A.n) out[t] = __float2half_rn(xh[t]);
            }
        } else {
            float* out = static_cast<float*>(A.xhat) + i;
            if (full[k]) {
                f4 v;
                v.x = xh[0]; v.y = xh[1]; v.z = xh[2]; v.w = xh[3];
                __builtin_nontemporal_store(v, reinterpret_cast<f4*>(out));
            } else {
#pragma unroll
                for (int t = 0; t < E; ++t) if (i + t < A.n) out[t] = xh[t];
            }
        }
    }
}

// ---- the whole step in one pass (qadam_step_fused) -----------------------------------------------
// U = number of workers whose loads are issued together (N must be a multiple of U).
// W = false: variant S (workers' g and e in, server moments).  W = true: second pass of variant W
// (the first pass left p_i = alpha m_i / sqrt(v_i + eps) + e_i in the error buffers; the server
// only subtracts the mean message).
template <int V, int ROUNDING, int U, bool W, bool INLINE = false, bool SH = false>
__device__ __forceinline__ void fused_tile(const FusedArgs& A, const Tile& t, const SmallLayerShared* sh = nullptr)
{
    constexpr int WAVE_ELEMS = 64 * V, BLOCK_ELEMS = (kBlockThreads / 64) * WAVE_ELEMS;
    const StepScalars& S = A.S;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const QgConst c = make_qg(S.k_g);
    const int N = S.num_workers;
    const Shift sf = make_shift(t);
    for (int base = wave * WAVE_ELEMS; base < t.len; base += BLOCK_ELEMS) {
        const int off = base + lane * V;
        const int nvalid = min(max(t.len - off, 0), V);
        const int64_t gi = t.start + off;
        // server state first: its latency hides behind the workers' arithmetic
        float xv[V], mv[V], vv[V], wi[V], wo[V];
        int jc[V];
#pragma unroll
        for (int j = 0; j < V; ++j) wi[j] = 0.0f;
        ld<V, SH>(A.sp.x, gi, nvalid, sf, xv);
        if constexpr (!W) {
            ld<V, SH>(A.sp.m, gi, nvalid, sf, mv);
            ld<V, SH>(A.sp.v, gi, nvalid, sf, vv);
        }
        const bool quantize_x = S.k_x >= 0;              // false: Q_x is the identity
        if (S.weight_ef && quantize_x) ld<V, SH>(A.sp.werr, gi, nvalid, sf, wi);
        float acc[V];
#pragma unroll
        for (int j = 0; j < V; ++j) acc[j] = 0.0f;
        for (int i0 = 0; i0 < N; i0 += U) {
            float g[U][V], e[U][V];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if constexpr (W) {
                    ld<V, SH>(A.err[i0 + u], gi, nvalid, sf, g[u]);       // parked p; p + 0 reproduces it
#pragma unroll
                    for (int j = 0; j < V; ++j) e[u][j] = 0.0f;
                } else {
                    ld<V, SH>(A.grad[i0 + u], gi, nvalid, sf, g[u]);
                    ld<V, SH>(A.err[i0 + u], gi, nvalid, sf, e[u]);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = i0 + u;
                const float s = INLINE ? sh->scale[i] : A.scales[i][t.seg];
                const float inv_s = INLINE ? sh->inv[i] : A.inv_scales[(size_t)i * A.num_segments + t.seg];
                float q[V], en[V], Ur[V];
#pragma unroll
                for (int j = 0; j < V; ++j) Ur[j] = 0.0f;
                if constexpr (ROUNDING == 1) unif<V, SH>(S, gi, (uint32_t)i, 0u, sf, Ur);
                uint32_t codes;
                worker_lane<V, ROUNDING>(g[u], e[u], s, inv_s, c, S.mu_bits, Ur, q, en, codes);
                st<V, SH>(A.err[i], gi, nvalid, sf, en);
                int slot; bool writes;
                const uint32_t word = pack_planes<V>(codes, S.code_bits, lane, slot, writes);
                store_chunk_words(A.codes[i], t, base, S.code_bits, word, slot, writes);
#pragma unroll
                for (int j = 0; j < V; ++j) acc[j] = acc[j] + q[j];
            }
        }
        // server: mean, (moments, step,) weight quantizer
        if constexpr (W) {
#pragma unroll
            for (int j = 0; j < V; ++j) xv[j] = xv[j] - mean_over_workers(S, acc[j]);
        } else {
#pragma unroll
            for (int j = 0; j < V; ++j) {
                const float u = adam_step(S, mean_over_workers(S, acc[j]), mv[j], vv[j]);
                xv[j] = xv[j] - u;
            }
        }
        if constexpr (!W) {
            st<V, SH>(A.sp.m, gi, nvalid, sf, mv);
            st<V, SH>(A.sp.v, gi, nvalid, sf, vv);
        }
        st<V, SH>(A.sp.x, gi, nvalid, sf, xv);
        if (quantize_x) {
            weight_lane<V, ROUNDING, SH>(S, xv, wi, gi, sf, wo, jc);
            if (A.sp.werr) st<V, SH>(A.sp.werr, gi, nvalid, sf, wo);
            stw<V, SH>(A.sp.wcodes, S.wcode_bytes, gi, nvalid, sf, jc);
        }
    }
    for (int i = 0; i < N; ++i) {
        write_pad_words(A.codes[i], t, S.code_bits);
        const float s = INLINE ? sh->scale[i] : A.scales[i][t.seg];
        if (!(s >= 0.0f && s < __builtin_inff()) && threadIdx.x == 0)
            atomicOr(A.status, QADAM_STATUS_NONFINITE_SCALE);
    }
}

// One workgroup does a whole small layer: the scales of all workers first (g and e read once, kept in
// cache), then the layer's tiles exactly as the separate workgroups would have done them.
template <int ROUNDING, int U>
__device__ __forceinline__ void fused_small_layer(const FusedArgs& A, const Tile& head)
{
    __shared__ SmallLayerShared sh;
    const int n = head.layer_len, N = A.S.num_workers;
    const bool unaligned = head.flags & kTileUnaligned;
    for (int i = 0; i < N; ++i) {
        const uint32_t wm = unaligned ? wave_max_u32(amax_range<false>(A.grad[i], A.err[i], head.start, n, 0u))
                                      : small_layer_wave_max<4>(A.grad[i], A.err[i], head.start, n);
        if ((threadIdx.x & 63) == 0) sh.part[i][threadIdx.x >> 6] = wm;
    }
    small_layer_finish(sh, 0, N, head.seg, A.num_segments, A.scales, A.inv_scales, A.err_bound, A.bound_factor, false);
    for (int o = 0; o < n; o += kDefaultTileElems) {
        const Tile t = small_layer_tile(head, o, A.S.code_bits);
        if (unaligned) fused_tile<4, ROUNDING, U, false, true, true>(A, t, &sh);
        else fused_tile<4, ROUNDING, U, false, true, false>(A, t, &sh);
    }
}

template <int ROUNDING, int U, bool W>
__global__ void __launch_bounds__(kBlockThreads) k_fused(FusedArgs A)
{
    const int ti = blockIdx.x;
    const Tile t = A.tiles[ti];
    if constexpr (!W) {
        // small layers: the workgroup of the first tile does the whole layer, scales included
        if (t.flags & kTileSmallBody) return;
        if (t.flags & kTileSmallHead) {
            fused_small_layer<ROUNDING, U>(A, t);
            return;
        }
    }
    if (t.flags & kTileMedium) {
        // the layer has few tiles: fold their maxima here instead of in a launch of its own
        __shared__ SmallLayerShared sh;
        const int N = A.S.num_workers;
        const int t0 = A.seg_tile_begin[t.seg], t1 = A.seg_tile_begin[t.seg + 1];
        for (int i = 0; i < N; ++i) {
            const uint32_t wm = medium_layer_wave_max(A.tile_max + (size_t)i * A.num_tiles, t0, t1);
            if ((threadIdx.x & 63) == 0) sh.part[i][threadIdx.x >> 6] = wm;
        }
        small_layer_finish(sh, 0, N, t.seg, A.num_segments, A.scales, A.inv_scales, A.err_bound, A.bound_factor, false,
                           ti == t0);
        if (t.flags & kTileUnaligned) fused_tile<4, ROUNDING, U, W, true, true>(A, t, &sh);
        else fused_tile<4, ROUNDING, U, W, true, false>(A, t, &sh);
        return;
    }
    if (t.flags & kTileUnaligned) fused_tile<4, ROUNDING, U, W, false, true>(A, t);
    else fused_tile<4, ROUNDING, U, W, false, false>(A, t);
}

// ---- Q_g = identity: the messages are fp32 values ------------------------------------------------
// W = false: the message of worker i is its gradient (plain distributed generic Adam on the mean
// gradient, then Q_x).  W = true: second pass of variant W with the identity quantizer: the message
// is the parked p_i = alpha m_i / sqrt(v_i + eps) + e_i, all of it is sent, so e_i <- 0.
template <int V, int ROUNDING, int U, bool W, bool SH = false>
__device__ __forceinline__ void plain_tile(const FusedArgs& A, const Tile& t)
{
    constexpr int WAVE_ELEMS = 64 * V, BLOCK_ELEMS = (kBlockThreads / 64) * WAVE_ELEMS;
    const StepScalars& S = A.S;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int N = S.num_workers;
    const bool quantize_x = S.k_x >= 0;
    const Shift sf = make_shift(t);
    for (int base = wave * WAVE_ELEMS; base < t.len; base += BLOCK_ELEMS) {
        const int off = base + lane * V;
        const int nvalid = min(max(t.len - off, 0), V);
        if (nvalid == 0) continue;
        const int64_t gi = t.start + off;
        float xv[V], mv[V], vv[V], wi[V], wo[V], acc[V], zero[V];
        int jc[V];
#pragma unroll
        for (int j = 0; j < V; ++j) { wi[j] = 0.0f; acc[j] = 0.0f; zero[j] = 0.0f; }
        ld<V, SH>(A.sp.x, gi, nvalid, sf, xv);
        if constexpr (!W) {
            ld<V, SH>(A.sp.m, gi, nvalid, sf, mv);
            ld<V, SH>(A.sp.v, gi, nvalid, sf, vv);
        }
        if (S.weight_ef && quantize_x) ld<V, SH>(A.sp.werr, gi, nvalid, sf, wi);
        for (int i0 = 0; i0 < N; i0 += U) {
            float p[U][V];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if constexpr (W) ld<V, SH>(A.err[i0 + u], gi, nvalid, sf, p[u]);
                else ld<V, SH>(A.grad[i0 + u], gi, nvalid, sf, p[u]);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int j = 0; j < V; ++j) acc[j] = acc[j] + p[u][j];
                if constexpr (W) st<V, SH>(A.err[i0 + u], gi, nvalid, sf, zero);
            }
        }
        if constexpr (W) {
#pragma unroll
            for (int j = 0; j < V; ++j) xv[j] = xv[j] - mean_over_workers(S, acc[j]);
        } else {
#pragma unroll
            for (int j = 0; j < V; ++j) {
                const float u = adam_step(S, mean_over_workers(S, acc[j]), mv[j], vv[j]);
                xv[j] = xv[j] - u;
            }
            st<V, SH>(A.sp.m, gi, nvalid, sf, mv);
            st<V, SH>(A.sp.v, gi, nvalid, sf, vv);
        }
        st<V, SH>(A.sp.x, gi, nvalid, sf, xv);
        if (quantize_x) {
            weight_lane<V, ROUNDING, SH>(S, xv, wi, gi, sf, wo, jc);
            if (A.sp.werr) st<V, SH>(A.sp.werr, gi, nvalid, sf, wo);
            stw<V, SH>(A.sp.wcodes, S.wcode_bytes, gi, nvalid, sf, jc);
        }
    }
}

template <int ROUNDING, int U, bool W>
__global__ void __launch_bounds__(kBlockThreads) k_plain_messages(FusedArgs A)
{
    const int ti = blockIdx.x;
    const Tile t = A.tiles[ti];
    if (t.flags & kTileUnaligned) plain_tile<4, ROUNDING, U, W, true>(A, t);
    else plain_tile<4, ROUNDING, U, W, false>(A, t);
}

// ---- variant W, first pass: local moments, park p = u + e in the error buffer, scale ------------
struct MomentsWArgs {
    const Tile* tiles;
    int num_tiles;
    StepScalars S;
    const float* grad[QADAM_MAX_WORKERS];
    float* mw[QADAM_MAX_WORKERS];
    float* vw[QADAM_MAX_WORKERS];
    float* err[QADAM_MAX_WORKERS];
    uint32_t* tile_max;     // [N][num_tiles]
    int first_worker;
};

template <int V, bool SH = false>
__device__ __forceinline__ uint32_t moments_w_tile(const StepScalars& S, const float* __restrict__ grad,
                                                   float* __restrict__ mw, float* __restrict__ vw,
                                                   float* __restrict__ err, const Tile& t)
{
    constexpr int BLOCK_ELEMS = kBlockThreads * V;
    uint32_t local = 0;
    const Shift sf = make_shift(t);
    for (int base = 0; base < t.len; base += BLOCK_ELEMS) {
        const int off = base + threadIdx.x * V;
        const int nvalid = min(max(t.len - off, 0), V);
        const int64_t gi = t.start + off;
        float g[V], mv[V], vv[V], e[V], p[V];
        ld<V, SH>(grad, gi, nvalid, sf, g);
        ld<V, SH>(mw, gi, nvalid, sf, mv);
        ld<V, SH>(vw, gi, nvalid, sf, vv);
        ld<V, SH>(err, gi, nvalid, sf, e);
#pragma unroll
        for (int j = 0; j < V; ++j) {
            const float u = adam_step(S, g[j], mv[j], vv[j]);
            p[j] = u + e[j];
            const uint32_t ab = j < nvalid ? (f2u(p[j]) & 0x7fffffffu) : 0u;
            local = ab > local ? ab : local;
        }
        st<V, SH>(mw, gi, nvalid, sf, mv);
        st<V, SH>(vw, gi, nvalid, sf, vv);
        st<V, SH>(err, gi, nvalid, sf, p);
    }
    return local;
}

// grid: (tiles, workers)
__global__ void __launch_bounds__(kBlockThreads) k_moments_w(MomentsWArgs A)
{
    const int ti = blockIdx.x;
    const Tile t = A.tiles[ti];
    const int w = A.first_worker + blockIdx.y;
    uint32_t local;
    if (t.flags & kTileUnaligned) local = moments_w_tile<4, true>(A.S, A.grad[w], A.mw[w], A.vw[w], A.err[w], t);
    else local = moments_w_tile<4, false>(A.S, A.grad[w], A.mw[w], A.vw[w], A.err[w], t);
    const uint32_t bm = block_max(local);
    if (threadIdx.x == 0) A.tile_max[(size_t)w * A.num_tiles + ti] = bm;
}

// ---- diagnostic: per-layer sum of squares in fp64, fixed order ---------------------------------
struct SumsqArgs {
    const Tile* tiles;
    const float* a;
    const float* b;         // may be null
    double* tile_sum;       // [num_tiles]
    const int32_t* seg_tile_begin;
    double* out;            // [num_segments]
};

// block-wide sum in a fixed order: butterfly inside each wavefront, then the wavefronts in index
// order; every thread gets the result
__device__ __forceinline__ double block_sum_f64(double v)
{
    __shared__ double wave_part[kBlockThreads / 64];
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    __syncthreads();                       // the array may still be read from an earlier call
    if (lane == 0) wave_part[wave] = v;
    __syncthreads();
    double s = wave_part[0];
#pragma unroll
    for (int w = 1; w < kBlockThreads / 64; ++w) s += wave_part[w];
    return s;
}

template <int V>
__device__ __forceinline__ double sumsq_tile(const float* __restrict__ a, const float* __restrict__ b, const Tile& t)
{
    constexpr int BLOCK_ELEMS = kBlockThreads * V;
    double local = 0.0;
    for (int off = threadIdx.x * V; off < t.len; off += BLOCK_ELEMS) {
        const int nvalid = min(t.len - off, V);
        float av[V], bv[V];
        load_v<V>(a + t.start + off, nvalid, av);
        if (b) {
            load_v<V>(b + t.start + off, nvalid, bv);
        } else {
#pragma unroll
            for (int j = 0; j < V; ++j) bv[j] = 0.0f;
        }
#pragma unroll
        for (int j = 0; j < V; ++j) {
            const double p = (double)(av[j] + bv[j]);     // the sum in fp32, as the step forms it
            local += p * p;                               // exact product of two 24-bit significands
        }
    }
    return local;
}

// grid: tiles
__global__ void __launch_bounds__(kBlockThreads) k_sumsq_tiles(SumsqArgs A)
{
    const int ti = blockIdx.x;
    const Tile t = A.tiles[ti];
    double local;
    if (t.flags & kTileUnaligned) local = sumsq_tile<1>(A.a, A.b, t);
    else local = sumsq_tile<4>(A.a, A.b, t);
    const double s = block_sum_f64(local);
    if (threadIdx.x == 0) A.tile_sum[ti] = s;
}

// grid: layers.  Thread k adds tiles k, k+256, ... of its layer in that order, then the block sum.
__global__ void __launch_bounds__(kBlockThreads) k_sumsq_layers(SumsqArgs A)
{
    const int l = blockIdx.x;
    const int t0 = A.seg_tile_begin[l], t1 = A.seg_tile_begin[l + 1];
    double local = 0.0;
    for (int t = t0 + threadIdx.x; t < t1; t += kBlockThreads) local += A.tile_sum[t];
    const double s = block_sum_f64(local);
    if (threadIdx.x == 0) A.out[l] = s;
}

}  // namespace

// ================================================================================================
// launchers
// ================================================================================================
// |p - Q_g(p)| <= factor * s: half the widest gap of the grid for nearest rounding (the gap between
// 1/2 and 1, or between 0 and 1 for the ternary grid), the whole gap for stochastic rounding; the
// small excess covers the rounding of the quotient p / s that takes the decision.
static float residual_bound_factor(const StepScalars& S)
{
    const float half_gap = S.k_g >= 1 ? 0.25f : 0.5f;
    return (S.rounding == 0 ? half_gap : 2.0f * half_gap) * (1.0f + 0x1p-20f);
}

static void fill_scale_args(ScaleArgs& A, const Launch& L, const StepScalars& S, const WorkerPtrs& W, int first_worker)
{
    A.tiles = L.tiles;
    for (int i = 0; i < QADAM_MAX_WORKERS; ++i) A.scales[i] = W.scales[i];
    A.inv_scales = L.inv_scales; A.tile_max = L.tile_max; A.seg_tile_begin = L.seg_tile_begin;
    A.first_worker = first_worker; A.num_segments = L.num_segments; A.num_tiles = L.num_tiles;
    A.err_bound = L.err_bound; A.thr = L.thr;
    A.bound_factor = residual_bound_factor(S);
    A.sample_stride = kSampleStride;
}

hipError_t launch_reduce_scales(const Launch& L, const StepScalars& S, const WorkerPtrs& W, int first_worker, int num)
{
    if (L.num_segments == 0 || num == 0) return hipSuccess;
    if (!L.need_reduce) return hipSuccess;      // every scale is folded by the quantizing kernel
    ScaleArgs A;
    fill_scale_args(A, L, S, W, first_worker);
    hipLaunchKernelGGL(k_reduce_scales, dim3(L.num_segments, num), dim3(kBlockThreads), 0, L.stream, A);
    return hipGetLastError();
}

static void fill_amax_args(AmaxArgs& A, const Launch& L, const WorkerPtrs& W, int first_worker)
{
    A.tiles = L.tiles; A.num_tiles = L.num_tiles;
    for (int i = 0; i < QADAM_MAX_WORKERS; ++i) { A.grad[i] = W.grad[i]; A.err[i] = W.err[i]; }
    A.tile_max = L.tile_max;
    A.first_worker = first_worker;
    A.tile_list = nullptr; A.thr = L.thr; A.num_segments = L.num_segments;
    A.err_bound = L.err_bound; A.status = L.status;
    A.seg_len = 0;
    A.skip_small = 1;       // only the server-moments path uses these kernels
}

hipError_t launch_check_error_bounds(const Launch& L, const WorkerPtrs& W, int first_worker, int num)
{
    if (L.num_tiles == 0 || num == 0) return hipSuccess;
    AmaxArgs A;
    fill_amax_args(A, L, W, first_worker);
    A.skip_small = 0;       // the check covers every tile
    hipLaunchKernelGGL(k_check_error_bounds, dim3(L.num_tiles, num), dim3(kBlockThreads), 0, L.stream, A);
    return hipGetLastError();
}

hipError_t launch_amax(const Launch& L, const StepScalars& S, const WorkerPtrs& W, int first_worker, int num)
{
    (void)S;
    if (L.num_tiles == 0 || num == 0 || !L.need_amax) return hipSuccess;
    AmaxArgs A;
    fill_amax_args(A, L, W, first_worker);
    hipLaunchKernelGGL(k_amax, dim3(L.num_tiles, num), dim3(kBlockThreads), 0, L.stream, A);
    return hipGetLastError();
}

// The scale pass when every |e_j| is known to be at most the bound the previous step left:
// exact maxima of the sampled tiles -> per-layer thresholds -> the other tiles, reading e only
// where |g| reaches the threshold.  launch_reduce_scales follows as usual.
hipError_t launch_amax_filtered(const Launch& L, const StepScalars& S, const WorkerPtrs& W, int first_worker, int num)
{
    if (L.num_tiles == 0 || num == 0 || !L.need_amax) return hipSuccess;
    AmaxArgs A;
    fill_amax_args(A, L, W, first_worker);
    A.tile_list = L.sample_tiles;
    hipLaunchKernelGGL(k_amax, dim3(L.num_sample_tiles, num), dim3(kBlockThreads), 0, L.stream, A);
    ScaleArgs R;
    fill_scale_args(R, L, S, W, first_worker);
    hipLaunchKernelGGL(k_reduce_lower_bounds, dim3(L.num_segments, num), dim3(kBlockThreads), 0, L.stream, R);
    A.tile_list = nullptr;
    hipLaunchKernelGGL(k_amax_filtered, dim3(L.num_tiles, num), dim3(kBlockThreads), 0, L.stream, A);
    return hipGetLastError();
}

hipError_t launch_worker_quantize(const Launch& L, const StepScalars& S, const WorkerPtrs& W, int worker)
{
    if (L.num_tiles == 0) return hipSuccess;
    WorkerArgs A;
    A.tiles = L.tiles; A.num_tiles = L.num_tiles;
    A.status = L.status; A.S = S;
    A.grad = W.grad[worker]; A.err = W.err[worker]; A.codes = W.codes[worker]; A.scales = W.scales[worker];
    A.inv_scales = L.inv_scales + (size_t)worker * L.num_segments;
    A.err_bound = L.err_bound + (size_t)worker * L.num_segments;
    A.bound_factor = residual_bound_factor(S);
    A.tile_max = L.tile_max + (size_t)worker * L.num_tiles;
    A.seg_tile_begin = L.seg_tile_begin;
    A.worker = worker;
    A.seg_len = 0;
    const bool parked = (A.grad == nullptr);
    const dim3 grid(L.num_tiles), block(kBlockThreads);
    if (S.rounding == 0) {
        if (parked) hipLaunchKernelGGL((k_worker_quantize<0, true>), grid, block, 0, L.stream, A);
        else hipLaunchKernelGGL((k_worker_quantize<0, false>), grid, block, 0, L.stream, A);
    } else {
        if (parked) hipLaunchKernelGGL((k_worker_quantize<1, true>), grid, block, 0, L.stream, A);
        else hipLaunchKernelGGL((k_worker_quantize<1, false>), grid, block, 0, L.stream, A);
    }
    return hipGetLastError();
}

static void fill_server_args(ServerArgs& A, const Launch& L, const StepScalars& S, const WorkerPtrs& W)
{
    A.tiles = L.tiles; A.num_tiles = L.num_tiles; A.S = S;
    for (int i = 0; i < QADAM_MAX_WORKERS; ++i) { A.codes[i] = W.codes[i]; A.scales[i] = W.scales[i]; }
}

static void launch_server_kernel(const Launch& L, const ServerArgs& A)
{
    const dim3 grid(L.num_tiles), block(kBlockThreads);
    const bool four = A.S.num_workers % 4 == 0;
#define QADAM_LAUNCH_SERVER(MB)                                                                       \
    do {                                                                                              \
        if (four) hipLaunchKernelGGL((k_server_step<4, MB>), grid, block, 0, L.stream, A);            \
        else hipLaunchKernelGGL((k_server_step<1, MB>), grid, block, 0, L.stream, A);                 \
    } while (0)
    if (A.S.mu_bits == 1) QADAM_LAUNCH_SERVER(1);
    else if (A.S.mu_bits == 2) QADAM_LAUNCH_SERVER(2);
    else QADAM_LAUNCH_SERVER(3);
#undef QADAM_LAUNCH_SERVER
}

hipError_t launch_server_step(const Launch& L, const StepScalars& S, const WorkerPtrs& W, const ServerPtrs& sp)
{
    if (L.num_tiles == 0) return hipSuccess;
    ServerArgs A;
    fill_server_args(A, L, S, W);
    A.x = sp.x; A.m = sp.m; A.v = sp.v; A.apply_only = 0;
    launch_server_kernel(L, A);
    return hipGetLastError();
}

hipError_t launch_server_apply_w(const Launch& L, const StepScalars& S, const WorkerPtrs& W, float* x)
{
    if (L.num_tiles == 0) return hipSuccess;
    ServerArgs A;
    fill_server_args(A, L, S, W);
    A.x = x; A.m = nullptr; A.v = nullptr; A.apply_only = 1;
    launch_server_kernel(L, A);
    return hipGetLastError();
}

hipError_t launch_weight_quantize(const Launch& L, const StepScalars& S, const float* x, float* werr, void* wcodes)
{
    if (L.num_params == 0) return hipSuccess;
    WeightArgs A;
    A.S = S; A.x = x; A.werr = werr; A.wcodes = wcodes; A.n = L.num_params;
    const dim3 grid((unsigned)((L.num_params + kBlockThreads * 16 - 1) / (kBlockThreads * 16))), block(kBlockThreads);
    if (S.rounding == 0) hipLaunchKernelGGL(k_weight_quantize<0>, grid, block, 0, L.stream, A);
    else hipLaunchKernelGGL(k_weight_quantize<1>, grid, block, 0, L.stream, A);
    return hipGetLastError();
}

hipError_t launch_weight_dequantize(const Launch& L, const StepScalars& S, const void* wcodes, void* xhat, bool half)
{
    if (L.num_params == 0) return hipSuccess;
    DequantArgs A;
    A.wcodes = wcodes; A.xhat = xhat; A.n = L.num_params; A.wcode_bytes = S.wcode_bytes;
    union { uint32_t u; float f; } cv;
    cv.u = (uint32_t)(127 - S.k_x - 1) << 23;
    A.inv_two_kx1 = cv.f;
    const int64_t per_block = (int64_t)kBlockThreads * 4 * (half ? 8 : 4);
    const dim3 grid((unsigned)((L.num_params + per_block - 1) / per_block)), block(kBlockThreads);
    if (S.wcode_bytes == 1) {
        if (half) hipLaunchKernelGGL((k_weight_dequantize<true, 1>), grid, block, 0, L.stream, A);
        else hipLaunchKernelGGL((k_weight_dequantize<false, 1>), grid, block, 0, L.stream, A);
    } else {
        if (half) hipLaunchKernelGGL((k_weight_dequantize<true, 2>), grid, block, 0, L.stream, A);
        else hipLaunchKernelGGL((k_weight_dequantize<false, 2>), grid, block, 0, L.stream, A);
    }
    return hipGetLastError();
}

static hipError_t launch_fused_any(const Launch& L, const StepScalars& S, const WorkerPtrs& W, const ServerPtrs& sp,
                                   bool variant_w)
{
    if (L.num_tiles == 0) return hipSuccess;
    FusedArgs A;
    A.tiles = L.tiles; A.num_tiles = L.num_tiles;
    A.status = L.status; A.inv_scales = L.inv_scales; A.num_segments = L.num_segments; A.S = S; A.sp = sp;
    A.err_bound = L.err_bound; A.bound_factor = residual_bound_factor(S);
    A.tile_max = L.tile_max; A.seg_tile_begin = L.seg_tile_begin;
    for (int i = 0; i < QADAM_MAX_WORKERS; ++i) {
        A.grad[i] = W.grad[i]; A.err[i] = W.err[i]; A.codes[i] = W.codes[i]; A.scales[i] = W.scales[i];
    }
    const dim3 grid(L.num_tiles), block(kBlockThreads);
    const int N = S.num_workers;
    // loads of up to four workers in flight per lane: more (eight) costs registers and occupancy
    // without a measurable gain
#define QADAM_LAUNCH_FUSED(R, WV)                                                                     \
    do {                                                                                              \
        if (N % 4 == 0) hipLaunchKernelGGL((k_fused<R, 4, WV>), grid, block, 0, L.stream, A);         \
        else if (N % 2 == 0 && R == 0) hipLaunchKernelGGL((k_fused<R, 2, WV>), grid, block, 0, L.stream, A); \
        else hipLaunchKernelGGL((k_fused<R, 1, WV>), grid, block, 0, L.stream, A);                    \
    } while (0)
    if (S.rounding == 0) {
        if (variant_w) QADAM_LAUNCH_FUSED(0, true); else QADAM_LAUNCH_FUSED(0, false);
    } else {
        if (variant_w) QADAM_LAUNCH_FUSED(1, true); else QADAM_LAUNCH_FUSED(1, false);
    }
#undef QADAM_LAUNCH_FUSED
    return hipGetLastError();
}

hipError_t launch_fused(const Launch& L, const StepScalars& S, const WorkerPtrs& W, const ServerPtrs& sp)
{
    return launch_fused_any(L, S, W, sp, false);
}

hipError_t launch_plain_messages(const Launch& L, const StepScalars& S, const WorkerPtrs& W, const ServerPtrs& sp,
                                 bool variant_w)
{
    if (L.num_tiles == 0) return hipSuccess;
    FusedArgs A;
    A.tiles = L.tiles; A.num_tiles = L.num_tiles;
    A.status = L.status; A.inv_scales = L.inv_scales; A.num_segments = L.num_segments; A.S = S; A.sp = sp;
    A.err_bound = L.err_bound; A.bound_factor = 0.0f;
    A.tile_max = L.tile_max; A.seg_tile_begin = L.seg_tile_begin;
    for (int i = 0; i < QADAM_MAX_WORKERS; ++i) {
        A.grad[i] = W.grad[i]; A.err[i] = W.err[i]; A.codes[i] = nullptr; A.scales[i] = nullptr;
    }
    const dim3 grid(L.num_tiles), block(kBlockThreads);
    const bool four = S.num_workers % 4 == 0;
#define QADAM_LAUNCH_PLAIN(R, WV)                                                                     \
    do {                                                                                              \
        if (four) hipLaunchKernelGGL((k_plain_messages<R, 4, WV>), grid, block, 0, L.stream, A);      \
        else hipLaunchKernelGGL((k_plain_messages<R, 1, WV>), grid, block, 0, L.stream, A);           \
    } while (0)
    if (S.rounding == 0) {
        if (variant_w) QADAM_LAUNCH_PLAIN(0, true); else QADAM_LAUNCH_PLAIN(0, false);
    } else {
        if (variant_w) QADAM_LAUNCH_PLAIN(1, true); else QADAM_LAUNCH_PLAIN(1, false);
    }
#undef QADAM_LAUNCH_PLAIN
    return hipGetLastError();
}

hipError_t launch_fused_w(const Launch& L, const StepScalars& S, const WorkerPtrs& W, const ServerPtrs& sp)
{
    return launch_fused_any(L, S, W, sp, true);
}

hipError_t launch_layer_sumsq(const Launch& L, const float* a, const float* b, double* out)
{
    if (L.num_segments == 0) return hipSuccess;
    SumsqArgs A;
    A.tiles = L.tiles; A.a = a; A.b = b; A.tile_sum = L.tile_sum; A.seg_tile_begin = L.seg_tile_begin; A.out = out;
    if (L.num_tiles > 0)
        hipLaunchKernelGGL(k_sumsq_tiles, dim3(L.num_tiles), dim3(kBlockThreads), 0, L.stream, A);
    hipLaunchKernelGGL(k_sumsq_layers, dim3(L.num_segments), dim3(kBlockThreads), 0, L.stream, A);
    return hipGetLastError();
}

hipError_t launch_worker_moments_w(const Launch& L, const StepScalars& S, const WorkerPtrs& W, int first_worker, int num)
{
    if (L.num_tiles == 0 || num == 0) return hipSuccess;
    MomentsWArgs A;
    A.tiles = L.tiles; A.num_tiles = L.num_tiles; A.S = S;
    for (int i = 0; i < QADAM_MAX_WORKERS; ++i) {
        A.grad[i] = W.grad[i]; A.mw[i] = W.mw[i]; A.vw[i] = W.vw[i]; A.err[i] = W.err[i];
    }
    A.tile_max = L.tile_max;
    A.first_worker = first_worker;
    hipLaunchKernelGGL(k_moments_w, dim3(L.num_tiles, num), dim3(kBlockThreads), 0, L.stream, A);
    return hipGetLastError();
}

// ================================================================================================
// Handle-free quantization of one segment without any allocation.
// The device memory the kernels need beyond the caller's buffers -- one maximum per tile, the
// reciprocal scale, the residual bound and a status word -- is this file-scope array.  Every GPU
// holds its own copy at its own address; host code must never pass the array's name to a kernel
// or a HIP call (on the host it is only a stand-in for the symbol): it uses the address that
// hipGetSymbolAddress returned for the current device.
// ================================================================================================
constexpr int kNoallocMaxTiles = (int)(kNoallocMaxElems / kDefaultTileElems);
constexpr int kNoallocExtraWords = 64;      // [0] reciprocal scale, [1] residual bound, [2] status, rest unused
constexpr int kMaxDevices = 64;
static __device__ __align__(256) uint32_t scratch[kNoallocMaxTiles + kNoallocExtraWords];

static uint32_t* g_scratch_ptr[kMaxDevices];          // per device, null until looked up
static std::mutex g_scratch_mutex;

static hipError_t scratch_for_current_device(uint32_t** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = static_cast<uint32_t*>(p);
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

hipError_t noalloc_prepare()
{
    uint32_t* p = nullptr;
    return scratch_for_current_device(&p);
}

// The three launches of qadam_worker_quantize for worker 0 of a one-segment vector of n elements,
// with tile records computed in the kernels and the scratch rows taken from the static array.
// Nothing of the array has to start at zero: every tile maximum, the reciprocal and the bound are
// written before they are read, and the status word is only ever OR-ed into and never read here.
hipError_t noalloc_quantize_segment(const StepScalars& S, int64_t n, const float* grad, float* err, uint32_t* codes,
                                    float* scale_out, hipStream_t stream)
{
    uint32_t* sc = nullptr;
    hipError_t e = scratch_for_current_device(&sc);
    if (e != hipSuccess) return e;
    const int num_tiles = (int)((n + kDefaultTileElems - 1) / kDefaultTileElems);
    uint32_t* tile_max = sc;
    float* inv_scale = reinterpret_cast<float*>(sc + kNoallocMaxTiles);
    float* err_bound = reinterpret_cast<float*>(sc + kNoallocMaxTiles + 1);
    uint32_t* status = sc + kNoallocMaxTiles + 2;

    if (num_tiles > 0) {
        AmaxArgs A;
        std::memset(&A, 0, sizeof A);
        A.tiles = nullptr; A.num_tiles = num_tiles; A.seg_len = n;
        A.grad[0] = grad; A.err[0] = err;
        A.tile_max = tile_max; A.first_worker = 0; A.num_segments = 1; A.status = status;
        hipLaunchKernelGGL(k_amax, dim3(num_tiles, 1), dim3(kBlockThreads), 0, stream, A);
    }
    ScaleArgs R;
    std::memset(&R, 0, sizeof R);
    R.scales[0] = scale_out; R.inv_scales = inv_scale; R.tile_max = tile_max; R.seg_tile_begin = nullptr;
    R.first_worker = 0; R.num_segments = 1; R.num_tiles = num_tiles;
    R.err_bound = err_bound; R.thr = nullptr;
    R.bound_factor = residual_bound_factor(S);
    R.sample_stride = kSampleStride;
    R.tiles = nullptr;
    hipLaunchKernelGGL(k_reduce_scales, dim3(1, 1), dim3(kBlockThreads), 0, stream, R);
    if (num_tiles > 0) {
        WorkerArgs W;
        std::memset(&W, 0, sizeof W);
        W.tiles = nullptr; W.num_tiles = num_tiles; W.seg_len = n;
        W.status = status; W.S = S;
        W.grad = grad; W.err = err; W.codes = codes; W.scales = scale_out; W.inv_scales = inv_scale;
        W.err_bound = err_bound; W.bound_factor = residual_bound_factor(S);
        W.tile_max = tile_max; W.seg_tile_begin = nullptr;
        W.worker = 0;
        hipLaunchKernelGGL((k_worker_quantize<0, false>), dim3(num_tiles), dim3(kBlockThreads), 0, stream, W);
    }
    return hipGetLastError();
}

}  // namespace qadam
