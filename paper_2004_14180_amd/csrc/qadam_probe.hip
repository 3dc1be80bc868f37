// Memory-system probes for MI355X (gfx950): the measurements behind the design decisions of the
// optimizer-step kernels.  A stand-alone program (no part of the library, nothing of the method's
// arithmetic): it prints what this GPU delivers to the access patterns the step uses, so that the
// kernels' bandwidth can be read against the part's practical ceilings rather than only against
// the published 8 TB/s.
//
//   streams    R read-only + U updated-in-place (+ small write-only) fp32 streams walked in lockstep,
//              one 16 KiB tile of every stream per workgroup, 128-bit non-temporal accesses:
//              the shape of the scale pass (R = 16, U = 0) and of the fused main pass
//              (R = 8 gradients, U = 12: errors, x, m, v, weight residual; codes as small writes);
//              then the write-heavy shapes of the code utilities (pure fill, 1 byte in per 4 bytes out)
//   placement  the main-pass shape again with its 20 buffers carved out of ONE allocation that spans the
//              device's memory: packed back to back from different offsets, and dealt alternately to the
//              two halves of the block -- where the buffers lie physically changes the rate by ~20 %
//   reread     one buffer of S bytes read many times inside one launch: where the caches
//              (4 MiB L2 per XCD, 256 MiB memory-side cache) stop helping
//   barrier    cost of a grid-wide wait among co-resident workgroups: cooperative-groups grid sync
//              and a hand-written hierarchical counter barrier (bounded spin), per barrier
//   parked     a single-pass worker quantize that keeps p = g + e in registers across a grid-wide
//              wait (scale of the round = max over all workgroups), against its byte count
//
// Build: hipcc --offload-arch=gfx950 -O3 (see build.py).  Run: qadam_probe.bin [streams|placement|reread|barrier|parked|all]
#include <hip/hip_cooperative_groups.h>
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

namespace cg = cooperative_groups;
typedef float f4 __attribute__((ext_vector_type(4)));

#define CK(x)                                                                               \
    do {                                                                                    \
        hipError_t err_ = (x);                                                              \
        if (err_ != hipSuccess) {                                                           \
            std::printf("HIP error %s at line %d\n", hipGetErrorString(err_), __LINE__);    \
            std::exit(1);                                                                   \
        }                                                                                   \
    } while (0)

static hipEvent_t ev0, ev1;

template <typename F>
static float best_ms(F launch, int reps = 5)
{
    float best = 1e30f;
    for (int r = 0; r < reps; ++r) {
        CK(hipEventRecord(ev0));
        launch();
        CK(hipEventRecord(ev1));
        CK(hipEventSynchronize(ev1));
        float ms;
        CK(hipEventElapsedTime(&ms, ev0, ev1));
        if (ms < best) best = ms;
    }
    return best;
}

// ------------------------------------------------------------------------------------------------
// streams
// ------------------------------------------------------------------------------------------------
constexpr int kMaxStreams = 24;
struct StreamArgs {
    const float* ro[kMaxStreams];   // read-only streams
    float* rw[kMaxStreams];         // updated in place ...
    float* wo[kMaxStreams];         // ... or, where non-null, read from rw[s] and written here (out of place)
    unsigned* small;                // one word per 32 elements and updated stream (stands in for the packed codes)
    int n_ro, n_rw;
};

// one workgroup = one tile of 4096 elements of every stream; a lane owns 4 x 4 consecutive floats
template <bool NT_STORE>
__global__ void __launch_bounds__(256) k_streams_t(StreamArgs A);
__global__ void __launch_bounds__(256) k_streams(StreamArgs A)
{
    const size_t base = (size_t)blockIdx.x * 4096 + threadIdx.x * 4;
    const bool out_of_place = A.wo[0] != nullptr;
    f4 acc[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) acc[k] = f4{0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < A.n_ro; ++s) {
        f4 v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(A.ro[s] + base + k * 1024));
#pragma unroll
        for (int k = 0; k < 4; ++k) acc[k] += v[k];
    }
    for (int s = 0; s < A.n_rw; ++s) {
        f4 v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(A.rw[s] + base + k * 1024));
        float* dst = out_of_place ? A.wo[s] : A.rw[s];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            acc[k] += v[k];
            __builtin_nontemporal_store(acc[k] * 0.5f, reinterpret_cast<f4*>(dst + base + k * 1024));
        }
        if ((threadIdx.x & 7) == 0) {
            const float t = acc[0].x + acc[1].y + acc[2].z + acc[3].w;
#pragma unroll
            for (int k = 0; k < 4; ++k)
                __builtin_nontemporal_store(__float_as_uint(t), A.small + ((size_t)s * gridDim.x * 4096 + base + k * 1024) / 32);
        }
    }
    if (A.n_rw == 0) {      // read-only: keep the loads alive
        const float t = acc[0].x + acc[1].y + acc[2].z + acc[3].w;
        if (t == 1234.5678f) A.small[0] = 1u;
    }
}

template <bool NT_STORE>
__global__ void __launch_bounds__(256) k_streams_t(StreamArgs A)
{
    const size_t base = (size_t)blockIdx.x * 4096 + threadIdx.x * 4;
    f4 acc[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) acc[k] = f4{0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < A.n_ro; ++s) {
        f4 v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(A.ro[s] + base + k * 1024));
#pragma unroll
        for (int k = 0; k < 4; ++k) acc[k] += v[k];
    }
    for (int s = 0; s < A.n_rw; ++s) {
        f4 v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(A.rw[s] + base + k * 1024));
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            acc[k] += v[k];
            if (NT_STORE) __builtin_nontemporal_store(acc[k] * 0.5f, reinterpret_cast<f4*>(A.rw[s] + base + k * 1024));
            else *reinterpret_cast<f4*>(A.rw[s] + base + k * 1024) = acc[k] * 0.5f;
        }
        if ((threadIdx.x & 7) == 0) {
            const float t = acc[0].x + acc[1].y + acc[2].z + acc[3].w;
#pragma unroll
            for (int k = 0; k < 4; ++k)
                __builtin_nontemporal_store(__float_as_uint(t), A.small + ((size_t)s * gridDim.x * 4096 + base + k * 1024) / 32);
        }
    }
    if (A.n_rw == 0) {      // read-only: keep the loads alive
        const float t = acc[0].x + acc[1].y + acc[2].z + acc[3].w;
        if (t == 1234.5678f) A.small[0] = 1u;
    }
}

// write-heavy shapes of the utilities: a workgroup writes one tile of 4096 floats and reads READ_Q quarters
// of a tile (0: pure fill; 1: the 1-byte-in / 4-bytes-out shape of a code-to-fp32 expansion)
template <int READ_Q, bool NT = true>
__global__ void __launch_bounds__(256) k_expand(const float* src, float* dst)
{
    const size_t base = (size_t)blockIdx.x * 4096 + threadIdx.x * 4;
    f4 a = f4{1.f, 2.f, 3.f, 4.f};
    if (READ_Q) a = __builtin_nontemporal_load(reinterpret_cast<const f4*>(src + (size_t)blockIdx.x * 1024 + threadIdx.x * 4));
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        if (NT) __builtin_nontemporal_store(a * (float)(k + 1), reinterpret_cast<f4*>(dst + base + k * 1024));
        else *reinterpret_cast<f4*>(dst + base + k * 1024) = a * (float)(k + 1);
    }
}

// the main-pass shape once more with every lane's 128-bit access ld_off / st_off floats (0..3) off the 16-byte
// grid (dword-aligned vector types): what a layer list whose offsets are not multiples of four costs
typedef f4 f4_a4 __attribute__((aligned(4)));
__global__ void __launch_bounds__(256) k_streams_off(StreamArgs A, int ld_off, int st_off)
{
    const size_t base = (size_t)blockIdx.x * 4096 + threadIdx.x * 4;
    f4 acc[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) acc[k] = f4{0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < A.n_ro; ++s) {
        f4 v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = *reinterpret_cast<const f4_a4*>(A.ro[s] + base + k * 1024 + ld_off);
#pragma unroll
        for (int k = 0; k < 4; ++k) acc[k] += v[k];
    }
    for (int s = 0; s < A.n_rw; ++s) {
        f4 v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = *reinterpret_cast<const f4_a4*>(A.rw[s] + base + k * 1024 + ld_off);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            acc[k] += v[k];
            __builtin_nontemporal_store(acc[k] * 0.5f, reinterpret_cast<f4_a4*>(A.rw[s] + base + k * 1024 + st_off));
        }
        if ((threadIdx.x & 7) == 0) {
            const float t = acc[0].x + acc[1].y + acc[2].z + acc[3].w;
#pragma unroll
            for (int k = 0; k < 4; ++k)
                __builtin_nontemporal_store(__float_as_uint(t), A.small + ((size_t)s * gridDim.x * 4096 + base + k * 1024) / 32);
        }
    }
}

static void probe_streams()
{
    const size_t n = (size_t)1 << 29;        // 2 GiB per stream
    const int total = 20;
    std::vector<float*> buf(total);
    for (int i = 0; i < total; ++i) {
        CK(hipMalloc(reinterpret_cast<void**>(&buf[i]), n * 4));
        CK(hipMemset(buf[i], 0, n * 4));
    }
    unsigned* small;
    CK(hipMalloc(reinterpret_cast<void**>(&small), (size_t)12 * n / 32 * 4 + 4096));
    std::printf("streams: %d buffers of 2 GiB, one 16 KiB tile of every stream per workgroup, 128-bit non-temporal accesses\n", total);
    struct Case { const char* name; int ro, rw; };
    const Case cases[] = {
        {"1 read-only stream", 1, 0},
        {"16 read-only streams (scale pass: g, e of 8 workers)", 16, 0},
        {"1 stream updated in place", 0, 1},
        {"12 streams updated in place", 0, 12},
        {"8 read-only + 12 updated in place + small writes (main pass: 20 reads, 13 writes)", 8, 12},
    };
    for (const Case& c : cases) {
        StreamArgs A;
        std::memset(&A, 0, sizeof A);
        A.n_ro = c.ro; A.n_rw = c.rw; A.small = small;
        for (int i = 0; i < c.ro; ++i) A.ro[i] = buf[i];
        for (int i = 0; i < c.rw; ++i) A.rw[i] = buf[c.ro + i];
        const float ms = best_ms([&] { hipLaunchKernelGGL(k_streams, dim3((unsigned)(n / 4096)), dim3(256), 0, 0, A); });
        const double bytes = (double)n * 4.0 * (c.ro + 2.0 * c.rw) + (double)c.rw * n / 8.0;
        std::printf("  %-84s %7.1f GB/s  (%.3f ms)\n", c.name, bytes / ms / 1e6, ms);
        if (c.rw) {
            const float ms2 = best_ms([&] { hipLaunchKernelGGL(k_streams_t<false>, dim3((unsigned)(n / 4096)), dim3(256), 0, 0, A); });
            std::printf("  %-84s %7.1f GB/s  (%.3f ms)\n", "  the same with ordinary (cached) stores", bytes / ms2 / 1e6, ms2);
        }
        std::fflush(stdout);
    }
    {
        // grid one workgroup short, so that the shifted accesses of the last one stay inside the buffers
        StreamArgs A;
        std::memset(&A, 0, sizeof A);
        A.n_ro = 8; A.n_rw = 12; A.small = small;
        for (int i = 0; i < 8; ++i) A.ro[i] = buf[i];
        for (int i = 0; i < 12; ++i) A.rw[i] = buf[8 + i];
        const unsigned wgs = (unsigned)(n / 4096) - 1;
        const double bytes = (double)wgs * 4096 * 4.0 * (8 + 24) + 12.0 * wgs * 4096 / 8.0;
        const int offs[4][2] = {{0, 0}, {1, 1}, {1, 0}, {0, 1}};
        const char* names[4] = {"main-pass shape through dword-aligned vector types, on the 16-byte grid (cached loads)",
                                "  loads and stores 4 bytes off the grid", "  loads 4 bytes off the grid, stores on it",
                                "  loads on the grid, stores 4 bytes off it"};
        for (int c = 0; c < 4; ++c) {
            const float ms = best_ms([&] { hipLaunchKernelGGL(k_streams_off, dim3(wgs), dim3(256), 0, 0, A, offs[c][0], offs[c][1]); });
            std::printf("  %-84s %7.1f GB/s  (%.3f ms)\n", names[c], bytes / ms / 1e6, ms);
        }
        std::fflush(stdout);
    }
    {
        const float ms = best_ms([&] { hipLaunchKernelGGL(k_expand<0>, dim3((unsigned)(n / 4096)), dim3(256), 0, 0, buf[0], buf[1]); });
        std::printf("  %-84s %7.1f GB/s  (%.3f ms)\n", "1 write-only stream", (double)n * 4.0 / ms / 1e6, ms);
    }
    {
        const float ms = best_ms([&] { hipLaunchKernelGGL((k_expand<0, false>), dim3((unsigned)(n / 4096)), dim3(256), 0, 0, buf[0], buf[1]); });
        std::printf("  %-84s %7.1f GB/s  (%.3f ms)\n", "1 write-only stream, ordinary (cached) stores", (double)n * 4.0 / ms / 1e6, ms);
    }
    {
        const float ms = best_ms([&] { hipLaunchKernelGGL(k_expand<1>, dim3((unsigned)(n / 4096)), dim3(256), 0, 0, buf[0], buf[1]); });
        std::printf("  %-84s %7.1f GB/s  (%.3f ms)\n", "1 byte read per 4 bytes written (expansion of 8-bit codes to fp32)", (double)n * 5.0 / ms / 1e6, ms);
    }
    {
        const float ms = best_ms([&] { hipLaunchKernelGGL((k_expand<1, false>), dim3((unsigned)(n / 4096)), dim3(256), 0, 0, buf[0], buf[1]); });
        std::printf("  %-84s %7.1f GB/s  (%.3f ms)\n", "1 byte read per 4 bytes written, ordinary (cached) stores", (double)n * 5.0 / ms / 1e6, ms);
    }
    std::fflush(stdout);
    for (float* p : buf) CK(hipFree(p));
    CK(hipFree(small));
}

// ------------------------------------------------------------------------------------------------
// placement: a fresh process's single large allocation is physically contiguous, so offsets inside
// it are (up to the small part of memory already in use) physical positions
// ------------------------------------------------------------------------------------------------
static void probe_placement()
{
    size_t free_b = 0, total_b = 0;
    CK(hipMemGetInfo(&free_b, &total_b));
    const size_t GiB = (size_t)1 << 30;
    const size_t arena_bytes = (free_b - 4 * GiB) / GiB * GiB;
    char* arena;
    CK(hipMalloc(reinterpret_cast<void**>(&arena), arena_bytes));
    const size_t n = (size_t)1 << 30;         // 4 GiB per stream, 20 streams = 80 GiB
    const size_t buf = n * 4;
    unsigned* small;
    CK(hipMalloc(reinterpret_cast<void**>(&small), (size_t)12 * n / 32 * 4 + 4096));
    std::printf("placement: main-pass shape (8 read-only + 12 updated in place, 4 GiB each) inside one allocation of %zu GiB "
                "(device total %zu GiB)\n", arena_bytes / GiB, total_b / GiB);
    auto run = [&](const char* name, const std::vector<size_t>& offs) {
        StreamArgs A;
        std::memset(&A, 0, sizeof A);
        A.n_ro = 8; A.n_rw = 12; A.small = small;
        for (int i = 0; i < 20; ++i) {
            if (offs[i] + buf > arena_bytes) { std::printf("  %-58s does not fit\n", name); return; }
            CK(hipMemsetAsync(arena + offs[i], 0, buf, 0));
        }
        // the updated streams first in the order of placement, as the library's layout deals them
        for (int i = 0; i < 12; ++i) A.rw[i] = reinterpret_cast<float*>(arena + offs[i]);
        for (int i = 0; i < 8; ++i) A.ro[i] = reinterpret_cast<const float*>(arena + offs[12 + i]);
        const float ms = best_ms([&] { hipLaunchKernelGGL(k_streams, dim3((unsigned)(n / 4096)), dim3(256), 0, 0, A); }, 3);
        const double bytes = (double)n * 4.0 * (8 + 2.0 * 12) + 12.0 * n / 8.0;
        std::printf("  %-58s %7.1f GB/s  (%.3f ms)\n", name, bytes / ms / 1e6, ms);
        std::fflush(stdout);
    };
    char name[128];
    for (size_t base_gib = 0; base_gib + 80 <= arena_bytes / GiB; base_gib += 24) {
        std::vector<size_t> offs(20);
        for (int i = 0; i < 20; ++i) offs[i] = base_gib * GiB + (size_t)i * buf;
        std::snprintf(name, sizeof name, "packed back to back from %3zu GiB", base_gib);
        run(name, offs);
    }
    for (int groups : {2, 3}) {
        std::vector<size_t> offs(20), fill(groups, 0);
        const size_t region = arena_bytes / groups / GiB * GiB;
        for (int i = 0; i < 20; ++i) {
            offs[i] = (size_t)(i % groups) * region + fill[i % groups];
            fill[i % groups] += buf;
        }
        std::snprintf(name, sizeof name, "dealt alternately to %d equal parts of the block", groups);
        run(name, offs);
    }
    // the same 20 reads and 13 writes with every updated stream written to a second buffer instead of in place
    // (32 buffers): does it pay to keep what is read and what is written in different parts of the memory?
    auto run_oop = [&](const char* name, const std::vector<size_t>& rd, const std::vector<size_t>& wr) {
        StreamArgs A;
        std::memset(&A, 0, sizeof A);
        A.n_ro = 8; A.n_rw = 12; A.small = small;
        for (size_t o : rd) if (o + buf > arena_bytes) { std::printf("  %-58s does not fit\n", name); return; }
        for (size_t o : wr) if (o + buf > arena_bytes) { std::printf("  %-58s does not fit\n", name); return; }
        for (int i = 0; i < 12; ++i) A.rw[i] = reinterpret_cast<float*>(arena + rd[i]);
        for (int i = 0; i < 8; ++i) A.ro[i] = reinterpret_cast<const float*>(arena + rd[12 + i]);
        for (int i = 0; i < 12; ++i) A.wo[i] = reinterpret_cast<float*>(arena + wr[i]);
        const float ms = best_ms([&] { hipLaunchKernelGGL(k_streams, dim3((unsigned)(n / 4096)), dim3(256), 0, 0, A); }, 3);
        const double bytes = (double)n * 4.0 * (8 + 2.0 * 12) + 12.0 * n / 8.0;
        std::printf("  %-58s %7.1f GB/s  (%.3f ms)\n", name, bytes / ms / 1e6, ms);
        std::fflush(stdout);
    };
    if (arena_bytes >= 136 * GiB) {
        const size_t half = arena_bytes / 2 / GiB * GiB;
        std::vector<size_t> rd(20), wr(12);
        for (int i = 0; i < 20; ++i) rd[i] = (size_t)i * buf;
        for (int i = 0; i < 12; ++i) wr[i] = half + (size_t)i * buf;
        run_oop("out of place: 20 read from the lower half, 12 written to the upper", rd, wr);
        for (int i = 0; i < 20; ++i) rd[i] = (size_t)(i & 1) * half + (size_t)(i / 2) * buf;
        for (int i = 0; i < 12; ++i) wr[i] = (size_t)((i + 1) & 1) * half + (size_t)(10 + i / 2) * buf;
        run_oop("out of place: reads and writes dealt to both halves", rd, wr);
        for (int i = 0; i < 20; ++i) rd[i] = (size_t)i * buf;
        for (int i = 0; i < 12; ++i) wr[i] = (size_t)(20 + i) * buf;
        run_oop("out of place: all 32 buffers packed back to back from 0", rd, wr);
    }
    CK(hipFree(small));
    CK(hipFree(arena));
}

// ------------------------------------------------------------------------------------------------
// reread
// ------------------------------------------------------------------------------------------------
template <int NT>
__global__ void __launch_bounds__(256) k_reread(const f4* __restrict__ p, size_t n4, int sweeps, float* out)
{
    float acc = 0.f;
    const size_t stride = (size_t)gridDim.x * 1024;
    for (int r = 0; r < sweeps; ++r) {
        for (size_t j = (size_t)blockIdx.x * 1024 + threadIdx.x; j < n4; j += stride) {
            f4 v[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const size_t jj = j + 256 * k < n4 ? j + 256 * k : j;
                v[k] = NT ? __builtin_nontemporal_load(p + jj) : p[jj];
            }
            acc += v[0].x + v[1].y + v[2].z + v[3].w;
        }
    }
    if (acc == 12345.678f) out[0] = acc;
}

static void probe_reread()
{
    float *a, *out;
    const size_t cap = (size_t)4 << 30;
    CK(hipMalloc(reinterpret_cast<void**>(&a), cap));
    CK(hipMalloc(reinterpret_cast<void**>(&out), 256));
    CK(hipMemset(a, 1, cap));
    std::printf("reread: one buffer read repeatedly inside one launch (2048 workgroups, 4 x 128-bit loads per lane in flight)\n");
    const size_t sizes_mib[] = {16, 32, 64, 128, 192, 256, 384, 512, 1024, 4096};
    for (int nt = 0; nt < 2; ++nt)
        for (size_t mib : sizes_mib) {
            const size_t bytes = mib << 20, n4 = bytes / 16;
            int sweeps = (int)(((size_t)16 << 30) / bytes);
            if (sweeps < 2) sweeps = 2;
            const float ms = best_ms([&] {
                if (nt) hipLaunchKernelGGL(k_reread<1>, dim3(2048), dim3(256), 0, 0, reinterpret_cast<const f4*>(a), n4, sweeps, out);
                else hipLaunchKernelGGL(k_reread<0>, dim3(2048), dim3(256), 0, 0, reinterpret_cast<const f4*>(a), n4, sweeps, out);
            }, 3);
            std::printf("  %-12s %5zu MiB x %4d sweeps: %7.0f GB/s\n", nt ? "non-temporal" : "plain", mib, sweeps,
                        (double)bytes * sweeps / ms / 1e6);
            std::fflush(stdout);
        }
    CK(hipFree(a));
    CK(hipFree(out));
}

// ------------------------------------------------------------------------------------------------
// barrier: every kernel here is launched cooperatively (the runtime refuses a grid that cannot be
// co-resident) and every wait is bounded, so all waves reach the end whatever happens
// ------------------------------------------------------------------------------------------------
struct Barrier {
    unsigned group[8][64];  // one counter per residue of the workgroup index mod 8, 256 bytes apart
    unsigned global[64];
    unsigned generation[64];
    unsigned timed_out[64];
};

__device__ __forceinline__ void counter_barrier(Barrier* b, unsigned round, unsigned per_group, unsigned spin_limit)
{
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned g = blockIdx.x & 7u;
        const unsigned seen = __hip_atomic_fetch_add(&b->group[g][0], 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        if (seen == per_group * (round + 1u) - 1u) {
            const unsigned seen2 = __hip_atomic_fetch_add(&b->global[0], 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
            if (seen2 == 8u * (round + 1u) - 1u)
                __hip_atomic_store(&b->generation[0], round + 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        }
        unsigned spins = 0;
        // once any wait has timed out the measurement is void: later barriers no longer wait at all
        while (__hip_atomic_load(&b->generation[0], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) < round + 1u &&
               __hip_atomic_load(&b->timed_out[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u) {
            __builtin_amdgcn_s_sleep(2);
            if (++spins > spin_limit) {
                __hip_atomic_store(&b->timed_out[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
        }
    }
    __syncthreads();
}

__global__ void __launch_bounds__(256) k_barrier_own(Barrier* b, int rounds, unsigned per_group, unsigned* out)
{
    unsigned acc = 0;
    for (int r = 0; r < rounds; ++r) {
        acc += r;
        counter_barrier(b, r, per_group, 1u << 18);
    }
    if (acc == 0xffffffffu) out[0] = acc;
}

__global__ void __launch_bounds__(256) k_barrier_cg(int rounds, unsigned* out)
{
    cg::grid_group grid = cg::this_grid();
    unsigned acc = 0;
    for (int r = 0; r < rounds; ++r) {
        acc += r;
        grid.sync();
    }
    if (acc == 0xffffffffu) out[0] = acc;
}

static void probe_barrier(int num_cus)
{
    unsigned* out;
    Barrier* bar;
    CK(hipMalloc(reinterpret_cast<void**>(&out), 256));
    CK(hipMalloc(reinterpret_cast<void**>(&bar), sizeof(Barrier)));
    std::printf("barrier: grid-wide wait among co-resident 256-thread workgroups, 1000 barriers per launch\n");
    for (int per_cu : {1, 2, 4}) {
        int grid = num_cus * per_cu, rounds = 1000;
        unsigned per_group = (unsigned)grid / 8u;
        {
            void* args[] = {&rounds, &out};
            const float ms = best_ms([&] { CK(hipLaunchCooperativeKernel((void*)k_barrier_cg, dim3(grid), dim3(256), args, 0, 0)); }, 3);
            std::printf("  cooperative-groups grid sync, %4d workgroups: %6.2f us per barrier\n", grid, ms * 1000.f / rounds);
        }
        {
            void* args[] = {&bar, &rounds, &per_group, &out};
            const float ms = best_ms([&] {
                CK(hipMemsetAsync(bar, 0, sizeof(Barrier), 0));
                CK(hipLaunchCooperativeKernel((void*)k_barrier_own, dim3(grid), dim3(256), args, 0, 0));
            }, 3);
            Barrier hb;
            CK(hipMemcpy(&hb, bar, sizeof hb, hipMemcpyDeviceToHost));
            std::printf("  counter barrier (8 groups + 1),  %4d workgroups: %6.2f us per barrier%s\n", grid, ms * 1000.f / rounds,
                        hb.timed_out[0] ? "  [a wait timed out: figure invalid]" : "");
        }
        std::fflush(stdout);
    }
    CK(hipFree(out));
    CK(hipFree(bar));
}

// ------------------------------------------------------------------------------------------------
// parked: per round every workgroup loads Q x 1024 elements of g and e, keeps p = g + e in
// registers, publishes its maximum, waits for all workgroups, folds their maxima into the scale of
// the round and only then quantizes (3-bit levels) and writes the residual and the codes: one trip
// through memory per buffer (12.375 B per element) at the price of one grid-wide wait per round
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ unsigned wave_max(unsigned v)
{
    for (int d = 32; d >= 1; d >>= 1) {
        const unsigned o = (unsigned)__shfl_xor((int)v, d, 64);
        v = o > v ? o : v;
    }
    return v;
}

template <int Q>
__global__ void __launch_bounds__(256, 2) k_parked(const float* __restrict__ g, float* __restrict__ e,
                                                   unsigned* __restrict__ codes, unsigned* __restrict__ wg_max,
                                                   Barrier* b, int rounds, unsigned per_group)
{
    __shared__ unsigned part[4];
    const size_t chunk = (size_t)gridDim.x * 1024 * Q;
    for (int r = 0; r < rounds; ++r) {
        f4 p[Q];
        unsigned local = 0;
#pragma unroll
        for (int k = 0; k < Q; ++k) {
            const size_t off = (size_t)r * chunk + ((size_t)k * gridDim.x + blockIdx.x) * 1024 + threadIdx.x * 4;
            p[k] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(g + off)) +
                   __builtin_nontemporal_load(reinterpret_cast<const f4*>(e + off));
        }
#pragma unroll
        for (int k = 0; k < Q; ++k)
            for (int j = 0; j < 4; ++j) {
                const unsigned ab = __float_as_uint(p[k][j]) & 0x7fffffffu;
                local = ab > local ? ab : local;
            }
        const unsigned wm = wave_max(local);
        if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = wm;
        __syncthreads();
        if (threadIdx.x == 0) {
            unsigned bm = part[0];
            for (int w = 1; w < 4; ++w) bm = part[w] > bm ? part[w] : bm;
            __hip_atomic_store(&wg_max[(r & 1) * gridDim.x + blockIdx.x], bm, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        counter_barrier(b, r, per_group, 1u << 18);
        unsigned m = 0;
        for (int i = threadIdx.x; i < (int)gridDim.x; i += 256) {
            const unsigned v = __hip_atomic_load(&wg_max[(r & 1) * gridDim.x + i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            m = v > m ? v : m;
        }
        m = wave_max(m);
        __syncthreads();
        if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = m;
        __syncthreads();
        m = part[0];
        for (int w = 1; w < 4; ++w) m = part[w] > m ? part[w] : m;
        const float s = __uint_as_float(m);
        const float inv_s = s > 0.f ? 1.0f / s : 0.f;
#pragma unroll
        for (int k = 0; k < Q; ++k) {
            const size_t off = (size_t)r * chunk + ((size_t)k * gridDim.x + blockIdx.x) * 1024 + threadIdx.x * 4;
            f4 en;
            unsigned cd = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const unsigned ab = __float_as_uint(p[k][j] * inv_s) & 0x7fffffffu;
                unsigned lvl = (ab + 0x00400000u) & 0x7f800000u;
                lvl = lvl > 0x3e800000u ? lvl : 0x3e800000u;
                lvl = ab >= 0x3e000000u ? lvl : 0u;
                float q = s * __uint_as_float(lvl);
                q = __uint_as_float(__float_as_uint(q) | (__float_as_uint(p[k][j]) & 0x80000000u));
                en[j] = p[k][j] - q;
                cd |= (lvl >> 23) << (8 * j);
            }
            __builtin_nontemporal_store(en, reinterpret_cast<f4*>(e + off));
            if ((threadIdx.x & 7) < 3) __builtin_nontemporal_store(cd, codes + (off >> 5) * 3 + (threadIdx.x & 7));
        }
    }
}

template <int Q>
static void run_parked(int num_cus, const float* g, float* e, unsigned* codes, unsigned* wg_max, Barrier* bar, size_t n)
{
    int grid = num_cus * 2;
    const size_t chunk = (size_t)grid * 1024 * Q;
    int rounds = (int)(n / chunk);
    unsigned per_group = (unsigned)grid / 8u;
    void* args[] = {&g, &e, &codes, &wg_max, &bar, &rounds, &per_group};
    const float ms = best_ms([&] {
        CK(hipMemsetAsync(bar, 0, sizeof(Barrier), 0));
        CK(hipLaunchCooperativeKernel((void*)k_parked<Q>, dim3(grid), dim3(256), args, 0, 0));
    }, 3);
    Barrier hb;
    CK(hipMemcpy(&hb, bar, sizeof hb, hipMemcpyDeviceToHost));
    const double bytes = (double)rounds * chunk * 12.375;
    std::printf("  %3d floats parked per lane: %4d rounds of %5.1f M elements, %6.1f us per round, %7.1f GB/s on 12.375 B/element%s\n",
                4 * Q, rounds, chunk / 1e6, ms * 1000.f / rounds, bytes / ms / 1e6,
                hb.timed_out[0] ? "  [a wait timed out: figure invalid]" : "");
    std::fflush(stdout);
}

static void probe_parked(int num_cus)
{
    const size_t n = (size_t)1 << 30;
    float *g, *e;
    unsigned *codes, *wg_max;
    Barrier* bar;
    CK(hipMalloc(reinterpret_cast<void**>(&g), n * 4));
    CK(hipMalloc(reinterpret_cast<void**>(&e), n * 4));
    CK(hipMalloc(reinterpret_cast<void**>(&codes), n / 32 * 3 * 4 + 4096));
    CK(hipMalloc(reinterpret_cast<void**>(&wg_max), 1 << 16));
    CK(hipMalloc(reinterpret_cast<void**>(&bar), sizeof(Barrier)));
    CK(hipMemset(g, 0x3c, n * 4));
    CK(hipMemset(e, 0x3b, n * 4));
    std::printf("parked: single-pass worker quantize with p kept in registers across a grid-wide wait, %d workgroups, 4 GiB of g and of e\n",
                num_cus * 2);
    std::printf("  (the two-pass design it would replace moves 20.4 B per element at the rates of the streams probe)\n");
    run_parked<16>(num_cus, g, e, codes, wg_max, bar, n);
    run_parked<24>(num_cus, g, e, codes, wg_max, bar, n);
    run_parked<32>(num_cus, g, e, codes, wg_max, bar, n);
    CK(hipFree(g)); CK(hipFree(e)); CK(hipFree(codes)); CK(hipFree(wg_max)); CK(hipFree(bar));
}

int main(int argc, char** argv)
{
    const char* what = argc > 1 ? argv[1] : "all";
    hipDeviceProp_t prop;
    CK(hipGetDeviceProperties(&prop, 0));
    std::printf("device: %s, %d compute units\n", prop.gcnArchName, prop.multiProcessorCount);
    CK(hipEventCreate(&ev0));
    CK(hipEventCreate(&ev1));
    const bool all = std::strcmp(what, "all") == 0;
    if (all || std::strcmp(what, "streams") == 0) probe_streams();
    if (all || std::strcmp(what, "placement") == 0) probe_placement();
    if (all || std::strcmp(what, "reread") == 0) probe_reread();
    if (all || std::strcmp(what, "barrier") == 0) probe_barrier(prop.multiProcessorCount);
    if (all || std::strcmp(what, "parked") == 0) probe_parked(prop.multiProcessorCount);
    return 0;
}
