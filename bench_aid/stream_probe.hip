// The benchmark's measurement aid, built into its own shared object: not part of the MG-WFBP library and not
// part of the method.
//   bench_aid_stream_probe  streams a chosen mix of read-only, write-only and updated-in-place binary32
//                           arrays through the GPU with the access shape of the pipeline kernels (one workgroup
//                           of 256 lanes per 2048-element tile, 16-byte non-temporal accesses, every load of a
//                           tile issued before its first store), so that bench.py can report what the bare
//                           access pattern of a mode reaches next to what the real kernel reaches;
//   bench_aid_cache_scrub   displaces the contents of the memory-side cache between timed steps.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "stream_probe.h"

#define AID_EINVAL (-1)
#define AID_EHIP (-3)

namespace {

constexpr int PROBE_MAX = 16;
constexpr int PROBE_TILE = 2048;
constexpr int PROBE_BLOCK = 256;

typedef float pf4 __attribute__((ext_vector_type(4)));
#define PROBE_GLOBAL __attribute__((address_space(1)))

struct ProbePtrs {
    const float* r[PROBE_MAX];
    float* w[PROBE_MAX];
    float* x[PROBE_MAX];
};

template <int R, int W, int X>
__global__ void __launch_bounds__(PROBE_BLOCK) bench_aid_probe_kernel(const ProbePtrs P) {
    const int64_t base = static_cast<int64_t>(blockIdx.x) * PROBE_TILE + threadIdx.x * 4;
    pf4 a[2][R > 0 ? R : 1], xv[2][X > 0 ? X : 1];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
#pragma unroll
        for (int i = 0; i < R; ++i)
            a[u][i] = __builtin_nontemporal_load((const PROBE_GLOBAL pf4*)(P.r[i] + base + u * 1024));
#pragma unroll
        for (int i = 0; i < X; ++i)
            xv[u][i] = __builtin_nontemporal_load((const PROBE_GLOBAL pf4*)(P.x[i] + base + u * 1024));
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        pf4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < R; ++i) s = s + a[u][i];
#pragma unroll
        for (int i = 0; i < W; ++i) {
            pf4 val = {1.f, 1.f, 1.f, 1.f};
            if constexpr (R > 0) val = a[u][i % (R > 0 ? R : 1)];
            __builtin_nontemporal_store(val, (PROBE_GLOBAL pf4*)(P.w[i] + base + u * 1024));
        }
#pragma unroll
        for (int i = 0; i < X; ++i)
            __builtin_nontemporal_store(xv[u][i] + s, (PROBE_GLOBAL pf4*)(P.x[i] + base + u * 1024));
        if constexpr (X == 0 && R > 0) {
            // nothing consumes the sum of the inputs in this mix: an empty asm statement does, so that every
            // read-only array is really read
            asm volatile("" ::"v"(s[0]), "v"(s[1]), "v"(s[2]), "v"(s[3]));
        }
    }
}

template <int R, int W, int X>
int probe_launch(const ProbePtrs& P, uint64_t tiles, hipStream_t stream) {
    hipLaunchKernelGGL((bench_aid_probe_kernel<R, W, X>), dim3(static_cast<unsigned>(tiles)), dim3(PROBE_BLOCK), 0,
                       stream, P);
    return hipGetLastError() == hipSuccess ? 0 : AID_EHIP;
}

template <int R, int W>
int probe_by_x(int x, const ProbePtrs& P, uint64_t tiles, hipStream_t s) {
    switch (x) {
        case 0: return probe_launch<R, W, 0>(P, tiles, s);
        case 1: return probe_launch<R, W, 1>(P, tiles, s);
        case 2: return probe_launch<R, W, 2>(P, tiles, s);
        default: return AID_EINVAL;
    }
}

template <int R>
int probe_by_w(int w, int x, const ProbePtrs& P, uint64_t tiles, hipStream_t s) {
    switch (w) {
        case 0: return probe_by_x<R, 0>(x, P, tiles, s);
        case 1: return probe_by_x<R, 1>(x, P, tiles, s);
        case 2: return probe_by_x<R, 2>(x, P, tiles, s);
        case 4: return probe_by_x<R, 4>(x, P, tiles, s);
        case 8: return probe_by_x<R, 8>(x, P, tiles, s);
        case 16: return probe_by_x<R, 16>(x, P, tiles, s);
        default: return AID_EINVAL;
    }
}

// The same traffic walked one array at a time: a workgroup of B lanes owns U * B * 4 consecutive elements, loads
// its part of read array i, stores it to write array i (if there is one), adds it to a running sum, goes on to
// array i + 1, and finally updates the X arrays one after the other.  A lane never has more than U loads in
// flight; the unused dynamic LDS of the launch bounds the workgroups per compute unit.
template <int B, int U>
__global__ void __launch_bounds__(B) bench_aid_paced_probe_kernel(const ProbePtrs P, int n_read, int n_write, int n_update) {
    const int64_t base = static_cast<int64_t>(blockIdx.x) * (U * B * 4) + threadIdx.x * 4;
    pf4 acc[U];
#pragma unroll
    for (int u = 0; u < U; ++u) acc[u] = pf4{0.f, 0.f, 0.f, 0.f};
    for (int i = 0; i < n_read; ++i) {
        pf4 g[U];
#pragma unroll
        for (int u = 0; u < U; ++u) g[u] = __builtin_nontemporal_load((const PROBE_GLOBAL pf4*)(P.r[i] + base + u * (B * 4)));
        if (i < n_write) {
#pragma unroll
            for (int u = 0; u < U; ++u) __builtin_nontemporal_store(g[u], (PROBE_GLOBAL pf4*)(P.w[i] + base + u * (B * 4)));
        }
#pragma unroll
        for (int u = 0; u < U; ++u) acc[u] = acc[u] + g[u];
        __builtin_amdgcn_sched_barrier(0);
    }
    for (int i = n_read; i < n_write; ++i) {            // more write arrays than read arrays: constants
#pragma unroll
        for (int u = 0; u < U; ++u)
            __builtin_nontemporal_store(pf4{1.f, 1.f, 1.f, 1.f}, (PROBE_GLOBAL pf4*)(P.w[i] + base + u * (B * 4)));
    }
    for (int j = 0; j < n_update; ++j) {
        pf4 xv[U];
#pragma unroll
        for (int u = 0; u < U; ++u) xv[u] = __builtin_nontemporal_load((const PROBE_GLOBAL pf4*)(P.x[j] + base + u * (B * 4)));
#pragma unroll
        for (int u = 0; u < U; ++u) __builtin_nontemporal_store(xv[u] + acc[u], (PROBE_GLOBAL pf4*)(P.x[j] + base + u * (B * 4)));
        __builtin_amdgcn_sched_barrier(0);
    }
    if (n_update == 0 && n_write == 0) {
        // nothing consumes the sums in a read-only mix: an empty asm statement does
#pragma unroll
        for (int u = 0; u < U; ++u) asm volatile("" ::"v"(acc[u][0]), "v"(acc[u][1]), "v"(acc[u][2]), "v"(acc[u][3]));
    }
}

template <int B, int U>
int paced_launch(const ProbePtrs& P, int r, int w, int x, uint64_t elems, size_t lds, hipStream_t s) {
    const uint64_t chunk = static_cast<uint64_t>(U) * B * 4;
    if (elems % chunk != 0 || elems / chunk > 0x7fffffffull) return AID_EINVAL;
    hipLaunchKernelGGL((bench_aid_paced_probe_kernel<B, U>), dim3(static_cast<unsigned>(elems / chunk)), dim3(B), lds, s,
                       P, r, w, x);
    return hipGetLastError() == hipSuccess ? 0 : AID_EHIP;
}

// first half -> second half, ordinary (cacheable) 16-byte accesses; one workgroup per 2048 elements
__global__ void __launch_bounds__(PROBE_BLOCK) bench_aid_scrub_kernel(const pf4* src, pf4* dst) {
    const int64_t v = static_cast<int64_t>(blockIdx.x) * (PROBE_TILE / 4) + threadIdx.x;
    const pf4 a = src[v], b = src[v + PROBE_BLOCK];
    dst[v] = a;
    dst[v + PROBE_BLOCK] = b;
}

}  // namespace

extern "C" int bench_aid_paced_probe(const float* const* read_ptrs, int32_t n_read, float* const* write_ptrs,
                                     int32_t n_write, float* const* update_ptrs, int32_t n_update, uint64_t elems,
                                     int32_t block_lanes, int32_t vectors_per_step, uint32_t lds_bytes,
                                     void* hip_stream) {
    if (n_read < 0 || n_write < 0 || n_update < 0 || n_read + n_write + n_update == 0) return AID_EINVAL;
    if (n_read > PROBE_MAX || n_write > PROBE_MAX || n_update > PROBE_MAX) return AID_EINVAL;
    if ((n_read && !read_ptrs) || (n_write && !write_ptrs) || (n_update && !update_ptrs)) return AID_EINVAL;
    if (elems == 0 || lds_bytes > (64u << 10)) return AID_EINVAL;
    ProbePtrs P = {};
    for (int i = 0; i < n_read; ++i) if ((P.r[i] = read_ptrs[i]) == nullptr) return AID_EINVAL;
    for (int i = 0; i < n_write; ++i) if ((P.w[i] = write_ptrs[i]) == nullptr) return AID_EINVAL;
    for (int i = 0; i < n_update; ++i) if ((P.x[i] = update_ptrs[i]) == nullptr) return AID_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const int key = block_lanes * 10 + vectors_per_step;
    switch (key) {
        case 641: return paced_launch<64, 1>(P, n_read, n_write, n_update, elems, lds_bytes, s);
        case 1281: return paced_launch<128, 1>(P, n_read, n_write, n_update, elems, lds_bytes, s);
        case 1282: return paced_launch<128, 2>(P, n_read, n_write, n_update, elems, lds_bytes, s);
        case 2561: return paced_launch<256, 1>(P, n_read, n_write, n_update, elems, lds_bytes, s);
        case 2562: return paced_launch<256, 2>(P, n_read, n_write, n_update, elems, lds_bytes, s);
        case 2564: return paced_launch<256, 4>(P, n_read, n_write, n_update, elems, lds_bytes, s);
        default: return AID_EINVAL;
    }
}

extern "C" int bench_aid_cache_scrub(void* buf, uint64_t bytes, void* hip_stream) {
    const uint64_t half = bytes / 2;
    if (buf == nullptr || bytes == 0 || half % (PROBE_TILE * sizeof(float)) != 0 ||
        (reinterpret_cast<uintptr_t>(buf) & 15u) != 0 || half / (PROBE_TILE * sizeof(float)) > 0x7fffffffull)
        return AID_EINVAL;
    const unsigned tiles = static_cast<unsigned>(half / (PROBE_TILE * sizeof(float)));
    hipLaunchKernelGGL(bench_aid_scrub_kernel, dim3(tiles), dim3(PROBE_BLOCK), 0, static_cast<hipStream_t>(hip_stream),
                       reinterpret_cast<const pf4*>(buf),
                       reinterpret_cast<pf4*>(static_cast<char*>(buf) + half));
    return hipGetLastError() == hipSuccess ? 0 : AID_EHIP;
}

extern "C" int bench_aid_stream_probe(const float* const* read_ptrs, int32_t n_read, float* const* write_ptrs,
                                   int32_t n_write, float* const* update_ptrs, int32_t n_update, uint64_t elems,
                                   void* hip_stream) {
    if (n_read < 0 || n_write < 0 || n_update < 0 || n_read + n_write + n_update == 0) return AID_EINVAL;
    if (n_read > PROBE_MAX || n_write > PROBE_MAX || n_update > PROBE_MAX) return AID_EINVAL;
    if ((n_read && !read_ptrs) || (n_write && !write_ptrs) || (n_update && !update_ptrs)) return AID_EINVAL;
    if (elems == 0 || elems % PROBE_TILE != 0 || elems / PROBE_TILE > 0x7fffffffull) return AID_EINVAL;
    ProbePtrs P = {};
    for (int i = 0; i < n_read; ++i) if ((P.r[i] = read_ptrs[i]) == nullptr) return AID_EINVAL;
    for (int i = 0; i < n_write; ++i) if ((P.w[i] = write_ptrs[i]) == nullptr) return AID_EINVAL;
    for (int i = 0; i < n_update; ++i) if ((P.x[i] = update_ptrs[i]) == nullptr) return AID_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const uint64_t tiles = elems / PROBE_TILE;
    switch (n_read) {
        case 0: return probe_by_w<0>(n_write, n_update, P, tiles, s);
        case 1: return probe_by_w<1>(n_write, n_update, P, tiles, s);
        case 2: return probe_by_w<2>(n_write, n_update, P, tiles, s);
        case 4: return probe_by_w<4>(n_write, n_update, P, tiles, s);
        case 8: return probe_by_w<8>(n_write, n_update, P, tiles, s);
        case 16: return probe_by_w<16>(n_write, n_update, P, tiles, s);
        default: return AID_EINVAL;
    }
}
