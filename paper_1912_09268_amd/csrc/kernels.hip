// Device side of the MG-WFBP library for gfx950 (MI355X): context management and the streaming
// kernels pack / reduce / unpack_update and their fused forms.
//
// All six operations are the same walk over the merge arena, tile by tile (by default one workgroup
// of 64 lanes = one wavefront per tile of 256 elements, dispatched in tile order):
//
//   kind            reads                          writes
//   PACK            per-layer gradients (P)        merge arenas (P)                     Sec. 5.3
//   REDUCE          merge arenas (P)               reduced arena                        Eq. 2 (sum, 1/P)
//   UPDATE          reduced arena, w, v            w, v                                 Eq. 2 (update)
//   REDUCE_UPDATE   merge arenas (P), w, v         w, v
//   PIPELINE        per-layer gradients (P), w, v  merge arenas (P), [reduced], w, v
//   DIRECT          per-layer gradients (P), w, v  [reduced], w, v
//
// The arena side of every access is 16-byte aligned (tiles start on multiples of the tile size and
// lanes step in 4-element vectors).  The per-layer side starts wherever the tensor starts, so it is
// accessed through vector types that only promise element alignment; gfx950 executes those as the
// same 16-byte (8-byte for 16-bit gradients) memory instructions.
//
// A tile that lies entirely inside one tensor takes the fast path: tensor index and source offset
// come from the tile header, the pointer table is read once with wave-uniform addresses, and the tile is
// walked in paced steps, one worker at a time (see paced_step).  Any other tile takes the general path:
// the tile-local start offsets of the segments it intersects are produced by a workgroup-wide prefix sum
// (wavefront scans via cross-lane shifts, combined through LDS) over the segment lengths, staged in LDS,
// and each lane finds the owner of its vector by binary search there.  Vectors that straddle two tensors,
// the end of the group or the edge of the interval a call is clipped to are taken element by element,
// one element per lane, after the whole vectors.
//
// This is bandwidth-bound streaming work (at most 4 flops per 12+ bytes), so there is no use for the
// matrix cores; the job is to present the traffic to the memory system in the form it serves fastest:
//   - SMALL LAUNCHES (too few tiles to fill the chip: one small group) are bound by the latency of a tile,
//     so they issue every load of a tile at once (the burst form, STEPV = 0); what follows is for the rest;
//   - PACING.  For these read/write mixes MI355X delivers most when every compute unit keeps about
//     16-24 KiB of loads in flight and a tenth less beyond that, so a lane has one 16-byte load outstanding
//     (one worker's share of the tile; two workers' in the kinds that only read between their stores) and each
//     launch asks for enough unused LDS that only about 16 workgroups share a compute unit (see run() and
//     lds_for_workgroups_per_cu());
//   - SMALL WORKGROUPS.  A workgroup is one wavefront and a tile the 256 elements it covers with one vector per
//     lane: the same bytes in flight spread over sixteen independent wavefronts per compute unit, each at its
//     own point of its walk, load the memory system more evenly than two workgroups of four wavefronts that
//     move in step (3-5 % of the peak on every shape);
//   - one workgroup per tile, dispatched in tile order, so that the bytes the chip has in flight form one
//     contiguous moving window per array;
//   - everything is streamed with non-temporal loads and stores; a caller may ask for a leading share of
//     the weights and momenta to use ordinary accesses and stay in the 256 MB memory-side cache (tile flag);
//   - PACK, which has no arithmetic across workers, runs as P single-worker copies (gridDim.y = P),
//     so the chip streams 2 arrays at a time instead of 2P; a workgroup copies 4 KiB of its worker's data,
//     two tiles per step (more per workgroup stretches the window its compute unit covers and costs 8 %).
//
// Arithmetic contract: binary32, one rounding per operation.  The file must be compiled with
// -ffp-contract=off so that mu*v + g and w - lr*v are never fused.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>

#include "mgwfbp.h"
#include "tables.h"

#ifndef MGWFBP_NT
#define MGWFBP_NT 3   // bit 0: non-temporal loads of gradients / merge / reduced, bit 1: non-temporal
                      // stores to merge / reduced, bit 2: non-temporal accesses to w and v
#endif
#ifndef MGWFBP_PACK_TILES
#define MGWFBP_PACK_TILES 2       // consecutive full tiles of one tensor that PACK copies in one step
#endif
#define MGWFBP_MAXSEG (2 * MGWFBP_BLOCK)   // segments per tile whose offsets are staged in LDS (two per lane)

// Table space of mgwfbp_group_pipeline_static: one copy per GPU, held until the process ends.  Host code must
// not pass this name to a kernel or a copy (on the host it is only a stand-in for the symbol); the device
// address comes from hipGetSymbolAddress, once per device.  (No `used` attribute here: the compiler exports a
// file-local device variable under a global symbol only when it sees host code refer to it, as
// mgwfbp_group_pipeline_static does; marked `used` it stays a local symbol that the runtime cannot look up.)
static __device__ __align__(256) unsigned char scratch[MGWFBP_STATIC_TABLE_MAX_BYTES];

namespace {

constexpr int BLOCK = MGWFBP_BLOCK;
constexpr int VEC = MGWFBP_VEC;
constexpr int TVECS = MGWFBP_TILE_VECS;
constexpr int TILE = MGWFBP_TILE_ELEMS;
constexpr int MAXSEG = MGWFBP_MAXSEG;
constexpr int PACK_TILES = MGWFBP_PACK_TILES;

enum Kind { K_PACK = 0, K_REDUCE = 1, K_UPDATE = 2, K_REDUCE_UPDATE = 3, K_PIPELINE = 4, K_DIRECT = 5 };

constexpr bool reads_grads(int k) { return k == K_PACK || k == K_PIPELINE || k == K_DIRECT; }
constexpr bool reads_merge(int k) { return k == K_REDUCE || k == K_REDUCE_UPDATE; }
constexpr bool writes_merge(int k) { return k == K_PACK || k == K_PIPELINE; }
constexpr bool sums(int k) { return k == K_REDUCE || k == K_REDUCE_UPDATE || k == K_PIPELINE || k == K_DIRECT; }
constexpr bool writes_reduced(int k) { return k == K_REDUCE || k == K_PIPELINE || k == K_DIRECT; }
constexpr bool updates(int k) { return k == K_UPDATE || k == K_REDUCE_UPDATE || k == K_PIPELINE || k == K_DIRECT; }
constexpr bool needs_owner(int k) { return k != K_REDUCE; }

// ---------------------------------------------------------------------------------------------
// vector types that promise only element alignment
// ---------------------------------------------------------------------------------------------
typedef float f32x4 __attribute__((ext_vector_type(4), aligned(4)));
typedef uint16_t u16x4 __attribute__((ext_vector_type(4), aligned(2)));   // bfloat16 bit patterns
typedef _Float16 f16x4 __attribute__((ext_vector_type(4), aligned(2)));   // IEEE binary16

template <typename T, int W> struct VecOf;
template <> struct VecOf<float, 4> { typedef f32x4 type; };
template <> struct VecOf<float, 1> { typedef float type; };
template <> struct VecOf<uint16_t, 4> { typedef u16x4 type; };
template <> struct VecOf<uint16_t, 1> { typedef uint16_t type; };
template <> struct VecOf<_Float16, 4> { typedef f16x4 type; };
template <> struct VecOf<_Float16, 1> { typedef _Float16 type; };

template <typename V> struct Lanes { static constexpr int n = 4; };
template <> struct Lanes<float> { static constexpr int n = 1; };
template <> struct Lanes<uint16_t> { static constexpr int n = 1; };
template <> struct Lanes<_Float16> { static constexpr int n = 1; };

__device__ __forceinline__ float comp(const f32x4& v, int c) { return v[c]; }
__device__ __forceinline__ float comp(const float& v, int) { return v; }
__device__ __forceinline__ uint16_t comp(const u16x4& v, int c) { return v[c]; }
__device__ __forceinline__ uint16_t comp(const uint16_t& v, int) { return v; }
__device__ __forceinline__ _Float16 comp(const f16x4& v, int c) { return v[c]; }
__device__ __forceinline__ _Float16 comp(const _Float16& v, int) { return v; }
__device__ __forceinline__ void setc(f32x4& v, int c, float x) { v[c] = x; }
__device__ __forceinline__ void setc(float& v, int, float x) { v = x; }

// Address spaces of the AMDGPU target: 1 = global memory, 4 = constant (read-only for the whole
// kernel; wave-uniform addresses are fetched through the scalar unit).  Pointers that were themselves
// read from memory carry no address space, so data accesses name it explicitly; otherwise they would
// become slower generic ("flat") instructions.
#define MGWFBP_GLOBAL __attribute__((address_space(1)))
#define MGWFBP_CONST __attribute__((address_space(4)))

template <typename T> __device__ __forceinline__ const MGWFBP_CONST T* ro(const T* p) {
    return (const MGWFBP_CONST T*)p;
}

template <bool NT, typename V> __device__ __forceinline__ V ld(const void* p) {
    const MGWFBP_GLOBAL V* q = (const MGWFBP_GLOBAL V*)p;
    if constexpr (NT) return __builtin_nontemporal_load(q);
    else return *q;
}
template <bool NT, typename V> __device__ __forceinline__ void st(void* p, const V& x) {
    MGWFBP_GLOBAL V* q = (MGWFBP_GLOBAL V*)p;
    if constexpr (NT) __builtin_nontemporal_store(x, q);
    else *q = x;
}

constexpr bool NT_LD = (MGWFBP_NT & 1) != 0;
constexpr bool NT_ST = (MGWFBP_NT & 2) != 0;
constexpr bool NT_WV = (MGWFBP_NT & 4) != 0;

__device__ __forceinline__ float widen(float x) { return x; }
__device__ __forceinline__ float widen(uint16_t bits) { return __uint_as_float(static_cast<uint32_t>(bits) << 16); }
__device__ __forceinline__ float widen(_Float16 x) { return static_cast<float>(x); }   // every binary16 value is a binary32 value

// ---------------------------------------------------------------------------------------------
// kernel arguments
// ---------------------------------------------------------------------------------------------
template <typename GradT> struct Args {
    const TileHdr* tiles;
    const uint32_t* seg_n;
    const int32_t* seg_layer;
    const uint64_t* seg_off;
    const GradT* const* grad_ptrs;   // [P*L]
    GradT* const* merge_bufs;        // [P]
    float* reduced;                  // arena or null
    float* const* w_ptrs;            // [L]
    float* const* v_ptrs;            // [L]
    float lr, mu, inv_p;
    int32_t L, P;
    int32_t tile_first, tile_count;
    int32_t xcd_contiguous;
    int32_t tiles_per_wg;            // consecutive tiles one workgroup handles per turn, >= 1
    int32_t n_units;                 // ceil(tile_count / tiles_per_wg)
    int32_t worker_split;            // 1: gridDim.y = P and every workgroup serves worker blockIdx.y alone
    int32_t clipped;                 // 0: whole tiles; 1: only arena elements in [clip_lo, clip_hi)
    int64_t clip_lo, clip_hi;
};

// First worker a workgroup serves.  PACK has no arithmetic across workers, so it is launched as P
// single-worker copies side by side in gridDim.y: workgroups are dispatched x-fastest, the chip then
// streams one worker's gradients at a time (2 streams instead of 2P), which the memory system serves
// faster.
template <typename GradT> __device__ __forceinline__ int worker_base(const Args<GradT>& A) {
    return A.worker_split ? static_cast<int>(blockIdx.y) : 0;
}

// Pointers of the P workers, either held in registers (P known at compile time) or re-read from the
// table on every use (any P).
template <typename T, int PT> struct WorkerPtrs {
    T* p[PT];
    __device__ __forceinline__ void fetch(T* const* table, int64_t stride, int64_t index, int w0) {
#pragma unroll
        for (int w = 0; w < PT; ++w) p[w] = ro(table)[(w0 + w) * stride + index];
    }
    __device__ __forceinline__ T* get(int w) const { return p[w]; }
};
template <typename T> struct WorkerPtrs<T, 0> {
    T* const* base;
    int64_t stride;
    __device__ __forceinline__ void fetch(T* const* table, int64_t s, int64_t index, int w0) {
        base = table + w0 * s + index;
        stride = s;
    }
    __device__ __forceinline__ T* get(int w) const { return ro(base)[w * stride]; }
};

// ---------------------------------------------------------------------------------------------
// one paced step: N vectors (W = 4) or one element (W = 1) per lane, at arena position `apos`, which is
// element `soff` of its tensor; the N vectors lie `stride` elements apart
// ---------------------------------------------------------------------------------------------
//
// The step is taken worker by worker: load one worker's values, store them into that worker's merge arena
// (kinds that fill the arenas), add them to the running sums -- acc = g_0, then acc = acc + g_w, the worker
// order 0..P-1 of Eq. 2 -- and go on to the next worker; then the reduced arena, then v, then w.  A lane never
// has more than N loads in flight (kinds without stores between the workers take MGWFBP_READ_GROUP workers at a
// time), and that is the point: the memory system serves this traffic fastest when each compute unit keeps
// only 16-24 KiB of loads in flight (the exact figure differs a little from one machine to the next) and about
// a tenth slower beyond.  N x 16 bytes per lane of the workgroup times the workgroups a compute unit is allowed
// to hold (see run()) sets that budget.
#ifndef MGWFBP_READ_GROUP
#define MGWFBP_READ_GROUP 2
#endif
#ifndef MGWFBP_GENERAL_GROUP
#define MGWFBP_GENERAL_GROUP 64   // workers whose loads the general path issues together (64: all of them)
#endif

// keeps the compiler from moving the next group's loads above this group's arithmetic
__device__ __forceinline__ void pace() { __builtin_amdgcn_sched_barrier(0); }

template <int KIND, typename GradT, int PT, int W, int N, bool WVNT, bool TOGETHER = false>
__device__ __forceinline__ void paced_step(const Args<GradT>& A, const WorkerPtrs<const GradT, PT>& src,
                                           const WorkerPtrs<GradT, PT>& mrg, float* wp, float* vp,
                                           int64_t soff, int64_t apos, int stride) {
    typedef typename VecOf<GradT, W>::type GV;
    typedef typename VecOf<float, W>::type FV;
    constexpr int C = Lanes<GV>::n;
    FV acc[N];
    // the general path wants everything under way at once: its v and w loads go out before the gradients'
    constexpr int NE = (updates(KIND) && TOGETHER) ? N : 1;
    FV v_early[NE], w_early[NE];
    if constexpr (updates(KIND) && TOGETHER) {
#pragma unroll
        for (int i = 0; i < N; ++i) v_early[i] = ld<WVNT, FV>(vp + soff + i * stride);
#pragma unroll
        for (int i = 0; i < N; ++i) w_early[i] = ld<WVNT, FV>(wp + soff + i * stride);
    }
    if constexpr (reads_grads(KIND) || reads_merge(KIND)) {
        // workers whose loads are issued together: one (kinds that store each worker's share before the next
        // load), MGWFBP_READ_GROUP (kinds that only read them), or all of them / four at a time (TOGETHER: the
        // general path, whose lanes also have to fetch their own pointers and gain from overlapping all of that)
        constexpr int GW = TOGETHER ? (PT > 0 ? (PT < MGWFBP_GENERAL_GROUP ? PT : MGWFBP_GENERAL_GROUP) : 4) : (writes_merge(KIND) ? 1 : MGWFBP_READ_GROUP);
        auto some_workers = [&](int w0, int count) {      // workers w0 .. w0 + count - 1, count <= GW
            GV g[GW][N];
#pragma unroll
            for (int j = 0; j < GW; ++j) {
                if (j < count) {
                    const GradT* from;
                    if constexpr (reads_grads(KIND)) from = src.get(w0 + j) + soff;
                    else from = mrg.get(w0 + j) + apos;
#pragma unroll
                    for (int i = 0; i < N; ++i) g[j][i] = ld<NT_LD, GV>(from + i * stride);
                }
            }
            // kinds that store and add each worker's share: every load of the step is issued before the first
            // value is used (left alone, the scheduler now and then puts an add, and with it a wait for the
            // first load, in front of the second load)
            if constexpr (writes_merge(KIND) && sums(KIND)) pace();
#pragma unroll
            for (int j = 0; j < GW; ++j) {
                if (j < count) {
                    if constexpr (writes_merge(KIND)) {
                        GradT* to = mrg.get(w0 + j) + apos;
#pragma unroll
                        for (int i = 0; i < N; ++i) st<NT_ST, GV>(to + i * stride, g[j][i]);
                    }
                    if constexpr (sums(KIND)) {
#pragma unroll
                        for (int i = 0; i < N; ++i)
#pragma unroll
                            for (int c = 0; c < C; ++c) {
                                const float x = widen(comp(g[j][i], c));
                                setc(acc[i], c, (w0 + j == 0) ? x : comp(acc[i], c) + x);
                            }
                    }
                }
            }
        };
        if constexpr (PT > 0) {
#pragma unroll
            for (int w0 = 0; w0 < PT; w0 += GW) {
                some_workers(w0, PT - w0 < GW ? PT - w0 : GW);
                pace();
            }
        } else {
            for (int w0 = 0; w0 < A.P; w0 += GW) {
                some_workers(w0, A.P - w0 < GW ? A.P - w0 : GW);
                pace();
            }
        }
        if constexpr (sums(KIND)) {
#pragma unroll
            for (int i = 0; i < N; ++i)
#pragma unroll
                for (int c = 0; c < C; ++c) setc(acc[i], c, comp(acc[i], c) * A.inv_p);
        }
    }
    if constexpr (KIND == K_UPDATE) {
#pragma unroll
        for (int i = 0; i < N; ++i) acc[i] = ld<NT_LD, FV>(A.reduced + apos + i * stride);
    }
    if constexpr (writes_reduced(KIND)) {
        if (KIND == K_REDUCE || A.reduced != nullptr) {
#pragma unroll
            for (int i = 0; i < N; ++i) st<NT_ST, FV>(A.reduced + apos + i * stride, acc[i]);
        }
    }
    if constexpr (updates(KIND) && TOGETHER) {
#pragma unroll
        for (int i = 0; i < N; ++i) {
#pragma unroll
            for (int c = 0; c < C; ++c) {
                const float t1 = A.mu * comp(v_early[i], c);
                setc(v_early[i], c, t1 + comp(acc[i], c));
                const float t2 = A.lr * comp(v_early[i], c);
                setc(w_early[i], c, comp(w_early[i], c) - t2);
            }
            st<WVNT, FV>(vp + soff + i * stride, v_early[i]);
            st<WVNT, FV>(wp + soff + i * stride, w_early[i]);
        }
    } else if constexpr (updates(KIND)) {
        FV v[N];
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] = ld<WVNT, FV>(vp + soff + i * stride);
#pragma unroll
        for (int i = 0; i < N; ++i) {
#pragma unroll
            for (int c = 0; c < C; ++c) {
                const float t1 = A.mu * comp(v[i], c);
                setc(v[i], c, t1 + comp(acc[i], c));
            }
            st<WVNT, FV>(vp + soff + i * stride, v[i]);
        }
        pace();
        FV w[N];
#pragma unroll
        for (int i = 0; i < N; ++i) w[i] = ld<WVNT, FV>(wp + soff + i * stride);
#pragma unroll
        for (int i = 0; i < N; ++i) {
#pragma unroll
            for (int c = 0; c < C; ++c) {
                const float t2 = A.lr * comp(v[i], c);
                setc(w[i], c, comp(w[i], c) - t2);
            }
            st<WVNT, FV>(wp + soff + i * stride, w[i]);
        }
    }
}

// one vector or element of the general path
template <int KIND, typename GradT, int PT, int W>
__device__ __forceinline__ void do_one(const Args<GradT>& A, const WorkerPtrs<GradT, PT>& mrg,
                                       int layer, int64_t soff, int64_t apos) {
    WorkerPtrs<const GradT, PT> src;
    float* wp = nullptr;
    float* vp = nullptr;
    if constexpr (reads_grads(KIND)) src.fetch(A.grad_ptrs, A.L, layer, worker_base(A));
    if constexpr (updates(KIND)) {
        wp = ro(A.w_ptrs)[layer];
        vp = ro(A.v_ptrs)[layer];
    }
    paced_step<KIND, GradT, PT, W, 1, NT_WV, true>(A, src, mrg, wp, vp, soff, apos, 0);
}

// ---------------------------------------------------------------------------------------------
// fast path: `nvec` vectors per lane (one or more whole tiles) that lie inside one tensor, taken STEPV
// vectors at a time; vector u of the chunk covers elements u * BLOCK * VEC + lane * VEC ...
// ---------------------------------------------------------------------------------------------
template <int KIND, typename GradT, int PT, bool WVNT, int STEPV>
__device__ __forceinline__ void fast_chunk(const Args<GradT>& A, const WorkerPtrs<GradT, PT>& mrg,
                                           int layer, int64_t tensor_off, int64_t tile_base, int nvec) {
    static_assert(STEPV == 0 || TVECS % STEPV == 0, "a tile is a whole number of steps");
    WorkerPtrs<const GradT, PT> src;
    float* wp = nullptr;
    float* vp = nullptr;
    if constexpr (reads_grads(KIND)) src.fetch(A.grad_ptrs, A.L, layer, worker_base(A));
    if constexpr (updates(KIND)) {
        wp = ro(A.w_ptrs)[layer];
        vp = ro(A.v_ptrs)[layer];
    }
    constexpr int STEP = BLOCK * VEC;
    const int lane_elem = static_cast<int>(threadIdx.x) * VEC;
    const int64_t soff = tensor_off + lane_elem;    // this lane's first element: in its tensor
    const int64_t apos = tile_base + lane_elem;     //                            in the arena
    if constexpr (STEPV == 0) {
        // burst: every load of the tile under way at once.  The form for a launch too small to fill the chip,
        // where the time is the tile's own latency and not the memory system's throughput.
        for (int u = 0; u < nvec; u += TVECS)
            paced_step<KIND, GradT, PT, VEC, TVECS, WVNT, true>(A, src, mrg, wp, vp,
                                                                soff + static_cast<int64_t>(u) * STEP,
                                                                apos + static_cast<int64_t>(u) * STEP, STEP);
    } else {
        for (int u = 0; u < nvec; u += STEPV) {
            paced_step<KIND, GradT, PT, VEC, STEPV, WVNT>(A, src, mrg, wp, vp, soff + static_cast<int64_t>(u) * STEP,
                                                          apos + static_cast<int64_t>(u) * STEP, STEP);
            pace();
        }
    }
}

// ---------------------------------------------------------------------------------------------
// general path
// ---------------------------------------------------------------------------------------------

// Inclusive prefix sum across the lanes of the workgroup: shift-and-add inside each wavefront,
// wavefront totals combined through LDS.  Every lane of the workgroup must call it.
__device__ __forceinline__ int block_inclusive_scan(int x, int* s_wave) {
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int y = __shfl_up(x, d, 64);
        if (lane >= d) x += y;
    }
    if (lane == 63) s_wave[wave] = x;
    __syncthreads();
    int carry = 0;
#pragma unroll
    for (int q = 0; q < BLOCK / 64; ++q)
        if (q < wave) carry += s_wave[q];
    return x + carry;
}

template <int KIND, typename GradT, int PT>
__device__ void general_tile(const Args<GradT>& A, const WorkerPtrs<GradT, PT>& mrg, const TileHdr& h,
                             int64_t tile_base, int clo, int chi, int* s_loc, int* s_layer, int* s_wave,
                             int* s_ragged, int* s_nragged) {
    // Only tile-local elements [clo, chi) are touched; 0 <= clo < chi <= h.valid.
    //
    // A lane takes the 4-element vectors it owns whole where it can.  A vector that is not wanted whole (it
    // crosses a tensor boundary, the end of the group or a clip edge) is set aside in LDS, and once every whole
    // vector is under way the elements of those vectors are dealt out one per lane: a tile pays for its ragged
    // spots with one more step, not with up to four dependent ones in a row on a single lane while the
    // rest of the workgroup waits.
    const int tid = threadIdx.x;
    const int valid = h.valid;
    const int nseg = h.nseg;
    const int p_first = (clo & ~(VEC - 1)) + tid * VEC;
    const bool staged = needs_owner(KIND) && nseg <= MAXSEG;     // uniform over the workgroup
    __syncthreads();                            // the previous tile's readers are done with LDS
    if (tid == 0) *s_nragged = 0;
    if (staged) {
        // Tile-local start of segment j (1 <= j < nseg) = first_end + sum of the lengths of the
        // segments 1..j-1, all of which lie wholly inside the tile.  Each lane owns entries
        // j = 1 + 2*tid and j = 2 + 2*tid.
        const int j0 = 1 + 2 * tid, j1 = j0 + 1;
        int x0 = 0, x1 = 0;
        if (j0 < nseg) x0 = (j0 == 1) ? h.first_end : static_cast<int>(ro(A.seg_n)[h.seg0 + j0 - 1]);
        if (j1 < nseg) x1 = static_cast<int>(ro(A.seg_n)[h.seg0 + j1 - 1]);
        const int incl = block_inclusive_scan(x0 + x1, s_wave);
        if (j0 < nseg) s_loc[j0] = incl - x1;
        if (j1 < nseg) s_loc[j1] = incl;
        for (int j = tid; j < nseg; j += BLOCK) s_layer[j] = ro(A.seg_layer)[h.seg0 + j];
        if (tid == 0) s_loc[nseg] = valid;
    }
    __syncthreads();
    auto start_of = [&](int j) -> int {         // j >= 1
        return staged ? s_loc[j] : static_cast<int>(static_cast<int64_t>(ro(A.seg_off)[h.seg0 + j]) - tile_base);
    };
    auto end_of = [&](int j) -> int { return (j + 1 < nseg) ? start_of(j + 1) : valid; };
    auto layer_of = [&](int j) -> int { return staged ? s_layer[j] : ro(A.seg_layer)[h.seg0 + j]; };
    auto owner_of = [&](int q) -> int {         // last j with start_of(j) <= q (segment 0 starts <= 0)
        int lo = 0, hi = nseg - 1;
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (start_of(mid) <= q) lo = mid; else hi = mid - 1;
        }
        return lo;
    };
    auto offset_in = [&](int j, int q) -> int64_t {   // element q of the tile is this element of segment j
        return (j == 0) ? (static_cast<int64_t>(q) - h.first_start) : static_cast<int64_t>(q - start_of(j));
    };
    for (int p = p_first; p < chi; p += BLOCK * VEC) {
        bool whole = p >= clo && p + VEC <= chi;
        int j = 0;
        if constexpr (needs_owner(KIND)) {
            j = owner_of(max(p, clo));
            whole = whole && p + VEC <= end_of(j);
        }
        if (whole) {
            if constexpr (needs_owner(KIND)) do_one<KIND, GradT, PT, VEC>(A, mrg, layer_of(j), offset_in(j, p), tile_base + p);
            else do_one<KIND, GradT, PT, VEC>(A, mrg, 0, 0, tile_base + p);
        } else {
            s_ragged[atomicAdd(s_nragged, 1)] = p;      // at most TILE / VEC entries: one per vector of the tile
        }
    }
    __syncthreads();
    const int n_ragged = *s_nragged;
    for (int e = tid; e < n_ragged * VEC; e += BLOCK) {
        const int q = s_ragged[e / VEC] + (e % VEC);
        if (q < clo || q >= chi) continue;
        if constexpr (needs_owner(KIND)) {
            const int j = owner_of(q);
            do_one<KIND, GradT, PT, 1>(A, mrg, layer_of(j), offset_in(j, q), tile_base + q);
        } else {
            do_one<KIND, GradT, PT, 1>(A, mrg, 0, 0, tile_base + q);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// the kernel
// ---------------------------------------------------------------------------------------------
typedef int i32x4 __attribute__((ext_vector_type(4)));

// The 32-byte tile header, fetched as two 16-byte read-only loads (wave-uniform address).
__device__ __forceinline__ TileHdr load_header(const TileHdr* p) {
    const MGWFBP_CONST i32x4* q = (const MGWFBP_CONST i32x4*)p;
    const i32x4 a = q[0], b = q[1];
    TileHdr h;
    h.first_start = static_cast<int64_t>((static_cast<uint64_t>(static_cast<uint32_t>(a[1])) << 32) |
                                         static_cast<uint32_t>(a[0]));
    h.first_end = a[2];
    h.seg0 = a[3];
    h.nseg = b[0];
    h.valid = b[1];
    h.layer0 = b[2];
    h.flags = b[3];
    return h;
}

// STEPV: vectors per lane a fast tile is walked in (1 or 2, see paced_step), or 0 for the burst form.
template <int KIND, typename GradT, int PT, int STEPV>
__global__ void __launch_bounds__(MGWFBP_BLOCK) mgwfbp_stream_kernel(const Args<GradT> A) {
    __shared__ int s_loc[MAXSEG + 1];
    __shared__ int s_layer[MAXSEG];
    __shared__ int s_wave[BLOCK / 64];
    __shared__ int s_ragged[TILE / VEC];
    __shared__ int s_nragged;

    WorkerPtrs<GradT, PT> mrg;
    if constexpr (reads_merge(KIND) || writes_merge(KIND)) mrg.fetch(A.merge_bufs, 1, 0, worker_base(A));

    // Work is dealt in units of `tiles_per_wg` consecutive tiles.
    const int K = A.tiles_per_wg;
    const int n_units = A.n_units;              // ceil(tile_count / K), computed on the host
    int u_begin, u_end, u_step;
    if (A.xcd_contiguous) {
        // workgroup ids are dealt round-robin to the 8 dies: die = id % 8.  Give each die one
        // contiguous eighth of the units.
        const int die = blockIdx.x & 7;
        const int per_die = (n_units + 7) >> 3;
        u_begin = die * per_die + static_cast<int>(blockIdx.x >> 3);
        u_end = min(n_units, (die + 1) * per_die);
        u_step = static_cast<int>(gridDim.x >> 3);
    } else {
        u_begin = blockIdx.x;
        u_end = n_units;
        u_step = gridDim.x;
    }
    for (int u = u_begin; u < u_end; u += u_step) {
        const int t_end = min((u + 1) * K, A.tile_count);
        for (int t = u * K; t < t_end; ++t) {
            const int tile = A.tile_first + t;
            const TileHdr h = load_header(A.tiles + tile);
            const int64_t tile_base = static_cast<int64_t>(tile) * TILE;
            int clo = 0, chi = h.valid;
            if (A.clipped) {                        // uniform over the workgroup
                const int64_t l = A.clip_lo - tile_base, r = A.clip_hi - tile_base;
                if (l > 0) clo = l < h.valid ? static_cast<int>(l) : h.valid;
                if (r < h.valid) chi = r > 0 ? static_cast<int>(r) : 0;
                if (chi <= clo) continue;
            }
            if (!(clo == 0 && chi == TILE && (!needs_owner(KIND) || h.nseg == 1))) {
                general_tile<KIND, GradT, PT>(A, mrg, h, tile_base, clo, chi, s_loc, s_layer, s_wave, s_ragged, &s_nragged);
                continue;
            }
            // A full tile inside one tensor.
            if constexpr (KIND == K_PACK && PACK_TILES > 1) {
                // Pack is a plain copy and wants more bytes in flight per lane than one tile holds: when the next
                // tiles of this workgroup's share are full tiles of the same tensor too, they are copied together.
                if (!A.clipped && t + PACK_TILES <= t_end) {
                    bool same = true;
#pragma unroll
                    for (int k = 1; k < PACK_TILES; ++k) {
                        const TileHdr hk = load_header(A.tiles + tile + k);
                        same = same && hk.valid == TILE && hk.nseg == 1 && hk.layer0 == h.layer0;
                    }
                    if (same) {
                        WorkerPtrs<const GradT, PT> src;
                        src.fetch(A.grad_ptrs, A.L, h.layer0, worker_base(A));
                        const int lane_elem = static_cast<int>(threadIdx.x) * VEC;
                        paced_step<KIND, GradT, PT, VEC, PACK_TILES * TVECS, true>(
                            A, src, mrg, nullptr, nullptr, -h.first_start + lane_elem, tile_base + lane_elem, BLOCK * VEC);
                        t += PACK_TILES - 1;
                        continue;
                    }
                }
            }
            // Tiles flagged "resident" keep their w and v in the memory-side cache between iterations
            // (ordinary loads and stores); all other w, v traffic is streamed past it like the gradients.
            // The two arms differ only in the cache policy of their memory instructions; the empty asm
            // statements keep the optimiser from merging them back into one (which drops the policy).
            const int64_t toff = -h.first_start;
            if (!updates(KIND) || (h.flags & 1)) {
                asm volatile("; w and v cacheable" ::: "memory");
                fast_chunk<KIND, GradT, PT, NT_WV, STEPV>(A, mrg, h.layer0, toff, tile_base, TVECS);
                asm volatile("; end w and v cacheable" ::: "memory");
            } else {
                asm volatile("; w and v streamed" ::: "memory");
                fast_chunk<KIND, GradT, PT, true, STEPV>(A, mrg, h.layer0, toff, tile_base, TVECS);
                asm volatile("; end w and v streamed" ::: "memory");
            }
        }
    }
}

thread_local int g_last_hip_error = 0;

int note(hipError_t e) {
    if (e == hipSuccess) return MGWFBP_OK;
    g_last_hip_error = static_cast<int>(e);
    return MGWFBP_EHIP;
}

}  // namespace

int mgwfbp_note_hip_result(int hip_error_code) { return note(static_cast<hipError_t>(hip_error_code)); }

// ---------------------------------------------------------------------------------------------
// context
// ---------------------------------------------------------------------------------------------
constexpr int32_t DEFAULT_BURST_TILES = 262144 / TILE;   // see run(): launches of at most 256 Ki elements

struct mgwfbp_ctx {
    HostTables host;
    int32_t P = 0;
    int32_t dtype = 0;
    bool on_device = false;
    int device = -1;
    int n_cu = 0;
    int32_t blocks_per_cu = 0;
    int32_t xcd_contiguous = 0;
    int32_t tiles_per_wg = 0;         // 0 = per-kernel default
    int32_t wg_per_cu = 0;            // 0 = per-kernel default, > 0 = cap, < 0 = no cap
    int32_t step_vecs = 0;            // 0 = per-kernel default, 1 or 2 = paced steps, -1 = always the burst form
    int32_t burst_tiles = DEFAULT_BURST_TILES;   // launches of at most this many tiles take the burst form
    uint64_t resident_bytes = 0;      // budget of w + v bytes kept cacheable
    uint64_t serial = 0;              // changes whenever the tables change; never reused within a process
    // device copies
    TileHdr* d_tiles = nullptr;
    uint32_t* d_seg_n = nullptr;
    int32_t* d_seg_layer = nullptr;
    uint64_t* d_seg_off = nullptr;
};

namespace {

// 0 = no cap: one workgroup per tile.  Workgroups are then dispatched in tile order, which keeps the
// chip's accesses to each of the 2P+2 streams inside a narrow moving window; measured faster than a
// persistent grid for every profile.
constexpr int32_t DEFAULT_BLOCKS_PER_CU = 0;

// Default share of the 256 MB memory-side cache given to weights and momenta: none.  In a training loop a
// forward and a backward pass run between two updates, so nothing of one update is still cached at the next.
constexpr uint64_t DEFAULT_RESIDENT_BYTES = 0;

std::atomic<uint64_t> g_next_serial{1};

// Marks the leading tiles whose w + v bytes (8 per element) fit into the budget.
void mark_resident_tiles(HostTables& h, uint64_t budget) {
    uint64_t used = 0;
    for (TileHdr& t : h.tiles) {
        const uint64_t need = static_cast<uint64_t>(t.valid) * 8u;
        if (used + need <= budget) {
            t.flags = 1;
            used += need;
        } else {
            t.flags = 0;
        }
    }
}

template <typename T> int upload(T** dst, const std::vector<T>& src) {
    const size_t bytes = (src.empty() ? 1 : src.size()) * sizeof(T);
    hipError_t e = hipMalloc(reinterpret_cast<void**>(dst), bytes);
    if (e != hipSuccess) {
        *dst = nullptr;
        g_last_hip_error = static_cast<int>(e);
        return e == hipErrorOutOfMemory ? MGWFBP_ENOMEM : MGWFBP_EHIP;
    }
    if (!src.empty()) return note(hipMemcpy(*dst, src.data(), src.size() * sizeof(T), hipMemcpyHostToDevice));
    return MGWFBP_OK;
}

int create_common(mgwfbp_ctx** out, const uint64_t* n_elems, int32_t L, const uint8_t* merged, int32_t P,
                  int32_t dtype, bool device) {
    if (out == nullptr) return MGWFBP_EINVAL;
    *out = nullptr;
    if (P < 1 || P > MGWFBP_MAX_P) return MGWFBP_EINVAL;
    if (dtype != MGWFBP_F32 && dtype != MGWFBP_BF16 && dtype != MGWFBP_F16) return MGWFBP_EINVAL;
    mgwfbp_ctx* c = new (std::nothrow) mgwfbp_ctx();
    if (c == nullptr) return MGWFBP_ENOMEM;
    int rc = mgwfbp_build_tables(n_elems, L, merged, c->host);
    if (rc != MGWFBP_OK) {
        delete c;
        return rc;
    }
    c->P = P;
    c->dtype = dtype;
    c->blocks_per_cu = DEFAULT_BLOCKS_PER_CU;
    c->resident_bytes = DEFAULT_RESIDENT_BYTES;
    c->serial = g_next_serial.fetch_add(1);
    mark_resident_tiles(c->host, c->resident_bytes);
    if (device) {
        hipDeviceProp_t prop;
        rc = note(hipGetDevice(&c->device));
        if (rc == MGWFBP_OK) rc = note(hipGetDeviceProperties(&prop, c->device));
        if (rc == MGWFBP_OK) {
            c->n_cu = prop.multiProcessorCount;
            rc = upload(&c->d_tiles, c->host.tiles);
        }
        if (rc == MGWFBP_OK) rc = upload(&c->d_seg_n, c->host.seg_n);
        if (rc == MGWFBP_OK) rc = upload(&c->d_seg_layer, c->host.seg_layer);
        if (rc == MGWFBP_OK) rc = upload(&c->d_seg_off, c->host.seg_off);
        if (rc != MGWFBP_OK) {
            mgwfbp_ctx_destroy(c);
            return rc;
        }
        c->on_device = true;
    }
    *out = c;
    return MGWFBP_OK;
}

// How a launch is paced (host side only).
struct Pace {
    size_t lds_bytes = 0;     // dynamic LDS per workgroup; unused by the kernel, it only bounds the workgroups per CU
    int step_vecs = 1;        // vectors per lane a fast tile is walked in: 1 or 2; 0 = burst (all at once)
};

template <int KIND, typename GradT, int PT>
int launch_one(const Args<GradT>& A, int grid, hipStream_t stream, const Pace& pc, int grid_y = 1) {
    bool launched = false;
    if (pc.step_vecs <= 0) {
        hipLaunchKernelGGL((mgwfbp_stream_kernel<KIND, GradT, PT, 0>), dim3(grid, grid_y), dim3(BLOCK), pc.lds_bytes,
                           stream, A);
        launched = true;
    }
    if constexpr (TVECS % 2 == 0) {
        if (!launched && pc.step_vecs >= 2) {
            hipLaunchKernelGGL((mgwfbp_stream_kernel<KIND, GradT, PT, 2>), dim3(grid, grid_y), dim3(BLOCK), pc.lds_bytes,
                               stream, A);
            launched = true;
        }
    }
    if (!launched)
        hipLaunchKernelGGL((mgwfbp_stream_kernel<KIND, GradT, PT, 1>), dim3(grid, grid_y), dim3(BLOCK), pc.lds_bytes,
                           stream, A);
    return note(hipGetLastError());
}

template <int KIND, typename GradT>
int launch_by_p(const Args<GradT>& A, int grid, hipStream_t stream, const Pace& pc) {
    if constexpr (KIND == K_UPDATE) {
        return launch_one<KIND, GradT, 0>(A, grid, stream, pc);   // no per-worker data
    } else if constexpr (KIND == K_PACK) {
        Args<GradT> B = A;                                     // P independent single-worker copies
        B.worker_split = 1;
        return launch_one<KIND, GradT, 1>(B, grid, stream, pc, A.P);
    } else {
        switch (A.P) {
            case 2: return launch_one<KIND, GradT, 2>(A, grid, stream, pc);
            case 4: return launch_one<KIND, GradT, 4>(A, grid, stream, pc);
            case 8: return launch_one<KIND, GradT, 8>(A, grid, stream, pc);
            case 16: return launch_one<KIND, GradT, 16>(A, grid, stream, pc);
            default: return launch_one<KIND, GradT, 0>(A, grid, stream, pc);
        }
    }
}

// Dynamic LDS per workgroup that lets at most n workgroups share the 160 KiB of a compute unit.  A workgroup's
// LDS (static + dynamic) is granted in blocks of 1280 bytes (a 128th of the compute unit's; seen in the cap
// sweeps, where 12 and 13, 14 and 15, 16 and 17 behave alike); the total aimed at is the smallest multiple of
// the block above 160 KiB / (n + 1), so n + 1 workgroups never fit, and n do wherever a multiple of the block
// lies in (160 KiB / (n + 1), 160 KiB / n]: 32, 25, 21, 18, 16, 14, 12, 11, 10, 9, 8, ... are the caps that
// exist, and a request in between gets the next lower one.  The request stays 64 bytes short of that total so
// that padding of the static part cannot push it into the next block.  62 KiB keeps clear of the 64 KiB a launch may ask for without special arrangements (so n = 1 is
// served as n = 2).  n <= 0 means no cap, and so does an n beyond what the waves of a compute unit allow anyway.
size_t lds_for_workgroups_per_cu(int32_t n) {
    constexpr int32_t MAX_WGS = 32 * 64 / BLOCK;         // 32 waves per compute unit
    if (n <= 0 || n >= MAX_WGS) return 0;
    if (n < 2) n = 2;
    constexpr size_t CU_LDS = 160u << 10;
    constexpr size_t GRAIN = 1280;
    constexpr size_t STATIC_LDS = sizeof(int) * (2 * MAXSEG + 1 + BLOCK / 64 + TILE / VEC + 1);
    size_t total = (CU_LDS / static_cast<size_t>(n + 1) / GRAIN + 1) * GRAIN;
    total = std::min<size_t>(total, 62u << 10);
    if (total <= STATIC_LDS + 64 + GRAIN) return 0;
    return total - STATIC_LDS - 64;
}

// Defaults measured with a cold memory-side cache on the DNN shapes (profiles/: pacing study).  With one
// 16-byte load per lane in flight a wavefront has 1 KiB of a binary32 array under way (512 bytes of a 16-bit
// one), so a cap of 16 wavefronts gives a compute unit 16 KiB; with 16-bit gradients every wave slot is needed
// to get there, and the update alone (20 bytes per element, nothing per worker) runs best uncapped.
int32_t default_step_vecs(int, int32_t) { return TVECS % 2 == 0 ? 2 : 1; }
int32_t default_workgroups_per_cu(int kind, int32_t dtype) {
    const bool wide = dtype == MGWFBP_F32;
    switch (kind) {
        case K_REDUCE: return 14;
        case K_UPDATE: return -1;
        case K_PACK:
        case K_REDUCE_UPDATE: return wide ? 14 : -1;
        default: return wide ? 16 : -1;                  // pipeline, direct
    }
}

// Where the kernels find the tables: normally the context's own device copies.
struct DevTables {
    const TileHdr* tiles;
    const uint32_t* seg_n;
    const int32_t* seg_layer;
    const uint64_t* seg_off;
};

// Tile range and element clip of one call: either a group (or all groups), or an arena interval.
struct Span {
    int32_t t0 = 0, t1 = 0;
    bool clipped = false;
    int64_t lo = 0, hi = 0;
};

template <int KIND>
int run(mgwfbp_ctx* c, int32_t group, const void* const* grad_ptrs, void* const* merge_bufs, float* reduced,
        float* const* w_ptrs, float* const* v_ptrs, float lr, float mu, void* stream_v,
        const Span* span = nullptr, const DevTables* tabs = nullptr) {
    if (c == nullptr || (tabs == nullptr && !c->on_device)) return MGWFBP_EINVAL;
    if (span == nullptr && (group < -1 || group >= c->host.G)) return MGWFBP_EINVAL;
    if (reads_grads(KIND) && grad_ptrs == nullptr) return MGWFBP_EINVAL;
    if ((reads_merge(KIND) || writes_merge(KIND)) && merge_bufs == nullptr) return MGWFBP_EINVAL;
    if ((KIND == K_REDUCE || KIND == K_UPDATE) && reduced == nullptr) return MGWFBP_EINVAL;
    if (updates(KIND) && (w_ptrs == nullptr || v_ptrs == nullptr)) return MGWFBP_EINVAL;

    int32_t t0, t1;
    if (span != nullptr) {
        t0 = span->t0;
        t1 = span->t1;
    } else if (group < 0) {
        t0 = 0;
        t1 = static_cast<int32_t>(c->host.tiles.size());
    } else {
        t0 = c->host.group_tile[static_cast<size_t>(group)];
        t1 = c->host.group_tile[static_cast<size_t>(group) + 1];
    }
    const int32_t count = t1 - t0;
    if (count <= 0) return MGWFBP_OK;             // nothing to move (empty group or empty model)

    DevTables T{c->d_tiles, c->d_seg_n, c->d_seg_layer, c->d_seg_off};
    if (tabs != nullptr) {
        T = *tabs;                                    // the caller vouches for the current device
    } else {
        int dev = -1;
        int rc = note(hipGetDevice(&dev));
        if (rc != MGWFBP_OK) return rc;
        if (dev != c->device) return MGWFBP_EINVAL;   // tables live on the device the context was made on
    }

    // tiles per workgroup: PACK runs as single-worker copies, whose tiles are small (one array in, one out),
    // so a workgroup takes 4 KiB of its worker's data (two tiles at a time, see the kernel); every other kind
    // takes one tile per workgroup.  More only stretches the set of bytes the chip has in flight: the window
    // the workgroups of a compute unit cover together should stay within a few hundred KiB per array.
    int32_t tpw = c->tiles_per_wg;
    if (tpw <= 0) tpw = (KIND == K_PACK) ? std::max(1, 4096 / (TILE * (c->dtype == MGWFBP_F32 ? 4 : 2))) : 1;
    const int32_t units = (count + tpw - 1) / tpw;
    int grid = units;
    if (c->blocks_per_cu > 0 && c->n_cu > 0 && static_cast<int64_t>(c->n_cu) * c->blocks_per_cu < units)
        grid = c->n_cu * c->blocks_per_cu;
    int32_t xcd = 0;
    if (c->xcd_contiguous && grid >= 64) {
        grid &= ~7;
        xcd = 1;
    }
    // Pacing: how many vectors a lane moves per step and how many workgroups may share a compute unit.
    // Together they set the loads a compute unit has in flight (step_vecs x 4 KiB x workgroups for binary32).
    // A launch too small to fill the chip is bound by the latency of its tiles, not by the memory system: it
    // takes the burst form (every load of a tile at once, no cap) unless the caller has fixed the pacing.
    Pace pc;
    const bool burst = c->step_vecs < 0 || (c->step_vecs == 0 && c->burst_tiles > 0 && count <= c->burst_tiles);
    pc.step_vecs = burst ? 0 : (c->step_vecs > 0 ? c->step_vecs : default_step_vecs(KIND, c->dtype));
    const int32_t wgs = c->wg_per_cu != 0 ? c->wg_per_cu
                                          : (burst ? -1 : default_workgroups_per_cu(KIND, c->dtype));
    pc.lds_bytes = lds_for_workgroups_per_cu(wgs);
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    const float inv_p = 1.0f / static_cast<float>(c->P);
    const int32_t clip_on = (span != nullptr && span->clipped) ? 1 : 0;
    const int64_t clip_lo = span ? span->lo : 0, clip_hi = span ? span->hi : 0;

    if (c->dtype == MGWFBP_F32) {
        Args<float> A{T.tiles, T.seg_n, T.seg_layer, T.seg_off,
                      reinterpret_cast<const float* const*>(grad_ptrs),
                      reinterpret_cast<float* const*>(merge_bufs), reduced, w_ptrs, v_ptrs,
                      lr, mu, inv_p, c->host.L, c->P, t0, count, xcd, tpw, units, 0,
                      clip_on, clip_lo, clip_hi};
        return launch_by_p<KIND, float>(A, grid, stream, pc);
    }
    if (c->dtype == MGWFBP_F16) {
        Args<_Float16> A{T.tiles, T.seg_n, T.seg_layer, T.seg_off,
                         reinterpret_cast<const _Float16* const*>(grad_ptrs),
                         reinterpret_cast<_Float16* const*>(merge_bufs), reduced, w_ptrs, v_ptrs,
                         lr, mu, inv_p, c->host.L, c->P, t0, count, xcd, tpw, units, 0,
                         clip_on, clip_lo, clip_hi};
        return launch_by_p<KIND, _Float16>(A, grid, stream, pc);
    }
    Args<uint16_t> A{T.tiles, T.seg_n, T.seg_layer, T.seg_off,
                     reinterpret_cast<const uint16_t* const*>(grad_ptrs),
                     reinterpret_cast<uint16_t* const*>(merge_bufs), reduced, w_ptrs, v_ptrs,
                     lr, mu, inv_p, c->host.L, c->P, t0, count, xcd, tpw, units, 0,
                     clip_on, clip_lo, clip_hi};
    return launch_by_p<KIND, uint16_t>(A, grid, stream, pc);
}

// Per device: where that GPU's copy of `scratch` lives and whose tables it holds.
struct StaticSlot {
    unsigned char* ptr = nullptr;
    bool loaded = false;
    uint64_t serial = 0;              // context serial of the tables last written there
    hipStream_t stream = nullptr;     // ... and the stream the copy was ordered on
};
constexpr int MAX_STATIC_DEVICES = 64;
StaticSlot g_static[MAX_STATIC_DEVICES];
std::mutex g_static_mutex;

}  // namespace

extern "C" {

int mgwfbp_ctx_create(mgwfbp_ctx** ctx_out, const uint64_t* n_elems, int32_t L, const uint8_t* merged,
                      int32_t P, int32_t grad_dtype) {
    return create_common(ctx_out, n_elems, L, merged, P, grad_dtype, true);
}

int mgwfbp_ctx_create_host(mgwfbp_ctx** ctx_out, const uint64_t* n_elems, int32_t L, const uint8_t* merged,
                           int32_t P, int32_t grad_dtype) {
    return create_common(ctx_out, n_elems, L, merged, P, grad_dtype, false);
}

void mgwfbp_ctx_destroy(mgwfbp_ctx* c) {
    if (c == nullptr) return;
    if (c->d_tiles) (void)hipFree(c->d_tiles);
    if (c->d_seg_n) (void)hipFree(c->d_seg_n);
    if (c->d_seg_layer) (void)hipFree(c->d_seg_layer);
    if (c->d_seg_off) (void)hipFree(c->d_seg_off);
    delete c;
}

int mgwfbp_ctx_dims(const mgwfbp_ctx* c, int32_t* L, int32_t* n_groups, int32_t* P, int32_t* grad_dtype,
                    uint64_t* arena_elems, int32_t* tile_elems, int32_t* n_tiles) {
    if (c == nullptr) return MGWFBP_EINVAL;
    if (L) *L = c->host.L;
    if (n_groups) *n_groups = c->host.G;
    if (P) *P = c->P;
    if (grad_dtype) *grad_dtype = c->dtype;
    if (arena_elems) *arena_elems = c->host.arena_elems;
    if (tile_elems) *tile_elems = TILE;
    if (n_tiles) *n_tiles = static_cast<int32_t>(c->host.tiles.size());
    return MGWFBP_OK;
}

int mgwfbp_ctx_layout(const mgwfbp_ctx* c, uint64_t* tensor_off, int32_t* tensor_group, uint64_t* group_base,
                      uint64_t* group_elems) {
    if (c == nullptr) return MGWFBP_EINVAL;
    const HostTables& h = c->host;
    if (tensor_off && h.L) std::memcpy(tensor_off, h.tensor_off.data(), sizeof(uint64_t) * static_cast<size_t>(h.L));
    if (tensor_group && h.L) std::memcpy(tensor_group, h.tensor_group.data(), sizeof(int32_t) * static_cast<size_t>(h.L));
    if (group_base && h.G) std::memcpy(group_base, h.group_base.data(), sizeof(uint64_t) * static_cast<size_t>(h.G));
    if (group_elems && h.G) std::memcpy(group_elems, h.group_elems.data(), sizeof(uint64_t) * static_cast<size_t>(h.G));
    return MGWFBP_OK;
}

int mgwfbp_ctx_tables(const mgwfbp_ctx* c, int32_t* n_segments, void* tiles_out, uint64_t* seg_off_out,
                      uint32_t* seg_n_out, int32_t* seg_layer_out, int32_t* group_tile_out) {
    if (c == nullptr) return MGWFBP_EINVAL;
    const HostTables& h = c->host;
    const size_t S = h.seg_layer.size();
    if (n_segments) *n_segments = static_cast<int32_t>(S);
    if (tiles_out && !h.tiles.empty()) std::memcpy(tiles_out, h.tiles.data(), sizeof(TileHdr) * h.tiles.size());
    if (seg_off_out) std::memcpy(seg_off_out, h.seg_off.data(), sizeof(uint64_t) * (S + 1));
    if (seg_n_out && S) std::memcpy(seg_n_out, h.seg_n.data(), sizeof(uint32_t) * S);
    if (seg_layer_out && S) std::memcpy(seg_layer_out, h.seg_layer.data(), sizeof(int32_t) * S);
    if (group_tile_out) std::memcpy(group_tile_out, h.group_tile.data(), sizeof(int32_t) * h.group_tile.size());
    return MGWFBP_OK;
}

int mgwfbp_ctx_set_launch(mgwfbp_ctx* c, int32_t blocks_per_cu, int32_t xcd_contiguous, int32_t tiles_per_workgroup) {
    if (c == nullptr || blocks_per_cu > 4096 || tiles_per_workgroup > 1024) return MGWFBP_EINVAL;
    c->tiles_per_wg = tiles_per_workgroup <= 0 ? 0 : tiles_per_workgroup;
    c->blocks_per_cu = blocks_per_cu <= 0 ? DEFAULT_BLOCKS_PER_CU : blocks_per_cu;
    c->xcd_contiguous = xcd_contiguous ? 1 : 0;
    return MGWFBP_OK;
}

int mgwfbp_ctx_set_pacing(mgwfbp_ctx* c, int32_t workgroups_per_cu, int32_t vectors_per_step) {
    if (c == nullptr || workgroups_per_cu > 64 || vectors_per_step < -1 || vectors_per_step > TVECS ||
        (vectors_per_step > 0 && TVECS % vectors_per_step != 0))
        return MGWFBP_EINVAL;
    c->wg_per_cu = workgroups_per_cu;
    c->step_vecs = vectors_per_step;
    return MGWFBP_OK;
}

int mgwfbp_ctx_set_small_launch(mgwfbp_ctx* c, int32_t max_tiles) {
    if (c == nullptr) return MGWFBP_EINVAL;
    c->burst_tiles = max_tiles < 0 ? DEFAULT_BURST_TILES : max_tiles;
    return MGWFBP_OK;
}

int mgwfbp_ctx_set_resident_bytes(mgwfbp_ctx* c, uint64_t bytes) {
    if (c == nullptr) return MGWFBP_EINVAL;
    c->resident_bytes = bytes;
    c->serial = g_next_serial.fetch_add(1);
    mark_resident_tiles(c->host, bytes);
    if (c->on_device && !c->host.tiles.empty())
        return note(hipMemcpy(c->d_tiles, c->host.tiles.data(), c->host.tiles.size() * sizeof(TileHdr),
                              hipMemcpyHostToDevice));
    return MGWFBP_OK;
}

int mgwfbp_pack(mgwfbp_ctx* c, int32_t group, const void* const* d_grad_ptrs, void* const* d_merge_bufs,
                void* hip_stream) {
    return run<K_PACK>(c, group, d_grad_ptrs, d_merge_bufs, nullptr, nullptr, nullptr, 0.f, 0.f, hip_stream);
}

int mgwfbp_pack_tensors(mgwfbp_ctx* c, int32_t first_tensor, int32_t last_tensor, const void* const* d_grad_ptrs,
                        void* const* d_merge_bufs, void* hip_stream) {
    if (c == nullptr || !c->on_device) return MGWFBP_EINVAL;
    const HostTables& h = c->host;
    if (last_tensor < 0 || first_tensor >= h.L || first_tensor < last_tensor) return MGWFBP_EINVAL;
    // Tensors lie in the arena in arrival order, so the run first_tensor, ..., last_tensor occupies one
    // arena interval (group padding inside it belongs to no tile's valid part and is skipped).
    uint64_t lo = UINT64_MAX, hi = 0;
    for (int32_t i = first_tensor; i >= last_tensor; --i) {
        const size_t q = static_cast<size_t>(i);
        if (h.tensor_n[q] == 0) continue;
        const uint64_t start = h.group_base[static_cast<size_t>(h.tensor_group[q])] + h.tensor_off[q];
        if (start < lo) lo = start;
        if (start + h.tensor_n[q] > hi) hi = start + h.tensor_n[q];
    }
    if (hi <= lo) return MGWFBP_OK;                               // only empty tensors
    Span s;
    s.t0 = static_cast<int32_t>(lo / TILE);
    s.t1 = static_cast<int32_t>((hi + TILE - 1) / TILE);
    s.clipped = true;
    s.lo = static_cast<int64_t>(lo);
    s.hi = static_cast<int64_t>(hi);
    return run<K_PACK>(c, 0, d_grad_ptrs, d_merge_bufs, nullptr, nullptr, nullptr, 0.f, 0.f, hip_stream, &s);
}

int mgwfbp_reduce(mgwfbp_ctx* c, int32_t group, const void* const* d_merge_bufs, float* d_reduced,
                  void* hip_stream) {
    return run<K_REDUCE>(c, group, nullptr, const_cast<void* const*>(d_merge_bufs), d_reduced, nullptr, nullptr,
                         0.f, 0.f, hip_stream);
}

int mgwfbp_unpack_update(mgwfbp_ctx* c, int32_t group, const float* d_reduced, float* const* d_w_ptrs,
                         float* const* d_v_ptrs, float lr, float momentum, void* hip_stream) {
    return run<K_UPDATE>(c, group, nullptr, nullptr, const_cast<float*>(d_reduced), d_w_ptrs, d_v_ptrs, lr,
                         momentum, hip_stream);
}

int mgwfbp_reduce_update(mgwfbp_ctx* c, int32_t group, const void* const* d_merge_bufs, float* const* d_w_ptrs,
                         float* const* d_v_ptrs, float lr, float momentum, void* hip_stream) {
    return run<K_REDUCE_UPDATE>(c, group, nullptr, const_cast<void* const*>(d_merge_bufs), nullptr, d_w_ptrs,
                                d_v_ptrs, lr, momentum, hip_stream);
}

int mgwfbp_group_pipeline(mgwfbp_ctx* c, int32_t group, const void* const* d_grad_ptrs, void* const* d_merge_bufs,
                          float* d_reduced, float* const* d_w_ptrs, float* const* d_v_ptrs, float lr,
                          float momentum, void* hip_stream) {
    return run<K_PIPELINE>(c, group, d_grad_ptrs, d_merge_bufs, d_reduced, d_w_ptrs, d_v_ptrs, lr, momentum,
                           hip_stream);
}

int mgwfbp_group_pipeline_span(mgwfbp_ctx* c, int32_t group_first, int32_t group_count,
                               const void* const* d_grad_ptrs, void* const* d_merge_bufs, float* d_reduced,
                               float* const* d_w_ptrs, float* const* d_v_ptrs, float lr, float momentum,
                               void* hip_stream) {
    if (c == nullptr || !c->on_device) return MGWFBP_EINVAL;
    if (group_first < 0 || group_count < 0 || group_first > c->host.G - group_count) return MGWFBP_EINVAL;
    Span s;                                   // consecutive groups own consecutive tiles
    s.t0 = c->host.group_tile[static_cast<size_t>(group_first)];
    s.t1 = c->host.group_tile[static_cast<size_t>(group_first + group_count)];
    return run<K_PIPELINE>(c, 0, d_grad_ptrs, d_merge_bufs, d_reduced, d_w_ptrs, d_v_ptrs, lr, momentum,
                           hip_stream, &s);
}

int mgwfbp_group_pipeline_static(mgwfbp_ctx* c, int32_t group, const void* const* d_grad_ptrs,
                                 void* const* d_merge_bufs, float* d_reduced, float* const* d_w_ptrs,
                                 float* const* d_v_ptrs, float lr, float momentum, void* hip_stream) {
    if (c == nullptr) return MGWFBP_EINVAL;
    const HostTables& h = c->host;
    if (group < -1 || group >= h.G) return MGWFBP_EINVAL;
    auto round256 = [](size_t x) { return (x + 255) & ~static_cast<size_t>(255); };
    const size_t b_tiles = h.tiles.size() * sizeof(TileHdr), b_n = h.seg_n.size() * sizeof(uint32_t);
    const size_t b_layer = h.seg_layer.size() * sizeof(int32_t), b_off = h.seg_off.size() * sizeof(uint64_t);
    const size_t o_n = round256(b_tiles), o_layer = o_n + round256(b_n), o_off = o_layer + round256(b_layer);
    if (o_off + round256(b_off) > MGWFBP_STATIC_TABLE_MAX_BYTES) return MGWFBP_ECAPACITY;
    if (h.tiles.empty()) return MGWFBP_OK;

    int dev = -1;
    int rc = note(hipGetDevice(&dev));
    if (rc != MGWFBP_OK) return rc;
    if (dev < 0 || dev >= MAX_STATIC_DEVICES) return MGWFBP_EINVAL;
    std::lock_guard<std::mutex> lock(g_static_mutex);
    StaticSlot& slot = g_static[dev];
    if (slot.ptr == nullptr) {                    // first call on this device: where does its copy live?
        void* p = nullptr;
        rc = note(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (rc != MGWFBP_OK) return rc;
        if (p == nullptr) return MGWFBP_EHIP;
        slot.ptr = static_cast<unsigned char*>(p);
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (!(slot.loaded && slot.serial == c->serial && slot.stream == stream)) {
        // The array still holds the previous call's tables: overwrite them, in stream order, with this model's.
        slot.loaded = false;
        const struct { size_t off, bytes; const void* src; } parts[4] = {
            {0, b_tiles, h.tiles.data()}, {o_n, b_n, h.seg_n.data()},
            {o_layer, b_layer, h.seg_layer.data()}, {o_off, b_off, h.seg_off.data()}};
        for (const auto& part : parts) {
            if (part.bytes == 0) continue;
            rc = note(hipMemcpyAsync(slot.ptr + part.off, part.src, part.bytes, hipMemcpyHostToDevice, stream));
            if (rc != MGWFBP_OK) return rc;
        }
        slot.loaded = true;
        slot.serial = c->serial;
        slot.stream = stream;
    }
    const DevTables T{reinterpret_cast<const TileHdr*>(slot.ptr), reinterpret_cast<const uint32_t*>(slot.ptr + o_n),
                      reinterpret_cast<const int32_t*>(slot.ptr + o_layer),
                      reinterpret_cast<const uint64_t*>(slot.ptr + o_off)};
    return run<K_PIPELINE>(c, group, d_grad_ptrs, d_merge_bufs, d_reduced, d_w_ptrs, d_v_ptrs, lr, momentum,
                           hip_stream, nullptr, &T);
}

int mgwfbp_handler_replay(mgwfbp_ctx* c, const double* group_ready_s, double time_scale,
                          int32_t max_groups_per_launch, void* const* streams, int32_t n_streams, const void* const* d_grad_ptrs, void* const* d_merge_bufs,
                          float* d_reduced, float* const* d_w_ptrs, float* const* d_v_ptrs, float lr, float momentum,
                          double* stats_out) {
    if (c == nullptr || !c->on_device || streams == nullptr || n_streams < 1 || n_streams > 16) return MGWFBP_EINVAL;
    if (!std::isfinite(time_scale) || time_scale < 0.0 || max_groups_per_launch < 0) return MGWFBP_EINVAL;
    const int32_t G = c->host.G;
    if (G > 0 && group_ready_s == nullptr) return MGWFBP_EINVAL;
    for (int32_t k = 0; k < G; ++k) {
        if (!std::isfinite(group_ready_s[k]) || group_ready_s[k] < 0.0) return MGWFBP_EINVAL;
        if (k > 0 && group_ready_s[k] < group_ready_s[k - 1]) return MGWFBP_EINVAL;
    }
    // Back-pressure for the batching forms: at most two launches queued per stream.  While a stream's earlier
    // launches are still running the GPU has work anyway, so the handler keeps collecting groups instead of
    // queueing ever more small launches behind them.  (One event per queue slot; created and destroyed here.)
    constexpr int DEPTH = 2;
    const bool throttle = max_groups_per_launch != 1;
    hipEvent_t slot_done[16 * DEPTH] = {};
    int rc = MGWFBP_OK;
    if (throttle) {
        for (int32_t j = 0; j < n_streams * DEPTH && rc == MGWFBP_OK; ++j)
            rc = note(hipEventCreateWithFlags(&slot_done[j], hipEventDisableTiming));
    }
    typedef std::chrono::steady_clock Clock;
    const Clock::time_point t0 = Clock::now();
    auto since_t0 = [&]() { return std::chrono::duration<double>(Clock::now() - t0).count(); };
    int32_t next = 0, launches = 0;
    while (next < G && rc == MGWFBP_OK) {
        const double due = time_scale * group_ready_s[next];
        double now = since_t0();
        while (now < due) now = since_t0();       // the backward pass has not produced this group yet
        const int32_t j = launches % n_streams;
        const int32_t slot = j * DEPTH + (launches / n_streams) % DEPTH;
        if (throttle && launches >= n_streams * DEPTH) {
            hipError_t q;
            while ((q = hipEventQuery(slot_done[slot])) == hipErrorNotReady) {
            }
            if (q != hipSuccess) {
                rc = note(q);
                break;
            }
            now = since_t0();
        }
        int32_t upto = next + 1;                  // everything that filled meanwhile goes into the same launch
        while (upto < G && time_scale * group_ready_s[upto] <= now &&
               (max_groups_per_launch == 0 || upto - next < max_groups_per_launch)) ++upto;
        Span s;
        s.t0 = c->host.group_tile[static_cast<size_t>(next)];
        s.t1 = c->host.group_tile[static_cast<size_t>(upto)];
        rc = run<K_PIPELINE>(c, 0, d_grad_ptrs, d_merge_bufs, d_reduced, d_w_ptrs, d_v_ptrs, lr, momentum,
                             streams[j], &s);
        if (rc == MGWFBP_OK && throttle) rc = note(hipEventRecord(slot_done[slot], static_cast<hipStream_t>(streams[j])));
        ++launches;
        next = upto;
    }
    // Drain every stream, also after a failed launch.  The handler thread has nothing else to do, so it polls
    // (a blocking wait sleeps, and waking up costs tens of microseconds per stream) and then confirms.
    for (int32_t j = 0; j < n_streams; ++j) {
        hipStream_t sj = static_cast<hipStream_t>(streams[j]);
        while (hipStreamQuery(sj) == hipErrorNotReady) {
        }
        const int rj = note(hipStreamSynchronize(sj));
        if (rc == MGWFBP_OK) rc = rj;
    }
    const double done = since_t0();
    for (hipEvent_t e : slot_done)
        if (e != nullptr) (void)hipEventDestroy(e);
    if (stats_out != nullptr) {
        const double last = G > 0 ? time_scale * group_ready_s[G - 1] : 0.0;
        stats_out[0] = static_cast<double>(launches);
        stats_out[1] = last;
        stats_out[2] = done;
        stats_out[3] = done - last;
    }
    return rc;
}

int mgwfbp_direct_update(mgwfbp_ctx* c, int32_t group, const void* const* d_grad_ptrs, float* d_reduced,
                         float* const* d_w_ptrs, float* const* d_v_ptrs, float lr, float momentum,
                         void* hip_stream) {
    return run<K_DIRECT>(c, group, d_grad_ptrs, nullptr, d_reduced, d_w_ptrs, d_v_ptrs, lr, momentum, hip_stream);
}

int mgwfbp_last_hip_error(void) { return g_last_hip_error; }

const char* mgwfbp_version(void) { return "mgwfbp-gfx950 0.1"; }

}  // extern "C"
