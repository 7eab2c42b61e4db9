/*
 * mgwfbp.h -- C ABI of the MI355X (gfx950) merged-gradient hot path of MG-WFBP
 *             (merged-gradient wait-free backpropagation).
 *
 * The library does two things:
 *   1. HOST: decide which layers' gradients travel together (Algorithm 1), evaluate the
 *      wait-free-backpropagation timeline of any such plan (Eq. 6-8 with the merged-layer
 *      properties Eq. 12-14), and derive the merge-buffer layout (Sec. 5.3, Algorithm 2).
 *   2. DEVICE: for one group or for all groups, on one GPU and one HIP stream,
 *        pack           copy many per-layer gradient tensors of P workers into P contiguous
 *                       merge buffers                                            (Sec. 5.3)
 *        reduce         the per-GPU arithmetic of the all-reduce: sum the P merge buffers in
 *                       worker order 0..P-1 and scale by 1/P                      (Eq. 2)
 *        unpack_update  read the averaged gradient back out of the buffer and apply
 *                       v <- mu*v + g ; w <- w - eta*v to the per-layer tensors   (Eq. 2,
 *                       Algorithm 2 line 15; the momentum buffer is an addition of this library)
 *      plus fused forms that produce bit-identical results with less memory traffic.
 *
 * Conventions
 *   - Tensor index i = 0..L-1 is the paper's layer l = i+1 (forward order).  Gradients become
 *     ready in the order L-1, L-2, ..., 0 ("arrival order").
 *   - merged[i] = 1 means layer i+1 is a merged-gradient layer: it sends nothing by itself and
 *     its gradient is communicated together with tensor i-1.  merged[0] is always 0.
 *   - A group is a maximal run hi >= ... >= lo with merged[i] = 1 for lo < i <= hi and
 *     merged[lo] = 0.  Groups are numbered in arrival order: group 0 contains tensor L-1.
 *   - Inside a group's slice of the merge buffer the tensors lie densely in arrival order
 *     (tensor hi at element offset 0); the slice holds exactly the sum of its members' elements.
 *   - All groups live in one "arena" per worker: group k's slice starts at element group_base[k],
 *     which is a multiple of the library's tile size.  Elements between the end of one slice and
 *     the next base are padding that no call reads or writes.
 *   - Times are seconds (double).  Message sizes are bytes.  a and b are the startup time and the
 *     per-byte time of the all-reduce cost model T(M) = a + b*M (Eq. 10).
 *   - "device array" = memory readable by the GPU; "host array" = ordinary host memory.
 *     The caller owns every buffer it passes in; the context owns only its own tables.
 *   - Device entry points enqueue work on `hip_stream` (a hipStream_t passed as void*; NULL is
 *     the default stream) and return without waiting for it.  They allocate nothing.
 *   - Arithmetic is binary32 with one rounding per operation (no fused multiply-add):
 *       r = ((..((g_0 + g_1) + g_2)..) + g_{P-1}) * (1.0f / P)
 *       t1 = mu * v ; v' = t1 + r ; t2 = eta * v' ; w' = w - t2
 *     bfloat16 and binary16 gradients are widened exactly to binary32 before the first addition.
 *   - A context is used by one host thread at a time (its launch settings are plain fields); different
 *     contexts are independent, and the host-only functions are re-entrant.
 *   - Every function returns MGWFBP_OK (0) or a negative mgwfbp_status.  Nothing throws or aborts.
 *     A failed call has enqueued nothing.
 */
#ifndef MGWFBP_H
#define MGWFBP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum mgwfbp_status {
    MGWFBP_OK = 0,
    MGWFBP_EINVAL = -1, /* null pointer, size or index out of range, non-finite or negative time */
    MGWFBP_ENOMEM = -2, /* host or device allocation failed                                       */
    MGWFBP_EHIP = -3,   /* a HIP runtime call failed; see mgwfbp_last_hip_error()                 */
    MGWFBP_ECAPACITY = -4 /* the model needs larger tables than a fixed-size entry point can hold         */
} mgwfbp_status;

typedef enum mgwfbp_dtype {
    MGWFBP_F32 = 0, /* gradients are binary32, 4 bytes per element            */
    MGWFBP_BF16 = 1, /* gradients are bfloat16 bit patterns, 2 bytes per element (Sec. 5.3:
                        BytesPerElement = 2 for half-precision training)        */
    MGWFBP_F16 = 2   /* gradients are IEEE binary16, 2 bytes per element: the half precision of the
                        paper's own mixed-precision runs (Sec. 5.3, Sec. 6.3)   */
} mgwfbp_dtype;

typedef struct mgwfbp_ctx mgwfbp_ctx; /* opaque; host + device copies of the group/offset tables */

/* ---------------------------------------------------------------------------------------------
 * Host: planning
 * ------------------------------------------------------------------------------------------- */

/* Algorithm 1 ("find optimal m").  For l = L..2 layer l becomes a merged-gradient layer iff
 *     tau_b[l-1] + t_b[l-1] - tau_c[l] < a          (evaluated left to right, strict)
 * where tau_b follows Eq. 6 with tau_b[L] = 0 and tau_c follows Eq. 7 under the merges decided so
 * far; a merge moves the layer's bytes to layer l-1 and recomputes that layer's message time
 * a + b*bytes.  The result equals the O(L^2) formulation of the paper bit for bit; this
 * implementation updates tau_c incrementally and runs in O(L).
 *
 *   size_bytes    host [L]  gradient bytes of each tensor (may be 0)
 *   t_backward_s  host [L]  backward time of each tensor, seconds, finite and >= 0
 *   a_s, b_s_per_byte       cost model, finite and >= 0
 *   merged_out    host [L]  out: 0 = normal layer, 1 = merged-gradient layer
 *   group_first_out host [L+1] or NULL  out: group_first[k] = highest tensor index of group k,
 *                           group_first[G] = -1
 *   n_groups_out  host [1] or NULL      out: G
 * L = 0 is accepted (G = 0).  Errors: MGWFBP_EINVAL. */
int mgwfbp_plan(const uint64_t* size_bytes, const double* t_backward_s, int32_t L,
                double a_s, double b_s_per_byte,
                uint8_t* merged_out, int32_t* group_first_out, int32_t* n_groups_out);

/* The exact minimiser of the paper's objective (Eq. 8 minimised over all plans with layer 1 normal),
 * which Algorithm 1 approximates: Theorem 1's optimality claim fails on some inputs, e.g. bytes
 * (0,0,100), t_b (49.1,0.9,0), a = b = 1 gives 102.9 with Algorithm 1 and 102.0 here.  Dynamic
 * programme over the arrival order, O(L^2) time: the earliest end of the first k arrivals' messages is
 * min over cuts i of max(end[i], ready[k]) + a + b*bytes(i+1..k).  Ties keep the longest last group.
 * Arguments as mgwfbp_plan; *t_iter_out (may be NULL) receives the optimum, which equals
 * mgwfbp_eval of the returned plan bit for bit. */
int mgwfbp_plan_opt(const uint64_t* size_bytes, const double* t_backward_s, int32_t L,
                    double a_s, double b_s_per_byte,
                    uint8_t* merged_out, int32_t* group_first_out, int32_t* n_groups_out,
                    double* t_iter_out);

/* Iteration time minus forward time, t_iter - t_f, of an arbitrary plan: Eq. 8 evaluated on the
 * timeline of Eq. 6-7 after applying Eq. 12 (no message for a merged layer), Eq. 13 (bytes move
 * down) and Eq. 14 (start of the lower layer).  merged[0] must be 0.  Result in *t_iter_out. */
int mgwfbp_eval(const uint8_t* merged, const uint64_t* size_bytes, const double* t_backward_s,
                int32_t L, double a_s, double b_s_per_byte, double* t_iter_out);

/* When each group's merge buffer is full, measured from the start of the backward pass: a buffer is full
 * (Sec. 5.3; Algorithm 2's handler sends it) once the gradient of the group's lowest layer exists, which is
 * at tau_b + t_b of that layer with tau_b from Eq. 6 and tau_b of the last layer = 0 as in Algorithm 1.
 *   merged, t_backward_s  host [L]   as for mgwfbp_eval
 *   ready_out             host [G] or NULL   out: seconds, group 0 (the first to fill) first; non-decreasing
 *   n_groups_out          host [1] or NULL   out: G
 * Errors: MGWFBP_EINVAL. */
int mgwfbp_group_ready_times(const uint8_t* merged, const double* t_backward_s, int32_t L,
                             double* ready_out, int32_t* n_groups_out);

/* ---------------------------------------------------------------------------------------------
 * Host: where a and b come from, and the worker-count sweep
 * ------------------------------------------------------------------------------------------- */

typedef enum mgwfbp_allreduce_algorithm {   /* rows of Table 2 */
    MGWFBP_AR_BINARY_TREE = 0,              /* a = 2 alpha log N      b = (2 beta + gamma) log N                 */
    MGWFBP_AR_RECURSIVE_DOUBLING = 1,       /* a = alpha log N        b = (beta + gamma) log N                   */
    MGWFBP_AR_HALVING_DOUBLING = 2,         /* a = 2 alpha log N      b = 2 beta - (2 beta + gamma)/N + gamma    */
    MGWFBP_AR_DOUBLE_BINARY_TREES = 3,      /* a = 2 alpha log N      b = beta + gamma   (the table prints the
                                               startup without alpha; read as for the other rows)               */
    MGWFBP_AR_RING = 4                      /* a = 2 (N-1) alpha      b = 2 (N-1)/N beta + (N-1)/N gamma         */
} mgwfbp_allreduce_algorithm;

/* Table 2: all-reduce startup a and per-byte cost b from the point-to-point latency alpha (s), the
 * per-byte transfer time beta (s/B), the per-byte summation time gamma (s/B) and the worker count N >= 1.
 * log is base 2.  Errors: MGWFBP_EINVAL (unknown algorithm, N < 1, negative or non-finite input). */
int mgwfbp_allreduce_ab(int32_t algorithm, int32_t n_workers, double alpha_s, double beta_s_per_byte,
                        double gamma_s_per_byte, double* a_out, double* b_out);

/* Sec. 6.2 (Fig. 4): a and b as the least-squares line through n >= 2 measured (message bytes, seconds)
 * points with at least two different sizes. */
int mgwfbp_fit_ab(const uint64_t* message_bytes, const double* seconds, int32_t n,
                  double* a_out, double* b_out);

/* Sec. 6.4: for every worker count, take (a, b) from Table 2 and report the iteration time
 * (t_forward_s + Eq. 8) of wait-free backpropagation (every layer normal), of single-layer
 * communication (everything merged, Eq. 9) and of MG-WFBP (Algorithm 1), plus the number of messages
 * MG-WFBP sends.  Any out array (host, [n_counts]) may be NULL.  The speedup over one worker is
 * N * (t_forward_s + sum t_backward_s) / t_iter. */
int mgwfbp_simulate(const uint64_t* size_bytes, const double* t_backward_s, int32_t L, double t_forward_s,
                    int32_t algorithm, double alpha_s, double beta_s_per_byte, double gamma_s_per_byte,
                    const int32_t* worker_counts, int32_t n_counts,
                    double* t_wfbp_out, double* t_single_out, double* t_mgwfbp_out, int32_t* groups_out);

/* ---------------------------------------------------------------------------------------------
 * Host: context = group/offset table for one (tensor sizes, plan, P, dtype), uploaded once
 * ------------------------------------------------------------------------------------------- */

/* Builds the layout described under "Conventions" and copies the tables that drive the kernels to
 * the current HIP device (synchronous; this is the only allocating call besides destroy).
 *   n_elems host [L]  element count of each tensor (0 allowed: such a tensor is skipped)
 *   merged  host [L]  plan, e.g. from mgwfbp_plan
 *   P       number of workers whose gradients are held on this GPU, 1..64
 *   grad_dtype        mgwfbp_dtype of the gradient tensors and merge buffers
 * Errors: MGWFBP_EINVAL, MGWFBP_ENOMEM, MGWFBP_EHIP. */
int mgwfbp_ctx_create(mgwfbp_ctx** ctx_out, const uint64_t* n_elems, int32_t L,
                      const uint8_t* merged, int32_t P, int32_t grad_dtype);

/* Same tables, host copies only: needs no GPU and touches none.  Such a context answers the
 * inspection calls below; every device entry point rejects it with MGWFBP_EINVAL. */
int mgwfbp_ctx_create_host(mgwfbp_ctx** ctx_out, const uint64_t* n_elems, int32_t L,
                           const uint8_t* merged, int32_t P, int32_t grad_dtype);

void mgwfbp_ctx_destroy(mgwfbp_ctx* ctx); /* frees the tables; NULL is ignored */

/* Sizes a caller needs before allocating: any out pointer may be NULL.
 *   arena_elems  elements each merge buffer (and the reduced buffer) must hold
 *   tile_elems   granule of the arena that one workgroup processes; group bases are multiples */
int mgwfbp_ctx_dims(const mgwfbp_ctx* ctx, int32_t* L, int32_t* n_groups, int32_t* P,
                    int32_t* grad_dtype, uint64_t* arena_elems, int32_t* tile_elems,
                    int32_t* n_tiles);

/* The layout, for inspection and tests.  Any out pointer may be NULL.
 *   tensor_off   host [L]  element offset of tensor i inside its group's slice (Sec. 5.3: dense,
 *                          arrival order)
 *   tensor_group host [L]  group number of tensor i
 *   group_base   host [G]  first arena element of group k
 *   group_elems  host [G]  elements in group k (sum of its members) */
int mgwfbp_ctx_layout(const mgwfbp_ctx* ctx, uint64_t* tensor_off, int32_t* tensor_group,
                      uint64_t* group_base, uint64_t* group_elems);

/* The tables the kernels walk, for tests of the host logic.  Any out pointer may be NULL.
 * A "segment" is one non-empty tensor's stretch of the arena; segments are numbered in arena order.
 *   n_segments     host [1]    S
 *   tiles_out      host [n_tiles] records of 32 bytes: int64 first_start (arena start of the tile's
 *                  first segment minus the tile's own start, <= 0), int32 first_end (tile-local end
 *                  of that segment), int32 seg0 (its number), int32 nseg (segments intersecting the
 *                  tile), int32 valid (leading elements of the tile inside the group), int32 layer0
 *                  (tensor index of seg0), int32 flags (bit 0: w and v of the tile use ordinary, cacheable accesses)
 *   seg_off_out    host [S+1]  arena element where each segment starts; [S] = arena_elems
 *   seg_n_out      host [S]    elements of each segment, saturated at 2^32-1
 *   seg_layer_out  host [S]    tensor index of each segment
 *   group_tile_out host [G+1]  first tile of each group; [G] = n_tiles */
int mgwfbp_ctx_tables(const mgwfbp_ctx* ctx, int32_t* n_segments, void* tiles_out,
                      uint64_t* seg_off_out, uint32_t* seg_n_out, int32_t* seg_layer_out,
                      int32_t* group_tile_out);

/* Launch shape.  A tile is 256 consecutive arena elements.  By default a call launches one workgroup of 64 lanes
 * (one wavefront) per tile it covers (per 4 KiB of each worker's data for mgwfbp_pack, which runs as P
 * single-worker copies).
 *   blocks_per_cu > 0        caps the grid at compute units * blocks_per_cu workgroups, which then stride
 *                            over the work; <= 0 restores the default
 *   xcd_contiguous != 0      renumbers workgroups so that each of the 8 accelerator dies walks one
 *                            contiguous eighth of the range instead of every eighth piece
 *   tiles_per_workgroup > 0  consecutive tiles a workgroup handles, one after the other; <= 0 restores the
 *                            default
 * Results never depend on the launch shape. */
int mgwfbp_ctx_set_launch(mgwfbp_ctx* ctx, int32_t blocks_per_cu, int32_t xcd_contiguous,
                          int32_t tiles_per_workgroup);

/* Pacing.  The kernels walk a tile one worker at a time with one 16-byte load per lane in flight, so that a
 * workgroup has 1 KiB of loads under way (half that for 16-bit gradients), and a launch asks for enough (unused)
 * LDS that at most `workgroups_per_cu` workgroups share a compute unit.  Their product is the load traffic a
 * compute unit keeps in flight; MI355X serves the mixes of this library fastest at about 16 KiB and about a
 * tenth slower beyond 20 KiB.
 *   workgroups_per_cu  2..31 = cap; 0 = the library's default for the kind of kernel; < 0 or >= 32 = no cap
 *                      (a compute unit holds 32 wavefronts).  LDS is granted in blocks, so the caps that exist
 *                      are 25, 21, 18, 16, 14, 12, 11, 10, 9, 8, ...; a value in between acts as the next lower one.
 *   vectors_per_step   1 (the only paced step of a one-vector tile); 0 = the library's default; -1 = the burst
 *                      form (below) for every launch
 * Results never depend on it. */
int mgwfbp_ctx_set_pacing(mgwfbp_ctx* ctx, int32_t workgroups_per_cu, int32_t vectors_per_step);

/* Small launches.  A launch that covers too few tiles to fill the chip (one small group, as Algorithm 2's
 * handler sends them) is bound by the latency of a tile, not by the memory system, and pacing only stretches
 * that latency: such a launch takes the burst form, in which a lane issues every load of its tile at once and
 * no cap on the workgroups per compute unit applies.  `max_tiles` is the largest launch (in tiles of 256
 * elements) that does so: 0 = none, < 0 = the library's default (1024 tiles = 256 Ki elements).  Ignored while vectors_per_step of
 * mgwfbp_ctx_set_pacing is not 0.  Results never depend on it. */
int mgwfbp_ctx_set_small_launch(mgwfbp_ctx* ctx, int32_t max_tiles);

/* How many bytes of weights + momenta (8 per element, counted from the start of the arena) are accessed
 * with ordinary loads and stores so that they stay in the GPU's 256 MB memory-side cache from one
 * iteration to the next; the rest of w and v is streamed with non-temporal accesses like the gradients.
 * Results do not depend on it.  Default 0 (everything is streamed: in a training loop a forward and a backward
 * pass run between two updates, so nothing would survive in that cache anyway); a caller whose next reader of
 * the weights comes soon may set up to about 232 MiB.  Synchronous: the tile table is rewritten with a blocking
 * copy, so the call is allowed only while no kernel launched with this context is still in flight (synchronise
 * the streams it was used on first). */
int mgwfbp_ctx_set_resident_bytes(mgwfbp_ctx* ctx, uint64_t bytes);

/* ---------------------------------------------------------------------------------------------
 * Device: the pipeline.  `group` is a group number 0..G-1, or -1 for every group in one launch.
 *
 * Pointer tables are DEVICE arrays of device pointers:
 *   d_grad_ptrs  [P*L]  d_grad_ptrs[w*L + i] -> gradient tensor i of worker w, n_elems[i] elements
 *                       of the context's dtype, element-aligned (16-byte alignment is faster)
 *   d_merge_bufs [P]    d_merge_bufs[w] -> worker w's merge arena, arena_elems elements of the
 *                       context's dtype, 16-byte aligned
 *   d_w_ptrs, d_v_ptrs [L]  -> binary32 weight / momentum tensor i, n_elems[i] elements, 4-byte aligned
 *   d_reduced           binary32 arena of arena_elems elements, 16-byte aligned
 * Entries of zero-element tensors are never dereferenced.  Buffers of different roles must not
 * overlap.  Calls on the same stream execute in order; calls for different groups touch disjoint
 * elements and may run on different streams.
 * Errors: MGWFBP_EINVAL (null argument, group out of range), MGWFBP_EHIP (launch failed).
 * ------------------------------------------------------------------------------------------- */

/* Sec. 5.3: copy the member gradients of `group`, for all P workers, into the merge arenas. */
int mgwfbp_pack(mgwfbp_ctx* ctx, int32_t group, const void* const* d_grad_ptrs,
                void* const* d_merge_bufs, void* hip_stream);

/* Algorithm 2, communication handler (`lb.push(l)`): as gradients arrive, copy the tensors
 * first_tensor, first_tensor-1, ..., last_tensor (a run in arrival order, first_tensor >= last_tensor;
 * it may cross group boundaries) of all P workers into their places in the merge arenas.  Covering every
 * tensor of a group with such calls, in any order and any split into runs, leaves the group's slices
 * exactly as mgwfbp_pack(group) does; the group's buffer is "full" (Sec. 5.3) once its lowest tensor,
 * the one with merged[i] = 0, has been packed.  Errors: MGWFBP_EINVAL for an empty or out-of-range run. */
int mgwfbp_pack_tensors(mgwfbp_ctx* ctx, int32_t first_tensor, int32_t last_tensor,
                        const void* const* d_grad_ptrs, void* const* d_merge_bufs, void* hip_stream);

/* Eq. 2, aggregation part: d_reduced[j] = (sum over w in order of merge[w][j]) * (1/P) for every
 * element j of the group's slice. */
int mgwfbp_reduce(mgwfbp_ctx* ctx, int32_t group, const void* const* d_merge_bufs,
                  float* d_reduced, void* hip_stream);

/* Eq. 2, update part (Algorithm 2 line 15) with momentum: for every member tensor i and element e,
 * g = d_reduced[group_base + tensor_off[i] + e]; v_i[e] <- mu*v_i[e] + g; w_i[e] <- w_i[e] - lr*v_i[e]. */
int mgwfbp_unpack_update(mgwfbp_ctx* ctx, int32_t group, const float* d_reduced,
                         float* const* d_w_ptrs, float* const* d_v_ptrs,
                         float lr, float momentum, void* hip_stream);

/* reduce + unpack_update in one pass: reads the P merge slices, writes only w and v.
 * Same bits as mgwfbp_reduce followed by mgwfbp_unpack_update. */
int mgwfbp_reduce_update(mgwfbp_ctx* ctx, int32_t group, const void* const* d_merge_bufs,
                         float* const* d_w_ptrs, float* const* d_v_ptrs,
                         float lr, float momentum, void* hip_stream);

/* pack + reduce + unpack_update in one pass: reads the per-layer gradients once, fills the merge
 * arenas (the buffers an all-reduce would transmit), optionally writes the averaged gradient to
 * d_reduced (NULL to skip), and updates w and v.  Same bits in every output as the three separate
 * calls. */
int mgwfbp_group_pipeline(mgwfbp_ctx* ctx, int32_t group, const void* const* d_grad_ptrs,
                          void* const* d_merge_bufs, float* d_reduced,
                          float* const* d_w_ptrs, float* const* d_v_ptrs,
                          float lr, float momentum, void* hip_stream);

/* reduce + update straight from the per-layer gradients, for the case in which all P workers'
 * gradients are on this device and nothing has to be transmitted: the merge buffers of Sec. 5.3 are
 * never written (they exist to give the all-reduce one contiguous message).  Walks the same group /
 * offset table, so `group` means what it means everywhere else; optionally writes the averaged
 * gradient to d_reduced (NULL to skip).  Same bits in w, v and d_reduced as mgwfbp_group_pipeline
 * (Eq. 2 with the sum taken in worker order). */
int mgwfbp_direct_update(mgwfbp_ctx* ctx, int32_t group, const void* const* d_grad_ptrs, float* d_reduced,
                         float* const* d_w_ptrs, float* const* d_v_ptrs,
                         float lr, float momentum, void* hip_stream);

/* mgwfbp_group_pipeline for the consecutive groups group_first .. group_first + group_count - 1 in one
 * launch (e.g. all groups whose buffers filled since the last call).  group_count = 0 is a no-op. */
int mgwfbp_group_pipeline_span(mgwfbp_ctx* ctx, int32_t group_first, int32_t group_count,
                               const void* const* d_grad_ptrs, void* const* d_merge_bufs, float* d_reduced,
                               float* const* d_w_ptrs, float* const* d_v_ptrs,
                               float lr, float momentum, void* hip_stream);

/* mgwfbp_group_pipeline for callers that must not allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  The context may come from mgwfbp_ctx_create_host (no device
 * allocation at all): instead of the context's own device tables the kernels read the group/offset/tile
 * tables from a fixed array of MGWFBP_STATIC_TABLE_MAX_BYTES that is part of the loaded library on every GPU
 * (held until the process ends).  The call copies the context's tables there in stream order (skipped when the
 * same unchanged context was the last one used on this device and on this stream) and launches the same
 * kernel with the same arguments otherwise; it calls no allocating routine.  Same results as
 * mgwfbp_group_pipeline.
 *   - Runs on the CURRENT device, whichever device the context was created on.
 *   - Every call on one GPU shares that GPU's array: calls whose work may overlap in time (different streams
 *     without ordering, different host threads) race unless they pass the same unchanged context.
 *   - The context must stay alive and unchanged until the work has finished.
 *   - A caller that captures the call into a HIP graph makes one ordinary call with the same context on the
 *     same stream first: the table copy reads ordinary host memory and does not belong in a graph; the
 *     captured calls then find the tables in place and only launch the kernel.
 * Errors: MGWFBP_ECAPACITY if the model's tables (32 bytes per tile of 256 elements + 16 bytes per non-empty
 * tensor, each table rounded up to 256 bytes) exceed the array -- about 400 M elements; MGWFBP_EINVAL;
 * MGWFBP_EHIP. */
#define MGWFBP_STATIC_TABLE_MAX_BYTES (48u << 20)
int mgwfbp_group_pipeline_static(mgwfbp_ctx* ctx, int32_t group, const void* const* d_grad_ptrs,
                                 void* const* d_merge_bufs, float* d_reduced,
                                 float* const* d_w_ptrs, float* const* d_v_ptrs,
                                 float lr, float momentum, void* hip_stream);

/* Algorithm 2's communication handler, driven by a recorded schedule instead of a live backward pass.
 * Group k's buffer counts as full at host time t0 + time_scale * group_ready_s[k], t0 being the moment of the
 * call.  The handler waits (spinning on the host's monotonic clock) until the next unlaunched group is full,
 * issues ONE fused pack + reduce + update launch (as mgwfbp_group_pipeline_span) covering every group that is
 * full by then, on the next of `streams` in round-robin order, and repeats until all groups are launched; then
 * it waits for all the streams.  Groups that fill while the handler is busy launching are therefore batched
 * into the next launch.  Unless max_groups_per_launch is 1 the handler also keeps at most two launches queued
 * per stream: while a stream's earlier launches are still running it goes on collecting groups, so a schedule
 * faster than the GPU degenerates into few, long launches instead of a long queue of small ones.
 * Unlike the other device entry points this call BLOCKS until the work is done (and creates and destroys a
 * few HIP events).
 *   group_ready_s  host [G]   e.g. from mgwfbp_group_ready_times; finite, >= 0, non-decreasing
 *   time_scale     >= 0; 1 replays the schedule in real time, 0 makes every group full at once
 *   max_groups_per_launch  0 = no limit; 1 = strictly one launch per group (groups that are already full
 *                  are then launched back to back), n = at most n groups per launch
 *   streams        host [n_streams] of hipStream_t, 1 <= n_streams <= 16, all of default priority; launches for
 *                  different groups touch disjoint elements, so they need no ordering among themselves
 *   stats_out      host [4] or NULL  out: [0] launches issued, [1] seconds from t0 at which the last group was
 *                  full, [2] seconds from t0 at which every stream had drained, [3] = [2] - [1], the part of
 *                  the pipeline left exposed after the last gradient
 * Errors: MGWFBP_EINVAL, MGWFBP_EHIP. */
int mgwfbp_handler_replay(mgwfbp_ctx* ctx, const double* group_ready_s, double time_scale,
                          int32_t max_groups_per_launch, void* const* streams, int32_t n_streams,
                          const void* const* d_grad_ptrs, void* const* d_merge_bufs, float* d_reduced,
                          float* const* d_w_ptrs, float* const* d_v_ptrs, float lr, float momentum,
                          double* stats_out);

/* ---------------------------------------------------------------------------------------------
 * Diagnostics
 * ------------------------------------------------------------------------------------------- */
int mgwfbp_last_hip_error(void);      /* hipError_t of the last failed HIP call on this thread, 0 if none */
const char* mgwfbp_version(void);     /* static string */

#ifdef __cplusplus
}
#endif
#endif /* MGWFBP_H */
