/*
 * libpxchg -- the per-GPU arithmetic of a data-parallel parameter exchange,
 * hand-written for AMD MI355X (gfx950).
 *
 * The operations are the ones the Theano-MPI report (arXiv 1605.08325) places
 * on each GPU during an exchange:
 *   - Section 3.2, "Alltoall-sum-Allgather": every rank receives the k ranks'
 *     copies of its slice and sums them on the GPU; in the half-precision
 *     variant the data travels as 16-bit floats and is summed at full precision;
 *   - Section 4: what is exchanged (weights, momentum, raw gradients), summing
 *     updates before descent versus averaging weights after it, momentum SGD as
 *     the optimiser, and elastic averaging (EASGD, moving rate alpha) for the
 *     asynchronous mode.
 *
 * Conventions
 *   - Plain C ABI.  Every function returns a PXCHG_* status (0 = success) unless
 *     stated otherwise; nothing throws or aborts, and only the set-up calls that
 *     say so (the two destroy calls, pxchg_table_set_multipliers) synchronise the
 *     device.  The exchange calls allocate nothing, copy nothing from the host and
 *     record no memset, so a sequence of them can be captured into a HIP graph.
 *   - "host" / "device" says where a pointer must live.  Data buffers are device
 *     memory owned by the caller; the library owns only tables and buffer sets.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Work is enqueued on it and the call returns without waiting.
 *   - A parameter set is a list of tensors (one device array per layer weight or
 *     bias, as in Section 3.1).  A `pxchg_table` fixes the element count of each
 *     tensor; a `pxchg_bufset` is one device pointer per tensor, all of one
 *     element type (a worker's gradients, its packed copy, the parameters, ...).
 *     Both are created once; steady-state calls do no per-tensor host work, no
 *     allocation and no host-to-device copies, and each call is ONE kernel
 *     launch however many tensors the set has.
 *   - Pointers must be aligned to their element size.  16-byte alignment is the
 *     fast path; other alignments are handled by a slower element-wise path.
 *   - Inputs must not overlap outputs except where a function says "in place".
 *   - All calls for one table must be made with the table's device current.
 *   - No call throws: every failure is a status (see pxchg_status), also when memory runs out.
 */
#ifndef PXCHG_H
#define PXCHG_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PXCHG_MAX_K 64 /* most workers one call can combine */

enum pxchg_status {
    PXCHG_OK = 0,
    PXCHG_ERR_INVALID_ARG = 1,    /* null pointer, bad enum, negative count, misaligned pointer */
    PXCHG_ERR_SHAPE_MISMATCH = 2, /* buffer set belongs to another table, or wrong element type */
    PXCHG_ERR_UNSUPPORTED = 3,    /* k outside 1..PXCHG_MAX_K, size beyond a stated limit */
    PXCHG_ERR_NO_DEVICE = 4,      /* no usable GPU, or the table's device is not current */
    PXCHG_ERR_RUNTIME = 5,        /* a HIP call failed (allocation, copy, launch), or host memory ran out in a set-up
                                     call: then nothing was created and nothing is left allocated */
    PXCHG_ERR_OUT_OF_RANGE = 6,   /* a tensor does not fit inside the device allocation it points into */
    PXCHG_ERR_IN_USE = 7          /* pxchg_table_destroy on a table that still has views or buffer sets */
};

enum pxchg_dtype { PXCHG_F32 = 0, PXCHG_F16 = 1 }; /* IEEE binary32 / binary16 */
enum pxchg_mode { PXCHG_AVG = 0, PXCHG_SUM = 1 };  /* divide the sum by k, or not */

/* Launch-shape controls (see pxchg_set_option). */
enum pxchg_option {
    PXCHG_OPT_CHUNK_ELEMS = 0,   /* elements per work chunk for tables created afterwards;
                                    multiple of 512, 512..1048576; default 512 */
    PXCHG_OPT_BLOCKS_PER_CU = 1, /* 0 (default): one workgroup per chunk (two for some kernels, each taking half
                                    of it); n>0: n persistent workgroups per compute unit, each looping over chunks */
    PXCHG_OPT_CHECK_RANGES = 2,  /* 1 (default): pxchg_bufset_create verifies that each tensor lies
                                    inside one device allocation */
    PXCHG_OPT_NONTEMPORAL = 3,   /* -1 (default): each kernel's own measured-best policy; 0: plain loads and
                                    stores everywhere.  A tuning build of the library (compiled with
                                    -DPXCHG_ALL_POLICIES, see PXCHG_OPT_ALL_POLICIES_BUILT) also takes 1..3:
                                    bit 0 puts the non-temporal hint on vector loads, bit 1 on vector stores;
                                    4: non-temporal loads, and stores that are streaming with agent scope;
                                    5: non-temporal loads, and agent-scope stores without the streaming hint;
                                    the regular build answers PXCHG_ERR_UNSUPPORTED to those.
                                    Results never depend on it.  One operand is exempt: a binary16 gradient
                                    of pxchg_sgd_momentum is always read with plain loads (it is usually the
                                    mean just written by pxchg_reduce_avg and may still be cached) */
    PXCHG_OPT_CENTER_RESIDENT = 4, /* 0 (default): the elastic calls stream both operands; 1: they read the
                                    center with plain loads and write it with agent-scope stores, so that
                                    a center that fits the memory-side cache (256 MB) stays there from one
                                    meeting to the next, as on a server that does nothing but meet workers
                                    (a meeting is then 7 % faster, a fused round of 8 workers 8 %); tables whose
                                    center is larger than that cache stream as with 0.  What is left
                                    dirty in that cache is written back during whatever runs next.
                                    Results never depend on it */
    PXCHG_OPT_ALL_POLICIES_BUILT = 5 /* read-only: 1 if this library was compiled with every cache policy for
                                    every kernel, 0 if only with each kernel's own and the plain one */
};

typedef struct pxchg_table pxchg_table;
typedef struct pxchg_bufset pxchg_bufset;

/* Text for a status code; never NULL; static storage. */
const char *pxchg_status_string(int status);

/* Library version as major*10000 + minor*100 + patch. */
int pxchg_version(void);

/* Set / read a launch-shape control.  Process-wide; each option is one atomic
 * word, so a call running in another thread sees the old or the new value.
 * pxchg_set_option returns PXCHG_ERR_INVALID_ARG for an unknown option or a
 * value outside the stated range; pxchg_get_option returns -1 for an unknown
 * option. */
int pxchg_set_option(int option, int64_t value);
int64_t pxchg_get_option(int option);

/*
 * Host-only planning helper (no GPU needed): splits tensors of `counts[t]`
 * elements into chunks of at most `chunk_elems` elements that never straddle
 * two tensors; empty tensors produce no chunk.  Writes up to `cap` chunks into
 * the three host arrays (any of which may be NULL when cap == 0) and the total
 * number of chunks into *n_chunks.  This is the work list the kernels walk.
 */
int pxchg_plan_chunks(int n_tensors, const int64_t *counts /*host*/, int64_t chunk_elems,
                      int64_t cap, int32_t *chunk_tensor /*host*/, int64_t *chunk_start /*host*/,
                      int32_t *chunk_len /*host*/, int64_t *n_chunks /*host*/);

/*
 * Host-only planning helper (no GPU needed) for a layer-wise exchange (Section 3.2 notes that the exchange could
 * overlap with the rest of the step; back-propagation hands gradients over last layer first): cuts the tensor
 * list into groups of consecutive tensors, each with at least `min_elems` elements in all, so that small layers
 * share a launch; the last group formed holds what is left and may be smaller.  With `reverse` != 0 the groups
 * are formed and listed from the last tensor backwards.  Writes up to `cap` groups into the two host arrays
 * (first tensor and number of tensors of each group, as pxchg_table_view takes them; either may be NULL when
 * cap == 0) and the total number of groups into *n_groups.
 */
int pxchg_plan_groups(int n_tensors, const int64_t *counts /*host*/, int64_t min_elems, int reverse, int cap,
                      int32_t *group_first /*host*/, int32_t *group_n /*host*/, int *n_groups /*host*/);

/*
 * Tensor table: element counts of the parameter set's tensors (Section 3.1: the
 * model's parameters are arrays in GPU memory, one per weight or bias).
 * `counts` is a host array of n_tensors non-negative counts (zero allowed).
 * The table is bound to the device current at creation; the library keeps a
 * device copy of the chunk list.  Destroying a table or a buffer set waits for
 * the device to go idle first (launches may still be reading their device-side
 * lists) and frees device memory; neither is allowed while any stream of the
 * process is being captured into a graph (the capture would be invalidated), so
 * destroy objects before a capture starts or after it has ended.
 *
 * Lifetime.  The library keeps a list of its live handles and never reads through
 * a pointer that is not on it: a handle that was destroyed (also twice), a handle
 * of the other kind and a pointer to anything else are PXCHG_ERR_INVALID_ARG in
 * every call, never a crash.  A table cannot be destroyed while views of it or
 * buffer sets on it exist: pxchg_table_destroy then changes nothing and returns
 * PXCHG_ERR_IN_USE; destroy those first.  A buffer set belongs to the one table it
 * was created on, not to whatever table later occupies the same address.  Calls on
 * handles may run concurrently from several threads; create and destroy calls wait
 * for calls in flight on other threads and exclude each other.
 */
int pxchg_table_create(int n_tensors, const int64_t *counts /*host*/, pxchg_table **out);
int pxchg_table_destroy(pxchg_table *table);
/*
 * A view of `n_tensors` consecutive tensors of `parent`, starting at `first_tensor`: a table handle that
 * every call accepts in place of the parent, together with the PARENT's buffer sets (a view has none of its
 * own), and that makes the call work on those tensors only.  It is how one layer, or a group of layers, is
 * exchanged on its own stream as soon as its gradients exist (Section 3.2 notes that the exchange could overlap
 * with the rest of the step) without a second set of tables and buffer sets.  A view owns no device memory
 * (it points into the parent's chunk list), is created and destroyed without synchronising, uses the parent's
 * multipliers, and must be destroyed before the parent (which refuses to go first: PXCHG_ERR_IN_USE).  Views of
 * views, buffer sets on a view and multipliers on a view are PXCHG_ERR_INVALID_ARG.
 */
int pxchg_table_view(const pxchg_table *parent, int first_tensor, int n_tensors, pxchg_table **out);
/*
 * Optional per-tensor multipliers for the update calls (the usual way to give biases another learning rate or
 * no weight decay; the paper names weight decay and the learning-rate policy among the hyper-parameters,
 * Section 4).  Host arrays of n_tensors floats, or NULL for "all ones"; both NULL removes the multipliers.
 * pxchg_sgd_momentum and pxchg_reduce_avg_sgd_momentum then use, for tensor t, lr * lr_mult[t] and
 * wd * wd_mult[t], each product rounded to binary32.  Synchronises the device (the values must not change
 * under a running launch); not for the hot path.
 */
int pxchg_table_set_multipliers(pxchg_table *table, const float *lr_mult /*host*/, const float *wd_mult /*host*/);
/*
 * The same controls for one table (and its views) only: PXCHG_OPT_NONTEMPORAL and PXCHG_OPT_CENTER_RESIDENT,
 * with the values pxchg_set_option takes for them, override the process-wide setting for calls on this table;
 * PXCHG_TABLE_OPTION_INHERIT (the state of a new table) goes back to the process-wide one.  So an elastic server's
 * table can keep its center cached while the tables of a synchronous exchange in the same process stream.
 * Other options are PXCHG_ERR_INVALID_ARG (the chunk size is fixed when a table is made, the rest is not per
 * table).  pxchg_table_get_option returns the table's own value, PXCHG_TABLE_OPTION_INHERIT if it has none, and
 * -3 for a bad handle or option.  Not for a table with calls in flight on another thread that should all see
 * one setting: a call reads the option once, when it is made.
 */
#define PXCHG_TABLE_OPTION_INHERIT (-2)
int pxchg_table_set_option(pxchg_table *table, int option, int64_t value);
int64_t pxchg_table_get_option(const pxchg_table *table, int option);
int64_t pxchg_table_total(const pxchg_table *table);   /* sum of counts; -1 if NULL */
int pxchg_table_n_tensors(const pxchg_table *table);   /* -1 if NULL */
int64_t pxchg_table_n_chunks(const pxchg_table *table); /* -1 if NULL */

/*
 * Buffer set: `ptrs` is a HOST array of n_tensors DEVICE pointers, tensor t
 * holding counts[t] contiguous elements of `dtype`.  The pointer values are
 * copied (host and device side); the memory they point to stays the caller's
 * and must outlive every call that uses the set.  A NULL pointer is accepted
 * only for an empty tensor.
 */
int pxchg_bufset_create(const pxchg_table *table, int dtype, const void *const *ptrs /*host array of device ptrs*/,
                        pxchg_bufset **out);
int pxchg_bufset_destroy(pxchg_bufset *set);

/*
 * Section 3.2, half-precision transfer, sending side: for each of k workers,
 * dst[i][j] = binary16(src[i][j]), IEEE round-to-nearest-even, overflow to
 * infinity, gradual underflow, NaN stays NaN.  src[i] are F32 sets, dst[i] F16
 * sets, given as host arrays of k set handles.  One launch for all k workers
 * and all tensors.
 */
int pxchg_pack_fp16(const pxchg_table *table, int k, const pxchg_bufset *const *src_f32 /*host*/,
                    pxchg_bufset *const *dst_f16 /*host*/, void *stream);

/* Receiving side of the same transfer: dst[i][j] = (binary32) src[i][j], exact. */
int pxchg_unpack_fp16(const pxchg_table *table, int k, const pxchg_bufset *const *src_f16 /*host*/,
                      pxchg_bufset *const *dst_f32 /*host*/, void *stream);

/*
 * Section 3.2, the sum step of Alltoall-sum-Allgather on this rank's slice, and
 * Section 4's averaging: for every element j,
 *     s = contrib[0][j]; s = s + contrib[i][j] for i = 1..k-1 (binary32, this order)
 *     a = s / k (mode PXCHG_AVG, one correctly rounded division) or s (PXCHG_SUM)
 *     out[j] = a, rounded to binary16 (nearest-even) if `out` is an F16 set.
 * contrib[] is a host array of k sets, all F32 or all F16 (F16 is widened
 * exactly before the sum).  `out` may be one of the contrib sets of the same
 * element type (in place); otherwise it must not overlap them.
 */
int pxchg_reduce_avg(const pxchg_table *table, int k, const pxchg_bufset *const *contrib /*host*/,
                     pxchg_bufset *out, int mode, void *stream);

/*
 * Section 4, momentum SGD on the exchanged gradient, in place on param and vel
 * (both F32 sets):   gg = grad + wd * param;  vel = mu * vel - lr * gg;
 *                    param = param + vel
 * with every product and sum rounded to binary32 separately (no fused
 * multiply-add).  `grad` is an F32 set or an F16 set (widened exactly, the
 * unpack of the second transfer leg).
 */
int pxchg_sgd_momentum(const pxchg_table *table, const pxchg_bufset *grad, pxchg_bufset *param,
                       pxchg_bufset *vel, float lr, float mu, float wd, void *stream);

/*
 * Section 4, asynchronous mode: one elastic-averaging meeting of a worker's
 * parameters x with the center c, in place on both (F32 sets):
 *     d = alpha * (x - c);  x = x - d;  c = c + d      (each op rounded to binary32)
 */
int pxchg_easgd(const pxchg_table *table, pxchg_bufset *x, pxchg_bufset *c, float alpha, void *stream);

/*
 * Section 4, asynchronous mode (workers exchange with the server one after the
 * other, first come first served, no round-robin): a whole round of such
 * meetings.  Workers x[0], x[1], ..., x[k-1] (host array of k distinct F32 sets,
 * in their order of arrival) meet the center one after the other.  Bit-identical to k calls of pxchg_easgd in that order.  Up to 8
 * workers take one launch that reads and writes the center once; more workers
 * take one launch per group of 8.
 */
int pxchg_easgd_round(const pxchg_table *table, int k, pxchg_bufset *const *x /*host*/, pxchg_bufset *c,
                      float alpha, void *stream);

/*
 * Section 3.2's sum step (with the 1/k of an average) and Section 4's momentum
 * SGD step on its result, as one operation: what the rank that owns a slice
 * does between the two transfer legs when it also holds the parameters.
 * pxchg_reduce_avg followed by pxchg_sgd_momentum in one launch, without the
 * intermediate buffer.  `wire_dtype` says how the average would have travelled
 * on the second transfer leg: PXCHG_F16 rounds it once to binary16 and widens it
 * again before the update, PXCHG_F32 uses it as is.  Bit-identical to the two
 * separate calls with an `out` set of that type.  1 to 8 workers take kernels
 * specialised for that number, 9 to PXCHG_MAX_K a general one.
 */
int pxchg_reduce_avg_sgd_momentum(const pxchg_table *table, int k, const pxchg_bufset *const *contrib /*host*/,
                                  int mode, int wire_dtype, pxchg_bufset *param, pxchg_bufset *vel,
                                  float lr, float mu, float wd, void *stream);

/*
 * Diagnostics of one buffer set, for watching the reduced-precision exchange
 * whose accuracy cost Section 4 reports (an overflow in the pack shows up as an
 * infinity in the packed copy): over all elements of all tensors of `set` (F32,
 * or F16 widened exactly),
 *     nonfinite = number of infinities and NaNs,
 *     max_abs   = largest magnitude among the finite elements (0 if none),
 *     sum_sq    = sum of squares of the finite elements, accumulated in binary64
 *                 (its square root is the L2 norm).
 * `out` is DEVICE memory, 8-byte aligned, written by this call (no need to clear
 * it); it is valid once the stream has reached this point.
 *
 * All three are reproducible bit for bit, run after run and whatever else the
 * device is doing: the sum is taken in a fixed tree order that is part of this
 * definition.  The table's chunk list (pxchg_plan_chunks with the table's chunk
 * size; for a view, the view's part of it), numbered g = 0, 1, ..., is cut into
 * blocks of PXCHG_STATS_BLOCK_CHUNKS consecutive chunks.  A block has
 * PXCHG_STATS_WAVES x 64 accumulators, each starting at +0; element i of the
 * chunk at place j in its block goes to accumulator (wave, lane) =
 * (j mod PXCHG_STATS_WAVES, (i div p) mod 64), p being the elements in 16 bytes
 * (4 for F32, 8 for F16), and an accumulator takes its elements in increasing
 * (g, i) as acc = acc + x*x (square exact, sum rounded once).  Values are then
 * combined like this: combine(values, T): thread t of T adds values t, t + T,
 * t + 2T, ... in that order onto +0; the 64 threads of each group t div 64
 * exchange in a butterfly, a[l] = a[l] + a[l xor off] for off = 32, 16, 8, 4, 2,
 * 1; the groups' a[0] are added in group order starting from group 0's.  A
 * block's sum is combine(its accumulators in (wave, lane) order,
 * PXCHG_STATS_WAVES * 64); sum_sq is combine(the blocks' sums in block order,
 * PXCHG_STATS_COMBINE_THREADS).  (Like any binary64 sum of n non-negative terms
 * it is within a few dozen units of 2^-53 relative of the exact sum.)
 *
 * Two launches: one workgroup per block writes the block's partial result into
 * device memory that belongs to the table (allocated with it; views use their
 * parent's), one workgroup then combines the partial results into `out`.  Every
 * partial result is written before it is read, so nothing needs clearing, and
 * there are no atomics.  Calls on one table (or its views) that may overlap on
 * the device, on different streams, would share that memory: give such calls
 * separate tables, or order them.
 */
#ifndef PXCHG_STATS_WAVES
#define PXCHG_STATS_WAVES 4            /* wavefronts, and so 64-lane accumulator groups, per block */
#endif
#ifndef PXCHG_STATS_BLOCK_CHUNKS
#define PXCHG_STATS_BLOCK_CHUNKS 32    /* consecutive chunks per block */
#endif
#define PXCHG_STATS_COMBINE_THREADS 1024 /* T of the final combine */
typedef struct pxchg_stats {
    uint64_t nonfinite;
    double sum_sq;
    float max_abs;
    uint32_t reserved;
} pxchg_stats;

int pxchg_buffer_stats(const pxchg_table *table, const pxchg_bufset *set, pxchg_stats *out /*device*/, void *stream);

/*
 * The same call for callers that can allocate nothing and must not depend on memory that some earlier call
 * allocated for them: code running under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  It differs from pxchg_buffer_stats only in where the partial results live: in a fixed array of
 * PXCHG_STATS_STATIC_MAX_BLOCKS entries (24 bytes each, 384 KiB) that is part of the library's code object, one
 * copy per GPU, held until the process ends.  Same arguments, same results, bit for bit.  The call allocates and
 * frees nothing, on the device or through any library.  The array's address on the current device is looked up
 * once per device: by pxchg_table_create, or else by the first call on that device.
 * Limits: a chunk list of more than PXCHG_STATS_STATIC_MAX_BLOCKS * PXCHG_STATS_BLOCK_CHUNKS chunks (268,435,456
 * elements at the default chunk size) is PXCHG_ERR_UNSUPPORTED and launches nothing; use pxchg_buffer_stats.
 * Every call on a GPU shares that GPU's array, whatever the table: calls that may overlap on one GPU (different
 * streams) race on it, so order them.  Nothing in the array needs clearing between calls: each call writes the
 * entries it reads.
 */
#define PXCHG_STATS_STATIC_MAX_BLOCKS 16384
int pxchg_buffer_stats_static(const pxchg_table *table, const pxchg_bufset *set, pxchg_stats *out /*device*/,
                              void *stream);

#ifdef __cplusplus
}
#endif
#endif /* PXCHG_H */
