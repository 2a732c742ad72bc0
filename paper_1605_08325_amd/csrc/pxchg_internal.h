// Internal structures of libpxchg shared by the host-side object code and the
// kernel launchers.  Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <shared_mutex>
#include <vector>

#include "pxchg.h"

// One unit of work for a workgroup: `len` consecutive elements of tensor
// `tensor`, starting `start` elements into it.  Chunks never straddle tensors.
struct PxChunk {
    int64_t start;
    int32_t len;
    int32_t tensor;
};
static_assert(sizeof(PxChunk) == 16, "chunk descriptors are read as one 16-byte load");

struct pxchg_table {
    uint64_t id;  // unique per creation in this process: a buffer set remembers it, so a new table that happens
                  // to be allocated at a destroyed table's address does not inherit that table's sets
    int device;
    int n_tensors;
    int64_t total;
    int64_t chunk_elems;
    int64_t n_chunks;
    std::vector<int64_t> counts;
    PxChunk *d_chunks;  // device copy of the chunk list (a view: the part of its parent's list it covers)
    float *d_mult;      // optional: n_tensors pairs (lr multiplier, decay multiplier); null = all ones
    pxchg_stats *d_partials;  // one partial result per block of chunks for pxchg_buffer_stats (views use the parent's)
    pxchg_table *parent;      // null for a table of its own; a view owns no device memory
    int first_tensor;         // a view covers the parent's tensors first_tensor .. first_tensor + n_tensors - 1
    int live_views;           // handles that point into this table; it cannot be destroyed before them
    int live_sets;            // (both changed only under the registry's exclusive lock)
    std::atomic<int64_t> opt_nontemporal;      // this table's own setting, or PXCHG_TABLE_OPTION_INHERIT
    std::atomic<int64_t> opt_center_resident;  // (a view uses its parent's)
};

// The table that owns the device-side lists, the multipliers and the buffer sets.
inline const pxchg_table *px_root(const pxchg_table *t) { return t->parent ? t->parent : t; }

struct pxchg_bufset {
    pxchg_table *table;
    uint64_t table_id;
    int dtype;
    std::vector<const void *> h_ptrs;  // host copy of the device pointers
    void **d_ptrs;                     // device array of n_tensors pointers
};

// Live handles.  A pointer is a valid handle exactly while the registry lists it with its kind: nothing is ever
// read through a pointer that is not listed, so a destroyed handle, a handle of the other kind and arbitrary
// memory are all told apart without touching them.  Calls that use handles hold the shared lock for their
// duration (they run concurrently); create and destroy take the exclusive lock, so a handle cannot disappear
// under a call that has validated it.
enum PxKind { PX_KIND_TABLE = 1, PX_KIND_BUFSET = 2 };
std::shared_mutex &px_registry_lock();
bool px_live(const void *handle, int kind);  // caller holds the lock (shared or exclusive)
inline bool px_valid(const pxchg_table *t) { return px_live(t, PX_KIND_TABLE); }
inline bool px_valid(const pxchg_bufset *s) { return px_live(s, PX_KIND_BUFSET); }

// Process-wide settings.  Each is one atomic word, so a thread that changes one while another thread is in a
// call is not a data race: that call sees the old or the new value of each option it reads.
struct PxOptions {
    std::atomic<int64_t> chunk_elems;
    std::atomic<int64_t> blocks_per_cu;
    std::atomic<int64_t> check_ranges;
    std::atomic<int64_t> nontemporal;
    std::atomic<int64_t> center_resident;
};
PxOptions &px_options();

// The cache policy and the center-resident switch in force for a call on `t`: the table's own setting (its
// parent's for a view) if it has one, else the process-wide option.
inline int64_t px_nontemporal_for(const pxchg_table *t) {
    const int64_t own = px_root(t)->opt_nontemporal.load();
    return own != PXCHG_TABLE_OPTION_INHERIT ? own : px_options().nontemporal.load();
}
inline bool px_center_resident_for(const pxchg_table *t) {
    const int64_t own = px_root(t)->opt_center_resident.load();
    return (own != PXCHG_TABLE_OPTION_INHERIT ? own : px_options().center_resident.load()) != 0;
}


// 1 if every cache policy of every kernel is compiled in (a tuning build), 0 if only each kernel's own policy and
// the plain one are.  Defined beside the kernels.
int px_all_policies_built();

// Looks up, once per device, this device's copy of the static array that pxchg_buffer_stats_static keeps its
// partial results in.  `device` must be current.  Called when a table is created, so that the exchange calls
// find the address ready.  Defined beside the array.
int px_prepare_static_scratch(int device);

// Compute units of the current device (cached per device).
int px_cu_count(int device);

// Blocks of PXCHG_STATS_BLOCK_CHUNKS chunks that pxchg_buffer_stats cuts a chunk list into.
inline int64_t px_stats_blocks(int64_t n_chunks) {
    return (n_chunks + PXCHG_STATS_BLOCK_CHUNKS - 1) / PXCHG_STATS_BLOCK_CHUNKS;
}
