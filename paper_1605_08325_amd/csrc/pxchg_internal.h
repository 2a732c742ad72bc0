// Internal structures of libpxchg shared by the host-side object code and the
// kernel launchers.  Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
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
    uint32_t magic;
    int device;
    int n_tensors;
    int64_t total;
    int64_t chunk_elems;
    int64_t n_chunks;
    std::vector<int64_t> counts;
    PxChunk *d_chunks;  // device copy of the chunk list (a view: the part of its parent's list it covers)
    float *d_mult;      // optional: n_tensors pairs (lr multiplier, decay multiplier); null = all ones
    const pxchg_table *parent;  // null for a table of its own; a view owns no device memory
    int first_tensor;           // a view covers the parent's tensors first_tensor .. first_tensor + n_tensors - 1
};

// The table that owns the device-side lists, the multipliers and the buffer sets.
inline const pxchg_table *px_root(const pxchg_table *t) { return t->parent ? t->parent : t; }

struct pxchg_bufset {
    uint32_t magic;
    const pxchg_table *table;
    int dtype;
    std::vector<const void *> h_ptrs;  // host copy of the device pointers
    void **d_ptrs;                     // device array of n_tensors pointers
};

constexpr uint32_t PX_TABLE_MAGIC = 0x70784354u;
constexpr uint32_t PX_BUFSET_MAGIC = 0x70784253u;

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

// Compute units of the current device (cached per device).
int px_cu_count(int device);

inline bool px_valid(const pxchg_table *t) { return t && t->magic == PX_TABLE_MAGIC; }
inline bool px_valid(const pxchg_bufset *s) { return s && s->magic == PX_BUFSET_MAGIC; }
