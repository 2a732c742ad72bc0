// Host-side objects of libpxchg: options, chunk planning, tensor tables and
// buffer sets.  Everything here runs at set-up time; the per-exchange calls live
// beside the kernels.
#include <algorithm>
#include <memory>
#include <mutex>
#include <new>
#include <unordered_map>

#include "pxchg_internal.h"

namespace {

constexpr int64_t kMinChunk = 512;
constexpr int64_t kMaxChunk = 1 << 20;

std::unordered_map<const void *, int> &registry() {
    static std::unordered_map<const void *, int> live;
    return live;
}
std::atomic<uint64_t> next_table_id{1};

using Shared = std::shared_lock<std::shared_mutex>;
using Exclusive = std::unique_lock<std::shared_mutex>;

// Owners for objects under construction: if a step fails, or host memory runs out (std::bad_alloc from a
// container), what has been allocated so far is given back and the call returns a status.  No exception crosses
// the C boundary.
struct TableDrop {
    void operator()(pxchg_table *t) const {
        if (!t->parent) {
            if (t->d_chunks) (void)hipFree(t->d_chunks);
            if (t->d_mult) (void)hipFree(t->d_mult);
            if (t->d_partials) (void)hipFree(t->d_partials);
        }
        delete t;
    }
};
struct SetDrop {
    void operator()(pxchg_bufset *s) const {
        if (s->d_ptrs) (void)hipFree(s->d_ptrs);
        delete s;
    }
};
using TableOwner = std::unique_ptr<pxchg_table, TableDrop>;
using SetOwner = std::unique_ptr<pxchg_bufset, SetDrop>;

}  // namespace

std::shared_mutex &px_registry_lock() {
    static std::shared_mutex mu;
    return mu;
}

bool px_live(const void *handle, int kind) {
    if (!handle) return false;
    const auto &live = registry();
    const auto it = live.find(handle);
    return it != live.end() && it->second == kind;
}

PxOptions &px_options() {
    static PxOptions o{{/*chunk_elems=*/512}, {/*blocks_per_cu=*/0}, {/*check_ranges=*/1}, {/*nontemporal=*/-1},
                       {/*center_resident=*/0}};
    return o;
}

int px_cu_count(int device) {
    // one word per device, filled on first use; two threads that race here look up the same number
    constexpr int kMaxDevices = 64;
    static std::atomic<int> cache[kMaxDevices];
    if (device < 0) return 0;
    if (device < kMaxDevices) {
        const int known = cache[device].load(std::memory_order_relaxed);
        if (known) return known;
    }
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || n <= 0) n = 256;
    if (device < kMaxDevices) cache[device].store(n, std::memory_order_relaxed);
    return n;
}

extern "C" {

const char *pxchg_status_string(int status) {
    switch (status) {
        case PXCHG_OK: return "ok";
        case PXCHG_ERR_INVALID_ARG: return "invalid argument";
        case PXCHG_ERR_SHAPE_MISMATCH: return "buffer set does not match the table or has the wrong element type";
        case PXCHG_ERR_UNSUPPORTED: return "unsupported size or worker count";
        case PXCHG_ERR_NO_DEVICE: return "no usable GPU, or the table's device is not current";
        case PXCHG_ERR_RUNTIME: return "HIP runtime call failed";
        case PXCHG_ERR_OUT_OF_RANGE: return "tensor does not fit inside its device allocation";
        case PXCHG_ERR_IN_USE: return "table still has views or buffer sets";
        default: return "unknown status";
    }
}

int pxchg_version(void) { return 200; }

int pxchg_set_option(int option, int64_t value) {
    PxOptions &o = px_options();
    switch (option) {
        case PXCHG_OPT_CHUNK_ELEMS:
            if (value < kMinChunk || value > kMaxChunk || value % kMinChunk) return PXCHG_ERR_INVALID_ARG;
            o.chunk_elems = value;
            return PXCHG_OK;
        case PXCHG_OPT_BLOCKS_PER_CU:
            if (value < 0 || value > 64) return PXCHG_ERR_INVALID_ARG;
            o.blocks_per_cu = value;
            return PXCHG_OK;
        case PXCHG_OPT_CHECK_RANGES:
            if (value != 0 && value != 1) return PXCHG_ERR_INVALID_ARG;
            o.check_ranges = value;
            return PXCHG_OK;
        case PXCHG_OPT_NONTEMPORAL:
            if (value < -1 || value > 5) return PXCHG_ERR_INVALID_ARG;
            // policies 1..5 exist for every kernel only in a tuning build of the library
            if (value > 0 && !px_all_policies_built()) return PXCHG_ERR_UNSUPPORTED;
            o.nontemporal = value;
            return PXCHG_OK;
        case PXCHG_OPT_CENTER_RESIDENT:
            if (value != 0 && value != 1) return PXCHG_ERR_INVALID_ARG;
            o.center_resident = value;
            return PXCHG_OK;
        default:
            return PXCHG_ERR_INVALID_ARG;
    }
}

int64_t pxchg_get_option(int option) {
    const PxOptions &o = px_options();
    switch (option) {
        case PXCHG_OPT_CHUNK_ELEMS: return o.chunk_elems;
        case PXCHG_OPT_BLOCKS_PER_CU: return o.blocks_per_cu;
        case PXCHG_OPT_CHECK_RANGES: return o.check_ranges;
        case PXCHG_OPT_NONTEMPORAL: return o.nontemporal;
        case PXCHG_OPT_CENTER_RESIDENT: return o.center_resident;
        case PXCHG_OPT_ALL_POLICIES_BUILT: return px_all_policies_built();
        default: return -1;
    }
}

int pxchg_plan_chunks(int n_tensors, const int64_t *counts, int64_t chunk_elems, int64_t cap,
                      int32_t *chunk_tensor, int64_t *chunk_start, int32_t *chunk_len, int64_t *n_chunks) {
    if (n_tensors < 1 || !counts || !n_chunks || cap < 0) return PXCHG_ERR_INVALID_ARG;
    if (chunk_elems < kMinChunk || chunk_elems > kMaxChunk || chunk_elems % kMinChunk) return PXCHG_ERR_INVALID_ARG;
    if (cap > 0 && (!chunk_tensor || !chunk_start || !chunk_len)) return PXCHG_ERR_INVALID_ARG;
    int64_t n = 0;
    for (int t = 0; t < n_tensors; ++t) {
        if (counts[t] < 0) return PXCHG_ERR_INVALID_ARG;
        for (int64_t s = 0; s < counts[t]; s += chunk_elems) {
            if (n < cap) {
                chunk_tensor[n] = t;
                chunk_start[n] = s;
                chunk_len[n] = (int32_t)std::min<int64_t>(chunk_elems, counts[t] - s);
            }
            ++n;
        }
    }
    *n_chunks = n;
    return PXCHG_OK;
}

int pxchg_plan_groups(int n_tensors, const int64_t *counts, int64_t min_elems, int reverse, int cap, int32_t *group_first,
                      int32_t *group_n, int *n_groups) {
    if (n_tensors < 1 || !counts || !n_groups || cap < 0 || min_elems < 0) return PXCHG_ERR_INVALID_ARG;
    if (cap > 0 && (!group_first || !group_n)) return PXCHG_ERR_INVALID_ARG;
    for (int t = 0; t < n_tensors; ++t)
        if (counts[t] < 0) return PXCHG_ERR_INVALID_ARG;
    int n = 0, run = 0;      // groups closed so far; tensors in the open group
    int64_t size = 0;        // elements in the open group
    for (int i = 0; i < n_tensors; ++i) {
        const int t = reverse ? n_tensors - 1 - i : i;
        ++run;
        size += counts[t];
        if (size >= min_elems || i == n_tensors - 1) {   // close the group (the last one takes what is left)
            if (n < cap) {
                group_first[n] = reverse ? t : t - run + 1;   // a group is a run of consecutive tensors either way
                group_n[n] = run;
            }
            ++n;
            run = 0;
            size = 0;
        }
    }
    *n_groups = n;
    return PXCHG_OK;
}

int pxchg_table_create(int n_tensors, const int64_t *counts, pxchg_table **out) try {
    if (!out) return PXCHG_ERR_INVALID_ARG;
    *out = nullptr;
    if (n_tensors < 1 || n_tensors > (1 << 24) || !counts) return PXCHG_ERR_INVALID_ARG;
    int64_t total = 0;
    for (int t = 0; t < n_tensors; ++t) {
        if (counts[t] < 0) return PXCHG_ERR_INVALID_ARG;
        if (counts[t] > ((int64_t)1 << 40) || total > ((int64_t)1 << 40)) return PXCHG_ERR_UNSUPPORTED;
        total += counts[t];
    }
    const int64_t chunk_elems = px_options().chunk_elems;
    int64_t n_chunks = 0;
    int rc = pxchg_plan_chunks(n_tensors, counts, chunk_elems, 0, nullptr, nullptr, nullptr, &n_chunks);
    if (rc != PXCHG_OK) return rc;
    // the grid (times up to PXCHG_MAX_K workers) must stay a 31-bit number
    if (n_chunks > ((int64_t)1 << 24)) return PXCHG_ERR_UNSUPPORTED;

    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device < 0) {
        (void)hipGetLastError();
        return PXCHG_ERR_NO_DEVICE;
    }

    TableOwner t(new pxchg_table());
    t->d_chunks = nullptr;
    t->d_mult = nullptr;
    t->d_partials = nullptr;
    t->parent = nullptr;
    t->id = next_table_id.fetch_add(1);
    t->device = device;
    t->n_tensors = n_tensors;
    t->total = total;
    t->chunk_elems = chunk_elems;
    t->n_chunks = n_chunks;
    t->counts.assign(counts, counts + n_tensors);
    t->first_tensor = 0;
    t->live_views = 0;
    t->live_sets = 0;
    t->opt_nontemporal = PXCHG_TABLE_OPTION_INHERIT;
    t->opt_center_resident = PXCHG_TABLE_OPTION_INHERIT;

    if (n_chunks > 0) {
        std::vector<PxChunk> h(n_chunks);
        int64_t n = 0;
        for (int i = 0; i < n_tensors; ++i)
            for (int64_t s = 0; s < counts[i]; s += chunk_elems) {
                h[n].start = s;
                h[n].len = (int32_t)std::min<int64_t>(chunk_elems, counts[i] - s);
                h[n].tensor = i;
                ++n;
            }
        // the chunk list, and one partial result per block of chunks for the diagnostics (written before it is
        // read in every call, so it needs no clearing)
        if (hipMalloc((void **)&t->d_chunks, n_chunks * sizeof(PxChunk)) != hipSuccess ||
            hipMemcpy(t->d_chunks, h.data(), n_chunks * sizeof(PxChunk), hipMemcpyHostToDevice) != hipSuccess ||
            hipMalloc((void **)&t->d_partials, px_stats_blocks(n_chunks) * sizeof(pxchg_stats)) != hipSuccess) {
            (void)hipGetLastError();
            return PXCHG_ERR_RUNTIME;
        }
    }
    // set-up for the allocation-free diagnostics call (the device is current here); if the look-up fails, that
    // call tries again and reports it
    (void)px_prepare_static_scratch(device);
    {
        Exclusive lock(px_registry_lock());
        registry()[t.get()] = PX_KIND_TABLE;
    }
    *out = t.release();
    return PXCHG_OK;
} catch (...) {
    return PXCHG_ERR_RUNTIME;  // host memory ran out
}

int pxchg_table_view(const pxchg_table *parent_c, int first_tensor, int n_tensors, pxchg_table **out) try {
    if (!out) return PXCHG_ERR_INVALID_ARG;
    *out = nullptr;
    Exclusive lock(px_registry_lock());
    pxchg_table *parent = const_cast<pxchg_table *>(parent_c);  // only its count of live views changes
    if (!px_valid(parent) || parent->parent) return PXCHG_ERR_INVALID_ARG;  // no views of views
    if (first_tensor < 0 || n_tensors < 1 || first_tensor > parent->n_tensors - n_tensors) return PXCHG_ERR_INVALID_ARG;
    // chunks never straddle tensors, so a run of tensors is a run of chunks
    const int64_t ce = parent->chunk_elems;
    int64_t first_chunk = 0, n_chunks = 0, total = 0;
    for (int t = 0; t < first_tensor; ++t) first_chunk += (parent->counts[t] + ce - 1) / ce;
    for (int t = first_tensor; t < first_tensor + n_tensors; ++t) {
        n_chunks += (parent->counts[t] + ce - 1) / ce;
        total += parent->counts[t];
    }
    TableOwner v(new pxchg_table());
    v->parent = parent;  // from here on the owner knows that this is a view: it frees no device memory
    v->id = next_table_id.fetch_add(1);
    v->device = parent->device;
    v->n_tensors = n_tensors;
    v->total = total;
    v->chunk_elems = ce;
    v->n_chunks = n_chunks;
    v->counts.assign(parent->counts.begin() + first_tensor, parent->counts.begin() + first_tensor + n_tensors);
    v->d_chunks = n_chunks ? parent->d_chunks + first_chunk : nullptr;
    v->d_mult = nullptr;      // the parent's multipliers apply (looked up at each call)
    v->d_partials = nullptr;  // and the parent's partial results
    v->first_tensor = first_tensor;
    v->live_views = 0;
    v->live_sets = 0;
    v->opt_nontemporal = PXCHG_TABLE_OPTION_INHERIT;      // unused: a view follows its parent
    v->opt_center_resident = PXCHG_TABLE_OPTION_INHERIT;
    registry()[v.get()] = PX_KIND_TABLE;
    ++parent->live_views;
    *out = v.release();
    return PXCHG_OK;
} catch (...) {
    return PXCHG_ERR_RUNTIME;  // host memory ran out
}

int pxchg_table_destroy(pxchg_table *table) {
    if (!table) return PXCHG_OK;
    {
        Exclusive lock(px_registry_lock());
        if (!px_valid(table)) return PXCHG_ERR_INVALID_ARG;  // never a handle, or destroyed already
        if (table->live_views || table->live_sets) return PXCHG_ERR_IN_USE;
        registry().erase(table);  // from here on every call rejects the handle
        if (table->parent) {      // a view owns nothing on the device
            --table->parent->live_views;
            delete table;
            return PXCHG_OK;
        }
    }
    int rc = PXCHG_OK;
    (void)hipDeviceSynchronize();  // launches still reading the chunk list must finish first
    if (table->d_chunks && hipFree(table->d_chunks) != hipSuccess) rc = PXCHG_ERR_RUNTIME;
    if (table->d_mult && hipFree(table->d_mult) != hipSuccess) rc = PXCHG_ERR_RUNTIME;
    if (table->d_partials && hipFree(table->d_partials) != hipSuccess) rc = PXCHG_ERR_RUNTIME;
    delete table;
    return rc;
}

int pxchg_table_set_multipliers(pxchg_table *table, const float *lr_mult, const float *wd_mult) try {
    Exclusive lock(px_registry_lock());  // no call may be reading d_mult while it changes
    if (!px_valid(table) || table->parent) return PXCHG_ERR_INVALID_ARG;  // set them on the parent
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device != table->device) {
        (void)hipGetLastError();
        return PXCHG_ERR_NO_DEVICE;
    }
    (void)hipDeviceSynchronize();  // no launch may be reading the old values while they change
    if (!lr_mult && !wd_mult) {
        if (table->d_mult && hipFree(table->d_mult) != hipSuccess) {
            (void)hipGetLastError();
            return PXCHG_ERR_RUNTIME;
        }
        table->d_mult = nullptr;
        return PXCHG_OK;
    }
    std::vector<float> h(2 * (size_t)table->n_tensors);
    for (int t = 0; t < table->n_tensors; ++t) {
        h[2 * t] = lr_mult ? lr_mult[t] : 1.0f;
        h[2 * t + 1] = wd_mult ? wd_mult[t] : 1.0f;
    }
    const size_t bytes = h.size() * sizeof(float);
    if (!table->d_mult && hipMalloc((void **)&table->d_mult, bytes) != hipSuccess) {
        (void)hipGetLastError();
        table->d_mult = nullptr;
        return PXCHG_ERR_RUNTIME;
    }
    if (hipMemcpy(table->d_mult, h.data(), bytes, hipMemcpyHostToDevice) != hipSuccess) {
        (void)hipGetLastError();
        return PXCHG_ERR_RUNTIME;
    }
    return PXCHG_OK;
} catch (...) {
    return PXCHG_ERR_RUNTIME;  // host memory ran out; the multipliers on the device are unchanged
}

int pxchg_table_set_option(pxchg_table *table, int option, int64_t value) {
    Shared lock(px_registry_lock());
    if (!px_valid(table) || table->parent) return PXCHG_ERR_INVALID_ARG;  // set them on the parent
    switch (option) {
        case PXCHG_OPT_NONTEMPORAL:
            if (value != PXCHG_TABLE_OPTION_INHERIT && (value < -1 || value > 5)) return PXCHG_ERR_INVALID_ARG;
            if (value > 0 && !px_all_policies_built()) return PXCHG_ERR_UNSUPPORTED;
            table->opt_nontemporal = value;
            return PXCHG_OK;
        case PXCHG_OPT_CENTER_RESIDENT:
            if (value != PXCHG_TABLE_OPTION_INHERIT && value != 0 && value != 1) return PXCHG_ERR_INVALID_ARG;
            table->opt_center_resident = value;
            return PXCHG_OK;
        default:
            return PXCHG_ERR_INVALID_ARG;
    }
}

int64_t pxchg_table_get_option(const pxchg_table *table, int option) {
    Shared lock(px_registry_lock());
    if (!px_valid(table)) return -3;
    switch (option) {
        case PXCHG_OPT_NONTEMPORAL: return px_root(table)->opt_nontemporal.load();
        case PXCHG_OPT_CENTER_RESIDENT: return px_root(table)->opt_center_resident.load();
        default: return -3;
    }
}

int64_t pxchg_table_total(const pxchg_table *table) {
    Shared lock(px_registry_lock());
    return px_valid(table) ? table->total : -1;
}
int pxchg_table_n_tensors(const pxchg_table *table) {
    Shared lock(px_registry_lock());
    return px_valid(table) ? table->n_tensors : -1;
}
int64_t pxchg_table_n_chunks(const pxchg_table *table) {
    Shared lock(px_registry_lock());
    return px_valid(table) ? table->n_chunks : -1;
}

int pxchg_bufset_create(const pxchg_table *table_c, int dtype, const void *const *ptrs, pxchg_bufset **out) try {
    if (!out) return PXCHG_ERR_INVALID_ARG;
    *out = nullptr;
    Exclusive lock(px_registry_lock());
    pxchg_table *table = const_cast<pxchg_table *>(table_c);  // only its count of live sets changes
    if (!px_valid(table) || !ptrs) return PXCHG_ERR_INVALID_ARG;
    if (table->parent) return PXCHG_ERR_INVALID_ARG;  // buffer sets belong to the parent and serve its views
    if (dtype != PXCHG_F32 && dtype != PXCHG_F16) return PXCHG_ERR_INVALID_ARG;
    const size_t es = dtype == PXCHG_F32 ? 4 : 2;
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device != table->device) {
        (void)hipGetLastError();
        return PXCHG_ERR_NO_DEVICE;
    }
    for (int t = 0; t < table->n_tensors; ++t) {
        const int64_t n = table->counts[t];
        if (n == 0) continue;
        const uintptr_t a = (uintptr_t)ptrs[t];
        if (a == 0 || a % es) return PXCHG_ERR_INVALID_ARG;
        if (px_options().check_ranges) {
            // The kernels trust counts[t]; make sure the whole tensor lies inside one
            // device allocation so that no launch can touch unmapped memory.
            hipDeviceptr_t base = nullptr;
            size_t size = 0;
            if (hipMemGetAddressRange(&base, &size, (hipDeviceptr_t)ptrs[t]) != hipSuccess) {
                (void)hipGetLastError();
                return PXCHG_ERR_OUT_OF_RANGE;
            }
            const uintptr_t b = (uintptr_t)base;
            if (a < b || a + (uintptr_t)n * es > b + size) return PXCHG_ERR_OUT_OF_RANGE;
        }
    }
    SetOwner s(new pxchg_bufset());
    s->d_ptrs = nullptr;
    s->table = table;
    s->table_id = table->id;
    s->dtype = dtype;
    s->h_ptrs.assign(ptrs, ptrs + table->n_tensors);
    const size_t bytes = (size_t)table->n_tensors * sizeof(void *);
    if (hipMalloc((void **)&s->d_ptrs, bytes) != hipSuccess ||
        hipMemcpy(s->d_ptrs, s->h_ptrs.data(), bytes, hipMemcpyHostToDevice) != hipSuccess) {
        (void)hipGetLastError();
        return PXCHG_ERR_RUNTIME;
    }
    registry()[s.get()] = PX_KIND_BUFSET;
    ++table->live_sets;
    *out = s.release();
    return PXCHG_OK;
} catch (...) {
    return PXCHG_ERR_RUNTIME;  // host memory ran out
}

int pxchg_bufset_destroy(pxchg_bufset *set) {
    if (!set) return PXCHG_OK;
    {
        Exclusive lock(px_registry_lock());
        if (!px_valid(set)) return PXCHG_ERR_INVALID_ARG;  // never a handle, or destroyed already
        registry().erase(set);
        // its table is alive: a table cannot be destroyed while it has sets
        --set->table->live_sets;
    }
    int rc = PXCHG_OK;
    (void)hipDeviceSynchronize();  // launches still reading the pointer table must finish first
    if (set->d_ptrs && hipFree(set->d_ptrs) != hipSuccess) rc = PXCHG_ERR_RUNTIME;
    delete set;
    return rc;
}

}  // extern "C"
