// Host-only driver for the library's host code: options, chunk planning, handle lifetime, argument validation
// and the launch arithmetic of every call, built with AddressSanitizer and UBSan on the host side by
// tests/test_abi_sanitizers.py.  No GPU is used: the few HIP runtime calls the library makes are defined below
// as a stand-in (device memory is host memory, a launch is recorded and not run), and since they are part of
// this program the library objects linked into it call them instead of the real runtime.  So every path that
// only decides what to launch runs here, under the sanitizers, including what happens to handles that were
// destroyed.  Prints "ok" and exits 0 when every check holds and the sanitizers saw nothing.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <new>
#include <thread>
#include <vector>

#include "pxchg.h"

// ---------------------------------------------------------------- stand-in runtime

namespace fake {
int current_device = 0;
std::mutex mu;                            // the real runtime is thread-safe; so is this one
std::map<uintptr_t, size_t> allocations;  // base -> size
std::atomic<int> launches{0}, get_last_error_calls{0}, synchronizes{0}, symbol_lookups{0}, mallocs{0};
bool fail_next_launch = false;
dim3 last_grid, last_block;
std::vector<dim3> grids;
// Failure injection: the n-th host allocation (operator new) or device allocation (hipMalloc) from now fails;
// -1 = none.  The stand-in runtime's own bookkeeping is exempt.
long new_countdown = -1, malloc_countdown = -1;
std::atomic<long> live_host_blocks{0};  // operator new minus operator delete
thread_local int exempt = 0;
struct Exempt {
    Exempt() { ++exempt; }
    ~Exempt() { --exempt; }
};
}  // namespace fake

// Replacements for the global allocation functions, so that running out of host memory can be rehearsed (left
// out with -DPXCHG_DRIVER_NO_ALLOC_HOOKS: ThreadSanitizer's runtime brings its own).
#ifndef PXCHG_DRIVER_NO_ALLOC_HOOKS
static void *counted_alloc(std::size_t size) {
    if (!fake::exempt && fake::new_countdown >= 0 && fake::new_countdown-- == 0) throw std::bad_alloc();
    void *p = std::malloc(size ? size : 1);
    if (!p) throw std::bad_alloc();
    ++fake::live_host_blocks;
    return p;
}
static void counted_free(void *p) {
    if (!p) return;
    --fake::live_host_blocks;
    std::free(p);
}
void *operator new(std::size_t size) { return counted_alloc(size); }
void *operator new[](std::size_t size) { return counted_alloc(size); }
void operator delete(void *p) noexcept { counted_free(p); }
void operator delete[](void *p) noexcept { counted_free(p); }
void operator delete(void *p, std::size_t) noexcept { counted_free(p); }
void operator delete[](void *p, std::size_t) noexcept { counted_free(p); }
constexpr int kFirstFailureKind = 0;
#else
constexpr int kFirstFailureKind = 1;  // device allocations only
#endif

extern "C" {
hipError_t hipGetDevice(int *device) {
    *device = fake::current_device;
    return hipSuccess;
}
hipError_t hipDeviceGetAttribute(int *value, hipDeviceAttribute_t, int) {
    *value = 256;
    return hipSuccess;
}
hipError_t hipMalloc(void **ptr, size_t size) {
    fake::Exempt exempt;
    *ptr = nullptr;
    if (fake::malloc_countdown >= 0 && fake::malloc_countdown-- == 0) return hipErrorOutOfMemory;
    *ptr = std::malloc(size ? size : 1);
    if (!*ptr) return hipErrorOutOfMemory;
    ++fake::mallocs;
    std::lock_guard<std::mutex> lock(fake::mu);
    fake::allocations[(uintptr_t)*ptr] = size;
    return hipSuccess;
}
hipError_t hipFree(void *ptr) {
    fake::Exempt exempt;
    if (!ptr) return hipSuccess;
    {
        std::lock_guard<std::mutex> lock(fake::mu);
        if (!fake::allocations.erase((uintptr_t)ptr)) return hipErrorInvalidValue;
    }
    std::free(ptr);
    return hipSuccess;
}
hipError_t hipMemcpy(void *dst, const void *src, size_t bytes, hipMemcpyKind) {
    std::memcpy(dst, src, bytes);
    return hipSuccess;
}
hipError_t hipDeviceSynchronize(void) {
    ++fake::synchronizes;
    return hipSuccess;
}
hipError_t hipGetLastError(void) {
    ++fake::get_last_error_calls;
    return hipSuccess;
}
hipError_t hipMemGetAddressRange(hipDeviceptr_t *base, size_t *size, hipDeviceptr_t ptr) {
    const uintptr_t a = (uintptr_t)ptr;
    std::lock_guard<std::mutex> lock(fake::mu);
    auto it = fake::allocations.upper_bound(a);
    if (it == fake::allocations.begin()) return hipErrorInvalidValue;
    --it;
    if (a >= it->first + it->second) return hipErrorInvalidValue;
    *base = (hipDeviceptr_t)it->first;
    *size = it->second;
    return hipSuccess;
}
hipError_t hipGetSymbolAddress(void **address, const void *symbol) {
    static pxchg_stats standin[PXCHG_STATS_STATIC_MAX_BLOCKS];  // what a device would hold
    if (!symbol) return hipErrorInvalidSymbol;
    ++fake::symbol_lookups;
    *address = standin;
    return hipSuccess;
}
hipError_t hipLaunchKernel(const void *function, dim3 grid, dim3 block, void **args, size_t, hipStream_t) {
    if (!function || !args) return hipErrorInvalidValue;
    fake::Exempt exempt;
    std::lock_guard<std::mutex> lock(fake::mu);
    if (fake::fail_next_launch) {
        fake::fail_next_launch = false;
        return hipErrorLaunchFailure;
    }
    ++fake::launches;
    fake::last_grid = grid;
    fake::last_block = block;
    fake::grids.push_back(grid);
    return hipSuccess;
}
}

#define CHECK(cond)                                                   \
    do {                                                              \
        if (!(cond)) {                                                \
            std::printf("check failed, line %d: %s\n", __LINE__, #cond); \
            return 1;                                                 \
        }                                                             \
    } while (0)

namespace {

// One "device" buffer per tensor.
struct Buffers {
    std::vector<void *> ptrs;
    Buffers(const std::vector<int64_t> &counts, size_t es) {
        for (int64_t c : counts) {
            void *p = nullptr;
            if (c) (void)hipMalloc(&p, (size_t)c * es);
            ptrs.push_back(p);
        }
    }
    ~Buffers() {
        for (void *p : ptrs) (void)hipFree(p);
    }
    const void *const *data() const { return ptrs.data(); }
};

int options_and_planning() {
    for (int s = -2; s < 12; ++s) CHECK(pxchg_status_string(s) != nullptr && std::strlen(pxchg_status_string(s)) > 0);
    CHECK(pxchg_version() >= 200);

    // options: defaults, limits, restore
    CHECK(pxchg_get_option(PXCHG_OPT_CHUNK_ELEMS) == 512);
    CHECK(pxchg_set_option(PXCHG_OPT_CHUNK_ELEMS, 500) == PXCHG_ERR_INVALID_ARG);
    CHECK(pxchg_set_option(PXCHG_OPT_CHUNK_ELEMS, 0) == PXCHG_ERR_INVALID_ARG);
    CHECK(pxchg_set_option(PXCHG_OPT_CHUNK_ELEMS, (int64_t)1 << 40) == PXCHG_ERR_INVALID_ARG);
    CHECK(pxchg_set_option(PXCHG_OPT_CHUNK_ELEMS, 2048) == PXCHG_OK && pxchg_get_option(PXCHG_OPT_CHUNK_ELEMS) == 2048);
    CHECK(pxchg_set_option(PXCHG_OPT_CHUNK_ELEMS, 512) == PXCHG_OK);
    CHECK(pxchg_set_option(PXCHG_OPT_NONTEMPORAL, 6) == PXCHG_ERR_INVALID_ARG);
    CHECK(pxchg_set_option(PXCHG_OPT_NONTEMPORAL, -2) == PXCHG_ERR_INVALID_ARG);
    CHECK(pxchg_set_option(PXCHG_OPT_NONTEMPORAL, 0) == PXCHG_OK && pxchg_set_option(PXCHG_OPT_NONTEMPORAL, -1) == PXCHG_OK);
    const int64_t all = pxchg_get_option(PXCHG_OPT_ALL_POLICIES_BUILT);
    CHECK(all == 0 || all == 1);
    // the other policies exist only in the tuning build; the regular one says so instead of falling back
    CHECK(pxchg_set_option(PXCHG_OPT_NONTEMPORAL, 4) == (all ? PXCHG_OK : PXCHG_ERR_UNSUPPORTED));
    CHECK(pxchg_set_option(PXCHG_OPT_NONTEMPORAL, -1) == PXCHG_OK);
    CHECK(pxchg_set_option(PXCHG_OPT_ALL_POLICIES_BUILT, 1) == PXCHG_ERR_INVALID_ARG);  // read-only
    CHECK(pxchg_set_option(PXCHG_OPT_BLOCKS_PER_CU, 65) == PXCHG_ERR_INVALID_ARG);
    CHECK(pxchg_set_option(PXCHG_OPT_CHECK_RANGES, 2) == PXCHG_ERR_INVALID_ARG);
    CHECK(pxchg_get_option(PXCHG_OPT_CENTER_RESIDENT) == 0);
    CHECK(pxchg_set_option(PXCHG_OPT_CENTER_RESIDENT, 2) == PXCHG_ERR_INVALID_ARG);
    CHECK(pxchg_set_option(PXCHG_OPT_CENTER_RESIDENT, 1) == PXCHG_OK && pxchg_get_option(PXCHG_OPT_CENTER_RESIDENT) == 1);
    CHECK(pxchg_set_option(PXCHG_OPT_CENTER_RESIDENT, 0) == PXCHG_OK);
    CHECK(pxchg_set_option(99, 0) == PXCHG_ERR_INVALID_ARG && pxchg_get_option(99) == -1);

    // chunk planning: count first, then fill exactly that many, then a too-small capacity
    const int64_t counts[] = {0, 1, 511, 512, 513, 1237, 0, 4096};
    const int nt = (int)(sizeof(counts) / sizeof(counts[0]));
    int64_t n = -1;
    CHECK(pxchg_plan_chunks(nt, counts, 512, 0, nullptr, nullptr, nullptr, &n) == PXCHG_OK);
    CHECK(n == 0 + 1 + 1 + 1 + 2 + 3 + 0 + 8);
    std::vector<int32_t> tensor(n), len(n);
    std::vector<int64_t> start(n);
    int64_t n2 = -1;
    CHECK(pxchg_plan_chunks(nt, counts, 512, n, tensor.data(), start.data(), len.data(), &n2) == PXCHG_OK && n2 == n);
    std::vector<int64_t> covered(nt, 0);
    for (int64_t i = 0; i < n; ++i) {
        CHECK(tensor[i] >= 0 && tensor[i] < nt && len[i] >= 1 && len[i] <= 512);
        CHECK(start[i] == covered[tensor[i]]);  // chunks of a tensor are consecutive and in order
        covered[tensor[i]] += len[i];
        if (i) CHECK(tensor[i] >= tensor[i - 1]);
    }
    for (int t = 0; t < nt; ++t) CHECK(covered[t] == counts[t]);
    std::vector<int32_t> small_t(3), small_l(3);
    std::vector<int64_t> small_s(3);
    CHECK(pxchg_plan_chunks(nt, counts, 512, 3, small_t.data(), small_s.data(), small_l.data(), &n2) == PXCHG_OK);
    CHECK(n2 == n);  // reports what is needed, writes only what fits
    const int64_t negative[] = {4, -1};
    CHECK(pxchg_plan_chunks(2, negative, 512, 0, nullptr, nullptr, nullptr, &n2) == PXCHG_ERR_INVALID_ARG);
    CHECK(pxchg_plan_chunks(nt, counts, 100, 0, nullptr, nullptr, nullptr, &n2) == PXCHG_ERR_INVALID_ARG);
    CHECK(pxchg_plan_chunks(nt, counts, 512, 4, nullptr, nullptr, nullptr, &n2) == PXCHG_ERR_INVALID_ARG);
    CHECK(pxchg_plan_chunks(0, counts, 512, 0, nullptr, nullptr, nullptr, &n2) == PXCHG_ERR_INVALID_ARG);

    // tables: argument errors come before any use of a device
    pxchg_table *table = (pxchg_table *)0x1;
    CHECK(pxchg_table_create(0, counts, &table) == PXCHG_ERR_INVALID_ARG && table == nullptr);
    CHECK(pxchg_table_create(nt, nullptr, &table) == PXCHG_ERR_INVALID_ARG);
    CHECK(pxchg_table_create(nt, counts, nullptr) == PXCHG_ERR_INVALID_ARG);
    CHECK(pxchg_table_create(2, negative, &table) == PXCHG_ERR_INVALID_ARG);
    const int64_t huge[] = {(int64_t)1 << 41};
    CHECK(pxchg_table_create(1, huge, &table) == PXCHG_ERR_UNSUPPORTED);
    const int64_t many_chunks[] = {((int64_t)1 << 24) * 512 + 1};
    CHECK(pxchg_table_create(1, many_chunks, &table) == PXCHG_ERR_UNSUPPORTED);
    CHECK(pxchg_table_create(nt, counts, &table) == PXCHG_OK && table != nullptr);
    CHECK(pxchg_table_total(table) == 1 + 511 + 512 + 513 + 1237 + 4096);
    CHECK(pxchg_table_n_tensors(table) == nt && pxchg_table_n_chunks(table) == n);
    CHECK(pxchg_table_destroy(table) == PXCHG_OK);
    CHECK(pxchg_table_destroy(nullptr) == PXCHG_OK && pxchg_bufset_destroy(nullptr) == PXCHG_OK);
    CHECK(pxchg_table_total(nullptr) == -1 && pxchg_table_n_tensors(nullptr) == -1 && pxchg_table_n_chunks(nullptr) == -1);

    // a block of memory that is not a handle must be rejected by every call that takes one, unread
    alignas(16) unsigned char junk[256];
    std::memset(junk, 0x5a, sizeof(junk));
    pxchg_table *not_a_table = (pxchg_table *)junk;
    pxchg_bufset *not_a_set = (pxchg_bufset *)junk;
    pxchg_bufset *set = nullptr;
    const void *ptrs[8] = {};
    CHECK(pxchg_table_destroy(not_a_table) == PXCHG_ERR_INVALID_ARG);
    CHECK(pxchg_bufset_destroy(not_a_set) == PXCHG_ERR_INVALID_ARG);
    CHECK(pxchg_table_total(not_a_table) == -1);
    CHECK(pxchg_bufset_create(not_a_table, PXCHG_F32, ptrs, &set) == PXCHG_ERR_INVALID_ARG && set == nullptr);
    CHECK(pxchg_bufset_create(nullptr, PXCHG_F32, ptrs, &set) == PXCHG_ERR_INVALID_ARG);
    CHECK(pxchg_table_set_multipliers(not_a_table, nullptr, nullptr) == PXCHG_ERR_INVALID_ARG);
    pxchg_table *view = (pxchg_table *)0x1;
    CHECK(pxchg_table_view(not_a_table, 0, 1, &view) == PXCHG_ERR_INVALID_ARG && view == nullptr);
    CHECK(pxchg_table_view(nullptr, 0, 1, &view) == PXCHG_ERR_INVALID_ARG);
    CHECK(pxchg_table_view(not_a_table, 0, 1, nullptr) == PXCHG_ERR_INVALID_ARG);
    return 0;
}

// Every call that takes handles, with `table`, `a`, `b`, `c` (F32 sets) and `h` (an F16 set); returns the
// statuses in a fixed order.
std::vector<int> every_hot_call(pxchg_table *table, pxchg_bufset *a, pxchg_bufset *b, pxchg_bufset *c, pxchg_bufset *h,
                                pxchg_stats *out) {
    const pxchg_bufset *in1[1] = {a};
    pxchg_bufset *out1[1] = {h};
    const pxchg_bufset *hin[1] = {h};
    pxchg_bufset *fout[1] = {b};
    const pxchg_bufset *two[2] = {a, b};
    pxchg_bufset *xs[2] = {a, b};
    return {
        pxchg_pack_fp16(table, 1, in1, out1, nullptr),
        pxchg_unpack_fp16(table, 1, hin, fout, nullptr),
        pxchg_reduce_avg(table, 2, two, c, PXCHG_AVG, nullptr),
        pxchg_sgd_momentum(table, h, a, b, 0.01f, 0.9f, 0.0f, nullptr),
        pxchg_easgd(table, a, c, 0.0625f, nullptr),
        pxchg_easgd_round(table, 2, xs, c, 0.0625f, nullptr),
        pxchg_reduce_avg_sgd_momentum(table, 1, hin, PXCHG_AVG, PXCHG_F16, a, b, 0.01f, 0.9f, 0.0f, nullptr),
        pxchg_buffer_stats(table, h, out, nullptr),
        pxchg_buffer_stats_static(table, h, out, nullptr),
    };
}

int lifetime_and_launches() {
    const std::vector<int64_t> counts = {1000, 0, 513, 40000};
    const int nt = (int)counts.size();
    const int64_t n_chunks = 2 + 0 + 2 + 79;
    pxchg_table *table = nullptr, *other = nullptr;
    CHECK(pxchg_table_create(nt, counts.data(), &table) == PXCHG_OK);
    CHECK(pxchg_table_create(nt, counts.data(), &other) == PXCHG_OK);
    CHECK(pxchg_table_n_chunks(table) == n_chunks);
    Buffers fa(counts, 4), fb(counts, 4), fc(counts, 4), hh(counts, 2);
    pxchg_bufset *a = nullptr, *b = nullptr, *c = nullptr, *h = nullptr, *foreign = nullptr;
    CHECK(pxchg_bufset_create(table, PXCHG_F32, fa.data(), &a) == PXCHG_OK);
    CHECK(pxchg_bufset_create(table, PXCHG_F32, fb.data(), &b) == PXCHG_OK);
    CHECK(pxchg_bufset_create(table, PXCHG_F32, fc.data(), &c) == PXCHG_OK);
    CHECK(pxchg_bufset_create(table, PXCHG_F16, hh.data(), &h) == PXCHG_OK);
    CHECK(pxchg_bufset_create(other, PXCHG_F32, fa.data(), &foreign) == PXCHG_OK);
    pxchg_stats *out = nullptr;
    CHECK(hipMalloc((void **)&out, sizeof(pxchg_stats)) == hipSuccess);

    // a binary16 buffer registered as float32 claims twice its size: refused when the set is made
    pxchg_bufset *too_long = nullptr;
    CHECK(pxchg_bufset_create(table, PXCHG_F32, hh.data(), &too_long) == PXCHG_ERR_OUT_OF_RANGE && too_long == nullptr);
    const void *misaligned[4] = {(const char *)fa.ptrs[0] + 2, nullptr, fa.ptrs[2], fa.ptrs[3]};
    CHECK(pxchg_bufset_create(table, PXCHG_F32, misaligned, &too_long) == PXCHG_ERR_INVALID_ARG);
    const void *missing[4] = {fa.ptrs[0], nullptr, nullptr, fa.ptrs[3]};  // only an empty tensor may have no buffer
    CHECK(pxchg_bufset_create(table, PXCHG_F32, missing, &too_long) == PXCHG_ERR_INVALID_ARG);

    // ---- valid handles: one launch per call (two for the diagnostics), of the expected shape, and no call
    // looks at (or clears) the runtime's last-error state
    const int errs_before = fake::get_last_error_calls, syncs_before = fake::synchronizes;
    fake::launches = 0;
    fake::grids.clear();
    for (int rc : every_hot_call(table, a, b, c, h, out)) CHECK(rc == PXCHG_OK);
    CHECK(fake::launches == 11);
    CHECK(fake::get_last_error_calls == errs_before && fake::synchronizes == syncs_before);
    // one workgroup per chunk, two for the single meeting (call 4)
    for (size_t i = 0; i < 7; ++i) CHECK(fake::grids[i].x == (unsigned)(i == 4 ? 2 * n_chunks : n_chunks) && fake::grids[i].y == 1);
    const int64_t n_blocks = (n_chunks + PXCHG_STATS_BLOCK_CHUNKS - 1) / PXCHG_STATS_BLOCK_CHUNKS;
    CHECK(fake::grids[7].x == (unsigned)n_blocks && fake::grids[8].x == 1);
    CHECK(fake::last_block.x == PXCHG_STATS_COMBINE_THREADS);
    // pack of 3 workers: one launch over 3 x n_chunks
    {
        const pxchg_bufset *src[3] = {a, b, c};
        Buffers h2(counts, 2), h3(counts, 2);
        pxchg_bufset *s2 = nullptr, *s3 = nullptr;
        CHECK(pxchg_bufset_create(table, PXCHG_F16, h2.data(), &s2) == PXCHG_OK);
        CHECK(pxchg_bufset_create(table, PXCHG_F16, h3.data(), &s3) == PXCHG_OK);
        pxchg_bufset *dst[3] = {h, s2, s3};
        fake::launches = 0;
        CHECK(pxchg_pack_fp16(table, 3, src, dst, nullptr) == PXCHG_OK);
        CHECK(fake::launches == 1 && fake::last_grid.x == (unsigned)(3 * n_chunks) && fake::last_block.x == 64);
        pxchg_bufset *same[3] = {h, s2, s2};
        CHECK(pxchg_pack_fp16(table, 3, src, same, nullptr) == PXCHG_ERR_INVALID_ARG);
        // a persistent grid: n workgroups per compute unit (the stand-in device has 256 units)
        CHECK(pxchg_set_option(PXCHG_OPT_BLOCKS_PER_CU, 1) == PXCHG_OK);
        CHECK(pxchg_pack_fp16(table, 3, src, dst, nullptr) == PXCHG_OK && fake::last_grid.x == 249);
        CHECK(pxchg_easgd(table, a, c, 0.5f, nullptr) == PXCHG_OK && fake::last_grid.x == (unsigned)(2 * n_chunks));
        CHECK(pxchg_set_option(PXCHG_OPT_BLOCKS_PER_CU, 0) == PXCHG_OK);
        CHECK(pxchg_bufset_destroy(s2) == PXCHG_OK && pxchg_bufset_destroy(s3) == PXCHG_OK);
    }
    // a launch that fails is this call's PXCHG_ERR_RUNTIME; the next call is unaffected
    fake::fail_next_launch = true;
    CHECK(pxchg_easgd(table, a, c, 0.5f, nullptr) == PXCHG_ERR_RUNTIME);
    CHECK(pxchg_easgd(table, a, c, 0.5f, nullptr) == PXCHG_OK);
    // more than 8 workers in a round: one launch per group of 8
    {
        std::vector<Buffers *> bufs;
        std::vector<pxchg_bufset *> sets;
        for (int i = 0; i < 11; ++i) {
            bufs.push_back(new Buffers(counts, 4));
            pxchg_bufset *s = nullptr;
            CHECK(pxchg_bufset_create(table, PXCHG_F32, bufs.back()->data(), &s) == PXCHG_OK);
            sets.push_back(s);
        }
        fake::launches = 0;
        CHECK(pxchg_easgd_round(table, 11, sets.data(), c, 0.1f, nullptr) == PXCHG_OK && fake::launches == 2);
        sets.push_back(sets[3]);
        CHECK(pxchg_easgd_round(table, 12, sets.data(), c, 0.1f, nullptr) == PXCHG_ERR_INVALID_ARG);  // a worker twice
        sets.pop_back();
        for (auto *s : sets) CHECK(pxchg_bufset_destroy(s) == PXCHG_OK);
        for (auto *p : bufs) delete p;
    }

    // ---- the allocation-free diagnostics call: same two launches, no allocation, the array's address looked up
    // once per device (table creation did it), and a size limit of its own
    {
        const int mallocs = fake::mallocs, lookups = fake::symbol_lookups;
        CHECK(lookups == 1);
        fake::launches = 0;
        fake::grids.clear();
        CHECK(pxchg_buffer_stats_static(table, h, out, nullptr) == PXCHG_OK);
        CHECK(pxchg_buffer_stats_static(table, a, out, nullptr) == PXCHG_OK);
        CHECK(fake::launches == 4 && fake::grids[0].x == (unsigned)n_blocks && fake::grids[1].x == 1);
        CHECK(fake::mallocs == mallocs && fake::symbol_lookups == lookups);
        CHECK(pxchg_buffer_stats_static(table, h, nullptr, nullptr) == PXCHG_ERR_INVALID_ARG);
        CHECK(pxchg_buffer_stats_static(table, foreign, out, nullptr) == PXCHG_ERR_SHAPE_MISMATCH);
        // one chunk too many for the static array: refused before anything is launched; the regular call takes it
        const int64_t limit = (int64_t)PXCHG_STATS_STATIC_MAX_BLOCKS * PXCHG_STATS_BLOCK_CHUNKS;
        const int64_t big_counts[2] = {limit * 512, 1};
        pxchg_table *big = nullptr;
        CHECK(pxchg_table_create(2, big_counts, &big) == PXCHG_OK && pxchg_table_n_chunks(big) == limit + 1);
        CHECK(pxchg_set_option(PXCHG_OPT_CHECK_RANGES, 0) == PXCHG_OK);  // no buffers of that size here
        const void *anywhere[2] = {fa.ptrs[0], fa.ptrs[0]};
        pxchg_bufset *bs = nullptr;
        CHECK(pxchg_bufset_create(big, PXCHG_F16, anywhere, &bs) == PXCHG_OK);
        CHECK(pxchg_set_option(PXCHG_OPT_CHECK_RANGES, 1) == PXCHG_OK);
        fake::launches = 0;
        CHECK(pxchg_buffer_stats_static(big, bs, out, nullptr) == PXCHG_ERR_UNSUPPORTED && fake::launches == 0);
        CHECK(pxchg_buffer_stats(big, bs, out, nullptr) == PXCHG_OK && fake::launches == 2);
        pxchg_table *fits = nullptr;   // a view of exactly the limit fits
        CHECK(pxchg_table_view(big, 0, 1, &fits) == PXCHG_OK && pxchg_table_n_chunks(fits) == limit);
        CHECK(pxchg_buffer_stats_static(fits, bs, out, nullptr) == PXCHG_OK);
        CHECK(fake::grids.back().x == 1 && fake::grids[fake::grids.size() - 2].x == (unsigned)PXCHG_STATS_STATIC_MAX_BLOCKS);
        CHECK(pxchg_table_destroy(fits) == PXCHG_OK && pxchg_bufset_destroy(bs) == PXCHG_OK && pxchg_table_destroy(big) == PXCHG_OK);
    }

    // ---- wrong arguments with live handles
    {
        const pxchg_bufset *mixed[2] = {a, h};
        const pxchg_bufset *with_foreign[2] = {a, foreign};
        std::vector<const pxchg_bufset *> many(PXCHG_MAX_K + 1, a);
        CHECK(pxchg_reduce_avg(table, 2, mixed, c, PXCHG_AVG, nullptr) == PXCHG_ERR_SHAPE_MISMATCH);
        CHECK(pxchg_reduce_avg(table, 2, with_foreign, c, PXCHG_AVG, nullptr) == PXCHG_ERR_SHAPE_MISMATCH);
        CHECK(pxchg_reduce_avg(table, PXCHG_MAX_K + 1, many.data(), c, PXCHG_AVG, nullptr) == PXCHG_ERR_UNSUPPORTED);
        CHECK(pxchg_reduce_avg(table, 0, many.data(), c, PXCHG_AVG, nullptr) == PXCHG_ERR_UNSUPPORTED);
        CHECK(pxchg_reduce_avg(table, 2, mixed, c, 7, nullptr) == PXCHG_ERR_INVALID_ARG);
        CHECK(pxchg_reduce_avg(table, 2, nullptr, c, PXCHG_AVG, nullptr) == PXCHG_ERR_INVALID_ARG);
        CHECK(pxchg_sgd_momentum(table, a, a, b, 0.1f, 0.9f, 0.0f, nullptr) == PXCHG_ERR_INVALID_ARG);
        CHECK(pxchg_sgd_momentum(table, a, h, b, 0.1f, 0.9f, 0.0f, nullptr) == PXCHG_ERR_SHAPE_MISMATCH);
        CHECK(pxchg_easgd(table, a, a, 0.1f, nullptr) == PXCHG_ERR_INVALID_ARG);
        CHECK(pxchg_buffer_stats(table, h, nullptr, nullptr) == PXCHG_ERR_INVALID_ARG);
        CHECK(pxchg_buffer_stats(table, h, (pxchg_stats *)((char *)out + 4), nullptr) == PXCHG_ERR_INVALID_ARG);
        // a table handle where a set is expected, and the other way round
        CHECK(pxchg_easgd(table, (pxchg_bufset *)table, c, 0.1f, nullptr) == PXCHG_ERR_INVALID_ARG);
        CHECK(pxchg_easgd((pxchg_table *)a, a, c, 0.1f, nullptr) == PXCHG_ERR_INVALID_ARG);
        CHECK(pxchg_table_destroy((pxchg_table *)a) == PXCHG_ERR_INVALID_ARG);
        CHECK(pxchg_bufset_destroy((pxchg_bufset *)table) == PXCHG_ERR_INVALID_ARG);
        // the table's device is not the current one
        fake::current_device = 1;
        CHECK(pxchg_easgd(table, a, c, 0.1f, nullptr) == PXCHG_ERR_NO_DEVICE);
        pxchg_bufset *s = nullptr;
        CHECK(pxchg_bufset_create(table, PXCHG_F32, fa.data(), &s) == PXCHG_ERR_NO_DEVICE);
        fake::current_device = 0;
    }

    // ---- views: a handle of their own on the parent's sets; the parent cannot go first
    pxchg_table *view = nullptr, *view2 = nullptr;
    CHECK(pxchg_table_view(table, 2, 2, &view) == PXCHG_OK);
    CHECK(pxchg_table_view(table, 0, 1, &view2) == PXCHG_OK);
    CHECK(pxchg_table_n_chunks(view) == 2 + 79 && pxchg_table_total(view) == 513 + 40000);
    pxchg_table *vv = nullptr;
    CHECK(pxchg_table_view(view, 0, 1, &vv) == PXCHG_ERR_INVALID_ARG);                  // no views of views
    CHECK(pxchg_table_view(table, 3, 2, &vv) == PXCHG_ERR_INVALID_ARG);                 // runs past the end
    pxchg_bufset *on_view = nullptr;
    CHECK(pxchg_bufset_create(view, PXCHG_F32, fa.data(), &on_view) == PXCHG_ERR_INVALID_ARG);
    CHECK(pxchg_table_set_multipliers(view, nullptr, nullptr) == PXCHG_ERR_INVALID_ARG);
    CHECK(pxchg_table_set_option(view, PXCHG_OPT_CENTER_RESIDENT, 1) == PXCHG_ERR_INVALID_ARG);     // set it on the parent
    CHECK(pxchg_table_get_option(view, PXCHG_OPT_CENTER_RESIDENT) == PXCHG_TABLE_OPTION_INHERIT);   // reads the parent's
    fake::launches = 0;
    for (int rc : every_hot_call(view, a, b, c, h, out)) CHECK(rc == PXCHG_OK);
    CHECK(fake::launches == 11);
    CHECK(pxchg_easgd(view, a, c, 0.1f, nullptr) == PXCHG_OK && fake::last_grid.x == 2 * 81);
    CHECK(pxchg_easgd(view, foreign, c, 0.1f, nullptr) == PXCHG_ERR_SHAPE_MISMATCH);
    CHECK(pxchg_table_destroy(table) == PXCHG_ERR_IN_USE);                              // views and sets alive
    for (int rc : every_hot_call(view, a, b, c, h, out)) CHECK(rc == PXCHG_OK);         // nothing was torn down
    CHECK(pxchg_table_destroy(view) == PXCHG_OK);
    CHECK(pxchg_table_destroy(view) == PXCHG_ERR_INVALID_ARG);                          // twice
    for (int rc : every_hot_call(view, a, b, c, h, out)) CHECK(rc == PXCHG_ERR_INVALID_ARG);  // a destroyed view
    CHECK(pxchg_table_destroy(table) == PXCHG_ERR_IN_USE);                              // one view and the sets are left
    CHECK(pxchg_table_destroy(view2) == PXCHG_OK);
    CHECK(pxchg_table_destroy(table) == PXCHG_ERR_IN_USE);                              // the sets are left

    // ---- per-table options: the table's own setting overrides the process-wide one; a view follows its parent
    {
        CHECK(pxchg_table_get_option(table, PXCHG_OPT_CENTER_RESIDENT) == PXCHG_TABLE_OPTION_INHERIT);
        CHECK(pxchg_table_set_option(table, PXCHG_OPT_CENTER_RESIDENT, 1) == PXCHG_OK);
        CHECK(pxchg_table_get_option(table, PXCHG_OPT_CENTER_RESIDENT) == 1);
        CHECK(pxchg_table_get_option(other, PXCHG_OPT_CENTER_RESIDENT) == PXCHG_TABLE_OPTION_INHERIT);
        CHECK(pxchg_get_option(PXCHG_OPT_CENTER_RESIDENT) == 0);                    // the process-wide one is untouched
        CHECK(pxchg_easgd(table, a, c, 0.1f, nullptr) == PXCHG_OK);                // same launch shape either way
        CHECK(pxchg_table_set_option(table, PXCHG_OPT_CENTER_RESIDENT, 2) == PXCHG_ERR_INVALID_ARG);
        CHECK(pxchg_table_set_option(table, PXCHG_OPT_CENTER_RESIDENT, PXCHG_TABLE_OPTION_INHERIT) == PXCHG_OK);
        CHECK(pxchg_table_set_option(table, PXCHG_OPT_NONTEMPORAL, 0) == PXCHG_OK);
        CHECK(pxchg_table_get_option(table, PXCHG_OPT_NONTEMPORAL) == 0);
        CHECK(pxchg_table_set_option(table, PXCHG_OPT_NONTEMPORAL, 6) == PXCHG_ERR_INVALID_ARG);
        CHECK(pxchg_table_set_option(table, PXCHG_OPT_NONTEMPORAL, 4) ==
              (pxchg_get_option(PXCHG_OPT_ALL_POLICIES_BUILT) ? PXCHG_OK : PXCHG_ERR_UNSUPPORTED));
        CHECK(pxchg_table_set_option(table, PXCHG_OPT_NONTEMPORAL, PXCHG_TABLE_OPTION_INHERIT) == PXCHG_OK);
        CHECK(pxchg_table_set_option(table, PXCHG_OPT_CHUNK_ELEMS, 1024) == PXCHG_ERR_INVALID_ARG);   // not per table
        CHECK(pxchg_table_get_option(table, PXCHG_OPT_CHUNK_ELEMS) == -3);
        CHECK(pxchg_table_set_option(nullptr, PXCHG_OPT_NONTEMPORAL, 0) == PXCHG_ERR_INVALID_ARG);
        CHECK(pxchg_table_get_option((pxchg_table *)a, PXCHG_OPT_NONTEMPORAL) == -3);
    }

    // ---- multipliers (a set-up call that waits for the device)
    {
        std::vector<float> lr(nt, 1.0f), wd(nt, 0.0f);
        const int syncs = fake::synchronizes;
        CHECK(pxchg_table_set_multipliers(table, lr.data(), wd.data()) == PXCHG_OK && fake::synchronizes > syncs);
        CHECK(pxchg_sgd_momentum(table, h, a, b, 0.01f, 0.9f, 5e-4f, nullptr) == PXCHG_OK);
        CHECK(pxchg_table_set_multipliers(table, nullptr, nullptr) == PXCHG_OK);
    }

    // ---- destroyed sets: every call refuses them, also the second destroy
    CHECK(pxchg_bufset_destroy(h) == PXCHG_OK);
    CHECK(pxchg_bufset_destroy(h) == PXCHG_ERR_INVALID_ARG);
    {
        const std::vector<int> rcs = every_hot_call(table, a, b, c, h, out);
        // pack, unpack, update with h as gradient, fused reduce+update and the diagnostics use h
        CHECK(rcs[0] == PXCHG_ERR_INVALID_ARG && rcs[1] == PXCHG_ERR_INVALID_ARG && rcs[3] == PXCHG_ERR_INVALID_ARG);
        CHECK(rcs[6] == PXCHG_ERR_INVALID_ARG && rcs[7] == PXCHG_ERR_INVALID_ARG && rcs[8] == PXCHG_ERR_INVALID_ARG);
        CHECK(rcs[2] == PXCHG_OK && rcs[4] == PXCHG_OK && rcs[5] == PXCHG_OK);
    }
    CHECK(pxchg_bufset_destroy(a) == PXCHG_OK && pxchg_bufset_destroy(b) == PXCHG_OK);
    CHECK(pxchg_table_destroy(table) == PXCHG_ERR_IN_USE);                              // c is left
    CHECK(pxchg_bufset_destroy(c) == PXCHG_OK);

    // ---- the destroyed table: every call refuses it, also with sets of another, live table
    CHECK(pxchg_table_destroy(table) == PXCHG_OK);
    CHECK(pxchg_table_destroy(table) == PXCHG_ERR_INVALID_ARG);
    CHECK(pxchg_table_total(table) == -1 && pxchg_table_n_chunks(table) == -1 && pxchg_table_n_tensors(table) == -1);
    fake::launches = 0;
    for (int rc : every_hot_call(table, foreign, foreign, foreign, foreign, out)) CHECK(rc == PXCHG_ERR_INVALID_ARG);
    for (int rc : every_hot_call(table, a, b, c, h, out)) CHECK(rc == PXCHG_ERR_INVALID_ARG);
    CHECK(fake::launches == 0);
    CHECK(pxchg_table_view(table, 0, 1, &vv) == PXCHG_ERR_INVALID_ARG);
    CHECK(pxchg_bufset_create(table, PXCHG_F32, fa.data(), &on_view) == PXCHG_ERR_INVALID_ARG);
    CHECK(pxchg_table_set_multipliers(table, nullptr, nullptr) == PXCHG_ERR_INVALID_ARG);

    // ---- a new table may land on the destroyed one's address; the old table's sets are gone, and a set of
    // another table stays that table's
    pxchg_table *fresh = nullptr;
    CHECK(pxchg_table_create(nt, counts.data(), &fresh) == PXCHG_OK);
    CHECK(pxchg_easgd(fresh, foreign, foreign, 0.1f, nullptr) != PXCHG_OK);
    pxchg_bufset *fx = nullptr, *fy = nullptr;
    CHECK(pxchg_bufset_create(fresh, PXCHG_F32, fa.data(), &fx) == PXCHG_OK);
    CHECK(pxchg_bufset_create(fresh, PXCHG_F32, fb.data(), &fy) == PXCHG_OK);
    CHECK(pxchg_easgd(fresh, fx, fy, 0.1f, nullptr) == PXCHG_OK);
    CHECK(pxchg_easgd(fresh, fx, foreign, 0.1f, nullptr) == PXCHG_ERR_SHAPE_MISMATCH);
    CHECK(pxchg_bufset_destroy(fx) == PXCHG_OK && pxchg_bufset_destroy(fy) == PXCHG_OK);
    CHECK(pxchg_table_destroy(fresh) == PXCHG_OK);

    // ---- a table of empty tensors: nothing to launch, the diagnostics still write their zeros
    {
        const int64_t zeros[2] = {0, 0};
        pxchg_table *empty = nullptr;
        CHECK(pxchg_table_create(2, zeros, &empty) == PXCHG_OK && pxchg_table_n_chunks(empty) == 0);
        const void *none[2] = {nullptr, nullptr};
        pxchg_bufset *e1 = nullptr, *e2 = nullptr, *eh = nullptr;
        CHECK(pxchg_bufset_create(empty, PXCHG_F32, none, &e1) == PXCHG_OK);
        CHECK(pxchg_bufset_create(empty, PXCHG_F32, none, &e2) == PXCHG_OK);
        CHECK(pxchg_bufset_create(empty, PXCHG_F16, none, &eh) == PXCHG_OK);
        fake::launches = 0;
        CHECK(pxchg_easgd(empty, e1, e2, 0.1f, nullptr) == PXCHG_OK && fake::launches == 0);
        CHECK(pxchg_buffer_stats(empty, eh, out, nullptr) == PXCHG_OK && fake::launches == 1 && fake::last_grid.x == 1);
        CHECK(pxchg_bufset_destroy(e1) == PXCHG_OK && pxchg_bufset_destroy(e2) == PXCHG_OK && pxchg_bufset_destroy(eh) == PXCHG_OK);
        CHECK(pxchg_table_destroy(empty) == PXCHG_OK);
    }

    CHECK(pxchg_bufset_destroy(foreign) == PXCHG_OK);
    CHECK(pxchg_table_destroy(other) == PXCHG_OK);
    CHECK(hipFree(out) == hipSuccess);
    return 0;
}

// Several threads use one table while others create and destroy tables, views and sets of their own, and one
// keeps trying to destroy the shared table: calls on live handles succeed, the shared table stays (it has sets),
// and a handle that another thread has destroyed is refused, not read.  Run under ThreadSanitizer as well.
int threads_share_handles() {
    const std::vector<int64_t> counts = {5000, 513, 0, 70001};
    pxchg_table *shared = nullptr;
    CHECK(pxchg_table_create((int)counts.size(), counts.data(), &shared) == PXCHG_OK);
    Buffers fa(counts, 4), fb(counts, 4);
    pxchg_bufset *a = nullptr, *b = nullptr;
    CHECK(pxchg_bufset_create(shared, PXCHG_F32, fa.data(), &a) == PXCHG_OK);
    CHECK(pxchg_bufset_create(shared, PXCHG_F32, fb.data(), &b) == PXCHG_OK);
    std::atomic<int> failures{0};
    std::atomic<pxchg_bufset *> passed_around{nullptr};
    auto user = [&](int id) {
        for (int i = 0; i < 300; ++i) {
            if (pxchg_easgd(shared, a, b, 0.1f, nullptr) != PXCHG_OK) ++failures;
            pxchg_table *view = nullptr;
            if (pxchg_table_view(shared, id % 2, 2, &view) != PXCHG_OK) ++failures;
            if (pxchg_easgd(view, a, b, 0.1f, nullptr) != PXCHG_OK) ++failures;
            if (pxchg_table_destroy(view) != PXCHG_OK) ++failures;
            if (pxchg_table_total(shared) != 5000 + 513 + 70001) ++failures;
        }
    };
    auto maker = [&]() {
        for (int i = 0; i < 100; ++i) {
            pxchg_table *t = nullptr;
            pxchg_bufset *x = nullptr, *y = nullptr;
            if (pxchg_table_create((int)counts.size(), counts.data(), &t) != PXCHG_OK) ++failures;
            if (pxchg_bufset_create(t, PXCHG_F32, fa.data(), &x) != PXCHG_OK) ++failures;
            if (pxchg_bufset_create(t, PXCHG_F32, fb.data(), &y) != PXCHG_OK) ++failures;
            if (pxchg_easgd(t, x, y, 0.1f, nullptr) != PXCHG_OK) ++failures;
            if (pxchg_easgd(shared, x, y, 0.1f, nullptr) != PXCHG_ERR_SHAPE_MISMATCH) ++failures;   // another table's sets
            if (pxchg_table_destroy(t) != PXCHG_ERR_IN_USE) ++failures;
            // hand one set to the breaker thread, which may destroy it at any moment: whoever comes second is refused
            pxchg_bufset *expected = nullptr;
            const bool handed = passed_around.compare_exchange_strong(expected, y);
            if (pxchg_bufset_destroy(x) != PXCHG_OK) ++failures;
            if (handed) {
                int rc;
                while ((rc = pxchg_table_destroy(t)) == PXCHG_ERR_IN_USE) std::this_thread::yield();   // until y is gone
                if (rc != PXCHG_OK) ++failures;
            } else {
                if (pxchg_bufset_destroy(y) != PXCHG_OK) ++failures;
                if (pxchg_table_destroy(t) != PXCHG_OK) ++failures;
            }
        }
    };
    std::atomic<bool> stop{false};
    auto breaker = [&]() {
        while (!stop) {
            if (pxchg_table_destroy(shared) != PXCHG_ERR_IN_USE) ++failures;     // it has sets: never goes
            pxchg_bufset *y = passed_around.exchange(nullptr);
            if (y) {
                if (pxchg_bufset_destroy(y) != PXCHG_OK) ++failures;
                if (pxchg_bufset_destroy(y) != PXCHG_ERR_INVALID_ARG) ++failures;   // twice
                if (pxchg_easgd(shared, y, b, 0.1f, nullptr) != PXCHG_ERR_INVALID_ARG) ++failures;
            }
            std::this_thread::yield();
        }
    };
    std::vector<std::thread> pool;
    for (int id = 0; id < 3; ++id) pool.emplace_back(user, id);
    pool.emplace_back(maker);
    pool.emplace_back(maker);
    std::thread br(breaker);
    for (auto &t : pool) t.join();
    stop = true;
    br.join();
    if (pxchg_bufset *left = passed_around.exchange(nullptr)) CHECK(pxchg_bufset_destroy(left) == PXCHG_OK);
    CHECK(failures == 0);
    CHECK(pxchg_bufset_destroy(a) == PXCHG_OK && pxchg_bufset_destroy(b) == PXCHG_OK);
    CHECK(pxchg_table_destroy(shared) == PXCHG_OK);
    return 0;
}


// Every way a set-up call can run out of memory half-way: the n-th host allocation throws, or the n-th device
// allocation fails, for n = 0, 1, ... until the call gets through.  Each failure must come back as a status (no
// exception leaves the library), hand out no handle, return every device allocation made so far, and leave the
// counts of live views and sets as they were (the objects can be destroyed afterwards), with as many host blocks
// alive as before.
int planted_failures = 0;  // failures met by the last exhaust()
template <typename Call>
int exhaust(const char *what, long &countdown, Call call) {
    planted_failures = 0;
    const size_t device_before = fake::allocations.size();
    const long host_before = fake::live_host_blocks;
    for (long n = 0;; ++n) {
        if (n > 200) {
            std::printf("%s: still failing after 200 allocations\n", what);
            return 1;
        }
        countdown = n;
        void *handle = (void *)0x1;
        const int rc = call(&handle);
        const bool fired = countdown < 0;  // the planted failure was reached
        countdown = -1;
        if (rc == PXCHG_OK) {
            CHECK(handle != nullptr && handle != (void *)0x1);
            CHECK(!fired);  // a call that got through met no failure
            return 0;
        }
        CHECK(fired);
        ++planted_failures;
        CHECK(rc == PXCHG_ERR_RUNTIME);
        CHECK(handle == nullptr);
        CHECK(fake::allocations.size() == device_before);
        CHECK(fake::live_host_blocks == host_before);  // and every host block
    }
}

int memory_runs_out() {
    const std::vector<int64_t> counts = {1000, 0, 513, 7, 4096};
    Buffers f32(counts, 4);
    for (int kind = kFirstFailureKind; kind < 2; ++kind) {
        long &countdown = kind == 0 ? fake::new_countdown : fake::malloc_countdown;
        pxchg_table *table = nullptr, *view = nullptr;
        pxchg_bufset *set = nullptr;
        if (exhaust("table_create", countdown, [&](void **h) {
                const int rc = pxchg_table_create((int)counts.size(), counts.data(), (pxchg_table **)h);
                table = (pxchg_table *)*h;
                return rc;
            }))
            return 1;
        // the rehearsal is not vacuous: the object, its vectors and its registry entry on the host side; the
        // chunk list and the partial results on the device side
        CHECK(planted_failures >= (kind == 0 ? 3 : 2));
        if (exhaust("table_view", countdown, [&](void **h) {
                const int rc = pxchg_table_view(table, 1, 3, (pxchg_table **)h);
                view = (pxchg_table *)*h;
                return rc;
            }))
            return 1;
        if (exhaust("bufset_create", countdown, [&](void **h) {
                const int rc = pxchg_bufset_create(table, PXCHG_F32, f32.data(), (pxchg_bufset **)h);
                set = (pxchg_bufset *)*h;
                return rc;
            }))
            return 1;
        CHECK(planted_failures >= (kind == 0 ? 3 : 1));
        // multipliers: a failure leaves the table usable and without multipliers or with the old ones
        std::vector<float> ones(counts.size(), 1.0f);
        for (long n = 0;; ++n) {
            CHECK(n <= 200);
            countdown = n;
            const int rc = pxchg_table_set_multipliers(table, ones.data(), nullptr);
            const bool fired = countdown < 0;
            countdown = -1;
            if (rc == PXCHG_OK) break;
            CHECK(fired && rc == PXCHG_ERR_RUNTIME);
        }
        {   // what was built works: a launch through the view with the set
            const int before = fake::launches;
            pxchg_bufset *one[1] = {set};
            pxchg_bufset *other = nullptr;
            Buffers out(counts, 4);
            CHECK(pxchg_bufset_create(table, PXCHG_F32, out.data(), &other) == PXCHG_OK);
            CHECK(pxchg_reduce_avg(view, 1, one, other, PXCHG_AVG, nullptr) == PXCHG_OK);
            CHECK(fake::launches == before + 1);
            CHECK(pxchg_bufset_destroy(other) == PXCHG_OK);
        }
        // exactly one view and one set are alive: the failed attempts left nothing behind
        CHECK(pxchg_table_destroy(table) == PXCHG_ERR_IN_USE);
        CHECK(pxchg_table_destroy(view) == PXCHG_OK);
        CHECK(pxchg_table_destroy(table) == PXCHG_ERR_IN_USE);
        CHECK(pxchg_bufset_destroy(set) == PXCHG_OK);
        CHECK(pxchg_table_destroy(table) == PXCHG_OK);
    }
    return 0;
}

}  // namespace

int main(int argc, char **argv) {
    const bool threads_only = argc > 1 && std::strcmp(argv[1], "threads") == 0;
    if (!threads_only) {
        if (options_and_planning()) return 1;
        if (lifetime_and_launches()) return 1;
        if (memory_runs_out()) return 1;
    }
    if (threads_share_handles()) return 1;
    if (!fake::allocations.empty()) {  // every device allocation of the library was returned
        std::printf("%zu device allocations were never freed\n", fake::allocations.size());
        return 1;
    }
    std::printf("ok\n");
    return 0;
}
