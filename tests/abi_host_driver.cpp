// Host-only driver for the library's set-up code (options, chunk planning, handle validation, error paths
// that need no GPU), built with AddressSanitizer and UBSan on the host side by tests/test_abi_sanitizers.py.
// Prints "ok" and exits 0 when every check holds and the sanitizers saw nothing.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "pxchg.h"

#define CHECK(cond)                                                   \
    do {                                                              \
        if (!(cond)) {                                                \
            std::printf("check failed, line %d: %s\n", __LINE__, #cond); \
            return 1;                                                 \
        }                                                             \
    } while (0)

int main() {
    for (int s = -2; s < 12; ++s) CHECK(pxchg_status_string(s) != nullptr && std::strlen(pxchg_status_string(s)) > 0);
    CHECK(pxchg_version() >= 100);

    // options: defaults, limits, restore
    CHECK(pxchg_get_option(PXCHG_OPT_CHUNK_ELEMS) == 512);
    CHECK(pxchg_set_option(PXCHG_OPT_CHUNK_ELEMS, 500) == PXCHG_ERR_INVALID_ARG);
    CHECK(pxchg_set_option(PXCHG_OPT_CHUNK_ELEMS, 0) == PXCHG_ERR_INVALID_ARG);
    CHECK(pxchg_set_option(PXCHG_OPT_CHUNK_ELEMS, (int64_t)1 << 40) == PXCHG_ERR_INVALID_ARG);
    CHECK(pxchg_set_option(PXCHG_OPT_CHUNK_ELEMS, 2048) == PXCHG_OK && pxchg_get_option(PXCHG_OPT_CHUNK_ELEMS) == 2048);
    CHECK(pxchg_set_option(PXCHG_OPT_CHUNK_ELEMS, 512) == PXCHG_OK);
    CHECK(pxchg_set_option(PXCHG_OPT_NONTEMPORAL, 6) == PXCHG_ERR_INVALID_ARG);
    CHECK(pxchg_set_option(PXCHG_OPT_NONTEMPORAL, -2) == PXCHG_ERR_INVALID_ARG);
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

    // tables and buffer sets: argument errors come before any use of a device
    pxchg_table *table = (pxchg_table *)0x1;
    CHECK(pxchg_table_create(0, counts, &table) == PXCHG_ERR_INVALID_ARG && table == nullptr);
    CHECK(pxchg_table_create(nt, nullptr, &table) == PXCHG_ERR_INVALID_ARG);
    CHECK(pxchg_table_create(nt, counts, nullptr) == PXCHG_ERR_INVALID_ARG);
    CHECK(pxchg_table_create(2, negative, &table) == PXCHG_ERR_INVALID_ARG);
    const int64_t huge[] = {(int64_t)1 << 41};
    CHECK(pxchg_table_create(1, huge, &table) == PXCHG_ERR_UNSUPPORTED);
    const int64_t many_chunks[] = {((int64_t)1 << 24) * 512 + 1};
    CHECK(pxchg_table_create(1, many_chunks, &table) == PXCHG_ERR_UNSUPPORTED);
    const int rc = pxchg_table_create(nt, counts, &table);
    CHECK(rc == PXCHG_OK || rc == PXCHG_ERR_NO_DEVICE || rc == PXCHG_ERR_RUNTIME);
    if (rc == PXCHG_OK) {
        CHECK(pxchg_table_total(table) == 1 + 511 + 512 + 513 + 1237 + 4096);
        CHECK(pxchg_table_n_tensors(table) == nt && pxchg_table_n_chunks(table) == n);
        CHECK(pxchg_table_destroy(table) == PXCHG_OK);
    } else {
        CHECK(table == nullptr);
    }
    CHECK(pxchg_table_destroy(nullptr) == PXCHG_OK && pxchg_bufset_destroy(nullptr) == PXCHG_OK);
    CHECK(pxchg_table_total(nullptr) == -1 && pxchg_table_n_tensors(nullptr) == -1 && pxchg_table_n_chunks(nullptr) == -1);

    // a block of memory that is not a handle must be rejected by every call that takes one
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
    std::printf("ok\n");
    return 0;
}
