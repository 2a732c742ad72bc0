/* A plain C program (no Python, no torch) that drives the exchange through the C ABI of libpxchg.so on GPU 0 and
 * compares every result, bit for bit, with the CPU oracle compiled into this same program.  It shows that the
 * boundary is the library itself: device memory comes from hipMalloc, and the handles, calls and status codes
 * are the ones pxchg.h declares.  Built by __graft_entry__.build() with gcc; run by tests/test_gpu_c_abi.py.
 * Prints one line per step and "ok" at the end; exits non-zero at the first mismatch or error. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <hip/hip_runtime_api.h>

#include "pxchg.h"
#include "../oracle/pxchg_oracle.c"

#define K 3
#define NT 6
static const int64_t counts[NT] = {1, 63, 1237, 70001, 0, 4096};

#define HIP_OK(call)                                                                      \
    do {                                                                                  \
        hipError_t e_ = (call);                                                           \
        if (e_ != hipSuccess) {                                                           \
            printf("%s failed: %s (line %d)\n", #call, hipGetErrorString(e_), __LINE__);  \
            return 1;                                                                     \
        }                                                                                 \
    } while (0)
#define PX_OK(call)                                                                       \
    do {                                                                                  \
        int s_ = (call);                                                                  \
        if (s_ != PXCHG_OK) {                                                             \
            printf("%s returned %d: %s (line %d)\n", #call, s_, pxchg_status_string(s_), __LINE__); \
            return 1;                                                                     \
        }                                                                                 \
    } while (0)

/* A small counter-based generator, only to have reproducible inputs: values in (-0.04, 0.04). */
static float draw(uint64_t role, uint64_t tensor, uint64_t j)
{
    uint64_t z = (role * 0x9e3779b97f4a7c15ull) ^ (tensor * 0xbf58476d1ce4e5b9ull) ^ (j + 0x94d049bb133111ebull);
    z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
    z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
    z ^= z >> 31;
    return ((float)(z >> 40) / 16777216.0f - 0.5f) * 0.08f;
}

/* One buffer of the exchange: a host copy per tensor, a device copy per tensor (separate allocations), and the
 * library's handle for the device side. */
typedef struct {
    int es;                 /* element size: 4 or 2 */
    void *host[NT];
    void *dev[NT];
    pxchg_bufset *set;
} buffer;

static int buffer_make(buffer *b, const pxchg_table *table, int dtype, uint64_t role, int fill)
{
    b->es = dtype == PXCHG_F32 ? 4 : 2;
    for (int t = 0; t < NT; ++t) {
        size_t bytes = (size_t)counts[t] * b->es;
        b->host[t] = calloc(bytes ? bytes : 1, 1);
        b->dev[t] = NULL;
        if (fill && dtype == PXCHG_F32)
            for (int64_t j = 0; j < counts[t]; ++j) ((float *)b->host[t])[j] = draw(role, (uint64_t)t, (uint64_t)j);
        if (bytes) {
            HIP_OK(hipMalloc(&b->dev[t], bytes));
            HIP_OK(hipMemcpy(b->dev[t], b->host[t], bytes, hipMemcpyHostToDevice));
        }
    }
    PX_OK(pxchg_bufset_create(table, dtype, (const void *const *)b->dev, &b->set));
    return 0;
}

/* Device contents against the host copy (which the oracle has advanced), bit for bit. */
static int buffer_same(const buffer *b, const char *what)
{
    for (int t = 0; t < NT; ++t) {
        size_t bytes = (size_t)counts[t] * b->es;
        if (!bytes) continue;
        void *back = malloc(bytes);
        HIP_OK(hipMemcpy(back, b->dev[t], bytes, hipMemcpyDeviceToHost));
        if (memcmp(back, b->host[t], bytes) != 0) {
            size_t at = 0;
            while (((unsigned char *)back)[at] == ((unsigned char *)b->host[t])[at]) ++at;
            printf("%s: tensor %d differs from the oracle at element %zu\n", what, t, at / b->es);
            free(back);
            return 1;
        }
        free(back);
    }
    printf("%s: identical to the oracle\n", what);
    return 0;
}

static int buffer_free(buffer *b)
{
    PX_OK(pxchg_bufset_destroy(b->set));
    for (int t = 0; t < NT; ++t) {
        free(b->host[t]);
        if (b->dev[t]) HIP_OK(hipFree(b->dev[t]));
    }
    return 0;
}

int main(void)
{
    int n_dev = 0;
    HIP_OK(hipGetDeviceCount(&n_dev));
    if (n_dev < 1) {
        printf("no GPU\n");
        return 2;
    }
    HIP_OK(hipSetDevice(0));
    hipStream_t stream;
    HIP_OK(hipStreamCreate(&stream));

    pxchg_table *table = NULL;
    PX_OK(pxchg_table_create(NT, counts, &table));

    static buffer g[K], h[K], x[K], mean, w, v, c;
    const pxchg_bufset *g_sets[K], *h_sets_c[K];
    pxchg_bufset *h_sets[K], *x_sets[K];
    for (int i = 0; i < K; ++i) {
        if (buffer_make(&g[i], table, PXCHG_F32, 10 + (uint64_t)i, 1)) return 1;
        if (buffer_make(&h[i], table, PXCHG_F16, 0, 0)) return 1;
        if (buffer_make(&x[i], table, PXCHG_F32, 20 + (uint64_t)i, 1)) return 1;
        g_sets[i] = g[i].set;
        h_sets[i] = h[i].set;
        h_sets_c[i] = h[i].set;
        x_sets[i] = x[i].set;
    }
    if (buffer_make(&mean, table, PXCHG_F16, 0, 0) || buffer_make(&w, table, PXCHG_F32, 30, 1) ||
        buffer_make(&v, table, PXCHG_F32, 0, 0) || buffer_make(&c, table, PXCHG_F32, 31, 1))
        return 1;

    const float lr = 0.01f, mu = 0.9f, wd = 5e-4f, alpha = 0.125f;

    /* two steps of pack -> reduce+average (binary16 out) -> momentum update, then a round of elastic meetings */
    for (int step = 0; step < 2; ++step) {
        PX_OK(pxchg_pack_fp16(table, K, g_sets, h_sets, stream));
        PX_OK(pxchg_reduce_avg(table, K, h_sets_c, mean.set, PXCHG_AVG, stream));
        PX_OK(pxchg_sgd_momentum(table, mean.set, w.set, v.set, lr, mu, wd, stream));
        for (int t = 0; t < NT; ++t) {
            const void *contrib[K];
            for (int i = 0; i < K; ++i) {
                oracle_pack_fp16((const float *)g[i].host[t], (uint16_t *)h[i].host[t], counts[t]);
                contrib[i] = h[i].host[t];
            }
            if (oracle_reduce_avg(K, contrib, ORACLE_F16, mean.host[t], ORACLE_F16, ORACLE_AVG, counts[t])) return 1;
            if (oracle_sgd_momentum(mean.host[t], ORACLE_F16, (float *)w.host[t], (float *)v.host[t], lr, mu, wd,
                                    counts[t]))
                return 1;
        }
    }
    PX_OK(pxchg_easgd_round(table, K, x_sets, c.set, alpha, stream));
    PX_OK(pxchg_easgd(table, x[1].set, c.set, alpha, stream));
    for (int t = 0; t < NT; ++t) {
        for (int i = 0; i < K; ++i)
            if (oracle_easgd((float *)x[i].host[t], (float *)c.host[t], alpha, counts[t])) return 1;
        if (oracle_easgd((float *)x[1].host[t], (float *)c.host[t], alpha, counts[t])) return 1;
    }
    /* one more meeting of worker 0, on tensors 2 and 3 only, through a view of the table */
    pxchg_table *view = NULL;
    PX_OK(pxchg_table_view(table, 2, 2, &view));
    if (pxchg_table_total(view) != counts[2] + counts[3] || pxchg_table_n_tensors(view) != 2) {
        printf("the view reports the wrong size\n");
        return 1;
    }
    PX_OK(pxchg_easgd(view, x[0].set, c.set, alpha, stream));
    for (int t = 2; t < 4; ++t)
        if (oracle_easgd((float *)x[0].host[t], (float *)c.host[t], alpha, counts[t])) return 1;
    HIP_OK(hipStreamSynchronize(stream));
    PX_OK(pxchg_table_destroy(view));

    int bad = 0;
    for (int i = 0; i < K; ++i) bad |= buffer_same(&h[i], "packed gradient");
    bad |= buffer_same(&mean, "mean");
    bad |= buffer_same(&w, "parameters");
    bad |= buffer_same(&v, "velocity");
    for (int i = 0; i < K; ++i) bad |= buffer_same(&x[i], "worker copy");
    bad |= buffer_same(&c, "center");

    /* error paths through the same boundary: a set of the wrong type, too many workers */
    if (pxchg_sgd_momentum(table, mean.set, mean.set, v.set, lr, mu, wd, stream) != PXCHG_ERR_SHAPE_MISMATCH) {
        printf("a binary16 parameter set was not rejected\n");
        bad = 1;
    }
    if (pxchg_reduce_avg(table, PXCHG_MAX_K + 1, h_sets_c, mean.set, PXCHG_AVG, stream) != PXCHG_ERR_UNSUPPORTED) {
        printf("k above the maximum was not rejected\n");
        bad = 1;
    }

    /* lifetime: a table with live buffer sets refuses to go, and stays usable */
    if (pxchg_table_destroy(table) != PXCHG_ERR_IN_USE) {
        printf("a table with live buffer sets was destroyed\n");
        return 1;
    }
    if (pxchg_table_total(table) < 0) {
        printf("the table did not survive the refused destroy\n");
        bad = 1;
    }

    for (int i = 0; i < K; ++i)
        if (buffer_free(&g[i]) || buffer_free(&h[i]) || buffer_free(&x[i])) return 1;
    if (buffer_free(&mean) || buffer_free(&w) || buffer_free(&v) || buffer_free(&c)) return 1;
    PX_OK(pxchg_table_destroy(table));
    if (pxchg_table_destroy(table) != PXCHG_ERR_INVALID_ARG || pxchg_table_total(table) != -1) {
        printf("a destroyed table was not rejected\n");
        bad = 1;
    }
    HIP_OK(hipStreamDestroy(stream));
    if (bad) return 1;
    printf("ok\n");
    return 0;
}
