/* Host-only driver: runs every oracle routine on small buffers whose sizes are
 * not multiples of anything, so that AddressSanitizer and UBSan see any read or
 * write past an end, misaligned access or undefined shift.  Built and run by
 * tests/test_oracle_sanitizers.py; prints "ok" and exits 0 when clean. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../oracle/pxchg_oracle.c"

int main(void)
{
    enum { N = 1237, K = 5 };
    /* every binary16 pattern through both conversions, every exponent of binary32 */
    for (uint32_t h = 0; h < 65536u; ++h) {
        uint32_t f = oracle_f16_to_f32_bits((uint16_t)h);
        uint16_t back = oracle_f32_to_f16_bits(f);
        if ((h & 0x7c00u) != 0x7c00u || (h & 0x3ffu) == 0) {
            if (back != h) { printf("round trip failed at %x\n", h); return 1; }
        }
    }
    for (uint32_t e = 0; e < 256; ++e)
        for (uint32_t m = 0; m < 8; ++m) {
            (void)oracle_f32_to_f16_bits((e << 23) | (m * 0x124925u & 0x7fffffu));
            (void)oracle_f32_to_f16_bits(0x80000000u | (e << 23) | (0x7fffffu - m));
        }
    float *g[K];
    uint16_t *h[K];
    const void *cf[K], *ch[K];
    for (int i = 0; i < K; ++i) {
        g[i] = malloc(N * sizeof(float));
        h[i] = malloc(N * sizeof(uint16_t));
        for (int j = 0; j < N; ++j) g[i][j] = (float)((j * 37 + i * 11) % 201 - 100) * 1e-3f;
        oracle_pack_fp16(g[i], h[i], N);
        cf[i] = g[i];
        ch[i] = h[i];
    }
    float *w = malloc(N * sizeof(float)), *v = malloc(N * sizeof(float)), *a32 = malloc(N * sizeof(float));
    uint16_t *a16 = malloc(N * sizeof(uint16_t));
    for (int j = 0; j < N; ++j) { w[j] = 0.01f * (float)(j % 17); v[j] = 0.0f; }
    oracle_unpack_fp16(h[0], a32, N);
    if (oracle_reduce_avg(K, cf, ORACLE_F32, a32, ORACLE_F32, ORACLE_AVG, N)) return 1;
    if (oracle_reduce_avg(K, cf, ORACLE_F32, a16, ORACLE_F16, ORACLE_SUM, N)) return 1;
    if (oracle_reduce_avg(K, ch, ORACLE_F16, a32, ORACLE_F32, ORACLE_SUM, N)) return 1;
    if (oracle_reduce_avg(K, ch, ORACLE_F16, a16, ORACLE_F16, ORACLE_AVG, N)) return 1;
    if (oracle_reduce_avg(1, ch, ORACLE_F16, a16, ORACLE_F16, ORACLE_AVG, 0)) return 1;
    if (!oracle_reduce_avg(0, ch, ORACLE_F16, a16, ORACLE_F16, ORACLE_AVG, N)) return 1;   /* must reject */
    if (oracle_sgd_momentum(a16, ORACLE_F16, w, v, 0.01f, 0.9f, 5e-4f, N)) return 1;
    if (oracle_sgd_momentum(a32, ORACLE_F32, w, v, 0.01f, 0.9f, 0.0f, N)) return 1;
    if (oracle_easgd(w, v, 0.0625f, N)) return 1;
    uint64_t bad;
    float mx;
    double ss;
    if (oracle_stats(a16, ORACLE_F16, N, &bad, &mx, &ss)) return 1;
    if (oracle_stats(w, ORACLE_F32, N, &bad, &mx, &ss)) return 1;
    /* the tree-ordered diagnostics: ragged tensors incl. empty ones, blocks that end mid-list, every parameter odd */
    {
        const void *ts16[4] = {a16, NULL, h[1], h[2]}, *ts32[3] = {w, a32, g[0]};
        const int64_t c16[4] = {N, 0, 700, 1}, c32[3] = {N, 513, N - 3};
        double ordered;
        if (oracle_stats_ordered(4, ts16, c16, ORACLE_F16, 512, 4, 32, 1024, &bad, &mx, &ordered)) return 1;
        if (oracle_stats_ordered(4, ts16, c16, ORACLE_F16, 7, 3, 5, 64, &bad, &mx, &ordered)) return 1;
        if (oracle_stats_ordered(3, ts32, c32, ORACLE_F32, 512, 1, 1, 128, &bad, &mx, &ordered)) return 1;
        if (oracle_stats_ordered(3, ts32, c32, ORACLE_F32, 100000, 16, 256, 1024, &bad, &mx, &ordered)) return 1;
        const int64_t none[2] = {0, 0};
        if (oracle_stats_ordered(2, ts16, none, ORACLE_F16, 512, 4, 32, 1024, &bad, &mx, &ordered) || ordered != 0.0) return 1;
        if (!oracle_stats_ordered(3, ts32, c32, ORACLE_F32, 512, 4, 32, 100, &bad, &mx, &ordered)) return 1;   /* must reject */
    }
    for (int i = 0; i < K; ++i) { free(g[i]); free(h[i]); }
    free(w); free(v); free(a32); free(a16);
    printf("ok\n");
    return 0;
}
