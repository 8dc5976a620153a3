/* Runs the CPU oracle over a spread of layer tables under AddressSanitizer / UBSan (host only).
 * Built and run by tests/test_sanitizers.py; exit status 0 means no report. */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "adacomp_oracle.h"

static unsigned long long lcg = 88172645463325252ull;
static float rnd(void)
{
    lcg = lcg * 6364136223846793005ull + 1442695040888963407ull;
    return (float)((double)(lcg >> 11) / 9007199254740992.0 - 0.5);
}

int main(void)
{
    static const struct { unsigned n, T; } shapes[] = {
        {1, 1}, {3, 1}, {1003, 1}, {4099, 2}, {10001, 3}, {12345, 7}, {5013, 50}, {64 * 70 + 5, 64},
        {65 * 70 + 5, 65}, {500 * 31 + 216, 500}, {3 * 4097 + 1, 4097}, {16384 * 2 + 5, 16384}, {5, 16384}};
    const unsigned n_shapes = sizeof shapes / sizeof shapes[0];
    adacomp_oracle_layer_t layers[16];
    unsigned long long off = 0;
    for (unsigned l = 0; l < n_shapes; ++l) {
        layers[l].elem_offset = off; layers[l].n_elems = shapes[l].n; layers[l].L_T = shapes[l].T; layers[l].reserved = 0;
        off += (shapes[l].n + 3u) / 4u * 4u;
    }
    const size_t n_total = (size_t)off;
    const size_t bound = adacomp_oracle_packet_bound(layers, n_shapes);
    if (!bound) return 2;
    enum { K = 5 };
    float *grad = malloc(n_total * 4), *residue[K], *dense = malloc(n_total * 4);
    float *w = calloc(n_total, 4), *s1 = calloc(n_total, 4), *s2 = calloc(n_total, 4);
    void *packet[K];
    unsigned long long checksum = 0;
    for (int k = 0; k < K; ++k) { residue[k] = calloc(n_total, 4); packet[k] = malloc(bound); }
    for (int step = 0; step < 4; ++step) {
        for (int k = 0; k < K; ++k) {
            for (size_t i = 0; i < n_total; ++i) grad[i] = (step == 2 && i % 3 == 0) ? 0.f : rnd() * (k + 1);
            int rule = (step + k) % 3;
            float factor = 1.0f + 0.5f * (float)((step + k) % 5);
            /* learn the size on a copy; one byte less must be refused and leave the residue alone;
             * the exact size must work */
            float *r2 = malloc(n_total * 4);
            memcpy(r2, residue[k], n_total * 4);
            long long bytes = adacomp_oracle_compress(layers, n_shapes, grad, r2, packet[k], bound, rule, factor);
            if (bytes <= 0 || (size_t)bytes > bound) return 3;
            memcpy(r2, residue[k], n_total * 4);
            void *tight = malloc((size_t)bytes);
            long long again = adacomp_oracle_compress(layers, n_shapes, grad, r2, tight, (size_t)bytes - 1, rule, factor);
            if (again != -4 || memcmp(r2, residue[k], n_total * 4) != 0) return 4;
            again = adacomp_oracle_compress(layers, n_shapes, grad, residue[k], tight, (size_t)bytes, rule, factor);
            if (again != bytes || memcmp(tight, packet[k], (size_t)bytes) != 0) return 4;
            free(tight); free(r2);
            checksum += (unsigned long long)bytes;
        }
        if (adacomp_oracle_unpack_accumulate(layers, n_shapes, (const void *const *)packet, K, dense) != 0) return 5;
        if (adacomp_oracle_update_sgd(layers, n_shapes, dense, K, w, s1, 0.01f, 0.9f) != 0) return 6;
        if (adacomp_oracle_update_adam(layers, n_shapes, dense, K, w, s1, s2, 0.001f, 0.9f, 0.999f, 1e-8f, 0.1f, 0.001f) != 0) return 7;
    }
    /* malformed packets are refused, not followed */
    memset(packet[0], 0xFF, 64);
    if (adacomp_oracle_unpack_accumulate(layers, n_shapes, (const void *const *)packet, K, dense) != -5) return 8;
    /* bad tables */
    adacomp_oracle_layer_t bad = {2, 10, 50, 0};
    if (adacomp_oracle_packet_bound(&bad, 1) != 0) return 9;
    printf("oracle sanitizer driver ok, checksum %llu\n", checksum);
    for (int k = 0; k < K; ++k) { free(residue[k]); free(packet[k]); }
    free(grad); free(dense); free(w); free(s1); free(s2);
    return 0;
}
