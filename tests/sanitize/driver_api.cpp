// Exercises the host-only parts of libadacomp (table validation, plan and size arithmetic, error
// paths that return before any HIP call) under AddressSanitizer / UBSan on the host side.
// Built and run by tests/test_sanitizers.py; no GPU is touched.
#include <cstdio>
#include <cstdint>
#include <cstdlib>
#include <vector>

#include "adacomp.h"

int main()
{
    uint64_t lcg = 12345;
    auto next = [&lcg]() { lcg = lcg * 6364136223846793005ull + 1442695040888963407ull; return uint32_t(lcg >> 33); };
    const uint32_t lts[] = {1, 2, 3, 7, 50, 63, 64, 65, 500, 4095, 4096, 4097, 8192, 16383, 16384};
    uint64_t checksum = 0;
    for (int rep = 0; rep < 200; ++rep) {
        const uint32_t n_layers = 1 + next() % 40;
        std::vector<adacomp_layer_t> t(n_layers);
        uint64_t off = 0;
        for (auto &l : t) {
            l.elem_offset = off;
            l.n_elems = 1 + next() % (rep % 10 == 0 ? 3000000u : 20000u);
            l.L_T = lts[next() % (sizeof lts / sizeof lts[0])];
            l.reserved = 0;
            off += (l.n_elems + 3) / 4 * 4 + 4 * (next() % 3);
        }
        const size_t bound = adacomp_packet_bound(t.data(), n_layers), fixed = adacomp_packet_fixed_bytes(t.data(), n_layers);
        const size_t ws1 = adacomp_workspace_bytes(t.data(), n_layers), ws5 = adacomp_workspace_bytes_batch(t.data(), n_layers, 5);
        if (!bound || !fixed || fixed > bound || !ws1 || ws5 <= ws1) return 2;
        size_t goff = 0, gn = 0, gstride = 0;
        if (adacomp_workspace_gmax(t.data(), n_layers, &goff, &gn, &gstride) != ADACOMP_OK || goff + 4 * gn > ws1) return 3;
        checksum += bound + fixed + ws1 + gn;
        // calls on a workspace that was never initialised return before touching any device
        alignas(256) static char fake[4096];
        const float *g = reinterpret_cast<const float *>(fake);
        float *r = reinterpret_cast<float *>(fake + 1024);
        void *pk = fake + 2048;
        if (adacomp_compress(t.data(), n_layers, g, r, pk, bound, fake + 3072, ws1, nullptr) != ADACOMP_EWORKSPACE) return 4;
        const void *pks[1] = {pk};
        if (adacomp_unpack_accumulate(t.data(), n_layers, pks, 1, r, fake + 3072, ws1, nullptr) != ADACOMP_EWORKSPACE) return 5;
        // a broken copy of the table is refused
        std::vector<adacomp_layer_t> b = t;
        b[next() % n_layers].L_T = 16385;
        if (adacomp_packet_bound(b.data(), n_layers) != 0) return 6;
        b = t;
        b[0].elem_offset += 2;
        if (adacomp_packet_bound(b.data(), n_layers) != 0) return 7;
        if (n_layers > 1) { b = t; b[1].elem_offset = b[0].elem_offset; if (adacomp_packet_bound(b.data(), n_layers) != 0) return 8; }
    }
    if (adacomp_selftest_binindex() != 0) return 9;
    for (int c = 1; c > -9; --c) if (!adacomp_strerror(c)) return 10;
    std::printf("api sanitizer driver ok, checksum %llu\n", (unsigned long long)checksum);
    return 0;
}
