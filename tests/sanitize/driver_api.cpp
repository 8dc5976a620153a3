// Exercises the host-only parts of libadacomp (table validation, plan and size arithmetic, error
// paths that return before any HIP call) under AddressSanitizer / UBSan on the host side.
// Built and run by tests/test_sanitizers.py; no GPU is touched.
#include <cstdio>
#include <cstdint>
#include <cstdlib>
#include <vector>

#include <hip/hip_runtime.h>

#include "adacomp.h"
#include "adacomp_debug.h"
#include "adacomp_plan.h"

// Invariants of the tile tables that the kernels index without further checks: every table is
// built on the host, so everything the kernels assume about it can be verified here.
static uint64_t g_tiles_checked = 0, g_groups_checked = 0;

static int check_plan(const std::vector<adacomp_layer_t> &t)
{
    using namespace adacomp;
    Plan p;
    if (build_plan(t.data(), uint32_t(t.size()), true, p) != ADACOMP_OK) return 100;
    if (p.ctiles.size() != p.n_ctiles || p.utiles.size() != p.n_utiles || p.ugroups.size() != p.n_ugroups ||
        p.usingles.size() != p.n_utiles)
        return 101;
    // compress tiles: whole bins, in order, covering each layer exactly; sizes fit the register class
    uint32_t ct = 0;
    uint64_t stage_next = 0;   // stretches of the staging array: one after the other in tile order, each a multiple of 4 entries
    for (uint32_t l = 0; l < p.n_layers; ++l) {
        const LayerDev &ld = p.layers[l];
        if (ld.ctile_start != ct) return 102;
        uint64_t e = 0;
        uint32_t bin = 0;
        for (uint32_t i = 0; i < ld.n_ctiles; ++i, ++ct) {
            const TileDev &td = p.ctiles[ct];
            const uint32_t cap = td.jcode() ? 16384u : 4096u;
            if (td.layer() != l || td.L_T != ld.L_T || td.first_bin != bin || td.elem_base != ld.elem_offset + e) return 103;
            if (td.n_elems == 0 || td.n_elems > cap || td.n_bins == 0 || td.n_bins > kMaxTileBins) return 104;
            if (td.n_bins != (td.n_elems + td.L_T - 1) / td.L_T) return 105;
            if (td.aligned() != (td.elem_base % 4 == 0)) return 106;
            // a tile that keeps 16-byte accesses although it is not aligned: larger class only, skip is its
            // misalignment, and the tile still fits its class with the misalignment added
            if (td.skip() != 0 && (td.aligned() || td.jcode() != 1 || td.skip() != td.elem_base % 4 || td.n_elems + td.skip() > 16384u)) return 119;
            if (td.skip() == 0 && !td.aligned() && td.jcode() == 1 && td.n_elems + td.elem_base % 4 <= 16384u) return 146;
            if (td.skip() != 0 && !p.has_shifted_tiles) return 147;
            if (td.magic != bin_magic(td.L_T)) return 107;
            if (td.n_elems > 16384u) return 108;  // the multiply-shift bin index is checked below this
            if (td.stage_base % 4u != 0 || td.stage_base < stage_next) return 117;   // stretches do not overlap
            stage_next = uint64_t(td.stage_base) + td.n_elems;
            if (stage_next > p.stage_entries) return 118;
            e += td.n_elems;
            bin += td.n_bins;
            if (i + 1 < ld.n_ctiles && td.n_elems % td.L_T != 0) return 109;  // only the last tile may end in a short bin
        }
        if (e != ld.n_elems || bin != ld.n_bins) return 110;
    }
    if (ct != p.n_ctiles) return 111;
    // tables with both tile sizes list the tile indices by size, each size in ascending order
    if (p.n_class_tiles[0] + p.n_class_tiles[1] != p.n_ctiles) return 112;
    if (p.n_class_tiles[0] && p.n_class_tiles[1]) {
        if (p.cclass.size() != p.n_ctiles) return 113;
        for (uint32_t i = 0; i < p.n_ctiles; ++i) {
            const uint32_t want = i < p.n_class_tiles[0] ? 0u : 1u;
            if (p.cclass[i] >= p.n_ctiles || p.ctiles[p.cclass[i]].jcode() != want) return 114;
            if (i && i != p.n_class_tiles[0] && p.cclass[i] <= p.cclass[i - 1]) return 115;
        }
    } else if (!p.cclass.empty()) return 116;
    // unpack tiles: cover each layer exactly, at most kUnpackTileElems each, whole bins inside one
    // 64-bin chunk or a slice of one long bin
    std::vector<uint64_t> covered(p.n_layers, 0);
    for (uint32_t i = 0; i < p.n_utiles; ++i) {
        const UTileDev &ut = p.utiles[i];
        if (ut.layer() >= p.n_layers) return 120;
        const LayerDev &ld = p.layers[ut.layer()];
        if (ut.L_T != ld.L_T || ut.n_elems == 0 || ut.n_elems > kUnpackTileElems) return 121;
        const uint64_t local = uint64_t(ut.first_bin) * ut.L_T + ut.idx_lo;
        if (ut.elem_base != ld.elem_offset + local || local != covered[ut.layer()]) return 122;
        covered[ut.layer()] += ut.n_elems;
        if (ut.L_T <= kUnpackTileElems) {
            if (ut.idx_lo != 0 || ut.n_bins == 0 || ut.n_bins > 64) return 123;
            if ((ut.first_bin >> 6) != ((ut.first_bin + ut.n_bins - 1) >> 6)) return 124;
            if (ut.n_bins != (ut.n_elems + ut.L_T - 1) / ut.L_T) return 125;
        } else {
            if (ut.n_bins != 1 || ut.idx_lo + ut.n_elems > ut.L_T) return 126;
        }
        if (ut.group_log2() < 3 || ut.group_log2() > 6) return 127;
        if (ut.aligned() != (ut.elem_base % 4 == 0)) return 128;
    }
    for (uint32_t l = 0; l < p.n_layers; ++l)
        if (covered[l] != p.layers[l].n_elems) return 129;
    // groups: consecutive tiles, every tile in exactly one group, at most kUnpackGroupTiles, all in
    // one layer and one chunk (or one long bin): the kernel's table rows stay below 64
    std::vector<uint8_t> seen(p.n_utiles, 0);
    for (const UGroupDev &g : p.ugroups) {
        if (g.n_tiles == 0 || g.n_tiles > kUnpackGroupTiles || uint64_t(g.first_tile) + g.n_tiles > p.n_utiles) return 130;
        const UTileDev &a = p.utiles[g.first_tile];
        for (uint32_t i = 0; i < g.n_tiles; ++i) {
            const UTileDev &ut = p.utiles[g.first_tile + i];
            if (seen[g.first_tile + i]++) return 131;
            if (ut.layer() != a.layer()) return 132;
            if (ut.L_T <= kUnpackTileElems ? (ut.first_bin >> 6) != (a.first_bin >> 6) : ut.first_bin != a.first_bin) return 133;
            if (ut.first_bin < a.first_bin || ut.first_bin + ut.n_bins - a.first_bin > 64) return 134;
        }
    }
    for (uint32_t i = 0; i < p.n_utiles; ++i)
        if (seen[i] != 1) return 135;
    // both tables list the groups of layers with 8-bit words first (they go to their own kernel)
    if (p.n_ugroups8 > p.n_ugroups || p.n_usingles8 > p.n_utiles) return 137;
    for (uint32_t i = 0; i < p.n_ugroups; ++i)
        if ((p.utiles[p.ugroups[i].first_tile].L_T <= 64u) != (i < p.n_ugroups8)) return 138;
    for (uint32_t i = 0; i < p.n_utiles; ++i)
        if ((p.utiles[p.usingles[i].first_tile].L_T <= 64u) != (i < p.n_usingles8)) return 139;
    std::fill(seen.begin(), seen.end(), 0);
    for (const UGroupDev &g : p.usingles) {
        if (g.n_tiles != 1 || g.first_tile >= p.n_utiles || seen[g.first_tile]++) return 136;
    }
    // workspace layout: sections in order, inside the advertised size
    const WorkspaceLayout &w = p.ws;
    if (w.cclass + 4 * size_t(p.n_ctiles) > w.utiles) return 144;
    if (!(w.layers < w.ctiles && w.ctiles <= w.cclass && w.cclass <= w.utiles && w.utiles <= w.ugroups && w.ugroups <= w.usingles && w.usingles <= w.scratch)) return 140;
    if (w.usingles + sizeof(UGroupDev) * size_t(p.n_utiles) > w.scratch) return 141;
    if (w.stage + 2 * size_t(p.stage_entries) + 128 > w.scratch_stride) return 142;  // k_place reads 64 entries from a tile's start
    if (p.stage_entries > p.n_elems_total + 3ull * p.n_ctiles) return 145;       // the array follows the element count, not the address span
    if (w.total(3) != adacomp_workspace_bytes_batch(t.data(), uint32_t(t.size()), 3)) return 143;
    g_tiles_checked += p.n_ctiles + p.n_utiles;
    g_groups_checked += p.n_ugroups;
    return 0;
}

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
        // tile tables, with the default grouping of unpack tiles and with runs forced on small tables
        adacomp_tuning_unpack_min_groups(rep % 2 ? 1u : 0u);
        const int pc = check_plan(t);
        adacomp_tuning_unpack_min_groups(0);
        if (pc) { std::printf("plan check failed with %d at rep %d\n", pc, rep); return pc; }
        // calls on a workspace that was never initialised return before touching any device
        alignas(256) static char fake[4096];
        const float *g = reinterpret_cast<const float *>(fake);
        float *r = reinterpret_cast<float *>(fake + 1024);
        void *pk = fake + 2048;
        if (adacomp_compress(t.data(), n_layers, g, r, pk, bound, fake + 3072, ws1, nullptr) != ADACOMP_EWORKSPACE) return 4;
        const void *pks[1] = {pk};
        if (adacomp_unpack_accumulate(t.data(), n_layers, pks, 1, r, fake + 3072, ws1, nullptr) != ADACOMP_EWORKSPACE) return 5;
        void *pko[1] = {pk};
        if (adacomp_compress_batch_lazy(t.data(), n_layers, 1, &g, &r, pko, bound, fake + 3072, ws1, nullptr) != ADACOMP_EWORKSPACE) return 9;
        if (adacomp_residue_sync(fake + 3072, nullptr) != ADACOMP_EWORKSPACE || adacomp_residue_sync(nullptr, nullptr) != ADACOMP_EINVAL) return 10;
        // a broken copy of the table is refused
        std::vector<adacomp_layer_t> b = t;
        b[next() % n_layers].L_T = 16385;
        if (adacomp_packet_bound(b.data(), n_layers) != 0) return 6;
        b = t;
        b[0].elem_offset += 2;
        if (adacomp_packet_bound(b.data(), n_layers) != 0) return 7;
        if (n_layers > 1) { b = t; b[1].elem_offset = b[0].elem_offset; if (adacomp_packet_bound(b.data(), n_layers) != 0) return 8; }
    }
    {   // the 125 M-element table of the benchmark: runs of 8 tiles that shorten towards the end
        std::vector<adacomp_layer_t> t(7);
        uint64_t off = 0;
        for (int l = 0; l < 7; ++l) { t[l] = adacomp_layer_t{off, l < 6 ? 4096ull * 4096 : 4096ull * 5999, 500, 0}; off += t[l].n_elems; }
        const int pc = check_plan(t);
        if (pc) { std::printf("plan check of the large table failed with %d\n", pc); return pc; }
        adacomp::Plan p;
        adacomp::build_plan(t.data(), 7, true, p);
        uint32_t longest = 0;
        for (const auto &g : p.ugroups) longest = g.n_tiles > longest ? g.n_tiles : longest;
        if (longest != adacomp::kUnpackGroupTiles || p.ugroups.back().n_tiles != 1) return 11;
    }
    {   // a workspace registered for one layer table serves that list of layers and no other: the
        // same table is found, tables of the same length that differ in one field of one layer are
        // refused (the kernels would index the tile tables of the wrong geometry otherwise)
        using namespace adacomp;
        std::vector<adacomp_layer_t> a = {{0, 5000, 50, 0}, {5000, 70000, 500, 0}, {75000, 130, 64, 0}};
        alignas(256) static char fake_ws[256];
        Plan p, found;
        if (build_plan(a.data(), 3, true, p) != ADACOMP_OK) return 20;
        const size_t bytes = p.ws.total(2);
        register_workspace(a.data(), 3, fake_ws, bytes, std::move(p));
        if (find_plan(a.data(), 3, fake_ws, bytes, 2, found) != ADACOMP_OK) return 21;
        if (found.n_ctiles == 0 || found.ws.total(2) != bytes) return 22;
        if (find_plan(a.data(), 3, fake_ws, bytes, 3, found) != ADACOMP_EWORKSPACE) return 23;  // too small for 3 learners
        if (find_plan(a.data(), 3, fake_ws + 16, bytes, 2, found) != ADACOMP_EWORKSPACE) return 24;
        for (int field = 0; field < 3; ++field)
            for (int l = 0; l < 3; ++l) {
                std::vector<adacomp_layer_t> b = a;
                if (field == 0) b[l].L_T += 1;
                if (field == 1) b[l].n_elems -= 1;
                if (field == 2) b[2].elem_offset += 4 * (l + 1);   // the last layer moved up: still no overlap
                if (adacomp_packet_bound(b.data(), 3) == 0) return 25;   // b is a valid table in its own right
                if (find_plan(b.data(), 3, fake_ws, bytes, 2, found) != ADACOMP_EWORKSPACE) return 26;
                const float *g = reinterpret_cast<const float *>(fake_ws);
                if (adacomp_compress(b.data(), 3, g + 4, const_cast<float *>(g) + 8, fake_ws + 64, 1 << 20, fake_ws, bytes, nullptr) !=
                    ADACOMP_EWORKSPACE)
                    return 27;
            }
        if (find_plan(a.data(), 2, fake_ws, bytes, 2, found) != ADACOMP_EWORKSPACE) return 28;  // a prefix of the list
        if (adacomp_workspace_release(fake_ws) != ADACOMP_OK) return 29;
        if (find_plan(a.data(), 3, fake_ws, bytes, 2, found) != ADACOMP_EWORKSPACE) return 30;
    }
    if (adacomp_selftest_binindex() != 0) return 9;
    for (int c = 1; c > -9; --c) if (!adacomp_strerror(c)) return 10;
    std::printf("api sanitizer driver ok, checksum %llu, %llu tiles and %llu groups checked\n", (unsigned long long)checksum,
                (unsigned long long)g_tiles_checked, (unsigned long long)g_groups_checked);
    return 0;
}
