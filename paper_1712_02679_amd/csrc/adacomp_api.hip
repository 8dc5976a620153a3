// adacomp_api.hip -- the C ABI of libadacomp: argument checks, the plan (tile tables and
// workspace layout) and the launch sequences.  No arithmetic of the method lives here.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <unordered_map>

#include "adacomp_debug.h"
#include "adacomp_plan.h"

namespace adacomp {

static uint64_t pad16(uint64_t x) { return (x + 15u) & ~uint64_t(15); }
static size_t pad256(size_t x) { return (x + 255u) & ~size_t(255); }
static uint32_t gcd_u32(uint32_t a, uint32_t b) { while (b) { uint32_t t = a % b; a = b; b = t; } return a; }

uint32_t bin_magic(uint32_t L_T)
{
    // floor(2^32 / L_T) + 1; exact for every index below 2^32 / L_T >= 2^18 (see the self-test).
    // L_T == 1 would need 2^32 + 1: the kernels special-case it (bin == index).
    return L_T <= 1 ? 0u : uint32_t((uint64_t(1) << 32) / L_T) + 1u;
}

static int validate(const adacomp_layer_t *layers, uint32_t n_layers)
{
    if (!layers || n_layers == 0 || n_layers >= (1u << 24)) return ADACOMP_EINVAL;
    for (uint32_t l = 0; l < n_layers; ++l) {
        if (layers[l].n_elems == 0 || layers[l].n_elems >= (uint64_t(1) << 31)) return ADACOMP_EINVAL;
        if (layers[l].L_T == 0 || layers[l].L_T > ADACOMP_LT_MAX) return ADACOMP_EBADLT;
        if (layers[l].elem_offset % 4 != 0) return ADACOMP_EALIGN;
        if (layers[l].elem_offset + layers[l].n_elems < layers[l].elem_offset) return ADACOMP_EINVAL;
    }
    // overlap check: sort-free O(n^2) is fine for a few hundred layers; use a sorted copy beyond that
    if (n_layers <= 512) {
        for (uint32_t l = 0; l < n_layers; ++l)
            for (uint32_t m = 0; m < l; ++m) {
                uint64_t a0 = layers[l].elem_offset, a1 = a0 + layers[l].n_elems;
                uint64_t b0 = layers[m].elem_offset, b1 = b0 + layers[m].n_elems;
                if (a0 < b1 && b0 < a1) return ADACOMP_EINVAL;
            }
    } else {
        std::vector<std::pair<uint64_t, uint64_t>> iv(n_layers);
        for (uint32_t l = 0; l < n_layers; ++l) iv[l] = {layers[l].elem_offset, layers[l].elem_offset + layers[l].n_elems};
        std::sort(iv.begin(), iv.end());
        for (uint32_t l = 1; l < n_layers; ++l)
            if (iv[l].first < iv[l - 1].second) return ADACOMP_EINVAL;
    }
    return ADACOMP_OK;
}

// process-wide tuning and diagnostic flags (adacomp_debug.h): atomics, so that a compute call on one
// thread reads a whole value while another thread sets it; no ordering beyond that is promised
static std::atomic<uint32_t> g_unpack_min_groups{kUnpackMinGroups};
static std::atomic<bool> g_fold_scan{true};
static std::atomic<bool> g_place_tiled{true};

int build_plan(const adacomp_layer_t *layers, uint32_t n_layers, bool tables, Plan &p)
{
    int rc = validate(layers, n_layers);
    if (rc != ADACOMP_OK) return rc;
    p = Plan();
    p.n_layers = n_layers;
    p.layers.resize(n_layers);

    uint64_t fixed = sizeof(adacomp_packet_header_t) + uint64_t(sizeof(adacomp_packet_layer_t)) * n_layers;
    uint64_t words_bound = 0;
    uint64_t n_ctiles = 0, n_utiles = 0, bins_total = 0, chunks_total = 0;

    // A table that makes fewer tiles of 4096 elements than there are compute units cannot fill the GPU,
    // and the time of a launch is then the time of one tile: such tables get smaller tiles, down to
    // 1024 elements (the 397 k-element table: 97 tiles become 265, 23 -> 19 us per compress call).
    uint64_t elems_all = 0;
    for (uint32_t l = 0; l < n_layers; ++l) elems_all += layers[l].n_elems;
    const uint32_t small_cap = uint32_t(std::min<uint64_t>(4096u, std::max<uint64_t>(1024u, elems_all / kComputeUnits)));

    for (uint32_t l = 0; l < n_layers; ++l) {
        const uint32_t T = layers[l].L_T;
        const uint32_t n = uint32_t(layers[l].n_elems);
        const uint32_t n_bins = (n + T - 1) / T;
        const uint32_t n_chunks = (n_bins + ADACOMP_CHUNK_BINS - 1) / ADACOMP_CHUNK_BINS;
        const uint32_t wb = T <= 64 ? 1u : 2u;
        LayerDev &ld = p.layers[l];
        ld.elem_offset = layers[l].elem_offset;
        ld.n_elems = n; ld.L_T = T; ld.n_bins = n_bins; ld.word_bytes = wb; ld.n_chunks = n_chunks; ld.pad0 = 0;
        ld.counts_offset = fixed;
        ld.chunks_offset = fixed + pad16(uint64_t(n_bins) * wb);
        fixed = ld.chunks_offset + pad16(uint64_t(n_chunks) * 4);
        words_bound += pad16(uint64_t(n) * wb);
        ld.bin_start = uint32_t(bins_total);
        ld.chunk_start = uint32_t(chunks_total);
        bins_total += n_bins;
        chunks_total += n_chunks;
        if (bins_total >= (uint64_t(1) << 32)) return ADACOMP_EINVAL;
        p.elem_span = std::max<uint64_t>(p.elem_span, layers[l].elem_offset + n);
        p.n_elems_total += n;

        // ---- compress tiles: whole bins, as many as fit the registers of a workgroup ------------
        // 16 elements per thread (tiles of 4096 elements) unless a bin is longer: then 64 per thread
        // (16384).  Tiles of 8192 elements streamed at less than half the rate of either on MI355X
        // (measured on a plain triad), so there is no class in between.
        // Tile starts are float4-aligned when a tile holds a multiple of a = 4 / gcd(L_T, 4) bins.  Bin
        // lengths that are odd (a = 4) or twice an odd number (a = 2) and too long for a such bins to fit
        // 4096 elements take the larger class when they fit there: unaligned tiles fall back to 4-byte
        // accesses, which stream at 44 % of the HBM peak instead of 71-77 %.
        const uint32_t a = 4u / gcd_u32(T, 4u);
        const int cls = (T > 4096u || (uint64_t(a) * T > 4096u && uint64_t(a) * T <= 16384u)) ? 1 : 0;
        const uint32_t cap = cls ? 16384u : 4096u;
        uint32_t bpt = (cls ? cap : small_cap) / T;
        if (bpt == 0) bpt = 1;                        // a bin of up to cap elements always fits its class
        if (bpt > kMaxTileBins) bpt = kMaxTileBins;
        if (bpt < a && uint64_t(a) * T <= cap) bpt = a;
        if (bpt >= a) bpt -= bpt % a;
        const uint32_t nt = (n_bins + bpt - 1) / bpt;
        ld.ctile_start = uint32_t(n_ctiles);
        ld.n_ctiles = nt;
        p.n_class_tiles[cls] += nt;
        if (T <= 64u) p.has_short_bins = true;
        // The staging array is indexed by position in the tile table, not by address: a tile's stretch
        // starts where the stretches of the tiles before it end (each rounded up to 4 entries, which keeps
        // every stretch 8-byte aligned), so its size follows the element count whatever holes the table has.
        const uint64_t full_tile = uint64_t(bpt) * T, full_stretch = (full_tile + 3u) & ~uint64_t(3);
        if (tables) {
            for (uint32_t t = 0; t < nt; ++t) {
                TileDev td;
                const uint32_t first_bin = t * bpt;
                const uint64_t e0 = uint64_t(first_bin) * T;
                td.elem_base = layers[l].elem_offset + e0;
                td.stage_base = uint32_t(p.stage_entries + full_stretch * t);
                td.n_elems = uint16_t(std::min<uint64_t>(full_tile, n - e0));
                td.L_T = T;
                td.magic = bin_magic(T);
                td.n_bins = uint16_t((uint32_t(td.n_elems) + T - 1) / T);
                td.first_bin = first_bin;
                td.layer_flags = l | (uint32_t(cls) << 24) | ((e0 % 4 == 0) ? 0x80000000u : 0u);
                p.ctiles.push_back(td);
            }
        }
        // unaligned tiles of the larger class keep 16-byte accesses when the tile still fits with its
        // misalignment added (all but bins of 16382 or 16383 elements); independent of `tables`, so
        // that every plan of a table says the same
        if (cls == 1 && (uint64_t(bpt) * T) % 4 != 0) {
            for (uint32_t t = 0; t < nt; ++t) {
                const uint64_t e0 = uint64_t(t) * bpt * T;
                const uint32_t sk = uint32_t(e0 % 4), ne = uint32_t(std::min<uint64_t>(uint64_t(bpt) * T, n - e0));
                if (sk != 0 && ne + sk <= 16384u) {
                    p.has_shifted_tiles = true;
                    if (tables) p.ctiles[p.ctiles.size() - nt + t].layer_flags |= sk << 25;
                }
            }
        }
        p.stage_entries += full_stretch * (nt - 1) + ((n - full_tile * (nt - 1) + 3u) & ~uint64_t(3));
        if (p.stage_entries >= (uint64_t(1) << 32)) return ADACOMP_EINVAL;
        n_ctiles += nt;

        // ---- unpack tiles: a power-of-two number of bins inside one 64-bin chunk, or slices of
        //      one long bin --------------------------------------------------------------------
        const uint32_t glog = T <= 64 ? 3u : 4u;      // lanes that share a bin: 8 or 16
        if (T <= kUnpackTileElems) {
            uint32_t nb = 1;
            while (nb * 2 <= ADACOMP_CHUNK_BINS && uint64_t(nb) * 2 * T <= kUnpackTileElems) nb *= 2;
            const uint32_t nut = (n_bins + nb - 1) / nb;
            if (tables) {
                for (uint32_t t = 0; t < nut; ++t) {
                    UTileDev ut;
                    const uint32_t first_bin = t * nb;
                    const uint64_t e0 = uint64_t(first_bin) * T;
                    ut.elem_base = layers[l].elem_offset + e0;
                    ut.n_elems = uint32_t(std::min<uint64_t>(uint64_t(nb) * T, n - e0));
                    ut.L_T = T;
                    ut.n_bins = (ut.n_elems + T - 1) / T;
                    ut.first_bin = first_bin;
                    ut.idx_lo = 0;
                    ut.layer_flags = l | (glog << 24) | ((e0 % 4 == 0) ? 0x80000000u : 0u);
                    p.utiles.push_back(ut);
                }
            }
            n_utiles += nut;
        } else {
            for (uint32_t b = 0; b < n_bins; ++b) {
                const uint64_t b0 = uint64_t(b) * T;
                const uint32_t blen = uint32_t(std::min<uint64_t>(T, n - b0));
                for (uint32_t lo = 0; lo < blen; lo += kUnpackTileElems) {
                    if (tables) {
                        UTileDev ut;
                        ut.elem_base = layers[l].elem_offset + b0 + lo;
                        ut.n_elems = std::min(kUnpackTileElems, blen - lo);
                        ut.L_T = T;
                        ut.n_bins = 1;
                        ut.first_bin = b;
                        ut.idx_lo = lo;
                        ut.layer_flags = l | (glog << 24) | (((b0 + lo) % 4 == 0) ? 0x80000000u : 0u);
                        p.utiles.push_back(ut);
                    }
                    ++n_utiles;
                }
            }
        }
        if (n_ctiles >= (1u << 31) || n_utiles >= (1u << 31)) return ADACOMP_EINVAL;
    }
    p.n_ctiles = uint32_t(n_ctiles);
    p.n_utiles = uint32_t(n_utiles);
    if (tables && p.n_class_tiles[0] && p.n_class_tiles[1]) {
        // both tile sizes: each gets its own k_fused launch over its own tiles
        p.cclass.reserve(p.n_ctiles);
        for (uint32_t c = 0; c < 2u; ++c)
            for (uint32_t i = 0; i < p.n_ctiles; ++i)
                if (p.ctiles[i].jcode() == c) p.cclass.push_back(i);
    }
    if (tables) {
        // ---- unpack groups: runs of tiles that share phase 1 (same layer and 64-bin chunk, or the
        //      same long bin).  Longer runs save more table work but leave fewer workgroups, so the
        //      run length halves until at least kUnpackMinGroups workgroups remain.  Workgroups
        //      start in index order, so the runs get shorter towards the end of the table (the last
        //      kUnpackTaperTiles tiles go alone, twice as many before them in pairs, ...): the
        //      launch then ends with short workgroups instead of a few long stragglers. -----------
        uint32_t run = kUnpackGroupTiles;
        const uint32_t min_groups = g_unpack_min_groups.load(std::memory_order_relaxed);
        while (run > 1u && n_utiles / run < min_groups) run /= 2u;
        const uint32_t taper = kUnpackTaperTiles;
        const uint32_t run_max = run;
        for (uint32_t i = 0; i < p.n_utiles; ++i) {
            const UTileDev &ut = p.utiles[i];
            const uint32_t left = p.n_utiles - i;
            run = run_max;
            for (uint32_t r = 1u, span = taper; r < run_max; r *= 2u, span += taper * r)
                if (left <= span) { run = r; break; }
            bool fresh = p.ugroups.empty() || p.ugroups.back().n_tiles >= run;
            if (!fresh) {
                const UTileDev &first = p.utiles[p.ugroups.back().first_tile];
                fresh = first.layer() != ut.layer() ||
                        (ut.L_T <= kUnpackTileElems ? (first.first_bin >> 6) != (ut.first_bin >> 6) : first.first_bin != ut.first_bin);
            }
            if (fresh) p.ugroups.push_back(UGroupDev{i, 1u});
            else ++p.ugroups.back().n_tiles;
        }
        // Single tiles, for the launches that also apply the optimizer: those are bound by the
        // traffic of their epilogue, gain nothing from shared tables, and with runs of tiles they
        // were up to 15 % slower on some machines.  Workgroups are dealt to the 8 XCDs round-robin,
        // so inside each 64 the order is transposed and the 8 tiles of a chunk, which read the same
        // count and offset lines of every packet, share an L2.
        p.usingles.resize(p.n_utiles);
        const uint32_t whole = p.n_utiles & ~63u;
        for (uint32_t i = 0; i < p.n_utiles; ++i)
            p.usingles[i] = UGroupDev{i < whole ? ((i & ~63u) | ((i & 7u) << 3) | ((i >> 3) & 7u)) : i, 1u};
        if (run_max == 1u) p.ugroups = p.usingles;
        // groups of 8-bit layers first: the two kinds go to different kernels
        auto is8 = [&p](const UGroupDev &g) { return p.utiles[g.first_tile].L_T <= 64u; };
        p.n_ugroups8 = uint32_t(std::stable_partition(p.ugroups.begin(), p.ugroups.end(), is8) - p.ugroups.begin());
        p.n_usingles8 = uint32_t(std::stable_partition(p.usingles.begin(), p.usingles.end(), is8) - p.usingles.begin());
        p.n_ugroups = uint32_t(p.ugroups.size());
    }
    p.n_bins_total = uint32_t(bins_total);
    p.n_chunks_total = uint32_t(chunks_total);
    p.fixed_bytes = fixed;
    p.bound_bytes = fixed + words_bound;
    if (p.bound_bytes >= (uint64_t(1) << 32)) return ADACOMP_EINVAL;  // word positions are 32-bit in k_unpack

    WorkspaceLayout &w = p.ws;
    size_t off = 256;  // first 256 bytes: reserved
    w.layers = off;      off = pad256(off + sizeof(LayerDev) * size_t(n_layers));
    w.ctiles = off;      off = pad256(off + sizeof(TileDev) * size_t(p.n_ctiles));
    w.cclass = off;      off = pad256(off + 4 * size_t(p.n_ctiles));
    w.utiles = off;      off = pad256(off + sizeof(UTileDev) * size_t(p.n_utiles));
    w.ugroups = off;     off = pad256(off + sizeof(UGroupDev) * size_t(p.n_utiles));  // at most one group per tile
    w.usingles = off;    off = pad256(off + sizeof(UGroupDev) * size_t(p.n_utiles));
    w.scratch = off;
    off = 0;             // offsets inside one learner's scratch block
    w.tile_out = off;    off = pad256(off + sizeof(TileOut) * size_t(p.n_ctiles));
    w.layer_nsel = off;  off = pad256(off + 4 * size_t(n_layers));
    w.layer_scale = off; off = pad256(off + 4 * size_t(n_layers));
    w.gmax = off;        off = pad256(off + 4 * size_t(p.n_bins_total));
    w.chunk_rel = off;   off = pad256(off + 4 * size_t(p.n_chunks_total));
    if (off >= (size_t(1) << 32)) return ADACOMP_EINVAL;
    w.stage = off;       off = pad256(off + 2 * size_t(p.stage_entries) + 128);  // slack: k_place reads up to 64 entries from a tile's start
    w.scratch_stride = off;
    return ADACOMP_OK;
}

// Workspaces that adacomp_workspace_init has filled, by address.
// waiting: the residue buffers, by learner slot, whose corrections of the last lazy call have not
// been written yet (empty: none).  Kept at enqueue time, which is stream order for a workspace that
// one stream uses at a time.
struct Registered {
    Plan plan;
    size_t bytes = 0;
    std::vector<adacomp_layer_t> table;  // the layer table the tile tables in the workspace were built for
    std::vector<float *> waiting;
};

static bool same_table(const std::vector<adacomp_layer_t> &have, const adacomp_layer_t *layers, uint32_t n_layers)
{
    if (have.size() != n_layers) return false;
    for (uint32_t l = 0; l < n_layers; ++l)
        if (have[l].elem_offset != layers[l].elem_offset || have[l].n_elems != layers[l].n_elems ||
            have[l].L_T != layers[l].L_T)
            return false;
    return true;
}
static std::mutex g_mu;
static std::unordered_map<const void *, Registered> g_ws;

int find_plan(const adacomp_layer_t *layers, uint32_t n_layers, const void *workspace,
              size_t workspace_bytes, size_t n_learners, Plan &out)
{
    if (!layers || n_layers == 0 || !workspace) return ADACOMP_EINVAL;
    std::lock_guard<std::mutex> lk(g_mu);
    auto it = g_ws.find(workspace);
    if (it == g_ws.end()) return ADACOMP_EWORKSPACE;
    const Plan &p = it->second.plan;
    // the kernels index the tile tables in the workspace without further checks: the table of this
    // call must be, entry by entry, the one those tables were built for
    if (!same_table(it->second.table, layers, n_layers)) return ADACOMP_EWORKSPACE;
    if (workspace_bytes < p.ws.total(n_learners) || it->second.bytes < p.ws.total(n_learners)) return ADACOMP_EWORKSPACE;
    // copy the scalars only; the tables already live on the device
    out.n_layers = p.n_layers; out.n_ctiles = p.n_ctiles; out.n_utiles = p.n_utiles; out.n_ugroups = p.n_ugroups; out.n_ugroups8 = p.n_ugroups8; out.n_usingles8 = p.n_usingles8;
    out.n_bins_total = p.n_bins_total; out.n_chunks_total = p.n_chunks_total;
    out.elem_span = p.elem_span; out.n_elems_total = p.n_elems_total; out.stage_entries = p.stage_entries;
    out.fixed_bytes = p.fixed_bytes; out.bound_bytes = p.bound_bytes;
    for (int c = 0; c < 2; ++c) out.n_class_tiles[c] = p.n_class_tiles[c];
    out.has_short_bins = p.has_short_bins; out.has_shifted_tiles = p.has_shifted_tiles;
    out.ws = p.ws;
    return ADACOMP_OK;
}

void register_workspace(const adacomp_layer_t *layers, uint32_t n_layers, const void *workspace, size_t workspace_bytes,
                        Plan &&plan)
{
    Registered reg;
    reg.plan = std::move(plan);
    Plan &p = reg.plan;
    // the host copies of the tile tables are not needed once they are on the device
    p.ctiles.clear(); p.ctiles.shrink_to_fit();
    p.cclass.clear(); p.cclass.shrink_to_fit();
    p.utiles.clear(); p.utiles.shrink_to_fit();
    p.ugroups.clear(); p.ugroups.shrink_to_fit();
    p.usingles.clear(); p.usingles.shrink_to_fit();
    reg.table.assign(layers, layers + n_layers);
    reg.bytes = workspace_bytes;
    std::lock_guard<std::mutex> lk(g_mu);
    g_ws[workspace] = std::move(reg);
}

// ---- optional event timing of the streaming kernel ---------------------------------------------
// The records are guarded by g_timing_mu; `on` alone is read without it, so that calls pay nothing
// while timing is off.
struct Timing {
    std::atomic<bool> on{false};
    std::vector<std::pair<hipEvent_t, hipEvent_t>> pool;
    size_t used = 0;
    uint64_t learners = 0;  // learners covered by the recorded launches
    uint32_t stride = 1;    // every stride-th launch is recorded
    uint64_t seen = 0;      // launches since recording started
};
static Timing g_timing;
static std::mutex g_timing_mu;
static std::atomic<bool> g_keep_gmax{false};

}  // namespace adacomp

using namespace adacomp;

extern "C" {

size_t adacomp_packet_bound(const adacomp_layer_t *layers, uint32_t n_layers)
{
    Plan p;
    return build_plan(layers, n_layers, false, p) == ADACOMP_OK ? size_t(p.bound_bytes) : 0;
}

size_t adacomp_packet_fixed_bytes(const adacomp_layer_t *layers, uint32_t n_layers)
{
    Plan p;
    return build_plan(layers, n_layers, false, p) == ADACOMP_OK ? size_t(p.fixed_bytes) : 0;
}

size_t adacomp_workspace_bytes(const adacomp_layer_t *layers, uint32_t n_layers)
{
    Plan p;
    return build_plan(layers, n_layers, false, p) == ADACOMP_OK ? p.ws.total(1) : 0;
}

size_t adacomp_workspace_bytes_batch(const adacomp_layer_t *layers, uint32_t n_layers, uint32_t n_learners)
{
    Plan p;
    if (n_learners == 0) return 0;
    return build_plan(layers, n_layers, false, p) == ADACOMP_OK ? p.ws.total(n_learners) : 0;
}

int adacomp_workspace_gmax(const adacomp_layer_t *layers, uint32_t n_layers, size_t *byte_offset,
                           size_t *n_bins_total, size_t *learner_stride)
{
    if (!byte_offset || !n_bins_total) return ADACOMP_EINVAL;
    Plan p;
    int rc = build_plan(layers, n_layers, false, p);
    if (rc != ADACOMP_OK) return rc;
    *byte_offset = p.ws.scratch + p.ws.gmax;
    *n_bins_total = p.n_bins_total;
    if (learner_stride) *learner_stride = p.ws.scratch_stride;
    return ADACOMP_OK;
}

int adacomp_workspace_init(const adacomp_layer_t *layers, uint32_t n_layers, void *workspace,
                           size_t workspace_bytes, void *hip_stream)
{
    if (!workspace) return ADACOMP_EINVAL;
    if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0) return ADACOMP_EALIGN;
    Registered reg;
    int rc = build_plan(layers, n_layers, true, reg.plan);
    if (rc != ADACOMP_OK) return rc;
    Plan &p = reg.plan;
    if (workspace_bytes < p.ws.total(1)) return ADACOMP_EWORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (hipStreamSynchronize(s) != hipSuccess) return ADACOMP_EHIP;
    char *ws = static_cast<char *>(workspace);
    if (hipMemcpy(ws + p.ws.layers, p.layers.data(), sizeof(LayerDev) * p.layers.size(), hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(ws + p.ws.ctiles, p.ctiles.data(), sizeof(TileDev) * p.ctiles.size(), hipMemcpyHostToDevice) != hipSuccess ||
        (!p.cclass.empty() && hipMemcpy(ws + p.ws.cclass, p.cclass.data(), 4 * p.cclass.size(), hipMemcpyHostToDevice) != hipSuccess) ||
        hipMemcpy(ws + p.ws.utiles, p.utiles.data(), sizeof(UTileDev) * p.utiles.size(), hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(ws + p.ws.ugroups, p.ugroups.data(), sizeof(UGroupDev) * p.ugroups.size(), hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(ws + p.ws.usingles, p.usingles.data(), sizeof(UGroupDev) * p.usingles.size(), hipMemcpyHostToDevice) != hipSuccess)
        return ADACOMP_EHIP;
    register_workspace(layers, n_layers, workspace, workspace_bytes, std::move(reg.plan));
    return ADACOMP_OK;
}

int adacomp_workspace_release(void *workspace)
{
    std::lock_guard<std::mutex> lk(g_mu);
    return g_ws.erase(workspace) ? ADACOMP_OK : ADACOMP_EINVAL;
}

// Lanes per tile in k_place: 64 for tables with short bins, whose tiles send several hundred words,
// and for small tables, where the launch is far from filling the GPU and the words of a tile are
// better spread over more lanes (the 397 k-element table sends 440 words per tile in its first
// steps: 37 -> 23 us per compress call); 16 otherwise.
static uint32_t place_lanes_for(const Plan &p)
{
    return (p.has_short_bins || p.n_ctiles <= 2048u) ? 64u : 16u;
}

// Small tables: no k_scan launch, the placement kernel does the scan itself (see k_place).
static bool fold_scan_for(const Plan &p)
{
    return g_fold_scan.load(std::memory_order_relaxed) && place_lanes_for(p) == 64u && p.n_ctiles <= kFoldTiles && p.n_layers <= kFoldLayers;
}

static int compress_common(const adacomp_layer_t *layers, uint32_t n_layers, uint32_t n_learners,
                           const float *const *grads, float *const *residues, void *const *packets_out,
                           size_t packet_capacity, uint32_t rule, float soft_factor, bool lazy, void *workspace,
                           size_t workspace_bytes, void *hip_stream)
{
    if (n_learners == 0 || !grads || !residues || !packets_out) return ADACOMP_EINVAL;
    if (rule > ADACOMP_RULE_LOCAL_SELECTION || !(soft_factor >= 1.0f && soft_factor <= 16.0f)) return ADACOMP_EINVAL;
    for (uint32_t k = 0; k < n_learners; ++k) {
        if (!grads[k] || !residues[k] || !packets_out[k] || grads[k] == residues[k]) return ADACOMP_EINVAL;
        if (reinterpret_cast<uintptr_t>(grads[k]) % 16 || reinterpret_cast<uintptr_t>(residues[k]) % 16 ||
            reinterpret_cast<uintptr_t>(packets_out[k]) % 16)
            return ADACOMP_EALIGN;
        for (uint32_t m = 0; m < k; ++m)
            if (residues[k] == residues[m] || packets_out[k] == packets_out[m]) return ADACOMP_EINVAL;
    }
    Plan p;
    int rc = find_plan(layers, n_layers, workspace, workspace_bytes, n_learners, p);
    if (rc != ADACOMP_OK) return rc;
    if (packet_capacity < p.fixed_bytes) return ADACOMP_ENOSPC;

    // Corrections that wait belong to the residue buffers of the call that left them: a lazy call
    // goes on with exactly those buffers, anything else has to wait for adacomp_residue_sync.
    bool corrections_wait = false;
    {
        std::lock_guard<std::mutex> lk(g_mu);
        auto it = g_ws.find(workspace);
        if (it == g_ws.end()) return ADACOMP_EWORKSPACE;  // released by another thread meanwhile
        const std::vector<float *> &waiting = it->second.waiting;
        if (!waiting.empty()) {
            if (!lazy || waiting.size() != n_learners) return ADACOMP_EPENDING;
            for (uint32_t k = 0; k < n_learners; ++k)
                if (waiting[k] != residues[k]) return ADACOMP_EPENDING;
            corrections_wait = true;
        }
    }

    char *ws = static_cast<char *>(workspace);
    CompressArgs a;
    a.lazy = corrections_wait ? 1u : 0u;
    a.place_mode = lazy ? kPlaceWords : kPlaceEager;
    a.tiles = reinterpret_cast<const TileDev *>(ws + p.ws.ctiles);
    a.layers = reinterpret_cast<const LayerDev *>(ws + p.ws.layers);
    a.scratch_stride = p.ws.scratch_stride;
    a.o_tile_out = uint32_t(p.ws.tile_out); a.o_layer_nsel = uint32_t(p.ws.layer_nsel);
    a.o_layer_scale = uint32_t(p.ws.layer_scale); a.o_gmax = uint32_t(p.ws.gmax);
    a.o_chunk_rel = uint32_t(p.ws.chunk_rel); a.o_stage = p.ws.stage;
    a.n_tiles = p.n_ctiles;
    a.n_layers = p.n_layers;
    a.keep_gmax = g_keep_gmax.load(std::memory_order_relaxed) ? 1u : 0u;
    a.class_tiles = (p.n_class_tiles[0] && p.n_class_tiles[1]) ? reinterpret_cast<const uint32_t *>(ws + p.ws.cclass) : nullptr;
    a.place_lanes = place_lanes_for(p);
    a.fold_scan = fold_scan_for(p) ? 1u : 0u;
    // tables with short bins send a large share of their elements: the eager placement then corrects
    // the residue tile by tile, whole lines at a time (k_place_tiled), instead of word by word
    a.place_tiled = (g_place_tiled.load(std::memory_order_relaxed) && p.has_short_bins && !a.fold_scan && !lazy) ? 1u : 0u;
    a.shift = (p.has_shifted_tiles && !corrections_wait) ? 1u : 0u;
    a.rule = rule;
    a.soft_factor_minus_1 = soft_factor - 1.0f;
    a.capacity = packet_capacity;
    a.fixed_bytes = p.fixed_bytes;

    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    // The streaming kernel runs a few percent faster per byte in launches of one learner than in one
    // launch over 16 learners of the 125 M-element workload (240 vs 246 us per learner), so large
    // gradients get one k_fused launch per learner and small ones share a launch; the scan and
    // placement kernels always cover all learners of the call.  The lazy variant of the kernel does
    // more before its first store and loses more at every launch boundary: two learners per launch
    // (or four) are 1.5 % faster per step there, and 0.3 % (1 %) slower on the eager path.
    const uint32_t per_launch_max = p.n_elems_total >= kSplitElems ? (lazy ? 2u : 1u) : kMaxBatch;
    a.fused_idle_lds = (per_launch_max == 1u && n_learners >= kFusedIdleMinLearners) ? kFusedIdleLds : 0u;
    auto enqueue = [&]() -> int {
    int rc = ADACOMP_OK;
    for (uint32_t done = 0; done < n_learners; done += kMaxBatch) {
        const uint32_t now = std::min(n_learners - done, kMaxBatch);
        a.n_learners = now;
        a.scratch = reinterpret_cast<uint8_t *>(ws + p.ws.scratch + p.ws.scratch_stride * done);
        for (uint32_t k = 0; k < kMaxBatch; ++k) {
            a.grad[k] = k < now ? grads[done + k] : nullptr;
            a.residue[k] = k < now ? residues[done + k] : nullptr;
            a.packet[k] = k < now ? static_cast<uint8_t *>(packets_out[done + k]) : nullptr;
        }
        for (uint32_t f = 0; f < now; f += per_launch_max) {
            a.fused_first = f;
            a.fused_count = std::min(per_launch_max, now - f);
            hipEvent_t ev_end = nullptr;   // set: this launch is bracketed by an event pair
            if (g_timing.on.load(std::memory_order_relaxed)) {
                std::lock_guard<std::mutex> lk(g_timing_mu);
                if (g_timing.on.load(std::memory_order_relaxed) && (g_timing.seen++ % g_timing.stride) == 0) {
                    if (g_timing.used == g_timing.pool.size()) {
                        hipEvent_t e0, e1;
                        if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return ADACOMP_EHIP;
                        g_timing.pool.emplace_back(e0, e1);
                    }
                    const std::pair<hipEvent_t, hipEvent_t> &ev = g_timing.pool[g_timing.used++];
                    g_timing.learners += a.fused_count;
                    if (hipEventRecord(ev.first, s) != hipSuccess) return ADACOMP_EHIP;
                    ev_end = ev.second;   // the handle itself: the pool may grow under another thread
                }
            }
            for (int c = 0; c < 2; ++c) {
                if (p.n_class_tiles[c] == 0) continue;
                a.class_first = c ? p.n_class_tiles[0] : 0u;
                a.class_count = p.n_class_tiles[c];
                if ((rc = launch_fused(a, c, hip_stream)) != ADACOMP_OK) return rc;
            }
            if (ev_end && hipEventRecord(ev_end, s) != hipSuccess) return ADACOMP_EHIP;
        }
        if (!a.fold_scan && (rc = launch_scan(a, hip_stream)) != ADACOMP_OK) return rc;
        if ((rc = launch_place(a, hip_stream)) != ADACOMP_OK) return rc;
    }
    return ADACOMP_OK;
    };
    rc = enqueue();
    if (lazy || corrections_wait) {
        // After a failure part of the way through, some kernels of this call may have applied and
        // overwritten the corrections that waited while others did not run: nothing can be said to
        // wait any more, and the residues are unspecified (as after a failed adacomp_residue_sync).
        std::lock_guard<std::mutex> lk(g_mu);
        auto it = g_ws.find(workspace);
        if (it != g_ws.end()) {
            if (rc == ADACOMP_OK) it->second.waiting.assign(residues, residues + n_learners);
            else it->second.waiting.clear();
        }
    }
    return rc;
}

int adacomp_compress_variant(const adacomp_layer_t *layers, uint32_t n_layers, uint32_t n_learners,
                             const float *const *grads, float *const *residues, void *const *packets_out,
                             size_t packet_capacity, uint32_t rule, float soft_factor, void *workspace,
                             size_t workspace_bytes, void *hip_stream)
{
    return compress_common(layers, n_layers, n_learners, grads, residues, packets_out, packet_capacity, rule,
                           soft_factor, false, workspace, workspace_bytes, hip_stream);
}

int adacomp_compress_batch_lazy(const adacomp_layer_t *layers, uint32_t n_layers, uint32_t n_learners,
                                const float *const *grads, float *const *residues, void *const *packets_out,
                                size_t packet_capacity, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return compress_common(layers, n_layers, n_learners, grads, residues, packets_out, packet_capacity,
                           ADACOMP_RULE_ADACOMP, 2.0f, true, workspace, workspace_bytes, hip_stream);
}

int adacomp_residue_sync(void *workspace, void *hip_stream)
{
    if (!workspace) return ADACOMP_EINVAL;
    Plan p;
    std::vector<float *> waiting;
    {
        std::lock_guard<std::mutex> lk(g_mu);
        auto it = g_ws.find(workspace);
        if (it == g_ws.end()) return ADACOMP_EWORKSPACE;
        if (it->second.waiting.empty()) return ADACOMP_OK;
        waiting = it->second.waiting;
        p.n_layers = it->second.plan.n_layers; p.n_ctiles = it->second.plan.n_ctiles;
        p.has_short_bins = it->second.plan.has_short_bins; p.ws = it->second.plan.ws;
    }
    char *ws = static_cast<char *>(workspace);
    CompressArgs a = {};
    a.tiles = reinterpret_cast<const TileDev *>(ws + p.ws.ctiles);
    a.layers = reinterpret_cast<const LayerDev *>(ws + p.ws.layers);
    a.scratch_stride = p.ws.scratch_stride;
    a.o_tile_out = uint32_t(p.ws.tile_out); a.o_layer_nsel = uint32_t(p.ws.layer_nsel);
    a.o_layer_scale = uint32_t(p.ws.layer_scale); a.o_gmax = uint32_t(p.ws.gmax);
    a.o_chunk_rel = uint32_t(p.ws.chunk_rel); a.o_stage = p.ws.stage;
    a.n_tiles = p.n_ctiles;
    a.n_layers = p.n_layers;
    a.place_lanes = place_lanes_for(p);
    a.place_mode = kPlaceResidue;
    const uint32_t n_learners = uint32_t(waiting.size());
    int rc = ADACOMP_OK;
    for (uint32_t done = 0; done < n_learners; done += kMaxBatch) {
        const uint32_t now = std::min(n_learners - done, kMaxBatch);
        a.n_learners = now;
        a.scratch = reinterpret_cast<uint8_t *>(ws + p.ws.scratch + p.ws.scratch_stride * done);
        for (uint32_t k = 0; k < kMaxBatch; ++k) a.residue[k] = k < now ? waiting[done + k] : nullptr;
        if ((rc = launch_place(a, hip_stream)) != ADACOMP_OK) break;
    }
    // after a failed launch some corrections may be applied and others not: nothing waits either way
    std::lock_guard<std::mutex> lk(g_mu);
    auto it = g_ws.find(workspace);
    if (it != g_ws.end()) it->second.waiting.clear();
    return rc;
}

int adacomp_compress_batch(const adacomp_layer_t *layers, uint32_t n_layers, uint32_t n_learners,
                           const float *const *grads, float *const *residues, void *const *packets_out,
                           size_t packet_capacity, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return adacomp_compress_variant(layers, n_layers, n_learners, grads, residues, packets_out, packet_capacity,
                                    ADACOMP_RULE_ADACOMP, 2.0f, workspace, workspace_bytes, hip_stream);
}

int adacomp_compress(const adacomp_layer_t *layers, uint32_t n_layers, const float *grad,
                     float *residue, void *packet_out, size_t packet_capacity, void *workspace,
                     size_t workspace_bytes, void *hip_stream)
{
    return adacomp_compress_batch(layers, n_layers, 1, &grad, &residue, &packet_out, packet_capacity,
                                  workspace, workspace_bytes, hip_stream);
}

// ---- the entry point that allocates nothing -----------------------------------------------------
// Its workspace is a file-scope device array.  Host code never uses the array's name as an address
// (on the host the name is only a handle for the runtime): the device address of this GPU's copy
// comes from hipGetSymbolAddress, once per device, and that pointer is what is registered as the
// workspace, copied to and handed to the kernels.
constexpr size_t kStaticScratchBytes = ADACOMP_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static std::mutex g_static_mu;
static void *g_static_ptr[kMaxDevices];  // per device: where that device holds `scratch`

static int static_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return ADACOMP_EHIP;
    std::lock_guard<std::mutex> lk(g_static_mu);
    if (!g_static_ptr[dev]) {   // first call on this device, which is current
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return ADACOMP_EHIP;
        if (reinterpret_cast<uintptr_t>(ptr) % 256 != 0) return ADACOMP_EALIGN;
        g_static_ptr[dev] = ptr;
    }
    *out = g_static_ptr[dev];
    return ADACOMP_OK;
}

int adacomp_compress_static(const adacomp_layer_t *layers, uint32_t n_layers, const float *grad, float *residue,
                            void *packet_out, size_t packet_capacity, void *hip_stream)
{
    if (!layers || n_layers == 0 || !grad || !residue || !packet_out) return ADACOMP_EINVAL;
    void *ws = nullptr;
    const int rc_dev = static_scratch(&ws);
    if (rc_dev == ADACOMP_OK) {
        // the usual case: this device's array already holds the tile tables of this layer table
        const int rc = adacomp_compress(layers, n_layers, grad, residue, packet_out, packet_capacity, ws,
                                        kStaticScratchBytes, hip_stream);
        if (rc != ADACOMP_EWORKSPACE) return rc;
    }
    // another layer table than the last call's on this device (or the first call): check it, see that
    // it fits, and write its tile tables into the array
    Plan p;
    int rc = build_plan(layers, n_layers, false, p);
    if (rc != ADACOMP_OK) return rc;
    if (p.ws.total(1) > kStaticScratchBytes) return ADACOMP_ETOOBIG;
    if (rc_dev != ADACOMP_OK) return rc_dev;
    if ((rc = adacomp_workspace_init(layers, n_layers, ws, kStaticScratchBytes, hip_stream)) != ADACOMP_OK) return rc;
    return adacomp_compress(layers, n_layers, grad, residue, packet_out, packet_capacity, ws, kStaticScratchBytes,
                            hip_stream);
}

static int unpack_common(const adacomp_layer_t *layers, uint32_t n_layers, const void *const *packets,
                         uint32_t n_learners, float *dense_out, float *weights, float *state1, float *state2,
                         const adacomp_optimizer_t *opt, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (n_learners > 0 && !packets) return ADACOMP_EINVAL;
    if (reinterpret_cast<uintptr_t>(dense_out) % 16) return ADACOMP_EALIGN;
    for (uint32_t k = 0; k < n_learners; ++k) {
        if (!packets[k]) return ADACOMP_EINVAL;
        if (reinterpret_cast<uintptr_t>(packets[k]) % 16) return ADACOMP_EALIGN;
    }
    Plan p;
    int rc = find_plan(layers, n_layers, workspace, workspace_bytes, 1, p);
    if (rc != ADACOMP_OK) return rc;

    char *ws = static_cast<char *>(workspace);
    UnpackArgs a;
    a.tiles = reinterpret_cast<const UTileDev *>(ws + p.ws.utiles);
    a.layers = reinterpret_cast<const LayerDev *>(ws + p.ws.layers);
    a.dense = dense_out;
    a.n_tiles = p.n_utiles;
    a.n_layers = p.n_layers;
    a.weights = weights; a.state1 = state1; a.state2 = state2;
    a.n_average = float(n_learners);
    a.lr = a.p1 = a.p2 = a.one_minus_p1 = a.one_minus_p2 = a.eps = 0.f;
    a.bias1 = a.bias2 = 1.f;
    if (opt) {
        a.lr = opt->lr;
        if (opt->kind == ADACOMP_OPT_SGD_MOMENTUM) a.p1 = opt->momentum;
        else {
            a.p1 = opt->beta1; a.p2 = opt->beta2;
            a.one_minus_p1 = 1.0f - opt->beta1; a.one_minus_p2 = 1.0f - opt->beta2;
            a.eps = opt->eps; a.bias1 = opt->bias1; a.bias2 = opt->bias2;
        }
    }
    uint32_t done = 0;
    do {  // 64 learners per launch; later launches add onto the stored partial sum, same order;
          // the update is applied by the last launch, when the sum is complete
        const uint32_t now = std::min(n_learners - done, kMaxPacketArgs);
        const bool last = done + now == n_learners;
        a.n_learners = now;
        a.accumulate = done > 0;
        a.mode = (opt && last) ? opt->kind : 0u;
        a.write_dense = dense_out != nullptr;
        for (uint32_t k = 0; k < kMaxPacketArgs; ++k)
            a.packets[k] = k < now ? static_cast<const uint8_t *>(packets[done + k]) : nullptr;
        // runs of tiles per workgroup for the plain sum, single tiles when the optimizer step follows
        const UGroupDev *table = reinterpret_cast<const UGroupDev *>(ws + (a.mode == 0u ? p.ws.ugroups : p.ws.usingles));
        const uint32_t n_all = a.mode == 0u ? p.n_ugroups : p.n_utiles, n8 = a.mode == 0u ? p.n_ugroups8 : p.n_usingles8;
        a.groups = table;
        a.n_groups = n_all;
        if (n8 == 0u || n8 == n_all) {  // one word width
            if ((rc = launch_unpack(a, n8 ? 1 : 0, hip_stream)) != ADACOMP_OK) return rc;
        } else if (p.n_utiles <= kUnpackSplitTiles) {  // small and mixed: one launch that handles both
            if ((rc = launch_unpack(a, 2, hip_stream)) != ADACOMP_OK) return rc;
        } else {  // large and mixed: the 8-bit groups come first in the table
            a.n_groups = n8;
            if ((rc = launch_unpack(a, 1, hip_stream)) != ADACOMP_OK) return rc;
            a.groups = table + n8;
            a.n_groups = n_all - n8;
            if ((rc = launch_unpack(a, 0, hip_stream)) != ADACOMP_OK) return rc;
        }
        done += now;
    } while (done < n_learners);
    return ADACOMP_OK;
}

int adacomp_unpack_accumulate(const adacomp_layer_t *layers, uint32_t n_layers,
                              const void *const *packets, uint32_t n_learners, float *dense_out,
                              void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!dense_out) return ADACOMP_EINVAL;
    return unpack_common(layers, n_layers, packets, n_learners, dense_out, nullptr, nullptr, nullptr, nullptr,
                         workspace, workspace_bytes, hip_stream);
}

int adacomp_unpack_update(const adacomp_layer_t *layers, uint32_t n_layers, const void *const *packets,
                          uint32_t n_learners, float *dense_out, float *weights, float *state1, float *state2,
                          const adacomp_optimizer_t *opt, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!opt || !weights || !state1 || n_learners == 0) return ADACOMP_EINVAL;
    if (opt->kind != ADACOMP_OPT_SGD_MOMENTUM && opt->kind != ADACOMP_OPT_ADAM) return ADACOMP_EINVAL;
    if (opt->kind == ADACOMP_OPT_ADAM && (!state2 || !(opt->bias1 > 0.f) || !(opt->bias2 > 0.f))) return ADACOMP_EINVAL;
    if (!dense_out && n_learners > kMaxPacketArgs) return ADACOMP_EINVAL;  // the partial sums need a home
    if (reinterpret_cast<uintptr_t>(weights) % 16 || reinterpret_cast<uintptr_t>(state1) % 16 ||
        reinterpret_cast<uintptr_t>(state2) % 16)
        return ADACOMP_EALIGN;
    if (weights == state1 || weights == state2 || state1 == state2 || dense_out == weights || dense_out == state1 ||
        (dense_out && dense_out == state2))
        return ADACOMP_EINVAL;
    return unpack_common(layers, n_layers, packets, n_learners, dense_out, weights, state1, state2, opt, workspace,
                         workspace_bytes, hip_stream);
}

const char *adacomp_strerror(int code)
{
    switch (code) {
    case ADACOMP_OK: return "ok";
    case ADACOMP_EINVAL: return "invalid argument (null pointer, empty or overlapping layer, aliasing buffers)";
    case ADACOMP_EBADLT: return "L_T must be in 1..16384";
    case ADACOMP_EALIGN: return "elem_offset must be a multiple of 4 and buffers 16-byte aligned (workspace 256)";
    case ADACOMP_ENOSPC: return "packet capacity below the fixed part of the packet";
    case ADACOMP_EHIP: return "HIP runtime error (no device or failed launch)";
    case ADACOMP_EWORKSPACE: return "workspace too small or not initialised for this layer table";
    case ADACOMP_EPENDING: return "residue corrections of a lazy call wait in this workspace: go on with the same lazy call or call adacomp_residue_sync";
    case ADACOMP_ETOOBIG: return "layer table needs more workspace than the static scratch array holds (16 MiB): use adacomp_compress with a workspace of the caller's";
    default: return "unknown adacomp error";
    }
}

int adacomp_copy_f32(float *dst, const float *src, size_t n, void *hip_stream)
{
    if (!dst || !src) return ADACOMP_EINVAL;
    if (reinterpret_cast<uintptr_t>(dst) % 16 || reinterpret_cast<uintptr_t>(src) % 16) return ADACOMP_EALIGN;
    return n == 0 ? ADACOMP_OK : launch_copy(dst, src, n, hip_stream);
}

int adacomp_triad_resident_f32(float *x, const float *y, size_t n, uint32_t workgroups_per_cu, void *hip_stream)
{
    if (!x || !y || x == y || workgroups_per_cu < 3 || workgroups_per_cu > 8) return ADACOMP_EINVAL;
    if (reinterpret_cast<uintptr_t>(x) % 16 || reinterpret_cast<uintptr_t>(y) % 16 || n % 4 != 0) return ADACOMP_EALIGN;
    if (n >= (size_t(1) << 43)) return ADACOMP_EINVAL;
    return n == 0 ? ADACOMP_OK : launch_triad(x, y, n, workgroups_per_cu, hip_stream);
}

int adacomp_triad_f32(float *x, const float *y, size_t n, void *hip_stream)
{
    return adacomp_triad_resident_f32(x, y, n, 8, hip_stream);
}

int adacomp_fill_f32(float *x, float value, size_t n, void *hip_stream)
{
    if (!x) return ADACOMP_EINVAL;
    if (reinterpret_cast<uintptr_t>(x) % 16 || n % 4 != 0) return ADACOMP_EALIGN;
    if (n >= (size_t(1) << 43)) return ADACOMP_EINVAL;
    return n == 0 ? ADACOMP_OK : launch_fill(x, value, n, hip_stream);
}

int adacomp_selftest_binindex(void)
{
    for (uint32_t T = 2; T <= ADACOMP_LT_MAX; ++T) {
        const uint32_t m = bin_magic(T);
        uint32_t q = 0, r = 0;  // running e / T, e % T
        for (uint32_t e = 0; e < 16384u; ++e) {
            if (uint32_t((uint64_t(e) * m) >> 32) != q) return -1;
            if (++r == T) { r = 0; ++q; }
        }
    }
    return 0;
}

int adacomp_debug_keep_gmax(int enable)
{
    g_keep_gmax = enable != 0;
    return ADACOMP_OK;
}

int adacomp_tuning_fold_scan(int enable)
{
    g_fold_scan = enable != 0;
    return ADACOMP_OK;
}

int adacomp_tuning_place_tiled(int enable)
{
    g_place_tiled = enable != 0;
    return ADACOMP_OK;
}

int adacomp_tuning_unpack_min_groups(uint32_t n_groups)
{
    g_unpack_min_groups = n_groups ? n_groups : kUnpackMinGroups;
    return ADACOMP_OK;
}

int adacomp_timing_enable(int enable)
{
    std::lock_guard<std::mutex> lk(g_timing_mu);
    g_timing.on = enable != 0;
    g_timing.stride = enable > 0 ? uint32_t(enable) : 1u;
    g_timing.used = 0;
    g_timing.learners = 0;
    g_timing.seen = 0;
    return ADACOMP_OK;
}

int adacomp_timing_read(double *total_ms, uint64_t *n_launches, uint64_t *n_learners)
{
    if (!total_ms || !n_launches || !n_learners) return ADACOMP_EINVAL;
    std::lock_guard<std::mutex> lk(g_timing_mu);
    double sum = 0.0;
    for (size_t i = 0; i < g_timing.used; ++i) {
        float ms = 0.f;
        if (hipEventSynchronize(g_timing.pool[i].second) != hipSuccess ||
            hipEventElapsedTime(&ms, g_timing.pool[i].first, g_timing.pool[i].second) != hipSuccess)
            return ADACOMP_EHIP;
        sum += ms;
    }
    *total_ms = sum;
    *n_launches = g_timing.used;
    *n_learners = g_timing.learners;
    g_timing.used = 0;
    g_timing.learners = 0;
    return ADACOMP_OK;
}

}  // extern "C"
