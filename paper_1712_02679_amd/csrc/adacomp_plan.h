// adacomp_plan.h -- host-side plan (tile tables, workspace layout) and the structures the
// kernels read from device memory.  Internal to libadacomp.
#pragma once

#include <cstddef>
#include <cstdint>
#include <vector>

#include "adacomp.h"

namespace adacomp {

constexpr uint32_t kWG = 256;            // threads per workgroup in every kernel (4 wave64)
constexpr uint32_t kMaxTileBins = 1024;  // bins per compress tile (LDS arrays)
constexpr uint32_t kFoldTiles = 512;     // tables up to this many compress tiles and
constexpr uint32_t kFoldLayers = 16;     // this many layers: the placement kernel does the scan itself
constexpr uint32_t kComputeUnits = 256;  // of an MI355X: what a small table's tiles are sized against
// elements per unpack tile: 16 KB of LDS accumulators (8192 was 10 % faster for the plain sum but
// 12 % slower with the optimizer epilogue)
constexpr uint32_t kUnpackTileElems = 4096;
constexpr uint32_t kLearnerGroup = 16;   // learners whose bin tables sit in LDS together in unpack
constexpr uint32_t kMaxPacketArgs = 64;  // packet pointers passed by value per unpack launch

// A layer as the kernels see it (64 bytes).
struct LayerDev {
    uint64_t elem_offset;
    uint64_t counts_offset;  // byte offsets inside a packet; fixed by the layer table alone
    uint64_t chunks_offset;
    uint32_t n_elems, L_T, n_bins, word_bytes;
    uint32_t ctile_start, n_ctiles;  // this layer's compress tiles in the tile table
    uint32_t bin_start, chunk_start; // first global bin / chunk index (g_max, chunk scratch arrays)
    uint32_t n_chunks, pad0;
};
static_assert(sizeof(LayerDev) == 64, "LayerDev layout");

// One workgroup's share of adacomp_compress: whole bins of one layer (32 bytes).
struct TileDev {
    uint64_t elem_base;   // first element in grad / residue (layer offset included)
    uint32_t stage_base;  // first entry of the tile's stretch of the staging array: the tiles' element counts,
                          // each rounded up to 4, summed over the tiles before it (so a multiple of 4)
    uint32_t L_T;
    uint32_t magic;       // floor(2^32 / L_T) + 1: bin = umulhi(e, magic) for e < 16384 (L_T > 1)
    uint16_t n_elems;     // elements in the tile, <= 4096 or 16384 by register class
    uint16_t n_bins;      // bins in the tile, <= kMaxTileBins
    uint32_t first_bin;   // index of the tile's first bin inside the layer
    uint32_t layer_flags; // bits 0..23 layer, bit 24 register class (0: 4096-element tiles, 1: 16384), bits 25..26 skip, bit 31 aligned
    __host__ __device__ uint32_t layer() const { return layer_flags & 0xFFFFFFu; }
    __host__ __device__ uint32_t jcode() const { return (layer_flags >> 24) & 1u; }
    // skip: for a tile of the larger class that is not 16-byte aligned but fits its class with the
    // misalignment added, the number of elements (1..3) between the 16-byte boundary below the tile
    // and its first element; 0 for aligned tiles and for unaligned ones that take 4-byte accesses
    __host__ __device__ uint32_t skip() const { return (layer_flags >> 25) & 3u; }
    __host__ __device__ bool aligned() const { return (layer_flags >> 31) != 0; }
};
static_assert(sizeof(TileDev) == 32, "TileDev layout");

// One workgroup's share of adacomp_unpack_accumulate: up to 64 whole bins inside one 64-bin
// chunk, or a slice [idx_lo, idx_lo + n_elems) of a single bin longer than the tile (32 bytes).
struct UTileDev {
    uint64_t elem_base;
    uint32_t n_elems;
    uint32_t L_T;
    uint32_t n_bins;
    uint32_t first_bin;
    uint32_t idx_lo;
    uint32_t layer_flags; // bits 0..23 layer, 24..27 log2(lanes per bin), bit 31 aligned
    __host__ __device__ uint32_t layer() const { return layer_flags & 0xFFFFFFu; }
    __host__ __device__ uint32_t group_log2() const { return (layer_flags >> 24) & 15u; }
    __host__ __device__ bool aligned() const { return (layer_flags >> 31) != 0; }
};
static_assert(sizeof(UTileDev) == 32, "UTileDev layout");

// Consecutive unpack tiles served by one workgroup: tiles of one 64-bin chunk, or slices of one bin.
struct UGroupDev {
    uint32_t first_tile, n_tiles;
};
static_assert(sizeof(UGroupDev) == 8, "UGroupDev layout");
constexpr uint32_t kUnpackGroupTiles = 8;   // at most this many tiles per group
constexpr uint32_t kUnpackMinGroups = 2048;  // groups of more than one tile only while this many workgroups remain (8 per compute unit)
constexpr uint32_t kUnpackSplitTiles = 2048;  // tables with both word widths and more tiles than this: one launch per width
constexpr uint32_t kUnpackTaperTiles = 768;  // tiles at the end of the table that go alone (3 per compute unit)

// What k_fused leaves per tile for k_scan and k_place: one 16-byte record, so that a tile makes one
// small store here instead of three.
struct TileOut {
    double gmax_sum;  // sum of the tile's g_max values
    uint32_t count;   // words the tile sends
    uint32_t base;    // words of the layer before this tile (written by k_scan)
};
static_assert(sizeof(TileOut) == 16, "TileOut layout");

// Byte offsets inside the caller's workspace.  The tables come first; then one scratch block per
// learner of a batched call (a single-learner call uses block 0).
struct WorkspaceLayout {
    size_t layers = 0, ctiles = 0, cclass = 0, utiles = 0, ugroups = 0, usingles = 0;  // tables written by workspace_init
    size_t scratch = 0;                                 // first scratch block
    size_t scratch_stride = 0;                          // bytes per learner
    // offsets inside a scratch block
    size_t tile_out = 0;                                // TileOut per compress tile
    size_t layer_nsel = 0, layer_scale = 0;             // per layer
    size_t gmax = 0, chunk_rel = 0;                     // per bin / per chunk
    size_t stage = 0;                                   // uint16 per element of the layers (not of the address span): words before placement
    size_t total(size_t n_learners) const { return scratch + scratch_stride * n_learners; }
};

struct Plan {
    uint32_t n_layers = 0;
    uint32_t n_ctiles = 0, n_utiles = 0, n_ugroups = 0;
    uint32_t n_ugroups8 = 0, n_usingles8 = 0;  // groups of layers with 8-bit words: they come first in both tables
    uint32_t n_bins_total = 0, n_chunks_total = 0;
    uint64_t elem_span = 0;     // max over layers of elem_offset + n_elems
    uint64_t n_elems_total = 0;
    uint64_t stage_entries = 0; // entries of the staging array: sum over the compress tiles of their element counts rounded up to 4
    uint64_t fixed_bytes = 0;   // packet bytes before the first word
    uint64_t bound_bytes = 0;   // packet bytes with every element sent
    uint32_t n_class_tiles[2] = {0, 0};  // compress tiles of 4096 / of 16384 elements
    std::vector<uint32_t> cclass;        // compress tile indices, the 4096-element ones first (tables with both kinds)
    bool has_short_bins = false;  // some layer has L_T <= 64 (8-bit words, many words per tile)
    bool has_shifted_tiles = false;  // some tile of the larger class has skip != 0
    WorkspaceLayout ws;
    std::vector<LayerDev> layers;
    std::vector<TileDev> ctiles;
    std::vector<UTileDev> utiles;
    std::vector<UGroupDev> ugroups, usingles;
};

// Validates the table (ADACOMP_E* on failure) and, with tables = true, fills the tile tables.
int build_plan(const adacomp_layer_t *layers, uint32_t n_layers, bool tables, Plan &plan);
uint32_t bin_magic(uint32_t L_T);
// Host bookkeeping of adacomp_workspace_init (which workspace holds the tile tables of which layer
// table) and the look-up every compute call starts with: ADACOMP_EWORKSPACE unless `workspace` was
// registered for exactly this list of layers and is large enough for n_learners scratch blocks.
void register_workspace(const adacomp_layer_t *layers, uint32_t n_layers, const void *workspace, size_t workspace_bytes,
                        Plan &&plan);
int find_plan(const adacomp_layer_t *layers, uint32_t n_layers, const void *workspace, size_t workspace_bytes,
              size_t n_learners, Plan &out);

// ---- kernel launchers (adacomp_kernels.hip) ---------------------------------------------------
constexpr uint32_t kMaxBatch = 32;  // learners per launch of the compress kernels
constexpr uint64_t kSplitElems = 32u * 1000u * 1000u;  // gradients at least this long: one k_fused launch per learner

// Dynamic LDS that no kernel touches, asked for with the launches of the eager 256-thread streaming
// kernel in calls that launch it once per learner, for many learners: with its 8.5 KB of arrays that leaves room for 6 workgroups per
// compute unit instead of the 8 its registers allow.  The kernel is bound by HBM, and HBM serves it
// better with fewer bytes in flight (a bare triad of the same shape gains up to 7 % between 8 and 4
// resident workgroups); since the layer record is fetched at the start of a workgroup and not in its
// tail, 6 workgroups still cover the LDS phases.  Measured per learner of the 125 M-element table,
// uncapped / capped: 235.5 / 247.9 us in calls of 1 learner, 243.3 / 251.2 of 2, 240.2 / 245.9 of 4,
// 242.1 / 239.0 of 8, 242.4 / 237.3 of 12, 243.8 / 238.0 of 16: a launch that follows another
// streaming launch gains, one that follows a placement and an unpack loses, hence the learner count.
// The kernel that first applies waiting corrections is longer per tile and loses with any cap.
constexpr uint32_t kFusedIdleLds = 18000;
constexpr uint32_t kFusedIdleMinLearners = 8;

struct CompressArgs {
    const TileDev *tiles;
    const LayerDev *layers;
    uint8_t *scratch;         // scratch block of learner 0 of this launch
    uint64_t scratch_stride;
    uint32_t o_tile_out, o_layer_nsel, o_layer_scale, o_gmax, o_chunk_rel;
    uint32_t n_tiles, n_layers, n_learners, keep_gmax;
    uint32_t fused_first, fused_count;  // learners covered by one k_fused launch
    const uint32_t *class_tiles;        // tile indices by register class, or null: the launch covers tiles 0 .. class_count - 1
    uint32_t class_first, class_count;  // this launch's stretch of class_tiles
    uint32_t place_lanes;               // lanes per tile in k_place: 16 or 64
    uint32_t place_mode;                // kPlaceEager / kPlaceWords / kPlaceResidue
    uint32_t fold_scan;                 // no k_scan launch: k_place computes word offsets and layer scales itself
    uint32_t place_tiled;               // the placement is k_place_tiled: one workgroup per tile, residue corrected line by line
    uint32_t lazy;                      // k_fused applies the waiting residue corrections of the previous call
    uint32_t shift;                     // the launch over the larger tiles uses the kernel that honours TileDev::skip
    uint32_t fused_idle_lds;            // bytes of dynamic LDS for the eager 256-thread k_fused launches (kFusedIdleLds or 0)
    uint32_t rule;                      // ADACOMP_RULE_*
    float soft_factor_minus_1;          // 1 for the paper's factor 2
    uint64_t o_stage;
    uint64_t capacity;        // bytes available in each packet buffer
    uint64_t fixed_bytes;
    const float *grad[kMaxBatch];
    float *residue[kMaxBatch];
    uint8_t *packet[kMaxBatch];
};

struct UnpackArgs {
    const UTileDev *tiles;
    const UGroupDev *groups;
    const LayerDev *layers;
    float *dense;
    uint32_t n_groups;
    uint32_t n_tiles, n_layers, n_learners, accumulate;
    uint32_t write_dense;              // 0: the sum is only consumed by the update
    uint32_t mode;                     // 0: sum only; 1: SGD with momentum; 2: Adam (applied by this launch)
    float *weights, *state1, *state2;  // momentum buffer, or Adam's m and v
    float n_average;                   // learner count the sum is divided by
    float lr, p1, p2, one_minus_p1, one_minus_p2, eps, bias1, bias2;
    const uint8_t *packets[kMaxPacketArgs];
};

int launch_fused(const CompressArgs &a, int jcode, void *stream);
int launch_scan(const CompressArgs &a, void *stream);
int launch_place(const CompressArgs &a, void *stream);
// what a k_place launch does: everything (the default); the words, offsets and header only, leaving
// the residue corrections waiting; or those corrections only
constexpr uint32_t kPlaceEager = 0, kPlaceWords = 1, kPlaceResidue = 2;
int launch_unpack(const UnpackArgs &a, int kind, void *stream);  // kind 0: 16-bit words, 1: 8-bit, 2: both
int launch_copy(float *dst, const float *src, size_t n, void *stream);
int launch_triad(float *x, const float *y, size_t n, uint32_t resident, void *stream);   // n a multiple of 4, below 2^44; resident 3 .. 8
int launch_fill(float *x, float value, size_t n, void *stream);

}  // namespace adacomp
