// adacomp_kernels.hip -- the hot path of libadacomp as hand-written HIP for gfx950 (CDNA4,
// wave64).  Everything here is bound by HBM traffic, not arithmetic: there is no dense
// contraction, hence no MFMA.  The floating-point work of the default method is single additions
// and subtractions in float32 (no multiplies, nothing to contract) plus one float64 sum and divide
// per layer; the soft-threshold factor of the variant entry point adds one multiply per element,
// the fused optimizer step a handful of separate float32 operations per element.
//
// adacomp_compress runs three launches:
//   k_fused  (streaming, dominant)  one pass over dW and the residue: G = R + dW, H = G + dW, the
//            per-bin maximum of |G|, the selection compare, and R <- G, all while the tile sits
//            in registers (Algorithm 2 of the AdaComp paper, both loops; selection is local to a
//            bin, so nothing outside the tile is needed).  Selected elements leave as 16-bit
//            (tile-local index, sign) entries in a staging area, counts per bin go straight into
//            the packet, g_max and its per-tile float64 sum go to scratch.
//   k_scan   one workgroup per layer: the layer scale = average of the g_max vector (section
//            "Pseudo code") and the exclusive scan of per-tile word counts.  (Small tables: no
//            launch; every k_place workgroup works these out itself.)
//   k_place  16 or 64 lanes per tile: moves the staged entries to their final place in the packet
//            as (index-in-bin, ternary code) words and applies the only step that needs the
//            layer-wide scale, residue <- G - Gq at the sent elements (a read-modify-write of
//            about 0.3-10 % of the elements); one extra workgroup writes header and records.
//            Large tables with short bins (L_T <= 64), which send several percent of their elements,
//            use k_place_tiled instead: a workgroup per tile, the residue corrected line by line.
// adacomp_compress_batch_lazy runs the same three, but k_place leaves that read-modify-write out
// and the next call's k_fused applies the corrections to the residue values while it has them in
// registers (same arithmetic, same results; adacomp_residue_sync writes them on request).
// adacomp_unpack_accumulate is one launch per word width, k_unpack: a workgroup owns a tile of the dense output
// in LDS, a lane group owns each bin and adds the learners' +-scale in learner order, then the
// tile is written out once with coalesced float4 stores; neighbouring tiles share a workgroup
// and the per-bin bookkeeping.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "adacomp_plan.h"

namespace adacomp {

// ---- small device helpers --------------------------------------------------------------------
// Streaming (non-temporal) 16-byte accesses: every element of dW and the residue is touched once
// per call, so nothing is gained by keeping it in L2, and on MI355X the streaming hint is worth
// about 15 % of bandwidth on a read-read-write pass.
typedef float vfloat4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ vfloat4 load_stream4(const float *p) { return __builtin_nontemporal_load(reinterpret_cast<const vfloat4 *>(p)); }
__device__ __forceinline__ void store_stream4(float *p, vfloat4 v) { __builtin_nontemporal_store(v, reinterpret_cast<vfloat4 *>(p)); }

// The same accesses as raw buffer instructions, for the Adam epilogue of k_unpack, which streams
// three arrays in and out per tile: addressing through a descriptor (scalar base, 32-bit offset)
// takes fewer registers there than 64-bit addresses, enough to stay within 80 without spilling,
// and the pass runs 4 % faster (k_fused and the plain sum measured the same with them, the
// SGD epilogue 4 % slower, so those keep global accesses).  A descriptor covers one tile:
// base = the tile's first element, size = its bytes; an access past the tile is dropped by the
// hardware.
typedef uint32_t vuint4 __attribute__((ext_vector_type(4)));
constexpr int kAuxStream = 2;  // cache-policy bits of a buffer access on gfx94x / gfx950: 1 = sc0, 2 = nt, 16 = sc1
__device__ __forceinline__ __amdgpu_buffer_rsrc_t tile_buffer(const float *base, uint32_t n_elems)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(base), 0, int(n_elems * 4u), 0x00020000);
}
__device__ __forceinline__ vfloat4 buffer_load_stream4(__amdgpu_buffer_rsrc_t rsrc, uint32_t elem)
{
    return __builtin_bit_cast(vfloat4, __builtin_amdgcn_raw_buffer_load_b128(rsrc, int(elem * 4u), 0, kAuxStream));
}
__device__ __forceinline__ void buffer_store_stream4(__amdgpu_buffer_rsrc_t rsrc, uint32_t elem, vfloat4 v)
{
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(vuint4, v), rsrc, int(elem * 4u), 0, kAuxStream);
}
// one element through the same descriptor (the first and last slot of a tile that is not 16-byte aligned)
__device__ __forceinline__ float buffer_load1(__amdgpu_buffer_rsrc_t rsrc, uint32_t elem)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrc, int(elem * 4u), 0, 0));
}
__device__ __forceinline__ void buffer_store1(__amdgpu_buffer_rsrc_t rsrc, uint32_t elem, float v)
{
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, v), rsrc, int(elem * 4u), 0, 0);
}

__device__ __forceinline__ uint32_t bin_of(uint32_t e, uint32_t L_T, uint32_t magic)
{
    return L_T == 1u ? e : __umulhi(e, magic);
}

// Inclusive prefix sum over the 64 lanes of a wave with DPP moves (no LDS traffic): four
// shift-and-add steps inside each row of 16 lanes, then the row totals are carried over with the
// two row broadcasts (lane 15 of rows 0 and 2 into rows 1 and 3, lane 31 into rows 2 and 3).
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v)
{
    v += uint32_t(__builtin_amdgcn_update_dpp(0, int(v), 0x111, 0xF, 0xF, false));  // row_shr:1
    v += uint32_t(__builtin_amdgcn_update_dpp(0, int(v), 0x112, 0xF, 0xF, false));  // row_shr:2
    v += uint32_t(__builtin_amdgcn_update_dpp(0, int(v), 0x114, 0xF, 0xF, false));  // row_shr:4
    v += uint32_t(__builtin_amdgcn_update_dpp(0, int(v), 0x118, 0xF, 0xF, false));  // row_shr:8
    v += uint32_t(__builtin_amdgcn_update_dpp(0, int(v), 0x142, 0xA, 0xF, false));  // row_bcast:15 -> rows 1, 3
    v += uint32_t(__builtin_amdgcn_update_dpp(0, int(v), 0x143, 0xC, 0xF, false));  // row_bcast:31 -> rows 2, 3
    return v;
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t v)
{
#pragma unroll
    for (uint32_t d = 32; d > 0; d >>= 1) v += __shfl_xor(v, d, 64);
    return v;
}

// Sum of one double per lane, fixed pairing (lane i with lane i + d): deterministic.
__device__ __forceinline__ double wave_sum_f64(double v)
{
#pragma unroll
    for (uint32_t d = 32; d > 0; d >>= 1) v += __shfl_down(v, d, 64);
    return v;  // valid in lane 0
}

// ==============================================================================================
// k_fused: Algorithm 2, both loops, on a tile of whole bins held in registers.
// Thread t owns float4 slots t, t + WG, ...: element e = 4 * (j * WG + t) + c of the tile, with WG = 256
// threads and 4 slots each for tiles of 4096 elements, 1024 threads and 4 slots each for tiles of 16384.
// ==============================================================================================
// VARIANT = false is the method as built by default (union rule, factor 2: additions only);
// VARIANT = true takes the selection rule and the soft-threshold factor from the arguments.
// LAZY = true: the residue corrections of the learner's previous call (residue <- G - Gq at the
// elements it sent) are still waiting in the scratch block instead of having been written (the host
// knows); they are applied here, to the residue values in registers, before anything else.
// SHIFT = true (launches over tiles of 16384 elements that hold bins of an odd length, or of twice an
// odd length): a tile that starts `skip` = 1..3 elements past a 16-byte boundary still moves whole
// 16-byte slots.  Slot q of the tile then covers the elements 4 q - skip .. 4 q + 3 - skip: the first
// slot begins in the tile before (those elements are left alone: loaded as zero, never stored) and
// everything after it is aligned.  With 4-byte accesses such tiles streamed at 44 % of the HBM peak.
template <int J, int WAVES, bool VARIANT, bool LAZY, bool SHIFT = false>
__global__ __launch_bounds__(WAVES * 64) void k_fused(const CompressArgs a)
{
    static_assert(!(SHIFT && LAZY), "the lazy kernel keeps 4-byte accesses on unaligned tiles");
    constexpr uint32_t WG = uint32_t(WAVES) * 64u;  // threads of the workgroup: a tile is J * WG float4 slots
    static_assert(J * WAVES <= 64, "the per-row word totals are scanned by one wave");
    // one-dimensional grid, learner-major: workgroups are dispatched in index order, so a batched
    // call streams one learner's buffers after the other instead of all of them at once.  A launch
    // covers the class_count tiles of one register class (all tiles, for most tables).
    const uint32_t lq = blockIdx.x / a.class_count;
    uint32_t pos = blockIdx.x - lq * a.class_count;
    const uint32_t lr = a.fused_first + lq;
    // Workgroups go to the 8 XCDs round-robin by index.  Inside each run of 64 the mapping is
    // transposed, so that the 8 workgroups landing on one XCD take 8 consecutive tiles (128 KB of
    // each stream): measured 6-9 % faster than the identity on a plain triad with these tiles,
    // and free of the slowdown of long launches.
    if (pos < (a.class_count & ~63u)) pos = (pos & ~63u) | ((pos & 7u) << 3) | ((pos >> 3) & 7u);
    const uint32_t tile = a.class_tiles ? a.class_tiles[a.class_first + pos] : pos;
    const TileDev td = a.tiles[tile];
    // The layer's record is needed only at the end, for the tile's outputs, but a dependent load in
    // the tail adds its whole latency to the life of the workgroup, so it is fetched early.  The
    // 256-thread kernel fetches it here, which holds its streaming loads back until the record is in
    // (they wait for the same counter as the buffer pointers); measured, that is as fast or faster
    // than the fetch behind the loads.  The 1024-thread kernel, of which a compute unit holds two
    // workgroups, cannot hide that wait (a third longer per launch) and fetches behind its loads
    // (2-4 % faster than in the tail).
    LayerDev ld;
    if (WAVES == 4) ld = a.layers[td.layer()];
    uint8_t *const sb = a.scratch + uint64_t(lr) * a.scratch_stride;
    TileOut *const tile_out = reinterpret_cast<TileOut *>(sb + a.o_tile_out);
    float *const gmax_out = reinterpret_cast<float *>(sb + a.o_gmax);
    uint32_t *const chunk_rel = reinterpret_cast<uint32_t *>(sb + a.o_chunk_rel);
    uint16_t *const stage_all = reinterpret_cast<uint16_t *>(sb + a.o_stage);
    uint8_t *const packet = a.packet[lr];

    __shared__ uint32_t s_gmax[kMaxTileBins];  // bit pattern of max |G|: for non-negative floats the
    __shared__ uint32_t s_cnt[kMaxTileBins];   // unsigned integer order is the float order
    __shared__ uint32_t s_wtot[64];
    __shared__ double s_red[WAVES];

    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform across the wave
    const uint32_t n = td.n_elems, T = td.L_T, M = td.magic, nb = td.n_bins;
    const uint32_t skip = SHIFT ? td.skip() : 0u;         // elements of the first slot that belong to the tile before
    const bool vec = td.aligned() || (SHIFT && skip != 0u);

    for (uint32_t i = tid; i < nb; i += WG) { s_gmax[i] = 0u; s_cnt[i] = 0u; }

    const float *__restrict__ gr = a.grad[lr] + td.elem_base;
    float *__restrict__ rs = a.residue[lr] + td.elem_base;

    // ---- G <- residue + dW ; H <- G + dW ; residue <- G (the "no transmission" value) ----------
    float r[J][4], w[J][4];
#pragma unroll
    for (int j = 0; j < J; ++j) {
        const uint32_t f0 = (uint32_t(j) * WG + tid) * 4u;
        const uint32_t e0 = f0 - skip;   // wraps to a huge value in the first slot of a shifted tile: its valid elements wrap back
        if (vec && f0 >= skip && e0 + 4u <= n) {
            const vfloat4 rv = load_stream4(rs + e0);
            const vfloat4 wv = load_stream4(gr + e0);
            r[j][0] = rv.x; r[j][1] = rv.y; r[j][2] = rv.z; r[j][3] = rv.w;
            w[j][0] = wv.x; w[j][1] = wv.y; w[j][2] = wv.z; w[j][3] = wv.w;
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const bool ok = e0 + uint32_t(c) < n;
                r[j][c] = ok ? rs[e0 + c] : 0.f;
                w[j][c] = ok ? gr[e0 + c] : 0.f;
            }
        }
    }
    if (WAVES != 4) ld = a.layers[td.layer()];
    if (LAZY) {
        // The previous call left, for this tile, its staged entries (tile-local index, sign), their
        // number and the layer's scale.  An entry becomes a code byte in LDS at the element's place;
        // every thread then reads the four codes of each of its slots and corrects its residues:
        // the same single float32 subtraction or addition that the eager placement performs.
        __shared__ __attribute__((aligned(16))) uint8_t s_fix[J * WG * 4];
        const uint32_t prev_count = tile_out[tile].count;
        const float prev_scale = reinterpret_cast<const float *>(sb + a.o_layer_scale)[td.layer()];
        for (uint32_t i = tid; i < uint32_t(J) * WG / 4u; i += WG) reinterpret_cast<uint4 *>(s_fix)[i] = make_uint4(0u, 0u, 0u, 0u);
        __syncthreads();
        // four entries per load: a tile's stretch of the staging area starts on an 8-byte boundary
        // (stretches are multiples of 4 entries) and what lies behind its last entry is readable
        const uint2 *prev_stage = reinterpret_cast<const uint2 *>(stage_all + td.stage_base);
        const uint32_t prev_n = prev_count < n ? prev_count : n;
        for (uint32_t q = tid; 4u * q < prev_n; q += WG) {
            const uint2 v = prev_stage[q];
            const uint32_t entry[4] = {v.x & 0xFFFFu, v.x >> 16, v.y & 0xFFFFu, v.y >> 16};
#pragma unroll
            for (uint32_t i = 0; i < 4u; ++i)
                if (4u * q + i < prev_n && (entry[i] >> 2) < n) s_fix[entry[i] >> 2] = uint8_t(entry[i] & 3u);
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < J; ++j) {
            const uint32_t e0 = (uint32_t(j) * WG + tid) * 4u;
            const uint32_t codes = *reinterpret_cast<const uint32_t *>(&s_fix[e0]);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t code = (codes >> (8 * c)) & 3u;
                if (code == 1u) r[j][c] = r[j][c] - prev_scale;
                else if (code == 3u) r[j][c] = r[j][c] + prev_scale;
            }
        }
    }
    uint32_t gb[J][4];  // bits of G (sign included)
    uint32_t mb[J][4];  // bits of max(|G|, |H|): what is compared with g_max
#pragma unroll
    for (int j = 0; j < J; ++j) {
        const uint32_t f0 = (uint32_t(j) * WG + tid) * 4u;
        const uint32_t e0 = f0 - skip;
        float G[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            G[c] = r[j][c] + w[j][c];
            float H;
            if (VARIANT) {
                const float extra = a.soft_factor_minus_1 * w[j][c];  // residue + f dW = G + (f - 1) dW
                H = G[c] + extra;
            } else {
                H = G[c] + w[j][c];
            }
            gb[j][c] = __float_as_uint(G[c]);
            const uint32_t ag = gb[j][c] & 0x7FFFFFFFu, ah = __float_as_uint(H) & 0x7FFFFFFFu;
            if (VARIANT && a.rule == ADACOMP_RULE_PRINTED_COMPARE) mb[j][c] = ah;          // |H| alone
            else if (VARIANT && a.rule == ADACOMP_RULE_LOCAL_SELECTION) mb[j][c] = ag;     // bin maxima only
            else mb[j][c] = ag > ah ? ag : ah;
        }
        if (vec && f0 >= skip && e0 + 4u <= n) {
            store_stream4(rs + e0, vfloat4{G[0], G[1], G[2], G[3]});
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (e0 + uint32_t(c) < n) rs[e0 + c] = G[c];
        }
    }

    __syncthreads();  // LDS arrays are zeroed

    // ---- first loop of Algorithm 2: g_max(i) per bin -------------------------------------------
#pragma unroll
    for (int j = 0; j < J; ++j) {
        const uint32_t f0 = (uint32_t(j) * WG + tid) * 4u;
        const uint32_t e0 = f0 - skip;
        if (WAVES == 16) {
            // Long bins: the 256 elements of a wave's row of slots nearly always lie in one bin, and
            // 64 lanes that bring their maxima to one LDS address are served one after the other
            // (2 cycles each, measured).  The wave reduces first; one lane goes to the LDS.
            const uint32_t w0f = (uint32_t(j) * WG + wave * 64u) * 4u;  // uniform: first slot of the row
            const uint32_t w0 = w0f - skip;                              // its first element (the row that holds a shifted tile's first slot takes the path below)
            if (w0f >= skip && w0 < n) {
                const uint32_t w1 = w0 + 255u < n ? w0 + 255u : n - 1u;
                const uint32_t bw = bin_of(w0, T, M);
                if (bw == bin_of(w1, T, M)) {
                    uint32_t m = gb[j][0] & 0x7FFFFFFFu;   // elements past n hold G = 0
#pragma unroll
                    for (int c = 1; c < 4; ++c) { const uint32_t v = gb[j][c] & 0x7FFFFFFFu; m = v > m ? v : m; }
#pragma unroll
                    for (uint32_t d = 32; d > 0; d >>= 1) { const uint32_t o = __shfl_xor(m, d, 64); m = o > m ? o : m; }
                    if (lane == 0) atomicMax(&s_gmax[bw], m);
                    continue;
                }
            }
        }
        if (SHIFT && f0 < skip) {   // the first slot of a shifted tile: only the elements from skip on are the tile's
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (e0 + uint32_t(c) < n) atomicMax(&s_gmax[bin_of(e0 + c, T, M)], gb[j][c] & 0x7FFFFFFFu);
        } else if (e0 < n) {
            const uint32_t e3 = e0 + 3u < n ? e0 + 3u : n - 1u;
            const uint32_t b0 = bin_of(e0, T, M), b3 = bin_of(e3, T, M);
            if (b0 == b3) {
                uint32_t m = gb[j][0] & 0x7FFFFFFFu;   // elements past n hold G = 0: they never raise a maximum
#pragma unroll
                for (int c = 1; c < 4; ++c) { const uint32_t v = gb[j][c] & 0x7FFFFFFFu; m = v > m ? v : m; }
                atomicMax(&s_gmax[b0], m);
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (e0 + uint32_t(c) < n) atomicMax(&s_gmax[bin_of(e0 + c, T, M)], gb[j][c] & 0x7FFFFFFFu);
            }
        }
    }
    __syncthreads();

    // ---- second loop: the local-max compare.  Sent iff G != 0 and max(|H|, |G|) >= g_max -------
    uint32_t before[J];  // sent elements of this wave's slot row that precede this lane
    uint32_t flags[J];   // bit c: element c of the slot is sent
    uint32_t wtot[J];
#pragma unroll
    for (int j = 0; j < J; ++j) {
        const uint32_t f0 = (uint32_t(j) * WG + tid) * 4u;
        const uint32_t e0 = f0 - skip;
        uint32_t f = 0u;
        if (e0 < n || (SHIFT && f0 < skip)) {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t e = e0 + uint32_t(c);
                if (e < n) {
                    const uint32_t gm = s_gmax[bin_of(e, T, M)];
                    // the printed compare alone also sends elements whose G is zero
                    const bool nonzero = (gb[j][c] & 0x7FFFFFFFu) != 0u ||
                                         (VARIANT && a.rule == ADACOMP_RULE_PRINTED_COMPARE);
                    const bool sent = nonzero && (mb[j][c] >= gm);
                    f |= sent ? (1u << c) : 0u;
                }
            }
        }
        flags[j] = f;
        uint32_t acc = 0u, tot = 0u;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint64_t m = __ballot((f >> c) & 1u);
            acc = __builtin_amdgcn_mbcnt_hi(uint32_t(m >> 32), __builtin_amdgcn_mbcnt_lo(uint32_t(m), acc));
            tot += uint32_t(__popcll(m));
        }
        before[j] = acc;
        wtot[j] = tot;
        if (lane == 0) s_wtot[j * WAVES + wave] = tot;
    }
    __syncthreads();

    // element order inside the tile is (j, wave, lane, c): exclusive prefix over the 4 J rows
    const uint32_t row_incl = wave_incl_scan(lane < uint32_t(WAVES * J) ? s_wtot[lane] : 0u);
    const uint32_t tile_total = __shfl(row_incl, WAVES * J - 1, 64);

    // ---- the pack vector of Algorithm 2: a sent element is staged as (tile-local index << 2 | code) --
    uint16_t *__restrict__ stage = stage_all + td.stage_base;
#pragma unroll
    for (int j = 0; j < J; ++j) {
        const uint32_t e0 = (uint32_t(j) * WG + tid) * 4u - skip;
        uint32_t pos = __shfl(row_incl, j * WAVES + int(wave), 64) - wtot[j] + before[j];
        const uint32_t f = flags[j];
        if (f) {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if ((f >> c) & 1u) {
                    const uint32_t e = e0 + uint32_t(c);
                    const uint32_t code = (gb[j][c] >> 31) ? 3u : 1u;  // ternary value: -scale / +scale
                    stage[pos] = uint16_t((e << 2) | code);
                    ++pos;
                    atomicAdd(&s_cnt[bin_of(e, T, M)], 1u);
                }
            }
        }
    }
    __syncthreads();

    // ---- tile outputs: counts (into the packet), g_max, sum of g_max, chunk prefixes, total ----
    if (ld.word_bytes == 1u) {
        uint8_t *cp = packet + ld.counts_offset + td.first_bin;
        for (uint32_t i = tid; i < nb; i += WG) cp[i] = uint8_t(s_cnt[i]);
    } else {
        uint16_t *cp = reinterpret_cast<uint16_t *>(packet + ld.counts_offset) + td.first_bin;
        for (uint32_t i = tid; i < nb; i += WG) cp[i] = uint16_t(s_cnt[i]);
    }
    double part = 0.0;
    float *gm_out = gmax_out + ld.bin_start + td.first_bin;
    for (uint32_t i = tid; i < nb; i += WG) {
        const float g = __uint_as_float(s_gmax[i]);
        if (a.keep_gmax) gm_out[i] = g;  // diagnostics only: no later kernel reads the g_max vector
        part += double(g);
    }
    part = wave_sum_f64(part);
    if (lane == 0) s_red[wave] = part;
    // running word count at every 64th bin of the layer that falls inside this tile
    const uint32_t t0 = (64u - (td.first_bin & 63u)) & 63u;
    for (uint32_t t = t0 + 64u * wave; t < nb; t += 64u * uint32_t(WAVES)) {
        uint32_t sum = 0u;
        for (uint32_t i = lane; i < t; i += 64u) sum += s_cnt[i];
        sum = wave_sum(sum);
        if (lane == 0) chunk_rel[ld.chunk_start + ((td.first_bin + t) >> 6)] = sum;
    }
    __syncthreads();
    if (tid == 0) {
        TileOut o;
        double sum = s_red[0];
        for (int wv = 1; wv < WAVES; ++wv) sum += s_red[wv];  // fixed order
        o.gmax_sum = sum;
        o.count = tile_total;
        o.base = 0u;  // filled in by k_scan
        tile_out[tile] = o;  // one 16-byte store
    }
}

// ==============================================================================================
// k_scan: per layer, scale = (sum of g_max) / n_bins in float64 rounded once to float32, and the
// exclusive scan of the tiles' word counts.  One workgroup of 1024 threads per layer; a thread
// owns a contiguous run of tiles so that its loads are independent and issue back to back.
// ==============================================================================================
constexpr uint32_t kScanWG = 1024;

__global__ __launch_bounds__(kScanWG) void k_scan(const CompressArgs a)
{
    const uint32_t l = blockIdx.x;
    if (l >= a.n_layers) return;
    // per-learner buffers: blockIdx.y selects the learner of a batched call
    const uint32_t lr = blockIdx.y;
    uint8_t *const sb = a.scratch + uint64_t(lr) * a.scratch_stride;
    TileOut *const tile_out = reinterpret_cast<TileOut *>(sb + a.o_tile_out);
    uint32_t *const layer_nsel = reinterpret_cast<uint32_t *>(sb + a.o_layer_nsel);
    float *const layer_scale = reinterpret_cast<float *>(sb + a.o_layer_scale);
    const LayerDev ld = a.layers[l];
    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform across the wave
    const uint32_t nt = ld.n_ctiles, ts = ld.ctile_start;
    const uint32_t per = (nt + kScanWG - 1) / kScanWG;
    const uint32_t lo = tid * per < nt ? tid * per : nt;
    const uint32_t hi = lo + per < nt ? lo + per : nt;

    __shared__ uint32_t s_wsum[16];
    __shared__ double s_dsum[16];

    // a thread's run of tiles is read once into registers when it is short (up to 8 records: layers of
    // up to 8192 tiles), so the kernel costs one memory round trip before the scan and one store after
    constexpr uint32_t kHold = 8;
    uint32_t cnt[kHold];
    uint32_t csum = 0u;
    double dsum = 0.0;
    if (per <= kHold) {
        TileOut rec[kHold];
#pragma unroll
        for (uint32_t i = 0; i < kHold; ++i) {
            rec[i].gmax_sum = 0.0; rec[i].count = 0u;
            if (lo + i < hi) rec[i] = tile_out[ts + lo + i];
        }
#pragma unroll
        for (uint32_t i = 0; i < kHold; ++i) { cnt[i] = rec[i].count; csum += rec[i].count; dsum += rec[i].gmax_sum; }
    } else {
        for (uint32_t i = lo; i < hi; ++i) { const TileOut o = tile_out[ts + i]; csum += o.count; dsum += o.gmax_sum; }
    }

    const uint32_t incl = wave_incl_scan(csum);
    dsum = wave_sum_f64(dsum);
    if (lane == 63) s_wsum[wave] = incl;
    if (lane == 0) s_dsum[wave] = dsum;
    __syncthreads();
    uint32_t wave_base = 0u;
    for (uint32_t wv = 0; wv < wave; ++wv) wave_base += s_wsum[wv];
    uint32_t run = wave_base + incl - csum;
    if (per <= kHold) {
#pragma unroll
        for (uint32_t i = 0; i < kHold; ++i)
            if (lo + i < hi) { tile_out[ts + lo + i].base = run; run += cnt[i]; }
    } else {
        for (uint32_t i = lo; i < hi; ++i) { tile_out[ts + i].base = run; run += tile_out[ts + i].count; }
    }
    if (tid == 0) {
        double total = 0.0;
        uint32_t nsel = 0u;
        for (uint32_t wv = 0; wv < kScanWG / 64u; ++wv) { total += s_dsum[wv]; nsel += s_wsum[wv]; }
        layer_scale[l] = float(total / double(ld.n_bins));
        layer_nsel[l] = nsel;
    }
}

// ==============================================================================================
// k_place: staged entries -> final words; residue <- G - Gq at the sent elements; chunk offsets;
// header, records and padding (last workgroup).  With long bins a tile sends a few dozen words at
// most in steady state, so 16 lanes serve a tile and a workgroup serves 16 tiles; the whole grid
// is resident at once and the kernel costs about three dependent memory round trips.  Its pace is
// set by the scattered read-modify-writes of the residue: a bare kernel that does nothing else
// needs as long for the same number of words.
// ==============================================================================================
__device__ __forceinline__ uint64_t pad16_dev(uint64_t x) { return (x + 15u) & ~uint64_t(15); }

// LANES lanes serve a tile: 16 where bins are long and a tile sends a few dozen words, 64 for tables
// with short bins, whose tiles send several hundred (5 % off the compress time of the ResNet-50
// table, 23 % off the small CIFAR table; 64 lanes cost the 125 M-element table half a percent).
// MODE kPlaceEager does all of it.  kPlaceWords leaves the residue alone: the corrections wait in
// the scratch block (staged entries, tile counts, layer scales) and the next lazy k_fused of this
// learner applies them in registers, where they cost next to nothing; until then the residue holds
// G at the sent elements.  kPlaceResidue applies waiting corrections and nothing else.
// FOLD = true (small tables: up to kFoldTiles tiles and kFoldLayers layers; 64 lanes per tile): there
// is no k_scan launch.  Every workgroup scans the word counts of all tiles itself (8 per thread, a
// few kilobytes from L2) and every wave sums the g_max totals of its tile's layer, in one fixed
// order (fold_layer_scale) that the header block uses as well; on tables that take 35-90 us per
// step this is cheaper than a launch of 4 us and the gap before it.
__device__ __forceinline__ float fold_layer_scale(const TileOut *tile_out, const uint32_t ctile_start,
                                                  const uint32_t n_ctiles, const uint32_t n_bins, const uint32_t lane)
{
    double s = 0.0;
    for (uint32_t t = lane; t < n_ctiles; t += 64u) s += tile_out[ctile_start + t].gmax_sum;
    s = wave_sum_f64(s);          // lane 0 holds the sum
    s = __shfl(s, 0, 64);
    return float(s / double(n_bins));
}

// Header, layer records and zero padding of one learner's packet, by one workgroup of kWG threads
// (the extra workgroup of a placement launch): 256 layers at a time, word offsets by a block scan
// of the padded section sizes (all below 2^32: the packet bound is).  FOLD: the layer totals come
// from s_excl (words of all tiles before each tile) and the scales are worked out here.
template <bool FOLD>
__device__ __forceinline__ void place_header(const CompressArgs &a, uint8_t *const packet, const TileOut *const tile_out,
                                             uint32_t *const layer_nsel, float *const layer_scale, const uint32_t *const s_excl)
{
    const uint32_t tid = threadIdx.x;
    __shared__ uint32_t s_wtot[4];
    __shared__ float s_fscale[FOLD ? kFoldLayers : 1u];
    const uint32_t lane = tid & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    if (FOLD) {
        for (uint32_t l = wave; l < a.n_layers; l += 4u) {
            const float sc = fold_layer_scale(tile_out, a.layers[l].ctile_start, a.layers[l].n_ctiles, a.layers[l].n_bins, lane);
            if (lane == 0u) s_fscale[l] = sc;
        }
        __syncthreads();
    }
    uint64_t carry = a.fixed_bytes, nsel_all = 0;
    for (uint32_t l0 = 0; l0 < a.n_layers; l0 += kWG) {
        const uint32_t l = l0 + tid;
        const bool live = l < a.n_layers;
        LayerDev ld;
        uint32_t nsel = 0u, bytes = 0u;
        float scale = 0.f;
        if (live) {
            ld = a.layers[l];
            if (FOLD) {   // and left in the scratch block for whoever applies the corrections later
                nsel = s_excl[ld.ctile_start + ld.n_ctiles] - s_excl[ld.ctile_start];
                scale = s_fscale[l];
                layer_nsel[l] = nsel;
                layer_scale[l] = scale;
            } else {
                nsel = layer_nsel[l];
                scale = layer_scale[l];
            }
            bytes = uint32_t(pad16_dev(uint64_t(nsel) * ld.word_bytes));
        }
        const uint32_t incl = wave_incl_scan(bytes);
        uint32_t nsum = wave_sum(nsel);
        __syncthreads();  // previous round's readers of s_wtot are done
        if (lane == 63) s_wtot[wave] = incl;
        __syncthreads();
        uint64_t before = carry;
        for (uint32_t wv = 0; wv < wave; ++wv) before += s_wtot[wv];
        const uint64_t woff = before + incl - bytes;
        carry += uint64_t(s_wtot[0]) + s_wtot[1] + s_wtot[2] + s_wtot[3];
        if (live) {
            adacomp_packet_layer_t rec;
            rec.elem_offset = ld.elem_offset; rec.n_elems = ld.n_elems;
            rec.L_T = ld.L_T; rec.n_bins = ld.n_bins; rec.word_bits = ld.word_bytes * 8u;
            rec.scale = scale;
            rec.n_selected = nsel;
            rec.counts_offset = ld.counts_offset; rec.chunks_offset = ld.chunks_offset; rec.words_offset = woff;
            reinterpret_cast<adacomp_packet_layer_t *>(packet + sizeof(adacomp_packet_header_t))[l] = rec;
            for (uint64_t b = ld.counts_offset + uint64_t(ld.n_bins) * ld.word_bytes; b < ld.chunks_offset; ++b) packet[b] = 0;
            const uint64_t chunks_end = ld.chunks_offset + 4ull * ld.n_chunks;
            for (uint64_t b = chunks_end; b < pad16_dev(chunks_end); ++b) packet[b] = 0;
            const uint64_t words_end = woff + uint64_t(nsel) * ld.word_bytes;
            for (uint64_t b = words_end; b < pad16_dev(words_end); ++b)
                if (b < a.capacity) packet[b] = 0;
        }
        // total word count: per-wave sums through the same LDS slots
        __syncthreads();
        if (lane == 0) s_wtot[wave] = nsum;
        __syncthreads();
        nsel_all += uint64_t(s_wtot[0]) + s_wtot[1] + s_wtot[2] + s_wtot[3];
    }
    if (tid == 0) {
        adacomp_packet_header_t h;
        h.magic = ADACOMP_PACKET_MAGIC; h.version = ADACOMP_PACKET_VERSION;
        h.status = carry > a.capacity ? ADACOMP_STATUS_TRUNCATED : ADACOMP_STATUS_COMPLETE;
        h.n_layers = a.n_layers; h.total_bytes = carry; h.n_selected = nsel_all;
        *reinterpret_cast<adacomp_packet_header_t *>(packet) = h;
    }
}

template <uint32_t LANES, uint32_t MODE, bool FOLD>
__global__ __launch_bounds__(kWG) void k_place(const CompressArgs a)
{
    static_assert(!FOLD || (LANES == 64u && MODE != kPlaceResidue), "the folded scan serves 64-lane placement launches");
    constexpr uint32_t kPlaceLanes = LANES, kPlaceTiles = kWG / LANES;
    const uint32_t tid = threadIdx.x;
    // per-learner buffers: blockIdx.y selects the learner of a batched call
    const uint32_t lr = blockIdx.y;
    uint8_t *const sb = a.scratch + uint64_t(lr) * a.scratch_stride;
    TileOut *const tile_out = reinterpret_cast<TileOut *>(sb + a.o_tile_out);
    uint32_t *const layer_nsel = reinterpret_cast<uint32_t *>(sb + a.o_layer_nsel);
    float *const layer_scale = reinterpret_cast<float *>(sb + a.o_layer_scale);
    uint32_t *const chunk_rel = reinterpret_cast<uint32_t *>(sb + a.o_chunk_rel);
    uint16_t *const stage_all = reinterpret_cast<uint16_t *>(sb + a.o_stage);
    uint8_t *const packet = a.packet[lr];

    // s_excl[t] = words of all tiles before tile t (tile table order: layer after layer)
    __shared__ uint32_t s_excl[FOLD ? kFoldTiles + 1u : 1u];
    if (FOLD) {
        __shared__ uint32_t s_fw[4];
        constexpr uint32_t kPer = kFoldTiles / kWG;
        const uint32_t lane = tid & 63u;
        const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
        uint32_t cnt[kPer], sum = 0u;
#pragma unroll
        for (uint32_t i = 0; i < kPer; ++i) {
            const uint32_t t = tid * kPer + i;
            cnt[i] = t < a.n_tiles ? tile_out[t].count : 0u;
            sum += cnt[i];
        }
        const uint32_t incl = wave_incl_scan(sum);
        if (lane == 63u) s_fw[wave] = incl;
        __syncthreads();
        uint32_t run = incl - sum;
        for (uint32_t wv = 0; wv < wave; ++wv) run += s_fw[wv];
#pragma unroll
        for (uint32_t i = 0; i < kPer; ++i) {
            s_excl[tid * kPer + i] = run;
            run += cnt[i];
        }
        if (tid == kWG - 1u) s_excl[kFoldTiles] = run;
        __syncthreads();
    }

    if (MODE == kPlaceResidue && blockIdx.x == gridDim.x - 1) return;
    if (MODE != kPlaceResidue && blockIdx.x == gridDim.x - 1) {
        place_header<FOLD>(a, packet, tile_out, layer_nsel, layer_scale, s_excl);
        return;
    }

    const uint32_t sub = tid & (kPlaceLanes - 1u);
    const uint32_t tile = blockIdx.x * kPlaceTiles + (tid / kPlaceLanes);
    if (tile >= a.n_tiles) return;
    const TileDev td = a.tiles[tile];
    const uint32_t l = td.layer();

    // independent loads first: the tile's counters, its first staged entries, the layer's fields
    const TileOut to = tile_out[tile];
    const uint32_t cnt = to.count;
    const uint32_t base = FOLD ? s_excl[tile] - s_excl[a.layers[l].ctile_start] : to.base;
    const uint16_t *__restrict__ stage = stage_all + td.stage_base;
    float *__restrict__ rs = a.residue[lr] + td.elem_base;
    const uint32_t s_first = stage[sub];  // speculative: the staging array has 64 entries of slack
    const float scale = FOLD ? fold_layer_scale(tile_out, a.layers[l].ctile_start, a.layers[l].n_ctiles, a.layers[l].n_bins, sub)
                             : layer_scale[l];
    const uint32_t wbytes = a.layers[l].word_bytes;
    const uint64_t chunks_offset = a.layers[l].chunks_offset;
    const uint32_t chunk_start = a.layers[l].chunk_start;

    // first word of this layer = end of the fixed part + the (padded) word sections before it
    uint64_t woff = 0;
    for (uint32_t m = sub; m < l; m += kPlaceLanes) {
        const uint32_t nsel_m = FOLD ? s_excl[a.layers[m].ctile_start + a.layers[m].n_ctiles] - s_excl[a.layers[m].ctile_start]
                                     : layer_nsel[m];
        woff += pad16_dev(uint64_t(nsel_m) * a.layers[m].word_bytes);
    }
#pragma unroll
    for (uint32_t d = kPlaceLanes / 2; d > 0; d >>= 1) {
        const uint32_t lo = __shfl_xor(uint32_t(woff), d, kPlaceLanes), hi = __shfl_xor(uint32_t(woff >> 32), d, kPlaceLanes);
        woff += (uint64_t(hi) << 32) | lo;
    }
    woff += a.fixed_bytes;

    // Eight words per lane and round, so that a tile with hundreds of words (short bins send several
    // percent of their elements) costs a few memory round trips instead of one per 16 words.
    const uint32_t T = td.L_T, M = td.magic;
    constexpr uint32_t kU = 8;
    for (uint32_t p0 = sub; p0 < cnt; p0 += kPlaceLanes * kU) {
        uint32_t s[kU];
        float g[kU];
#pragma unroll
        for (uint32_t u = 0; u < kU; ++u) {
            const uint32_t p = p0 + kPlaceLanes * u;
            s[u] = p < cnt ? (p == sub ? s_first : uint32_t(stage[p])) : 0u;  // 0: code 0, never a real entry
        }
        // The sent elements' residue update of Algorithm 2: G minus sign(G) * scale; G is what k_fused left in the
        // residue: a read-modify-write, measured at a 64-byte read and a 32-byte write per word.
        // (Keeping G next to the staged entry, so that this becomes a plain store, was built and
        // measured three times: in an array of its own for all layers, for short-bin layers only,
        // and as 8-byte entries in the same staging stretch.  The scattered partial writes, not
        // the reads, set the pace here, and k_fused lost more to the wider staging stores, about
        // 1 %, than this kernel gained.)
#pragma unroll
        for (uint32_t u = 0; u < kU; ++u)
            g[u] = (MODE != kPlaceWords && (s[u] & 1u)) ? rs[s[u] >> 2] : 0.f;
#pragma unroll
        for (uint32_t u = 0; u < kU; ++u) {
            if (!(s[u] & 1u)) continue;  // codes are 1 or 3
            const uint32_t p = p0 + kPlaceLanes * u;
            const uint32_t e = s[u] >> 2, code = s[u] & 3u;
            if (MODE != kPlaceResidue) {
                const uint32_t b = bin_of(e, T, M);
                const uint32_t word = ((e - b * T) << 2) | code;  // index inside the bin, ternary code
                const uint64_t at = woff + uint64_t(base + p) * wbytes;
                if (at + wbytes <= a.capacity) {
                    if (wbytes == 1u) packet[at] = uint8_t(word);
                    else *reinterpret_cast<uint16_t *>(packet + at) = uint16_t(word);
                }
            }
            if (MODE != kPlaceWords) rs[e] = code == 1u ? g[u] - scale : g[u] + scale;
        }
    }
    if (MODE == kPlaceResidue) return;

    // chunks[c] = words of the layer in bins < 64 c, for the chunk starts inside this tile
    const uint32_t t0 = (64u - (td.first_bin & 63u)) & 63u;
    for (uint32_t t = t0 + 64u * sub; t < td.n_bins; t += 64u * kPlaceLanes) {
        const uint32_t c = (td.first_bin + t) >> 6;
        reinterpret_cast<uint32_t *>(packet + chunks_offset)[c] = base + chunk_rel[chunk_start + c];
    }
}

// ==============================================================================================
// k_place_tiled: the eager placement for tables with short bins.  Where L_T <= 64 several percent of
// the elements are sent (7.9 % on the ResNet-50 table) and three quarters of the residue's 64-byte
// lines hold a sent element, so correcting the residue word by word (a scattered read-modify-write
// per word, as k_place does) moves far more than the lines themselves.  Here a workgroup owns one
// compress tile: it places the tile's words, marks the sent elements in an LDS byte map (the
// scheme of the lazy k_fused), and then streams over the tile's residue line by line: a line with a
// mark is loaded whole, corrected with the same single float32 subtraction or addition, and written
// back whole; a line without one is not touched.  Tiles that send only a few words (the fully
// connected layers of such a table) and tiles that are not 16-byte aligned correct word by word.
// ==============================================================================================
constexpr uint32_t kTiledMinWords = 24;  // fewer words than this in a tile: word-by-word corrections

__global__ __launch_bounds__(kWG) void k_place_tiled(const CompressArgs a)
{
    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t lr = blockIdx.y;   // the learner of a batched call
    uint8_t *const sb = a.scratch + uint64_t(lr) * a.scratch_stride;
    TileOut *const tile_out = reinterpret_cast<TileOut *>(sb + a.o_tile_out);
    uint32_t *const layer_nsel = reinterpret_cast<uint32_t *>(sb + a.o_layer_nsel);
    float *const layer_scale = reinterpret_cast<float *>(sb + a.o_layer_scale);
    const uint32_t *const chunk_rel = reinterpret_cast<const uint32_t *>(sb + a.o_chunk_rel);
    const uint16_t *const stage_all = reinterpret_cast<const uint16_t *>(sb + a.o_stage);
    uint8_t *const packet = a.packet[lr];

    if (blockIdx.x == gridDim.x - 1) {
        place_header<false>(a, packet, tile_out, layer_nsel, layer_scale, nullptr);
        return;
    }
    const uint32_t tile = blockIdx.x;   // the grid has one workgroup per tile and one for the header
    const TileDev td = a.tiles[tile];
    const uint32_t l = td.layer();
    const TileOut to = tile_out[tile];
    const uint32_t cnt = to.count, base = to.base;
    const uint32_t n = td.n_elems, T = td.L_T, M = td.magic;
    const float scale = layer_scale[l];
    const uint32_t wbytes = a.layers[l].word_bytes;
    const uint64_t chunks_offset = a.layers[l].chunks_offset;
    const uint32_t chunk_start = a.layers[l].chunk_start;
    const uint16_t *__restrict__ stage = stage_all + td.stage_base;
    float *__restrict__ rs = a.residue[lr] + td.elem_base;
    const bool tiled = td.aligned() && cnt >= kTiledMinWords;   // uniform over the workgroup

    __shared__ __attribute__((aligned(16))) uint8_t s_fix[16384];   // code of the word an element was sent with, or 0
    __shared__ uint64_t s_part[kWG / 64u];
    if (tiled)
        for (uint32_t i = tid; i < (n + 15u) / 16u; i += kWG) reinterpret_cast<uint4 *>(s_fix)[i] = make_uint4(0u, 0u, 0u, 0u);

    // first word of this layer = end of the fixed part + the (padded) word sections before it
    uint64_t part = 0;
    for (uint32_t m = tid; m < l; m += kWG) part += pad16_dev(uint64_t(layer_nsel[m]) * a.layers[m].word_bytes);
#pragma unroll
    for (uint32_t d = 32; d > 0; d >>= 1) {
        const uint32_t lo = __shfl_xor(uint32_t(part), d, 64), hi = __shfl_xor(uint32_t(part >> 32), d, 64);
        part += (uint64_t(hi) << 32) | lo;
    }
    if (lane == 0) s_part[wave] = part;
    __syncthreads();   // the byte map is cleared, the partial sums are there
    uint64_t woff = a.fixed_bytes;
    for (uint32_t wv = 0; wv < kWG / 64u; ++wv) woff += s_part[wv];

    for (uint32_t p = tid; p < cnt; p += kWG) {
        const uint32_t s = stage[p];
        const uint32_t e = s >> 2, code = s & 3u;
        if (!(code & 1u) || e >= n) continue;   // codes are 1 or 3 and indices lie inside the tile
        const uint32_t b = bin_of(e, T, M);
        const uint32_t word = ((e - b * T) << 2) | code;   // index inside the bin, ternary code
        const uint64_t at = woff + uint64_t(base + p) * wbytes;
        if (at + wbytes <= a.capacity) {
            if (wbytes == 1u) packet[at] = uint8_t(word);
            else *reinterpret_cast<uint16_t *>(packet + at) = uint16_t(word);
        }
        if (tiled) s_fix[e] = uint8_t(code);
        else {   // the sent elements' residue update of Algorithm 2, one element at a time
            const float g = rs[e];
            rs[e] = code == 1u ? g - scale : g + scale;
        }
    }

    if (tiled) {
        __syncthreads();   // the byte map is complete
        // Lines of the residue: four consecutive 16-byte slots, the first on a 64-byte boundary.  The
        // tile starts `shift` slots past such a boundary; virtual slot v = shift + (slot in the tile),
        // so that the four lanes v & ~3 .. v | 3 share a line and decide together.
        const uint32_t shift = uint32_t(reinterpret_cast<uintptr_t>(rs) >> 4) & 3u;
        const uint32_t n_virtual = (shift + (n + 3u) / 4u + 3u) & ~3u;
        for (uint32_t v = tid; v < n_virtual; v += kWG) {
            const uint32_t e0 = (v - shift) * 4u;   // wraps to a huge value below the tile's start
            const bool ok = v >= shift && e0 < n;
            const uint32_t codes = ok ? *reinterpret_cast<const uint32_t *>(&s_fix[e0]) : 0u;   // bytes past n are 0
            uint32_t any = codes;
            any |= uint32_t(__shfl_xor(int(any), 1, 64));
            any |= uint32_t(__shfl_xor(int(any), 2, 64));
            if (!ok || any == 0u) continue;
            if (e0 + 4u <= n) {
                const vfloat4 r = load_stream4(rs + e0);
                float g[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const uint32_t code = (codes >> (8 * c)) & 3u;
                    if (code == 1u) g[c] = g[c] - scale;
                    else if (code == 3u) g[c] = g[c] + scale;
                }
                store_stream4(rs + e0, vfloat4{g[0], g[1], g[2], g[3]});
            } else {   // the layer's last elements: what follows them is not ours to write
                for (uint32_t c = 0; c < 4u && e0 + c < n; ++c) {
                    const uint32_t code = (codes >> (8u * c)) & 3u;
                    if (code == 1u) rs[e0 + c] = rs[e0 + c] - scale;
                    else if (code == 3u) rs[e0 + c] = rs[e0 + c] + scale;
                }
            }
        }
    }

    // chunks[c] = words of the layer in bins < 64 c, for the chunk starts inside this tile
    const uint32_t t0 = (64u - (td.first_bin & 63u)) & 63u;
    for (uint32_t t = t0 + 64u * tid; t < td.n_bins; t += 64u * kWG) {
        const uint32_t c = (td.first_bin + t) >> 6;
        reinterpret_cast<uint32_t *>(packet + chunks_offset)[c] = base + chunk_rel[chunk_start + c];
    }
}

// ==============================================================================================
// k_unpack: dense_out <- sum over learners, in learner order, of the decoded packets.
// A workgroup owns a tile of the output in LDS, and serves a run of up to 8 neighbouring tiles one
// after the other.  Phase 1 gathers, for every (bin, learner) of the run, the word count and the
// position of the first word (one wave per learner, all learners' loads in flight together); with
// up to 16 learners this is done once per run, which is what the runs are for: at L_T = 500 the
// 8 tiles of a 64-bin chunk need the same count lines and the same prefix sums.  Phase 2, per
// tile: a lane group per bin reads the 16 learners' table entries with a few wide LDS loads,
// fetches the words of all 16 learners, and adds +-scale in learner order: with LDS float atomics
// where bins are long and few lanes have a word, with plain LDS loads and stores where bins are
// short (see lds_add).  All adds to one address come from one wave in program order and the LDS
// unit executes a wave's operations in order, so the sum order is fixed: learner 0 first.  (LDS
// float adds round to nearest even and keep denormals, like v_add_f32.)  On the 125 M-element table with 16 learners
// a pass that only clears and writes the tiles takes 88 us, phase 1 per tile added 79 us and
// phase 2 adds 63 us; sharing phase 1 over a run brought the whole launch from 230-250 to 185 us.
// ==============================================================================================
// Row strides of the two LDS tables.  With the natural strides (16 words, 8 words) the 64 lanes of
// phase 1, which write one row each, would hit 2 and 4 of the 32 banks; 20 and 12 words spread
// them over 8 banks and keep the rows 16-byte aligned for the wide reads of phase 2.
constexpr uint32_t kOffStride = 20;  // uint32 per row, 16 used
constexpr uint32_t kCntStride = 24;  // uint16 per row, 16 used

// Phase 1 for learners k0 .. k0 + 15 and the bins [row0_bin, scan_end) of one 64-bin chunk: word
// count and position of the first word of every (bin, learner), into the LDS tables (row = bin -
// row0_bin).  The caller has a barrier before (the tables are free) and after (they are filled).
template <bool W8>
__device__ __forceinline__ void unpack_tables(const UnpackArgs &a, const LayerDev &ld, const uint32_t layer,
                                              const uint32_t row0_bin, const uint32_t scan_end, const uint32_t k0,
                                              uint32_t (*s_off)[kOffStride], uint16_t (*s_cnt)[kCntStride],
                                              float *s_scale, uint32_t *s_cmax)
{
    typedef typename std::conditional<W8, uint8_t, uint16_t>::type word_t;
    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform across the wave
    const uint32_t chunk = row0_bin >> 6;
    const uint32_t b = (chunk << 6) + lane;           // the bin this lane looks up
    const bool in_scan = b < scan_end;                // bins of the chunk up to the end of the group
    const bool in_rows = in_scan && b >= row0_bin;
    constexpr uint32_t kPerWave = kLearnerGroup / 4u;
    const uint32_t nk = a.n_learners - k0 < kLearnerGroup ? a.n_learners - k0 : kLearnerGroup;

    if (tid == 0) *s_cmax = 0u;
    __syncthreads();

    // wave w serves learners w, w + 4, ...; all their loads are issued first
    uint32_t c[kPerWave], coff[kPerWave], wbase[kPerWave], limit[kPerWave];
    float sc[kPerWave];
    bool ok[kPerWave];
#pragma unroll
    for (uint32_t q = 0; q < kPerWave; ++q) {
        const uint32_t kk = wave + 4u * q;
        c[q] = 0u; coff[q] = 0u; wbase[q] = 0u; limit[q] = 0u; sc[q] = 0.f; ok[q] = false;
        if (kk < nk) {
            const uint8_t *pk = a.packets[k0 + kk];
            const uint4 hv = *reinterpret_cast<const uint4 *>(pk);  // magic, version, status, n_layers
            const uint2 tb = *reinterpret_cast<const uint2 *>(pk + 16);  // total_bytes
            ok[q] = (hv.x == ADACOMP_PACKET_MAGIC) & (hv.y == ADACOMP_PACKET_VERSION) &
                    (hv.z == ADACOMP_STATUS_COMPLETE) & (hv.w == a.n_layers) & (tb.y == 0u);
            limit[q] = tb.x / uint32_t(sizeof(word_t));  // words that fit in the packet
            // counts and chunk offsets sit in the fixed part, which every packet buffer holds
            if (in_scan) c[q] = reinterpret_cast<const word_t *>(pk + ld.counts_offset)[b];
            coff[q] = reinterpret_cast<const uint32_t *>(pk + ld.chunks_offset)[chunk];
            const adacomp_packet_layer_t *rec =
                reinterpret_cast<const adacomp_packet_layer_t *>(pk + sizeof(adacomp_packet_header_t)) + layer;
            sc[q] = rec->scale;
            wbase[q] = uint32_t(rec->words_offset / sizeof(word_t));  // packets stay below 2^32 words (host check)
        }
    }
    uint32_t wmax = 0u;
#pragma unroll
    for (uint32_t q = 0; q < kPerWave; ++q) {
        const uint32_t kk = wave + 4u * q;  // < kLearnerGroup; learners past nk get empty entries
        const uint32_t cq = ok[q] ? c[q] : 0u;   // a packet that does not match contributes nothing
        const uint32_t incl = wave_incl_scan(cq);
        // A bin whose words would lie past the packet's total_bytes (counts or offsets that do not
        // belong together) contributes nothing: no word is read from outside the packet.
        const uint64_t first = uint64_t(wbase[q]) + coff[q] + (incl - cq);
        const bool inside = first + cq <= limit[q];
        const uint32_t cw = inside ? cq : 0u;
        if (in_rows) {
            s_off[b - row0_bin][kk] = inside ? uint32_t(first) : 0u;
            s_cnt[b - row0_bin][kk] = uint16_t(cw);
        }
        if (lane == 0) s_scale[kk] = sc[q];
        wmax = (in_rows && cw > wmax) ? cw : wmax;
    }
#pragma unroll
    for (uint32_t d = 32; d > 0; d >>= 1) { const uint32_t o = __shfl_xor(wmax, d, 64); wmax = o > wmax ? o : wmax; }
    if (lane == 0) atomicMax(s_cmax, wmax);
}

// acc[idx] <- acc[idx] + v as an LDS load, a float add and an LDS store.  The LDS float atomic of
// this GPU works through its active lanes one after the other (3 cycles per lane, measured: a wave
// with all lanes busy holds the unit for 194 cycles, whatever the addresses), which made the adds
// the bottleneck of the short-bin path.  The plain sequence is safe here: the words of one learner
// name different elements, so no two lanes write one address in the same step; steps of different
// learners that do meet on an address come from lanes of one wave in program order, and the LDS
// unit executes a wave's instructions in order.  The accesses are volatile so that the compiler
// keeps that order.  The sum, a single float32 addition per word, is the one the atomic gives.
typedef __attribute__((address_space(3))) float lds_float;  // a float in LDS: ds_read / ds_write, not flat accesses
__device__ __forceinline__ volatile lds_float *lds_volatile(float *p) { return (volatile lds_float *)p; }
__device__ __forceinline__ void lds_add(float *acc, const uint32_t idx, const float v)
{
    volatile lds_float *p = lds_volatile(acc) + idx;
    const float cur = *p;
    *p = cur + v;
}

// Phase 2 for one tile: a lane group owns a bin (table row row0 + bin index inside the tile).
template <bool W8>
__device__ __forceinline__ void unpack_adds(const UnpackArgs &a, const UTileDev &ut, const uint32_t row0, const uint32_t k0,
                                            float *s_acc, uint32_t (*s_off)[kOffStride],
                                            uint16_t (*s_cnt)[kCntStride], const float *s_scale, const uint32_t *s_cmax)
{
    typedef typename std::conditional<W8, uint8_t, uint16_t>::type word_t;
    const uint32_t tid = threadIdx.x;
    const uint32_t n = ut.n_elems, T = ut.L_T, nb = ut.n_bins;
    const uint32_t nk = a.n_learners - k0 < kLearnerGroup ? a.n_learners - k0 : kLearnerGroup;
    if (W8) {
        // Short bins (8-bit words) send several words each, about 8 % of the elements on the
        // ResNet-50 table.  Four lanes own a bin and lane j fetches the aligned 4 bytes number j of
        // the bin's run of words, for all 16 learners at once (16 words per bin and learner; longer
        // runs are finished with byte loads), then adds learner after learner in program order.
        const uint32_t lb = tid >> 2, sub = tid & 3u;
        if (lb >= nb) return;
        const uint32_t row = row0 + lb;
        const uint32_t span = T < n - lb * T ? T : n - lb * T;  // elements of this bin held by the tile
        float *acc = s_acc + lb * T;
        // 8 learners at a time, to keep the register count (and with it the number of resident
        // workgroups) where the 16-bit path has it
#pragma unroll 1
        for (uint32_t h0 = 0; h0 < kLearnerGroup; h0 += 8u) {
            if (h0 >= nk) break;
            uint32_t cc[8], off[8], packed[8];
            {
                const uint4 t = *reinterpret_cast<const uint4 *>(&s_cnt[row][h0]);
                cc[0] = t.x & 0xFFFFu; cc[1] = t.x >> 16; cc[2] = t.y & 0xFFFFu; cc[3] = t.y >> 16;
                cc[4] = t.z & 0xFFFFu; cc[5] = t.z >> 16; cc[6] = t.w & 0xFFFFu; cc[7] = t.w >> 16;
                const uint4 o0 = *reinterpret_cast<const uint4 *>(&s_off[row][h0]);
                const uint4 o1 = *reinterpret_cast<const uint4 *>(&s_off[row][h0 + 4u]);
                off[0] = o0.x; off[1] = o0.y; off[2] = o0.z; off[3] = o0.w;
                off[4] = o1.x; off[5] = o1.y; off[6] = o1.z; off[7] = o1.w;
            }
#pragma unroll
            for (uint32_t kk = 0; kk < 8u; ++kk) {
                packed[kk] = 0u;
                // word sections start on 16-byte boundaries and are padded to them, so the aligned
                // 4 bytes around any word of the run lie inside the packet
                if (cc[kk] != 0u && 4u * sub < (off[kk] & 3u) + cc[kk])
                    packed[kk] = reinterpret_cast<const uint32_t *>(a.packets[k0 + (h0 + kk < nk ? h0 + kk : 0u)])[(off[kk] >> 2) + sub];
            }
#pragma unroll
            for (uint32_t kk = 0; kk < 8u; ++kk) {
                __builtin_amdgcn_sched_barrier(0);  // one learner at a time: keeps the register count down
                const uint32_t skew = off[kk] & 3u, cck = cc[kk];
                const float sck = s_scale[h0 + kk];
                // The words of this lane: bytes [beg, end) of its four, moved to the front so that
                // slot j is in use in every lane that has more than j words and a slot that no lane
                // of the wave uses costs nothing.  All loads of the accumulators first, then the
                // stores (one learner's words name different elements).
                volatile lds_float *vacc = lds_volatile(acc);
                const uint32_t lo = 4u * sub, end_all = skew + cck;
                const uint32_t beg = skew > lo ? (skew - lo < 4u ? skew - lo : 4u) : 0u;
                const uint32_t end = end_all > lo ? (end_all - lo < 4u ? end_all - lo : 4u) : 0u;
                const uint32_t nw = end > beg ? end - beg : 0u;
                const uint32_t mine = beg < 4u ? packed[kk] >> (8u * beg) : 0u;
                float cur[4];
                uint32_t at_idx[4];
#pragma unroll
                for (uint32_t j = 0; j < 4u; ++j) {
                    at_idx[j] = 0xFFFFFFFFu;  // all ones: no word
                    cur[j] = 0.f;
                    if (__builtin_amdgcn_ballot_w64(j < nw) != 0ull) {
                        const uint32_t wd = (mine >> (8u * j)) & 0xFFu;
                        const uint32_t idx = wd >> 2, code = wd & 3u;
                        const bool on = j < nw && (code & 1u) && idx < span;
                        if (on) { at_idx[j] = idx | (code << 30); cur[j] = vacc[idx]; }  // code 1 or 3 in the top bits
                    }
                }
#pragma unroll
                for (uint32_t j = 0; j < 4u; ++j)
                    if (at_idx[j] != 0xFFFFFFFFu) vacc[at_idx[j] & 0x3FFFFFFFu] = cur[j] + ((at_idx[j] >> 30) == 1u ? sck : -sck);
                if (skew + cck > 16u) {  // the words of this learner beyond the fetched 16 bytes
                    const word_t *wp = reinterpret_cast<const word_t *>(a.packets[k0 + (h0 + kk < nk ? h0 + kk : 0u)]);
                    for (uint32_t q = 16u - skew + sub; q < cck; q += 4u) {
                        const uint32_t wd = wp[off[kk] + q];
                        const uint32_t idx = wd >> 2, code = wd & 3u;
                        if ((code & 1u) && idx < span) lds_add(acc, idx, code == 1u ? sck : -sck);
                    }
                }
            }
        }
        return;
    }
    // lanes per bin: the smallest power of two that holds the largest word count of the tables,
    // between the layer's default (8 or 16) and the whole wave
    uint32_t glog = ut.group_log2();
    while (glog < 6u && (1u << glog) < *s_cmax) ++glog;
    const uint32_t gsz = 1u << glog;

    for (uint32_t s = tid; s < (nb << glog); s += kWG) {
        const uint32_t lb = s >> glog, sub = s & (gsz - 1u);
        const uint32_t row = row0 + lb;
        const uint32_t span = T < n - lb * T ? T : n - lb * T;  // elements of this bin held by the tile
        float *acc = s_acc + lb * T;
        uint32_t cc[kLearnerGroup], off[kLearnerGroup];
#pragma unroll
        for (uint32_t v = 0; v < kLearnerGroup / 8u; ++v) {
            const uint4 t = *reinterpret_cast<const uint4 *>(&s_cnt[row][8u * v]);
            cc[8 * v] = t.x & 0xFFFFu; cc[8 * v + 1] = t.x >> 16; cc[8 * v + 2] = t.y & 0xFFFFu; cc[8 * v + 3] = t.y >> 16;
            cc[8 * v + 4] = t.z & 0xFFFFu; cc[8 * v + 5] = t.z >> 16; cc[8 * v + 6] = t.w & 0xFFFFu; cc[8 * v + 7] = t.w >> 16;
        }
#pragma unroll
        for (uint32_t v = 0; v < kLearnerGroup / 4u; ++v) {
            const uint4 t = *reinterpret_cast<const uint4 *>(&s_off[row][4u * v]);
            off[4 * v] = t.x; off[4 * v + 1] = t.y; off[4 * v + 2] = t.z; off[4 * v + 3] = t.w;
        }
        uint32_t word[kLearnerGroup];
        uint32_t cmax = 0u;
#pragma unroll
        for (uint32_t kk = 0; kk < kLearnerGroup; ++kk) {
            cmax = cc[kk] > cmax ? cc[kk] : cmax;
            word[kk] = 0u;
            if (sub < cc[kk]) {
                const word_t *wp = reinterpret_cast<const word_t *>(a.packets[k0 + (kk < nk ? kk : 0u)]);
                word[kk] = wp[off[kk] + sub];
            }
        }
        if (cmax <= gsz) {
#pragma unroll
            for (uint32_t kk = 0; kk < kLearnerGroup; ++kk) {
                const uint32_t idx = (word[kk] >> 2) - ut.idx_lo;  // wraps to a huge value below idx_lo
                const uint32_t code = word[kk] & 3u;
                if ((code & 1u) && idx < span) { const float sck = s_scale[kk]; atomicAdd(&acc[idx], code == 1u ? sck : -sck); }
            }
        } else {
            // some learner sends more words from this bin than the group has lanes: plain loops,
            // one learner after the other (same order)
            for (uint32_t kk = 0; kk < nk; ++kk) {
                const word_t *wp = reinterpret_cast<const word_t *>(a.packets[k0 + kk]);
                const uint32_t cck = s_cnt[row][kk], st = s_off[row][kk];
                const float sck = s_scale[kk];
                for (uint32_t jw = sub; jw < cck; jw += gsz) {
                    const uint32_t wd = wp[st + jw];
                    const uint32_t idx = (wd >> 2) - ut.idx_lo;
                    const uint32_t code = wd & 3u;
                    if ((code & 1u) && idx < span) atomicAdd(&acc[idx], code == 1u ? sck : -sck);
                }
            }
        }
    }
}

// averageGradients() and updateWeights() of Algorithm 1 on one element of the finished sum: every
// operation is a separate float32 operation (contraction is off), division and square root are
// the correctly rounded ones.
template <int MODE>
__device__ __forceinline__ void apply_update(const UnpackArgs &a, float sum, float &w, float &s1, float &s2)
{
    const float g = sum / a.n_average;
    if (MODE == 1) {  // SGD with momentum: v <- mu v + g; w <- w - lr v
        const float mv = a.p1 * s1;
        const float v = mv + g;
        s1 = v;
        const float step = a.lr * v;
        w = w - step;
    } else {          // Adam
        const float m1 = a.p1 * s1, m2 = a.one_minus_p1 * g;
        const float m = m1 + m2;
        const float g2 = g * g;
        const float v1 = a.p2 * s2, v2 = a.one_minus_p2 * g2;
        const float v = v1 + v2;
        s1 = m;
        s2 = v;
        const float m_hat = m / a.bias1;
        const float v_hat = v / a.bias2;
        const float denom = sqrtf(v_hat) + a.eps;
        const float ratio = m_hat / denom;
        const float step = a.lr * ratio;
        w = w - step;
    }
}

// MODE 0: dense_out <- sum.  MODE 1 / 2: also (or only) the SGD / Adam step on weights and state.
// KIND 0 / 1: all groups of this launch belong to layers with 16-bit / 8-bit words; 2: either (the
// layer says which).  Large tables get one launch per kind: each path alone needs fewer registers
// than a kernel that holds both, which buys resident workgroups (8 % of the 16-bit path's time on
// the 125 M-element table).  Small tables, where a second launch would cost more than that, use
// the kernel that holds both.  The single-width kernels are held to 80 registers (6 waves per
// SIMD, what the LDS tile allows; the 16-bit path spills two).
template <int MODE, int KIND>
__global__ __launch_bounds__(kWG, (KIND == 2 ? 4 : 6)) void k_unpack(const UnpackArgs a)
{
    // A workgroup serves a group of consecutive tiles that lie in one 64-bin chunk (or are slices
    // of one long bin).  With up to 16 learners the tables of phase 1 are built once for the group.
    if (blockIdx.x >= a.n_groups) return;
    const UGroupDev grp = a.groups[blockIdx.x];
    const UTileDev ut0 = a.tiles[grp.first_tile];
    const UTileDev ut_last = a.tiles[grp.first_tile + grp.n_tiles - 1u];
    const uint32_t layer = ut0.layer();
    const LayerDev ld = a.layers[layer];
    const uint32_t tid = threadIdx.x;
    const uint32_t row0_bin = ut0.first_bin, scan_end = ut_last.first_bin + ut_last.n_bins;
    const bool tables_once = a.n_learners <= kLearnerGroup;
    const bool w8 = KIND == 2 ? ld.word_bytes == 1u : KIND == 1;

    __shared__ float s_acc[kUnpackTileElems];
    __shared__ __attribute__((aligned(16))) uint32_t s_off[64][kOffStride];  // first word of (bin, learner), counted from the packet start
    __shared__ __attribute__((aligned(16))) uint16_t s_cnt[64][kCntStride];
    __shared__ __attribute__((aligned(16))) float s_scale[kLearnerGroup];
    __shared__ uint32_t s_cmax;                                                // largest word count of a (bin, learner) in the tables

  for (uint32_t ti = 0; ti < grp.n_tiles; ++ti) {
    const UTileDev ut = ti == 0u ? ut0 : a.tiles[grp.first_tile + ti];
    const uint32_t n = ut.n_elems;
    const bool vec = ut.aligned();
    float *__restrict__ out = a.dense + ut.elem_base;

    __syncthreads();  // the previous tile has been written out and its adds are done with the tables
    // ---- tile accumulators: zero, or the partial sum of an earlier launch ----------------------
    for (uint32_t i = tid * 4u; i < n; i += kWG * 4u) {
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (a.accumulate) {
            if (vec && i + 4u <= n) v = *reinterpret_cast<const float4 *>(out + i);
            else {
                v.x = out[i];
                v.y = i + 1u < n ? out[i + 1] : 0.f;
                v.z = i + 2u < n ? out[i + 2] : 0.f;
                v.w = i + 3u < n ? out[i + 3] : 0.f;
            }
        }
        *reinterpret_cast<float4 *>(&s_acc[i]) = v;  // s_acc has room for the rounded-up tail
    }

    for (uint32_t k0 = 0; k0 < a.n_learners; k0 += kLearnerGroup) {
        if (!tables_once || ti == 0u) {
            if (k0 != 0u) __syncthreads();  // the adds of the previous 16 learners are done with the tables
            if (w8) unpack_tables<true>(a, ld, layer, row0_bin, scan_end, k0, s_off, s_cnt, s_scale, &s_cmax);
            else unpack_tables<false>(a, ld, layer, row0_bin, scan_end, k0, s_off, s_cnt, s_scale, &s_cmax);
        }
        __syncthreads();  // tables filled, accumulators initialised
        if (w8) unpack_adds<true>(a, ut, ut.first_bin - row0_bin, k0, s_acc, s_off, s_cnt, s_scale, &s_cmax);
        else unpack_adds<false>(a, ut, ut.first_bin - row0_bin, k0, s_acc, s_off, s_cnt, s_scale, &s_cmax);
    }
    __syncthreads();

    float *const W = MODE == 1 ? a.weights + ut.elem_base : nullptr;
    float *const S1 = MODE == 1 ? a.state1 + ut.elem_base : nullptr;
    const __amdgpu_buffer_rsrc_t w_buf = tile_buffer(MODE == 2 ? a.weights + ut.elem_base : out, MODE == 2 ? n : 0u);
    const __amdgpu_buffer_rsrc_t s1_buf = tile_buffer(MODE == 2 ? a.state1 + ut.elem_base : out, MODE == 2 ? n : 0u);
    const __amdgpu_buffer_rsrc_t s2_buf = tile_buffer(MODE == 2 ? a.state2 + ut.elem_base : out, MODE == 2 ? n : 0u);
    // The write-out moves 16-byte slots of memory whatever the tile's alignment.  A tile that starts
    // `skip` elements past a 16-byte boundary reads its accumulators from the LDS tile at the matching
    // offset (four 4-byte reads per slot instead of one 16-byte read): slot f (a multiple of 4) holds
    // the elements f - skip .. f + 3 - skip; in the first slot that wraps below zero, and `< n` on the
    // wrapped value tells the elements that are the tile's.  (With 4-byte accesses to memory such
    // tiles were written at 3.1 instead of 5 TB/s.)
    // (The Adam epilogue sits at its register limit and keeps 4-byte accesses on unaligned tiles: the
    // few registers this costs spilled there and slowed the aligned case by 4 %.)
    const uint32_t skip = MODE == 2 ? 0u : uint32_t(ut.elem_base) & 3u;
    for (uint32_t f = tid * 4u; f < n + skip; f += kWG * 4u) {
        const uint32_t e = f - skip;
        const bool full = (MODE != 2 || vec) && f >= skip && e + 4u <= n;
        float sum[4];
        if (skip == 0u) {
            const float4 v = *reinterpret_cast<const float4 *>(&s_acc[f]);
            sum[0] = v.x; sum[1] = v.y; sum[2] = v.z; sum[3] = v.w;
        } else {
#pragma unroll
            for (uint32_t c = 0; c < 4u; ++c) sum[c] = e + c < n ? s_acc[e + c] : 0.f;
        }
        if (a.write_dense) {
            if (full) store_stream4(out + e, vfloat4{sum[0], sum[1], sum[2], sum[3]});
            else {
#pragma unroll
                for (uint32_t c = 0; c < 4u; ++c)
                    if (e + c < n) out[e + c] = sum[c];
            }
        }
        if (MODE != 0) {
            if (full) {
                vfloat4 w4, s14, s24 = vfloat4{0.f, 0.f, 0.f, 0.f};
                if (MODE == 2) { w4 = buffer_load_stream4(w_buf, e); s14 = buffer_load_stream4(s1_buf, e); s24 = buffer_load_stream4(s2_buf, e); }
                else { w4 = load_stream4(W + e); s14 = load_stream4(S1 + e); }
                float w[4] = {w4.x, w4.y, w4.z, w4.w}, s1[4] = {s14.x, s14.y, s14.z, s14.w}, s2[4] = {s24.x, s24.y, s24.z, s24.w};
#pragma unroll
                for (int c = 0; c < 4; ++c) apply_update<MODE>(a, sum[c], w[c], s1[c], s2[c]);
                if (MODE == 2) {
                    buffer_store_stream4(w_buf, e, vfloat4{w[0], w[1], w[2], w[3]});
                    buffer_store_stream4(s1_buf, e, vfloat4{s1[0], s1[1], s1[2], s1[3]});
                    buffer_store_stream4(s2_buf, e, vfloat4{s2[0], s2[1], s2[2], s2[3]});
                } else {
                    store_stream4(W + e, vfloat4{w[0], w[1], w[2], w[3]});
                    store_stream4(S1 + e, vfloat4{s1[0], s1[1], s1[2], s1[3]});
                }
            } else {
                for (uint32_t c = 0; c < 4u; ++c) {
                    const uint32_t ec = e + c;   // wraps back into the tile for the elements of the first slot that are the tile's
                    if (ec >= n) continue;
                    float w, s1, s2 = 0.f;
                    if (MODE == 2) { w = buffer_load1(w_buf, ec); s1 = buffer_load1(s1_buf, ec); s2 = buffer_load1(s2_buf, ec); }
                    else { w = W[ec]; s1 = S1[ec]; }
                    apply_update<MODE>(a, sum[c], w, s1, s2);
                    if (MODE == 2) { buffer_store1(w_buf, ec, w); buffer_store1(s1_buf, ec, s1); buffer_store1(s2_buf, ec, s2); }
                    else { W[ec] = w; S1[ec] = s1; }
                }
            }
        }
    }
  }  // tiles of the group
}

// ==============================================================================================
// k_copy: plain float4 copy, the calibration kernel for byte counters and copy bandwidth.
// ==============================================================================================
__global__ __launch_bounds__(kWG) void k_copy(float *__restrict__ dst, const float *__restrict__ src, size_t n)
{
    const size_t n4 = n / 4;
    const size_t stride = size_t(gridDim.x) * kWG;
    for (size_t i = size_t(blockIdx.x) * kWG + threadIdx.x; i < n4; i += stride)
        reinterpret_cast<float4 *>(dst)[i] = reinterpret_cast<const float4 *>(src)[i];
    if (blockIdx.x == 0 && threadIdx.x < n % 4) dst[n4 * 4 + threadIdx.x] = src[n4 * 4 + threadIdx.x];
}

// ==============================================================================================
// k_triad, k_fill: the two streaming ceilings the hot kernels are measured against, with the access
// pattern of k_fused and nothing else.  k_triad: x <- x + y in place, 12 bytes per element (read,
// read, write) in tiles of 4096 elements, 16 per thread, streaming loads and stores, the same
// transposed tile order inside every 64 workgroups.  k_fill: 4 bytes per element written.
// ==============================================================================================
__global__ __launch_bounds__(kWG) void k_triad(float *__restrict__ x, const float *__restrict__ y, uint32_t n_tiles, size_t n)
{
    uint32_t tile = blockIdx.x;
    if (tile < (n_tiles & ~63u)) tile = (tile & ~63u) | ((tile & 7u) << 3) | ((tile >> 3) & 7u);
    const size_t base = size_t(tile) * 4096u;
    if (base + 4096u <= n) {   // a whole tile: eight loads in flight per thread, no branch between them
        vfloat4 a[4], b[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const size_t e = base + (uint32_t(j) * kWG + threadIdx.x) * 4u;
            a[j] = load_stream4(x + e);
            b[j] = load_stream4(y + e);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const size_t e = base + (uint32_t(j) * kWG + threadIdx.x) * 4u;
            store_stream4(x + e, a[j] + b[j]);
        }
        return;
    }
    for (int j = 0; j < 4; ++j) {   // the ragged last tile
        const size_t e = base + (uint32_t(j) * kWG + threadIdx.x) * 4u;
        if (e + 4u <= n) store_stream4(x + e, load_stream4(x + e) + load_stream4(y + e));
    }
}

__global__ __launch_bounds__(kWG) void k_fill(float *__restrict__ x, float value, size_t n)
{
    const size_t base = size_t(blockIdx.x) * 4096u;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const size_t e = base + (uint32_t(j) * kWG + threadIdx.x) * 4u;
        if (e + 4u <= n) store_stream4(x + e, vfloat4{value, value, value, value});
    }
}

// ---- launchers ---------------------------------------------------------------------------------
static int check_launch() { return hipGetLastError() == hipSuccess ? ADACOMP_OK : ADACOMP_EHIP; }

// a.fused_idle_lds: dynamic LDS that no kernel touches, asked for with the launches of the eager
// 256-thread kernel (the host decides when, adacomp_plan.h says why).
int launch_fused(const CompressArgs &a, int jcode, void *stream)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    // tiles of 4096 elements: 256 threads; tiles of 16384 (a bin longer than 4096): 1024 threads.  Either
    // way a thread holds 16 elements, and a compute unit holds 32 waves of them.  (With 256 threads
    // and 64 elements each the long-bin tiles had two workgroups per compute unit and streamed at
    // 51-55 % of the HBM peak instead of 75-80 %.)
    const dim3 grid(a.class_count * a.fused_count), wg(jcode == 0 ? 256 : 1024);
    const bool variant = a.rule != ADACOMP_RULE_ADACOMP || a.soft_factor_minus_1 != 1.0f;
    if (a.lazy) {  // the host offers lazy residues for the default method only
        if (jcode == 0) hipLaunchKernelGGL((k_fused<4, 4, false, true>), grid, wg, 0, s, a);
        else hipLaunchKernelGGL((k_fused<4, 16, false, true>), grid, wg, 0, s, a);
    } else if (!variant) {
        if (jcode == 0) hipLaunchKernelGGL((k_fused<4, 4, false, false>), grid, wg, a.fused_idle_lds, s, a);
        else if (a.shift) hipLaunchKernelGGL((k_fused<4, 16, false, false, true>), grid, wg, 0, s, a);
        else hipLaunchKernelGGL((k_fused<4, 16, false, false>), grid, wg, 0, s, a);
    } else {
        if (jcode == 0) hipLaunchKernelGGL((k_fused<4, 4, true, false>), grid, wg, a.fused_idle_lds, s, a);
        else if (a.shift) hipLaunchKernelGGL((k_fused<4, 16, true, false, true>), grid, wg, 0, s, a);
        else hipLaunchKernelGGL((k_fused<4, 16, true, false>), grid, wg, 0, s, a);
    }
    return check_launch();
}

int launch_scan(const CompressArgs &a, void *stream)
{
    hipLaunchKernelGGL(k_scan, dim3(a.n_layers, a.n_learners), dim3(kScanWG), 0, static_cast<hipStream_t>(stream), a);
    return check_launch();
}

int launch_place(const CompressArgs &a, void *stream)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    const dim3 wg(kWG);
    if (a.place_tiled) {
        if (a.fold_scan || a.place_mode != kPlaceEager) return ADACOMP_EINVAL;  // the host picks it for eager calls after a k_scan launch only
        hipLaunchKernelGGL(k_place_tiled, dim3(a.n_tiles + 1u, a.n_learners), wg, 0, s, a);
        return check_launch();
    }
    if (a.fold_scan && (a.place_lanes != 64u || a.place_mode == kPlaceResidue || a.n_tiles > kFoldTiles || a.n_layers > kFoldLayers))
        return ADACOMP_EINVAL;  // the host picks the folded scan only where the kernel is built for it
    if (a.place_lanes == 64u) {
        const dim3 grid((a.n_tiles + 3u) / 4u + 1u, a.n_learners);
        if (a.fold_scan) {
            if (a.place_mode == kPlaceWords) hipLaunchKernelGGL((k_place<64, kPlaceWords, true>), grid, wg, 0, s, a);
            else hipLaunchKernelGGL((k_place<64, kPlaceEager, true>), grid, wg, 0, s, a);
        } else if (a.place_mode == kPlaceWords) hipLaunchKernelGGL((k_place<64, kPlaceWords, false>), grid, wg, 0, s, a);
        else if (a.place_mode == kPlaceResidue) hipLaunchKernelGGL((k_place<64, kPlaceResidue, false>), grid, wg, 0, s, a);
        else hipLaunchKernelGGL((k_place<64, kPlaceEager, false>), grid, wg, 0, s, a);
    } else {
        const dim3 grid((a.n_tiles + 15u) / 16u + 1u, a.n_learners);
        if (a.place_mode == kPlaceWords) hipLaunchKernelGGL((k_place<16, kPlaceWords, false>), grid, wg, 0, s, a);
        else if (a.place_mode == kPlaceResidue) hipLaunchKernelGGL((k_place<16, kPlaceResidue, false>), grid, wg, 0, s, a);
        else hipLaunchKernelGGL((k_place<16, kPlaceEager, false>), grid, wg, 0, s, a);
    }
    return check_launch();
}

int launch_unpack(const UnpackArgs &a, int kind, void *stream)
{
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (a.n_groups == 0) return ADACOMP_OK;
    const dim3 grid(a.n_groups), wg(kWG);
    if (kind == 1) {
        if (a.mode == 1) hipLaunchKernelGGL((k_unpack<1, 1>), grid, wg, 0, s, a);
        else if (a.mode == 2) hipLaunchKernelGGL((k_unpack<2, 1>), grid, wg, 0, s, a);
        else hipLaunchKernelGGL((k_unpack<0, 1>), grid, wg, 0, s, a);
    } else if (kind == 0) {
        if (a.mode == 1) hipLaunchKernelGGL((k_unpack<1, 0>), grid, wg, 0, s, a);
        else if (a.mode == 2) hipLaunchKernelGGL((k_unpack<2, 0>), grid, wg, 0, s, a);
        else hipLaunchKernelGGL((k_unpack<0, 0>), grid, wg, 0, s, a);
    } else {
        if (a.mode == 1) hipLaunchKernelGGL((k_unpack<1, 2>), grid, wg, 0, s, a);
        else if (a.mode == 2) hipLaunchKernelGGL((k_unpack<2, 2>), grid, wg, 0, s, a);
        else hipLaunchKernelGGL((k_unpack<0, 2>), grid, wg, 0, s, a);
    }
    return check_launch();
}

int launch_triad(float *x, const float *y, size_t n, uint32_t resident, void *stream)
{
    const uint32_t n_tiles = uint32_t((n + 4095u) / 4096u);
    // fewer than 8 workgroups per compute unit: each asks for dynamic LDS it never touches, sized so that
    // `resident` of them fit the 160 KB of a compute unit and one more does not
    const uint32_t idle_lds = resident >= 8u ? 0u : 163840u / resident - 1024u;
    hipLaunchKernelGGL(k_triad, dim3(n_tiles), dim3(kWG), idle_lds, static_cast<hipStream_t>(stream), x, y, n_tiles, n);
    return check_launch();
}

int launch_fill(float *x, float value, size_t n, void *stream)
{
    hipLaunchKernelGGL(k_fill, dim3(uint32_t((n + 4095u) / 4096u)), dim3(kWG), 0, static_cast<hipStream_t>(stream), x, value, n);
    return check_launch();
}

int launch_copy(float *dst, const float *src, size_t n, void *stream)
{
    const size_t n4 = n / 4;
    size_t blocks = (n4 + kWG - 1) / kWG;
    if (blocks > 256u * 32u) blocks = 256u * 32u;
    if (blocks == 0) blocks = 1;
    hipLaunchKernelGGL(k_copy, dim3(uint32_t(blocks)), dim3(kWG), 0, static_cast<hipStream_t>(stream), dst, src, n);
    return check_launch();
}

}  // namespace adacomp
