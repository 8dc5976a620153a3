/*
 * adacomp.h -- C ABI of libadacomp: AdaComp residual-gradient compression on one AMD MI355X
 * (gfx950).  Hand-written HIP kernels; no CPU fallback exists: without a GPU every compute
 * entry point returns ADACOMP_EHIP.
 *
 * The method is that of "AdaComp: Adaptive Residual Gradient Compression for Data-Parallel
 * Distributed Training" (arXiv 1712.02679).  Per learner and per mini-batch, pack() (Algorithm 2)
 * adds the new gradient dW to the residue (G = residue + dW), forms H = G + dW, cuts every
 * layer's flat vector into bins of length L_T, finds each bin's largest |G| (g_max), sends the
 * elements whose |H| reaches their bin's g_max (together with the bin maximum itself, section
 * "Adaptive Residual Gradient Compression (AdaComp) Technique"), quantises every sent value to
 * sign(G) * scale with one scale per layer = average of the g_max vector (section "Pseudo
 * code"), and keeps G - Gq (sent) or G (not sent) as the new residue.  Sent values travel as
 * sparse-index words, 8 bits for L_T <= 64 and 16 bits up to L_T = 16384, two bits of which hold
 * the ternary value (section "Experiment Results").  unpack() (Algorithm 1) decodes the packets a
 * learner received; here it also sums them into one dense gradient.
 *
 * Conventions
 *   - Pointers are DEVICE pointers unless the comment says host.  The library allocates and
 *     frees no caller memory; the caller owns every buffer, including the workspace.
 *   - Work is enqueued on the HIP stream passed in (a hipStream_t cast to void*, NULL = the
 *     default stream) and the call returns without synchronising.  Results, including the packet
 *     header, are in device memory once the stream has drained.
 *   - Calls that share a workspace must be ordered on one stream; calls on different streams
 *     need different workspaces.
 *   - Every function returns 0 (ADACOMP_OK) or a negative ADACOMP_E* code; nothing throws or
 *     aborts.  Inputs must be finite; NaN / Inf give unspecified values but stay memory-safe.
 *   - Arithmetic is IEEE float32 with round-to-nearest-even and denormals kept; the layer scale
 *     is summed and divided in float64 and rounded once.  The kernels add the g_max values in a
 *     fixed tree (so a call repeats bit for bit), a sequential program adds them bin after bin; the
 *     two agree in every bit while the float64 sum is exact, which holds when the layer's nonzero
 *     g_max values span at most 2^(29 - log2(n_bins)) in magnitude (e.g. a factor of 2000 over
 *     250 000 bins, 10^6 over 500 bins).  Beyond that the float32 scale can differ from the
 *     sequential one in its last bit (2^-24 relative, against the 1e-6 this library promises),
 *     and with it the residue at the sent elements by one unit in the last place of the scale.
 *
 * Packet container written by adacomp_compress (little-endian, offsets in bytes from the packet
 * start, every padding byte zero, every section start a multiple of 16):
 *
 *   adacomp_packet_header_t                      32 bytes
 *   adacomp_packet_layer_t[n_layers]             64 bytes each
 *   per layer, in order:  counts[n_bins]  (uint8 when word_bits == 8, else uint16), pad to 16
 *                         chunks[ceil(n_bins / 64)] uint32, pad to 16
 *        counts[b] = words contributed by bin b; chunks[c] = words of this layer in bins < 64 c
 *   per layer, in order:  words[n_selected] (uint8 | uint16), pad to 16
 *        word = (index_in_bin << 2) | code;  code 1 = +scale, code 3 = -scale (2-bit two's
 *        complement of the ternary value; 0 and 2 never occur); words are ordered by bin, then by
 *        index inside the bin.
 *   Compression rate by the paper's accounting = 32 * n_elems / (word_bits * n_selected);
 *   on the wire = 4 * n_elems / total_bytes.
 */
#ifndef ADACOMP_H
#define ADACOMP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ADACOMP_OK 0
#define ADACOMP_EINVAL (-1)     /* null pointer, n_layers == 0, n_elems == 0 or >= 2^31, overlapping layers,
                                   or a table whose adacomp_packet_bound would reach 4 GiB             */
#define ADACOMP_EBADLT (-2)     /* L_T == 0 or L_T > 16384                                               */
#define ADACOMP_EALIGN (-3)     /* elem_offset not a multiple of 4, or a buffer not 16-byte aligned      */
#define ADACOMP_ENOSPC (-4)     /* packet_capacity below the fixed part of the packet                    */
#define ADACOMP_EHIP (-5)       /* a HIP call failed (no device, launch failure)                         */
#define ADACOMP_EWORKSPACE (-6) /* workspace too small, or not initialised for this layer table          */
#define ADACOMP_EPENDING (-7)   /* residue corrections of a lazy call wait in this workspace and the call
                                   is not the lazy call that goes on with the same residue buffers      */

#define ADACOMP_ETOOBIG (-8)    /* adacomp_compress_static: the table needs more than ADACOMP_STATIC_SCRATCH_BYTES */

#define ADACOMP_LT_MAX 16384u
#define ADACOMP_CHUNK_BINS 64u
#define ADACOMP_PACKET_MAGIC 0x50434441u /* bytes 'A' 'D' 'C' 'P' */
#define ADACOMP_PACKET_VERSION 1u
#define ADACOMP_STATUS_COMPLETE 0u
#define ADACOMP_STATUS_TRUNCATED 1u /* capacity was too small: words beyond it were not written */

/* One layer of the flat gradient: the method treats every layer on its own (section "Adaptive
 * Residual Gradient Compression (AdaComp) Technique"); L_T is its one hyper-parameter, chosen per
 * layer type: 50 for convolutions, 500 for FC / LSTM (Table 2). */
typedef struct {
    uint64_t elem_offset; /* first element in grad / residue / dense_out; multiple of 4        */
    uint64_t n_elems;     /* 1 .. 2^31-1; need not be a multiple of L_T (the last bin is short) */
    uint32_t L_T;         /* bin length, 1 .. 16384                                             */
    uint32_t reserved;    /* 0                                                                  */
} adacomp_layer_t;

typedef struct {
    uint32_t magic, version, status, n_layers;
    uint64_t total_bytes; /* size of the complete packet (what a transport has to move)   */
    uint64_t n_selected;  /* words in all layers                                           */
} adacomp_packet_header_t;

typedef struct {
    uint64_t elem_offset, n_elems;
    uint32_t L_T, n_bins, word_bits; /* 8 or 16 */
    float scale;                     /* decoded magnitude of every word of this layer */
    uint64_t n_selected;
    uint64_t counts_offset, chunks_offset, words_offset;
} adacomp_packet_layer_t;

/* ---- sizes (host-only arithmetic; layers is a host array) ---------------------------------- */

/* Bytes of a packet in which every element of every layer is sent: a capacity that can never
 * overflow.  Returns 0 if the layer table is invalid. */
size_t adacomp_packet_bound(const adacomp_layer_t *layers, uint32_t n_layers);

/* Bytes before the first word (header, records, counts, chunks): the least capacity accepted. */
size_t adacomp_packet_fixed_bytes(const adacomp_layer_t *layers, uint32_t n_layers);

/* Bytes of workspace adacomp_workspace_init / compress / unpack need for this table (device
 * tables, per-bin g_max, per-tile counters, staging for unplaced words). 0 if the table is invalid. */
size_t adacomp_workspace_bytes(const adacomp_layer_t *layers, uint32_t n_layers);

/* Same, for adacomp_compress_batch with up to n_learners learners per call: the tables once plus
 * one scratch block per learner (about 2 bytes per gradient element each). */
size_t adacomp_workspace_bytes_batch(const adacomp_layer_t *layers, uint32_t n_layers, uint32_t n_learners);

/* ---- set-up --------------------------------------------------------------------------------- */

/* Writes the device-side tile tables for this layer table into the head of `workspace`
 * (256-byte aligned device memory of at least adacomp_workspace_bytes()).  Call once per
 * workspace and layer table, before the first compress / unpack that uses it.  The tables are
 * copied with a blocking host-to-device copy ordered after the work already on `hip_stream`, so
 * this call is not capturable in a HIP graph; compress and unpack only launch kernels.  The
 * caller must leave the workspace contents alone between calls. */
int adacomp_workspace_init(const adacomp_layer_t *layers, uint32_t n_layers, void *workspace,
                           size_t workspace_bytes, void *hip_stream);

/* Forgets a workspace registered by adacomp_workspace_init (host bookkeeping only). */
int adacomp_workspace_release(void *workspace);

/* ---- pack(): Algorithm 2 over every layer of one learner ------------------------------------- */

/* grad       dW of this mini-batch, read only; 16-byte aligned; layers at their elem_offset.
 * residue    in: residue carried from the previous mini-batch (zeros at the start of training);
 *            out: the new residue.  Must not alias grad.
 * packet_out receives the packet; 16-byte aligned.  packet_capacity >= adacomp_packet_fixed_bytes
 *            or ADACOMP_ENOSPC is returned and nothing is enqueued.  If the words do not fit,
 *            header.status = ADACOMP_STATUS_TRUNCATED, header.total_bytes is the size that was
 *            needed, no byte past packet_capacity is written, and the residue is updated as if
 *            everything had been sent (the packet must then be discarded by the caller).
 * Elements of grad / residue outside every layer are neither read nor written. */
int adacomp_compress(const adacomp_layer_t *layers, uint32_t n_layers, const float *grad,
                     float *residue, void *packet_out, size_t packet_capacity, void *workspace,
                     size_t workspace_bytes, void *hip_stream);

/* adacomp_compress for callers that cannot allocate device memory or hand in a workspace: code
 * that runs under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results and error codes as adacomp_compress (packet and residue are bit for bit the
 * same), but the workspace is an array of ADACOMP_STATIC_SCRATCH_BYTES (16 MiB) that the library
 * holds in the memory of every GPU it runs on until the process ends; there is no
 * adacomp_workspace_init to call.  No device memory is allocated or freed by this call, or by
 * anything it calls.
 *   - A layer table whose adacomp_workspace_bytes exceeds the array (about 2.1 bytes per gradient
 *     element: tables beyond roughly 7.5 M elements) is refused with ADACOMP_ETOOBIG before
 *     anything is enqueued.
 *   - The first call on a device, and every call whose layer table differs from the previous
 *     call's on that device, writes the tile tables into the array with blocking host-to-device
 *     copies ordered after the work already on hip_stream (so that call is not capturable in a
 *     graph and waits for the stream); calls that repeat the table only launch kernels and touch
 *     no allocator, host or device.
 *   - All calls on one GPU share that GPU's array, which keeps what the last call left in it.
 *     Nothing in it has to start at zero (every field a kernel reads is written earlier in the
 *     same call), but two calls that overlap in time on one GPU (different streams, different
 *     threads) race on it: give them one stream, or use adacomp_compress with workspaces of the
 *     caller's. */
#define ADACOMP_STATIC_SCRATCH_BYTES (16u << 20)
int adacomp_compress_static(const adacomp_layer_t *layers, uint32_t n_layers, const float *grad,
                            float *residue, void *packet_out, size_t packet_capacity, void *hip_stream);

/* pack() for several learners that share one layer table, in one set of launches (the simulated
 * learners of a single-GPU run, or several model replicas on one device).  grads, residues and
 * packets_out are HOST arrays of n_learners DEVICE pointers; residues and packets must be
 * distinct buffers; every packet buffer has packet_capacity bytes.  Learner k's result is exactly
 * what adacomp_compress gives for (grads[k], residues[k], packets_out[k]).  The workspace must
 * have been initialised with at least adacomp_workspace_bytes_batch(layers, n_layers, n_learners)
 * bytes.  Cites: every learner runs Algorithm 2 on its own gradient and residue (Algorithm 1,
 * "pack()" precedes "exchange()"), so learners are independent until unpack. */
int adacomp_compress_batch(const adacomp_layer_t *layers, uint32_t n_layers, uint32_t n_learners,
                           const float *const *grads, float *const *residues, void *const *packets_out,
                           size_t packet_capacity, void *workspace, size_t workspace_bytes, void *hip_stream);

/* pack() with another selection rule or soft-threshold factor: the mechanisms of the paper's
 * ablations (section "Robustness of the AdaComp Technique": Local Selection keeps the selection
 * inside bins and leaves the soft threshold out, so only bin maxima go; section "Adaptive Residual
 * Gradient Compression (AdaComp) Technique": factors 1.5 - 3.0 were studied, 2 chosen so that only
 * additions are needed).  Everything else (bins, g_max, scale, quantiser, residue, packet) is as
 * in adacomp_compress_batch, which is this call with ADACOMP_RULE_ADACOMP and factor 2.
 *   rule         ADACOMP_RULE_ADACOMP          sent iff G != 0 and max(|H|, |G|) >= g_max
 *                ADACOMP_RULE_PRINTED_COMPARE  sent iff |H| >= g_max, exactly the compare printed in
 *                                              Algorithm 2 (may drop a bin maximum, sends zeros of
 *                                              an all-zero bin)
 *                ADACOMP_RULE_LOCAL_SELECTION  sent iff G != 0 and |G| >= g_max (bin maxima only)
 *   soft_factor  f in [1, 16]: H = residue + f dW, computed as G + (f - 1) dW with one float
 *                multiplication and one addition; f = 2 is G + dW.  Other values: ADACOMP_EINVAL. */
#define ADACOMP_RULE_ADACOMP 0u
#define ADACOMP_RULE_PRINTED_COMPARE 1u
#define ADACOMP_RULE_LOCAL_SELECTION 2u
int adacomp_compress_variant(const adacomp_layer_t *layers, uint32_t n_layers, uint32_t n_learners,
                             const float *const *grads, float *const *residues, void *const *packets_out,
                             size_t packet_capacity, uint32_t rule, float soft_factor, void *workspace,
                             size_t workspace_bytes, void *hip_stream);

/* pack() with the residue corrections deferred.  The last step of Algorithm 2, the subtraction of
 * the quantised value from G at the sent elements, is a scattered read-modify-write that costs about 6 %
 * of the whole pack() on a large fully connected table; nothing needs its result before the same
 * learner's next pack(), which reads the whole residue anyway.  This call sends exactly the
 * packets adacomp_compress_batch sends, but leaves the corrections in the workspace and applies
 * them at the start of the next lazy call, in registers.  Between the two calls residues[k] holds
 * G (not G - Gq) at the elements that were sent.
 *   - The next call on this workspace must be adacomp_compress_batch_lazy with the same
 *     n_learners and the same residues[k] in the same order, or adacomp_residue_sync; every other
 *     compress call returns ADACOMP_EPENDING and enqueues nothing.  Unpack calls are not affected.
 *   - Before the residues are read, written, zeroed, checkpointed or freed by anyone else, and
 *     before adacomp_workspace_init / adacomp_workspace_release of this workspace (which drop the
 *     waiting corrections), call adacomp_residue_sync.
 *   - The host keeps the books when a call is enqueued: use one stream per workspace.  A HIP graph
 *     holds the kernels of the call as it was captured: capture a lazy call while corrections
 *     wait (after a first lazy call outside the capture) and replay it only in that state.
 * After the sync the residues are bit for bit those of the eager calls.  If a launch of this call
 * fails (ADACOMP_EHIP) the residues are unspecified and nothing is left waiting. */
int adacomp_compress_batch_lazy(const adacomp_layer_t *layers, uint32_t n_layers, uint32_t n_learners,
                                const float *const *grads, float *const *residues, void *const *packets_out,
                                size_t packet_capacity, void *workspace, size_t workspace_bytes, void *hip_stream);

/* Applies the residue corrections that the last adacomp_compress_batch_lazy on this workspace left
 * waiting, to the residue buffers that call was given (one kernel launch on hip_stream).  Does
 * nothing if none wait.  ADACOMP_EWORKSPACE if the workspace is not registered.  If a launch fails
 * (ADACOMP_EHIP) the residues are unspecified and nothing is left waiting. */
int adacomp_residue_sync(void *workspace, void *hip_stream);

/* ---- unpack() of all learners, summed ("unpack()" then the sum inside "averageGradients()") -- */

/* packets    HOST array of n_learners DEVICE pointers to complete packets made by
 *            adacomp_compress with the same layer table.  A packet whose header does not match
 *            (magic, version, status, n_layers) contributes nothing.  The counts and offsets
 *            inside a packet are otherwise taken as they are; the only check is that no word is
 *            read at or beyond the header's total_bytes (a bin whose words would lie there
 *            contributes nothing), so the buffer must hold total_bytes bytes: a caller that
 *            received the packet from elsewhere compares the header's total_bytes with the
 *            number of bytes it received before it calls.  Whatever a packet holds, nothing
 *            outside dense_out is written.
 * dense_out  every element of every layer is overwritten with the float32 sum, taken in learner
 *            order 0..n-1, of the decoded values (+-scale of that learner's layer where it sent
 *            the element, 0 elsewhere); 16-byte aligned.  n_learners == 0 writes zeros.
 * The division by the learner count is left to the caller. */
int adacomp_unpack_accumulate(const adacomp_layer_t *layers, uint32_t n_layers,
                              const void *const *packets, uint32_t n_learners, float *dense_out,
                              void *workspace, size_t workspace_bytes, void *hip_stream);

/* ---- unpack() + averageGradients() + updateWeights() in one pass (Algorithm 1, last three steps) */

#define ADACOMP_OPT_SGD_MOMENTUM 1u /* v <- momentum v + g;  w <- w - lr v                                  */
#define ADACOMP_OPT_ADAM 2u         /* m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2;
                                       w <- w - lr (m / bias1) / (sqrt(v / bias2) + eps)                    */
typedef struct {
    uint32_t kind;  /* ADACOMP_OPT_* */
    float lr;
    float momentum; /* SGD */
    float beta1, beta2, eps;
    float bias1, bias2; /* Adam's 1 - beta1^t and 1 - beta2^t for this step, computed by the caller */
} adacomp_optimizer_t;

/* Like adacomp_unpack_accumulate, then g = sum / n_learners (averageGradients() of Algorithm 1) and
 * one optimizer step on the weights (updateWeights(), which every learner does for itself), without writing the dense
 * gradient to memory and reading it back.  The paper trains with SGD with momentum 0.9 and with
 * Adam (sections "Experiment Results", "Robustness of the AdaComp Technique") and leaves the
 * update rule to the framework; the forms above are the usual ones, each arithmetic operation a
 * separate float32 operation in the order written.
 * dense_out  may be NULL (the sum is then never stored) unless n_learners > 64; if given it
 *            receives the un-averaged sum as in adacomp_unpack_accumulate.
 * weights, state1 (momentum buffer, or Adam's m), state2 (Adam's v; NULL for SGD): float32 buffers
 *            laid out like the gradient, 16-byte aligned, updated in place on every layer element.
 * n_learners must be >= 1. */
int adacomp_unpack_update(const adacomp_layer_t *layers, uint32_t n_layers, const void *const *packets,
                          uint32_t n_learners, float *dense_out, float *weights, float *state1, float *state2,
                          const adacomp_optimizer_t *opt, void *workspace, size_t workspace_bytes, void *hip_stream);

/* ---- errors as text ------------------------------------------------------------------------ */

const char *adacomp_strerror(int code);

/* Diagnostics, tuning knobs and kernel timing are declared in adacomp_debug.h; they are not part of
 * the stable contract. */

#ifdef __cplusplus
}
#endif
#endif
