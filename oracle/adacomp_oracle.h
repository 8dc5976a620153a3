/*
 * adacomp_oracle.h -- plain, slow, single-threaded CPU statement of AdaComp's pack() and unpack().
 *
 * TEST INFRASTRUCTURE ONLY.  This is the checker the GPU library is compared against; it is not
 * part of the product, it is never a fallback, and nothing in the product path links, loads or
 * calls it.  It shares no code, header, table or constant with the HIP path: the packet layout
 * below is written out a second time here, on purpose.
 *
 * What it follows (AdaComp paper, arXiv 1712.02679):
 *   - Algorithm 2 "Details of pack()": G = residue + dW, H = G + dW, bins of size T, g_max per
 *     bin, the local-max compare, Quantize, the pack vector, both residue updates.
 *   - Section "Pseudo code": the quantiser is a sign bit and one scale per layer, the scale being
 *     the average of the g_max vector.
 *   - Section "Adaptive Residual Gradient Compression (AdaComp) Technique": bins are a uniform cut
 *     of the flat layer vector; the bin maximum itself is sent and the soft-threshold picks are
 *     sent in addition to it; every layer is treated separately; one scale factor per layer per
 *     learner travels with the sparse vector.
 *   - Section "Experiment Results": 8-bit sparse-index words for L_T < 64 (here: <= 64, index
 *     0..63 fits 6 bits), 16-bit words up to L_T = 16K, 2 bits of each word hold the ternary value.
 *   - Algorithm 1: unpack() then averageGradients() are separate steps; unpack here produces the
 *     plain sum over learners; averageGradients() and updateWeights() follow as update_sgd /
 *     update_adam.
 *
 * Readings taken where the paper is silent or at odds with itself:
 *   union rule      an element is sent when G != 0 and (|H| >= g_max or |G| >= g_max), so the bin
 *                   maximum always goes out (prose) even when dW opposes it (the printed compare
 *                   alone would drop it);
 *   zeros           G == 0 (either sign of zero) is never sent;
 *   ragged layers   the last bin is short and counts as one bin in the scale average;
 *   scale           sum of g_max in double precision in bin order, one divide by the bin count,
 *                   one rounding to float;
 *   H               two float additions, fl(fl(R + dW) + dW), as the assignment is printed.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_pins.py (worked example,
 * closed forms, invariants, reductions to numpy routines, brute force on tiny inputs, planted
 * mistakes).  Nothing in this file is "parity unpinned"; what no paper value can confirm is the
 * choice of the readings above and of the container layout.
 *
 * Packet container (little-endian, all offsets in bytes from the packet start, every padding byte
 * zero, every section start a multiple of 16):
 *
 *   header, 32 bytes
 *     u32 magic 0x50434441 ("ADCP")   u32 version 1   u32 status (0 complete, 1 truncated)
 *     u32 n_layers                    u64 total_bytes u64 n_selected (all layers)
 *   n_layers records, 64 bytes each
 *     u64 elem_offset  u64 n_elems  u32 L_T  u32 n_bins  u32 word_bits (8|16)  f32 scale
 *     u64 n_selected   u64 counts_offset  u64 chunks_offset  u64 words_offset
 *   for each layer in order:  counts[n_bins] (u8 when word_bits == 8, else u16), pad to 16,
 *                             chunks[ceil(n_bins/64)] u32, pad to 16
 *        counts[b]  = number of words bin b contributes
 *        chunks[c]  = number of words this layer holds in bins < 64*c
 *   for each layer in order:  words[n_selected] (u8 | u16), pad to 16
 *        word = (index_in_bin << 2) | code,  code 1 = +scale, code 3 = -scale (0 and 2 unused),
 *        ordered by bin, then by index inside the bin
 */
#ifndef ADACOMP_ORACLE_H
#define ADACOMP_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    uint64_t elem_offset; /* first element of the layer in the flat gradient / residue / dense buffers */
    uint64_t n_elems;     /* > 0; need not be a multiple of L_T                                       */
    uint32_t L_T;         /* bin length, 1..16384                                                      */
    uint32_t reserved;
} adacomp_oracle_layer_t;

/* selection rules: 0 is the one the library implements; 1 and 2 exist for the ablation mechanism
 * of section "Robustness of the AdaComp Technique" and for planted-difference tests. */
#define ADACOMP_ORACLE_RULE_UNION   0 /* G != 0 and max(|H|,|G|) >= g_max                     */
#define ADACOMP_ORACLE_RULE_LITERAL 1 /* |H| >= g_max exactly as the printed compare           */
#define ADACOMP_ORACLE_RULE_LS      2 /* local selection: G != 0 and |G| >= g_max (max only)   */

/* One layer, one mini-batch of Algorithm 2.  All arrays are host memory.  residue_in and
 * residue_out may be the same array.  G, H (n floats), gmax (ceil(n/T) floats), selected (n bytes,
 * 0 or 1) and scale receive the intermediate values; none of them may be NULL.  soft_factor is
 * the multiple of dW in the soft-threshold operand (section "Adaptive Residual Gradient
 * Compression (AdaComp) Technique": factors 1.5 - 3.0 were studied, 2 chosen), 1 <= f <= 16;
 * 2.0f gives H = G + dW exactly as printed.
 * Returns the number of selected elements, or -1 on a bad argument. */
long long adacomp_oracle_pack_layer(const float *residue_in, const float *dW, uint64_t n, uint32_t T,
                                    int rule, float soft_factor, float *G, float *H, float *gmax,
                                    float *scale, uint8_t *selected, float *residue_out);

/* Size of the packet when every element of every layer is selected; 0 on a bad layer table. */
size_t adacomp_oracle_packet_bound(const adacomp_oracle_layer_t *layers, uint32_t n_layers);

/* pack() over a whole layer table: residue is updated in place, the packet is written to
 * packet_out.  Returns total_bytes (> 0) or a negative value: -1 bad argument, -2 bad L_T,
 * -3 elem_offset not a multiple of 4, -4 capacity too small (nothing is written, residue
 * untouched). */
long long adacomp_oracle_compress(const adacomp_oracle_layer_t *layers, uint32_t n_layers,
                                  const float *grad, float *residue, void *packet_out,
                                  size_t packet_capacity, int rule, float soft_factor);

/* unpack() of n_learners packets summed into dense_out in learner order 0..n-1 (float adds);
 * every element of every layer is written (0 where no learner sent it).  Returns 0, or -1 on a
 * bad argument, -5 when a packet does not match the layer table or is malformed. */
int adacomp_oracle_unpack_accumulate(const adacomp_oracle_layer_t *layers, uint32_t n_layers,
                                     const void *const *packets, uint32_t n_learners,
                                     float *dense_out);

/* averageGradients() then updateWeights() (Algorithm 1) on the dense sum of n_learners decoded
 * packets.  The paper trains with "SGD with momentum (=0.9)" and with Adam and leaves the update
 * rule to the framework; the forms taken here are the usual ones:
 *   SGD     g = sum / n;  v <- momentum * v + g;  w <- w - lr * v
 *   Adam    g = sum / n;  m <- beta1 m + (1 - beta1) g;  v <- beta2 v + (1 - beta2) g^2;
 *           w <- w - lr * (m / bias1) / (sqrt(v / bias2) + eps),  bias_k = 1 - beta_k^t passed in
 * Each arithmetic operation is one float operation, in that order.  Returns 0 or -1. */
int adacomp_oracle_update_sgd(const adacomp_oracle_layer_t *layers, uint32_t n_layers,
                              const float *dense_sum, uint32_t n_learners, float *weights,
                              float *momentum_buf, float lr, float momentum);
int adacomp_oracle_update_adam(const adacomp_oracle_layer_t *layers, uint32_t n_layers,
                               const float *dense_sum, uint32_t n_learners, float *weights, float *m_buf,
                               float *v_buf, float lr, float beta1, float beta2, float eps,
                               float bias1, float bias2);

#ifdef __cplusplus
}
#endif
#endif
