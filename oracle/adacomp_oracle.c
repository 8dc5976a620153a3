/*
 * adacomp_oracle.c -- see adacomp_oracle.h.  TEST INFRASTRUCTURE ONLY: the slow CPU checker.
 *
 * Plain C, one thread.  The steps of Algorithm 2 of the AdaComp paper are taken in the paper's
 * order and notation (G, H, T, g_max, Gq, residue), each as a small function of its own and a
 * driver that calls them; no blocking, no fusion, no reordering.
 * Build without value-changing options: gcc -O2 -ffp-contract=off, no fast-math.
 */
#include "adacomp_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

#define PK_MAGIC 0x50434441u /* "ADCP" */
#define PK_VERSION 1u
#define PK_HEADER_BYTES 32u
#define PK_RECORD_BYTES 64u
#define PK_CHUNK_BINS 64u
#define LT_MAX 16384u

/* ------------------------------------------------------------------------------------------
 * Algorithm 2, one layer: small pieces first, then the driver that strings them together.
 * ---------------------------------------------------------------------------------------- */

/* Elements [*lo, *hi) of bin i when a vector of n elements is cut into bins of T (section
 * "Adaptive Residual Gradient Compression (AdaComp) Technique": a uniform cut; the last bin is
 * short when T does not divide n). */
static void bin_range(uint64_t i, uint32_t T, uint64_t n, uint64_t *lo, uint64_t *hi)
{
    *lo = i * T;
    *hi = *lo + T < n ? *lo + T : n;
}

/* g_max of one bin: the largest absolute value of G over [lo, hi). */
static float bin_max_abs(const float *G, uint64_t lo, uint64_t hi)
{
    float m = 0.0f;
    for (uint64_t index = lo; index < hi; ++index) {
        float a = fabsf(G[index]);
        if (a > m) m = a;
    }
    return m;
}

/* The quantiser's scale: the average of the g_max vector over all bins of the layer (section
 * "Pseudo code"), accumulated in double in bin order and rounded to float once. */
static float mean_of_gmax(const float *gmax, uint64_t n_bins)
{
    double sum = 0.0;
    for (uint64_t i = 0; i < n_bins; ++i) sum += (double)gmax[i];
    return (float)(sum / (double)n_bins);
}

/* The soft-threshold operand for one element: the stored G plus dW once more.  That is residue +
 * 2 dW, the paper's choice among the factors 1.5 - 3.0 it studied; another factor f gives residue +
 * f dW, formed as G + (f - 1) dW with one multiplication and one addition. */
static float soft_operand(float g, float dw, float soft_factor)
{
    if (soft_factor == 2.0f) return g + dw;
    float f_minus_1 = soft_factor - 1.0f;
    float extra = f_minus_1 * dw;
    return g + extra;
}

/* Is the element sent?  m is its bin's g_max. */
static int is_sent(int rule, float g, float h, float m)
{
    if (rule == ADACOMP_ORACLE_RULE_LITERAL) return fabsf(h) >= m;
    if (rule == ADACOMP_ORACLE_RULE_LS) return (g != 0.0f) && (fabsf(g) >= m);
    return (g != 0.0f) && (fabsf(h) >= m || fabsf(g) >= m);
}

long long adacomp_oracle_pack_layer(const float *residue_in, const float *dW, uint64_t n, uint32_t T,
                                    int rule, float soft_factor, float *G, float *H, float *gmax,
                                    float *scale, uint8_t *selected, float *residue_out)
{
    if (!residue_in || !dW || !G || !H || !gmax || !scale || !selected || !residue_out) return -1;
    if (n == 0 || T == 0 || T > LT_MAX) return -1;
    if (rule < 0 || rule > 2) return -1;
    if (!(soft_factor >= 1.0f && soft_factor <= 16.0f)) return -1;

    uint64_t n_bins = (n + T - 1) / T;

    /* the two element-wise vectors */
    for (uint64_t index = 0; index < n; ++index) {
        G[index] = residue_in[index] + dW[index];
        H[index] = soft_operand(G[index], dW[index], soft_factor);
    }

    /* every bin's maximum, then the one scale of the layer */
    for (uint64_t i = 0; i < n_bins; ++i) {
        uint64_t lo, hi;
        bin_range(i, T, n, &lo, &hi);
        gmax[i] = bin_max_abs(G, lo, hi);
    }
    float s = mean_of_gmax(gmax, n_bins);
    *scale = s;

    /* bin by bin, index by index: compare with the bin's maximum, quantise what is sent, and leave
     * the rest of G (all of it when nothing is sent) as the new residue */
    long long n_sent = 0;
    for (uint64_t i = 0; i < n_bins; ++i) {
        uint64_t lo, hi;
        bin_range(i, T, n, &lo, &hi);
        for (uint64_t index = lo; index < hi; ++index) {
            float g = G[index];
            if (is_sent(rule, g, H[index], gmax[i])) {
                float Gq = copysignf(s, g); /* sign bit and the layer scale */
                residue_out[index] = g - Gq;
                selected[index] = 1;
                ++n_sent;
            } else {
                residue_out[index] = g;
                selected[index] = 0;
            }
        }
    }
    return n_sent;
}

/* ------------------------------------------------------------------------------------------
 * Packet container.
 * ---------------------------------------------------------------------------------------- */
static uint64_t pad16(uint64_t x) { return (x + 15u) & ~(uint64_t)15u; }

static void put_u32(uint8_t *p, uint32_t v)
{
    p[0] = (uint8_t)v; p[1] = (uint8_t)(v >> 8); p[2] = (uint8_t)(v >> 16); p[3] = (uint8_t)(v >> 24);
}
static void put_u64(uint8_t *p, uint64_t v)
{
    put_u32(p, (uint32_t)v); put_u32(p + 4, (uint32_t)(v >> 32));
}
static uint32_t get_u32(const uint8_t *p)
{
    return (uint32_t)p[0] | ((uint32_t)p[1] << 8) | ((uint32_t)p[2] << 16) | ((uint32_t)p[3] << 24);
}
static uint64_t get_u64(const uint8_t *p)
{
    return (uint64_t)get_u32(p) | ((uint64_t)get_u32(p + 4) << 32);
}

static int check_layers(const adacomp_oracle_layer_t *layers, uint32_t n_layers)
{
    if (!layers || n_layers == 0) return -1;
    for (uint32_t l = 0; l < n_layers; ++l) {
        if (layers[l].n_elems == 0 || layers[l].n_elems >= ((uint64_t)1 << 31)) return -1;
        if (layers[l].L_T == 0 || layers[l].L_T > LT_MAX) return -2;
        if (layers[l].elem_offset % 4 != 0) return -3;
        /* layers must not overlap */
        for (uint32_t m = 0; m < l; ++m) {
            uint64_t a0 = layers[l].elem_offset, a1 = a0 + layers[l].n_elems;
            uint64_t b0 = layers[m].elem_offset, b1 = b0 + layers[m].n_elems;
            if (a0 < b1 && b0 < a1) return -1;
        }
    }
    return 0;
}

static uint32_t word_bits_of(uint32_t T) { return T <= 64 ? 8u : 16u; }

/* bytes of header + records + all counts/chunks sections: everything before the first word */
static uint64_t fixed_part_bytes(const adacomp_oracle_layer_t *layers, uint32_t n_layers)
{
    uint64_t off = PK_HEADER_BYTES + (uint64_t)PK_RECORD_BYTES * n_layers;
    for (uint32_t l = 0; l < n_layers; ++l) {
        uint64_t n_bins = (layers[l].n_elems + layers[l].L_T - 1) / layers[l].L_T;
        uint64_t n_chunks = (n_bins + PK_CHUNK_BINS - 1) / PK_CHUNK_BINS;
        off += pad16(n_bins * (word_bits_of(layers[l].L_T) / 8));
        off += pad16(n_chunks * 4);
    }
    return off;
}

size_t adacomp_oracle_packet_bound(const adacomp_oracle_layer_t *layers, uint32_t n_layers)
{
    if (check_layers(layers, n_layers) != 0) return 0;
    uint64_t off = fixed_part_bytes(layers, n_layers);
    for (uint32_t l = 0; l < n_layers; ++l)
        off += pad16(layers[l].n_elems * (word_bits_of(layers[l].L_T) / 8));
    return (size_t)off;
}

long long adacomp_oracle_compress(const adacomp_oracle_layer_t *layers, uint32_t n_layers,
                                  const float *grad, float *residue, void *packet_out,
                                  size_t packet_capacity, int rule, float soft_factor)
{
    int rc = check_layers(layers, n_layers);
    if (rc != 0) return rc;
    if (!grad || !residue || !packet_out) return -1;

    /* run Algorithm 2 on every layer into temporaries first, so that a packet that does not fit
     * leaves the residue untouched */
    typedef struct { float *R_new; uint8_t *sel; float *G; float scale; long long n_sent; } tmp_t;
    tmp_t *tmp = (tmp_t *)calloc(n_layers, sizeof(tmp_t));
    if (!tmp) return -1;
    long long result = -1;
    uint64_t total = fixed_part_bytes(layers, n_layers);
    int ok = 1;
    for (uint32_t l = 0; l < n_layers && ok; ++l) {
        uint64_t n = layers[l].n_elems;
        uint32_t T = layers[l].L_T;
        uint64_t n_bins = (n + T - 1) / T;
        float *H = (float *)malloc(n * sizeof(float));
        float *gmax = (float *)malloc(n_bins * sizeof(float));
        tmp[l].G = (float *)malloc(n * sizeof(float));
        tmp[l].R_new = (float *)malloc(n * sizeof(float));
        tmp[l].sel = (uint8_t *)malloc(n);
        if (!H || !gmax || !tmp[l].G || !tmp[l].R_new || !tmp[l].sel) ok = 0;
        if (ok) {
            tmp[l].n_sent = adacomp_oracle_pack_layer(residue + layers[l].elem_offset,
                                                      grad + layers[l].elem_offset, n, T, rule, soft_factor,
                                                      tmp[l].G, H, gmax, &tmp[l].scale, tmp[l].sel,
                                                      tmp[l].R_new);
            if (tmp[l].n_sent < 0) ok = 0;
            else total += pad16((uint64_t)tmp[l].n_sent * (word_bits_of(T) / 8));
        }
        free(H);
        free(gmax);
    }
    if (!ok) goto done;
    if (total > packet_capacity) { result = -4; goto done; }

    uint8_t *pk = (uint8_t *)packet_out;
    memset(pk, 0, (size_t)total);

    /* header */
    uint64_t n_sel_all = 0;
    for (uint32_t l = 0; l < n_layers; ++l) n_sel_all += (uint64_t)tmp[l].n_sent;
    put_u32(pk + 0, PK_MAGIC);
    put_u32(pk + 4, PK_VERSION);
    put_u32(pk + 8, 0);
    put_u32(pk + 12, n_layers);
    put_u64(pk + 16, total);
    put_u64(pk + 24, n_sel_all);

    uint64_t fixed_off = PK_HEADER_BYTES + (uint64_t)PK_RECORD_BYTES * n_layers;
    uint64_t words_off = fixed_part_bytes(layers, n_layers);
    for (uint32_t l = 0; l < n_layers; ++l) {
        uint64_t n = layers[l].n_elems;
        uint32_t T = layers[l].L_T;
        uint64_t n_bins = (n + T - 1) / T;
        uint64_t n_chunks = (n_bins + PK_CHUNK_BINS - 1) / PK_CHUNK_BINS;
        uint32_t wbytes = word_bits_of(T) / 8;
        uint64_t counts_off = fixed_off;
        uint64_t chunks_off = counts_off + pad16(n_bins * wbytes);
        fixed_off = chunks_off + pad16(n_chunks * 4);

        /* record */
        uint8_t *rec = pk + PK_HEADER_BYTES + (uint64_t)PK_RECORD_BYTES * l;
        uint32_t scale_bits;
        memcpy(&scale_bits, &tmp[l].scale, 4);
        put_u64(rec + 0, layers[l].elem_offset);
        put_u64(rec + 8, n);
        put_u32(rec + 16, T);
        put_u32(rec + 20, (uint32_t)n_bins);
        put_u32(rec + 24, wbytes * 8);
        put_u32(rec + 28, scale_bits);
        put_u64(rec + 32, (uint64_t)tmp[l].n_sent);
        put_u64(rec + 40, counts_off);
        put_u64(rec + 48, chunks_off);
        put_u64(rec + 56, words_off);

        /* the pack vector: walk bins, then indices within each bin, appending one word per sent
         * element; count per bin; a running total at every 64th bin */
        uint64_t w = 0; /* words of this layer so far */
        for (uint64_t i = 0; i < n_bins; ++i) {
            if (i % PK_CHUNK_BINS == 0) put_u32(pk + chunks_off + 4 * (i / PK_CHUNK_BINS), (uint32_t)w);
            uint64_t lo = i * T, hi = lo + T < n ? lo + T : n;
            uint32_t count = 0;
            for (uint64_t index = lo; index < hi; ++index) {
                if (!tmp[l].sel[index]) continue;
                uint32_t j = (uint32_t)(index - lo);              /* index inside the bin        */
                uint32_t code = signbit(tmp[l].G[index]) ? 3u : 1u; /* ternary value: -scale / +scale */
                uint32_t word = (j << 2) | code;
                if (wbytes == 1) pk[words_off + w] = (uint8_t)word;
                else { pk[words_off + 2 * w] = (uint8_t)word; pk[words_off + 2 * w + 1] = (uint8_t)(word >> 8); }
                ++w;
                ++count;
            }
            if (wbytes == 1) pk[counts_off + i] = (uint8_t)count;
            else { pk[counts_off + 2 * i] = (uint8_t)count; pk[counts_off + 2 * i + 1] = (uint8_t)(count >> 8); }
        }
        words_off += pad16(w * wbytes);
    }

    /* commit the residue */
    for (uint32_t l = 0; l < n_layers; ++l)
        memcpy(residue + layers[l].elem_offset, tmp[l].R_new, layers[l].n_elems * sizeof(float));
    result = (long long)total;

done:
    for (uint32_t l = 0; l < n_layers; ++l) {
        free(tmp[l].G);
        free(tmp[l].R_new);
        free(tmp[l].sel);
    }
    free(tmp);
    return result;
}

/* ------------------------------------------------------------------------------------------
 * unpack(): decode every learner's packet and sum, learner 0 first.
 * ---------------------------------------------------------------------------------------- */
int adacomp_oracle_unpack_accumulate(const adacomp_oracle_layer_t *layers, uint32_t n_layers,
                                     const void *const *packets, uint32_t n_learners,
                                     float *dense_out)
{
    if (check_layers(layers, n_layers) != 0 || !dense_out) return -1;
    if (n_learners > 0 && !packets) return -1;

    for (uint32_t l = 0; l < n_layers; ++l)
        for (uint64_t e = 0; e < layers[l].n_elems; ++e) dense_out[layers[l].elem_offset + e] = 0.0f;

    for (uint32_t k = 0; k < n_learners; ++k) {
        const uint8_t *pk = (const uint8_t *)packets[k];
        if (!pk) return -1;
        if (get_u32(pk + 0) != PK_MAGIC || get_u32(pk + 4) != PK_VERSION) return -5;
        if (get_u32(pk + 8) != 0 || get_u32(pk + 12) != n_layers) return -5;
        for (uint32_t l = 0; l < n_layers; ++l) {
            const uint8_t *rec = pk + PK_HEADER_BYTES + (uint64_t)PK_RECORD_BYTES * l;
            uint64_t n = layers[l].n_elems;
            uint32_t T = layers[l].L_T;
            uint64_t n_bins = (n + T - 1) / T;
            uint32_t wbytes = word_bits_of(T) / 8;
            if (get_u64(rec + 0) != layers[l].elem_offset || get_u64(rec + 8) != n ||
                get_u32(rec + 16) != T || get_u32(rec + 20) != n_bins || get_u32(rec + 24) != wbytes * 8)
                return -5;
            uint32_t scale_bits = get_u32(rec + 28);
            float scale;
            memcpy(&scale, &scale_bits, 4);
            uint64_t counts_off = get_u64(rec + 40), words_off = get_u64(rec + 56);
            uint64_t w = 0;
            for (uint64_t i = 0; i < n_bins; ++i) {
                uint64_t lo = i * T, hi = lo + T < n ? lo + T : n;
                uint32_t count = wbytes == 1 ? pk[counts_off + i]
                                             : (uint32_t)pk[counts_off + 2 * i] | ((uint32_t)pk[counts_off + 2 * i + 1] << 8);
                for (uint32_t c = 0; c < count; ++c, ++w) {
                    uint32_t word = wbytes == 1 ? pk[words_off + w]
                                                : (uint32_t)pk[words_off + 2 * w] | ((uint32_t)pk[words_off + 2 * w + 1] << 8);
                    uint32_t j = word >> 2, code = word & 3u;
                    if (lo + j >= hi || (code != 1u && code != 3u)) return -5;
                    float v = code == 1u ? scale : -scale;
                    dense_out[layers[l].elem_offset + lo + j] += v;
                }
            }
            if (w != get_u64(rec + 32)) return -5;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------------------------
 * averageGradients() and updateWeights() of Algorithm 1, applied to the dense sum unpack() made.
 * Every operation is a separate float operation in the order written (no fused multiply-add).
 * ---------------------------------------------------------------------------------------- */
int adacomp_oracle_update_sgd(const adacomp_oracle_layer_t *layers, uint32_t n_layers,
                              const float *dense_sum, uint32_t n_learners, float *weights,
                              float *momentum_buf, float lr, float momentum)
{
    if (check_layers(layers, n_layers) != 0 || !dense_sum || !weights || !momentum_buf || n_learners == 0) return -1;
    float n = (float)n_learners;
    for (uint32_t l = 0; l < n_layers; ++l)
        for (uint64_t e = 0; e < layers[l].n_elems; ++e) {
            uint64_t i = layers[l].elem_offset + e;
            float g = dense_sum[i] / n;      /* average among all learners */
            float mv = momentum * momentum_buf[i];
            float v = mv + g;                /* v <- momentum * v + g      */
            momentum_buf[i] = v;
            float step = lr * v;
            weights[i] = weights[i] - step;  /* w <- w - lr * v            */
        }
    return 0;
}

int adacomp_oracle_update_adam(const adacomp_oracle_layer_t *layers, uint32_t n_layers,
                               const float *dense_sum, uint32_t n_learners, float *weights, float *m_buf,
                               float *v_buf, float lr, float beta1, float beta2, float eps,
                               float bias1, float bias2)
{
    if (check_layers(layers, n_layers) != 0 || !dense_sum || !weights || !m_buf || !v_buf || n_learners == 0) return -1;
    float n = (float)n_learners;
    float one_minus_b1 = 1.0f - beta1, one_minus_b2 = 1.0f - beta2;
    for (uint32_t l = 0; l < n_layers; ++l)
        for (uint64_t e = 0; e < layers[l].n_elems; ++e) {
            uint64_t i = layers[l].elem_offset + e;
            float g = dense_sum[i] / n;                 /* average among all learners          */
            float a = beta1 * m_buf[i], b = one_minus_b1 * g;
            float m = a + b;                            /* m <- beta1 m + (1 - beta1) g        */
            float g2 = g * g;
            float c = beta2 * v_buf[i], d = one_minus_b2 * g2;
            float v = c + d;                            /* v <- beta2 v + (1 - beta2) g^2      */
            m_buf[i] = m;
            v_buf[i] = v;
            float m_hat = m / bias1;                    /* bias1 = 1 - beta1^t                 */
            float v_hat = v / bias2;                    /* bias2 = 1 - beta2^t                 */
            float denom = sqrtf(v_hat) + eps;
            float ratio = m_hat / denom;
            float step = lr * ratio;
            weights[i] = weights[i] - step;             /* w <- w - lr m_hat / (sqrt(v_hat)+eps) */
        }
    return 0;
}
