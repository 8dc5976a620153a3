"""Pin strength: a copy of the oracle with ONE planted mistake must fail at least one pin.

Each mutant is the oracle's C source with one snippet replaced (a dropped term, a wrong sign or
index, a wrong operand, a wrong bound), compiled on the CPU into a temporary library.  Nothing
here runs on a GPU.
"""
import os
import subprocess

import pytest

import oracle
import oracle_pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "adacomp_oracle.c")

MUTANTS = {
    "G_minus_dW": ("G[index] = residue_in[index] + dW[index];", "G[index] = residue_in[index] - dW[index];"),
    "H_minus_dW": ("if (soft_factor == 2.0f) return g + dw;", "if (soft_factor == 2.0f) return g - dw;"),
    "H_from_residue_once": ("H[index] = soft_operand(G[index], dW[index], soft_factor);", "H[index] = soft_factor == 2.0f ? residue_in[index] + 2.0f * dW[index] : soft_operand(G[index], dW[index], soft_factor);"),
    "factor_not_reduced_by_one": ("float f_minus_1 = soft_factor - 1.0f;", "float f_minus_1 = soft_factor;"),
    "factor_applied_to_G": ("float extra = f_minus_1 * dw;", "float extra = f_minus_1 * g;"),
    "sgd_no_average": ("float g = dense_sum[i] / n;      /* average among all learners */", "float g = dense_sum[i];"),
    "sgd_plus_step": ("weights[i] = weights[i] - step;  /* w <- w - lr * v            */", "weights[i] = weights[i] + step;"),
    "sgd_momentum_on_gradient": ("float mv = momentum * momentum_buf[i];", "float mv = momentum * g;"),
    "sgd_step_uses_gradient": ("float step = lr * v;", "float step = lr * g;"),
    "adam_v_not_squared": ("float g2 = g * g;", "float g2 = g;"),
    "adam_no_bias_correction": ("float m_hat = m / bias1;                    /* bias1 = 1 - beta1^t                 */", "float m_hat = m;"),
    "adam_eps_inside_sqrt": ("float denom = sqrtf(v_hat) + eps;", "float denom = sqrtf(v_hat + eps);"),
    "adam_swapped_betas": ("float a = beta1 * m_buf[i], b = one_minus_b1 * g;", "float a = beta2 * m_buf[i], b = one_minus_b2 * g;"),
    "gmax_from_H": ("gmax[i] = bin_max_abs(G, lo, hi);", "gmax[i] = bin_max_abs(H, lo, hi);"),
    "gmax_signed": ("float a = fabsf(G[index]);", "float a = G[index];"),
    "bin_end_off_by_one": ("*hi = *lo + T < n ? *lo + T : n;", "*hi = *lo + T - 1 < n ? *lo + T - 1 : n;"),
    "scale_over_elements": ("float s = mean_of_gmax(gmax, n_bins);", "float s = mean_of_gmax(gmax, n_bins) * (float)n_bins / (float)n;"),
    "scale_float_sum": ("double sum = 0.0;", "float sum = 0.0f;"),
    "scale_skips_last_bin": ("for (uint64_t i = 0; i < n_bins; ++i) sum += (double)gmax[i];",
                             "for (uint64_t i = 0; i + 1 < n_bins; ++i) sum += (double)gmax[i];"),
    "strict_compare": ("return (g != 0.0f) && (fabsf(h) >= m || fabsf(g) >= m);", "return (g != 0.0f) && (fabsf(h) > m || fabsf(g) > m);"),
    "no_union": ("return (g != 0.0f) && (fabsf(h) >= m || fabsf(g) >= m);", "return (g != 0.0f) && (fabsf(h) >= m);"),
    "no_soft_threshold": ("return (g != 0.0f) && (fabsf(h) >= m || fabsf(g) >= m);", "return (g != 0.0f) && (fabsf(g) >= m);"),
    "zeros_sent": ("return (g != 0.0f) && (fabsf(h) >= m || fabsf(g) >= m);", "return (fabsf(h) >= m || fabsf(g) >= m);"),
    "wrong_bin_for_threshold": ("if (is_sent(rule, g, H[index], gmax[i])) {", "if (is_sent(rule, g, H[index], gmax[0])) {"),
    "residue_plus_Gq": ("residue_out[index] = g - Gq;", "residue_out[index] = g + Gq;"),
    "residue_zeroed_when_sent": ("residue_out[index] = g - Gq;", "residue_out[index] = 0.0f;"),
    "Gq_sign_of_H": ("float Gq = copysignf(s, g);", "float Gq = copysignf(s, H[index]);"),
    "Gq_unsigned": ("float Gq = copysignf(s, g);", "float Gq = s;"),
    "unsent_residue_keeps_old": ("residue_out[index] = g;\n", "residue_out[index] = residue_in[index];\n"),
    "code_sign_flipped": ("? 3u : 1u;", "? 1u : 3u;"),
    "index_shift": ("uint32_t word = (j << 2) | code;", "uint32_t word = (j << 1) | code;"),
    "index_global": ("uint32_t j = (uint32_t)(index - lo);              /* index inside the bin        */",
                     "uint32_t j = (uint32_t)(index);"),
    "word_width_boundary": ("static uint32_t word_bits_of(uint32_t T) { return T <= 64 ? 8u : 16u; }",
                            "static uint32_t word_bits_of(uint32_t T) { return T < 64 ? 8u : 16u; }"),
    "chunk_offsets_inclusive": ("put_u32(pk + chunks_off + 4 * (i / PK_CHUNK_BINS), (uint32_t)w);",
                                "put_u32(pk + chunks_off + 4 * (i / PK_CHUNK_BINS), (uint32_t)(w + 1));"),
    "unpack_overwrites": ("dense_out[layers[l].elem_offset + lo + j] += v;", "dense_out[layers[l].elem_offset + lo + j] = v;"),
    "unpack_sign_flipped": ("float v = code == 1u ? scale : -scale;", "float v = code == 1u ? -scale : scale;"),
    "unpack_ignores_bin": ("dense_out[layers[l].elem_offset + lo + j] += v;", "dense_out[layers[l].elem_offset + j] += v;"),
    "residue_committed_on_overflow": ("if (total > packet_capacity) { result = -4; goto done; }",
                                      "if (total > packet_capacity) { result = -4; for (uint32_t l = 0; l < n_layers; ++l) memcpy(residue + layers[l].elem_offset, tmp[l].R_new, layers[l].n_elems * sizeof(float)); goto done; }"),
    "soft_operand_ignores_factor": ("float extra = f_minus_1 * dw;", "float extra = dw;"),
    "sent_compare_swapped_operands": ("if (is_sent(rule, g, H[index], gmax[i])) {", "if (is_sent(rule, H[index], g, gmax[i])) {"),
    "bound_doubled": ("return (size_t)off;", "return (size_t)(2 * off);"),
    "bound_one_byte_per_element": ("off += pad16(layers[l].n_elems * (word_bits_of(layers[l].L_T) / 8));",
                                   "off += pad16(layers[l].n_elems);"),
    "bound_counts_one_byte_per_bin": ("off += pad16(n_bins * (word_bits_of(layers[l].L_T) / 8));", "off += pad16(n_bins);"),
    "bound_without_chunk_table": ("off += pad16(n_chunks * 4);", "off += 0;"),
    "padding_not_zero": ("memset(pk, 0, (size_t)total);", "memset(pk, 0xAB, (size_t)total);"),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_is_caught(tmp_path, name):
    old, new = MUTANTS[name]
    src = open(SRC).read()
    assert src.count(old) == 1, f"mutation site for {name} not unique / not found"
    csrc = tmp_path / "mutant.c"
    csrc.write_text(src.replace(old, new))
    lib = tmp_path / f"libmutant_{name}.so"
    subprocess.run(["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-shared", "-fPIC", "-w",
                    f"-I{os.path.dirname(SRC)}", "-o", str(lib), str(csrc), "-lm"], check=True)
    mutant = oracle.Oracle(str(lib))
    failed = []
    for pin in oracle_pins.PINS:
        try:
            pin(mutant)
        except Exception:   # any failed assertion or refused call counts
            failed.append(pin.__name__)
    assert failed, f"planted mistake '{name}' passes every pin"
