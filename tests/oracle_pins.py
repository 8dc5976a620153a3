"""Pins for the CPU oracle: each function takes an ``oracle.Oracle`` and asserts facts that the
AdaComp paper or plain mathematics fix, none of them computed by the oracle itself.

Citations are to the AdaComp paper (arXiv 1712.02679): Algorithm 2 "Details of pack()", section
"Pseudo code" (the quantiser and its scale), section "Adaptive Residual Gradient Compression
(AdaComp) Technique" (bins, the bin maximum is sent, the soft threshold adds to it) and section
"Experiment Results" (word widths, the 40x / 200x arithmetic).

test_oracle_pins.py runs every pin on the real oracle (all must pass); test_oracle_planted.py
compiles copies of the oracle with one planted mistake each and requires that some pin fails.
"""
import os

import numpy as np

import packet_format as pf

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
f32 = np.float32


def _read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            out[key] = vals
    return out


def _rand(seed, n, scale=1.0):
    return (np.random.default_rng(seed).standard_normal(n) * scale).astype(f32)


def _binmax(a, T):
    """max |a| per bin via numpy's reshape/max on a zero-padded copy (zeros never win a max of
    absolute values, and an all-zero bin has maximum 0)."""
    n = a.size
    nb = (n + T - 1) // T
    p = np.zeros(nb * T, f32)
    p[:n] = np.abs(a)
    return p.reshape(nb, T).max(axis=1)


# ---------------------------------------------------------------------------------------------
def pin_worked_example(o):
    """Hand-worked 16-element example (tests/golden/worked_example_T4.txt): every intermediate of
    Algorithm 2, the words, the counts and the decoded vector."""
    g = _read_golden("worked_example_T4.txt")
    T = int(g["T"][0])
    R = np.array(g["residue"], f32)
    dW = np.array(g["dW"], f32)
    r = o.pack_layer(R, dW, T)
    assert np.array_equal(r["G"], np.array(g["G"], f32))
    assert np.array_equal(r["H"], np.array(g["H"], f32))
    assert np.array_equal(r["gmax"], np.array(g["gmax"], f32))
    assert r["scale"] == f32(g["scale"][0])
    assert np.flatnonzero(r["selected"]).tolist() == [int(v) for v in g["selected"]]
    assert np.array_equal(r["residue"], np.array(g["residue_new"], f32))
    # whole-table call: same residue, and the packet holds the hand-written words and counts
    R2 = R.copy()
    pk = o.compress([(0, R.size, T)], dW, R2)
    assert np.array_equal(R2, np.array(g["residue_new"], f32))
    h, layers = pf.parse(pk)
    assert layers[0]["words"].tolist() == [int(v) for v in g["words"]]
    assert layers[0]["counts"].tolist() == [int(v) for v in g["counts"]]
    assert layers[0]["rec"]["word_bits"] == 8 and layers[0]["rec"]["scale"] == f32(g["scale"][0])
    dense = o.unpack_accumulate([(0, R.size, T)], [pk], R.size)
    assert np.array_equal(dense, np.array(g["decoded"], f32))
    # paper accounting: dense bits over packed word bits
    assert 32 * R.size == int(g["paper_ratio_num"][0]) and 8 * int(h["n_selected"]) == int(g["paper_ratio_den"][0])


def pin_G_H_gmax_against_numpy(o):
    """G and H are single float additions and g_max a max of absolute values: they must equal
    numpy's float32 add and reshape/abs/max bit for bit, ragged last bin included."""
    for seed, n, T in [(1, 1000, 50), (2, 1234, 50), (3, 7777, 500), (4, 129, 64), (5, 33, 7), (6, 5, 16384)]:
        R, dW = _rand(seed, n), _rand(seed + 100, n, 0.3)
        r = o.pack_layer(R, dW, T)
        G = R + dW
        assert G.dtype == f32 and np.array_equal(r["G"], G)
        assert np.array_equal(r["H"], G + dW)
        assert np.array_equal(r["gmax"], _binmax(G, T))
        assert r["gmax"].size == (n + T - 1) // T


def pin_H_uses_two_additions(o):
    """H = fl(fl(R + dW) + dW) as the assignment is printed, not fl(R + 2 dW).  With R = 1 and
    dW = 0.625 ulp(1): R + dW = 1 + 0.625 ulp rounds to 1 + 1 ulp; adding dW again gives
    1 + 1.625 ulp which rounds to 1 + 2 ulp; the single-rounding value 1 + 1.25 ulp would round
    to 1 + 1 ulp."""
    R = np.array([1.0], f32)
    dW = np.array([5.0 * 2.0 ** -26], f32)
    r = o.pack_layer(R, dW, 1)
    ulp = 2.0 ** -23
    assert float(r["G"][0]) == 1.0 + ulp
    assert float(r["H"][0]) == 1.0 + 2 * ulp          # two roundings
    assert float(f32(1.0 + 2 * 5.0 * 2.0 ** -26)) == 1.0 + ulp  # what one rounding would give


def pin_scale_closed_forms(o):
    """Scale = average of g_max over ALL bins (zero bins and the short last bin included)."""
    # all bins share one maximum -> scale is exactly that maximum
    T, nb = 8, 37
    R = np.zeros(T * nb, f32)
    R[::T] = f32(0.3)
    r = o.pack_layer(R, np.zeros_like(R), T)
    assert r["scale"] == f32(0.3)
    # bins with maxima 1,2,...,10 and 6 all-zero bins: mean = 55/16
    R = np.zeros(4 * 16, f32)
    R[0:40:4] = np.arange(1, 11, dtype=f32)
    r = o.pack_layer(R, np.zeros_like(R), 4)
    assert r["scale"] == f32(55.0 / 16.0)
    # ragged: 10 elements, T = 4 -> 3 bins, the short one counts as a bin: (4 + 8 + 3)/3 = 5
    R = np.array([4, 0, 0, 0, 0, -8, 0, 0, 3, 0], f32)
    r = o.pack_layer(R, np.zeros_like(R), 4)
    assert r["gmax"].tolist() == [4.0, 8.0, 3.0] and r["scale"] == f32(5.0)
    # double-precision mean, one rounding: compare with numpy float64 mean of a random g_max
    R = _rand(11, 50 * 400)
    r = o.pack_layer(R, np.zeros_like(R), 50)
    assert r["scale"] == f32(np.mean(_binmax(R, 50).astype(np.float64)))


def pin_LT1_selects_every_nonzero(o):
    """With L_T = 1 each element is its own bin maximum: every nonzero G is sent and the scale
    is the mean of |G|."""
    R, dW = _rand(21, 500), _rand(22, 500)
    R[::7] = 0
    dW[::7] = 0
    dW[3] = -R[3]                      # exact cancellation -> G == 0 -> not sent
    r = o.pack_layer(R, dW, 1)
    G = R + dW
    assert np.array_equal(r["selected"], G != 0)
    assert r["n_selected"] == np.count_nonzero(G)
    assert r["scale"] == f32(np.mean(np.abs(G).astype(np.float64)))


def pin_bin_maximum_always_sent(o):
    """'In addition to this value' (the bin maximum): every bin with g_max > 0 sends at least
    one element and all of its arg-max elements; an all-zero bin sends nothing; signed zeros in G
    are never sent."""
    for seed, n, T in [(31, 5000, 50), (32, 5013, 500), (33, 640, 64)]:
        R, dW = _rand(seed, n), _rand(seed + 1, n, 2.0)   # large dW so it often opposes G
        R[:T] = 0
        dW[:T] = 0                                         # first bin all zero
        r = o.pack_layer(R, dW, T)
        G = R + dW
        gm = _binmax(G, T)
        bins = np.arange(n) // T
        is_max = (np.abs(G) == gm[bins]) & (G != 0)
        assert np.all(r["selected"][is_max])
        per_bin = np.bincount(bins, weights=r["selected"], minlength=gm.size)
        assert np.all(per_bin[gm > 0] >= 1) and np.all(per_bin[gm == 0] == 0)
    # -0.0 and +0.0 with H large: not sent
    R = np.array([0.0, -0.0, 1.0, 0.0], f32)
    dW = np.array([0.0, 0.0, 0.0, 0.0], f32)
    R[0], dW[0] = 5.0, -5.0            # G = 0, H = -5
    r = o.pack_layer(R, dW, 4)
    assert r["selected"].tolist() == [False, False, True, False]


def pin_dW_zero_sends_exactly_the_maxima(o):
    """dW = 0 gives H = G = R: the sent set is exactly the set of bin maxima, ties included."""
    n, T = 3000, 50
    R = np.round(_rand(41, n) * 4).astype(f32) / 4       # coarse grid -> many ties
    r = o.pack_layer(R, np.zeros(n, f32), T)
    gm = _binmax(R, T)
    expect = (np.abs(R) == gm[np.arange(n) // T]) & (R != 0)
    assert np.array_equal(r["selected"], expect)
    assert expect.sum() > gm.size                          # ties really occur
    # a bin of equal magnitudes sends all of them
    R = np.array([2, -2, 2, -2, 1, 0, 0, 0], f32)
    r = o.pack_layer(R, np.zeros(8, f32), 4)
    assert r["selected"].tolist() == [True, True, True, True, True, False, False, False]


def pin_zero_residue_threshold_is_half_the_maximum(o):
    """First mini-batch (residue = 0): G = dW and H = 2 dW exactly, so the soft threshold sends
    exactly the elements with 2|dW| >= bin max |dW| (the self-adjusting rule with factor 2)."""
    n, T = 20000, 500
    dW = _rand(51, n, 1e-3)
    r = o.pack_layer(np.zeros(n, f32), dW, T)
    gm = _binmax(dW, T)
    expect = (np.abs(dW) * f32(2) >= gm[np.arange(n) // T]) & (dW != 0)
    assert np.array_equal(r["selected"], expect)
    # statistics of the mechanism: a Gaussian bin of 500 sends roughly a tenth of its elements
    assert 40 < r["n_selected"] / (n / T) < 70


def pin_expected_selection_count_of_a_gaussian_bin(o):
    """First mini-batch with independent Gaussian dW: an element is sent iff 2|x| >= max|x| of its bin
    (factor 2 of the soft threshold), so the expected number sent per bin of T elements is
    T * integral of f(a) F(2a)^(T-1) da, with f and F the density and distribution of |x|.
    The integral gives about 55 for T = 500 and 11 for T = 50, the self-adjusting rate the paper
    describes (more is sent where the distribution is flat); the oracle must meet it within the
    sampling error."""
    from scipy.special import erf
    a = np.linspace(0.0, 12.0, 240001)
    f = np.sqrt(2.0 / np.pi) * np.exp(-0.5 * a * a)
    values = {}
    for T, n_bins, seed in ((500, 4000, 61), (50, 40000, 62)):
        F2 = erf(2.0 * a / np.sqrt(2.0))
        y = f * F2 ** (T - 1)
        expected = T * float(np.sum((y[1:] + y[:-1]) * 0.5 * (a[1] - a[0])))
        n = T * n_bins
        r = o.pack_layer(np.zeros(n, f32), _rand(seed, n, 3e-3), T)
        got = r["n_selected"] / n_bins
        assert abs(got - expected) < 0.02 * expected, (T, got, expected)
        values[T] = expected
    # what the integral comes to, so that a slip in it shows too
    assert abs(values[500] - 55.12) < 0.02 and abs(values[50] - 11.05) < 0.01


def pin_comparison_is_greater_or_equal(o):
    """The printed compare is >=: an element whose |H| equals g_max is sent."""
    R = np.array([2.0, 1.0, 0.5, 0.0], f32)
    dW = np.array([0.0, 0.5, 0.0, 0.0], f32)             # G = [2, 1.5, .5, 0], H = [2, 2, .5, 0]
    r = o.pack_layer(R, dW, 4)
    assert r["selected"].tolist() == [True, True, False, False]


def pin_soft_threshold_uses_H_not_G(o):
    """An element below the bin maximum in |G| is sent exactly when |G + dW| reaches it; the
    threshold is the maximum of |G| (not of |H|)."""
    #            max        picked by H   not picked    H large but gmax from G
    R = np.array([4.0,       2.5,          3.0,          0.0], f32)
    dW = np.array([0.0,      1.0,          0.25,         0.0], f32)
    # G = [4, 3.5, 3.25, 0], H = [4, 4.5, 3.5, 0]; g_max = 4 (from G; max|H| would be 4.5)
    r = o.pack_layer(R, dW, 4)
    assert r["gmax"].tolist() == [4.0]
    assert r["selected"].tolist() == [True, True, False, False]
    # opposite-sign gradient lowers |H|: the element is not an extra pick
    R = np.array([4.0, 3.9], f32)
    dW = np.array([0.0, -0.5], f32)                        # G = [4, 3.4], H = [4, 2.9]
    r = o.pack_layer(R, dW, 2)
    assert r["selected"].tolist() == [True, False]


def pin_residue_update(o):
    """Not sent: residue = G bit for bit.  Sent: residue = G - Gq with Gq = sign(G) * scale, one
    float subtraction, so residue + Gq reconstructs G to within half an ulp."""
    n, T = 10000, 50
    R, dW = _rand(61, n), _rand(62, n, 0.5)
    r = o.pack_layer(R, dW, T)
    G, sel, s = r["G"], r["selected"], r["scale"]
    assert np.array_equal(r["residue"][~sel].view(np.uint32), G[~sel].view(np.uint32))
    Gq = np.copysign(np.float64(s), G[sel].astype(np.float64))
    exact = G[sel].astype(np.float64) - Gq
    assert np.array_equal(r["residue"][sel], exact.astype(f32))   # correctly rounded difference
    assert np.all(np.abs(r["residue"][sel].astype(np.float64) + Gq - G[sel]) <=
                  0.5 * np.spacing(np.maximum(np.abs(G[sel]), s)).astype(np.float64))
    # the magnitude of a sent residue shrinks toward zero by scale (sign convention of Gq)
    big = sel & (np.abs(G) > s)
    assert big.any() and np.all(np.abs(r["residue"][big]) < np.abs(G[big]))
    assert np.all(np.sign(r["residue"][big]) == np.sign(G[big]))
    small = sel & (np.abs(G) < s)
    assert small.any() and np.all(np.sign(r["residue"][small]) == -np.sign(G[small]))


def pin_telescoping_over_steps(o):
    """Residues keep what was not sent: after t mini-batches,
    residue_t + sum of decoded packets = sum of dW, up to the float rounding of t additions."""
    n, T, steps = 6000, 50, 12
    layers = [(0, n, T)]
    R = np.zeros(n, f32)
    sent = np.zeros(n, np.float64)
    total = np.zeros(n, np.float64)
    for t in range(steps):
        dW = _rand(70 + t, n, 1e-2)
        pk = o.compress(layers, dW, R)
        sent += pf.decode_dense(pk, n).astype(np.float64)
        total += dW.astype(np.float64)
    err = np.abs(R.astype(np.float64) + sent - total)
    assert err.max() <= steps * 2.0 ** -24 * (np.abs(total).max() + np.abs(sent).max())
    assert np.abs(sent).max() > 0


def pin_packet_structure_and_roundtrip(o):
    """Container invariants on a mixed layer table (8- and 16-bit layers, ragged bins, > 64 bins
    so chunk offsets matter), and unpack of one packet = +-scale exactly at the sent elements."""
    table = [(0, 5013, 50), (5016, 70000, 500), (75016, 130, 64), (75148, 777, 65), (75928, 3, 16384)]
    n_total = 75928 + 3
    R, dW = _rand(81, n_total), _rand(82, n_total, 0.7)
    R0 = R.copy()
    pk = o.compress(table, dW, R)
    h, layers = pf.parse(pk)                              # asserts all structural invariants
    assert h["total_bytes"] == pk.size and h["status"] == 0 and h["n_layers"] == len(table)
    dense = o.unpack_accumulate(table, [pk], n_total)
    for (off, n, T), l in zip(table, layers):
        r = o.pack_layer(R0[off:off + n], dW[off:off + n], T)
        assert l["rec"]["elem_offset"] == off and l["rec"]["n_elems"] == n and l["rec"]["L_T"] == T
        assert l["rec"]["word_bits"] == (8 if T <= 64 else 16)
        idx, sign = pf.selected_indices(l)
        assert np.array_equal(idx, np.flatnonzero(r["selected"]))
        assert np.array_equal(sign, np.where(r["G"][idx] > 0, 1, -1))
        assert l["rec"]["scale"] == r["scale"]
        expect = np.zeros(n, f32)
        expect[idx] = sign.astype(f32) * r["scale"]
        assert np.array_equal(dense[off:off + n], expect)
        assert np.array_equal(R[off:off + n], r["residue"])
    # gaps between layers are not written by unpack
    assert np.isnan(dense[5013:5016]).all()
    assert o.packet_bound(table) >= pk.size


def pin_packet_bound_exact(o):
    """The capacity that can never overflow, against byte counts worked out by hand from the
    container layout (32-byte header, 64-byte record per layer, counts of 1 or 2 bytes per bin,
    one 4-byte running count per 64 bins, words of 1 or 2 bytes, every section padded to 16), and
    against a packet in which every element is sent, which has exactly that size."""
    # the worked example's table: 16 elements, L_T 4 -> 4 bins, 8-bit words
    #   32 + 64 | counts 4 -> 16 | chunks 4 -> 16 | words 16 -> 16
    assert o.packet_bound([(0, 16, 4)]) == 96 + 16 + 16 + 16 == 144
    # one layer with more than 64 bins: 6500 elements, L_T 50 -> 130 bins, 3 chunks
    #   96 | counts 130 -> 144 | chunks 12 -> 16 | words 6500 -> 6512
    assert o.packet_bound([(0, 6500, 50)]) == 96 + 144 + 16 + 6512 == 6768
    # mixed word widths, every last bin short
    table = [(0, 1003, 50),     # 21 bins:  counts 21 -> 32, chunks 4 -> 16, words 1003 -> 1008
             (1004, 777, 500),  # 2 bins:   counts 4 -> 16,  chunks 16,      words 1554 -> 1568
             (1784, 130, 64),   # 3 bins:   counts 3 -> 16,  chunks 16,      words 130 -> 144
             (1916, 66, 65)]    # 2 bins:   counts 4 -> 16,  chunks 16,      words 132 -> 144
    fixed = 32 + 4 * 64 + (32 + 16) + (16 + 16) + (16 + 16) + (16 + 16)
    words = 1008 + 1568 + 144 + 144
    assert fixed == 432 and words == 2864
    assert o.packet_bound(table) == 3296
    # every element sent (equal magnitudes: each one ties with its bin's maximum): the packet is
    # exactly as long as the bound, and one byte less of capacity is refused
    n_total = 1916 + 66
    for tbl, n in [(table, n_total), ([(0, 16, 4)], 16), ([(0, 6500, 50)], 6500)]:
        dW = np.where(np.arange(n) % 3 == 0, -0.25, 0.25).astype(f32)
        pk = o.compress(tbl, dW, np.zeros(n, f32))
        h, layers = pf.parse(pk)
        assert int(h["n_selected"]) == sum(t[1] for t in tbl)
        assert pk.size == o.packet_bound(tbl)
        try:
            o.compress(tbl, dW, np.zeros(n, f32), capacity=o.packet_bound(tbl) - 1)
            raise AssertionError("a capacity one byte below the bound must not hold the all-sent packet")
        except Exception as e:
            assert getattr(e, "code", None) == -4
    assert o.packet_bound([(0, 0, 50)]) == 0 and o.packet_bound([(0, 10, 0)]) == 0


def pin_word_width_boundary(o):
    """8-bit words while the in-bin index fits 6 bits (L_T <= 64), 16-bit words above, up to
    L_T = 16384 where the index needs all 14 bits."""
    for T, bits in [(1, 8), (63, 8), (64, 8), (65, 16), (500, 16), (16384, 16)]:
        n = 2 * T + 1
        R = np.zeros(n, f32)
        R[T - 1] = -1.0                                   # last index of bin 0
        R[2 * T - 1] = 2.0                                # last index of bin 1
        R[2 * T] = 3.0                                    # ragged bin of one element
        pk = o.compress([(0, n, T)], np.zeros(n, f32), R)
        h, layers = pf.parse(pk)
        l = layers[0]
        assert l["rec"]["word_bits"] == bits
        assert l["words"].tolist() == [((T - 1) << 2) | 3, ((T - 1) << 2) | 1, 1]
        assert l["counts"].tolist() == [1, 1, 1]
    try:
        o.compress([(0, 10, 16385)], np.zeros(10, f32), np.zeros(10, f32))
        raise AssertionError("L_T above 16K must be rejected")
    except Exception as e:
        assert getattr(e, "code", None) == -2
    try:
        o.compress([(0, 10, 0)], np.zeros(10, f32), np.zeros(10, f32))
        raise AssertionError("L_T = 0 must be rejected")
    except Exception as e:
        assert getattr(e, "code", None) == -2


def pin_paper_compression_rates(o):
    """Five sent elements per bin give the paper's rates exactly: 50*32/(5*8) = 40 for L_T = 50
    and 500*32/(5*16) = 200 for L_T = 500 (dense bits over word bits)."""
    for T, expect in [(50, 40.0), (500, 200.0)]:
        nb = 130
        n = nb * T
        R = np.full(n, 0.001, f32) * np.where(np.arange(n) % 2 == 0, 1, -1).astype(f32)
        for b in range(nb):                                # five equal maxima per bin, spread out
            R[b * T + np.array([0, 7, T // 2, T - 9, T - 1])] = [1.0, -1.0, 1.0, -1.0, 1.0]
        Rw = R.copy()
        pk = o.compress([(0, n, T)], np.zeros(n, f32), Rw)
        h, layers = pf.parse(pk)
        l = layers[0]
        assert np.all(l["counts"] == 5)
        assert 32.0 * n / (int(l["rec"]["word_bits"]) * int(l["rec"]["n_selected"])) == expect


def pin_unpack_sums_in_learner_order(o):
    """unpack over several learners = plain float32 sum of the decoded vectors, learner 0 first,
    every layer element written (zeros where nobody sent)."""
    table = [(0, 4000, 50), (4000, 9000, 500)]
    n_total = 13000
    pks, decs = [], []
    for k in range(7):
        R = _rand(90 + k, n_total, 10.0 ** (k - 3))        # very different scales -> order matters
        pk = o.compress(table, _rand(190 + k, n_total, 10.0 ** (k - 3)), R)
        pks.append(pk)
        decs.append(pf.decode_dense(pk, n_total))
    acc = np.zeros(n_total, f32)
    for d in decs:
        acc = acc + d                                       # float32 adds in learner order
    got = o.unpack_accumulate(table, pks, n_total)
    assert np.array_equal(got, acc)
    rev = np.zeros(n_total, f32)
    for d in decs[::-1]:
        rev = rev + d
    assert not np.array_equal(rev, acc)                     # the order is observable on this input
    assert np.array_equal(o.unpack_accumulate(table, [], n_total), np.zeros(n_total, f32))


def pin_brute_force_tiny(o):
    """Every (residue, dW) pair over a small dyadic grid, 2 bins of 2: with dyadic values the
    mathematical result is exact in double precision, so selection, scale and residue are checked
    against the set definition evaluated in exact arithmetic."""
    vals = [-1.0, -0.5, 0.0, 0.25, 1.0]
    grid = np.array(np.meshgrid(*[vals] * 4, indexing="ij")).reshape(4, -1).T   # 625 residues
    rng = np.random.default_rng(5)
    for R in grid[::3]:
        for dW in grid[rng.integers(0, len(grid), 12)]:
            r = o.pack_layer(R.astype(f32), dW.astype(f32), 2)
            G = R + dW
            H = R + 2 * dW
            M = [max(abs(G[0]), abs(G[1])), max(abs(G[2]), abs(G[3]))]
            s = (M[0] + M[1]) / 2
            for e in range(4):
                m = M[e // 2]
                sent = G[e] != 0 and (abs(H[e]) >= m or abs(G[e]) >= m)
                assert bool(r["selected"][e]) == sent
                want = G[e] - (s if G[e] > 0 else -s) if sent else G[e]
                assert float(r["residue"][e]) == want
            assert float(r["scale"]) == s


def pin_capacity_and_bad_arguments(o):
    """A packet that does not fit is refused and leaves the residue untouched; bad tables are
    refused: zero-length layer, misaligned offset, overlapping layers."""
    n = 1000
    R, dW = _rand(1, n), _rand(2, n)
    R0 = R.copy()
    try:
        o.compress([(0, n, 50)], dW, R, capacity=200)
        raise AssertionError("must not fit")
    except Exception as e:
        assert getattr(e, "code", None) == -4
    assert np.array_equal(R, R0)
    for bad, code in [([(0, 0, 50)], -1), ([(2, 10, 50)], -3), ([(0, 100, 50), (96, 100, 50)], -1)]:
        try:
            o.compress(bad, np.zeros(300, f32), np.zeros(300, f32))
            raise AssertionError("bad table accepted")
        except Exception as e:
            assert getattr(e, "code", None) == code, (bad, e)


def pin_variant_rules(o):
    """The two ablation rules: the printed compare alone (drops a maximum that dW opposes, sends a
    zero whose H is large) and local selection (maxima only)."""
    import oracle as om
    g = _read_golden("worked_example_T4.txt")
    R, dW = np.array(g["residue"], f32), np.array(g["dW"], f32)
    lit = o.pack_layer(R, dW, 4, rule=om.RULE_LITERAL)
    assert np.flatnonzero(lit["selected"]).tolist() == [1, 2, 6, 7, 12, 13]
    ls = o.pack_layer(R, dW, 4, rule=om.RULE_LS)
    assert np.flatnonzero(ls["selected"]).tolist() == [1, 6, 8, 13]


def pin_soft_threshold_factor(o):
    """Other soft-threshold factors (the paper studied 1.5 - 3.0 and chose 2): the operand is
    residue + f dW.  With residue = 0 and dyadic gradients everything is exact, so the sent set is
    {f |dW| >= bin max |dW|}; f = 1 adds nothing to local selection; f = 2 is the default path;
    for random inputs H equals numpy's float32 G + (f - 1) * dW bit for bit."""
    import oracle as om
    n, T = 4000, 50
    dW = (np.round(_rand(91, n) * 64) / 64).astype(f32)
    gm = _binmax(dW, T)[np.arange(n) // T]
    for f in (1.5, 3.0, 2.0):
        r = o.pack_layer(np.zeros(n, f32), dW, T, soft_factor=f)
        expect = (np.abs(dW.astype(np.float64)) * f >= gm) & (dW != 0)
        assert np.array_equal(r["selected"], expect), f
    counts = [o.pack_layer(np.zeros(n, f32), dW, T, soft_factor=f)["n_selected"] for f in (1.0, 1.5, 2.0, 3.0)]
    assert counts == sorted(counts) and counts[0] < counts[-1]      # a larger factor sends more here
    R, g = _rand(92, n), _rand(93, n, 0.4)
    base = o.pack_layer(R, g, T)
    same = o.pack_layer(R, g, T, soft_factor=2.0)
    assert np.array_equal(base["H"], same["H"]) and np.array_equal(base["selected"], same["selected"])
    one = o.pack_layer(R, g, T, soft_factor=1.0)
    ls = o.pack_layer(R, g, T, rule=om.RULE_LS)
    assert np.array_equal(one["selected"], ls["selected"]) and np.array_equal(one["residue"], ls["residue"])
    for f in (1.5, 2.5, 3.0):
        r = o.pack_layer(R, g, T, soft_factor=f)
        G = R + g
        assert np.array_equal(r["H"], G + f32(f - 1.0) * g)
        assert np.array_equal(r["G"], G) and np.array_equal(r["gmax"], _binmax(G, T))   # the threshold does not move
    for bad in (0.5, 17.0, float("nan")):
        try:
            o.pack_layer(R, g, T, soft_factor=bad)
            raise AssertionError("factor outside 1..16 accepted")
        except ValueError:
            pass


def pin_update_sgd(o):
    """averageGradients + SGD with momentum: closed forms.  lr = 0 leaves the weights alone; with
    momentum 0 the step is lr * sum / n; a constant gradient builds the geometric series
    v_k = g (1 - mu^k) / (1 - mu); elements outside the layers are untouched."""
    table = [(0, 1001, 50), (1004, 700, 500)]
    n = 1704
    mask = np.zeros(n, bool)
    mask[:1001] = True
    mask[1004:] = True
    s = _rand(101, n)
    w0 = _rand(102, n)
    w, v = w0.copy(), np.zeros(n, f32)
    o.update_sgd(table, s, 4, w, v, 0.0, 0.9)
    assert np.array_equal(w[mask], w0[mask]) and np.array_equal(v[mask], s[mask] / f32(4))
    assert np.all(v[~mask] == 0) and np.array_equal(w[~mask], w0[~mask])
    w, v = w0.copy(), np.zeros(n, f32)
    o.update_sgd(table, s, 8, w, v, 0.5, 0.0)             # all dyadic factors: exact
    assert np.array_equal(w[mask], (w0 - f32(0.5) * (s / f32(8)))[mask])
    # geometric series with dyadic numbers (mu = 0.5, g = 1): v_k = 2 - 2^(1-k) exactly
    ones = np.ones(n, f32) * f32(3)
    w, v = np.zeros(n, f32), np.zeros(n, f32)
    for k in range(1, 11):
        o.update_sgd(table, ones, 3, w, v, 0.25, 0.5)
        assert np.all(v[mask] == f32(2.0 - 2.0 ** (1 - k)))
    assert np.all(w[mask] == f32(-0.25 * sum(2.0 - 2.0 ** (1 - k) for k in range(1, 11))))
    # general values: the same sequence of float32 operations in numpy
    w, v = w0.copy(), _rand(103, n)
    v0 = v.copy()
    o.update_sgd(table, s, 7, w, v, 0.01, 0.9)
    g = s / f32(7)
    v_ref = f32(0.9) * v0 + g
    assert np.array_equal(v[mask], v_ref[mask]) and np.array_equal(w[mask], (w0 - f32(0.01) * v_ref)[mask])


def pin_update_adam(o):
    """averageGradients + Adam: from zero state at t = 1, m_hat = g and v_hat = g^2, so the first
    step is lr * g / (|g| + eps): magnitude lr (to within eps / |g|), sign of g, whatever the
    gradient's size (the scale invariance of Adam); a zero gradient moves nothing."""
    table = [(0, 900, 50)]
    n = 900
    g4 = _rand(111, n) * f32(10.0) ** np.random.default_rng(5).integers(-3, 3, n).astype(f32)
    g4[::50] = 0
    lr, b1, b2, eps = 1e-3, 0.9, 0.999, 1e-8
    w, m, v = np.zeros(n, f32), np.zeros(n, f32), np.zeros(n, f32)
    o.update_adam(table, g4 * f32(4), 4, w, m, v, lr, b1, b2, eps, 1 - b1, 1 - b2)
    nz = g4 != 0
    assert np.all(w[~nz] == 0) and np.all(m[~nz] == 0) and np.all(v[~nz] == 0)
    assert np.all(np.sign(w[nz]) == -np.sign(g4[nz]))
    a64 = np.abs(g4[nz].astype(np.float64))
    assert np.allclose(np.abs(w[nz]), lr * a64 / (a64 + eps), rtol=1e-5)
    assert np.all(np.abs(w[nz]) <= lr * (1 + 2e-5)) and np.median(np.abs(w[nz])) > 0.99 * lr
    omb1, omb2 = float(f32(1) - f32(b1)), float(f32(1) - f32(b2))   # the one-minus-beta factors are float32
    assert np.allclose(m[nz], omb1 * g4[nz].astype(np.float64), rtol=1e-6)
    assert np.allclose(v[nz], omb2 * g4[nz].astype(np.float64) ** 2, rtol=1e-6)
    # steady state with a constant gradient: m -> g, v -> g^2, step -> lr * sign(g)
    w, m, v = np.zeros(n, f32), np.zeros(n, f32), np.zeros(n, f32)
    for t in range(1, 60):
        w_before = w.copy()
        o.update_adam(table, g4, 1, w, m, v, lr, b1, b2, eps, 1 - b1 ** t, 1 - b2 ** t)
    big = np.abs(g4) > 1e-4
    assert np.allclose((w_before - w)[big], lr * np.sign(g4[big]), rtol=2e-3)
    # general values: the same sequence of float32 operations in numpy (sqrt and divide are
    # correctly rounded in both)
    w0, m0, v0 = _rand(112, n), _rand(113, n, 0.1), np.abs(_rand(114, n, 0.01))
    w, m, v = w0.copy(), m0.copy(), v0.copy()
    o.update_adam(table, g4, 3, w, m, v, lr, b1, b2, eps, 0.19, 0.002)
    g = g4 / f32(3)
    m_ref = f32(b1) * m0 + (f32(1) - f32(b1)) * g
    v_ref = f32(b2) * v0 + (f32(1) - f32(b2)) * (g * g)
    w_ref = w0 - f32(lr) * ((m_ref / f32(0.19)) / (np.sqrt(v_ref / f32(0.002)) + f32(eps)))
    assert np.array_equal(m, m_ref) and np.array_equal(v, v_ref) and np.array_equal(w, w_ref)


PINS = [v for k, v in sorted(globals().items()) if k.startswith("pin_")]
