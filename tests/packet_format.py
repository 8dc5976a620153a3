"""Packet reader used by the tests only: a third, independent statement of the container layout
(the oracle's C and the library's header are the other two).  numpy views, no method arithmetic.

Layout: 32-byte header {u32 magic 'ADCP', u32 version, u32 status, u32 n_layers, u64 total_bytes,
u64 n_selected}; n_layers 64-byte records {u64 elem_offset, u64 n_elems, u32 L_T, u32 n_bins,
u32 word_bits, f32 scale, u64 n_selected, u64 counts_offset, u64 chunks_offset, u64 words_offset};
per layer counts (u8|u16) and chunk offsets (u32 per 64 bins); then per layer words (u8|u16);
every section 16-byte aligned, padding zero.  The 8/16-bit word widths and the 2-bit ternary
field are those of the paper's section "Experiment Results".
"""
import numpy as np

MAGIC = 0x50434441
HEADER = np.dtype([("magic", "<u4"), ("version", "<u4"), ("status", "<u4"), ("n_layers", "<u4"),
                   ("total_bytes", "<u8"), ("n_selected", "<u8")])
RECORD = np.dtype([("elem_offset", "<u8"), ("n_elems", "<u8"), ("L_T", "<u4"), ("n_bins", "<u4"),
                   ("word_bits", "<u4"), ("scale", "<f4"), ("n_selected", "<u8"),
                   ("counts_offset", "<u8"), ("chunks_offset", "<u8"), ("words_offset", "<u8")])
assert HEADER.itemsize == 32 and RECORD.itemsize == 64


def header(buf):
    return np.frombuffer(np.asarray(buf, np.uint8)[:32].tobytes(), HEADER)[0]


def parse(buf, check=True):
    """Return (header, [layer dicts]) and, with check=True, assert every structural invariant."""
    buf = np.ascontiguousarray(buf, dtype=np.uint8)
    h = header(buf)
    recs = np.frombuffer(buf[32:32 + 64 * int(h["n_layers"])].tobytes(), RECORD)
    layers = []
    covered = np.zeros(int(h["total_bytes"]), bool) if check else None
    if check:
        assert h["magic"] == MAGIC and h["version"] == 1
        assert h["total_bytes"] % 16 == 0 and h["total_bytes"] <= buf.size
        covered[:32 + 64 * len(recs)] = True
    for r in recs:
        wdt = np.dtype("<u1") if r["word_bits"] == 8 else np.dtype("<u2")
        nb, ns = int(r["n_bins"]), int(r["n_selected"])
        nch = (nb + 63) // 64
        co, cho, wo = int(r["counts_offset"]), int(r["chunks_offset"]), int(r["words_offset"])
        counts = np.frombuffer(buf[co:co + nb * wdt.itemsize].tobytes(), wdt).astype(np.int64)
        chunks = np.frombuffer(buf[cho:cho + 4 * nch].tobytes(), "<u4").astype(np.int64)
        if h["status"] == 0:
            words = np.frombuffer(buf[wo:wo + ns * wdt.itemsize].tobytes(), wdt).astype(np.int64)
        else:
            words = None
        layers.append({"rec": r, "counts": counts, "chunks": chunks, "words": words})
        if check:
            T, n = int(r["L_T"]), int(r["n_elems"])
            assert r["word_bits"] == (8 if T <= 64 else 16)
            assert nb == (n + T - 1) // T
            assert co % 16 == 0 and cho % 16 == 0 and wo % 16 == 0
            assert counts.sum() == ns
            prefix = np.concatenate([[0], np.cumsum(counts)])
            assert np.array_equal(chunks, prefix[0:nb:64])
            if words is not None:
                assert len(words) == ns
                code = words & 3
                assert np.all((code == 1) | (code == 3))
                idx = words >> 2
                bin_of_word = np.repeat(np.arange(nb), counts)
                bin_len = np.minimum(T, n - bin_of_word * T)
                assert np.all(idx < bin_len)
                same_bin = bin_of_word[1:] == bin_of_word[:-1]
                assert np.all(idx[1:][same_bin] > idx[:-1][same_bin])  # strictly ascending in a bin
                covered[wo:wo + ns * wdt.itemsize] = True
            covered[co:co + nb * wdt.itemsize] = True
            covered[cho:cho + 4 * nch] = True
    if check:
        assert h["n_selected"] == sum(int(l["rec"]["n_selected"]) for l in layers)
        # sections sit back to back in the stated order, each padded to 16 bytes
        pad16 = lambda x: (x + 15) // 16 * 16
        off = 32 + 64 * len(recs)
        for l in layers:
            r = l["rec"]
            wb = int(r["word_bits"]) // 8
            assert r["counts_offset"] == off
            off += pad16(int(r["n_bins"]) * wb)
            assert r["chunks_offset"] == off
            off += pad16(4 * ((int(r["n_bins"]) + 63) // 64))
        for l in layers:
            r = l["rec"]
            assert r["words_offset"] == off
            off += pad16(int(r["n_selected"]) * (int(r["word_bits"]) // 8))
        assert h["total_bytes"] == off
        if h["status"] == 0:
            assert np.all(buf[:int(h["total_bytes"])][~covered] == 0), "padding bytes must be zero"
    return h, layers


def selected_indices(layer):
    """Layer-local element indices of the words, in packet order, and their signs (+1 / -1)."""
    r = layer["rec"]
    bin_of_word = np.repeat(np.arange(int(r["n_bins"])), layer["counts"])
    idx = bin_of_word * int(r["L_T"]) + (layer["words"] >> 2)
    sign = np.where((layer["words"] & 3) == 1, 1, -1)
    return idx, sign


def decode_dense(buf, n_total):
    """Dense float32 vector of one packet: +-scale at the sent positions, 0 elsewhere in layers."""
    h, layers = parse(buf, check=False)
    out = np.zeros(n_total, np.float32)
    for l in layers:
        idx, sign = selected_indices(l)
        out[int(l["rec"]["elem_offset"]) + idx] = sign.astype(np.float32) * np.float32(l["rec"]["scale"])
    return out
