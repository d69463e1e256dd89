"""Pins for the CPU oracle: what the paper and the mathematics fix, checked
without any reference to the HIP library.

Each test names the passage it pins.  The brute-force re-implementations here
are deliberately written in another style (numpy / pure-Python loops / scipy)
than the C oracle, on inputs small enough to check by eye.
"""
from __future__ import annotations

import os

import numpy as np
import pytest
import scipy.sparse as sp

import gqsa_inputs as gi
import oracle


# ----------------------------------------------------------------------------- helpers

def unpack_codes(c):
    """Canonical `values` -> integer codes [nnzg, G] (low nibble = even element)."""
    v = np.asarray(c.values, dtype=np.uint8)
    if c.bits == 8:
        return v.reshape(c.nnzg, c.G).astype(np.int64)
    out = np.empty((c.nnzg, c.G), dtype=np.int64)
    v = v.reshape(c.nnzg, c.G // 2)
    out[:, 0::2] = v & 0xF
    out[:, 1::2] = v >> 4
    return out


def half(bits):
    return np.asarray(bits, dtype=np.uint16).view(np.float16).astype(np.float64)


def brute_dense(c):
    """Pure-Python densification of Eq. 3, pruned groups zero."""
    Wd = np.zeros((c.N, c.K))
    q = unpack_codes(c)
    s = half(c.scales)
    z = half(c.zeros)
    for n in range(c.N):
        for g in range(int(c.rowIndex[n]), int(c.rowIndex[n + 1])):
            col = int(c.groups[g])
            for j in range(c.G):
                Wd[n, col * c.G + j] = (q[g, j] - z[g]) * s[g]
    return Wd


def numpy_group_quant(W, G, bits):
    """Dense per-group asymmetric quantiser (Eq. 1-2) in numpy fp32, every group kept."""
    N, K = W.shape
    w = W.reshape(N, K // G, G).astype(np.float32)
    qmax = np.float32(2 ** bits - 1)
    mn = w.min(-1)
    mx = w.max(-1)
    s16 = ((mx - mn) / qmax).astype(np.float16)
    s16 = np.where(s16 >= np.float16(2.0 ** -14), s16, np.float16(2.0 ** -14)).astype(np.float16)
    sf = s16.astype(np.float32)
    z = np.clip(np.rint(-mn / sf), -2048, 2048).astype(np.float32)
    q = np.clip(np.rint(w / sf[..., None]) + z[..., None], 0, qmax)
    return q.astype(np.int64), s16, z.astype(np.float16)


# ----------------------------------------------------------------------------- fp16

def test_f16_to_f32_all_patterns():
    """Every binary16 pattern widens exactly as IEEE-754 says (numpy as the library)."""
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float32)
    got = np.array([oracle.f16_bits_to_f32(int(b)) for b in bits], dtype=np.float32)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), ref[~nan].view(np.uint32))


def test_f32_to_f16_round_to_nearest_even():
    rng = np.random.default_rng(5)
    vals = np.concatenate([
        rng.standard_normal(20000).astype(np.float32) * np.float32(0.01),
        rng.standard_normal(20000).astype(np.float32) * np.float32(100.0),
        (rng.standard_normal(5000) * 1e-6).astype(np.float32),       # subnormal halves
        np.array([0.0, -0.0, 65504.0, 65519.9, 65520.0, 1e9, -1e9, 2.0 ** -24, 2.0 ** -25,
                  1.5 * 2.0 ** -24, 2.5 * 2.0 ** -24, 2.0 ** -14, 1024.5, 1025.5, 2049.0,
                  2051.0, np.inf, -np.inf], dtype=np.float32),
    ])
    # exact ties between neighbouring halves
    h = rng.integers(0, 0x7BFF, size=5000).astype(np.uint16)
    lo = h.view(np.float16).astype(np.float64)
    hi = (h + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    ties = ((lo + hi) / 2).astype(np.float32)
    vals = np.concatenate([vals, ties, -ties])
    ref = vals.astype(np.float16).view(np.uint16)
    got = np.array([oracle.f32_to_f16_bits(float(v)) for v in vals], dtype=np.uint16)
    assert np.array_equal(got, ref)


# ----------------------------------------------------------------------------- quantiser (Eq. 1-2)

def test_quantiser_hand_example_exact():
    """Eq. 1-2 by hand: w = -1, -0.875, ..., 0.875 -> s = 1.875/15 = 0.125, z = 8, q = 0..15."""
    w = (np.arange(16, dtype=np.float32) - 8) * np.float32(0.125)
    c = oracle.pack(w[None, :], G=16, bits=4, sparsity=0.0)
    assert c.nnzg == 1 and list(c.rowIndex) == [0, 1] and list(c.groups) == [0]
    assert half(c.scales)[0] == 0.125
    assert half(c.zeros)[0] == 8.0
    assert list(unpack_codes(c)[0]) == list(range(16))
    # nibble order: byte b holds element 2b in the low nibble, 2b+1 in the high nibble
    assert list(c.values) == [(2 * b) | ((2 * b + 1) << 4) for b in range(8)]


def test_quantiser_hand_example_8bit():
    """Same with n = 8: w = k/4 for k = -100..155 sampled at 16 points incl. both ends."""
    ks = np.array([-100, 155, 0, 1, -1, 17, 33, 64, 100, 127, -50, -99, 154, 3, 5, 7])
    w = ks.astype(np.float32) * np.float32(0.25)
    c = oracle.pack(w[None, :], G=16, bits=8, sparsity=0.0)
    assert half(c.scales)[0] == 0.25            # 63.75 / 255
    assert half(c.zeros)[0] == 100.0
    assert list(unpack_codes(c)[0]) == list(ks + 100)
    assert c.values.size == 16


def test_quantiser_closed_form_properties():
    """For a non-degenerate group: code(min) = 0, code(max) in {2^n-2, 2^n-1},
    and |W - W^| <= (1/2 + (2^n-1) 2^-11) s  (rounding of q plus the fp16 rounding of s)."""
    W = gi.dense_weight(64, 512, seed=11, outliers=True)
    for bits in (4, 8):
        qmax = 2 ** bits - 1
        c = oracle.pack(W, G=16, bits=bits, sparsity=0.0)
        q = unpack_codes(c).reshape(64, 32, 16)
        w = W.reshape(64, 32, 16)
        amin = w.argmin(-1)
        amax = w.argmax(-1)
        qmin = np.take_along_axis(q, amin[..., None], -1)[..., 0]
        qmaxc = np.take_along_axis(q, amax[..., None], -1)[..., 0]
        assert (qmin == 0).all()
        assert ((qmaxc == qmax) | (qmaxc == qmax - 1)).all()
        s = half(c.scales).reshape(64, 32)
        z = half(c.zeros).reshape(64, 32)
        what = (q - z[..., None]) * s[..., None]
        bound = (0.5 + qmax * 2.0 ** -11) * s[..., None] * (1 + 1e-6)
        assert (np.abs(what - w) <= bound).all()
        assert (z == np.rint(z)).all()


def test_quantiser_lossless_construction():
    """W built as (q - z) * s with s a power of two and q covering 0 and 2^n-1 packs
    back to exactly q, z, s: pins sign of z, the clamp and the order of the codes."""
    rng = np.random.default_rng(3)
    for bits in (4, 8):
        qmax = 2 ** bits - 1
        N, KG, G = 8, 6, 16
        q = rng.integers(0, qmax + 1, size=(N, KG, G))
        q[..., 3] = 0
        q[..., 9] = qmax
        z = rng.integers(-20, qmax + 20, size=(N, KG))
        s = 2.0 ** rng.integers(-9, -3, size=(N, KG))
        W = ((q - z[..., None]) * s[..., None]).astype(np.float32).reshape(N, KG * G)
        c = oracle.pack(W, G=G, bits=bits, sparsity=0.0)
        assert np.array_equal(unpack_codes(c).reshape(N, KG, G), q)
        assert np.array_equal(half(c.zeros).reshape(N, KG), z)
        assert np.array_equal(half(c.scales).reshape(N, KG), s)
        assert np.array_equal(oracle.densify(c), W.astype(np.float64))


def test_quantiser_degenerate_group_gets_scale_floor():
    W = np.full((2, 32), 0.03, dtype=np.float32)
    W[1, 16:] = np.float32(0.03) + np.arange(16, dtype=np.float32) * np.float32(1e-7)  # fp16 underflow of s
    c = oracle.pack(W, G=16, bits=4, sparsity=0.0)
    assert (c.scales == 0x0400).all()            # 2^-14
    what = oracle.densify(c)
    assert (np.abs(what - W) <= 0.5 * 2.0 ** -14 + 1e-12).all()


def test_quantiser_matches_numpy_dense_group_quant():
    """S = 0 reduces to ordinary dense per-group quantisation (library: numpy fp32/fp16)."""
    W = gi.dense_weight(48, 256, seed=21, outliers=True)
    for bits in (4, 8):
        c = oracle.pack(W, G=16, bits=bits, sparsity=0.0)
        q, s16, z16 = numpy_group_quant(W, 16, bits)
        assert np.array_equal(unpack_codes(c).reshape(48, 16, 16), q)
        assert np.array_equal(c.scales.reshape(48, 16), s16.view(np.uint16))
        assert np.array_equal(c.zeros.reshape(48, 16), z16.view(np.uint16))
        assert np.array_equal(c.groups.reshape(48, 16), np.tile(np.arange(16), (48, 1)))


# ----------------------------------------------------------------------------- pruning (Sec. 3.2, Fig. 3)

def test_keep_count_rounding():
    assert oracle.keep_counts(1, 4096, 16, 0.3)[0] == 256 - 77
    assert oracle.keep_counts(1, 4096, 16, 0.7)[0] == 256 - 179
    assert oracle.keep_counts(1, 14336, 16, 0.3)[0] == 896 - 269
    assert oracle.keep_counts(1, 14336, 16, 0.7)[0] == 896 - 627
    assert oracle.keep_counts(1, 4096, 16, 0.5)[0] == 128
    assert oracle.keep_counts(1, 4096, 16, 0.0)[0] == 256
    assert oracle.keep_counts(1, 4096, 16, 1.0)[0] == 0
    assert oracle.keep_counts(1, 48, 16, 0.5)[0] == 1          # 1.5 pruned -> 2


def test_pruning_matches_brute_force_argsort():
    W, _ = gi.tiny_config()
    c = oracle.pack(W, G=16, bits=4, sparsity=0.5)
    norms = np.sqrt((W.astype(np.float64).reshape(256, 16, 16) ** 2).sum(-1))
    for n in range(256):
        kept = np.sort(np.argsort(norms[n], kind="stable")[8:])
        got = c.groups[c.rowIndex[n]:c.rowIndex[n + 1]]
        assert np.array_equal(got, kept)
    assert np.array_equal(np.diff(c.rowIndex), np.full(256, 8))


def test_pruning_ties_lower_column_pruned_first():
    g = np.linspace(-1, 1, 16).astype(np.float32)
    W = np.zeros((3, 6 * 16), dtype=np.float32)
    for col in range(6):
        W[0, col * 16:(col + 1) * 16] = g              # six identical groups
    W[1, 2 * 16:3 * 16] = g                            # zero groups tie too
    W[1, 5 * 16:6 * 16] = g * 2
    W[2] = W[0]
    c = oracle.pack(W, G=16, bits=4, keep_per_row=np.array([2, 3, 6], dtype=np.int32))
    assert list(c.groups[c.rowIndex[0]:c.rowIndex[1]]) == [4, 5]
    assert list(c.groups[c.rowIndex[1]:c.rowIndex[2]]) == [2, 4, 5]   # zeros 0,1,3 pruned first, 4 survives
    assert list(c.groups[c.rowIndex[2]:c.rowIndex[3]]) == [0, 1, 2, 3, 4, 5]


def test_hessian_saliency_matches_brute_force():
    """Eq. 4: saliency of a weight = w^2 / d_k^2, d = diag(H^-1); a group's = the sum over it."""
    rng = np.random.default_rng(21)
    N, K, G = 24, 192, 16
    W = rng.standard_normal((N, K)).astype(np.float32)
    d = np.exp(rng.standard_normal(K)).astype(np.float32)          # positive, spread over ~2 decades
    c = oracle.pack(W, G=G, bits=4, sparsity=0.5, hinv_diag=d)
    sal = ((W.astype(np.float64) / d.astype(np.float64)) ** 2).reshape(N, K // G, G).sum(-1)
    for n in range(N):
        kept = np.sort(np.argsort(sal[n], kind="stable")[K // G // 2:])
        assert np.array_equal(c.groups[c.rowIndex[n]:c.rowIndex[n + 1]], kept)
    # the selection differs from plain magnitude pruning here, the quantiser does not: every
    # stored group carries the codes magnitude packing gives that same group
    m = oracle.pack(W, G=G, bits=4, sparsity=0.0)
    differs = False
    for n in range(N):
        cols = c.groups[c.rowIndex[n]:c.rowIndex[n + 1]]
        mag = np.sort(np.argsort((W[n].astype(np.float64) ** 2).reshape(-1, G).sum(-1), kind="stable")[K // G // 2:])
        differs |= not np.array_equal(cols, mag)
        for i, col in enumerate(cols):
            g, gm = c.rowIndex[n] + i, m.rowIndex[n] + col
            assert np.array_equal(c.values[8 * g:8 * g + 8], m.values[8 * gm:8 * gm + 8])
            assert c.scales[g] == m.scales[gm] and c.zeros[g] == m.zeros[gm]
    assert differs


def test_hessian_saliency_special_cases():
    W = gi.dense_weight(32, 256, seed=22)
    base = oracle.pack(W, sparsity=0.5)
    for const in (1.0, 0.5, 4.0):          # a constant d (exact powers of two) changes nothing
        c = oracle.pack(W, sparsity=0.5, hinv_diag=np.full(256, const, dtype=np.float32))
        assert np.array_equal(c.groups, base.groups) and np.array_equal(c.values, base.values)
    # a huge d on some input columns makes their groups the first to go, a tiny d the last
    d = np.ones(256, dtype=np.float32)
    d[0:16] = 1e6          # group-column 0: irrelevant inputs
    d[32:48] = 1e-6        # group-column 2: inputs that matter most
    c = oracle.pack(W, sparsity=0.5, hinv_diag=d)
    for n in range(32):
        cols = list(c.groups[c.rowIndex[n]:c.rowIndex[n + 1]])
        assert 0 not in cols and 2 in cols
    for bad in (0.0, -1.0, np.inf, np.nan):
        d = np.ones(256, dtype=np.float32)
        d[7] = bad
        with pytest.raises(ValueError):
            oracle.pack(W, sparsity=0.5, hinv_diag=d)


def test_sparsity_extremes():
    W = gi.dense_weight(16, 128, seed=4)
    c0 = oracle.pack(W, sparsity=0.0)
    c1 = oracle.pack(W, sparsity=1.0)
    assert c0.nnzg == 16 * 8 and c1.nnzg == 0
    assert np.array_equal(c1.rowIndex, np.zeros(17, dtype=np.int32))
    x = gi.activations(2, 128, seed=4)
    y = oracle.gemv(c1, x)
    assert y.shape == (2, 16) and not y.any() and not np.signbit(y).any()


# ----------------------------------------------------------------------------- BSR structure (Sec. 3.2 listing)

def _read_golden(path):
    out = {}
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, v = line.split("=")
        out[k.strip()] = [int(t) for t in v.split()]
    return out


def test_paper_worked_bsr_example_structure(golden_dir):
    gold = _read_golden(os.path.join(golden_dir, "paper_bsr_example.txt"))
    G = gold["group_size"][0]
    rows = gold["rows"][0]
    kg = gold["group_columns"][0]
    # a matrix whose group norms force the kept pattern of the listing
    rng = np.random.default_rng(0)
    W = rng.standard_normal((rows, kg * G)).astype(np.float32)
    W[0, :G] *= 0.01           # row 0 keeps column 1
    W[3, :G] *= 0.01           # row 3 keeps column 1
    keep = np.array([1, 2, 0, 1], dtype=np.int32)
    c = oracle.pack(W, G=G, bits=4, keep_per_row=keep)
    assert list(c.rowIndex) == gold["rowIndex"]
    assert list(c.groups) == gold["groups"]
    assert unpack_codes(c).size == gold["n_values"][0]
    assert c.rowIndex[rows] == c.nnzg == len(gold["groups"])
    # values are stored row after row, group after group: group 2 is row 1's column-1 group
    q, s16, z16 = numpy_group_quant(W, G, 4)
    assert np.array_equal(unpack_codes(c)[2], q[1, 1])
    assert np.array_equal(unpack_codes(c)[0], q[0, 1])


def test_bsr_invariants_balanced_and_imbalanced():
    W = gi.dense_weight(200, 512, seed=9)
    keep = gi.imbalanced_keep_counts(200, 32, seed=9)
    for kw in (dict(sparsity=0.3), dict(keep_per_row=keep)):
        c = oracle.pack(W, **kw)
        assert c.rowIndex[0] == 0 and c.rowIndex[-1] == c.nnzg
        d = np.diff(c.rowIndex)
        assert (d >= 0).all()
        if "keep_per_row" in kw:
            assert np.array_equal(d, keep)
        else:
            assert (d == 32 - 10).all()          # floor(0.3*32+0.5) = 10 pruned
        for n in range(200):
            g = c.groups[c.rowIndex[n]:c.rowIndex[n + 1]]
            assert (np.diff(g) > 0).all() and (g >= 0).all() and (g < 32).all()


# ----------------------------------------------------------------------------- GEMV value (Sec. 3.5, Eq. 3)

@pytest.mark.parametrize("bits", [4, 8])
def test_gemv_matches_brute_force_dense_product(bits):
    W, x = gi.tiny_config()
    keep = gi.imbalanced_keep_counts(256, 16, seed=1)
    for kw in (dict(sparsity=0.5), dict(keep_per_row=keep)):
        c = oracle.pack(W, bits=bits, **kw)
        Wd = brute_dense(c)
        assert np.array_equal(oracle.densify(c), Wd)
        xb = gi.activations(3, 256, seed=7)
        ref = xb.astype(np.float64) @ Wd.T
        got = oracle.gemv(c, xb)
        assert np.allclose(got, ref, rtol=1e-12, atol=1e-13)
        # pruned groups are exactly zero in the dense view
        mask = np.zeros((256, 16), dtype=bool)
        for n in range(256):
            mask[n, c.groups[c.rowIndex[n]:c.rowIndex[n + 1]]] = True
        assert not Wd.reshape(256, 16, 16)[~mask].any()


def test_gemv_matches_scipy_bsr_product():
    W = gi.dense_weight(96, 640, seed=13)
    keep = gi.imbalanced_keep_counts(96, 40, seed=13)
    c = oracle.pack(W, keep_per_row=keep)
    q = unpack_codes(c).astype(np.float64)
    data = (q - half(c.zeros)[:, None]) * half(c.scales)[:, None]
    A = sp.bsr_matrix((data.reshape(c.nnzg, 1, 16), c.groups, c.rowIndex), shape=(96, 640))
    x = gi.activations(2, 640, seed=13)
    ref = (A @ x.astype(np.float64).T).T
    got = oracle.gemv(c, x)
    assert np.allclose(got, ref, rtol=1e-12, atol=1e-13)


def test_gemv_s0_is_plain_group_quantised_gemv():
    W = gi.dense_weight(40, 320, seed=17)
    q, s16, z16 = numpy_group_quant(W, 16, 4)
    Wd = ((q - z16.astype(np.float64)[..., None]) * s16.astype(np.float64)[..., None]).reshape(40, 320)
    x = gi.activations(1, 320, seed=17)
    c = oracle.pack(W, sparsity=0.0)
    assert np.allclose(oracle.gemv(c, x), x.astype(np.float64) @ Wd.T, rtol=1e-12, atol=1e-13)


def test_gemv_empty_rows_are_exact_plus_zero():
    W = gi.dense_weight(12, 64, seed=2)
    keep = np.array([0, 4, 0, 0, 2, 1, 0, 4, 3, 0, 0, 0], dtype=np.int32)
    c = oracle.pack(W, keep_per_row=keep)
    y = oracle.gemv(c, gi.activations(2, 64, seed=2))
    assert (y[:, keep == 0] == 0).all() and not np.signbit(y[:, keep == 0]).any()
    assert (y[:, keep > 0] != 0).all()


def test_gemv_unit_and_ones_vectors():
    """x = e_k picks column k of W^; x = 1 gives its row sums."""
    W = gi.dense_weight(32, 128, seed=23)
    c = oracle.pack(W, sparsity=0.5)
    Wd = brute_dense(c)
    for k in (0, 17, 127):
        assert np.array_equal(oracle.gemv(c, gi.unit_vector(128, k))[0], Wd[:, k])
    assert np.allclose(oracle.gemv(c, gi.ones_vector(128))[0], Wd.sum(1), rtol=1e-13, atol=1e-15)


def test_gemv_linearity_and_batch_independence():
    W = gi.dense_weight(32, 256, seed=29)
    c = oracle.pack(W, sparsity=0.5)
    x = gi.activations(4, 256, seed=29)
    y = oracle.gemv(c, x)
    for b in range(4):
        assert np.array_equal(oracle.gemv(c, x[b:b + 1])[0], y[b])
    # exact halves so that x1 + x2 is representable: use small integers
    x1 = np.rint(x[0].astype(np.float32) * 4).astype(np.float16)
    x2 = np.rint(x[1].astype(np.float32) * 4).astype(np.float16)
    y12 = oracle.gemv(c, (x1 + x2)[None])[0]
    assert np.allclose(y12, oracle.gemv(c, x1[None])[0] + oracle.gemv(c, x2[None])[0],
                       rtol=1e-12, atol=1e-12)


def test_gemv_threads_do_not_change_the_result():
    W = gi.dense_weight(64, 256, seed=31)
    c = oracle.pack(W, sparsity=0.5)
    x = gi.activations(1, 256, seed=31)
    assert np.array_equal(oracle.gemv(c, x, threads=1), oracle.gemv(c, x, threads=4))


def test_rel_error_metric():
    ref = np.array([1.0, -2.0, 0.0, 1e-6])
    rms = np.sqrt(np.mean(ref ** 2))
    y = ref + np.array([1e-3, 0.0, 1e-4, 0.0])
    exp = max(1e-3 / 1.0, 1e-4 / (1e-2 * rms))
    assert abs(oracle.rel_error(y, ref) - exp) < 1e-15


def test_algorithmic_bytes_formula():
    # 4096x4096 W4 G16 S50, batch 1: 524288 groups * 14 B + row pointers + x + y
    assert oracle.algorithmic_bytes(4096, 4096, 16, 4, 524288, 1) == 524288 * 14 + 4097 * 4 + 8192 * 2
    assert oracle.algorithmic_bytes(4096, 4096, 16, 8, 524288, 16) == 524288 * 22 + 4097 * 4 + 16 * 8192 * 2
