"""Pins of the oracle's other value widths (1, 2, 3, 4 bits and unquantized fp32;
the paper's ablation "Effect of quantization on loss") against things other than
itself: the 2-bit functions pinned elsewhere, exact rational arithmetic, values
placed by hand on the bin edges, hand-worked record bytes, a big-integer model
of the bit stream, closed forms, and the identities of Eq. (2).  CPU only.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from test_oracle_pins import FLAT, TILE, bits, f32_round, small_list, tensor_mask

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "quantizer_ablation.txt")
WIDTHS = (1, 2, 3, 4)


def paper_rows():
    return [line.split("#")[0].split() for line in open(GOLDEN) if line.split("#")[0].split()]


def test_widths_are_the_ones_the_paper_ablates():
    assert [int(b) for b, _ in paper_rows()] == list(WIDTHS) + [32]


# --------------------------------------------------------------------------- quantizer
def test_two_bits_is_the_pinned_two_bit_quantizer(oracle):
    rng = np.random.default_rng(100)
    for nc, k in ((1, 8), (7, 64), (33, 32), (300, 64)):
        x = (rng.standard_t(3, nc * k) * 1e-3).astype(np.float32)
        c2, l2, s2 = oracle.quantize_tensor(x, nc, k)
        cb, lb, sb = oracle.quantize_tensor_b(x, nc, k, 2)
        assert np.array_equal(c2, cb) and np.array_equal(bits(l2), bits(lb)) and np.array_equal(s2, sb)


def exact_quantizer_b(x, b):
    """Section 4's description in exact rational arithmetic: centre by the mean, cut
    [-6 sigma, 6 sigma] into 2^b uniform half-open bins, clamp to the end bins.  A
    value is at or above the edge c*sigma (c rational) iff sign-aware d^2 vs c^2 var."""
    X = [Fraction(float(v)) for v in x]
    M = len(X)
    mu = sum(X) / M
    var = sum(v * v for v in X) / M - mu * mu
    nb = 1 << b
    codes = []
    for v in X:
        d = v - mu
        q = 0
        for j in range(1, nb):
            c = Fraction(12 * j, nb) - 6
            if c < 0:
                reached = d >= 0 or d * d <= c * c * var
            else:
                reached = d >= 0 and d * d >= c * c * var
            q += reached
        codes.append(q)
    lut = []
    for q in range(nb):
        sel = [v for v, c in zip(X, codes) if c == q]
        lut.append(f32_round(sum(sel) / len(sel)) if sel else np.float32(0))
    return mu, var, np.array(codes), np.array(lut, dtype=np.float32)


@pytest.mark.parametrize("b", WIDTHS)
def test_quantizer_exact_rational_on_dyadic_inputs(oracle, b):
    rng = np.random.default_rng(110 + b)
    for trial in range(120):
        k = int(rng.choice([4, 8, 16]))
        nc = int(rng.choice([1, 2, 4, 8]))
        M = nc * k
        x = (rng.integers(-64, 65, M) / 16.0).astype(np.float32)
        if trial % 4 == 0:
            x[rng.integers(0, M, 2)] = rng.choice([-32.0, 32.0, 48.0], 2)
        if trial % 7 == 0:
            x[:] = x[0]
        mu, var, codes, lut = exact_quantizer_b(x, b)
        code, got, st = oracle.quantize_tensor_b(x, nc, k, b)
        assert Fraction(st[2]) == mu and Fraction(st[3]) == var
        assert np.array_equal(code, codes)
        for q in range(1 << b):
            assert got[q] == lut[q] or abs(float(got[q]) - float(lut[q])) <= abs(float(lut[q])) * 2.0**-23
        assert st[4:].tolist() == [int((codes == q).sum()) for q in range(1 << b)]


def edge_multiset():
    """128 values with mean 0 and variance 1 exactly: two each of +-1.5, +-3, +-4.5
    (sum of squares 126), one +-1 (2), 114 zeros.  Every inner edge of the 2-, 3-
    and 4-bit quantizers that is a multiple of 1.5 sigma has a value sitting on it."""
    x = np.zeros(128, dtype=np.float32)
    vals = [1.5, -1.5, 3.0, -3.0, 4.5, -4.5, 1.5, -1.5, 3.0, -3.0, 4.5, -4.5, 1.0, -1.0]
    pos = [3, 9, 17, 22, 31, 40, 47, 55, 64, 70, 85, 99, 110, 127]
    x[pos] = vals
    return x


def test_values_on_the_bin_edges_by_hand(oracle):
    x = edge_multiset()
    # bin q = [c_q, c_q+1) sigma with c_j = 12 j / 2^b - 6: a value on an edge opens the bin above it
    want = {
        1: {-4.5: 0, -3.0: 0, -1.5: 0, -1.0: 0, 0.0: 1, 1.0: 1, 1.5: 1, 3.0: 1, 4.5: 1},
        2: {-4.5: 0, -3.0: 1, -1.5: 1, -1.0: 1, 0.0: 2, 1.0: 2, 1.5: 2, 3.0: 3, 4.5: 3},
        3: {-4.5: 1, -3.0: 2, -1.5: 3, -1.0: 3, 0.0: 4, 1.0: 4, 1.5: 5, 3.0: 6, 4.5: 7},
        4: {-4.5: 2, -3.0: 4, -1.5: 6, -1.0: 6, 0.0: 8, 1.0: 9, 1.5: 10, 3.0: 12, 4.5: 14},
    }
    for b in WIDTHS:
        for nc, k in ((1, 128), (4, 32), (16, 8)):
            code, lut, st = oracle.quantize_tensor_b(x, nc, k, b)
            assert st[2] == 0.0 and st[3] == 1.0
            assert code.tolist() == [want[b][float(v)] for v in x]
            for q in range(1 << b):                      # centroid = plain mean of the bin's values
                sel = x[code == q]
                cen = np.float32(sel.astype(np.float64).mean()) if sel.size else np.float32(0)
                assert bits(lut[q] + np.float32(0)) == bits(cen + np.float32(0)) and bits(lut[q]) != 0x80000000


def test_one_bit_is_the_side_of_the_mean(oracle):
    rng = np.random.default_rng(120)
    for nc, k in ((5, 8), (40, 64)):
        x = rng.normal(3e-4, 1e-3, nc * k).astype(np.float32)
        code, lut, st = oracle.quantize_tensor_b(x, nc, k, 1)
        mu = st[2]
        assert abs(mu - x.astype(np.float64).mean()) < 1e-15
        assert np.array_equal(code, (x.astype(np.float64) >= mu).astype(np.uint8))
        for q in (0, 1):
            assert abs(lut[q] - x[code == q].astype(np.float64).mean()) <= abs(lut[q]) * 2.0**-23


@pytest.mark.parametrize("b", WIDTHS)
def test_plus_minus_c_is_lossless_at_every_width(oracle, b):
    """+-c in equal numbers: mu = 0, sigma = c, the two values fall in the bins that
    contain -1 sigma and +1 sigma, whose centroids are the values themselves."""
    lo = {1: 0, 2: 1, 3: 3, 4: 6}[b]           # bin of -sigma: floor((-1 + 6) * 2^b / 12)
    assert lo == math.floor(5 * (1 << b) / 12) and (1 << b) - 1 - lo == math.floor(7 * (1 << b) / 12)
    for c in (1e-3, 0.37, 5.0):
        c32 = np.float32(c)
        x = np.tile(np.array([c32, -c32, -c32, c32], dtype=np.float32), 8 * 5)
        code, lut, st = oracle.quantize_tensor_b(x, 5, 32, b)
        assert st[2] == 0.0 and st[3] == float(c32) ** 2
        assert np.array_equal(code, np.where(x > 0, (1 << b) - 1 - lo, lo))
        assert np.array_equal(bits(lut[code]), bits(x))
        assert np.count_nonzero(lut) == 2


@pytest.mark.parametrize("b", WIDTHS)
def test_quantizer_invariants_random(oracle, b):
    rng = np.random.default_rng(130 + b)
    nb = 1 << b
    for nc, k in ((7, 64), (33, 32), (300, 64)):
        mag = np.abs(rng.normal(0, 1e-3, nc * k)) + 2e-3
        x = (mag * rng.choice([-1, 1], nc * k)).astype(np.float32)
        x[rng.integers(0, x.size, 5)] *= 30
        code, lut, st = oracle.quantize_tensor_b(x, nc, k, b)
        S1, S2, mu, var = st[:4]
        assert abs(var - x.astype(np.float64).var()) < 1e-12 * var
        order = np.argsort(x, kind="stable")
        assert np.all(np.diff(code[order].astype(int)) >= 0)
        sig = math.sqrt(var)
        edges = [-math.inf] + [mu + (12.0 * j / nb - 6.0) * sig for j in range(1, nb)] + [math.inf]
        # the floor formula of a uniform quantizer, away from the edges
        d = (x.astype(np.float64) - mu) / sig
        near = np.min(np.abs(d[:, None] - (12.0 * np.arange(1, nb) / nb - 6.0)[None, :]), axis=1) < 1e-9
        floor_code = np.clip(np.floor((d + 6.0) * nb / 12.0), 0, nb - 1).astype(int)
        assert np.array_equal(code[~near], floor_code[~near])
        tot = 0.0
        for q in range(nb):
            n_q = int((code == q).sum())
            assert st[4 + q] == n_q
            if n_q:
                assert edges[q] - 1e-9 <= lut[q] <= edges[q + 1] + 1e-9
                tot += n_q * float(lut[q])
            else:
                assert bits(lut[q]) == 0
        assert abs(tot - S1) <= 2.0**-22 * np.abs(x).sum()
        assert st[4:].sum() == nc * k


# --------------------------------------------------------------------------- wire format
def bigint_record_b(idx, sent, b):
    k = len(idx)
    stream = sum(int(v) << (12 * m) for m, v in enumerate(idx))
    head = stream.to_bytes(3 * k // 2, "little")
    if b == 32:
        tail = np.asarray(sent, dtype="<f4").tobytes()
    else:
        tail = sum(int(c) << (b * m) for m, c in enumerate(sent)).to_bytes(k * b // 8, "little")
    return np.frombuffer(head + tail, dtype=np.uint8)


def test_record_bytes_worked_by_hand(oracle):
    idx = [0, 1, 2, 3, 4, 5, 6, 4095]
    head = "001000" "023000" "045000" "06f0ff"
    assert oracle.pack_record_b(idx, [1, 0, 1, 1, 0, 0, 1, 0], 1).tobytes().hex() == head + "4d"
    assert oracle.pack_record_b(idx, [0, 1, 2, 3, 0, 1, 2, 3], 2).tobytes().hex() == head + "e4e4"
    assert oracle.pack_record_b(idx, [0, 1, 2, 3, 4, 5, 6, 7], 3).tobytes().hex() == head + "88c6fa"
    assert oracle.pack_record_b(idx, [0, 1, 2, 3, 12, 13, 14, 15], 4).tobytes().hex() == head + "1032dcfe"
    v = [1.0, -2.0, 0.5, 0.0, -0.0, 3.0, 1e-3, -1e-3]
    assert oracle.pack_record_b(idx, v, 32).tobytes().hex() == head + "".join(
        h for h in ("0000803f", "000000c0", "0000003f", "00000000", "00000080", "00004040", "6f12833a", "6f1283ba"))


@pytest.mark.parametrize("b", WIDTHS + (32,))
def test_records_match_bigint_model_and_round_trip(oracle, b):
    rng = np.random.default_rng(140 + b)
    for k in (8, 32, 64, 128, 256, 4096):
        for _ in range(10):
            idx = np.sort(rng.choice(4096, k, replace=False)).astype(np.uint16)
            sent = (rng.normal(0, 1, k).astype(np.float32) if b == 32
                    else rng.integers(0, 1 << b, k).astype(np.uint8))
            rec = oracle.pack_record_b(idx, sent, b)
            assert rec.size == oracle.record_bytes_b(k, b) == (12 + b) * k // 8
            assert np.array_equal(rec, bigint_record_b(idx, sent, b))
            i2, s2 = oracle.unpack_record_b(rec, k, b)
            assert np.array_equal(i2, idx)
            assert np.array_equal(bits(s2), bits(sent)) if b == 32 else np.array_equal(s2, sent)
    if b == 2:                                           # same bytes as the 2-bit record
        idx = np.sort(rng.choice(4096, 64, replace=False)).astype(np.uint16)
        code = rng.integers(0, 4, 64).astype(np.uint8)
        assert np.array_equal(oracle.pack_record_b(idx, code, 2), oracle.pack_record(idx, code))


def test_sizes(oracle):
    descs, n = small_list()
    assert [oracle.header_bytes_b(b) for b in (1, 2, 3, 4, 32)] == [16, 16, 32, 64, 0]
    for b in (1, 2, 3, 4, 32):
        for k in (8, 64):
            want = 0
            for d in descs:
                blk = oracle.header_bytes_b(b) + oracle.tensor_chunks(d) * (12 + b) * k // 8
                assert oracle.tensor_block_bytes_b(d, k, b) == (blk + 15) // 16 * 16
                want += (blk + 15) // 16 * 16
            assert oracle.payload_bytes_b(descs, k, b) == want
    assert oracle.payload_bytes_b(descs, 64, 2) == oracle.payload_bytes(descs, 64)


# --------------------------------------------------------------------------- whole path
def rand_state(n, descs, seed):
    rng = np.random.default_rng(seed)
    m = tensor_mask(descs, n)
    e = np.where(m, rng.normal(0, 2e-3, n), 0).astype(np.float32)
    d = np.where(m, rng.standard_t(3, n) * 1e-3, 0).astype(np.float32)
    return e, d


def test_compress_two_bits_is_the_pinned_path(oracle):
    descs, n = small_list()
    e, d = rand_state(n, descs, 150)
    e2 = e.copy()
    p2 = oracle.compress(descs, 64, e2, d, 0.95)
    eb = e.copy()
    pb, det = oracle.compress_b(descs, 64, 2, eb, d, 0.95, want_detail=True)
    assert np.array_equal(p2, pb) and np.array_equal(bits(e2), bits(eb))
    rng = np.random.default_rng(151)
    th = rng.normal(0, 0.02, n).astype(np.float32)
    t2, tb = th.copy(), th.copy()
    oracle.decompress_avg_apply(descs, 64, t2, [p2, p2], 0.7)
    oracle.decompress_avg_apply_b(descs, 64, 2, tb, [pb, pb], 0.7)
    assert np.array_equal(bits(t2), bits(tb))


@pytest.mark.parametrize("b", WIDTHS + (32,))
def test_compress_identities_of_eq2(oracle, b):
    """Selection does not depend on the value width; e = a where nothing was sent; at
    sent positions e = a - sent (one fp32 subtract); the dense view of the payload is
    what was subtracted; full-precision values leave a zero residual."""
    descs, n = small_list()
    k = 64
    e0, d = rand_state(n, descs, 160)
    e_ref = e0.copy()
    p_ref, det_ref = oracle.compress(descs, k, e_ref, d, 0.95, want_detail=True)
    e = e0.copy()
    pay, det = oracle.compress_b(descs, k, b, e, d, 0.95, want_detail=True)
    assert pay.size == oracle.payload_bytes_b(descs, k, b)
    assert np.array_equal(det["idx"], det_ref["idx"]) and np.array_equal(bits(det["val"]), bits(det_ref["val"]))
    acc = e0.copy()
    oracle.accumulate(acc, d, 0.95)
    dense = oracle.decompress_dense_b(descs, k, b, pay, n)
    probe = oracle.decompress_dense_b(descs, k, b, pay, n, out=np.full(n, np.nan, dtype=np.float32))
    sent = ~np.isnan(probe)                              # the positions the payload names
    assert sent.sum() == oracle.num_chunks(descs) * k
    assert np.array_equal(bits(e[~sent]), bits(acc[~sent]))
    assert np.array_equal(bits(e[sent]), bits(acc[sent] - dense[sent]))
    if b == 32:
        assert np.array_equal(bits(dense[sent]), bits(acc[sent]))
        assert not e[sent].any() and not np.signbit(e[sent]).any()
    else:
        lut = det["lut"].reshape(len(descs), 1 << b)
        assert np.isin(bits(dense[sent]), bits(lut)).all()
        # finer quantizers leave a smaller residual on the same selection
        if b > 1:
            e1 = e0.copy()
            oracle.compress_b(descs, k, b - 1, e1, d, 0.95)
            assert np.square(e[sent].astype(np.float64)).sum() < np.square(e1[sent].astype(np.float64)).sum()


@pytest.mark.parametrize("b", (1, 3, 4, 32))
def test_aggregate_matches_dense_numpy_model(oracle, b):
    descs = [(70, 130, 0, TILE), (1, 5000, 70 * 130 + 4, FLAT)]
    n = 70 * 130 + 4 + 5000
    k, R, lr = 8, 3, 0.7
    rng = np.random.default_rng(170 + b)
    payloads = []
    for r in range(R):
        e = np.zeros(n, dtype=np.float32)
        d = np.where(tensor_mask(descs, n), rng.normal(0, 1e-3, n), 0).astype(np.float32)
        payloads.append(oracle.compress_b(descs, k, b, e, d, 0.95))
    theta0 = rng.normal(0, 0.02, n).astype(np.float32)
    theta = theta0.copy()
    oracle.decompress_avg_apply_b(descs, k, b, theta, payloads, lr)
    acc = np.zeros(n, dtype=np.float32)
    for p in payloads:
        acc = acc + oracle.decompress_dense_b(descs, k, b, p, n)
    upd = (acc * (np.float32(1.0) / np.float32(R))).astype(np.float32)
    want = theta0.copy()
    for i in np.flatnonzero(upd):
        want[i] = f32_round(Fraction(float(theta0[i])) - Fraction(float(np.float32(lr))) * Fraction(float(upd[i])))
    assert np.array_equal(bits(theta), bits(want))
    assert np.array_equal(bits(theta[acc == 0]), bits(theta0[acc == 0])) and (acc != 0).sum() > 0


def test_argument_errors(oracle):
    descs, n = small_list()
    e = np.zeros(n, dtype=np.float32)
    for k, b in ((64, 5), (64, 0), (64, 8), (12, 3), (4, 1)):
        with pytest.raises(ValueError):
            oracle.compress_b(descs, k, b, e, e.copy(), 0.95)
    oracle.compress_b(descs, 12, 2, e, e.copy(), 0.95)       # k a multiple of 4 is enough at 2 bits
