"""Pins of the CPU oracle against things other than itself (CPU only).

Each test names what it pins the oracle to: exact rational arithmetic, brute
force on tiny inputs, a library routine on a special case, a hand-computed
value, a number printed in the paper, or an invariant of Eq. (2).
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_numbers.txt")
FLAT, TILE = 0, 1


def paper_numbers():
    out = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].split()
        if len(line) == 2:
            out[line[0]] = float(line[1])
    return out


# --------------------------------------------------------------------------- helpers
def f32_round(fr: Fraction) -> np.float32:
    """Round an exact rational to fp32, nearest-even, with integer arithmetic only."""
    if fr == 0:
        return np.float32(0.0)
    sign = -1 if fr < 0 else 1
    fr = abs(fr)
    e = math.floor(math.log2(fr)) if fr > 0 else 0
    while Fraction(2) ** e > fr:
        e -= 1
    while Fraction(2) ** (e + 1) <= fr:
        e += 1
    e = max(e, -126)                       # denormal range shares the exponent of 2^-126
    ulp = Fraction(2) ** (e - 23)
    q = fr / ulp
    n = q.numerator // q.denominator
    rem = q - n
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and n % 2 == 1):
        n += 1
    val = sign * n * ulp
    assert val.denominator & (val.denominator - 1) == 0
    return np.float32(float(val))          # exact: val is representable


def bits(x):
    return np.asarray(x, dtype=np.float32).view(np.uint32)


# --------------------------------------------------------------------------- step 1: accumulate
def test_accumulate_is_one_correctly_rounded_fma(oracle):
    """Exact rational arithmetic: a = round_f32(beta*e + delta), a single rounding."""
    rng = np.random.default_rng(1)
    n = 400
    e = rng.normal(0, 1e-3, n).astype(np.float32)
    d = rng.normal(0, 1e-3, n).astype(np.float32)
    # cases that tell a fused from a two-rounding evaluation, plus denormals
    e[:4] = np.array([1.0 + 2.0**-23, 3.0, 2.0**-140, -2.0**-130], dtype=np.float32)
    d[:4] = np.array([-1.0, 2.0**-24, 2.0**-149, 2.0**-131], dtype=np.float32)
    for beta in (0.95, 0.9, 0.999, 1.0 - 2.0**-23):
        b32 = np.float32(beta)
        got = e.copy()
        oracle.accumulate(got, d, b32)
        want = np.array([f32_round(Fraction(float(b32)) * Fraction(float(x)) + Fraction(float(y)))
                         for x, y in zip(e, d)], dtype=np.float32)
        assert np.array_equal(bits(got), bits(want))
    # a two-rounding evaluation would differ somewhere in this set
    two = (np.float32(0.95) * e).astype(np.float32) + d
    fused = e.copy()
    oracle.accumulate(fused, d, np.float32(0.95))
    assert not np.array_equal(bits(two), bits(fused))


def test_accumulate_special_cases(oracle):
    rng = np.random.default_rng(2)
    d = rng.normal(0, 1e-3, 1000).astype(np.float32)
    e = np.zeros_like(d)
    oracle.accumulate(e, d, 0.95)
    assert np.array_equal(bits(e), bits(d))            # e = 0  ->  a = delta
    e = rng.normal(0, 1, 1000).astype(np.float32)
    e0 = e.copy()
    oracle.accumulate(e, d, 0.0)
    assert np.array_equal(e, d)                        # beta = 0
    e = e0.copy()
    oracle.accumulate(e, np.zeros_like(d), 1.0)
    assert np.array_equal(bits(e), bits(e0))           # beta = 1, delta = 0


# --------------------------------------------------------------------------- step 2: chunk geometry
def test_tile_geometry_matches_numpy_blocking(oracle):
    """64x64 blocks of a row-major matrix == reshape/transpose blocking in numpy."""
    rows, cols = 192, 320
    a = np.arange(rows * cols, dtype=np.int64).reshape(rows, cols)
    blocks = a.reshape(rows // 64, 64, cols // 64, 64).transpose(0, 2, 1, 3).reshape(-1, 4096)
    desc = (rows, cols, 0, TILE)
    assert oracle.tensor_chunks(desc) == blocks.shape[0]
    rng = np.random.default_rng(0)
    for _ in range(300):
        c = int(rng.integers(blocks.shape[0]))
        j = int(rng.integers(4096))
        assert oracle.element_of(desc, c, j) == blocks[c, j]
    # with an arena offset
    assert oracle.element_of((rows, cols, 1000, TILE), 7, 65) == 1000 + blocks[7, 65]


def test_partial_tiles_and_flat_runs(oracle):
    rows, cols = 81, 70           # 2x2 tile grid, both edges ragged
    desc = (rows, cols, 5, TILE)
    assert oracle.tensor_chunks(desc) == 4
    seen = set()
    for c in range(4):
        tr, tc = divmod(c, 2)
        for j in range(4096):
            r, q = tr * 64 + j // 64, tc * 64 + j % 64
            want = 5 + r * cols + q if (r < rows and q < cols) else -1
            got = oracle.element_of(desc, c, j)
            assert got == want
            if got >= 0:
                seen.add(got)
    assert seen == set(range(5, 5 + rows * cols))      # a partition: every element exactly once
    # 1-D rule
    desc = (1, 10000, 64, FLAT)
    assert oracle.tensor_chunks(desc) == 3
    assert oracle.element_of(desc, 2, 1807) == 64 + 2 * 4096 + 1807
    assert oracle.element_of(desc, 2, 1808) == -1
    # chunk counts of the benchmark lists against the closed form
    assert oracle.tensor_chunks((50257, 2048, 0, TILE)) == 786 * 32


# --------------------------------------------------------------------------- step 3: Top-k
def brute_topk(vals, valid_js, k):
    """k rounds of arg-max on |x|; among equal magnitudes the lowest index wins."""
    chosen, remaining = [], list(valid_js)
    for _ in range(k):
        best = None
        for j in remaining:
            if best is None or abs(float(vals[j])) > abs(float(vals[best])):
                best = j
        chosen.append(best)
        remaining.remove(best)
    return sorted(chosen)


@pytest.mark.parametrize("tile,layout", [(2, FLAT), (4, FLAT), (4, TILE), (3, TILE)])
def test_topk_brute_force_tiny(oracle, tile, layout):
    rng = np.random.default_rng(10 + tile)
    C = tile * tile
    for trial in range(300):
        if layout == TILE:
            rows, cols = int(rng.integers(tile, 3 * tile + 1)), int(rng.integers(tile, 3 * tile + 1))
        else:
            rows, cols = 1, int(rng.integers(C, 4 * C))
        n = rows * cols
        mode = trial % 3
        if mode == 0:
            a = rng.normal(0, 1, n)
        elif mode == 1:   # many ties, signed zeros
            a = rng.choice([-2.0, -1.0, -0.0, 0.0, 1.0, 2.0], n)
        else:
            a = np.zeros(n)
        a = a.astype(np.float32)
        desc = (rows, cols, 0, layout)
        for c in range(oracle.tensor_chunks(desc, tile)):
            valid = [j for j in range(C) if oracle.element_of(desc, c, j, tile) >= 0]
            ks = [k for k in (4, 8, 12, 16) if k <= len(valid)]
            if not ks:
                with pytest.raises(ValueError):
                    oracle.topk_chunk(desc, c, a, 4, tile)
                continue
            k = ks[int(rng.integers(len(ks)))]
            local = {j: a[oracle.element_of(desc, c, j, tile)] for j in valid}
            want = brute_topk(local, valid, k)
            idx, val = oracle.topk_chunk(desc, c, a, k, tile)
            assert idx.tolist() == want
            assert np.array_equal(bits(val), bits([local[j] for j in want]))


def test_topk_equals_stable_sort_and_invariants(oracle):
    """Special case that reduces to a library routine: stable argsort of -|a| bits."""
    rng = np.random.default_rng(3)
    rows, cols = 128, 192
    a = rng.standard_t(3, rows * cols).astype(np.float32)
    a[rng.integers(0, a.size, 3000)] = np.float32(0.5)      # plant ties
    desc = (rows, cols, 0, TILE)
    blocks = a.reshape(rows // 64, 64, cols // 64, 64).transpose(0, 2, 1, 3).reshape(-1, 4096)
    for c in range(blocks.shape[0]):
        key = blocks[c].view(np.uint32) & 0x7FFFFFFF
        for k in (4, 32, 64, 128, 2048, 4096):
            order = np.argsort(-(key.astype(np.int64)), kind="stable")[:k]
            idx, val = oracle.topk_chunk(desc, c, a, k)
            assert np.array_equal(np.sort(order), idx)
            assert np.all(np.diff(idx.astype(int)) > 0)                 # ascending, distinct
            sel = np.zeros(4096, bool)
            sel[idx] = True
            if k < 4096:
                assert key[sel].min() >= key[~sel].max()
                thr = key[sel].min()
                tie_sel = np.nonzero(sel & (key == thr))[0]
                tie_uns = np.nonzero(~sel & (key == thr))[0]
                if tie_uns.size:
                    assert tie_sel.max() < tie_uns.min()                # lowest index wins
            assert np.array_equal(bits(val), bits(blocks[c][idx]))


def test_topk_all_zero_chunk_selects_first_k(oracle):
    a = np.zeros(8192, dtype=np.float32)
    idx, val = oracle.topk_chunk((1, 8192, 0, FLAT), 1, a, 32)
    assert idx.tolist() == list(range(32)) and not val.any()


# --------------------------------------------------------------------------- fixed summation tree
def test_tree_sum_shape_by_hand(oracle):
    big = 2.0**60
    # ((big + 1) + (-big + 1)) = big + (-big) = 0 ; a left-to-right sum gives 1
    assert oracle.tree_sum([big, 1.0, -big, 1.0]) == 0.0
    # three values are padded to four: (a + b) + (c + 0)
    assert oracle.tree_sum([1.0, big, -big]) == (1.0 + big) + (-big + 0.0) == 0.0
    assert oracle.tree_sum([big, -big, 1.0]) == 1.0
    # five values -> eight leaves: ((a+b)+(c+d)) + ((e+0)+(0+0))
    v = [1.0, big, 1.0, -big, 3.0]
    assert oracle.tree_sum(v) == ((1.0 + big) + (1.0 + -big)) + ((3.0 + 0.0) + (0.0 + 0.0)) == 3.0
    # a pairing (a + (b + (c + ...))) or a split at n/2 instead of the power of two would give:
    assert oracle.tree_sum([1.0, 1.0, big, -big, 1.0, 1.0]) == ((2.0) + (0.0)) + ((2.0) + 0.0)
    assert oracle.tree_sum([big, 1.0, 1.0, -big, 1.0, 1.0]) == (big + (1.0 - big)) + 2.0
    assert oracle.tree_sum([]) == 0.0 and oracle.tree_sum([7.5]) == 7.5
    rng = np.random.default_rng(0)
    x = rng.normal(size=1000)
    assert abs(oracle.tree_sum(x) - math.fsum(x)) < 1e-11


def test_two_level_sum_is_chunk_tree_then_tensor_tree(oracle):
    """S1 of the quantizer: per chunk a tree over its k entries (k = 12 padded to 16),
    then a tree over the chunk leaves (3 padded to 4) - written out by hand."""
    big = 2.0**60                      # fp32-representable; big + 1 == big in fp64
    k, nc = 12, 3
    c0 = [big, 1, 1, 1, 1, 1, 1, 1, -big, 1, 1, 1]
    c1 = [1, 1, big, 1, 1, -big, 1, 1, 1, 1, 1, 1]
    c2 = [3, 3, 3, 3, 3, 3, 3, 3, 3, 3, 3, 3]
    x = np.array(c0 + c1 + c2, dtype=np.float32)

    def leaf(v):                       # ((p0+p1)+(p2+p3)) + ((p4+p5)+(0+0)), p_i = v[2i]+v[2i+1]
        p = [float(v[2 * i]) + float(v[2 * i + 1]) for i in range(6)]
        return ((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (0.0 + 0.0))

    leaves = [leaf(c0), leaf(c1), leaf(c2)]
    assert leaves == [0.0, 4.0, 36.0]  # chunk 0 loses all its ones, chunk 1 six of them
    want = (leaves[0] + leaves[1]) + (leaves[2] + 0.0)
    _, _, st = oracle.quantize_tensor(x, nc, k)
    assert st[0] == want == 40.0
    assert oracle.tree_sum(x.astype(np.float64)) != want      # one flat tree pairs differently
    assert [oracle.tree_sum(np.array(c, dtype=np.float64)) for c in (c0, c1, c2)] == leaves


# --------------------------------------------------------------------------- step 4: quantizer
def test_quantizer_closed_form_plus_minus_c(oracle):
    """All selected values are +-c in equal numbers: mu = 0, var = c^2, lossless."""
    for c in (1e-3, 0.37, 5.0):
        c32 = np.float32(c)
        x = np.tile(np.array([c32, -c32, -c32, c32], dtype=np.float32), 8 * 5)
        code, lut, st = oracle.quantize_tensor(x, 5, 32)
        assert st[2] == 0.0 and st[3] == float(c32) ** 2
        assert np.array_equal(code, np.where(x > 0, 2, 1))
        assert np.array_equal(bits(lut), bits([0.0, -c32, c32, 0.0]))
        assert np.array_equal(bits(lut[code]), bits(x))


def test_quantizer_bin_edges_half_open(oracle):
    """36 values: 2x(+3), 2x(-3), 32 zeros -> mu = 0, var = 1, T = 9 exactly.
    d = +3 sits on the upper edge (goes up: code 3), d = -3 on the lower edge
    (stays in the inner bin: code 1), d = 0 opens bin 2."""
    x = np.zeros(36, dtype=np.float32)
    x[[1, 20]] = 3.0
    x[[5, 30]] = -3.0
    for nc, k in ((1, 36), (3, 12), (9, 4)):
        code, lut, st = oracle.quantize_tensor(x, nc, k)
        assert st[2] == 0.0 and st[3] == 1.0
        want = np.full(36, 2)
        want[[1, 20]] = 3
        want[[5, 30]] = 1
        assert np.array_equal(code, want)
        assert np.array_equal(bits(lut), bits([0.0, -3.0, 0.0, 3.0]))
        assert st[4:].tolist() == [0, 2, 32, 2]


def exact_quantizer(x):
    """The quantizer's definition in exact rational arithmetic."""
    X = [Fraction(float(v)) for v in x]
    M = len(X)
    mu = sum(X) / M
    var = sum(v * v for v in X) / M - mu * mu
    T = 9 * var
    codes = []
    for v in X:
        d = v - mu
        codes.append((0 if d * d > T else 1) if d < 0 else (3 if d * d >= T else 2))
    lut = []
    for b in range(4):
        sel = [v for v, c in zip(X, codes) if c == b]
        lut.append(f32_round(sum(sel) / len(sel)) if sel else np.float32(0))
    return mu, var, np.array(codes), np.array(lut, dtype=np.float32)


def test_quantizer_exact_rational_on_dyadic_inputs(oracle):
    """Small dyadic values, M a power of two: every fp64 operation of the oracle is
    exact, so it must agree with exact rational arithmetic, edges included."""
    rng = np.random.default_rng(5)
    for trial in range(200):
        k = int(rng.choice([4, 8, 16]))
        nc = int(rng.choice([1, 2, 4, 8]))
        M = nc * k
        x = (rng.integers(-64, 65, M) / 16.0).astype(np.float32)
        if trial % 4 == 0:                    # outliers beyond 3 sigma
            x[rng.integers(0, M, 2)] = rng.choice([-32.0, 32.0, 48.0], 2)
        if trial % 7 == 0:
            x[:] = x[0]                       # sigma = 0
        mu, var, codes, lut = exact_quantizer(x)
        code, got_lut, st = oracle.quantize_tensor(x, nc, k)
        assert Fraction(st[2]) == mu and Fraction(st[3]) == var
        assert np.array_equal(code, codes)
        # centroids: sums are exact, the division is rounded once to fp64 then to fp32;
        # accept the directly rounded value or its double-rounded neighbour
        for b in range(4):
            assert got_lut[b] == lut[b] or abs(float(got_lut[b]) - float(lut[b])) <= abs(float(lut[b])) * 2.0**-23
        assert st[4:].tolist() == [int((codes == b).sum()) for b in range(4)]


def test_quantizer_sigma_zero_and_signed_zero(oracle):
    """sigma = 0: every edge sits on the mean; d = 0 is not below the upper edge of the
    half-open bins, so everything lands in the top bin, whose centroid is the value."""
    code, lut, st = oracle.quantize_tensor(np.zeros(64, dtype=np.float32), 2, 32)
    assert np.all(code == 3) and np.array_equal(bits(lut), bits([0, 0, 0, 0]))
    code, lut, st = oracle.quantize_tensor(np.full(64, -0.0, dtype=np.float32), 2, 32)
    assert np.array_equal(bits(lut), bits([0, 0, 0, 0]))        # never -0.0 on the wire
    code, lut, _ = oracle.quantize_tensor(np.full(64, 0.25, dtype=np.float32), 2, 32)
    assert np.all(code == 3) and lut[3] == np.float32(0.25) and not lut[:3].any()


def test_quantizer_invariants_random(oracle):
    rng = np.random.default_rng(6)
    for nc, k in ((7, 64), (33, 32), (1, 128), (300, 64)):
        mag = np.abs(rng.normal(0, 1e-3, nc * k)) + 2e-3
        x = (mag * rng.choice([-1, 1], nc * k)).astype(np.float32)
        x[rng.integers(0, x.size, 5)] *= 30
        code, lut, st = oracle.quantize_tensor(x, nc, k)
        S1, S2, mu, var = st[:4]
        assert abs(S1 - math.fsum(x.astype(np.float64))) <= 1e-12 * np.abs(x).sum()
        assert abs(mu - x.astype(np.float64).mean()) < 1e-15
        assert abs(var - x.astype(np.float64).var()) < 1e-12 * var        # population variance
        order = np.argsort(x, kind="stable")
        assert np.all(np.diff(code[order].astype(int)) >= 0)             # codes monotone in x
        sig = math.sqrt(var)
        edges = [-math.inf, mu - 3 * sig, mu, mu + 3 * sig, math.inf]
        tot = 0.0
        for b in range(4):
            n_b = int((code == b).sum())
            assert st[4 + b] == n_b
            if n_b:
                assert edges[b] - 1e-9 <= lut[b] <= edges[b + 1] + 1e-9   # centroid inside its bin
                assert abs(lut[b] - x[code == b].astype(np.float64).mean()) <= abs(lut[b]) * 2.0**-23
                tot += n_b * float(lut[b])
        assert abs(tot - S1) <= 2.0**-22 * np.abs(x).sum()               # centroids preserve the sum
        assert st[4:].sum() == nc * k


# --------------------------------------------------------------------------- wire format
def bigint_record(idx, code):
    """Independent model: the index fields form one little-endian integer."""
    k = len(idx)
    stream = sum(int(v) << (12 * m) for m, v in enumerate(idx))
    cstream = sum(int(c) << (2 * m) for m, c in enumerate(code))
    return np.frombuffer(stream.to_bytes(3 * k // 2, "little") + cstream.to_bytes(k // 4, "little"),
                         dtype=np.uint8)


def test_pack_worked_example_bytes(oracle):
    rec = oracle.pack_record([1, 2, 7, 4095], [0, 1, 2, 3])
    assert rec.tobytes().hex() == "0120000" "7f0ff" "e4"
    assert rec.tobytes() == bytes([0x01, 0x20, 0x00, 0x07, 0xF0, 0xFF, 0xE4])


def test_pack_matches_bigint_model_and_round_trips(oracle):
    rng = np.random.default_rng(7)
    for k in (4, 8, 32, 64, 128, 256, 4096):
        for _ in range(20):
            idx = np.sort(rng.choice(4096, k, replace=False)).astype(np.uint16)
            code = rng.integers(0, 4, k).astype(np.uint8)
            rec = oracle.pack_record(idx, code)
            assert rec.size == 7 * k // 4 == oracle.record_bytes(k)
            assert np.array_equal(rec, bigint_record(idx, code))
            i2, c2 = oracle.unpack_record(rec, k)
            assert np.array_equal(i2, idx) and np.array_equal(c2, code)
    idx = np.sort(rng.choice(4096, (5, 32), replace=False), axis=1).astype(np.uint16)
    code = rng.integers(0, 4, (5, 32)).astype(np.uint8)
    out = oracle.pack_indices(idx.ravel(), code.ravel(), 5, 32)
    assert np.array_equal(out, np.concatenate([bigint_record(i, c) for i, c in zip(idx, code)]))


def test_wire_size_is_14_bits_per_value_and_paper_context(oracle):
    """Paper: 12 bits per index naively + 2-bit values.  Table 1's own sizes come from
    the paper's index coder (8.9 / 6.6 bits); they must decode to 2 + coder bits."""
    p = paper_numbers()
    P = int(p["params_512M"])
    assert p["naive_index_bits"] + p["value_bits"] == 14
    for k in (32, 64, 128):
        assert oracle.record_bytes(k) * 8 == 14 * k
    descs = [(1024, 1024, 0, TILE), (1, 768, 1024 * 1024, FLAT), (100, 130, 2 * 1024 * 1024, TILE)]
    for k in (32, 64):
        want = sum((16 + oracle.tensor_chunks(d) * 7 * k // 4 + 15) // 16 * 16 for d in descs)
        assert oracle.payload_bytes(descs, k) == want
    for k, size_key, coder_key in ((32, "table1_size_MB_density_0p78", "coder_bits_k32"),
                                   (128, "table1_size_MB_density_3p12", "coder_bits_k128")):
        n_values = P * k / 4096
        bits_per_value = p[size_key] * 1e6 * 8 / n_values
        assert abs(bits_per_value - (p["value_bits"] + p[coder_key])) < 0.05
        assert abs(100.0 * k / 4096 - p["density_k%d" % k]) < 0.01
    for k in (32, 128, 256):
        bound = (math.lgamma(4097) - math.lgamma(k + 1) - math.lgamma(4097 - k)) / math.log(2) / k
        assert abs(bound - p["entropy_bits_k%d" % k]) < 0.1
        assert bound < p["coder_bits_k%d" % k] < p["naive_index_bits"]


def test_tensor_list_generator_reproduces_paper_parameter_counts():
    from paper_2508_15706_amd import synth
    p = paper_numbers()
    for name in ("178M", "512M", "2B"):
        assert synth.total_numel(synth.paper_shape_list(name)) == int(p["params_" + name])
    assert abs(int(p["params_512M"]) / 1e6 - p["table1_dense_8bit_MB"]) < 0.01   # 1 byte / param


# --------------------------------------------------------------------------- whole compress
def small_list():
    """Several tiles, ragged edges, a 1-D tensor with a ragged tail, 16-column matrix."""
    shapes = [(140, 200, TILE), (1, 9000, FLAT), (64, 64, TILE), (1024, 16, TILE), (1, 768, FLAT)]
    descs, off = [], 0
    for r, c, lay in shapes:
        descs.append((r, c, off, lay))
        off += (r * c + 63) // 64 * 64
    return descs, off


def tensor_mask(descs, n):
    m = np.zeros(n, bool)
    for r, c, off, _ in descs:
        m[off:off + r * c] = True
    return m


def chunk_elements(oracle, descs):
    """[(tensor index, chunk, element index array over j, -1 = outside)]"""
    out = []
    for ti, d in enumerate(descs):
        for c in range(oracle.tensor_chunks(d)):
            out.append((ti, c, np.array([oracle.element_of(d, c, j) for j in range(4096)])))
    return out


@pytest.mark.parametrize("k", [32, 64])
def test_compress_invariants_of_eq2(oracle, k):
    descs, n = small_list()
    rng = np.random.default_rng(8)
    e0 = rng.normal(0, 1e-3, n).astype(np.float32)
    delta = rng.normal(0, 1e-3, n).astype(np.float32)
    beta = np.float32(0.95)
    a = e0.copy()
    oracle.accumulate(a, delta, beta)
    e = e0.copy()
    payload, det = oracle.compress(descs, k, e, delta, beta, want_detail=True)
    chunks = chunk_elements(oracle, descs)
    assert det["idx"].size == len(chunks) * k                       # exactly k per chunk
    sel_mask = np.zeros(n, bool)
    pos = 0
    for (ti, c, elems), ci in zip(chunks, range(len(chunks))):
        idx = det["idx"][ci * k:(ci + 1) * k]
        assert np.all(np.diff(idx.astype(int)) > 0)
        ei = elems[idx]
        assert np.all(ei >= 0)                                      # only in-range positions
        sel_mask[ei] = True
        valid = elems[elems >= 0]
        uns = np.setdiff1d(valid, ei)
        assert np.abs(a[ei]).min() >= (np.abs(a[uns]).max() if uns.size else 0)
        assert np.array_equal(bits(det["val"][ci * k:(ci + 1) * k]), bits(a[ei]))
        lut = det["lut"][4 * ti:4 * ti + 4]
        dq = lut[det["code"][ci * k:(ci + 1) * k]]
        assert np.array_equal(bits(e[ei]), bits(a[ei] - dq))        # residual at sent coordinates
    in_tensor = np.zeros(n, bool)
    for r_, c_, off_, _ in descs:
        in_tensor[off_:off_ + r_ * c_] = True
    rest = in_tensor & ~sel_mask
    assert np.array_equal(bits(e[rest]), bits(a[rest]))             # e = a where nothing was sent, bit-exact
    assert np.array_equal(bits(e[~in_tensor]), bits(e0[~in_tensor]))  # arena padding is never touched
    # payload decodes to the same selection, tensor blocks 16-byte aligned
    dense = oracle.decompress_dense(descs, k, payload, n)
    assert np.array_equal(bits((a - dense)[sel_mask]), bits(e[sel_mask]))
    assert not dense[~sel_mask].any()
    a[~in_tensor] = e0[~in_tensor]
    off = 0
    for ti, d in enumerate(descs):
        assert off % 16 == 0
        assert np.array_equal(payload[off:off + 16].view(np.float32), det["lut"][4 * ti:4 * ti + 4])
        off += oracle.tensor_block_bytes(d, k)
    assert off == payload.size
    # a second tensor list made of the same tensors one at a time gives the same blocks
    off = 0
    for d in descs:
        e1 = e0.copy()
        p1 = oracle.compress([d], k, e1, delta, beta)
        assert np.array_equal(p1, payload[off:off + p1.size])
        off += p1.size


def test_compress_dense_case_k_equals_chunk(oracle):
    """k = chunk size: everything is sent; e keeps only the quantization error
    (the dense special case the paper identifies with DiLoCo without outer momentum)."""
    rng = np.random.default_rng(9)
    n = 2 * 4096
    descs = [(64, 128, 0, TILE)]
    e = rng.normal(0, 1e-3, n).astype(np.float32)
    delta = rng.normal(0, 1e-3, n).astype(np.float32)
    a = e.copy()
    oracle.accumulate(a, delta, 0.95)
    payload, det = oracle.compress(descs, 4096, e, delta, 0.95, want_detail=True)
    assert np.array_equal(det["idx"].reshape(2, 4096), np.tile(np.arange(4096), (2, 1)))
    blocks = a.reshape(1, 64, 2, 64).transpose(0, 2, 1, 3).reshape(-1)
    code, lut, _ = oracle.quantize_tensor(blocks, 2, 4096)
    assert np.array_equal(lut, det["lut"])
    dense = oracle.decompress_dense(descs, 4096, payload, n)
    assert np.array_equal(bits(e), bits(a - dense))
    frac_outer = np.mean((det["code"] == 0) | (det["code"] == 3))
    assert 0.0005 < frac_outer < 0.008                              # Gaussian: 0.27% beyond 3 sigma


def test_compress_rejects_chunks_smaller_than_k(oracle):
    e = np.zeros(4096, dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.compress([(1, 100, 0, FLAT)], 128, e, e.copy(), 0.95)
    with pytest.raises(ValueError):
        oracle.compress([(64, 64, 0, TILE)], 6, e, e.copy(), 0.95)   # k not a multiple of 4


def test_ef_freeze_neither_uses_nor_accumulates(oracle):
    """Freeze (appendix on freezing error feedback): payload = Q(Top-k(delta)), e untouched."""
    descs, n = small_list()
    rng = np.random.default_rng(11)
    e0 = rng.normal(0, 1e-3, n).astype(np.float32)
    delta = rng.normal(0, 1e-3, n).astype(np.float32)
    e = e0.copy()
    p_frozen = oracle.compress(descs, 32, e, delta, 0.95, ef_frozen=True)
    assert np.array_equal(bits(e), bits(e0))
    z = np.zeros_like(e0)
    p_zero = oracle.compress(descs, 32, z, delta, 0.95)             # e = 0 => a = delta
    assert np.array_equal(p_frozen, p_zero)


# --------------------------------------------------------------------------- aggregation
def numpy_dense_aggregate(oracle, descs, k, theta, payloads, lr, n):
    R = len(payloads)
    acc = np.zeros(n, dtype=np.float32)
    for p in payloads:                                   # r ascending, fp32 adds
        acc = acc + oracle.decompress_dense(descs, k, p, n)
    invR = np.float32(1.0) / np.float32(R)
    upd = (acc * invR).astype(np.float32)
    # fma(-lr, upd, theta): exact in fp64 for the product, then one rounding
    out = np.empty_like(theta)
    lr32 = np.float32(lr)
    for i in range(n):
        out[i] = f32_round(Fraction(float(theta[i])) - Fraction(float(lr32)) * Fraction(float(upd[i]))) \
            if upd[i] != 0 else theta[i]
    return out, acc


@pytest.mark.parametrize("R,lr", [(1, 1.0), (3, 0.7), (4, 0.7), (8, 1.0)])
def test_aggregate_matches_dense_numpy_model(oracle, R, lr):
    descs = [(70, 130, 0, TILE), (1, 5000, 70 * 130 + 4, FLAT)]
    n = 70 * 130 + 4 + 5000
    k = 8
    rng = np.random.default_rng(20 + R)
    payloads = []
    for r in range(R):
        e = np.zeros(n, dtype=np.float32)
        d = rng.normal(0, 1e-3, n).astype(np.float32)
        payloads.append(oracle.compress(descs, k, e, d, 0.95))
    theta0 = rng.normal(0, 0.02, n).astype(np.float32)
    theta = theta0.copy()
    oracle.decompress_avg_apply(descs, k, theta, payloads, lr)
    want, acc = numpy_dense_aggregate(oracle, descs, k, theta0, payloads, lr, n)
    assert np.array_equal(bits(theta), bits(want))
    untouched = acc == 0
    assert np.array_equal(bits(theta[untouched]), bits(theta0[untouched]))
    assert (~untouched).sum() > 0
    if R == 1 and lr == 1.0:                             # theta' = theta - dequantised payload
        dense = oracle.decompress_dense(descs, k, payloads[0], n)
        assert np.array_equal(bits(theta), bits(theta0 - dense))
    t2 = theta0.copy()
    oracle.decompress_avg_apply(descs, k, t2, payloads, 0.0)
    assert np.array_equal(bits(t2), bits(theta0))        # lr = 0


def test_aggregate_overlapping_indices_sum_in_worker_order(oracle):
    """Three workers send the same coordinate with values whose fp32 sum depends on
    the order: ((a + b) + c) with a = 1, b = 2^-24, c = 2^-24 gives 1, not 1 + 2^-23."""
    descs = [(1, 4096, 0, FLAT)]
    k = 4
    vals = [1.0, 2.0**-24, 2.0**-24]
    payloads = []
    for v in vals:
        blk = np.zeros(oracle.payload_bytes(descs, k), dtype=np.uint8)
        blk[:16] = np.array([0, 0, v, 0], dtype=np.float32).view(np.uint8)
        blk[16:23] = oracle.pack_record([5, 6, 7, 8], [2, 1, 1, 1])
        payloads.append(blk)
    theta = np.zeros(4096, dtype=np.float32)
    oracle.decompress_avg_apply(descs, k, theta, payloads, 1.0)
    invR = np.float32(1) / np.float32(3)
    assert theta[5] == -(np.float32(1.0) * invR) and not theta[6:9].any()
    theta = np.zeros(4096, dtype=np.float32)
    oracle.decompress_avg_apply(descs, k, theta, payloads[::-1], 1.0)
    assert theta[5] == -(np.float32(1.0 + 2.0**-23) * invR)


def test_multi_round_state_carry(oracle):
    """Three rounds, two workers: e and theta after T rounds equal a straight
    re-computation from the per-round payloads (Algorithm 1's loop)."""
    descs, n = small_list()
    k, R, beta, lr = 32, 2, 0.95, 0.7
    rng = np.random.default_rng(30)
    es = [np.zeros(n, dtype=np.float32) for _ in range(R)]
    theta = rng.normal(0, 0.02, n).astype(np.float32)
    theta_ref = theta.copy()
    inside = tensor_mask(descs, n)
    for t in range(3):
        ds = [rng.normal(0, 1e-3, n).astype(np.float32) for _ in range(R)]
        a = []
        for r in range(R):
            ar = es[r].copy()
            oracle.accumulate(ar, ds[r], beta)
            a.append(ar)
        payloads = [oracle.compress(descs, k, es[r], ds[r], beta) for r in range(R)]
        dense = [oracle.decompress_dense(descs, k, p, n) for p in payloads]
        for r in range(R):
            assert np.array_equal(bits(es[r][inside]), bits((a[r] - dense[r])[inside]))   # e = a - sent
            assert not es[r][~inside].any()
        oracle.decompress_avg_apply(descs, k, theta, payloads, lr)
        upd = ((dense[0] + dense[1]) * (np.float32(1) / np.float32(2))).astype(np.float32)
        theta_ref = (theta_ref.astype(np.float64) - float(np.float32(lr)) * upd.astype(np.float64)).astype(np.float32)
        assert np.array_equal(bits(theta), bits(theta_ref))


# --------------------------------------------------------------------------- payload well-formedness
def test_validate_payload_by_hand(oracle):
    """Hand-built records for a 70 x 100 tile-layout tensor (chunks: 64x64, 64x36, 6x64, 6x36):
    the checker accepts exactly the records whose positions ascend strictly and lie inside the
    tensor - each violation planted alone is caught."""
    descs, k = [(70, 100, 0, TILE)], 4
    rec = oracle.record_bytes(k)

    def payload(records):
        buf = np.zeros(oracle.payload_bytes(descs, k), dtype=np.uint8)
        for c, idx in enumerate(records):
            buf[16 + c * rec:16 + (c + 1) * rec] = oracle.pack_record(idx, [0, 1, 2, 3])
        return buf

    good = [[0, 63, 64, 4095], [0, 35, 64, 63 * 64 + 35], [0, 63, 5 * 64, 5 * 64 + 63], [0, 35, 64, 5 * 64 + 35]]
    assert oracle.validate_payload(descs, k, payload(good))
    for c, bad_rec in [
        (0, [0, 64, 63, 4095]),            # descending pair
        (0, [0, 63, 63, 4095]),            # repeated position
        (1, [0, 36, 64, 100]),             # column 36 of a 36-column edge tile
        (2, [0, 63, 64, 6 * 64]),          # row 6 of a 6-row edge tile
        (3, [0, 35, 64, 5 * 64 + 36]),     # corner tile, one column too far
        (3, [0, 35, 64, 4095]),            # corner tile, far outside
    ]:
        recs = [list(r) for r in good]
        recs[c] = bad_rec
        assert not oracle.validate_payload(descs, k, payload(recs)), (c, bad_rec)

    flat = [(1, 4096 + 10, 0, FLAT)]
    buf = np.zeros(oracle.payload_bytes(flat, k), dtype=np.uint8)
    buf[16:16 + rec] = oracle.pack_record([0, 1, 2, 4095], [0, 0, 0, 0])
    buf[16 + rec:16 + 2 * rec] = oracle.pack_record([0, 1, 2, 9], [0, 0, 0, 0])
    assert oracle.validate_payload(flat, k, buf)
    buf[16 + rec:16 + 2 * rec] = oracle.pack_record([0, 1, 2, 10], [0, 0, 0, 0])   # only 10 valid positions
    assert not oracle.validate_payload(flat, k, buf)


def test_validate_accepts_every_compressed_payload(oracle):
    descs, n = small_list()
    rng = np.random.default_rng(77)
    for k in (4, 32, 64):
        e = rng.normal(0, 1e-3, n).astype(np.float32)
        pay = oracle.compress(descs, k, e, rng.normal(0, 1e-3, n).astype(np.float32), 0.95)
        assert oracle.validate_payload(descs, k, pay)
