"""Pins of the oracle's Random-k selection (the paper's ablation "Random-k vs. Top-k":
the same pipeline with k random positions per chunk) against things other than itself:
published values of the generator's finalizer, a brute-force subset on tiny chunks,
uniformity of the chosen positions, independence from the data, and the pinned quantizer
and wire format applied to the chosen values.  CPU only."""
import os

import numpy as np
import pytest

from test_oracle_pins import FLAT, TILE, bits, small_list, tensor_mask

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "murmur3_vectors.txt")


def test_finalizer_matches_published_values(oracle):
    rows = [l.split("#")[0].split() for l in open(GOLDEN)]
    rows = [r for r in rows if len(r) == 2]
    assert len(rows) == 3
    for seed, want in rows:
        assert oracle.fmix32(int(seed, 16)) == int(want, 16)
    # a bijection on 32 bits: no two of many inputs collide
    xs = np.arange(200000, dtype=np.uint64) * 20011
    assert len({oracle.fmix32(int(x)) for x in xs[:20000]}) == 20000
    assert oracle.random_key(5, 7, 9) == oracle.fmix32(oracle.fmix32(oracle.fmix32(5) ^ 7) ^ 9) >> 1 < 2**31


def test_selection_is_the_k_largest_keys_brute_force(oracle):
    """The selected set is the k positions with the largest keys (ties to the lower index),
    listed in ascending index, over ragged tiles and a ragged tail; it does not depend on the data."""
    descs = [(70, 100, 0, TILE), (1, 5000, 7008, FLAT)]
    n = 7008 + 5000
    rng = np.random.default_rng(2)
    for k, seed in ((4, 0), (8, 12345), (32, 0xFFFFFFFF)):
        e = np.zeros(n, dtype=np.float32)
        d = np.where(tensor_mask(descs, n), rng.normal(0, 1e-3, n), 0).astype(np.float32)
        _, idx = oracle.compress_random_b(descs, k, 2, e, d, 0.95, seed, want_idx=True)
        _, idx2 = oracle.compress_random_b(descs, k, 2, np.ones(n, dtype=np.float32), -d, 0.5, seed, want_idx=True)
        assert np.array_equal(idx, idx2)                       # the data plays no part
        chunk = 0
        for desc in descs:
            for c in range(oracle.tensor_chunks(desc)):
                valid = [j for j in range(4096) if oracle.element_of(desc, c, j) >= 0]
                keys = {j: oracle.random_key(seed, chunk, j) for j in valid}
                want = sorted(sorted(valid, key=lambda j: (-keys[j], j))[:k])
                assert idx[chunk * k:(chunk + 1) * k].tolist() == want, (desc, c)
                chunk += 1


def test_selected_positions_are_uniform(oracle):
    """Over many chunks and seeds every position is chosen about equally often
    (chi-square against the uniform distribution, 4095 degrees of freedom)."""
    nc, k = 512, 64
    descs = [(1, 4096 * nc, 0, FLAT)]
    counts = np.zeros(4096)
    z = np.zeros(4096 * nc, dtype=np.float32)
    for seed in (1, 2, 3, 4):
        _, idx = oracle.compress_random_b(descs, k, 2, z.copy(), z, 0.95, seed, want_idx=True)
        counts += np.bincount(idx, minlength=4096)
        sets = idx.reshape(nc, k)
        assert len({tuple(s) for s in sets}) == nc             # chunks get different subsets
    expect = counts.sum() / 4096
    chi2 = ((counts - expect) ** 2 / expect).sum()
    assert 4095 - 5 * np.sqrt(2 * 4095) < chi2 < 4095 + 5 * np.sqrt(2 * 4095)
    _, a = oracle.compress_random_b(descs, k, 2, z.copy(), z, 0.95, 10, want_idx=True)
    _, b = oracle.compress_random_b(descs, k, 2, z.copy(), z, 0.95, 11, want_idx=True)
    overlap = np.mean([len(set(x) & set(y)) for x, y in zip(a.reshape(nc, k), b.reshape(nc, k))])
    assert abs(overlap - k * k / 4096) < 0.3                    # two seeds: independent subsets


@pytest.mark.parametrize("b", (2, 4, 32))
def test_everything_after_the_selection_is_the_pinned_pipeline(oracle, b):
    """Payload and error buffer equal what the pinned pieces give on the chosen positions:
    accumulate, the tensor's quantizer on the chosen values, the record encoder, the residual."""
    descs, n = small_list()
    k, seed = 32, 99
    rng = np.random.default_rng(3 + b)
    inside = tensor_mask(descs, n)
    e0 = np.where(inside, rng.normal(0, 1e-3, n), 0).astype(np.float32)
    d = np.where(inside, rng.standard_t(3, n) * 1e-3, 0).astype(np.float32)
    e = e0.copy()
    pay, idx = oracle.compress_random_b(descs, k, b, e, d, 0.95, seed, want_idx=True)
    a = e0.copy()
    oracle.accumulate(a, d, 0.95)
    want_e, blocks, chunk = a.copy(), [], 0
    for desc in descs:
        nc = oracle.tensor_chunks(desc)
        el = np.array([[oracle.element_of(desc, c, int(j)) for j in idx[(chunk + c) * k:(chunk + c + 1) * k]]
                       for c in range(nc)])
        assert (el >= 0).all()
        vals = a[el.ravel()]
        if b == 32:
            sent, lut_bytes = vals, b""
            recs = [oracle.pack_record_b(idx[(chunk + c) * k:(chunk + c + 1) * k], vals[c * k:(c + 1) * k], 32)
                    for c in range(nc)]
        else:
            code, lut, _ = oracle.quantize_tensor_b(vals, nc, k, b)
            sent = lut[code]
            lut_bytes = lut.tobytes().ljust(oracle.header_bytes_b(b), b"\0")
            recs = [oracle.pack_record_b(idx[(chunk + c) * k:(chunk + c + 1) * k], code[c * k:(c + 1) * k], b)
                    for c in range(nc)]
        want_e[el.ravel()] = vals - sent
        blk = lut_bytes + b"".join(r.tobytes() for r in recs)
        blocks.append(blk.ljust((len(blk) + 15) // 16 * 16, b"\0"))
        chunk += nc
    assert pay.tobytes() == b"".join(blocks)
    assert np.array_equal(bits(e), bits(want_e))
    # k = chunk size: nothing is left to chance
    full = [(64, 64, 0, TILE)]
    e1, e2 = np.zeros(4096, dtype=np.float32), np.zeros(4096, dtype=np.float32)
    d1 = rng.normal(0, 1e-3, 4096).astype(np.float32)
    assert np.array_equal(oracle.compress_random_b(full, 4096, b, e1, d1, 0.95, 7),
                          oracle.compress_b(full, 4096, b, e2, d1, 0.95))
