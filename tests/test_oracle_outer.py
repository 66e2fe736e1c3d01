"""Pins of the oracle's DiLoCo-family outer steps (Eq. (1); Section 3.2; appendix
"Exact algorithmic description of DiLoCo variants") against things other than
itself: exact rational arithmetic for every fused step, closed forms of the
momentum recursion, the paper's proposition that local outer momentum equals
global outer momentum (exact on dyadic inputs), brute-force Top-k for Sub-k,
and the pinned dense view of the payloads for the sparse Nesterov step.  CPU only.
"""
from fractions import Fraction

import numpy as np
import pytest

from test_oracle_pins import (FLAT, TILE, bits, brute_topk, chunk_elements, f32_round, small_list,
                              tensor_mask)


def fr(x):
    return Fraction(float(x))


def fma32(a, b, c):
    """One correctly rounded fp32 fused multiply-add, in exact arithmetic."""
    return f32_round(fr(a) * fr(b) + fr(c))


def tiny_list():
    return [(5, 9, 0, TILE), (1, 23, 48, FLAT)], 48 + 23 + 5     # gaps before, between and after


# --------------------------------------------------------------------------- local outer momentum
def test_lom_direction_is_two_fused_steps_and_touches_only_tensors(oracle):
    descs, n = tiny_list()
    rng = np.random.default_rng(200)
    mu = np.float32(0.9)
    m0 = rng.normal(0, 1e-2, n).astype(np.float32)
    d = rng.normal(0, 1e-3, n).astype(np.float32)
    m = m0.copy()
    out = np.full(n, np.float32(7.0))
    oracle.lom_direction(descs, m, d, mu, out=out)
    inside = tensor_mask(descs, n)
    for i in range(n):
        if inside[i]:
            mn = fma32(mu, m0[i], d[i])
            assert bits(m[i]) == bits(mn)
            assert bits(out[i]) == bits(fma32(mu, mn, d[i]))
        else:
            assert bits(m[i]) == bits(m0[i]) and out[i] == 7.0
    # in place: dir may overwrite delta
    m2, d2 = m0.copy(), d.copy()
    oracle.lom_direction(descs, m2, d2, mu, out=d2)
    assert np.array_equal(bits(d2[inside]), bits(out[inside])) and np.array_equal(bits(m2), bits(m))


def test_momentum_closed_form_for_a_constant_pseudo_gradient(oracle):
    """delta = c every round, mu = 1/2: m_t = c (2 - 2^(1-t)), dir_t = c + m_t / 2,
    exactly (dyadic c: nothing is rounded)."""
    descs = [(1, 64, 0, FLAT)]
    c = np.float32(0.375)
    m = np.zeros(64, dtype=np.float32)
    d = np.full(64, c)
    for t in range(1, 9):
        out = oracle.lom_direction(descs, m, d, 0.5)
        assert np.all(m == c * (2 - 2.0 ** (1 - t)))
        assert np.all(out == c + m / 2)
    # mu = 0: no momentum, the direction is the pseudo-gradient
    m = np.ones(64, dtype=np.float32)
    assert np.array_equal(oracle.lom_direction(descs, m, d, 0.0), d) and np.array_equal(m, d)


# --------------------------------------------------------------------------- dense aggregate
@pytest.mark.parametrize("R", [1, 3, 8])
@pytest.mark.parametrize("with_m", [False, True])
def test_dense_avg_apply_exact_rational(oracle, R, with_m):
    descs, n = tiny_list()
    rng = np.random.default_rng(210 + R)
    lr, mu = np.float32(0.7), np.float32(0.9)
    dirs = [rng.normal(0, 1e-3, n).astype(np.float32) for _ in range(R)]
    th0 = rng.normal(0, 0.02, n).astype(np.float32)
    m0 = rng.normal(0, 1e-3, n).astype(np.float32)
    th, m = th0.copy(), m0.copy()
    oracle.dense_avg_apply(descs, th, dirs, lr, m=m if with_m else None, mu=mu)
    inside = tensor_mask(descs, n)
    invR = np.float32(1.0) / np.float32(R)
    for i in range(n):
        if not inside[i]:
            assert bits(th[i]) == bits(th0[i]) and bits(m[i]) == bits(m0[i])
            continue
        acc = np.float32(0.0)
        for r in range(R):                      # r ascending, one rounding per add
            acc = f32_round(fr(acc) + fr(dirs[r][i]))
        dd = f32_round(fr(acc) * fr(invR))
        if with_m:
            mn = fma32(mu, m0[i], dd)
            assert bits(m[i]) == bits(mn)
            dd = fma32(mu, mn, dd)
        else:
            assert bits(m[i]) == bits(m0[i])
        assert bits(th[i]) == bits(f32_round(fr(th0[i]) - fr(lr) * fr(dd)))


def test_dense_avg_order_is_r_ascending(oracle):
    descs = [(1, 4, 0, FLAT)]
    vals = [1.0, 2.0 ** -24, 2.0 ** -24]      # (1 + e) + e = 1 in fp32, (e + e) + 1 = 1 + 2e
    for order, want in ((vals, 1.0), (vals[::-1], 1.0 + 2.0 ** -23)):
        th = np.zeros(4, dtype=np.float32)
        oracle.dense_avg_apply(descs, th, [np.full(4, v, dtype=np.float32) for v in order], -1.0)
        assert np.all(th == np.float32(np.float32(want) * (np.float32(1) / np.float32(3))))


def test_local_outer_momentum_equals_global_outer_momentum(oracle):
    """The paper's proposition (appendix "Equivalence of LOM and Global Outer Momentum"):
    with zero initial momenta the average of the local momenta is the global momentum
    and the parameters of DiLoCo-LOM and DiLoCo coincide at every step.  On dyadic
    inputs with mu = 1/2, lr = 1/2, R = 4 no operation rounds, so the two oracles
    paths must agree bit for bit; with ordinary inputs they agree to rounding."""
    descs, n = small_list()
    inside = tensor_mask(descs, n)
    R, T = 4, 4
    for exact in (True, False):
        rng = np.random.default_rng(220 + exact)
        mu, lr = (0.5, 0.5) if exact else (0.9, 0.7)
        th_lom = np.where(inside, rng.integers(-64, 65, n) / 64.0, 0).astype(np.float32)
        th_dil = th_lom.copy()
        m_loc = [np.zeros(n, dtype=np.float32) for _ in range(R)]
        m_glob = np.zeros(n, dtype=np.float32)
        for t in range(T):
            if exact:
                deltas = [np.where(inside, rng.integers(-32, 33, n) / 256.0, 0).astype(np.float32) for _ in range(R)]
            else:
                deltas = [np.where(inside, rng.normal(0, 1e-3, n), 0).astype(np.float32) for _ in range(R)]
            dirs = [oracle.lom_direction(descs, m_loc[r], deltas[r], mu) for r in range(R)]
            oracle.dense_avg_apply(descs, th_lom, dirs, lr)                       # DiLoCo-LOM
            oracle.dense_avg_apply(descs, th_dil, deltas, lr, m=m_glob, mu=mu)    # DiLoCo, Eq. (1)
            m_bar = sum(x.astype(np.float64) for x in m_loc) / R
            if exact:
                assert np.array_equal(m_bar, m_glob.astype(np.float64)), t
                assert np.array_equal(bits(th_lom), bits(th_dil)), t
            else:
                assert np.allclose(m_bar, m_glob, rtol=1e-5, atol=1e-9)
                assert np.allclose(th_lom, th_dil, rtol=1e-5, atol=1e-8)
        assert np.abs(th_lom[inside]).sum() > 0


# --------------------------------------------------------------------------- Sub-k
def test_sub_topk_removes_exactly_the_brute_force_top_k(oracle):
    rng = np.random.default_rng(230)
    for tile, layout, rows, cols in ((4, TILE, 7, 10), (4, FLAT, 1, 75), (3, TILE, 9, 9)):
        descs = [(rows, cols, 4, layout)]
        n = 4 + rows * cols + 3
        for k in (1, 2, 3):
            m0 = rng.choice([-2.0, -1.0, -0.5, 0.0, -0.0, 0.5, 1.0, 2.0, 3.0], n).astype(np.float32)
            m = m0.copy()
            idx = oracle.sub_topk(descs, k, m, tile=tile, want_idx=True)
            changed = np.zeros(n, bool)
            for c in range(oracle.tensor_chunks(descs[0], tile)):
                el = np.array([oracle.element_of(descs[0], c, j, tile) for j in range(tile * tile)])
                valid = [j for j in range(tile * tile) if el[j] >= 0]
                want = brute_topk(m0[el], valid, k)
                assert idx[c * k:(c + 1) * k].tolist() == sorted(want)
                changed[el[sorted(want)]] = True
            assert np.array_equal(bits(m[~changed]), bits(m0[~changed]))      # everything else untouched
            assert np.all(bits(m[changed]) == 0)                              # m - m = +0.0


def test_sub_topk_on_the_small_list(oracle):
    descs, n = small_list()
    rng = np.random.default_rng(231)
    m0 = rng.standard_t(3, n).astype(np.float32)
    chunks = chunk_elements(oracle, descs)
    for k in (32, 64):
        m = m0.copy()
        idx = oracle.sub_topk(descs, k, m, want_idx=True)
        # same selection as the compression path makes on a = m (beta = 1, delta = 0 keeps m)
        e = m0.copy()
        _, det = oracle.compress(descs, k, e, np.zeros(n, dtype=np.float32), 1.0, want_detail=True)
        assert np.array_equal(idx, det["idx"])
        zeroed = bits(m) != bits(m0)                      # the inputs hold no zeros
        assert zeroed.sum() == oracle.num_chunks(descs) * k and not m[zeroed].any()
        for _, _, el in chunks:                            # per chunk: what is left is no larger than what went
            el = el[el >= 0]
            z = zeroed[el]
            assert z.sum() == k and np.abs(m0[el][~z]).max() <= np.abs(m0[el][z]).min()
    m = m0.copy()
    oracle.sub_topk([(64, 64, 0, TILE)], 4096, m)                              # k = chunk: nothing is left
    assert not m[:4096].any() and np.array_equal(bits(m[4096:]), bits(m0[4096:]))


# --------------------------------------------------------------------------- sparse aggregate + Nesterov
@pytest.mark.parametrize("b", (2, 32))
def test_sparse_nesterov_equals_dense_step_on_the_dense_views(oracle, b):
    """The aggregate of the payloads, then Eq. (1)'s momentum: the same as feeding the dense
    views of the payloads (pinned elsewhere) to the dense step (pinned above in exact
    arithmetic) - adding the +0.0 of a worker that did not send a coordinate changes nothing."""
    descs = [(70, 130, 0, TILE), (1, 5000, 70 * 130 + 4, FLAT)]
    n = 70 * 130 + 4 + 5000
    k, R, lr, mu = 8, 5, 0.7, 0.9
    rng = np.random.default_rng(240 + b)
    inside = tensor_mask(descs, n)
    pays = []
    for r in range(R):
        e = np.zeros(n, dtype=np.float32)
        d = np.where(inside, rng.normal(0, 1e-3, n), 0).astype(np.float32)
        pays.append(oracle.compress_b(descs, k, b, e, d, 0.95))
    th0 = rng.normal(0, 0.02, n).astype(np.float32)
    m0 = np.where(inside, rng.normal(0, 1e-3, n), 0).astype(np.float32)
    th, m = th0.copy(), m0.copy()
    oracle.decompress_avg_apply_nesterov_b(descs, k, b, th, m, pays, lr, mu)
    th_d, m_d = th0.copy(), m0.copy()
    oracle.dense_avg_apply(descs, th_d, [oracle.decompress_dense_b(descs, k, b, p, n) for p in pays], lr,
                           m=m_d, mu=mu)
    assert np.array_equal(bits(th), bits(th_d)) and np.array_equal(bits(m), bits(m_d))
    assert (m != m0).sum() > inside.sum() // 2           # the momentum moves everywhere, not only where data was sent
    # mu = 0 is the plain sparse aggregate
    th1, th2, m1 = th0.copy(), th0.copy(), m0.copy()
    oracle.decompress_avg_apply_nesterov_b(descs, k, b, th1, m1, pays, lr, 0.0)
    oracle.decompress_avg_apply_b(descs, k, b, th2, pays, lr)
    assert np.array_equal(bits(th1), bits(th2))
