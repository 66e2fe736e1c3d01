"""GPU parity for the outer steps of the DiLoCo family (local outer momentum, dense
aggregate with and without Nesterov momentum, sparse aggregate with global
momentum, Sub-k) and for the paper's variants composed from them, against the
CPU oracle: bit-identical fp32, else within 1e-6 relative."""
import numpy as np
import pytest
import torch

from test_gpu_parity import FLAT, TILE, assert_f32_close, layout_list, sl  # noqa: F401 (fixture)

pytestmark = pytest.mark.gpu

SHAPES = [(150, 210, TILE), (1, 9000, FLAT), (128, 192, TILE), (1024, 16, TILE), (1, 4096 + 1030, FLAT)]


def inside_mask(descs, n):
    m = np.zeros(n, bool)
    for r, c, off, _ in descs:
        m[off:off + r * c] = True
    return m


def dev(x):
    return torch.from_numpy(x.copy()).cuda()


def test_lom_direction(sl, oracle):
    descs, n = layout_list(SHAPES)
    n += 64
    rng = np.random.default_rng(2000)
    plan = sl.sl_plan_create(descs, 32)
    m0 = rng.normal(0, 1e-2, n).astype(np.float32)
    d0 = rng.normal(0, 1e-3, n).astype(np.float32)
    m, d = dev(m0), dev(d0)
    out = torch.full((n,), 7.0, dtype=torch.float32, device="cuda")
    sl.sl_lom_direction(plan, m, d, 0.9, out)
    torch.cuda.synchronize()
    m_ref = m0.copy()
    out_ref = oracle.lom_direction(descs, m_ref, d0, 0.9, out=np.full(n, np.float32(7.0)))
    assert_f32_close(m.cpu().numpy(), m_ref, "m")
    assert_f32_close(out.cpu().numpy(), out_ref, "dir")
    # in place: the direction overwrites the pseudo-gradient
    m2, d2 = dev(m0), dev(d0)
    sl.sl_lom_direction(plan, m2, d2, 0.9, d2)
    torch.cuda.synchronize()
    ins = inside_mask(descs, n)
    assert_f32_close(d2.cpu().numpy()[ins], out_ref[ins], "dir in place")
    assert np.array_equal(d2.cpu().numpy()[~ins].view(np.uint32), d0[~ins].view(np.uint32))


@pytest.mark.parametrize("R", [1, 3, 8, 16])
@pytest.mark.parametrize("with_m", [False, True])
def test_dense_avg_apply(sl, oracle, R, with_m):
    descs, n = layout_list(SHAPES)
    n += 64
    rng = np.random.default_rng(2100 + R)
    plan = sl.sl_plan_create(descs, 32)
    dirs = [(1e-3 * rng.standard_t(3, n)).astype(np.float32) for _ in range(R)]
    th0 = rng.normal(0, 0.02, n).astype(np.float32)
    m0 = rng.normal(0, 1e-3, n).astype(np.float32)
    th, m = dev(th0), dev(m0)
    sl.sl_dense_avg_apply(plan, th, m if with_m else None, [dev(x) for x in dirs], 0.7, 0.9)
    torch.cuda.synchronize()
    th_ref, m_ref = th0.copy(), m0.copy()
    oracle.dense_avg_apply(descs, th_ref, dirs, 0.7, m=m_ref if with_m else None, mu=0.9)
    assert_f32_close(th.cpu().numpy(), th_ref, "theta")
    assert_f32_close(m.cpu().numpy(), m_ref, "momentum")


@pytest.mark.parametrize("k", [8, 32, 64, 128, 256, 512])
def test_sub_topk(sl, oracle, k):
    shapes = SHAPES if k <= 256 else [(160, 224, TILE), (1024, 16, TILE), (1, 8192 + 1000, FLAT)]
    descs, n = layout_list(shapes)
    n += 64
    rng = np.random.default_rng(2200 + k)
    plan = sl.sl_plan_create_bits(descs, k, 32)
    m0 = (1e-3 * rng.standard_t(3, n)).astype(np.float32)
    r, c, off, _ = descs[2]
    m0[off:off + r * c] = rng.choice([-1e-3, 0.0, -0.0, 1e-3, 2e-3], r * c).astype(np.float32)   # ties
    m = dev(m0)
    sl.sl_sub_topk(plan, m)
    torch.cuda.synchronize()
    m_ref = m0.copy()
    oracle.sub_topk(descs, k, m_ref)
    assert np.array_equal(m.cpu().numpy().view(np.uint32), m_ref.view(np.uint32))
    plan2 = sl.sl_plan_create(descs, k)                    # the value width of the plan plays no part
    m2 = dev(m0)
    sl.sl_sub_topk(plan2, m2)
    torch.cuda.synchronize()
    assert np.array_equal(m2.cpu().numpy().view(np.uint32), m_ref.view(np.uint32))


@pytest.mark.parametrize("bits", [2, 32])
@pytest.mark.parametrize("R,k", [(1, 32), (8, 64), (5, 128)])
def test_sparse_aggregate_with_nesterov_momentum(sl, oracle, bits, R, k):
    descs, n = layout_list(SHAPES)
    rng = np.random.default_rng(2300 + R + bits)
    plan = sl.sl_plan_create_bits(descs, k, bits)
    ws = sl.alloc_workspace(plan)
    pays_dev, pays = [], []
    for r in range(R):
        delta = (1e-3 * rng.standard_t(3, n)).astype(np.float32)
        e = torch.zeros(n, dtype=torch.float32, device="cuda")
        pay = sl.alloc_payload(plan)
        sl.sl_compress(plan, e, dev(delta), 0.95, pay, ws)
        torch.cuda.synchronize()
        pays_dev.append(pay)
        pays.append(oracle.compress_b(descs, k, bits, np.zeros(n, dtype=np.float32), delta, 0.95))
        assert np.array_equal(pay[:plan.payload_bytes].cpu().numpy(), pays[-1])
    th0 = rng.normal(0, 0.02, n).astype(np.float32)
    m0 = rng.normal(0, 1e-3, n).astype(np.float32)
    th, m = dev(th0), dev(m0)
    for _ in range(2):                                     # two outer steps: the momentum carries over
        sl.sl_decompress_avg_apply_nesterov(plan, th, m, pays_dev, 0.7, 0.9)
    torch.cuda.synchronize()
    th_ref, m_ref = th0.copy(), m0.copy()
    for _ in range(2):
        oracle.decompress_avg_apply_nesterov_b(descs, k, bits, th_ref, m_ref, pays, 0.7, 0.9)
    assert_f32_close(th.cpu().numpy(), th_ref, "theta")
    assert_f32_close(m.cpu().numpy(), m_ref, "momentum")


def test_variants_three_outer_steps(sl, oracle):
    """DiLoCo-LOM-Sub-k and DiLoCo-LOM+Top-k+EF, three outer steps with R = 4 workers,
    composed from the entry points as the header describes, against the same composition
    of oracle functions (all state carried: theta, m_r, e_r)."""
    descs, n = layout_list(SHAPES)
    rng = np.random.default_rng(2400)
    R, k, mu, rho, lr = 4, 64, 0.9, 0.95, 0.7
    ins = inside_mask(descs, n)
    plan = sl.sl_plan_create_bits(descs, k, 32)
    ws = sl.alloc_workspace(plan)
    th0 = rng.normal(0, 0.02, n).astype(np.float32)
    # --- DiLoCo-LOM-Sub-k
    th, th_ref = dev(th0), th0.copy()
    m = [torch.zeros(n, dtype=torch.float32, device="cuda") for _ in range(R)]
    m_ref = [np.zeros(n, dtype=np.float32) for _ in range(R)]
    for t in range(3):
        deltas = [rng.normal(0, 1e-3, n).astype(np.float32) for _ in range(R)]
        dirs, dirs_ref = [], []
        for r in range(R):
            out = torch.empty(n, dtype=torch.float32, device="cuda")
            sl.sl_lom_direction(plan, m[r], dev(deltas[r]), mu, out)
            dirs.append(out)
            dirs_ref.append(oracle.lom_direction(descs, m_ref[r], deltas[r], mu))
        sl.sl_dense_avg_apply(plan, th, None, dirs, lr)
        oracle.dense_avg_apply(descs, th_ref, dirs_ref, lr)
        for r in range(R):
            sl.sl_sub_topk(plan, m[r])
            oracle.sub_topk(descs, k, m_ref[r])
        torch.cuda.synchronize()
        assert_f32_close(th.cpu().numpy()[ins], th_ref[ins], f"Sub-k theta step {t}")
        for r in range(R):
            assert_f32_close(m[r].cpu().numpy()[ins], m_ref[r][ins], f"Sub-k m[{r}] step {t}")
    # --- DiLoCo-LOM+Top-k+EF
    th, th_ref = dev(th0), th0.copy()
    m = [torch.zeros(n, dtype=torch.float32, device="cuda") for _ in range(R)]
    e = [torch.zeros(n, dtype=torch.float32, device="cuda") for _ in range(R)]
    m_ref = [np.zeros(n, dtype=np.float32) for _ in range(R)]
    e_ref = [np.zeros(n, dtype=np.float32) for _ in range(R)]
    pays = [sl.alloc_payload(plan) for _ in range(R)]
    for t in range(3):
        refs = []
        for r in range(R):
            delta = rng.normal(0, 1e-3, n).astype(np.float32)
            d = dev(delta)
            sl.sl_lom_direction(plan, m[r], d, mu, d)                       # direction in place
            sl.sl_compress(plan, e[r], d, rho, pays[r], ws)
            dir_ref = oracle.lom_direction(descs, m_ref[r], delta, mu, out=np.zeros(n, dtype=np.float32))
            refs.append(oracle.compress_b(descs, k, 32, e_ref[r], dir_ref, rho))
            torch.cuda.synchronize()
            assert np.array_equal(pays[r][:plan.payload_bytes].cpu().numpy(), refs[-1]), (t, r)
            assert_f32_close(e[r].cpu().numpy()[ins], e_ref[r][ins], f"LOM+Top-k e[{r}] step {t}")
        sl.sl_decompress_avg_apply(plan, th, pays, lr)
        oracle.decompress_avg_apply_b(descs, k, 32, th_ref, refs, lr)
        torch.cuda.synchronize()
        assert_f32_close(th.cpu().numpy(), th_ref, f"LOM+Top-k theta step {t}")


def test_argument_errors(sl):
    plan = sl.sl_plan_create([(64, 64, 0, TILE)], 32)
    a = torch.zeros(4096, dtype=torch.float32, device="cuda")
    b = torch.zeros(4096, dtype=torch.float32, device="cuda")
    with pytest.raises(sl.SparseLoCoError):
        sl.sl_lom_direction(plan, a, a, 0.9, b)                 # m aliases delta
    with pytest.raises(sl.SparseLoCoError):
        sl.sl_lom_direction(plan, a, b, 0.9, a)                 # m aliases dir
    with pytest.raises(sl.SparseLoCoError):
        sl.sl_dense_avg_apply(plan, a, None, [], 0.7)           # R = 0
    with pytest.raises(sl.SparseLoCoError):
        sl.sl_dense_avg_apply(plan, a, None, [a], 0.7)          # a direction aliases theta
    with pytest.raises(sl.SparseLoCoError):
        sl.sl_dense_avg_apply(plan, a, a, [b], 0.7)             # momentum aliases theta
    with pytest.raises(sl.SparseLoCoError):
        sl.sl_decompress_avg_apply_nesterov(plan, a, a, [sl.alloc_payload(plan)], 0.7, 0.9)
