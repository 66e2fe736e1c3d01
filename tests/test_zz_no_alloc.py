"""sl_compress_noalloc (the entry point that allocates nothing) against sl_compress.

Through the C ABI: the same inputs go through sl_compress with a caller's workspace and
through sl_compress_noalloc with the library's fixed scratch array; payload bytes and the
error buffer must be bit-identical (and equal the CPU oracle's).  Two calls in a row, the
second on a smaller list with another k, so that whatever the first call left in the shared
array lies under the second call's sections; then a deferred-residual chain, and a plan that
needs more scratch than the array holds.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

FLAT, TILE = 0, 1


@pytest.fixture(scope="module")
def sl():
    from paper_2508_15706_amd import binding
    binding.lib()
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return binding


def layout_list(shapes):
    descs, off = [], 0
    for r, c, lay in shapes:
        descs.append((r, c, off, lay))
        off += (r * c + 63) // 64 * 64
    return descs, off


def both_ways(sl, oracle, shapes, k, seed, beta=0.95):
    descs, n = layout_list(shapes)
    rng = np.random.default_rng(seed)
    e0 = rng.normal(0, 1e-3, n).astype(np.float32)
    d0 = rng.normal(0, 1e-3, n).astype(np.float32)
    plan = sl.sl_plan_create(descs, k)
    assert plan.workspace_bytes <= sl.SL_NOALLOC_SCRATCH_BYTES

    e_a = torch.from_numpy(e0).cuda()
    pay_a = sl.alloc_payload(plan).fill_(0xAB)
    sl.sl_compress(plan, e_a, torch.from_numpy(d0).cuda(), beta, pay_a, sl.alloc_workspace(plan))

    e_b = torch.from_numpy(e0).cuda()
    pay_b = sl.alloc_payload(plan).fill_(0xCD)
    sl.sl_compress_noalloc(plan, e_b, torch.from_numpy(d0).cuda(), beta, pay_b)
    torch.cuda.synchronize()

    nb = plan.payload_bytes
    assert torch.equal(pay_a[:nb], pay_b[:nb]), f"k={k}: payload bytes differ between the two entry points"
    assert torch.equal(e_a.view(torch.int32), e_b.view(torch.int32)), f"k={k}: e differs between the two entry points"
    e_ref = e0.copy()
    pay_ref = oracle.compress(descs, k, e_ref, d0, beta)
    assert np.array_equal(pay_b[:nb].cpu().numpy(), pay_ref), f"k={k}: payload differs from the oracle"
    assert np.array_equal(e_b.cpu().numpy().view(np.uint32), e_ref.view(np.uint32)), f"k={k}: e differs from the oracle"
    plan.close()


def test_noalloc_equals_compress_on_two_calls_in_a_row(sl, oracle):
    # first call: several tensors, ragged edges, 2,400 chunks; second call: fewer and smaller, another k
    both_ways(sl, oracle, [(1536, 6144, TILE), (150, 210, TILE), (1, 9000, FLAT), (1024, 16, TILE)], 64, seed=1)
    both_ways(sl, oracle, [(256, 320, TILE), (1, 5000, FLAT)], 32, seed=2)
    # and a third, at a density that takes the other kernel routes, on top of the same array
    both_ways(sl, oracle, [(320, 250, TILE), (1, 4096 + 1030, FLAT)], 512, seed=3)


def test_noalloc_deferred_chain_equals_compress(sl, oracle):
    """Three rounds with the error update left pending, each round through both entry points."""
    shapes = [(200, 330, TILE), (1, 7000, FLAT)]
    descs, n = layout_list(shapes)
    k, beta = 64, 0.95
    rng = np.random.default_rng(7)
    plan = sl.sl_plan_create(descs, k)
    ws = sl.alloc_workspace(plan)
    e_a = torch.zeros(n, dtype=torch.float32, device="cuda")
    e_b = torch.zeros(n, dtype=torch.float32, device="cuda")
    pays_a = [sl.alloc_payload(plan) for _ in range(2)]
    pays_b = [sl.alloc_payload(plan) for _ in range(2)]
    e_ref = np.zeros(n, dtype=np.float32)
    for rnd in range(3):
        d = rng.normal(0, 1e-3, n).astype(np.float32)
        dg = torch.from_numpy(d).cuda()
        pend_a = pays_a[(rnd + 1) % 2] if rnd else None
        pend_b = pays_b[(rnd + 1) % 2] if rnd else None
        sl.sl_compress(plan, e_a, dg, beta, pays_a[rnd % 2], ws, flags=sl.SL_COMPRESS_DEFER_RESIDUAL, pending=pend_a)
        sl.sl_compress_noalloc(plan, e_b, dg, beta, pays_b[rnd % 2], flags=sl.SL_COMPRESS_DEFER_RESIDUAL,
                               pending=pend_b)
        torch.cuda.synchronize()
        nb = plan.payload_bytes
        assert torch.equal(pays_a[rnd % 2][:nb], pays_b[rnd % 2][:nb]), f"round {rnd}: payloads differ"
        assert torch.equal(e_a.view(torch.int32), e_b.view(torch.int32)), f"round {rnd}: e differs"
        pay_ref = oracle.compress(descs, k, e_ref, d, beta)
        assert np.array_equal(pays_b[rnd % 2][:nb].cpu().numpy(), pay_ref), f"round {rnd}: payload differs from the oracle"
    sl.sl_residual_apply(plan, e_b, pays_b[0])
    torch.cuda.synchronize()
    assert np.array_equal(e_b.cpu().numpy().view(np.uint32), e_ref.view(np.uint32))
    plan.close()


def test_noalloc_rejects_a_plan_beyond_its_scratch(sl):
    """A list whose workspace exceeds the fixed array is refused before anything is launched."""
    rows = 64 * 700                                     # 700 x 400 = 280,000 chunks at k = 64: about 90 MB of scratch
    descs = [(rows, 64 * 400, 0, TILE)]
    plan = sl.sl_plan_create(descs, 64)
    assert plan.workspace_bytes > sl.SL_NOALLOC_SCRATCH_BYTES
    e = torch.zeros(16, dtype=torch.float32, device="cuda")      # never touched: the call must fail first
    d = torch.zeros(16, dtype=torch.float32, device="cuda")
    pay = torch.full((64,), 0x5A, dtype=torch.uint8, device="cuda")
    with pytest.raises(sl.SparseLoCoError) as err:
        sl.sl_compress_noalloc(plan, e, d, 0.95, pay)
    assert err.value.status == sl.SL_ERR_TOO_LARGE
    torch.cuda.synchronize()
    assert bool((pay == 0x5A).all())
    plan.close()
