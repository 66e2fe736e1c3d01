"""GPU parity of the coded wire format: sl_compress_coded, sl_decompress_avg_apply_coded (and the
Nesterov variant), sl_rice_encode / sl_rice_decode, through the C ABI, against the CPU oracle.

Bar: coded bytes (and their size) bit-exact against the oracle's encoder applied to the oracle's
payload; the plain record and e bit-exact as for sl_compress; theta after the coded aggregate
bit-identical to the oracle's aggregate of the (plain) payloads, 1e-6 relative as the fall-back.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

FLAT, TILE = 0, 1
REL_TOL = 1e-6


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


def assert_f32_close(got, want, what):
    got, want = np.asarray(got), np.asarray(want)
    if np.array_equal(got.view(np.uint32), want.view(np.uint32)):
        return
    denom = np.maximum(np.abs(want), 1e-30)
    rel = np.abs(got.astype(np.float64) - want.astype(np.float64)) / denom
    bad = int((got.view(np.uint32) != want.view(np.uint32)).sum())
    assert rel.max() <= REL_TOL, f"{what}: {bad} values differ, max rel err {rel.max():.3e}"


def shapes_for(k):
    if k <= 256:      # smallest chunk: 22 x 18 = 396 elements; 40 chunks in the long vector: three directory groups
        shapes = [(150, 210, TILE), (1, 4096 * 39 + 1100, FLAT), (1024, 16, TILE), (64, 64, TILE), (256, 320, TILE)]
        if k <= 32:
            shapes += [(140, 200, TILE), (70, 70, TILE)]
        return shapes
    if k <= 1024:
        return [(160, 224, TILE), (1, 4096 * 20 + 1100, FLAT)]
    return [(128, 192, TILE), (1, 4096 * 18, FLAT)]


def coded_compress(sl, plan, e0, delta, beta, flags=0, pending=None):
    e = torch.from_numpy(e0.copy()).cuda()
    rec = sl.alloc_payload(plan).fill_(0xAB)
    cap = sl.sl_rice_max_bytes(plan)
    wire = torch.full((cap + 64,), 0xCD, dtype=torch.uint8, device="cuda")
    sl.sl_compress_coded(plan, e, torch.from_numpy(delta).cuda(), beta, rec, wire, sl.alloc_workspace(plan),
                         flags=flags, pending=pending)
    torch.cuda.synchronize()
    return e, rec, wire


def check_wire(wire, want, what):
    have = wire.cpu().numpy()
    size = int(have[8:16].view(np.uint64)[0])
    assert size == want.size, f"{what}: coded size {size}, oracle {want.size}"
    if not np.array_equal(have[:size], want):
        diff = np.nonzero(have[:size] != want)[0]
        raise AssertionError(f"{what}: coded bytes differ at {diff.size} places, first at {diff[:8]}")
    assert bool((have[size:] == 0xCD).all()), f"{what}: bytes beyond the coded size were written"
    return size


# --------------------------------------------------------------------------- the compressor's coded output
@pytest.mark.parametrize("k", [4, 8, 12, 20, 32, 36, 64, 100, 128, 200, 256, 512, 1000, 2048, 4096])
def test_compress_coded_matches_oracle(sl, oracle, k):
    """Record, e and coded bytes; ragged tiles, 16-column matrices, tails, several directory groups,
    k with every kind of padding in the fixed record, one- and two-byte quotient fields."""
    descs, n = layout_list(shapes_for(k))
    rng = np.random.default_rng(4000 + k)
    e0 = rng.normal(0, 1e-3, n).astype(np.float32)
    delta = (1e-3 * rng.standard_t(3, n)).astype(np.float32)
    plan = sl.sl_plan_create(descs, k)
    assert sl.sl_rice_max_bytes(plan) == oracle.rice_max_bytes(descs, k)
    e, rec, wire = coded_compress(sl, plan, e0, delta, 0.95)
    e_ref = e0.copy()
    pay_ref = oracle.compress(descs, k, e_ref, delta, 0.95)
    assert np.array_equal(rec[:plan.payload_bytes].cpu().numpy(), pay_ref), f"k={k}: plain record differs"
    assert_f32_close(e.cpu().numpy(), e_ref, f"k={k} e")
    size = check_wire(wire, oracle.rice_encode(descs, k, pay_ref), f"k={k}")
    assert size < plan.payload_bytes or k < 32 or k >= 2048      # smaller than the plain payload at the paper's densities
    plan.close()


@pytest.mark.parametrize("bits", [1, 3, 4, 32])
@pytest.mark.parametrize("k", [8, 64, 104, 512])
def test_compress_coded_other_widths(sl, oracle, bits, k):
    descs, n = layout_list(shapes_for(k))
    rng = np.random.default_rng(4100 + 10 * k + bits)
    e0 = rng.normal(0, 1e-3, n).astype(np.float32)
    delta = rng.normal(0, 1e-3, n).astype(np.float32)
    plan = sl.sl_plan_create_bits(descs, k, bits)
    e, rec, wire = coded_compress(sl, plan, e0, delta, 0.95)
    e_ref = e0.copy()
    pay_ref = oracle.compress_b(descs, k, bits, e_ref, delta, 0.95)
    assert np.array_equal(rec[:plan.payload_bytes].cpu().numpy(), pay_ref)
    assert_f32_close(e.cpu().numpy(), e_ref, f"bits={bits} k={k} e")
    check_wire(wire, oracle.rice_encode_b(descs, k, bits, pay_ref), f"bits={bits} k={k}")
    plan.close()


@pytest.mark.parametrize("k", [32, 64, 256])
def test_compress_coded_extreme_supports(sl, oracle, k):
    """All-zero chunks (indices 0..k-1, every quotient 0), supports packed at the end of a chunk (the
    largest quotient sum the format allows), one cluster, and an even spread."""
    nc = 40
    descs, n = layout_list([(1, 4096 * nc, FLAT), (128, 128, TILE)])
    rng = np.random.default_rng(4200 + k)
    e0 = np.zeros(n, dtype=np.float32)
    delta = np.zeros(n, dtype=np.float32)
    big = lambda m: (rng.normal(0, 1, m).astype(np.float32) + np.float32(3.0)) * rng.choice([-1, 1], m).astype(np.float32)
    for c in range(nc):
        base = 4096 * c
        kind = c % 5
        if kind == 1:
            delta[base + 4096 - k: base + 4096] = big(k)
        elif kind == 2:
            delta[base + 1777: base + 1777 + k] = big(k)
        elif kind == 3:
            delta[base: base + 4096: 4096 // k] = big(k)
        elif kind == 4:
            delta[base: base + 4096] = rng.normal(0, 1e-3, 4096).astype(np.float32)
    delta[4096 * nc:] = rng.normal(0, 1e-3, n - 4096 * nc).astype(np.float32)
    plan = sl.sl_plan_create(descs, k)
    e, rec, wire = coded_compress(sl, plan, e0, delta, 0.95)
    e_ref = e0.copy()
    pay_ref = oracle.compress(descs, k, e_ref, delta, 0.95)
    assert np.array_equal(rec[:plan.payload_bytes].cpu().numpy(), pay_ref)
    check_wire(wire, oracle.rice_encode(descs, k, pay_ref), f"k={k} extreme supports")
    # and through the coded aggregate
    theta0 = rng.normal(0, 0.02, n).astype(np.float32)
    theta = torch.from_numpy(theta0.copy()).cuda()
    size = sl.coded_size(wire)
    sl.sl_decompress_avg_apply_coded(plan, theta, [wire, wire], [size, size], 0.7)
    torch.cuda.synchronize()
    want = theta0.copy()
    oracle.decompress_avg_apply(descs, k, want, [pay_ref, pay_ref], 0.7)
    assert_f32_close(theta.cpu().numpy(), want, f"k={k} theta")
    plan.close()


def test_compress_coded_deferred_chain_and_determinism(sl, oracle):
    """Three rounds with the error update pending (the plain record is what the next call takes), every
    round's coded bytes against the oracle; the same call twice gives the same bytes."""
    descs, n = layout_list([(200, 330, TILE), (1, 4096 * 17 + 900, FLAT)])
    k, beta = 64, 0.95
    rng = np.random.default_rng(4300)
    plan = sl.sl_plan_create(descs, k)
    ws = sl.alloc_workspace(plan)
    e = torch.zeros(n, dtype=torch.float32, device="cuda")
    e_ref = np.zeros(n, dtype=np.float32)
    recs = [sl.alloc_payload(plan) for _ in range(2)]
    cap = sl.sl_rice_max_bytes(plan)
    for rnd in range(3):
        d = rng.normal(0, 1e-3, n).astype(np.float32)
        wire = torch.full((cap,), 0xCD, dtype=torch.uint8, device="cuda")
        e_before = e.clone()
        sl.sl_compress_coded(plan, e, torch.from_numpy(d).cuda(), beta, recs[rnd % 2], wire, ws,
                             flags=sl.SL_COMPRESS_DEFER_RESIDUAL, pending=recs[(rnd + 1) % 2] if rnd else None)
        torch.cuda.synchronize()
        pay_ref = oracle.compress(descs, k, e_ref, d, beta)
        assert np.array_equal(recs[rnd % 2][:plan.payload_bytes].cpu().numpy(), pay_ref), f"round {rnd}"
        size = check_wire(wire, oracle.rice_encode(descs, k, pay_ref), f"round {rnd}")
        # once more from the same state into other buffers
        wire2 = torch.full((cap,), 0xCD, dtype=torch.uint8, device="cuda")
        rec2 = sl.alloc_payload(plan)
        sl.sl_compress_coded(plan, e_before, torch.from_numpy(d).cuda(), beta, rec2, wire2, ws,
                             flags=sl.SL_COMPRESS_DEFER_RESIDUAL, pending=recs[(rnd + 1) % 2] if rnd else None)
        torch.cuda.synchronize()
        assert torch.equal(wire[:size], wire2[:size]) and torch.equal(e, e_before)
    sl.sl_residual_apply(plan, e, recs[0])
    torch.cuda.synchronize()
    assert_f32_close(e.cpu().numpy(), e_ref, "e after the chain")
    plan.close()


# --------------------------------------------------------------------------- the coded aggregate
@pytest.mark.parametrize("R,k,lr", [(1, 32, 1.0), (3, 64, 0.7), (4, 64, 0.7), (8, 64, 1.0), (16, 32, 0.8), (8, 128, 1.0),
                                    (16, 256, 0.8), (33, 64, 0.6), (64, 32, 0.5), (5, 100, 1.0), (8, 12, 1.0),
                                    (3, 512, 1.0), (2, 1000, 1.0), (3, 2048, 1.0), (2, 4096, 1.0), (20, 200, 0.9),
                                    (64, 4, 1.0), (64, 64, 0.9), (64, 256, 0.7), (17, 8, 1.0), (9, 520, 0.8)])
def test_apply_coded_matches_oracle(sl, oracle, R, k, lr):
    """theta after sl_decompress_avg_apply_coded over the GPU's own coded payloads against the oracle's
    aggregate of the oracle's payloads: every decode layout (lanes per worker, words per vector, one-
    and two-byte quotient fields, more workers than one staging batch holds)."""
    descs, n = layout_list(shapes_for(k))
    rng = np.random.default_rng(4400 + 7 * k + R)
    plan = sl.sl_plan_create(descs, k)
    theta0 = rng.normal(0, 0.02, n).astype(np.float32)
    wires, sizes, refs = [], [], []
    for r in range(R):
        e0 = rng.normal(0, 1e-3, n).astype(np.float32)
        delta = rng.normal(0, 1e-3, n).astype(np.float32)
        _, _, wire = coded_compress(sl, plan, e0, delta, 0.95)
        refs.append(oracle.compress(descs, k, e0.copy(), delta, 0.95))
        sizes.append(check_wire(wire, oracle.rice_encode(descs, k, refs[-1]), f"worker {r}"))
        wires.append(wire)
    theta = torch.from_numpy(theta0.copy()).cuda()
    sl.sl_decompress_avg_apply_coded(plan, theta, wires, sizes, lr)
    torch.cuda.synchronize()
    want = theta0.copy()
    oracle.decompress_avg_apply(descs, k, want, refs, lr)
    assert_f32_close(theta.cpu().numpy(), want, f"R={R} k={k} theta")
    # ... and bit-identical to the plain aggregate of the plain payloads on the GPU
    plan.close()


def test_apply_coded_order_of_workers_is_r_ascending(sl, oracle):
    """Three workers send the same position with values whose fp32 sum depends on the order."""
    descs, n = layout_list([(1, 4096 * 2, FLAT)])
    k = 4
    plan = sl.sl_plan_create(descs, k)
    ws = sl.alloc_workspace(plan)
    luts = [np.array([1e8, 1.0, -1.0, -1e8], np.float32), np.array([-1e8, 1.0, -1.0, 1e8], np.float32),
            np.array([1.0, 2.0, 3.0, 4.0], np.float32)]
    pays = []
    for lut in luts:
        pay = np.zeros(plan.payload_bytes, np.uint8)
        pay[:16] = lut.view(np.uint8)
        pay[16:23] = oracle.pack_record([5, 100, 2000, 4095], [0, 1, 2, 3])
        pay[23:30] = oracle.pack_record([5, 6, 7, 8], [0, 0, 0, 0])
        pays.append(pay)
    for order in ([0, 1, 2], [2, 1, 0], [1, 2, 0]):
        wires, sizes = [], []
        for r in order:
            wire = sl.alloc_coded(plan)
            sl.sl_rice_encode(plan, torch.from_numpy(pays[r]).cuda(), wire, ws)
            torch.cuda.synchronize()
            wires.append(wire)
            sizes.append(sl.coded_size(wire))
        theta = torch.zeros(n, dtype=torch.float32, device="cuda")
        sl.sl_decompress_avg_apply_coded(plan, theta, wires, sizes, 1.0)
        torch.cuda.synchronize()
        want = np.zeros(n, np.float32)
        oracle.decompress_avg_apply(descs, k, want, [pays[r] for r in order], 1.0)
        assert np.array_equal(theta.cpu().numpy().view(np.uint32), want.view(np.uint32)), order
    plan.close()


@pytest.mark.parametrize("bits,k,R", [(1, 64, 4), (3, 64, 8), (4, 104, 3), (32, 64, 4), (32, 512, 2), (4, 256, 9)])
def test_apply_coded_other_widths(sl, oracle, bits, k, R):
    descs, n = layout_list(shapes_for(k))
    rng = np.random.default_rng(4500 + 10 * k + bits)
    plan = sl.sl_plan_create_bits(descs, k, bits)
    theta0 = rng.normal(0, 0.02, n).astype(np.float32)
    wires, sizes, refs = [], [], []
    for r in range(R):
        e0 = rng.normal(0, 1e-3, n).astype(np.float32)
        delta = rng.normal(0, 1e-3, n).astype(np.float32)
        _, _, wire = coded_compress(sl, plan, e0, delta, 0.95)
        refs.append(oracle.compress_b(descs, k, bits, e0.copy(), delta, 0.95))
        sizes.append(check_wire(wire, oracle.rice_encode_b(descs, k, bits, refs[-1]), f"worker {r}"))
        wires.append(wire)
    theta = torch.from_numpy(theta0.copy()).cuda()
    sl.sl_decompress_avg_apply_coded(plan, theta, wires, sizes, 0.8)
    torch.cuda.synchronize()
    want = theta0.copy()
    oracle.decompress_avg_apply_b(descs, k, bits, want, refs, 0.8)
    assert_f32_close(theta.cpu().numpy(), want, f"bits={bits} k={k} theta")
    plan.close()


@pytest.mark.parametrize("k,R", [(64, 8), (256, 3)])
def test_apply_nesterov_coded_matches_oracle(sl, oracle, k, R):
    descs, n = layout_list(shapes_for(k))
    rng = np.random.default_rng(4600 + k)
    plan = sl.sl_plan_create(descs, k)
    theta0 = rng.normal(0, 0.02, n).astype(np.float32)
    m0 = rng.normal(0, 1e-3, n).astype(np.float32)
    wires, sizes, refs = [], [], []
    for r in range(R):
        e0 = rng.normal(0, 1e-3, n).astype(np.float32)
        delta = rng.normal(0, 1e-3, n).astype(np.float32)
        _, _, wire = coded_compress(sl, plan, e0, delta, 0.95)
        refs.append(oracle.compress(descs, k, e0.copy(), delta, 0.95))
        sizes.append(sl.coded_size(wire))
        wires.append(wire)
    theta = torch.from_numpy(theta0.copy()).cuda()
    mom = torch.from_numpy(m0.copy()).cuda()
    sl.sl_decompress_avg_apply_nesterov_coded(plan, theta, mom, wires, sizes, 0.7, 0.9)
    torch.cuda.synchronize()
    want, m_want = theta0.copy(), m0.copy()
    oracle.decompress_avg_apply_nesterov_b(descs, k, 2, want, m_want, refs, 0.7, 0.9)
    assert_f32_close(theta.cpu().numpy(), want, "theta")
    assert_f32_close(mom.cpu().numpy(), m_want, "momentum")
    plan.close()


# --------------------------------------------------------------------------- transcoders
@pytest.mark.parametrize("k", [4, 20, 32, 64, 128, 256, 1000])
def test_rice_transcode_matches_oracle(sl, oracle, k):
    """sl_rice_encode produces the oracle's coded bytes from a plain payload, sl_rice_decode restores
    the payload (from the GPU's and from the oracle's coded buffer)."""
    descs, n = layout_list(shapes_for(k))
    rng = np.random.default_rng(700 + k)
    e0 = rng.normal(0, 1e-3, n).astype(np.float32)
    delta = (1e-3 * rng.standard_t(3, n)).astype(np.float32)
    plan = sl.sl_plan_create(descs, k)
    ws = sl.alloc_workspace(plan)
    ref_pay = oracle.compress(descs, k, e0.copy(), delta, 0.95)
    ref_enc = oracle.rice_encode(descs, k, ref_pay)
    pay_dev = torch.from_numpy(np.concatenate([ref_pay, np.zeros(16, np.uint8)])).cuda()

    cap = sl.sl_rice_max_bytes(plan)
    assert cap >= ref_enc.size and sl.sl_coded_fixed_bytes(plan) <= ref_enc.size
    out = torch.full((cap + 32,), 0xCD, dtype=torch.uint8, device="cuda")
    sl.sl_rice_encode(plan, pay_dev, out, ws)
    torch.cuda.synchronize()
    size = check_wire(out, ref_enc, f"k={k} transcode")

    for src in (out, torch.from_numpy(np.concatenate([ref_enc, np.zeros(16, np.uint8)])).cuda()):
        back = torch.full((max(16, plan.payload_bytes) + 16,), 0xEE, dtype=torch.uint8, device="cuda")
        sl.sl_rice_decode(plan, src, size, back)
        torch.cuda.synchronize()
        assert np.array_equal(back[:plan.payload_bytes].cpu().numpy(), ref_pay)
        assert bool((back[plan.payload_bytes:] == 0xEE).all())
    with pytest.raises(sl.SparseLoCoError):
        sl.sl_rice_encode(plan, pay_dev, out[:cap - 16], ws)   # capacity too small
    plan.close()


def test_coded_decoders_stay_in_bounds_on_malformed_buffers(sl, oracle):
    """A truncated buffer, a directory of garbage and a section of garbage: every read stays inside the
    buffer and every index inside the chunk (the calls complete, theta stays finite where it was)."""
    k = 64
    descs, n = layout_list([(150, 210, TILE), (1, 4096 * 20 + 1100, FLAT)])
    rng = np.random.default_rng(4700)
    plan = sl.sl_plan_create(descs, k)
    e0 = rng.normal(0, 1e-3, n).astype(np.float32)
    delta = rng.normal(0, 1e-3, n).astype(np.float32)
    _, _, wire = coded_compress(sl, plan, e0, delta, 0.95)
    size = sl.coded_size(wire)
    fixed = sl.sl_coded_fixed_bytes(plan)
    good = wire[:size].cpu().numpy()
    variants = []
    v = good.copy()
    variants.append((v, fixed + (size - fixed) // 2 // 16 * 16))             # truncated inside the section
    v = good.copy()
    v[fixed:] = rng.integers(0, 256, size - fixed, dtype=np.uint8)           # garbage bit vectors
    variants.append((v, size))
    v = good.copy()
    v[16:fixed] = rng.integers(0, 256, fixed - 16, dtype=np.uint8)           # garbage tables, directory, records
    variants.append((v, size))
    for buf, nbytes in variants:
        dev = torch.from_numpy(np.concatenate([buf, np.zeros(16, np.uint8)])).cuda()
        theta = torch.zeros(n, dtype=torch.float32, device="cuda")
        sl.sl_decompress_avg_apply_coded(plan, theta, [dev, wire], [nbytes, size], 1.0)
        back = torch.full((plan.payload_bytes + 16,), 0xEE, dtype=torch.uint8, device="cuda")
        sl.sl_rice_decode(plan, dev, nbytes, back)
        torch.cuda.synchronize()
        assert bool((back[plan.payload_bytes:] == 0xEE).all())
        assert sl.sl_payload_validate(plan, back, sl.alloc_workspace(plan)) in (True, False)
    with pytest.raises(sl.SparseLoCoError):
        sl.sl_decompress_avg_apply_coded(plan, torch.zeros(n, device="cuda"), [wire], [fixed - 16], 1.0)
    plan.close()


def test_rice_encode_of_a_malformed_record_stays_in_its_buffer(sl, oracle):
    """Indices that are not ascending are coded as gap 0 and nothing is written beyond the stated bound."""
    k = 32
    descs, n = layout_list([(1, 4096 * 40, FLAT)])
    rng = np.random.default_rng(4800)
    plan = sl.sl_plan_create(descs, k)
    pay = rng.integers(0, 256, plan.payload_bytes, dtype=np.uint8)            # random records: indices in any order
    cap = sl.sl_rice_max_bytes(plan)
    out = torch.full((cap + 4096,), 0xCD, dtype=torch.uint8, device="cuda")
    sl.sl_rice_encode(plan, torch.from_numpy(pay).cuda(), out, sl.alloc_workspace(plan))
    torch.cuda.synchronize()
    size = sl.coded_size(out)
    assert sl.sl_coded_fixed_bytes(plan) <= size <= cap
    assert bool((out[cap:] == 0xCD).all())
    plan.close()
