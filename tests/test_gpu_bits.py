"""GPU parity for the other value widths (1, 3, 4 bits and unquantized fp32; 2 bits
through the same entry point): the HIP path through the C ABI against the CPU
oracle.  Payload bytes bit-exact; e and theta bit-identical, else within 1e-6
relative."""
import numpy as np
import pytest
import torch

from test_gpu_parity import FLAT, TILE, assert_f32_close, layout_list, sl  # noqa: F401 (fixture)

pytestmark = pytest.mark.gpu

WIDTHS = (1, 2, 3, 4, 32)


def degenerate_inputs(descs, n, rng):
    """Tensor 0 all zero (sigma = 0), tensor 1 few distinct magnitudes, the rest heavy-tailed."""
    delta = (1e-3 * rng.standard_t(3, n)).astype(np.float32)
    e0 = rng.normal(0, 1e-3, n).astype(np.float32)
    r, c, off, _ = descs[0]
    delta[off:off + r * c] = 0
    e0[off:off + r * c] = 0
    r, c, off, _ = descs[1]
    delta[off:off + r * c] = rng.choice([-3e-3, -1e-3, -0.0, 0.0, 1e-3, 3e-3], r * c).astype(np.float32)
    e0[off:off + r * c] = 0
    return e0, delta


@pytest.mark.parametrize("bits", WIDTHS)
@pytest.mark.parametrize("k", [8, 32, 64, 128, 512])
def test_compress_matches_oracle(sl, oracle, bits, k):
    if k <= 256:
        shapes = [(128, 128, TILE), (1, 8192, FLAT), (150, 210, TILE), (1, 9000, FLAT), (1024, 16, TILE),
                  (128, 192, TILE)]
    else:
        shapes = [(128, 128, TILE), (1, 8192, FLAT), (160, 224, TILE), (1, 8192 + 1000, FLAT)]
    descs, n = layout_list(shapes)
    rng = np.random.default_rng(1000 + 10 * k + bits)
    e0, delta = degenerate_inputs(descs, n, rng)
    plan = sl.sl_plan_create_bits(descs, k, bits)
    assert plan.value_bits == bits
    assert plan.payload_bytes == oracle.payload_bytes_b(descs, k, bits)
    e = torch.from_numpy(e0.copy()).cuda()
    pay = sl.alloc_payload(plan)
    pay.fill_(0xAB)
    ws = sl.alloc_workspace(plan)
    sl.sl_compress(plan, e, torch.from_numpy(delta).cuda(), 0.95, pay, ws)
    torch.cuda.synchronize()
    e_ref = e0.copy()
    ref = oracle.compress_b(descs, k, bits, e_ref, delta, 0.95)
    got = pay[:plan.payload_bytes].cpu().numpy()
    if not np.array_equal(got, ref):
        diff = np.nonzero(got != ref)[0]
        raise AssertionError(f"bits={bits} k={k}: payload differs at {diff.size} bytes, first at {diff[:8]}")
    assert_f32_close(e.cpu().numpy(), e_ref, f"bits={bits} k={k} e")
    assert sl.sl_payload_validate(plan, pay, ws)
    # the same list again with the list-length knob of the code kernel at zero (at 2 bits: a lane per chunk
    # instead of a wave per chunk)
    sl.sl_plan_set_codes_wave_below(plan, 0)
    e2 = torch.from_numpy(e0.copy()).cuda()
    pay2 = sl.alloc_payload(plan)
    pay2.fill_(0x5A)
    sl.sl_compress(plan, e2, torch.from_numpy(delta).cuda(), 0.95, pay2, ws)
    torch.cuda.synchronize()
    assert np.array_equal(pay2[:plan.payload_bytes].cpu().numpy(), ref), f"bits={bits} k={k}: the other route differs"
    assert torch.equal(e2.view(torch.int32), e.view(torch.int32))
    sl.sl_plan_set_codes_wave_below(plan, 32768)
    # the index coder at this width: the oracle's coded bytes, and back
    ref_enc = oracle.rice_encode_b(descs, k, bits, ref)
    cap = sl.sl_rice_max_bytes(plan)
    assert cap == oracle.rice_max_bytes_b(descs, k, bits) >= ref_enc.size
    out = torch.full((cap,), 0xCD, dtype=torch.uint8, device="cuda")
    sl.sl_rice_encode(plan, pay, out, ws)
    torch.cuda.synchronize()
    coded = out.cpu().numpy()
    size = int(coded[8:16].view(np.uint64)[0])
    assert size == ref_enc.size and np.array_equal(coded[:size], ref_enc)
    back = torch.full((max(16, plan.payload_bytes),), 0xEE, dtype=torch.uint8, device="cuda")
    sl.sl_rice_decode(plan, out, size, back)
    torch.cuda.synchronize()
    assert np.array_equal(back[:plan.payload_bytes].cpu().numpy(), ref)
    plan.close()


@pytest.mark.parametrize("bits", WIDTHS)
def test_ef_frozen(sl, oracle, bits):
    descs, n = layout_list([(140, 200, TILE), (1, 9000, FLAT)])
    rng = np.random.default_rng(1100 + bits)
    e0 = rng.normal(0, 1e-3, n).astype(np.float32)
    delta = rng.normal(0, 1e-3, n).astype(np.float32)
    plan = sl.sl_plan_create_bits(descs, 32, bits)
    e = torch.from_numpy(e0.copy()).cuda()
    pay = sl.alloc_payload(plan)
    sl.sl_compress(plan, e, torch.from_numpy(delta).cuda(), 0.95, pay, sl.alloc_workspace(plan),
                   flags=sl.SL_COMPRESS_EF_FROZEN)
    torch.cuda.synchronize()
    ref = oracle.compress_b(descs, 32, bits, e0.copy(), delta, 0.95, ef_frozen=True)
    assert np.array_equal(pay[:plan.payload_bytes].cpu().numpy(), ref)
    assert np.array_equal(e.cpu().numpy().view(np.uint32), e0.view(np.uint32))


@pytest.mark.parametrize("bits", (1, 3, 4, 32))
@pytest.mark.parametrize("k", [8, 64, 128, 512])
def test_deferred_residual_chain(sl, oracle, bits, k):
    run_deferred_chain(sl, oracle, bits, k)


# Large records reach the accumulate kernel through LDS as whole words (k a multiple of 8, record a
# multiple of 4 bytes, at most 8 KB); 264, 520 and 1032 fall outside that at some widths, 2048 and
# 4096 are more than the words fetched ahead, and fp32 values at k = 2048 are too large to stage.
@pytest.mark.parametrize("bits", WIDTHS)
@pytest.mark.parametrize("k", [256, 264, 520, 1024, 1032, 2048, 4096])
def test_deferred_residual_chain_high_density(sl, oracle, bits, k):
    run_deferred_chain(sl, oracle, bits, k)


def run_deferred_chain(sl, oracle, bits, k):
    if k <= 256:
        shapes = [(150, 210, TILE), (1, 9000, FLAT), (1024, 16, TILE), (128, 192, TILE), (1, 4096 + 1030, FLAT)]
    elif k <= 1000:
        shapes = [(160, 224, TILE), (1024, 16, TILE), (1, 8192 + 1000, FLAT)]
    elif k <= 2048:
        shapes = [(128, 192, TILE), (1, 8192 + 2100, FLAT)]
    else:
        shapes = [(128, 128, TILE), (1, 8192, FLAT)]
    descs, n = layout_list(shapes)
    rng = np.random.default_rng(1200 + 10 * k + bits)
    plan = sl.sl_plan_create_bits(descs, k, bits)
    ws = sl.alloc_workspace(plan)
    e_ref = rng.normal(0, 1e-3, n).astype(np.float32)
    e = torch.from_numpy(e_ref.copy()).cuda()
    pays = [sl.alloc_payload(plan), sl.alloc_payload(plan)]
    pending = None
    for rnd in range(4):
        if rnd == 2:
            delta_h = np.zeros(n, dtype=np.float32)
            delta_h[::7] = 1e-3
        else:
            delta_h = (1e-3 * rng.standard_t(3, n)).astype(np.float32)
        out = pays[rnd % 2]
        out.fill_(0xAB)
        sl.sl_compress(plan, e, torch.from_numpy(delta_h).cuda(), 0.95, out, ws,
                       flags=sl.SL_COMPRESS_DEFER_RESIDUAL, pending=pending)
        torch.cuda.synchronize()
        ref = oracle.compress_b(descs, k, bits, e_ref, delta_h, 0.95)
        assert np.array_equal(out[:plan.payload_bytes].cpu().numpy(), ref), f"payload round {rnd}"
        e_chk = e.clone()
        sl.sl_residual_apply(plan, e_chk, out)
        torch.cuda.synchronize()
        assert_f32_close(e_chk.cpu().numpy(), e_ref, f"e round {rnd}")
        pending = out
    sl.sl_residual_apply(plan, e, pending)
    torch.cuda.synchronize()
    assert_f32_close(e.cpu().numpy(), e_ref, "e after the final flush")


@pytest.mark.parametrize("bits", (1, 3, 4, 32))
@pytest.mark.parametrize("R,k,lr", [(1, 32, 1.0), (5, 24, 0.6), (8, 64, 1.0), (16, 128, 0.8), (3, 1024, 0.7)])
def test_apply_matches_oracle(sl, oracle, bits, R, k, lr):
    run_apply_case(sl, oracle, bits, R, k, lr)


# From k = 256 a lane of the aggregate decodes eight entries at a time (word reads of the
# record); k = 264 and 328 give records that are not a whole number of words, R = 24 at k = 2048
# more records than are staged at once, R*k below and above the switch to two half-chunk passes.
@pytest.mark.parametrize("bits", WIDTHS)
@pytest.mark.parametrize("R,k,lr", [(2, 256, 1.0), (16, 256, 0.8), (2, 264, 0.9), (5, 328, 0.7), (8, 512, 1.0),
                                    (4, 1024, 0.6), (24, 2048, 0.5), (2, 4096, 1.0)])
def test_apply_high_density_matches_oracle(sl, oracle, bits, R, k, lr):
    run_apply_case(sl, oracle, bits, R, k, lr)


@pytest.mark.parametrize("bits", (2, 32))
@pytest.mark.parametrize("R,k", [(8, 64), (16, 128), (4, 512)])
def test_apply_keeps_subnormal_sums(sl, oracle, bits, R, k):
    """Payload values in the subnormal range (multiples of 2^-149): every partial sum of the
    aggregate, the average and the update of a zero theta are subnormal too, so a flush to zero
    anywhere on the way shows as a difference from the oracle."""
    shapes = [(128, 128, TILE), (1, 8192 + 1100, FLAT)]
    descs, n = layout_list(shapes)
    rng = np.random.default_rng(1700 + R + bits)
    plan = sl.sl_plan_create_bits(descs, k, bits)
    ws = sl.alloc_workspace(plan)
    dev, host = [], []
    for r in range(R):
        delta = (rng.integers(-4000, 4000, n) * 2.0**-149).astype(np.float32)
        e = torch.zeros(n, dtype=torch.float32, device="cuda")
        pay = sl.alloc_payload(plan)
        sl.sl_compress(plan, e, torch.from_numpy(delta).cuda(), 0.95, pay, ws)
        torch.cuda.synchronize()
        ref = oracle.compress_b(descs, k, bits, np.zeros(n, dtype=np.float32), delta, 0.95)
        assert np.array_equal(pay[:plan.payload_bytes].cpu().numpy(), ref)
        dev.append(pay)
        host.append(ref)
    theta = torch.zeros(n, dtype=torch.float32, device="cuda")
    sl.sl_decompress_avg_apply(plan, theta, dev, 1.0)
    torch.cuda.synchronize()
    want = np.zeros(n, dtype=np.float32)
    oracle.decompress_avg_apply_b(descs, k, bits, want, host, 1.0)
    got = theta.cpu().numpy()
    assert np.count_nonzero(want) > n // 100 and np.abs(want).max() < 2.0**-126   # the case is what it claims
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def run_apply_case(sl, oracle, bits, R, k, lr):
    shapes = [(150, 210, TILE), (1, 9000, FLAT), (128, 128, TILE), (1024, 16, TILE)] if k <= 256 \
        else [(160, 224, TILE), (1, 8192 + 1100, FLAT)] if k <= 1024 else [(128, 192, TILE), (1, 3 * 4096, FLAT)]
    descs, n = layout_list(shapes)
    rng = np.random.default_rng(1300 + 10 * R + bits)
    plan = sl.sl_plan_create_bits(descs, k, bits)
    ws = sl.alloc_workspace(plan)
    dev, host = [], []
    for r in range(R):
        delta = (1e-3 * rng.standard_t(3, n)).astype(np.float32)
        e = torch.zeros(n, dtype=torch.float32, device="cuda")
        pay = sl.alloc_payload(plan)
        sl.sl_compress(plan, e, torch.from_numpy(delta).cuda(), 0.95, pay, ws)
        torch.cuda.synchronize()
        ref = oracle.compress_b(descs, k, bits, np.zeros(n, dtype=np.float32), delta, 0.95)
        assert np.array_equal(pay[:plan.payload_bytes].cpu().numpy(), ref)
        dev.append(pay)
        host.append(ref)
    theta0 = rng.normal(0, 0.02, n).astype(np.float32)
    theta = torch.from_numpy(theta0).cuda()
    sl.sl_decompress_avg_apply(plan, theta, dev, lr)
    torch.cuda.synchronize()
    want = theta0.copy()
    oracle.decompress_avg_apply_b(descs, k, bits, want, host, lr)
    assert_f32_close(theta.cpu().numpy(), want, f"theta bits={bits} R={R}")


@pytest.mark.parametrize("bits", WIDTHS)
@pytest.mark.parametrize("k", [8, 64, 104, 4096])
def test_pack_indices_bits(sl, oracle, bits, k):
    rng = np.random.default_rng(1400 + bits + k)
    nc = 29
    idx = np.stack([np.sort(rng.choice(4096, k, replace=False)) for _ in range(nc)]).astype(np.uint16)
    rec = oracle.record_bytes_b(k, bits)
    out = torch.full((nc * rec,), 0xCD, dtype=torch.uint8, device="cuda")
    idx_dev = torch.from_numpy(idx.view(np.int16)).cuda().view(torch.uint16)
    if bits == 32:
        sent = rng.normal(0, 1, (nc, k)).astype(np.float32)
        sl.sl_pack_indices_bits(idx_dev, None, torch.from_numpy(sent).cuda(), nc, k, bits, out)
    else:
        sent = rng.integers(0, 1 << bits, (nc, k)).astype(np.uint8)
        sl.sl_pack_indices_bits(idx_dev, torch.from_numpy(sent).cuda(), None, nc, k, bits, out)
    torch.cuda.synchronize()
    want = np.concatenate([oracle.pack_record_b(i, s, bits) for i, s in zip(idx, sent)])
    assert np.array_equal(out.cpu().numpy(), want)


def test_argument_errors(sl):
    for k, bits in ((64, 0), (64, 5), (64, 8), (64, 16), (12, 3), (4, 1), (20, 32)):
        with pytest.raises(sl.SparseLoCoError):
            sl.sl_plan_create_bits([(64, 64, 0, TILE)], k, bits)
    plan = sl.sl_plan_create_bits([(64, 64, 0, TILE)], 12, 2)      # a multiple of 4 is enough at 2 bits
    assert plan.value_bits == 2 and sl.sl_rice_max_bytes(plan) > 0
    plan = sl.sl_plan_create_bits([(64, 64, 0, TILE)], 16, 3)
    assert plan.value_bits == 3 and sl.sl_rice_max_bytes(plan) > 0


# --------------------------------------------------------------------------- Random-k ablation
@pytest.mark.parametrize("bits", (2, 3, 32))
@pytest.mark.parametrize("k", [8, 64, 512])
def test_random_k_matches_oracle(sl, oracle, bits, k):
    """sl_compress_random_k: the oracle's payload bytes and error buffer, over two rounds (the
    second with the first round's update still pending), ragged tiles and tails included."""
    if k <= 256:
        shapes = [(150, 210, TILE), (1, 9000, FLAT), (1024, 16, TILE), (128, 192, TILE)]
    else:
        shapes = [(160, 224, TILE), (1, 8192 + 1000, FLAT)]
    descs, n = layout_list(shapes)
    rng = np.random.default_rng(1500 + k + bits)
    plan = sl.sl_plan_create_bits(descs, k, bits)
    ws = sl.alloc_workspace(plan)
    e_ref = rng.normal(0, 1e-3, n).astype(np.float32)
    e = torch.from_numpy(e_ref.copy()).cuda()
    pays = [sl.alloc_payload(plan), sl.alloc_payload(plan)]
    pending = None
    for rnd, seed in enumerate((0, 0xC0FFEE11)):
        delta = (1e-3 * rng.standard_t(3, n)).astype(np.float32)
        out = pays[rnd]
        out.fill_(0xAB)
        sl.sl_compress_random_k(plan, e, torch.from_numpy(delta).cuda(), 0.95, out, ws, seed,
                                flags=sl.SL_COMPRESS_DEFER_RESIDUAL, pending=pending)
        torch.cuda.synchronize()
        ref = oracle.compress_random_b(descs, k, bits, e_ref, delta, 0.95, seed)
        got = out[:plan.payload_bytes].cpu().numpy()
        assert np.array_equal(got, ref), f"round {rnd}: payload differs at {np.nonzero(got != ref)[0][:8]}"
        assert sl.sl_payload_validate(plan, out, ws)
        pending = out
    sl.sl_residual_apply(plan, e, pending)
    torch.cuda.synchronize()
    assert_f32_close(e.cpu().numpy(), e_ref, "e")
    # another seed gives another selection
    e2 = torch.zeros(n, dtype=torch.float32, device="cuda")
    d2 = torch.from_numpy(delta).cuda()
    a, b = sl.alloc_payload(plan), sl.alloc_payload(plan)
    sl.sl_compress_random_k(plan, e2, d2, 0.95, a, ws, 1)
    e2.zero_()
    sl.sl_compress_random_k(plan, e2, d2, 0.95, b, ws, 2)
    torch.cuda.synchronize()
    assert not torch.equal(a, b)
