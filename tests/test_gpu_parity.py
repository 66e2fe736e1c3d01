"""GPU parity: the HIP path (through the C ABI) against the CPU oracle.

Bar: selected indices and payload bytes bit-exact; fp32 values (e, theta, LUT)
within 1e-6 relative - the tests first check bit-identity, which the pinned
operation order makes attainable, and report the relative error otherwise.
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


def gpu_compress(sl, plan, e_host, d_host, beta, flags=0):
    e = torch.from_numpy(e_host).cuda()
    d = torch.from_numpy(d_host).cuda()
    pay = sl.alloc_payload(plan)
    pay.fill_(0xAB)                      # every byte must be written by the library
    ws = sl.alloc_workspace(plan)
    sl.sl_compress(plan, e, d, beta, pay, ws, flags=flags)
    torch.cuda.synchronize()
    return e.cpu().numpy(), pay[:plan.payload_bytes].cpu().numpy(), pay


def check_compress(sl, oracle, descs, n, k, e0, delta, beta, flags=0, what="", wave_below=None):
    plan = sl.sl_plan_create(descs, k)
    if wave_below is not None:
        sl.sl_plan_set_codes_wave_below(plan, wave_below)
    assert plan.num_chunks == oracle.num_chunks(descs)
    assert plan.payload_bytes == oracle.payload_bytes(descs, k)
    e_gpu, pay_gpu, _ = gpu_compress(sl, plan, e0, delta, beta, flags)
    e_ref = e0.copy()
    pay_ref = oracle.compress(descs, k, e_ref, delta, beta, ef_frozen=bool(flags & 1))
    if not np.array_equal(pay_gpu, pay_ref):
        diff = np.nonzero(pay_gpu != pay_ref)[0]
        raise AssertionError(f"{what} k={k}: payload differs at {diff.size} bytes, first at {diff[:8]}")
    assert_f32_close(e_gpu, e_ref, f"{what} k={k} e")
    plan.close()
    return pay_ref, e_ref


# --------------------------------------------------------------------------- compress
@pytest.mark.parametrize("k,lane_codes", [(k, False) for k in (4, 8, 20, 32, 64, 128, 256, 512, 1000)] +
                         [(k, True) for k in (4, 8, 20, 32, 64, 128)])
def test_compress_small_list_all_k_paths(sl, oracle, k, lane_codes):
    """Several tiles, ragged edges in both directions, 16-column matrix, 1-D tails;
    k covers every pruning width, the byte-wise record writer and the unpruned path.
    Up to k = 128 the code kernel is chosen by the length of the list: both choices are run."""
    if k <= 256:      # smallest chunk: 22 x 18 = 396 elements
        shapes = [(150, 210, TILE), (1, 9000, FLAT), (1024, 16, TILE), (64, 64, TILE),
                  (1, 4096 + 1030, FLAT), (128, 192, TILE)]
        if k <= 32:   # smallest chunk: 6 x 6 = 36 elements
            shapes += [(140, 200, TILE), (70, 70, TILE)]
    else:             # smallest chunk: 1000 elements
        shapes = [(160, 224, TILE), (1024, 16, TILE), (1, 8192 + 1000, FLAT), (100, 133, FLAT)]
    descs, n = layout_list(shapes)
    rng = np.random.default_rng(100 + k)
    e0 = rng.normal(0, 1e-3, n).astype(np.float32)
    delta = rng.normal(0, 1e-3, n).astype(np.float32)
    check_compress(sl, oracle, descs, n, k, e0, delta, 0.95, what="small list", wave_below=0 if lane_codes else None)


def test_compress_dense_case_k_4096(sl, oracle):
    descs, n = layout_list([(64, 128, TILE), (1, 8192, FLAT)])
    rng = np.random.default_rng(7)
    e0 = rng.normal(0, 1e-3, n).astype(np.float32)
    delta = rng.normal(0, 1e-3, n).astype(np.float32)
    check_compress(sl, oracle, descs, n, 4096, e0, delta, 0.95, what="dense")


@pytest.mark.parametrize("k", [32, 64, 128, 256, 320, 512, 640])
def test_compress_ties_zeros_and_heavy_tails(sl, oracle, k):
    """Degenerate inputs: all-zero tensors (all ties), few distinct magnitudes, signed
    zeros, denormals, a heavy-tailed tensor, a tensor with one hot column."""
    shapes = [(128, 128, TILE), (128, 128, TILE), (128, 128, TILE), (1, 8192, FLAT), (128, 128, TILE),
              (128, 128, TILE), (1, 4096 + 700, FLAT)]
    descs, n = layout_list(shapes)
    rng = np.random.default_rng(200 + k)
    delta = np.zeros(n, dtype=np.float32)
    e0 = np.zeros(n, dtype=np.float32)
    o = [d[2] for d in descs]
    sz = [d[0] * d[1] for d in descs]
    # tensor 0: all zero.  tensor 1: few distinct magnitudes with both signs
    delta[o[1]:o[1] + sz[1]] = rng.choice([-3e-3, -1e-3, -0.0, 0.0, 1e-3, 3e-3], sz[1]).astype(np.float32)
    # tensor 2: fewer than k non-zeros per chunk
    t2 = np.zeros(sz[2], dtype=np.float32)
    t2[rng.choice(sz[2], 40, replace=False)] = rng.normal(0, 1e-3, 40)
    delta[o[2]:o[2] + sz[2]] = t2
    # tensor 3: denormals and tiny values
    delta[o[3]:o[3] + sz[3]] = (rng.integers(-200, 200, sz[3]) * 2.0**-149).astype(np.float32)
    # tensor 4: heavy tails
    delta[o[4]:o[4] + sz[4]] = (1e-3 * rng.standard_t(3, sz[4])).astype(np.float32)
    # tensor 5: one hot column on top of noise
    t5 = rng.normal(0, 1e-4, (128, 128)).astype(np.float32)
    t5[:, 37] += 1.0
    delta[o[5]:o[5] + sz[5]] = t5.ravel()
    # tensor 6: constant (every value ties)
    delta[o[6]:o[6] + sz[6]] = np.float32(2.5e-4)
    e0[o[4]:o[4] + sz[4]] = rng.normal(0, 1e-3, sz[4]).astype(np.float32)
    check_compress(sl, oracle, descs, n, k, e0, delta, 0.95, what="degenerate")


@pytest.mark.parametrize("k", [64, 512, 520, 1024, 2048, 3000])
def test_compress_ties_at_the_threshold(sl, oracle, k):
    """Ties exactly at the k-th largest magnitude, a few per chunk and with both signs, so that
    the lowest indices must win (the general route narrows the threshold to a short list of
    keys first and resolves the ties from it); magnitudes cut to a coarse grid, so that many
    keys coincide around the threshold; magnitudes from so narrow a band that they share all
    leading bits, which overflows that list."""
    shapes = [(128, 192, TILE), (1, 2 * 4096 + 4000, FLAT), (64, 64, TILE), (128, 128, TILE), (128, 64, TILE)]
    descs, n = layout_list(shapes)
    rng = np.random.default_rng(300 + k)
    e0 = np.zeros(n, dtype=np.float32)
    delta = rng.normal(0, 1e-3, n).astype(np.float32)
    # tensors 0-2: copy each chunk's k-th largest magnitude to positions that hold smaller ones
    for r, c, off, layout in descs[:3]:
        x = delta[off:off + r * c]
        if layout == TILE:
            t = x.reshape(r // 64, 64, c // 64, 64).transpose(0, 2, 1, 3).reshape(-1, 4096).copy()
        else:
            t = None
        chunks = t if t is not None else [x[i:i + 4096] for i in range(0, r * c, 4096)]
        for ch in chunks:
            if ch.size <= k:
                continue
            mag = np.abs(ch)
            order = np.argsort(-mag, kind="stable")
            thr = mag[order[k - 1]]
            below = order[k:]
            take = rng.choice(below, size=min(7, below.size), replace=False)
            ch[take] = thr * rng.choice([-1.0, 1.0], take.size).astype(np.float32)
        if t is not None:
            x[:] = t.reshape(r // 64, c // 64, 64, 64).transpose(0, 2, 1, 3).reshape(-1)
    # tensor 3: five mantissa bits only
    r, c, off, _ = descs[3]
    u = delta[off:off + r * c].view(np.uint32)
    u &= np.uint32(0xFFFC0000)
    # tensor 4: all magnitudes within 2^-12 of one another (relative)
    r, c, off, _ = descs[4]
    delta[off:off + r * c] = (1e-3 * (1.0 + rng.integers(0, 1500, r * c) * 2.0**-23)).astype(np.float32) * \
        rng.choice([-1.0, 1.0], r * c).astype(np.float32)
    check_compress(sl, oracle, descs, n, k, e0, delta, 0.0, what="threshold ties")


@pytest.mark.parametrize("beta", [0.0, 0.9, 0.999, 1.0])
def test_compress_other_ef_decays(sl, oracle, beta):
    """The EF decay values of the paper's ablation (0.9, 0.95, 0.999; 1 = plain error feedback;
    0 = no memory), two rounds so that the decay acts on a non-zero buffer."""
    descs, n = layout_list([(150, 210, TILE), (1, 9000, FLAT), (128, 192, TILE)])
    rng = np.random.default_rng(int(beta * 1000) + 11)
    e0 = rng.normal(0, 1e-3, n).astype(np.float32)
    for rnd in range(2):
        delta = rng.normal(0, 1e-3, n).astype(np.float32)
        _, e0 = check_compress(sl, oracle, descs, n, 64, e0, delta, beta, what=f"beta={beta} round {rnd}")


@pytest.mark.parametrize("k", [1024, 2048, 4088])
def test_compress_high_densities(sl, oracle, k):
    """Densities of 25 %, 50 % and almost everything (the paper sweeps densities up to 50 %)."""
    descs, n = layout_list([(128, 192, TILE), (1, 3 * 4096 + 4090, FLAT), (64, 64, TILE)])
    rng = np.random.default_rng(k)
    e0 = rng.normal(0, 1e-3, n).astype(np.float32)
    delta = (1e-3 * rng.standard_t(3, n)).astype(np.float32)
    check_compress(sl, oracle, descs, n, k, e0, delta, 0.95, what="high density")


def test_compress_ef_frozen(sl, oracle):
    descs, n = layout_list([(140, 200, TILE), (1, 9000, FLAT)])
    rng = np.random.default_rng(9)
    e0 = rng.normal(0, 1e-3, n).astype(np.float32)
    delta = rng.normal(0, 1e-3, n).astype(np.float32)
    _, e_ref = check_compress(sl, oracle, descs, n, 32, e0, delta, 0.95, flags=sl.SL_COMPRESS_EF_FROZEN,
                              what="frozen")
    assert np.array_equal(e_ref, e0)


def test_compress_is_deterministic_and_leaves_padding(sl, oracle):
    descs, n = layout_list([(200, 140, TILE), (1, 5000, FLAT), (64, 64, TILE)])
    n += 64
    rng = np.random.default_rng(10)
    e0 = rng.normal(0, 1e-3, n).astype(np.float32)
    delta = rng.normal(0, 1e-3, n).astype(np.float32)
    plan = sl.sl_plan_create(descs, 64)
    e1, p1, _ = gpu_compress(sl, plan, e0, delta, 0.95)
    e2, p2, _ = gpu_compress(sl, plan, e0, delta, 0.95)
    assert np.array_equal(p1, p2) and np.array_equal(e1.view(np.uint32), e2.view(np.uint32))
    inside = np.zeros(n, bool)
    for r, c, off, _ in descs:
        inside[off:off + r * c] = True
    assert np.array_equal(e1[~inside].view(np.uint32), e0[~inside].view(np.uint32))


# --------------------------------------------------------------------------- deferred residual
@pytest.mark.parametrize("k", [8, 32, 64, 128, 512])
def test_deferred_residual_chain_equals_eager(sl, oracle, k):
    """Rounds chained with SL_COMPRESS_DEFER_RESIDUAL + `pending`: every payload equals the
    oracle's, e minus the pending payload equals the oracle's e after every round
    (checked through sl_residual_apply on a copy), and a final sl_residual_apply
    leaves exactly the oracle's e."""
    if k <= 256:
        shapes = [(150, 210, TILE), (1, 9000, FLAT), (1024, 16, TILE), (128, 192, TILE), (1, 4096 + 1030, FLAT)]
    else:
        shapes = [(160, 224, TILE), (1024, 16, TILE), (1, 8192 + 1000, FLAT)]
    descs, n = layout_list(shapes)
    rng = np.random.default_rng(500 + k)
    plan = sl.sl_plan_create(descs, k)
    ws = sl.alloc_workspace(plan)
    e_ref = rng.normal(0, 1e-3, n).astype(np.float32)
    e = torch.from_numpy(e_ref.copy()).cuda()
    pays = [sl.alloc_payload(plan), sl.alloc_payload(plan)]
    pending = None
    for rnd in range(4):
        if rnd == 2:
            delta_h = np.zeros(n, dtype=np.float32)          # a round with ties everywhere
            delta_h[::7] = 1e-3
        else:
            delta_h = rng.normal(0, 1e-3, n).astype(np.float32)
        out = pays[rnd % 2]
        out.fill_(0xAB)
        sl.sl_compress(plan, e, torch.from_numpy(delta_h).cuda(), 0.95, out, ws,
                       flags=sl.SL_COMPRESS_DEFER_RESIDUAL, pending=pending)
        torch.cuda.synchronize()
        ref = oracle.compress(descs, k, e_ref, delta_h, 0.95)
        assert np.array_equal(out[:plan.payload_bytes].cpu().numpy(), ref), f"payload round {rnd}"
        e_chk = e.clone()
        sl.sl_residual_apply(plan, e_chk, out)
        torch.cuda.synchronize()
        assert_f32_close(e_chk.cpu().numpy(), e_ref, f"e round {rnd}")
        pending = out
    sl.sl_residual_apply(plan, e, pending)
    torch.cuda.synchronize()
    assert_f32_close(e.cpu().numpy(), e_ref, "e after the final flush")
    # an eager call may follow a deferred one: pending is consumed, nothing stays pending
    e2 = torch.from_numpy(e_ref.copy()).cuda()
    d1 = rng.normal(0, 1e-3, n).astype(np.float32)
    d2 = rng.normal(0, 1e-3, n).astype(np.float32)
    sl.sl_compress(plan, e2, torch.from_numpy(d1).cuda(), 0.95, pays[0], ws, flags=sl.SL_COMPRESS_DEFER_RESIDUAL)
    sl.sl_compress(plan, e2, torch.from_numpy(d2).cuda(), 0.95, pays[1], ws, pending=pays[0])
    torch.cuda.synchronize()
    oracle.compress(descs, k, e_ref, d1, 0.95)
    ref2 = oracle.compress(descs, k, e_ref, d2, 0.95)
    assert np.array_equal(pays[1][:plan.payload_bytes].cpu().numpy(), ref2)
    assert_f32_close(e2.cpu().numpy(), e_ref, "e after deferred then eager")


# --------------------------------------------------------------------------- aggregate
@pytest.mark.parametrize("R,k,lr", [(1, 32, 1.0), (3, 64, 0.7), (4, 64, 0.7), (8, 64, 1.0), (16, 32, 0.8),
                                     (5, 20, 0.6), (33, 128, 0.5)])
def test_apply_matches_oracle(sl, oracle, R, k, lr):
    shapes = [(150, 210, TILE), (1, 9000, FLAT), (128, 128, TILE), (1024, 16, TILE)]
    descs, n = layout_list(shapes)
    rng = np.random.default_rng(300 + R)
    plan = sl.sl_plan_create(descs, k)
    payloads_dev, payloads_host = [], []
    for r in range(R):
        e0 = np.zeros(n, dtype=np.float32)
        delta = rng.normal(0, 1e-3, n).astype(np.float32)
        _, pay_host, pay_dev = gpu_compress(sl, plan, e0, delta, 0.95)
        ref = oracle.compress(descs, k, e0.copy(), delta, 0.95)
        assert np.array_equal(pay_host, ref)
        payloads_dev.append(pay_dev)
        payloads_host.append(ref)
    theta0 = rng.normal(0, 0.02, n).astype(np.float32)
    theta = torch.from_numpy(theta0).cuda()
    sl.sl_decompress_avg_apply(plan, theta, payloads_dev, lr)
    torch.cuda.synchronize()
    want = theta0.copy()
    oracle.decompress_avg_apply(descs, k, want, payloads_host, lr)
    assert_f32_close(theta.cpu().numpy(), want, f"theta R={R}")


@pytest.mark.parametrize("k", [16, 32, 64, 128, 136, 160, 200, 248, 256])
def test_apply_every_worker_count_boundary(sl, oracle, k):
    """The aggregate fetches the first words of the records ahead of theta, stages the rest in rounds,
    and switches its decode route and the number of passes with R*k: worker counts on both sides of
    those switches (and the largest, 64), each checked against the oracle on the same payloads."""
    shapes = [(150, 210, TILE), (1, 9000, FLAT), (128, 128, TILE)]
    descs, n = layout_list(shapes)
    rng = np.random.default_rng(3300 + k)
    plan = sl.sl_plan_create(descs, k)
    dev, host = [], []
    for r in range(64):
        delta = (1e-3 * rng.standard_t(3, n)).astype(np.float32)
        _, pay_host, pay_dev = gpu_compress(sl, plan, np.zeros(n, dtype=np.float32), delta, 0.95)
        ref = oracle.compress(descs, k, np.zeros(n, dtype=np.float32), delta, 0.95)
        assert np.array_equal(pay_host, ref)
        dev.append(pay_dev)
        host.append(ref)
    theta0 = rng.normal(0, 0.02, n).astype(np.float32)
    for R in (1, 2, 5, 8, 9, 11, 12, 13, 16, 17, 23, 24, 25, 31, 32, 33, 47, 48, 49, 63, 64):
        theta = torch.from_numpy(theta0).cuda()
        sl.sl_decompress_avg_apply(plan, theta, dev[:R], 0.9)
        torch.cuda.synchronize()
        want = theta0.copy()
        oracle.decompress_avg_apply(descs, k, want, host[:R], 0.9)
        assert_f32_close(theta.cpu().numpy(), want, f"theta k={k} R={R}")


def test_apply_order_of_workers_is_r_ascending(sl, oracle):
    """Hand-made payloads: the fp32 sum at one coordinate depends on the order."""
    descs = [(1, 4096, 0, FLAT)]
    k = 4
    plan = sl.sl_plan_create(descs, k)
    vals = [1.0, 2.0**-24, 2.0**-24]
    host = []
    for v in vals:
        blk = np.zeros(oracle.payload_bytes(descs, k), dtype=np.uint8)
        blk[:16] = np.array([0, 0, v, 0], dtype=np.float32).view(np.uint8)
        blk[16:23] = oracle.pack_record([5, 6, 7, 8], [2, 1, 1, 1])
        host.append(blk)
    for order in (host, host[::-1]):
        dev = [torch.from_numpy(p).cuda() for p in order]
        theta = torch.zeros(4096, dtype=torch.float32, device="cuda")
        sl.sl_decompress_avg_apply(plan, theta, dev, 1.0)
        want = np.zeros(4096, dtype=np.float32)
        oracle.decompress_avg_apply(descs, k, want, order, 1.0)
        assert np.array_equal(theta.cpu().numpy().view(np.uint32), want.view(np.uint32))


# --------------------------------------------------------------------------- configuration 1, all rounds
def test_config1_three_rounds_four_workers(sl, oracle):
    from paper_2508_15706_amd import synth
    w = synth.workload(1)
    descs = [s.desc() for s in w.specs]
    n = w.arena
    plan = sl.sl_plan_create(descs, w.k)
    ws = sl.alloc_workspace(plan)
    e_dev = [torch.zeros(n, dtype=torch.float32, device="cuda") for _ in range(w.R)]
    e_ref = [np.zeros(n, dtype=np.float32) for _ in range(w.R)]
    theta = torch.empty(n, dtype=torch.float32, device="cuda")
    synth.fill_theta(w, theta)
    theta_ref = theta.cpu().numpy().copy()
    delta = torch.empty(n, dtype=torch.float32, device="cuda")
    pays = [sl.alloc_payload(plan) for _ in range(w.R)]
    for rnd in range(1, w.rounds + 1):
        ref_pays = []
        for r in range(w.R):
            synth.fill_delta(w, delta, rnd, r)
            sl.sl_compress(plan, e_dev[r], delta, w.beta, pays[r], ws)
            torch.cuda.synchronize()
            ref = oracle.compress(descs, w.k, e_ref[r], delta.cpu().numpy(), w.beta)
            assert np.array_equal(pays[r][:plan.payload_bytes].cpu().numpy(), ref), (rnd, r)
            assert_f32_close(e_dev[r].cpu().numpy(), e_ref[r], f"e round {rnd} worker {r}")
            ref_pays.append(ref)
        sl.sl_decompress_avg_apply(plan, theta, pays, w.lr)
        torch.cuda.synchronize()
        oracle.decompress_avg_apply(descs, w.k, theta_ref, ref_pays, w.lr)
        assert_f32_close(theta.cpu().numpy(), theta_ref, f"theta round {rnd}")


# --------------------------------------------------------------------------- record encoder
@pytest.mark.parametrize("shift", [0, 1, 2])
@pytest.mark.parametrize("k", [4, 16, 32, 48, 64, 100, 264, 1040, 4096])
def test_pack_indices(sl, oracle, k, shift):
    """Records of whole words take a word-wise encoder, the rest (and buffers that are not 4-byte
    aligned: shift != 0) a byte-wise one; the bytes are the same."""
    rng = np.random.default_rng(400 + k)
    nc = 37
    idx = np.stack([np.sort(rng.choice(4096, k, replace=False)) for _ in range(nc)]).astype(np.uint16)
    code = rng.integers(0, 4, (nc, k)).astype(np.uint8)
    rec = 7 * k // 4
    buf = torch.full((nc * rec + 16,), 0xCD, dtype=torch.uint8, device="cuda")
    out = buf[shift:shift + nc * rec]
    code_buf = torch.zeros(nc * k + 16, dtype=torch.uint8, device="cuda")
    code_dev = code_buf[shift:shift + nc * k]
    code_dev.copy_(torch.from_numpy(code.ravel()).cuda())
    idx_dev = torch.from_numpy(idx.view(np.int16)).cuda().view(torch.uint16)
    sl.sl_pack_indices(idx_dev, code_dev, nc, k, out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), oracle.pack_indices(idx.ravel(), code.ravel(), nc, k))
    host = buf.cpu().numpy()
    assert (host[:shift] == 0xCD).all() and (host[shift + nc * rec:] == 0xCD).all()   # nothing written outside


# --------------------------------------------------------------------------- argument errors
def test_argument_errors_are_reported_not_launched(sl):
    with pytest.raises(sl.SparseLoCoError):
        sl.sl_plan_create([(64, 64, 0, TILE)], 6)                 # k not a multiple of 4
    with pytest.raises(sl.SparseLoCoError):
        sl.sl_plan_create([(1, 100, 0, FLAT)], 128)               # chunk smaller than k
    with pytest.raises(sl.SparseLoCoError):
        sl.sl_plan_create([(64, 64, 2, TILE)], 32)                # offset not 16-byte aligned
    with pytest.raises(sl.SparseLoCoError):
        sl.sl_plan_create([(64, 64, 0, TILE), (64, 64, 4000, TILE)], 32)   # overlap
    plan = sl.sl_plan_create([(64, 64, 0, TILE)], 32)
    theta = torch.zeros(4096, dtype=torch.float32, device="cuda")
    pay = sl.alloc_payload(plan)
    with pytest.raises(sl.SparseLoCoError):
        sl.sl_decompress_avg_apply(plan, theta, [], 1.0)          # R = 0
    with pytest.raises(sl.SparseLoCoError):
        sl.sl_decompress_avg_apply(plan, theta, [pay] * 65, 1.0)  # R too large
    with pytest.raises(sl.SparseLoCoError):
        sl.sl_compress(plan, theta, theta, 0.95, pay, sl.alloc_workspace(plan))   # e aliases delta
    d = torch.zeros_like(theta)
    with pytest.raises(sl.SparseLoCoError):                       # pending is the output buffer
        sl.sl_compress(plan, theta, d, 0.95, pay, sl.alloc_workspace(plan), pending=pay)
    with pytest.raises(sl.SparseLoCoError):                       # frozen excludes a deferred residual
        sl.sl_compress(plan, theta, d, 0.95, pay, sl.alloc_workspace(plan),
                       flags=sl.SL_COMPRESS_EF_FROZEN | sl.SL_COMPRESS_DEFER_RESIDUAL)


# --------------------------------------------------------------------------- index coder
# --------------------------------------------------------------------------- pseudo-gradient formed on the fly
@pytest.mark.parametrize("k,flags", [(32, 0), (64, 0), (64, 1), (512, 0)])
def test_compress_params_equals_compress_of_the_difference(sl, oracle, k, flags):
    """delta = theta_outer - theta_local (one fp32 subtraction per element) inside the kernel:
    same payload and e as the oracle fed with the numpy difference."""
    shapes = [(150, 210, TILE), (1, 9000, FLAT), (128, 192, TILE)] if k <= 256 else [(160, 224, TILE), (1, 8192 + 1000, FLAT)]
    descs, n = layout_list(shapes)
    rng = np.random.default_rng(800 + k)
    theta_o = rng.normal(0, 0.02, n).astype(np.float32)
    theta_l = (theta_o - rng.normal(0, 1e-3, n)).astype(np.float32)
    e0 = rng.normal(0, 1e-3, n).astype(np.float32)
    delta = theta_o - theta_l                     # fp32 subtraction, rounded once
    assert delta.dtype == np.float32
    plan = sl.sl_plan_create(descs, k)
    ws = sl.alloc_workspace(plan)
    e = torch.from_numpy(e0.copy()).cuda()
    pay = sl.alloc_payload(plan)
    sl.sl_compress_params(plan, e, torch.from_numpy(theta_o).cuda(), torch.from_numpy(theta_l).cuda(), 0.95,
                          pay, ws, flags=flags)
    torch.cuda.synchronize()
    e_ref = e0.copy()
    ref = oracle.compress(descs, k, e_ref, delta, 0.95, ef_frozen=bool(flags & 1))
    assert np.array_equal(pay[:plan.payload_bytes].cpu().numpy(), ref)
    assert_f32_close(e.cpu().numpy(), e_ref, "e")


# --------------------------------------------------------------------------- payload check
def test_payload_validate_agrees_with_oracle(sl, oracle):
    """A compressed payload passes; one planted violation (descending pair, repeated position,
    position outside an edge chunk) anywhere in the buffer is reported, as by the oracle."""
    k = 32
    shapes = [(150, 210, TILE), (1, 4096 * 5 + 1100, FLAT), (70, 100, TILE)]
    descs, n = layout_list(shapes)
    rng = np.random.default_rng(900)
    plan = sl.sl_plan_create(descs, k)
    ws = sl.alloc_workspace(plan)
    _, pay_host, pay_dev = gpu_compress(sl, plan, rng.normal(0, 1e-3, n).astype(np.float32),
                                        rng.normal(0, 1e-3, n).astype(np.float32), 0.95)
    assert oracle.validate_payload(descs, k, pay_host)
    assert sl.sl_payload_validate(plan, pay_dev, ws)

    rec = oracle.record_bytes(k)
    offs, off = [], 0
    for d in descs:
        offs.append(off)
        off += oracle.tensor_block_bytes(d, k)
    nc0 = oracle.tensor_chunks(descs[0])
    cases = [
        (0, 0, lambda idx: idx[[1, 0] + list(range(2, k))]),                # first chunk, first pair swapped
        (0, nc0 - 1, lambda idx: np.r_[idx[:-1], idx[-2]]),                 # last chunk of tensor 0, repeat
        (0, nc0 - 1, lambda idx: np.r_[idx[:-1], 4095]),                    # corner tile 22 x 18: outside
        (1, 5, lambda idx: np.r_[idx[:-1], 1100]),                          # flat tail holds 1100 positions
        (2, 1, lambda idx: np.r_[idx[:-1], 63 * 64 + 36]),                  # 64 x 36 edge tile, column 36
        (2, 3, lambda idx: np.r_[idx[:-1], 6 * 64]),                        # 6 x 36 corner tile, row 6
    ]
    for ti, c, mutate in cases:
        bad = pay_host.copy()
        at = offs[ti] + 16 + c * rec
        idx, code = oracle.unpack_record(bad[at:at + rec], k)
        bad[at:at + rec] = oracle.pack_record(np.asarray(mutate(idx), dtype=np.uint16), code)
        assert not oracle.validate_payload(descs, k, bad), (ti, c)
        dev = sl.alloc_payload(plan)
        dev[:bad.size] = torch.from_numpy(bad).cuda()
        assert not sl.sl_payload_validate(plan, dev, ws), (ti, c)
    assert sl.sl_payload_validate(plan, pay_dev, ws)        # the flag is cleared per call
    plan.close()


# --------------------------------------------------------------------------- non-finite inputs, streams
def test_non_finite_inputs_are_handled_in_bounds_and_deterministically(sl, oracle):
    """NaN and infinities in the pseudo-gradient: behaviour is defined only as deterministic
    and memory-safe.  Selection works on integer keys (NaN > Inf > finite), so the selected
    positions still equal the oracle's; the payload is well formed and reproducible."""
    descs, n = layout_list([(150, 210, TILE), (1, 9000, FLAT), (128, 128, TILE)])
    k = 32
    rng = np.random.default_rng(77)
    e0 = rng.normal(0, 1e-3, n).astype(np.float32)
    delta = rng.normal(0, 1e-3, n).astype(np.float32)
    bad = rng.choice(n, 200, replace=False)
    delta[bad[:80]] = np.nan
    delta[bad[80:140]] = np.inf
    delta[bad[140:]] = -np.inf
    plan = sl.sl_plan_create(descs, k)
    ws = sl.alloc_workspace(plan)
    e1, p1, dev1 = gpu_compress(sl, plan, e0, delta, 0.95)
    e2, p2, _ = gpu_compress(sl, plan, e0, delta, 0.95)
    assert np.array_equal(p1, p2) and np.array_equal(e1.view(np.uint32), e2.view(np.uint32))
    assert sl.sl_payload_validate(plan, dev1, ws)
    _, det = oracle.compress(descs, k, e0.copy(), delta, 0.95, want_detail=True)
    rec, off, c0 = oracle.record_bytes(k), 0, 0
    for d in descs:
        for c in range(oracle.tensor_chunks(d)):
            at = off + 16 + c * rec
            idx, _ = oracle.unpack_record(p1[at:at + rec], k)
            assert np.array_equal(idx, det["idx"][(c0 + c) * k:(c0 + c + 1) * k]), (d, c)
        c0 += oracle.tensor_chunks(d)
        off += oracle.tensor_block_bytes(d, k)
    theta = torch.zeros(n, dtype=torch.float32, device="cuda")
    sl.sl_decompress_avg_apply(plan, theta, [dev1, dev1], 0.7)       # decodes without leaving the chunk
    torch.cuda.synchronize()


def test_two_streams_with_their_own_workspaces(sl, oracle):
    """One plan, two workers compressed concurrently on two streams (each with its own
    workspace, payload and error buffer): both results equal the oracle's."""
    descs, n = layout_list([(256, 320, TILE), (1, 9000, FLAT), (150, 210, TILE)])
    k = 64
    rng = np.random.default_rng(78)
    plan = sl.sl_plan_create(descs, k)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    hosts = [(rng.normal(0, 1e-3, n).astype(np.float32), rng.normal(0, 1e-3, n).astype(np.float32)) for _ in range(2)]
    devs = []
    for (e0, d0) in hosts:
        devs.append(dict(e=torch.from_numpy(e0.copy()).cuda(), d=torch.from_numpy(d0).cuda(),
                         pay=sl.alloc_payload(plan), ws=sl.alloc_workspace(plan)))
    torch.cuda.synchronize()
    for rep in range(3):
        for s, b in zip(streams, devs):
            sl.sl_compress(plan, b["e"], b["d"], 0.95, b["pay"], b["ws"], stream=s)
    torch.cuda.synchronize()
    for (e0, d0), b in zip(hosts, devs):
        e_ref = e0.copy()
        for rep in range(3):
            ref = oracle.compress(descs, k, e_ref, d0, 0.95)
        assert np.array_equal(b["pay"][:plan.payload_bytes].cpu().numpy(), ref)
        assert_f32_close(b["e"].cpu().numpy(), e_ref, "e")


# --------------------------------------------------------------------------- empty and tiny lists
def test_empty_list_and_single_partial_chunks(sl, oracle):
    plan = sl.sl_plan_create([], 64)
    assert plan.num_chunks == 0 and plan.num_elements == 0 and plan.payload_bytes == 0
    x = torch.full((64,), 3.0, dtype=torch.float32, device="cuda")
    y = torch.full((64,), 5.0, dtype=torch.float32, device="cuda")
    pay, ws = sl.alloc_payload(plan), sl.alloc_workspace(plan)
    pay.fill_(0xAB)
    sl.sl_compress(plan, x, y, 0.95, pay, ws)
    sl.sl_decompress_avg_apply(plan, x, [pay], 1.0)
    sl.sl_residual_apply(plan, x, pay)
    assert sl.sl_payload_validate(plan, pay, ws)
    torch.cuda.synchronize()
    assert bool((x == 3.0).all()) and bool((y == 5.0).all()) and bool((pay == 0xAB).all())
    plan.close()
    # lists whose only chunks are partial, with k equal or close to the number of elements
    for descs, k in (([(1, 100, 0, FLAT)], 64), ([(7, 9, 0, TILE)], 32), ([(1, 64, 0, FLAT), (3, 24, 64, TILE)], 64),
                     ([(1, 4097, 0, FLAT)], 1)):
        if k % 4:
            with pytest.raises(sl.SparseLoCoError):
                sl.sl_plan_create(descs, k)
            continue
        n = max(d[2] + d[0] * d[1] for d in descs) + 12
        rng = np.random.default_rng(len(descs) + k)
        e0 = rng.normal(0, 1e-3, n).astype(np.float32)
        delta = rng.normal(0, 1e-3, n).astype(np.float32)
        pay_ref, _ = check_compress(sl, oracle, descs, n, k, e0, delta, 0.95, what=f"tiny {descs}")
        plan = sl.sl_plan_create(descs, k)
        theta0 = rng.normal(0, 0.02, n).astype(np.float32)
        theta = torch.from_numpy(theta0).cuda()
        dev = sl.alloc_payload(plan)
        dev[:pay_ref.size] = torch.from_numpy(pay_ref).cuda()
        sl.sl_decompress_avg_apply(plan, theta, [dev, dev, dev], 0.7)
        torch.cuda.synchronize()
        want = theta0.copy()
        oracle.decompress_avg_apply(descs, k, want, [pay_ref] * 3, 0.7)
        assert_f32_close(theta.cpu().numpy(), want, f"tiny {descs} theta")
        plan.close()


# --------------------------------------------------------------------------- changing R, checkpoint / resume
def test_worker_count_may_change_every_round_and_state_survives_a_checkpoint(sl, oracle):
    """The number of contributing workers is a run-time argument (peers may come and go:
    the average divides by the R actually passed).  The only state of the path is (theta, e_r):
    five rounds in one go equal two rounds, a copy of the state out and back into fresh
    buffers (after the pending error update has been flushed), and three more rounds."""
    descs, n = layout_list([(150, 210, TILE), (1, 9000, FLAT), (128, 192, TILE)])
    k, beta, lr = 64, 0.95, 0.7
    Rs = [4, 2, 3, 1, 4]
    rng = np.random.default_rng(99)
    deltas = [[rng.normal(0, 1e-3, n).astype(np.float32) for _ in range(4)] for _ in Rs]
    theta0 = rng.normal(0, 0.02, n).astype(np.float32)
    plan = sl.sl_plan_create(descs, k)
    ws = sl.alloc_workspace(plan)

    def run(first, last, theta, e, pend):
        """Rounds first..last-1, every worker in deferred mode; returns the pending payloads."""
        for t in range(first, last):
            cur = []
            for r in range(Rs[t]):
                out = sl.alloc_payload(plan)
                sl.sl_compress(plan, e[r], torch.from_numpy(deltas[t][r]).cuda(), beta, out, ws,
                               flags=sl.SL_COMPRESS_DEFER_RESIDUAL, pending=pend[r])
                pend[r] = out
                cur.append(out)
            sl.sl_decompress_avg_apply(plan, theta, cur, lr)
        return pend

    def flush(e, pend):
        for r in range(4):
            if pend[r] is not None:
                sl.sl_residual_apply(plan, e[r], pend[r])
                pend[r] = None

    # straight through
    th_a = torch.from_numpy(theta0.copy()).cuda()
    e_a = [torch.zeros(n, dtype=torch.float32, device="cuda") for _ in range(4)]
    pend_a = run(0, 5, th_a, e_a, [None] * 4)
    flush(e_a, pend_a)
    # with a checkpoint after round 2
    th_b = torch.from_numpy(theta0.copy()).cuda()
    e_b = [torch.zeros(n, dtype=torch.float32, device="cuda") for _ in range(4)]
    pend_b = run(0, 2, th_b, e_b, [None] * 4)
    flush(e_b, pend_b)
    torch.cuda.synchronize()
    saved = (th_b.cpu().numpy().copy(), [x.cpu().numpy().copy() for x in e_b])
    del th_b, e_b
    th_c = torch.from_numpy(saved[0]).cuda()
    e_c = [torch.from_numpy(x).cuda() for x in saved[1]]
    pend_c = run(2, 5, th_c, e_c, [None] * 4)
    flush(e_c, pend_c)
    torch.cuda.synchronize()
    assert torch.equal(th_a, th_c) and all(torch.equal(x, y) for x, y in zip(e_a, e_c))
    # and both are the oracle's
    th_ref = theta0.copy()
    e_ref = [np.zeros(n, dtype=np.float32) for _ in range(4)]
    for t, R in enumerate(Rs):
        pays = [oracle.compress(descs, k, e_ref[r], deltas[t][r], beta) for r in range(R)]
        oracle.decompress_avg_apply(descs, k, th_ref, pays, lr)
    assert_f32_close(th_a.cpu().numpy(), th_ref, "theta after five rounds")
    for r in range(4):
        assert_f32_close(e_a[r].cpu().numpy(), e_ref[r], f"e[{r}] after five rounds")


# --------------------------------------------------------------------------- fragments of the list
def test_fragments_of_the_list_equal_the_whole(sl, oracle):
    """The appendix "Streaming SparseLoCo" synchronises the model in three fragments at staggered
    steps.  A fragment is a plan over a subset of the tensors in the same arenas: its payload is
    the concatenation of those tensors' blocks of the whole list's payload, its error update
    touches those tensors only, and aggregating fragment by fragment gives the whole update."""
    shapes = [(150, 210, TILE), (1, 768, FLAT), (128, 192, TILE), (1, 9000, FLAT), (256, 64, TILE), (1, 4096, FLAT)]
    descs, n = layout_list(shapes)
    frags = [descs[0:2], descs[2:4], descs[4:6]]
    k, R, lr = 32, 3, 0.7
    rng = np.random.default_rng(123)
    whole = sl.sl_plan_create(descs, k)
    plans = [sl.sl_plan_create(f, k) for f in frags]
    assert sum(p.payload_bytes for p in plans) == whole.payload_bytes
    ws = sl.alloc_workspace(whole)
    theta0 = rng.normal(0, 0.02, n).astype(np.float32)
    th_w, th_f = torch.from_numpy(theta0.copy()).cuda(), torch.from_numpy(theta0.copy()).cuda()
    pays_w, pays_f = [], [[] for _ in frags]
    for r in range(R):
        e0 = rng.normal(0, 1e-3, n).astype(np.float32)
        d0 = rng.normal(0, 1e-3, n).astype(np.float32)
        e_w, e_f, d = torch.from_numpy(e0.copy()).cuda(), torch.from_numpy(e0.copy()).cuda(), torch.from_numpy(d0).cuda()
        pw = sl.alloc_payload(whole)
        sl.sl_compress(whole, e_w, d, 0.95, pw, ws)
        pays_w.append(pw)
        parts = []
        for i, p in enumerate(plans):
            pf = sl.alloc_payload(p)
            sl.sl_compress(p, e_f, d, 0.95, pf, ws)
            torch.cuda.synchronize()
            pays_f[i].append(pf)
            parts.append(pf[:p.payload_bytes])
        torch.cuda.synchronize()
        assert torch.equal(torch.cat(parts), pw[:whole.payload_bytes]) and torch.equal(e_w, e_f)
    sl.sl_decompress_avg_apply(whole, th_w, pays_w, lr)
    for i, p in enumerate(plans):                      # one fragment at a time, as the streaming schedule would
        before = th_f.clone()
        sl.sl_decompress_avg_apply(p, th_f, pays_f[i], lr)
        torch.cuda.synchronize()
        changed = (before != th_f).cpu().numpy()
        lo, hi = frags[i][0][2], frags[i][-1][2] + frags[i][-1][0] * frags[i][-1][1]
        assert changed[lo:hi].any() and not changed[:lo].any() and not changed[hi:].any()
    torch.cuda.synchronize()
    assert torch.equal(th_w, th_f)
