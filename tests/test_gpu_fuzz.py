"""Seeded random configurations of the whole path against the oracle: random tensor lists
(odd column counts, single-row and single-column matrices, tiny and multi-chunk tensors,
gaps between tensors), random k, value width, worker count, EF decay and mode (eager,
deferred chain, frozen, Random-k, pseudo-gradient from parameters).  Every case is valid
input; payload bytes must be bit-exact, e and theta bit-identical or within 1e-6."""
import os

import numpy as np
import pytest
import torch

from test_gpu_parity import FLAT, TILE, assert_f32_close, sl  # noqa: F401 (fixture)

pytestmark = pytest.mark.gpu


def random_list(rng, k):
    """Tensors whose every chunk holds at least k elements."""
    descs, off = [], int(rng.integers(0, 4)) * 4
    for _ in range(int(rng.integers(1, 7))):
        kind = rng.integers(0, 5)
        if kind == 0:                                     # 1-D with a tail of at least k
            n = int(rng.integers(1, 4)) * 4096 + int(rng.integers(k, 4097))
            r, c, lay = 1, n, FLAT
        elif kind == 1:                                   # matrix, arbitrary columns (also not multiples of 4)
            side = int(np.ceil(np.sqrt(k)))
            r = 64 * int(rng.integers(0, 3)) + int(rng.integers(side, 65))
            c = 64 * int(rng.integers(0, 4)) + int(rng.integers(side, 65))
            lay = TILE
        elif kind == 2:                                   # narrow matrix: 16 or fewer columns
            c = int(rng.integers(1, 17))
            r = 64 * int(rng.integers(-(-k // (64 * c)) + 0, -(-k // (64 * c)) + 3)) if 64 * c >= k else 0
            if r == 0:
                r, c = 64 * (-(-k // c) // 64 + 1), c
            lay = TILE
            if min(64, r) * c < k or (r % 64 and (r % 64) * c < k):
                r = 64 * (r // 64 + 1)
                if 64 * c < k:
                    continue
        elif kind == 3:                                   # matrix cut into flat runs
            r, c, lay = int(rng.integers(40, 90)), int(rng.integers(90, 200)), FLAT
            if (r * c) % 4096 and (r * c) % 4096 < k:
                c += 64
            if (r * c) % 4096 and (r * c) % 4096 < k:
                continue
        else:                                             # exactly full tiles
            r, c, lay = 64 * int(rng.integers(1, 3)), 64 * int(rng.integers(1, 4)), TILE
        descs.append((r, c, off, lay))
        off += r * c + int(rng.integers(0, 6)) * 4
        off = (off + 3) // 4 * 4
    return descs, off + 8


# SL_FUZZ_CASES / SL_FUZZ_SEED: more cases, other seeds (the defaults are what the suite runs)
N_CASES = int(os.environ.get("SL_FUZZ_CASES", "200"))
SEED0 = int(os.environ.get("SL_FUZZ_SEED", "7000"))


@pytest.mark.parametrize("case", range(N_CASES))
def test_random_configuration(sl, oracle, case):
    rng = np.random.default_rng(SEED0 + case)
    coded = (case // 2) % 2 == 1      # every other pair of cases travels in the coded wire format
    bits = int(rng.choice([1, 2, 2, 2, 3, 4, 32]))
    k = int(rng.choice([4, 8, 12, 16, 32, 40, 64, 100, 128, 136, 160, 200, 248, 256, 320, 512, 520, 1024, 2048]))
    if bits != 2:
        k = max(8, k // 8 * 8)
    descs, n = [], 0
    while not descs:
        descs, n = random_list(rng, k)
    R = int(rng.choice([1, 2, 3, 4, 8, 13, 16, 33]))
    beta = float(rng.choice([0.0, 0.9, 0.95, 1.0]))
    lr = float(rng.choice([0.5, 0.7, 1.0]))
    mode = str(rng.choice(["eager", "deferred", "frozen", "random", "params"]))
    try:
        plan = sl.sl_plan_create_bits(descs, k, bits)
    except sl.SparseLoCoError:
        pytest.skip("generator produced a chunk smaller than k")   # the oracle rejects it as well
    assert plan.num_chunks == oracle.num_chunks(descs)
    if case % 2:      # short lists take the wave-per-chunk code kernel: every other case forces the other one
        sl.sl_plan_set_codes_wave_below(plan, 0)
    ws = sl.alloc_workspace(plan)
    theta0 = rng.normal(0, 0.02, n).astype(np.float32)
    theta = torch.from_numpy(theta0.copy()).cuda()
    theta_ref = theta0.copy()
    e = [torch.from_numpy(x).cuda() for x in (rng.normal(0, 1e-3, (R, n)).astype(np.float32))]
    e_ref = [x.cpu().numpy().copy() for x in e]
    pend = [None] * R
    for rnd in range(2):
        pays, refs, wires, sizes = [], [], [], []
        for r in range(R):
            heavy = rng.random() < 0.5
            delta = ((rng.standard_t(3, n) if heavy else rng.normal(0, 1, n)) * 1e-3).astype(np.float32)
            if rng.random() < 0.2:
                delta[rng.integers(0, n, n // 3)] = 0            # many exact zeros: ties
            out = sl.alloc_payload(plan)
            out.fill_(0xAB)
            d = torch.from_numpy(delta).cuda()
            wire = torch.full((sl.sl_rice_max_bytes(plan) + 32,), 0xCD, dtype=torch.uint8, device="cuda") if coded else None

            def compress(flags=0, pending=None):
                if coded:      # the same call, emitting the coded format next to the plain record
                    sl.sl_compress_coded(plan, e[r], d, beta, out, wire, ws, flags=flags, pending=pending)
                else:
                    sl.sl_compress(plan, e[r], d, beta, out, ws, flags=flags, pending=pending)
            emitted = coded and mode in ("eager", "deferred", "frozen")
            if mode == "eager":
                compress()
                ref = oracle.compress_b(descs, k, bits, e_ref[r], delta, beta)
            elif mode == "deferred":
                compress(flags=sl.SL_COMPRESS_DEFER_RESIDUAL, pending=pend[r])
                pend[r] = out
                ref = oracle.compress_b(descs, k, bits, e_ref[r], delta, beta)
            elif mode == "frozen":
                compress(flags=sl.SL_COMPRESS_EF_FROZEN)
                ref = oracle.compress_b(descs, k, bits, e_ref[r], delta, beta, ef_frozen=True)
            elif mode == "random":
                seed = int(rng.integers(0, 2**32))
                sl.sl_compress_random_k(plan, e[r], d, beta, out, ws, seed)
                ref = oracle.compress_random_b(descs, k, bits, e_ref[r], delta, beta, seed)
            else:
                outer = rng.normal(0, 0.02, n).astype(np.float32)
                local = (outer - delta).astype(np.float32)
                sl.sl_compress_params(plan, e[r], torch.from_numpy(outer).cuda(), torch.from_numpy(local).cuda(),
                                      beta, out, ws)
                ref = oracle.compress_b(descs, k, bits, e_ref[r], outer - local, beta)
            torch.cuda.synchronize()
            got = out[:plan.payload_bytes].cpu().numpy()
            assert np.array_equal(got, ref), (f"case {case} {mode} bits={bits} k={k} round {rnd} worker {r}: "
                                              f"payload differs at {np.nonzero(got != ref)[0][:6]}; {descs}")
            assert sl.sl_payload_validate(plan, out, ws)
            if coded:
                if not emitted:   # these modes have no coded variant: the payload is transcoded
                    sl.sl_rice_encode(plan, out, wire, ws)
                    torch.cuda.synchronize()
                want = oracle.rice_encode_b(descs, k, bits, ref)
                have = wire.cpu().numpy()
                assert int(have[8:16].view(np.uint64)[0]) == want.size, f"case {case} {mode}: coded size"
                assert np.array_equal(have[:want.size], want), (
                    f"case {case} {mode} bits={bits} k={k} round {rnd} worker {r}: coded bytes differ at "
                    f"{np.nonzero(have[:want.size] != want)[0][:6]}; {descs}")
                assert bool((have[want.size:] == 0xCD).all()), "bytes beyond the coded size were written"
                wires.append(wire)
                sizes.append(want.size)
            pays.append(out)
            refs.append(ref)
        if coded:
            sl.sl_decompress_avg_apply_coded(plan, theta, wires, sizes, lr)
        else:
            sl.sl_decompress_avg_apply(plan, theta, pays, lr)
        oracle.decompress_avg_apply_b(descs, k, bits, theta_ref, refs, lr)
        torch.cuda.synchronize()
        assert_f32_close(theta.cpu().numpy(), theta_ref, f"case {case} theta round {rnd}")
    for r in range(R):
        if pend[r] is not None:
            sl.sl_residual_apply(plan, e[r], pend[r])
    torch.cuda.synchronize()
    for r in range(R):
        assert_f32_close(e[r].cpu().numpy(), e_ref[r], f"case {case} {mode} e[{r}]")
    plan.close()
