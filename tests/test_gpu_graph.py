"""A worker-round (sl_compress + sl_decompress_avg_apply, or their coded counterparts) captured into a HIP graph:
the entry points allocate nothing, do not synchronise and enqueue kernels only, so a
caller may capture them to take the launch overhead out of small rounds.  Every replay
is checked against the same calls made eagerly, with eager work and synchronisations
between the replays."""
import numpy as np
import pytest
import torch

from test_gpu_parity import FLAT, TILE, layout_list, sl  # noqa: F401 (fixture)

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("wire", ["plain", "coded"])
def test_captured_round_replays_like_eager(sl, oracle, wire):
    descs, n = layout_list([(256, 320, TILE), (1, 9000, FLAT), (150, 210, TILE)])
    k, R, beta, lr = 64, 4, 0.95, 0.7
    rng = np.random.default_rng(3000)
    plan = sl.sl_plan_create(descs, k)
    ws = sl.alloc_workspace(plan)
    cap = sl.sl_rice_max_bytes(plan)
    others, other_wires, other_sizes = [], [], []
    for r in range(1, R):
        e = torch.zeros(n, dtype=torch.float32, device="cuda")
        pay, coded = sl.alloc_payload(plan), sl.alloc_coded(plan)
        sl.sl_compress_coded(plan, e, torch.from_numpy(rng.normal(0, 1e-3, n).astype(np.float32)).cuda(), beta, pay,
                             coded, ws)
        others.append(pay)
        other_wires.append(coded)
        other_sizes.append(sl.coded_size(coded))
    deltas = [rng.normal(0, 1e-3, n).astype(np.float32) for _ in range(4)]
    theta0 = rng.normal(0, 0.02, n).astype(np.float32)

    def state():
        return dict(e=torch.zeros(n, dtype=torch.float32, device="cuda"),
                    theta=torch.from_numpy(theta0.copy()).cuda(),
                    delta=torch.empty(n, dtype=torch.float32, device="cuda"),
                    pay=sl.alloc_payload(plan), coded=sl.alloc_coded(plan))

    def round_(s):
        if wire == "plain":
            sl.sl_compress(plan, s["e"], s["delta"], beta, s["pay"], ws)
            sl.sl_decompress_avg_apply(plan, s["theta"], [s["pay"]] + others, lr)
        else:
            # (the size of the worker's own coded payload is known on the device only: the buffer's capacity
            # is passed, the reader takes the size from the header)
            sl.sl_compress_coded(plan, s["e"], s["delta"], beta, s["pay"], s["coded"], ws)
            sl.sl_decompress_avg_apply_coded(plan, s["theta"], [s["coded"]] + other_wires, [cap] + other_sizes, lr)

    g_state, e_state = state(), state()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    g_state["delta"].copy_(torch.from_numpy(deltas[0]))
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            round_(g_state)
    torch.cuda.synchronize()
    # capture does not execute: the graph's buffers are still in their initial state
    for i, d in enumerate(deltas):
        g_state["delta"].copy_(torch.from_numpy(d))
        e_state["delta"].copy_(torch.from_numpy(d))
        graph.replay()
        round_(e_state)                                    # the program's own eager work between replays
        torch.cuda.synchronize()
        for key in ("e", "theta", "pay") + (("coded",) if wire == "coded" else ()):
            assert torch.equal(g_state[key], e_state[key]), f"replay {i}: {key} differs from the eager round"
    # and the eager chain is the oracle's
    e_ref, th_ref = np.zeros(n, dtype=np.float32), theta0.copy()
    other_host = [p[:plan.payload_bytes].cpu().numpy() for p in others]
    for d in deltas:
        ref = oracle.compress(descs, k, e_ref, d, beta)
        oracle.decompress_avg_apply(descs, k, th_ref, [ref] + other_host, lr)
    assert np.array_equal(g_state["theta"].cpu().numpy().view(np.uint32), th_ref.view(np.uint32))
    assert np.array_equal(g_state["e"].cpu().numpy().view(np.uint32), e_ref.view(np.uint32))
