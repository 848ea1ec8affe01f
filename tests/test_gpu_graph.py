"""The decode step under HIP graph capture: the library allocates nothing, never synchronises and
keeps the cache lengths on the device, so one captured csp_decode_step replays as successive
decode steps.  Every replay is checked bit for bit against the eager call sequence."""
import numpy as np
import pytest

import csp_workloads as W

pytestmark = pytest.mark.gpu

torch = None  # imported by the `gpu` fixture: runs that select no GPU test never load it


@pytest.fixture(scope="module")
def gpu():
    global torch
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2412_04652_amd as P
    P.load_library()
    return torch.device("cuda:0")


def test_decode_step_graph_replays_match_eager(gpu, oracle):
    import gpu_util as U
    steps = 5
    case = W.make_case("graph", dtype="bf16", H_q=8, H_kv=4, D=128, O=16, R=16, sel_group=2,
                       layouts=[[(0, 300), (1, 900), (0, 200)], [(0, 100), (1, 400), (0, 60)]], budgets=[600, 300],
                       seed=12, decode_steps=steps)
    dc = U.DeviceCase(case, decode_cap=steps)
    lay = dc.layer
    lay.prune(dc.q_win, dc.k, dc.v, dc.modality)
    torch.cuda.synchronize()
    k0, v0, len0 = lay.k_cache.clone(), lay.v_cache.clone(), lay.kv_len.clone()
    dq, dk, dv = (U.to_dev(a, case.dtype) for a in (case.dec_q, case.dec_k, case.dec_v))

    eager = []
    for t in range(steps):
        eager.append(lay.decode_step(dq[t], dk[t], dv[t]).clone())
    torch.cuda.synchronize()
    k1, v1, len1 = lay.k_cache.clone(), lay.v_cache.clone(), lay.kv_len.clone()
    # the eager sequence itself against the oracle (last step, two heads)
    kc, vc = U.from_dev_bits(k1, "bf16"), U.from_dev_bits(v1, "bf16")
    for b, hq in [(0, 0), (1, 7)]:
        n = int(len1[b, hq // 2])
        ref = oracle.decode(oracle.to_f64(case.dec_q[steps - 1, b, hq], "bf16"), oracle.to_f64(kc[b, hq // 2, :n], "bf16"),
                            oracle.to_f64(vc[b, hq // 2, :n], "bf16"), 1.0)
        U.assert_decode_close(eager[-1][b, hq].cpu().numpy(), ref, f"eager b{b} h{hq}")

    # back to the state after pruning; capture ONE step on static input buffers
    lay.k_cache.copy_(k0); lay.v_cache.copy_(v0); lay.kv_len.copy_(len0)
    sq, sk, sv = dq[0].clone(), dk[0].clone(), dv[0].clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):       # warm-up on the capture stream, then undo it
        lay.decode_step(sq, sk, sv)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    lay.k_cache.copy_(k0); lay.v_cache.copy_(v0); lay.kv_len.copy_(len0)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        lay.decode_step(sq, sk, sv)
    torch.cuda.synchronize()
    assert torch.equal(lay.kv_len, len0)            # capturing executes nothing
    for t in range(steps):
        sq.copy_(dq[t]); sk.copy_(dk[t]); sv.copy_(dv[t])
        graph.replay()
        torch.cuda.synchronize()                     # eager work and a sync between replays
        assert torch.equal(lay.out, eager[t]), f"replay {t} differs from the eager step"
        assert torch.equal(lay.kv_len, len0 + t + 1)
    # bit patterns: rows past the live length are uninitialised memory and may hold NaNs
    assert torch.equal(lay.k_cache.view(torch.int16), k1.view(torch.int16))
    assert torch.equal(lay.v_cache.view(torch.int16), v1.view(torch.int16))
