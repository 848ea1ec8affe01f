"""GPU parity on randomly drawn problem shapes (seeded): head counts and grouping, head dimension,
storage type, window and recent sizes, ragged batches, budgets from a tenth of the length to above
it, cross ratio, n of the scoring softmax.  Each case runs score -> select -> compact -> two decode
steps and is checked against the oracle problem by problem."""
import numpy as np
import pytest

import csp_workloads as W

pytestmark = pytest.mark.gpu

torch = None  # imported by the `gpu` fixture: runs that select no GPU test never load it


@pytest.fixture(scope="module")
def gpu():
    global torch
    torch = pytest.importorskip("torch")
    import test_gpu_parity
    test_gpu_parity.torch = torch   # _end_to_end lives there
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2412_04652_amd as P
    P.load_library()
    return torch.device("cuda:0")


def draw_case(seed: int):
    rng = np.random.default_rng(4000 + seed)
    dtype = "bf16" if rng.random() < 0.7 else "f32"
    D = int(rng.choice([64, 128]))
    H_kv = int(rng.integers(1, 5))
    G = int(rng.choice([1, 1, 2, 4, 7]))
    H_q = H_kv * G
    groups = [g for g in (G, 2 * G, H_q) if H_q % g == 0]
    sel_group = int(rng.choice(groups))
    O = int(rng.choice([1, 3, 8, 17, 32, 33, 64, 100, 128]))
    R = int(rng.choice([0, 1, 5, O, O, 2 * O, 150]))
    B = int(rng.integers(1, 5))
    layouts, budgets = [], []
    for _ in range(B):
        tail_mod = int(rng.random() < 0.25)                      # the window's modality (visual now and then)
        tail = O + int(rng.integers(0, 40))
        body = int(rng.integers(max(R - tail, 0) + 8, 2600))
        spans, left = [], body
        while left > 0:
            n = int(min(left, rng.integers(1, 700)))
            m = int(rng.random() < 0.6)
            if spans and spans[-1][0] == m:
                spans[-1] = (m, spans[-1][1] + n)
            else:
                spans.append((m, n))
            left -= n
        if spans and spans[-1][0] == tail_mod:
            spans[-1] = (tail_mod, spans[-1][1] + tail)
        else:
            spans.append((tail_mod, tail))
        L = body + tail
        T = int(L * rng.choice([0.1, 0.25, 0.5, 0.8, 1.0, 1.2]))
        layouts.append(spans)
        budgets.append(max(T, R, 1))
    return W.make_case(f"random{seed}", dtype=dtype, H_q=H_q, H_kv=H_kv, D=D, O=O, R=R, sel_group=sel_group,
                       cross_ratio=float(rng.choice([0.0, 0.2, 0.5, 0.5, 0.77, 1.0])),
                       n_score=float(rng.choice([0.0, 0.0, 1.0, 0.3])), layouts=layouts, budgets=budgets,
                       seed=seed, decode_steps=2)


@pytest.mark.parametrize("seed", range(24))
def test_random_shape_end_to_end(gpu, oracle, seed):
    import gpu_util as U
    from test_gpu_parity import _end_to_end
    case = draw_case(seed)
    print(f"[random] seed={seed} {case.dtype} D={case.D} H_q={case.H_q} H_kv={case.H_kv} group={case.sel_group} O={case.O} "
          f"R={case.R} lens={np.diff(case.cu_seqlens).tolist()} T={case.budget_T.tolist()} ratio={case.cross_ratio} "
          f"n={case.n_score}", flush=True)
    heads = [(b, s) for b in range(case.B) for s in range(case.H_q // case.sel_group)]
    _end_to_end(U, oracle, case, heads, 2)
