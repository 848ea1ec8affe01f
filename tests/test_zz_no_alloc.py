"""csp_decode_attn_static (the entry point for callers that cannot allocate device memory: the
split-KV partials live in a device array of the library) against csp_decode_attn, through the C
ABI: two calls in a row, the second on a smaller input, must each return what the workspace
entry point returns on the same inputs (the same kernels run: bit for bit), and what the oracle
says.  Collected last on purpose."""
import ctypes as C
import os
import sys

import numpy as np
import pytest

import csp_workloads as W

pytestmark = pytest.mark.gpu
HERE = os.path.dirname(os.path.abspath(__file__))


def test_decode_attn_static_matches_workspace_entry_point(oracle):
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2412_04652_amd as P
    from paper_2412_04652_amd import binding as B_
    sys.path.insert(0, HERE)
    import gpu_util as U
    lib = P.load_library()
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(5)
    # first call: 5 sequences, 14 query heads on 2 KV heads, up to 5000 cached keys; second call: smaller
    # in every size (fewer sequences and heads, shorter cache, other split of the key axis)
    for call, (Bn, H_q, H_kv, D, lens) in enumerate([(5, 14, 2, 128, [0, 1, 63, 5000, 1024]), (2, 4, 4, 128, [700, 257])]):
        print(f"[static] call {call}: B={Bn} H_q={H_q} H_kv={H_kv} D={D} lens={lens}", flush=True)
        cap, G = max(lens) + 3, H_q // H_kv
        kc = W.f32_to_bf16_bits(rng.standard_normal((Bn, H_kv, cap, D), dtype=np.float32))
        vc = W.f32_to_bf16_bits(rng.standard_normal((Bn, H_kv, cap, D), dtype=np.float32))
        q = W.f32_to_bf16_bits(rng.standard_normal((Bn, H_q, D), dtype=np.float32))
        kvl = np.array([[l + (h % 2 if l > 1 else 0) for h in range(H_kv)] for l in lens], np.int32)
        d_k, d_v, d_q = U.to_dev(kc, "bf16"), U.to_dev(vc, "bf16"), U.to_dev(q, "bf16")
        d_len = torch.from_numpy(kvl).to(dev)
        cu = list(range(Bn + 1))
        desc = B_.Desc(dtype="bf16", B=Bn, H_q=H_q, H_kv=H_kv, D=D, sel_group=G, window_O=1, recent_R=1, max_seqlen=1,
                       cu_seqlens_host=cu, budget_T_host=[cap] * Bn, cu_seqlens=torch.tensor(cu, dtype=torch.int32, device=dev),
                       budget_T=torch.tensor([cap] * Bn, dtype=torch.int32, device=dev),
                       k_strides=(D, D), v_strides=(D, D), n_decode=1.0)
        need = P.csp_decode_workspace_bytes(desc, cap)
        assert 0 < need <= P.csp_static_scratch_bytes()
        ws = torch.empty(need, dtype=torch.uint8, device=dev)
        out_ws = torch.full((Bn, H_q, D), float("nan"), dtype=torch.float32, device=dev)
        out_st = torch.full((Bn, H_q, D), float("nan"), dtype=torch.float32, device=dev)
        strides = (H_kv * cap * D, cap * D, D)
        stream = torch.cuda.current_stream().cuda_stream
        vp = lambda t: C.c_void_p(t.data_ptr())
        rc = lib.csp_decode_attn(desc.ref(), vp(d_q), vp(d_k), vp(d_v), strides[0], strides[1], strides[2], vp(d_len), cap,
                                 vp(out_ws), vp(ws), need, C.c_void_p(stream))
        assert rc == 0, P.csp_strerror(rc)
        rc = lib.csp_decode_attn_static(desc.ref(), vp(d_q), vp(d_k), vp(d_v), strides[0], strides[1], strides[2], vp(d_len),
                                        cap, vp(out_st), C.c_void_p(stream))
        assert rc == 0, P.csp_strerror(rc)
        torch.cuda.synchronize()
        assert torch.equal(out_ws, out_st), f"call {call}: static scratch and workspace entry points disagree"
        o = out_st.cpu().numpy()
        for b in range(Bn):
            for hq in range(H_q):
                T = int(kvl[b, hq // G])
                ref = oracle.decode(oracle.to_f64(q[b, hq], "bf16"), oracle.to_f64(kc[b, hq // G, :T], "bf16"),
                                    oracle.to_f64(vc[b, hq // G, :T], "bf16"), 1.0)
                U.assert_decode_close(o[b, hq], ref, f"static decode call{call} b{b} h{hq} T{T}")
    # a size beyond the library's scratch is refused, nothing is launched
    big = B_.Desc(dtype="bf16", B=64, H_q=64, H_kv=64, D=128, sel_group=1, window_O=1, recent_R=1, max_seqlen=1,
                  cu_seqlens_host=list(range(65)), budget_T_host=[1] * 64, cu_seqlens=0x1000, budget_T=0x1000,
                  k_strides=(128, 128), v_strides=(128, 128))
    assert P.csp_decode_workspace_bytes(big, 1 << 16) > P.csp_static_scratch_bytes()
    rc = lib.csp_decode_attn_static(big.ref(), C.c_void_p(16), C.c_void_p(16), C.c_void_p(16), 128, 128, 128, C.c_void_p(16),
                                    1 << 16, C.c_void_p(16), None)
    assert rc == -3, rc
