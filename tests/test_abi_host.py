"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol include/csp.h declares, and rejects bad arguments before it
launches anything."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def P():
    import paper_2412_04652_amd as pkg
    if not os.path.exists(pkg.lib_path()):
        from paper_2412_04652_amd.build import build_lib
        build_lib()
    pkg.load_library()
    return pkg


def test_every_declared_symbol_is_exported(P):
    hdr = open(os.path.join(ROOT, "include", "csp.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(csp_[a-z_]+)\s*\(", hdr))
    assert declared == set(P.EXPORTED_SYMBOLS), declared ^ set(P.EXPORTED_SYMBOLS)
    lib = C.CDLL(P.lib_path())
    for name in declared:
        assert getattr(lib, name) is not None


def test_strerror_and_version(P):
    assert P.csp_strerror(0) == "ok"
    assert "invalid" in P.csp_strerror(-1)
    assert "workspace" in P.csp_strerror(-3)
    assert P.csp_version().startswith("csp-gfx950")


def _desc(P, **kw):
    base = dict(dtype="bf16", B=2, H_q=8, H_kv=8, D=128, sel_group=1, window_O=64, recent_R=64, max_seqlen=4096,
                cu_seqlens_host=[0, 4096, 8192], budget_T_host=[2048, 2048], cu_seqlens=0x1000, budget_T=0x2000,
                k_strides=(128, 8192 * 128), v_strides=(128, 8192 * 128))
    base.update(kw)
    return P.Desc(**base)


def test_workspace_sizes(P):
    d = _desc(P)
    # 16 bytes of counters, then the statistics of whichever path needs more: two passes with chunks of
    # 128 keys at this size (2*8*32 chunks * 64 rows * 2 floats) against one float per (head, 512-key
    # chunk, row) of the single-read kernel
    assert P.csp_score_workspace_bytes(d) == 16 + 2 * 8 * 32 * 64 * 2 * 4
    # benchmark shape: the single-read statistics (32 chunks of 512 keys), its task table (a 64-byte
    # record per (sequence, head, window part, chunk), and one more) and the keys' modality as bits (a
    # word per 32 keys of every (sequence, selection group)) are more than the two-pass statistics
    # (4 chunks of 4096 keys, two floats each)
    L = 16384
    big = dict(B=4, H_q=32, H_kv=32, max_seqlen=L, cu_seqlens_host=[0, L, 2 * L, 3 * L, 4 * L], budget_T_host=[L // 2] * 4,
               k_strides=(128, 4 * L * 128), v_strides=(128, 4 * L * 128))
    table = (4 * 32 * 32 + 1) * 64
    bits = lambda groups: (4 * groups * 32 * 16 + 2) * 4
    assert P.csp_score_workspace_bytes(_desc(P, **big)) == 16 + 4 * 32 * 32 * 64 * 4 + table + bits(32)
    # all heads in one selection group: one score array pair per head on top of that
    assert P.csp_score_workspace_bytes(_desc(P, sel_group=32, **big)) == 16 + 4 * 32 * 32 * 64 * 4 + table + bits(1) + 2 * 32 * 4 * L * 4
    # a window of 128 rows is scored in two parts of 64: statistics and score arrays per part
    assert P.csp_score_workspace_bytes(_desc(P, window_O=128, recent_R=128, **big)) == 16 + 4 * 32 * 2 * 32 * 64 * 4 + (4 * 32 * 2 * 32 + 1) * 64 + bits(32) + 2 * 2 * 32 * 4 * L * 4
    # fp32 keeps the two passes
    assert P.csp_score_workspace_bytes(_desc(P, dtype="f32", **big)) == 16 + 4 * 32 * 4 * 64 * 2 * 4
    assert P.csp_select_workspace_bytes(d) == 0
    n = P.csp_decode_workspace_bytes(d, 2048 + 16)
    assert n % ((128 + 2) * 4 * 2 * 8) == 0 and n > 0


FAKE = 0x10000  # a 16-byte aligned non-null "device pointer"; never dereferenced: validation fails first


@pytest.mark.parametrize("kw,code", [
    (dict(D=96), -2),
    (dict(dtype=7), -2),
    (dict(H_q=8, H_kv=3), -1),
    (dict(sel_group=3), -1),
    (dict(H_q=8, H_kv=2, sel_group=2), -1),         # not a multiple of the GQA group (4)
    (dict(window_O=5000), -2),
    (dict(window_O=100, cu_seqlens_host=[0, 50, 8192]), -1),   # window longer than a sequence
    (dict(recent_R=5000), -1),
    (dict(cross_ratio=1.5), -1),
    (dict(n_score=-1.0), -1),
    (dict(cu_seqlens_host=[0, 5000, 8192]), -1),    # longer than max_seqlen
    (dict(k_strides=(100, 8192 * 128)), -1),        # rows would overlap
    (dict(k_strides=(132, 8192 * 132)), -1),        # rows not 16-byte aligned
    (dict(cu_seqlens=None), -1),
])
def test_score_rejects_bad_descriptors(P, kw, code):
    d = _desc(P, **kw)
    with pytest.raises(P.CspError) as e:
        P.load_library()  # noqa
        rc = P.load_library().csp_score(d.ref(), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 30, None)
        if rc != 0:
            raise P.CspError(rc, "csp_score")
    assert e.value.code == code


def test_null_pointers_and_workspace(P):
    L = P.load_library()
    d = _desc(P)
    assert L.csp_score(d.ref(), None, FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == -1
    assert L.csp_score(d.ref(), FAKE, FAKE, FAKE, FAKE, FAKE, None, 0, None) == -3
    assert L.csp_score(d.ref(), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 16, None) == -3
    assert L.csp_score(d.ref(), FAKE + 4, FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == -1   # misaligned q
    assert L.csp_score(None, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == -1
    assert L.csp_score_lse(d.ref(), FAKE, FAKE, FAKE, None, FAKE, FAKE, FAKE, 1 << 30, None) == -1
    assert L.csp_score_lse(d.ref(), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 16, None) == -3
    assert L.csp_select(d.ref(), FAKE, FAKE, FAKE, None, 2048, FAKE, None, 0, None) == -1
    assert L.csp_select(d.ref(), FAKE, FAKE, FAKE, FAKE, 100, FAKE, None, 0, None) == -1       # kept_cap < min(T, L)
    assert L.csp_compact(d.ref(), FAKE, FAKE, FAKE, 2048, FAKE, FAKE, None, 1, 1, 128, None, None) == -1
    assert L.csp_compact(d.ref(), FAKE, FAKE, FAKE, 2048, FAKE, FAKE, FAKE, 8 * 2064 * 128, 2064 * 128, 64, None, None) == -1
    assert L.csp_decode_attn(d.ref(), FAKE, FAKE, FAKE, 8 * 2064 * 128, 2064 * 128, 128, FAKE, 2064, FAKE, None, 0, None) == -3
    assert L.csp_decode_attn(d.ref(), FAKE, FAKE, FAKE, 8 * 2064 * 128, 2064 * 128, 128, FAKE, 0, FAKE, FAKE, 1 << 30, None) == -1
    assert L.csp_decode_step_phase(d.ref(), 3, FAKE, FAKE, FAKE, FAKE, FAKE, 8 * 2064 * 128, 2064 * 128, 128, 2064, FAKE, FAKE, FAKE, 1 << 30, None) == -1
    assert L.csp_decode_step(d.ref(), FAKE, None, FAKE, FAKE, FAKE, 8 * 2064 * 128, 2064 * 128, 128, 2064, FAKE, FAKE, FAKE, 1 << 30, None) == -1
    assert L.csp_append_kv(d.ref(), FAKE, FAKE, FAKE, FAKE, 8 * 2064 * 128, 2064 * 128, 128, 0, FAKE, None) == -1
    assert L.csp_probe_stream(None, None, 1 << 20, FAKE, None) == -1
    assert L.csp_probe_stream(FAKE, None, 1 << 20, None, None) == -1
    assert L.csp_probe_stream(FAKE, None, (1 << 20) + 8, FAKE, None) == -1                      # not a multiple of 16
    assert L.csp_probe_stream(FAKE, FAKE + 4, 1 << 20, FAKE, None) == -1                        # misaligned dst
    assert L.csp_probe_stream(FAKE, None, 0, FAKE, None) == -1


def test_budget_below_recent_is_rejected(P):
    L = P.load_library()
    d = _desc(P, budget_T_host=[32, 2048])          # T < R while L > T
    assert L.csp_select(d.ref(), FAKE, FAKE, FAKE, FAKE, 4096, FAKE, None, 0, None) == -1
    d = _desc(P, budget_T_host=[9000, 2048])        # T >= L: identity, fine as far as validation goes
    assert d.c.budget_T_host is not None


def test_reprune_validation(P):
    L = P.load_library()
    d = _desc(P)
    cap = 2048 + 64
    sb, sh, st = 8 * cap * 128, cap * 128, 128
    ws = P.csp_reprune_workspace_bytes(d, cap)
    # ordered window (2*8*64 rows of 256 bytes) + counters + softmax statistics per chunk; no slices for sel_group 1
    n_chunks = -(-cap // 128)
    assert ws == 2 * 8 * 64 * 256 + 16 + 2 * 8 * n_chunks * 64 * 2 * 4
    dg = _desc(P, H_q=32, H_kv=8, sel_group=4, B=1, cu_seqlens_host=[0, 4096], budget_T_host=[2048])
    assert P.csp_reprune_workspace_bytes(dg, cap) > 1 * 32 * 64 * 256 + 2 * 4 * 1 * 8 * cap * 4   # slices of the group

    def call(desc=d, ring=FAKE, start=0, k=FAKE, s_tok=st, mod=FAKE, kept_cap=2048, wsp=FAKE, wsb=1 << 30):
        return L.csp_reprune(desc.ref(), ring, start, k, FAKE, sb, sh, s_tok, cap, mod, FAKE, FAKE, FAKE, FAKE, kept_cap,
                             FAKE, wsp, wsb, None)

    assert call(ring=None) == -1
    assert call(mod=None) == -1
    assert call(start=64) == -1 and call(start=-1) == -1
    assert call(k=FAKE + 8) == -1
    assert call(s_tok=100) == -1
    assert call(kept_cap=2047) == -1                                   # below a budget
    assert call(desc=_desc(P, budget_T_host=[32, 2048])) == -1          # budget below the window
    assert call(desc=_desc(P, budget_T=None)) == -1
    assert call(wsp=None) == -3 and call(wsb=ws - 1) == -3
    assert call(desc=_desc(P, window_O=200, recent_R=64)) == -2
    # companions
    assert L.csp_window_push(d.ref(), FAKE, FAKE, 64, None) == -1
    assert L.csp_window_push(d.ref(), None, FAKE, 0, None) == -1
    assert L.csp_gather_modality(d.ref(), FAKE, FAKE, 2048, FAKE, None, cap, None) == -1
    assert L.csp_gather_modality(d.ref(), FAKE, FAKE, 0, FAKE, FAKE, cap, None) == -1


def test_binding_fails_loudly_without_library(monkeypatch, P):
    import paper_2412_04652_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "_LIB_PATH", "/nonexistent/libcsp.so")
    with pytest.raises(RuntimeError):
        b.load_library()


def test_one_hip_runtime_in_the_process(P):
    """libcsp.so must resolve against the HIP runtime torch ships (the owner of the streams and
    the device memory it is handed), not map the system runtime beside it: two runtimes in one
    process are what made finished test processes abort in their exit handlers."""
    import torch  # noqa: F401
    maps = open("/proc/self/maps").read()
    hip = set(re.findall(r"(/\S*libamdhip64[^\s]*)", maps))
    hsa = set(re.findall(r"(/\S*libhsa-runtime64[^\s]*)", maps))
    assert len(hip) == 1, hip
    assert len(hsa) == 1, hsa
