"""The CPU oracle under AddressSanitizer + UndefinedBehaviorSanitizer: a copy of
oracle/csp_oracle.c is compiled (host compiler, temporary directory) together with
tests/oracle_san_driver.c into an executable that calls every oracle function on
exact-size heap buffers; it must exit cleanly, report nothing, and return the
very bytes the ordinary build returns."""
import os
import struct
import subprocess

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)

CASES = [
    # L, O, R, D, T, causal, problems, n_score, n_decode, cross_ratio, window modality mix
    dict(L=96, O=16, R=16, D=8, T=40, causal=1, P=3, n_score=0.0, n_decode=1.0, ratio=0.5, mixed=False),
    dict(L=70, O=9, R=5, D=4, T=33, causal=1, P=2, n_score=1.0, n_decode=1.0, ratio=0.3, mixed=True),
    dict(L=40, O=8, R=8, D=4, T=40, causal=1, P=2, n_score=0.0, n_decode=0.0, ratio=0.5, mixed=False),   # identity
    dict(L=33, O=4, R=0, D=2, T=1, causal=0, P=1, n_score=2.5, n_decode=1.0, ratio=1.0, mixed=False),     # one key kept
]


@pytest.fixture(scope="module")
def san_exe(tmp_path_factory):
    d = tmp_path_factory.mktemp("san")
    exe = str(d / "oracle_san")
    # sanitizer runtimes linked statically: the executable does not depend on the order of preloaded libraries
    cmd = ["gcc", "-O1", "-g", "-std=c99", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-static-libubsan", "-fno-omit-frame-pointer", "-o", exe, os.path.join(HERE, "oracle_san_driver.c"),
           os.path.join(ROOT, "oracle", "csp_oracle.c"), "-lm"]
    subprocess.check_call(cmd)
    return exe


def _inputs(c, seed):
    rng = np.random.default_rng(seed)
    L, O, D, P = c["L"], c["O"], c["D"], c["P"]
    q = rng.standard_normal((P, O, D))
    k = rng.standard_normal((P, L, D))
    v = rng.standard_normal((P, L, D))
    mod = (rng.random((P, L)) < 0.6).astype(np.uint8)
    mod[:, L - O:] = 0
    if c["mixed"]:
        mod[:, L - O: L - O // 2] = 1
    return q, k, v, mod


@pytest.mark.parametrize("ci", range(len(CASES)))
def test_oracle_is_clean_under_asan_ubsan(san_exe, oracle, tmp_path, ci):
    c = CASES[ci]
    q, k, v, mod = _inputs(c, 100 + ci)
    L, O, R, D, T, P = c["L"], c["O"], c["R"], c["D"], c["T"], c["P"]
    fin, fout = str(tmp_path / "in.bin"), str(tmp_path / "out.bin")
    with open(fin, "wb") as f:
        f.write(struct.pack("<7i", L, O, R, D, T, c["causal"], P))
        f.write(struct.pack("<3d", c["n_score"], c["n_decode"], c["ratio"]))
        for p in range(P):
            f.write(q[p].tobytes()); f.write(k[p].tobytes()); f.write(v[p].tobytes()); f.write(mod[p].tobytes())
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="2")
    res = subprocess.run([san_exe, fin, fout], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, env=env, timeout=120)
    assert res.returncode == 0, res.stderr[-4000:]
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr, res.stderr[-4000:]
    raw = open(fout, "rb").read()
    off = 0

    def take(dtype, n):
        nonlocal off
        a = np.frombuffer(raw, dtype=dtype, count=n, offset=off)
        off += a.nbytes
        return a

    cap = min(T, L)
    kc_all = np.zeros((P, cap, D)); vc_all = np.zeros((P, cap, D))
    for p in range(P):
        a_s, a_c, rs = take(np.float64, L), take(np.float64, L), take(np.float64, O)
        kept = int(take(np.int32, 1)[0]); cnt = take(np.int32, 4); idx = take(np.int32, L); o = take(np.float64, D)
        r_s, r_c, r_rs = oracle.head_scores(q[p], k[p], mod[p], R, c["n_score"], bool(c["causal"]), want_row_sum=True)
        np.testing.assert_array_equal(a_s, r_s); np.testing.assert_array_equal(a_c, r_c); np.testing.assert_array_equal(rs, r_rs)
        r_idx, r_cnt = oracle.select(r_s, r_c, mod[p], O, R, T, c["ratio"])
        assert kept == len(r_idx) and idx[:kept].tolist() == r_idx.tolist() and (idx[kept:] == -1).all()
        assert cnt.tolist() == [r_cnt["kept"], r_cnt["K_s"], r_cnt["K_c"], r_cnt["both"]]
        kc, vc = oracle.gather(k[p], r_idx), oracle.gather(v[p], r_idx)
        np.testing.assert_array_equal(o, oracle.decode(q[p, 0], kc, vc, c["n_decode"]))
        kc_all[p, :kept] = kc; vc_all[p, :kept] = vc
    bs, bc = take(np.float64, P * L).reshape(P, L), take(np.float64, P * L).reshape(P, L)
    r_bs, r_bc = oracle.scores_batch(q, k, mod, R, c["n_score"], bool(c["causal"]))
    np.testing.assert_array_equal(bs, r_bs); np.testing.assert_array_equal(bc, r_bc)
    bo = take(np.float64, P * D).reshape(P, D)
    np.testing.assert_array_equal(bo, oracle.decode_batch(q[:, 0], kc_all, vc_all, c["n_decode"]))
    assert off == len(raw)
