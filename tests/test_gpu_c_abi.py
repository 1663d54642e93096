"""The boundary in its pure form: tests/c_abi/abi_check.c, a C11 program compiled with gcc, calls the
library with hipMalloc'ed buffers (no Python, no PyTorch in that process) and prints what it got;
this test regenerates its inputs and compares every printed value with the CPU oracle."""
import os
import subprocess

import numpy as np
import pytest

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))
BIN = os.path.join(HERE, "c_abi", "abi_check")


def _lcg_stream(count: int, seed: int = 20241016) -> np.ndarray:
    """The program's generator: state <- state * a + c (mod 2^64), output = state >> 33."""
    out = np.empty(count, np.uint32)
    state = seed
    mask = (1 << 64) - 1
    for i in range(count):
        state = (state * 6364136223846793005 + 1442695040888963407) & mask
        out[i] = state >> 33
    return out


def _inputs(N, K, M):
    r = _lcg_stream(N * K + M * K + K)
    w = (r[: N * K] % 3).astype(np.int8).reshape(N, K) - 1
    x = ((r[N * K: N * K + M * K] % 2001).astype(np.int32) - 1000).astype(np.float32) / np.float32(256.0)
    gamma = np.float32(0.5) + (r[N * K + M * K:] % 1024).astype(np.float32) / np.float32(1024.0)
    return w, x.reshape(M, K), gamma


def _parse(text):
    rec = {}
    for line in text.splitlines():
        name, _, rest = line.partition(" ")
        rec[name] = rest.split()
    return rec


def _ints(tokens):
    return np.array([int(t) for t in tokens], np.int64)


def _floats(tokens):
    return np.array([int(t, 16) for t in tokens], np.uint32).view(np.float32)


@pytest.mark.gpu
@pytest.mark.parametrize("N,K,M", [(200, 1000, 3), (130, 4160, 8), (64, 64, 1)])
def test_c_program_matches_oracle(N, K, M):
    assert os.path.exists(BIN), "tests/c_abi/abi_check is not built: run __graft_entry__.build()"
    r = subprocess.run([BIN, str(N), str(K), str(M)], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]
    rec = _parse(r.stdout)
    assert rec["done"] == []
    w, x, gamma = _inputs(N, K, M)
    ref = oracle.bitlinear(x, w, np.float32(0.03125))
    Kp, Np = -(-K // 64) * 64, -(-N // 64) * 64
    assert _ints(rec["desc"]).tolist() == [N, K, Np, Kp, Np * Kp // 4]
    assert rec["roundtrip"] == ["1", "bad", "0"]
    q = _ints(rec["q"]).reshape(M, Kp)
    assert np.array_equal(q[:, :K], ref["q"])
    assert not q[:, K:].any()                      # the padding of every row is zero
    assert np.array_equal(_floats(rec["a_scale"]), ref["a_scale"])
    assert np.array_equal(_ints(rec["q_sum"]), ref["q_sum"])
    assert np.array_equal(_ints(rec["acc_gemv"]).reshape(M, N), ref["acc"])
    out = _floats(rec["out_gemv"]).reshape(M, N)
    assert np.all(np.abs(out - ref["out"]) <= 1e-6 * np.abs(ref["out"]))
    assert rec["gemm_equals_gemv"] == ["1", "1"]
    assert np.array_equal(_ints(rec["acc_fused"]), ref["acc"][0])
    assert rec["fused_pair_equal"] == ["1"]
    KC3 = -(-K // 72)
    assert _ints(rec["tl2_desc"]).tolist() == [72 * KC3, Np * KC3 * 16]
    assert rec["tl2_roundtrip"] == ["1"]
    assert np.array_equal(_ints(rec["acc_tl2"]), ref["acc"][0])
    assert rec["tl2_equals_gemv"] == ["1", "1"]
    assert rec["err_m_range"] == ["3"] and rec["err_null"] == ["1"]
    # the decoder block's norm, stand-alone: y against the fp64 formula, the codes against the oracle's quantizer on y
    from oracle import decoder as D
    y = _floats(rec["norm_y"])
    want_y = D.rmsnorm(x[0].astype(np.float64), gamma, 1e-5)
    assert np.all(np.abs(y - want_y) <= 3e-6 * np.abs(want_y).max())
    qn, an, sn = oracle.quant_act(y[None, :])
    got_q = _ints(rec["norm_q"])
    assert np.array_equal(got_q[:K], qn[0]) and not got_q[K:].any()
    assert np.array_equal(_floats(rec["norm_a_scale"]), an) and _ints(rec["norm_q_sum"]).tolist() == sn.tolist()
    assert rec["err_norm_null"] == ["1"]
    if K % 8 == 0:   # ... and folded into the product, on x' = x + x
        xp = x[0] + x[0]
        assert np.array_equal(_floats(rec["fold_h"]), xp)
        qz, az, _ = oracle.quant_act((xp * gamma)[None, :])
        acc = oracle.matmul_i32(qz, w)[0]
        assert np.array_equal(_ints(rec["fold_acc"]), acc)
        r64 = 1.0 / np.sqrt(np.mean(xp.astype(np.float64) ** 2) + 1e-5)
        a_got = _floats(rec["fold_a_scale"])
        assert abs(float(a_got[0]) - float(az[0]) * r64) <= 3e-6 * float(az[0]) * r64
        want = oracle.dequant(acc[None, :], np.float32(0.03125), a_got)[0]
        assert np.all(np.abs(_floats(rec["fold_out"]) - want) <= 1e-6 * np.abs(want))


def test_lcg_stream_is_the_documented_recurrence():
    # two steps by hand: (seed * a + c) mod 2^64, then again
    a, c, m = 6364136223846793005, 1442695040888963407, 1 << 64
    s1 = (20241016 * a + c) % m
    s2 = (s1 * a + c) % m
    assert _lcg_stream(2).tolist() == [s1 >> 33, s2 >> 33]


def test_c_program_links_and_loads_without_a_gpu():
    # with no arguments the program prints its usage and exits 1 before any GPU call; getting that
    # far means the dynamic loader resolved the library and every symbol the program uses
    assert os.path.exists(BIN), "tests/c_abi/abi_check is not built: run __graft_entry__.build()"
    r = subprocess.run([BIN], capture_output=True, text=True, timeout=60)
    assert r.returncode == 1 and "usage" in r.stderr
