"""The hand-counted vector-memory waits of the prefill kernel's operand pipeline and of the decode kernel's activation
copy, checked without a GPU.

1. A host-side model (tests/ring_model/ring_check.cpp, plain C++) replays the kernels' per-thread issue order for every
   instantiation the library launches and every step count up to 48, with the constants of the header the kernels
   themselves use (csrc/bl_gemm_ring.hpp), under the ISA's rule "operations complete in issue order, vmcnt(n) = at most n
   outstanding": every LDS read of an activation tile must lie behind a barrier that followed the tile's completion,
   every overwrite of a stage behind a barrier that followed its last read -- whether the compiler keeps the dead weight
   loads of the loop's tail or removes them.  With the tail's count set to the main loop's (the kernel's earlier form)
   the model must fail: that is the mistake it is there to catch.
2. The model's premise -- which loads each step issues -- is checked against the compiler's output: the kernels are
   compiled to assembly for gfx950 and every barrier of the K loop must be preceded by the expected wait and by the
   expected number of global -> LDS requests and weight loads since the barrier before it.
"""
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2410_16144_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.fixture(scope="module")
def model(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("ring") / "ring_check")
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-Wall", "-Werror", "-I", CSRC,
                           os.path.join(ROOT, "tests", "ring_model", "ring_check.cpp"), "-o", exe])
    return exe


def test_model_accepts_the_kernels_wait_counts(model):
    r = subprocess.run([model], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout[-2000:]
    assert "0 failing cases" in r.stdout


def test_model_rejects_the_main_loop_count_in_the_tail(model):
    r = subprocess.run([model, "--old-tail"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 1
    n = int(re.search(r"(\d+) failing cases", r.stdout).group(1))
    assert n > 0


def _functions(asm_path):
    cur, out = None, {}
    with open(asm_path) as f:
        for line in f:
            m = re.match(r"^(_Z\S+):", line)
            if m:
                cur = m.group(1)
                out[cur] = []
            elif line.startswith(".Lfunc_end"):
                cur = None
            elif cur:
                out[cur].append(line.strip())
    return out


def _barriers(lines):
    """Per s_barrier: (vmcnt of the last wait since the previous barrier, global->LDS loads, 128-bit loads since it)."""
    seq, lds, w, wait = [], 0, 0, None
    for l in lines:
        if l.startswith("global_load_lds_dwordx4"):
            lds += 1
        elif l.startswith("global_load_dwordx4"):
            w += 1
        elif l.startswith("s_waitcnt"):
            m = re.search(r"vmcnt\((\d+)\)", l)
            if m:
                wait = int(m.group(1))
        elif l.startswith("s_barrier"):
            seq.append((wait, lds, w))
            lds, w, wait = 0, 0, None
    return seq


def _compile_to_asm(tmp, name, extra=()):
    out = str(tmp / (name + ".s"))
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-ffp-contract=off", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-Wno-unused-command-line-argument", *extra, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           "-S", "--cuda-device-only", "-o", out, os.path.join(CSRC, name)]
    subprocess.run(cmd, check=True, stderr=subprocess.DEVNULL, timeout=600)
    return out


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="needs hipcc")
def test_compiled_prefill_kernels_issue_what_the_model_assumes(tmp_path):
    fns = _functions(_compile_to_asm(tmp_path, "bl_gemm.hip"))
    seen = 0
    for name, lines in fns.items():
        m = re.search(r"gemm_(?:batch_)?kernelILi(\d)ELi(\d)ELi(\d)ELi(\d)E", name)
        if not m:
            continue
        seen += 1
        mb, h, wk, wn = (int(x) for x in m.groups())
        nt, lead = (h + 1) // 2, 4
        wr = 8 if nt == 1 else 4
        rq = -(-(wk * 2 * mb) // (wn * wk))          # requests per loader thread and step
        younger, younger_tail, prologue = (lead - 2) * (rq + nt), (lead - 2) * rq, (lead - 3) * rq
        seq = _barriers(lines)
        # prologue: the weight ring's first tiles and the first kLead requests, a wait that leaves kPrologueWait outstanding
        assert seq[0][1] == lead * rq and seq[0][2] == (wr - 1) * nt and seq[0][0] is not None and seq[0][0] <= prologue, (name, seq[0])
        main = [b for b in seq[1:] if b[0] == younger]
        tail = [b for b in seq[1:] if b[0] == younger_tail]
        assert len(main) == 8 and len(tail) == 7, (name, seq)
        for wait, lds, w in main:          # a step of the main loop: kRQ requests, at least the kNT weight loads
            assert lds == rq and w >= nt, (name, seq)
        for wait, lds, w in tail:          # a step of the tail: kRQ requests; its weight loads may be gone
            assert lds == rq, (name, seq)
    assert seen == 14                      # seven forms, single and batched


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="needs hipcc")
def test_compiled_decode_copy_waits_for_the_copy_only(tmp_path):
    fns = _functions(_compile_to_asm(tmp_path, "bl_gemv.hip", ("-mllvm", "-amdgpu-kernarg-preload-count=7")))
    seen = 0
    for name, lines in fns.items():
        # QMODE 1 (activations copied into LDS), either kind of weight load, not the publishing form (which issues
        # the copy last and waits for everything)
        if not re.search(r"decode_mfma_kernelILi\dELi1ELb\dELb\dELb0E", name):
            continue
        seen += 1
        first = _barriers(lines)[0]
        # the copy's requests, then exactly the 6 weight tiles of the first batch, and a wait that lets those 6 fly
        assert first[1] >= 1 and first[2] == 6 and first[0] == 6, (name, first)
    assert seen == 16
