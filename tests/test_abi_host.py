"""CPU-side checks of the C-ABI library: it loads, exports every declared symbol, and rejects
bad arguments on the host before anything is launched (no GPU needed for any of this)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2603_11243_amd", "libssd.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2603_11243_amd.build import build_library
        build_library(verbose=False)
    from paper_2603_11243_amd import binding
    return binding.load_library()


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "ssd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(\w+)\s*\([^;{]*\)\s*;", text)))


def test_every_declared_symbol_is_exported(lib):
    from paper_2603_11243_amd import binding
    names = _declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_host_side_argument_errors(lib):
    h = C.c_void_p()
    assert lib.ssd_create(C.byref(h), None, None, None) == 0
    i32 = lambda a: np.asarray(a, dtype=np.int32)
    cu = i32([0, 4])
    fake = C.c_void_p(0x1000)      # never dereferenced: every call below fails on the host first
    args = lambda **k: [h, k.get("logits", fake), k.get("dtype", 1), k.get("cu", cu).ctypes.data, k.get("B", 1),
                        k.get("V", 16), k.get("blank", 0), C.c_float(0.7), None, None, fake, fake, fake, fake]
    assert lib.ctc_gate(*args(logits=None)) == -1
    assert lib.ctc_gate(*args(B=0)) == -1
    assert lib.ctc_gate(*args(V=0)) == -1
    assert lib.ctc_gate(*args(blank=16)) == -1
    assert lib.ctc_gate(*args(dtype=7)) == -5
    assert lib.ctc_gate(*args(cu=i32([0, 0]))) == -1            # utterance without frames
    assert lib.ctc_gate(*args(cu=i32([1, 4]))) == -1
    assert lib.ctc_gate(*args()) == -3                          # no workspace set
    assert b"workspace" in lib.ssd_last_error(h)
    assert lib.ssd_set_workspace(h, C.c_void_p(0x1001), 1 << 20) == -1      # misaligned
    # a context without a model refuses the decoder calls
    assert lib.verify_forward(h, fake, cu.ctypes.data, fake, cu.ctypes.data, fake, cu.ctypes.data, 1, fake) == -1
    assert lib.accept_prefix(h, fake, fake, cu.ctypes.data, 1, C.c_float(0.1), fake, fake, fake, None) == -1
    assert lib.ssd_workspace_bytes(h, 1000, 0, 0, 4) >= 2 * 4000
    assert lib.ssd_workspace_bytes(h, -1, 0, 0, 4) == 0
    lib.ssd_destroy(h)


def test_create_rejects_bad_model(lib):
    from paper_2603_11243_amd.binding import ModelCfgC, WeightsC
    h = C.c_void_p()
    w = WeightsC()
    cfg = ModelCfgC(2, 256, 4, 4, 64, 1024, 4096, 1e-5, 10000.0, 1, 512)       # bf16 with head_dim 64
    assert lib.ssd_create(C.byref(h), C.byref(cfg), C.byref(w), None) == -2 and not h
    cfg = ModelCfgC(2, 256, 4, 3, 64, 1024, 4096, 1e-5, 10000.0, 0, 512)       # heads not divisible
    assert lib.ssd_create(C.byref(h), C.byref(cfg), C.byref(w), None) == -2
    cfg = ModelCfgC(2, 256, 4, 4, 64, 1024, 4096, 1e-5, 10000.0, 0, 512)       # fine shape, NULL weights
    assert lib.ssd_create(C.byref(h), C.byref(cfg), C.byref(w), None) == -1
    assert lib.ssd_create(C.byref(h), C.byref(cfg), None, None) == -1


def test_plan_batches_matches_oracle(lib):
    """The batch planner is host code: compared with the oracle here, no GPU involved."""
    from oracle import ssd_oracle as O
    from paper_2603_11243_amd.binding import plan_batches
    rng = np.random.default_rng(21)
    for padded in (False, True):
        for _ in range(100):
            n = int(rng.integers(1, 40))
            L = rng.integers(1, 800, size=n)
            budget = int(rng.integers(100, 5000))
            got = [list(map(int, b)) for b in plan_batches(L, budget, padded)]
            assert got == O.plan_batches(L, budget, padded)
    # the paper's budget on a corpus-like length mix (frames of 1-30 s utterances)
    L = np.rint(rng.uniform(1, 30, size=500) * 25).astype(np.int32)
    got = plan_batches(L, 50000, False)
    assert [list(map(int, b)) for b in got] == O.plan_batches(L, 50000, False)
    assert all(L[b].sum() <= 50000 for b in got) and sum(len(b) for b in got) == 500
    h = C.c_int32()
    assert lib.ssd_plan_batches(None, 3, 10, 0, None, None, C.byref(h)) == -1
    bad = np.array([3, 0, 2], dtype=np.int32); o = np.empty(3, np.int32); s = np.empty(4, np.int32)
    assert lib.ssd_plan_batches(bad.ctypes.data, 3, 10, 0, o.ctypes.data, s.ctypes.data, C.byref(h)) == -1


def test_bench_refuses_more_than_one_gpu_and_has_no_cpu_fallback():
    """bench.py is a one-GPU measurement of the HIP path: --gpus 2 exits with a message that says so, and
    on a machine without a GPU it stops instead of timing anything else."""
    import os
    import subprocess
    import sys
    bench = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "bench.py")
    r = subprocess.run([sys.executable, bench, "--gpus", "2"], capture_output=True, text=True, timeout=300)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
    import torch
    if not torch.cuda.is_available():
        r = subprocess.run([sys.executable, bench, "--steps", "1"], capture_output=True, text=True, timeout=300)
        assert r.returncode == 1 and "no CPU fallback" in r.stderr and r.stdout.strip() == ""


def test_noalloc_gate_rejects_bad_arguments_on_the_host(lib):
    """ctc_gate_noalloc: argument and size errors come back before anything touches a device."""
    fake = C.c_void_p(0x1000)
    err = C.create_string_buffer(200)
    call = lambda **k: lib.ctc_gate_noalloc(None, k.get("logits", fake), k.get("dtype", 1), fake, k.get("B", 2),
                                            k.get("n", 100), k.get("V", 16), k.get("blank", 0), C.c_float(0.7),
                                            fake, fake, fake, fake, err, len(err))
    assert call(logits=None) == -1
    assert call(B=0) == -1
    assert call(n=0) == -1
    assert call(V=0) == -1
    assert call(blank=16) == -1
    assert call(dtype=9) == -5
    from paper_2603_11243_amd import binding
    assert call(n=binding.NOALLOC_MAX_FRAMES + 1) == -2
    assert b"at most 262144" in err.value
    text = open(os.path.join(ROOT, "include", "ssd.h")).read()
    assert re.search(r"#define\s+SSD_NOALLOC_MAX_FRAMES\s+(\d+)", text).group(1) == str(binding.NOALLOC_MAX_FRAMES)
