"""Host-side checks of the C boundary that need no GPU: the library loads, exports every
declared symbol, rejects bad arguments before touching the device, and its scheduler
(host-only) agrees with the paper's example and with the oracle."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2601_11676_amd as H
from paper_2601_11676_amd import binding as B
from oracle import ref
from tests.util import read_golden

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    names = []
    for fn in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if fn.endswith(".h"):
            text = open(os.path.join(ROOT, "include", fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names += re.findall(r"\b(halo_[a-z_0-9]+)\s*\(", text)
    return sorted(set(names))


def test_library_exports_every_declared_symbol():
    lib = H.load_library()
    names = _declared_functions()
    assert {"halo_predict_scores", "halo_build_group_mask", "halo_group_sparse_ffn",
            "halo_ffn_forward", "halo_build_schedule", "halo_workspace_bytes"} <= set(names)
    for n in names:
        assert getattr(lib, n) is not None


def test_schedule_paper_example_and_oracle_agreement():
    g = read_golden("alg3_example.txt")
    pd = H.halo_build_schedule(g["n_groups"][0], g["plr"], g["ratios"])
    runs = {dev: [p + 1 for p in range(len(pd)) if pd[p] == dev] for dev in range(3)}
    assert runs == g["device"]
    rng = np.random.default_rng(1)
    for _ in range(200):
        n_dev = int(rng.integers(1, 9))
        n = int(rng.integers(0, 260))
        plr = rng.choice([0.0, 0.02, 0.05, 0.1, 0.2, 0.3], size=n_dev)
        rat = None
        if rng.random() < 0.5:
            rat = rng.random(n_dev) + 0.01
            rat /= rat.sum()
        assert np.array_equal(H.halo_build_schedule(n, plr, rat), ref.schedule(n, plr, rat))


def test_schedule_rejects_bad_arguments():
    for args in [(4, [0.1, float("nan")], None), (4, [0.1, 1.5], None), (-1, [0.1], None),
                 (4, [0.1, 0.2], [-1.0, 2.0])]:
        with pytest.raises(H.HaloError):
            H.halo_build_schedule(*args)


def test_status_strings():
    lib = H.load_library()
    seen = {lib.halo_status_string(c).decode() for c in range(-6, 1)}
    assert len(seen) == 7 and "ok" in seen


def test_workspace_bytes():
    s = H.Shape(4096, 11008, 128, 256, "bf16")
    a = H.halo_workspace_bytes(s, 1, 43)
    b = H.halo_workspace_bytes(s, 8, 43)
    assert 0 < a < b
    assert H.halo_workspace_bytes(H.Shape(4096, 11000, 128, 256, "bf16", n_groups=86), 1, 43) == 0
    assert H.halo_workspace_bytes(s, 1, 87) == 0
    # a workspace sized for T tokens serves every smaller call: the size never falls as T grows
    # (the number of group ranges in the prefill down projection does)
    sizes = [H.halo_workspace_bytes(s, T, 43) for T in range(1, 2200, 7)]
    assert all(b >= a > 0 for a, b in zip(sizes, sizes[1:]))
    assert H.halo_workspace_bytes(H.Shape(4090, 11008, 128, 256), 1, 4) == 0


def test_workspace_bytes_q4():
    # the bound for callers of the 4-bit entry points: the plain one, plus one block's weights as bf16 once
    # more than 16 tokens can run on the bf16 kernels; never smaller, never falling as T grows
    s = H.Shape(4096, 11008, 128, 256, "bf16")
    for T in (1, 2, 16):
        assert H.halo_workspace_bytes_q4(s, T, 43) == H.halo_workspace_bytes(s, T, 43)
    for T in (17, 64, 512, 2000):
        assert H.halo_workspace_bytes_q4(s, T, 43) == H.halo_workspace_bytes(s, T, 43) + 3 * 11008 * 4096 * 2
    sizes = [H.halo_workspace_bytes_q4(s, T, 43) for T in range(1, 2200, 7)]
    assert all(b >= a > 0 for a, b in zip(sizes, sizes[1:]))
    assert H.halo_workspace_bytes_q4(s, 1, 87) == 0 and H.halo_workspace_bytes_q4(s, -1, 4) == 0
    f = H.Shape(4096, 11008, 128, 256, "f32")                  # float32 activations: the plain path, no extra room
    assert H.halo_workspace_bytes_q4(f, 512, 43) == H.halo_workspace_bytes(f, 512, 43)


def test_entry_points_validate_before_any_gpu_work():
    lib = H.load_library()
    s = H.Shape(256, 1024, 128, 64, "f32")
    bad_dtype = H.Shape(256, 1024, 128, 64, "fp8")
    bad_shape = H.Shape(256, 1000, 128, 64, "f32", n_groups=8)
    one = C.c_void_p(0x1000)     # never dereferenced: validation fails first
    null = None
    st = C.c_void_p(0)
    f = lib.halo_predict_scores
    assert f(C.byref(bad_dtype.c), one, 1, one, one, one, one, 1 << 30, st) == -3
    assert f(C.byref(bad_shape.c), one, 1, one, one, one, one, 1 << 30, st) == -2
    assert f(C.byref(s.c), null, 1, one, one, one, one, 1 << 30, st) == -1
    assert f(C.byref(s.c), one, -1, one, one, one, one, 1 << 30, st) == -4
    assert f(C.byref(s.c), C.c_void_p(0x1001), 1, one, one, one, one, 1 << 30, st) == -4
    assert f(C.byref(s.c), one, 1, one, one, one, one, 16, st) == -5
    assert f(C.byref(s.c), one, 1, one, one, one, null, 1 << 30, st) == -5
    assert f(C.byref(s.c), one, 0, one, one, one, one, 0, st) == 0      # T == 0: no-op
    g = lib.halo_build_group_mask
    assert g(one, 1, 0, 0, one, 1, null, null, null, one, null, null, st) == -2
    assert g(one, 1, 8, 9, one, 1, null, null, null, one, null, null, st) == -4
    assert g(one, 1, 8, 4, one, 0, null, null, null, one, null, null, st) == -4
    assert g(one, 1, 8, 4, one, 1, null, null, null, null, null, null, st) == -1
    assert g(null, 1, 8, 4, one, 1, null, null, null, one, null, null, st) == -1
    ffn = lib.halo_group_sparse_ffn
    assert ffn(C.byref(s.c), one, 1, one, one, one, null, one, one, 1 << 30, st) == -1
    assert ffn(C.byref(s.c), one, 1, one, one, one, one, one, one, 8, st) == -5
    assert ffn(C.byref(bad_shape.c), one, 1, one, one, one, one, one, one, 1 << 30, st) == -2
    fw = lib.halo_ffn_forward
    args = [C.byref(s.c), one, one, 1, one, one, one, one, one, 4, one, 4, null, one,
            null, null, null, null, null, null, one, 1 << 30, st]
    for idx, val, code in [(9, 9, -4), (11, 0, -4), (13, null, -1), (20, null, -5), (21, 64, -5),
                           (10, null, -1)]:
        a = list(args)
        a[idx] = val
        assert fw(*a) == code, (idx, code)


def test_binding_refuses_host_tensors():
    import torch
    s = H.Shape(256, 1024, 128, 64, "f32")
    x = torch.zeros(1, 256)
    with pytest.raises(ValueError):
        H.halo_predict_scores(s, x, x, x, x, x)


def test_bench_refuses_more_than_one_gpu():
    # one GPU by design: the benchmark says so instead of starting ranks
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    p = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert p.returncode != 0
    assert "single-GPU" in p.stderr and p.stdout.strip() == ""


def test_prepared_records_in_its_own_thread_and_nests():
    # prepared() marshals a call once; while it records, other threads still reach the real library
    import threading
    seen = {}

    def inner():
        return H.halo_build_schedule(4, [0.0, 0.1])

    def outer():
        seen["nested"] = H.prepared(inner)           # a prepared() inside the recorded function
        return H.halo_build_schedule(6, [0.0, 0.1, 0.2])

    def other_thread():
        seen["other"] = H.halo_build_schedule(4, [0.0, 0.1]).tolist()

    def recorded():
        t = threading.Thread(target=other_thread)
        t.start()
        t.join()
        return outer()

    call = H.prepared(recorded)
    assert seen["other"] == [0, 0, 1, 1]                 # the real library answered the other thread
    call()
    seen["nested"]()
    assert H.halo_build_schedule(4, [0.0, 0.1]).tolist() == [0, 0, 1, 1]   # and this thread, afterwards
    with pytest.raises(RuntimeError):
        H.prepared(lambda: None)
