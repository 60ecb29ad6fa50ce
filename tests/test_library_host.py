"""CPU-only checks of the C boundary: the library loads, exports what include/psgd.h declares,
builds tables bit-identical to the oracle's, and rejects bad arguments before touching a
device.  No kernel runs here."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import psgd_oracle as orc
from paper_2002_01119_amd import psgd

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    lib = psgd.load()
    with open(os.path.join(ROOT, "include", "psgd.h")) as f:
        text = re.sub(r"/\*.*?\*/", "", f.read(), flags=re.S)
    declared = sorted(set(re.findall(r"\b(psgd_[a-z0-9_]+)\s*\(", text)))
    assert len(declared) >= 15
    for name in declared:
        assert hasattr(lib, name), name
    assert sorted(psgd.EXPORTS) == declared
    assert psgd.version() >= 1
    assert psgd.MAX_N == 512 and psgd.DEG == 3


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 8, 16, 33, 64, 128, 512])
def test_tables_bit_identical_to_oracle(n):
    for topo in (psgd.TOPO_RING, psgd.TOPO_RAND_RING):
        for seed in (0, 1, 3001, 3005, 2 ** 63 + 5, 2 ** 64 - 1):
            for step in (0, 1, 7, 99, 2 ** 40 + 3):
                nbr, w = psgd.build_mixing(topo, n, seed, step)
                onbr, ow = orc.neighbour_table(topo, n, seed, step)
                assert nbr.dtype == np.int32 and w.dtype == np.float32
                assert np.array_equal(nbr, onbr), (topo, n, seed, step)
                assert np.array_equal(w.view(np.uint32), ow.view(np.uint32))


def test_tables_match_frozen_golden(golden_dir):
    with open(os.path.join(golden_dir, "mixing_tables.txt")) as f:
        lines = [l for l in f if l.strip() and not l.startswith("#")]
    for line in lines:
        head, rest = line.split(":")
        n, seed, step = (int(x) for x in head.split())
        nbr, _ = psgd.build_mixing(psgd.TOPO_RAND_RING, n, seed, step)
        assert [int(v) for v in nbr.reshape(-1)] == [int(x) for x in rest.split("|")[1].split()]


def test_tables_same_seed_same_ring_and_ring_ignores_seed():
    a = psgd.build_mixing(psgd.TOPO_RAND_RING, 64, 42, 5)[0]
    b = psgd.build_mixing(psgd.TOPO_RAND_RING, 64, 42, 5)[0]
    c = psgd.build_mixing(psgd.TOPO_RAND_RING, 64, 42, 6)[0]
    assert np.array_equal(a, b) and not np.array_equal(a, c)
    assert np.array_equal(psgd.build_mixing(psgd.TOPO_RING, 9, 1, 2)[0],
                          psgd.build_mixing(psgd.TOPO_RING, 9, 3, 4)[0])


def test_build_mixing_rejects_bad_arguments():
    lib = psgd.load()
    nbr = (ctypes.c_int32 * 12)()
    w = (ctypes.c_float * 12)()
    assert lib.psgd_build_mixing(0, 0, 0, 0, nbr, w) == psgd.EINVAL
    assert "n=0" in psgd.last_error()
    assert lib.psgd_build_mixing(0, psgd.MAX_N + 1, 0, 0, nbr, w) == psgd.EINVAL
    assert lib.psgd_build_mixing(7, 4, 0, 0, nbr, w) == psgd.EINVAL
    assert "topology" in psgd.last_error()
    assert lib.psgd_build_mixing(psgd.TOPO_FULL, 4, 0, 0, nbr, w) == psgd.EINVAL
    assert "psgd_mix_full" in psgd.last_error()
    assert lib.psgd_build_mixing(0, 4, 0, 0, None, w) == psgd.EINVAL
    assert lib.psgd_build_mixing(0, 4, 0, 0, nbr, None) == psgd.EINVAL
    assert lib.psgd_build_mixing(0, 4, 0, 0, nbr, w) == psgd.OK
    assert psgd.last_error() == ""
    with pytest.raises(psgd.PsgdError):
        psgd.build_mixing(psgd.TOPO_RING, 0)


def test_build_mixing_device_argument_checks():
    lib = psgd.load()
    A, B, S = 0x100000, 0x200000, 0x300000
    fn = lib.psgd_build_mixing_device
    assert fn(0, 0, 0, None, 0, 0, A, B, None) == psgd.EINVAL
    assert fn(0, psgd.MAX_N + 1, 0, None, 0, 0, A, B, None) == psgd.EINVAL
    assert fn(5, 4, 0, None, 0, 0, A, B, None) == psgd.EINVAL and "topology" in psgd.last_error()
    assert fn(psgd.TOPO_FULL, 4, 0, None, 0, 0, A, B, None) == psgd.EINVAL
    assert fn(1, 4, 0, None, 0, 0, None, B, None) == psgd.EINVAL
    assert fn(1, 4, 0, None, 0, 0, A, None, None) == psgd.EINVAL
    assert fn(1, 4, 0, S, 0, -1, A, B, None) == psgd.EINVAL and "advance" in psgd.last_error()
    assert fn(1, 4, 0, S + 4, 0, 0, A, B, None) == psgd.EALIGN
    assert fn(1, 4, 0, None, 0, 0, A + 2, B, None) == psgd.EALIGN
    assert fn(1, 4, 0, None, 0, 0, A, A + 16, None) == psgd.EALIAS
    assert fn(1, 4, 0, A + 8, 0, 1, A, B, None) == psgd.EALIAS
    assert fn(1, 4, 0, S, 0, 1, A, B, None) in (psgd.OK, psgd.EHIP)      # valid: only a device is missing here


def test_mix_step_argument_checks_need_no_device():
    """Validation runs before any HIP call, so fake (never dereferenced) addresses do."""
    lib = psgd.load()
    A, B, C, T1, T2 = 0x100000, 0x900000, 0x1100000, 0x2000000, 0x2001000
    n, d = 4, 1000

    def call(fn=lib.psgd_mix_step, X=A, O=B, G=C, nbr=T1, w=T2, n=n, d=d, lr=0.1, mode=0):
        return fn(X, O, G, nbr, w, n, d, lr, mode, None)

    assert call(X=None) == psgd.EINVAL and "null" in psgd.last_error()
    assert call(O=None) == psgd.EINVAL
    assert call(G=None) == psgd.EINVAL
    assert call(nbr=None) == psgd.EINVAL
    assert call(w=None) == psgd.EINVAL
    assert call(n=0) == psgd.EINVAL
    assert call(n=psgd.MAX_N + 1) == psgd.EINVAL
    assert call(d=-1) == psgd.EINVAL
    assert call(mode=2) == psgd.EINVAL
    assert call(n=512, d=2 ** 61) == psgd.EINVAL and "overflow" in psgd.last_error()
    assert call(X=A + 2) == psgd.EALIGN
    assert call(G=C + 1) == psgd.EALIGN
    assert call(fn=lib.psgd_mix_step_bf16g, G=C + 1) == psgd.EALIGN
    assert call(O=A + 16) == psgd.EALIAS and "partially" in psgd.last_error()
    assert call(O=A, mode=1) == psgd.EALIAS and "delay" in psgd.last_error()
    assert call(G=B + 4 * 100) == psgd.EALIAS
    assert lib.psgd_mix_step_cd(A, B, C, T1, T2, n, d, 0.1, 0, None, None) == psgd.EINVAL
    assert lib.psgd_mix_step_cd(A, B, C, T1, T2, n, d, 0.1, 0, 0x3000004, None) == psgd.EALIGN
    assert lib.psgd_mix_step_cd(A, B, C, T1, T2, n, d, 0.1, 0, B + 8, None) == psgd.EALIAS
    assert lib.psgd_mix_step_cd_bf16g(A, A, C, T1, T2, n, d, 0.1, 1, 0x3000000, None) == psgd.EALIAS
    dg = lib.psgd_mix_step_deg
    assert dg(A, d, B, d, C, d, 0, T1, T2, 0, n, d, 0.1, 0, None, None) == psgd.EINVAL
    assert dg(A, d, B, d, C, d, 0, T1, T2, 33, n, d, 0.1, 0, None, None) == psgd.EINVAL
    assert dg(A, d, B, d, C, d, 0, T1, T2, 16, 512, d, 0.1, 0, None, None) == psgd.EINVAL      # n * deg too large
    assert dg(A, d, A + 4, d, C, d, 0, T1, T2, 5, n, d, 0.1, 0, None, None) == psgd.EALIAS
    assert dg(A, d, B, d, C, d, 0, T1, T2, 5, n, 0, 0.1, 0, None, None) == psgd.OK
    full = lib.psgd_mix_full
    assert full(A, d, B, d, C, d, 0, n, d, 0.1, 0, None, None) in (psgd.OK, psgd.EHIP)
    assert full(None, d, B, d, C, d, 0, n, d, 0.1, 0, None, None) == psgd.EINVAL
    assert full(A, d, A, d, C, d, 0, n, d, 0.1, 1, None, None) == psgd.EALIAS
    assert full(A, d, A + 8, d, C, d, 0, n, d, 0.1, 0, None, None) == psgd.EALIAS
    assert full(A, d, B, d, C, d, 3, n, d, 0.1, 0, None, None) == psgd.EINVAL
    assert full(A, d - 1, B, d, C, d, 0, n, d, 0.1, 0, None, None) == psgd.EINVAL
    assert full(A, d, A, d, C, d, 0, n, 0, 0.1, 0, None, None) == psgd.OK
    ex = lib.psgd_mix_step_ex
    # pitched rows: arrays may interleave (X rows at A + i*P, X_out rows right behind them) ...
    P = 3 * d            # elements
    assert ex(A, P, A + 4 * d, P, A + 8 * d, 2 * P, 1, T1, T2, n, d, 0.1, 0, None, None) in (psgd.OK, psgd.EHIP)
    # ... but must not share bytes, pitches must cover a row, in-place needs equal pitches
    assert ex(A, P, A + 4 * d - 4, P, C, d, 0, T1, T2, n, d, 0.1, 0, None, None) == psgd.EALIAS
    assert ex(A, d - 1, B, d, C, d, 0, T1, T2, n, d, 0.1, 0, None, None) == psgd.EINVAL
    assert ex(A, P, A, 2 * P, C, d, 0, T1, T2, n, d, 0.1, 0, None, None) == psgd.EALIAS
    assert ex(A, P, A, P, C, d, 0, T1, T2, n, d, 0.1, 1, None, None) == psgd.EALIAS
    assert ex(A, P, B, d, C, d, 2, T1, T2, n, d, 0.1, 0, None, None) == psgd.EINVAL
    assert ex(A, P, A, P, C, d, 0, T1, T2, n, 0, 0.1, 0, None, None) == psgd.OK
    # an empty model is a no-op that needs no device either; in-place is legal in mode 0
    assert call(d=0) == psgd.OK
    assert call(O=A, d=0) == psgd.OK


def test_other_entry_points_argument_checks():
    lib = psgd.load()
    A = 0x100000
    assert np.isnan(lib.psgd_consensus_dist(None, 4, 10))
    assert "null" in psgd.last_error()
    assert np.isnan(lib.psgd_consensus_dist(A, 0, 10))
    assert np.isnan(lib.psgd_consensus_dist(A + 1, 4, 10))
    assert lib.psgd_consensus_dist(A, 1, 10) == 0.0          # one learner is always at consensus
    assert lib.psgd_consensus_dist(A, 4, 0) == 0.0
    assert lib.psgd_consensus_dist_async(A, 4, 10, None, None) == psgd.EINVAL
    assert lib.psgd_consensus_dist_async(A, 4, 10, A + 4, None) == psgd.EALIGN
    assert lib.psgd_consensus_dist_async(None, 4, 10, A, None) == psgd.EINVAL
    assert lib.psgd_consensus_dist_ex(A, 5, 4, 10, A, None) == psgd.EINVAL      # pitch < d
    assert lib.psgd_consensus_dist_ex(A, 50, 4, 10, None, None) == psgd.EINVAL
    assert lib.psgd_synth_grad_ex(A, 5, A + 4096, 50, A + 8192, 50, 4, 10, 0.1, None) == psgd.EINVAL
    assert lib.psgd_synth_grad_ex(A, 50, A + 4096, 50, A + 220, 50, 4, 10, 0.1, None) == psgd.EALIAS
    assert lib.psgd_synth_grad(None, A, A, 10, 0.1, None) == psgd.EINVAL
    assert lib.psgd_synth_grad(A, A + 4096, A + 8, 10, 0.1, None) == psgd.EALIAS
    assert lib.psgd_synth_grad(A, A + 4096, A + 8192, -1, 0.1, None) == psgd.EINVAL
    assert lib.psgd_synth_grad(A, A + 4096, A + 8192, 0, 0.1, None) == psgd.OK


def test_no_device_is_reported_not_crashed():
    """On a box without a GPU a real launch request must come back as PSGD_EHIP."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    lib = psgd.load()
    rc = lib.psgd_mix_step(0x100000, 0x900000, 0x1100000, 0x2000000, 0x2001000, 4, 1000, 0.1, 0, None)
    assert rc == psgd.EHIP and psgd.last_error() != ""


def test_pitched_overlap_answer_matches_brute_force():
    """The alias check of the row-pitched entry points against a plain double loop over all row
    pairs, on random interleavings (fake addresses: the answer is given before any device call)."""
    lib = psgd.load()
    rng = np.random.default_rng(3)
    T1, T2 = 0x7000000000, 0x7000001000
    G = 0x6000000000              # gradients far away from both
    hits = 0
    for _ in range(400):
        n = int(rng.integers(1, 9))
        d = int(rng.integers(1, 40))
        P = d + int(rng.integers(0, 60))                  # pitch in elements
        a0 = 0x1000000 + 4 * int(rng.integers(0, 50))
        b0 = a0 + 4 * int(rng.integers(-3 * P, 3 * P + 1))
        if b0 == a0:
            continue                                       # exact aliasing is the in-place case
        same = bool(rng.integers(0, 2))
        Pb = P if same else d + int(rng.integers(0, 60))
        brute = False
        for i in range(n):
            for j in range(n):
                ai, bj = a0 + 4 * i * (P if n > 1 else d), b0 + 4 * j * (Pb if n > 1 else d)
                brute |= ai < bj + 4 * d and bj < ai + 4 * d
        rc = lib.psgd_mix_step_ex(a0, P, b0, Pb, G, d, 0, T1, T2, n, d, 0.1, 0, None, None)
        assert (rc == psgd.EALIAS) == brute, (n, d, P, Pb, a0, b0, rc, brute)
        hits += brute
    assert 50 < hits < 350


def test_binding_refuses_host_tensors():
    """The binding hands raw pointers to kernels, so anything that is not memory of the current
    GPU must be stopped in Python (here, or on a GPU machine, a host tensor would otherwise fault)."""
    import torch
    n, d = 4, 16
    X = torch.zeros(n, d)
    nbr, w = psgd.build_mixing(psgd.TOPO_RING, n)
    with pytest.raises(ValueError):
        psgd.mix_step(X, X.clone(), X.clone(), torch.from_numpy(nbr), torch.from_numpy(w), 0.1)
    with pytest.raises(ValueError):
        psgd.mix_full(X, X.clone(), X.clone(), 0.1)
    with pytest.raises(ValueError):
        psgd.consensus_dist(X)
    with pytest.raises(ValueError):
        psgd.consensus_dist_async(X, torch.zeros(1, dtype=torch.float64))
    with pytest.raises(ValueError):
        psgd.synth_grad(X, X.clone(), X.clone(), 0.1)
    with pytest.raises(ValueError):
        psgd.build_mixing_device(psgd.TOPO_RING, n, 0, torch.from_numpy(nbr), torch.from_numpy(w))


def test_host_calls_are_thread_safe_and_errors_are_per_thread():
    import threading
    lib = psgd.load()
    results, errors = {}, {}

    def good(k):
        for rep in range(50):
            nbr, w = psgd.build_mixing(psgd.TOPO_RAND_RING, 64, 1000 + k, rep)
            if not np.array_equal(nbr, orc.neighbour_table(orc.TOPO_RAND_RING, 64, 1000 + k, rep)[0]):
                results[k] = False
                return
        results[k] = True

    def bad(k):
        nbr = (ctypes.c_int32 * 12)()
        w = (ctypes.c_float * 12)()
        for rep in range(200):
            rc = lib.psgd_build_mixing(0, -k - 1, 0, 0, nbr, w)
            text = psgd.last_error()
            if rc != psgd.EINVAL or ("n=%d " % (-k - 1)) not in text:
                errors[k] = text
                return
        errors[k] = None

    ts = [threading.Thread(target=good, args=(k,)) for k in range(4)] + \
         [threading.Thread(target=bad, args=(k,)) for k in range(4)]
    for t in ts:
        t.start()
    for t in ts:
        t.join()
    assert all(results[k] for k in range(4))
    assert all(errors[k] is None for k in range(4)), errors


def test_launch_arithmetic_covers_every_column_group_once_and_clamps_grids(tmp_path):
    """The persistent-grid arithmetic of the launchers (csrc/psgd_internal.h), compiled for the CPU: every
    column group has exactly one owner, chunks start on 256-byte boundaries, and no grid exceeds the
    partials buffer for any compute-unit count."""
    import shutil
    import subprocess
    gxx = shutil.which("g++") or shutil.which("c++")
    if gxx is None:
        pytest.skip("no host C++ compiler")
    exe = str(tmp_path / "launch_plan_check")
    subprocess.run([gxx, "-std=c++17", "-O1", "-Wall", "-Werror",
                    "-I", os.path.join(ROOT, "paper_2002_01119_amd", "csrc"),
                    os.path.join(ROOT, "tests", "launch_plan_check.cpp"), "-o", exe], check=True)
    r = subprocess.run([exe], capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "launch plan ok" in r.stdout
