"""psgd_mix_step_cd_static, the entry point that allocates nothing, called through the C ABI with raw device
addresses and compared with psgd_mix_step_ex (same kernels, library-allocated partials) and with the CPU
oracle, on two calls in a row, the second with a smaller input: the static array then still holds the
first call's partial sums beyond what the second call uses.

Collected last on purpose (file name): it must pass alone in a fresh process and after every other test.
"""
import ctypes

import numpy as np
import pytest

from oracle import psgd_oracle as orc
from paper_2002_01119_amd import inputs as inp

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

REL = 1e-6


@pytest.fixture(scope="module")
def lib():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2002_01119_amd import psgd as m
    torch.cuda.set_device(0)
    return m.load()


def _case(lib, n, d, gkind, topo, seed, pitched):
    """One call of each entry point on the same inputs; returns nothing, asserts."""
    from paper_2002_01119_amd import psgd as m
    lr = 0.1
    X = inp.host_normal_f32((n, d), 1.0, seed)
    G = (inp.host_normal_bf16_bits if gkind == "bf16" else inp.host_normal_f32)((n, d), 0.1, seed + 1)
    nbr, w = orc.neighbour_table(topo, n, 77, seed)
    ld = d + 24 if pitched else d                       # row pitch in elements
    dev = "cuda:0"
    Xd = torch.zeros((n, ld), dtype=torch.float32, device=dev)
    Xd[:, :d] = torch.from_numpy(X).to(dev)
    if gkind == "bf16":
        Gd = torch.zeros((n, ld), dtype=torch.int16, device=dev)
        Gd[:, :d] = torch.from_numpy(G.view(np.int16)).to(dev)
    else:
        Gd = torch.zeros((n, ld), dtype=torch.float32, device=dev)
        Gd[:, :d] = torch.from_numpy(G).to(dev)
    out_ref = torch.full((n, ld), float("nan"), dtype=torch.float32, device=dev)
    out_new = torch.full((n, ld), float("nan"), dtype=torch.float32, device=dev)
    nbr_d, w_d = torch.from_numpy(nbr).to(dev), torch.from_numpy(w).to(dev)
    cd = torch.full((2,), float("nan"), dtype=torch.float64, device=dev)
    torch.cuda.synchronize()
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    args = lambda out, slot: (Xd.data_ptr(), ld, out.data_ptr(), ld, Gd.data_ptr(), ld, int(gkind == "bf16"),
                              nbr_d.data_ptr(), w_d.data_ptr(), n, d, ctypes.c_float(lr), 0,
                              cd.data_ptr() + 8 * slot, stream)
    rc = lib.psgd_mix_step_ex(*args(out_ref, 0))
    assert rc == m.OK, m.last_error()
    rc = lib.psgd_mix_step_cd_static(*args(out_new, 1))
    assert rc == m.OK, m.last_error()
    torch.cuda.synchronize()
    got_ref, got_new = out_ref[:, :d].cpu().numpy(), out_new[:, :d].cpu().numpy()
    # same kernels, same grid, same order of the partial sums: the two entry points agree bit for bit
    assert np.array_equal(got_ref.view(np.uint32), got_new.view(np.uint32))
    c_ref, c_new = cd.cpu().numpy()
    assert c_new == c_ref
    # and both meet the oracle's bar
    want = orc.mix_step(X, G, orc.densify(nbr, w), lr)
    scale = np.abs(want).max()
    assert np.abs(got_new.astype(np.float64) - want).max() <= REL * scale
    c_want = orc.consensus_dist(got_new)
    assert abs(c_new - c_want) <= REL * c_want
    if pitched:                                          # nothing outside the rows was written
        assert torch.isnan(out_new[:, d:]).all()
    assert m.device_status() == 0


def test_static_entry_point_twice_second_call_smaller(lib):
    # long rows: 768-lane workgroups, many sweeps, one workgroup per CU -> about 256 partials
    _case(lib, 16, 1_600_004, "bf16", orc.TOPO_RAND_RING, 5, pitched=True)
    # then a small ragged one: 256-lane workgroups, a handful of partials, scalar columns (d odd)
    _case(lib, 5, 1001, "f32", orc.TOPO_RING, 6, pitched=False)
    # and a mid-sized one whose grid is the largest the kernel uses (4 workgroups per CU)
    _case(lib, 8, 300_000, "f32", orc.TOPO_RAND_RING, 7, pitched=False)


def test_static_entry_point_argument_checks_and_empty_input(lib):
    from paper_2002_01119_amd import psgd as m
    dev = "cuda:0"
    n, d = 4, 64
    X = torch.zeros((n, d), device=dev)
    Y = torch.zeros((n, d), device=dev)
    G = torch.zeros((n, d), device=dev)
    nbr, w = orc.neighbour_table(orc.TOPO_RING, n)
    nbr_d, w_d = torch.from_numpy(nbr).to(dev), torch.from_numpy(w).to(dev)
    cd = torch.full((1,), float("nan"), dtype=torch.float64, device=dev)
    f = lib.psgd_mix_step_cd_static
    lr = ctypes.c_float(0.1)
    assert f(X.data_ptr(), d, Y.data_ptr(), d, G.data_ptr(), d, 0, nbr_d.data_ptr(), w_d.data_ptr(), n, d, lr, 0,
             None, None) == m.EINVAL                                    # the distance output is required
    assert f(X.data_ptr(), d, Y.data_ptr(), d, G.data_ptr(), d, 2, nbr_d.data_ptr(), w_d.data_ptr(), n, d, lr, 0,
             cd.data_ptr(), None) == m.EINVAL
    assert f(X.data_ptr(), d, X.data_ptr(), d, G.data_ptr(), d, 0, nbr_d.data_ptr(), w_d.data_ptr(), n, d, lr, 1,
             cd.data_ptr(), None) == m.EALIAS                           # delay-by-one forbids in place
    assert f(X.data_ptr(), d, Y.data_ptr(), d, G.data_ptr(), d, 0, nbr_d.data_ptr(), w_d.data_ptr(), m.MAX_N + 1, d,
             lr, 0, cd.data_ptr(), None) == m.EINVAL
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    assert f(X.data_ptr(), 0, Y.data_ptr(), 0, G.data_ptr(), 0, 0, nbr_d.data_ptr(), w_d.data_ptr(), n, 0, lr, 0,
             cd.data_ptr(), stream) == m.OK                             # d = 0 writes distance 0
    torch.cuda.synchronize()
    assert cd.item() == 0.0
