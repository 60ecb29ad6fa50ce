"""psgd_spread_alloc and psgd_interleaved_alloc (placement support): the memory is usable at the promised
addresses, only what was asked for stays allocated, the step runs on views of it and matches the oracle, and
bad arguments are refused."""
import ctypes

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import psgd_oracle as orc
from paper_2002_01119_amd import inputs as inp
from paper_2002_01119_amd import placement as plc

pytestmark = pytest.mark.gpu
REL = 1e-6


@pytest.fixture(scope="module")
def psgd():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2002_01119_amd import psgd as m
    m.load()
    return m


def test_step_on_spread_rows_matches_the_oracle_and_only_the_slots_stay_allocated(psgd):
    dev = torch.device("cuda:0")
    n, d = 12, 300_004
    specs = [("X", torch.float32), ("Y", torch.float32), ("G", torch.bfloat16)]
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info()[0]
    views, owner, pitch = plc.spread_layout(n, d, specs, n * (96 << 20), dev)
    used = free0 - torch.cuda.mem_get_info()[0]
    row_bytes = 2 * ((d * 4 + 4095) // 4096 * 4096) + (d * 2 + 4095) // 4096 * 4096
    assert pitch >= 96 << 20 and pitch % 4096 == 0
    assert n * row_bytes <= used <= n * row_bytes + (256 << 20) < n * pitch // 2, (used, n * row_bytes)   # not n * pitch
    for name, dt in specs:
        v = views[name]
        assert v.shape == (n, d) and v.dtype == dt and v.stride() == (pitch // v.element_size(), 1)
        assert v.data_ptr() >= owner.base and v.data_ptr() + d * v.element_size() <= owner.base + row_bytes + 3 * 4096
    X = inp.fill_normal_rows_(views["X"], 1.0, 11)
    G = inp.fill_normal_rows_(views["G"], 0.1, 12)
    Y = views["Y"]
    Y.fill_(float("nan"))
    nbr, w = psgd.build_mixing(psgd.TOPO_RAND_RING, n, 5, 3)
    cd = torch.zeros(1, dtype=torch.float64, device=dev)
    psgd.mix_step(X, Y, G, torch.from_numpy(nbr).to(dev), torch.from_numpy(w).to(dev), 0.1, cdist_out=cd)
    torch.cuda.synchronize()
    Xh, Gh, Yh = X.contiguous().cpu().numpy(), inp.bf16_tensor_bits(G), Y.contiguous().cpu().numpy()
    want = orc.mix_step(Xh, Gh, orc.densify(nbr, w), 0.1)
    assert np.abs(Yh - want).max() <= REL * np.abs(want).max()
    c_ref = orc.consensus_dist(Yh)
    assert abs(cd.item() - c_ref) <= REL * c_ref
    # rows written through one view are read back through another tensor of the same memory, slot by slot
    Y.fill_(0.0)
    Y[:, 7] = torch.arange(n, dtype=torch.float32, device=dev)
    assert Y.sum().item() == n * (n - 1) / 2
    del views, X, Y, G, v
    torch.cuda.empty_cache()
    free1 = torch.cuda.mem_get_info()[0]
    owner.close()
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] - free1 >= n * row_bytes         # the slots went back to the driver
    owner.close()                                            # a second close is a no-op


def test_bad_arguments_are_refused(psgd):
    lib = psgd.load()
    base, pitch = ctypes.c_void_p(), ctypes.c_int64()
    for n, slot, pit in ((0, 4096, 8192), (513, 4096, 8192), (4, 0, 8192), (4, 8192, 4096), (4, -1, 8192)):
        rc = lib.psgd_spread_alloc(n, slot, pit, ctypes.byref(base), ctypes.byref(pitch))
        assert rc == psgd.EINVAL and base.value is None and psgd.last_error(), (n, slot, pit)
    assert lib.psgd_spread_alloc(4, 4096, 8192, None, ctypes.byref(pitch)) == psgd.EINVAL
    assert lib.psgd_spread_free(None) == psgd.OK
    assert lib.psgd_spread_free(ctypes.c_void_p(0x1000)) == psgd.EINVAL
    # slots as close as they can be: pitch == slot, nothing between them
    b, p = psgd.spread_alloc(3, 10_000, 10_000)
    assert p >= 10_000 and p % 4096 == 0
    t = torch.as_tensor(plc._StridedDeviceArray(type("O", (), {"base": b, "pitch": p})(), 0, 3, 2500, "<f4", 4), device="cuda:0")
    t.fill_(2.0)
    assert t.sum().item() == 3 * 2500 * 2.0
    del t
    psgd.spread_free(b)
    with pytest.raises(psgd.PsgdError):
        psgd.spread_free(b)


def test_step_on_dense_arrays_in_an_interleaved_block_matches_the_oracle(psgd):
    dev = torch.device("cuda:0")
    n, d = 10, 30_000_004                                   # X and Y 1.2 GB each, G 0.6 GB: the block spans 3 GiB pieces
    specs = [("X", torch.float32), ("Y", torch.float32), ("G", torch.bfloat16)]
    torch.cuda.empty_cache()
    free0 = torch.cuda.mem_get_info()[0]
    views, owner = plc.interleaved_layout(n, d, specs, dev)
    used = free0 - torch.cuda.mem_get_info()[0]
    assert (3 << 30) - (64 << 20) <= used <= (3 << 30) + (256 << 20), used    # three 1 GiB pieces, and nothing else kept
    for name, dt in specs:
        v = views[name]
        assert v.shape == (n, d) and v.dtype == dt and v.is_contiguous() and v.data_ptr() % 4096 == 0
    assert views["X"].data_ptr() == owner.base and views["Y"].data_ptr() > views["X"].data_ptr()
    X = inp.fill_normal_rows_(views["X"], 1.0, 21)
    G = inp.fill_normal_rows_(views["G"], 0.1, 22)
    Y = views["Y"]
    Y.fill_(float("nan"))
    nbr, w = psgd.build_mixing(psgd.TOPO_RAND_RING, n, 6, 1)
    cd = torch.zeros(1, dtype=torch.float64, device=dev)
    psgd.mix_step(X, Y, G, torch.from_numpy(nbr).to(dev), torch.from_numpy(w).to(dev), 0.1, cdist_out=cd)
    torch.cuda.synchronize()
    assert psgd.device_status() == 0
    T = orc.densify(nbr, w)
    c_sum = 0.0
    for lo in range(0, d, 6_000_000):                       # column blocks: the oracle works in fp64
        hi = min(lo + 6_000_000, d)
        Xh, Gh = X[:, lo:hi].contiguous().cpu().numpy(), inp.bf16_tensor_bits(G[:, lo:hi])
        Yh = Y[:, lo:hi].contiguous().cpu().numpy()
        want = orc.mix_step(Xh, Gh, T, 0.1)
        assert np.abs(Yh - want).max() <= REL * np.abs(want).max(), lo
        c_sum += orc.consensus_dist(Yh)
    assert abs(cd.item() - c_sum) <= REL * c_sum
    del views, X, Y, G, v
    torch.cuda.empty_cache()
    free1 = torch.cuda.mem_get_info()[0]
    owner.close()
    assert torch.cuda.mem_get_info()[0] - free1 >= (3 << 30) - (64 << 20)
    owner.close()


def test_interleaved_bad_arguments_are_refused(psgd):
    lib = psgd.load()
    ptr = ctypes.c_void_p()
    assert lib.psgd_interleaved_alloc(0, ctypes.byref(ptr)) == psgd.EINVAL and ptr.value is None
    assert lib.psgd_interleaved_alloc(-5, ctypes.byref(ptr)) == psgd.EINVAL
    assert lib.psgd_interleaved_alloc(4096, None) == psgd.EINVAL
    assert lib.psgd_interleaved_alloc(1 << 50, ctypes.byref(ptr)) == psgd.EHIP and "fit" in psgd.last_error()
    assert lib.psgd_interleaved_free(None) == psgd.OK
    assert lib.psgd_interleaved_free(ctypes.c_void_p(0x2000)) == psgd.EINVAL
    p = psgd.interleaved_alloc(100)                          # rounded up to one piece
    psgd.interleaved_free(p)
    with pytest.raises(psgd.PsgdError):
        psgd.interleaved_free(p)
