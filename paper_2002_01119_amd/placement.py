"""Placement of the replica buffers inside HBM.

On MI355X the sustained rate of a kernel that writes a multi-gigabyte buffer depends on where that buffer lies
physically.  Measured: the device's memory behaves as three ranks, the thirds of its physical address range; a
stream that writes rows which all lie in one third runs at about 71 % of the 8 TB/s peak, rows split evenly over
two or three thirds at 88-89 %, and the mixing step follows its output buffer (76-78 % against 59-72 %).  Virtual
addresses do not matter.  The remedies offered here, all of them only device-memory plumbing (the timed work is
the library's own kernels):

  pitched_layout        rows of all arrays interleaved in one pool that spans most of the device (deterministic,
                        the benchmark's default; the pool is 2.6 times the data)
  spread_layout         the same slots on psgd_spread_alloc memory: physically as far apart, only the slots resident
  interleaved_layout    plain dense arrays in one psgd_interleaved_alloc block, whose 1 GiB pieces come from the
                        three thirds in turn
  place_replica_buffers dense arrays on the fastest windows of a probed pool (the step itself, in place, is timed
                        on candidate windows)

spread_layout infers physical positions from the order in which the driver hands out memory, which is the
address order in a process that has not freed large allocations before: call it first.  interleaved_layout
measures them (a few seconds) and does not care.
"""
import torch

from . import psgd


def settled_pool(nbytes, device):
    """A uint8 pool of `nbytes`, allocated twice: the first allocation is touched and handed back
    to the driver, the second is the one returned.  A process that follows a memory-hungry one
    (a test suite, say) is given whatever pages that one left, and the step then runs about 2 %
    slower (75.9 instead of 77.9 % of the HBM peak, reproducibly); once the whole pool has been
    freed in one piece the driver hands out a better-ordered range."""
    pool = torch.empty(nbytes, dtype=torch.uint8, device=device)
    pool.zero_()
    torch.cuda.synchronize(device)
    del pool
    torch.cuda.empty_cache()
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def settle_allocator(nbytes, device):
    """Allocate, touch and free `nbytes` in one piece: afterwards the driver hands out physical memory in address
    order again (see settled_pool), which is what spread_layout() relies on in a process with an allocation
    history."""
    pool = torch.empty(nbytes, dtype=torch.uint8, device=device)
    pool.zero_()
    torch.cuda.synchronize(device)
    del pool
    torch.cuda.empty_cache()


def pitched_layout(n, d, specs, span_bytes, device, settle=True):
    """Interleave the rows of several [n, d] arrays in ONE pool so that every array spans
    `span_bytes` of device memory: slot i (at i * pitch) holds row i of each array back to
    back.  `specs` is a list of (name, torch dtype).  Returns (dict name -> [n, d] strided view,
    pool tensor, pitch in bytes).  Row starts are 4 KB aligned.  With `settle` the pool comes
    from settled_pool()."""
    def up(v, a):
        return (v + a - 1) // a * a
    offs, cur = {}, 0
    for name, dt in specs:
        offs[name] = cur
        cur += up(d * torch.empty((), dtype=dt).element_size(), 4096)
    pitch = max(cur, (span_bytes // max(n, 1)) // 4096 * 4096)
    pool_bytes = (n - 1) * pitch + cur
    pool = settled_pool(pool_bytes, device) if settle else torch.empty(pool_bytes, dtype=torch.uint8, device=device)
    views = {}
    for name, dt in specs:
        es = torch.empty((), dtype=dt).element_size()
        flat = pool.view(dt)
        views[name] = flat.as_strided((n, d), (pitch // es, 1), offs[name] // es)
    return views, pool, pitch


class SpreadSlots:
    """Owner of a psgd_spread_alloc allocation: frees it when the last tensor view is gone."""

    def __init__(self, n, slot_bytes, pitch_bytes):
        self.base, self.pitch = psgd.spread_alloc(n, slot_bytes, pitch_bytes)
        self.n, self.slot_bytes = n, slot_bytes

    def resident_bytes(self):
        return self.n * self.slot_bytes

    def close(self):
        if self.base:
            base, self.base = self.base, 0
            psgd.spread_free(base)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class _StridedDeviceArray:
    """[n, d] rows inside the slots of a SpreadSlots, exposed through the CUDA array interface so that
    torch.as_tensor() wraps the memory without copying; keeps the owner alive."""

    def __init__(self, owner, offset, n, d, typestr, itemsize):
        self._owner = owner
        self.__cuda_array_interface__ = {
            "shape": (n, d), "typestr": typestr, "data": (owner.base + offset, False), "version": 3,
            "strides": (owner.pitch, itemsize),
        }


def spread_layout(n, d, specs, span_bytes, device):
    """The same interleaved layout as pitched_layout() - slot i holds row i of each array back to back, slots
    `pitch` bytes apart - on memory from psgd_spread_alloc: the slots lie `pitch` apart PHYSICALLY as well, and
    only the slots are resident (the memory between them has been given back to the driver).  Returns (dict
    name -> [n, d] strided view, owner, pitch in bytes).  The views keep the owner alive; the memory is not
    cleared."""
    def up(v, a):
        return (v + a - 1) // a * a
    offs, cur = {}, 0
    for name, dt in specs:
        offs[name] = cur
        cur += up(d * torch.empty((), dtype=dt).element_size(), 4096)
    pitch = max(cur, (span_bytes // max(n, 1)) // 4096 * 4096)
    with torch.cuda.device(device):
        owner = SpreadSlots(n, cur, pitch)
        views = {}
        for name, dt in specs:
            es = torch.empty((), dtype=dt).element_size()
            typestr = {4: "<f4", 2: "<i2"}[es]
            t = torch.as_tensor(_StridedDeviceArray(owner, offs[name], n, d, typestr, es), device=device)
            views[name] = t.view(dt) if t.dtype != dt else t
    return views, owner, owner.pitch


class InterleavedBlock:
    """Owner of a psgd_interleaved_alloc block: frees it when the last tensor view is gone."""

    def __init__(self, nbytes):
        self.base = psgd.interleaved_alloc(nbytes)
        self.pitch = 0                       # unused: the arrays carved from the block are dense
        self.nbytes = nbytes

    def close(self):
        if self.base:
            base, self.base = self.base, 0
            psgd.interleaved_free(base)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class _DenseDeviceArray:
    def __init__(self, owner, offset, shape, typestr):
        self._owner = owner
        self.__cuda_array_interface__ = {"shape": tuple(shape), "typestr": typestr, "data": (owner.base + offset, False),
                                         "version": 3, "strides": None}


def interleaved_layout(n, d, specs, device):
    """Plain dense [n, d] arrays, one per (name, torch dtype) in `specs`, back to back (4 KB aligned) in ONE block
    from psgd_interleaved_alloc: wherever an array starts, its rows are spread evenly over the three thirds of
    the device's physical memory (measured by the call: it takes a few seconds and needs the device's free memory
    for that long).  Returns (dict name
    -> [n, d] contiguous tensor, owner).  The tensors keep the owner alive; the memory is not cleared."""
    def up(v, a):
        return (v + a - 1) // a * a
    offs, cur = {}, 0
    for name, dt in specs:
        offs[name] = cur
        cur += up(n * d * torch.empty((), dtype=dt).element_size(), 4096)
    with torch.cuda.device(device):
        owner = InterleavedBlock(cur)
        views = {}
        for name, dt in specs:
            es = torch.empty((), dtype=dt).element_size()
            t = torch.as_tensor(_DenseDeviceArray(owner, offs[name], (n, d), {4: "<f4", 2: "<i2"}[es]), device=device)
            views[name] = t.view(dt) if t.dtype != dt else t
    return views, owner


def _window(pool, offset, n, d):
    return pool[offset:offset + n * d * 4].view(torch.float32).view(n, d)


def probe_windows(pool, n, d, G, nbr, w, step_bytes, stream=None, repeats=2):
    """Time an in-place psgd_mix_step on every window [off, off + n*d*4) of `pool` (a uint8
    device tensor) with off = 0, step_bytes, 2*step_bytes, ...  Returns [(offset, ms), ...].
    The windows' contents are overwritten."""
    nbytes = n * d * 4
    stream = stream or torch.cuda.current_stream()
    out = []
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    off = 0
    while off + nbytes <= pool.numel():
        X = _window(pool, off, n, d)
        best = float("inf")
        for r in range(repeats + 1):
            e0.record(stream)
            psgd.mix_step(X, X, G, nbr, w, 0.0, stream=stream)
            e1.record(stream)
            e1.synchronize()
            if r > 0:
                best = min(best, e0.elapsed_time(e1))
        out.append((off, best))
        off += step_bytes
    return out


def choose_windows(timings, nbytes, count):
    """Greedy pick of `count` mutually non-overlapping windows with the smallest times."""
    chosen = []
    for off, ms in sorted(timings, key=lambda t: t[1]):
        if all(abs(off - c) >= nbytes for c, _ in chosen):
            chosen.append((off, ms))
            if len(chosen) == count:
                break
    return chosen


def place_replica_buffers(n, d, count, G, nbr, w, reserve_bytes, max_pool_bytes=None, log=None):
    """Allocate one pool, probe it, and return (`count` [n, d] fp32 views on the fastest
    windows, pool tensor, report dict).  Raises torch.OutOfMemoryError if the pool does not fit."""
    nbytes = n * d * 4
    free, _total = torch.cuda.mem_get_info()
    pool_bytes = free - reserve_bytes
    if max_pool_bytes is not None:
        pool_bytes = min(pool_bytes, max_pool_bytes)
    step = max((nbytes // 4) // 4096 * 4096, 4096)
    pool_bytes = pool_bytes // 4096 * 4096
    if pool_bytes < count * nbytes:
        raise torch.OutOfMemoryError("pool of %d bytes cannot hold %d buffers" % (pool_bytes, count))
    pool = settled_pool(pool_bytes, G.device)
    pool.zero_()
    timings = probe_windows(pool, n, d, G, nbr, w, step)
    chosen = choose_windows(timings, nbytes, count)
    if len(chosen) < count:
        raise RuntimeError("could not place %d non-overlapping windows" % count)
    if log:
        log("placement probe (in-place mix step per window, ms): "
            + " ".join("%.1fGB:%.2f" % (o / 1e9, ms) for o, ms in timings))
        log("placement: chose windows at " + ", ".join("%.1f GB (%.2f ms)" % (o / 1e9, ms) for o, ms in chosen))
    views = [_window(pool, off, n, d) for off, _ in chosen]
    report = {
        "pool_GB": pool_bytes / 1e9, "windows_probed": len(timings),
        "probe_ms_min": min(t for _, t in timings), "probe_ms_max": max(t for _, t in timings),
        "chosen_offsets_GB": [o / 1e9 for o, _ in chosen], "chosen_probe_ms": [ms for _, ms in chosen],
    }
    return views, pool, report
