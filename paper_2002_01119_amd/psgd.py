"""ctypes binding of libpsgd.so: argument marshalling only, same names as include/psgd.h.

Device buffers are torch tensors (PyTorch is used for HBM allocation and streams); every
step of the computation runs in the library's HIP kernels.  There is no fallback: if the
shared library is missing or a call fails, an exception is raised.
"""
import ctypes
import math
import os

import numpy as np

TOPO_RING = 0
TOPO_RAND_RING = 1
TOPO_FULL = 2
DEG = 3
MAX_N = 512
STATIC_SLOTS = 2048

OK, EINVAL, EALIAS, EALIGN, EHIP = 0, -1, -2, -3, -4

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libpsgd.so")
_lib = None

EXPORTS = (
    "psgd_build_mixing", "psgd_build_mixing_device", "psgd_mix_step", "psgd_mix_step_bf16g", "psgd_mix_step_cd",
    "psgd_mix_step_cd_bf16g", "psgd_mix_step_ex", "psgd_mix_step_cd_static", "psgd_mix_step_deg", "psgd_mix_full", "psgd_consensus_dist", "psgd_consensus_dist_ex",
    "psgd_consensus_dist_async", "psgd_synth_grad", "psgd_synth_grad_ex", "psgd_reference_stream", "psgd_spread_alloc", "psgd_spread_free", "psgd_interleaved_alloc", "psgd_interleaved_free", "psgd_device_status", "psgd_last_error",
    "psgd_version",
)


class PsgdError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("psgd status %d: %s" % (code, text))
        self.code = code


def load(reload=False):
    """Load libpsgd.so (built in-tree by __graft_entry__.build()) and declare its signatures."""
    global _lib
    if _lib is not None and not reload:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError("%s not found: run `python __graft_entry__.py` to build the HIP library"
                          % _LIB_PATH)
    lib = ctypes.CDLL(_LIB_PATH)
    c_i32p = ctypes.POINTER(ctypes.c_int32)
    c_f32p = ctypes.POINTER(ctypes.c_float)
    vp = ctypes.c_void_p
    lib.psgd_build_mixing.restype = ctypes.c_int
    lib.psgd_build_mixing.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_uint64, ctypes.c_uint64,
                                      c_i32p, c_f32p]
    lib.psgd_build_mixing_device.restype = ctypes.c_int
    lib.psgd_build_mixing_device.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_uint64, vp, ctypes.c_uint64,
                                             ctypes.c_int, vp, vp, vp]
    for name in ("psgd_mix_step", "psgd_mix_step_bf16g"):
        fn = getattr(lib, name)
        fn.restype = ctypes.c_int
        fn.argtypes = [vp, vp, vp, vp, vp, ctypes.c_int, ctypes.c_int64, ctypes.c_float,
                       ctypes.c_int, vp]
    for name in ("psgd_mix_step_cd", "psgd_mix_step_cd_bf16g"):
        fn = getattr(lib, name)
        fn.restype = ctypes.c_int
        fn.argtypes = [vp, vp, vp, vp, vp, ctypes.c_int, ctypes.c_int64, ctypes.c_float,
                       ctypes.c_int, vp, vp]
    lib.psgd_mix_step_ex.restype = ctypes.c_int
    lib.psgd_mix_step_ex.argtypes = [vp, ctypes.c_int64, vp, ctypes.c_int64, vp, ctypes.c_int64, ctypes.c_int,
                                     vp, vp, ctypes.c_int, ctypes.c_int64, ctypes.c_float, ctypes.c_int, vp, vp]
    lib.psgd_mix_step_cd_static.restype = ctypes.c_int
    lib.psgd_mix_step_cd_static.argtypes = list(lib.psgd_mix_step_ex.argtypes)
    lib.psgd_mix_step_deg.restype = ctypes.c_int
    lib.psgd_mix_step_deg.argtypes = [vp, ctypes.c_int64, vp, ctypes.c_int64, vp, ctypes.c_int64, ctypes.c_int,
                                      vp, vp, ctypes.c_int, ctypes.c_int, ctypes.c_int64, ctypes.c_float,
                                      ctypes.c_int, vp, vp]
    lib.psgd_mix_full.restype = ctypes.c_int
    lib.psgd_mix_full.argtypes = [vp, ctypes.c_int64, vp, ctypes.c_int64, vp, ctypes.c_int64, ctypes.c_int,
                                  ctypes.c_int, ctypes.c_int64, ctypes.c_float, ctypes.c_int, vp, vp]
    lib.psgd_consensus_dist_ex.restype = ctypes.c_int
    lib.psgd_consensus_dist_ex.argtypes = [vp, ctypes.c_int64, ctypes.c_int, ctypes.c_int64, vp, vp]
    lib.psgd_consensus_dist.restype = ctypes.c_double
    lib.psgd_consensus_dist.argtypes = [vp, ctypes.c_int, ctypes.c_int64]
    lib.psgd_consensus_dist_async.restype = ctypes.c_int
    lib.psgd_consensus_dist_async.argtypes = [vp, ctypes.c_int, ctypes.c_int64, vp, vp]
    lib.psgd_synth_grad.restype = ctypes.c_int
    lib.psgd_synth_grad.argtypes = [vp, vp, vp, ctypes.c_int64, ctypes.c_float, vp]
    lib.psgd_synth_grad_ex.restype = ctypes.c_int
    lib.psgd_synth_grad_ex.argtypes = [vp, ctypes.c_int64, vp, ctypes.c_int64, vp, ctypes.c_int64, ctypes.c_int,
                                       ctypes.c_int64, ctypes.c_float, vp]
    lib.psgd_reference_stream.restype = ctypes.c_int
    lib.psgd_reference_stream.argtypes = [ctypes.c_int, vp, ctypes.c_int64, vp, ctypes.c_int64, vp, ctypes.c_int64,
                                          ctypes.c_int, ctypes.c_int, ctypes.c_int64, ctypes.c_float, vp]
    lib.psgd_spread_alloc.restype = ctypes.c_int
    lib.psgd_spread_alloc.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.POINTER(ctypes.c_void_p),
                                      ctypes.POINTER(ctypes.c_int64)]
    lib.psgd_spread_free.restype = ctypes.c_int
    lib.psgd_spread_free.argtypes = [vp]
    lib.psgd_interleaved_alloc.restype = ctypes.c_int
    lib.psgd_interleaved_alloc.argtypes = [ctypes.c_int64, ctypes.POINTER(ctypes.c_void_p)]
    lib.psgd_interleaved_free.restype = ctypes.c_int
    lib.psgd_interleaved_free.argtypes = [vp]
    lib.psgd_device_status.restype = ctypes.c_int
    lib.psgd_device_status.argtypes = [ctypes.c_int]
    lib.psgd_last_error.restype = ctypes.c_char_p
    lib.psgd_last_error.argtypes = []
    lib.psgd_version.restype = ctypes.c_int
    lib.psgd_version.argtypes = []
    _lib = lib
    return lib


def last_error():
    return load().psgd_last_error().decode("utf-8", "replace")


def _check(rc):
    if rc != OK:
        raise PsgdError(rc, last_error())


def _stream_handle(stream):
    """hipStream_t of a torch stream (None = torch's current stream)."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _on_current_device(*tensors):
    """Every pointer handed to the library must be device memory of the CURRENT device: a host
    pointer or another GPU's would be dereferenced by a kernel."""
    import torch
    if not torch.cuda.is_available():
        raise ValueError("no GPU visible: the library works on device memory only")
    cur = torch.cuda.current_device()
    for t in tensors:
        if t is None:
            continue
        if not isinstance(t, torch.Tensor) or not t.is_cuda or t.device.index != cur:
            raise ValueError("expected tensors on the current GPU (cuda:%d)" % cur)


def _rows_cols(t):
    if t.dim() != 2 or not t.is_contiguous():
        raise ValueError("expected a contiguous [n, d] tensor")
    return int(t.shape[0]), int(t.shape[1])


def _rows_cols_pitch(t):
    """(n, d, pitch in elements) of a 2-D tensor whose rows are contiguous (stride(1) == 1)."""
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError("expected an [n, d] tensor with unit stride along d")
    n, d = int(t.shape[0]), int(t.shape[1])
    return n, d, (int(t.stride(0)) if n > 1 else d)


def build_mixing(topology, n, seed=0, step=0):
    """Returns (nbr int32 [n,3], w float32 [n,3]) as host numpy arrays."""
    nbr = np.empty((max(n, 0), DEG), dtype=np.int32)
    w = np.empty((max(n, 0), DEG), dtype=np.float32)
    _check(load().psgd_build_mixing(
        int(topology), int(n), ctypes.c_uint64(seed & (2 ** 64 - 1)), ctypes.c_uint64(step & (2 ** 64 - 1)),
        nbr.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), w.ctypes.data_as(ctypes.POINTER(ctypes.c_float))))
    return nbr, w


def build_mixing_device(topology, n, seed, nbr, w, step_dev=None, step_offset=0, advance=0, stream=None):
    """Enqueue the construction of the same table in device memory: nbr int32 [n,3], w float32
    [n,3] (device tensors, written).  The iteration is step_offset plus, if given, the value of
    step_dev (device int64 / uint64 tensor, >= 1 element), which is then advanced by `advance`."""
    import torch
    if nbr.dtype != torch.int32 or w.dtype != torch.float32 or nbr.numel() != 3 * n or w.numel() != 3 * n \
            or not nbr.is_contiguous() or not w.is_contiguous():
        raise ValueError("nbr must be int32 [n,3] and w float32 [n,3], contiguous")
    _on_current_device(nbr, w, step_dev)
    sp = None
    if step_dev is not None:
        if step_dev.dtype not in (torch.int64, torch.uint64) or step_dev.numel() < 1 or step_dev.device != nbr.device:
            raise ValueError("step_dev must be a 64-bit integer device tensor")
        sp = step_dev.data_ptr()
    _check(load().psgd_build_mixing_device(
        int(topology), int(n), ctypes.c_uint64(seed & (2 ** 64 - 1)), sp, ctypes.c_uint64(step_offset & (2 ** 64 - 1)),
        int(advance), nbr.data_ptr(), w.data_ptr(), _stream_handle(stream)))


def mix_step(X, X_out, G, nbr, w, lr, delay_mode=0, stream=None, cdist_out=None):
    """Enqueue X_out = mix(X) - lr * G.  All arguments are device tensors; G is float32, or
    bfloat16 / int16 / uint16 (bf16 bit patterns).  nbr / w are [n, deg] tables (deg = 3 for
    the ring tables of build_mixing; any other deg selects psgd_mix_step_deg).  X, X_out and G are [n, d] with unit
    stride along d; their rows may be pitched (stride(0) >= d), which selects
    psgd_mix_step_ex.  With cdist_out (device float64 tensor, >= 1 element) the fused
    variant also writes the consensus distance of X_out there."""
    import torch
    n, d, ldx = _rows_cols_pitch(X)
    no, do, ldo = _rows_cols_pitch(X_out)
    ng, dg, ldg = _rows_cols_pitch(G)
    if (no, do) != (n, d) or (ng, dg) != (n, d):
        raise ValueError("X, X_out and G must have one shape")
    if X.dtype != torch.float32 or X_out.dtype != torch.float32:
        raise ValueError("X and X_out must be float32")
    if nbr.dtype != torch.int32 or w.dtype != torch.float32 or nbr.numel() % n or nbr.numel() != w.numel() \
            or not nbr.is_contiguous() or not w.is_contiguous():
        raise ValueError("nbr must be int32 [n,deg] and w float32 [n,deg], contiguous")
    deg = nbr.numel() // n
    _on_current_device(X, X_out, G, nbr, w, cdist_out)
    lib = load()
    if G.dtype == torch.float32:
        bf16 = False
    elif G.dtype in (torch.bfloat16, torch.int16, torch.uint16):
        bf16 = True
    else:
        raise ValueError("G must be float32 or bfloat16 bit patterns")
    cd_ptr = None
    if cdist_out is not None:
        if cdist_out.dtype != torch.float64 or cdist_out.numel() < 1 or cdist_out.device != X.device:
            raise ValueError("cdist_out must be a float64 device tensor")
        cd_ptr = cdist_out.data_ptr()
    sh = _stream_handle(stream)
    if deg != DEG:
        _check(lib.psgd_mix_step_deg(X.data_ptr(), ldx, X_out.data_ptr(), ldo, G.data_ptr(), ldg, int(bf16),
                                     nbr.data_ptr(), w.data_ptr(), deg, n, d, float(lr), int(delay_mode), cd_ptr, sh))
    elif (ldx, ldo, ldg) != (d, d, d):
        _check(lib.psgd_mix_step_ex(X.data_ptr(), ldx, X_out.data_ptr(), ldo, G.data_ptr(), ldg, int(bf16),
                                    nbr.data_ptr(), w.data_ptr(), n, d, float(lr), int(delay_mode), cd_ptr, sh))
    elif cd_ptr is None:
        fn = lib.psgd_mix_step_bf16g if bf16 else lib.psgd_mix_step
        _check(fn(X.data_ptr(), X_out.data_ptr(), G.data_ptr(), nbr.data_ptr(), w.data_ptr(), n, d,
                  float(lr), int(delay_mode), sh))
    else:
        fn = lib.psgd_mix_step_cd_bf16g if bf16 else lib.psgd_mix_step_cd
        _check(fn(X.data_ptr(), X_out.data_ptr(), G.data_ptr(), nbr.data_ptr(), w.data_ptr(), n, d,
                  float(lr), int(delay_mode), cd_ptr, sh))


def mix_step_cd_static(X, X_out, G, nbr, w, lr, cdist_out, delay_mode=0, stream=None):
    """psgd_mix_step_cd_static: the fused step + distance of mix_step (3-slot tables, any row pitch) through
    the entry point that allocates nothing."""
    import torch
    n, d, ldx = _rows_cols_pitch(X)
    no, do, ldo = _rows_cols_pitch(X_out)
    ng, dg, ldg = _rows_cols_pitch(G)
    if (no, do) != (n, d) or (ng, dg) != (n, d):
        raise ValueError("X, X_out and G must have one shape")
    if X.dtype != torch.float32 or X_out.dtype != torch.float32:
        raise ValueError("X and X_out must be float32")
    if nbr.dtype != torch.int32 or w.dtype != torch.float32 or nbr.numel() != DEG * n or w.numel() != DEG * n \
            or not nbr.is_contiguous() or not w.is_contiguous():
        raise ValueError("nbr must be int32 [n,3] and w float32 [n,3], contiguous")
    if G.dtype == torch.float32:
        bf16 = 0
    elif G.dtype in (torch.bfloat16, torch.int16, torch.uint16):
        bf16 = 1
    else:
        raise ValueError("G must be float32 or bfloat16 bit patterns")
    if cdist_out is None or cdist_out.dtype != torch.float64 or cdist_out.numel() < 1 or cdist_out.device != X.device:
        raise ValueError("cdist_out must be a float64 device tensor")
    _on_current_device(X, X_out, G, nbr, w, cdist_out)
    _check(load().psgd_mix_step_cd_static(X.data_ptr(), ldx, X_out.data_ptr(), ldo, G.data_ptr(), ldg, bf16,
                                          nbr.data_ptr(), w.data_ptr(), n, d, float(lr), int(delay_mode),
                                          cdist_out.data_ptr(), _stream_handle(stream)))


def mix_full(X, X_out, G, lr, delay_mode=0, stream=None, cdist_out=None):
    """Enqueue X_out[i] = mean_j X[j] - lr * G[i] (global averaging, T_u).  Tensors as in mix_step."""
    import torch
    n, d, ldx = _rows_cols_pitch(X)
    no, do, ldo = _rows_cols_pitch(X_out)
    ng, dg, ldg = _rows_cols_pitch(G)
    if (no, do) != (n, d) or (ng, dg) != (n, d):
        raise ValueError("X, X_out and G must have one shape")
    if X.dtype != torch.float32 or X_out.dtype != torch.float32:
        raise ValueError("X and X_out must be float32")
    if G.dtype == torch.float32:
        bf16 = 0
    elif G.dtype in (torch.bfloat16, torch.int16, torch.uint16):
        bf16 = 1
    else:
        raise ValueError("G must be float32 or bfloat16 bit patterns")
    _on_current_device(X, X_out, G, cdist_out)
    cd_ptr = None
    if cdist_out is not None:
        if cdist_out.dtype != torch.float64 or cdist_out.numel() < 1 or cdist_out.device != X.device:
            raise ValueError("cdist_out must be a float64 device tensor")
        cd_ptr = cdist_out.data_ptr()
    _check(load().psgd_mix_full(X.data_ptr(), ldx, X_out.data_ptr(), ldo, G.data_ptr(), ldg, bf16, n, d, float(lr),
                                int(delay_mode), cd_ptr, _stream_handle(stream)))


def consensus_dist(X):
    """Synchronous sum_i ||x_i - xbar||^2 of a device tensor [n, d]."""
    import torch
    n, d = _rows_cols(X)
    _on_current_device(X)
    if X.dtype != torch.float32:
        raise ValueError("X must be float32")
    v = load().psgd_consensus_dist(X.data_ptr(), n, d)
    if math.isnan(v):
        err = last_error()
        if err:
            raise PsgdError(EINVAL, err)
    return v


def consensus_dist_async(X, out, stream=None):
    """Enqueue the consensus distance of X into out (device float64 tensor, 1 element)."""
    import torch
    n, d, ldx = _rows_cols_pitch(X)
    _on_current_device(X, out)
    if X.dtype != torch.float32:
        raise ValueError("X must be float32")
    if out.dtype != torch.float64 or out.numel() < 1 or out.device != X.device:
        raise ValueError("out must be a float64 device tensor")
    if ldx != d:
        _check(load().psgd_consensus_dist_ex(X.data_ptr(), ldx, n, d, out.data_ptr(), _stream_handle(stream)))
    else:
        _check(load().psgd_consensus_dist_async(X.data_ptr(), n, d, out.data_ptr(), _stream_handle(stream)))


def synth_grad(X_prev, noise, G, c, stream=None):
    """Enqueue G = c * X_prev + noise (fp32, elementwise) for the delay-by-one workload.
    Contiguous tensors of any shape, or [n, d] tensors with pitched rows."""
    import torch
    if X_prev.shape != noise.shape or X_prev.shape != G.shape:
        raise ValueError("X_prev, noise and G must have one shape")
    _on_current_device(X_prev, noise, G)
    if X_prev.dtype != torch.float32 or noise.dtype != torch.float32 or G.dtype != torch.float32:
        raise ValueError("X_prev, noise and G must be float32")
    if X_prev.is_contiguous() and noise.is_contiguous() and G.is_contiguous():
        _check(load().psgd_synth_grad(X_prev.data_ptr(), noise.data_ptr(), G.data_ptr(), X_prev.numel(),
                                      float(c), _stream_handle(stream)))
        return
    n, d, ldx = _rows_cols_pitch(X_prev)
    _, _, ldn = _rows_cols_pitch(noise)
    _, _, ldg = _rows_cols_pitch(G)
    _check(load().psgd_synth_grad_ex(X_prev.data_ptr(), ldx, noise.data_ptr(), ldn, G.data_ptr(), ldg, n, d,
                                     float(c), _stream_handle(stream)))


REF_READ, REF_WRITE, REF_AXPY = 0, 1, 2


def reference_stream(kind, X, X_out, G, a=0.0, stream=None):
    """Enqueue a reference stream over [n, d] tensors laid out as for mix_step (measurement support):
    REF_READ reads X and G, REF_WRITE fills X_out with `a`, REF_AXPY writes X_out = X + a * G."""
    import torch
    n, d, ldx = _rows_cols_pitch(X)
    no, do, ldo = _rows_cols_pitch(X_out)
    ng, dg, ldg = _rows_cols_pitch(G)
    if (no, do) != (n, d) or (ng, dg) != (n, d):
        raise ValueError("X, X_out and G must have one shape")
    if X.dtype != torch.float32 or X_out.dtype != torch.float32:
        raise ValueError("X and X_out must be float32")
    if G.dtype == torch.float32:
        bf16 = 0
    elif G.dtype in (torch.bfloat16, torch.int16, torch.uint16):
        bf16 = 1
    else:
        raise ValueError("G must be float32 or bfloat16 bit patterns")
    _on_current_device(X, X_out, G)
    _check(load().psgd_reference_stream(int(kind), X.data_ptr(), ldx, X_out.data_ptr(), ldo, G.data_ptr(), ldg, bf16,
                                        n, d, float(a), _stream_handle(stream)))


def spread_alloc(n, slot_bytes, pitch_bytes):
    """n slots of device memory, `pitch` bytes apart in one address range and physically spread out likewise,
    with only the slots resident (psgd_spread_alloc).  Returns (base address, pitch in bytes); free it with
    spread_free(base).  Addresses between the slots are not mapped."""
    base = ctypes.c_void_p()
    pitch = ctypes.c_int64()
    _check(load().psgd_spread_alloc(int(n), int(slot_bytes), int(pitch_bytes), ctypes.byref(base), ctypes.byref(pitch)))
    return base.value, pitch.value


def spread_free(base):
    _check(load().psgd_spread_free(ctypes.c_void_p(base)))


def interleaved_alloc(nbytes):
    """One block of device memory at consecutive addresses whose 1 GiB pieces come from the three thirds of the
    device's physical memory in turn (psgd_interleaved_alloc).  Returns its address; free it with
    interleaved_free()."""
    ptr = ctypes.c_void_p()
    _check(load().psgd_interleaved_alloc(int(nbytes), ctypes.byref(ptr)))
    return ptr.value


def interleaved_free(ptr):
    _check(load().psgd_interleaved_free(ctypes.c_void_p(ptr)))


def device_status(clear=True):
    rc = load().psgd_device_status(1 if clear else 0)
    if rc < 0:
        raise PsgdError(rc, last_error())
    return rc


def version():
    return load().psgd_version()
