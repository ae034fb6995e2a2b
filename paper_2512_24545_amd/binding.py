"""ctypes binding of libmdbf.so: argument marshalling only.

PyTorch supplies device memory and streams; every step of the forward product runs in
the library's HIP kernels.  There is no CPU or PyTorch fallback: if the library cannot
be loaded (and cannot be built), importing callers get an exception.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

MDBF_F16, MDBF_BF16, MDBF_F32 = 0, 1, 2
MDBF_FLAG_PRECISE = 1
MDBF_FLAG_BLOCK_SCALED = 2
MDBF_FLAG_ACCUMULATE = 4
MDBF_FLAG_FP16_STAGED = 8
DTYPE_CODE = {"f16": MDBF_F16, "bf16": MDBF_BF16, "f32": MDBF_F32}

STATUS = {0: "MDBF_OK", -1: "MDBF_EINVAL", -2: "MDBF_EALIGN", -3: "MDBF_EDTYPE", -4: "MDBF_EWORKSPACE",
          -5: "MDBF_EUNSUPPORTED", -6: "MDBF_EHIP"}

EXPORTS = [
    "mdbf_bpw", "mdbf_rank_for_budget", "mdbf_packed_bytes", "mdbf_pack", "mdbf_unpack", "mdbf_pad_envelope",
    "mdbf_stream_read", "mdbf_workspace_bytes", "mdbf_forward", "mdbf_forward_static", "mdbf_batch_plan_bytes", "mdbf_batch_plan_build",
    "mdbf_forward_batch", "mdbf_forward_batch_part", "mdbf_batch_plan_kernel", "mdbf_batch_plan_launches", "mdbf_strerror", "mdbf_last_hip_error", "mdbf_version",
    "mdbf_msvid_block", "mdbf_msvid_workspace_bytes", "mdbf_msvid",
]


class MdbfError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = "%s failed: %s (%d)" % (where, STATUS.get(status, "?"), status)
        if status == -6:
            msg += ": " + lib().mdbf_last_hip_error().decode()
        super().__init__(msg)


class Desc(C.Structure):
    _fields_ = [("m", C.c_int32), ("n", C.c_int32), ("k", C.c_int32), ("l", C.c_int32),
                ("x_dtype", C.c_int32), ("env_dtype", C.c_int32), ("y_dtype", C.c_int32),
                ("flags", C.c_uint32)]


class Env(C.Structure):
    _fields_ = [("A_dev", C.c_void_p), ("Q_dev", C.c_void_p), ("G_dev", C.c_void_p), ("B_dev", C.c_void_p)]


class Layer(C.Structure):
    _fields_ = [("desc", Desc), ("SA_packed_dev", C.c_void_p), ("SB_packed_dev", C.c_void_p), ("env", Env),
                ("X_dev", C.c_void_p), ("ldx", C.c_int64), ("Y_dev", C.c_void_p), ("ldy", C.c_int64),
                ("T", C.c_int32)]


_lib = None


def lib():
    """Load libmdbf.so (building it first only if it does not exist)."""
    global _lib
    if _lib is not None:
        return _lib
    path = os.environ.get("MDBF_LIB_PATH", _build.LIB_PATH)  # override: an alternative build of this library
    if path == _build.LIB_PATH and not os.path.exists(path):
        _build.build_library()
    L = C.CDLL(path)
    L.mdbf_bpw.restype = C.c_double
    L.mdbf_bpw.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int]
    L.mdbf_rank_for_budget.restype = C.c_int
    L.mdbf_rank_for_budget.argtypes = [C.c_int, C.c_int, C.c_int, C.c_double, C.c_int, C.c_int]
    L.mdbf_packed_bytes.argtypes = [C.c_int, C.c_int, C.POINTER(C.c_size_t)]
    L.mdbf_pack.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int64, C.c_void_p, C.c_size_t, C.c_void_p]
    L.mdbf_unpack.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_int64, C.c_void_p]
    L.mdbf_pad_envelope.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_int, C.c_void_p]
    L.mdbf_stream_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_int, C.c_void_p]
    L.mdbf_workspace_bytes.argtypes = [C.POINTER(Desc), C.c_int, C.POINTER(C.c_size_t)]
    L.mdbf_forward.argtypes = [C.POINTER(Desc), C.c_void_p, C.c_void_p, C.POINTER(Env), C.c_void_p, C.c_int64,
                               C.c_void_p, C.c_int64, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]
    L.mdbf_forward_static.argtypes = [C.POINTER(Desc), C.c_void_p, C.c_void_p, C.POINTER(Env), C.c_void_p, C.c_int64,
                                      C.c_void_p, C.c_int64, C.c_int, C.c_void_p]
    L.mdbf_batch_plan_bytes.argtypes = [C.c_int, C.POINTER(Layer), C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
    L.mdbf_batch_plan_build.argtypes = [C.c_int, C.POINTER(Layer), C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t]
    L.mdbf_forward_batch.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    L.mdbf_forward_batch_part.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int, C.c_int, C.c_void_p]
    L.mdbf_batch_plan_launches.argtypes = [C.c_void_p, C.c_size_t]
    L.mdbf_batch_plan_kernel.restype = C.c_char_p
    L.mdbf_batch_plan_kernel.argtypes = [C.c_void_p, C.c_size_t, C.c_int]
    L.mdbf_msvid_block.argtypes = [C.c_int]
    L.mdbf_msvid_workspace_bytes.argtypes = [C.c_int, C.c_int, C.c_int, C.POINTER(C.c_size_t)]
    L.mdbf_msvid.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int64, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                             C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    L.mdbf_strerror.restype = C.c_char_p
    L.mdbf_strerror.argtypes = [C.c_int]
    L.mdbf_last_hip_error.restype = C.c_char_p
    L.mdbf_version.restype = C.c_int
    for name in EXPORTS:
        getattr(L, name)
    _lib = L
    return L


def _check(status, where):
    if status != 0:
        raise MdbfError(status, where)


# ---- host-only calls ------------------------------------------------------------------------
def mdbf_bpw(m, n, k, l, env_bits=16, merge_inner=False):
    return lib().mdbf_bpw(m, n, k, l, env_bits, int(merge_inner))


def mdbf_rank_for_budget(m, n, l, bpw, env_bits=16, multiple=1):
    return lib().mdbf_rank_for_budget(m, n, l, float(bpw), env_bits, multiple)


def mdbf_packed_bytes(rows, cols):
    out = C.c_size_t(0)
    _check(lib().mdbf_packed_bytes(rows, cols, C.byref(out)), "mdbf_packed_bytes")
    return out.value


def mdbf_version():
    return lib().mdbf_version()


# ---- device calls (torch tensors carry the device memory) -----------------------------------
def _torch():
    import torch
    return torch


def _stream_ptr(stream=None):
    torch = _torch()
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def _torch_dtype(name):
    torch = _torch()
    return {"f16": torch.float16, "bf16": torch.bfloat16, "f32": torch.float32}[name]


def _dtype_name(t):
    torch = _torch()
    return {torch.float16: "f16", torch.bfloat16: "bf16", torch.float32: "f32"}[t.dtype]


def mdbf_pack(signs, stream=None):
    """signs: int8 CUDA tensor (rows, cols), entries +-1 (>= 0 packs as +1).  Returns a uint8 CUDA tensor."""
    torch = _torch()
    assert signs.is_cuda and signs.dtype == torch.int8 and signs.dim() == 2 and signs.stride(1) == 1
    rows, cols = signs.shape
    nbytes = mdbf_packed_bytes(rows, cols)
    packed = torch.empty(nbytes, dtype=torch.uint8, device=signs.device)
    _check(lib().mdbf_pack(signs.data_ptr(), rows, cols, signs.stride(0), packed.data_ptr(), nbytes,
                           _stream_ptr(stream)), "mdbf_pack")
    return packed


def mdbf_unpack(packed, rows, cols, stream=None):
    torch = _torch()
    out = torch.empty((rows, cols), dtype=torch.int8, device=packed.device)
    _check(lib().mdbf_unpack(packed.data_ptr(), rows, cols, out.data_ptr(), out.stride(0), _stream_ptr(stream)),
           "mdbf_unpack")
    return out


def mdbf_pad_envelope(env, l_to, stream=None):
    """env: CUDA tensor (rows, l), contiguous.  Returns (rows, l_to) with zero modes appended."""
    torch = _torch()
    assert env.is_cuda and env.dim() == 2 and env.is_contiguous()
    out = torch.empty((env.shape[0], l_to), dtype=env.dtype, device=env.device)
    _check(lib().mdbf_pad_envelope(env.data_ptr(), env.shape[0], env.shape[1], DTYPE_CODE[_dtype_name(env)],
                                   out.data_ptr(), l_to, _stream_ptr(stream)), "mdbf_pad_envelope")
    return out


def mdbf_stream_read(src, sink, stream=None):
    """src: contiguous CUDA tensor whose size in bytes is a multiple of 16; sink: int32 CUDA tensor with a
    multiple of 4 elements, one per wave of the launch.  XOR of sink = XOR of the 32-bit words of src."""
    assert src.is_cuda and src.is_contiguous() and sink.is_cuda and sink.is_contiguous()
    _check(lib().mdbf_stream_read(src.data_ptr(), src.numel() * src.element_size(), sink.data_ptr(), sink.numel(),
                                  _stream_ptr(stream)), "mdbf_stream_read")
    return sink


class DeviceLayer:
    """Device-resident MDBF layer: packed sign bases and envelope factors."""

    def __init__(self, m, n, k, l, SA_packed, SB_packed, A, Q, G, B):
        self.m, self.n, self.k, self.l = m, n, k, l
        self.SA_packed, self.SB_packed = SA_packed, SB_packed
        self.A, self.Q, self.G, self.B = A, Q, G, B
        self.env_dtype = _dtype_name(A)

    @staticmethod
    def from_host(layer, device="cuda:0"):
        """layer: dict from synth.make_layer (numpy).  Uploads, then packs the signs on the GPU."""
        torch = _torch()
        dt = _torch_dtype(layer["env_dtype"])
        up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(device)
        SA = mdbf_pack(up(layer["SA"]))
        SB = mdbf_pack(up(layer["SB"]))
        env = [up(layer[kname]).to(dt).contiguous() for kname in ("A", "Q", "G", "B")]
        return DeviceLayer(layer["m"], layer["n"], layer["k"], layer["l"], SA, SB, *env)

    def padded(self, l_to):
        """The same layer with envelope rank l_to >= l (zero modes appended through mdbf_pad_envelope)."""
        env = [mdbf_pad_envelope(e, l_to) for e in (self.A, self.Q, self.G, self.B)]
        return DeviceLayer(self.m, self.n, self.k, l_to, self.SA_packed, self.SB_packed, *env)

    def desc(self, x_dtype, y_dtype, precise=False, block_scaled=False, accumulate=False, fp16_staged=False):
        flags = ((MDBF_FLAG_PRECISE if precise else 0) | (MDBF_FLAG_BLOCK_SCALED if block_scaled else 0) |
                 (MDBF_FLAG_ACCUMULATE if accumulate else 0) | (MDBF_FLAG_FP16_STAGED if fp16_staged else 0))
        return Desc(self.m, self.n, self.k, self.l, DTYPE_CODE[x_dtype], DTYPE_CODE[self.env_dtype],
                    DTYPE_CODE[y_dtype], flags)

    def env(self):
        return Env(self.A.data_ptr(), self.Q.data_ptr(), self.G.data_ptr(), self.B.data_ptr())


def mdbf_workspace_bytes(desc, T):
    out = C.c_size_t(0)
    _check(lib().mdbf_workspace_bytes(C.byref(desc), T, C.byref(out)), "mdbf_workspace_bytes")
    return out.value


def mdbf_forward(layer, X, y_dtype="f32", precise=False, Y=None, workspace=None, stream=None, block_scaled=False,
                 accumulate=False, fp16_staged=False):
    """Y[b,:] = What X[b,:].  X: CUDA tensor (T, n) of f16/bf16/f32; returns Y (T, m) of y_dtype."""
    torch = _torch()
    assert X.is_cuda and X.dim() == 2 and X.shape[1] == layer.n and X.stride(1) == 1
    T = X.shape[0]
    d = layer.desc(_dtype_name(X), y_dtype, precise, block_scaled, accumulate, fp16_staged)
    assert not (accumulate and Y is None), "accumulate needs the Y to add to"
    if Y is None:
        Y = torch.empty((T, layer.m), dtype=_torch_dtype(y_dtype), device=X.device)
    if workspace is None:
        workspace = torch.empty(mdbf_workspace_bytes(d, T), dtype=torch.uint8, device=X.device)
    env = layer.env()
    _check(lib().mdbf_forward(C.byref(d), layer.SA_packed.data_ptr(), layer.SB_packed.data_ptr(), C.byref(env),
                              X.data_ptr(), X.stride(0), Y.data_ptr(), Y.stride(0), T, workspace.data_ptr(),
                              workspace.numel(), _stream_ptr(stream)), "mdbf_forward")
    return Y


def mdbf_forward_static(layer, X, Y, stream=None, block_scaled=False, fp16_staged=False, precise=False):
    """mdbf_forward on the library's static scratch array: no workspace argument, nothing allocated here
    either (the caller passes Y)."""
    assert X.is_cuda and X.dim() == 2 and X.shape[1] == layer.n and X.stride(1) == 1
    assert Y.is_cuda and Y.shape == (X.shape[0], layer.m) and Y.stride(1) == 1
    d = layer.desc(_dtype_name(X), _dtype_name(Y), precise, block_scaled, False, fp16_staged)
    env = layer.env()
    _check(lib().mdbf_forward_static(C.byref(d), layer.SA_packed.data_ptr(), layer.SB_packed.data_ptr(),
                                     C.byref(env), X.data_ptr(), X.stride(0), Y.data_ptr(), Y.stride(0),
                                     X.shape[0], _stream_ptr(stream)), "mdbf_forward_static")
    return Y


class BatchPlan:
    """Plan for many independent layers: two launches for all of them."""

    def __init__(self, layers, Xs, Ys, precise=False, block_scaled=False, accumulate=False, fp16_staged=False,
                 workspace=None):
        torch = _torch()
        assert len(layers) == len(Xs) == len(Ys) and len(layers) > 0
        n = len(layers)
        arr = (Layer * n)()
        for i, (L, X, Y) in enumerate(zip(layers, Xs, Ys)):
            acc = accumulate[i] if isinstance(accumulate, (list, tuple)) else accumulate
            arr[i].desc = L.desc(_dtype_name(X), _dtype_name(Y), precise, block_scaled, acc, fp16_staged)
            arr[i].SA_packed_dev = L.SA_packed.data_ptr()
            arr[i].SB_packed_dev = L.SB_packed.data_ptr()
            arr[i].env = L.env()
            arr[i].X_dev = X.data_ptr()
            arr[i].ldx = X.stride(0)
            arr[i].Y_dev = Y.data_ptr()
            arr[i].ldy = Y.stride(0)
            arr[i].T = X.shape[0]
        pb, wb = C.c_size_t(0), C.c_size_t(0)
        _check(lib().mdbf_batch_plan_bytes(n, arr, C.byref(pb), C.byref(wb)), "mdbf_batch_plan_bytes")
        self.keep = (layers, Xs, Ys)
        self.workspace_bytes = wb.value
        if workspace is None:
            workspace = torch.empty(max(wb.value, 16), dtype=torch.uint8, device=Xs[0].device)
        self.workspace = workspace   # caller-supplied: a uint8 CUDA tensor of at least workspace_bytes
        self.plan_host = torch.empty(pb.value, dtype=torch.uint8)
        _check(lib().mdbf_batch_plan_build(n, arr, self.workspace.data_ptr(), self.workspace.numel(),
                                           self.plan_host.data_ptr(), pb.value), "mdbf_batch_plan_build")
        self.plan_dev = self.plan_host.to(Xs[0].device)
        self.plan_bytes = pb.value

    def run(self, stream=None):
        _check(lib().mdbf_forward_batch(self.plan_host.data_ptr(), self.plan_dev.data_ptr(), self.plan_bytes,
                                        _stream_ptr(stream)), "mdbf_forward_batch")

    def kernel(self, stage):
        """Name of the product kernel the plan runs for stage 1 or 2."""
        return lib().mdbf_batch_plan_kernel(self.plan_host.data_ptr(), self.plan_bytes, stage).decode()

    def launches(self):
        """Kernel launches one run() issues."""
        return lib().mdbf_batch_plan_launches(self.plan_host.data_ptr(), self.plan_bytes)

    def run_part(self, stages, kernels, stream=None):
        """One part of the plan (bit masks: stages 1|2, kernels 1 = scale-in, 2 = product)."""
        _check(lib().mdbf_forward_batch_part(self.plan_host.data_ptr(), self.plan_dev.data_ptr(), self.plan_bytes,
                                             stages, kernels, _stream_ptr(stream)), "mdbf_forward_batch_part")


def mdbf_forward_batch(plan, stream=None):
    plan.run(stream)


def mdbf_forward_batch_part(plan, stages, kernels, stream=None):
    plan.run_part(stages, kernels, stream)


# ---- quantizer projection --------------------------------------------------------------------
def mdbf_msvid_block(l):
    b = lib().mdbf_msvid_block(l)
    if b < 0:
        raise MdbfError(b, "mdbf_msvid_block")
    return b


def mdbf_msvid(Z, l, X0, iters=8, stream=None, workspace=None):
    """MSVID_l of the CUDA fp32 matrix Z (rows x cols): returns (S int8 +-1, A rows x l, Q cols x l, sigma b).
    X0: the start block of the subspace iteration, cols x mdbf_msvid_block(l), fp32, on the device."""
    torch = _torch()
    assert Z.is_cuda and Z.dim() == 2 and Z.dtype == torch.float32 and Z.stride(1) == 1
    rows, cols = Z.shape
    b = mdbf_msvid_block(l)
    assert X0.is_cuda and X0.dtype == torch.float32 and tuple(X0.shape) == (cols, b) and X0.is_contiguous()
    need = C.c_size_t(0)
    _check(lib().mdbf_msvid_workspace_bytes(rows, cols, l, C.byref(need)), "mdbf_msvid_workspace_bytes")
    if workspace is None:
        workspace = torch.empty(need.value, dtype=torch.uint8, device=Z.device)
    S = torch.empty((rows, cols), dtype=torch.int8, device=Z.device)
    A = torch.empty((rows, l), dtype=torch.float32, device=Z.device)
    Q = torch.empty((cols, l), dtype=torch.float32, device=Z.device)
    sigma = torch.empty((b,), dtype=torch.float32, device=Z.device)
    _check(lib().mdbf_msvid(Z.data_ptr(), rows, cols, Z.stride(0), l, iters, X0.data_ptr(), S.data_ptr(), A.data_ptr(),
                            Q.data_ptr(), sigma.data_ptr(), workspace.data_ptr(), workspace.numel(),
                            _stream_ptr(stream)), "mdbf_msvid")
    return S, A, Q, sigma
