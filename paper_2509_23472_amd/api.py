"""Thin Python binding of the C ABI in include/loract.h: argument marshalling only.

Every function takes torch tensors that already live on the GPU (torch supplies device memory
and the current HIP stream), checks shapes and dtypes, and forwards raw pointers to the
library.  Names match the C entry points.  No step of the method runs in Python.
"""
from __future__ import annotations

import ctypes
from typing import Dict, Optional, Sequence, Tuple

import torch

from . import _lib
from ._lib import LoractParams

F32, BF16 = 0, 1
MAX_RANK = 320
STATUS_RANK_DEFICIENT = 1


class LoractError(RuntimeError):
    def __init__(self, code: int, where: str):
        lib = _lib.load()
        msg = lib.loract_strerror(code).decode()
        hip = lib.loract_last_hip_error().decode()
        super().__init__("%s failed: %s (%d)%s" % (where, msg, code, (" [" + hip + "]") if hip else ""))
        self.code = code


def _check(code: int, where: str) -> None:
    if code != 0:
        raise LoractError(code, where)


def _dtype_code(dt: torch.dtype) -> int:
    if dt == torch.float32:
        return F32
    if dt == torch.bfloat16:
        return BF16
    raise TypeError("unsupported dtype %s (float32 or bfloat16)" % dt)


def _torch_dtype(code: int) -> torch.dtype:
    return torch.bfloat16 if code == BF16 else torch.float32


def _stream_ptr() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


def _require_cuda(*tensors: torch.Tensor) -> None:
    for t in tensors:
        if not t.is_cuda:
            raise ValueError("tensors must live on the GPU")


_workspaces: Dict[Tuple[int, int], torch.Tensor] = {}


def _workspace(nbytes: int, device: torch.device) -> torch.Tensor:
    """A cached uint8 device buffer of at least `nbytes` (grown on demand, never shrunk)."""
    key = (device.index if device.index is not None else torch.cuda.current_device(), _stream_ptr())
    ws = _workspaces.get(key)
    if ws is None or ws.numel() < nbytes:
        ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
        _workspaces[key] = ws
    return ws


def loract_version() -> str:
    return _lib.load().loract_version().decode()


def loract_sample_indices(m: int, l: int, seed: int) -> list:
    """Algorithm 1, row sampling (host): the l ascending distinct row ids for `seed`."""
    buf = (ctypes.c_int32 * max(l, 1))()
    _check(_lib.load().loract_sample_indices(m, l, seed & (2 ** 64 - 1), buf), "loract_sample_indices")
    return [int(buf[i]) for i in range(l)]


def make_params(x: torch.Tensor, k: int, l: int = 0, t: int = 0, seed: int = 0,
                factor_dtype: Optional[torch.dtype] = None) -> LoractParams:
    if x.dim() != 2 or x.stride(1) != 1:
        raise ValueError("X must be a 2-D tensor with unit column stride")
    fd = x.dtype if factor_dtype is None else factor_dtype
    return LoractParams(m=x.shape[0], n=x.shape[1], ldx=x.stride(0) if x.shape[0] > 1 else x.shape[1],
                        k=k, l=l, t=t, x_dtype=_dtype_code(x.dtype), factor_dtype=_dtype_code(fd),
                        seed=seed & (2 ** 64 - 1))


def loract_workspace_bytes(params: LoractParams) -> int:
    out = ctypes.c_size_t(0)
    _check(_lib.load().loract_workspace_bytes(ctypes.byref(params), ctypes.byref(out)),
           "loract_workspace_bytes")
    return int(out.value)


def loract_compress(x: torch.Tensor, k: int, t: int = 0, seed: int = 0,
                    idx: Optional[Sequence[int]] = None,
                    factor_dtype: Optional[torch.dtype] = None,
                    out: Optional[Tuple[torch.Tensor, torch.Tensor]] = None,
                    status: Optional[torch.Tensor] = None, l: int = 0
                    ) -> Tuple[torch.Tensor, torch.Tensor]:
    """U (m x k), V (k x n) of Algorithm 1 for the GPU matrix `x`; enqueued on the current stream.

    `l` > k samples l rows (Theorem 4.3) and cuts the result to rank k; 0 means l = k.
    """
    _require_cuda(x)
    lib = _lib.load()
    p = make_params(x, k, l, t, seed, factor_dtype)
    fdt = _torch_dtype(p.factor_dtype)
    if out is None:
        u = torch.empty((p.m, k), dtype=fdt, device=x.device)
        v = torch.empty((k, p.n), dtype=fdt, device=x.device)
    else:
        u, v = out
        if u.shape != (p.m, k) or v.shape != (k, p.n) or u.dtype != fdt or v.dtype != fdt \
                or not u.is_contiguous() or not v.is_contiguous():
            raise ValueError("out=(U, V) must be contiguous m x k and k x n tensors of the factor dtype")
    ws = _workspace(loract_workspace_bytes(p), x.device)
    idx_arr = None
    if idx is not None:
        n_idx = l if l else k
        if len(idx) != n_idx:
            raise ValueError("idx must hold l row ids (k when l is 0)")
        idx_arr = (ctypes.c_int32 * n_idx)(*[int(i) for i in idx])
    if status is not None and (status.dtype != torch.int32 or not status.is_cuda):
        raise ValueError("status must be an int32 GPU tensor")
    _check(lib.loract_compress(x.data_ptr(), ctypes.byref(p), idx_arr, u.data_ptr(), v.data_ptr(),
                               ws.data_ptr(), ws.numel(), _stream_ptr(),
                               status.data_ptr() if status is not None else None),
           "loract_compress")
    return u, v


def loract_compress_adaptive(x: torch.Tensor, k_max: int, energy: float = 0.9, l: int = 0, t: int = 0,
                             seed: int = 0, idx: Optional[Sequence[int]] = None,
                             factor_dtype: Optional[torch.dtype] = None,
                             status: Optional[torch.Tensor] = None
                             ) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """Algorithm 1 with the rank chosen by the retained-energy count of Section 2 (sum of singular
    values of the l x n factor), at most k_max.  Returns U (m x k_max), V (k_max x n) whose columns /
    rows from the chosen rank on are zero, and the chosen rank as an int32 GPU tensor (read it when
    convenient: nothing here synchronises)."""
    _require_cuda(x)
    lib = _lib.load()
    p = make_params(x, k_max, l, t, seed, factor_dtype)
    fdt = _torch_dtype(p.factor_dtype)
    u = torch.empty((p.m, k_max), dtype=fdt, device=x.device)
    v = torch.empty((k_max, p.n), dtype=fdt, device=x.device)
    k_out = torch.zeros((1,), dtype=torch.int32, device=x.device)
    ws = _workspace(loract_workspace_bytes(p), x.device)
    idx_arr = None
    if idx is not None:
        n_idx = l if l else k_max
        if len(idx) != n_idx:
            raise ValueError("idx must hold l row ids (k_max when l is 0)")
        idx_arr = (ctypes.c_int32 * n_idx)(*[int(i) for i in idx])
    if status is not None and (status.dtype != torch.int32 or not status.is_cuda):
        raise ValueError("status must be an int32 GPU tensor")
    _check(lib.loract_compress_adaptive(x.data_ptr(), ctypes.byref(p), idx_arr, float(energy), u.data_ptr(),
                                        v.data_ptr(), k_out.data_ptr(), ws.data_ptr(), ws.numel(),
                                        _stream_ptr(), status.data_ptr() if status is not None else None),
           "loract_compress_adaptive")
    return u, v, k_out


def loract_reconstruct(u: torch.Tensor, v: torch.Tensor, out_dtype: Optional[torch.dtype] = None,
                       out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Xhat = U V (Section 3.1, Eq. 4)."""
    _require_cuda(u, v)
    if u.dim() != 2 or v.dim() != 2 or u.shape[1] != v.shape[0] or u.dtype != v.dtype:
        raise ValueError("need U (m x k) and V (k x n) of one dtype")
    if not u.is_contiguous() or not v.is_contiguous():
        raise ValueError("U and V must be contiguous")
    m, k = u.shape
    n = v.shape[1]
    odt = u.dtype if out_dtype is None else out_dtype
    if out is None:
        out = torch.empty((m, n), dtype=odt, device=u.device)
    elif out.shape != (m, n) or out.dtype != odt or out.stride(1) != 1:
        raise ValueError("out must be an m x n tensor of the output dtype with unit column stride")
    _check(_lib.load().loract_reconstruct(u.data_ptr(), v.data_ptr(), m, n, k, _dtype_code(u.dtype),
                                          out.data_ptr(), out.stride(0) if m > 1 else n,
                                          _dtype_code(odt), _stream_ptr()),
           "loract_reconstruct")
    return out


def loract_lora_grad(u: torch.Tensor, v: torch.Tensor, dy: torch.Tensor, b_lora: torch.Tensor,
                     scale: float = 1.0, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """dA = (U V)^T (dY B_lora^T) * scale, n x r float32, without forming U V."""
    _require_cuda(u, v, dy, b_lora)
    m, k = u.shape
    n = v.shape[1]
    if v.shape[0] != k or dy.shape[0] != m or b_lora.shape[1] != dy.shape[1] or u.dtype != v.dtype \
            or dy.dtype != b_lora.dtype:
        raise ValueError("shape or dtype mismatch")
    for tns in (u, v, dy, b_lora):
        if not tns.is_contiguous():
            raise ValueError("operands must be contiguous")
    n_out, r = dy.shape[1], b_lora.shape[0]
    lib = _lib.load()
    nbytes = ctypes.c_size_t(0)
    _check(lib.loract_lora_grad_workspace_bytes(m, n, k, n_out, r, ctypes.byref(nbytes)),
           "loract_lora_grad_workspace_bytes")
    ws = _workspace(int(nbytes.value), u.device)
    if out is None:
        out = torch.empty((n, r), dtype=torch.float32, device=u.device)
    elif out.shape != (n, r) or out.dtype != torch.float32 or not out.is_contiguous():
        raise ValueError("out must be a contiguous n x r float32 tensor")
    _check(lib.loract_lora_grad(u.data_ptr(), v.data_ptr(), m, n, k, _dtype_code(u.dtype),
                                dy.data_ptr(), n_out, b_lora.data_ptr(), r, _dtype_code(dy.dtype),
                                float(scale), out.data_ptr(), ws.data_ptr(), ws.numel(), _stream_ptr()),
           "loract_lora_grad")
    return out


def loract_lora_grad_static(u: torch.Tensor, v: torch.Tensor, dy: torch.Tensor, b_lora: torch.Tensor,
                            out: torch.Tensor, scale: float = 1.0) -> torch.Tensor:
    """loract_lora_grad on the scratch buffer built into the library: nothing is allocated, here or
    in the library, so `out` (n x r float32) must be given.  Shapes that need more than
    loract_static_scratch_bytes() of scratch raise LoractError."""
    _require_cuda(u, v, dy, b_lora, out)
    m, k = u.shape
    n = v.shape[1]
    if v.shape[0] != k or dy.shape[0] != m or b_lora.shape[1] != dy.shape[1] or u.dtype != v.dtype \
            or dy.dtype != b_lora.dtype:
        raise ValueError("shape or dtype mismatch")
    for tns in (u, v, dy, b_lora, out):
        if not tns.is_contiguous():
            raise ValueError("operands must be contiguous")
    n_out, r = dy.shape[1], b_lora.shape[0]
    if out.shape != (n, r) or out.dtype != torch.float32:
        raise ValueError("out must be a contiguous n x r float32 tensor")
    _check(_lib.load().loract_lora_grad_static(
        u.data_ptr(), v.data_ptr(), m, n, k, _dtype_code(u.dtype), dy.data_ptr(), n_out,
        b_lora.data_ptr(), r, _dtype_code(dy.dtype), float(scale), out.data_ptr(), _stream_ptr()),
        "loract_lora_grad_static")
    return out


def loract_static_scratch_bytes() -> int:
    return int(_lib.load().loract_static_scratch_bytes())


def loract_gaussian_omega_t(l: int, n: int, dtype: torch.dtype, seed: int,
                            device: Optional[torch.device] = None) -> torch.Tensor:
    """The comparator's Gaussian test matrix, stored transposed (l x n), generated on the GPU."""
    device = torch.device("cuda", torch.cuda.current_device()) if device is None else device
    out = torch.empty((l, n), dtype=dtype, device=device)
    _check(_lib.load().loract_gaussian_omega_t(out.data_ptr(), l, n, _dtype_code(dtype),
                                               seed & (2 ** 64 - 1), _stream_ptr()),
           "loract_gaussian_omega_t")
    return out


def loract_rsvd(x: torch.Tensor, k: int, oversample: int = 0, power_iters: int = 0, seed: int = 0,
                omega_t: Optional[torch.Tensor] = None,
                factor_dtype: Optional[torch.dtype] = None,
                status: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Randomized-SVD comparator (Section 3.2): rank-k factors U (m x k), V (k x n)."""
    _require_cuda(x)
    lib = _lib.load()
    l = k + oversample
    p = make_params(x, k, l, power_iters, seed, factor_dtype)
    fdt = _torch_dtype(p.factor_dtype)
    if omega_t is not None:
        _require_cuda(omega_t)
        if omega_t.shape != (l, p.n) or omega_t.dtype != x.dtype or not omega_t.is_contiguous():
            raise ValueError("omega_t must be a contiguous l x n tensor of X's dtype")
    u = torch.empty((p.m, k), dtype=fdt, device=x.device)
    v = torch.empty((k, p.n), dtype=fdt, device=x.device)
    ws = _workspace(loract_workspace_bytes(p), x.device)
    _check(lib.loract_rsvd(x.data_ptr(), ctypes.byref(p),
                           omega_t.data_ptr() if omega_t is not None else None,
                           u.data_ptr(), v.data_ptr(), ws.data_ptr(), ws.numel(), _stream_ptr(),
                           status.data_ptr() if status is not None else None),
           "loract_rsvd")
    return u, v


def loract_prenorm_forward(x: torch.Tensor, gamma: torch.Tensor, eps: float = 0.0
                           ) -> Tuple[torch.Tensor, torch.Tensor]:
    """Section 3.3, Eqs. (6)-(7): A = X / RMS(X) * gamma and the RMS vector (float32, m)."""
    _require_cuda(x, gamma)
    if x.dim() != 2 or x.stride(1) != 1 or gamma.dtype != torch.float32 or gamma.numel() != x.shape[1] \
            or not gamma.is_contiguous():
        raise ValueError("need a 2-D X with unit column stride and a contiguous float32 gamma of length n")
    m, n = x.shape
    a = torch.empty((m, n), dtype=x.dtype, device=x.device)
    rms = torch.empty((m,), dtype=torch.float32, device=x.device)
    _check(_lib.load().loract_prenorm_forward(x.data_ptr(), m, n, x.stride(0) if m > 1 else n,
                                              _dtype_code(x.dtype), gamma.data_ptr(), float(eps),
                                              a.data_ptr(), n, rms.data_ptr(), _stream_ptr()),
           "loract_prenorm_forward")
    return a, rms


def loract_prenorm_backward(a: torch.Tensor, rms: torch.Tensor, gamma: torch.Tensor,
                            grad_a: torch.Tensor) -> torch.Tensor:
    """Section 3.3, Eqs. (8)-(10): dL/dX from the (reconstructed) A, the RMS vector and dL/dA."""
    _require_cuda(a, rms, gamma, grad_a)
    if a.shape != grad_a.shape or a.dtype != grad_a.dtype or a.stride(1) != 1 or grad_a.stride(1) != 1:
        raise ValueError("A and dA must have the same shape and dtype, unit column stride")
    m, n = a.shape
    if rms.dtype != torch.float32 or rms.numel() != m or gamma.dtype != torch.float32 or gamma.numel() != n:
        raise ValueError("rms (m) and gamma (n) must be float32")
    dx = torch.empty((m, n), dtype=a.dtype, device=a.device)
    _check(_lib.load().loract_prenorm_backward(a.data_ptr(), m, n, a.stride(0) if m > 1 else n,
                                               _dtype_code(a.dtype), rms.data_ptr(), gamma.data_ptr(),
                                               grad_a.data_ptr(), grad_a.stride(0) if m > 1 else n,
                                               dx.data_ptr(), n, _stream_ptr()),
           "loract_prenorm_backward")
    return dx


def loract_profile_begin() -> None:
    _check(_lib.load().loract_profile_begin(), "loract_profile_begin")


def loract_profile_end() -> Dict[str, Tuple[float, int]]:
    """Stops per-kernel timing; returns {kernel name: (total milliseconds, launches)}."""
    lib = _lib.load()
    _check(lib.loract_profile_end(), "loract_profile_end")
    out: Dict[str, Tuple[float, int]] = {}
    buf = ctypes.create_string_buffer(128)
    for i in range(lib.loract_profile_count()):
        ms = ctypes.c_double(0.0)
        cnt = ctypes.c_int64(0)
        _check(lib.loract_profile_get(i, buf, 128, ctypes.byref(ms), ctypes.byref(cnt)),
               "loract_profile_get")
        out[buf.value.decode()] = (float(ms.value), int(cnt.value))
    return out
