"""ctypes binding of the C ABI in include/svdcache.h (argument marshalling only)."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

PKG_DIR = os.path.dirname(os.path.abspath(__file__))

SVDC_F32, SVDC_BF16 = 0, 1
SVDC_PRECISE, SVDC_FAST = 0, 1
_DTYPES = {torch.float32: SVDC_F32, torch.bfloat16: SVDC_BF16}


class SvdcError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {svdcache_strerror(code)} (status {code})")


class Shape(C.Structure):
    """Mirror of svdc_shape."""
    _fields_ = [("B", C.c_int32), ("N", C.c_int32), ("D", C.c_int32), ("k", C.c_int32),
                ("ldf", C.c_int64), ("block_stride", C.c_int64), ("dtype", C.c_int32), ("precision", C.c_int32)]


class FitParams(C.Structure):
    """Mirror of svdc_fit_params."""
    _fields_ = [("oversample_p", C.c_int32), ("power_iters_q", C.c_int32), ("seed", C.c_uint64),
                ("jacobi_max_sweeps", C.c_int32), ("reserved", C.c_int32)]


EXPORTS = {
    "svdcache_version": (C.c_int32, []),
    "svdcache_strerror": (C.c_char_p, [C.c_int32]),
    "svdcache_fit_workspace_bytes": (C.c_size_t, [C.POINTER(Shape), C.POINTER(FitParams)]),
    "svdcache_workspace_bytes": (C.c_size_t, [C.POINTER(Shape), C.POINTER(FitParams)]),
    "svdcache_fit_status_offset": (C.c_size_t, [C.POINTER(Shape), C.POINTER(FitParams)]),
    "svdcache_packed_basis_bytes": (C.c_size_t, [C.POINTER(Shape)]),
    "svdcache_has_mfma_path": (C.c_int32, [C.POINTER(Shape)]),
    "svdcache_fit_basis": (C.c_int32, [C.POINTER(Shape), C.POINTER(FitParams), C.c_void_p, C.c_void_p, C.c_void_p,
                                       C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "svdcache_fit_basis_static": (C.c_int32, [C.POINTER(Shape), C.POINTER(FitParams), C.c_void_p, C.c_void_p,
                                              C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "svdcache_pack_basis": (C.c_int32, [C.POINTER(Shape), C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "svdcache_full_step": (C.c_int32, [C.POINTER(Shape), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                       C.c_void_p, C.c_void_p, C.c_float, C.c_int32, C.c_void_p]),
    "svdcache_full_step_residual_ema": (C.c_int32, [C.POINTER(Shape), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                                    C.c_void_p, C.c_void_p, C.c_void_p, C.c_float, C.c_float,
                                                    C.c_int32, C.c_void_p]),
    "svdcache_forecast": (C.c_int32, [C.POINTER(Shape), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_void_p]),
    "svdcache_packed_state_bytes": (C.c_size_t, [C.POINTER(Shape)]),
    "svdcache_pack_state": (C.c_int32, [C.POINTER(Shape), C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]),
    "svdcache_full_step_packed": (C.c_int32, [C.POINTER(Shape), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                              C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_float, C.c_int32,
                                              C.c_void_p]),
    "svdcache_forecast_packed": (C.c_int32, [C.POINTER(Shape), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                             C.c_void_p]),
    "svdcache_select_rank": (C.c_int32, [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_float, C.c_void_p,
                                         C.c_void_p, C.c_void_p]),
    "svdcache_truncate_basis": (C.c_int32, [C.POINTER(Shape), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "svdcache_extrapolation_weights": (C.c_int32, [C.c_int32, C.c_double, C.c_double, C.POINTER(C.c_float)]),
    "svdcache_basis_overlap": (C.c_int32, [C.POINTER(Shape), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "svdcache_rebase_state": (C.c_int32, [C.POINTER(Shape), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "svdcache_basis_similarity": (C.c_int32, [C.POINTER(Shape), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                              C.c_void_p, C.c_void_p, C.c_void_p]),
    "svdcache_forecast_combine": (C.c_int32, [C.POINTER(Shape), C.c_int32, C.POINTER(C.c_void_p),
                                              C.POINTER(C.c_float), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                              C.c_void_p, C.c_void_p]),
}

_lib = None


def lib_path() -> str:
    return os.path.join(PKG_DIR, "libsvdcache.so")


def exported_symbols():
    return sorted(EXPORTS)


def load_library():
    """Load libsvdcache.so from the package directory; raises if it was not built."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it with `python -m paper_2601_07396_amd.build` "
                           "(there is no fallback path)")
    lib = C.CDLL(path)
    for name, (res, args) in EXPORTS.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def svdcache_version() -> int:
    return load_library().svdcache_version()


def svdcache_strerror(code: int) -> str:
    return load_library().svdcache_strerror(code).decode()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _need_gpu(*ts):
    for t in ts:
        if t is not None and not t.is_cuda:
            raise RuntimeError("svdcache: tensors must live in GPU memory (no CPU path exists)")


def make_shape(F: torch.Tensor, k: int, precision: int = SVDC_PRECISE) -> Shape:
    """Shape descriptor of a feature tensor [B, N, D] (or [N, D]) whose last dim is contiguous."""
    if F.dim() == 2:
        F = F.unsqueeze(0)
    if F.dim() != 3 or F.stride(2) != 1:
        raise ValueError("F must be [B, N, D] with a contiguous last dimension")
    if F.dtype not in _DTYPES:
        raise ValueError("F must be float32 or bfloat16")
    B, N, D = F.shape
    bs = F.stride(0) if B > 1 else max(F.stride(0), (N - 1) * F.stride(1) + D)
    return Shape(B, N, D, k, F.stride(1), bs, _DTYPES[F.dtype], precision)


_TORCH_OF = {SVDC_F32: torch.float32, SVDC_BF16: torch.bfloat16}


def _like_features(shape: Shape, **tensors):
    """The C ABI describes F, R, Fhat, X and R_prev by ONE (ldf, block_stride, dtype): refuse a tensor whose own
    layout differs (e.g. `empty_like` of a row-strided view comes back contiguous), which the kernels would
    otherwise address with the wrong strides, past the end of its allocation."""
    for name, t in tensors.items():
        if t is None:
            continue
        if t.dtype != _TORCH_OF[shape.dtype]:
            raise ValueError(f"{name}: dtype {t.dtype} differs from the feature dtype {_TORCH_OF[shape.dtype]}")
        u = t.unsqueeze(0) if t.dim() == 2 else t
        if u.dim() != 3 or tuple(u.shape) != (shape.B, shape.N, shape.D):
            raise ValueError(f"{name}: shape {tuple(t.shape)} is not [B={shape.B}, N={shape.N}, D={shape.D}]")
        if u.stride(2) != 1 or u.stride(1) != shape.ldf or (shape.B > 1 and u.stride(0) != shape.block_stride):
            raise ValueError(f"{name}: strides {tuple(u.stride())} differ from the features' "
                             f"(block {shape.block_stride}, row {shape.ldf}, 1)")


def _dense_f32(count: int, what: str, **tensors):
    """V, S, C and their like are float32, contiguous, with exactly the element count the shape implies."""
    for name, t in tensors.items():
        if t is None:
            continue
        if t.dtype != torch.float32 or not t.is_contiguous() or t.numel() != count:
            raise ValueError(f"{name}: need a contiguous float32 tensor of {count} elements ({what}), got "
                             f"{t.dtype} {tuple(t.shape)} contiguous={t.is_contiguous()}")


def _check_step_args(shape: Shape, V, packed, coefs: dict, feats: dict):
    _like_features(shape, **feats)
    _dense_f32(shape.B * shape.D * shape.k, "[B, D, k]", V=V)
    _dense_f32(shape.B * shape.N * shape.k, "[B, N, k]", **coefs)
    if packed is not None:
        need = svdcache_packed_basis_bytes(shape)
        if need == 0 or packed.numel() * packed.element_size() < need or not packed.is_contiguous():
            raise ValueError(f"packed: {packed.numel() * packed.element_size()} bytes, this shape needs {need} "
                             "(a buffer packed for another rank or width?)")


def _check(code: int, where: str):
    if code != 0:
        raise SvdcError(code, where)


SVDC_FIT_JACOBI_CAPPED, SVDC_FIT_RANK_DEFICIENT = 1, 2


def svdcache_fit_workspace_bytes(shape: Shape, p: int = 0, q: int = 0, seed: int = 0, max_sweeps: int = 0) -> int:
    fp = FitParams(p, q, seed, max_sweeps, 0)
    return load_library().svdcache_fit_workspace_bytes(C.byref(shape), C.byref(fp))


def svdcache_workspace_bytes(shape: Shape, p: int = 0, q: int = 0, seed: int = 0, max_sweeps: int = 0) -> int:
    fp = FitParams(p, q, seed, max_sweeps, 0)
    return load_library().svdcache_workspace_bytes(C.byref(shape), C.byref(fp))


def svdcache_fit_status_offset(shape: Shape, p: int = 0, q: int = 0, seed: int = 0, max_sweeps: int = 0) -> int:
    fp = FitParams(p, q, seed, max_sweeps, 0)
    return load_library().svdcache_fit_status_offset(C.byref(shape), C.byref(fp))


def svdcache_packed_basis_bytes(shape: Shape) -> int:
    return load_library().svdcache_packed_basis_bytes(C.byref(shape))


def svdcache_has_mfma_path(shape: Shape) -> bool:
    return bool(load_library().svdcache_has_mfma_path(C.byref(shape)))


def svdcache_fit_basis(shape: Shape, F, V, sigma, fro2, workspace, p: int = 0, q: int = 0, seed: int = 0,
                       max_sweeps: int = 0):
    _like_features(shape, F=F)
    _dense_f32(shape.B * shape.D * shape.k, "[B, D, k]", V=V)
    _dense_f32(shape.B * shape.k, "[B, k]", sigma=sigma)
    _dense_f32(shape.B, "[B]", fro2=fro2)
    _need_gpu(F, V, sigma, fro2, workspace)
    fp = FitParams(p, q, seed, max_sweeps, 0)
    rc = load_library().svdcache_fit_basis(C.byref(shape), C.byref(fp), _ptr(F), _ptr(V), _ptr(sigma), _ptr(fro2),
                                           _ptr(workspace), workspace.numel() * workspace.element_size(), _stream())
    _check(rc, "svdcache_fit_basis")


SVDC_STATIC_SCRATCH_BYTES = 32 << 20


def svdcache_fit_basis_static(shape: Shape, F, V, sigma, fro2, status=None, p: int = 0, q: int = 0, seed: int = 0,
                              max_sweeps: int = 0):
    """The fit on the library's static device workspace (no allocation inside the call)."""
    _like_features(shape, F=F)
    _dense_f32(shape.B * shape.D * shape.k, "[B, D, k]", V=V)
    _dense_f32(shape.B * shape.k, "[B, k]", sigma=sigma)
    _dense_f32(shape.B, "[B]", fro2=fro2)
    if status is not None and (status.dtype != torch.int32 or not status.is_contiguous() or status.numel() != shape.B):
        raise ValueError("status: need a contiguous int32 tensor of B elements")
    _need_gpu(F, V, sigma, fro2, status)
    fp = FitParams(p, q, seed, max_sweeps, 0)
    rc = load_library().svdcache_fit_basis_static(C.byref(shape), C.byref(fp), _ptr(F), _ptr(V), _ptr(sigma),
                                                  _ptr(fro2), _ptr(status), _stream())
    _check(rc, "svdcache_fit_basis_static")


def svdcache_pack_basis(shape: Shape, V, packed):
    _dense_f32(shape.B * shape.D * shape.k, "[B, D, k]", V=V)
    _need_gpu(V, packed)
    rc = load_library().svdcache_pack_basis(C.byref(shape), _ptr(V), _ptr(packed),
                                            packed.numel() * packed.element_size(), _stream())
    _check(rc, "svdcache_pack_basis")


def svdcache_full_step(shape: Shape, F, V, packed, R, S, Cout, alpha: float, init: bool):
    _check_step_args(shape, V, packed, {"S": S, "C": Cout}, {"F": F, "R": R})
    _need_gpu(F, V, packed, R, S, Cout)
    rc = load_library().svdcache_full_step(C.byref(shape), _ptr(F), _ptr(V), _ptr(packed), _ptr(R), _ptr(S),
                                           _ptr(Cout), float(alpha), int(bool(init)), _stream())
    _check(rc, "svdcache_full_step")


def svdcache_full_step_residual_ema(shape: Shape, F, V, packed, R_prev, R, S, Cout, alpha: float, alpha_r: float,
                                    init: bool):
    _check_step_args(shape, V, packed, {"S": S, "C": Cout}, {"F": F, "R": R, "R_prev": R_prev})
    _need_gpu(F, V, packed, R_prev, R, S, Cout)
    rc = load_library().svdcache_full_step_residual_ema(C.byref(shape), _ptr(F), _ptr(V), _ptr(packed), _ptr(R_prev),
                                                        _ptr(R), _ptr(S), _ptr(Cout), float(alpha), float(alpha_r),
                                                        int(bool(init)), _stream())
    _check(rc, "svdcache_full_step_residual_ema")


def svdcache_forecast(shape: Shape, S, V, packed, R, Fhat):
    _check_step_args(shape, V, packed, {"S": S}, {"R": R, "Fhat": Fhat})
    _need_gpu(S, V, packed, R, Fhat)
    rc = load_library().svdcache_forecast(C.byref(shape), _ptr(S), _ptr(V), _ptr(packed), _ptr(R), _ptr(Fhat),
                                          _stream())
    _check(rc, "svdcache_forecast")


def svdcache_packed_state_bytes(shape: Shape) -> int:
    return load_library().svdcache_packed_state_bytes(C.byref(shape))


def _check_packed_state(shape: Shape, S_packed):
    need = svdcache_packed_state_bytes(shape)
    if need == 0 or not S_packed.is_contiguous() or S_packed.numel() * S_packed.element_size() < need:
        raise ValueError(f"S_packed: {S_packed.numel() * S_packed.element_size()} bytes, this shape needs {need}")


def svdcache_pack_state(shape: Shape, S, S_packed):
    _dense_f32(shape.B * shape.N * shape.k, "[B, N, k]", S=S)
    _check_packed_state(shape, S_packed)
    _need_gpu(S, S_packed)
    rc = load_library().svdcache_pack_state(C.byref(shape), _ptr(S), _ptr(S_packed),
                                            S_packed.numel() * S_packed.element_size(), _stream())
    _check(rc, "svdcache_pack_state")


def svdcache_full_step_packed(shape: Shape, F, V, packed, R, S, Cout, S_packed, alpha: float, init: bool):
    if packed is None:
        raise ValueError("packed: the packed-state full step needs the packed basis")
    _check_step_args(shape, V, packed, {"S": S, "C": Cout}, {"F": F, "R": R})
    _check_packed_state(shape, S_packed)
    _need_gpu(F, V, packed, R, S, Cout, S_packed)
    rc = load_library().svdcache_full_step_packed(C.byref(shape), _ptr(F), _ptr(V), _ptr(packed), _ptr(R), _ptr(S),
                                                  _ptr(Cout), _ptr(S_packed),
                                                  S_packed.numel() * S_packed.element_size(), float(alpha),
                                                  int(bool(init)), _stream())
    _check(rc, "svdcache_full_step_packed")


def svdcache_forecast_packed(shape: Shape, S_packed, packed, R, Fhat):
    if packed is None:
        raise ValueError("packed: the packed-state cached step needs the packed basis")
    _like_features(shape, R=R, Fhat=Fhat)
    _check_packed_state(shape, S_packed)
    need = svdcache_packed_basis_bytes(shape)
    if need == 0 or packed.numel() * packed.element_size() < need:
        raise ValueError("packed: too small for this shape")
    _need_gpu(S_packed, packed, R, Fhat)
    rc = load_library().svdcache_forecast_packed(C.byref(shape), _ptr(S_packed), _ptr(packed), _ptr(R), _ptr(Fhat),
                                                 _stream())
    _check(rc, "svdcache_forecast_packed")


def svdcache_select_rank(sigma, fro2, tau: float, k_star, reached=None):
    """k_star [B] int32 (and reached [B] int32, optional) from sigma [B,k] float32 and fro2 [B] float32."""
    _need_gpu(sigma, fro2, k_star, reached)
    B, k = sigma.shape
    rc = load_library().svdcache_select_rank(B, k, _ptr(sigma), _ptr(fro2), float(tau), _ptr(k_star), _ptr(reached),
                                             _stream())
    _check(rc, "svdcache_select_rank")


def svdcache_truncate_basis(shape: Shape, V, sigma, k_star):
    _need_gpu(V, sigma, k_star)
    rc = load_library().svdcache_truncate_basis(C.byref(shape), _ptr(V), _ptr(sigma), _ptr(k_star), _stream())
    _check(rc, "svdcache_truncate_basis")


def svdcache_extrapolation_weights(order: int, offset: float, interval: float):
    """Host-side: the order+1 weights as a list of Python floats (float32 values)."""
    w = (C.c_float * (order + 1 if order >= 0 else 1))()
    rc = load_library().svdcache_extrapolation_weights(int(order), float(offset), float(interval), w)
    _check(rc, "svdcache_extrapolation_weights")
    return [float(x) for x in w]


def svdcache_forecast_combine(shape: Shape, S_list, weights, V, packed, R, X, Out):
    m = len(S_list)
    if m != len(weights):
        raise ValueError("one weight per state")
    _check_step_args(shape, V, packed, {f"S_list[{i}]": t for i, t in enumerate(S_list)}, {"R": R, "X": X, "Out": Out})
    _need_gpu(*S_list, V, packed, R, X, Out)
    ptrs = (C.c_void_p * max(m, 1))(*[t.data_ptr() for t in S_list])
    w = (C.c_float * max(m, 1))(*[float(x) for x in weights])
    rc = load_library().svdcache_forecast_combine(C.byref(shape), m, ptrs, w, _ptr(V), _ptr(packed), _ptr(R),
                                                  _ptr(X), _ptr(Out), _stream())
    _check(rc, "svdcache_forecast_combine")


def svdcache_basis_overlap(shape: Shape, V_old, V_new, M):
    _need_gpu(V_old, V_new, M)
    rc = load_library().svdcache_basis_overlap(C.byref(shape), _ptr(V_old), _ptr(V_new), _ptr(M), _stream())
    _check(rc, "svdcache_basis_overlap")


def svdcache_rebase_state(shape: Shape, M, S_in, S_out):
    _need_gpu(M, S_in, S_out)
    rc = load_library().svdcache_rebase_state(C.byref(shape), _ptr(M), _ptr(S_in), _ptr(S_out), _stream())
    _check(rc, "svdcache_rebase_state")


def svdcache_basis_similarity(shape: Shape, V_a, sigma_a, V_b, sigma_b, sim_dir, sim_sigma):
    _need_gpu(V_a, sigma_a, V_b, sigma_b, sim_dir, sim_sigma)
    rc = load_library().svdcache_basis_similarity(C.byref(shape), _ptr(V_a), _ptr(sigma_a), _ptr(V_b), _ptr(sigma_b),
                                                  _ptr(sim_dir), _ptr(sim_sigma), _stream())
    _check(rc, "svdcache_basis_similarity")


# ---- conveniences that only allocate (torch owns the memory) ------------------------------------

def fit_basis(F: torch.Tensor, k: int, p: int = 0, q: int = 0, seed: int = 0, max_sweeps: int = 0,
              return_status: bool = False):
    """Allocate outputs + workspace and call svdcache_fit_basis. Returns (V [B,D,k], sigma [B,k], fro2 [B]) and,
    with return_status, the per-block status words [B] int32 (SVDC_FIT_* flags) copied out of the workspace."""
    shape = make_shape(F, k)
    dev = F.device
    V = torch.empty(shape.B, shape.D, k, device=dev, dtype=torch.float32)
    sigma = torch.empty(shape.B, k, device=dev, dtype=torch.float32)
    fro2 = torch.empty(shape.B, device=dev, dtype=torch.float32)
    nbytes = svdcache_workspace_bytes(shape, p, q, seed, max_sweeps)
    if nbytes == 0:
        raise SvdcError(-2, "svdcache_workspace_bytes")
    ws = torch.empty(nbytes, device=dev, dtype=torch.uint8)
    svdcache_fit_basis(shape, F, V, sigma, fro2, ws, p, q, seed, max_sweeps)
    if not return_status:
        return V, sigma, fro2
    off = svdcache_fit_status_offset(shape, p, q, seed, max_sweeps)
    status = ws[off:off + 4 * shape.B].view(torch.int32).clone()
    return V, sigma, fro2, status


def fit_basis_for_energy(F: torch.Tensor, tau: float = 0.85, k_init: int = 32, k_max: int = 128, p: int = 0,
                         q: int = 0, seed: int = 0):
    """Rank chosen by the energy rule (Eq. 6): fit with k_init, let the device pick k*_b per block, and fit
    again with twice the rank (up to k_max) while some block has not reached tau within the fitted values
    (the sketch must be at least as wide as the rank it is asked about).  The loop and its one device-to-host
    read per pass are host policy; every arithmetic step is a library call.
    Returns (V [B,D,k] with the columns >= k*_b zeroed, sigma [B,k] likewise, fro2 [B], k_star [B] int32,
    reached [B] int32) where k is the rank of the last fit."""
    if F.dim() == 2:
        F = F.unsqueeze(0)
    B, N, D = F.shape
    k = max(1, min(k_init, N, D))
    while True:
        V, sigma, fro2 = fit_basis(F, k, p, q, seed)
        k_star = torch.empty(B, dtype=torch.int32, device=F.device)
        reached = torch.empty(B, dtype=torch.int32, device=F.device)
        svdcache_select_rank(sigma, fro2, tau, k_star, reached)
        k_next = min(2 * k, k_max, N, D)
        if bool(reached.all()) or k_next <= k:
            break
        k = k_next
    svdcache_truncate_basis(make_shape(F, k), V, sigma, k_star)
    return V, sigma, fro2, k_star, reached


def save_basis(path: str, V: torch.Tensor, sigma: torch.Tensor, fro2: Optional[torch.Tensor] = None):
    """Write a fitted basis to a file (numpy .npz, plain arrays only): the one-time SVD of a model is done
    offline on a reference prompt and its V and sigma are reused for every later prompt (Sec. 3.3)."""
    import numpy as np
    arrays = {"V": V.detach().float().cpu().numpy(), "sigma": sigma.detach().float().cpu().numpy()}
    if fro2 is not None:
        arrays["fro2"] = fro2.detach().float().cpu().numpy()
    with open(path, "wb") as f:
        np.savez(f, **arrays)


def load_basis(path: str, device="cuda:0"):
    """(V [B,D,k], sigma [B,k], fro2 [B] or None) from a file written by save_basis, as float32 tensors on
    `device`.  Nothing in the file is executed (no pickled objects are accepted)."""
    import numpy as np
    with np.load(path, allow_pickle=False) as z:
        V = torch.from_numpy(z["V"]).to(device).contiguous()
        sigma = torch.from_numpy(z["sigma"]).to(device).contiguous()
        fro2 = torch.from_numpy(z["fro2"]).to(device).contiguous() if "fro2" in z.files else None
    if V.dim() != 3 or sigma.shape != (V.shape[0], V.shape[2]):
        raise ValueError("not a basis file: V must be [B, D, k] and sigma [B, k]")
    return V, sigma, fro2


def alloc_packed_state(shape: Shape, device):
    """Buffer for the packed coefficient state, or None when the shape has no matrix-core path."""
    n = svdcache_packed_state_bytes(shape)
    return torch.empty(n, device=device, dtype=torch.uint8) if n else None


def pack_basis(shape: Shape, V: torch.Tensor):
    """Packed copy of V for the matrix-core kernels, or None when the shape has no such path."""
    n = svdcache_packed_basis_bytes(shape)
    if n == 0:
        return None
    packed = torch.empty(n, device=V.device, dtype=torch.uint8)
    svdcache_pack_basis(shape, V, packed)
    return packed
