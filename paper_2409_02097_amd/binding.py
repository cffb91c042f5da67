"""ctypes binding of include/linfusion.h: same names, argument marshalling only.

Tensors are torch tensors used purely as device-memory handles (`data_ptr()`), and the stream
is torch's current HIP stream unless one is given.  Every step of the method runs inside the
shared library; there is no fallback.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "liblinfusion.so"

DTYPE_F32, DTYPE_F16, DTYPE_BF16 = 0, 1, 2
PHI_ELU_PLUS_ONE, PHI_RELU, PHI_IDENTITY = 0, 1, 2
FLAG_NONE, FLAG_UNNORMALIZED, FLAG_FORCE_SPLIT, FLAG_FORCE_FUSED, FLAG_FORCE_SOLO = 0, 1, 2, 4, 8

_lib = None


class LinFusionError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: status {status} ({linfusion_status_string(status)})")
        self.status = status


def library_path() -> str:
    """The in-tree library; LINFUSION_LIBRARY names another build of it (for A/B timing of two builds)."""
    return os.environ.get("LINFUSION_LIBRARY") or os.path.join(_HERE, _LIB_NAME)


def library() -> ctypes.CDLL:
    """Loads the built shared library; builds it first if it has never been built."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        from . import build as _build
        _build.build()
    lib = ctypes.CDLL(path)
    vp, i32, i64, f32, u32, sz = (ctypes.c_void_p, ctypes.c_int, ctypes.c_longlong, ctypes.c_float,
                                  ctypes.c_uint, ctypes.c_size_t)
    lib.linfusion_attn_fwd_ex.argtypes = [vp, vp, vp, vp, i32, i32, i64, i32, i32, i32, f32, u32, vp, sz, vp]
    lib.linfusion_attn_fwd_ex.restype = i32
    st3 = ctypes.POINTER(ctypes.c_longlong * 3)
    lib.linfusion_attn_fwd_strided.argtypes = [vp, vp, vp, vp, i32, i32, i64, i32, i32, i32, f32, u32, st3, st3, st3,
                                               vp, sz, vp]
    lib.linfusion_attn_fwd_strided.restype = i32
    lib.linfusion_attn_fwd_profile.argtypes = [vp, vp, vp, vp, i32, i32, i64, i32, i32, i32, f32, u32, st3, st3, st3,
                                               vp, sz, vp, ctypes.POINTER(ctypes.c_void_p * 4)]
    lib.linfusion_attn_fwd_profile.restype = i32
    lib.linfusion_attn_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i64, i32, i32, i32, f32, u32, vp, sz, vp]
    lib.linfusion_attn_bwd.restype = i32
    lib.linfusion_attn_bwd_strided.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i64, i32, i32, i32, f32, u32,
                                               st3, st3, st3, st3, st3, vp, sz, vp]
    lib.linfusion_attn_bwd_strided.restype = i32
    lib.linfusion_attn_workspace_state_offset.argtypes = [i32, i32, i64, i32, i32]
    lib.linfusion_attn_workspace_state_offset.restype = sz
    lib.linfusion_attn_bwd_workspace_bytes.argtypes = [i32, i32, i64, i32, i32]
    lib.linfusion_attn_bwd_workspace_bytes.restype = sz
    lib.linfusion_attn_fwd_mlp.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i64, i32, i32, i32, f32,
                                           f32, f32, u32, vp, sz, vp, ctypes.POINTER(ctypes.c_void_p * 4)]
    lib.linfusion_attn_fwd_mlp.restype = i32
    st2 = ctypes.POINTER(ctypes.c_longlong * 2)
    lib.linfusion_attn_fwd_mlp_strided.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i64, i32, i32, i32,
                                                   f32, f32, f32, u32, st2, st2, vp, sz, vp,
                                                   ctypes.POINTER(ctypes.c_void_p * 4)]
    lib.linfusion_attn_fwd_mlp_strided.restype = i32
    lib.linfusion_attn_mlp_workspace_bytes.argtypes = [i32, i32, i64, i32, i32]
    lib.linfusion_attn_mlp_workspace_bytes.restype = sz
    lib.linfusion_attn_fwd_qv.argtypes = [vp, vp, vp, vp, i32, i32, i64, i32, i32, i32, i32, f32, u32, vp, sz, vp,
                                          ctypes.POINTER(ctypes.c_void_p * 4)]
    lib.linfusion_attn_fwd_qv.restype = i32
    lib.linfusion_attn_qv_workspace_bytes.argtypes = [i32, i32, i64, i32, i32, i32]
    lib.linfusion_attn_qv_workspace_bytes.restype = sz
    lib.linfusion_attn_last_error.argtypes = [vp, sz, i32, i32, i64, i32, i32, vp]
    lib.linfusion_attn_last_error.restype = i32
    lib.linfusion_attn_workspace_bytes.argtypes = [i32, i32, i64, i32, i32]
    lib.linfusion_attn_workspace_bytes.restype = sz
    for name in ("linfusion_attn_fwd", "linfusion_attn_fwd_f16", "linfusion_attn_fwd_bf16", "linfusion_attn_fwd_f32"):
        fn = getattr(lib, name)
        fn.argtypes = [vp, vp, vp, vp, i32, i32, i64, i32, i32, f32, vp]
        fn.restype = i32
    lib.linfusion_attn_state.argtypes = [vp, vp, vp, i32, i32, i64, i32, i32, i32, vp, sz, vp]
    lib.linfusion_attn_state.restype = i32
    lib.linfusion_release.argtypes = []
    lib.linfusion_release.restype = None
    lib.linfusion_status_string.argtypes = [i32]
    lib.linfusion_status_string.restype = ctypes.c_char_p
    lib.linfusion_version.argtypes = []
    lib.linfusion_version.restype = i32
    lib.linfusion_attn_fwd_static.argtypes = [vp, vp, vp, vp, i32, i32, i64, i32, i32, i32, f32, u32, vp]
    lib.linfusion_attn_fwd_static.restype = i32
    lib.linfusion_attn_static_scratch_bytes.argtypes = []
    lib.linfusion_attn_static_scratch_bytes.restype = sz
    lib.linfusion_init.argtypes = []
    lib.linfusion_init.restype = i32
    lib.linfusion_hbm_probe.argtypes = [i32, i32, vp, vp, vp, vp, sz, i32, vp, vp]
    lib.linfusion_hbm_probe.restype = i32
    lib.linfusion_launch_probe.argtypes = [i32, i32, vp, vp]
    lib.linfusion_launch_probe.restype = i32
    lib.linfusion_set_tuning.argtypes = [i32]
    lib.linfusion_set_tuning.restype = None
    lib.linfusion_attn_apply_kernel.argtypes = [i32, i32, i64, i32, i32, u32]
    lib.linfusion_attn_apply_kernel.restype = ctypes.c_char_p
    lib.linfusion_attn_plan.argtypes = [i32, i32, i64, i32, i32, u32, ctypes.POINTER(ctypes.c_int * 4)]
    lib.linfusion_attn_plan.restype = i32
    _lib = lib
    return lib


def _dtype_code(t) -> int:
    import torch
    return {torch.float32: DTYPE_F32, torch.float16: DTYPE_F16, torch.bfloat16: DTYPE_BF16}[t.dtype]


def _stream_ptr(stream) -> int:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def _check_layout(*tensors):
    shape = tensors[0].shape
    for t in tensors:
        if t.dim() != 4 or t.shape != shape or not t.is_contiguous() or t.dtype != tensors[0].dtype:
            raise ValueError("q, k, v, out must be contiguous [B, H, N, d] tensors of one dtype and shape")
        if not t.is_cuda:
            raise ValueError("tensors must live in device memory")
    return shape


def _check_views(q, k, v, out):
    """[B, H, N, d]-shaped views with any batch / head / token strides and contiguous channels."""
    shape = q.shape
    for t in (q, k, v, out):
        if t.dim() != 4 or t.shape != shape or t.dtype != q.dtype or not t.is_cuda:
            raise ValueError("q, k, v, out must be [B, H, N, d]-shaped device views of one dtype and shape")
        if t.shape[3] > 1 and t.stride(3) != 1:
            raise ValueError("the d channels of a token must be contiguous")
    if k.stride() != v.stride():
        raise ValueError("k and v must share their strides")
    return shape


def _strides3(t):
    return (ctypes.c_longlong * 3)(t.stride(0), t.stride(1), t.stride(2))


def linfusion_status_string(status: int) -> str:
    return library().linfusion_status_string(int(status)).decode()


def linfusion_version() -> int:
    return library().linfusion_version()


def linfusion_attn_workspace_bytes(B: int, H: int, N: int, d: int, dtype: int) -> int:
    return int(library().linfusion_attn_workspace_bytes(B, H, N, d, dtype))


def linfusion_attn_bwd_workspace_bytes(B: int, H: int, N: int, d: int, dtype: int) -> int:
    return int(library().linfusion_attn_bwd_workspace_bytes(B, H, N, d, dtype))


def linfusion_attn_workspace_state_offset(B: int, H: int, N: int, d: int, dtype: int) -> int:
    return int(library().linfusion_attn_workspace_state_offset(B, H, N, d, dtype))


def linfusion_attn_bwd(q, k, v, dout, dq, dk, dv, feature_map: int = PHI_ELU_PLUS_ONE, eps: float = 1e-6,
                       flags: int = FLAG_NONE, workspace=None, stream=None, check: bool = True, state=None) -> int:
    """dq, dk, dv <- gradients of the mixer for upstream gradient dout (contiguous [B, H, N, d] tensors).
    `state`: optional fp32 device tensor holding the forward state of q, k, v."""
    B, H, N, d = _check_layout(q, k, v, dout, dq, dk, dv)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = library().linfusion_attn_bwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), dout.data_ptr(),
                                      state.data_ptr() if state is not None else None, dq.data_ptr(),
                                      dk.data_ptr(), dv.data_ptr(), B, H, N, d, _dtype_code(q), feature_map, eps,
                                      flags, ws_ptr, ws_bytes, _stream_ptr(stream))
    if check and rc != 0:
        raise LinFusionError(rc, "linfusion_attn_bwd")
    return rc


def linfusion_attn_qv_workspace_bytes(B: int, H: int, N: int, d_qk: int, d_v: int, dtype: int) -> int:
    return int(library().linfusion_attn_qv_workspace_bytes(B, H, N, d_qk, d_v, dtype))


def linfusion_attn_fwd_qv(q, k, v, out, feature_map: int = PHI_ELU_PLUS_ONE, eps: float = 1e-6, flags: int = FLAG_NONE,
                          workspace=None, stream=None, events=None, check: bool = True) -> int:
    """out <- mixer(q, k, v) with q, k contiguous [B, H, N, d_qk] and v, out contiguous [B, H, N, d_v], d_qk != d_v."""
    if q.shape != k.shape or v.shape != out.shape or q.shape[:3] != v.shape[:3] or q.dim() != 4:
        raise ValueError("q, k: [B, H, N, d_qk]; v, out: [B, H, N, d_v]")
    if any(not t.is_contiguous() or t.dtype != q.dtype or t.device != q.device for t in (q, k, v, out)):
        raise ValueError("q, k, v, out must be contiguous tensors of one dtype on one device")
    B, H, N, dk = q.shape
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = library().linfusion_attn_fwd_qv(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), B, H, N, dk,
                                         v.shape[3], _dtype_code(q), feature_map, eps, flags, ws_ptr, ws_bytes,
                                         _stream_ptr(stream),
                                         ctypes.byref((ctypes.c_void_p * 4)(*[ctypes.c_void_p(int(e)) for e in events]))
                                         if events is not None else None)
    if check and rc != 0:
        raise LinFusionError(rc, "linfusion_attn_fwd_qv")
    return rc


def linfusion_attn_mlp_workspace_bytes(B: int, H: int, N: int, d: int, dtype: int) -> int:
    return int(library().linfusion_attn_mlp_workspace_bytes(B, H, N, d, dtype))


def linfusion_attn_fwd_mlp(a_q, t_q, a_k, t_k, v, out, gamma_q, beta_q, gamma_k, beta_k, H: int,
                           feature_map: int = PHI_ELU_PLUS_ONE, eps: float = 1e-6, ln_eps: float = 1e-5,
                           slope: float = 0.01, flags: int = FLAG_NONE, workspace=None, stream=None,
                           events=None, check: bool = True) -> int:
    """out <- mixer(a_q + LeakyReLU(LayerNorm(t_q)), a_k + LeakyReLU(LayerNorm(t_k)), v) on token-major
    contiguous [B, N, H*d] tensors; gamma_*, beta_*: fp32 device vectors of H*d values.
    `events`: optional list of four hipEvent_t handles (ints) recorded around the kernels."""
    import torch
    ts = (a_q, t_q, a_k, t_k, v, out)
    if any(t.dim() != 3 or not t.is_contiguous() or t.shape != a_q.shape or t.dtype != a_q.dtype
           or t.device != a_q.device for t in ts):
        raise ValueError("a_q, t_q, a_k, t_k, v, out must be contiguous [B, N, H*d] tensors of one dtype and device")
    B, N, C = a_q.shape
    if C % H:
        raise ValueError("the channel count must be a multiple of H")
    for g in (gamma_q, beta_q, gamma_k, beta_k):
        if g.dtype != torch.float32 or g.numel() != C or not g.is_contiguous() or g.device != a_q.device:
            raise ValueError("gamma / beta must be contiguous fp32 vectors of H*d values on the tensors' device")
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = library().linfusion_attn_fwd_mlp(a_q.data_ptr(), t_q.data_ptr(), a_k.data_ptr(), t_k.data_ptr(), v.data_ptr(),
                                          out.data_ptr(), gamma_q.data_ptr(), beta_q.data_ptr(), gamma_k.data_ptr(),
                                          beta_k.data_ptr(), B, H, N, C // H, _dtype_code(a_q), feature_map, eps,
                                          ln_eps, slope, flags, ws_ptr, ws_bytes, _stream_ptr(stream),
                                          ctypes.byref((ctypes.c_void_p * 4)(*[ctypes.c_void_p(int(e)) for e in events]))
                                          if events is not None else None)
    if check and rc != 0:
        raise LinFusionError(rc, "linfusion_attn_fwd_mlp")
    return rc


def linfusion_attn_fwd_mlp_strided(a_q, t_q, a_k, t_k, v, out, gamma_q, beta_q, gamma_k, beta_k, H: int,
                                   feature_map: int = PHI_ELU_PLUS_ONE, eps: float = 1e-6, ln_eps: float = 1e-5,
                                   slope: float = 0.01, flags: int = FLAG_NONE, workspace=None, stream=None,
                                   events=None, check: bool = True) -> int:
    """linfusion_attn_fwd_mlp on [B, N, H*d] views with contiguous channels, e.g. column blocks of one wider
    [B, N, 5 H d] tensor; the five inputs must share their strides."""
    import torch
    ins = (a_q, t_q, a_k, t_k, v)
    for t in ins + (out,):
        if (t.dim() != 3 or t.shape != a_q.shape or t.dtype != a_q.dtype or t.device != a_q.device
                or (t.shape[2] > 1 and t.stride(2) != 1)):
            raise ValueError("a_q, t_q, a_k, t_k, v, out must be [B, N, H*d] views of one dtype and device with "
                             "contiguous channels")
    if any(t.stride() != a_q.stride() for t in ins):
        raise ValueError("a_q, t_q, a_k, t_k and v must share their strides")
    B, N, C = a_q.shape
    if C % H:
        raise ValueError("the channel count must be a multiple of H")
    for g in (gamma_q, beta_q, gamma_k, beta_k):
        if g.dtype != torch.float32 or g.numel() != C or not g.is_contiguous() or g.device != a_q.device:
            raise ValueError("gamma / beta must be contiguous fp32 vectors of H*d values on the tensors' device")
    sin = (ctypes.c_longlong * 2)(a_q.stride(0), a_q.stride(1))
    sout = (ctypes.c_longlong * 2)(out.stride(0), out.stride(1))
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = library().linfusion_attn_fwd_mlp_strided(
        a_q.data_ptr(), t_q.data_ptr(), a_k.data_ptr(), t_k.data_ptr(), v.data_ptr(), out.data_ptr(),
        gamma_q.data_ptr(), beta_q.data_ptr(), gamma_k.data_ptr(), beta_k.data_ptr(), B, H, N, C // H,
        _dtype_code(a_q), feature_map, eps, ln_eps, slope, flags, ctypes.byref(sin), ctypes.byref(sout), ws_ptr,
        ws_bytes, _stream_ptr(stream),
        ctypes.byref((ctypes.c_void_p * 4)(*[ctypes.c_void_p(int(e)) for e in events])) if events is not None else None)
    if check and rc != 0:
        raise LinFusionError(rc, "linfusion_attn_fwd_mlp_strided")
    return rc


def linfusion_attn_bwd_strided(q, k, v, dout, dq, dk, dv, feature_map: int = PHI_ELU_PLUS_ONE, eps: float = 1e-6,
                               flags: int = FLAG_NONE, workspace=None, stream=None, check: bool = True,
                               state=None) -> int:
    """linfusion_attn_bwd on [B, H, N, d] views with contiguous channels; k and v must share their strides, and
    so must dk and dv."""
    B, H, N, d = _check_views(q, k, v, dout)
    for t in (dq, dk, dv):
        if t.dim() != 4 or t.shape != q.shape or t.dtype != q.dtype or not t.is_cuda or (d > 1 and t.stride(3) != 1):
            raise ValueError("dq, dk, dv must be [B, H, N, d]-shaped device views like q with contiguous channels")
    if dk.stride() != dv.stride():
        raise ValueError("dk and dv must share their strides")
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = library().linfusion_attn_bwd_strided(q.data_ptr(), k.data_ptr(), v.data_ptr(), dout.data_ptr(),
                                              state.data_ptr() if state is not None else None, dq.data_ptr(),
                                              dk.data_ptr(), dv.data_ptr(), B, H, N, d, _dtype_code(q), feature_map,
                                              eps, flags, ctypes.byref(_strides3(q)), ctypes.byref(_strides3(k)),
                                              ctypes.byref(_strides3(dout)), ctypes.byref(_strides3(dq)),
                                              ctypes.byref(_strides3(dk)), ws_ptr, ws_bytes, _stream_ptr(stream))
    if check and rc != 0:
        raise LinFusionError(rc, "linfusion_attn_bwd_strided")
    return rc


def linfusion_attn_last_error(workspace, B: int, H: int, N: int, d: int, dtype: int, stream=None) -> int:
    """Synchronises the stream; 0, or LINFUSION_ERR_TIMEOUT (-8) if the last single-launch call gave up."""
    return int(library().linfusion_attn_last_error(workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                                   B, H, N, d, dtype, _stream_ptr(stream)))


def linfusion_attn_apply_kernel(B: int, H: int, N: int, d: int, dtype: int, flags: int = 0) -> str:
    return library().linfusion_attn_apply_kernel(B, H, N, d, dtype, flags).decode()


def linfusion_attn_plan(B: int, H: int, N: int, d: int, dtype: int, flags: int = 0):
    arr = (ctypes.c_int * 4)()
    rc = library().linfusion_attn_plan(B, H, N, d, dtype, flags, ctypes.byref(arr))
    if rc != 0:
        raise LinFusionError(rc, "linfusion_attn_plan")
    return {"path": arr[0], "reduce_wgs_per_head": arr[1], "apply_wgs_per_head": arr[2], "tile_tokens": arr[3]}


def linfusion_attn_fwd_ex(q, k, v, out, feature_map: int = PHI_ELU_PLUS_ONE, eps: float = 1e-6,
                          flags: int = FLAG_NONE, workspace=None, stream=None, check: bool = True) -> int:
    """out <- mixer(q, k, v).  `workspace`: a uint8 device tensor of at least
    linfusion_attn_workspace_bytes(...) bytes (the caller allocates it)."""
    B, H, N, d = _check_layout(q, k, v, out)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = library().linfusion_attn_fwd_ex(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), B, H, N, d,
                                         _dtype_code(q), feature_map, eps, flags, ws_ptr, ws_bytes,
                                         _stream_ptr(stream))
    if check and rc != 0:
        raise LinFusionError(rc, "linfusion_attn_fwd_ex")
    return rc


def linfusion_attn_fwd_ex_bound(q, k, v, out, feature_map: int = PHI_ELU_PLUS_ONE, eps: float = 1e-6,
                                flags: int = FLAG_NONE, workspace=None, stream=None):
    """The same call as linfusion_attn_fwd_ex with the marshalling done once: returns a function of no arguments
    that enqueues the call on the stream current now (or `stream`) and returns the status.  For loops that repeat
    one call on the same buffers: checking four tensors and looking up the stream costs this binding about 5 us a
    call, as much as two of the library's three kernel launches, which matters where a whole call takes 15 us.
    The tensors and the workspace must stay alive as long as the function is used."""
    B, H, N, d = _check_layout(q, k, v, out)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    fn = library().linfusion_attn_fwd_ex
    args = (q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), B, H, N, d, _dtype_code(q), feature_map, eps,
            flags, ws_ptr, ws_bytes, _stream_ptr(stream))

    def call() -> int:
        return fn(*args)
    return call


def linfusion_attn_fwd_static(q, k, v, out, feature_map: int = PHI_ELU_PLUS_ONE, eps: float = 1e-6,
                              flags: int = FLAG_NONE, stream=None, check: bool = True) -> int:
    """out <- mixer(q, k, v) with the library's fixed scratch array: no workspace argument, no allocation."""
    B, H, N, d = _check_layout(q, k, v, out)
    rc = library().linfusion_attn_fwd_static(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), B, H, N, d,
                                             _dtype_code(q), feature_map, eps, flags, _stream_ptr(stream))
    if check and rc != 0:
        raise LinFusionError(rc, "linfusion_attn_fwd_static")
    return rc


def linfusion_attn_static_scratch_bytes() -> int:
    return int(library().linfusion_attn_static_scratch_bytes())


def linfusion_init(check: bool = True) -> int:
    rc = library().linfusion_init()
    if check and rc != 0:
        raise LinFusionError(rc, "linfusion_init")
    return rc


def linfusion_attn_fwd_strided(q, k, v, out, feature_map: int = PHI_ELU_PLUS_ONE, eps: float = 1e-6,
                               flags: int = FLAG_NONE, workspace=None, stream=None, check: bool = True) -> int:
    """out <- mixer(q, k, v) on [B, H, N, d]-shaped VIEWS (e.g. `x.view(B, N, H, d).permute(0, 2, 1, 3)` of a
    token-major activation): the views' strides are handed to the library, nothing is copied."""
    B, H, N, d = _check_views(q, k, v, out)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = library().linfusion_attn_fwd_strided(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), B, H, N, d,
                                              _dtype_code(q), feature_map, eps, flags, ctypes.byref(_strides3(q)),
                                              ctypes.byref(_strides3(k)), ctypes.byref(_strides3(out)), ws_ptr,
                                              ws_bytes, _stream_ptr(stream))
    if check and rc != 0:
        raise LinFusionError(rc, "linfusion_attn_fwd_strided")
    return rc


def linfusion_attn_fwd_profile(q, k, v, out, feature_map, eps, flags, workspace, events, stream=None,
                               check: bool = True) -> int:
    """Like linfusion_attn_fwd_strided; `events` = four hipEvent_t handles (ints) recorded around the kernels."""
    B, H, N, d = _check_views(q, k, v, out)
    ev = (ctypes.c_void_p * 4)(*[ctypes.c_void_p(int(e)) for e in events])
    rc = library().linfusion_attn_fwd_profile(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), B, H, N, d,
                                              _dtype_code(q), feature_map, eps, flags, ctypes.byref(_strides3(q)),
                                              ctypes.byref(_strides3(k)), ctypes.byref(_strides3(out)),
                                              workspace.data_ptr(),
                                              workspace.numel() * workspace.element_size(), _stream_ptr(stream),
                                              ctypes.byref(ev))
    if check and rc != 0:
        raise LinFusionError(rc, "linfusion_attn_fwd_profile")
    return rc


def _fwd_owned(name, q, k, v, out, feature_map, eps, stream, check):
    B, H, N, d = _check_layout(q, k, v, out)
    rc = getattr(library(), name)(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), B, H, N, d,
                                  feature_map, eps, _stream_ptr(stream))
    if check and rc != 0:
        raise LinFusionError(rc, name)
    return rc


def linfusion_attn_fwd(q, k, v, out, feature_map: int = PHI_ELU_PLUS_ONE, eps: float = 1e-6, stream=None,
                       check: bool = True) -> int:
    return _fwd_owned("linfusion_attn_fwd", q, k, v, out, feature_map, eps, stream, check)


def linfusion_attn_fwd_f16(q, k, v, out, feature_map: int = PHI_ELU_PLUS_ONE, eps: float = 1e-6, stream=None,
                           check: bool = True) -> int:
    return _fwd_owned("linfusion_attn_fwd_f16", q, k, v, out, feature_map, eps, stream, check)


def linfusion_attn_fwd_bf16(q, k, v, out, feature_map: int = PHI_ELU_PLUS_ONE, eps: float = 1e-6, stream=None,
                            check: bool = True) -> int:
    return _fwd_owned("linfusion_attn_fwd_bf16", q, k, v, out, feature_map, eps, stream, check)


def linfusion_attn_fwd_f32(q, k, v, out, feature_map: int = PHI_ELU_PLUS_ONE, eps: float = 1e-6, stream=None,
                           check: bool = True) -> int:
    return _fwd_owned("linfusion_attn_fwd_f32", q, k, v, out, feature_map, eps, stream, check)


def linfusion_attn_state(k, v, state_out, feature_map: int = PHI_ELU_PLUS_ONE, workspace=None, stream=None,
                         check: bool = True) -> int:
    """state_out <- per head [d*d + d] fp32: S row-major then z."""
    B, H, N, d = _check_layout(k, v)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = library().linfusion_attn_state(k.data_ptr(), v.data_ptr(), state_out.data_ptr(), B, H, N, d,
                                        _dtype_code(k), feature_map, ws_ptr, ws_bytes, _stream_ptr(stream))
    if check and rc != 0:
        raise LinFusionError(rc, "linfusion_attn_state")
    return rc


def linfusion_hbm_probe(reads: int, writes: int, a, b, c, d, nbytes: int, workgroups: int, sink, stream=None,
                        check: bool = True) -> int:
    """One plain streaming kernel: reads `reads` of the uint8 device tensors a, b, c and writes `writes` of d,
    `nbytes` bytes each (measurement aid)."""
    ptr = lambda t: t.data_ptr() if t is not None else None
    rc = library().linfusion_hbm_probe(reads, writes, ptr(a), ptr(b), ptr(c), ptr(d), nbytes, workgroups, ptr(sink),
                                       _stream_ptr(stream))
    if check and rc != 0:
        raise LinFusionError(rc, "linfusion_hbm_probe")
    return rc


def linfusion_launch_probe(launches: int, workgroups: int, sink, stream=None, check: bool = True) -> int:
    """`launches` empty kernels back to back on the stream (measurement aid)."""
    rc = library().linfusion_launch_probe(launches, workgroups, sink.data_ptr() if sink is not None else None,
                                          _stream_ptr(stream))
    if check and rc != 0:
        raise LinFusionError(rc, "linfusion_launch_probe")
    return rc


def linfusion_set_tuning(on: bool) -> None:
    """Switches on / off whether the library looks at the LINFUSION_* environment variables (development aids)."""
    library().linfusion_set_tuning(1 if on else 0)


def linfusion_release() -> None:
    library().linfusion_release()
