"""ctypes binding of ``librodimus_hip.so`` -- argument marshalling only.

Every step of the path runs in the HIP kernels; this module checks tensor
shapes/dtypes/devices, hands raw device pointers and the current HIP stream to the
C ABI declared in ``include/rodimus.h`` and turns a non-zero status into an
exception.  torch is used for device memory and streams, nothing else.  There is no
CPU fallback: if the library has not been built, loading raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librodimus_hip.so")

F32, BF16 = 0, 1
PATH_NONE, PATH_GENERIC, PATH_MFMA = 0, 1, 2
_DTYPES = {torch.float32: F32, torch.bfloat16: BF16}

_lib = None


class RodimusError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"rodimus status {status}: {message}")
        self.status = status


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2410_06577_amd.build` "
                "(there is no fallback implementation)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
        L.rodimus_status_string.argtypes = [i]
        L.rodimus_status_string.restype = ctypes.c_char_p
        L.rodimus_chunk_scan_fwd.argtypes = [vp] * 8 + [i] * 7 + [vp, sz, vp]
        L.rodimus_chunk_scan_fwd.restype = i
        L.rodimus_chunk_scan_fwd_noalloc.argtypes = [vp] * 8 + [i] * 7 + [vp]
        L.rodimus_chunk_scan_fwd_noalloc.restype = i
        L.rodimus_chunk_scan_fwd_noalloc_scratch_bytes.argtypes = []
        L.rodimus_chunk_scan_fwd_noalloc_scratch_bytes.restype = sz
        L.rodimus_chunk_scan_workspace_bytes.argtypes = [i] * 7
        L.rodimus_chunk_scan_workspace_bytes.restype = sz
        L.rodimus_chunk_scan_path.argtypes = [i] * 7
        L.rodimus_chunk_scan_path.restype = i
        L.rodimus_decode_step.argtypes = [vp] * 7 + [i] * 5 + [vp]
        L.rodimus_decode_step.restype = i
        L.rodimus_chunk_scan_fwd_zbeta.argtypes = L.rodimus_chunk_scan_fwd.argtypes
        L.rodimus_chunk_scan_fwd_zbeta.restype = i
        L.rodimus_decode_step_zbeta.argtypes = L.rodimus_decode_step.argtypes
        L.rodimus_decode_step_zbeta.restype = i
        L.rodimus_chunk_scan_varlen_fwd.argtypes = [vp] * 5 + [i] + [vp] * 4 + [i] * 7 + [vp]
        L.rodimus_chunk_scan_varlen_fwd.restype = i
        L.rodimus_chunk_scan_varlen_fwd_gated_block.argtypes = [vp] * 10 + [i] + [vp] * 3 + [i] * 7 + [vp, sz, vp]
        L.rodimus_chunk_scan_varlen_fwd_gated_block.restype = i
        L.rodimus_hbm_stream_probe.argtypes = [vp, vp, sz, i, i, vp]
        L.rodimus_hbm_stream_probe.restype = i
        L.rodimus_chunk_scan_varlen_fwd_cut.argtypes = [vp] * 5 + [i] + [vp] * 4 + [i] * 7 + [vp, sz, vp]
        L.rodimus_chunk_scan_varlen_fwd_cut.restype = i
        L.rodimus_chunk_scan_varlen_workspace_bytes.argtypes = [i] * 7
        L.rodimus_chunk_scan_varlen_workspace_bytes.restype = sz
        L.rodimus_chunk_scan_bwd.argtypes = [vp] * 14 + [i] * 6 + [vp, sz, vp]
        L.rodimus_chunk_scan_bwd.restype = i
        L.rodimus_chunk_scan_bwd_zbeta.argtypes = L.rodimus_chunk_scan_bwd.argtypes
        L.rodimus_chunk_scan_bwd_zbeta.restype = i
        L.rodimus_chunk_scan_bwd_gated.argtypes = [vp] * 16 + [i] * 6 + [vp, sz, vp]
        L.rodimus_chunk_scan_bwd_gated.restype = i
        L.rodimus_chunk_scan_bwd_gated_workspace_bytes.argtypes = [i] * 6
        L.rodimus_chunk_scan_bwd_gated_workspace_bytes.restype = sz
        L.rodimus_chunk_scan_varlen_bwd_gated.argtypes = [vp] * 17 + [i] * 7 + [vp, sz, vp]
        L.rodimus_chunk_scan_varlen_bwd_gated.restype = i
        L.rodimus_chunk_scan_varlen_bwd_gated_workspace_bytes.argtypes = [i] * 7
        L.rodimus_chunk_scan_varlen_bwd_gated_workspace_bytes.restype = sz
        L.rodimus_chunk_scan_bwd_workspace_bytes.argtypes = [i] * 6
        L.rodimus_chunk_scan_bwd_workspace_bytes.restype = sz
        L.rodimus_chunk_scan_varlen_bwd.argtypes = [vp] * 15 + [i] * 6 + [vp, sz, vp]
        L.rodimus_chunk_scan_varlen_bwd.restype = i
        L.rodimus_chunk_scan_varlen_bwd_workspace_bytes.argtypes = [i] * 6
        L.rodimus_chunk_scan_varlen_bwd_workspace_bytes.restype = sz
        L.rodimus_chunk_scan_varlen_bwd_cut.argtypes = [vp] * 15 + [i] * 6 + [vp, sz, vp]
        L.rodimus_chunk_scan_varlen_bwd_cut.restype = i
        L.rodimus_chunk_scan_varlen_bwd_cut_workspace_bytes.argtypes = [i] * 6
        L.rodimus_chunk_scan_varlen_bwd_cut_workspace_bytes.restype = sz
        L.rodimus_chunk_scan_fwd_block.argtypes = [vp] * 5 + [i] + [vp] * 4 + [i] + [vp] * 2 + [i] * 7 + [vp, sz, vp]
        L.rodimus_chunk_scan_fwd_block.restype = i
        L.rodimus_decode_step_block.argtypes = [vp] * 5 + [i] + [vp] * 3 + [i] + [vp] * 2 + [i] * 5 + [vp]
        L.rodimus_decode_step_block.restype = i
        L.rodimus_ddts_gates.argtypes = [vp] * 9 + [ctypes.c_longlong, i, i, i, vp]
        L.rodimus_ddts_gates.restype = i
        L.rodimus_chunk_scan_fwd_gated.argtypes = [vp] * 9 + [i] * 7 + [vp, sz, vp]
        L.rodimus_chunk_scan_fwd_gated.restype = i
        L.rodimus_decode_step_gated.argtypes = [vp] * 8 + [i] * 5 + [vp]
        L.rodimus_decode_step_gated.restype = i
        L.rodimus_chunk_scan_fwd_gated_block.argtypes = [vp] * 10 + [i] + [vp] * 2 + [i] * 7 + [vp, sz, vp]
        L.rodimus_chunk_scan_fwd_gated_block.restype = i
        L.rodimus_decode_step_gated_block.argtypes = [vp] * 9 + [i] + [vp] * 2 + [i] * 5 + [vp]
        L.rodimus_decode_step_gated_block.restype = i
        L.rodimus_chunk_scan_fwd_general.argtypes = [vp] * 9 + [i] * 7 + [vp]
        L.rodimus_chunk_scan_fwd_general.restype = i
        L.rodimus_decode_step_general.argtypes = [vp] * 8 + [i] * 5 + [vp]
        L.rodimus_decode_step_general.restype = i
        L.rodimus_short_conv_fwd.argtypes = [vp] * 6 + [i] * 6 + [vp]
        L.rodimus_short_conv_fwd.restype = i
        L.rodimus_short_conv_step.argtypes = [vp] * 5 + [i] * 5 + [vp]
        L.rodimus_short_conv_step.restype = i
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().rodimus_status_string(int(status)).decode()


def _check(status: int):
    if status != 0:
        raise RodimusError(status, status_string(status))


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _require(t, name, shape, dtype, device):
    if t is None:
        return
    if tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: shape {tuple(t.shape)} != expected {tuple(shape)}")
    if t.dtype != dtype:
        raise ValueError(f"{name}: dtype {t.dtype} != expected {dtype}")
    if t.device != device:
        raise ValueError(f"{name}: device {t.device} != {device}")
    if not t.is_contiguous():
        raise ValueError(f"{name}: must be contiguous")


def _stream(device):
    return ctypes.c_void_p(torch.cuda.current_stream(device).cuda_stream)


def rodimus_chunk_scan_workspace_bytes(B, T, H, dk, dv, chunk, io_dtype) -> int:
    return int(lib().rodimus_chunk_scan_workspace_bytes(B, T, H, dk, dv, chunk, _DTYPES[io_dtype]))


def rodimus_chunk_scan_path(B, T, H, dk, dv, chunk, io_dtype) -> int:
    return int(lib().rodimus_chunk_scan_path(B, T, H, dk, dv, chunk, _DTYPES[io_dtype]))


def rodimus_chunk_scan_fwd(q, k, v, log_alpha, beta=None, S0=None, *, chunk=64, o=None, S_T=None,
                           want_state=True, workspace=None, _preact=False):
    """Chunkwise forward scan.  q,k,log_alpha [B,T,H,dk]; v,beta [B,T,H,dv]; S0 [B,H,dk,dv] fp32.

    Returns (o, S_T); S_T is None when ``want_state`` is False.  Output and workspace
    tensors are allocated with torch unless passed in.
    """
    if q.dtype not in _DTYPES:
        raise ValueError(f"q: unsupported dtype {q.dtype}")
    if not q.is_cuda:
        raise ValueError("rodimus_chunk_scan_fwd needs device tensors (no CPU path exists)")
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    dev, io = q.device, q.dtype
    _require(q, "q", (B, T, H, dk), io, dev)
    _require(k, "k", (B, T, H, dk), io, dev)
    _require(v, "v", (B, T, H, dv), io, dev)
    _require(log_alpha, "log_alpha", (B, T, H, dk), torch.float32, dev)
    if _preact and beta is None:
        raise ValueError("z_beta is required")
    _require(beta, "z_beta" if _preact else "beta", (B, T, H, dv), io if _preact else torch.float32, dev)
    _require(S0, "S0", (B, H, dk, dv), torch.float32, dev)
    if o is None:
        o = torch.empty((B, T, H, dv), dtype=io, device=dev)
    _require(o, "o", (B, T, H, dv), io, dev)
    if S_T is None and want_state:
        S_T = torch.empty((B, H, dk, dv), dtype=torch.float32, device=dev)
    _require(S_T, "S_T", (B, H, dk, dv), torch.float32, dev)
    need = rodimus_chunk_scan_workspace_bytes(B, T, H, dk, dv, chunk, io)
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    with torch.cuda.device(dev):
        entry = lib().rodimus_chunk_scan_fwd_zbeta if _preact else lib().rodimus_chunk_scan_fwd
        _check(entry(_ptr(q), _ptr(k), _ptr(v), _ptr(log_alpha), _ptr(beta), _ptr(S0), _ptr(o), _ptr(S_T),
                     B, T, H, dk, dv, int(chunk), _DTYPES[io], _ptr(workspace), ws_bytes, _stream(dev)))
    return o, S_T


def rodimus_chunk_scan_fwd_noalloc(q, k, v, log_alpha, beta, S0, o, S_T, *, chunk=64):
    """``rodimus_chunk_scan_fwd`` through the entry point that allocates nothing: the caller passes every tensor, outputs
    included (S_T may be None); a call that is cut along the sequence uses the library's built-in scratch buffer."""
    if q.dtype not in _DTYPES:
        raise ValueError(f"q: unsupported dtype {q.dtype}")
    if not q.is_cuda:
        raise ValueError("rodimus_chunk_scan_fwd_noalloc needs device tensors (no CPU path exists)")
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    dev, io = q.device, q.dtype
    _require(q, "q", (B, T, H, dk), io, dev)
    _require(k, "k", (B, T, H, dk), io, dev)
    _require(v, "v", (B, T, H, dv), io, dev)
    _require(log_alpha, "log_alpha", (B, T, H, dk), torch.float32, dev)
    _require(beta, "beta", (B, T, H, dv), torch.float32, dev)
    _require(S0, "S0", (B, H, dk, dv), torch.float32, dev)
    if o is None:
        raise ValueError("o: the caller passes the output tensor")
    _require(o, "o", (B, T, H, dv), io, dev)
    _require(S_T, "S_T", (B, H, dk, dv), torch.float32, dev)
    with torch.cuda.device(dev):
        _check(lib().rodimus_chunk_scan_fwd_noalloc(_ptr(q), _ptr(k), _ptr(v), _ptr(log_alpha), _ptr(beta), _ptr(S0), _ptr(o),
                                                    _ptr(S_T), B, T, H, dk, dv, int(chunk), _DTYPES[io], _stream(dev)))
    return o, S_T


def rodimus_chunk_scan_fwd_zbeta(q, k, v, log_alpha, z_beta, S0=None, **kw):
    """``rodimus_chunk_scan_fwd`` with the value gate given as its pre-activation z_beta [B,T,H,dv] (dtype of v)."""
    return rodimus_chunk_scan_fwd(q, k, v, log_alpha, z_beta, S0, _preact=True, **kw)


def rodimus_chunk_scan_bwd_gated(q, k, v, z_g, z_tau, z_beta, S0, d_o, dS_T=None, *, want_dS0=True, workspace=None):
    """Backward of ``rodimus_chunk_scan_fwd_gated``: cotangents of the raw q, k, v, of the pre-activations z_g, z_tau,
    z_beta (None: no value gate) and of S0.  Returns a dict ``dq, dk, dv, dz_g, dz_tau, dz_beta, dS0``."""
    if q.dtype not in _DTYPES:
        raise ValueError(f"q: unsupported dtype {q.dtype}")
    if not q.is_cuda:
        raise ValueError("rodimus_chunk_scan_bwd_gated needs device tensors (no CPU path exists)")
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    dev, io = q.device, q.dtype
    for name, t in (("k", k), ("z_g", z_g), ("z_tau", z_tau)):
        _require(t, name, (B, T, H, dk), io, dev)
    for name, t in (("v", v), ("z_beta", z_beta), ("d_o", d_o)):
        _require(t, name, (B, T, H, dv), io, dev)
    _require(S0, "S0", (B, H, dk, dv), torch.float32, dev)
    _require(dS_T, "dS_T", (B, H, dk, dv), torch.float32, dev)
    out = {"dq": torch.empty_like(q), "dk": torch.empty_like(k), "dv": torch.empty_like(v), "dz_g": torch.empty_like(q),
           "dz_tau": torch.empty_like(q), "dz_beta": torch.empty_like(v) if z_beta is not None else None,
           "dS0": torch.empty((B, H, dk, dv), dtype=torch.float32, device=dev) if want_dS0 else None}
    need = int(lib().rodimus_chunk_scan_bwd_gated_workspace_bytes(B, T, H, dk, dv, _DTYPES[io]))
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
    ws_bytes = workspace.numel() * workspace.element_size()
    with torch.cuda.device(dev):
        _check(lib().rodimus_chunk_scan_bwd_gated(_ptr(q), _ptr(k), _ptr(v), _ptr(z_g), _ptr(z_tau), _ptr(z_beta), _ptr(S0), _ptr(d_o),
                                                  _ptr(dS_T), _ptr(out["dq"]), _ptr(out["dk"]), _ptr(out["dv"]), _ptr(out["dz_g"]),
                                                  _ptr(out["dz_tau"]), _ptr(out["dz_beta"]), _ptr(out["dS0"]), B, T, H, dk, dv,
                                                  _DTYPES[io], _ptr(workspace), ws_bytes, _stream(dev)))
    return out


def rodimus_chunk_scan_varlen_bwd_gated(q, k, v, z_g, z_tau, z_beta, cu_seqlens, S0, d_o, dS_T=None, *, cut=False, want_dS0=True,
                                        workspace=None):
    """``rodimus_chunk_scan_bwd_gated`` over a packed variable-length batch (token tensors [total,H,.], states [N,H,dk,dv],
    cu_seqlens [N+1] int32 on the device); ``cut``: the kernels cut long sequences into segments that run side by side."""
    if q.dtype not in _DTYPES:
        raise ValueError(f"q: unsupported dtype {q.dtype}")
    if not q.is_cuda:
        raise ValueError("rodimus_chunk_scan_varlen_bwd_gated needs device tensors (no CPU path exists)")
    total, H, dk = q.shape
    dv = v.shape[-1]
    dev, io = q.device, q.dtype
    N = cu_seqlens.numel() - 1
    _require(cu_seqlens, "cu_seqlens", (N + 1,), torch.int32, dev)
    for name, t in (("k", k), ("z_g", z_g), ("z_tau", z_tau)):
        _require(t, name, (total, H, dk), io, dev)
    for name, t in (("v", v), ("z_beta", z_beta), ("d_o", d_o)):
        _require(t, name, (total, H, dv), io, dev)
    _require(S0, "S0", (N, H, dk, dv), torch.float32, dev)
    _require(dS_T, "dS_T", (N, H, dk, dv), torch.float32, dev)
    out = {"dq": torch.empty_like(q), "dk": torch.empty_like(k), "dv": torch.empty_like(v), "dz_g": torch.empty_like(q),
           "dz_tau": torch.empty_like(q), "dz_beta": torch.empty_like(v) if z_beta is not None else None,
           "dS0": torch.empty((N, H, dk, dv), dtype=torch.float32, device=dev) if want_dS0 else None}
    need = int(lib().rodimus_chunk_scan_varlen_bwd_gated_workspace_bytes(N, total, H, dk, dv, _DTYPES[io], int(bool(cut))))
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
    ws_bytes = workspace.numel() * workspace.element_size()
    with torch.cuda.device(dev):
        _check(lib().rodimus_chunk_scan_varlen_bwd_gated(_ptr(q), _ptr(k), _ptr(v), _ptr(z_g), _ptr(z_tau), _ptr(z_beta), _ptr(S0),
                                                         _ptr(d_o), _ptr(dS_T), _ptr(out["dq"]), _ptr(out["dk"]), _ptr(out["dv"]),
                                                         _ptr(out["dz_g"]), _ptr(out["dz_tau"]), _ptr(out["dz_beta"]), _ptr(out["dS0"]),
                                                         _ptr(cu_seqlens), N, total, H, dk, dv, _DTYPES[io], int(bool(cut)),
                                                         _ptr(workspace), ws_bytes, _stream(dev)))
    return out


def rodimus_chunk_scan_varlen_bwd_cut(q, k, v, log_alpha, cu_seqlens, beta, S0, d_o, dS_T=None, *, want_dbeta=True, want_dS0=True,
                                      workspace=None):
    """``rodimus_chunk_scan_varlen_bwd`` for a batch dominated by few long sequences: the kernels cut every sequence into
    segments that run side by side."""
    return rodimus_chunk_scan_varlen_bwd(q, k, v, log_alpha, cu_seqlens, beta, S0, d_o, dS_T, want_dbeta=want_dbeta, want_dS0=want_dS0,
                                         workspace=workspace, _cut=True)


def rodimus_chunk_scan_varlen_bwd(q, k, v, log_alpha, cu_seqlens, beta, S0, d_o, dS_T=None, *, want_dbeta=True, want_dS0=True,
                                  workspace=None, _cut=False):
    """Backward over a packed variable-length batch.  q, k, log_alpha [total,H,dk]; v, beta, d_o [total,H,dv];
    S0, dS_T [N,H,dk,dv] fp32; cu_seqlens [N+1] int32 on the device.  Returns the same dict as ``rodimus_chunk_scan_bwd``."""
    if q.dtype not in _DTYPES:
        raise ValueError(f"q: unsupported dtype {q.dtype}")
    if not q.is_cuda:
        raise ValueError("rodimus_chunk_scan_varlen_bwd needs device tensors (no CPU path exists)")
    total, H, dk = q.shape
    dv = v.shape[-1]
    dev, io = q.device, q.dtype
    N = cu_seqlens.numel() - 1
    _require(cu_seqlens, "cu_seqlens", (N + 1,), torch.int32, dev)
    _require(k, "k", (total, H, dk), io, dev)
    _require(v, "v", (total, H, dv), io, dev)
    _require(log_alpha, "log_alpha", (total, H, dk), torch.float32, dev)
    _require(beta, "beta", (total, H, dv), torch.float32, dev)
    _require(S0, "S0", (N, H, dk, dv), torch.float32, dev)
    _require(d_o, "d_o", (total, H, dv), io, dev)
    _require(dS_T, "dS_T", (N, H, dk, dv), torch.float32, dev)
    out = {"dq": torch.empty_like(q), "dk": torch.empty_like(k), "dv": torch.empty_like(v),
           "dlog_alpha": torch.empty_like(log_alpha),
           "dbeta": torch.empty((total, H, dv), dtype=torch.float32, device=dev) if want_dbeta else None,
           "dS0": torch.empty((N, H, dk, dv), dtype=torch.float32, device=dev) if want_dS0 else None}
    size_fn = lib().rodimus_chunk_scan_varlen_bwd_cut_workspace_bytes if _cut else lib().rodimus_chunk_scan_varlen_bwd_workspace_bytes
    call = lib().rodimus_chunk_scan_varlen_bwd_cut if _cut else lib().rodimus_chunk_scan_varlen_bwd
    need = int(size_fn(N, total, H, dk, dv, _DTYPES[io]))
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    with torch.cuda.device(dev):
        _check(call(_ptr(q), _ptr(k), _ptr(v), _ptr(log_alpha), _ptr(beta), _ptr(S0), _ptr(d_o), _ptr(dS_T), _ptr(out["dq"]),
                    _ptr(out["dk"]), _ptr(out["dv"]), _ptr(out["dlog_alpha"]), _ptr(out["dbeta"]), _ptr(out["dS0"]), _ptr(cu_seqlens),
                    N, total, H, dk, dv, _DTYPES[io], _ptr(workspace), ws_bytes, _stream(dev)))
    return out


def rodimus_chunk_scan_fwd_gated(q, k, v, z_g, z_tau, z_beta=None, S0=None, *, chunk=64, o=None, S_T=None,
                                 want_state=True, workspace=None):
    """Chunkwise forward scan with the DDTS gate front-end fused in: raw q, k and the pre-activations z_g, z_tau
    [B,T,H,dk], z_beta [B,T,H,dv] or None (all in q's dtype).  Returns (o, S_T)."""
    if q.dtype not in _DTYPES:
        raise ValueError(f"q: unsupported dtype {q.dtype}")
    if not q.is_cuda:
        raise ValueError("rodimus_chunk_scan_fwd_gated needs device tensors (no CPU path exists)")
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    dev, io = q.device, q.dtype
    for name, t in (("q", q), ("k", k), ("z_g", z_g), ("z_tau", z_tau)):
        if t is None:
            raise ValueError(f"{name} is required")
        _require(t, name, (B, T, H, dk), io, dev)
    _require(v, "v", (B, T, H, dv), io, dev)
    _require(z_beta, "z_beta", (B, T, H, dv), io, dev)
    _require(S0, "S0", (B, H, dk, dv), torch.float32, dev)
    if o is None:
        o = torch.empty((B, T, H, dv), dtype=io, device=dev)
    _require(o, "o", (B, T, H, dv), io, dev)
    if S_T is None and want_state:
        S_T = torch.empty((B, H, dk, dv), dtype=torch.float32, device=dev)
    _require(S_T, "S_T", (B, H, dk, dv), torch.float32, dev)
    need = rodimus_chunk_scan_workspace_bytes(B, T, H, dk, dv, chunk, io)
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    with torch.cuda.device(dev):
        _check(lib().rodimus_chunk_scan_fwd_gated(_ptr(q), _ptr(k), _ptr(v), _ptr(z_g), _ptr(z_tau), _ptr(z_beta), _ptr(S0),
                                                  _ptr(o), _ptr(S_T), B, T, H, dk, dv, int(chunk), _DTYPES[io],
                                                  _ptr(workspace), ws_bytes, _stream(dev)))
    return o, S_T


def rodimus_decode_step_gated(q, k, v, z_g, z_tau, z_beta, S, *, o=None):
    """One recurrent step with the gate front-end fused in.  q, k, z_g, z_tau [N,H,dk]; v, z_beta (or None) [N,H,dv];
    S [N,H,dk,dv] fp32, updated in place.  Returns o [N,H,dv]."""
    if q.dtype not in _DTYPES:
        raise ValueError(f"q: unsupported dtype {q.dtype}")
    if not q.is_cuda:
        raise ValueError("rodimus_decode_step_gated needs device tensors (no CPU path exists)")
    N, H, dk = q.shape
    dv = v.shape[-1]
    dev, io = q.device, q.dtype
    for name, t in (("q", q), ("k", k), ("z_g", z_g), ("z_tau", z_tau)):
        if t is None:
            raise ValueError(f"{name} is required")
        _require(t, name, (N, H, dk), io, dev)
    _require(v, "v", (N, H, dv), io, dev)
    _require(z_beta, "z_beta", (N, H, dv), io, dev)
    _require(S, "S", (N, H, dk, dv), torch.float32, dev)
    if o is None:
        o = torch.empty((N, H, dv), dtype=io, device=dev)
    _require(o, "o", (N, H, dv), io, dev)
    with torch.cuda.device(dev):
        _check(lib().rodimus_decode_step_gated(_ptr(q), _ptr(k), _ptr(v), _ptr(z_g), _ptr(z_tau), _ptr(z_beta), _ptr(S), _ptr(o),
                                               N, H, dk, dv, _DTYPES[io], _stream(dev)))
    return o


def rodimus_chunk_scan_fwd_gated_block(q, k, v, z_g, z_tau, z_beta=None, S0=None, *, x_prime=None, d=None, z_gate=None,
                                       gate_act="sigmoid", chunk=64, o=None, S_T=None, want_state=True, workspace=None):
    """The whole block around the recurrence in one call: gates and pre-processing as ``rodimus_chunk_scan_fwd_gated``, output
    stage as ``rodimus_chunk_scan_fwd_block``: y = (q / sqrt(dk) S + d .* x') .* act(z_gate).  Returns (y, S_T)."""
    if q.dtype not in _DTYPES:
        raise ValueError(f"q: unsupported dtype {q.dtype}")
    if not q.is_cuda:
        raise ValueError("rodimus_chunk_scan_fwd_gated_block needs device tensors (no CPU path exists)")
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    dev, io = q.device, q.dtype
    for name, t in (("q", q), ("k", k), ("z_g", z_g), ("z_tau", z_tau)):
        if t is None:
            raise ValueError(f"{name} is required")
        _require(t, name, (B, T, H, dk), io, dev)
    for name, t in (("v", v), ("z_beta", z_beta), ("x_prime", x_prime), ("z_gate", z_gate)):
        _require(t, name, (B, T, H, dv), io, dev)
    _require(d, "d", (H, dv), torch.float32, dev)
    _require(S0, "S0", (B, H, dk, dv), torch.float32, dev)
    if o is None:
        o = torch.empty((B, T, H, dv), dtype=io, device=dev)
    _require(o, "o", (B, T, H, dv), io, dev)
    if S_T is None and want_state:
        S_T = torch.empty((B, H, dk, dv), dtype=torch.float32, device=dev)
    _require(S_T, "S_T", (B, H, dk, dv), torch.float32, dev)
    need = rodimus_chunk_scan_workspace_bytes(B, T, H, dk, dv, chunk, io)
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    with torch.cuda.device(dev):
        _check(lib().rodimus_chunk_scan_fwd_gated_block(_ptr(q), _ptr(k), _ptr(v), _ptr(z_g), _ptr(z_tau), _ptr(z_beta), _ptr(S0),
                                                        _ptr(x_prime), _ptr(d), _ptr(z_gate), _GATE_ACTS[gate_act], _ptr(o), _ptr(S_T),
                                                        B, T, H, dk, dv, int(chunk), _DTYPES[io], _ptr(workspace), ws_bytes,
                                                        _stream(dev)))
    return o, S_T


def rodimus_decode_step_gated_block(q, k, v, z_g, z_tau, z_beta, S, *, x_prime=None, d=None, z_gate=None, gate_act="sigmoid",
                                    o=None):
    """One recurrent step of the whole block (see ``rodimus_chunk_scan_fwd_gated_block``); S updated in place.  Returns y."""
    if q.dtype not in _DTYPES:
        raise ValueError(f"q: unsupported dtype {q.dtype}")
    if not q.is_cuda:
        raise ValueError("rodimus_decode_step_gated_block needs device tensors (no CPU path exists)")
    N, H, dk = q.shape
    dv = v.shape[-1]
    dev, io = q.device, q.dtype
    for name, t in (("q", q), ("k", k), ("z_g", z_g), ("z_tau", z_tau)):
        if t is None:
            raise ValueError(f"{name} is required")
        _require(t, name, (N, H, dk), io, dev)
    for name, t in (("v", v), ("z_beta", z_beta), ("x_prime", x_prime), ("z_gate", z_gate)):
        _require(t, name, (N, H, dv), io, dev)
    _require(d, "d", (H, dv), torch.float32, dev)
    _require(S, "S", (N, H, dk, dv), torch.float32, dev)
    if o is None:
        o = torch.empty((N, H, dv), dtype=io, device=dev)
    _require(o, "o", (N, H, dv), io, dev)
    with torch.cuda.device(dev):
        _check(lib().rodimus_decode_step_gated_block(_ptr(q), _ptr(k), _ptr(v), _ptr(z_g), _ptr(z_tau), _ptr(z_beta), _ptr(x_prime),
                                                     _ptr(d), _ptr(z_gate), _GATE_ACTS[gate_act], _ptr(S), _ptr(o), N, H, dk, dv,
                                                     _DTYPES[io], _stream(dev)))
    return o


def rodimus_chunk_scan_fwd_general(q, k, v, log_alpha, log_beta_t, beta=None, S0=None, *, chunk=64, o=None, S_T=None,
                                   want_state=True):
    """Forward scan with the general transition of Sec. 3.1.1: log_beta_t [B,T,H,dv] fp32 gates the state along the value
    dimension; ``beta`` is the input gate on the value.  Returns (o, S_T)."""
    if q.dtype not in _DTYPES:
        raise ValueError(f"q: unsupported dtype {q.dtype}")
    if not q.is_cuda:
        raise ValueError("rodimus_chunk_scan_fwd_general needs device tensors (no CPU path exists)")
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    dev, io = q.device, q.dtype
    _require(k, "k", (B, T, H, dk), io, dev)
    _require(v, "v", (B, T, H, dv), io, dev)
    _require(log_alpha, "log_alpha", (B, T, H, dk), torch.float32, dev)
    if log_beta_t is None:
        raise ValueError("log_beta_t is required")
    _require(log_beta_t, "log_beta_t", (B, T, H, dv), torch.float32, dev)
    _require(beta, "beta", (B, T, H, dv), torch.float32, dev)
    _require(S0, "S0", (B, H, dk, dv), torch.float32, dev)
    if o is None:
        o = torch.empty((B, T, H, dv), dtype=io, device=dev)
    _require(o, "o", (B, T, H, dv), io, dev)
    if S_T is None and want_state:
        S_T = torch.empty((B, H, dk, dv), dtype=torch.float32, device=dev)
    _require(S_T, "S_T", (B, H, dk, dv), torch.float32, dev)
    with torch.cuda.device(dev):
        _check(lib().rodimus_chunk_scan_fwd_general(_ptr(q), _ptr(k), _ptr(v), _ptr(log_alpha), _ptr(log_beta_t), _ptr(beta),
                                                    _ptr(S0), _ptr(o), _ptr(S_T), B, T, H, dk, dv, int(chunk), _DTYPES[io],
                                                    _stream(dev)))
    return o, S_T


def rodimus_decode_step_general(q, k, v, log_alpha, log_beta_t, beta, S, *, o=None):
    """One recurrent step with the general transition.  log_beta_t [N,H,dv] fp32; S updated in place.  Returns o."""
    if q.dtype not in _DTYPES:
        raise ValueError(f"q: unsupported dtype {q.dtype}")
    if not q.is_cuda:
        raise ValueError("rodimus_decode_step_general needs device tensors (no CPU path exists)")
    N, H, dk = q.shape
    dv = v.shape[-1]
    dev, io = q.device, q.dtype
    _require(k, "k", (N, H, dk), io, dev)
    _require(v, "v", (N, H, dv), io, dev)
    _require(log_alpha, "log_alpha", (N, H, dk), torch.float32, dev)
    if log_beta_t is None:
        raise ValueError("log_beta_t is required")
    _require(log_beta_t, "log_beta_t", (N, H, dv), torch.float32, dev)
    _require(beta, "beta", (N, H, dv), torch.float32, dev)
    _require(S, "S", (N, H, dk, dv), torch.float32, dev)
    if o is None:
        o = torch.empty((N, H, dv), dtype=io, device=dev)
    _require(o, "o", (N, H, dv), io, dev)
    with torch.cuda.device(dev):
        _check(lib().rodimus_decode_step_general(_ptr(q), _ptr(k), _ptr(v), _ptr(log_alpha), _ptr(log_beta_t), _ptr(beta),
                                                 _ptr(S), _ptr(o), N, H, dk, dv, _DTYPES[io], _stream(dev)))
    return o


_GATE_ACTS = {"sigmoid": 0, "silu": 1}


def rodimus_chunk_scan_fwd_block(q, k, v, log_alpha, beta=None, S0=None, *, z_beta=None, x_prime=None, d=None, z_gate=None,
                                 gate_act="sigmoid", chunk=64, o=None, S_T=None, want_state=True, workspace=None):
    """Chunkwise forward scan with the block's output stage fused: o = (q S + d .* x') .* act(z_gate).

    x_prime, z_gate [B,T,H,dv] (dtype of v) or None; d [H,dv] fp32; the value gate as ``beta`` (fp32) or ``z_beta``."""
    if q.dtype not in _DTYPES:
        raise ValueError(f"q: unsupported dtype {q.dtype}")
    if not q.is_cuda:
        raise ValueError("rodimus_chunk_scan_fwd_block needs device tensors (no CPU path exists)")
    if beta is not None and z_beta is not None:
        raise ValueError("give beta or z_beta, not both")
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    dev, io = q.device, q.dtype
    _require(k, "k", (B, T, H, dk), io, dev)
    _require(v, "v", (B, T, H, dv), io, dev)
    _require(log_alpha, "log_alpha", (B, T, H, dk), torch.float32, dev)
    _require(beta, "beta", (B, T, H, dv), torch.float32, dev)
    _require(z_beta, "z_beta", (B, T, H, dv), io, dev)
    _require(S0, "S0", (B, H, dk, dv), torch.float32, dev)
    _require(x_prime, "x_prime", (B, T, H, dv), io, dev)
    _require(d, "d", (H, dv), torch.float32, dev)
    _require(z_gate, "z_gate", (B, T, H, dv), io, dev)
    if o is None:
        o = torch.empty((B, T, H, dv), dtype=io, device=dev)
    _require(o, "o", (B, T, H, dv), io, dev)
    if S_T is None and want_state:
        S_T = torch.empty((B, H, dk, dv), dtype=torch.float32, device=dev)
    _require(S_T, "S_T", (B, H, dk, dv), torch.float32, dev)
    need = rodimus_chunk_scan_workspace_bytes(B, T, H, dk, dv, chunk, io)
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    gate, kind = (z_beta, 1) if z_beta is not None else (beta, 0)
    with torch.cuda.device(dev):
        _check(lib().rodimus_chunk_scan_fwd_block(_ptr(q), _ptr(k), _ptr(v), _ptr(log_alpha), _ptr(gate), kind, _ptr(S0),
                                                  _ptr(x_prime), _ptr(d), _ptr(z_gate), _GATE_ACTS[gate_act], _ptr(o), _ptr(S_T),
                                                  B, T, H, dk, dv, int(chunk), _DTYPES[io], _ptr(workspace), ws_bytes, _stream(dev)))
    return o, S_T


def rodimus_decode_step_block(q, k, v, log_alpha, beta, S, *, z_beta=None, x_prime=None, d=None, z_gate=None,
                              gate_act="sigmoid", o=None):
    """One recurrent step with the block's output stage fused (see ``rodimus_chunk_scan_fwd_block``)."""
    if q.dtype not in _DTYPES:
        raise ValueError(f"q: unsupported dtype {q.dtype}")
    if not q.is_cuda:
        raise ValueError("rodimus_decode_step_block needs device tensors (no CPU path exists)")
    if beta is not None and z_beta is not None:
        raise ValueError("give beta or z_beta, not both")
    N, H, dk = q.shape
    dv = v.shape[-1]
    dev, io = q.device, q.dtype
    _require(k, "k", (N, H, dk), io, dev)
    _require(v, "v", (N, H, dv), io, dev)
    _require(log_alpha, "log_alpha", (N, H, dk), torch.float32, dev)
    _require(beta, "beta", (N, H, dv), torch.float32, dev)
    _require(z_beta, "z_beta", (N, H, dv), io, dev)
    _require(S, "S", (N, H, dk, dv), torch.float32, dev)
    _require(x_prime, "x_prime", (N, H, dv), io, dev)
    _require(d, "d", (H, dv), torch.float32, dev)
    _require(z_gate, "z_gate", (N, H, dv), io, dev)
    if o is None:
        o = torch.empty((N, H, dv), dtype=io, device=dev)
    _require(o, "o", (N, H, dv), io, dev)
    gate, kind = (z_beta, 1) if z_beta is not None else (beta, 0)
    with torch.cuda.device(dev):
        _check(lib().rodimus_decode_step_block(_ptr(q), _ptr(k), _ptr(v), _ptr(log_alpha), _ptr(gate), kind, _ptr(x_prime),
                                               _ptr(d), _ptr(z_gate), _GATE_ACTS[gate_act], _ptr(S), _ptr(o), N, H, dk, dv,
                                               _DTYPES[io], _stream(dev)))
    return o


def _scan_bwd(fn_name, gate_key, q, k, v, log_alpha, gate, S0, d_o, dS_T, want_gate, want_dS0, workspace):
    """Shared by the two dense backward calls: ``gate`` is beta (fp32) or z_beta (dtype of v), ``gate_key`` names its
    cotangent in the returned dict."""
    if q.dtype not in _DTYPES:
        raise ValueError(f"q: unsupported dtype {q.dtype}")
    if not q.is_cuda:
        raise ValueError(f"{fn_name} needs device tensors (no CPU path exists)")
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    dev, io = q.device, q.dtype
    preact = gate_key == "dz_beta"
    gate_dtype = io if preact else torch.float32
    _require(k, "k", (B, T, H, dk), io, dev)
    _require(v, "v", (B, T, H, dv), io, dev)
    _require(log_alpha, "log_alpha", (B, T, H, dk), torch.float32, dev)
    if preact and gate is None:
        raise ValueError("z_beta is required")
    _require(gate, "z_beta" if preact else "beta", (B, T, H, dv), gate_dtype, dev)
    _require(S0, "S0", (B, H, dk, dv), torch.float32, dev)
    _require(d_o, "d_o", (B, T, H, dv), io, dev)
    _require(dS_T, "dS_T", (B, H, dk, dv), torch.float32, dev)
    out = {"dq": torch.empty_like(q), "dk": torch.empty_like(k), "dv": torch.empty_like(v),
           "dlog_alpha": torch.empty_like(log_alpha),
           gate_key: torch.empty((B, T, H, dv), dtype=gate_dtype, device=dev) if want_gate else None,
           "dS0": torch.empty((B, H, dk, dv), dtype=torch.float32, device=dev) if want_dS0 else None}
    need = int(lib().rodimus_chunk_scan_bwd_workspace_bytes(B, T, H, dk, dv, _DTYPES[io]))
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    with torch.cuda.device(dev):
        _check(getattr(lib(), fn_name)(_ptr(q), _ptr(k), _ptr(v), _ptr(log_alpha), _ptr(gate), _ptr(S0), _ptr(d_o),
                                       _ptr(dS_T), _ptr(out["dq"]), _ptr(out["dk"]), _ptr(out["dv"]),
                                       _ptr(out["dlog_alpha"]), _ptr(out[gate_key]), _ptr(out["dS0"]), B, T, H, dk, dv,
                                       _DTYPES[io], _ptr(workspace), ws_bytes, _stream(dev)))
    return out


def rodimus_chunk_scan_bwd(q, k, v, log_alpha, beta, S0, d_o, dS_T=None, *, want_dbeta=True, want_dS0=True, workspace=None):
    """Backward of ``rodimus_chunk_scan_fwd``.  Returns a dict with dq, dk [B,T,H,dk] and dv [B,T,H,dv] (dtype of q),
    dlog_alpha [B,T,H,dk], dbeta [B,T,H,dv] and dS0 [B,H,dk,dv] in fp32 (dbeta / dS0 None when not wanted)."""
    return _scan_bwd("rodimus_chunk_scan_bwd", "dbeta", q, k, v, log_alpha, beta, S0, d_o, dS_T, want_dbeta, want_dS0, workspace)


def rodimus_chunk_scan_bwd_zbeta(q, k, v, log_alpha, z_beta, S0, d_o, dS_T=None, *, want_dz_beta=True, want_dS0=True,
                                 workspace=None):
    """Backward of ``rodimus_chunk_scan_fwd_zbeta``: ``z_beta`` [B,T,H,dv] (dtype of v) is the value gate's pre-activation.
    Returns the dict of ``rodimus_chunk_scan_bwd`` with ``dz_beta`` (dtype of v) in place of ``dbeta``."""
    return _scan_bwd("rodimus_chunk_scan_bwd_zbeta", "dz_beta", q, k, v, log_alpha, z_beta, S0, d_o, dS_T, want_dz_beta, want_dS0,
                     workspace)


def rodimus_hbm_stream_probe(src, dst, reads_per_write, workgroups=2048):
    """Plain streaming kernel (measurement aid): dst (any dtype, a multiple of 16 bytes) <- constant + sum of the
    ``reads_per_write`` streams of dst's size laid end to end in src."""
    if not dst.is_cuda:
        raise ValueError("rodimus_hbm_stream_probe needs device tensors (no CPU path exists)")
    nbytes = dst.numel() * dst.element_size()
    if nbytes % 16 or (reads_per_write and src.numel() * src.element_size() < nbytes * reads_per_write):
        raise ValueError("dst must hold whole 16-byte units and src reads_per_write times as many")
    with torch.cuda.device(dst.device):
        _check(lib().rodimus_hbm_stream_probe(_ptr(src) if reads_per_write else None, _ptr(dst), nbytes // 16, int(reads_per_write),
                                              int(workgroups), _stream(dst.device)))
    return dst


def rodimus_chunk_scan_varlen_fwd_gated_block(q, k, v, z_g, z_tau, cu_seqlens, z_beta=None, S0=None, *, x_prime=None, d=None,
                                              z_gate=None, gate_act="sigmoid", chunk=64, o=None, S_T=None, want_state=True,
                                              cut=False, workspace=None):
    """The whole block around the recurrence over a packed variable-length batch, one launch (three with ``cut``, which lets
    the kernels cut long sequences into segments that run side by side; the workspace is allocated here when missing).
    Returns (y [total,H,dv], S_T or None)."""
    if q.dtype not in _DTYPES:
        raise ValueError(f"q: unsupported dtype {q.dtype}")
    if not q.is_cuda:
        raise ValueError("rodimus_chunk_scan_varlen_fwd_gated_block needs device tensors (no CPU path exists)")
    total, H, dk = q.shape
    dv = v.shape[-1]
    dev, io = q.device, q.dtype
    N = cu_seqlens.numel() - 1
    _require(cu_seqlens, "cu_seqlens", (N + 1,), torch.int32, dev)
    for name, t in (("q", q), ("k", k), ("z_g", z_g), ("z_tau", z_tau)):
        if t is None:
            raise ValueError(f"{name} is required")
        _require(t, name, (total, H, dk), io, dev)
    for name, t in (("v", v), ("z_beta", z_beta), ("x_prime", x_prime), ("z_gate", z_gate)):
        _require(t, name, (total, H, dv), io, dev)
    _require(d, "d", (H, dv), torch.float32, dev)
    _require(S0, "S0", (N, H, dk, dv), torch.float32, dev)
    if o is None:
        o = torch.empty((total, H, dv), dtype=io, device=dev)
    _require(o, "o", (total, H, dv), io, dev)
    if S_T is None and want_state:
        S_T = torch.empty((N, H, dk, dv), dtype=torch.float32, device=dev)
    _require(S_T, "S_T", (N, H, dk, dv), torch.float32, dev)
    ws = None
    if cut or workspace is not None:
        need = rodimus_chunk_scan_varlen_workspace_bytes(N, total, H, dk, dv, chunk, io)
        ws = workspace
        if ws is None and need > 0:
            ws = torch.empty(need, dtype=torch.uint8, device=dev)
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    with torch.cuda.device(dev):
        _check(lib().rodimus_chunk_scan_varlen_fwd_gated_block(_ptr(q), _ptr(k), _ptr(v), _ptr(z_g), _ptr(z_tau), _ptr(z_beta), _ptr(S0),
                                                               _ptr(x_prime), _ptr(d), _ptr(z_gate), _GATE_ACTS[gate_act], _ptr(o),
                                                               _ptr(S_T), _ptr(cu_seqlens), N, total, H, dk, dv, int(chunk), _DTYPES[io],
                                                               _ptr(ws), ws_bytes, _stream(dev)))
    return o, S_T


def rodimus_chunk_scan_varlen_workspace_bytes(N, total_tokens, H, dk, dv, chunk, io_dtype):
    """Workspace bytes of ``rodimus_chunk_scan_varlen_fwd_cut`` (0: the batch is not cut along its sequences)."""
    code = _DTYPES[io_dtype] if isinstance(io_dtype, torch.dtype) else int(io_dtype)
    return int(lib().rodimus_chunk_scan_varlen_workspace_bytes(int(N), int(total_tokens), int(H), int(dk), int(dv), int(chunk), code))


def rodimus_chunk_scan_varlen_fwd_cut(q, k, v, log_alpha, cu_seqlens, beta=None, S0=None, *, z_beta=None, chunk=64, o=None,
                                      S_T=None, want_state=True, workspace=None):
    """``rodimus_chunk_scan_varlen_fwd`` for a batch of few long sequences: the kernels cut every sequence into segments that
    run side by side.  ``workspace``: a uint8 device tensor of ``rodimus_chunk_scan_varlen_workspace_bytes`` bytes
    (allocated here when missing)."""
    return rodimus_chunk_scan_varlen_fwd(q, k, v, log_alpha, cu_seqlens, beta, S0, z_beta=z_beta, chunk=chunk, o=o, S_T=S_T,
                                         want_state=want_state, _cut=True, _workspace=workspace)


def rodimus_chunk_scan_varlen_fwd(q, k, v, log_alpha, cu_seqlens, beta=None, S0=None, *, z_beta=None, chunk=64, o=None,
                                  S_T=None, want_state=True, _cut=False, _workspace=None):
    """Chunkwise forward scan over a packed variable-length batch.

    q,k,log_alpha [total,H,dk]; v, beta (fp32) or z_beta (dtype of v) [total,H,dv]; cu_seqlens [N+1] int32 on the
    device; S0, S_T [N,H,dk,dv] fp32.  Returns (o [total,H,dv], S_T or None).
    """
    if q.dtype not in _DTYPES:
        raise ValueError(f"q: unsupported dtype {q.dtype}")
    if not q.is_cuda:
        raise ValueError("rodimus_chunk_scan_varlen_fwd needs device tensors (no CPU path exists)")
    if beta is not None and z_beta is not None:
        raise ValueError("give beta or z_beta, not both")
    total, H, dk = q.shape
    dv = v.shape[-1]
    dev, io = q.device, q.dtype
    N = cu_seqlens.numel() - 1
    _require(cu_seqlens, "cu_seqlens", (N + 1,), torch.int32, dev)
    _require(q, "q", (total, H, dk), io, dev)
    _require(k, "k", (total, H, dk), io, dev)
    _require(v, "v", (total, H, dv), io, dev)
    _require(log_alpha, "log_alpha", (total, H, dk), torch.float32, dev)
    _require(beta, "beta", (total, H, dv), torch.float32, dev)
    _require(z_beta, "z_beta", (total, H, dv), io, dev)
    _require(S0, "S0", (N, H, dk, dv), torch.float32, dev)
    if o is None:
        o = torch.empty((total, H, dv), dtype=io, device=dev)
    _require(o, "o", (total, H, dv), io, dev)
    if S_T is None and want_state:
        S_T = torch.empty((N, H, dk, dv), dtype=torch.float32, device=dev)
    _require(S_T, "S_T", (N, H, dk, dv), torch.float32, dev)
    gate, kind = (z_beta, 1) if z_beta is not None else (beta, 0)
    if _cut:
        need = rodimus_chunk_scan_varlen_workspace_bytes(N, total, H, dk, dv, chunk, io)
        ws = _workspace
        if ws is None and need > 0:
            ws = torch.empty(need, dtype=torch.uint8, device=dev)
        ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
        with torch.cuda.device(dev):
            _check(lib().rodimus_chunk_scan_varlen_fwd_cut(_ptr(q), _ptr(k), _ptr(v), _ptr(log_alpha), _ptr(gate), kind, _ptr(S0),
                                                           _ptr(o), _ptr(S_T), _ptr(cu_seqlens), N, total, H, dk, dv, int(chunk),
                                                           _DTYPES[io], _ptr(ws), ws_bytes, _stream(dev)))
        return o, S_T
    with torch.cuda.device(dev):
        _check(lib().rodimus_chunk_scan_varlen_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(log_alpha), _ptr(gate), kind, _ptr(S0),
                                                   _ptr(o), _ptr(S_T), _ptr(cu_seqlens), N, total, H, dk, dv, int(chunk),
                                                   _DTYPES[io], _stream(dev)))
    return o, S_T


def rodimus_decode_step(q, k, v, log_alpha, beta, S, *, o=None, _preact=False):
    """One recurrent step.  q,k,log_alpha [N,H,dk]; v,beta [N,H,dv]; S [N,H,dk,dv] fp32, updated in place.

    Returns o [N,H,dv].
    """
    if q.dtype not in _DTYPES:
        raise ValueError(f"q: unsupported dtype {q.dtype}")
    if not q.is_cuda:
        raise ValueError("rodimus_decode_step needs device tensors (no CPU path exists)")
    N, H, dk = q.shape
    dv = v.shape[-1]
    dev, io = q.device, q.dtype
    _require(q, "q", (N, H, dk), io, dev)
    _require(k, "k", (N, H, dk), io, dev)
    _require(v, "v", (N, H, dv), io, dev)
    _require(log_alpha, "log_alpha", (N, H, dk), torch.float32, dev)
    if _preact and beta is None:
        raise ValueError("z_beta is required")
    _require(beta, "z_beta" if _preact else "beta", (N, H, dv), io if _preact else torch.float32, dev)
    _require(S, "S", (N, H, dk, dv), torch.float32, dev)
    if o is None:
        o = torch.empty((N, H, dv), dtype=io, device=dev)
    _require(o, "o", (N, H, dv), io, dev)
    with torch.cuda.device(dev):
        entry = lib().rodimus_decode_step_zbeta if _preact else lib().rodimus_decode_step
        _check(entry(_ptr(q), _ptr(k), _ptr(v), _ptr(log_alpha), _ptr(beta), _ptr(S), _ptr(o),
                     N, H, dk, dv, _DTYPES[io], _stream(dev)))
    return o


def rodimus_decode_step_zbeta(q, k, v, log_alpha, z_beta, S, *, o=None):
    """``rodimus_decode_step`` with the value gate given as its pre-activation z_beta [N,H,dv] (dtype of v)."""
    return rodimus_decode_step(q, k, v, log_alpha, z_beta, S, o=o, _preact=True)


def rodimus_ddts_gates(z_g, z_tau, z_beta, q, k, *, log_alpha=None, beta=None, q_out=None, k_out=None):
    """DDTS gate front-end.  z_g, z_tau, q, k [..., dk]; z_beta [..., dv] or None (same leading shape).

    Returns (log_alpha fp32, beta fp32 or None, q_out, k_out); q_out / k_out may be passed as q / k for in-place use.
    """
    if q.dtype not in _DTYPES:
        raise ValueError(f"q: unsupported dtype {q.dtype}")
    if not q.is_cuda:
        raise ValueError("rodimus_ddts_gates needs device tensors (no CPU path exists)")
    dev, io = q.device, q.dtype
    lead, dk = tuple(q.shape[:-1]), q.shape[-1]
    rows = 1
    for d in lead:
        rows *= d
    for name, t in (("z_g", z_g), ("z_tau", z_tau), ("q", q), ("k", k)):
        _require(t, name, lead + (dk,), io, dev)
    dv = 0
    if z_beta is not None:
        dv = z_beta.shape[-1]
        _require(z_beta, "z_beta", lead + (dv,), io, dev)
        if beta is None:
            beta = torch.empty(lead + (dv,), dtype=torch.float32, device=dev)
        _require(beta, "beta", lead + (dv,), torch.float32, dev)
    if log_alpha is None:
        log_alpha = torch.empty(lead + (dk,), dtype=torch.float32, device=dev)
    if q_out is None:
        q_out = torch.empty_like(q)
    if k_out is None:
        k_out = torch.empty_like(k)
    _require(log_alpha, "log_alpha", lead + (dk,), torch.float32, dev)
    _require(q_out, "q_out", lead + (dk,), io, dev)
    _require(k_out, "k_out", lead + (dk,), io, dev)
    with torch.cuda.device(dev):
        _check(lib().rodimus_ddts_gates(_ptr(z_g), _ptr(z_tau), _ptr(z_beta), _ptr(q), _ptr(k), _ptr(log_alpha), _ptr(beta),
                                        _ptr(q_out), _ptr(k_out), rows, dk, dv, _DTYPES[io], _stream(dev)))
    return log_alpha, beta, q_out, k_out


CONV_NONE, CONV_SILU = 0, 1
_CONV_ACTS = {"none": CONV_NONE, "silu": CONV_SILU}


def rodimus_short_conv_fwd(x, w, bias=None, state=None, *, act="silu", y=None, state_out=None, want_state=True):
    """ShortConv over a sequence.  x [B,T,C]; w [C,W] fp32; bias [C] fp32 or None; state [B,W-1,C] (x's dtype) or None.

    Returns (y [B,T,C], state_out [B,W-1,C] or None)."""
    if x.dtype not in _DTYPES:
        raise ValueError(f"x: unsupported dtype {x.dtype}")
    if not x.is_cuda:
        raise ValueError("rodimus_short_conv_fwd needs device tensors (no CPU path exists)")
    dev, io = x.device, x.dtype
    B, T, C = x.shape
    W = w.shape[-1]
    _require(x, "x", (B, T, C), io, dev)
    _require(w, "w", (C, W), torch.float32, dev)
    _require(bias, "bias", (C,), torch.float32, dev)
    _require(state, "state", (B, W - 1, C), io, dev)
    if y is None:
        y = torch.empty_like(x)
    if state_out is None and want_state:
        state_out = torch.empty((B, W - 1, C), dtype=io, device=dev)
    _require(y, "y", (B, T, C), io, dev)
    _require(state_out, "state_out", (B, W - 1, C), io, dev)
    with torch.cuda.device(dev):
        _check(lib().rodimus_short_conv_fwd(_ptr(x), _ptr(w), _ptr(bias), _ptr(state), _ptr(y), _ptr(state_out),
                                            B, T, C, W, _CONV_ACTS[act], _DTYPES[io], _stream(dev)))
    return y, state_out


def rodimus_short_conv_step(x, w, bias, state, *, act="silu", y=None):
    """One decode step of ShortConv.  x [N,C]; state [N,W-1,C] is updated in place.  Returns y [N,C]."""
    if x.dtype not in _DTYPES:
        raise ValueError(f"x: unsupported dtype {x.dtype}")
    if not x.is_cuda:
        raise ValueError("rodimus_short_conv_step needs device tensors (no CPU path exists)")
    dev, io = x.device, x.dtype
    N, C = x.shape
    W = w.shape[-1]
    _require(x, "x", (N, C), io, dev)
    _require(w, "w", (C, W), torch.float32, dev)
    _require(bias, "bias", (C,), torch.float32, dev)
    _require(state, "state", (N, W - 1, C), io, dev)
    if y is None:
        y = torch.empty_like(x)
    _require(y, "y", (N, C), io, dev)
    with torch.cuda.device(dev):
        _check(lib().rodimus_short_conv_step(_ptr(x), _ptr(w), _ptr(bias), _ptr(state), _ptr(y), N, C, W,
                                             _CONV_ACTS[act], _DTYPES[io], _stream(dev)))
    return y
