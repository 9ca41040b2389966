"""ctypes binding of include/pf.h.  Argument marshalling only: every step of the computation
runs in the HIP kernels of libpf.so.  PyTorch appears here only as the owner of device memory
and of the stream; there is no CPU or eager fallback - without libpf.so this module raises.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libpf.so")

(PF_OK, PF_ERR_NULL, PF_ERR_SHAPE, PF_ERR_UNSUPPORTED, PF_ERR_ALIGN, PF_ERR_WORKSPACE, PF_ERR_LAUNCH,
 PF_ERR_SCRATCH_LIMIT) = range(8)
PF_F32, PF_BF16 = 0, 1

EXPORTS = ["pf_version", "pf_status_str", "pf_delta_fwd_supported", "pf_delta_fwd_block", "pf_delta_fwd_workspace_bytes",
           "pf_delta_fwd_describe", "pf_delta_fwd", "pf_init", "pf_delta_fwd_static_limit", "pf_delta_fwd_static", "pf_delta_product_fwd", "pf_delta_fwd_fused_supported", "pf_delta_fwd_fused", "pf_beta_exponential", "pf_flow_fwd_supported", "pf_flow_fwd", "pf_flow_fwd_mfma_block", "pf_flow_fwd_mfma_workspace_bytes", "pf_flow_fwd_mfma", "pf_delta_chunk_supported", "pf_delta_chunk_flow", "pf_delta_chunk_scan",
           "pf_delta_chunk_sigdelta_supported", "pf_delta_chunk_sigdelta_workspace_bytes", "pf_delta_chunk_sigdelta"]


class PfError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: pf_status {status} ({pf_status_str(status)})")


def _load() -> ctypes.CDLL:
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2504_00492_amd.build` "
                          "(there is no fallback path)")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    lib.pf_version.restype = i
    lib.pf_version.argtypes = []
    lib.pf_status_str.restype = ctypes.c_char_p
    lib.pf_status_str.argtypes = [i]
    lib.pf_delta_fwd_supported.restype = i
    lib.pf_delta_fwd_supported.argtypes = [i, i, i, i, i]
    lib.pf_delta_fwd_block.restype = i
    lib.pf_delta_fwd_block.argtypes = [i, i, i, i, i]
    lib.pf_delta_fwd_workspace_bytes.restype = sz
    lib.pf_delta_fwd_workspace_bytes.argtypes = [i] * 8
    lib.pf_delta_fwd_describe.restype = sz
    lib.pf_delta_fwd_describe.argtypes = [i] * 8 + [ctypes.c_char_p, sz]
    lib.pf_delta_fwd.restype = i
    lib.pf_delta_fwd.argtypes = [vp] * 7 + [i] * 8 + [vp, sz, vp]
    lib.pf_init.restype = i
    lib.pf_init.argtypes = []
    lib.pf_delta_fwd_static_limit.restype = sz
    lib.pf_delta_fwd_static_limit.argtypes = []
    lib.pf_delta_fwd_static.restype = i
    lib.pf_delta_fwd_static.argtypes = [vp] * 7 + [i] * 8 + [vp]
    lib.pf_delta_product_fwd.restype = i
    lib.pf_delta_product_fwd.argtypes = [vp] * 7 + [i] * 8 + [vp, sz, vp]
    lib.pf_delta_fwd_fused_supported.restype = i
    lib.pf_delta_fwd_fused_supported.argtypes = [i] * 4
    lib.pf_delta_fwd_fused.restype = i
    lib.pf_delta_fwd_fused.argtypes = [vp] * 7 + [i] * 8 + [vp]
    lib.pf_beta_exponential.restype = i
    lib.pf_beta_exponential.argtypes = [vp] * 3 + [i] * 6 + [vp]
    lib.pf_flow_fwd_supported.restype = i
    lib.pf_flow_fwd_supported.argtypes = [i, i, i, i, i]
    lib.pf_flow_fwd.restype = i
    lib.pf_flow_fwd.argtypes = [vp] * 7 + [i] * 8 + [vp]
    lib.pf_flow_fwd_mfma_block.restype = i
    lib.pf_flow_fwd_mfma_block.argtypes = [i] * 5
    lib.pf_flow_fwd_mfma_workspace_bytes.restype = sz
    lib.pf_flow_fwd_mfma_workspace_bytes.argtypes = [i] * 8
    lib.pf_flow_fwd_mfma.restype = i
    lib.pf_flow_fwd_mfma.argtypes = [vp] * 7 + [i] * 8 + [vp, sz, vp]
    lib.pf_delta_chunk_supported.restype = i
    lib.pf_delta_chunk_supported.argtypes = [i] * 4
    lib.pf_delta_chunk_flow.restype = i
    lib.pf_delta_chunk_flow.argtypes = [vp] * 5 + [i] * 7 + [vp]
    lib.pf_delta_chunk_scan.restype = i
    lib.pf_delta_chunk_scan.argtypes = [vp] * 9 + [i] * 7 + [vp]
    lib.pf_delta_chunk_sigdelta_supported.restype = i
    lib.pf_delta_chunk_sigdelta_supported.argtypes = [i] * 5
    lib.pf_delta_chunk_sigdelta_workspace_bytes.restype = sz
    lib.pf_delta_chunk_sigdelta_workspace_bytes.argtypes = [i] * 5
    lib.pf_delta_chunk_sigdelta.restype = i
    lib.pf_delta_chunk_sigdelta.argtypes = [vp] * 5 + [i] * 8 + [vp, sz, vp]
    return lib


_lib = _load()


def _ptr(x):
    """torch tensor -> device address; int / None pass through."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _stream_handle(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def pf_version() -> int:
    return int(_lib.pf_version())


def pf_status_str(status: int) -> str:
    return _lib.pf_status_str(int(status)).decode()


def pf_delta_fwd_supported(d_k, d_v, r, chunk, dt) -> int:
    return int(_lib.pf_delta_fwd_supported(d_k, d_v, r, chunk, dt))


def pf_delta_fwd_block(d_k, d_v, r, chunk, dt) -> int:
    return int(_lib.pf_delta_fwd_block(d_k, d_v, r, chunk, dt))


def pf_delta_fwd_workspace_bytes(B, H, L, d_k, d_v, r, chunk, dt) -> int:
    return int(_lib.pf_delta_fwd_workspace_bytes(B, H, L, d_k, d_v, r, chunk, dt))


def pf_delta_fwd_describe(B, H, L, d_k, d_v, r, chunk, dt) -> list:
    """Kernel instantiations one pf_delta_fwd call enqueues, in launch order (list of names)."""
    need = int(_lib.pf_delta_fwd_describe(B, H, L, d_k, d_v, r, chunk, dt, None, 0))
    if need == 0:
        return []
    buf = ctypes.create_string_buffer(need + 1)
    _lib.pf_delta_fwd_describe(B, H, L, d_k, d_v, r, chunk, dt, buf, need + 1)
    return buf.value.decode().split(";")


def pf_delta_fwd(Q, K, V, beta, S0, O, S_L, B, H, L, d_k, d_v, r, chunk, dt, workspace, workspace_bytes,
                 stream=None) -> int:
    """Raw call; returns the pf_status.  Pointers may be torch tensors, ints or None."""
    return int(_lib.pf_delta_fwd(_ptr(Q), _ptr(K), _ptr(V), _ptr(beta), _ptr(S0), _ptr(O), _ptr(S_L),
                                 B, H, L, d_k, d_v, r, chunk, dt, _ptr(workspace), workspace_bytes,
                                 _stream_handle(stream)))


def pf_init() -> int:
    return int(_lib.pf_init())


def pf_delta_fwd_static_limit() -> int:
    return int(_lib.pf_delta_fwd_static_limit())


def pf_delta_fwd_static(Q, K, V, beta, S0, O, S_L, B, H, L, d_k, d_v, r, chunk, dt, stream=None) -> int:
    """Raw call (no workspace argument, nothing allocated); returns the pf_status."""
    return int(_lib.pf_delta_fwd_static(_ptr(Q), _ptr(K), _ptr(V), _ptr(beta), _ptr(S0), _ptr(O), _ptr(S_L),
                                        B, H, L, d_k, d_v, r, chunk, dt, _stream_handle(stream)))


def pf_delta_product_fwd(Q, K, V, beta, S0, O, S_L, B, H, L, d_k, d_v, r, chunk, dt, workspace, workspace_bytes,
                         stream=None) -> int:
    """Raw call; returns the pf_status.  Pointers may be torch tensors, ints or None."""
    return int(_lib.pf_delta_product_fwd(_ptr(Q), _ptr(K), _ptr(V), _ptr(beta), _ptr(S0), _ptr(O), _ptr(S_L),
                                         B, H, L, d_k, d_v, r, chunk, dt, _ptr(workspace), workspace_bytes,
                                         _stream_handle(stream)))


def pf_delta_fwd_fused_supported(d_k, d_v, r, chunk) -> int:
    return int(_lib.pf_delta_fwd_fused_supported(d_k, d_v, r, chunk))


def pf_delta_fwd_fused(Q, K, V, beta, S0, O, S_L, B, H, L, d_k, d_v, r, chunk, product=0, stream=None) -> int:
    """Raw call; returns the pf_status.  Pointers may be torch tensors, ints or None."""
    return int(_lib.pf_delta_fwd_fused(_ptr(Q), _ptr(K), _ptr(V), _ptr(beta), _ptr(S0), _ptr(O), _ptr(S_L),
                                       B, H, L, d_k, d_v, r, chunk, int(product), _stream_handle(stream)))


def pf_beta_exponential(K, beta, beta_out, B, H, L, d_k, r, dt, stream=None) -> int:
    return int(_lib.pf_beta_exponential(_ptr(K), _ptr(beta), _ptr(beta_out), B, H, L, d_k, r, dt,
                                        _stream_handle(stream)))


def pf_flow_fwd_supported(d_k, d_v, r, chunk, dt) -> int:
    return int(_lib.pf_flow_fwd_supported(d_k, d_v, r, chunk, dt))


def pf_flow_fwd(Q, A, Atil, Bm, S0, O, S_L, B, H, L, d_k, d_v, r, chunk, dt, stream=None) -> int:
    """Raw call; returns the pf_status.  Pointers may be torch tensors, ints or None."""
    return int(_lib.pf_flow_fwd(_ptr(Q), _ptr(A), _ptr(Atil), _ptr(Bm), _ptr(S0), _ptr(O), _ptr(S_L),
                                B, H, L, d_k, d_v, r, chunk, dt, _stream_handle(stream)))


def pf_flow_fwd_mfma_block(d_k, d_v, r, chunk, dt) -> int:
    return int(_lib.pf_flow_fwd_mfma_block(d_k, d_v, r, chunk, dt))


def pf_flow_fwd_mfma_workspace_bytes(B, H, L, d_k, d_v, r, chunk, dt) -> int:
    return int(_lib.pf_flow_fwd_mfma_workspace_bytes(B, H, L, d_k, d_v, r, chunk, dt))


def pf_flow_fwd_mfma(Q, A, Atil, Bm, S0, O, S_L, B, H, L, d_k, d_v, r, chunk, dt, workspace, workspace_bytes,
                     stream=None) -> int:
    """Raw call; returns the pf_status.  Pointers may be torch tensors, ints or None."""
    return int(_lib.pf_flow_fwd_mfma(_ptr(Q), _ptr(A), _ptr(Atil), _ptr(Bm), _ptr(S0), _ptr(O), _ptr(S_L),
                                     B, H, L, d_k, d_v, r, chunk, dt, _ptr(workspace), workspace_bytes,
                                     _stream_handle(stream)))


def pf_delta_chunk_supported(d_k, d_v, r, chunk) -> int:
    return int(_lib.pf_delta_chunk_supported(d_k, d_v, r, chunk))


def pf_delta_chunk_flow(Q, K, beta, Tt, Pt, B, H, L, d_k, d_v, r, chunk, stream=None) -> int:
    return int(_lib.pf_delta_chunk_flow(_ptr(Q), _ptr(K), _ptr(beta), _ptr(Tt), _ptr(Pt),
                                        B, H, L, d_k, d_v, r, chunk, _stream_handle(stream)))


def pf_delta_chunk_scan(Q, K, V, beta, Tt, Pt, S0, O, S_L, B, H, L, d_k, d_v, r, chunk, stream=None) -> int:
    return int(_lib.pf_delta_chunk_scan(_ptr(Q), _ptr(K), _ptr(V), _ptr(beta), _ptr(Tt), _ptr(Pt), _ptr(S0),
                                        _ptr(O), _ptr(S_L), B, H, L, d_k, d_v, r, chunk,
                                        _stream_handle(stream)))


def pf_delta_chunk_sigdelta_supported(d_k, d_v, r, chunk, dt) -> int:
    return int(_lib.pf_delta_chunk_sigdelta_supported(d_k, d_v, r, chunk, dt))


def pf_delta_chunk_sigdelta_workspace_bytes(B, H, L, r, chunk) -> int:
    return int(_lib.pf_delta_chunk_sigdelta_workspace_bytes(B, H, L, r, chunk))


def pf_delta_chunk_sigdelta(K, V, beta, W, U, B, H, L, d_k, d_v, r, chunk, dt, workspace, workspace_bytes,
                            stream=None) -> int:
    return int(_lib.pf_delta_chunk_sigdelta(_ptr(K), _ptr(V), _ptr(beta), _ptr(W), _ptr(U), B, H, L, d_k, d_v,
                                            r, chunk, dt, _ptr(workspace), workspace_bytes,
                                            _stream_handle(stream)))


def delta_fwd(Q, K, V, beta, S0=None, *, chunk: int, workspace=None, stream=None, product: bool = False):
    """Convenience wrapper over pf_delta_fwd (pf_delta_product_fwd with product=True) for torch CUDA tensors.

    Q [B,H,L,dk], K [B,H,L,r,dk], V [B,H,L,r,dv], beta [B,H,L,r] (float32 or bfloat16, contiguous),
    S0 [B,H,dv,dk] float32 or None.  Allocates O, S_L (and the workspace unless given) with torch,
    then makes exactly one library call.  Returns (O, S_L)."""
    import torch
    if not (Q.is_cuda and K.is_cuda and V.is_cuda and beta.is_cuda):
        raise ValueError("delta_fwd needs CUDA (HIP) tensors; there is no CPU path")
    for t in (Q, K, V, beta):
        if not t.is_contiguous():
            raise ValueError("inputs must be contiguous")
    B, H, L, r, d_k = K.shape
    d_v = V.shape[-1]
    if Q.dtype == torch.float32:
        dt = PF_F32
    elif Q.dtype == torch.bfloat16:
        dt = PF_BF16
    else:
        raise ValueError("dtype must be float32 or bfloat16")
    if not (K.dtype == V.dtype == beta.dtype == Q.dtype):
        raise ValueError("Q, K, V, beta must share one dtype")
    if Q.shape != (B, H, L, d_k) or V.shape != (B, H, L, r, d_v) or beta.shape != (B, H, L, r):
        raise ValueError("inconsistent shapes")
    if S0 is not None and (S0.dtype != torch.float32 or S0.shape != (B, H, d_v, d_k) or not S0.is_contiguous()):
        raise ValueError("S0 must be contiguous float32 [B,H,dv,dk]")
    O = torch.empty((B, H, L, d_v), dtype=Q.dtype, device=Q.device)
    S_L = torch.empty((B, H, d_v, d_k), dtype=torch.float32, device=Q.device)
    need = pf_delta_fwd_workspace_bytes(B, H, L, d_k, d_v, r, chunk, dt)
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=Q.device)
    wbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    call = pf_delta_product_fwd if product else pf_delta_fwd
    st = call(Q, K, V, beta, S0, O, S_L, B, H, L, d_k, d_v, r, chunk, dt, workspace, wbytes, stream)
    if st != PF_OK:
        raise PfError(st, call.__name__)
    return O, S_L


def flow_fwd(Q, A, Atil, Bm, S0=None, *, chunk: int, stream=None):
    """Convenience wrapper over pf_flow_fwd (general drivers of Section 3.1) for torch CUDA tensors.

    Q [B,H,L,dk], A [B,H,L,r,dk], Atil [B,H,L,r,dv], Bm [B,H,L,r,dk] (float32 or bfloat16,
    contiguous), S0 [B,H,dv,dk] float32 or None.  Allocates O and S_L with torch, then makes
    exactly one library call.  Returns (O, S_L)."""
    import torch
    for t in (Q, A, Atil, Bm):
        if not t.is_cuda:
            raise ValueError("flow_fwd needs CUDA (HIP) tensors; there is no CPU path")
        if not t.is_contiguous():
            raise ValueError("inputs must be contiguous")
    B, H, L, r, d_k = A.shape
    d_v = Atil.shape[-1]
    if Q.dtype == torch.float32:
        dt = PF_F32
    elif Q.dtype == torch.bfloat16:
        dt = PF_BF16
    else:
        raise ValueError("dtype must be float32 or bfloat16")
    if not (A.dtype == Atil.dtype == Bm.dtype == Q.dtype):
        raise ValueError("Q, A, Atil, Bm must share one dtype")
    if Q.shape != (B, H, L, d_k) or Atil.shape != (B, H, L, r, d_v) or Bm.shape != (B, H, L, r, d_k):
        raise ValueError("inconsistent shapes")
    if S0 is not None and (S0.dtype != torch.float32 or S0.shape != (B, H, d_v, d_k) or not S0.is_contiguous()):
        raise ValueError("S0 must be contiguous float32 [B,H,dv,dk]")
    O = torch.empty((B, H, L, d_v), dtype=Q.dtype, device=Q.device)
    S_L = torch.empty((B, H, d_v, d_k), dtype=torch.float32, device=Q.device)
    st = pf_flow_fwd(Q, A, Atil, Bm, S0, O, S_L, B, H, L, d_k, d_v, r, chunk, dt, stream)
    if st != PF_OK:
        raise PfError(st, "pf_flow_fwd")
    return O, S_L
