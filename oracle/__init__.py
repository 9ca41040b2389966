"""fp64 CPU oracle of the low-rank delta-rule recurrence (ParallelFlow, arXiv 2504.00492).

TEST INFRASTRUCTURE ONLY: imported by tests/, by ``__graft_entry__.smoke()`` and by the
``cpu_baseline`` leg of ``bench.py``.  Nothing in the product package imports this, and this
package imports nothing from the product package.

* ``pf_oracle.c``      token-by-token recurrence (Section 1.1 recurrence/readout, Section 3.1
                       discretised dynamics, delta mapping of the Remark in Section 3.1), plain C.
                       ``delta_product_fwd`` (product form of the rank-r transition, the contrast
                       case) is that same routine on the sequence of L*r virtual tokens.
                       ``delta_compare`` runs that recurrence per head and returns only error sums
                       against a candidate result (every head of a full-size workload).
* ``chunk_flow_ref.py`` numpy fp64 transcription of the chunk flow (Theorem 3.2, Proposition 3.3,
                       Theorem 3.4); used by the tests only, to pin the recurrence from a second,
                       independent direction.

Parity status: every function here is pinned by tests/test_oracle_pins.py (closed forms,
textbook special cases, library routines, brute force); nothing is "parity unpinned".
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pf_oracle.c")
_LIB = os.path.join(_HERE, "libpf_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile pf_oracle.c with gcc (no HIP, no ROCm headers).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        fp = ctypes.POINTER(ctypes.c_float)
        lib.pf_oracle_flow_head.restype = ctypes.c_int
        lib.pf_oracle_flow_head.argtypes = [dp, dp, dp, dp, dp, dp, dp] + [ctypes.c_int] * 4
        lib.pf_oracle_delta_fwd.restype = ctypes.c_int
        lib.pf_oracle_delta_fwd.argtypes = [fp, fp, fp, fp, fp, dp, dp] + [ctypes.c_int] * 6
        lib.pf_oracle_delta_compare.restype = ctypes.c_int
        lib.pf_oracle_delta_compare.argtypes = [fp] * 7 + [dp] * 5 + [ctypes.c_int] * 6
        lib.pf_oracle_max_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _dptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _fptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def max_threads() -> int:
    return int(_load().pf_oracle_max_threads())


def flow_head(A, Atil, Bm, Q, S0=None, want_O=True):
    """General-driver recurrence for one head.

    A, Bm: [L, R, dk]; Atil: [L, R, dv]; Q: [L, dk]; S0: [dv, dk] or None.
    Returns (O [L, dv] or None, S_L [dv, dk]) in float64.
    """
    A = np.ascontiguousarray(A, dtype=np.float64)
    Atil = np.ascontiguousarray(Atil, dtype=np.float64)
    Bm = np.ascontiguousarray(Bm, dtype=np.float64)
    Q = np.ascontiguousarray(Q, dtype=np.float64)
    L, R, dk = A.shape
    dv = Atil.shape[2]
    assert Bm.shape == (L, R, dk) and Atil.shape == (L, R, dv) and Q.shape == (L, dk)
    S0c = None if S0 is None else np.ascontiguousarray(S0, dtype=np.float64)
    if S0c is not None:
        assert S0c.shape == (dv, dk)
    O = np.empty((L, dv), dtype=np.float64) if want_O else None
    SL = np.empty((dv, dk), dtype=np.float64)
    rc = _load().pf_oracle_flow_head(_dptr(A), _dptr(Atil), _dptr(Bm), _dptr(Q), _dptr(S0c),
                                     _dptr(O), _dptr(SL), L, R, dk, dv)
    if rc != 0:
        raise MemoryError("pf_oracle_flow_head")
    return O, SL


def delta_fwd(Q, K, V, beta, S0=None, want_O=True, nthreads=0):
    """Delta-rule recurrence over independent heads.

    Q: [..., L, dk]; K: [..., L, R, dk]; V: [..., L, R, dv]; beta: [..., L, R];
    S0: [..., dv, dk] or None.  Leading dims (e.g. B, H) are flattened.  Inputs are taken as
    float32 (a bf16 workload passes its already-rounded values) and widened to float64.
    Returns (O [..., L, dv] or None, S_L [..., dv, dk]) in float64.
    """
    K = np.ascontiguousarray(K, dtype=np.float32)
    lead = K.shape[:-3]
    L, R, dk = K.shape[-3:]
    V = np.ascontiguousarray(V, dtype=np.float32)
    dv = V.shape[-1]
    Q = np.ascontiguousarray(Q, dtype=np.float32)
    beta = np.ascontiguousarray(beta, dtype=np.float32)
    assert V.shape == lead + (L, R, dv) and Q.shape == lead + (L, dk) and beta.shape == lead + (L, R)
    N = int(np.prod(lead)) if lead else 1
    S0c = None
    if S0 is not None:
        S0c = np.ascontiguousarray(S0, dtype=np.float32)
        assert S0c.shape == lead + (dv, dk)
    O = np.empty(lead + (L, dv), dtype=np.float64) if want_O else None
    SL = np.empty(lead + (dv, dk), dtype=np.float64)
    rc = _load().pf_oracle_delta_fwd(_fptr(Q), _fptr(K), _fptr(V), _fptr(beta), _fptr(S0c),
                                     _dptr(O), _dptr(SL), N, L, R, dk, dv, int(nthreads))
    if rc != 0:
        raise MemoryError("pf_oracle_delta_fwd")
    return O, SL


def delta_compare(Q, K, V, beta, S0, O_cand, SL_cand=None, nthreads=0):
    """Hold a candidate result against the recurrence, head by head, without keeping the fp64
    outputs: runs ``delta_fwd`` per head inside the C library and returns only sums.

    Inputs as for ``delta_fwd`` with ONE leading axis N (heads); O_cand [N, L, dv] and
    SL_cand [N, dv, dk] (or None) are the candidate's outputs as float32.
    Returns a dict of float64 arrays: err2 [N, L] = |o_t(cand) - o_t|^2, ref2 [N, L] = |o_t|^2,
    maxabs [N], and s_err2 [N], s_ref2 [N] for the final state (None without SL_cand)."""
    K = np.ascontiguousarray(K, dtype=np.float32)
    V = np.ascontiguousarray(V, dtype=np.float32)
    Q = np.ascontiguousarray(Q, dtype=np.float32)
    beta = np.ascontiguousarray(beta, dtype=np.float32)
    N, L, R, dk = K.shape
    dv = V.shape[-1]
    assert V.shape == (N, L, R, dv) and Q.shape == (N, L, dk) and beta.shape == (N, L, R)
    S0c = None if S0 is None else np.ascontiguousarray(S0, dtype=np.float32)
    assert S0c is None or S0c.shape == (N, dv, dk)
    Oc = np.ascontiguousarray(O_cand, dtype=np.float32)
    assert Oc.shape == (N, L, dv)
    Sc = None if SL_cand is None else np.ascontiguousarray(SL_cand, dtype=np.float32)
    assert Sc is None or Sc.shape == (N, dv, dk)
    err2 = np.zeros((N, L)); ref2 = np.zeros((N, L)); maxabs = np.zeros(N)
    s_err2 = np.zeros(N); s_ref2 = np.zeros(N)
    rc = _load().pf_oracle_delta_compare(_fptr(Q), _fptr(K), _fptr(V), _fptr(beta), _fptr(S0c), _fptr(Oc), _fptr(Sc),
                                         _dptr(err2), _dptr(ref2), _dptr(maxabs), _dptr(s_err2), _dptr(s_ref2),
                                         N, L, R, dk, dv, int(nthreads))
    if rc != 0:
        raise MemoryError("pf_oracle_delta_compare")
    return dict(err2=err2, ref2=ref2, maxabs=maxabs, s_err2=None if Sc is None else s_err2,
                s_ref2=None if Sc is None else s_ref2)


def delta_product_fwd(Q, K, V, beta, S0=None, want_O=True, nthreads=0):
    """Product form of the rank-r transition: the r (k, v, beta) triples of a token are applied one
    after another, S <- S (I - beta k k^T) + beta v k^T for j = 0 .. r-1, and o_t = S q_t is read after
    the r-th.  By definition this is the rank-1 delta rule (Section 1.3) over the L*r virtual tokens
    in (t, j) order, read out at every r-th of them, so it is computed by ``delta_fwd`` on that
    re-indexed sequence (queries of the other virtual tokens are zero and their outputs dropped).
    Shapes as for ``delta_fwd``."""
    K = np.ascontiguousarray(K, dtype=np.float32)
    V = np.ascontiguousarray(V, dtype=np.float32)
    Q = np.ascontiguousarray(Q, dtype=np.float32)
    beta = np.ascontiguousarray(beta, dtype=np.float32)
    lead = K.shape[:-3]
    L, R, dk = K.shape[-3:]
    dv = V.shape[-1]
    Kv = K.reshape(lead + (L * R, 1, dk))
    Vv = V.reshape(lead + (L * R, 1, dv))
    bv = beta.reshape(lead + (L * R, 1))
    Qv = np.zeros(lead + (L, R, dk), dtype=np.float32)
    Qv[..., R - 1, :] = Q
    Qv = Qv.reshape(lead + (L * R, dk))
    Ov, SL = delta_fwd(Qv, Kv, Vv, bv, S0, want_O=want_O, nthreads=nthreads)
    if not want_O:
        return None, SL
    return np.ascontiguousarray(Ov.reshape(lead + (L, R, dv))[..., R - 1, :]), SL
