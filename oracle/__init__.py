"""CPU oracle for the SEA attention forward pass -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper around ``sea_oracle.c`` (plain C, fp64).  Only the tests,
the smoke check and the benchmark's cpu_baseline leg may import this package;
the product path never does.  It shares no code with the HIP library.

Every function takes NumPy arrays (any float dtype; converted to float64, which
holds fp32 and bf16 values exactly) and returns NumPy arrays.

Stage functions follow the paper's Sec. 3 (FAVOR+), Sec. 3.1 (estimation,
per-query top-k^ selection, mask generation), App. A.5.3 (sparse interpolation)
and Sec. 3.1.1 (sparse attention); see the header of ``sea_oracle.c``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sea_oracle.c")
_LIB = os.path.join(_HERE, "libsea_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over heads).  Returns the path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-D_GNU_SOURCE",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _RefParams(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("T", ctypes.c_int32),
                ("d", ctypes.c_int32), ("m", ctypes.c_int32), ("K", ctypes.c_int32),
                ("k_hat", ctypes.c_int32), ("k_budget", ctypes.c_int32),
                ("causal", ctypes.c_int32), ("round8", ctypes.c_int32),
                ("grouping", ctypes.c_int32), ("geometry", ctypes.c_int32), ("scale", ctypes.c_double)]


@dataclass
class Params:
    B: int
    H: int
    T: int
    d: int
    m: int
    K: int
    k_hat: int
    k_budget: int = 0
    causal: bool = True
    scale: float = 0.125
    round8: bool = False  # True for the bf16 contract (rounding of phi(Q) and key state)
    grouping: int = 0     # 0 per-query top-k^, 1 causal-per-batch (H k^ per time step over all heads)
    geometry: int = 0     # 0 fixed key buckets; 1 a causal row spreads its K columns over its own t + 1 keys

    def c(self) -> _RefParams:
        return _RefParams(self.B, self.H, self.T, self.d, self.m, self.K, self.k_hat,
                          self.k_budget, int(self.causal), int(self.round8), int(self.grouping),
                          int(self.geometry), float(self.scale))


_lib = None


def _open(path):
    """Load a build of the oracle (the tests also load deliberately broken builds this way)."""
    lib = ctypes.CDLL(path)
    lib.ref_k_hat.restype = ctypes.c_int32
    lib.ref_k_hat.argtypes = [ctypes.c_int32] * 3
    lib.ref_row_stride.restype = ctypes.c_int32
    lib.ref_row_stride.argtypes = [ctypes.POINTER(_RefParams)]
    lib.ref_sel_stride.restype = ctypes.c_int32
    lib.ref_sel_stride.argtypes = [ctypes.POINTER(_RefParams)]
    lib.ref_round8.restype = ctypes.c_double
    lib.ref_round8.argtypes = [ctypes.c_double]
    for name in ("ref_estimate", "ref_topk_mask", "ref_sparse_attn", "ref_forward", "ref_output_mix"):
        getattr(lib, name).restype = ctypes.c_int
    return lib


def _load():
    global _lib
    if _lib is None:
        _lib = _open(build())
    return _lib


def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _i32(a):
    return None if a is None else np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def k_hat_from_k(k: int, K: int, T: int) -> int:
    """k^ = max(1, round(k K / T)) -- Sec. 3.1 "Mask Generation"."""
    return int(_load().ref_k_hat(k, K, T))


def row_stride(p: Params) -> int:
    cp = p.c()
    return int(_load().ref_row_stride(ctypes.byref(cp)))


def sel_stride(p: Params) -> int:
    cp = p.c()
    return int(_load().ref_sel_stride(ctypes.byref(cp)))


def round8(x: float) -> float:
    return float(_load().ref_round8(float(x)))


def _nrows(p, rows):
    return p.T if rows is None else len(rows)


def estimate(p: Params, Q, K, W, seq_len=None, rows=None):
    """A_hat [B,H,n_rows,K] float64 -- steps a1..a3."""
    Q, K, W = _f64(Q), _f64(K), _f64(W)
    assert Q.shape == (p.B, p.H, p.T, p.d) and K.shape == Q.shape and W.shape == (p.m, p.d)
    sl, rw = _i32(seq_len), _i32(rows)
    n = _nrows(p, rows)
    A = np.empty((p.B, p.H, n, p.K), dtype=np.float64)
    cp = p.c()
    rc = _load().ref_estimate(ctypes.byref(cp), _ptr(Q), _ptr(K), _ptr(W), _ptr(sl), _ptr(rw),
                              ctypes.c_int32(n), _ptr(A))
    if rc != 0:
        raise MemoryError("ref_estimate failed")
    return A


def topk_mask(p: Params, A_hat, seq_len=None, rows=None):
    """(sel [.,k_hat], idx [.,L], cnt [.]) int32 -- steps a4..a5."""
    A = _f64(A_hat)
    n = _nrows(p, rows)
    assert A.shape == (p.B, p.H, n, p.K)
    sl, rw = _i32(seq_len), _i32(rows)
    L = row_stride(p)
    sel = np.empty((p.B, p.H, n, sel_stride(p)), dtype=np.int32)
    idx = np.empty((p.B, p.H, n, L), dtype=np.int32)
    cnt = np.empty((p.B, p.H, n), dtype=np.int32)
    cp = p.c()
    rc = _load().ref_topk_mask(ctypes.byref(cp), _ptr(A), _ptr(sl), _ptr(rw), ctypes.c_int32(n),
                               _ptr(sel), _ptr(idx), _ptr(cnt))
    if rc != 0:
        raise MemoryError("ref_topk_mask failed")
    return sel, idx, cnt


def sparse_attn(p: Params, Q, K, V, idx, cnt, rows=None):
    """O [B,H,n_rows,d] float64 -- step a6 (softmax over the listed keys only)."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    idx, cnt = _i32(idx), _i32(cnt)
    n = _nrows(p, rows)
    L = idx.shape[-1]
    assert idx.shape == (p.B, p.H, n, L) and cnt.shape == (p.B, p.H, n)
    rw = _i32(rows)
    O = np.empty((p.B, p.H, n, p.d), dtype=np.float64)
    cp = p.c()
    rc = _load().ref_sparse_attn(ctypes.byref(cp), _ptr(Q), _ptr(K), _ptr(V), _ptr(idx), _ptr(cnt),
                                 _ptr(rw), ctypes.c_int32(n), ctypes.c_int32(L), _ptr(O))
    if rc != 0:
        raise MemoryError("ref_sparse_attn failed")
    return O


def forward(p: Params, Q, K, V, W, seq_len=None, rows=None, heads=None, n_threads=0,
            want_aux=True):
    """Whole path a1..a6.  Returns dict(O, A_hat, sel, idx, cnt, threads).

    ``heads`` = (lo, hi) restricts the work to a range of the flattened B*H axis
    (outputs of other heads are left zero); used to time a bounded sample.
    """
    Q, K, V, W = _f64(Q), _f64(K), _f64(V), _f64(W)
    sl, rw = _i32(seq_len), _i32(rows)
    n = _nrows(p, rows)
    L = row_stride(p)
    lo, hi = heads if heads is not None else (0, p.B * p.H)
    O = np.zeros((p.B, p.H, n, p.d), dtype=np.float64)
    A = np.zeros((p.B, p.H, n, p.K), dtype=np.float64) if want_aux else None
    sel = np.full((p.B, p.H, n, sel_stride(p)), -1, dtype=np.int32) if want_aux else None
    idx = np.full((p.B, p.H, n, L), -1, dtype=np.int32) if want_aux else None
    cnt = np.zeros((p.B, p.H, n), dtype=np.int32) if want_aux else None
    cp = p.c()
    rc = _load().ref_forward(ctypes.byref(cp), _ptr(Q), _ptr(K), _ptr(V), _ptr(W), _ptr(sl),
                             _ptr(rw), ctypes.c_int32(n), ctypes.c_int32(lo), ctypes.c_int32(hi),
                             _ptr(O), _ptr(A), _ptr(sel), _ptr(idx), _ptr(cnt),
                             ctypes.c_int32(n_threads))
    if rc == -2:
        raise ValueError("with the causal-per-batch grouping the head range must cover whole batch elements")
    if rc < 0:
        raise MemoryError("ref_forward failed")
    return dict(O=O, A_hat=A, sel=sel, idx=idx, cnt=cnt, threads=rc)


def output_mix(p: Params, C, V, s_mix, s_prob=None, A_hat=None, seq_len=None):
    """C_sea [B,H,T,d] = s_mix (s_prob C) + (1 - s_mix) C_avg -- Sec. 3.1.1 "Output Calculation".

    A_hat [B,H,T,K] is needed for bidirectional attention only (importance pooling)."""
    C, V, s_mix = _f64(C), _f64(V), _f64(s_mix)
    assert C.shape == (p.B, p.H, p.T, p.d) and V.shape == C.shape and s_mix.shape == (p.B, p.H, p.T)
    sp = None if s_prob is None else _f64(s_prob)
    A = None
    if not p.causal:
        A = _f64(A_hat)
        assert A.shape == (p.B, p.H, p.T, p.K)
    sl = _i32(seq_len)
    O = np.empty_like(C)
    cp = p.c()
    rc = _load().ref_output_mix(ctypes.byref(cp), _ptr(C), _ptr(V), _ptr(A), _ptr(sp), _ptr(s_mix),
                                _ptr(sl), _ptr(O))
    if rc != 0:
        raise MemoryError("ref_output_mix failed")
    return O


def flatcsr(p: Params, idx, cnt):
    """FlatCSR tensor of the expanded mask -- Sec. 3.1.1 "FlatCSR" and App. A.5 "FlatCSR: Modified
    CSR Format To Handle Grouped Mask": M* [B][H][T][T] with the head and query axes exchanged and
    (head, key) flattened into one column axis, stored as CSR.  Row b T + t holds, ascending, the
    columns h T + j of the keys j that head h attends from query t.

    Returns (crow int64 [B T + 1], col int32 [nnz])."""
    idx, cnt = _i32(idx), _i32(cnt)
    assert cnt.shape == (p.B, p.H, p.T) and idx.shape[:3] == cnt.shape
    crow = np.zeros(p.B * p.T + 1, dtype=np.int64)
    col = []
    for b in range(p.B):
        for t in range(p.T):
            n = 0
            for h in range(p.H):
                keys = idx[b, h, t, :cnt[b, h, t]]
                col.append(h * p.T + keys.astype(np.int64))
                n += len(keys)
            crow[b * p.T + t + 1] = crow[b * p.T + t] + n
    col = np.concatenate(col) if col else np.zeros(0, dtype=np.int64)
    return crow, col.astype(np.int32)


def flatcsr_attn(p: Params, Q, K, V, crow, col):
    """Sparse attention (Sec. 3.1.1) read from the FlatCSR tensor: entry h T + j of row b T + t is
    key j of head h for query t; the softmax runs over the entries of one head in one row.
    The tensor is taken apart into per-head key lists, then attended as in ``sparse_attn``."""
    crow = np.asarray(crow, dtype=np.int64)
    col = np.asarray(col, dtype=np.int64)
    lists = {}
    L = 1
    for b in range(p.B):
        for t in range(p.T):
            e = col[crow[b * p.T + t]:crow[b * p.T + t + 1]]
            for h in range(p.H):
                keys = e[e // p.T == h] - h * p.T
                lists[b, h, t] = keys
                L = max(L, len(keys))
    idx = np.full((p.B, p.H, p.T, L), -1, dtype=np.int32)
    cnt = np.zeros((p.B, p.H, p.T), dtype=np.int32)
    for (b, h, t), keys in lists.items():
        idx[b, h, t, :len(keys)] = keys
        cnt[b, h, t] = len(keys)
    return sparse_attn(p, Q, K, V, idx, cnt)
