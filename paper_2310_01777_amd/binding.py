"""ctypes binding of libsea_hip.so: same names as the C ABI in include/sea.h.

Argument marshalling only -- every step of the path runs in the HIP kernels.  Tensors are
torch CUDA (ROCm) tensors used purely as device memory; the HIP stream is torch's current
stream unless one is given.  If the shared library is missing the import of this module
fails loudly; there is no fallback.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsea_hip.so")

SEA_F32, SEA_BF16 = 0, 1
SEA_OK, SEA_EINVAL, SEA_ENOTSUP, SEA_EWORKSPACE, SEA_EHIP, SEA_ETOOBIG = 0, -1, -2, -3, -4, -5
STAGES = ("features", "state", "contract", "topk_mask", "sparse", "dense", "compact")


class SeaParamsC(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("T", ctypes.c_int32),
                ("d", ctypes.c_int32), ("m", ctypes.c_int32), ("K", ctypes.c_int32),
                ("k_hat", ctypes.c_int32), ("k_budget", ctypes.c_int32),
                ("causal", ctypes.c_int32), ("scale", ctypes.c_float),
                ("dtype", ctypes.c_int32), ("seq_len", ctypes.c_void_p),
                ("grouping", ctypes.c_int32), ("geometry", ctypes.c_int32)]


class SeaDecoderWeightsC(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in ("mu_w", "mu_b", "nu1_w", "nu1_b", "nu2_w", "nu2_b", "conv1_w", "conv1_b",
                                               "conv2_w", "conv2_b", "conv3_w", "conv3_b", "mix_w", "mix_b",
                                               "prob_w", "prob_b")]


class SeaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = _lib.sea_strerror(status).decode()
        if status == SEA_EHIP:
            msg += f" [hipError {_lib.sea_last_hip_error()}]"
        super().__init__(f"{where}: {msg} ({status})")


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'` "
            "(hipcc --offload-arch=gfx950).  There is no CPU fallback.")
    lib = ctypes.CDLL(LIB_PATH)
    P = ctypes.POINTER(SeaParamsC)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    lib.sea_k_hat.restype, lib.sea_k_hat.argtypes = i32, [i32, i32, i32]
    lib.sea_row_stride.restype, lib.sea_row_stride.argtypes = i32, [P]
    lib.sea_sel_stride.restype, lib.sea_sel_stride.argtypes = i32, [P]
    lib.sea_workspace_bytes.restype, lib.sea_workspace_bytes.argtypes = sz, [P]
    lib.sea_estimate.restype, lib.sea_estimate.argtypes = ctypes.c_int, [P, vp, vp, vp, vp, vp, sz, vp]
    lib.sea_topk_mask.restype, lib.sea_topk_mask.argtypes = ctypes.c_int, [P, vp, vp, vp, vp, vp]
    lib.sea_sparse_attn.restype, lib.sea_sparse_attn.argtypes = ctypes.c_int, [P, vp, vp, vp, vp, vp, i32, vp, vp]
    lib.sea_forward.restype, lib.sea_forward.argtypes = ctypes.c_int, [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.sea_static_scratch_bytes.restype, lib.sea_static_scratch_bytes.argtypes = sz, []
    lib.sea_forward_static_bytes.restype, lib.sea_forward_static_bytes.argtypes = sz, [P]
    lib.sea_forward_static.restype, lib.sea_forward_static.argtypes = ctypes.c_int, [P, vp, vp, vp, vp, vp, vp]
    DW = ctypes.POINTER(SeaDecoderWeightsC)
    lib.sea_decoder_workspace_bytes.restype, lib.sea_decoder_workspace_bytes.argtypes = sz, [P]
    lib.sea_decoder_estimate.restype = ctypes.c_int
    lib.sea_decoder_estimate.argtypes = [P, DW, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.sea_decoder_forward.restype = ctypes.c_int
    lib.sea_decoder_forward.argtypes = [P, DW, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.sea_dense_workspace_bytes.restype, lib.sea_dense_workspace_bytes.argtypes = sz, [P]
    lib.sea_dense_attn.restype, lib.sea_dense_attn.argtypes = ctypes.c_int, [P, vp, vp, vp, vp, vp, sz, vp]
    lib.sea_output_mix_workspace_bytes.restype, lib.sea_output_mix_workspace_bytes.argtypes = sz, [P]
    lib.sea_output_mix.restype, lib.sea_output_mix.argtypes = ctypes.c_int, [P, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.sea_profile_enable.restype, lib.sea_profile_enable.argtypes = ctypes.c_int, [ctypes.c_int]
    lib.sea_profile_collect.restype = ctypes.c_int
    lib.sea_profile_collect.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
    lib.sea_strerror.restype, lib.sea_strerror.argtypes = ctypes.c_char_p, [ctypes.c_int]
    lib.sea_last_hip_error.restype, lib.sea_last_hip_error.argtypes = ctypes.c_int, []
    lib.sea_attention_path.restype, lib.sea_attention_path.argtypes = ctypes.c_int, [P]
    lib.sea_flatcsr_workspace_bytes.restype, lib.sea_flatcsr_workspace_bytes.argtypes = sz, [P]
    lib.sea_flatcsr.restype = ctypes.c_int
    lib.sea_flatcsr.argtypes = [P, vp, vp, ctypes.c_int32, vp, vp, ctypes.c_int64, vp, sz, vp]
    lib.sea_flatcsr_attn.restype, lib.sea_flatcsr_attn.argtypes = ctypes.c_int, [P, vp, vp, vp, vp, vp, vp, vp]
    lib.sea_key_mask.restype, lib.sea_key_mask.argtypes = ctypes.c_int, [P, vp, vp, vp]
    lib.sea_mask_attn_workspace_bytes.restype, lib.sea_mask_attn_workspace_bytes.argtypes = sz, [P]
    lib.sea_mask_attn.restype, lib.sea_mask_attn.argtypes = ctypes.c_int, [P, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.sea_version.restype, lib.sea_version.argtypes = ctypes.c_char_p, []
    return lib


_lib = _load()


@dataclass
class SeaParams:
    """Mirror of ``sea_params``.  ``dtype`` is 'f32' or 'bf16'; ``seq_len`` a CUDA int32 [B] tensor or None."""
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
    dtype: str = "bf16"
    seq_len: Optional[torch.Tensor] = None
    grouping: int = 0   # 0 per-query top-k^, 1 causal-per-batch
    geometry: int = 0   # 0 fixed key buckets, 1 a causal row spreads its columns over its own t + 1 keys

    def c(self) -> SeaParamsC:
        sl = None
        if self.seq_len is not None:
            t = self.seq_len
            assert t.is_cuda and t.dtype == torch.int32 and t.is_contiguous() and t.numel() == self.B
            sl = t.data_ptr()
        return SeaParamsC(self.B, self.H, self.T, self.d, self.m, self.K, self.k_hat, self.k_budget,
                          int(self.causal), float(self.scale), SEA_BF16 if self.dtype == "bf16" else SEA_F32,
                          sl, int(self.grouping), int(self.geometry))

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.bfloat16 if self.dtype == "bf16" else torch.float32


def _ptr(t: Optional[torch.Tensor], dtype=None, numel=None, name="tensor"):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name}: expected a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name}: expected dtype {dtype}, got {t.dtype}")
    if numel is not None and t.numel() < numel:
        raise ValueError(f"{name}: needs {numel} elements, has {t.numel()}")
    return t.data_ptr()


def _nbytes(t: Optional[torch.Tensor]) -> int:
    """Size of a workspace tensor; no tensor = 0 bytes, which the library answers with SEA_EWORKSPACE
    wherever it needs any."""
    return 0 if t is None else t.numel() * t.element_size()


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _check(rc: int, where: str):
    if rc != SEA_OK:
        raise SeaError(rc, where)


def sea_k_hat(k: int, K: int, T: int) -> int:
    return int(_lib.sea_k_hat(k, K, T))


def sea_row_stride(p: SeaParams) -> int:
    cp = p.c()
    L = int(_lib.sea_row_stride(ctypes.byref(cp)))
    if L < 0:
        raise SeaError(L, "sea_row_stride")
    return L


def sea_sel_stride(p: SeaParams) -> int:
    cp = p.c()
    S = int(_lib.sea_sel_stride(ctypes.byref(cp)))
    if S < 0:
        raise SeaError(S, "sea_sel_stride")
    return S


def sea_workspace_bytes(p: SeaParams) -> int:
    cp = p.c()
    return int(_lib.sea_workspace_bytes(ctypes.byref(cp)))


def sea_estimate(p: SeaParams, Q, K, W, A_hat, workspace, stream=None):
    n = p.B * p.H * p.T
    cp = p.c()
    _check(_lib.sea_estimate(ctypes.byref(cp), _ptr(Q, p.torch_dtype, n * p.d, "Q"),
                             _ptr(K, p.torch_dtype, n * p.d, "K"),
                             _ptr(W, p.torch_dtype, p.m * p.d, "W"),
                             _ptr(A_hat, torch.float32, n * p.K, "A_hat"),
                             _ptr(workspace, None, None, "workspace"),
                             _nbytes(workspace), _stream(stream)),
           "sea_estimate")


def sea_topk_mask(p: SeaParams, A_hat, sel, idx, cnt, stream=None):
    n = p.B * p.H * p.T
    L = sea_row_stride(p)
    cp = p.c()
    _check(_lib.sea_topk_mask(ctypes.byref(cp), _ptr(A_hat, torch.float32, n * p.K, "A_hat"),
                              _ptr(sel, torch.int32, n * sea_sel_stride(p), "sel"),
                              _ptr(idx, torch.int32, n * L, "idx"),
                              _ptr(cnt, torch.int32, n, "cnt"), _stream(stream)),
           "sea_topk_mask")


def sea_sparse_attn(p: SeaParams, Q, K, V, idx, cnt, row_stride, O, stream=None):
    n = p.B * p.H * p.T
    cp = p.c()
    _check(_lib.sea_sparse_attn(ctypes.byref(cp), _ptr(Q, p.torch_dtype, n * p.d, "Q"),
                                _ptr(K, p.torch_dtype, n * p.d, "K"),
                                _ptr(V, p.torch_dtype, n * p.d, "V"),
                                _ptr(idx, torch.int32, n * row_stride, "idx"),
                                _ptr(cnt, torch.int32, n, "cnt"), int(row_stride),
                                _ptr(O, p.torch_dtype, n * p.d, "O"), _stream(stream)),
           "sea_sparse_attn")


def sea_flatcsr_workspace_bytes(p: SeaParams) -> int:
    cp = p.c()
    return int(_lib.sea_flatcsr_workspace_bytes(ctypes.byref(cp)))


def sea_flatcsr(p: SeaParams, idx, cnt, row_stride, crow, col, workspace, stream=None):
    n = p.B * p.H * p.T
    cp = p.c()
    _check(_lib.sea_flatcsr(ctypes.byref(cp), _ptr(idx, torch.int32, n * row_stride, "idx"),
                            _ptr(cnt, torch.int32, n, "cnt"), int(row_stride),
                            _ptr(crow, torch.int64, p.B * p.T + 1, "crow"),
                            _ptr(col, torch.int32, None, "col"), col.numel(),
                            _ptr(workspace, None, None, "workspace"),
                            _nbytes(workspace), _stream(stream)),
           "sea_flatcsr")


def sea_flatcsr_attn(p: SeaParams, Q, K, V, crow, col, O, stream=None):
    n = p.B * p.H * p.T
    cp = p.c()
    _check(_lib.sea_flatcsr_attn(ctypes.byref(cp), _ptr(Q, p.torch_dtype, n * p.d, "Q"),
                                 _ptr(K, p.torch_dtype, n * p.d, "K"),
                                 _ptr(V, p.torch_dtype, n * p.d, "V"),
                                 _ptr(crow, torch.int64, p.B * p.T + 1, "crow"),
                                 _ptr(col, torch.int32, None, "col"),
                                 _ptr(O, p.torch_dtype, n * p.d, "O"), _stream(stream)),
           "sea_flatcsr_attn")


def sea_key_mask(p: SeaParams, mhat, key_bits, stream=None):
    """mhat [B, H, T, ceil(K/32)] int32 -> key_bits [B, H, T, ceil(T/32)] int32 (one bit per key)."""
    n = p.B * p.H * p.T
    cp = p.c()
    _check(_lib.sea_key_mask(ctypes.byref(cp), _ptr(mhat, torch.int32, n * ((p.K + 31) // 32), "mhat"),
                             _ptr(key_bits, torch.int32, n * ((p.T + 31) // 32), "key_bits"), _stream(stream)),
           "sea_key_mask")


def sea_mask_attn_workspace_bytes(p: SeaParams) -> int:
    cp = p.c()
    return int(_lib.sea_mask_attn_workspace_bytes(ctypes.byref(cp)))


def sea_mask_attn(p: SeaParams, Q, K, V, mhat, O, workspace=None, stream=None):
    n = p.B * p.H * p.T
    cp = p.c()
    _check(_lib.sea_mask_attn(ctypes.byref(cp), _ptr(Q, p.torch_dtype, n * p.d, "Q"),
                              _ptr(K, p.torch_dtype, n * p.d, "K"),
                              _ptr(V, p.torch_dtype, n * p.d, "V"),
                              _ptr(mhat, torch.int32, n * ((p.K + 31) // 32), "mhat"),
                              _ptr(O, p.torch_dtype, n * p.d, "O"),
                              _ptr(workspace, None, None, "workspace"),
                              _nbytes(workspace),
                              _stream(stream)),
           "sea_mask_attn")


def sea_forward(p: SeaParams, Q, K, V, W, O, A_hat=None, sel=None, idx=None, cnt=None,
                workspace=None, stream=None, mhat=None):
    n = p.B * p.H * p.T
    L = sea_row_stride(p)
    cp = p.c()
    _check(_lib.sea_forward(ctypes.byref(cp), _ptr(Q, p.torch_dtype, n * p.d, "Q"),
                            _ptr(K, p.torch_dtype, n * p.d, "K"),
                            _ptr(V, p.torch_dtype, n * p.d, "V"),
                            _ptr(W, p.torch_dtype, p.m * p.d, "W"),
                            _ptr(O, p.torch_dtype, n * p.d, "O"),
                            _ptr(A_hat, torch.float32, n * p.K, "A_hat"),
                            _ptr(sel, torch.int32, n * sea_sel_stride(p), "sel"),
                            _ptr(idx, torch.int32, n * L, "idx"),
                            _ptr(cnt, torch.int32, n, "cnt"),
                            _ptr(mhat, torch.int32, n * ((p.K + 31) // 32), "mhat"),
                            _ptr(workspace, None, None, "workspace"),
                            _nbytes(workspace),
                            _stream(stream)),
           "sea_forward")


def sea_static_scratch_bytes() -> int:
    return int(_lib.sea_static_scratch_bytes())


def sea_forward_static_bytes(p: SeaParams) -> int:
    cp = p.c()
    return int(_lib.sea_forward_static_bytes(ctypes.byref(cp)))


def sea_forward_static(p: SeaParams, Q, K, V, W, O, stream=None):
    n = p.B * p.H * p.T
    cp = p.c()
    _check(_lib.sea_forward_static(ctypes.byref(cp), _ptr(Q, p.torch_dtype, n * p.d, "Q"),
                                   _ptr(K, p.torch_dtype, n * p.d, "K"),
                                   _ptr(V, p.torch_dtype, n * p.d, "V"),
                                   _ptr(W, p.torch_dtype, p.m * p.d, "W"),
                                   _ptr(O, p.torch_dtype, n * p.d, "O"), _stream(stream)),
           "sea_forward_static")


def _decoder_weights(p: SeaParams, w: dict) -> SeaDecoderWeightsC:
    """dict of device tensors (matrices in bf16, biases in fp32) -> the C struct of pointers."""
    C, Wd = 4 * p.H, p.K // 2
    shapes = dict(mu_w=128 * 192, mu_b=128, nu1_w=128 * 128, nu1_b=128, nu2_w=Wd * 4 * 128, nu2_b=Wd * 4,
                  conv1_w=C * 9 * C, conv1_b=C, conv2_w=C * 9 * C, conv2_b=C, conv3_w=p.H * 9 * C, conv3_b=p.H,
                  mix_w=128, mix_b=1, prob_w=128, prob_b=1)
    out = SeaDecoderWeightsC()
    for name, n in shapes.items():
        dt = torch.float32 if name.endswith("_b") else torch.bfloat16
        setattr(out, name, _ptr(w[name], dt, n, name))
    return out


def sea_decoder_workspace_bytes(p: SeaParams) -> int:
    cp = p.c()
    return int(_lib.sea_decoder_workspace_bytes(ctypes.byref(cp)))


def sea_decoder_estimate(p: SeaParams, weights: dict, Q, K, V, W, A_hat, workspace, s_mix=None, s_prob=None, stream=None):
    n = p.B * p.H * p.T
    cp, cw = p.c(), _decoder_weights(p, weights)
    _check(_lib.sea_decoder_estimate(ctypes.byref(cp), ctypes.byref(cw), _ptr(Q, p.torch_dtype, n * p.d, "Q"),
                                     _ptr(K, p.torch_dtype, n * p.d, "K"), _ptr(V, p.torch_dtype, n * p.d, "V"),
                                     _ptr(W, p.torch_dtype, p.m * p.d, "W"),
                                     _ptr(A_hat, torch.float32, n * p.K, "A_hat"),
                                     _ptr(s_mix, torch.float32, n, "s_mix"), _ptr(s_prob, torch.float32, n, "s_prob"),
                                     _ptr(workspace, None, None, "workspace"),
                                     _nbytes(workspace),
                                     _stream(stream)),
           "sea_decoder_estimate")


def sea_decoder_forward(p: SeaParams, weights: dict, Q, K, V, W, O, workspace, A_hat=None, stream=None):
    n = p.B * p.H * p.T
    cp, cw = p.c(), _decoder_weights(p, weights)
    _check(_lib.sea_decoder_forward(ctypes.byref(cp), ctypes.byref(cw), _ptr(Q, p.torch_dtype, n * p.d, "Q"),
                                    _ptr(K, p.torch_dtype, n * p.d, "K"), _ptr(V, p.torch_dtype, n * p.d, "V"),
                                    _ptr(W, p.torch_dtype, p.m * p.d, "W"), _ptr(O, p.torch_dtype, n * p.d, "O"),
                                    _ptr(A_hat, torch.float32, n * p.K, "A_hat"),
                                    _ptr(workspace, None, None, "workspace"),
                                    _nbytes(workspace),
                                    _stream(stream)),
           "sea_decoder_forward")


def sea_dense_workspace_bytes(p: SeaParams) -> int:
    cp = p.c()
    return int(_lib.sea_dense_workspace_bytes(ctypes.byref(cp)))


def sea_dense_attn(p: SeaParams, Q, K, V, O, workspace=None, stream=None):
    n = p.B * p.H * p.T
    cp = p.c()
    _check(_lib.sea_dense_attn(ctypes.byref(cp), _ptr(Q, p.torch_dtype, n * p.d, "Q"),
                               _ptr(K, p.torch_dtype, n * p.d, "K"),
                               _ptr(V, p.torch_dtype, n * p.d, "V"),
                               _ptr(O, p.torch_dtype, n * p.d, "O"),
                               _ptr(workspace, None, None, "workspace"),
                               _nbytes(workspace),
                               _stream(stream)),
           "sea_dense_attn")


def sea_output_mix_workspace_bytes(p: SeaParams) -> int:
    cp = p.c()
    return int(_lib.sea_output_mix_workspace_bytes(ctypes.byref(cp)))


def sea_output_mix(p: SeaParams, C, V, s_mix, O, workspace, s_prob=None, A_hat=None, stream=None):
    n = p.B * p.H * p.T
    cp = p.c()
    _check(_lib.sea_output_mix(ctypes.byref(cp), _ptr(C, p.torch_dtype, n * p.d, "C"),
                               _ptr(V, p.torch_dtype, n * p.d, "V"),
                               _ptr(A_hat, torch.float32, n * p.K, "A_hat"),
                               _ptr(s_prob, torch.float32, n, "s_prob"),
                               _ptr(s_mix, torch.float32, n, "s_mix"),
                               _ptr(O, p.torch_dtype, n * p.d, "O"),
                               _ptr(workspace, None, None, "workspace"),
                               _nbytes(workspace), _stream(stream)),
           "sea_output_mix")


def sea_profile_enable(stages=True):
    """True/False for all/none, or an iterable of stage names from STAGES."""
    if stages is True:
        mask = -1
    elif not stages:
        mask = 0
    else:
        mask = sum(1 << STAGES.index(s) for s in stages)
    _check(_lib.sea_profile_enable(mask), "sea_profile_enable")


def sea_profile_collect():
    """{stage: (milliseconds, launches)} accumulated since the last collect."""
    ms = (ctypes.c_double * len(STAGES))()
    cnt = (ctypes.c_int64 * len(STAGES))()
    _check(_lib.sea_profile_collect(ms, cnt), "sea_profile_collect")
    return {name: (ms[i], cnt[i]) for i, name in enumerate(STAGES)}


def sea_attention_path(p: "SeaParams") -> int:
    """1 = tiled matrix-core attention (bf16), 2 = its fp32 counterpart, 3 = tiled on per-key bits (row-width geometry), 0 = per-row index lists, negative = rejected parameters."""
    cp = p.c()
    return int(_lib.sea_attention_path(ctypes.byref(cp)))


def sea_version() -> str:
    return _lib.sea_version().decode()


# ---- conveniences that only allocate device memory ----

def alloc_workspace(p: SeaParams, device="cuda") -> torch.Tensor:
    nbytes = sea_workspace_bytes(p)
    if nbytes == 0:
        raise SeaError(SEA_EINVAL, "sea_workspace_bytes")
    return torch.empty(nbytes, dtype=torch.uint8, device=device)   # torch allocations are 512-B aligned


def alloc_outputs(p: SeaParams, device="cuda", aux=True):
    n = (p.B, p.H, p.T)
    out = dict(O=torch.empty(*n, p.d, dtype=p.torch_dtype, device=device))
    if aux:
        L = sea_row_stride(p)
        out.update(A_hat=torch.empty(*n, p.K, dtype=torch.float32, device=device),
                   sel=torch.empty(*n, sea_sel_stride(p), dtype=torch.int32, device=device),
                   idx=torch.empty(*n, L, dtype=torch.int32, device=device),
                   cnt=torch.empty(*n, dtype=torch.int32, device=device),
                   mhat=torch.empty(*n, (p.K + 31) // 32, dtype=torch.int32, device=device))
    return out
