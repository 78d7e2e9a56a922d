"""Host-side checks of the C-ABI library (no GPU needed): it loads, exports every symbol the
header declares, validates arguments, and its integer helpers agree with the paper's formulas."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "sea.h")


@pytest.fixture(scope="module")
def sea():
    from paper_2310_01777_amd import binding, build
    if build.is_stale():
        build.build()
    return binding


def _declared_symbols():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(sea_[a-z_0-9]+)\s*\(", src)))


def test_library_exports_every_declared_symbol(sea):
    names = _declared_symbols()
    assert {"sea_estimate", "sea_topk_mask", "sea_sparse_attn", "sea_forward", "sea_dense_attn",
            "sea_workspace_bytes", "sea_row_stride", "sea_k_hat", "sea_strerror"} <= set(names)
    lib = ctypes.CDLL(sea.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in sea.h but not exported"


def test_k_hat_helper_matches_golden(sea):
    with open(os.path.join(ROOT, "tests", "golden", "k_hat_cases.txt")) as f:
        rows = [ln.split("#")[0].split() for ln in f if ln.split("#")[0].strip()]
    for k, K, T, want in rows:
        assert sea.sea_k_hat(int(k), int(K), int(T)) == int(want)
    assert sea.sea_k_hat(0, 4, 8) == sea.SEA_EINVAL


def test_row_stride_closed_forms(sea):
    P = sea.SeaParams
    # whole columns: k_hat * ceil(T / K)
    assert sea.sea_row_stride(P(1, 1, 2048, 64, 128, 128, 64)) == 64 * 16
    assert sea.sea_row_stride(P(1, 1, 1000, 64, 128, 7, 3)) == 3 * 143
    # budget: k* = min(k, ceil(T/K)) when k_hat = 1 (App. A.5.3)
    assert sea.sea_row_stride(P(1, 1, 131072, 64, 128, 128, 1, k_budget=64)) == 64
    assert sea.sea_row_stride(P(1, 1, 4096, 64, 128, 128, 1, k_budget=64)) == 32
    assert sea.sea_row_stride(P(1, 1, 32768, 64, 256, 256, 64, k_budget=512)) == 512
    assert sea.sea_row_stride(P(1, 1, 4096, 64, 256, 256, 64, k_budget=3)) == 64


def test_argument_validation_returns_codes_not_crashes(sea):
    P = sea.SeaParams
    bad = [
        (P(1, 1, 64, 64, 32, 128, 4), sea.SEA_EINVAL),        # K > T
        (P(1, 1, 64, 64, 32, 16, 17), sea.SEA_EINVAL),        # k_hat > K
        (P(0, 1, 64, 64, 32, 16, 4), sea.SEA_EINVAL),         # empty batch
        (P(1, 1, 64, 64, 32, 16, 4, scale=0.0), sea.SEA_EINVAL),
        (P(1, 1, 64, 32, 32, 16, 4), sea.SEA_ENOTSUP),        # d != 64
        (P(1, 1, 4096, 64, 32, 2048, 4), sea.SEA_ENOTSUP),    # K > 1024
    ]
    for p, code in bad:
        with pytest.raises(sea.SeaError) as e:
            sea.sea_row_stride(p)
        assert e.value.status == code
        assert sea.sea_workspace_bytes(p) == 0
    ok = P(1, 2, 128, 64, 64, 16, 4)
    assert sea.sea_workspace_bytes(ok) > 0
    cp = ok.c()
    lib = sea._lib
    # NULL tensors are rejected before anything is launched
    assert lib.sea_estimate(ctypes.byref(cp), None, None, None, None, None, 0, None) == sea.SEA_EINVAL
    assert lib.sea_topk_mask(ctypes.byref(cp), None, None, None, None, None) == sea.SEA_EINVAL
    assert lib.sea_sparse_attn(ctypes.byref(cp), None, None, None, None, None, 8, None, None) == sea.SEA_EINVAL
    assert lib.sea_forward(ctypes.byref(cp), None, None, None, None, None, None, None, None, None,
                           None, None, 0, None) == sea.SEA_EINVAL
    assert lib.sea_mask_attn(ctypes.byref(cp), None, None, None, None, None, None, 0, None) == sea.SEA_EINVAL
    assert lib.sea_flatcsr(ctypes.byref(cp), None, None, 8, None, None, 0, None, 0, None) == sea.SEA_EINVAL
    assert lib.sea_flatcsr_attn(ctypes.byref(cp), None, None, None, None, None, None, None) == sea.SEA_EINVAL
    assert sea.sea_flatcsr_workspace_bytes(ok) >= 8
    odd = P(1, 2, 300, 64, 96, 17, 5).c()            # K does not divide T: no column-structured form
    assert lib.sea_mask_attn_workspace_bytes(ctypes.byref(odd)) == 0
    m48 = P(1, 1, 128, 64, 48, 16, 4).c()
    one = ctypes.c_void_p(256)
    assert lib.sea_estimate(ctypes.byref(m48), one, one, one, one, one, 1 << 30, None) == sea.SEA_ENOTSUP
    # workspace too small / misaligned
    assert lib.sea_estimate(ctypes.byref(cp), one, one, one, one, one, 16, None) == sea.SEA_EWORKSPACE
    assert lib.sea_estimate(ctypes.byref(cp), one, one, one, one, ctypes.c_void_p(8), 1 << 30, None) \
        == sea.SEA_EWORKSPACE
    assert lib.sea_mask_attn(ctypes.byref(odd), one, one, one, one, one, None, 0, None) == sea.SEA_ENOTSUP
    assert lib.sea_flatcsr(ctypes.byref(cp), one, one, 8, one, one, 16, None, 0, None) == sea.SEA_EWORKSPACE
    assert lib.sea_flatcsr(ctypes.byref(cp), one, one, 0, one, one, 16, one, 1 << 20, None) == sea.SEA_EINVAL
    one_col = P(1, 2, 1024, 64, 64, 32, 1, k_budget=16)      # rows bucketed by column need scratch
    assert sea.sea_mask_attn_workspace_bytes(one_col) > 0
    assert lib.sea_mask_attn(ctypes.byref(one_col.c()), one, one, one, one, one, None, 0, None) \
        == sea.SEA_EWORKSPACE
    assert b"workspace" in lib.sea_strerror(sea.SEA_EWORKSPACE)
    assert sea.sea_version().startswith("sea-hip")
    # which attention kernel a forward call takes: tiles need bf16, K | T and a power-of-two r
    assert sea.sea_attention_path(P(1, 2, 2048, 64, 128, 128, 64)) == 1
    assert sea.sea_attention_path(P(1, 2, 2048, 64, 128, 128, 64, dtype="f32")) == 2
    assert sea.sea_attention_path(P(1, 2, 300, 64, 96, 17, 5, dtype="f32")) == 0
    assert sea.sea_attention_path(P(1, 2, 300, 64, 96, 17, 5)) == 0            # K does not divide T
    assert sea.sea_attention_path(P(1, 2, 768, 64, 64, 64, 8, k_budget=24)) == 0   # r = 3
    assert sea.sea_attention_path(P(1, 1, 64, 64, 32, 16, 17)) == sea.SEA_EINVAL
    # per-row width geometry: causal only, key lists for the attention
    assert sea.sea_attention_path(P(1, 2, 2048, 64, 128, 128, 64, geometry=1)) == 3
    assert sea.sea_attention_path(P(1, 2, 8192, 64, 128, 128, 64, geometry=1)) == 3
    assert sea.sea_attention_path(P(1, 2, 8192, 64, 128, 128, 64, geometry=1, dtype="f32")) == 0
    assert sea.sea_attention_path(P(1, 2, 16384, 64, 128, 128, 64, geometry=1)) == 0
    for bad, code in ((P(1, 2, 256, 64, 64, 16, 4, causal=False, geometry=1), sea.SEA_EINVAL),
                      (P(1, 2, 256, 64, 64, 16, 4, geometry=2), sea.SEA_EINVAL)):
        with pytest.raises(sea.SeaError) as e:
            sea.sea_row_stride(bad)
        assert e.value.status == code
    assert sea.sea_workspace_bytes(P(1, 2, 256, 64, 96, 16, 4, geometry=1)) == 0      # m = 96
    assert sea.sea_workspace_bytes(P(1, 2, 256, 64, 128, 16, 4, geometry=1)) > 0


def test_row_stride_agrees_with_oracle_helper(sea):
    import oracle
    for (T, K, kh, kb) in [(2048, 128, 64, 0), (1000, 7, 3, 0), (777, 100, 33, 70), (4096, 256, 64, 512),
                           (64, 64, 1, 5), (65, 64, 2, 1)]:
        p = sea.SeaParams(1, 1, T, 64, 32, K, kh, k_budget=kb)
        po = oracle.Params(B=1, H=1, T=T, d=64, m=32, K=K, k_hat=kh, k_budget=kb)
        assert sea.sea_row_stride(p) == oracle.row_stride(po)


def test_workspace_sizes_closed_forms(sea):
    """Host arithmetic of the scratch sizes the stage entry points ask for."""
    P = sea.SeaParams
    a256 = lambda n: (n + 255) // 256 * 256
    for (B, H, T) in [(1, 2, 128), (3, 5, 1000), (2, 12, 2048)]:
        p = P(B, H, T, 64, 64, 8, 2)
        assert sea.sea_flatcsr_workspace_bytes(p) == a256((B * T + 255) // 256 * 8)
    # the attention stage on a mask needs scratch only where rows are grouped by column
    assert sea.sea_mask_attn_workspace_bytes(P(1, 2, 2048, 64, 128, 128, 64)) == 0
    assert sea.sea_mask_attn_workspace_bytes(P(1, 2, 1024, 64, 64, 32, 1, k_budget=16)) > 0
    assert sea.sea_mask_attn_workspace_bytes(P(1, 2, 2048, 64, 128, 128, 64, geometry=1)) == 0   # not offered
    # per-row width geometry: both feature tensors dominate the estimator scratch -- bf16 for bf16
    # tensors (T rounded up to whole 32-token chunks), fp64 for fp32 tensors
    p1 = P(2, 3, 500, 64, 128, 32, 4, geometry=1)
    assert sea.sea_workspace_bytes(p1) >= 2 * (2 * 3 * 512 * 128 * 2)
    p2 = P(2, 3, 500, 64, 128, 32, 4, geometry=1, dtype="f32")
    assert sea.sea_workspace_bytes(p2) >= 2 * (2 * 3 * 500 * 128 * 8)
