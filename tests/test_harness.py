"""Host-side checks of the harness around the library: workload definitions and bench.py's
argument contract (nothing here touches a GPU)."""
import subprocess
import sys
from pathlib import Path

import oracle
from paper_2310_01777_amd import synth

ROOT = Path(__file__).resolve().parent.parent


def test_bench_refuses_more_than_one_gpu():
    res = subprocess.run([sys.executable, str(ROOT / "bench.py"), "--gpus", "2", "--steps", "1", "--warmup", "0"],
                         capture_output=True, text=True, timeout=120)
    assert res.returncode != 0
    assert "one GPU" in res.stderr
    assert res.stdout.strip() == ""          # no JSON line that could be mistaken for a measurement


def test_fixed_k_workloads_follow_the_k_hat_rule():
    """c6 / c7 derive k^ from a fixed k with k^ = max(1, round(k K / T)) (Sec. 3.1 "Linear Sparse
    Attention Mask Generation"); the oracle's helper is the reference for the rounding."""
    for T in synth.C6_LENGTHS:
        for name in (f"c6_T{T}", f"c6c_T{T}"):
            wl = synth.get_workload(name)
            assert wl.k_hat == oracle.k_hat_from_k(synth.C6_K, wl.K, T)
            assert wl.k_budget == synth.C6_K and wl.T == T and wl.T % wl.K == 0
            assert wl.causal == name.startswith("c6c")
    assert [synth.get_workload(f"c6_T{T}").k_hat for T in synth.C6_LENGTHS] == [2, 1, 1, 1, 1, 1]
    for T, kh in zip(synth.C4_LENGTHS, (32, 16, 8, 4)):
        wl = synth.get_workload(f"c7_T{T}")
        assert wl.k_hat == kh == oracle.k_hat_from_k(512, wl.K, T)
        assert wl.k_budget == 0 and wl.causal
        # whole columns: every active row far enough from the start gets k^ * (T / K) = 512 keys
        p = oracle.Params(B=1, H=1, T=T, d=64, m=wl.m, K=wl.K, k_hat=wl.k_hat, k_budget=0, causal=True)
        assert oracle.row_stride(p) == 512


def test_headline_workloads_match_the_baseline_shapes():
    c2 = synth.get_workload("c2")
    assert (c2.B, c2.H, c2.T, c2.d, c2.m, c2.K, c2.k_hat, c2.causal, c2.dtype) == \
        (4, 12, 2048, 64, 128, 128, 64, True, "bf16")
    c4 = synth.get_workload("c4_T32768")
    p = oracle.Params(B=1, H=1, T=c4.T, d=64, m=c4.m, K=c4.K, k_hat=c4.k_hat, k_budget=c4.k_budget, causal=True)
    assert oracle.row_stride(p) == 512       # 64 columns x 8 keys at every length of the sweep
