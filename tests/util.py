"""Shared helpers for the parity tests: tensor conversion, tolerance checks, near-tie analysis."""
from __future__ import annotations

import numpy as np
import torch

import oracle

# Tolerances of the contract: relative to the per-head scale of the reference (max and RMS).
TOL = {"f32": 1e-5, "bf16": 2e-2}
# Index sets must agree unless the oracle's own score gap at the selection boundary is below
# this.  fp32: the stated 1e-5.  bf16: two bf16 units in the last place (2^-7): the GPU and the
# fp64 oracle can round a feature or state element to neighbouring bf16 values when the
# pre-rounding values differ in the last fp32 bits, which moves a score by at most 2^-8 of itself.
GAP = {"f32": 1e-5, "bf16": 2.0 ** -7}


def to_np64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu", torch.float64).numpy()


def oracle_params(wl_or_p, round8=None) -> oracle.Params:
    p = wl_or_p
    geometry = int(getattr(p, "geometry", 0))
    r8 = (p.dtype == "bf16") if round8 is None else round8
    return oracle.Params(B=p.B, H=p.H, T=p.T, d=p.d, m=p.m, K=p.K, k_hat=p.k_hat,
                         k_budget=p.k_budget, causal=bool(p.causal), scale=float(p.scale), round8=r8,
                         grouping=int(getattr(p, "grouping", 0)), geometry=geometry)


def rel_errors(got: np.ndarray, ref: np.ndarray):
    """Per-head (max-abs error / max-abs ref, rms error / rms ref); arrays [B,H,...]."""
    B, H = ref.shape[:2]
    g = got.reshape(B * H, -1).astype(np.float64)
    r = ref.reshape(B * H, -1).astype(np.float64)
    dmax = np.abs(g - r).max(1)
    rmax = np.abs(r).max(1)
    drms = np.sqrt(((g - r) ** 2).mean(1))
    rrms = np.sqrt((r ** 2).mean(1))
    safe = lambda a, b: np.where(b > 0, a / np.where(b > 0, b, 1), np.where(a > 0, np.inf, 0.0))
    return safe(dmax, rmax), safe(drms, rrms)


def assert_close(got, ref, tol, what=""):
    emax, erms = rel_errors(np.asarray(got), np.asarray(ref))
    assert np.isfinite(np.asarray(got, dtype=np.float64)).all(), f"{what}: non-finite output"
    assert emax.max() <= tol, f"{what}: max-rel error {emax.max():.3e} > {tol:g} (head {emax.argmax()})"
    assert erms.max() <= tol, f"{what}: rms-rel error {erms.max():.3e} > {tol:g} (head {erms.argmax()})"
    return float(emax.max()), float(erms.max())


def selection_gaps(A_ref: np.ndarray, sel_ref: np.ndarray, ncand: np.ndarray) -> np.ndarray:
    """Relative gap between the smallest selected and the largest unselected candidate score of
    each row of the oracle's A_hat ([..., K]); +inf where every candidate is selected."""
    flat_A = A_ref.reshape(-1, A_ref.shape[-1])
    flat_s = sel_ref.reshape(-1, sel_ref.shape[-1])
    flat_n = ncand.reshape(-1)
    gaps = np.full(flat_A.shape[0], np.inf)
    for r in range(flat_A.shape[0]):
        s = flat_s[r][flat_s[r] >= 0]
        n = flat_n[r]
        if len(s) == 0 or len(s) >= n:
            continue
        mask = np.ones(n, dtype=bool)
        mask[s] = False
        lo = flat_A[r, s].min()
        hi = flat_A[r, :n][mask].max()
        gaps[r] = (lo - hi) / lo if lo > 0 else 0.0
    return gaps.reshape(sel_ref.shape[:-1])


def candidate_counts(B, H, T, K, causal, seq_len, rows=None) -> np.ndarray:
    """Number of candidate columns per row (0 for inactive rows); fixed key buckets."""
    rows = np.arange(T) if rows is None else np.asarray(rows)
    out = np.zeros((B, H, len(rows)), dtype=np.int64)
    for b in range(B):
        ln = T if seq_len is None else int(seq_len[b])
        for r, t in enumerate(rows):
            if t >= ln:
                continue
            jmax = min(t, ln - 1) if causal else ln - 1
            out[b, :, r] = (jmax * K) // T + 1
    return out


def group_selection_gaps(A_ref: np.ndarray, mask_ref: np.ndarray, ncand: np.ndarray) -> np.ndarray:
    """Causal-per-batch grouping: relative gap between the smallest selected and the largest
    unselected candidate score of each time step's H x K slab.  A_ref, mask_ref: [B,H,T,K];
    ncand: [B,H,T] (same for every head).  Returns [B,T]; +inf where every candidate is taken."""
    B, H, T, K = A_ref.shape
    gaps = np.full((B, T), np.inf)
    for b in range(B):
        for t in range(T):
            n = int(ncand[b, 0, t])
            if n == 0:
                continue
            a = A_ref[b, :, t, :n].reshape(-1)
            m = mask_ref[b, :, t, :n].reshape(-1)
            if m.all() or not m.any():
                continue
            lo, hi = a[m].min(), a[~m].max()
            gaps[b, t] = (lo - hi) / lo if lo > 0 else 0.0
    return gaps
