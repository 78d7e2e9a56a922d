"""CPU oracle of SEA's decoder path -- TEST INFRASTRUCTURE ONLY (tests, smoke, bench cpu leg).

Sec. 3.1 "CNN Decoder" and App. A.5.1 "Attention Estimator CNN": the Performer output on the
concatenated values [V_I; V], the MLPs mu and nu, the three-layer CNN with a nearest-neighbour
resize before its last layer, and the final softmax that yields the compressed attention matrix
A_hat; plus the scalers s_mix, s_prob of Sec. 3.1.1 "Output Calculation" (a linear map of the
shared hidden state Z followed by a sigmoid).  Plain fp64, one head / one batch element after the
other, in the paper's order; library primitives (matmul, torch's conv2d) serve as steps.

Readings where the paper is silent (the same list is in the repository's design notes):
  - features: phi(x)[i] = exp(w_i.x - |x|^2/2), x = sqrt(scale) q, as in the estimator oracle;
    the Performer output is normalised per row, C_perf[t] = sum_j a_tj u_j / sum_j a_tj with
    a_tj = phi(q_t).phi(k_j), u_j = [V_I(j); v_j], V_I the T x d nearest-neighbour stretch of I_d
    (V_I[j][floor(j d / T)] = 1); causal rows sum j <= t (the paper's learned positional
    embedding for causal V_I does not exist here, the stretched identity is kept);
  - hidden width d' = 2 d; mu = linear + ReLU; nu = linear + ReLU + linear (App. A.5.1 writes nu as
    R^d' -> R^d' -> R^(K c_h / c_s)); output index of nu: x c_h + ch (x the compressed column, ch the
    extra channel), which with random or learned weights is a permutation of the other order;
  - CNN: channels h c_h + ch; 3x3 kernels, zero padding of one column left and right; ReLU after the
    first two layers; bidirectional: the first layer has height stride c_s and rows i c_s - 1 .. + 1,
    the others rows i - 1 .. i + 1; causal: no height reduction (as the paper states) and every
    layer reads rows t - 2 .. t (a causal convolution: zero padding above only);
  - nearest resize to T x K: source = floor(dst * src_size / dst_size) on both axes;
  - right padding: keys >= seq_len contribute nothing, hidden rows >= seq_len enter the CNN as
    zeros, rows of A_hat >= seq_len are zero;
  - reduced-precision mode (`round_bf16`): every tensor the bf16 path stores is rounded to an
    8-bit significand, ties to even: phi(Q) (after a power-of-two row scale), phi(K), C_perf, Z,
    the hidden layer of nu, Z^ and the outputs of the first two convolutions.  Sums are not rounded.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
import torch


@dataclass
class DecoderParams:
    B: int
    H: int
    T: int
    d: int
    m: int
    K: int
    causal: bool = True
    scale: float = 0.125
    c_s: int = 2          # width (and, bidirectional, height) reduction of the CNN's hidden image
    c_h: int = 4          # channel expansion
    round_bf16: bool = False

    @property
    def d_hidden(self) -> int:
        return 2 * self.d

    @property
    def channels(self) -> int:
        return self.H * self.c_h


def round8(x: np.ndarray) -> np.ndarray:
    """Round to an 8-bit significand (bf16 precision, unbounded exponent), ties to even."""
    x = np.asarray(x, dtype=np.float64)
    f, e = np.frexp(x)                       # |f| in [0.5, 1)
    return np.ldexp(np.rint(np.ldexp(f, 8)), e - 8)


def _r(p: DecoderParams, x):
    return round8(x) if p.round_bf16 else x


def features(p: DecoderParams, X, W, query: bool):
    """phi of the rows of X [T, d] -> [T, m]; queries get a power-of-two row scale (cancels)."""
    y = np.sqrt(p.scale) * X
    arg = y @ W.T - 0.5 * (y * y).sum(-1, keepdims=True)
    if query:
        arg = arg - np.ceil(arg.max(-1, keepdims=True) / np.log(2.0)) * np.log(2.0)
    return _r(p, np.exp(arg))


def performer_encoding(p: DecoderParams, Q, K, V, W, seq_len=None):
    """C_perf [B, H, T, 2 d] = FAVOR+(Q, K, [V_I; V]) with the linear-attention normaliser."""
    B, H, T, d = p.B, p.H, p.T, p.d
    out = np.zeros((B, H, T, 2 * d))
    VI = np.zeros((T, d))
    VI[np.arange(T), (np.arange(T) * d) // T] = 1.0
    for b in range(B):
        ln = T if seq_len is None else int(seq_len[b])
        for h in range(H):
            fq = features(p, Q[b, h], W, True)
            fk = features(p, K[b, h], W, False)
            fk[ln:] = 0.0
            U = np.concatenate([VI, V[b, h]], -1)           # [T, 2d]
            if p.causal:
                S = np.zeros((p.m, 2 * d))                  # running phi(K)^T [V_I; V]
                z = np.zeros(p.m)                           # running sum of phi(k_j)
                for t in range(ln):
                    S += np.outer(fk[t], U[t])
                    z += fk[t]
                    out[b, h, t] = (fq[t] @ S) / (fq[t] @ z)
            else:
                S = fk.T @ U
                z = fk.sum(0)
                out[b, h, :ln] = (fq[:ln] @ S) / (fq[:ln] @ z)[:, None]
    return _r(p, out)


def _conv3x3(p: DecoderParams, x, w, bias, stride_h, causal):
    """x [C_in, Hh, Ww], w [C_out, 3, 3, C_in] (out, ky, kx, in) -> [C_out, Ho, Ww].  Width: one
    zero column on each side.  Height: causal -> two zero rows above (rows i-2..i); otherwise one
    above and one below, stride `stride_h` (rows i s - 1 .. i s + 1)."""
    xt = torch.from_numpy(np.ascontiguousarray(x))[None]
    wt = torch.from_numpy(np.ascontiguousarray(np.transpose(w, (0, 3, 1, 2))))   # [out, in, ky, kx]
    pad = (1, 1, 2, 0) if causal else (1, 1, 1, 1)                               # left, right, top, bottom
    xt = torch.nn.functional.pad(xt, pad)
    y = torch.nn.functional.conv2d(xt, wt, torch.from_numpy(np.asarray(bias, dtype=np.float64)),
                                   stride=(1 if causal else stride_h, 1))
    return y[0].numpy()


def _resize_nearest(x, Ho, Wo):
    C, Hi, Wi = x.shape
    rows = (np.arange(Ho) * Hi) // Ho
    cols = (np.arange(Wo) * Wi) // Wo
    return x[:, rows][:, :, cols]


def decoder_estimate(p: DecoderParams, Q, K, V, W, wts, seq_len=None):
    """Returns dict(A_hat [B,H,T,K], Z [B,H,T,d'], s_mix [B,H,T], s_prob [B,H,T], C_perf).
    `wts`: dict of float arrays mu_w [d',3d], mu_b, nu1_w [d',d'], nu1_b, nu2_w [K c_h/c_s, d'], nu2_b,
    conv1_w [C,3,3,C], conv1_b, conv2_w [C,3,3,C], conv2_b, conv3_w [H,3,3,C], conv3_b,
    mix_w [d'], mix_b, prob_w [d'], prob_b."""
    B, H, T, d, Kc = p.B, p.H, p.T, p.d, p.K
    f64 = lambda a: np.asarray(a, dtype=np.float64)
    Q, K, V, W = f64(Q), f64(K), f64(V), f64(W)
    w = {k: f64(v) for k, v in wts.items()}
    Wd = Kc // p.c_s
    C_perf = performer_encoding(p, Q, K, V, W, seq_len)
    A = np.zeros((B, H, T, Kc))
    Zs = np.zeros((B, H, T, p.d_hidden))
    s_mix = np.zeros((B, H, T))
    s_prob = np.zeros((B, H, T))
    sig = lambda a: 1.0 / (1.0 + np.exp(-a))
    for b in range(B):
        ln = T if seq_len is None else int(seq_len[b])
        img = np.zeros((p.channels, T, Wd))
        for h in range(H):
            x = np.concatenate([C_perf[b, h], V[b, h]], -1)                       # [T, 3d]
            Z = _r(p, np.maximum(x @ w["mu_w"].T + w["mu_b"], 0.0))               # mu
            hid = _r(p, np.maximum(Z @ w["nu1_w"].T + w["nu1_b"], 0.0))           # nu, first layer
            Zh = _r(p, hid @ w["nu2_w"].T + w["nu2_b"])                           # [T, Wd * c_h]
            Zh[ln:] = 0.0
            img[h * p.c_h:(h + 1) * p.c_h] = np.transpose(Zh.reshape(T, Wd, p.c_h), (2, 0, 1))
            Zs[b, h] = Z
            s_mix[b, h] = sig(Z @ w["mix_w"] + w["mix_b"])
            s_prob[b, h] = sig(Z @ w["prob_w"] + w["prob_b"])
        y = _r(p, np.maximum(_conv3x3(p, img, w["conv1_w"], w["conv1_b"], p.c_s, p.causal), 0.0))
        y = _r(p, np.maximum(_conv3x3(p, y, w["conv2_w"], w["conv2_b"], 1, p.causal), 0.0))
        y = _resize_nearest(y, T, Kc)
        logits = _conv3x3(p, y, w["conv3_w"], w["conv3_b"], 1, p.causal)          # [H, T, K]
        e = np.exp(logits - logits.max(-1, keepdims=True))
        soft = e / e.sum(-1, keepdims=True)
        soft[:, ln:] = 0.0
        A[b] = soft
        s_mix[b, :, ln:] = 0.0
        s_prob[b, :, ln:] = 0.0
    return dict(A_hat=A, Z=Zs, s_mix=s_mix, s_prob=s_prob, C_perf=C_perf)
