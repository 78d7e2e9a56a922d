"""Pins for the decoder oracle (oracle/decoder.py): Sec. 3.1 "CNN Decoder", App. A.5.1.  CPU only.
Each test checks the oracle against something other than itself: the already pinned estimator
oracle, the exact softmax attention the Performer output converges to, hand-enumerated
convolutions, a library resize, closed forms."""
import numpy as np
import pytest
import torch

import oracle
from oracle import decoder as dec
from paper_2310_01777_amd import synth


def _qkv(B, H, T, d, seed, std=1.0):
    g = np.random.default_rng(seed)
    return [g.standard_normal((B, H, T, d)) * std for _ in range(3)]


def _wts(H, d, K, seed=7):
    return {k: v.to(torch.float64).numpy() for k, v in synth.decoder_weights(H, d, K, seed=seed).items()}


def test_round8_is_the_library_bf16_cast():
    g = np.random.default_rng(0)
    x = (g.standard_normal(5000) * 10.0 ** g.integers(-20, 20, 5000)).astype(np.float32)
    x = np.concatenate([x, np.float32([1.00390625, 1.01171875, 255.5, 256.5, 0.0, -3.0])])
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(dec.round8(x.astype(np.float64)), want)


@pytest.mark.parametrize("causal", [False, True])
def test_identity_half_of_the_performer_output_is_the_estimate_with_d_columns(causal):
    """FAVOR+(Q, K, V_I) with V_I the T x d stretched identity is the compressed estimate of the
    estimator oracle (plain C, pinned on its own) with K = d columns."""
    B, H, T, d, m = 2, 2, 48, 8, 32
    Q, K, V = _qkv(B, H, T, d, 3, 0.7)
    W = synth.gaussian_orthogonal(m, d, 1).numpy().astype(np.float64)
    seq_len = np.array([T, 37], dtype=np.int32)
    p = dec.DecoderParams(B=B, H=H, T=T, d=d, m=m, K=16, causal=causal, scale=0.4)
    C = dec.performer_encoding(p, Q, K, V, W, seq_len)
    po = oracle.Params(B=B, H=H, T=T, d=d, m=m, K=d, k_hat=1, causal=causal, scale=0.4)
    A = oracle.estimate(po, Q, K, W, seq_len=seq_len)
    np.testing.assert_allclose(C[..., :d], A, rtol=1e-10, atol=1e-14)
    assert np.all(C[1, :, 37:] == 0.0)


@pytest.mark.parametrize("causal", [False, True])
def test_value_half_of_the_performer_output_converges_to_softmax_attention(causal):
    """FAVOR+(Q, K, V) is an unbiased estimate of softmax(scale QK^T) V: the error shrinks with m.
    A wrong normaliser, a dropped norm term or a non-causal state would all miss the limit."""
    B, H, T, d = 1, 2, 32, 8
    Q, K, V = _qkv(B, H, T, d, 5, 0.4)
    S = 0.5 * torch.from_numpy(Q) @ torch.from_numpy(K).transpose(-1, -2)
    if causal:
        S = S.masked_fill(~torch.tril(torch.ones(T, T, dtype=torch.bool)), float("-inf"))
    exact = (torch.softmax(S, -1) @ torch.from_numpy(V)).numpy()
    errs = []
    for m in (256, 16384):
        W = np.random.default_rng(m).standard_normal((m, d))
        p = dec.DecoderParams(B=B, H=H, T=T, d=d, m=m, K=8, causal=causal, scale=0.5)
        C = dec.performer_encoding(p, Q, K, V, W)
        errs.append(np.abs(C[..., d:] - exact).max())
    assert errs[1] < 0.02 and errs[1] < errs[0] / 3, errs


def test_convolution_taps_padding_and_stride_hand_enumerated():
    """One input channel, delta kernels: the output is the input shifted by the tap's offset, with
    zeros where the tap falls outside.  Fixes which rows a causal layer reads (t-2..t), which a
    bidirectional one reads (i s - 1 .. i s + 1) and the one-column padding."""
    p = dec.DecoderParams(B=1, H=1, T=5, d=4, m=4, K=8)
    x = np.arange(1.0, 21.0).reshape(1, 5, 4)
    for ky in range(3):
        for kx in range(3):
            w = np.zeros((1, 3, 3, 1))
            w[0, ky, kx, 0] = 1.0
            y = dec._conv3x3(p, x, w, np.zeros(1), 1, True)             # causal: row t + ky - 2, col c + kx - 1
            want = np.zeros((5, 4))
            for t in range(5):
                for c in range(4):
                    tt, cc = t + ky - 2, c + kx - 1
                    if 0 <= tt < 5 and 0 <= cc < 4:
                        want[t, c] = x[0, tt, cc]
            assert np.array_equal(y[0], want), (ky, kx)
            y = dec._conv3x3(p, x, w, np.zeros(1), 2, False)            # stride 2: row 2 i + ky - 1
            want = np.zeros((3, 4))
            for i in range(3):
                for c in range(4):
                    tt, cc = 2 * i + ky - 1, c + kx - 1
                    if 0 <= tt < 5 and 0 <= cc < 4:
                        want[i, c] = x[0, tt, cc]
            assert np.array_equal(y[0], want), (ky, kx)
    # channel mixing and bias: all-ones kernel over two channels of ones counts the taps in bounds
    ones = np.ones((2, 4, 3))
    y = dec._conv3x3(p, ones, np.ones((1, 3, 3, 2)), np.array([0.5]), 1, True)
    rows = np.minimum(np.arange(4) + 1, 3)[:, None]                      # rows t-2..t that exist
    cols = np.array([2, 3, 2])[None, :]
    assert np.array_equal(y[0], 2.0 * rows * cols + 0.5)


def test_resize_is_the_library_nearest_interpolation():
    x = np.random.default_rng(1).standard_normal((3, 6, 8))
    for Ho, Wo in [(12, 16), (6, 16), (11, 24)]:
        want = torch.nn.functional.interpolate(torch.from_numpy(x)[None], size=(Ho, Wo), mode="nearest")[0].numpy()
        assert np.array_equal(dec._resize_nearest(x, Ho, Wo), want)


def _run(p, seed=11, seq_len=None, Wseed=2):
    Q, K, V = _qkv(p.B, p.H, p.T, p.d, seed, 0.8)
    W = synth.gaussian_orthogonal(p.m, p.d, Wseed).numpy().astype(np.float64)
    return Q, K, V, W, dec.decoder_estimate(p, Q, K, V, W, _wts(p.H, p.d, p.K), seq_len)


@pytest.mark.parametrize("causal", [False, True])
def test_rows_are_softmaxes_padding_is_inert_and_scalers_are_sigmoids(causal):
    p = dec.DecoderParams(B=2, H=2, T=24, d=8, m=16, K=8, causal=causal, scale=0.35)
    seq_len = np.array([24, 17], dtype=np.int32)
    Q, K, V, W, o = _run(p, seq_len=seq_len)
    np.testing.assert_allclose(o["A_hat"][0].sum(-1), 1.0, atol=1e-12)
    np.testing.assert_allclose(o["A_hat"][1, :, :17].sum(-1), 1.0, atol=1e-12)
    assert np.all(o["A_hat"][1, :, 17:] == 0.0) and o["A_hat"].min() >= 0.0
    assert np.all((o["s_mix"][0] > 0) & (o["s_mix"][0] < 1))
    # positions >= seq_len are inert
    Q2, K2, V2 = Q.copy(), K.copy(), V.copy()
    for X in (Q2, K2, V2):
        X[1, :, 17:] = 50.0
    o2 = dec.decoder_estimate(p, Q2, K2, V2, W, _wts(p.H, p.d, p.K), seq_len)
    for k in ("A_hat", "s_mix", "s_prob"):
        assert np.array_equal(o[k], o2[k]), k
    # zero scaler weights: sigmoid(bias)
    w = _wts(p.H, p.d, p.K)
    w["mix_w"][:] = 0.0
    w["mix_b"][:] = 0.0
    o3 = dec.decoder_estimate(p, Q, K, V, W, w, seq_len)
    assert np.all(o3["s_mix"][0] == 0.5)


def test_causal_decoder_never_looks_ahead():
    """Causal mode (causal Performer state, causal convolutions, no height reduction): rows <= t0
    are bit-identical when later positions change."""
    p = dec.DecoderParams(B=1, H=2, T=40, d=8, m=16, K=8, causal=True, scale=0.35)
    Q, K, V, W, a = _run(p)
    t0 = 22
    g = np.random.default_rng(0)
    Q2, K2, V2 = Q.copy(), K.copy(), V.copy()
    for X in (Q2, K2, V2):
        X[:, :, t0 + 1:] = g.standard_normal(X[:, :, t0 + 1:].shape) * 3
    b = dec.decoder_estimate(p, Q2, K2, V2, W, _wts(p.H, p.d, p.K))
    for k in ("A_hat", "s_mix", "s_prob", "Z"):
        assert np.array_equal(a[k][:, :, :t0 + 1], b[k][:, :, :t0 + 1]), k
    assert not np.array_equal(a["A_hat"][:, :, t0 + 1:], b["A_hat"][:, :, t0 + 1:])


def test_mlp_and_channel_layout_with_hand_set_weights():
    """mu = identity on the first 2d inputs, nu = pass-through of one hidden unit to one (column,
    channel) output, CNN = centre taps copying channel 0 of head 0: A_hat is then the softmax of
    a known image.  Fixes the order of the concatenation [C_perf; V], the ReLU placement and the
    x c_h + ch layout of nu's output."""
    B, H, T, d, Kc = 1, 1, 6, 4, 4
    p = dec.DecoderParams(B=B, H=H, T=T, d=d, m=8, K=Kc, causal=True, scale=0.5)
    Q, K, V = _qkv(B, H, T, d, 9, 0.5)
    W = np.random.default_rng(3).standard_normal((8, d))
    C, Wd, dh = p.channels, Kc // p.c_s, p.d_hidden
    w = {k: np.zeros_like(v) for k, v in _wts(H, d, Kc).items()}
    w["mu_w"][:, :2 * d] = np.eye(dh)[:, :2 * d]                # Z = relu(C_perf), all of it >= 0 on the V_I half
    w["nu1_w"][:] = np.eye(dh)
    src = [1, 2]                                               # hidden units feeding columns 0 and 1 of channel 0
    for x in range(Wd):
        w["nu2_w"][x * p.c_h + 0, src[x]] = 1.0
    for name in ("conv1_w", "conv2_w"):
        w[name][0, 2, 1, 0] = 1.0                              # centre tap of the causal window (row t, same column)
    w["conv3_w"][0, 2, 1, 0] = 1.0
    o = dec.decoder_estimate(p, Q, K, V, W, w)
    Cp = dec.performer_encoding(p, Q, K, V, W)[0, 0]
    img = np.stack([np.maximum(Cp[:, src[0]], 0), np.maximum(Cp[:, src[1]], 0)], -1)     # [T, Wd]
    logits = img[:, (np.arange(Kc) * Wd) // Kc]
    want = np.exp(logits) / np.exp(logits).sum(-1, keepdims=True)
    np.testing.assert_allclose(o["A_hat"][0, 0], want, rtol=1e-12)


def test_reduced_precision_mode_stays_close_to_the_plain_definition():
    p = dec.DecoderParams(B=1, H=2, T=64, d=16, m=32, K=16, causal=True, scale=0.25)
    Q, K, V, W, a = _run(p)
    pr = dec.DecoderParams(**{**p.__dict__, "round_bf16": True})
    b = dec.decoder_estimate(pr, Q, K, V, W, _wts(p.H, p.d, p.K))
    assert not np.array_equal(a["A_hat"], b["A_hat"])
    assert np.abs(a["A_hat"] - b["A_hat"]).max() <= 2e-2 * np.abs(a["A_hat"]).max()
