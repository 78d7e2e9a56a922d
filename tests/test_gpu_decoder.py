"""GPU parity of the decoder path (Sec. 3.1 "CNN Decoder", App. A.5.1) against oracle/decoder.py on
the same seeded inputs and random stand-in weights, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from oracle import decoder as dec
from paper_2310_01777_amd import synth
from tests.util import TOL, assert_close, oracle_params, to_np64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sea():
    from paper_2310_01777_amd import binding
    return binding


def _wl(name, B, H, T, m, K, k_hat, k_budget=0, causal=True, pad_frac=0.0, grouping=0):
    return synth.Workload(name, B, H, T, 64, m, K, k_hat, k_budget, causal, "bf16", 4, pad_frac, grouping=grouping)


CASES = [
    _wl("dec_causal", 2, 2, 203, 64, 16, 4),
    _wl("dec_causal_m128_tiles", 1, 4, 256, 128, 32, 8),
    _wl("dec_bidir_pad", 2, 2, 192, 64, 16, 4, causal=False, pad_frac=0.3),
    _wl("dec_bidir_odd_T", 1, 2, 151, 128, 8, 2, causal=False),
    _wl("dec_causal_pad_m256", 2, 2, 160, 256, 32, 6, pad_frac=0.3),
    _wl("dec_grouped", 1, 4, 128, 64, 32, 4, grouping=1),
    _wl("dec_c2_one_batch", 1, 12, 2048, 128, 128, 64),
]


def _params(sea, wl, seq_len_dev=None):
    return sea.SeaParams(B=wl.B, H=wl.H, T=wl.T, d=wl.d, m=wl.m, K=wl.K, k_hat=wl.k_hat, k_budget=wl.k_budget,
                         causal=wl.causal, scale=wl.scale, dtype=wl.dtype, seq_len=seq_len_dev, grouping=wl.grouping)


@pytest.mark.parametrize("wl", CASES, ids=lambda w: w.name)
def test_decoder_matches_oracle(sea, wl):
    x = synth.make_inputs(wl)
    wts = synth.decoder_weights(wl.H, wl.d, wl.K)
    d = {k: x[k].cuda() for k in "QKVW"}
    sl_dev = None if x["seq_len"] is None else x["seq_len"].cuda()
    sl = None if x["seq_len"] is None else x["seq_len"].numpy()
    wd = {k: v.cuda() for k, v in wts.items()}
    p = _params(sea, wl, sl_dev)
    n = (wl.B, wl.H, wl.T)
    ws = torch.empty(sea.sea_decoder_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    assert ws.numel() > 0
    A = torch.full((*n, wl.K), float("nan"), dtype=torch.float32, device="cuda")
    s_mix = torch.empty(*n, dtype=torch.float32, device="cuda")
    s_prob = torch.empty(*n, dtype=torch.float32, device="cuda")
    print(f"[case] decoder {wl.name} B{wl.B} H{wl.H} T{wl.T} m{wl.m} K{wl.K} causal{int(wl.causal)} grouping{wl.grouping}", flush=True)
    sea.sea_decoder_estimate(p, wd, d["Q"], d["K"], d["V"], d["W"], A, ws, s_mix=s_mix, s_prob=s_prob)
    torch.cuda.synchronize()
    A_g = A.cpu().numpy().astype(np.float64)

    pd = dec.DecoderParams(B=wl.B, H=wl.H, T=wl.T, d=wl.d, m=wl.m, K=wl.K, causal=wl.causal, scale=wl.scale,
                           round_bf16=True)
    f = {k: to_np64(v) for k, v in wts.items()}
    o = dec.decoder_estimate(pd, to_np64(x["Q"]), to_np64(x["K"]), to_np64(x["V"]), to_np64(x["W"]), f, sl)
    tol = TOL["bf16"]
    assert_close(A_g, o["A_hat"], tol, "decoder A_hat")
    active = o["A_hat"].sum(-1) > 0
    np.testing.assert_allclose(A_g.sum(-1)[active], 1.0, atol=1e-5)
    assert (A_g[~active] == 0).all()
    assert_close(s_mix.cpu().numpy(), o["s_mix"], tol, "s_mix")
    assert_close(s_prob.cpu().numpy(), o["s_prob"], tol, "s_prob")
    # and against the plain fp64 definition (no rounding points): looser, the CNN amplifies bf16 steps
    pp = dec.DecoderParams(**{**pd.__dict__, "round_bf16": False})
    if wl.T <= 512:
        op = dec.decoder_estimate(pp, to_np64(x["Q"]), to_np64(x["K"]), to_np64(x["V"]), to_np64(x["W"]), f, sl)
        assert_close(A_g, op["A_hat"], 2 * tol, "decoder A_hat vs plain")

    # the whole layer: selection and lists on the GPU's own A_hat, attention, output mixing
    O = torch.full((*n, wl.d), float("nan"), dtype=torch.bfloat16, device="cuda")
    A2 = torch.empty_like(A)
    sea.sea_decoder_forward(p, wd, d["Q"], d["K"], d["V"], d["W"], O, ws, A_hat=A2)
    torch.cuda.synchronize()
    assert torch.equal(A2, A)
    po = oracle_params(wl)
    sel, idx, cnt = oracle.topk_mask(po, A_g, seq_len=sl)
    C = oracle.sparse_attn(po, to_np64(x["Q"]), to_np64(x["K"]), to_np64(x["V"]), idx, cnt)
    want = oracle.output_mix(po, C, to_np64(x["V"]), s_mix.cpu().numpy(), s_prob=s_prob.cpu().numpy(), A_hat=A_g,
                             seq_len=sl if sl is not None else np.full(wl.B, wl.T, dtype=np.int32))
    assert_close(to_np64(O), want, tol, "C_sea")


def test_decoder_rejects_unsupported_shapes(sea):
    wl = _wl("dec_bad", 1, 3, 64, 64, 16, 4)        # 4 H = 12 channels: not a multiple of 8
    p = _params(sea, wl)
    assert sea.sea_decoder_workspace_bytes(p) == 0
    wl = _wl("dec_bad_m", 1, 2, 64, 96, 16, 4)
    assert sea.sea_decoder_workspace_bytes(_params(sea, wl)) == 0
