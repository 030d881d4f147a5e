"""The full-precision modes of the HIP path (shape.bits_proj / bits_q / bits_prob = 16) against the oracle.

With every K/V row protected and nothing quantized, Eq. (2) and Eq. (3) reduce to plain softmax attention: the GPU
result must then agree with the oracle run in the same mode AND with torch's float64 scaled_dot_product_attention
(which shares nothing with either). The mixed cases switch one quantizer off at a time.
"""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import taq_oracle as O
from paper_2603_22943_amd import synth
from paper_2603_22943_amd import taq as T
from tests import gpu_helpers as G

pytestmark = pytest.mark.gpu


def run_gpu(L, bits_kv, bits_q, bits_prob, bits_proj, prob_grid="linear"):
    s = T.make_shape(B=L.B, N=L.N, C=L.C, H=L.H, T=L.T, Cc=L.Cc, bits_kv=bits_kv, bits_q=bits_q, bits_prob=bits_prob,
                     bits_proj=bits_proj, prob_grid={"linear": 0, "log2": 1, "rowmax": 2}[prob_grid])
    mask = G.dev(L.mask)
    if bits_proj == 16:
        wq, wo = G.dev(L.Wq), G.dev(L.Wo)
        scales = torch.cat([torch.full((2 * L.C,), float("nan"), device=G.DEV), G.dev(L.bias_o)]).contiguous()  # only the bias is read
    else:
        wq, swq = T.taq_quantize_weight(G.dev(L.Wq))
        wo, swo = T.taq_quantize_weight(G.dev(L.Wo))
        scales = torch.cat([swq, swo, G.dev(L.bias_o)]).contiguous()
    packed = torch.full((T.taq_kv_packed_bytes(s),), 0xFF, dtype=torch.uint8, device=G.DEV)
    ws = torch.full((T.taq_workspace_bytes(s),), 0xFF, dtype=torch.uint8, device=G.DEV)
    T.taq_quantize_kv(G.dev(L.context), mask, G.dev(L.Wk), G.dev(L.Wv), bits_kv, s, packed, ws)
    kvd = {k: v.cpu().numpy() for k, v in T.taq_unpack_kv(packed, s).items()}
    dbg, taps = T.make_debug(s, G.DEV)
    ws.fill_(0xFF)
    out = T.taq_cross_attn(G.dev(L.hidden), packed, wq, wo, scales, mask, s, workspace=ws, debug=dbg)
    torch.cuda.synchronize()
    return out.cpu().numpy(), kvd, {k: v.cpu().numpy() for k, v in taps.items()}


def oracle_on_device_rows(L, kvd, bits_kv, bits_q, bits_prob, bits_proj, prob_grid):
    """The oracle in the same mode; protected rows (float sums rounded to fp16: within one step of the oracle's, checked
    by the caller) are taken from the device so that everything downstream compares at float32-vs-float64 level."""
    kv = O.quantize_kv(L.context, L.mask, L.Wk, L.Wv, bits_kv, L.H, bits_proj=bits_proj)
    for name, full in (("K16", kv.K16), ("V16", kv.V16)):
        got = kvd[name].astype(np.float64)
        step = np.spacing(np.abs(full).astype(np.float16)).astype(np.float64)
        absx = np.abs(L.context.astype(np.float64))
        W = (L.Wk if name == "K16" else L.Wv).astype(np.float64)
        if bits_proj == 8:
            W = np.abs(kv.aux[name[0].lower() + "_w_code"].astype(np.float64)) * kv.aux[name[0].lower() + "_s_w"].astype(np.float64)[:, None]
        bound = step + (L.Cc + 4) * 2.0 ** -24 * np.einsum("btk,ck->btc", absx, np.abs(W))
        assert np.all(np.abs(got - full)[kv.mask] <= bound[kv.mask]), name
        assert np.all(kvd[name][~kv.mask] == 0)
    kv = dataclasses.replace(kv, K16=np.where(kv.mask[:, :, None], kvd["K16"].astype(np.float64), 0.0),
                             V16=np.where(kv.mask[:, :, None], kvd["V16"].astype(np.float64), 0.0))
    wq_code, s_wq = O.quantize_weight(L.Wq)
    wo_code, s_wo = O.quantize_weight(L.Wo)
    out, aux = O.cross_attn(L.hidden, kv, wq_code, s_wq, wo_code, s_wo, L.bias_o, bits_prob=bits_prob, bits_q=bits_q,
                            bits_proj=bits_proj, Wq_f16=L.Wq, Wo_f16=L.Wo, return_aux=True, prob_grid=prob_grid)
    return out, aux, kv


@pytest.mark.parametrize("C,H,N,T_", [(320, 8, 100, 77), (96, 4, 70, 33), (1280, 8, 40, 77), (128, 2, 33, 96)])
def test_everything_unquantized_is_plain_softmax_attention(C, H, N, T_):
    L = synth.make_layer("ident", seed=C + N, B=2, N=N, C=C, H=H, Cc=96, T=T_, bits_kv=16, trigger_positions=(2,),
                         trigger_scale=3.0, bias=True, outlier_frac=0.01)
    out, kvd, taps = run_gpu(L, 16, 16, 16, 16)
    ref, aux, kv = oracle_on_device_rows(L, kvd, 16, 16, 16, 16, "linear")
    # independent of the oracle's attention code: torch float64 SDPA on the same (device) K/V rows
    d = C // H
    Q = torch.from_numpy(L.hidden.astype(np.float64) @ L.Wq.astype(np.float64).T).reshape(L.B, N, H, d).transpose(1, 2)
    K = torch.from_numpy(kv.K16).reshape(L.B, T_, H, d).transpose(1, 2)
    V = torch.from_numpy(kv.V16).reshape(L.B, T_, H, d).transpose(1, 2)
    Osd = torch.nn.functional.scaled_dot_product_attention(Q, K, V).transpose(1, 2).reshape(L.B, N, C).numpy()
    Ysd = (Osd @ L.Wo.astype(np.float64).T + L.bias_o.astype(np.float64)).astype(np.float16)
    assert np.max(np.abs(Osd - aux["O"])) <= 1e-10 * max(1.0, np.abs(Osd).max())
    scale = np.abs(aux["O"]).max()
    dO = np.abs(taps["O"].astype(np.float64) - aux["O"])
    print(f"[case] identity C={C} H={H} N={N} T={T_}: max|dO|/max|O| = {dO.max() / scale:.2e}", flush=True)
    assert dO.max() <= 2e-5 * scale  # float32 (to_q sums of C terms, softmax, T-term sums) against float64
    # to_out in float32 (C-term sums, O itself within dO of the oracle's), one rounding to fp16 on both sides
    absWo = np.abs(L.Wo.astype(np.float64))
    slack = (C + 4) * 2.0 ** -24 * (np.abs(aux["O"]) @ absWo.T) + dO.max() * absWo.sum(axis=1)[None, None, :]
    for want in (ref, Ysd):
        gap = np.abs(out.astype(np.float64) - want.astype(np.float64))
        step = np.spacing(np.abs(want).astype(np.float16)).astype(np.float64)
        assert np.all(gap <= step + slack), float((gap - step - slack).max())
        assert np.mean(gap != 0) < 2e-2


@pytest.mark.parametrize("bits_kv,bits_q,bits_prob,bits_proj,grid", [
    (8, 16, 8, 8, "linear"),    # Q unquantized only
    (8, 8, 16, 8, "linear"),    # probabilities unquantized only
    (4, 16, 16, 8, "linear"),   # W8A8 projections, 4-bit K/V rows, nothing else quantized
    (8, 8, 8, 16, "linear"),    # unquantized projections, quantized attention
    (8, 16, 4, 16, "log2"),     # ... with the 4-bit logarithmic grid
    (4, 4, 16, 16, "linear"),
    (8, 16, 8, 16, "rowmax"),
])
@pytest.mark.parametrize("C,H,N", [(320, 8, 90), (96, 4, 70)])
def test_one_quantizer_switched_off_at_a_time(C, H, N, bits_kv, bits_q, bits_prob, bits_proj, grid):
    L = synth.make_layer("mixed", seed=C + N + bits_q + bits_prob, B=2, N=N, C=C, H=H, Cc=64, T=77, bits_kv=bits_kv,
                         trigger_positions=(3, 40), trigger_scale=3.0, bias=True)
    out, kvd, taps = run_gpu(L, bits_kv, bits_q, bits_prob, bits_proj, grid)
    ref, aux, kv = oracle_on_device_rows(L, kvd, bits_kv, bits_q, bits_prob, bits_proj, grid)
    if bits_proj == 8:  # exact integer projections: codes and scales bit for bit, as on the quantized path
        assert np.array_equal(kvd["k_code"].astype(np.int32), kv.k_code) and np.array_equal(kvd["s_K"], kv.s_K)
        assert np.array_equal(kvd["v_code"].astype(np.int32), kv.v_code) and np.array_equal(kvd["s_V"], kv.s_V)
        if bits_q != 16:
            assert np.array_equal(taps["q_code"].astype(np.int32), aux["q_code"]) and np.array_equal(taps["s_Q"], aux["s_Q"])
    else:  # rows are float sums: a code may move by one where the sum is within float32 rounding of a tie
        for name, code in (("k_code", kv.k_code), ("v_code", kv.v_code)):
            dcode = np.abs(kvd[name].astype(np.int32) - code)
            assert dcode.max() <= 1 and np.mean(dcode != 0) < 1e-3, name
    max_abs, rel_l2 = G.out_errors(out, ref)
    print(f"[case] kv{bits_kv} q{bits_q} p{bits_prob} proj{bits_proj} {grid} C={C}: out max_abs={max_abs:.3e} rel_l2={rel_l2:.3e}", flush=True)
    assert max_abs <= 2e-2 and rel_l2 <= 5e-3
