"""Token-sensitivity sweep (Section III-B, Eq. 1, on block outputs with MSE) on the HIP path against
the same sweep through the oracle: one text token's K/V rows quantized at a time."""
import numpy as np
import pytest
import torch

from oracle import taq_oracle as O
from paper_2603_22943_amd import sensitivity, synth
from paper_2603_22943_amd import taq as T
from tests import gpu_helpers as G

pytestmark = pytest.mark.gpu


def oracle_sweep(L, bits, tokens, full):
    """Eq. (1) through the oracle: y* with every row kept in fp16; full = everything else unquantized too."""
    wq_code, s_wq = O.quantize_weight(L.Wq)
    wo_code, s_wo = O.quantize_weight(L.Wo)
    w = 16 if full else 8

    def block(mask, b):
        kv = O.quantize_kv(L.context, mask, L.Wk, L.Wv, b, L.H, bits_proj=w)
        return O.cross_attn(L.hidden, kv, wq_code, s_wq, wo_code, s_wo, L.bias_o, bits_q=w, bits_prob=w, bits_proj=w,
                            Wq_f16=L.Wq, Wo_f16=L.Wo).astype(np.float64)

    all_on = np.ones_like(L.mask)
    y_star = block(all_on, 16)
    out = {}
    for b in bits:
        d = []
        for i in tokens:
            m = all_on.copy()
            m[:, i] = 0
            d.append(float(np.mean((block(m, b) - y_star) ** 2)))
        out[b] = np.array(d)
    return out


@pytest.mark.parametrize("full", [True, False])
@pytest.mark.parametrize("C,H,N", [(320, 8, 96), (96, 4, 64)])  # single-kernel path (when quantized), kernel-per-stage path
def test_token_sensitivity_matches_oracle_and_triggers_are_fragile(C, H, N, full):
    """full: everything but token i's rows in full precision, as Eq. (1) states (bits_q = bits_prob = bits_proj = 16);
    otherwise the same sweep inside the W8A8 block."""
    trig = (3, 4)
    L = synth.make_layer("sens", seed=C + N, B=2, N=N, C=C, H=H, Cc=64, T=20, bits_kv=8,
                         trigger_positions=trig, trigger_scale=3.0)
    tokens = list(range(L.T))
    if full:
        s = T.make_shape(B=L.B, N=L.N, C=L.C, H=L.H, T=L.T, Cc=L.Cc, bits_kv=8, bits_q=16, bits_prob=16, bits_proj=16)
        wq, wo = G.dev(L.Wq), G.dev(L.Wo)
        scales = torch.cat([torch.zeros(2 * C, dtype=torch.float32, device=G.DEV), G.dev(L.bias_o)]).contiguous()
    else:
        s = G.shape_of(L)
        wq, swq = T.taq_quantize_weight(G.dev(L.Wq))
        wo, swo = T.taq_quantize_weight(G.dev(L.Wo))
        scales = torch.cat([swq, swo, G.dev(L.bias_o)]).contiguous()
    got = sensitivity.token_sensitivity(G.dev(L.hidden), G.dev(L.context), G.dev(L.Wk), G.dev(L.Wv), wq, wo, scales, s,
                                        bits=(8, 4), tokens=tokens)
    ref = oracle_sweep(L, (8, 4), tokens, full)
    for b in (8, 4):
        g, r = got[b].numpy(), ref[b]
        print(f"[sens C={C} full={full}] b={b}: oracle median {np.median(r):.3e} trig {r[list(trig)]}  gpu/oracle max dev "
              f"{np.max(np.abs(g / r - 1)):.3e}", flush=True)
        # both sides round the outputs to fp16, and the HIP path's outputs carry its float32 arithmetic, so the two
        # Delta differ by the occasional fp16 step of an output (measured: < 1e-3 relative at 4 bits); at 8 bits in
        # the full-precision sweep Delta itself is only a few fp16 steps of the outputs, hence the wider bar there
        assert np.all(np.abs(g / r - 1) <= (5e-2 if (full and b == 8) else 1e-2))
        others = np.delete(g, list(trig))
        assert np.all(g[list(trig)] > np.median(others)) and g[list(trig)].mean() > 2.0 * others.mean()
    assert np.all(got[4].numpy() > got[8].numpy())  # fewer bits hurt more, token by token


def test_mse_kernel_against_numpy():
    rng = np.random.Generator(np.random.PCG64(11))
    x = rng.standard_normal(100003).astype(np.float16)
    y = (x.astype(np.float32) + 0.01 * rng.standard_normal(100003)).astype(np.float16)
    got = float(T.taq_mse_f16(G.dev(x), G.dev(y)).cpu()[0])
    want = float(np.mean((x.astype(np.float64) - y.astype(np.float64)) ** 2))
    assert abs(got / want - 1) < 1e-12


def test_token_sensitivity_argument_checks():
    L = synth.make_layer("sensargs", seed=5, B=1, N=8, C=64, H=2, Cc=64, T=5, bits_kv=8, trigger_positions=(1,))
    s = G.shape_of(L)
    wq, swq = T.taq_quantize_weight(G.dev(L.Wq))
    wo, swo = T.taq_quantize_weight(G.dev(L.Wo))
    scales = torch.cat([swq, swo, G.dev(L.bias_o)]).contiguous()
    args = (G.dev(L.hidden), G.dev(L.context), G.dev(L.Wk), G.dev(L.Wv), wq, wo, scales, s)
    with pytest.raises(ValueError):
        sensitivity.token_sensitivity(*args, bits=(16,))
    with pytest.raises(ValueError):
        sensitivity.token_sensitivity(*args, tokens=[L.T])
    d = sensitivity.token_sensitivity(*args, bits=(4,), tokens=[0, 1])
    assert d[4].shape == (2,) and torch.all(d[4] >= 0)
