"""Pins of the oracle's TAQ block against textbook attention, closed forms,
pass-through invariants, metamorphic properties and a separately written scalar
brute force (CPU only)."""
import numpy as np
import pytest
import torch

from oracle import taq_oracle as O
from oracle import brute
from paper_2603_22943_amd import synth


def small_layer(seed=3, B=2, N=24, C=48, H=4, T=13, Cc=40, bits_kv=8, trig=(2, 3), scale=3.0, bias=True):
    return synth.make_layer("small", seed=seed, B=B, N=N, C=C, H=H, T=T, Cc=Cc, bits_kv=bits_kv,
                            trigger_positions=trig, trigger_scale=scale, bias=bias)


# ---------------------------------------------------------------- textbook special case

def test_all_protected_16bit_equals_textbook_attention():
    """Mask all ones and 16 bits everywhere: Eq. (2),(3) reduce to plain
    softmax(QK^T/sqrt(d))V with fp projections. Checked against torch's float64
    scaled_dot_product_attention, a routine the oracle does not use."""
    L = small_layer(trig=tuple(range(13)))
    out = O.taq_block(L, bits_prob=16, bits_q=16, bits_proj=16, bits_kv=16, store_f16=False)
    x = torch.from_numpy(L.hidden.astype(np.float64))
    ctx = torch.from_numpy(L.context.astype(np.float64))
    Wq, Wk, Wv, Wo = (torch.from_numpy(w.astype(np.float64)) for w in (L.Wq, L.Wk, L.Wv, L.Wo))
    B, N, C = x.shape
    H, d = L.H, L.d
    q = (x @ Wq.T).view(B, N, H, d).transpose(1, 2)
    k = (ctx @ Wk.T).view(B, L.T, H, d).transpose(1, 2)
    v = (ctx @ Wv.T).view(B, L.T, H, d).transpose(1, 2)
    o = torch.nn.functional.scaled_dot_product_attention(q, k, v)
    ref = o.transpose(1, 2).reshape(B, N, C) @ Wo.T + torch.from_numpy(L.bias_o.astype(np.float64))
    assert np.max(np.abs(out - ref.numpy())) < 1e-12
    # bits_kv=16 alone protects every row whatever the mask says
    L2 = small_layer(trig=())
    out2 = O.taq_block(L2, bits_prob=16, bits_q=16, bits_proj=16, bits_kv=16, store_f16=False)
    L3 = small_layer(trig=tuple(range(13)), scale=1.0)
    out3 = O.taq_block(L3, bits_prob=16, bits_q=16, bits_proj=16, bits_kv=16, store_f16=False)
    assert np.max(np.abs(out2 - out3)) < 1e-12


def test_quantized_block_is_close_to_textbook_and_closer_with_more_bits():
    L = small_layer(N=64)
    ref = O.taq_block(L, bits_prob=16, bits_q=16, bits_proj=16, bits_kv=16, store_f16=False)
    e8 = np.linalg.norm(O.taq_block(L, bits_kv=8).astype(np.float64) - ref) / np.linalg.norm(ref)
    e4 = np.linalg.norm(O.taq_block(L, bits_kv=4).astype(np.float64) - ref) / np.linalg.norm(ref)
    assert e8 < 0.05 and e8 < e4 < 0.5


# ---------------------------------------------------------------- pass-through invariants

def test_trigger_rows_and_columns_pass_through():
    L = small_layer(bits_kv=4)
    out, aux = O.taq_block(L, return_aux=True)
    kv = aux["kv"]
    # protected rows of K~ / V~ are what the all-protected run stores for those rows
    Lall = small_layer(bits_kv=4, trig=(2, 3))
    kv_all = O.quantize_kv(Lall.context, Lall.mask, Lall.Wk, Lall.Wv, 16, Lall.H)
    for t in (2, 3):
        assert np.array_equal(kv.dequant("k")[:, t], kv_all.K16[:, t])
        assert np.array_equal(kv.dequant("v")[:, t], kv_all.V16[:, t])
        assert np.all(kv.k_code[:, t] == 0) and np.all(kv.s_K[:, :, t] == 0)
    # those rows are fp16-representable (stored as fp16)
    assert np.array_equal(kv.K16, kv.K16.astype(np.float16).astype(np.float64))
    # trigger columns of A^ are A itself; other columns sit on the 1/255 grid
    A, Ah = aux["A"], aux["A_hat"]
    assert np.array_equal(Ah[..., [2, 3]], A[..., [2, 3]])
    other = [t for t in range(L.T) if t not in (2, 3)]
    grid = Ah[..., other] * 255.0
    assert np.max(np.abs(grid - np.rint(grid))) < 1e-12
    # unprotected rows really are on their int grid: |code| <= 7 and some row reaches 7
    assert np.abs(kv.k_code).max() == 7 and np.abs(kv.v_code).max() == 7


def test_q_is_quantized_even_against_trigger_rows():
    """Eq. (2) third line has no mask: with every K/V row protected and
    probabilities unquantized, the only difference to the fp block is Q~."""
    L = small_layer(trig=tuple(range(13)))
    out, aux = O.taq_block(L, bits_prob=16, return_aux=True)
    B, N, C = L.hidden.shape
    q = aux["q_code"].reshape(B, N, L.H, L.d)
    assert np.all(np.abs(q).max(axis=-1) == 127)
    # scores are formed from the dequantised codes: recompute one by hand
    b, n, h, t = 1, 5, 2, 7
    qd = q[b, n, h].astype(np.float64) * float(aux["s_Q"][b, n, h])
    kd = aux["kv"].K16[b, :, h * L.d:(h + 1) * L.d]
    s = (kd @ qd) / np.sqrt(L.d)
    a = np.exp(s - s.max())
    a /= a.sum()
    assert aux["A"][b, n, h, t] == pytest.approx(a[t], rel=1e-12)


# ---------------------------------------------------------------- softmax / probability grid

def test_softmax_rows_sum_to_one_and_quantized_rows_within_bound():
    L = small_layer(N=40)
    _, aux = O.taq_block(L, return_aux=True)
    A, Ah = aux["A"], aux["A_hat"]
    assert np.all(A >= 0) and np.max(np.abs(A.sum(-1) - 1.0)) < 1e-12
    n_other = L.T - 2
    assert np.max(np.abs(Ah.sum(-1) - 1.0)) <= n_other / 510.0 + 1e-12
    assert np.max(np.abs(Ah - A)) <= 1.0 / 510.0 + 1e-7


def test_uniform_scores_closed_form():
    """All K codes zero -> every score is 0 -> A = 1/77 exactly. With one
    protected column: sum(A^) = 76*rint(255/77)/255 + 1/77 = 76*3/255 + 1/77,
    and with identical V rows v the output is that sum times v."""
    B, N, H, d, T = 1, 3, 2, 4, 77
    C = H * d
    mask = np.zeros((B, T), dtype=bool)
    mask[0, 5] = True
    v_row = np.arange(1, C + 1, dtype=np.float64) / 8.0  # fp16-exact
    v_code = np.zeros((B, T, C), dtype=np.int32)
    s_V = np.zeros((B, H, T), dtype=np.float32)
    # unprotected rows: codes c with scale 1/8 reproduce v_row exactly
    v_code[:, ~mask[0]] = np.arange(1, C + 1)
    s_V[:, :, ~mask[0]] = 0.125
    V16 = np.zeros((B, T, C))
    V16[0, 5] = v_row
    kv = O.QuantKV(B=B, T=T, C=C, H=H, bits_kv=8, mask=mask,
                   k_code=np.zeros((B, T, C), dtype=np.int32), v_code=v_code,
                   s_K=np.ones((B, H, T), dtype=np.float32), s_V=s_V,
                   K16=np.zeros((B, T, C)), V16=V16)
    rng = np.random.Generator(np.random.PCG64(1))
    hidden = rng.standard_normal((B, N, C)).astype(np.float16)
    wq, swq = O.quantize_weight(np.eye(C, dtype=np.float16))
    out, aux = O.cross_attn(hidden, kv, wq, swq, wq, swq, return_aux=True)
    total = 76 * 3 / 255.0 + 1 / 77.0
    assert np.max(np.abs(aux["A"] - 1 / 77.0)) < 1e-15
    assert np.max(np.abs(aux["A_hat"].sum(-1) - total)) < 1e-14
    assert total == pytest.approx(0.907, abs=5e-4)
    assert np.max(np.abs(aux["O"] - total * v_row[None, None, :])) < 1e-13


# ---------------------------------------------------------------- brute force

@pytest.mark.parametrize("case", [
    dict(seed=7, B=1, N=4, C=4, H=1, T=5, Cc=6, bits_kv=8, trig=(1,)),
    dict(seed=8, B=2, N=3, C=8, H=2, T=4, Cc=5, bits_kv=4, trig=(0, 3)),
    dict(seed=9, B=1, N=4, C=6, H=3, T=3, Cc=4, bits_kv=8, trig=()),
    dict(seed=10, B=1, N=2, C=4, H=1, T=4, Cc=3, bits_kv=16, trig=(2,)),
    dict(seed=12, B=1, N=3, C=8, H=2, T=5, Cc=7, bits_kv=4, trig=(0, 1, 2, 3, 4)),
])
def test_block_matches_scalar_brute_force(case):
    L = synth.make_layer("t", seed=case["seed"], B=case["B"], N=case["N"], C=case["C"], H=case["H"],
                         T=case["T"], Cc=case["Cc"], bits_kv=case["bits_kv"],
                         trigger_positions=case["trig"], trigger_scale=3.0, bias=True)
    out, aux = O.taq_block(L, return_aux=True)
    ref, dump = brute.taq_block_brute(L.context, L.mask, L.Wq, L.Wk, L.Wv, L.Wo, L.bias_o, L.hidden,
                                      L.H, L.bits_kv)
    kv = aux["kv"]
    for (b, t, c), v in dump["k_code"].items():
        assert kv.k_code[b, t, c] == v
    for (b, t, c), v in dump["v_code"].items():
        assert kv.v_code[b, t, c] == v
    for (b, t, c), v in dump["K16"].items():
        assert kv.K16[b, t, c] == v
    for (b, t, c), v in dump["V16"].items():
        assert kv.V16[b, t, c] == v
    for (b, n, c), v in dump["q_code"].items():
        assert aux["q_code"][b, n, c] == v
    for (b, n, h, t), v in dump["p_code"].items():
        assert aux["p_code"][b, n, h, t] == v
    for (b, n, c), v in dump["o_code"].items():
        assert aux["o_code"][b, n, c] == v
    # number of quantized entries is what the mask says
    n_prot = int(kv.mask.sum())
    assert len(dump["k_code"]) == (L.B * L.T - n_prot) * L.C
    assert len(dump["K16"]) == n_prot * L.C
    ref = np.array(ref)
    assert np.max(np.abs(out.astype(np.float64) - ref)) <= 1e-3 * max(1.0, np.abs(ref).max())
    assert np.mean(out.astype(np.float64) == ref) > 0.95  # same fp16 value almost everywhere


# ---------------------------------------------------------------- metamorphic properties

def test_text_token_permutation_invariance():
    L = small_layer(N=16)
    out = O.taq_block(L).astype(np.float64)
    perm = np.random.Generator(np.random.PCG64(4)).permutation(L.T)
    L2 = small_layer(N=16)
    L2.context = L.context[:, perm]
    L2.mask = L.mask[:, perm]
    out2 = O.taq_block(L2).astype(np.float64)
    # identical up to summation order (one fp16 step at most, rarely)
    assert np.max(np.abs(out - out2)) <= 2e-3 * np.abs(out).max()
    assert np.mean(out == out2) > 0.98


def test_query_rows_and_batch_elements_are_independent():
    L = small_layer(N=16)
    out = O.taq_block(L)
    L2 = small_layer(N=16)
    L2.hidden = L.hidden[:, 4:9].copy()
    out2 = O.taq_block(L2)
    assert np.array_equal(out[:, 4:9], out2)
    L3 = small_layer(N=16)
    L3.hidden, L3.context, L3.mask = L.hidden[1:], L.context[1:], L.mask[1:]
    L3.B = 1
    assert np.array_equal(O.taq_block(L3), out[1:])


def test_empty_mask_is_plain_uniform_quantization():
    """'Separate trigger tokens: no' in the paper's ablation = the same block
    with nothing protected: every K/V row on its int grid, every probability on
    the 1/255 grid."""
    L = small_layer(trig=())
    _, aux = O.taq_block(L, return_aux=True)
    kv = aux["kv"]
    assert not kv.mask.any() and np.all(kv.K16 == 0) and np.all(kv.V16 == 0)
    assert np.all(np.abs(kv.k_code.reshape(L.B, L.T, L.H, L.d)).max(-1) == 127)
    g = aux["A_hat"] * 255.0
    assert np.max(np.abs(g - np.rint(g))) < 1e-12
    # protecting a row moves the output towards the unquantized block (direction of the ablation)
    Lp = small_layer(trig=(2, 3))
    ref = O.taq_block(Lp, bits_prob=16, bits_q=16, bits_proj=16, bits_kv=16, store_f16=False)
    e_prot = np.linalg.norm(O.taq_block(Lp, bits_kv=4).astype(np.float64) - ref)
    Lu = small_layer(trig=(2, 3))
    Lu.mask[:] = 0
    e_unprot = np.linalg.norm(O.taq_block(Lu, bits_kv=4).astype(np.float64) - ref)
    assert e_prot < e_unprot


def test_token_sensitivity_trigger_rows_are_more_fragile():
    """Per-token sensitivity (Eq. 1) on block outputs with MSE: quantize only
    token i's K/V rows to 4 bits (protect every other row, keep everything else
    in full precision). The x3 trigger rows must hurt more than a typical word."""
    L = small_layer(N=64, T=13, trig=(2, 3))
    ref = O.taq_block(L, bits_prob=16, bits_q=16, bits_proj=16, bits_kv=16, store_f16=False)
    delta = []
    for i in range(L.T):
        Li = small_layer(N=64, T=13, trig=(2, 3))
        Li.mask[:] = 1
        Li.mask[:, i] = 0
        kv = O.quantize_kv(Li.context, Li.mask, Li.Wk, Li.Wv, 4, Li.H, bits_proj=16, store_f16=False)
        out = O.cross_attn(Li.hidden, kv, None, None, None, None, Li.bias_o, bits_prob=16, bits_q=16,
                           bits_proj=16, store_f16=False, Wq_f16=Li.Wq, Wo_f16=Li.Wo)
        delta.append(float(np.mean((out - ref) ** 2)))
    delta = np.array(delta)
    others = np.delete(delta, [2, 3])
    assert delta[2] > np.median(others) and delta[3] > np.median(others)
    assert delta[[2, 3]].mean() > 2.0 * others.mean()


def test_int4_codes_and_scales_shapes_and_ranges():
    L = small_layer(bits_kv=4)
    kv = O.quantize_kv(L.context, L.mask, L.Wk, L.Wv, 4, L.H)
    assert kv.k_code.shape == (L.B, L.T, L.C) and kv.s_K.shape == (L.B, L.H, L.T)
    assert kv.k_code.min() >= -7 and kv.k_code.max() <= 7
    # W8A8 projection accumulators equal an int64 matmul done token by token
    acc = kv.aux["k_acc"]
    xc, wc = kv.aux["k_x_code"], kv.aux["k_w_code"]
    for b in range(L.B):
        for t in (0, 5, 12):
            assert np.array_equal(acc[b, t], wc.astype(np.int64) @ xc[b, t].astype(np.int64))


# ---------------------------------------------------------------- 4-bit activations (the paper's "8/4" setting)

def test_a4_uniform_scores_closed_form():
    """4-bit probabilities: 1/77 rounds to code 0 on the 1/15 grid, so with uniform scores every unprotected
    column vanishes and only the protected column (kept exactly, Eq. 3) reaches the output: O = V_trigger / 77."""
    B, N, H, d, T = 1, 3, 2, 4, 77
    C = H * d
    mask = np.zeros((B, T), dtype=bool)
    mask[0, 5] = True
    v_row = np.arange(1, C + 1, dtype=np.float64) / 8.0
    v_code = np.zeros((B, T, C), dtype=np.int32)
    v_code[:, ~mask[0]] = 7
    s_V = np.full((B, H, T), 0.5, dtype=np.float32)
    V16 = np.zeros((B, T, C))
    V16[0, 5] = v_row
    kv = O.QuantKV(B=B, T=T, C=C, H=H, bits_kv=4, mask=mask, k_code=np.zeros((B, T, C), dtype=np.int32), v_code=v_code,
                   s_K=np.ones((B, H, T), dtype=np.float32), s_V=s_V, K16=np.zeros((B, T, C)), V16=V16)
    hidden = np.random.Generator(np.random.PCG64(1)).standard_normal((B, N, C)).astype(np.float16)
    wq, swq = O.quantize_weight(np.eye(C, dtype=np.float16))
    out, aux = O.cross_attn(hidden, kv, wq, swq, wq, swq, bits_prob=4, bits_q=4, return_aux=True)
    assert np.all(aux["p_code"] == 0)
    assert np.max(np.abs(aux["O"] - v_row[None, None, :] / 77.0)) < 1e-14
    assert np.abs(aux["q_code"]).max() == 7


@pytest.mark.parametrize("case", [
    dict(seed=21, B=1, N=4, C=8, H=2, T=5, Cc=6, bits_kv=4, trig=(1,)),
    dict(seed=22, B=2, N=3, C=4, H=1, T=4, Cc=5, bits_kv=8, trig=()),
])
def test_a4_block_matches_scalar_brute_force(case):
    L = synth.make_layer("t", seed=case["seed"], B=case["B"], N=case["N"], C=case["C"], H=case["H"], T=case["T"],
                         Cc=case["Cc"], bits_kv=case["bits_kv"], trigger_positions=case["trig"], trigger_scale=3.0, bias=True)
    out, aux = O.taq_block(L, bits_prob=4, bits_q=4, return_aux=True)
    ref, dump = brute.taq_block_brute(L.context, L.mask, L.Wq, L.Wk, L.Wv, L.Wo, L.bias_o, L.hidden, L.H, L.bits_kv,
                                      bits_q=4, bits_prob=4)
    for (b, n, c), v in dump["q_code"].items():
        assert aux["q_code"][b, n, c] == v and abs(v) <= 7
    for (b, n, h, t), v in dump["p_code"].items():
        assert aux["p_code"][b, n, h, t] == v and 0 <= v <= 15
    for (b, n, c), v in dump["o_code"].items():
        assert aux["o_code"][b, n, c] == v
    ref = np.array(ref)
    assert np.max(np.abs(out.astype(np.float64) - ref)) <= 1e-3 * max(1.0, np.abs(ref).max())


def test_a4_is_coarser_than_a8_and_trigger_columns_still_pass_through():
    L = small_layer(N=64)
    ref = O.taq_block(L, bits_prob=16, bits_q=16, bits_proj=16, bits_kv=16, store_f16=False)
    out8, aux8 = O.taq_block(L, return_aux=True)
    out4, aux4 = O.taq_block(L, bits_prob=4, bits_q=4, return_aux=True)
    e8 = np.linalg.norm(out8.astype(np.float64) - ref) / np.linalg.norm(ref)
    e4 = np.linalg.norm(out4.astype(np.float64) - ref) / np.linalg.norm(ref)
    assert e8 < e4 < 1.0
    assert np.array_equal(aux4["A_hat"][..., [2, 3]], aux4["A"][..., [2, 3]])
    g = aux4["A_hat"][..., [t for t in range(L.T) if t not in (2, 3)]] * 15.0
    assert np.max(np.abs(g - np.rint(g))) < 1e-12


# ---------------------------------------------------------------- logarithmic probability grid

def test_log2_grid_is_exact_on_uniform_attention_over_a_power_of_two_tokens():
    """Zero keys give uniform attention A = 1/T. With T = 64 that is a power of two, so the logarithmic grid keeps
    it exactly (codes 6) and the block equals the one with unquantized probabilities, while the linear 8-bit grid
    does not (255/64 rounds to 4, A^ = 4/255)."""
    B, N, H, d, T = 1, 5, 2, 4, 64
    C = H * d
    rng = np.random.Generator(np.random.PCG64(12))
    mask = np.zeros((B, T), dtype=bool)
    v_code = rng.integers(-127, 128, size=(B, T, C)).astype(np.int32)
    s_V = rng.uniform(0.01, 0.02, size=(B, H, T)).astype(np.float32)
    kv = O.QuantKV(B=B, T=T, C=C, H=H, bits_kv=8, mask=mask, k_code=np.zeros((B, T, C), dtype=np.int32), v_code=v_code,
                   s_K=np.ones((B, H, T), dtype=np.float32), s_V=s_V, K16=np.zeros((B, T, C)), V16=np.zeros((B, T, C)))
    hidden = rng.standard_normal((B, N, C)).astype(np.float16)
    wq, swq = O.quantize_weight(np.eye(C, dtype=np.float16))
    for bits in (4, 8):
        out_log, aux_log = O.cross_attn(hidden, kv, wq, swq, wq, swq, bits_prob=bits, prob_grid="log2", return_aux=True)
        out_fp, aux_fp = O.cross_attn(hidden, kv, wq, swq, wq, swq, bits_prob=16, return_aux=True)
        assert np.all(aux_log["p_code"] == 6)
        assert np.array_equal(aux_log["O"], aux_fp["O"]) and np.array_equal(out_log, out_fp)
    # column mean of V~ by hand
    Vt = kv.dequant("v")
    assert np.max(np.abs(aux_log["O"] - Vt.mean(axis=1)[:, None, :])) < 1e-15
    _, aux_lin = O.cross_attn(hidden, kv, wq, swq, wq, swq, bits_prob=8, return_aux=True)
    assert np.all(aux_lin["p_code"] == 4) and not np.allclose(aux_lin["O"], aux_fp["O"], rtol=1e-3)


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("case", [
    dict(seed=31, B=1, N=4, C=8, H=2, T=5, Cc=6, bits_kv=4, trig=(1,)),
    dict(seed=32, B=2, N=3, C=4, H=1, T=9, Cc=5, bits_kv=8, trig=()),
])
def test_log2_grid_block_matches_scalar_brute_force(case, bits):
    L = synth.make_layer("t", seed=case["seed"], B=case["B"], N=case["N"], C=case["C"], H=case["H"], T=case["T"],
                         Cc=case["Cc"], bits_kv=case["bits_kv"], trigger_positions=case["trig"], trigger_scale=3.0, bias=True)
    out, aux = O.taq_block(L, bits_prob=bits, prob_grid="log2", return_aux=True)
    ref, dump = brute.taq_block_brute(L.context, L.mask, L.Wq, L.Wk, L.Wv, L.Wo, L.bias_o, L.hidden, L.H, L.bits_kv,
                                      bits_prob=bits, prob_grid="log2")
    assert len(dump["p_code"]) == L.B * L.N * L.H * (L.T - len(case["trig"]))
    for (b, n, h, t), v in dump["p_code"].items():
        assert aux["p_code"][b, n, h, t] == v and 0 <= v <= (1 << bits) - 1
    for (b, n, c), v in dump["o_code"].items():
        assert aux["o_code"][b, n, c] == v
    ref = np.array(ref)
    assert np.max(np.abs(out.astype(np.float64) - ref)) <= 1e-3 * max(1.0, np.abs(ref).max())


def test_log2_grid_keeps_trigger_columns_and_puts_the_rest_on_powers_of_two():
    L = small_layer(N=64)
    out, aux = O.taq_block(L, bits_prob=4, prob_grid="log2", return_aux=True)
    assert np.array_equal(aux["A_hat"][..., [2, 3]], aux["A"][..., [2, 3]])       # Eq. (3): M_A columns keep A
    rest = aux["A_hat"][..., [t for t in range(L.T) if t not in (2, 3)]]
    e = -np.log2(rest)
    assert np.array_equal(e, np.rint(e)) and e.min() >= 0 and e.max() <= 15
    # nearest power of two in the log domain: within sqrt(2) unless clipped at 2^-15
    A_rest = aux["A"][..., [t for t in range(L.T) if t not in (2, 3)]]
    inside = A_rest >= 2.0 ** -15.5
    r = rest[inside] / A_rest[inside]
    assert r.max() <= 2 ** 0.5 * (1 + 1e-6) and r.min() >= 2 ** -0.5 * (1 - 1e-6)
    assert np.all(rest[~inside] == 2.0 ** -15)
    # at 8 bits the grid reaches 2^-255, so nothing is clipped and the relative error bound holds everywhere
    _, aux8 = O.taq_block(L, bits_prob=8, prob_grid="log2", return_aux=True)
    r8 = aux8["A_hat"] / aux8["A"]
    assert r8.max() <= 2 ** 0.5 * (1 + 1e-6) and r8.min() >= 2 ** -0.5 * (1 - 1e-6)
    with pytest.raises(ValueError):
        O.taq_block(L, prob_grid="sqrt")


# ---------------------------------------------------------------- per-row dynamic probability scale

def test_rowmax_grid_is_exact_on_uniform_attention_of_any_length():
    """Uniform attention A = 1/T with nothing protected: every entry equals the row maximum, takes the last code,
    and code * scale reproduces float32(1/T), so the block matches unquantized probabilities to float32 rounding
    (the fixed 1/255 grid is off by percents here)."""
    B, N, H, d, T = 1, 4, 2, 4, 77
    C = H * d
    rng = np.random.Generator(np.random.PCG64(13))
    mask = np.zeros((B, T), dtype=bool)
    v_code = rng.integers(-127, 128, size=(B, T, C)).astype(np.int32)
    s_V = rng.uniform(0.01, 0.02, size=(B, H, T)).astype(np.float32)
    kv = O.QuantKV(B=B, T=T, C=C, H=H, bits_kv=8, mask=mask, k_code=np.zeros((B, T, C), dtype=np.int32), v_code=v_code,
                   s_K=np.ones((B, H, T), dtype=np.float32), s_V=s_V, K16=np.zeros((B, T, C)), V16=np.zeros((B, T, C)))
    hidden = rng.standard_normal((B, N, C)).astype(np.float16)
    wq, swq = O.quantize_weight(np.eye(C, dtype=np.float16))
    _, aux_fp = O.cross_attn(hidden, kv, wq, swq, wq, swq, bits_prob=16, return_aux=True)
    for bits in (4, 8):
        _, aux = O.cross_attn(hidden, kv, wq, swq, wq, swq, bits_prob=bits, prob_grid="rowmax", return_aux=True)
        assert np.all(aux["p_code"] == (1 << bits) - 1)
        assert np.max(np.abs(aux["O"] - aux_fp["O"])) <= 2e-7 * np.abs(aux_fp["O"]).max()
    _, aux_lin = O.cross_attn(hidden, kv, wq, swq, wq, swq, bits_prob=8, return_aux=True)
    assert np.max(np.abs(aux_lin["O"] - aux_fp["O"])) > 1e-3 * np.abs(aux_fp["O"]).max()


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("case", [
    dict(seed=41, B=1, N=4, C=8, H=2, T=5, Cc=6, bits_kv=4, trig=(1,)),
    dict(seed=42, B=2, N=3, C=4, H=1, T=9, Cc=5, bits_kv=8, trig=()),
])
def test_rowmax_grid_block_matches_scalar_brute_force(case, bits):
    L = synth.make_layer("t", seed=case["seed"], B=case["B"], N=case["N"], C=case["C"], H=case["H"], T=case["T"],
                         Cc=case["Cc"], bits_kv=case["bits_kv"], trigger_positions=case["trig"], trigger_scale=3.0, bias=True)
    out, aux = O.taq_block(L, bits_prob=bits, prob_grid="rowmax", return_aux=True)
    ref, dump = brute.taq_block_brute(L.context, L.mask, L.Wq, L.Wk, L.Wv, L.Wo, L.bias_o, L.hidden, L.H, L.bits_kv,
                                      bits_prob=bits, prob_grid="rowmax")
    assert len(dump["p_code"]) == L.B * L.N * L.H * (L.T - len(case["trig"]))
    for (b, n, h, t), v in dump["p_code"].items():
        assert aux["p_code"][b, n, h, t] == v
    for (b, n, c), v in dump["o_code"].items():
        assert aux["o_code"][b, n, c] == v
    ref = np.array(ref)
    assert np.max(np.abs(out.astype(np.float64) - ref)) <= 1e-3 * max(1.0, np.abs(ref).max())


def test_rowmax_grid_keeps_trigger_columns_and_is_finer_than_the_fixed_grid():
    L = small_layer(N=64)
    ref = O.taq_block(L, bits_prob=16, store_f16=False)
    _, aux = O.taq_block(L, bits_prob=4, prob_grid="rowmax", return_aux=True)
    assert np.array_equal(aux["A_hat"][..., [2, 3]], aux["A"][..., [2, 3]])       # Eq. (3): M_A columns keep A
    rest = [t for t in range(L.T) if t not in (2, 3)]
    # the range comes from the quantized columns only, and the largest of them takes the last code
    assert np.all(aux["p_code"][..., rest].max(axis=-1) == 15)
    assert np.array_equal(aux["s_P"], (aux["A"][..., rest].astype(np.float32).max(axis=-1) / np.float32(15)).astype(np.float32))
    assert np.all(np.abs(aux["A_hat"][..., rest] - aux["A"][..., rest]) <= aux["s_P"][..., None] * (0.5 + 1e-5))
    e = {}
    for grid in ("linear", "rowmax"):
        out = O.taq_block(L, bits_prob=4, prob_grid=grid, store_f16=False)
        e[grid] = np.linalg.norm(out - ref) / np.linalg.norm(ref)
    assert e["rowmax"] < e["linear"]
