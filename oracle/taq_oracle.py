"""CPU oracle for Trigger-Aware Quantization (TAQ) of a cross-attention block.

TEST INFRASTRUCTURE ONLY. This is a plain, slow, float64 numpy statement of what
the TAQ cross-attention block computes. It exists so that the HIP library can
be checked against something written independently from the paper. It shares
no code with the HIP path and must never be imported by the product package:
only tests, the smoke check and the benchmark's CPU-baseline leg use it.

What it follows (PersonalQ, Section III-B "Trigger-Aware Quantization"):

* the attention definition A = softmax(Q K^T / sqrt(d)), one K/V row per text
  token, in each head;
* the masks M_KV (1 on trigger-token rows of K and V) and M_A (1 on the same
  token indices, as columns of A);
* Eq. (2): K~ = M_KV*K + (1-M_KV)*Q_a(K), same for V, and Q~ = Q_a(Q) with no mask;
* Eq. (3): A^ = M_A*A + (1-M_A)*Q_a(A);
* the block output A^ V~ followed by the output projection.

The paper gives the structure only. Every numeric detail below that it leaves
open (quantizer formula, scale granularity, which projections are W8A8) is a
reading chosen for this build; each is marked "reading:" where it is taken.

Precision: every contraction is float64. The quantizers are *defined* as short
sequences of IEEE float32 operations (so that a GPU can reproduce their integer
codes bit for bit); those sequences are carried out here with numpy float32
arrays. Storage points that the method defines as fp16 (protected K/V rows, the
block output) are rounded to fp16 unless ``store_f16=False``.

Parity status: every function here is pinned by tests/test_oracle_*.py (exact
rational quantizer, textbook attention when nothing is quantized, closed forms,
pass-through of trigger rows/columns, a separately written scalar brute force).
Image-quality numbers of the paper (FID/CLIP) are parity unpinned: they need the
paper's checkpoints and caption sets.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np

f32 = np.float32
f64 = np.float64


# --------------------------------------------------------------------------
# Quantizers  (reading: the "standard affine quantizer" Q_b of Section III-B,
# taken in its symmetric, zero-point-0 form with round-half-to-even)
# --------------------------------------------------------------------------

def symq(x, bits: int, axis: int = -1):
    """Symmetric b-bit quantizer over one axis ("row").

    qmax = 2^(b-1)-1;  amax = max|x| over the row;  scale = amax / qmax;
    code = clamp(rint((x * qmax) / amax), -qmax, +qmax);  dequantised = code * scale.
    All in float32: one multiply, one correctly rounded divide, rint half-to-even.
    A row of zeros gets scale 1 and codes 0.

    Multiplying by qmax before dividing by amax (instead of dividing by a
    pre-rounded scale) makes the code the exactly rounded value of x*qmax/amax
    whenever x*qmax is exact in float32, which holds for fp16-valued inputs.

    Returns (codes int32 with x's shape, scales float32 with ``axis`` removed).
    """
    if bits not in (4, 8):
        raise ValueError("symq: bits must be 4 or 8")
    x = np.asarray(x, dtype=f32)
    qmax = (1 << (bits - 1)) - 1
    qmaxf = f32(qmax)
    amax = np.max(np.abs(x), axis=axis, keepdims=True).astype(f32)
    zero = amax == f32(0)
    scale = (amax / qmaxf).astype(f32)
    scale = np.where(zero, f32(1), scale).astype(f32)
    safe = np.where(zero, f32(1), amax).astype(f32)
    q = ((x * qmaxf).astype(f32) / safe).astype(f32)
    code = np.clip(np.rint(q), -qmax, qmax).astype(np.int32)
    return code, np.squeeze(scale, axis=axis)


def uq(p, bits: int = 8):
    """Unsigned b-bit quantizer of a probability in [0,1] (reading: the affine
    quantizer with the a-priori range of a softmax output, zero-point 0, fixed
    scale 1/(2^b - 1)):  code = rint(p * (2^b - 1)) in float32, half-to-even.
    b = 8 gives the 1/255 grid, b = 4 (the paper's 4-bit activation setting) 1/15."""
    if bits not in (4, 8):
        raise ValueError("uq: bits must be 4 or 8")
    pmax = f32((1 << bits) - 1)
    p32 = np.asarray(p, dtype=f32)
    code = np.rint((p32 * pmax).astype(f32))
    return np.clip(code, 0, int(pmax)).astype(np.int32)


def uq8(p):
    """8-bit case of ``uq``."""
    return uq(p, 8)


def uq_log2(p, bits: int = 8):
    """Logarithmic b-bit quantizer of a probability (the "Logarithmic" rows of the
    TAQ ablation table in Section IV). The paper names this quantizer without a
    formula; reading: the power-of-two grid customary for post-softmax activations,
        code = clip(rint(-log2 p), 0, 2^b - 1),   p^ = 2^(-code),
    with -log2 p evaluated in float64, rounded once to float32, then rint
    half-to-even. p = 0 takes the last code (its p^ = 2^-(2^b-1) is not zero)."""
    if bits not in (4, 8):
        raise ValueError("uq_log2: bits must be 4 or 8")
    last = (1 << bits) - 1
    p64 = np.asarray(p, dtype=f64)
    with np.errstate(divide="ignore"):
        x = (-np.log2(p64)).astype(f32)          # +inf where p == 0
    code = np.rint(np.minimum(x, f32(last)))
    return np.clip(code, 0, last).astype(np.int32)


def uq_rowmax(p, bits: int = 8, quantized=None):
    """Unsigned b-bit quantizer of a row of probabilities with the row's own range (reading of the
    "standard affine quantizer" of Section III-B with a dynamic per-row scale instead of the a-priori
    range [0, 1]): over the entries of the last axis that are quantized at all (``quantized`` mask;
    default: all),
        amax = max p,  scale = amax / (2^b - 1),  code = clamp(rint((p * (2^b - 1)) / amax), 0, 2^b - 1),
    in float32 with the multiply-then-divide order of ``symq``; a row whose quantized entries are all zero
    gets scale 1 and codes 0. Returns (codes int32, scale float32 [...]); p^ = code * scale."""
    if bits not in (4, 8):
        raise ValueError("uq_rowmax: bits must be 4 or 8")
    pmax = f32((1 << bits) - 1)
    p32 = np.asarray(p, dtype=f32)
    q = np.ones(p32.shape, dtype=bool) if quantized is None else np.broadcast_to(np.asarray(quantized, dtype=bool), p32.shape)
    amax = np.where(q, p32, f32(0)).max(axis=-1).astype(f32)
    zero = amax == 0
    safe = np.where(zero, f32(1), amax).astype(f32)
    scale = np.where(zero, f32(1), (amax / pmax).astype(f32)).astype(f32)
    t = (np.where(q, p32, f32(0)) * pmax).astype(f32)      # entries outside the mask get no code
    code = np.rint((t / safe[..., None]).astype(f32))
    code = np.where(q, np.clip(code, 0, int(pmax)), 0).astype(np.int32)
    return code, scale


def pack_int4(codes):
    """Two's-complement nibbles, element 2j in the low nibble of byte j."""
    c = np.asarray(codes).astype(np.int32)
    if c.shape[-1] % 2:
        raise ValueError("pack_int4: last axis must be even")
    lo = c[..., 0::2] & 0xF
    hi = c[..., 1::2] & 0xF
    return (lo | (hi << 4)).astype(np.uint8)


def quantize_weight(W):
    """Per-output-channel symmetric int8 codes of a weight matrix [out, in]
    (reading: round-to-nearest 8-bit weights; the paper uses 8-bit weights in
    every setting of Table 1 but calibrates them with data this build lacks)."""
    code, scale = symq(np.asarray(W, dtype=np.float16).astype(f32), 8, axis=1)
    return code.astype(np.int8), scale


# --------------------------------------------------------------------------
# K/V side: Eq. (2), first two lines
# --------------------------------------------------------------------------

@dataclass
class QuantKV:
    """K~ and V~ in the mixed-precision form the block consumes."""

    B: int
    T: int
    C: int
    H: int
    bits_kv: int
    mask: np.ndarray  # bool [B, T]  effective protection mask (all True when bits_kv == 16)
    k_code: np.ndarray  # int32 [B, T, C]  zeros on protected rows
    v_code: np.ndarray
    s_K: np.ndarray  # f32 [B, H, T]   zeros on protected rows
    s_V: np.ndarray
    K16: np.ndarray  # f64 [B, T, C]  protected rows (fp16-valued if stored as fp16), zeros elsewhere
    V16: np.ndarray
    aux: Dict[str, np.ndarray] = field(default_factory=dict)

    def dequant(self, which: str) -> np.ndarray:
        """The matrix K~ (or V~) of Eq. (2) as float64 [B, T, C]."""
        code = self.k_code if which == "k" else self.v_code
        s = self.s_K if which == "k" else self.s_V
        full = self.K16 if which == "k" else self.V16
        d = self.C // self.H
        sc = np.repeat(np.transpose(s, (0, 2, 1)).astype(f64), d, axis=2)  # [B,T,C]
        M = self.mask[:, :, None]
        return np.where(M, full, code.astype(f64) * sc)


def _int_matmul(x_code, w_code):
    """Exact integer contraction sum_k x[..., k] * w[c, k] -> int64 [..., c].

    Done as a float64 matrix product: every product is below 2^14 and every
    partial sum below K * 2^14 << 2^53, so each intermediate is an integer that
    float64 represents exactly, whatever the summation order."""
    x = np.asarray(x_code)
    w = np.asarray(w_code)
    assert x.shape[-1] * 127 * 127 < 2 ** 52
    acc = np.matmul(x.astype(f64), w.astype(f64).T)
    return np.rint(acc).astype(np.int64)


def _project_rows(x16, W16, bits_proj, mask, store_f16):
    """One projection of the text context (K or V side).

    Returns (rows for unprotected tokens as float32 [B,T,C],
             rows for protected tokens as float64 [B,T,C], aux dict)."""
    x = np.asarray(x16, dtype=np.float16)
    W = np.asarray(W16, dtype=np.float16)
    aux = {}
    if bits_proj == 8:
        # reading: the projection itself is W8A8 for unprotected tokens
        w_code, s_w = symq(W.astype(f32), 8, axis=1)  # per output channel
        x_code, s_x = symq(x.astype(f32), 8, axis=-1)  # per token
        acc = _int_matmul(x_code, w_code)
        rows_q = (acc.astype(f32) * (s_x[:, :, None] * s_w[None, None, :]).astype(f32)).astype(f32)
        # reading: a protected token keeps its unquantized fp16 context row and
        # fp accumulation, but meets the same 8-bit weight codes
        full = np.einsum("btk,ck->btc", x.astype(f64), w_code.astype(f64)) * s_w.astype(f64)[None, None, :]
        aux.update(w_code=w_code, s_w=s_w, x_code=x_code, s_x=s_x, acc=acc)
    elif bits_proj == 16:
        full = np.einsum("btk,ck->btc", x.astype(f64), W.astype(f64))
        rows_q = full.astype(f32)
    else:
        raise ValueError("bits_proj must be 8 or 16")
    if store_f16:
        full = full.astype(np.float16).astype(f64)
    full = np.where(mask[:, :, None], full, 0.0)
    return rows_q, full, aux


def quantize_kv(context, trigger_mask, Wk, Wv, bits_kv: int, H: int,
                bits_proj: int = 8, store_f16: bool = True) -> QuantKV:
    """Eq. (2), K and V lines: protected rows stay in full precision, every
    other row is quantized per (head, token) over the head's d channels
    (reading: "one row per text token, in each head" fixes the row)."""
    context = np.asarray(context)
    B, T, _ = context.shape
    C = Wk.shape[0]
    if C % H:
        raise ValueError("C must be a multiple of H")
    if bits_kv not in (4, 8, 16):
        raise ValueError("bits_kv must be 4, 8 or 16")
    d = C // H
    mask = np.asarray(trigger_mask).astype(bool).reshape(B, T)
    if bits_kv == 16:
        mask = np.ones_like(mask)
    out = {}
    aux_all = {}
    for name, W in (("k", Wk), ("v", Wv)):
        rows_q, full, aux = _project_rows(context, W, bits_proj, mask, store_f16)
        if bits_kv == 16:
            code = np.zeros((B, T, C), dtype=np.int32)
            s = np.zeros((B, H, T), dtype=f32)
        else:
            code4, s4 = symq(rows_q.reshape(B, T, H, d), bits_kv, axis=-1)  # [B,T,H,d], [B,T,H]
            code = code4.reshape(B, T, C)
            s = np.transpose(s4, (0, 2, 1)).copy()  # [B,H,T]
            code = np.where(mask[:, :, None], 0, code)
            s = np.where(mask[:, None, :], f32(0), s).astype(f32)
        out[name] = (code, s, full)
        aux_all.update({f"{name}_{k}": v for k, v in aux.items()})
        aux_all[f"{name}_rows_q"] = rows_q
    return QuantKV(B=B, T=T, C=C, H=H, bits_kv=bits_kv, mask=mask,
                   k_code=out["k"][0], v_code=out["v"][0], s_K=out["k"][1], s_V=out["v"][1],
                   K16=out["k"][2], V16=out["v"][2], aux=aux_all)


# --------------------------------------------------------------------------
# Query side and the attention block: Eq. (2) third line, Eq. (3)
# --------------------------------------------------------------------------

def _linear_w8a8(x, w_code, s_w):
    """Per-token int8 activation codes, exact integer contraction with the
    weight codes, float32 dequantisation: acc * (s_x * s_w)."""
    x_code, s_x = symq(np.asarray(x, dtype=f32), 8, axis=-1)
    acc = _int_matmul(x_code, w_code)
    y = (acc.astype(f32) * (s_x[:, :, None] * np.asarray(s_w, dtype=f32)[None, None, :]).astype(f32)).astype(f32)
    return y, x_code, s_x, acc


def cross_attn(hidden, kv: QuantKV, wq_code, s_wq, wo_code, s_wo, bias_o=None,
               bits_prob: int = 8, bits_q: int = 8, bits_proj: int = 8,
               softmax_scale: Optional[float] = None, store_f16: bool = True,
               Wq_f16=None, Wo_f16=None, return_aux: bool = False, prob_grid: str = "linear"):
    """The TAQ cross-attention block for image tokens ``hidden`` [B, N, C].

    Steps, in the paper's order:
      Q  = to_q(hidden)                       (W8A8: reading)
      Q~ = Q_a(Q)                             Eq. (2), third line; per (token, head): reading; 8 or 4 bits
      A  = softmax(Q~ K~^T / sqrt(d))         attention definition, per head
      A^ = M_A*A + (1-M_A)*Q_a(A)             Eq. (3); no renormalisation; 8 or 4 bits;
                                              Q_a on the fixed linear grid (uq), on powers of two (prob_grid="log2",
                                              uq_log2) or on the row's own range (prob_grid="rowmax", uq_rowmax)
      O  = A^ V~
      out = to_out(O) + bias                  (W8A8: reading), stored as fp16
    With bits_proj == 16 the two projections use ``Wq_f16`` / ``Wo_f16`` unquantized.
    """
    hidden = np.asarray(hidden, dtype=np.float16)
    B, N, C = hidden.shape
    H, T = kv.H, kv.T
    d = C // H
    sigma = (1.0 / np.sqrt(f64(d))) if not softmax_scale else f64(softmax_scale)
    aux = {}

    # ---- to_q
    if bits_proj == 8:
        Qf, h_code, s_h, acc_q = _linear_w8a8(hidden.astype(f32), wq_code, s_wq)
        aux.update(h_code=h_code, s_h=s_h, acc_q=acc_q)
    else:
        Qf = np.einsum("bnk,ck->bnc", hidden.astype(f64), np.asarray(Wq_f16).astype(f64))
    aux["Qf"] = Qf

    # ---- Q~ = Q_a(Q)
    if bits_q in (4, 8):
        q_code, s_Q = symq(np.asarray(Qf, dtype=f32).reshape(B, N, H, d), bits_q, axis=-1)
        Qt = q_code.astype(f64) * s_Q.astype(f64)[..., None]  # [B,N,H,d]
        aux.update(q_code=q_code.reshape(B, N, C), s_Q=s_Q)
    elif bits_q == 16:
        Qt = np.asarray(Qf, dtype=f64).reshape(B, N, H, d)
    else:
        raise ValueError("bits_q must be 4, 8 or 16")

    # ---- K~, V~ as matrices (Eq. 2), split by head
    Kt = kv.dequant("k").reshape(B, T, H, d)
    Vt = kv.dequant("v").reshape(B, T, H, d)

    # ---- A = softmax(Q~ K~^T / sqrt(d)) over the T text tokens (all attended)
    S = sigma * np.einsum("bnhj,bthj->bnht", Qt, Kt)
    S = S - S.max(axis=-1, keepdims=True)
    E = np.exp(S)
    A = E / E.sum(axis=-1, keepdims=True)  # [B,N,H,T]
    aux["A"] = A

    # ---- A^ (Eq. 3): trigger columns keep A, the others are quantized
    M_A = kv.mask[:, None, None, :]  # [B,1,1,T] -> broadcast over N and heads
    if prob_grid not in ("linear", "log2", "rowmax"):
        raise ValueError("prob_grid must be 'linear', 'log2' or 'rowmax'")
    if bits_prob in (4, 8) and prob_grid == "rowmax":
        p_code, s_P = uq_rowmax(A, bits_prob, quantized=~M_A)
        A_q = p_code.astype(f64) * s_P.astype(f64)[..., None]
        aux.update(p_code=p_code, s_P=s_P)
    elif bits_prob in (4, 8) and prob_grid == "log2":
        p_code = uq_log2(A, bits_prob)
        A_q = np.exp2(-p_code.astype(f64))
        aux["p_code"] = p_code
    elif bits_prob in (4, 8):
        p_code = uq(A, bits_prob)
        A_q = p_code.astype(f64) / f64((1 << bits_prob) - 1)
        aux["p_code"] = p_code
    elif bits_prob == 16:
        A_q = A
    else:
        raise ValueError("bits_prob must be 4, 8 or 16")
    A_hat = np.where(M_A, A, A_q)
    aux["A_hat"] = A_hat

    # ---- O = A^ V~
    O = np.einsum("bnht,bthj->bnhj", A_hat, Vt).reshape(B, N, C)
    aux["O"] = O

    # ---- to_out
    if bias_o is None:
        bias_o = np.zeros(C, dtype=f32)
    if bits_proj == 8:
        Yq, o_code, s_o, acc_o = _linear_w8a8(O.astype(f32), wo_code, s_wo)
        Y = (Yq + np.asarray(bias_o, dtype=f32)[None, None, :]).astype(f32)
        aux.update(o_code=o_code, s_o=s_o, acc_o=acc_o)
    else:
        Y = np.einsum("bnk,ck->bnc", O, np.asarray(Wo_f16).astype(f64)) + np.asarray(bias_o, dtype=f64)
    out = Y.astype(np.float16) if store_f16 else np.asarray(Y, dtype=f64)
    if return_aux:
        return out, aux
    return out


def taq_block(layer, bits_prob: int = 8, bits_q: int = 8, bits_proj: int = 8,
              bits_kv: Optional[int] = None, store_f16: bool = True, return_aux: bool = False,
              prob_grid: str = "linear"):
    """Whole path for one synthetic layer: weight codes, K~/V~, then the block."""
    bk = layer.bits_kv if bits_kv is None else bits_kv
    kv = quantize_kv(layer.context, layer.mask, layer.Wk, layer.Wv, bk, layer.H,
                     bits_proj=bits_proj, store_f16=store_f16)
    wq_code, s_wq = quantize_weight(layer.Wq)
    wo_code, s_wo = quantize_weight(layer.Wo)
    res = cross_attn(layer.hidden, kv, wq_code, s_wq, wo_code, s_wo, layer.bias_o,
                     bits_prob=bits_prob, bits_q=bits_q, bits_proj=bits_proj,
                     store_f16=store_f16, Wq_f16=layer.Wq, Wo_f16=layer.Wo, return_aux=return_aux,
                     prob_grid=prob_grid)
    if return_aux:
        out, aux = res
        aux["kv"] = kv
        aux.update(wq_code=wq_code, s_wq=s_wq, wo_code=wo_code, s_wo=s_wo)
        return out, aux
    return res


# --------------------------------------------------------------------------
# Bit-operations of the block (Section III-C: BOPs = FLOPs * b_w * b_a)
# --------------------------------------------------------------------------

def block_bops(B, N, C, T, Cc, b_w: int, b_a: int) -> float:
    """BOPs of the block's five contractions at weight/activation widths b_w/b_a.
    FLOPs counted as 2 per multiply-accumulate."""
    flops = 2.0 * B * (N * C * C  # to_q
                       + 2 * T * Cc * C  # to_k, to_v
                       + 2 * N * T * C  # Q K^T and A V over all heads
                       + N * C * C)  # to_out
    return flops * b_w * b_a
