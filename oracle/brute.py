"""Scalar brute force of the TAQ cross-attention block, for tiny inputs only.

TEST INFRASTRUCTURE ONLY. Written separately from the vectorised oracle (no
shared helpers, no numpy array arithmetic: one Python scalar at a time), so that
an indexing, transposition or masking mistake in either shows up as a
disagreement. It follows PersonalQ Section III-B: the attention definition,
Eq. (2) (K~, V~, Q~) and Eq. (3) (A^), with the same readings of the open
details as the vectorised oracle (symmetric round-half-even quantizer, per
(head, token) K/V rows, per (token, head) Q rows, per-token activations,
per-output-channel 8-bit weights, probabilities on a fixed 1/255 or 1/15 grid, or on
powers of two for the logarithmic quantizer).

Float32 steps of the quantizer definition are done with numpy float32 *scalars*;
everything else is Python float (float64) or exact Fractions.
"""
from __future__ import annotations

import math
from fractions import Fraction

import numpy as np

_f32 = np.float32


def round_half_even(fr: Fraction) -> int:
    """Exact round-half-to-even of a rational."""
    fl = math.floor(fr)
    rem = fr - fl
    if rem > Fraction(1, 2):
        return fl + 1
    if rem < Fraction(1, 2):
        return fl
    return fl if fl % 2 == 0 else fl + 1


def symq_exact(row, bits):
    """Exact-rational symmetric quantizer of a list of floats: the code is the
    half-even rounding of the exact quotient x*qmax/amax. Returns (codes, amax)."""
    qmax = (1 << (bits - 1)) - 1
    fr = [Fraction(float(v)) for v in row]
    amax = max(abs(v) for v in fr) if fr else Fraction(0)
    if amax == 0:
        return [0] * len(fr), Fraction(0)
    codes = [max(-qmax, min(qmax, round_half_even(v * qmax / amax))) for v in fr]
    return codes, amax


def symq_f32(row, bits):
    """The float32 op sequence, scalar by scalar: t = x*qmax; q = t/amax; rint."""
    qmax = (1 << (bits - 1)) - 1
    xs = [_f32(v) for v in row]
    amax = _f32(0)
    for v in xs:
        a = _f32(abs(v))
        if a > amax:
            amax = a
    if amax == _f32(0):
        return [0] * len(xs), _f32(1)
    scale = _f32(amax / _f32(qmax))
    codes = []
    for v in xs:
        t = _f32(v * _f32(qmax))
        q = _f32(t / amax)
        r = int(np.rint(q))
        codes.append(max(-qmax, min(qmax, r)))
    return codes, scale


def taq_block_brute(context, mask, Wq, Wk, Wv, Wo, bias_o, hidden, H, bits_kv, bits_q=8, bits_prob=8,
                    prob_grid="linear"):
    """context [B][T][Cc], mask [B][T], W* [C][in], hidden [B][N][C] as nested
    lists / arrays of fp16-valued numbers. Returns out [B][N][C] (Python floats,
    rounded through fp16) and a dict of intermediates."""
    B = len(context)
    T = len(context[0])
    Cc = len(context[0][0])
    N = len(hidden[0])
    C = len(Wq)
    d = C // H
    sigma = 1.0 / math.sqrt(d)

    def wquant(W):
        codes, scales = [], []
        for c in range(len(W)):
            cr, sc = symq_f32([float(v) for v in W[c]], 8)
            codes.append(cr)
            scales.append(sc)
        return codes, scales

    wq_c, wq_s = wquant(Wq)
    wk_c, wk_s = wquant(Wk)
    wv_c, wv_s = wquant(Wv)
    wo_c, wo_s = wquant(Wo)

    out = [[[0.0] * C for _ in range(N)] for _ in range(B)]
    dump = {"k_code": {}, "v_code": {}, "q_code": {}, "p_code": {}, "o_code": {}, "K16": {}, "V16": {}}
    for b in range(B):
        trig = [bool(mask[b][t]) or bits_kv == 16 for t in range(T)]
        # ---- K~ / V~ rows, Eq. (2)
        Kt = [[0.0] * C for _ in range(T)]
        Vt = [[0.0] * C for _ in range(T)]
        for (Wc, Ws, dst, nm) in ((wk_c, wk_s, Kt, "k"), (wv_c, wv_s, Vt, "v")):
            for t in range(T):
                xrow = [float(v) for v in context[b][t]]
                if trig[t]:
                    for c in range(C):
                        s = 0.0
                        for k in range(Cc):
                            s += xrow[k] * Wc[c][k]
                        val = float(np.float16(s * float(Ws[c])))
                        dst[t][c] = val
                        dump["K16" if nm == "k" else "V16"][(b, t, c)] = val
                else:
                    xc, xs = symq_f32(xrow, 8)
                    rowf = []
                    for c in range(C):
                        acc = 0
                        for k in range(Cc):
                            acc += xc[k] * Wc[c][k]
                        rowf.append(_f32(_f32(acc) * _f32(xs * Ws[c])))
                    for h in range(H):
                        seg = rowf[h * d:(h + 1) * d]
                        cr, sc = symq_f32(seg, bits_kv)
                        for j in range(d):
                            dst[t][h * d + j] = cr[j] * float(sc)
                            dump[nm + "_code"][(b, t, h * d + j)] = cr[j]
        for n in range(N):
            # ---- to_q, W8A8
            hc, hs = symq_f32([float(v) for v in hidden[b][n]], 8)
            Qf = []
            for c in range(C):
                acc = 0
                for k in range(C):
                    acc += hc[k] * wq_c[c][k]
                Qf.append(_f32(_f32(acc) * _f32(hs * wq_s[c])))
            O = [0.0] * C
            for h in range(H):
                # ---- Q~ = Q_a(Q), Eq. (2) third line
                qc, qs = symq_f32(Qf[h * d:(h + 1) * d], bits_q)
                for j in range(d):
                    dump["q_code"][(b, n, h * d + j)] = qc[j]
                # ---- A = softmax(Q~ K~^T / sqrt(d))
                S = []
                for t in range(T):
                    s = 0.0
                    for j in range(d):
                        s += (qc[j] * float(qs)) * Kt[t][h * d + j]
                    S.append(sigma * s)
                m = max(S)
                E = [math.exp(v - m) for v in S]
                Z = sum(E)
                A = [e / Z for e in E]
                # ---- A^, Eq. (3)
                Ah = []
                row_amax = _f32(0)  # "rowmax" grid: largest float32 probability among the columns that get quantized
                for t in range(T):
                    if not trig[t] and _f32(A[t]) > row_amax:
                        row_amax = _f32(A[t])
                for t in range(T):
                    if trig[t]:
                        Ah.append(A[t])
                    elif prob_grid == "rowmax":
                        pmax = (1 << bits_prob) - 1
                        if row_amax == _f32(0):
                            pc, sc = 0, _f32(1)
                        else:
                            sc = _f32(row_amax / _f32(pmax))
                            pc = int(np.rint(_f32(_f32(_f32(A[t]) * _f32(pmax)) / row_amax)))
                            pc = min(pmax, max(0, pc))
                        dump["p_code"][(b, n, h, t)] = pc
                        Ah.append(pc * float(sc))
                    elif prob_grid == "log2":
                        # power-of-two grid: the exponent -log2 A, to float32, rounded half-even, clipped
                        last = (1 << bits_prob) - 1
                        ex = float(_f32(-math.log2(A[t]))) if A[t] > 0.0 else float(last)
                        pc = min(last, max(0, int(np.rint(_f32(min(ex, float(last)))))))
                        dump["p_code"][(b, n, h, t)] = pc
                        Ah.append(math.ldexp(1.0, -pc))
                    else:
                        pmax = (1 << bits_prob) - 1
                        pc = int(np.rint(_f32(_f32(A[t]) * _f32(pmax))))
                        dump["p_code"][(b, n, h, t)] = pc
                        Ah.append(pc / float(pmax))
                # ---- O = A^ V~
                for j in range(d):
                    s = 0.0
                    for t in range(T):
                        s += Ah[t] * Vt[t][h * d + j]
                    O[h * d + j] = s
            # ---- to_out, W8A8 + bias, fp16 store
            oc, os_ = symq_f32(O, 8)
            for c in range(C):
                dump["o_code"][(b, n, c)] = oc[c]
                acc = 0
                for k in range(C):
                    acc += oc[k] * wo_c[c][k]
                y = _f32(_f32(_f32(acc) * _f32(os_ * wo_s[c])) + _f32(bias_o[c]))
                out[b][n][c] = float(np.float16(y))
    return out, dump
