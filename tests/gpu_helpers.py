"""Shared plumbing of the GPU parity tests: move a synthetic layer to the GPU,
run the HIP path through the C ABI, run the oracle on the same inputs."""
from __future__ import annotations

import numpy as np
import torch

from oracle import taq_oracle as O
from paper_2603_22943_amd import taq as T

DEV = "cuda:0"


def shape_of(L, bits_kv=None, N=None, w_layout=0, bits_q=8, bits_prob=8, prob_grid="linear", tok_tile=0):
    return T.make_shape(B=L.B, N=L.N if N is None else N, C=L.C, H=L.H, T=L.T, Cc=L.Cc,
                        bits_kv=L.bits_kv if bits_kv is None else bits_kv, bits_q=bits_q, bits_prob=bits_prob,
                        w_layout=w_layout, tok_tile=tok_tile, prob_grid={"linear": T.TAQ_PROB_LINEAR, "log2": T.TAQ_PROB_LOG2,
                                                       "rowmax": T.TAQ_PROB_ROWMAX}[prob_grid])


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.to(DEV)


class GpuRun:
    """Everything the HIP path produces for one layer (tensors brought back as numpy)."""

    def __init__(self, L, taps=True, hidden=None, w_layout=0, bits_q=8, bits_prob=8, prob_grid="linear", tok_tile=0):
        self.L = L
        self.shape = s = shape_of(L, w_layout=w_layout, bits_q=bits_q, bits_prob=bits_prob, prob_grid=prob_grid, tok_tile=tok_tile)
        ctx, mask = dev(L.context), dev(L.mask)
        Wq, Wk, Wv, Wo = dev(L.Wq), dev(L.Wk), dev(L.Wv), dev(L.Wo)
        self.wq_code, self.s_wq = T.taq_quantize_weight(Wq)
        self.wo_code, self.s_wo = T.taq_quantize_weight(Wo)
        self.wq_plain, self.wo_plain = self.wq_code, self.wo_code
        if w_layout == 1:  # row-major codes followed by the operand-ordered copy
            self.wq_code = T.taq_pack_weight(self.wq_plain, s)
            self.wo_code = T.taq_pack_weight(self.wo_plain, s)
        self.scales = torch.cat([self.s_wq, self.s_wo, dev(L.bias_o)]).contiguous()
        # qkv_packed and the workspace start as 0xFF bytes (NaN as fp16 / float32, -1 as int8): a kernel that reads a
        # byte nobody wrote (alignment gaps, rows past the end of a section) shows up as NaN instead of passing by luck
        self.packed = torch.full((T.taq_kv_packed_bytes(s),), 0xFF, dtype=torch.uint8, device=DEV)
        self.ws = torch.full((T.taq_workspace_bytes(s),), 0xFF, dtype=torch.uint8, device=DEV)
        T.taq_quantize_kv(ctx, mask, Wk, Wv, L.bits_kv, s, self.packed, self.ws)
        self.kv = {k: v.cpu().numpy() for k, v in T.taq_unpack_kv(self.packed, s).items()}
        self.mask_d = mask
        self.hidden_d = dev(L.hidden if hidden is None else hidden)
        if hidden is not None:
            self.shape = s = shape_of(L, N=hidden.shape[1], w_layout=w_layout, bits_q=bits_q, bits_prob=bits_prob,
                                      prob_grid=prob_grid, tok_tile=tok_tile)
        if taps:
            dbg, t = T.make_debug(s, DEV)
            self.ws.fill_(0xFF)
            self.out_d = T.taq_cross_attn(self.hidden_d, self.packed, self.wq_code, self.wo_code, self.scales,
                                          mask, s, workspace=self.ws, debug=dbg)
            torch.cuda.synchronize()
            self.taps = {k: v.cpu().numpy() for k, v in t.items()}
        else:
            self.ws.fill_(0xFF)
            self.out_d = T.taq_cross_attn(self.hidden_d, self.packed, self.wq_code, self.wo_code, self.scales,
                                          mask, s, workspace=self.ws)
            torch.cuda.synchronize()
            self.taps = {}
        self.out = self.out_d.cpu().numpy()


def oracle_run(L, hidden=None, bits_q=8, bits_prob=8, prob_grid="linear"):
    kv = O.quantize_kv(L.context, L.mask, L.Wk, L.Wv, L.bits_kv, L.H)
    wq_code, s_wq = O.quantize_weight(L.Wq)
    wo_code, s_wo = O.quantize_weight(L.Wo)
    out, aux = O.cross_attn(L.hidden if hidden is None else hidden, kv, wq_code, s_wq, wo_code, s_wo, L.bias_o,
                            bits_q=bits_q, bits_prob=bits_prob, prob_grid=prob_grid, return_aux=True)
    aux.update(kv=kv, wq_code=wq_code, s_wq=s_wq, wo_code=wo_code, s_wo=s_wo)
    return out, aux


def fp16_ulp_distance(a, b):
    """Distance in units of fp16 steps between two fp16-valued arrays (same sign assumed near 0)."""
    ia = np.asarray(a, dtype=np.float16).view(np.int16).astype(np.int32)
    ib = np.asarray(b, dtype=np.float16).view(np.int16).astype(np.int32)
    ia = np.where(ia < 0, -(ia & 0x7FFF), ia)
    ib = np.where(ib < 0, -(ib & 0x7FFF), ib)
    return np.abs(ia - ib)


def out_errors(out, ref):
    o = np.asarray(out, dtype=np.float64)
    r = np.asarray(ref, dtype=np.float64)
    max_abs = float(np.max(np.abs(o - r))) if o.size else 0.0
    rel_l2 = float(np.linalg.norm(o - r) / max(np.linalg.norm(r), 1e-30))
    return max_abs, rel_l2
