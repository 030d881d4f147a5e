"""Per-token quantization sensitivity of the TAQ cross-attention block on the HIP path.

The experiment of Section III-B, Eq. (1), restricted to what this library computes: for each text
token i, only the K and V rows of token i are quantized to b bits (every other row is protected,
i.e. kept in fp16, through the trigger mask of Eq. (2)); the block output y^(i,b) is compared with
the output y* obtained with every row protected,

    Delta_i(b) = MSE(y^(i,b), y*),      b in {8, 4}.

Everything on the path (taq_quantize_kv, taq_cross_attn) runs in the HIP kernels; this module only
builds the masks, loops over tokens and reduces the squared difference (torch, on the GPU). Q~, the
probabilities outside the protected columns and the projections keep the widths given in `shape`
for both y^(i,b) and y*, so Delta isolates the effect of token i's rows.
"""
from __future__ import annotations

from typing import Dict, Iterable, Optional, Sequence

import torch

from . import taq as T


def _shape_with_bits(shape: "T.taq_shape", bits_kv: int) -> "T.taq_shape":
    s = T.taq_shape.from_buffer_copy(shape)
    s.bits_kv = bits_kv
    return s


def token_sensitivity(hidden: torch.Tensor, context: torch.Tensor, Wk: torch.Tensor, Wv: torch.Tensor,
                      wq_code: torch.Tensor, wo_code: torch.Tensor, scales: torch.Tensor, shape: "T.taq_shape",
                      bits: Sequence[int] = (8, 4), tokens: Optional[Iterable[int]] = None) -> Dict[int, torch.Tensor]:
    """Delta_i(b) for the given text tokens (default: all T) and bit widths.

    hidden f16 [B,N,C], context f16 [B,T,Cc], Wk/Wv f16 [C,Cc], wq_code/wo_code/scales as for
    taq_cross_attn (layout per shape.w_layout), all on the GPU. Returns {b: float64 tensor [len(tokens)]}
    on the CPU. Tokens are quantized one at a time, in every batch element alike."""
    B, Tn = shape.B, shape.T
    tokens = list(range(Tn)) if tokens is None else [int(t) for t in tokens]
    dev = hidden.device
    ws = torch.empty(T.taq_workspace_bytes(shape), dtype=torch.uint8, device=dev)
    all_on = torch.ones((B, Tn), dtype=torch.uint8, device=dev)
    s_ref = _shape_with_bits(shape, 8)
    packed = T.taq_quantize_kv(context, all_on, Wk, Wv, 8, s_ref, workspace=ws)
    y_star = T.taq_cross_attn(hidden, packed, wq_code, wo_code, scales, all_on, s_ref, workspace=ws).float()
    out: Dict[int, torch.Tensor] = {}
    y = torch.empty_like(hidden)
    for b in bits:
        if b not in (4, 8):
            raise ValueError("bits must be 4 or 8")
        s_b = _shape_with_bits(shape, b)
        packed_b = torch.empty(T.taq_kv_packed_bytes(s_b), dtype=torch.uint8, device=dev)
        delta = torch.zeros(len(tokens), dtype=torch.float64, device=dev)
        for k, i in enumerate(tokens):
            if not 0 <= i < Tn:
                raise ValueError("token index out of range")
            mask = all_on.clone()
            mask[:, i] = 0
            T.taq_quantize_kv(context, mask, Wk, Wv, b, s_b, packed_b, ws)
            T.taq_cross_attn(hidden, packed_b, wq_code, wo_code, scales, mask, s_b, y, ws)
            delta[k] = ((y.float() - y_star).double() ** 2).mean()
        out[b] = delta.cpu()
    return out
