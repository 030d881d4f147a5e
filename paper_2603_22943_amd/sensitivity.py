"""Per-token quantization sensitivity of the TAQ cross-attention block on the HIP path.

The experiment of Section III-B, Eq. (1), restricted to what this library computes: for each text
token i, only the K and V rows of token i are quantized to b bits (every other row is protected,
i.e. kept in fp16, through the trigger mask of Eq. (2)); the block output y^(i,b) is compared with
the output y* obtained with every row protected,

    Delta_i(b) = MSE(y^(i,b), y*),      b in {8, 4}.

Everything runs in the library's kernels, the squared-difference reduction included (taq_mse_f16);
this module only builds the masks and loops over tokens. What "everything else" is computed at is
the caller's choice through `shape`: with bits_q = bits_prob = bits_proj = 16 (Wq / Wo / Wk / Wv
the fp16 matrices) all other parameters and activations stay in full precision, as Eq. (1) states;
with the 8- or 4-bit widths the sweep isolates the effect of token i's rows inside the quantized
block.
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
                      wq: torch.Tensor, wo: torch.Tensor, scales: torch.Tensor, shape: "T.taq_shape",
                      bits: Sequence[int] = (8, 4), tokens: Optional[Iterable[int]] = None) -> Dict[int, torch.Tensor]:
    """Delta_i(b) for the given text tokens (default: all T) and bit widths.

    hidden f16 [B,N,C], context f16 [B,T,Cc], Wk/Wv f16 [C,Cc], wq/wo/scales as taq_cross_attn takes them
    for `shape` (weight codes, or the fp16 matrices with shape.bits_proj = 16), all on the GPU.
    Returns {b: float64 tensor [len(tokens)]} on the CPU. Tokens are quantized one at a time, in every
    batch element alike."""
    B, Tn = shape.B, shape.T
    tokens = list(range(Tn)) if tokens is None else [int(t) for t in tokens]
    for b in bits:
        if b not in (4, 8):
            raise ValueError("bits must be 4 or 8")
    for i in tokens:
        if not 0 <= i < Tn:
            raise ValueError("token index out of range")
    dev = hidden.device
    ws = torch.empty(T.taq_workspace_bytes(shape), dtype=torch.uint8, device=dev)
    all_on = torch.ones((B, Tn), dtype=torch.uint8, device=dev)
    s_ref = _shape_with_bits(shape, 16)  # every row kept in fp16
    packed = T.taq_quantize_kv(context, all_on, Wk, Wv, 16, s_ref, workspace=ws)
    y_star = T.taq_cross_attn(hidden, packed, wq, wo, scales, all_on, s_ref, workspace=ws)
    out: Dict[int, torch.Tensor] = {}
    y = torch.empty_like(y_star)
    masks = all_on.repeat(len(tokens), 1, 1)  # one mask per swept token (plain memory set-up, no arithmetic)
    for k, i in enumerate(tokens):
        masks[k, :, i] = 0
    for b in bits:
        s_b = _shape_with_bits(shape, b)
        packed_b = torch.empty(T.taq_kv_packed_bytes(s_b), dtype=torch.uint8, device=dev)
        delta = torch.zeros(len(tokens), dtype=torch.float64, device=dev)
        for k in range(len(tokens)):
            T.taq_quantize_kv(context, masks[k], Wk, Wv, b, s_b, packed_b, ws)
            T.taq_cross_attn(hidden, packed_b, wq, wo, scales, masks[k], s_b, y, ws)
            T.taq_mse_f16(y, y_star, delta[k:k + 1])
        out[b] = delta.cpu()
    return out
