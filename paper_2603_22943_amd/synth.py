"""Seeded synthetic inputs shaped like the paper's SD v1.5 / SDXL cross-attention workloads.

This module only draws random numbers and reshapes them: it holds none of the
method's arithmetic (no quantizer, no projection, no attention), so both the
CPU oracle's tests and the HIP path's tests may take their inputs from it.

The paper evaluates on personalised Stable Diffusion checkpoints prompted with
caption sets (Section III-C); neither the checkpoints nor the captions ship with
this repository, so these inputs reproduce only the shapes and rough value
structure of those workloads:

* text context: 77 tokens x 768 (SD v1.5) or 2048 (SDXL) channels, N(0,1), with
  the trigger-token rows scaled up (a fine-tuned trigger embedding is an outlier
  among ordinary word embeddings);
* projection weights N(0, 1/fan_in);
* image hidden states N(0,1) with about 1 % outlier channels scaled x20 where the
  configuration asks for them.

Everything is drawn in float64 from numpy's PCG64 in a fixed order and cast to
fp16, which is the storage type the library takes.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np

T_TEXT = 77


@dataclass
class Layer:
    """One cross-attention layer's inputs (numpy, host memory)."""

    name: str
    B: int
    N: int
    C: int
    H: int
    T: int
    Cc: int
    bits_kv: int
    context: np.ndarray  # f16 [B, T, Cc]
    mask: np.ndarray  # u8  [B, T]   1 = trigger token
    Wq: np.ndarray  # f16 [C, C]   out x in
    Wk: np.ndarray  # f16 [C, Cc]
    Wv: np.ndarray  # f16 [C, Cc]
    Wo: np.ndarray  # f16 [C, C]
    bias_o: np.ndarray  # f32 [C]
    hidden: np.ndarray  # f16 [B, N, C]
    seed: int = 0
    notes: str = ""

    @property
    def d(self) -> int:
        return self.C // self.H


def make_layer(
    name: str,
    seed: int,
    B: int,
    N: int,
    C: int,
    H: int,
    Cc: int = 768,
    T: int = T_TEXT,
    bits_kv: int = 8,
    trigger_positions: Optional[Sequence[int]] = None,
    n_random_triggers: int = 0,
    trigger_scale: float = 1.0,
    outlier_frac: float = 0.0,
    outlier_scale: float = 20.0,
    per_batch_masks: bool = False,
    bias: bool = False,
) -> Layer:
    """Draw one layer. Draw order is fixed: context, Wq, Wk, Wv, Wo, hidden,
    outlier channels, trigger positions, bias."""
    rng = np.random.Generator(np.random.PCG64(seed))
    context = rng.standard_normal((B, T, Cc))
    Wq = rng.standard_normal((C, C)) / np.sqrt(C)
    Wk = rng.standard_normal((C, Cc)) / np.sqrt(Cc)
    Wv = rng.standard_normal((C, Cc)) / np.sqrt(Cc)
    Wo = rng.standard_normal((C, C)) / np.sqrt(C)
    hidden = rng.standard_normal((B, N, C))
    n_out = int(round(outlier_frac * C))
    if n_out > 0:
        ch = rng.choice(C, size=n_out, replace=False)
        hidden[:, :, ch] *= outlier_scale
    mask = np.zeros((B, T), dtype=np.uint8)
    if trigger_positions is not None:
        for b in range(B):
            mask[b, list(trigger_positions)] = 1
    elif n_random_triggers > 0:
        if per_batch_masks:
            for b in range(B):
                pos = rng.choice(np.arange(1, T), size=n_random_triggers, replace=False)
                mask[b, pos] = 1
        else:
            pos = rng.choice(np.arange(1, T), size=n_random_triggers, replace=False)
            mask[:, pos] = 1
    if trigger_scale != 1.0:
        context = context * np.where(mask[:, :, None] != 0, trigger_scale, 1.0)
    bias_o = rng.standard_normal(C) * 0.1 if bias else np.zeros(C)
    return Layer(
        name=name, B=B, N=N, C=C, H=H, T=T, Cc=Cc, bits_kv=bits_kv,
        context=context.astype(np.float16), mask=mask,
        Wq=Wq.astype(np.float16), Wk=Wk.astype(np.float16),
        Wv=Wv.astype(np.float16), Wo=Wo.astype(np.float16),
        bias_o=bias_o.astype(np.float32), hidden=hidden.astype(np.float16), seed=seed,
    )


def config1() -> Layer:
    """SD1.5 lowest-resolution layer, batch 1, two-token trigger at positions 1-2 (x3)."""
    return make_layer("cfg1_sd15_8x8", seed=0, B=1, N=64, C=1280, H=8, Cc=768, bits_kv=8,
                      trigger_positions=(1, 2), trigger_scale=3.0)


def config2(seed: int = 1, B: int = 2, N: int = 4096) -> Layer:
    """SD1.5 highest-resolution layer, CFG pair, 1 trigger at position 5; the headline shape."""
    return make_layer("cfg2_sd15_64x64", seed=seed, B=B, N=N, C=320, H=8, Cc=768, bits_kv=8,
                      trigger_positions=(5,), outlier_frac=0.01)


SD15_LAYER_SHAPES = [(4096, 320)] * 5 + [(1024, 640)] * 5 + [(256, 1280)] * 5 + [(64, 1280)]


def config3(layers: Optional[Sequence[int]] = None) -> List[Layer]:
    """The 16 cross-attention layers of one SD1.5 UNet step, batch 2, int4 K/V,
    3 trigger rows at random positions in 1..76 (same positions in every layer:
    the prompt is the same). The 5/5/5/1 split over resolutions follows the
    usual SD1.5 UNet layout (down 2+2+2, mid 1, up 3+3+3)."""
    out = []
    pos_rng = np.random.Generator(np.random.PCG64(2))
    pos = tuple(int(p) for p in pos_rng.choice(np.arange(1, T_TEXT), size=3, replace=False))
    for i, (N, C) in enumerate(SD15_LAYER_SHAPES):
        if layers is not None and i not in layers:
            continue
        out.append(make_layer(f"cfg3_layer{i:02d}_{N}x{C}", seed=200 + i, B=2, N=N, C=C, H=8,
                              Cc=768, bits_kv=4, trigger_positions=pos))
    return out


def config4() -> List[Layer]:
    """SDXL-shaped layers: 10 or 20 heads of 64, context 77 x 2048, int4 K/V, outliers."""
    a = make_layer("cfg4_sdxl_4096x640", seed=3, B=2, N=4096, C=640, H=10, Cc=2048, bits_kv=4,
                   n_random_triggers=2, outlier_frac=0.01)
    b = make_layer("cfg4_sdxl_1024x1280", seed=4, B=2, N=1024, C=1280, H=20, Cc=2048, bits_kv=4,
                   n_random_triggers=2, outlier_frac=0.01)
    return [a, b]


def config5(R: int = 16, N: int = 4096) -> List[Layer]:
    """R concurrent requests at the SD1.5 4096-query layer, each with its own
    weights (as from R personalised checkpoints), context and 1-4 trigger rows."""
    out = []
    for r in range(R):
        ntrig = 1 + (r % 4)
        out.append(make_layer(f"cfg5_req{r:02d}", seed=1000 + r, B=1, N=N, C=320, H=8, Cc=768,
                              bits_kv=8, n_random_triggers=ntrig))
    return out


def tiny(seed: int = 7, B: int = 1, N: int = 4, C: int = 8, H: int = 1, T: int = 5, Cc: int = 6,
         bits_kv: int = 8, trigger_positions: Sequence[int] = (1,), trigger_scale: float = 3.0) -> Layer:
    """A few-element layer for brute-force checks."""
    return make_layer("tiny", seed=seed, B=B, N=N, C=C, H=H, Cc=Cc, T=T, bits_kv=bits_kv,
                      trigger_positions=trigger_positions, trigger_scale=trigger_scale, bias=True)
