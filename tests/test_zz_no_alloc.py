"""taq_cross_attn_static (the entry point that allocates nothing: its scratch is a fixed array inside the
library) against taq_cross_attn with a caller-owned workspace, through the C ABI: bit-identical outputs on two
calls in a row, the second on a smaller input, for the head-group path and the kernel-per-stage path (the two
that use scratch memory) and for a single-kernel shape (which uses none)."""
import numpy as np
import pytest
import torch

from paper_2603_22943_amd import synth
from paper_2603_22943_amd import taq as T
from tests import gpu_helpers as G

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("C,H,N1,N2,bits_kv", [
    (1280, 8, 200, 45, 8),    # head groups, d = 160: float32 A^ V~ and the row maxima pass through the scratch
    (1280, 20, 70, 33, 4),    # head groups, d = 64
    (96, 4, 300, 130, 8),     # one kernel per stage: codes, float32 Q and O in the scratch
    (320, 8, 150, 64, 8),     # single kernel: no scratch
])
def test_static_scratch_entry_matches_workspace_entry(C, H, N1, N2, bits_kv):
    print(f"[case] static scratch C={C} H={H} N={N1} then N={N2} bits_kv={bits_kv}", flush=True)
    L = synth.make_layer("noalloc", seed=C + H + N1, B=2, N=N1, C=C, H=H, Cc=64, T=77, bits_kv=bits_kv,
                         trigger_positions=(3, 40), trigger_scale=3.0, bias=True, outlier_frac=0.01)
    g = G.GpuRun(L, taps=False)                                  # taq_cross_attn, own workspace
    small = np.ascontiguousarray(L.hidden[:, 7:7 + N2])
    g2 = G.GpuRun(L, taps=False, hidden=small)
    # two calls in a row on the library's scratch, the second smaller; outputs start as NaN patterns
    out1 = torch.full_like(g.out_d, float("nan"))
    out2 = torch.full_like(g2.out_d, float("nan"))
    T.taq_cross_attn_static(g.hidden_d, g.packed, g.wq_code, g.wo_code, g.scales, g.mask_d, g.shape, out1)
    T.taq_cross_attn_static(g2.hidden_d, g.packed, g.wq_code, g.wo_code, g.scales, g.mask_d, g2.shape, out2)
    torch.cuda.synchronize()
    assert np.array_equal(out1.cpu().numpy().view(np.uint16), g.out.view(np.uint16))
    assert np.array_equal(out2.cpu().numpy().view(np.uint16), g2.out.view(np.uint16))


def test_static_scratch_entry_rejects_shapes_beyond_its_array():
    s = T.make_shape(B=2, N=4096, C=1280, H=8, T=77, Cc=768)
    x = torch.zeros(16, dtype=torch.float16, device=G.DEV)
    with pytest.raises(T.TaqError) as e:
        T.taq_cross_attn_static(x, x, x, x, x, None, s, x)
    assert e.value.status == T.TAQ_ERR_SCRATCH_TOO_SMALL
    torch.cuda.synchronize()
