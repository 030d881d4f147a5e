"""The five benchmark configurations at full size, HIP path against the oracle.

The oracle runs each whole layer in about a second, so every output element is
compared (no sampling needed). Same bars as tests/test_gpu_parity.py. The launch
configuration is the one bench.py times: same entry points, same shapes.
"""
import numpy as np
import pytest
import torch

from paper_2603_22943_amd import synth
from paper_2603_22943_amd import taq as T
from tests import gpu_helpers as G
from tests.test_gpu_parity import check_layer

pytestmark = pytest.mark.gpu


def test_config1_lowest_resolution_layer():
    check_layer(synth.config1())


def test_config2_headline_shape():
    check_layer(synth.config2())


@pytest.mark.parametrize("bits_kv,bits_q,bits_prob,prob_grid", [
    (4, 4, 4, "linear"),    # the 8/4 setting of Table 1
    (4, 4, 4, "log2"),      # ... with the logarithmic probability grid of the ablation table
    (8, 8, 8, "rowmax"),    # per-row dynamic probability scale
])
def test_config2_headline_shape_other_settings(bits_kv, bits_q, bits_prob, prob_grid):
    """The headline shape at full size in the other activation settings bench.py times."""
    import dataclasses
    L = dataclasses.replace(synth.config2(), bits_kv=bits_kv)
    check_layer(L, f"config2 kv{bits_kv} q{bits_q} p{bits_prob} {prob_grid}", bits_q=bits_q, bits_prob=bits_prob,
                prob_grid=prob_grid, w_layout=1)


@pytest.mark.parametrize("layer", list(range(16)))
def test_config3_unet_step_layers_int4(layer):
    # the 16 cross-attention layers of one UNet step: 4096x320 (x5), 1024x640 (x5), 256x1280 (x5), 64x1280
    (L,) = synth.config3(layers=[layer])
    check_layer(L)


def test_config4_sdxl_shapes_int4():
    for L in synth.config4():
        check_layer(L)


def test_config5_multi_checkpoint_batch():
    reqs = synth.config5(R=16)
    runs = [G.GpuRun(L, taps=False) for L in reqs]
    s = runs[0].shape
    outs, table = [], []
    for r in runs:
        o = torch.zeros_like(r.out_d)
        outs.append(o)
        table.append(dict(hidden=r.hidden_d, qkv_packed=r.packed, Wq=r.wq_code, Wo=r.wo_code, scales=r.scales,
                          trigger_mask=r.mask_d, out=o))
    T.taq_cross_attn_batched(table, s)
    torch.cuda.synchronize()
    for i, (L, o) in enumerate(zip(reqs, outs)):
        ref, _ = G.oracle_run(L)
        max_abs, rel_l2 = G.out_errors(o.cpu().numpy(), ref)
        print(f"[case] {L.name} ntrig={int(L.mask.sum())}: max_abs={max_abs:.3e} rel_l2={rel_l2:.3e}", flush=True)
        assert max_abs <= 2e-2 and rel_l2 <= 5e-3


def test_unet_step_of_16_layers_from_one_graph_matches_the_oracle():
    """The 16 cross-attention layers of one UNet step (configs[2]) captured into ONE HIP graph, as bench.py replays
    them: after each of several replays (eager work of the library in between) every layer's output must be bit-identical
    to its eager output, and that output must meet the oracle's within the block tolerance."""
    layers = synth.config3()
    runs = [G.GpuRun(L, taps=False, w_layout=1) for L in layers]
    wss = [torch.empty(T.taq_workspace_bytes(r.shape), dtype=torch.uint8, device=G.DEV) for r in runs]
    outs = [torch.zeros_like(r.out_d) for r in runs]

    def enqueue():
        for r, o, ws in zip(runs, outs, wss):
            T.taq_cross_attn(r.hidden_d, r.packed, r.wq_code, r.wo_code, r.scales, r.mask_d, r.shape, o, ws)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        enqueue()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        enqueue()
    for rep in range(3):
        for o in outs:
            o.zero_()
        r0 = runs[rep]
        T.taq_cross_attn(r0.hidden_d, r0.packed, r0.wq_code, r0.wo_code, r0.scales, r0.mask_d, r0.shape)  # eager, in between
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, (r, o) in enumerate(zip(runs, outs)):
            assert np.array_equal(o.cpu().numpy().view(np.uint16), r.out.view(np.uint16)), (rep, i)
    for i, (L, r) in enumerate(zip(layers, runs)):
        ref, _ = G.oracle_run(L)
        max_abs, rel_l2 = G.out_errors(r.out, ref)
        print(f"[case] graph layer {i} {L.name}: max_abs={max_abs:.3e} rel_l2={rel_l2:.3e}", flush=True)
        assert max_abs <= 2e-2 and rel_l2 <= 5e-3


def test_hip_graph_replays_match_eager():
    """bench.py replays the steps from a HIP graph. Replay several times with eager work and
    synchronisations in between; every replay must reproduce the eager result bit for bit."""
    L = synth.config2(N=1024)
    g = G.GpuRun(L, taps=False)
    s = g.shape
    ws = torch.empty(T.taq_workspace_bytes(s), dtype=torch.uint8, device=G.DEV)
    outs = [torch.zeros_like(g.out_d) for _ in range(3)]
    hid = [g.hidden_d.clone() for _ in range(3)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for h, o in zip(hid, outs):
            T.taq_cross_attn(h, g.packed, g.wq_code, g.wo_code, g.scales, g.mask_d, s, o, ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for h, o in zip(hid, outs):
            T.taq_cross_attn(h, g.packed, g.wq_code, g.wo_code, g.scales, g.mask_d, s, o, ws)
    ref = g.out.view(np.uint16)
    rng = np.random.Generator(np.random.PCG64(3))
    for rep in range(4):
        for o in outs:
            o.zero_()
        # eager work of the program itself between replays, on other data
        other = torch.from_numpy(rng.standard_normal((L.B, 1024, L.C)).astype(np.float16)).to(G.DEV)
        T.taq_cross_attn(other, g.packed, g.wq_code, g.wo_code, g.scales, g.mask_d, s)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for o in outs:
            assert np.array_equal(o.cpu().numpy().view(np.uint16), ref), rep
