"""The library's launches under HIP graph capture: a captured layer (PTS quantizer + W8A8 linear for in_proj and
out_proj, the fused launch for x_proj and dt_proj) replays to the bits of the eager result, on replays after
the first and with eager work in between.  The library allocates nothing and records no memset nodes."""
import pytest
import torch

import paper_2412_20386_amd as ptq
from paper_2412_20386_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _layer(cfg):
    lins = []
    for li in range(len(synth.CONFIGS[cfg].linears)):
        c = synth.make_linear_case(cfg, 0, li, device=DEV)
        wq, s_w, inv_m = ptq.fold_smoothing(c.w, c.m)
        M = c.B * c.L
        lins.append(dict(c=c, wq=wq, s_w=s_w, inv_m=inv_m, fused=(c.K <= 128 or c.N <= 128),
                         xq=torch.empty((M, c.K), dtype=torch.int8, device=DEV),
                         y=torch.empty((M, c.N), dtype=torch.float16, device=DEV)))
    return lins


def _run(lins):
    for d in lins:
        c = d["c"]
        if d["fused"]:
            ptq.w8a8_linear_fused(c.x, d["inv_m"], c.s_tok, d["wq"], d["s_w"], c.bias, c.B, c.L, y=d["y"])
        else:
            ptq.quantize_pts(c.x, d["inv_m"], c.s_tok, c.B, c.L, xq=d["xq"])
            ptq.w8a8_linear(d["xq"], d["wq"], c.s_tok, d["s_w"], c.bias, c.B, c.L, y=d["y"])


@pytest.mark.parametrize("cfg", [1, 3])
def test_captured_layer_replays_to_the_eager_bits(cfg):
    print(f"graph capture cfg{cfg}", flush=True)
    lins = _layer(cfg)
    _run(lins)
    torch.cuda.synchronize()
    want = [d["y"].clone() for d in lins]
    want_xq = [d["xq"].clone() for d in lins]

    side = torch.cuda.Stream()  # default priority
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        _run(lins)  # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        _run(lins)
    torch.cuda.synchronize()

    other = _layer(0)  # eager work between the replays (config 0: one small linear)
    for rep in range(4):
        for d in lins:  # fill kernels, not memsets
            d["y"].fill_(float(rep + 1))
            d["xq"].fill_(rep + 1)
        _run(other[:1])
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for d, y_ref, xq_ref in zip(lins, want, want_xq):
            assert torch.equal(d["y"].view(torch.int16), y_ref.view(torch.int16)), (rep, d["c"].name)
            if not d["fused"]:
                assert torch.equal(d["xq"], xq_ref), (rep, d["c"].name)
