"""The five stages recorded into a HIP graph (torch.cuda.CUDAGraph on torch's capture stream) and
replayed: the library allocates nothing, synchronises nothing and clears nothing with memset calls, so
its launches can be captured.  Every replay is checked against the eager result, with eager work and
synchronisations between the replays."""
import numpy as np
import pytest

from paper_2512_02371_amd import synth
from hbtest import up

pytestmark = pytest.mark.gpu


def test_five_stages_replay_from_a_graph():
    import torch
    from paper_2512_02371_amd import hb
    dev = "cuda:0"
    H, W = 192, 320
    img = [up(synth.uniform01_f16(7000 + i, (H, W))) for i in range(2)]
    taps8 = synth.random_taps_f16(7010, 8)
    gau = synth.gaussian_taps_f16(16, 3.0)
    x = up(synth.uniform_pm1_f16(7011, (1, 40, 64, 64)))
    w = up(synth.normal_f16(7012, (3, 3, 64, 64), 1.0 / 24.0))
    ws = torch.empty(hb.hb_sat2d_workspace_size(H, W), dtype=torch.uint8, device=dev)

    def buffers():
        return dict(fir=torch.zeros((H, W), dtype=torch.float32, device=dev),
                    blur=torch.zeros((H, W), dtype=torch.float32, device=dev),
                    sat=torch.zeros((H, W), dtype=torch.float32, device=dev),
                    conv=torch.zeros((1, 40, 64, 64), dtype=torch.float16, device=dev),
                    res=torch.zeros((H, W), dtype=torch.float32, device=dev),
                    down=torch.zeros((H // 2, W // 2), dtype=torch.float16, device=dev))

    def step(src, o):
        hb.hb_fir1d(src, o["fir"], taps8, 3)
        hb.hb_sepblur(src, o["blur"], gau, 7, gau, 7)
        hb.hb_sat2d(src, o["sat"], ws)
        hb.hb_conv3x3(x, w, o["conv"])
        hb.hb_pyr_level(src, o["res"], o["down"])

    # eager results for both inputs
    want = []
    for i in range(2):
        o = buffers()
        step(img[i], o)
        torch.cuda.synchronize()
        want.append({k: v.clone() for k, v in o.items()})

    # capture one step on a static input buffer
    static_in = img[0].clone()
    out = buffers()
    step(static_in, out)                       # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(static_in, out)
    for rep in range(4):
        i = rep & 1
        static_in.copy_(img[i])                # eager work between the replays
        for v in out.values():
            v.fill_(-1.0)
        torch.cuda.synchronize()
        print(f"replay {rep} on input {i}", flush=True)
        graph.replay()
        torch.cuda.synchronize()
        for k, v in out.items():
            assert torch.equal(v, want[i][k]), f"replay {rep}: {k} differs from the eager result"
