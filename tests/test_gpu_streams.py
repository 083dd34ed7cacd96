"""Calls on two HIP streams at once (default priorities): the library keeps no state between calls, so
stages with their own buffers and workspaces may overlap; every result equals the one computed alone."""
import numpy as np
import pytest

from paper_2512_02371_amd import synth
from hbtest import up

pytestmark = pytest.mark.gpu


def test_stages_on_two_streams_match_the_serial_results():
    import torch
    from paper_2512_02371_amd import hb
    dev = "cuda:0"
    H, W = 512, 1024
    imgs = [up(synth.uniform01_f16(7100 + i, (H, W))) for i in range(2)]
    gau = synth.gaussian_taps_f16(16, 3.0)
    k2 = synth.random_kernel2d_f16(7110, 16, 16)
    taps = synth.random_taps_f16(7111, 100)

    def run_all(img, ws):
        o = [torch.zeros((H, W), dtype=torch.float32, device=dev) for _ in range(5)]
        hb.hb_sepblur(img, o[0], gau, 7, gau, 7)
        hb.hb_sat2d(img, o[1], ws)
        hb.hb_pyr_level(img, o[2], None)
        hb.hb_conv2d(img, o[3], k2, 7, 7)
        hb.hb_fir1d(img, o[4], taps, 49)
        return o

    wss = [torch.empty(hb.hb_sat2d_workspace_size(H, W), dtype=torch.uint8, device=dev) for _ in range(2)]
    want = [run_all(imgs[i], wss[i]) for i in range(2)]
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(device=dev), torch.cuda.Stream(device=dev)]
    for rep in range(3):
        got = [None, None]
        for i in range(2):
            with torch.cuda.stream(streams[i]):
                got[i] = run_all(imgs[i], wss[i])
        torch.cuda.synchronize()
        for i in range(2):
            for a, b in zip(got[i], want[i]):
                assert torch.equal(a, b), f"round {rep}, stream {i}: a result differs from the serial one"
