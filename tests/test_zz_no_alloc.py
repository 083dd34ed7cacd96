"""hb_sat2d_noalloc (the entry point for callers that cannot allocate: its carry tables live in a
fixed array inside the library) against hb_sat2d on the same inputs: the two run the same kernels,
so the outputs must be bit-identical, on two calls in a row that share the array, the second one
on a smaller image.  The first result is also held to the oracle's bar."""
import numpy as np
import pytest

from paper_2512_02371_amd import synth
from hbtest import TOL, scaled_err, up

pytestmark = pytest.mark.gpu


def _both(img):
    import torch
    from paper_2512_02371_amd import hb
    H, W = img.shape
    d_in = up(img)
    ref = torch.full((H, W), -1.0, dtype=torch.float32, device="cuda:0")
    got = torch.full((H, W), -2.0, dtype=torch.float32, device="cuda:0")
    ws = torch.empty(hb.hb_sat2d_workspace_size(H, W), dtype=torch.uint8, device="cuda:0")
    print(f"hb_sat2d_noalloc H={H} W={W}", flush=True)
    hb.hb_sat2d(d_in, ref, ws)
    hb.hb_sat2d_noalloc(d_in, got)
    torch.cuda.synchronize()
    return got.cpu().numpy(), ref.cpu().numpy()


def test_noalloc_matches_workspace_entry_point_twice(orc):
    big = synth.uniform01_f16(9101, (1000, 1500))
    got, ref = _both(big)
    assert np.array_equal(got, ref)
    o = orc.sat2d(big)
    assert np.abs(got - o).max() / o[-1, -1] <= TOL
    assert scaled_err(got, o).max() <= TOL
    small = synth.uniform01_f16(9102, (130, 77))          # second call: smaller, shares the array
    got, ref = _both(small)
    assert np.array_equal(got, ref)
    o = orc.sat2d(small)
    assert scaled_err(got, o).max() <= TOL


def test_noalloc_benchmark_size_and_limit():
    import torch
    from paper_2512_02371_amd import hb
    got, ref = _both(synth.binary01_f16(9103, (4096, 4096)))
    assert np.array_equal(got, ref)
    # one tile row more than the array can hold: refused before any launch
    H, W = 64 * 80, 64 * 64
    assert hb.hb_sat2d_workspace_size(H, W) > hb.HB_SAT2D_NOALLOC_SCRATCH_BYTES
    x = torch.zeros((H, W), dtype=torch.float16, device="cuda:0")
    out = torch.zeros((H, W), dtype=torch.float32, device="cuda:0")
    with pytest.raises(hb.HbError) as e:
        hb.hb_sat2d_noalloc(x, out)
    assert e.value.code == hb.HB_ERR_UNSUPPORTED
