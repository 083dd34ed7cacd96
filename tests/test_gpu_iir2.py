"""hb_iir2 / hb_iir2_valu (second-order recursive filter, Sec. V-D) against the fp64 oracle."""
import numpy as np
import pytest

from paper_2512_02371_amd import synth
from hbtest import assert_close, up

pytestmark = pytest.mark.gpu

FILTERS = [
    (1.6, -0.8),      # resonant: complex poles of radius 0.894
    (1.2, -0.52),
    (0.5, 0.3),       # two real poles
    (-0.9, 0.0),      # first order, alternating sign
    (1.0, 0.0),       # the running sum (a pole on the unit circle)
    (0.0, 0.0),       # the identity
]


def run(fn, sig, alpha, beta, pitch_extra=0):
    import torch
    from paper_2512_02371_amd import hb
    C, T = sig.shape
    d_in = up(sig)
    if pitch_extra:
        base = torch.full((C, T + pitch_extra), 3.0, dtype=torch.float16, device="cuda:0")
        base[:, :T] = d_in
        d_in = base[:, :T]
    obuf = torch.full((C, T + pitch_extra), 7.0, dtype=torch.float32, device="cuda:0")
    out = obuf[:, :T]
    ws = torch.empty(hb.hb_iir2_workspace_size(C, T), dtype=torch.uint8, device="cuda:0")
    print(f"{fn} C={C} T={T} alpha={alpha} beta={beta} pitch+{pitch_extra}", flush=True)
    getattr(hb, fn)(d_in, out, alpha, beta, ws)
    torch.cuda.synchronize()
    return out.cpu().numpy(), obuf.cpu().numpy()


@pytest.mark.parametrize("fn", ["hb_iir2", "hb_iir2_valu"])
@pytest.mark.parametrize("alpha,beta", FILTERS)
@pytest.mark.parametrize("C,T", [(2, 5000), (1, 512), (3, 513), (1, 1), (2, 31), (1, 40000)])
def test_iir2_matches_oracle(orc, fn, alpha, beta, C, T):
    from paper_2512_02371_amd import hb
    sig = synth.uniform_pm1_f16(9500 + T, (C, T))
    if hb.hb_iir2_abs_gain(alpha, beta, T) > 16384:
        # the running sum over 40000 samples: its error magnification is beyond what the call accepts
        assert (alpha, beta, T) == (1.0, 0.0, 40000)
        with pytest.raises(hb.HbError) as e:
            run(fn, sig, alpha, beta)
        assert e.value.code == hb.HB_ERR_UNSUPPORTED
        return
    got, _ = run(fn, sig, alpha, beta)
    # the oracle filters with the fp32 coefficients the library receives
    ref = orc.iir2(sig, float(np.float32(alpha)), float(np.float32(beta)))
    assert_close(got, ref, f"{fn} {C}x{T} ({alpha}, {beta})")


@pytest.mark.parametrize("fn", ["hb_iir2", "hb_iir2_valu"])
def test_iir2_pitched_rows(orc, fn):
    sig = synth.uniform_pm1_f16(9600, (2, 3000))
    got, obuf = run(fn, sig, 1.6, -0.8, pitch_extra=5)
    assert_close(got, orc.iir2(sig, float(np.float32(1.6)), float(np.float32(-0.8))), fn)
    assert np.all(obuf[:, 3000:] == 7.0), "wrote past the end of the signal"


@pytest.mark.parametrize("fn", ["hb_iir2", "hb_iir2_valu"])
def test_iir2_impulse_response(fn):
    """Needs no oracle: an impulse late in the signal (tile 3, block 5) gives h_k = (p1^(k+1) - p2^(k+1)) / (p1 - p2)."""
    alpha, beta = np.float32(1.6), np.float32(-0.8)
    p1, p2 = np.roots([1.0, -float(alpha), -float(beta)])
    T, t0 = 4096, 3 * 512 + 5 * 32 + 7
    sig = np.zeros((1, T), dtype=np.float16)
    sig[0, t0] = 1.0
    got, _ = run(fn, sig.view(np.uint16), float(alpha), float(beta))
    k = np.arange(T - t0)
    h = ((p1 ** (k + 1) - p2 ** (k + 1)) / (p1 - p2)).real
    assert np.all(got[0, :t0] == 0.0)
    assert np.max(np.abs(got[0, t0:] - h)) < 2e-5


def test_iir2_long_signal(orc):
    """More than eight tiles per lane of the state scan (the path that moves tile states as 16-byte
    pieces), an odd number of them, and a ragged last tile."""
    C, T = 1, (1 << 23) + 777
    sig = synth.uniform_pm1_f16(9650, (C, T))
    for fn in ("hb_iir2", "hb_iir2_valu"):
        got, _ = run(fn, sig, 1.2, -0.52)
        assert_close(got, orc.iir2(sig, float(np.float32(1.2)), float(np.float32(-0.52))), f"{fn} 1 x {T}")


def test_iir2_full_size(orc):
    """The paper's workload: 2^21 stereo samples."""
    C, T = 2, 1 << 21
    sig = synth.uniform_pm1_f16(9700, (C, T))
    got, _ = run("hb_iir2", sig, 1.6, -0.8)
    assert_close(got, orc.iir2(sig, float(np.float32(1.6)), float(np.float32(-0.8))), "2 x 2^21")
