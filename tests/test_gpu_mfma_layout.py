"""The operand-to-lane maps every kernel relies on, checked on the device: one
MFMA on random dense operands must equal the host matrix product."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

SHAPES = {0: (16, 32, 16), 1: (16, 16, 16), 2: (32, 16, 32), 3: (16, 4, 16)}


@pytest.mark.parametrize("which", [0, 1, 2, 3])
def test_mfma_probe_matches_host_product(which):
    import torch
    from paper_2512_02371_amd import hb
    M, K, N = SHAPES[which]
    rng = np.random.default_rng(100 + which)
    A = rng.integers(-8, 9, size=(M, K)).astype(np.float64)       # small integers: exact everywhere
    B = rng.integers(-8, 9, size=(K, N)).astype(np.float64)
    dt = torch.float32 if which == 3 else torch.float16
    dA = torch.tensor(A, dtype=dt, device="cuda:0")
    dB = torch.tensor(B, dtype=dt, device="cuda:0")
    dD = torch.zeros((M, N), dtype=torch.float32, device="cuda:0")
    print(f"mfma probe which={which}", flush=True)
    hb.hb_mfma_probe(which, dA, dB, dD)
    torch.cuda.synchronize()
    assert np.array_equal(dD.cpu().numpy().astype(np.float64), A @ B)


@pytest.mark.parametrize("n", [8, 2048, 2049, 4096 * 3 + 5, 1 << 20])
def test_copy_reference_converts_every_element(n):
    """hb_copy_f16_f32 (the bandwidth reference) is an exact fp16 -> fp32 conversion, tails included."""
    import torch
    from paper_2512_02371_amd import hb
    x = (torch.rand(n, device="cuda:0") * 4 - 2).half()
    out = torch.full((n + 8,), -7.0, dtype=torch.float32, device="cuda:0")
    hb.hb_copy_f16_f32(x, out[:n])
    torch.cuda.synchronize()
    assert torch.equal(out[:n], x.float())
    assert torch.all(out[n:] == -7.0), "wrote past the end"
