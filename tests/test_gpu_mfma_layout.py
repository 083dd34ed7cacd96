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


def test_mfma_probe_two_shapes_chained_on_one_accumulator():
    """A K = 16 product issued straight after a K = 32 product on the same accumulator: the order
    that once produced a wrong tile inside an unrolled kernel and that the stage kernels cannot
    express any more (the shared header offers one shape).  Exact small integers; if the pair still
    misbehaves the case is reported as an expected failure, with the worst difference."""
    import torch
    from paper_2512_02371_amd import hb
    rng = np.random.default_rng(104)
    A1 = rng.integers(-8, 9, size=(16, 32)).astype(np.float64)
    B1 = rng.integers(-8, 9, size=(32, 16)).astype(np.float64)
    A2 = rng.integers(-8, 9, size=(16, 16)).astype(np.float64)
    B2 = rng.integers(-8, 9, size=(16, 16)).astype(np.float64)
    dA = torch.tensor(np.concatenate([A1.ravel(), A2.ravel()]), dtype=torch.float16, device="cuda:0")
    dB = torch.tensor(np.concatenate([B1.ravel(), B2.ravel()]), dtype=torch.float16, device="cuda:0")
    dD = torch.zeros((16, 16), dtype=torch.float32, device="cuda:0")
    print("mfma probe which=4", flush=True)
    hb.hb_mfma_probe(4, dA, dB, dD)
    torch.cuda.synchronize()
    got, want = dD.cpu().numpy().astype(np.float64), A1 @ B1 + A2 @ B2
    if not np.array_equal(got, want):
        pytest.xfail(f"chained 16x16x32 -> 16x16x16 on one accumulator: max difference {np.abs(got - want).max()}")


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
