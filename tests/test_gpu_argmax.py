"""GPU parity of reader_target_argmax with the oracle (bit-exact indices)."""
import numpy as np
import pytest

from paper_2508_09072_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def R():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2508_09072_amd import binding
    binding.load()
    return binding


def gpu_argmax(R, bits):
    import torch
    t = torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    out = torch.full(bits.shape[:-1], -1, dtype=torch.int32, device="cuda")
    R.reader_target_argmax(t, out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


@pytest.mark.parametrize("rows,V", [(3, 1), (5, 7), (4, 255), (6, 4099), (2, 128256), (33, 32000)])
def test_random_logits(R, oracle_mod, rows, V):
    print("argmax parity: rows", rows, "V", V, flush=True)
    rng = np.random.Generator(np.random.PCG64(rows * 131 + V))
    bits = W.to_bf16_bits(rng.standard_normal((rows, V), dtype=np.float32) * 4)   # bf16 makes ties common
    assert np.array_equal(gpu_argmax(R, bits), oracle_mod.target_argmax(bits))


def test_odd_row_starts_ties_and_specials(R, oracle_mod):
    # V odd: rows start at every 2-byte phase of a 16-byte line; maxima planted at both ends
    rng = np.random.Generator(np.random.PCG64(5))
    V = 1001
    vals = rng.standard_normal((16, V), dtype=np.float32)
    for r in range(16):
        vals[r, (0, V - 1, r, V - 1 - r)[r % 4]] = 9.0
        vals[r, V // 2] = 9.0 if r % 2 else -9.0
    bits = W.to_bf16_bits(vals)
    bits[3, 10] = 0x7FC0      # NaN
    bits[4, :] = 0x7FC0       # nothing but NaNs
    bits[5, :] = 0xFF80       # nothing but -inf
    bits[6, 500] = 0x7F80     # +inf
    assert np.array_equal(gpu_argmax(R, bits), oracle_mod.target_argmax(bits))
