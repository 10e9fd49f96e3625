"""GPU parity of reader_kv_rearrange with the oracle: bit-exact caches, flags and lengths."""
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


def run_gpu(R, c):
    import torch
    k = torch.from_numpy(c.k_pad.view(np.int16)).cuda().view(torch.bfloat16)
    v = torch.from_numpy(c.v_pad.view(np.int16)).cuda().view(torch.bfloat16)
    valid = torch.from_numpy(c.valid.copy()).cuda()
    B, S = c.valid.shape
    new_len = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    scratch = torch.empty(max(R.reader_kv_rearrange_scratch_bytes(B, S), 256), dtype=torch.uint8, device="cuda")
    R.reader_kv_rearrange(k, v, valid, new_len, scratch)
    torch.cuda.synchronize()
    bits = lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16)
    return bits(k), bits(v), valid.cpu().numpy(), new_len.cpu().numpy()


def check(R, oracle_mod, c):
    print("rearrange parity:", c.name, c.shape, flush=True)
    k_ref, v_ref, valid_ref = c.k_pad.copy(), c.v_pad.copy(), c.valid.copy()
    len_ref = oracle_mod.kv_rearrange(k_ref, v_ref, valid_ref)
    k, v, valid, new_len = run_gpu(R, c)
    assert np.array_equal(new_len, len_ref) and np.array_equal(valid, valid_ref)
    assert np.array_equal(k, k_ref), "K differs in %d elements" % int((k != k_ref).sum())
    assert np.array_equal(v, v_ref), "V differs in %d elements" % int((v != v_ref).sum())


@pytest.mark.parametrize("D,Hkv,NL", [(128, 8, 3), (64, 4, 2), (128, 1, 1)])
def test_random_padded_caches(R, oracle_mod, D, Hkv, NL):
    c = W.make_padded_cache("rand_D%d" % D, NL=NL, B=6, Hkv=Hkv, D=D, prompt_lens=[300, 17, 64, 1, 129, 255], steps=25,
                            p_long=0.15, seed=D + NL)
    check(R, oracle_mod, c)


def test_many_steps_ragged_batch(R, oracle_mod):
    rng = np.random.Generator(np.random.PCG64(9))
    c = W.make_padded_cache("many", NL=2, B=16, Hkv=2, D=128, prompt_lens=rng.integers(5, 400, size=16), steps=50,
                            p_long=0.1, seed=21)
    check(R, oracle_mod, c)


def test_more_slots_than_one_round_of_the_scan(R, oracle_mod):
    # the flags are scanned in rounds of 8192 slots per sample: two rounds here, with holes in both
    c = W.make_padded_cache("long", NL=2, B=3, Hkv=2, D=64, prompt_lens=[9000, 100, 8190], steps=30, p_long=0.2, seed=33)
    check(R, oracle_mod, c)


def test_hand_made_patterns(R, oracle_mod):
    # no hole; nothing valid; a single far entry; alternating flags; a hole of exactly one pass
    NL, B, S, Hkv, D = 1, 6, 200, 2, 128
    rng = np.random.Generator(np.random.PCG64(3))
    k = W.to_bf16_bits(rng.standard_normal((NL, B, S, Hkv, D), dtype=np.float32))
    v = W.to_bf16_bits(rng.standard_normal((NL, B, S, Hkv, D), dtype=np.float32))
    valid = np.zeros((B, S), dtype=np.uint8)
    valid[0, :150] = 1
    valid[2, 199] = 1
    valid[3, ::2] = 1
    valid[4, :16] = 1
    valid[4, 32:48] = 1
    valid[5, 1:] = 1
    c = W.PaddedCache("hand", np.ascontiguousarray(k), np.ascontiguousarray(v), valid)
    check(R, oracle_mod, c)


def test_second_pass_changes_nothing(R, oracle_mod):
    import torch
    c = W.make_padded_cache("twice", NL=2, B=4, Hkv=2, D=64, prompt_lens=[40, 3, 77, 20], steps=12, seed=8)
    k, v, valid, new_len = run_gpu(R, c)
    c2 = W.PaddedCache("twice2", k.copy(), v.copy(), valid.copy())
    k2, v2, valid2, new_len2 = run_gpu(R, c2)
    assert np.array_equal(k2, k) and np.array_equal(v2, v) and np.array_equal(valid2, valid)
    assert np.array_equal(new_len2, new_len)
