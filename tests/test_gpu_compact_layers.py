"""GPU parity of reader_kv_compact_layers with the oracle: bit-exact caches and lengths."""
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


def run_gpu(R, s, Hq=None):
    import torch
    NL, num_pages, Hkv, page_size, D = s.k_cache.shape
    B = s.path.shape[0]
    dims = R.make_dims(B, s.T, Hq or Hkv, Hkv, D, s.page_table.shape[1], s.max_path, num_pages)
    k = torch.from_numpy(s.k_cache.view(np.int16)).cuda().view(torch.bfloat16)
    v = torch.from_numpy(s.v_cache.view(np.int16)).cuda().view(torch.bfloat16)
    L = torch.from_numpy(s.seq_lens.copy()).cuda()
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    R.reader_kv_compact_layers(dims, torch.from_numpy(s.path).cuda(), torch.from_numpy(s.accept_len).cuda(), k, v,
                               torch.from_numpy(s.page_table).cuda(), L, status)
    torch.cuda.synchronize()
    bits = lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16)
    return bits(k), bits(v), L.cpu().numpy(), int(status.item())


def check(R, oracle_mod, s):
    print("layered compaction parity:", s.name, s.k_cache.shape, "accept", s.accept_len.tolist(), flush=True)
    k_ref, v_ref, L_ref = s.k_cache.copy(), s.v_cache.copy(), s.seq_lens.copy()
    oracle_mod.kv_compact_layers(k_ref, v_ref, s.path, s.accept_len, s.page_table, L_ref)
    k, v, L, status = run_gpu(R, s)
    assert status == 0 and np.array_equal(L, L_ref)
    assert np.array_equal(k, k_ref), "K differs in %d elements" % int((k != k_ref).sum())
    assert np.array_equal(v, v_ref), "V differs in %d elements" % int((v != v_ref).sum())


@pytest.mark.parametrize("D,Hkv,NL,T,max_path", [(128, 8, 4, 32, 9), (64, 4, 2, 16, 16), (128, 1, 1, 128, 128),
                                                 (128, 2, 3, 64, 33)])
def test_random_steps(R, oracle_mod, D, Hkv, NL, T, max_path):
    s = W.make_incache_step("rand_D%d_T%d" % (D, T), B=5, T=T, Hkv=Hkv, D=D, num_layers=NL,
                            seq_lens=[0, 15, 16, 300, 1023], max_path=max_path, seed=D + T)
    check(R, oracle_mod, s)


def test_long_paths_need_more_than_one_pass(R, oracle_mod):
    # 8 heads x 127 rows x 16 chunks x 2 = far more items than a workgroup carries at once; every
    # second node is accepted, so every destination is the source of an earlier row
    s = W.make_incache_step("long", B=2, T=128, Hkv=8, D=128, num_layers=2, seq_lens=[7, 100], max_path=128, seed=5)
    for b in range(2):
        s.parents[b] = np.arange(-1, 127)
        nodes = [0] + list(range(1, 128, 2))
        s.path[b, :] = -1
        s.path[b, : len(nodes)] = nodes
        s.accept_len[b] = len(nodes) - 1
    check(R, oracle_mod, s)


def test_paths_already_in_place_and_single_roots(R, oracle_mod):
    s = W.make_incache_step("inplace", B=3, T=8, Hkv=2, D=128, num_layers=2, seq_lens=[9, 30, 31], max_path=8, seed=6)
    s.path[0] = np.arange(8); s.accept_len[0] = 7             # a fully accepted chain: nothing moves
    s.path[1] = [0] + [-1] * 7; s.accept_len[1] = 0           # nothing but the root
    check(R, oracle_mod, s)


def test_bad_sequences_are_left_alone_and_reported(R, oracle_mod):
    s = W.make_incache_step("bad", B=4, T=16, Hkv=2, D=64, num_layers=2, seq_lens=[5, 20, 33, 40], max_path=8, seed=7)
    good = W.make_incache_step("bad", B=4, T=16, Hkv=2, D=64, num_layers=2, seq_lens=[5, 20, 33, 40], max_path=8, seed=7)
    s.path[1, :3] = [0, 5, 3]; s.accept_len[1] = 2            # not increasing
    s.accept_len[2] = 8                                        # longer than a path can be
    s.page_table[3, 40 // 16] = s.k_cache.shape[1] + 4         # a page id outside the pool
    k, v, L, status = run_gpu(R, s)
    assert status == (R.STATUS_BAD_PATH | R.STATUS_BAD_PAGE)
    # sequence 0 is moved as the oracle moves it; the others keep cache and length
    k_ref, v_ref, L_ref = good.k_cache.copy(), good.v_cache.copy(), good.seq_lens.copy()
    only0 = W.make_incache_step("bad", B=4, T=16, Hkv=2, D=64, num_layers=2, seq_lens=[5, 20, 33, 40], max_path=8, seed=7)
    only0.path[1:, 0] = 0; only0.path[1:, 1:] = -1; only0.accept_len[1:] = 0     # roots only: nothing moves
    oracle_mod.kv_compact_layers(k_ref, v_ref, only0.path, only0.accept_len, good.page_table, L_ref)
    assert L.tolist() == [int(L_ref[0]), 20, 33, 40]
    assert np.array_equal(k, k_ref) and np.array_equal(v, v_ref)


def test_serving_shape(R, oracle_mod):
    # the batched preset's step with all 32 layers of an 8B-class model (per-layer cache as in
    # the attention benchmark would be 6.7 GB; the lengths are scaled down, the shapes kept)
    rng = np.random.Generator(np.random.PCG64(8))
    s = W.make_incache_step("serving", B=16, T=32, Hkv=8, D=128, num_layers=32,
                            seq_lens=[int(x) for x in rng.integers(64, 257, size=16)], max_path=9, seed=9)
    check(R, oracle_mod, s)


def test_two_calls_in_a_row_on_the_same_tensors(R, oracle_mod):
    # The workgroups of a sequence elect the one that writes the new length through counters inside the library,
    # which must be back at zero when a call ends: a second call (lengths put back, caches as the first call
    # left them) has to move its rows and grow the lengths exactly like the oracle does.
    import torch
    s = W.make_incache_step("twice", B=6, T=16, Hkv=4, D=128, num_layers=5, seq_lens=[3, 40, 41, 100, 15, 16],
                            max_path=8, seed=11)
    k_ref, v_ref, L_ref = s.k_cache.copy(), s.v_cache.copy(), s.seq_lens.copy()
    NL, num_pages, Hkv, page_size, D = s.k_cache.shape
    dims = R.make_dims(6, s.T, Hkv, Hkv, D, s.page_table.shape[1], s.max_path, num_pages)
    k = torch.from_numpy(s.k_cache.view(np.int16)).cuda().view(torch.bfloat16)
    v = torch.from_numpy(s.v_cache.view(np.int16)).cuda().view(torch.bfloat16)
    L = torch.from_numpy(s.seq_lens.copy()).cuda()
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    path, acc, table = torch.from_numpy(s.path).cuda(), torch.from_numpy(s.accept_len).cuda(), torch.from_numpy(s.page_table).cuda()
    bits = lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16)
    for call in range(2):
        L.copy_(torch.from_numpy(s.seq_lens))
        L_ref[:] = s.seq_lens
        oracle_mod.kv_compact_layers(k_ref, v_ref, s.path, s.accept_len, s.page_table, L_ref)
        R.reader_kv_compact_layers(dims, path, acc, k, v, table, L, status)
        torch.cuda.synchronize()
        assert int(status.item()) == 0
        assert np.array_equal(L.cpu().numpy(), L_ref), "lengths after call %d" % call
        assert np.array_equal(bits(k), k_ref) and np.array_equal(bits(v), v_ref), "caches after call %d" % call
