"""GPU parity of reader_target_sample with the oracle (Appendix C, randomized decoding).

The kernel adds its weights in fp32, the oracle in double precision.  A row's token is
compared exactly wherever u * total keeps a margin of EPS * total to the neighbouring token
boundaries of the oracle's cumulative weights; inside that margin either neighbour is right,
and the kernel's token must be one whose interval of cumulative weight touches the margin.
EPS: a weight carries the relative error of exp2 of a rounded argument (argument up to ~100,
so ~100 * 2^-24 * ln 2 ~ 4e-6) and the sums add ~log2(512) + V/512/256 roundings: 1e-5 covers it."""
import numpy as np
import pytest

from paper_2508_09072_amd import workloads as W

pytestmark = pytest.mark.gpu
EPS = 1e-5


@pytest.fixture(scope="module")
def R():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2508_09072_amd import binding
    binding.load()
    return binding


def gpu_sample(R, bits, parents, uniforms, temperature):
    import torch
    t = torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    out = torch.full(bits.shape[:2], -1, dtype=torch.int32, device="cuda")
    R.reader_target_sample(t, torch.from_numpy(parents).cuda(), torch.from_numpy(uniforms.astype(np.float32)).cuda(),
                           temperature, out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def check(R, oracle_mod, bits, parents, uniforms, temperature, min_exact=0.0):
    got = gpu_sample(R, bits, parents, uniforms, temperature)
    ref, thr, tot = oracle_mod.target_sample(bits, parents, uniforms.astype(np.float32), temperature, with_cdf=True)
    B, T, V = bits.shape
    exact = 0
    for b in range(B):
        for n in range(T):
            k, r = int(got[b, n]), int(ref[b, n])
            assert 0 <= k < V
            if k == r:
                exact += 1
                continue
            cdf = oracle_mod.target_sample_weights(bits[b, n], temperature)
            eps = EPS * tot[b, n]
            lo_k = cdf[k - 1] if k else 0.0
            assert cdf[k] > lo_k, "token %d of row (%d, %d) has no weight" % (k, b, n)
            assert lo_k <= thr[b, n] + eps and cdf[k] >= thr[b, n] - eps, \
                "row (%d, %d): token %d, oracle %d, threshold %.9g of %.9g, interval [%.9g, %.9g]" % (
                    b, n, k, r, thr[b, n], tot[b, n], lo_k, cdf[k])
    assert exact >= min_exact * B * T, "only %d of %d rows agree exactly" % (exact, B * T)
    return got


def trees(B, T, rng):
    parents = np.full((B, T), -1, dtype=np.int32)
    for b in range(B):
        for n in range(1, T):
            parents[b, n] = rng.integers(max(0, n - 4), n)
    return parents


@pytest.mark.parametrize("B,T,V,tau", [(2, 5, 1, 1.0), (3, 4, 7, 1.0), (2, 8, 255, 0.7), (2, 6, 4099, 1.0),
                                       (3, 16, 32000, 1.0), (1, 12, 128256, 1.0), (2, 3, 1001, 3.0)])
def test_random_trees_and_peaked_logits(R, oracle_mod, B, T, V, tau):
    print("sample parity: B", B, "T", T, "V", V, "tau", tau, flush=True)
    rng = np.random.Generator(np.random.PCG64(B * 1009 + T * 31 + V))
    bits = W.make_logits(B, T, V, rng, peaked=True)
    check(R, oracle_mod, bits, trees(B, T, rng), W.make_uniforms(B, T, rng), tau, min_exact=0.9)


def test_diffuse_logits_stay_within_the_rounding_margin(R, oracle_mod):
    # no peak: every token holds ~1e-5 of the mass, so fp32 sums may pick a neighbour
    rng = np.random.Generator(np.random.PCG64(77))
    bits = W.make_logits(2, 8, 128256, rng, peaked=False)
    check(R, oracle_mod, bits, trees(2, 8, rng), W.make_uniforms(2, 8, rng), 1.0)


def test_low_temperature_gives_the_greedy_token(R, oracle_mod):
    rng = np.random.Generator(np.random.PCG64(78))
    bits = W.make_logits(2, 6, 5000, rng, peaked=True)
    got = check(R, oracle_mod, bits, trees(2, 6, rng), W.make_uniforms(2, 6, rng) * np.float32(0.99), 0.02, min_exact=1.0)
    assert np.array_equal(got, oracle_mod.target_argmax(bits))


def test_specials_edges_of_u_and_rows_without_weight(R, oracle_mod):
    rng = np.random.Generator(np.random.PCG64(79))
    B, T, V = 1, 10, 1003                      # odd V: rows start at every 2-byte phase
    bits = W.make_logits(B, T, V, rng, peaked=True)
    bits[0, 1, ::2] = 0xFF80                   # -inf on every other token
    bits[0, 2, 5:900] = 0x7FC0                 # NaNs carry no probability
    bits[0, 3, :] = 0xFF80                     # no weight at all -> 0
    bits[0, 4, :] = 0x7FC0
    bits[0, 5, :V - 1] = 0xFF80                # only the last token (in the tail) has weight
    bits[0, 6, 1:] = 0xFF80                    # only the first token (in the head) has weight
    parents = np.arange(-1, T - 1, dtype=np.int32)[None]      # a chain: node d has depth d
    u = W.make_uniforms(B, T, rng)
    u[0, 0] = 0.0
    u[0, 7] = np.float32(1.0 - 2.0 ** -24)     # the largest float below 1
    u[0, 8] = 0.0
    got = check(R, oracle_mod, bits, parents, u, 1.0, min_exact=0.9)
    assert got[0, 3] == 0 and got[0, 4] == 0 and got[0, 5] == V - 1 and got[0, 6] == 0


def test_infinite_and_huge_logits(R, oracle_mod):
    rng = np.random.Generator(np.random.PCG64(82))
    B, T, V = 1, 8, 2000
    bits = W.make_logits(B, T, V, rng, peaked=True)
    bits[0, 0, [3, 700, 1999]] = 0x7F80          # +inf in the head block, a middle block, the last block
    bits[0, 1, 1500] = 0x7F80                    # a single +inf
    bits[0, 2, 100:110] = 0x7F7F                 # the largest finite bf16 (3.4e38): scaling overflows
    bits[0, 3, :] = 0x7F80                       # everything +inf: uniform over the vocabulary
    parents = np.arange(-1, T - 1, dtype=np.int32)[None]
    u = W.make_uniforms(B, T, rng)
    got = check(R, oracle_mod, bits, parents, u, 1.0)
    assert got[0, 0] in (3, 700, 1999) and got[0, 1] == 1500 and 100 <= got[0, 2] < 110
    # the lowest temperature the entry point takes: the greedy token
    small = W.make_logits(1, 4, 1000, rng, peaked=True)
    got = check(R, oracle_mod, small, parents[:, :4], u[:, :4] * np.float32(0.99), 1e-6, min_exact=1.0)
    assert np.array_equal(got, oracle_mod.target_argmax(small))


def test_nodes_of_one_depth_draw_the_same_token(R, oracle_mod):
    rng = np.random.Generator(np.random.PCG64(80))
    parents = np.array([[-1, 0, 0, 1, 1, 2, 3, 5, 0]], dtype=np.int32)
    depth = np.array([0, 1, 1, 2, 2, 2, 3, 3, 1])
    T, V = parents.shape[1], 3000
    row = W.make_logits(1, 1, V, rng, peaked=True)[0, 0]
    bits = np.tile(row, (1, T, 1))
    got = check(R, oracle_mod, bits, parents, W.make_uniforms(1, T, rng), 1.0)[0]
    for d in range(4):
        assert len(set(got[depth == d].tolist())) == 1


def test_headline_step_shape(R, oracle_mod):
    # the rows of one verification step of the batched preset: 16 sequences x 32 nodes, vocabulary 128256
    w = W.make_config(2)
    rng = np.random.Generator(np.random.PCG64(81))
    V = 128256
    bits = W.make_logits(w.B, w.T, V, rng, peaked=True)
    u = W.make_uniforms(w.B, w.T, rng)
    got = gpu_sample(R, bits, w.parents, u, 1.0)
    # the oracle on a sample of rows
    pick = [(b, n) for b in (0, 7, 15) for n in (0, 1, 13, 31)]
    exact = 0
    for b, n in pick:
        ref, thr, tot = oracle_mod.target_sample(bits[b:b + 1], w.parents[b:b + 1], u[b:b + 1], 1.0, with_cdf=True)
        k = int(got[b, n])
        if k == ref[0, n]:
            exact += 1
            continue
        cdf = oracle_mod.target_sample_weights(bits[b, n], 1.0)
        eps = EPS * tot[0, n]
        lo_k = cdf[k - 1] if k else 0.0
        assert cdf[k] > lo_k and lo_k <= thr[0, n] + eps and cdf[k] >= thr[0, n] - eps
    assert exact >= len(pick) - 2
    # and the sampled tokens drive the acceptance like any other target tokens
    acc, path, bonus = oracle_mod.accept_path((w.draft_tokens % V).astype(np.int32), got.astype(np.int32), w.parents,
                                              w.max_path)
    assert acc.min() >= 0 and np.all(bonus == got[np.arange(w.B), path[np.arange(w.B), acc]])
