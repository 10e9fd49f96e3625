"""Pins for oracle.target_sample: the base model's tokens under a sampling policy with
coupled uniforms (Appendix C, randomized decoding)."""
import numpy as np
import scipy.special

from paper_2508_09072_amd import workloads as W


def chain(T):
    return np.arange(-1, T - 1, dtype=np.int32)


def test_equal_logits_give_the_floor_of_u_times_v(oracle_mod):
    # uniform distribution over V tokens: inverse CDF is floor(u * V)
    V, T = 10, 6
    logits = W.to_bf16_bits(np.full((1, T, V), 0.75, dtype=np.float32))
    u = np.array([[0.0, 0.05, 0.31, 0.55, 0.87, 0.999]])
    got = oracle_mod.target_sample(logits, chain(T)[None], u)
    assert got[0].tolist() == [0, 0, 3, 5, 8, 9]


def test_two_tokens_follow_the_logistic_function(oracle_mod):
    # two tokens: P(token 0) = 1 / (1 + exp(-(a - b) / tau))
    a, b, tau = 1.5, -0.25, 0.7           # exactly representable in bf16
    p0 = 1.0 / (1.0 + np.exp(-(a - b) / tau))
    us = np.array([0.0, p0 - 1e-9, p0 + 1e-9, 0.5, 0.99])
    T = len(us)
    logits = W.to_bf16_bits(np.tile(np.array([a, b], dtype=np.float32), (1, T, 1)))
    got = oracle_mod.target_sample(logits, chain(T)[None], us[None], temperature=tau)
    assert got[0].tolist() == [0, 0, 1, int(0.5 >= p0), 1]


def test_low_temperature_is_the_greedy_token(oracle_mod):
    rng = np.random.Generator(np.random.PCG64(11))
    bits = W.to_bf16_bits(rng.standard_normal((3, 4, 300), dtype=np.float32) * 4)
    # make the maximum unique and well separated
    vals = W.bf16_bits_to_f32(bits)
    top = np.argmax(vals, axis=-1)
    np.put_along_axis(vals, top[..., None], 30.0, axis=-1)
    bits = W.to_bf16_bits(vals)
    parents = np.tile(chain(4), (3, 1))
    u = rng.random((3, 4)) * 0.999
    got = oracle_mod.target_sample(bits, parents, u, temperature=0.01)
    assert np.array_equal(got, oracle_mod.target_argmax(bits)) and np.array_equal(got, top)


def test_token_is_monotone_in_u_and_zero_weight_tokens_never_come_out(oracle_mod):
    rng = np.random.Generator(np.random.PCG64(12))
    V, T = 64, 50
    row = rng.standard_normal(V).astype(np.float32) * 2
    row[[3, 17, 63]] = -np.inf                     # no probability
    bits = W.to_bf16_bits(np.tile(row, (1, T, 1)))
    bits[0, :, 40] = 0x7FC0                        # NaN: no probability either
    u = np.sort(rng.random(T))[None]
    got = oracle_mod.target_sample(bits, chain(T)[None], u)[0]
    assert np.all(np.diff(got) >= 0)
    assert not set(got.tolist()) & {3, 17, 40, 63}
    last = oracle_mod.target_sample(bits[:, :1], chain(1)[None], np.array([[np.nextafter(1.0, 0.0)]]))
    assert last[0, 0] == 62                        # u next to 1: the last token that has weight


def test_infinite_logits_take_everything_and_share_it(oracle_mod):
    # the limit of the softmax when some logits go to +inf: those tokens, equally
    V, T = 12, 6
    row = np.linspace(-1.0, 1.0, V).astype(np.float32)
    row[[2, 5, 9]] = np.inf
    bits = W.to_bf16_bits(np.tile(row, (1, T, 1)))
    u = np.array([[0.0, 0.3, 0.34, 0.6, 0.67, 0.99]])
    got = oracle_mod.target_sample(bits, chain(T)[None], u)[0]
    assert got.tolist() == [2, 2, 5, 5, 9, 9]


def test_frequencies_follow_the_softmax(oracle_mod):
    rng = np.random.Generator(np.random.PCG64(13))
    V, n, tau = 12, 40000, 1.3
    row = W.to_bf16_bits((rng.standard_normal(V) * 1.5).astype(np.float32))
    p = scipy.special.softmax(W.bf16_bits_to_f32(row).astype(np.float64) / tau)
    # n independent draws: n sequences, root only
    bits = np.tile(row, (n, 1, 1))
    got = oracle_mod.target_sample(bits, np.full((n, 1), -1, dtype=np.int32), rng.random((n, 1)), temperature=tau)
    freq = np.bincount(got[:, 0], minlength=V) / n
    assert np.all(np.abs(freq - p) < 4.5 * np.sqrt(p * (1 - p) / n) + 1e-4)


def test_nodes_of_one_depth_share_their_uniform(oracle_mod):
    # a tree whose nodes all see the same distribution: the token depends on the depth only
    rng = np.random.Generator(np.random.PCG64(14))
    parents = np.array([[-1, 0, 0, 1, 1, 2, 3, 5, 0]], dtype=np.int32)
    depth = np.array([0, 1, 1, 2, 2, 2, 3, 3, 1])
    T, V = parents.shape[1], 40
    row = W.to_bf16_bits((rng.standard_normal(V) * 2).astype(np.float32))
    bits = np.tile(row, (1, T, 1))
    u = rng.random((1, T))
    got = oracle_mod.target_sample(bits, parents, u)[0]
    for d in range(4):
        assert len(set(got[depth == d].tolist())) == 1
    by_depth = oracle_mod.target_sample(bits[:, :4], chain(4)[None], u[:, :4])[0]   # a chain: node d has depth d
    assert [int(got[np.flatnonzero(depth == d)[0]]) for d in range(4)] == by_depth.tolist()


def test_speculative_run_with_the_same_uniforms_repeats_the_plain_run(oracle_mod):
    # Randomized losslessness: drive a toy base model (logits are a fixed function of the last two
    # tokens) once token by token and once through draft trees + acceptance, with one uniform per
    # position.  Both runs must produce the same tokens.
    rng = np.random.Generator(np.random.PCG64(15))
    V, steps, tau = 24, 60, 0.8
    table = W.to_bf16_bits((rng.standard_normal((V, V, V)) * 2.5).astype(np.float32))   # logits after (prev2, prev1)
    uniforms = rng.random(4 * steps + 8)                                                # one per position
    start = [1, 2]

    def sample_after(prefix, pos):
        bits = table[prefix[-2], prefix[-1]][None, None]
        return int(oracle_mod.target_sample(bits, np.array([[-1]], dtype=np.int32),
                                            np.array([[uniforms[pos]]]), temperature=tau)[0, 0])

    plain = list(start)
    while len(plain) < len(start) + steps:
        plain.append(sample_after(plain, len(plain)))

    spec = list(start)
    max_path = 6
    while len(spec) < len(start) + steps:
        # a random draft tree under the last committed token; half of the time one branch is the true continuation
        T = 12
        parents = np.full(T, -1, dtype=np.int32)
        tokens = np.zeros(T, dtype=np.int32)
        tokens[0] = spec[-1]
        for n in range(1, T):
            parents[n] = rng.integers(0, n)
            tokens[n] = rng.integers(0, V)
        if rng.random() < 0.7:      # plant the plain run's continuation along the chain 0 -> 1 -> 2 -> 3
            for d in range(1, 4):
                parents[d] = d - 1
                if len(spec) - 1 + d < len(plain):
                    tokens[d] = plain[len(spec) - 1 + d]
        depth = np.zeros(T, dtype=np.int64)
        for n in range(1, T):
            depth[n] = depth[parents[n]] + 1
        # the base model's logits at every node: a function of the two tokens that end its path
        bits = np.zeros((1, T, V), dtype=np.uint16)
        for n in range(T):
            prev1 = tokens[n]
            prev2 = tokens[parents[n]] if n else spec[-2]
            bits[0, n] = table[prev2, prev1]
        # node n's successor sits at position len(spec) + depth(n): row d of this step's uniforms
        u_step = np.zeros((1, T))
        for d in range(T):
            u_step[0, d] = uniforms[len(spec) + d]
        target = oracle_mod.target_sample(bits, parents[None], u_step, temperature=tau)
        acc, path, bonus = oracle_mod.accept_path(tokens[None], target.astype(np.int32), parents[None], max_path)
        for j in range(1, int(acc[0]) + 1):
            spec.append(int(tokens[path[0, j]]))
        spec.append(int(bonus[0]))
    n = len(start) + steps
    assert spec[:n] == plain[:n]
