"""The library's launches under HIP graph capture: a chain of whole steps (logits -> target tokens ->
fused verification step, which feeds the next step's lengths and cache) is captured once and replayed
several times, with eager work and synchronisations between the replays; every replay must leave
exactly what the eager run leaves.  The entry points allocate nothing and record no memset nodes."""
import numpy as np
import pytest

from paper_2508_09072_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def R():
    from paper_2508_09072_amd import binding
    binding.load()
    return binding


def _bits(t):
    import torch
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("D,T,lens", [(128, 24, [700, 65, 1300, 0]), (64, 64, [2000, 333])])
def test_replays_of_a_captured_chain_of_steps_equal_eager(R, D, T, lens):
    import torch
    n_steps, vocab, depth = 3, 4096, 5
    # max_path = T: pages are mapped for T more positions per sequence, room for what three steps append
    w = W.make_custom("graph_T%d" % T, B=len(lens), Hq=8, Hkv=2, D=D, T=T, seq_lens=lens, tree="trie", depth=depth,
                      max_path=T, seed=440 + T)
    assert n_steps * (depth + 1) <= T
    dw = R.to_device(w)
    bound = int(max(lens)) + n_steps * (depth + 1)
    ws = torch.empty(max(R.reader_workspace_bytes(dw.dims, bound), 256), dtype=torch.uint8, device="cuda")
    gen = torch.Generator(device="cuda").manual_seed(77)
    logits = torch.randn((w.B, w.T, vocab), device="cuda", dtype=torch.bfloat16, generator=gen)
    # the drafted tokens are made to agree with the arg max often, so that paths are accepted
    greedy = logits.float().argmax(-1).to(torch.int32)
    draft = dw.draft_tokens.clone()
    par = dw.parents.long().clamp(min=0)
    agree = torch.rand((w.B, w.T), device="cuda", generator=gen) < 0.7
    draft = torch.where(agree, torch.gather(greedy, 1, par), draft % vocab).contiguous()
    target = torch.zeros((w.B, w.T), dtype=torch.int32, device="cuda")
    seq0, kc0, vc0 = dw.seq_lens.clone(), dw.k_cache.clone(), dw.v_cache.clone()
    outs = [torch.empty_like(dw.out) for _ in range(n_steps)]
    lens = [torch.empty_like(dw.accept_len) for _ in range(n_steps)]

    def reset():
        dw.seq_lens.copy_(seq0)
        dw.k_cache.copy_(kc0)
        dw.v_cache.copy_(vc0)
        dw.status.zero_()
        for t in outs + lens:
            t.zero_()

    def chain():
        for k in range(n_steps):
            R.reader_target_argmax(logits, target)
            R.reader_verify_step(dw.dims, dw.q, dw.k_tree, dw.v_tree, dw.k_cache, dw.v_cache, dw.page_table,
                                 dw.seq_lens, dw.parents, draft, target, outs[k], None, lens[k], dw.path, dw.bonus,
                                 bound, ws, dw.status)

    reset()
    chain()
    torch.cuda.synchronize()
    assert int(dw.status.item()) == 0
    want = [t.clone() for t in outs + lens] + [dw.seq_lens.clone()]
    want_cache = (_bits(dw.k_cache), _bits(dw.v_cache))
    assert int((dw.seq_lens - seq0).min()) >= n_steps          # every step appended at least the root
    assert int(lens[0].max()) >= 1                              # and some draft was accepted

    reset()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        chain()
    for replay in range(4):
        reset()
        scratch = torch.randn(1 << 20, device="cuda").sum()    # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert float(scratch) == float(scratch)
        got = outs + lens + [dw.seq_lens]
        for a, b in zip(got, want):
            assert torch.equal(a, b), "replay %d differs from the eager run" % replay
        assert np.array_equal(_bits(dw.k_cache), want_cache[0]) and np.array_equal(_bits(dw.v_cache), want_cache[1])
        assert int(dw.status.item()) == 0


def test_an_error_left_behind_by_somebody_else_is_not_taken_for_a_failed_launch(R):
    # the runtime keeps a thread's last error until it is read; the library must not report it as its own
    import ctypes
    import torch
    logits = torch.randn((4, 1000), device="cuda", dtype=torch.bfloat16)
    tok = torch.zeros(4, dtype=torch.int32, device="cuda")
    hip = ctypes.CDLL("libamdhip64.so")
    assert hip.hipSetDevice(1 << 20) != 0            # refused, no side effect, leaves an error behind
    R.reader_target_argmax(logits, tok)
    torch.cuda.synchronize()
    assert torch.equal(tok.long(), logits.float().argmax(-1))


def test_measured_peaks_are_plausible_and_bad_sizes_are_refused():
    # the two bare loops behind the roofline discussion: a copy ring (HBM -> LDS) and a matrix-instruction loop
    import torch
    from paper_2508_09072_amd import binding as R
    R.load()
    src = torch.empty(512 << 20, dtype=torch.uint8, device="cuda").fill_(3)
    scratch = torch.empty(1 << 19, dtype=torch.uint8, device="cuda")
    R.reader_measure_peaks(src, scratch)
    got = R.reader_measure_peaks(src, scratch)
    print("measured peaks:", got, flush=True)
    assert 2000.0 < got["hbm_read_gbs"] < 8000.0
    assert 800.0 < got["mfma_bf16_tflops"] < 2600.0
    assert 900.0 < got["mfma_clock_mhz"] < 2600.0
    # the rate is what 1024 matrix pipes do at that clock, one 32-cycle instruction after the other
    assert abs(got["mfma_bf16_tflops"] - 1024 * 32768 / 32 * got["mfma_clock_mhz"] * 1e-6) < 0.05 * got["mfma_bf16_tflops"]
    with pytest.raises(RuntimeError):
        R.reader_measure_peaks(src[: 1 << 20], scratch)
    with pytest.raises(RuntimeError):
        R.reader_measure_peaks(src, scratch[:1024])
