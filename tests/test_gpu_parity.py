"""Parity of the HIP library (through its C ABI) against the CPU oracle, on a real MI355X.

Attention: |gpu - oracle| <= 2e-2 + 2e-2 * |oracle| element by element (bf16 outputs,
fp32 accumulation).  Acceptance and compaction: bit-exact.
"""
import numpy as np
import pytest

from paper_2508_09072_amd import workloads as W
from helpers import assert_close

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def R():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2508_09072_amd import binding
    binding.load()          # raises if the HIP library was not built: no fallback
    return binding


@pytest.fixture
def tune(R):
    """Planner overrides for one test; cleared afterwards whatever happens."""
    touched = []

    def set_(which, value):
        touched.append(which)
        R.reader_tuning_override(which, value)
    yield set_
    for which in touched:
        R.reader_tuning_override(which, -1)


def bf16_to_np(t):
    return t.float().cpu().numpy().astype(np.float64)


def run_attn(R, w, variant=0, want_status=0, sm_scale=0.0):
    import torch
    dw = R.to_device(w, variant=variant, sm_scale=sm_scale)
    dw.out.fill_(float("nan"))
    dw.lse.fill_(float("nan"))
    R.reader_tree_attn(dw.dims, dw.q, dw.k_tree, dw.v_tree, dw.k_cache, dw.v_cache, dw.page_table,
                       dw.seq_lens, dw.parents, dw.out, dw.lse, dw.max_seq_len, dw.workspace, dw.status)
    torch.cuda.synchronize()
    assert int(dw.status.item()) == want_status
    return bf16_to_np(dw.out), dw.lse.cpu().numpy().astype(np.float64)


def check_attn(R, oracle_mod, w, variants=(0, 1), sm_scale=0.0):
    ref, ref_lse = oracle_mod.tree_attn(w.q, w.k_tree, w.v_tree, w.k_cache, w.v_cache, w.page_table,
                                        w.seq_lens, w.parents, sm_scale=sm_scale)
    for variant in variants:
        print("attn parity:", w.name, "variant", variant, "B", w.B, "T", w.T, "L", w.seq_lens[:6], flush=True)
        out, lse = run_attn(R, w, variant=variant, sm_scale=sm_scale)
        assert_close(out, ref, what="%s variant %d out" % (w.name, variant))
        assert_close(lse, ref_lse, what="%s variant %d lse" % (w.name, variant))


# ------------------------------------------------------------------ attention, whole outputs

@pytest.mark.parametrize("index,scale", [(0, 1.0), (1, 1.0), (2, 0.25), (3, 0.03), (4, 0.04)])
def test_attn_presets_element_by_element(R, oracle_mod, index, scale):
    # presets 0 and 1 at full size; 2-4 with shortened prefixes (still several 64-key tiles,
    # ragged tails, several workgroups per pair) so that the oracle finishes in seconds
    w = W.make_config(index, length_scale=scale)
    check_attn(R, oracle_mod, w, variants=(0, 1) if index < 2 else (0,))


@pytest.mark.parametrize("L", [0, 1, 15, 16, 63, 64, 65, 127, 129, 500])
def test_attn_prefix_length_edges(R, oracle_mod, L):
    w = W.make_custom("edge_L%d" % L, B=2, Hq=8, Hkv=2, D=128, T=20, seq_lens=[L, max(0, L - 1)],
                      tree="uniform", depth=5, seed=100 + L)
    check_attn(R, oracle_mod, w)


@pytest.mark.parametrize("T,tree", [(1, "chain"), (2, "chain"), (31, "uniform"), (64, "trie"), (65, "uniform"),
                                    (128, "chain"), (128, "star"), (128, "trie")])
def test_attn_tree_shapes(R, oracle_mod, T, tree):
    w = W.make_custom("tree_%s_T%d" % (tree, T), B=2, Hq=4, Hkv=2, D=128, T=T, seq_lens=[70, 200],
                      tree=tree, depth=12, branch=8, seed=200 + T)
    check_attn(R, oracle_mod, w)


@pytest.mark.parametrize("Hq,Hkv,D", [(8, 8, 64), (8, 2, 64), (16, 2, 64), (4, 4, 128), (16, 2, 128), (32, 2, 128)])
def test_attn_head_layouts(R, oracle_mod, Hq, Hkv, D):
    w = W.make_custom("heads_%d_%d_%d" % (Hq, Hkv, D), B=3, Hq=Hq, Hkv=Hkv, D=D, T=24,
                      seq_lens=[130, 5, 321], tree="trie", depth=6, branch=3, seed=300 + Hq + D)
    check_attn(R, oracle_mod, w)


def test_attn_many_short_sequences(R, oracle_mod):
    # more pairs than a workgroup range holds tiles: ranges cover several whole pairs
    rng = np.random.Generator(np.random.PCG64(5))
    w = W.make_custom("many_short", B=40, Hq=8, Hkv=4, D=128, T=8, seq_lens=rng.integers(0, 90, size=40),
                      tree="uniform", depth=4, seed=401)
    check_attn(R, oracle_mod, w)


def test_attn_more_sequences_than_lengths_fit_in_lds(R, oracle_mod):
    # above 1024 sequences the clamped lengths are re-read from memory while the tile list is written
    rng = np.random.Generator(np.random.PCG64(6))
    w = W.make_custom("very_many", B=1100, Hq=4, Hkv=2, D=64, T=4, seq_lens=rng.integers(0, 40, size=1100),
                      tree="uniform", depth=3, seed=404)
    check_attn(R, oracle_mod, w)


@pytest.mark.parametrize("T,Hq", [(16, 8), (48, 16)])
def test_attn_ranges_longer_than_the_tile_list(R, oracle_mod, T, Hq, tune):
    # few, long ranges: a workgroup walks more items than its list holds at once and has to
    # extend the list on the way (both kernel flavours: up to 128 query rows, and more)
    tune(R.TUNE_ATTN_RANGES, 8)
    w = W.make_custom("long_ranges", B=1, Hq=Hq, Hkv=4, D=128, T=T, seq_lens=[35000], tree="trie", depth=6,
                      seed=405)
    check_attn(R, oracle_mod, w)


@pytest.mark.parametrize("T,Hq", [(16, 8), (48, 16)])
def test_attn_ranges_cut_with_64_bit_arithmetic(R, oracle_mod, T, Hq, tune):
    # the kernel cuts its ranges in 32-bit arithmetic when the host can show that nothing
    # overflows, else in 64-bit: force the second path on a ragged batch
    tune(R.TUNE_ATTN_AXIS64, 1)
    w = W.make_custom("axis64", B=5, Hq=Hq, Hkv=4, D=128, T=T, seq_lens=[1, 900, 64, 2051, 130], tree="trie",
                      depth=5, seed=406)
    check_attn(R, oracle_mod, w)


@pytest.mark.parametrize("cost,front", [(0, 0), (1, 0), (3, 0), (3, 3), (5, 2), (9, 0), (9, 9)])
@pytest.mark.parametrize("axis64", [0, 1])
def test_attn_pair_cost_in_front_of_and_behind_the_tiles(R, oracle_mod, cost, front, axis64, tune):
    # what a pair costs beyond its tiles is booked partly in front of its tiles and partly behind them when
    # the ranges are cut: any split gives the same result, whichever padding a cut falls into (ranges that
    # end up empty included), in the 32-bit cut (found by votes) and the 64-bit one (found by search)
    tune(R.TUNE_ATTN_PAIR_COST, cost)
    tune(R.TUNE_ATTN_PAIR_FRONT, front)
    if axis64:
        tune(R.TUNE_ATTN_AXIS64, 1)
    w = W.make_custom("pair_cost", B=6, Hq=8, Hkv=4, D=128, T=24, seq_lens=[0, 64, 700, 3, 129, 260], tree="trie",
                      depth=5, seed=409)
    check_attn(R, oracle_mod, w, variants=(0,))


@pytest.mark.parametrize("lens", [[300, 40], [2500]])
def test_attn_most_query_rows_per_kv_head(R, oracle_mod, lens):
    # 128 nodes x 16 grouped heads = 2048 query rows per kv head: sixteen 128-row chunks (short contexts) or
    # eight 256-row chunks per key range, and so few ranges that all workgroups run at once
    w = W.make_custom("rows2048", B=len(lens), Hq=32, Hkv=2, D=128, T=128, seq_lens=lens, tree="trie", depth=9,
                      branch=3, seed=411)
    plan = R.reader_attn_plan(R.make_dims(w.B, w.T, w.Hq, w.Hkv, w.D, w.page_table.shape[1], w.max_path, w.k_cache.shape[0]),
                              int(max(lens)))
    assert plan["row_chunks"] * plan["key_ranges"] <= 256, plan
    check_attn(R, oracle_mod, w, variants=(0,))


@pytest.mark.parametrize("case", range(16))
def test_attn_seeded_random_shapes(R, oracle_mod, case):
    # a seeded sweep over batch, tree size, head layout and length mix (empty sequences included), both
    # kernel flavours (up to 128 query rows per kv head, and more)
    rng = np.random.Generator(np.random.PCG64(9000 + case))
    D = int(rng.choice([64, 128]))
    Hkv = int(rng.choice([1, 2, 4]))
    G = int(rng.choice([1, 2, 4, 8]))
    T = int(rng.choice([1, 3, 16, 33, 64, 100, 128]))
    B = int(rng.integers(1, 10))
    kind = case % 4
    if kind == 0:
        L = rng.integers(0, 40, size=B)                    # very short, some empty
    elif kind == 1:
        L = rng.integers(0, 700, size=B)
    elif kind == 2:
        L = np.where(rng.random(B) < 0.3, 0, rng.integers(60, 70, size=B))   # around one tile, or nothing
    else:
        L = rng.integers(900, 1400, size=B) if B <= 3 else rng.integers(100, 300, size=B)
    w = W.make_custom("rand%d" % case, B=B, Hq=Hkv * G, Hkv=Hkv, D=D, T=T, seq_lens=[int(x) for x in L],
                      tree=str(rng.choice(["trie", "uniform", "chain", "star"])), depth=int(rng.integers(2, 12)),
                      branch=int(rng.integers(1, 6)), seed=9100 + case)
    check_attn(R, oracle_mod, w, variants=(0,))


@pytest.mark.parametrize("rows", [128, 256, 257])
@pytest.mark.parametrize("T,Hq", [(64, 16), (128, 16), (100, 32)])
def test_attn_more_than_128_query_rows_both_decompositions(R, oracle_mod, rows, T, Hq, tune):
    # more than 128 query rows per kv head: workgroups of 128 rows (several row chunks per key range) and of
    # 256 rows (eight wavefronts of 32 rows, or, "257", four of 64) must agree with the oracle; the library
    # picks between them by problem size
    tune(R.TUNE_ATTN_WIDE, 1 if rows == 257 else 0)
    rows = min(rows, 256)
    tune(R.TUNE_ATTN_ROWS, rows)
    w = W.make_custom("rows%d_T%d" % (rows, T), B=3, Hq=Hq, Hkv=4, D=128, T=T, seq_lens=[700, 0, 131], tree="trie",
                      depth=7, seed=407)
    check_attn(R, oracle_mod, w, variants=(0,))


@pytest.mark.parametrize("T,Hq,D,lens", [(16, 8, 128, [0, 1, 15, 16, 200]), (32, 32, 128, [333, 1024, 77]),
                                         (64, 16, 128, [500, 31]), (128, 16, 128, [260]), (100, 32, 128, [64, 129]),
                                         (16, 8, 64, [5, 700]), (1, 8, 128, [40, 0])])
def test_attn_tree_rows_in_the_cache(R, oracle_mod, T, Hq, D, lens):
    check_attn_tree_rows_in_the_cache(R, oracle_mod, T, Hq, D, lens, variants=(0, 1))


@pytest.mark.parametrize("T,Hq,D,lens", [(64, 16, 128, [500, 31]), (128, 16, 128, [260, 1500]), (100, 32, 128, [64, 129]),
                                         (128, 8, 64, [300, 5, 0]), (33, 32, 128, [15])])
@pytest.mark.parametrize("wide", [0, 1])
def test_attn_tree_rows_in_the_cache_with_256_row_workgroups(R, oracle_mod, T, Hq, D, lens, wide, tune):
    # the planner picks 256-row workgroups only for large problems; forced here so that their copy loop
    # (which fetches tree tiles two tiles ahead) meets tree tiles that have to be gathered from the cache;
    # both 256-row kernels (eight wavefronts of 32 rows, four of 64)
    tune(R.TUNE_ATTN_ROWS, 256)
    tune(R.TUNE_ATTN_WIDE, wide)
    check_attn_tree_rows_in_the_cache(R, oracle_mod, T, Hq, D, lens, variants=(0,))


def check_attn_tree_rows_in_the_cache(R, oracle_mod, T, Hq, D, lens, variants):
    # the in-cache layout: no tree tensors, node n of sequence b sits at cache position L_b + n (any alignment
    # to the 16-position pages); the result must be what the oracle gives for the separate-tensor layout
    import torch
    print("in-cache attn: T", T, "Hq", Hq, "D", D, "lens", lens, "variants", variants, flush=True)
    w = W.make_custom("incache_T%d" % T, B=len(lens), Hq=Hq, Hkv=4, D=D, T=T, seq_lens=lens, tree="trie", depth=6,
                      seed=408 + T)
    ref, ref_lse = oracle_mod.tree_attn(w.q, w.k_tree, w.v_tree, w.k_cache, w.v_cache, w.page_table, w.seq_lens,
                                        w.parents)
    kc, vc, table = W.place_tree_in_cache(w, seed=5)
    dw = R.to_device(w)
    bf16 = lambda a: torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    dims = R.make_dims(w.B, w.T, w.Hq, w.Hkv, w.D, table.shape[1], w.max_path, kc.shape[0])
    bound = int(max(lens))
    ws = torch.empty(max(R.reader_workspace_bytes(dims, bound), 256), dtype=torch.uint8, device="cuda")
    for variant in variants:
        dims.variant = variant
        dw.out.fill_(float("nan"))
        dw.status.zero_()
        R.reader_tree_attn(dims, dw.q, None, None, bf16(kc), bf16(vc), torch.from_numpy(table).cuda(), dw.seq_lens,
                           dw.parents, dw.out, dw.lse, bound, ws, dw.status)
        torch.cuda.synchronize()
        assert int(dw.status.item()) == 0
        assert_close(bf16_to_np(dw.out), ref, what="in-cache variant %d" % variant)
        assert_close(dw.lse.cpu().numpy().astype(np.float64), ref_lse, what="in-cache lse variant %d" % variant)
    # one tree tensor without the other, or a page table too short for the tree rows, is refused
    with pytest.raises(R.ReaderError):
        R.reader_tree_attn(dims, dw.q, dw.k_tree, None, bf16(kc), bf16(vc), torch.from_numpy(table).cuda(), dw.seq_lens,
                           dw.parents, dw.out, dw.lse, bound, ws, dw.status)
    with pytest.raises(R.ReaderError):
        R.reader_tree_attn(dims, dw.q, None, None, bf16(kc), bf16(vc), torch.from_numpy(table).cuda(), dw.seq_lens,
                           dw.parents, dw.out, dw.lse, table.shape[1] * 16, ws, dw.status)


def test_attn_custom_scale_and_peaked_scores(R, oracle_mod):
    w = W.make_custom("peaked", B=1, Hq=8, Hkv=2, D=128, T=16, seq_lens=[700], tree="trie", depth=5,
                      k_outlier_frac=0.05, seed=402)
    check_attn(R, oracle_mod, w)
    check_attn(R, oracle_mod, w, sm_scale=0.2)


def test_attn_max_seq_len_bound_may_be_loose(R, oracle_mod):
    import torch
    w = W.make_custom("loose", B=2, Hq=8, Hkv=2, D=128, T=12, seq_lens=[100, 333], seed=403)
    ref, _ = oracle_mod.tree_attn(w.q, w.k_tree, w.v_tree, w.k_cache, w.v_cache, w.page_table, w.seq_lens, w.parents)
    dw = R.to_device(w)
    bound = w.max_pages * 16
    ws = torch.empty(R.reader_workspace_bytes(dw.dims, bound), dtype=torch.uint8, device="cuda")
    R.reader_tree_attn(dw.dims, dw.q, dw.k_tree, dw.v_tree, dw.k_cache, dw.v_cache, dw.page_table,
                       dw.seq_lens, dw.parents, dw.out, None, bound, ws, dw.status)
    torch.cuda.synchronize()
    assert_close(bf16_to_np(dw.out), ref, what="loose bound")


# ------------------------------------------------------------------ attention, full size, sampled rows

def stratified_rows(w, rng):
    """Output rows (b, hq, node) to check at full size: for every (sequence, kv head) pair one random row in each
    chunk of 128 query rows (a query row is node * G + grouped head; workgroups carry 128 or 256 of them), and
    the pair's first and last query row.  Pairs that are cut between workgroups, second row chunks and merged
    pairs are all hit this way, whatever the launch plan is."""
    G = w.Hq // w.Hkv
    M = w.T * G
    rows = []
    for b in range(w.B):
        for hkv in range(w.Hkv):
            picks = {0, M - 1}
            for lo in range(0, M, 128):
                picks.add(int(rng.integers(lo, min(lo + 128, M))))
            for m in sorted(picks):
                rows.append((b, hkv * G + m % G, m // G))
    return np.asarray(rows, dtype=np.int32)


def check_sampled_rows(oracle_mod, w, out, lse, rows, what):
    ref, ref_lse = oracle_mod.tree_attn_rows(w.q, w.k_tree, w.v_tree, w.k_cache, w.v_cache, w.page_table,
                                             w.seq_lens, w.parents, rows)
    got = np.stack([out[b, i, hq] for b, hq, i in rows])
    got_lse = np.asarray([lse[b, hq, i] for b, hq, i in rows])
    assert_close(got, ref, what=what + " sampled rows")
    assert_close(got_lse, ref_lse, what=what + " sampled lse")
    assert np.isfinite(out).all()


@pytest.mark.parametrize("index", [2, 3, 4])
def test_attn_full_size_sampled_rows(R, oracle_mod, index):
    # the launch configuration the benchmark times; the oracle checks a stratified sample of output rows
    w = W.make_config(index)
    out, lse = run_attn(R, w)
    rows = stratified_rows(w, np.random.Generator(np.random.PCG64(900 + index)))
    print("full-size attn:", w.name, len(rows), "rows", flush=True)
    check_sampled_rows(oracle_mod, w, out, lse, rows, w.name)


@pytest.mark.parametrize("wide", [0, 1])
@pytest.mark.parametrize("index", [3, 4])
def test_attn_full_size_sampled_rows_either_256_row_kernel(R, oracle_mod, index, wide, tune):
    # both 256-row kernels by name at the two matrix-bound presets: eight wavefronts of 32 rows (moving softmax
    # reference), and four of 64 rows (one per SIMD, fixed reference, second pass for workgroups whose scores
    # outgrew it), whichever of them the planner would take
    tune(R.TUNE_ATTN_WIDE, wide)
    w = W.make_config(index)
    out, lse = run_attn(R, w)
    rows = stratified_rows(w, np.random.Generator(np.random.PCG64(930 + index)))
    print("full-size attn, 256-row kernel", wide, ":", w.name, len(rows), "rows", flush=True)
    check_sampled_rows(oracle_mod, w, out, lse, rows, w.name + " kernel %d" % wide)


@pytest.mark.parametrize("wide", [0, 1])
@pytest.mark.parametrize("case", range(8))
def test_attn_seeded_random_shapes_either_256_row_kernel(R, oracle_mod, case, wide, tune):
    tune(R.TUNE_ATTN_ROWS, 256)
    tune(R.TUNE_ATTN_WIDE, wide)
    rng = np.random.Generator(np.random.PCG64(9300 + case))
    D = int(rng.choice([64, 128]))
    Hkv, G = int(rng.choice([1, 2, 4])), int(rng.choice([4, 8, 16]))
    T = int(rng.choice([16, 33, 64, 100, 128]))
    B = int(rng.integers(1, 6))
    L = [int(x) for x in (rng.integers(0, 700, size=B) if case % 2 else rng.integers(900, 2600, size=B))]
    w = W.make_custom("randwide%d" % case, B=B, Hq=Hkv * G, Hkv=Hkv, D=D, T=T, seq_lens=L,
                      tree=str(rng.choice(["trie", "uniform", "chain", "star"])), depth=int(rng.integers(2, 12)),
                      branch=int(rng.integers(1, 6)), k_outlier_frac=0.05 if case % 3 == 0 else 0.0, seed=9400 + case)
    check_attn(R, oracle_mod, w, variants=(0,))


def test_attn_scores_that_outgrow_the_fixed_reference_are_computed_again(R, oracle_mod, tune):
    # The four-wavefront kernel fixes a row's softmax reference at the first tile of a segment.  Keys late
    # in the context that score 2^100 and more above everything before them cannot be held by that; the
    # workgroups concerned flag it and the second pass (moving reference) has to produce the right rows.
    tune(R.TUNE_ATTN_ROWS, 256)
    tune(R.TUNE_ATTN_WIDE, 1)
    w = W.make_custom("outgrow", B=2, Hq=16, Hkv=2, D=128, T=40, seq_lens=[1500, 900], tree="trie", depth=6, seed=470)
    # one late key per sequence aligned with every query of the first kv head: q . k large and positive
    f32 = W.bf16_bits_to_f32
    for b, pos in ((0, 1400), (1, 700)):
        page, slot = int(w.page_table[b, pos // 16]), pos % 16
        w.q[b, :, :8, :] = W.to_bf16_bits(np.abs(f32(w.q[b, :, :8, :])) * 4.0 + 1.0)
        w.k_cache[page, 0, slot, :] = W.to_bf16_bits(np.full(w.D, 9.0, dtype=np.float32))
    check_attn(R, oracle_mod, w, variants=(0,))


def test_attn_full_size_head_dim_64_with_256_row_workgroups(R, oracle_mod):
    # D = 64 on a problem large enough for the planner to pick 256-row workgroups by itself (512 query rows per
    # kv head, > 10000 workgroup-tiles), ragged lengths, stratified sample of rows
    rng = np.random.Generator(np.random.PCG64(77))
    L = [int(x) for x in rng.integers(3000, 5000, size=16)]
    w = W.make_custom("d64_rows256", B=16, Hq=32, Hkv=4, D=64, T=64, seq_lens=L, tree="trie", depth=8, branch=4, seed=460)
    print("full-size attn:", w.name, "L", L, flush=True)
    plan = R.reader_attn_plan(R.make_dims(w.B, w.T, w.Hq, w.Hkv, w.D, w.page_table.shape[1], w.max_path, w.k_cache.shape[0]),
                              int(max(L)))
    assert plan["rows_per_workgroup"] == 256, plan
    out, lse = run_attn(R, w)
    check_sampled_rows(oracle_mod, w, out, lse, stratified_rows(w, rng), w.name)


# ------------------------------------------------------------------ device-side input errors

def test_malformed_tree_and_bad_page_set_status_without_faulting(R, oracle_mod):
    w = W.make_custom("status", B=2, Hq=4, Hkv=2, D=128, T=10, seq_lens=[40, 90], tree="uniform", depth=4, seed=404)
    w.parents[1, 5] = 7                    # parent after child
    for variant in (0, 1):
        run_attn(R, w, variant=variant, want_status=R.STATUS_BAD_TREE)
    w = W.make_custom("status2", B=2, Hq=4, Hkv=2, D=128, T=10, seq_lens=[40, 90], tree="uniform", depth=4, seed=405)
    w.page_table[1, 2] = w.num_pages + 5   # outside the pool
    for variant in (0, 1):
        out, _ = run_attn(R, w, variant=variant, want_status=R.STATUS_BAD_PAGE)
        ref, _ = oracle_mod.tree_attn(w.q[:1], w.k_tree[:1], w.v_tree[:1], w.k_cache, w.v_cache,
                                      w.page_table[:1], w.seq_lens[:1], w.parents[:1])
        assert_close(out[:1], ref, what="sequence next to the bad one")
    # the keys behind a bad page id are skipped: with the bad id in the last (partial) page of a sequence
    # the result is that of the sequence cut in front of that page; with the bad id in the middle the two
    # device implementations must agree
    w = W.make_custom("status3", B=2, Hq=4, Hkv=2, D=128, T=10, seq_lens=[40, 90], tree="uniform", depth=4, seed=406)
    w.page_table[1, 5] = -3
    cut = w.seq_lens.copy()
    cut[1] = 80
    ref, ref_lse = oracle_mod.tree_attn(w.q, w.k_tree, w.v_tree, w.k_cache, w.v_cache, w.page_table, cut, w.parents)
    for variant in (0, 1):
        out, lse = run_attn(R, w, variant=variant, want_status=R.STATUS_BAD_PAGE)
        assert_close(out, ref, what="bad last page, variant %d" % variant)
        assert_close(lse, ref_lse, what="bad last page lse, variant %d" % variant)
    w = W.make_custom("status4", B=2, Hq=8, Hkv=2, D=128, T=40, seq_lens=[300, 200], tree="trie", depth=5, seed=407)
    w.page_table[0, 0] = w.num_pages          # first quarter of the first tile
    w.page_table[0, 9] = -1
    w.page_table[1, 4] = w.num_pages + 1      # a whole tile of sequence 1 (pages 4..7)
    w.page_table[1, 5] = w.page_table[1, 6] = w.page_table[1, 7] = -1
    outs = [run_attn(R, w, variant=v, want_status=R.STATUS_BAD_PAGE) for v in (0, 1)]
    assert np.isfinite(outs[0][0]).all() and np.isfinite(outs[0][1]).all()
    assert_close(outs[0][0], outs[1][0], what="bad pages in the middle: matrix-core kernel against the scalar one")
    assert_close(outs[0][1], outs[1][1], what="bad pages in the middle, lse")


# ------------------------------------------------------------------ acceptance

def run_accept(R, w):
    import torch
    dw = R.to_device(w)
    dw.path.fill_(-7)
    R.reader_accept_path(dw.dims, dw.draft_tokens, dw.target_tokens, dw.parents, dw.accept_len, dw.path,
                         dw.bonus, dw.status)
    torch.cuda.synchronize()
    return dw.accept_len.cpu().numpy(), dw.path.cpu().numpy(), dw.bonus.cpu().numpy(), int(dw.status.item())


@pytest.mark.parametrize("index", [0, 1, 2, 3, 4])
def test_accept_presets_bit_exact(R, oracle_mod, index):
    w = W.make_config(index, length_scale=0.01)          # acceptance does not look at the prefix
    al, path, bonus, status = run_accept(R, w)
    ral, rpath, rbonus = oracle_mod.accept_path(w.draft_tokens, w.target_tokens, w.parents, w.max_path)
    assert status == 0
    assert np.array_equal(al, ral) and np.array_equal(path, rpath) and np.array_equal(bonus, rbonus)


@pytest.mark.parametrize("T", [1, 2, 63, 64, 65, 128])
def test_accept_random_trees_with_duplicate_siblings(R, oracle_mod, T):
    rng = np.random.Generator(np.random.PCG64(500 + T))
    B = 64
    w = W.make_custom("acc_T%d" % T, B=B, Hq=1, Hkv=1, D=64, T=T, seq_lens=[0] * B, tree="uniform",
                      depth=min(T - 1, 9) if T > 1 else 0, seed=501 + T, max_path=min(T, 10))
    w.draft_tokens[:] = rng.integers(0, 3, size=(B, T))     # tiny vocabulary: ties and duplicates
    w.target_tokens[:] = rng.integers(0, 3, size=(B, T))
    w.target_tokens[0] = w.draft_tokens[0, 0] = 1            # one sequence where everything matches
    w.draft_tokens[0] = 1
    al, path, bonus, status = run_accept(R, w)
    ral, rpath, rbonus = oracle_mod.accept_path(w.draft_tokens, w.target_tokens, w.parents, w.max_path)
    assert status == 0 and al.max() >= min(T - 1, 1)
    assert np.array_equal(al, ral) and np.array_equal(path, rpath) and np.array_equal(bonus, rbonus)


def test_accept_path_longer_than_max_path_is_cut_and_flagged(R):
    w = W.make_custom("cut", B=1, Hq=1, Hkv=1, D=64, T=8, seq_lens=[0], tree="chain", seed=7, max_path=4)
    w.draft_tokens[:] = 5
    w.target_tokens[:] = 5
    w.target_tokens[0, 3] = 9
    w.draft_tokens[0, 4] = 9                 # still a match: all 7 drafted nodes are acceptable
    al, path, bonus, status = run_accept(R, w)
    assert status == R.STATUS_BAD_PATH and al[0] == 3 and path[0].tolist() == [0, 1, 2, 3] and bonus[0] == 9


# ------------------------------------------------------------------ compaction and the whole step

def run_step(R, w, with_attn=True):
    """attention -> acceptance -> compaction on one stream, as the benchmark does."""
    import torch
    dw = R.to_device(w)
    if with_attn:
        R.reader_tree_attn(dw.dims, dw.q, dw.k_tree, dw.v_tree, dw.k_cache, dw.v_cache, dw.page_table,
                           dw.seq_lens, dw.parents, dw.out, dw.lse, dw.max_seq_len, dw.workspace, dw.status)
    R.reader_accept_path(dw.dims, dw.draft_tokens, dw.target_tokens, dw.parents, dw.accept_len, dw.path,
                         dw.bonus, dw.status)
    R.reader_kv_compact(dw.dims, dw.k_tree, dw.v_tree, dw.path, dw.accept_len, dw.k_cache, dw.v_cache,
                        dw.page_table, dw.seq_lens, dw.status)
    torch.cuda.synchronize()
    return dw


def oracle_step(oracle_mod, w):
    kc, vc, sl = w.k_cache.copy(), w.v_cache.copy(), w.seq_lens.copy()
    al, path, bonus = oracle_mod.accept_path(w.draft_tokens, w.target_tokens, w.parents, w.max_path)
    oracle_mod.kv_compact(w.k_tree, w.v_tree, path, al, kc, vc, w.page_table, sl)
    return al, path, bonus, kc, vc, sl


def cache_bits(t):
    import torch
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("index,scale", [(0, 1.0), (1, 0.1), (2, 0.1), (3, 0.01), (4, 0.02)])
def test_compact_presets_bit_exact(R, oracle_mod, index, scale):
    w = W.make_config(index, length_scale=scale)
    dw = run_step(R, w, with_attn=False)
    al, path, bonus, kc, vc, sl = oracle_step(oracle_mod, w)
    assert int(dw.status.item()) == 0
    assert np.array_equal(dw.seq_lens.cpu().numpy(), sl)
    assert np.array_equal(cache_bits(dw.k_cache), kc) and np.array_equal(cache_bits(dw.v_cache), vc)


def test_compact_page_boundaries_and_long_paths(R, oracle_mod):
    w = W.make_custom("compact_edges", B=8, Hq=4, Hkv=4, D=64, T=40, seq_lens=[0, 1, 15, 16, 17, 31, 32, 200],
                      tree="chain", vocab=2, p_match=0.97, seed=601)
    dw = run_step(R, w, with_attn=False)
    al, path, bonus, kc, vc, sl = oracle_step(oracle_mod, w)
    assert al.max() >= 17                                   # spans more than one whole page
    assert int(dw.status.item()) == 0 and np.array_equal(dw.seq_lens.cpu().numpy(), sl)
    assert np.array_equal(cache_bits(dw.k_cache), kc) and np.array_equal(cache_bits(dw.v_cache), vc)


def test_compact_refuses_bad_items_and_leaves_the_sequence_alone(R):
    import torch
    w = W.make_custom("compact_bad", B=3, Hq=2, Hkv=2, D=64, T=6, seq_lens=[20, 30, 40], tree="chain", seed=602)
    dw = R.to_device(w)
    dw.accept_len.copy_(torch.tensor([1, 9, 1], dtype=torch.int32))           # 9 > max_path - 1
    dw.path.copy_(torch.tensor([[0, 1, -1, -1, -1, -1], [0, 1, 2, 3, 4, 5], [0, 77, -1, -1, -1, -1]], dtype=torch.int32))
    R.reader_kv_compact(dw.dims, dw.k_tree, dw.v_tree, dw.path, dw.accept_len, dw.k_cache, dw.v_cache,
                        dw.page_table, dw.seq_lens, dw.status)
    torch.cuda.synchronize()
    assert int(dw.status.item()) == R.STATUS_BAD_PATH
    assert dw.seq_lens.cpu().tolist() == [22, 30, 40]
    k = cache_bits(dw.k_cache)
    changed = (k != w.k_cache).any(axis=(1, 3)).sum()
    assert changed == 2


@pytest.mark.parametrize("index,scale", [(0, 1.0), (2, 0.1)])
def test_whole_step_then_next_step_attention(R, oracle_mod, index, scale):
    # One full step, then attention again over the grown cache: what a decoding loop does.
    import torch
    w = W.make_config(index, length_scale=scale)
    dw = run_step(R, w)
    al, path, bonus, kc, vc, sl = oracle_step(oracle_mod, w)
    assert np.array_equal(dw.accept_len.cpu().numpy(), al) and np.array_equal(dw.bonus.cpu().numpy(), bonus)
    assert np.array_equal(dw.seq_lens.cpu().numpy(), sl)
    assert np.array_equal(cache_bits(dw.k_cache), kc) and np.array_equal(cache_bits(dw.v_cache), vc)
    # second step: same tree tensors over the grown prefix
    ref, _ = oracle_mod.tree_attn(w.q, w.k_tree, w.v_tree, kc, vc, w.page_table, sl, w.parents)
    R.reader_tree_attn(dw.dims, dw.q, dw.k_tree, dw.v_tree, dw.k_cache, dw.v_cache, dw.page_table,
                       dw.seq_lens, dw.parents, dw.out, dw.lse, int(sl.max()), dw.workspace, dw.status)
    torch.cuda.synchronize()
    assert_close(bf16_to_np(dw.out), ref, what="second step")


# ---------------------------------------------------------------- fused step (two launches)

def random_step_workload(case):
    rng = np.random.Generator(np.random.PCG64(9500 + case))
    Hkv, G = int(rng.choice([1, 2, 4])), int(rng.choice([1, 2, 4, 8]))
    B, T = int(rng.integers(1, 8)), int(rng.choice([1, 5, 16, 40, 64, 128]))
    L = [int(x) for x in rng.integers(0, 400, size=B)]
    return W.make_custom("randstep%d" % case, B=B, Hq=Hkv * G, Hkv=Hkv, D=int(rng.choice([64, 128])), T=T, seq_lens=L,
                         tree=str(rng.choice(["trie", "uniform", "chain"])), depth=int(rng.integers(2, 14)),
                         branch=int(rng.integers(1, 5)), vocab=int(rng.choice([3, 50])), p_match=float(rng.uniform(0.3, 0.95)),
                         seed=9600 + case)


@pytest.mark.parametrize("index,scale", [(0, 1.0), (1, 0.1), (2, 0.1), (2, 1.0), (3, 0.02), (4, 0.05)] +
                         [(-1 - c, 1.0) for c in range(10)])
def test_verify_step_equals_the_three_calls_and_the_oracle(R, oracle_mod, index, scale):
    import torch
    # the presets, and a seeded sweep of random shapes (negative index)
    w = W.make_config(index, length_scale=scale) if index >= 0 else random_step_workload(-1 - index)
    # the three entry points, one after the other
    dw3 = run_step(R, w)
    # the fused entry point on a fresh upload of the same workload
    dw = R.to_device(w)
    R.reader_verify_step(dw.dims, dw.q, dw.k_tree, dw.v_tree, dw.k_cache, dw.v_cache, dw.page_table, dw.seq_lens,
                         dw.parents, dw.draft_tokens, dw.target_tokens, dw.out, dw.lse, dw.accept_len, dw.path,
                         dw.bonus, dw.max_seq_len, dw.workspace, dw.status)
    torch.cuda.synchronize()
    assert int(dw.status.item()) == 0
    for name in ("out", "lse", "accept_len", "path", "bonus", "seq_lens"):
        a, b = getattr(dw, name), getattr(dw3, name)
        assert torch.equal(a, b), "fused step differs from the three calls in " + name
    for name in ("k_cache", "v_cache"):   # bit patterns: unused slots hold NaN canaries
        assert np.array_equal(cache_bits(getattr(dw, name)), cache_bits(getattr(dw3, name))), name
    # and against the oracle
    ref, _ = oracle_mod.tree_attn(w.q, w.k_tree, w.v_tree, w.k_cache, w.v_cache, w.page_table, w.seq_lens, w.parents)
    assert_close(bf16_to_np(dw.out), ref, what="fused step attention")
    al, path, bonus, kc, vc, sl = oracle_step(oracle_mod, w)
    assert np.array_equal(dw.accept_len.cpu().numpy(), al) and np.array_equal(dw.bonus.cpu().numpy(), bonus)
    assert np.array_equal(dw.path.cpu().numpy(), path)
    assert np.array_equal(dw.seq_lens.cpu().numpy(), sl)
    assert np.array_equal(cache_bits(dw.k_cache), kc) and np.array_equal(cache_bits(dw.v_cache), vc)


@pytest.mark.parametrize("T,Hq,D,lens", [(16, 8, 128, [0, 1, 15, 16, 200]), (40, 16, 64, [333, 1024, 77, 5]),
                                         (128, 16, 128, [50, 700])])
def test_verify_step_with_the_tree_rows_in_the_cache(R, oracle_mod, T, Hq, D, lens):
    check_verify_step_with_the_tree_rows_in_the_cache(R, oracle_mod, T, Hq, D, lens)


@pytest.mark.parametrize("T,Hq,D,lens", [(64, 16, 128, [333, 1024, 77]), (128, 16, 64, [50, 700])])
def test_verify_step_with_the_tree_rows_in_the_cache_and_256_row_workgroups(R, oracle_mod, T, Hq, D, lens, tune):
    tune(R.TUNE_ATTN_ROWS, 256)
    check_verify_step_with_the_tree_rows_in_the_cache(R, oracle_mod, T, Hq, D, lens)


def check_verify_step_with_the_tree_rows_in_the_cache(R, oracle_mod, T, Hq, D, lens):
    # in-cache layout, one layer: attention over the cache, acceptance, the accepted rows move in place
    import torch
    print("in-cache step: T", T, "Hq", Hq, "D", D, "lens", lens, flush=True)
    w = W.make_custom("incache_step_T%d" % T, B=len(lens), Hq=Hq, Hkv=4, D=D, T=T, seq_lens=lens, tree="trie", depth=7,
                      p_match=0.8, seed=418 + T)
    ref, ref_lse = oracle_mod.tree_attn(w.q, w.k_tree, w.v_tree, w.k_cache, w.v_cache, w.page_table, w.seq_lens,
                                        w.parents)
    kc, vc, table = W.place_tree_in_cache(w, seed=6)
    al, path, bonus = oracle_mod.accept_path(w.draft_tokens, w.target_tokens, w.parents, w.max_path)
    kc_ref, vc_ref, sl_ref = kc[None].copy(), vc[None].copy(), w.seq_lens.copy()
    oracle_mod.kv_compact_layers(kc_ref, vc_ref, path, al, table, sl_ref)
    assert al.max() >= 1   # something moves

    dw = R.to_device(w)
    bf16 = lambda a: torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    dims = R.make_dims(w.B, w.T, w.Hq, w.Hkv, w.D, table.shape[1], w.max_path, kc.shape[0])
    bound = int(max(lens))
    ws = torch.empty(max(R.reader_workspace_bytes(dims, bound), 256), dtype=torch.uint8, device="cuda")
    d_kc, d_vc, d_table = bf16(kc), bf16(vc), torch.from_numpy(table).cuda()
    dw.out.fill_(float("nan"))
    R.reader_verify_step(dims, dw.q, None, None, d_kc, d_vc, d_table, dw.seq_lens, dw.parents, dw.draft_tokens,
                         dw.target_tokens, dw.out, dw.lse, dw.accept_len, dw.path, dw.bonus, bound, ws, dw.status)
    torch.cuda.synchronize()
    assert int(dw.status.item()) == 0
    assert_close(bf16_to_np(dw.out), ref, what="in-cache step attention")
    assert_close(dw.lse.cpu().numpy().astype(np.float64), ref_lse, what="in-cache step lse")
    assert np.array_equal(dw.accept_len.cpu().numpy(), al) and np.array_equal(dw.bonus.cpu().numpy(), bonus)
    assert np.array_equal(dw.path.cpu().numpy(), path)
    assert np.array_equal(dw.seq_lens.cpu().numpy(), sl_ref)
    assert np.array_equal(cache_bits(d_kc), kc_ref[0]) and np.array_equal(cache_bits(d_vc), vc_ref[0])
    # one tree tensor without the other is refused, nothing changes
    with pytest.raises(R.ReaderError):
        R.reader_verify_step(dims, dw.q, dw.k_tree, None, d_kc, d_vc, d_table, dw.seq_lens, dw.parents,
                             dw.draft_tokens, dw.target_tokens, dw.out, dw.lse, dw.accept_len, dw.path, dw.bonus,
                             bound, ws, dw.status)
    torch.cuda.synchronize()
    assert np.array_equal(dw.seq_lens.cpu().numpy(), sl_ref)


@pytest.mark.parametrize("index", [3, 4])
def test_verify_step_full_size_sampled_rows(R, oracle_mod, index):
    # the fused step exactly as the benchmark launches it, at the presets' full sizes: a stratified sample of attention
    # rows against the oracle; acceptance, appended rows and new lengths bit for bit (the oracle does those at any size)
    import torch
    w = W.make_config(index)
    print("full-size fused step:", w.name, flush=True)
    dw = R.to_device(w)
    R.reader_verify_step(dw.dims, dw.q, dw.k_tree, dw.v_tree, dw.k_cache, dw.v_cache, dw.page_table, dw.seq_lens,
                         dw.parents, dw.draft_tokens, dw.target_tokens, dw.out, dw.lse, dw.accept_len, dw.path,
                         dw.bonus, dw.max_seq_len, dw.workspace, dw.status)
    torch.cuda.synchronize()
    assert int(dw.status.item()) == 0
    out, lse = bf16_to_np(dw.out), dw.lse.cpu().numpy().astype(np.float64)
    rows = stratified_rows(w, np.random.Generator(np.random.PCG64(950 + index)))
    check_sampled_rows(oracle_mod, w, out, lse, rows, w.name + " fused step")
    al, path, bonus, kc, vc, sl = oracle_step(oracle_mod, w)
    assert np.array_equal(dw.accept_len.cpu().numpy(), al) and np.array_equal(dw.bonus.cpu().numpy(), bonus)
    assert np.array_equal(dw.path.cpu().numpy(), path) and np.array_equal(dw.seq_lens.cpu().numpy(), sl)
    assert np.array_equal(cache_bits(dw.k_cache), kc) and np.array_equal(cache_bits(dw.v_cache), vc)


def test_verify_step_full_size_with_the_tree_rows_in_the_cache(R, oracle_mod):
    # the batched ragged preset at full size in the in-cache layout: the fused step (attention over the cache,
    # acceptance, in-place move of the accepted rows); stratified attention rows against the oracle, everything
    # else bit for bit
    import torch
    w = W.make_config(2)
    print("full-size in-cache fused step:", w.name, flush=True)
    kc, vc, table = W.place_tree_in_cache(w, seed=11)
    al, path, bonus = oracle_mod.accept_path(w.draft_tokens, w.target_tokens, w.parents, w.max_path)
    kc_ref, vc_ref, sl_ref = kc[None].copy(), vc[None].copy(), w.seq_lens.copy()
    oracle_mod.kv_compact_layers(kc_ref, vc_ref, path, al, table, sl_ref)
    dw = R.to_device(w)
    bf16 = lambda a: torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    dims = R.make_dims(w.B, w.T, w.Hq, w.Hkv, w.D, table.shape[1], w.max_path, kc.shape[0])
    bound = int(w.seq_lens.max())
    ws = torch.empty(max(R.reader_workspace_bytes(dims, bound), 256), dtype=torch.uint8, device="cuda")
    d_kc, d_vc, d_table = bf16(kc), bf16(vc), torch.from_numpy(table).cuda()
    dw.out.fill_(float("nan"))
    R.reader_verify_step(dims, dw.q, None, None, d_kc, d_vc, d_table, dw.seq_lens, dw.parents, dw.draft_tokens,
                         dw.target_tokens, dw.out, dw.lse, dw.accept_len, dw.path, dw.bonus, bound, ws, dw.status)
    torch.cuda.synchronize()
    assert int(dw.status.item()) == 0
    out, lse = bf16_to_np(dw.out), dw.lse.cpu().numpy().astype(np.float64)
    check_sampled_rows(oracle_mod, w, out, lse, stratified_rows(w, np.random.Generator(np.random.PCG64(961))),
                       w.name + " in-cache fused step")
    assert np.array_equal(dw.accept_len.cpu().numpy(), al) and np.array_equal(dw.bonus.cpu().numpy(), bonus)
    assert np.array_equal(dw.path.cpu().numpy(), path) and np.array_equal(dw.seq_lens.cpu().numpy(), sl_ref)
    assert np.array_equal(cache_bits(d_kc), kc_ref[0]) and np.array_equal(cache_bits(d_vc), vc_ref[0])


def test_two_host_threads_on_their_own_streams(R, oracle_mod):
    # the entry points keep no state between calls: two host threads, each with its own stream, workspace and
    # outputs, run whole steps of different shapes at the same time and get what a single thread gets
    import threading
    import torch
    shapes = [W.make_custom("thr_a", B=3, Hq=8, Hkv=2, D=128, T=24, seq_lens=[700, 65, 1300], tree="trie", depth=6,
                            seed=431),
              W.make_custom("thr_b", B=2, Hq=16, Hkv=2, D=64, T=64, seq_lens=[2000, 900], tree="uniform", depth=5,
                            seed=432)]
    single = [run_step(R, w) for w in shapes]
    results, errors = [None, None], []

    def work(k):
        try:
            torch.cuda.set_device(0)
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                for _ in range(20):
                    dw = R.to_device(shapes[k])
                    R.reader_verify_step(dw.dims, dw.q, dw.k_tree, dw.v_tree, dw.k_cache, dw.v_cache, dw.page_table,
                                         dw.seq_lens, dw.parents, dw.draft_tokens, dw.target_tokens, dw.out, dw.lse,
                                         dw.accept_len, dw.path, dw.bonus, dw.max_seq_len, dw.workspace, dw.status)
                    stream.synchronize()
                    results[k] = dw
        except Exception as e:      # reported by the main thread
            errors.append(e)

    threads = [threading.Thread(target=work, args=(k,)) for k in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for k in range(2):
        assert int(results[k].status.item()) == 0
        for name in ("out", "lse", "accept_len", "path", "bonus", "seq_lens"):
            assert torch.equal(getattr(results[k], name), getattr(single[k], name)), (k, name)
        for name in ("k_cache", "v_cache"):
            assert np.array_equal(cache_bits(getattr(results[k], name)), cache_bits(getattr(single[k], name))), (k, name)


def test_status_word_is_optional(R, oracle_mod):
    # every device entry point takes status = NULL: same results, and a malformed input is still skipped, not followed
    import torch
    w = W.make_custom("nostatus", B=3, Hq=8, Hkv=2, D=128, T=12, seq_lens=[40, 90, 300], tree="uniform", depth=4, seed=451)
    ref = run_step(R, w)
    dw = R.to_device(w)
    R.reader_verify_step(dw.dims, dw.q, dw.k_tree, dw.v_tree, dw.k_cache, dw.v_cache, dw.page_table, dw.seq_lens,
                         dw.parents, dw.draft_tokens, dw.target_tokens, dw.out, dw.lse, dw.accept_len, dw.path,
                         dw.bonus, dw.max_seq_len, dw.workspace, None)
    torch.cuda.synchronize()
    for name in ("out", "accept_len", "path", "bonus", "seq_lens"):
        assert torch.equal(getattr(dw, name), getattr(ref, name)), name
    # a page id outside the pool and a parent after its child, no status word: the other sequences come out right
    w.page_table[1, 2] = w.num_pages + 5
    w.parents[2, 5] = 7
    good, _ = oracle_mod.tree_attn(w.q[:1], w.k_tree[:1], w.v_tree[:1], w.k_cache, w.v_cache, w.page_table[:1],
                                   w.seq_lens[:1], w.parents[:1])
    for variant in (0, 1):
        dw = R.to_device(w)
        dw.dims.variant = variant
        R.reader_tree_attn(dw.dims, dw.q, dw.k_tree, dw.v_tree, dw.k_cache, dw.v_cache, dw.page_table, dw.seq_lens,
                           dw.parents, dw.out, None, dw.max_seq_len, dw.workspace, None)
        torch.cuda.synchronize()
        assert_close(bf16_to_np(dw.out)[:1], good, what="sequence next to the bad ones, no status word")
    dw = R.to_device(w)
    R.reader_accept_path(dw.dims, dw.draft_tokens, dw.target_tokens, dw.parents, dw.accept_len, dw.path, dw.bonus, None)
    R.reader_kv_compact(dw.dims, dw.k_tree, dw.v_tree, dw.path, dw.accept_len, dw.k_cache, dw.v_cache, dw.page_table,
                        dw.seq_lens, None)
    torch.cuda.synchronize()
    assert int(dw.seq_lens[1].item()) == int(w.seq_lens[1]) or int(dw.seq_lens[1].item()) == int(w.seq_lens[1]) + int(dw.accept_len[1].item()) + 1


def test_verify_step_rejects_bad_arguments(R):
    import torch
    w = W.make_config(0)
    dw = R.to_device(w)
    with pytest.raises(R.ReaderError):   # workspace too small
        R.reader_verify_step(dw.dims, dw.q, dw.k_tree, dw.v_tree, dw.k_cache, dw.v_cache, dw.page_table, dw.seq_lens,
                             dw.parents, dw.draft_tokens, dw.target_tokens, dw.out, dw.lse, dw.accept_len, dw.path,
                             dw.bonus, dw.max_seq_len, dw.workspace[:256], dw.status)
    torch.cuda.synchronize()
    assert int(dw.status.item()) == 0 and torch.equal(dw.seq_lens.cpu(), torch.from_numpy(w.seq_lens))


@pytest.mark.parametrize("wide", [0, 1])
def test_attn_repeated_launches_are_bit_identical(R, wide, tune):
    # Nothing in a launch depends on timing: the cut of the tile axis, the order in which a pair's parts are merged
    # and the hand-placed instruction order of the four-wavefront kernel (whose matrix results are read without any
    # hazard check by the compiler) give the same bits every time.
    import torch
    tune(R.TUNE_ATTN_WIDE, wide)
    w = W.make_config(3)
    dw = R.to_device(w)
    first = None
    for rep in range(8):
        dw.out.fill_(float("nan"))
        dw.lse.fill_(float("nan"))
        R.reader_tree_attn(dw.dims, dw.q, dw.k_tree, dw.v_tree, dw.k_cache, dw.v_cache, dw.page_table, dw.seq_lens,
                           dw.parents, dw.out, dw.lse, dw.max_seq_len, dw.workspace, dw.status)
        torch.cuda.synchronize()
        got = (dw.out.view(torch.int16).clone(), dw.lse.view(torch.int32).clone())
        if first is None:
            first = got
        else:
            assert torch.equal(got[0], first[0]), "outputs differ at repetition %d" % rep
            assert torch.equal(got[1], first[1]), "lse differs at repetition %d" % rep
    assert int(dw.status.item()) == 0
