"""reader_tree_attn_noalloc (the entry point that allocates nothing: its workspace is part of the
library's device code) against reader_tree_attn, through the C ABI, on a real MI355X.

Same kernels, so the outputs must be equal bit for bit; and within the attention tolerance of the
CPU oracle.  Two calls in a row, the second on a smaller problem: the shared workspace keeps the
first call's records and the second must not be disturbed by them.
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
    binding.load()
    return binding


def both_ways(R, w):
    import torch
    dw = R.to_device(w)
    dw.out.fill_(float("nan"))
    dw.lse.fill_(float("nan"))
    R.reader_tree_attn(dw.dims, dw.q, dw.k_tree, dw.v_tree, dw.k_cache, dw.v_cache, dw.page_table, dw.seq_lens,
                       dw.parents, dw.out, dw.lse, dw.max_seq_len, dw.workspace, dw.status)
    torch.cuda.synchronize()
    out_ws, lse_ws = dw.out.clone(), dw.lse.clone()
    dw.out.fill_(float("nan"))
    dw.lse.fill_(float("nan"))
    R.reader_tree_attn_noalloc(dw.dims, dw.q, dw.k_tree, dw.v_tree, dw.k_cache, dw.v_cache, dw.page_table,
                               dw.seq_lens, dw.parents, dw.out, dw.lse, dw.max_seq_len, dw.status)
    torch.cuda.synchronize()
    assert int(dw.status.item()) == 0
    return (out_ws, lse_ws), (dw.out.clone(), dw.lse.clone())


def test_noalloc_equals_the_workspace_entry_point_twice_in_a_row(R, oracle_mod):
    import torch
    # set-up call (B = 0): looks up the workspace's device address, launches nothing
    R.reader_tree_attn_noalloc(R.make_dims(0, 1, 1, 1, 128, 1, 1, 1), None, None, None, None, None, None, None, None,
                               None, None, 0)
    # first a problem whose pairs are cut between many workgroups (partial records in every slot),
    # then a smaller one with fewer ranges, fewer rows and another head dimension
    big = W.make_custom("noalloc_big", B=6, Hq=32, Hkv=4, D=128, T=48, seq_lens=[2100, 700, 0, 4097, 1300, 65],
                        tree="trie", depth=7, branch=3, seed=4401)
    small = W.make_custom("noalloc_small", B=2, Hq=8, Hkv=2, D=64, T=20, seq_lens=[333, 90], tree="uniform", depth=5,
                          seed=4402)
    for w in (big, small):
        print("no-alloc attention:", w.name, "B", w.B, "T", w.T, "L", w.seq_lens.tolist(), flush=True)
        (out_ws, lse_ws), (out_na, lse_na) = both_ways(R, w)
        assert torch.equal(out_na.view(torch.int16), out_ws.view(torch.int16)), w.name + ": outputs differ"
        assert torch.equal(lse_na, lse_ws), w.name + ": lse differs"
        ref, ref_lse = oracle_mod.tree_attn(w.q, w.k_tree, w.v_tree, w.k_cache, w.v_cache, w.page_table, w.seq_lens,
                                            w.parents)
        assert_close(out_na.float().cpu().numpy().astype(np.float64), ref, what=w.name + " no-alloc out")
        assert_close(lse_na.cpu().numpy().astype(np.float64), ref_lse, what=w.name + " no-alloc lse")


def test_noalloc_refuses_what_does_not_fit(R):
    import torch
    # 2048 query rows per kv head (eight row chunks) in 256 ranges need far more than the built-in workspace:
    # refused on the host, nothing is launched, the detail text says why.  (The planner itself keeps
    # ranges x chunks within the number of compute units, which always fits: the ranges are forced here.)
    dims = R.make_dims(64, 128, 128, 8, 128, 600, 16, 64 * 600)
    x = torch.zeros(16, dtype=torch.bfloat16, device="cuda")
    i = torch.zeros(16, dtype=torch.int32, device="cuda")
    assert R.reader_workspace_bytes(dims, 8192) <= R.NOALLOC_WORKSPACE_BYTES
    R.reader_tuning_override(R.TUNE_ATTN_RANGES, 256)
    try:
        need = R.reader_workspace_bytes(dims, 8192)
        assert need > R.NOALLOC_WORKSPACE_BYTES
        with pytest.raises(R.ReaderError) as e:
            R.reader_tree_attn_noalloc(dims, x, x, x, x, x, i, i, i, x, None, 8192)
        assert e.value.code == R.READER_EWORKSPACE
        assert "workspace" in R.load().reader_last_error_detail().decode()
    finally:
        R.reader_tuning_override(R.TUNE_ATTN_RANGES, -1)
    dims = R.make_dims(1, 8, 8, 8, 128, 4, 4, 4, variant=1)
    with pytest.raises(R.ReaderError) as e:
        R.reader_tree_attn_noalloc(dims, x, x, x, x, x, i, i, i, x, None, 16)
    assert e.value.code == R.READER_EINVAL
