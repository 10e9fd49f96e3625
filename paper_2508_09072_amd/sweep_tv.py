"""Verification time as a function of the draft-tree size on one MI355X.

The paper sizes its draft tree from the shape of T_V(T), the base model's verification
time for a tree of T nodes: flat while the step is bound by reading the KV cache, then
growing once the tree makes it compute bound (Section 3.2: reads grow with b*h*(gamma+s),
flops with b*h*gamma*(gamma+s); Section 3.3 and Appendix E take T_V as given).  This
script measures that curve for the attention part of the step with the library's own
kernels, on the shapes of three presets: the single prompt (B=1, L=4096; the paper's case for
large trees), the batched ragged serving shape (B=16, L in [1024,4096]) and the large batch
(B=64, 64/8 heads, L in [2048,8192]):

    python -m paper_2508_09072_amd.sweep_tv [--steps 50] [--shapes single,batched,large]

One line per tree size: query rows per kv head, time of the attention main kernel and of
the whole fused step, tree tokens per second, achieved HBM bandwidth and matrix rate.
Then the curve is handed to the tree-shape selection of Appendix E (reader_tree_select): a
seed tree of 128 nodes with synthetic acceptance frequencies (a child's at most its parent's)
is pruned leaf by leaf and the size with the best modelled throughput sum(alpha) / (T_D + T_V)
is reported, for drafting that is free (retrieval on the host, in parallel) and for a drafter
that costs 2 us per node.  Inputs are seeded and synthetic (same recipe as the benchmark presets).
"""
from __future__ import annotations

import argparse
import ctypes
import time

import numpy as np


def measure(R, torch, w, steps: int, warmup: int = 5):
    dw = R.to_device(w)
    lib = R.load()
    n = warmup + steps
    kv_bytes = 2 * w.k_cache.nbytes
    copies = int(max(1, min(8, -(-(512 << 20) // max(kv_bytes, 1)))))   # defeat the 256 MB Infinity Cache
    kc = [dw.k_cache] + [dw.k_cache.clone() for _ in range(copies - 1)]
    vc = [dw.v_cache] + [dw.v_cache.clone() for _ in range(copies - 1)]
    seq_rows = dw.seq_lens.unsqueeze(0).repeat(n, 1).contiguous()      # compaction grows the lengths
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    ws_bytes = dw.workspace.numel()

    def step(k):
        r = k % copies
        rc = lib.reader_verify_step(ctypes.byref(dw.dims), p(dw.q), p(dw.k_tree), p(dw.v_tree), p(kc[r]), p(vc[r]),
                                    p(dw.page_table), ctypes.c_void_p(seq_rows[k].data_ptr()), p(dw.parents),
                                    p(dw.draft_tokens), p(dw.target_tokens), p(dw.out), None, p(dw.accept_len),
                                    p(dw.path), p(dw.bonus), dw.max_seq_len, p(dw.workspace), ws_bytes,
                                    p(dw.status), stream)
        if rc:
            raise RuntimeError("reader_verify_step failed: %d" % rc)

    for k in range(warmup):
        step(k)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(warmup, n):
        step(k)
    torch.cuda.synchronize()
    step_s = (time.perf_counter() - t0) / steps
    assert int(dw.status.item()) == 0

    seq_rows.copy_(dw.seq_lens.unsqueeze(0).expand(n, -1))
    torch.cuda.synchronize()
    R.reader_profile_enable(True)
    for k in range(warmup, n):
        step(k)
    torch.cuda.synchronize()
    ms_sum, launches = R.reader_profile_collect()
    R.reader_profile_enable(False)
    return step_s, ms_sum / max(launches, 1) * 1e-3


SHAPES = {
    # name: (B, Hq, Hkv, (L lo, L hi), trie depth, branching)
    "single": (1, 32, 8, (4096, 4096), 8, 4),
    "batched": (16, 32, 8, (1024, 4096), 6, 3),
    "large": (64, 64, 8, (2048, 8192), 10, 4),
}


def seed_tree(T, rng):
    """An overprovisioned seed tree in the manner of Appendix E: a trie-shaped tree whose k-th child is accepted
    less often than the (k-1)-th and whose acceptance decays with depth; alpha = product along the root path."""
    parents, alpha, rank = [-1], [1.0], [0]
    n_children = [0]
    while len(parents) < T:
        p = int(rng.integers(0, len(parents)))
        if n_children[p] >= 4:
            continue
        k = n_children[p]
        n_children[p] += 1
        parents.append(p)
        n_children.append(0)
        rank.append(k)
        alpha.append(alpha[p] * (0.62, 0.2, 0.08, 0.04)[k] * float(rng.uniform(0.85, 1.0)))
    return np.asarray(parents, dtype=np.int32), np.asarray(alpha, dtype=np.float32)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--sizes", type=str, default="1,2,4,8,16,24,32,48,64,96,128")
    ap.add_argument("--shapes", type=str, default="single,batched,large")
    args = ap.parse_args()

    import torch
    from . import binding as R
    from . import workloads as W

    R.load()
    torch.cuda.set_device(0)
    sizes = [int(x) for x in args.sizes.split(",")]
    for shape in [x for x in args.shapes.split(",") if x]:
        B, Hq, Hkv, (lo, hi), depth, branch = SHAPES[shape]
        rng = np.random.Generator(np.random.PCG64(W.SEED_BASE + 2))
        L = [int(x) for x in rng.integers(lo, hi + 1, size=B)]
        G = Hq // Hkv
        print("# T_V(T), shape %s: attention of one verification step, B=%d Hq=%d Hkv=%d D=128 sum_L=%d, eager launches"
              % (shape, B, Hq, Hkv, sum(L)))
        print("# %4s %5s %10s %10s %14s %9s %9s" % ("T", "rows", "kernel_us", "step_us", "tree_tok_per_s", "HBM_GB/s", "TFLOP/s"))
        step_us = {}
        for T in sizes:
            w = W.make_custom("sweep_%s_T%d" % (shape, T), B=B, Hq=Hq, Hkv=Hkv, D=128, T=T, seq_lens=L,
                              tree="trie" if T > 1 else "chain", depth=min(depth, max(T - 1, 1)), branch=branch,
                              vocab=128256, p_match=0.7, seed=W.SEED_BASE + 3000 + T)
            step_s, kern_s = measure(R, torch, w, args.steps)
            step_us[T] = step_s * 1e6
            print("  %4d %5d %10.1f %10.1f %14.0f %9.0f %9.1f" % (
                T, T * G, kern_s * 1e6, step_s * 1e6, B * T / step_s, w.algorithmic_bytes() / kern_s / 1e9,
                w.attention_flops() / kern_s / 1e12), flush=True)
            del w
            torch.cuda.empty_cache()
        # Appendix E on the measured curve (linear between the measured sizes)
        T0 = max(sizes)
        tv = np.interp(np.arange(1, T0 + 1), sizes, [step_us[t] for t in sizes]).astype(np.float32)
        parents, alpha = seed_tree(T0, np.random.Generator(np.random.PCG64(W.SEED_BASE + 4)))
        for label, per_node in (("free drafting", 0.0), ("2 us per drafted node", 2.0)):
            t_draft = np.full(T0, per_node, dtype=np.float32)
            n, keep, thr, evals = R.reader_tree_select(parents, alpha, t_draft, tv)
            n_x, keep_x, thr_x, _ = R.reader_tree_select(parents, alpha, t_draft, tv, exhaustive=True)
            print("# tree-shape selection, %s: seed tree of %d nodes (sum alpha %.2f) -> %d nodes kept, expected tokens per step %.2f, "
                  "modelled %.0f tokens/s per sequence (%d trees scored; exhaustive search: %d nodes, %.0f tokens/s)"
                  % (label, T0, float(alpha.sum()), int(keep.sum()), float(alpha[keep].sum()), thr * 1e6, evals,
                     int(keep_x.sum()), thr_x * 1e6), flush=True)
        print(flush=True)


if __name__ == "__main__":
    main()
