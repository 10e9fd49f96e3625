"""Verification time as a function of the draft-tree size on one MI355X.

The paper sizes its draft tree from the shape of T_V(T), the base model's verification
time for a tree of T nodes: flat while the step is bound by reading the KV cache, then
growing once the tree makes it compute bound (Section 3.2: reads grow with b*h*(gamma+s),
flops with b*h*gamma*(gamma+s); Section 3.3 and Appendix E take T_V as given).  This
script measures that curve for the attention part of the step with the library's own
kernels, on the batched ragged serving shape (B=16, 32/8 heads, D=128, L in [1024,4096]):

    python -m paper_2508_09072_amd.sweep_tv [--steps 50]

One line per tree size: query rows per kv head, time of the attention main kernel and of
the whole fused step, tree tokens per second, achieved HBM bandwidth and matrix rate.
Inputs are seeded and synthetic (same recipe as the benchmark presets).
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--sizes", type=str, default="1,2,4,8,16,24,32,48,64,96,128")
    args = ap.parse_args()

    import torch
    from . import binding as R
    from . import workloads as W

    R.load()
    torch.cuda.set_device(0)
    rng = np.random.Generator(np.random.PCG64(W.SEED_BASE + 2))
    L = [int(x) for x in rng.integers(1024, 4096 + 1, size=16)]
    print("# T_V(T): attention of one verification step, B=16 Hq=32 Hkv=8 D=128 sum_L=%d, eager launches" % sum(L))
    print("# %4s %5s %10s %10s %14s %9s %9s" % ("T", "rows", "kernel_us", "step_us", "tree_tok_per_s", "HBM_GB/s", "TFLOP/s"))
    for T in [int(x) for x in args.sizes.split(",")]:
        w = W.make_custom("sweep_T%d" % T, B=16, Hq=32, Hkv=8, D=128, T=T, seq_lens=L,
                          tree="trie" if T > 1 else "chain", depth=min(6, max(T - 1, 1)), branch=3, vocab=128256,
                          p_match=0.7, seed=W.SEED_BASE + 3000 + T)
        step_s, kern_s = measure(R, torch, w, args.steps)
        print("  %4d %5d %10.1f %10.1f %14.0f %9.0f %9.1f" % (
            T, T * 4, kern_s * 1e6, step_s * 1e6, 16 * T / step_s, w.algorithmic_bytes() / kern_s / 1e9,
            w.attention_flops() / kern_s / 1e12), flush=True)


if __name__ == "__main__":
    main()
