#!/usr/bin/env python3
"""Benchmark of the draft-tree verification step on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input:
attention over the draft tree, acceptance of the longest matching path, compaction of
its rows into the cache (reader_verify_step: the three operations in two kernel launches;
`--separate-calls` times reader_tree_attn -> reader_accept_path -> reader_kv_compact
instead), all on one stream, inputs resident in HBM before the clock starts.  The metric is tree tokens per
second (B * T draft-tree nodes verified per step) together with the achieved HBM
bandwidth of the attention kernel, which streams the K/V cache and dominates.

    python bench.py --gpus 1 --steps 200 --warmup 20

prints ONE JSON line.  The headline workload is the largest single-GPU preset (cfg4:
B=64, Hq=64, L in [2048,8192], T=64, the whole step timed end to end); the other four
presets are timed the same way and reported inside the same line under
"other_workloads", each with its own roofline object and its own CPU-oracle baseline.
Before the timed steps of a workload the same steps run untimed for at least
SETTLE_MS (the GPU needs some tens of milliseconds of load to reach its clocks; the
`warmup` argument is honoured on top of that and echoed unchanged).  `--gpus N` with
N > 1 is refused: this build is single-GPU.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 matrix rate
ROTATE_BYTES = 512 << 20       # K/V copies cycled per step so the 256 MB Infinity Cache cannot serve the stream
CALIBRATION_BYTES = 256 << 20  # size of the plain elementwise pass the counter runs are scaled by
SETTLE_MS = 60.0               # untimed load in front of every timed region
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "tree_attn_hbm_traffic_all_presets.txt")


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class StepRunner:
    """Pre-marshalled C-ABI calls for K steps of one workload (no per-step Python marshalling)."""

    def __init__(self, R, torch, w, n_steps, fused=True, rotate=True, attention_only=False):
        self.R, self.torch, self.w, self.fused = R, torch, w, fused
        self.attention_only = attention_only
        self.lib = R.load()
        dw = R.to_device(w)
        self.dw = dw
        kv_bytes = 2 * w.k_cache.nbytes
        self.n_copies = int(max(1, min(32, -(-ROTATE_BYTES // max(kv_bytes, 1))))) if rotate else 1
        self.kc = [dw.k_cache] + [dw.k_cache.clone() for _ in range(self.n_copies - 1)]
        self.vc = [dw.v_cache] + [dw.v_cache.clone() for _ in range(self.n_copies - 1)]
        # compaction grows seq_lens: every step gets its own fresh copy of the lengths
        self.seq_rows = dw.seq_lens.unsqueeze(0).repeat(n_steps, 1).contiguous()
        self.n_steps = n_steps
        self.dims = ctypes.byref(dw.dims)
        p = lambda t: ctypes.c_void_p(t.data_ptr())
        self.attn_args, self.compact_args, self.step_args = [], [], []
        ws_bytes = dw.workspace.numel()
        for k in range(n_steps):
            r = k % self.n_copies
            seq = ctypes.c_void_p(self.seq_rows[k].data_ptr())
            self.attn_args.append((self.dims, p(dw.q), p(dw.k_tree), p(dw.v_tree), p(self.kc[r]), p(self.vc[r]),
                                   p(dw.page_table), seq, p(dw.parents), p(dw.out), None, dw.max_seq_len,
                                   p(dw.workspace), ws_bytes, p(dw.status)))
            self.compact_args.append((self.dims, p(dw.k_tree), p(dw.v_tree), p(dw.path), p(dw.accept_len),
                                      p(self.kc[r]), p(self.vc[r]), p(dw.page_table), seq, p(dw.status)))
            self.step_args.append((self.dims, p(dw.q), p(dw.k_tree), p(dw.v_tree), p(self.kc[r]), p(self.vc[r]),
                                   p(dw.page_table), seq, p(dw.parents), p(dw.draft_tokens), p(dw.target_tokens),
                                   p(dw.out), None, p(dw.accept_len), p(dw.path), p(dw.bonus), dw.max_seq_len,
                                   p(dw.workspace), ws_bytes, p(dw.status)))
        self.accept_args = (self.dims, p(dw.draft_tokens), p(dw.target_tokens), p(dw.parents), p(dw.accept_len),
                            p(dw.path), p(dw.bonus), p(dw.status))

    def reset(self):
        self.seq_rows.copy_(self.dw.seq_lens.unsqueeze(0).expand(self.n_steps, -1))

    def run(self, first, count):
        lib = self.lib
        stream = ctypes.c_void_p(self.torch.cuda.current_stream().cuda_stream)
        for k in range(first, first + count):
            if self.attention_only:
                rc = lib.reader_tree_attn(*self.attn_args[k], stream)
            elif self.fused:
                rc = lib.reader_verify_step(*self.step_args[k], stream)
            else:
                rc = lib.reader_tree_attn(*self.attn_args[k], stream)
                rc |= lib.reader_accept_path(*self.accept_args, stream)
                rc |= lib.reader_kv_compact(*self.compact_args[k], stream)
            if rc:
                raise RuntimeError("library call failed in step %d" % k)


def settle(run, torch, warmup, min_ms=SETTLE_MS):
    """The workload's own steps, untimed, until the GPU has been under load for min_ms: `warmup` steps at
    least.  Returns (milliseconds spent, steps run)."""
    t0 = time.perf_counter()
    n = 0
    while True:
        run.run(0, max(warmup, 1))
        run.reset()
        torch.cuda.synchronize()
        n += max(warmup, 1)
        ms = (time.perf_counter() - t0) * 1e3
        if ms >= min_ms or n >= 100000:
            return ms, n


def roofline_of(w, each):
    """Roofline object of the attention main kernel from its per-launch times (ms, HIP events bound to the kernel)."""
    import numpy as np
    n = len(each)
    kernel_ms = float(each.sum()) / max(n, 1)
    alg_bytes = w.algorithmic_bytes()
    flops = w.attention_flops()
    gbs = alg_bytes / (kernel_ms * 1e-3) / 1e9
    tflops = flops / (kernel_ms * 1e-3) / 1e12
    hbm_t = alg_bytes / (HBM_PEAK_GBS * 1e9)
    mfma_t = flops / (MFMA_BF16_PEAK_TFLOPS * 1e12)
    if hbm_t >= mfma_t:
        roof = {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS}
    else:
        roof = {"bound": "mfma", "achieved": tflops, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": tflops / MFMA_BF16_PEAK_TFLOPS}
    from paper_2508_09072_amd import binding as R
    plan = R.reader_attn_plan(R.make_dims(w.B, w.T, w.Hq, w.Hkv, w.D, w.max_pages, w.max_path, w.num_pages),
                              int(w.seq_lens.max()))
    roof.update({"kernel": plan["kernel"], "workgroups": plan["key_ranges"] * plan["row_chunks"],
                 "rows_per_workgroup": plan["rows_per_workgroup"], "kernel_ms": kernel_ms, "launches_timed": n,
                 "kernel_ms_median": float(np.median(each)) if n else None,
                 "kernel_ms_min": float(each.min()) if n else None,
                 "algorithmic_bytes": alg_bytes, "algorithmic_flops": flops, "hbm_gbs": gbs,
                 "hbm_frac": gbs / HBM_PEAK_GBS, "mfma_tflops": tflops, "mfma_frac": tflops / MFMA_BF16_PEAK_TFLOPS,
                 "traffic": measured_traffic(w.name)})
    return roof


def time_workload(R, torch, w, steps, warmup, use_graph=True, fused=True):
    total = warmup + steps
    run = StepRunner(R, torch, w, total, fused=fused)
    res = {"workload": w.name, "kv_copies_rotated": run.n_copies,
           "entry_points": "reader_verify_step" if fused else "reader_tree_attn+reader_accept_path+reader_kv_compact"}

    # ---- untimed load until the clocks have settled, then `warmup` steps, then exactly `steps` steps
    # between two synchronisations
    res["settle_ms"], res["settle_steps"] = settle(run, torch, warmup)
    run.run(0, warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run.run(warmup, steps)
    torch.cuda.synchronize()
    eager_s = time.perf_counter() - t0
    assert int(run.dw.status.item()) == 0, "device status flagged an input problem"
    out_eager = run.dw.out.clone()
    seq_eager = run.seq_rows.clone()
    res["eager_ms_per_step"] = eager_s / steps * 1e3

    # ---- the same `steps` steps captured once into a HIP graph and replayed
    graph_s = None
    if use_graph:
        try:
            run.reset()
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                run.run(warmup, steps)
            for _ in range(3):                      # replay is checked against eager every time
                run.reset()
                run.dw.out.zero_()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                g.replay()
                torch.cuda.synchronize()
                dt = time.perf_counter() - t0
                ok = torch.equal(run.dw.out, out_eager) and torch.equal(run.seq_rows[warmup:], seq_eager[warmup:])
                if not ok:
                    raise RuntimeError("graph replay differs from eager execution")
                graph_s = dt if graph_s is None else min(graph_s, dt)
            res["graph_ms_per_step"] = graph_s / steps * 1e3
        except Exception as e:  # the eager number stands on its own
            log("graph mode unavailable:", repr(e))
            graph_s = None
    best_s = eager_s if graph_s is None else min(graph_s, eager_s)
    res["launch_mode"] = "hip_graph" if (graph_s is not None and graph_s <= eager_s) else "eager"
    res["ms_per_step"] = best_s / steps * 1e3
    res["tree_tokens_per_s"] = w.B * w.T * steps / best_s

    # ---- roofline of the dominant kernel: HIP events around the attention main kernel,
    # recorded by the library on the launch stream, over the same `steps` steps
    run.reset()
    torch.cuda.synchronize()
    R.reader_profile_enable(True)
    run.run(warmup, steps)
    torch.cuda.synchronize()
    each = R.reader_profile_collect_each()
    R.reader_profile_enable(False)
    res["roofline"] = roofline_of(w, each)
    return res


def time_steps_only(R, torch, w, steps, warmup, **runner_kw):
    """Eager launches of `steps` steps after `warmup`, and the main kernel's own time: for the side figures
    of the headline preset (attention alone; K/V not rotated)."""
    total = warmup + steps
    run = StepRunner(R, torch, w, total, **runner_kw)
    settle(run, torch, warmup)
    run.run(0, warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run.run(warmup, steps)
    torch.cuda.synchronize()
    step_ms = (time.perf_counter() - t0) / steps * 1e3
    run.reset()
    torch.cuda.synchronize()
    R.reader_profile_enable(True)
    run.run(warmup, steps)
    torch.cuda.synchronize()
    each = R.reader_profile_collect_each()
    R.reader_profile_enable(False)
    kernel_ms = float(each.mean()) if len(each) else None
    res = {"ms_per_step": step_ms, "kernel_ms": kernel_ms, "kv_copies_rotated": run.n_copies}
    if kernel_ms:
        res["algorithmic_gbs"] = w.algorithmic_bytes() / (kernel_ms * 1e-3) / 1e9
    return res


def cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for ln in f:
                if ln.startswith("model name"):
                    return ln.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def measured_traffic(workload_name):
    """HBM bytes per launch of the attention kernel from the committed counter runs, or None.

    bench.py cannot run the counter collector around itself; the figure is taken from the
    summary of the two counter runs of this same command (one line per workload,
    `traffic <workload> <bytes>`), which is re-made whenever the kernel changes.
    """
    try:
        with open(TRAFFIC_FILE) as f:
            for ln in f:
                tok = ln.split()
                if len(tok) == 3 and tok[0] == "traffic" and tok[1] == workload_name:
                    return float(tok[2])
    except OSError:
        pass
    return None


def calibration_pass(torch):
    """One elementwise pass that reads and writes CALIBRATION_BYTES: the known-size kernel
    the FETCH_SIZE / WRITE_SIZE readings of a counter run are scaled by."""
    n = CALIBRATION_BYTES // 4
    x = torch.ones(n, dtype=torch.int32, device="cuda")
    y = torch.empty_like(x)
    torch.cuda.synchronize()
    for _ in range(3):
        torch.add(x, 1, out=y)
    torch.cuda.synchronize()
    assert int(y[-1].item()) == 2
    del x, y


def oracle_steps(w, budget_s, max_reps):
    """Whole steps of the CPU oracle, as it stands, on workload w until the budget is used.  Returns (steps, seconds)."""
    import oracle
    reps, t0 = 0, time.perf_counter()
    while True:
        kc, vc, sl = w.k_cache, w.v_cache, w.seq_lens.copy()
        oracle.tree_attn(w.q, w.k_tree, w.v_tree, kc, vc, w.page_table, sl, w.parents)
        al, path, bonus = oracle.accept_path(w.draft_tokens, w.target_tokens, w.parents, w.max_path)
        # compaction writes behind the sequences' ends (canary slots); lengths are a scratch copy
        oracle.kv_compact(w.k_tree, w.v_tree, path, al, kc, vc, w.page_table, sl)
        reps += 1
        dt = time.perf_counter() - t0
        if dt >= budget_s or reps >= max_reps:
            return reps, dt


def cpu_baseline(w, budget_s=12.0, max_reps=50, one_thread_index=None):
    """The CPU oracle on the same workload, on the host cores of the GPU machine: a bounded sample (whole steps
    until the budget is used; at least one).  one_thread_index: also time it with a single thread (a child
    process, the thread count is fixed when the OpenMP runtime starts) on preset number one_thread_index."""
    import oracle
    reps, dt = oracle_steps(w, budget_s, max_reps)
    res = {"value": w.B * w.T * reps / dt, "unit": "tree tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
           "cpu_model": cpu_model(), "host_cpus": os.cpu_count(),
           "sample": "%d whole step(s) of %s (attention + acceptance + compaction), %.1f s" % (reps, w.name, dt)}
    if one_thread_index is not None:
        import subprocess
        code = ("import sys, json; sys.path.insert(0, %r); import bench; from paper_2508_09072_amd import workloads as W; "
                "w = W.make_config(%d); r, t = bench.oracle_steps(w, 3.0, 20); print(json.dumps([r, t]))" % (ROOT, one_thread_index))
        try:
            out = subprocess.run([sys.executable, "-c", code], env=dict(os.environ, OMP_NUM_THREADS="1"), stdout=subprocess.PIPE,
                                 stderr=subprocess.DEVNULL, text=True, timeout=120).stdout
            r1, t1 = json.loads(out.strip().splitlines()[-1])
            res["one_thread"] = {"value": w.B * w.T * r1 / t1, "cores": 1, "sample": "%d whole step(s), %.1f s" % (r1, t1)}
        except Exception as e:      # the all-cores figure stands on its own
            log("one-thread oracle timing failed:", repr(e))
    return res


def time_rearrange(R, torch, W, reps=10):
    """The periodic rearrangement pass on a padded cache (Section 4.3): 16 samples with the prompt
    lengths of the headline preset, 25 decoding steps of holes (the paper's N), 8 layers.  The values
    are filled on the device (they do not matter for the timing; parity is the tests' business)."""
    import numpy as np
    NL, B, Hkv, D, steps = 8, 16, 8, 128, 25
    rng = np.random.Generator(np.random.PCG64(W.SEED_BASE + 77))
    prompts = rng.integers(1024, 4096 + 1, size=B)
    valid_np = W.padded_valid_flags(prompts, steps, 0.1, rng)
    S = valid_np.shape[1]
    rows_moved = rows_zeroed = 0
    for b in range(B):
        holes = np.flatnonzero(valid_np[b] == 0)
        n, last = int(valid_np[b].sum()), int(np.flatnonzero(valid_np[b]).max()) + 1
        if holes.size and holes[0] < last:
            rows_moved += int(valid_np[b, holes[0]:].sum())
            rows_zeroed += last - n
    row_bytes = NL * Hkv * D * 2 * 2                               # K and V, all layers, one position
    alg_bytes = rows_moved * row_bytes * 2 + rows_zeroed * row_bytes
    k0 = torch.randn((NL, B, S, Hkv, D), device="cuda", dtype=torch.bfloat16)
    v0 = torch.randn((NL, B, S, Hkv, D), device="cuda", dtype=torch.bfloat16)
    valid0 = torch.from_numpy(valid_np).cuda()
    k, v, valid = k0.clone(), v0.clone(), valid0.clone()
    new_len = torch.zeros(B, dtype=torch.int32, device="cuda")
    scratch = torch.empty(R.reader_kv_rearrange_scratch_bytes(B, S), dtype=torch.uint8, device="cuda")
    times = []
    for rep in range(reps + 2):
        k.copy_(k0); v.copy_(v0); valid.copy_(valid0)               # holes again (not timed)
        a, b_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        R.reader_kv_rearrange(k, v, valid, new_len, scratch)
        b_.record()
        torch.cuda.synchronize()
        if rep >= 2:
            times.append(a.elapsed_time(b_))
    assert np.array_equal(new_len.cpu().numpy(), valid_np.sum(axis=1))
    ms = float(np.median(times))
    return {"workload": "padded cache B=%d S=%d layers=%d Hkv=%d D=%d, %d steps of holes" % (B, S, NL, Hkv, D, steps),
            "ms_per_pass": ms, "rows_moved": rows_moved, "rows_zeroed": rows_zeroed, "algorithmic_bytes": alg_bytes,
            "hbm_gbs": alg_bytes / (ms * 1e-3) / 1e9, "hbm_frac": alg_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "ms_per_step_amortised_over_25": ms / 25}


def time_compact_layers(R, torch, W, reps=20):
    """Compaction in the in-cache layout over the 32 layers of an 8B-class model, for the 16 sequences and
    32-node trees of the headline preset (lengths scaled down: a full-length cache of 32 layers does not
    change what the pass touches, only what sits beside it).  Each call moves the same accepted paths
    again (the lengths are reset between calls, not timed)."""
    import numpy as np
    rng = np.random.Generator(np.random.PCG64(W.SEED_BASE + 78))
    s = W.make_incache_step("bench", B=16, T=32, Hkv=8, D=128, num_layers=32,
                            seq_lens=[int(x) for x in rng.integers(64, 257, size=16)], max_path=9, seed=W.SEED_BASE + 79)
    NL, num_pages, Hkv, _, D = s.k_cache.shape
    dims = R.make_dims(16, 32, 32, Hkv, D, s.page_table.shape[1], s.max_path, num_pages)
    k = torch.from_numpy(s.k_cache.view(np.int16)).cuda().view(torch.bfloat16)
    v = torch.from_numpy(s.v_cache.view(np.int16)).cuda().view(torch.bfloat16)
    L0 = torch.from_numpy(s.seq_lens.copy()).cuda()
    L = L0.clone()
    path, acc, table = torch.from_numpy(s.path).cuda(), torch.from_numpy(s.accept_len).cuda(), torch.from_numpy(s.page_table).cuda()
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    times = []
    for rep in range(reps + 2):
        L.copy_(L0)
        a, b_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        R.reader_kv_compact_layers(dims, path, acc, k, v, table, L, status)
        b_.record()
        torch.cuda.synchronize()
        if rep >= 2:
            times.append(a.elapsed_time(b_))
    assert int(status.item()) == 0
    ms = float(np.median(times))
    # the same call as one of a stream of kernels (as in a decoding loop): `reps` calls back to back, each behind
    # the copy that resets the lengths, minus the time of those copies alone
    def streamed(with_call):
        a, b_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(reps):
            L.copy_(L0)
            if with_call:
                R.reader_kv_compact_layers(dims, path, acc, k, v, table, L, status)
        b_.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b_) / reps
    both = float(np.median([streamed(True) for _ in range(5)]))
    resets = float(np.median([streamed(False) for _ in range(5)]))
    assert int(status.item()) == 0
    return {"workload": "in-cache step B=16 T=32 layers=32 Hkv=8 D=128, accepted lengths %s" % s.accept_len.tolist(),
            "ms_per_call": ms, "ms_per_call_in_a_stream": both - resets, "launches_per_call": 1,
            "algorithmic_bytes": s.moved_bytes(), "hbm_gbs": s.moved_bytes() / (ms * 1e-3) / 1e9}


def time_target_tokens(R, torch, reps=20):
    """Target tokens from base-model logits (vocabulary 128256) for the rows of one step of the headline
    preset (B*T = 512) and of the large-batch preset (4096): the greedy arg max, and the sampling policy with
    coupled uniforms (temperature 1, a chain of 32 nodes per sequence).  The logits are filled on the device."""
    greedy, sampled = {}, {}
    V, T = 128256, 32
    for name, rows in (("rows_512", 512), ("rows_4096", 4096)):
        n_buf = max(2, -(-ROTATE_BYTES // (rows * V * 2)))         # rotate so that the 256 MB cache cannot serve it
        logits = [torch.randn((rows // T, T, V), device="cuda", dtype=torch.bfloat16) for _ in range(n_buf)]
        tok = torch.zeros((rows // T, T), dtype=torch.int32, device="cuda")
        parents = (torch.arange(T, dtype=torch.int32, device="cuda") - 1).repeat(rows // T, 1).contiguous()
        uniforms = torch.rand((rows // T, T), device="cuda", dtype=torch.float32).clamp_(max=1.0 - 2.0 ** -24)
        nbytes = rows * V * 2
        for label, res, call in (("argmax", greedy, lambda l: R.reader_target_argmax(l, tok)),
                                 ("sample", sampled, lambda l: R.reader_target_sample(l, parents, uniforms, 1.0, tok))):
            for l in logits[:2]:
                call(l)
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for k in range(reps):
                call(logits[k % n_buf])
            b.record()
            torch.cuda.synchronize()
            ms = a.elapsed_time(b) / reps
            res[name] = {"ms": ms, "bytes": nbytes, "hbm_gbs": nbytes / (ms * 1e-3) / 1e9,
                         "hbm_frac": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
        del logits
        torch.cuda.empty_cache()
    return greedy, sampled


def time_drafter(R, W, n_tokens=65536, n_trees=2000):
    """The host-side retrieval drafter (plain C++ on the host cores, one thread): n-gram trie of depth 8
    over a self-repetitive token stream, then one draft tree of at most 32 nodes (5 levels) and a search
    path of 8 tokens per context of 3 tokens, for contexts taken along the stream."""
    import numpy as np
    text = W.make_token_stream(n_tokens, seed=W.SEED_BASE + 95)
    trie = R.Trie(8)
    t0 = time.perf_counter()
    for lo in range(0, n_tokens, 4096):            # appended piece by piece, as decoding does
        trie.insert(text[lo:lo + 4096])
    t_insert = time.perf_counter() - t0
    rng = np.random.Generator(np.random.PCG64(W.SEED_BASE + 96))
    ends = rng.integers(8, n_tokens, size=n_trees)
    nodes = 0
    t0 = time.perf_counter()
    for e in ends:
        tokens, _ = trie.extract_tree(text[e - 3:e], 5, 32)
        nodes += len(tokens)
    t_tree = time.perf_counter() - t0
    t0 = time.perf_counter()
    for e in ends:
        trie.search_path(text[e - 3:e], 8)
    t_path = time.perf_counter() - t0
    res = {"stream_tokens": n_tokens, "trie_nodes": len(trie), "insert_tokens_per_s": n_tokens / t_insert,
           "extract_tree_us": t_tree / n_trees * 1e6, "mean_tree_nodes": nodes / n_trees,
           "search_path_us": t_path / n_trees * 1e6, "threads": 1,
           "note": "per-call times include the Python binding"}
    trie.close()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20,
                    help="untimed steps right before the timed ones (on top of the time-based settle phase)")
    ap.add_argument("--config", type=int, default=4, help="headline preset (0..4)")
    ap.add_argument("--others", type=str, default="0,1,2,3", help="presets also timed (comma list, '' for none)")
    ap.add_argument("--other-steps", type=int, default=0, help="timed steps of the other presets (0: as --steps)")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--separate-calls", action="store_true",
                    help="time the three entry points called one after the other instead of the fused step")
    ap.add_argument("--no-scaled-shapes", action="store_true",
                    help="skip the two larger HBM-bound shapes (headline shape with longer contexts / more sequences)")
    ap.add_argument("--no-rearrange", action="store_true", help="skip the timings of the padded-cache rearrangement and of the logits arg max")
    ap.add_argument("--calibration-pass", action="store_true",
                    help="also run a plain elementwise pass of known size (for counter runs)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only; --gpus N with N > 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2508_09072_amd import binding as R
    from paper_2508_09072_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    R.load()   # raises if the HIP library is missing: there is no fallback path
    torch.cuda.set_device(0)

    if args.calibration_pass:
        calibration_pass(torch)
    log("generating", W.CONFIG_NAMES[args.config])
    w = W.make_config(args.config)
    head = time_workload(R, torch, w, args.steps, args.warmup, use_graph=not args.no_graph,
                         fused=not args.separate_calls)
    log("headline:", json.dumps(head))

    line = {
        "metric": "tree_verify_tokens_per_sec",
        "value": head["tree_tokens_per_s"],
        "unit": "tree tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "T": w.T, "Hq": w.Hq, "Hkv": w.Hkv, "D": w.D,
                   "sum_L": int(w.seq_lens.sum()), "page_size": w.page_size,
                   "launch_mode": head["launch_mode"], "kv_copies_rotated": head["kv_copies_rotated"],
                   "entry_points": head["entry_points"]},
        "eager_ms_per_step": head["eager_ms_per_step"],
        "graph_ms_per_step": head.get("graph_ms_per_step"),
        "settle_ms": head["settle_ms"],
        "roofline": head["roofline"],
    }
    if not args.no_cpu_baseline:
        log("timing the CPU oracle on the headline workload")
        line["cpu_baseline"] = cpu_baseline(w, budget_s=8.0, max_reps=50,
                                            one_thread_index=args.config if args.config in (0, 1) else None)
    del head, w
    torch.cuda.empty_cache()

    others = {}
    other_steps = args.other_steps if args.other_steps > 0 else args.steps
    for idx in [int(x) for x in args.others.split(",") if x.strip() != ""]:
        if idx == args.config:
            continue
        log("generating", W.CONFIG_NAMES[idx])
        wo = W.make_config(idx)
        r = time_workload(R, torch, wo, other_steps, args.warmup, use_graph=not args.no_graph,
                          fused=not args.separate_calls)
        others[wo.name] = {"tree_tokens_per_s": r["tree_tokens_per_s"], "ms_per_step": r["ms_per_step"],
                           "launch_mode": r["launch_mode"], "steps": other_steps, "settle_ms": r["settle_ms"],
                           "roofline": r["roofline"]}
        if idx == 2 and not args.no_scaled_shapes:
            # side figures of the batched HBM-bound preset: the attention entry point alone (its two launches),
            # and the step with K/V not rotated (one copy, small enough for the 256 MB Infinity Cache)
            side_steps = min(other_steps, 200)
            others[wo.name]["attention_only"] = time_steps_only(R, torch, wo, side_steps, args.warmup, attention_only=True)
            others[wo.name]["cache_resident"] = time_steps_only(R, torch, wo, side_steps, args.warmup, rotate=False)
        if not args.no_cpu_baseline:
            # the two long presets run once (several seconds each); the small ones also with one thread
            others[wo.name]["cpu_baseline"] = cpu_baseline(wo, budget_s=4.0, max_reps=20,
                                                           one_thread_index=idx if idx in (0, 1) else None)
        log(wo.name, json.dumps(others[wo.name]))
        del wo, r
        torch.cuda.empty_cache()
    line["other_workloads"] = others
    # what a bare copy ring and a bare matrix loop reach on this GPU (beside the published peaks of the roofline objects)
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
    scratch = torch.empty(1 << 19, dtype=torch.uint8, device="cuda")
    peaks = [R.reader_measure_peaks(src, scratch) for _ in range(3)][1:]
    line["measured_peaks"] = {"hbm_read_gbs": max(p["hbm_read_gbs"] for p in peaks),
                              "mfma_bf16_tflops": max(p["mfma_bf16_tflops"] for p in peaks),
                              "mfma_clock_mhz": peaks[-1]["mfma_clock_mhz"],
                              "note": "bare LDS copy ring over 1 GiB; bare v_mfma_f32_32x32x16_bf16 loop, one wavefront per SIMD"}
    del src, scratch
    torch.cuda.empty_cache()
    if not args.no_scaled_shapes:
        # The batched HBM-bound shape (cfg2) with more bytes per launch (longer contexts, or more sequences): the
        # fixed part of a launch (start, first latency, end) weighs less, the achieved fraction of the HBM peak rises.
        import numpy as np
        scaled = {}
        rng = np.random.Generator(np.random.PCG64(W.SEED_BASE + 90))
        for name, B, lo, hi in (("hbm_bound_B16_L8192-16384_T32", 16, 8192, 16384), ("hbm_bound_B64_L1024-4096_T32", 64, 1024, 4096)):
            log("generating", name)
            L = [int(x) for x in rng.integers(lo, hi + 1, size=B)]
            wo = W.make_custom(name, B=B, Hq=32, Hkv=8, D=128, T=32, seq_lens=L, tree="trie", depth=6, branch=3,
                               vocab=128256, p_match=0.7, seed=W.SEED_BASE + 91)
            r = time_workload(R, torch, wo, min(other_steps, 100), args.warmup, use_graph=not args.no_graph,
                              fused=not args.separate_calls)
            scaled[name] = {"tree_tokens_per_s": r["tree_tokens_per_s"], "ms_per_step": r["ms_per_step"],
                            "kernel_ms": r["roofline"]["kernel_ms"], "algorithmic_bytes": r["roofline"]["algorithmic_bytes"],
                            "hbm_gbs": r["roofline"]["hbm_gbs"], "hbm_frac": r["roofline"]["hbm_frac"]}
            log(name, json.dumps(scaled[name]))
            del wo, r
            torch.cuda.empty_cache()
        line["scaled_shapes"] = scaled
    if not args.no_rearrange:
        log("timing the periodic rearrangement pass")
        line["kv_rearrange"] = time_rearrange(R, torch, W)
        log("timing the arg max over logits")
        line["kv_compact_layers"] = time_compact_layers(R, torch, W)
        line["target_argmax"], line["target_sample"] = time_target_tokens(R, torch)
        log("timing the host drafter")
        line["drafter"] = time_drafter(R, W)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
