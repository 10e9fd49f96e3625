"""Where the attention main kernel's time goes, workgroup by workgroup, on one MI355X.

The profiling build of the library (python -m paper_2508_09072_amd.build --stamps, a second .so next to the
normal one) has thread 0 of every workgroup of the 128-row attention kernel note the GPU's constant-rate
counter (100 MHz) at these points: kernel entry, share of the tile axis known, tile list written, copy
constants made, first key tile asked for, first two asked for, first item complete in LDS, first key tile computed, last tile computed, exit.  This
script runs one preset with it and prints, over all workgroups and over the last launches of the run,
when each point is reached (relative to the first workgroup's entry), how long a workgroup takes per
tile in between, and how far apart the workgroups finish:

    python -m paper_2508_09072_amd.wg_timeline [--config 2] [--steps 40] [--tune ATTN_PAIR_COST=3]

The stamps cost a few stores per workgroup; the kernel is otherwise the one the benchmark times.
Inputs are seeded and synthetic (the benchmark presets).
"""
from __future__ import annotations

import argparse
import ctypes
import os

import numpy as np

STAMP_NAMES = ["entry", "range known", "list written", "first two key tiles asked for", "first item in LDS",
               "first tile computed", "last tile computed", "exit", "copy constants made", "first key tile asked for",
               "iteration 8: copier at the top", "iteration 8: copier past the barrier", "iteration 8: next item asked for",
               "first key tile in LDS", "first key tile computed (one wavefront)"]
ORDER = [0, 1, 2, 8, 9, 3, 4, 13, 14, 5, 10, 11, 12, 6, 7]     # in the order a workgroup reaches them
N_STAMPS = len(STAMP_NAMES)
MAX_WG = 2048


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--tune", action="append", default=[], metavar="NAME=VALUE",
                    help="planner override for the run, e.g. ATTN_PAIR_COST=3 (see reader_tuning_override)")
    args = ap.parse_args()

    import torch
    from . import binding as R, build as B, workloads as W
    if not os.path.exists(B.STAMPS_LIB):
        raise SystemExit("profiling build missing: run `python -m paper_2508_09072_amd.build --stamps` first")
    R.LIB_PATH = B.STAMPS_LIB
    lib = R.load()
    lib.reader_profile_wg_stamps.argtypes = [ctypes.c_void_p]
    lib.reader_profile_wg_stamps.restype = ctypes.c_int
    torch.cuda.set_device(0)
    for item in args.tune:
        name, value = item.split("=")
        R.reader_tuning_override(getattr(R, "TUNE_" + name), int(value))
        print("planner override: %s = %s" % (name, value))

    w = W.make_config(args.config)
    dw = R.to_device(w)
    kv_bytes = 2 * w.k_cache.nbytes
    copies = int(max(1, min(8, -(-(512 << 20) // max(kv_bytes, 1)))))   # more K/V than the 256 MB Infinity Cache holds
    kc = [dw.k_cache] + [dw.k_cache.clone() for _ in range(copies - 1)]
    vc = [dw.v_cache] + [dw.v_cache.clone() for _ in range(copies - 1)]
    stamps = torch.zeros((MAX_WG, N_STAMPS), dtype=torch.int64, device="cuda")
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)

    def attn(k):
        rc = lib.reader_tree_attn(ctypes.byref(dw.dims), p(dw.q), p(dw.k_tree), p(dw.v_tree), p(kc[k % copies]),
                                  p(vc[k % copies]), p(dw.page_table), p(dw.seq_lens), p(dw.parents), p(dw.out), None,
                                  dw.max_seq_len, p(dw.workspace), dw.workspace.numel(), p(dw.status), stream)
        if rc:
            raise RuntimeError("reader_tree_attn failed: %d" % rc)

    for k in range(10):
        attn(k)
    torch.cuda.synchronize()
    lib.reader_profile_wg_stamps(p(stamps))
    rows = []
    for k in range(args.steps):
        stamps.zero_()
        attn(10 + k)
        torch.cuda.synchronize()
        rows.append(stamps.cpu().numpy().copy())
    lib.reader_profile_wg_stamps(None)
    assert int(dw.status.item()) == 0

    ranges = dw.workspace[:256 * 4].view(torch.int32).cpu().numpy()    # tiles per range, first words of the workspace
    use = rows[len(rows) // 2:]                                          # the second half of the launches
    n_wg = int((use[0][:, 0] != 0).sum())
    print("preset %s: %d workgroups with stamps, %d launches summarised; times in us from the first workgroup's entry"
          % (w.name, n_wg, len(use)))
    rel = []
    for s in use:
        live = s[s[:, 0] != 0].astype(np.float64)
        rel.append((live - live[:, 0].min()) / 100.0)                   # 100 MHz -> us
    rel = np.stack(rel)                                                  # [launch, wg, stamp]
    print("%-38s %8s %8s %8s %8s %8s" % ("point", "min", "p10", "median", "p90", "max"))
    for i in ORDER:
        name = STAMP_NAMES[i]
        v = rel[:, :, i]
        v = v[v >= 0]
        if v.size == 0:                 # (a point no workgroup reached: fewer than nine iterations)
            continue
        print("%-38s %8.2f %8.2f %8.2f %8.2f %8.2f" % (name, v.min(), np.percentile(v, 10), np.median(v),
                                                        np.percentile(v, 90), v.max()))
    tiles = ranges[:n_wg].astype(np.float64) if n_wg <= 256 else None
    stream_us = rel[:, :, 6] - rel[:, :, 5]
    print("first tile computed -> last tile computed: median %.2f us per workgroup" % np.median(stream_us))
    if tiles is not None and (tiles > 1).all():
        per_tile = np.median(stream_us, axis=0) / (tiles - 1)
        print("  per tile: median %.3f us, p10 %.3f, p90 %.3f   (tiles per workgroup: %d..%d)"
              % (np.median(per_tile), np.percentile(per_tile, 10), np.percentile(per_tile, 90), tiles.min(), tiles.max()))
        row_bytes = 2 * w.D * 2                                          # K and V row of one kv head, bf16
        print("  = %.0f GB/s while streaming, all workgroups together (64 keys x %d bytes per tile)"
              % (n_wg * 64 * row_bytes / np.median(per_tile) / 1e3, row_bytes))
    end = rel[:, :, 7]
    print("kernel span (first entry -> last exit): median %.2f us; last exit - median exit: %.2f us; "
          "last entry - first entry: %.2f us" % (np.median(end.max(axis=1)), np.median(end.max(axis=1) - np.median(end, axis=1)),
                                                 np.median(rel[:, :, 0].max(axis=1))))
    late = np.argsort(-np.median(end, axis=0))[:5]
    print("the five workgroups that finish last (median over launches): " +
          ", ".join("wg %d at %.1f us%s" % (i, np.median(end[:, i]), "" if tiles is None else " (%d tiles)" % tiles[i]) for i in late))


if __name__ == "__main__":
    main()
