"""The host-side code under AddressSanitizer and UndefinedBehaviorSanitizer, on the CPU.

The retrieval drafter and the tree-shape selection (plain C++ of the library) and the CPU oracle
(plain C) are compiled here with -fsanitize=address,undefined into two small driver programs
(tests/sanitize/) and run on the inputs of the drafter, tree-shape and oracle tests: their
answers must be the oracle's (drafter, selection) respectively the ordinary oracle build's, and
the sanitizers must stay silent.  No GPU code is involved (the kernels cannot be run this way).
"""
import os
import subprocess
import sys

import numpy as np
import pytest

from oracle import drafter as D
from oracle import tree_shape as TS
from paper_2508_09072_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-static-libasan", "-static-libubsan",
       "-fno-omit-frame-pointer", "-g", "-O1"]
# the drivers are ordinary programs; a library somebody preloads into every process must not trip the
# link-order check of the sanitizer's own start-up
ENV = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def build(tmp, name, compiler, sources, extra=()):
    exe = os.path.join(tmp, name)
    cmd = [compiler] + SAN + list(extra) + ["-I" + os.path.join(ROOT, "include")] + sources + ["-o", exe]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout
    return exe


@pytest.fixture(scope="module")
def host_driver(tmp_path_factory):
    csrc = os.path.join(ROOT, "paper_2508_09072_amd", "csrc")
    # reader_validate_tree lives with the GPU entry points; the driver gets a copy of that one host function
    shim = os.path.join(str(tmp_path_factory.mktemp("shim")), "validate_tree.cpp")
    text = open(os.path.join(csrc, "reader_api.hip")).read()
    a = text.index('extern "C" int reader_validate_tree')
    b = text.index("\n}\n", a) + 3
    open(shim, "w").write('#include "reader.h"\n' + text[a:b])
    return build(str(tmp_path_factory.mktemp("san")), "host_driver", "g++",
                 [os.path.join(ROOT, "tests", "sanitize", "host_driver.cpp"), os.path.join(csrc, "trie_drafter.cpp"),
                  os.path.join(csrc, "tree_shape.cpp"), shim], extra=["-std=c++17"])


@pytest.fixture(scope="module")
def oracle_driver(tmp_path_factory):
    return build(str(tmp_path_factory.mktemp("san")), "oracle_driver", "gcc",
                 [os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"), os.path.join(ROOT, "oracle", "reader_oracle.c")],
                 extra=["-std=c11", "-fopenmp", "-lm"])


def run_lines(exe, lines):
    res = subprocess.run([exe], input="\n".join(lines) + "\n", stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True,
                         env=ENV, timeout=300)
    assert res.returncode == 0 and "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr, res.stderr[-3000:]
    out = res.stdout.strip().split("\n")
    assert len(out) == len(lines), (len(out), len(lines))
    return out


def ints(xs):
    return " ".join(str(int(x)) for x in xs)


def synthetic_text(rng, n, vocab=50, n_phrases=12, p_phrase=0.5):
    phrases = [rng.integers(0, vocab, size=rng.integers(3, 12)).tolist() for _ in range(n_phrases)]
    out = []
    while len(out) < n:
        if rng.random() < p_phrase:
            out += phrases[int(rng.integers(0, n_phrases))]
        else:
            out.append(int(min(vocab - 1, rng.zipf(1.5) - 1)))
    return out[:n]


def test_drafter_under_sanitizers_gives_the_oracles_answers(host_driver):
    rng = np.random.Generator(np.random.PCG64(71))
    lines, want = [], []
    for max_depth in (2, 5, 9):
        text = synthetic_text(rng, 500)
        ix = D.NgramIndex(max_depth)
        lines.append("trie %d" % max_depth); want.append("1")
        for lo in range(0, 500, 125):
            lines.append("insert 125 " + ints(text[lo:lo + 125])); want.append("0")
            ix.insert(text[lo:lo + 125])
        lines.append("nodes"); want.append(str(len(ix.count) + 1))
        for _ in range(40):
            at = int(rng.integers(1, 500))
            ctx = text[max(0, at - int(rng.integers(1, max_depth + 3))):at]
            if rng.random() < 0.2:
                ctx = [999] + ctx
            depth = int(rng.integers(0, 16))
            lines.append("path %d %d %s" % (depth, len(ctx), ints(ctx)))
            path = ix.search_path(ctx, depth)
            want.append(("%d %s" % (len(path), ints(path))).strip())
            md, budget = int(rng.integers(0, max_depth + 2)), int(rng.integers(1, 48))
            lines.append("tree %d %d %d %s" % (md, budget, len(ctx), ints(ctx)))
            tok, par = ix.extract_tree(ctx, md, budget)
            want.append("%d %s %s" % (len(tok), ints(tok), ints(par)))
    for _ in range(3):
        prompt, resp = synthetic_text(rng, 100), synthetic_text(rng, 150)
        lines.append("selfrep %d %s %d %s" % (len(prompt), ints(prompt), len(resp), ints(resp)))
        want.append(repr(float(D.self_repetition(prompt, resp))))
    lines.append("selfrep 0 0"); want.append("0")
    lines.append("attach 3 8 1 3 7 8 9 -1 0 0 20 21 22"); want.append("6 7 8 9 20 21 22 -1 0 0 1 3 4")
    lines.append("attach 3 4 0 3 7 8 9 -1 0 0 30 31 32"); want.append("4 7 8 9 30 -1 0 0 0")
    lines.append("bad"); want.append("0")
    got = run_lines(host_driver, lines)
    for ln, g, w_ in zip(lines, got, want):
        if ln.startswith("selfrep"):
            assert abs(float(g) - float(w_)) <= 1e-12 * max(1.0, abs(float(w_))), (ln[:60], g, w_)
        else:
            assert g.split() == w_.split(), (ln[:80], g, w_)


def test_tree_shape_selection_under_sanitizers_gives_the_oracles_answers(host_driver):
    rng = np.random.Generator(np.random.PCG64(72))
    lines, want = [], []
    for T in (1, 2, 3, 9, 40, 128):
        parents, alpha = [-1], [1.0]
        for i in range(1, T):
            parents.append(int(rng.integers(0, i)))
            alpha.append(alpha[parents[i]] * float(rng.uniform(0.1, 1.0)))
        alpha = np.asarray(alpha, dtype=np.float32)
        t_draft = np.asarray([0.0] + [float(rng.uniform(0, 0.5)) for _ in range(T - 1)], dtype=np.float32)
        tv = np.asarray([30.0 + 1.5 * max(0, k - T // 3) for k in range(1, T + 1)], dtype=np.float32)
        fl = lambda a: " ".join(repr(float(x)) for x in a)
        lines.append("order %d %s %s" % (T, ints(parents), fl(alpha)))
        order = TS.prune_order(parents, alpha)
        want.append(("%d %s" % (len(order), ints(order))).strip())
        n, nodes, thr, scores = TS.select(parents, alpha, t_draft, tv)
        lines.append("select 1 %d %s %s %s %s" % (T, ints(parents), fl(alpha), fl(t_draft), fl(tv)))
        want.append((n, thr, [1 if i in nodes else 0 for i in range(T)]))
        lines.append("select 0 %d %s %s %s %s" % (T, ints(parents), fl(alpha), fl(t_draft), fl(tv)))
        want.append(None)                          # golden-section: must run clean and return a prefix subtree
    got = run_lines(host_driver, lines)
    for ln, g, w_ in zip(lines, got, want):
        tok = g.split()
        if ln.startswith("order"):
            assert tok == w_.split(), (ln[:60], g, w_)
        elif w_ is not None:
            assert int(tok[0]) == w_[0] and abs(float(tok[1]) - w_[1]) < 1e-9 * max(1.0, w_[1]) and [int(x) for x in tok[2:]] == w_[2]
        else:
            assert int(tok[0]) >= 0 and int(tok[2]) == 1


@pytest.mark.parametrize("case", [0, 1, 2])
def test_oracle_under_sanitizers_equals_the_ordinary_build(oracle_driver, oracle_mod, tmp_path, case):
    if case == 0:
        w = W.make_custom("san_a", B=3, Hq=8, Hkv=2, D=64, T=20, seq_lens=[0, 37, 130], tree="trie", depth=5, seed=801)
    elif case == 1:
        w = W.make_custom("san_b", B=2, Hq=4, Hkv=4, D=128, T=1, seq_lens=[16, 1], tree="chain", seed=802)
    else:
        w = W.make_custom("san_c", B=1, Hq=2, Hkv=1, D=64, T=128, seq_lens=[65], tree="uniform", depth=9, seed=803)
    rng = np.random.Generator(np.random.PCG64(810 + case))
    n_rows = 7
    rows = np.stack([rng.integers(0, w.B, n_rows), rng.integers(0, w.Hq, n_rows), rng.integers(0, w.T, n_rows)], axis=1).astype(np.int32)
    V, ar = 37, 5
    logits = rng.integers(0, 1 << 16, size=(ar, V)).astype(np.uint16)          # any bit pattern: NaNs and infinities included
    head = np.asarray([w.B, w.T, w.Hq, w.Hkv, w.D, w.page_size, w.max_pages, w.num_pages, w.max_path, n_rows, V, ar], dtype=np.int32)
    src, dst = str(tmp_path / "in.bin"), str(tmp_path / "out.bin")
    with open(src, "wb") as f:
        for a in (head, w.q, w.k_tree, w.v_tree, w.k_cache, w.v_cache, w.page_table.astype(np.int32), w.seq_lens.astype(np.int32),
                  w.parents.astype(np.int32), w.draft_tokens.astype(np.int32), w.target_tokens.astype(np.int32), rows, logits):
            f.write(np.ascontiguousarray(a).tobytes())
    res = subprocess.run([oracle_driver, src, dst], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, env=ENV, timeout=300)
    assert res.returncode == 0 and "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr, res.stderr[-3000:]
    blob = open(dst, "rb").read()
    pos = 0

    def take(dtype, shape):
        nonlocal pos
        n = int(np.prod(shape)) * np.dtype(dtype).itemsize
        a = np.frombuffer(blob[pos:pos + n], dtype=dtype).reshape(shape)
        pos += n
        return a

    for b in range(w.B):
        mask, depth = oracle_mod.ancestor_mask(w.parents[b])
        assert np.array_equal(take(np.uint8, (w.T, w.T)), np.asarray(mask, dtype=np.uint8))
        assert np.array_equal(take(np.int32, (w.T,)), depth)
    ref, ref_lse = oracle_mod.tree_attn(w.q, w.k_tree, w.v_tree, w.k_cache, w.v_cache, w.page_table, w.seq_lens, w.parents)
    assert np.array_equal(take(np.float64, ref.shape), ref) and np.array_equal(take(np.float64, ref_lse.shape), ref_lse)
    rref, rlse = oracle_mod.tree_attn_rows(w.q, w.k_tree, w.v_tree, w.k_cache, w.v_cache, w.page_table, w.seq_lens, w.parents, rows)
    assert np.array_equal(take(np.float64, rref.shape), rref) and np.array_equal(take(np.float64, rlse.shape), rlse)
    al, path, bonus = oracle_mod.accept_path(w.draft_tokens, w.target_tokens, w.parents, w.max_path)
    assert np.array_equal(take(np.int32, al.shape), al) and np.array_equal(take(np.int32, path.shape), path)
    assert np.array_equal(take(np.int32, bonus.shape), bonus)
    kc, vc, sl = w.k_cache.copy(), w.v_cache.copy(), w.seq_lens.copy()
    oracle_mod.kv_compact(w.k_tree, w.v_tree, path, al, kc, vc, w.page_table, sl)
    assert np.array_equal(take(np.uint16, kc.shape), kc) and np.array_equal(take(np.uint16, vc.shape), vc)
    assert np.array_equal(take(np.int32, sl.shape), sl)
    assert np.array_equal(take(np.int32, (ar,)), oracle_mod.target_argmax(logits))
    assert pos == len(blob)
