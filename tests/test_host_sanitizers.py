"""The library's host-side C++ (strategy selector, n-gram drafter, static template) and the oracle's C
acceptance rules under AddressSanitizer + UndefinedBehaviorSanitizer (host compiler, no GPU): a small
driver program built with -fsanitize=address,undefined is fed the host parity cases and must print what
the Python oracles compute, bad arguments included, without a sanitizer report."""
import os
import subprocess

import numpy as np
import pytest

from oracle import accept as oa
from oracle import sample_draft as osd
from oracle.mab import BEG
from oracle.ngram import NGramDB
from synth import synthetic_logits, uniforms_u32


@pytest.fixture(scope="module")
def driver(repo_root, tmp_path_factory):
    out = tmp_path_factory.mktemp("san")
    csrc = os.path.join(repo_root, "paper_2511_16665_amd", "csrc")
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
    obj = str(out / "accept.o")
    subprocess.check_call(["gcc", *san, "-std=c11", "-ffp-contract=off", "-c", os.path.join(repo_root, "oracle", "accept.c"), "-o", obj])
    exe = str(out / "host_sanitize")
    subprocess.check_call(["g++", *san, "-std=c++17", "-static-libasan", "-static-libubsan",
                           os.path.join(repo_root, "tests", "host_sanitize_main.cpp"), os.path.join(csrc, "mab.cpp"),
                           os.path.join(csrc, "ngram.cpp"), os.path.join(csrc, "tmpl.cpp"), obj, "-o", exe, "-lm"])

    def run(text):
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
        r = subprocess.run([exe], input=text, capture_output=True, text=True, env=env, timeout=300)
        assert r.returncode == 0 and "Sanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-3000:]
        return r.stdout.split("\n")
    return run


def test_template_under_sanitizers(driver):
    cases = [(1, 4, 3), (2, 2, 4), (2, 4, 8), (3, 4, 25), (8, 6, 48), (10, 8, 64), (16, 16, 64), (2, 16, 64), (5, 1, 64), (3, 3, 1)]
    bad = [(0, 2, 4), (17, 2, 4), (2, -1, 4), (2, 17, 4), (2, 2, 0), (2, 2, 65)]
    lines = driver("".join(f"tmpl {K} {D} {N}\n" for K, D, N in cases + bad))
    for (K, D, N), line in zip(cases, lines):
        v = [int(x) for x in line.split()]
        p, r, d = osd.static_template(K, D, N)
        n = len(p)
        assert v[0] == 0 and v[1] == n and v[2:2 + n] == list(p) and v[2 + n:2 + 2 * n] == list(r) and v[2 + 2 * n:] == list(d)
    for line in lines[len(cases):len(cases) + len(bad)]:
        assert line.split()[0] == "-1"


def test_selector_under_sanitizers(driver):
    rng = np.random.default_rng(3)
    strategies = [(4, 2, 8), (6, 8, 32), (2, 2, 8), (8, 8, 32), (3, 3, 16)]
    thresholds, eps, w, thr = [1, 4, 16], 0.3, 3, 24
    ref = BEG(strategies, thresholds, eps, w, thr)
    ops, want = [], []
    for step in range(300):
        B = int(rng.integers(0, 40))
        u1, u2 = int(rng.integers(2 ** 32)), int(rng.integers(2 ** 32))
        s = ref.select(B, u1, u2)
        ops.append(f"s {B} {u1} {u2}")
        want.append(("s", -1 if s is None else s))
        if s is None or B == 0:
            continue
        lens = rng.integers(0, strategies[s][0] + 1, size=B).tolist()
        t = float(rng.uniform(1e-3, 5e-2))
        ops.append(f"r {s} {t!r} {B} " + " ".join(map(str, lens)))
        want.append(("r",) + ref.record(s, t, lens, B))
        ops.append(f"m {s}")
        want.append(("m", ref.median(ref.R[s]), len(ref.R[s])))
    ops += ["r 9 0.1 1 1", "r 0 0.0 1 1", "r 0 0.1 1 -1"]                     # no such strategy, no time, negative length
    head = f"mab {len(strategies)} " + " ".join(f"{d} {k} {n}" for d, k, n in strategies) + f" {len(thresholds)} " + \
        " ".join(map(str, thresholds)) + f" {eps} {w} {thr} {len(ops)}\n"
    lines = driver(head + "\n".join(ops) + "\nmab 1 4 2 0 1 1 0.1 4 32 0\n")      # second: a strategy verifying 0 tokens
    assert lines[0] == "0"
    for wv, line in zip(want, lines[1:]):
        v = line.split()
        assert v[0] == "0"
        if wv[0] == "s":
            assert int(v[1]) == wv[1]
        elif wv[0] == "r":
            assert float(v[1]) == wv[1] and float(v[2]) == wv[2]                # bit-identical doubles (17 digits)
        else:
            assert float(v[1]) == wv[1] and int(v[2]) == wv[2]
    tail = lines[1 + len(want):]
    assert [t.split()[0] for t in tail[:3]] == ["-1", "-1", "-1"] and tail[3] == "-1"


def test_ngram_drafter_under_sanitizers(driver):
    rng = np.random.default_rng(1)
    order, vocab = 4, 12
    ref = NGramDB(order)
    ins, props, want = [], [], []
    for p in range(3):
        phrases = [rng.integers(0, vocab, size=int(rng.integers(3, 9))).tolist() for _ in range(4)]
        for _ in range(3):
            s = []
            while len(s) < 60:
                s += phrases[int(rng.integers(len(phrases)))] if rng.random() < 0.7 else rng.integers(0, vocab, size=2).tolist()
            ref.insert(p, s[:60])
            ins.append(f"{p} 60 " + " ".join(map(str, s[:60])))
        probe = phrases[0] + phrases[1]
        for pos in range(1, len(probe), 2):
            K, D, N = int(rng.integers(1, 5)), int(rng.integers(0, 6)), int(rng.integers(1, 20))
            ctx = probe[max(0, pos - 5):pos]
            props.append(f"{p} {len(ctx)} " + " ".join(map(str, ctx)) + f" {D} {K} {N}")
            want.append(ref.propose(p, ctx, D, K, N))
    props += ["0 0 2 2 4", "0 1 1 2 0 4", "99 1 3 4 2 3"]                          # empty context, topk 0, unknown prompt
    lines = driver(f"ngram {order} {len(ins)}\n" + "\n".join(ins) + f"\n{len(props)}\n" + "\n".join(props) + "\nngram 1 0 0\n")
    assert lines[0] == "0"
    for (tok, par, sc), line in zip(want, lines[1:]):
        v = line.split()
        n = len(tok)
        assert v[0] == "0" and [int(x) for x in v[1:1 + n]] == tok and [int(x) for x in v[1 + n:1 + 2 * n]] == par
        np.testing.assert_array_equal(np.array([float(x) for x in v[1 + 2 * n:]], dtype=np.float32), np.asarray(sc, dtype=np.float32))
    tail = lines[1 + len(want):]
    assert tail[0].split()[0] == "-1" and tail[1].split()[0] == "-1"
    assert tail[2].split() == ["0", "3", "0", "1", "-1", "0", "0", "0", "-inf", "-inf"]   # root + padding
    assert tail[3] == "-1"                                                                # order 1 is refused


@pytest.mark.parametrize("mode", [0, 1, 2])
def test_acceptance_rules_under_sanitizers(driver, mode):
    B, n, V, stride, tau = 5, 9, 23, 4, 0.8
    rng = np.random.default_rng(mode)
    logits = synthetic_logits((B, n, V), seed=mode + 1)
    ql = logits + rng.standard_normal(size=logits.shape).astype(np.float32)
    q = np.exp(ql - ql.max(axis=-1, keepdims=True))
    q = (q / q.sum(axis=-1, keepdims=True)).astype(np.float32)
    token = rng.integers(0, V, size=(B, n)).astype(np.int32)
    parent = np.full((B, n), -1, dtype=np.int32)
    parent[:, 1:] = (np.arange(1, n) - 1) // 2
    token[0, 1], token[1, 2] = -1, V + 3                                # outside the vocabulary: skipped, never indexed
    if mode == 0:
        token[:, 1] = logits[:, 0].argmax(-1)                           # some greedy accepts
    u_acc, u_fin = uniforms_u32((B, n), 5), uniforms_u32((B,), 6)
    flat = lambda a, f="{}": " ".join(f.format(x) for x in np.asarray(a).ravel().tolist())
    text = f"accept {mode} {B} {n} {V} {stride} {tau}\n{flat(token)}\n{flat(parent)}\n{flat(logits, '{!r}')}\n{flat(q, '{!r}')}\n" \
           f"{flat(u_acc)}\n{flat(u_fin)}\n"
    lines = driver(text)
    if mode == 0:
        want = oa.accept_greedy(token, parent, logits, stride) + (np.zeros(B, np.int32),)
    elif mode == 1:
        want = oa.accept_sample(token, parent, logits, q, u_acc, u_fin, tau, stride, with_near=True)
    else:
        want = oa.accept_target_only(token, parent, logits, u_acc, u_fin, tau, stride, with_near=True)
    al, path, out, n_out, near = want
    for b in range(B):
        v = [int(x) for x in lines[b].split()]
        assert v[0] == al[b] and v[1] == n_out[b] and v[2] == near[b]
        assert v[3::2] == path[b].tolist() and v[4::2] == out[b].tolist()
