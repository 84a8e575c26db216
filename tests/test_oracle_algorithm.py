"""Pins for the oracle's Algorithm 1: what the paper and the method's definition fix about the schedule.

1. Output parity: AdaDecode's tokens equal plain greedy decoding's (Sec. 4.2), by brute force over
   thresholds, caps, forced schedules and scripted wrong drafts.
2. Deferred layers computed later, in parallel, leave the same KV cache as sequential decoding (Sec. 2.2).
3. The worked example of Fig. 2 (left), and the gamma = 0 / gamma = 1 extremes of Sec. 4.4.
4. Bookkeeping identities that hold for any run.
"""
import os

import numpy as np
import pytest

from oracle import oracle as orc
from paper_2506_03700_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")

UNTIED = synth.TINY.with_(name="tiny-untied", tied_head=False, vocab=512, exit_layers=(1, 2, 3))
SHAPES = {s.name: s for s in (synth.TINY, UNTIED, synth.TINY_GQA)}
_cache = {}


def model(name, seed=0):
    key = (name, seed)
    if key not in _cache:
        s = SHAPES[name]
        w = synth.make_weights(s, seed)
        o = orc.Oracle(s, w, max_pos=256)
        p = synth.make_prompt(s, seed, n=12)
        g, margins = o.generate_greedy(p, 48)
        kv = [o.kv_read(l, 0, 12 + 47) for l in range(1, s.n_layers + 1)]
        _cache[key] = (s, o, p, g, kv)
    return _cache[key]


def steps(ev):
    return [(int(e["layer"]), int(e["pos"]), int(e["m"])) for e in ev if e["kind"] == orc.EV_LAYER_STEP]


def check_bookkeeping(s, ev, st, n_prompt, cap):
    L = s.n_layers
    ls = steps(ev)
    assert st["layer_steps"] == len(ls) and st["layer_step_rows"] == sum(m for _, _, m in ls)
    assert all(1 <= m <= cap + 1 for _, _, m in ls)
    # every (layer, position) that is processed is processed in order, restarting only after a rollback
    length = [n_prompt - 1] * (L + 1)
    n_tokens_entered = 0
    for e in ev:
        if e["kind"] == orc.EV_LAYER_STEP:
            l, p, m = int(e["layer"]), int(e["pos"]), int(e["m"])
            assert p == length[l], "a layer step must continue that layer's cache"
            length[l] += m
            if l == 1:
                assert m == 1                      # only the current token is ever pending at layer 1
                n_tokens_entered += 1
            # deeper layers never run ahead of shallower ones
            assert all(length[a] >= length[a + 1] for a in range(1, L))
        elif e["kind"] == orc.EV_VERIFY:
            assert len(set(length[1:])) == 1       # at a verification every layer has caught up
            keep = int(e["pos"]) + int(e["flag"]) + 1
            length = [min(x, keep) for x in length]
    # each token that entered the model went through each layer exactly once
    assert st["layer_step_rows"] == L * n_tokens_entered
    assert st["early_preds"] == sum(1 for e in ev if e["kind"] == orc.EV_HEAD and e["flag"] == 1)
    assert st["verifies"] == sum(1 for e in ev if e["kind"] == orc.EV_VERIFY)
    assert n_tokens_entered == st["tokens"] + st["rejections"] + st["rolled_back"]


@pytest.mark.parametrize("name", list(SHAPES))
@pytest.mark.parametrize("cap", [1, 5, 7])
@pytest.mark.parametrize("gamma", [0.0, 0.004, 0.05, 0.5, 0.9, 1.0])
def test_parity_with_greedy_by_threshold(name, cap, gamma):
    s, o, p, g, kv = model(name)
    a, st, ev = o.generate_ada(p, 48, gamma, cap)
    np.testing.assert_array_equal(a, g)
    check_bookkeeping(s, ev, st, len(p), cap)
    # invariant 2: the cache equals the sequential run's, at every layer, for every kept position
    n = min(o.kv_lens())
    assert n >= len(p) + 47 - 1
    for l in range(1, s.n_layers + 1):
        k, v = o.kv_read(l, 0, len(p) + 46)
        np.testing.assert_allclose(k, kv[l - 1][0][:len(p) + 46], rtol=0, atol=1e-12)
        np.testing.assert_allclose(v, kv[l - 1][1][:len(p) + 46], rtol=0, atol=1e-12)


@pytest.mark.parametrize("name", list(SHAPES))
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_parity_under_forced_schedules_and_wrong_drafts(name, seed):
    s, o, p, g, kv = model(name)
    k = len(s.exit_layers)
    forced = synth.make_forced_schedule(s, seed, 256, probs=[0.6 / k] * k)
    a, st, ev = o.generate_ada(p, 48, 0.9, 7, forced_exit=forced)
    np.testing.assert_array_equal(a, g)
    check_bookkeeping(s, ev, st, len(p), 7)
    assert st["early_preds"] > 5 and max(m for _, _, m in steps(ev)) >= 3
    # scripted wrong drafts at a third of the positions: each one must be rejected and repaired
    rng = np.random.default_rng(seed)
    script = np.full(256, -1, dtype=np.int32)
    idx = rng.choice(np.arange(len(p) - 1, len(p) + 47), size=16, replace=False)
    script[idx] = rng.integers(0, s.vocab, size=16)
    a2, st2, ev2 = o.generate_ada(p, 48, 0.9, 5, forced_exit=forced, scripted_draft=script)
    np.testing.assert_array_equal(a2, g)
    check_bookkeeping(s, ev2, st2, len(p), 5)
    assert st2["rejections"] >= 3
    for l in range(1, s.n_layers + 1):
        kk, vv = o.kv_read(l, 0, len(p) + 46)
        np.testing.assert_allclose(kk, kv[l - 1][0][:len(p) + 46], rtol=0, atol=1e-12)
        np.testing.assert_allclose(vv, kv[l - 1][1][:len(p) + 46], rtol=0, atol=1e-12)


def test_fig2_left_worked_example():
    # 3 layers with heads at layers 1 and 2; t1 (the last prompt token) exits at layer 2, t2 at layer 1.
    with open(os.path.join(GOLDEN, "fig2_left_trace.txt")) as f:
        want = [line.split() for line in f if line.strip() and not line.startswith("#")]
    s = synth.TINY.with_(n_layers=3, exit_layers=(1, 2))
    w = synth.make_weights(s, 4)
    o = orc.Oracle(s, w, max_pos=64)
    p = synth.make_prompt(s, 4, n=6)
    forced = np.zeros(64, dtype=np.uint8)
    forced[5], forced[6] = 2, 1                    # positions of t1 and t2
    a, st, ev = o.generate_ada(p, 3, 0.9, 5, forced_exit=forced)
    name = {5: "t1", 6: "t2", 7: "t3"}
    got = [[str(l)] + [name[q] for q in range(pos, pos + m)] for l, pos, m in steps(ev)]
    assert got == want
    assert st["layer_steps"] == 6 and st["layer_step_rows"] == 9 and st["verifies"] == 1
    np.testing.assert_array_equal(a, o.generate_greedy(p, 3)[0])


@pytest.mark.parametrize("name", list(SHAPES))
def test_gamma_extremes(name):
    s, o, p, g, kv = model(name)
    L = s.n_layers
    # gamma = 1: no probability exceeds 1, so there are no early predictions and the step list is the
    # sequential one: every token through layers 1..L alone, then a one-row verification
    a, st, ev = o.generate_ada(p, 20, 1.0, 5)
    assert st["early_preds"] == 0 and st["rejections"] == 0 and st["verifies"] == 20
    assert steps(ev) == [(l, len(p) - 1 + i, 1) for i in range(20) for l in range(1, L + 1)]
    # gamma = 0: every head evaluation exits (a softmax probability is positive), always at the first
    # head layer, until the cap forces a full-depth token
    cap = 3
    a, st, ev = o.generate_ada(p, 21, 0.0, cap)
    heads = [e for e in ev if e["kind"] == orc.EV_HEAD]
    assert all(e["flag"] == 1 and e["layer"] == s.exit_layers[0] for e in heads)
    ver = [e for e in ev if e["kind"] == orc.EV_VERIFY]
    assert all(e["m"] == cap + 1 for e in ver[:-1])
    np.testing.assert_array_equal(a, g[:21])


def test_budget_and_eos_rules():
    s, o, p, g, kv = model("tiny-untied")
    for n in (1, 2, 3, 7):
        a, st, ev = o.generate_ada(p, n, 0.0, 5)
        np.testing.assert_array_equal(a, g[:n])            # exactly n tokens, all verified
        assert ev[-1]["kind"] == orc.EV_VERIFY_ROW
    # stop at an EOS id: take the 6th greedy token as EOS; generation ends with its first occurrence
    eos = int(g[5])
    first = int(np.argmax(g == eos))
    a, st, ev = o.generate_ada(p, 48, 0.0, 5, eos_id=eos)
    np.testing.assert_array_equal(a, g[:first + 1])
    ge, _ = o.generate_greedy(p, 48, eos_id=eos)
    np.testing.assert_array_equal(ge, g[:first + 1])
    # an early prediction of EOS is never taken: no HEAD event fires with that token
    assert not any(e["kind"] == orc.EV_HEAD and e["flag"] == 1 and e["token"] == eos for e in ev)


def test_rejection_accounting():
    s, o, p, g, kv = model("tiny-untied")
    # all tokens exit at the first head; every draft is scripted to the right (greedy) token except the
    # 3rd early prediction, which is scripted wrong
    forced = np.full(256, s.exit_layers[0], dtype=np.uint8)
    script = np.full(256, -1, dtype=np.int32)
    script[len(p) - 1:len(p) - 1 + 48] = g            # the token after position M-1+i is g[i]
    bad_pos = len(p) - 1 + 2
    script[bad_pos] = (int(g[2]) + 1) % s.vocab
    a, st, ev = o.generate_ada(p, 30, 0.9, 5, forced_exit=forced, scripted_draft=script)
    np.testing.assert_array_equal(a, g[:30])
    ver = [e for e in ev if e["kind"] == orc.EV_VERIFY]
    # first verification: 6 rows (cap 5), drafts 0 and 1 accepted, draft 2 rejected, 2 later drafts dropped
    assert (ver[0]["m"], ver[0]["flag"], ver[0]["token"]) == (6, 2, g[2])
    assert st["rejections"] == 1 and st["rolled_back"] == 2
    rows = [e for e in ev if e["kind"] == orc.EV_VERIFY_ROW][:6]
    assert [int(e["flag"]) for e in rows] == [1, 1, 0, -1, -1, -1]
    # after the rollback every layer's cache ends right after the last accepted row
    k_first_ver = [i for i, e in enumerate(ev) if e["kind"] == orc.EV_VERIFY][0]
    nxt = [e for e in ev[k_first_ver:] if e["kind"] == orc.EV_LAYER_STEP][0]
    assert (nxt["layer"], nxt["pos"], nxt["m"]) == (1, bad_pos + 1, 1)


# ---- ablation switches (Table 3 of the paper, in shape only): a single exit head, no verification ------------

def test_head_mask_with_one_bit_is_the_one_head_model():
    s, o, p, g, kv = model("tiny-untied")                      # heads at layers 1, 2, 3
    w = synth.make_weights(s, 0)
    for i, layer in enumerate(s.exit_layers):
        one = s.with_(name=f"one-head-{layer}", exit_layers=(layer,))
        o1 = orc.Oracle(one, w, max_pos=256)
        for gamma, cap in [(0.0, 5), (0.004, 7)]:
            a, st, ev = o.generate_ada(p, 40, gamma, cap, head_mask=1 << i)
            a1, st1, ev1 = o1.generate_ada(p, 40, gamma, cap)
            np.testing.assert_array_equal(a, a1)
            assert st == st1
            for f in ("kind", "layer", "pos", "m", "token", "flag"):
                np.testing.assert_array_equal(ev[f], ev1[f])
            assert {int(e["layer"]) for e in ev if e["kind"] == orc.EV_HEAD} <= {layer}
            np.testing.assert_array_equal(a, g[:40])            # still exactly greedy decoding
        o1.close()
    # every bit set is the same as no mask
    a, st, ev = o.generate_ada(p, 40, 0.004, 7, head_mask=0b111)
    a0, st0, ev0 = o.generate_ada(p, 40, 0.004, 7)
    assert st == st0 and np.array_equal(ev["flag"], ev0["flag"]) and np.array_equal(a, a0)


def test_no_verify_keeps_drafts_unchecked():
    s, o, p, g, kv = model("tiny-untied")
    n = 30
    # without early predictions there is nothing to verify: the run is plain decoding, one final-head row per token
    a, st, ev = o.generate_ada(p, n, 1.0, 5, no_verify=True)
    np.testing.assert_array_equal(a, g[:n])
    assert st["early_preds"] == 0 and st["verifies"] == n and st["rejections"] == 0
    # drafts that happen to be right (scripted to the greedy tokens): same output, nothing rolled back
    forced = np.full(256, s.exit_layers[0], dtype=np.uint8)
    script = np.full(256, -1, dtype=np.int32)
    script[len(p) - 1:len(p) - 1 + 48] = g
    a, st, ev = o.generate_ada(p, n, 0.9, 5, forced_exit=forced, scripted_draft=script, no_verify=True)
    np.testing.assert_array_equal(a, g[:n])
    assert st["early_preds"] > 10 and st["rejections"] == 0 and st["rolled_back"] == 0
    check_bookkeeping(s, ev, st, len(p), 5)
    # one wrong draft, at the k-th generated token, everything else at full depth: it is emitted as it is, and what
    # follows is plain decoding from the sequence that contains it (brute force: greedy decoding of that prefix)
    k = 7
    bad_pos = len(p) - 1 + k
    forced = np.zeros(256, dtype=np.uint8)
    forced[bad_pos] = s.exit_layers[1]
    script = np.full(256, -1, dtype=np.int32)
    wrong = (int(g[k]) + 5) % s.vocab
    script[bad_pos] = wrong
    a, st, ev = o.generate_ada(p, n, 0.9, 5, forced_exit=forced, scripted_draft=script, no_verify=True)
    np.testing.assert_array_equal(a[:k], g[:k])
    assert a[k] == wrong and st["rejections"] == 0 and st["early_preds"] == 1
    cache = [o.kv_read(l, 0, len(p) + n - 1) for l in range(1, s.n_layers + 1)]
    o2 = orc.Oracle(s, o.weights, max_pos=256)
    cont, _ = o2.generate_greedy(np.concatenate([p, a[:k + 1]]), n - k - 1)
    np.testing.assert_array_equal(a[k + 1:], cont)
    # ... and the cache is the sequential one of prompt + output
    for l in range(1, s.n_layers + 1):
        k2, v2 = o2.kv_read(l, 0, len(p) + n - 1)
        np.testing.assert_allclose(cache[l - 1][0], k2, rtol=0, atol=1e-12)
        np.testing.assert_allclose(cache[l - 1][1], v2, rtol=0, atol=1e-12)
    o2.close()
    # with verification the same schedule repairs the token
    a, st, ev = o.generate_ada(p, n, 0.9, 5, forced_exit=forced, scripted_draft=script)
    np.testing.assert_array_equal(a, g[:n])
    assert st["rejections"] == 1


def test_restart_from_kept_cache_rows_equals_a_run_from_scratch():
    # A cache row depends on the tokens up to its position only, so a run whose prompt extends an earlier run's
    # prompt by that run's own verified tokens may take the shared rows over (keep_cache): every event, token and
    # cache entry must equal those of the same call made on an empty cache.
    shape = synth.TINY.with_(name="tiny-untied", tied_head=False, vocab=512, exit_layers=(1, 2, 3))
    w = synth.make_weights(shape, seed=0)
    p = synth.make_prompt(shape, 0)[:12]
    forced = synth.make_forced_schedule(shape, 1, 96, probs=[0.2, 0.2, 0.2])
    a, b = orc.Oracle(shape, w, max_pos=96), orc.Oracle(shape, w, max_pos=96)
    t0, _, _ = a.generate_ada(p, 40, 0.9, 5, forced_exit=forced)
    for j in (1, 7, 23):
        p2 = np.concatenate([p, t0[:j]])
        keep = len(p2) - 1                       # rows of every prompt position but the last are in a's cache
        ta, sa, ea = a.generate_ada(p2, 40 - j, 0.9, 5, forced_exit=forced, keep_cache=keep)
        tb, sb, eb = b.generate_ada(p2, 40 - j, 0.9, 5, forced_exit=forced)
        np.testing.assert_array_equal(ta, tb)
        np.testing.assert_array_equal(ta, t0[j:])
        assert sa == sb and ea.tobytes() == eb.tobytes()
        n = min(a.kv_lens())
        assert a.kv_lens() == b.kv_lens()
        for l in (1, shape.n_layers):
            ka, va = a.kv_read(l, 0, n)
            kb, vb = b.kv_read(l, 0, n)
            np.testing.assert_array_equal(ka, kb)
            np.testing.assert_array_equal(va, vb)
        # what must be refused: more rows than the prompt's own, or more than the cache holds
        a.generate_ada(p2, 40 - j, 0.9, 5, forced_exit=forced)
    with pytest.raises(RuntimeError):
        a.generate_ada(p, 8, 0.9, 5, keep_cache=len(p))
    a.kv_truncate(3)
    with pytest.raises(RuntimeError):
        a.generate_ada(p, 8, 0.9, 5, keep_cache=5)
