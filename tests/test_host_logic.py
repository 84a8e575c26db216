"""CPU-only tests of the library's host side: the C ABI exports, argument checks that need no GPU, and the
host scheduler (Algorithm 1) driven through a scripted backend -- including a replay of the oracle's
recorded decisions, which the scheduler must reproduce event for event."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import oracle as orc
from paper_2506_03700_amd import binding as ad
from paper_2506_03700_amd import build as ad_build
from paper_2506_03700_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def _built():
    ad_build.build_sched_test(force=False)


def test_library_exports_every_declared_symbol():
    if not os.path.exists(ad.LIB_PATH):
        ad_build.build_hip(force=False)
    header = open(os.path.join(ROOT, "include", "adadecode.h")).read()
    declared = set(re.findall(r"\b(ad_[a-z_]+)\s*\(", header))
    assert declared == set(ad.EXPORTS)
    L = C.CDLL(ad.LIB_PATH)
    for name in declared:
        assert hasattr(L, name), name


def test_size_queries_and_config_checks_without_gpu():
    L = ad.lib()
    cfg = ad.make_config(synth.LLAMA8B)
    ws = L.ad_workspace_bytes(C.byref(cfg))
    # the library keeps one copy of every weight (same bytes as the originals for bf16), room for one d x d
    # transform per exit head (Sec. 2.1), the logits of up to 8 draft and 8 final rows for sampled decoding, and
    # small scratch
    s = synth.LLAMA8B
    weights = (s.n_layers * s.layer_weight_elems() + 2 * s.vocab * s.d_model + len(s.exit_layers) * s.d_model ** 2) * 2
    logits = 2 * 8 * s.vocab * 4
    assert weights + logits <= ws <= weights + logits + (8 << 20)
    kvb = L.ad_kv_bytes(C.byref(cfg), 4096 + 8)
    assert kvb >= s.n_layers * 2 * s.n_kv_heads * s.head_dim * (4096 + 8) * 2
    # per cached position, one layer reads K and V rows of 2 * Hkv * dh * 2 bytes = 4096 B (8B shape)
    assert 2 * s.n_kv_heads * s.head_dim * s.elem_bytes() == 4096
    bad = ad.make_config(synth.LLAMA8B.with_(head_dim=96))
    assert L.ad_workspace_bytes(C.byref(bad)) == 0 and b"head_dim" in L.ad_last_error()
    bad = ad.make_config(synth.TINY.with_(exit_layers=(4,)))
    assert L.ad_workspace_bytes(C.byref(bad)) == 0 and b"exit layer" in L.ad_last_error()
    bad = ad.make_config(synth.TINY, m_max=9)
    assert L.ad_workspace_bytes(C.byref(bad)) == 0
    assert L.ad_kv_bytes(C.byref(cfg), 0) == 0
    assert L.ad_model_create(None, None, None, None, 0, None, None) == ad.AD_EINVAL
    assert L.ad_kv_truncate(None, 0) == ad.AD_EINVAL


# ---- scheduler over scripted heads -------------------------------------------------------------------

def _events(ev):
    return [(int(e["kind"]), int(e["layer"]), int(e["pos"]), int(e["m"]), int(e["token"]), int(e["flag"])) for e in ev]


def test_fig2_left_schedule():
    # 3 layers, heads at 1 and 2; position 5 (t1) exits at layer 2, position 6 (t2) at layer 1
    n_pos = 16
    head_tok = np.zeros((n_pos, 2), dtype=np.int32)
    head_conf = np.zeros((n_pos, 2), dtype=np.float32)
    final_tok = np.arange(100, 100 + n_pos, dtype=np.int32)       # the token after position p is 100 + p
    head_tok[5] = [0, 105]; head_conf[5] = [0.1, 0.95]
    head_tok[6] = [106, 0]; head_conf[6] = [0.99, 0.0]
    rc, out, st, ev = ad.sched_test_run(3, [1, 2], 8, head_tok, head_conf, final_tok, prompt=[1, 2, 3, 4, 5, 6], max_new=3,
                                        gamma=0.9, max_pending=5)
    assert rc == ad.AD_OK and list(out) == [105, 106, 107]
    steps = [(l, p, m) for k, l, p, m, _, _ in _events(ev) if k == ad.EV_LAYER_STEP]
    assert steps == [(1, 5, 1), (2, 5, 1), (1, 6, 1), (1, 7, 1), (2, 6, 2), (3, 5, 3)]
    assert st["layer_steps"] == 6 and st["layer_step_rows"] == 9 and st["early_preds"] == 2 and st["verifies"] == 1
    assert st["steps_by_m"][1:4] == [4, 1, 1]


def _check_stretches(ev, n_layers):
    """The backend gets the layer steps as stretches: expanded, they are the run's layer steps in order; a stretch ends
    at the last layer, at a layer after which a head was evaluated, or where the next layer's step has other rows."""
    evs = _events(ev)
    steps = [(l, p, m) for k, l, p, m, _, _ in evs if k == ad.EV_LAYER_STEP]
    st = ad.sched_test_stretches()
    expanded = [(int(f) + i, int(p0), int(m)) for f, c, r0, m, p0 in st for i in range(int(c))]
    assert expanded == steps
    # the event that follows each stretch's last layer step
    idx = [i for i, e in enumerate(evs) if e[0] == ad.EV_LAYER_STEP]
    at = 0
    for f, c, r0, m, p0 in st:
        last = idx[at + int(c) - 1]
        at += int(c)
        layer = int(f) + int(c) - 1
        nxt = evs[last + 1] if last + 1 < len(evs) else None
        if layer == n_layers:
            continue
        assert nxt is not None
        if nxt[0] == ad.EV_LAYER_STEP:
            # no head in between: the next step must be this token's next layer with more rows (deferred rows join)
            assert nxt[1] == layer + 1 and nxt[3] > int(m)
        else:
            assert nxt[0] == ad.EV_HEAD and nxt[1] == layer
    return st


def test_layer_steps_reach_the_backend_as_maximal_stretches():
    # 12 layers, heads at 4 and 8: a token that goes to full depth alone is three stretches (1-4, 5-8, 9-12); after an
    # exit at layer 4 the next token runs 1-4 alone, then both rows 5-8 and 9-12
    n_pos = 32
    head_tok = np.zeros((n_pos, 2), dtype=np.int32)
    head_conf = np.zeros((n_pos, 2), dtype=np.float32)
    final_tok = np.arange(100, 100 + n_pos, dtype=np.int32)
    head_tok[3] = [103, 0]; head_conf[3] = [0.99, 0.0]          # position 3 exits at layer 4 with the right token
    head_tok[5] = [0, 105]; head_conf[5] = [0.0, 0.99]          # position 5 exits at layer 8
    rc, out, stt, ev = ad.sched_test_run(12, [4, 8], 8, head_tok, head_conf, final_tok, prompt=[1, 2, 3, 4], max_new=6,
                                         gamma=0.9, max_pending=5)
    assert rc == ad.AD_OK and list(out) == [103, 104, 105, 106, 107, 108]
    st = _check_stretches(ev, 12)
    assert [tuple(int(v) for v in r) for r in st[:7]] == [
        (1, 4, 0, 1, 3),            # position 3 alone up to the head at 4: exits
        (1, 4, 1, 1, 4),            # position 4 alone up to the head at 4 (stays)
        (5, 4, 0, 2, 3),            # both rows, layers 5-8 (head at 8: stays)
        (9, 4, 0, 2, 3),            # both rows to the last layer: verified
        (1, 4, 0, 1, 5), (5, 4, 0, 1, 5),    # position 5 exits at layer 8
        (1, 4, 1, 1, 6)]
    # with the exits switched off (gamma 1 never fires but the heads are still evaluated) the stretches are the same
    # three per token; with no heads in the schedule at all (head_mask cannot be empty, so: a cap of 0) one per token
    rc, out, stt, ev = ad.sched_test_run(12, [4, 8], 8, head_tok, head_conf, final_tok, prompt=[1, 2, 3, 4], max_new=3,
                                         gamma=0.9, max_pending=0)
    assert rc == ad.AD_OK
    st = _check_stretches(ev, 12)
    assert [tuple(int(v) for v in r) for r in st] == [(1, 12, 0, 1, 3), (1, 12, 0, 1, 4), (1, 12, 0, 1, 5)]
    # a single head (the fixed-layer variant): stretches 1-8 and 9-12
    rc, out, stt, ev = ad.sched_test_run(12, [4, 8], 8, head_tok, head_conf, final_tok, prompt=[1, 2, 3, 4], max_new=2,
                                         gamma=0.9, max_pending=5, head_mask=2)
    assert rc == ad.AD_OK
    st = _check_stretches(ev, 12)
    assert [tuple(int(v) for v in r) for r in st[:2]] == [(1, 8, 0, 1, 3), (9, 4, 0, 1, 3)]


def test_threshold_is_strict_and_cap_and_budget():
    n_pos, L = 64, 4
    final_tok = (np.arange(n_pos) * 7 % 50).astype(np.int32)
    head_tok = final_tok[:, None].copy()                           # the head always drafts the right token
    head_conf = np.full((n_pos, 1), 0.9, dtype=np.float32)
    prompt = [3, 1, 4, 1, 5]
    # conf == gamma does not exit (Eq. 1 uses >)
    rc, out, st, ev = ad.sched_test_run(L, [2], 8, head_tok, head_conf, final_tok, prompt, 10, np.float32(0.9), 5)
    assert rc == ad.AD_OK and st["early_preds"] == 0 and st["head_evals"] == 9
    assert list(out) == list(final_tok[4:14])
    # just below: every token exits until the cap of 3 unverified drafts, then one runs to depth L
    rc, out, st, ev = ad.sched_test_run(L, [2], 8, head_tok, head_conf, final_tok, prompt, 10, 0.89, 3)
    assert rc == ad.AD_OK and list(out) == list(final_tok[4:14])
    ver = [e for e in _events(ev) if e[0] == ad.EV_VERIFY]
    assert [v[3] for v in ver] == [4, 4, 2] and all(v[5] == v[3] - 1 for v in ver)    # all drafts accepted
    # budget: the last token is never drafted -> last verify has the remaining rows only, 10 tokens exactly
    assert st["tokens"] == 10 and st["early_preds"] == 7 and st["rejections"] == 0
    # max_pending = 0 is plain sequential decoding, no head is ever evaluated
    rc, out, st, ev = ad.sched_test_run(L, [2], 8, head_tok, head_conf, final_tok, prompt, 6, 0.0, 0)
    assert st["head_evals"] == 0 and st["layer_steps"] == 6 * L and list(out) == list(final_tok[4:10])
    # a cap that would need more rows than m_max is refused
    rc, *_ = ad.sched_test_run(L, [2], 4, head_tok, head_conf, final_tok, prompt, 6, 0.0, 4)
    assert rc == ad.AD_ERANGE


def test_rejection_rolls_back_and_resumes():
    n_pos, L = 64, 4
    final_tok = (np.arange(n_pos) * 11 % 97).astype(np.int32)
    head_tok = final_tok[:, None].copy()
    head_conf = np.ones((n_pos, 1), dtype=np.float32)
    head_tok[6, 0] = 1000                                           # wrong draft for the token after position 6
    prompt = [9, 8, 7, 6, 5]
    rc, out, st, ev = ad.sched_test_run(L, [1], 8, head_tok, head_conf, final_tok, prompt, 12, 0.5, 5)
    assert rc == ad.AD_OK and list(out) == list(final_tok[4:16])
    ver = [e for e in _events(ev) if e[0] == ad.EV_VERIFY]
    # first verification: rows at positions 4..9; drafts after 4 and 5 accepted, the one after 6 rejected
    assert ver[0][2:] == (4, 6, int(final_tok[6]), 2)
    assert st["rejections"] == 1 and st["rolled_back"] == 2
    rows = [e for e in _events(ev) if e[0] == ad.EV_VERIFY_ROW][:6]
    assert [r[5] for r in rows] == [1, 1, 0, -1, -1, -1]
    # the scripted backend checks on every layer step that the step continues the layer's (truncated) cache
    after = [e for e in _events(ev)[_events(ev).index(ver[0]):] if e[0] == ad.EV_LAYER_STEP][0]
    assert after[1:4] == (1, 7, 1)


def test_eos_only_from_the_last_layer():
    n_pos, L = 32, 3
    final_tok = np.arange(200, 200 + n_pos, dtype=np.int32)
    head_tok = final_tok[:, None].copy()
    head_conf = np.ones((n_pos, 1), dtype=np.float32)
    eos = int(final_tok[7])
    rc, out, st, ev = ad.sched_test_run(L, [1], 8, head_tok, head_conf, final_tok, [1, 2, 3], 20, 0.5, 5, eos_id=eos)
    assert rc == ad.AD_OK and list(out) == list(final_tok[2:8]) and out[-1] == eos
    assert not any(e[0] == ad.EV_HEAD and e[5] == 1 and e[4] == eos for e in _events(ev))


UNTIED = synth.TINY.with_(name="tiny-untied", tied_head=False, vocab=512, exit_layers=(1, 2, 3))


@pytest.mark.parametrize("shape", [UNTIED, synth.TINY_GQA], ids=lambda s: s.name)
@pytest.mark.parametrize("gamma,cap,forced_seed", [(0.0, 5, None), (0.0045, 7, None), (0.9, 7, 3), (0.9, 2, 4)])
def test_scheduler_replays_the_oracle_run(shape, gamma, cap, forced_seed):
    """Feed the oracle's recorded head outputs to the library's scheduler: tokens, statistics and the whole
    event sequence must be identical (the two loops are separate implementations of Algorithm 1)."""
    w = synth.make_weights(shape, 0)
    o = orc.Oracle(shape, w, max_pos=128)
    p = synth.make_prompt(shape, 0, n=10)
    forced = None if forced_seed is None else synth.make_forced_schedule(shape, forced_seed, 128, probs=[0.7 / len(shape.exit_layers)] * len(shape.exit_layers))
    script = None
    if forced_seed == 4:
        script = np.full(128, -1, dtype=np.int32)
        script[[12, 15, 21, 30]] = [1, 2, 3, 4]
    toks, st_o, ev_o = o.generate_ada(p, 40, gamma, cap, forced_exit=forced, scripted_draft=script)
    heads = ev_o[ev_o["kind"] == orc.EV_HEAD]
    rows = ev_o[ev_o["kind"] == orc.EV_VERIFY_ROW]
    # with a scripted draft the recorded token is the scripted one; the scheduler applies the script itself
    rc, out, st, ev = ad.sched_test_run(shape.n_layers, shape.exit_layers, 8, heads["token"], heads["conf"].astype(np.float32),
                                        rows["token"], p, 40, gamma, cap, forced_exit=forced, scripted_draft=script,
                                        max_pos=128, sequence=True)
    assert rc == ad.AD_OK
    _check_stretches(ev, shape.n_layers)
    np.testing.assert_array_equal(out, toks)
    for k in ("tokens", "layer_steps", "layer_step_rows", "head_evals", "verifies", "early_preds", "rejections", "rolled_back"):
        assert st[k] == st_o[k], k
    assert st["steps_by_m"] == st_o["steps_by_m"]
    assert _events(ev) == [(int(e["kind"]), int(e["layer"]), int(e["pos"]), int(e["m"]), int(e["token"]), int(e["flag"])) for e in ev_o]


def test_sampled_schedule_uses_the_draw_table_by_position_and_column():
    """Sampled decoding over a scripted backend: drafts are accepted iff their acceptance draw is below 0.5, and the
    scheduler must hand each use the draw of the right position and column of the caller's table."""
    n_pos, L = 32, 4
    final_tok = (100 + np.arange(n_pos)).astype(np.int32)
    head_tok = np.stack([200 + np.arange(n_pos), 300 + np.arange(n_pos)], axis=1).astype(np.int32)
    head_conf = np.zeros((n_pos, 2), dtype=np.float32)
    head_conf[:, 0] = 0.95                                        # every token exits at the first head (layer 1)
    u = np.zeros((n_pos, 5), dtype=np.float32)                    # columns: head 0, head 1, final, accept, replace
    u[:, 0] = 0.01 + np.arange(n_pos) * 1e-3
    u[:, 2] = 0.02 + np.arange(n_pos) * 1e-3
    u[:, 3] = 0.1                                                 # accept ...
    u[6, 3] = 0.9                                                 # ... except the token drafted after position 6
    u[:, 4] = 0.03 + np.arange(n_pos) * 1e-3
    prompt = [1, 2, 3, 4, 5]
    rc, out, st, ev, draws = ad.sched_test_run(L, [1, 3], 8, head_tok, head_conf, final_tok, prompt, 8, 0.9, 3,
                                               temperature=0.7, uniforms=u)
    assert rc == ad.AD_OK
    # positions 4, 5, 6 exit (cap 3), position 7 runs to the end; the draft after 6 is rejected -> next = final_tok[6]
    assert list(out[:3]) == [204, 205, 106] and st["rejections"] >= 1
    ver = [e for e in ev if e["kind"] == ad.EV_VERIFY]
    assert int(ver[0]["pos"]) == 4 and int(ver[0]["m"]) == 4 and int(ver[0]["flag"]) == 2 and int(ver[0]["token"]) == 106
    rows = [e for e in ev if e["kind"] == ad.EV_VERIFY_ROW][:4]
    assert [(int(r["token"]), int(r["flag"])) for r in rows] == [(204, 1), (205, 1), (106, 0), (-1, -1)]
    assert [float(r["conf"]) for r in rows] == [0.5, 0.5, 0.5, 0.0]
    assert len(out) == 8 and st["tokens"] == 8
    # the last verification of the run: check which table entries reached the backend
    last = [e for e in ev if e["kind"] == ad.EV_VERIFY][-1]
    p0, m = int(last["pos"]), int(last["m"])
    assert draws[1] == u[p0 + m - 1, 2]                           # final-layer draw of the newest row
    if m > 1:
        assert draws[2] == u[p0, 3] and draws[3] == u[p0, 4]
    heads = [e for e in ev if e["kind"] == ad.EV_HEAD]
    assert draws[0] == u[int(heads[-1]["pos"]), 0]
    # without the table a sampled run is refused
    rc, *_ = ad.sched_test_run(L, [1, 3], 8, head_tok, head_conf, final_tok, prompt, 8, 0.9, 3, temperature=0.7, uniforms=None)
    assert rc == ad.AD_EINVAL


def test_ablation_switches_in_the_scheduler():
    n_pos, L = 48, 4
    final_tok = (100 + np.arange(n_pos)).astype(np.int32)
    head_tok = np.stack([100 + np.arange(n_pos), 100 + np.arange(n_pos)], axis=1).astype(np.int32)
    head_tok[9, 0] = 7                                            # the first head drafts a wrong token after position 9
    head_conf = np.full((n_pos, 2), 0.95, dtype=np.float32)
    prompt = [1, 2, 3, 4, 5]
    # both heads on: every exit happens at the first head (layer 1)
    rc, out, st, ev = ad.sched_test_run(L, [1, 3], 8, head_tok, head_conf, final_tok, prompt, 12, 0.9, 3)
    assert rc == ad.AD_OK and {int(e["layer"]) for e in ev if e["kind"] == ad.EV_HEAD} == {1}
    assert list(out) == list(final_tok[4:16]) and st["rejections"] == 1
    # only the second head (bit 1): exits at layer 3, the wrong draft of head 0 is never seen
    rc, out, st, ev = ad.sched_test_run(L, [1, 3], 8, head_tok, head_conf, final_tok, prompt, 12, 0.9, 3, head_mask=0b10)
    assert rc == ad.AD_OK and {int(e["layer"]) for e in ev if e["kind"] == ad.EV_HEAD} == {3}
    assert list(out) == list(final_tok[4:16]) and st["rejections"] == 0 and st["early_preds"] > 0
    # no verification: the wrong draft stays in the output, nothing is rolled back, every layer still sees every token once
    rc, out, st, ev = ad.sched_test_run(L, [1, 3], 8, head_tok, head_conf, final_tok, prompt, 12, 0.9, 3, no_verify=True)
    assert rc == ad.AD_OK and st["rejections"] == 0 and st["rolled_back"] == 0
    want = list(final_tok[4:16])
    want[5] = 7                                                   # the token after position 9 is the 6th generated one
    assert list(out) == want
    assert st["layer_step_rows"] == L * 12
    rows = [e for e in ev if e["kind"] == ad.EV_VERIFY_ROW]
    assert all(int(r["flag"]) == -1 for r in rows)


def test_hints_of_the_expected_continuation_match_what_the_schedule_then_asks_for():
    """Before a greedy head evaluation the scheduler tells the backend what it will ask for next if the evaluation
    turns out as expected (the forced outcome, else the head's last decision).  Whenever the outcome is the
    expected one, the calls that follow must be exactly the hinted work; the hints never change the run."""
    rng = np.random.default_rng(5)
    n_pos, L, exits = 400, 12, [3, 6, 9]
    final_tok = rng.integers(0, 50, n_pos).astype(np.int32)
    head_tok = np.repeat(final_tok[:, None], 3, axis=1)
    wrong = rng.random((n_pos, 3)) < 0.15
    head_tok[wrong] = 77                                            # some drafts get rejected
    head_conf = rng.random((n_pos, 3)).astype(np.float32)           # about one head in three fires at gamma 0.65
    prompt = [1, 2, 3]
    rc, out, st, ev = ad.sched_test_run(L, exits, 8, head_tok, head_conf, final_tok, prompt, 200, 0.65, 5)
    assert rc == ad.AD_OK and st["early_preds"] > 40 and st["rejections"] > 5
    hints = ad.sched_test_hints()
    evs = [e for e in _events(ev) if e[0] in (ad.EV_HEAD, ad.EV_VERIFY)]
    # one per head evaluation and per verification, except a verification that certainly ends the run
    assert len(hints) in (len(evs) - 1, len(evs))
    last = {}
    n_hit = 0
    for i, (h, e) in enumerate(zip(hints, evs)):
        kind, layer, row0, m, hit = (int(v) for v in h)
        if e[0] == ad.EV_VERIFY:
            assert (kind, layer, row0, m) == (2, 1, 0, 1)
            assert hit == (1 if i + 1 < len(evs) else 0)            # the next token starts in row 0, unless the run is over
        else:
            take, expected = bool(e[5]), last.get(e[1], False)
            assert kind == (2 if expected else 1)
            if kind == 1:
                assert layer == e[1] + 1
            assert hit == (1 if take == expected else 0), (i, h, e)
            last[e[1]] = take
        n_hit += hit
    assert 0.4 * len(hints) < n_hit < len(hints)
    # the run is the same without hints
    rc, out2, st2, ev2 = ad.sched_test_run(L, exits, 8, head_tok, head_conf, final_tok, prompt, 200, 0.65, 5, no_issue_ahead=True)
    assert rc == ad.AD_OK and len(ad.sched_test_hints()) == 0
    np.testing.assert_array_equal(out, out2)
    assert st == st2 and _events(ev) == _events(ev2)
    # a forced schedule is known in advance: every hint is right (the last verification's aside)
    forced = np.zeros(n_pos, dtype=np.uint8)
    forced[rng.random(n_pos) < 0.5] = 6
    forced[rng.random(n_pos) < 0.2] = 9
    rc, out, st, ev = ad.sched_test_run(L, exits, 8, head_tok, head_conf, final_tok, prompt, 120, 0.9, 5, forced_exit=forced)
    hints = ad.sched_test_hints()
    n_dec = st["head_evals"] + st["verifies"]
    assert rc == ad.AD_OK and st["early_preds"] > 30 and len(hints) in (n_dec - 1, n_dec)
    assert hints[:n_dec - 1, 4].all() and not hints[n_dec - 1:, 4].any()
    # sampled decoding and the run without verification give no hints
    u = rng.random((n_pos, 6)).astype(np.float32)
    rc, *_ = ad.sched_test_run(L, exits, 8, head_tok, head_conf, final_tok, prompt, 40, 0.65, 5, temperature=1.0, uniforms=u)
    assert rc == ad.AD_OK and len(ad.sched_test_hints()) == 0
    rc, *_ = ad.sched_test_run(L, exits, 8, head_tok, head_conf, final_tok, prompt, 40, 0.65, 5, no_verify=True)
    assert rc == ad.AD_OK and len(ad.sched_test_hints()) == 0


def test_a_matrix_of_4_gib_or_more_is_refused():
    """The kernels address a packed weight matrix with a 32-bit byte offset: a configuration whose LM head (or any
    other matrix) would reach 4 GiB in the library's layout is an invalid configuration, not a silent wrap."""
    import ctypes as C
    from paper_2506_03700_amd import binding
    L = binding.lib()
    ok = synth.LLAMA8B
    assert L.ad_workspace_bytes(C.byref(binding.make_config(ok))) > 0
    big = ok.with_(d_model=8192, n_q_heads=64, vocab=262144)            # 262144 x 8192 x 2 B = 4 GiB
    assert L.ad_workspace_bytes(C.byref(binding.make_config(big))) == 0
    assert b"4 GiB" in L.ad_last_error()
    f32 = ok.with_(dtype=synth.F32, d_model=5120, n_q_heads=40, n_kv_heads=40, vocab=152064)     # three planes
    assert L.ad_workspace_bytes(C.byref(binding.make_config(f32))) == 0


def test_small_division_multipliers_are_exact():
    """The kernels divide small indices by multiplying with a rounded-up reciprocal the host derives
    (x / d == (x * mul) >> 32, with 0 standing for d == 1): exact over the whole range the kernels use."""
    def mul(d):
        return 0 if d <= 1 else (2 ** 32 + d - 1) // d
    x = np.arange(0, 65536, dtype=np.uint64)
    for d in list(range(1, 300)) + [511, 512, 513, 1000, 4095, 4096, 9217, 65535]:
        m = mul(d)
        got = x if m == 0 else (x * np.uint64(m)) >> np.uint64(32)
        np.testing.assert_array_equal(got, x // np.uint64(d), err_msg=f"d={d}")
