"""Free-run comparison of a GPU generation with the oracle's, decision by decision, over the whole run.

Every event of the two traces (layer steps with their row counts, head evaluations with token / exit decision /
confidence, verifications with their per-row outcome) must be identical.  A difference is tolerated only at a
decision that the oracle itself reports as a near tie: a greedy token whose top-2 logit margin is below NEAR_TIE,
an exit whose confidence is within rounding of the threshold, or (sampled decoding) a draw within `tie` of a
boundary of the cumulative distribution or of the acceptance ratio.  After a tolerated difference the two runs
would differ for good, so the comparison re-synchronises: both sides start again from the prompt extended by
the oracle's own output up to and including the token that was decided there, and the comparison goes on over
the rest of the run (schedules, scripted drafts and draws are indexed by absolute position, so they carry over).
The result says how many decisions were compared, how many agreed and how many re-synchronisations it took;
callers bound the latter, so a run that keeps parting from the oracle fails even if each parting is a near tie.
"""
from dataclasses import dataclass, field

import numpy as np

from oracle import oracle as orc

NEAR_TIE = 1e-2

# Largest error of a logit on the GPU path against the oracle (absolute, logits are O(1) here), per storage type
# of the model: measured on the deepest models of the suite (32 layers, d 4096) and rounded up; the sampled
# comparison turns it into a tolerance on probabilities.
LOGIT_ERR = {0: 5e-5, 1: 4e-3, 2: 6e-4}          # synth.F32, BF16, F16

STAT_KEYS = ("tokens", "layer_steps", "layer_step_rows", "head_evals", "verifies", "early_preds", "rejections", "rolled_back")


@dataclass
class Comparison:
    agreed: int = 0           # decisions (events) that were identical
    total: int = 0            # decisions compared (agreed ones plus one per tolerated difference)
    resyncs: int = 0          # tolerated differences, each followed by a restart from the oracle's prefix
    tokens: int = 0           # generated tokens covered by the comparison
    stats: dict = field(default_factory=dict)      # the oracle's statistics of the first segment
    notes: list = field(default_factory=list)

    def __str__(self):
        s = f"{self.agreed}/{self.total} decisions agree over {self.tokens} tokens, {self.resyncs} re-synchronisations"
        return s + ("" if not self.notes else " (" + "; ".join(self.notes) + ")")


class ResumingOracle:
    """The oracle's free runs for the full-size models, made affordable: results are remembered by their arguments
    (the two layer modes of a model are compared with the same oracle run), and a run whose prompt begins with
    tokens whose rows the oracle's cache still holds from its last run takes those rows over instead of
    recomputing them (the oracle's keep_cache; pinned in test_oracle_algorithm.py)."""

    def __init__(self, o):
        self.o = o
        self.memo = {}
        self.in_cache = []          # tokens whose rows the oracle's cache holds, by position

    def generate_ada(self, prompt, max_new, gamma, cap, **kw):
        prompt = np.asarray(prompt, dtype=np.int32)
        key = (prompt.tobytes(), max_new, gamma, cap,
               tuple(sorted((k, v.tobytes() if isinstance(v, np.ndarray) else v) for k, v in kw.items())))
        if key not in self.memo:
            keep = 0
            while keep < min(len(prompt) - 1, len(self.in_cache)) and self.in_cache[keep] == int(prompt[keep]):
                keep += 1
            keep = min([keep] + self.o.kv_lens())
            out = self.o.generate_ada(prompt, max_new, gamma, cap, keep_cache=keep, **kw)
            # a run ends after a verification: the cache holds the prompt and every emitted token but the last
            self.in_cache = [int(t) for t in prompt] + [int(t) for t in out[0][:-1]]
            self.memo[key] = out
        return self.memo[key]


def events(ev):
    return [(int(e["kind"]), int(e["layer"]), int(e["pos"]), int(e["m"]), int(e["token"]), int(e["flag"])) for e in ev]


def sampled_tie(dtype: int, temperature: float) -> float:
    """A logit error d changes every exp(z / T) by a factor within exp(+-d / T), hence a probability, a cumulative
    sum or an acceptance ratio by at most expm1(2 d / T) of its value (and these are at most 1, or compared near 1)."""
    return float(min(0.25, np.expm1(2.0 * LOGIT_ERR[dtype] / temperature)))


def _segment(g, o, prompt, max_new, gamma, cap, conf_rtol, tie, sampled, kw):
    """One free run of both sides.  Returns (events agreed, finished, position decided at the difference, oracle
    tokens, oracle stats, note)."""
    tg, sg, eg = g.ad_generate(prompt, max_new, gamma, cap, **kw)
    to, so, eo = o.generate_ada(prompt, max_new, gamma, cap, **kw)
    a, b = events(eg), events(eo)
    n = min(len(a), len(b))
    first = next((i for i in range(n) if a[i] != b[i]), None)
    if first is None:
        assert len(a) == len(b), f"traces have {len(a)} and {len(b)} events"
        np.testing.assert_array_equal(tg, to)
        for k in STAT_KEYS:
            assert sg[k] == so[k], k
        if not sampled:
            hg, ho = eg[eg["kind"] == orc.EV_HEAD], eo[eo["kind"] == orc.EV_HEAD]
            np.testing.assert_allclose(hg["conf"], ho["conf"], rtol=conf_rtol, atol=1e-6)
        else:
            for kind in (orc.EV_HEAD, orc.EV_VERIFY_ROW):            # drawn tokens' probabilities, ratios of Eq. 2
                cg, co = eg[eg["kind"] == kind]["conf"], eo[eo["kind"] == kind]["conf"]
                np.testing.assert_allclose(np.minimum(cg, 1e6), np.minimum(co, 1e6), rtol=max(tie, 1e-5), atol=1e-6)
        return len(a), True, None, to, so, ""
    e = eo[first]
    bar = tie if sampled else NEAR_TIE
    pos = int(e["pos"])
    if e["kind"] == orc.EV_VERIFY:
        # the verification's outcome differs: one of its rows decided differently; that row's margin counts
        rows_o = [x for x in eo[first + 1:first + 1 + int(e["m"])] if x["kind"] == orc.EV_VERIFY_ROW]
        rows_g = [x for x in eg[first + 1:first + 1 + int(e["m"])] if x["kind"] == orc.EV_VERIFY_ROW]
        diff = [ro for ro, rg in zip(rows_o, rows_g) if (ro["token"], ro["flag"]) != (rg["token"], rg["flag"])]
        ok = len(diff) > 0 and diff[0]["margin"] < bar
        why = f"row margin {diff[0]['margin'] if diff else None}"
        if diff:
            pos = int(diff[0]["pos"])
    elif e["kind"] == orc.EV_HEAD:
        near_gamma = abs(e["conf"] - gamma) < (tie if sampled else conf_rtol * gamma)
        ok = e["margin"] < bar or (near_gamma and a[first][:5] == b[first][:5])
        why = f"head margin {e['margin']} conf {e['conf']}"
    elif e["kind"] == orc.EV_VERIFY_ROW:
        ok = e["margin"] < bar
        why = f"row margin {e['margin']}"
    else:
        ok, why = False, "a layer step differs without an earlier decision differing"
    assert ok, f"decision {first} differs: gpu {a[first]} oracle {b[first]} ({why}; tolerated below {bar})"
    return first, False, pos, to, so, f"pos {pos}: {why}"


def _run(g, o, prompt, max_new, gamma, cap, conf_rtol, tie, sampled, max_resyncs, kw):
    res = Comparison()
    p = [int(t) for t in prompt]
    remaining = max_new
    while True:
        n, done, pos, to, so, note = _segment(g, o, np.asarray(p, dtype=np.int32), remaining, gamma, cap, conf_rtol, tie, sampled, kw)
        if not res.stats:
            res.stats = so
        res.agreed += n
        if done:
            res.total += n
            res.tokens += remaining
            break
        res.total += n + 1
        res.resyncs += 1
        res.notes.append(note)
        assert res.resyncs <= max_resyncs, f"more than {max_resyncs} tolerated differences: {res}"
        # the token at position pos + 1 was decided there: continue from the oracle's output up to and including it
        j = min(pos + 2 - len(p), len(to))
        assert j >= 1
        res.tokens += j
        p += [int(t) for t in to[:j]]
        remaining -= j
        if remaining < 1:
            break
    print(f"    compared: {res}", flush=True)
    return res


def compare_runs(g, o, prompt, max_new, gamma, cap, tol, max_resyncs=0, **kw) -> Comparison:
    """Greedy decoding (Algorithm 1 at temperature 0).  tol: the tensor tolerance of the model's storage type; the
    confidences of the heads must agree within 5 tol."""
    return _run(g, o, prompt, max_new, gamma, cap, 5 * tol, 0.0, False, max_resyncs, kw)


def compare_sampled_runs(g, o, prompt, max_new, gamma, cap, dtype, temperature, uniforms, max_resyncs=0, **kw) -> Comparison:
    """Sampled decoding (temperature > 0) with the same table of draws on both sides."""
    kw = dict(kw, temperature=temperature, uniforms=uniforms)
    return _run(g, o, prompt, max_new, gamma, cap, 0.0, sampled_tie(dtype, temperature), True, max_resyncs, kw)
