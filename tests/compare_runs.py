"""Free-run comparison of a GPU generation with the oracle's, decision by decision.

A divergence is tolerated only at a decision whose oracle top-2 logit margin is below the near-tie threshold
(or, for an exit decision, whose confidence is within rounding of the threshold); the comparison then stops
there and returns how many decisions agreed.
"""
import numpy as np

from oracle import oracle as orc

NEAR_TIE = 1e-2


def events(ev):
    return [(int(e["kind"]), int(e["layer"]), int(e["pos"]), int(e["m"]), int(e["token"]), int(e["flag"])) for e in ev]


def compare_runs(g, o, prompt, max_new, gamma, cap, tol, **kw):
    tg, sg, eg = g.ad_generate(prompt, max_new, gamma, cap, **kw)
    to, so, eo = o.generate_ada(prompt, max_new, gamma, cap, **kw)
    a, b = events(eg), events(eo)
    n = min(len(a), len(b))
    first = next((i for i in range(n) if a[i] != b[i]), None)
    if first is None:
        assert len(a) == len(b)
        np.testing.assert_array_equal(tg, to)
        for k in ("tokens", "layer_steps", "layer_step_rows", "head_evals", "verifies", "early_preds", "rejections", "rolled_back"):
            assert sg[k] == so[k], k
        hg, ho = eg[eg["kind"] == 2], eo[eo["kind"] == 2]
        np.testing.assert_allclose(hg["conf"], ho["conf"], rtol=5 * tol, atol=1e-6)
        return len(a), so
    e = eo[first]
    if e["kind"] == orc.EV_VERIFY:
        # the verification's outcome differs: one of its rows must have a different argmax; that row's margin decides
        rows_o = [x for x in eo[first + 1:first + 1 + int(e["m"])] if x["kind"] == orc.EV_VERIFY_ROW]
        rows_g = [x for x in eg[first + 1:first + 1 + int(e["m"])] if x["kind"] == 4]
        diff = [ro for ro, rg in zip(rows_o, rows_g) if ro["token"] != rg["token"]]
        ok = len(diff) > 0 and diff[0]["margin"] < NEAR_TIE
        why = f"row margin {diff[0]['margin'] if diff else None}"
    elif e["kind"] == orc.EV_HEAD:
        ok = e["margin"] < NEAR_TIE or (abs(e["conf"] - gamma) < 5 * tol * gamma and a[first][:5] == b[first][:5])
        why = f"head margin {e['margin']} conf {e['conf']}"
    elif e["kind"] == orc.EV_VERIFY_ROW:
        ok = e["margin"] < NEAR_TIE
        why = f"row margin {e['margin']}"
    else:
        ok, why = False, "a layer step differs without an earlier decision differing"
    assert ok, f"decision {first} differs: gpu {a[first]} oracle {b[first]} ({why})"
    return first, so


def compare_sampled_runs(g, o, prompt, max_new, gamma, cap, tol, temperature, uniforms, **kw):
    """Sampled decoding (temperature > 0) with the same table of draws on both sides.  A logit error e moves a
    cumulative-distribution boundary, a token's probability and the ratio of Eq. 2 by at most about e / temperature,
    so a divergence is tolerated only at a decision whose draw the oracle reports within that distance of a
    boundary; the comparison stops there.  Returns (decisions that agreed, decisions of the oracle's run, its stats)."""
    tg, sg, eg = g.ad_generate(prompt, max_new, gamma, cap, temperature=temperature, uniforms=uniforms, **kw)
    to, so, eo = o.generate_ada(prompt, max_new, gamma, cap, temperature=temperature, uniforms=uniforms, **kw)
    tie = min(0.5, 8 * tol / temperature)
    a, b = events(eg), events(eo)
    n = min(len(a), len(b))
    first = next((i for i in range(n) if a[i] != b[i]), None)
    if first is None:
        assert len(a) == len(b)
        np.testing.assert_array_equal(tg, to)
        for k in ("tokens", "layer_steps", "layer_step_rows", "head_evals", "verifies", "early_preds", "rejections", "rolled_back"):
            assert sg[k] == so[k], k
        for kind in (orc.EV_HEAD, orc.EV_VERIFY_ROW):            # drawn tokens' probabilities, ratios of Eq. 2
            cg, co = eg[eg["kind"] == kind]["conf"], eo[eo["kind"] == kind]["conf"]
            np.testing.assert_allclose(np.minimum(cg, 1e6), np.minimum(co, 1e6), rtol=tie, atol=1e-6)
        return len(a), len(b), so
    e = eo[first]
    if e["kind"] == orc.EV_VERIFY:
        rows_o = [x for x in eo[first + 1:first + 1 + int(e["m"])] if x["kind"] == orc.EV_VERIFY_ROW]
        rows_g = [x for x in eg[first + 1:first + 1 + int(e["m"])] if x["kind"] == 4]
        diff = [ro for ro, rg in zip(rows_o, rows_g) if (ro["token"], ro["flag"]) != (rg["token"], rg["flag"])]
        ok = len(diff) > 0 and diff[0]["margin"] < tie
        why = f"row margin {diff[0]['margin'] if diff else None}"
    elif e["kind"] == orc.EV_HEAD:
        ok = e["margin"] < tie or (abs(e["conf"] - gamma) < tie and a[first][:5] == b[first][:5])
        why = f"head draw margin {e['margin']} prob {e['conf']}"
    elif e["kind"] == orc.EV_VERIFY_ROW:
        ok = e["margin"] < tie
        why = f"row margin {e['margin']}"
    else:
        ok, why = False, "a layer step differs without an earlier decision differing"
    assert ok, f"decision {first} differs: gpu {a[first]} oracle {b[first]} ({why}; tolerated below {tie})"
    return first, len(b), so
