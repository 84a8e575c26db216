"""GPU parity of sampled decoding (Sec. 2.2: Eq. 1 with a drawn token, Eq. 2 in its general form) with the oracle.

A sampled decision is a floating-point comparison that decides an integer: the draw u against the cumulative
distribution, or against the ratio of Eq. 2.  The oracle reports how far each draw was from the nearest value
that would change the decision (in probability units); decisions must agree except within a margin that covers
the fp32 summation of the kernel (kernel-level tests, both sides start from the same fp32 logits: 1e-6) or the
logit error of the model's storage type (free runs: compare_runs.sampled_tie; after a tolerated difference the
comparison re-synchronises on the oracle's output and goes on, so whole runs are compared for every type).
"""
import numpy as np
import pytest

from oracle import oracle as orc
from paper_2506_03700_amd import synth

pytestmark = pytest.mark.gpu

KERNEL_MARGIN = 1e-6
# tolerated differences (each a draw the oracle reports within the logit error of a boundary) per free run of 48 tokens
MAX_RESYNCS = {synth.F32: 1, synth.BF16: 6, synth.F16: 3}


@pytest.fixture(scope="module")
def ad():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2506_03700_amd import binding
    binding.lib()
    return binding


def _logit_rows(rng, n, V, kind):
    if kind == "flat":
        return (rng.standard_normal((n, V)) * 0.3).astype(np.float32)
    if kind == "peaked":
        return (rng.standard_normal((n, V)) * 6.0).astype(np.float32)
    z = (rng.standard_normal((n, V)) * 0.5).astype(np.float32)          # "spike": one dominant token per row
    z[np.arange(n), rng.integers(0, V, n)] += 12.0
    return z


VOCABS = [pytest.param(synth.TINY.with_(name="v2048"), id="v2048"),
          pytest.param(synth.TINY.with_(name="v301", vocab=301, tied_head=False), id="v301"),
          pytest.param(synth.TINY.with_(name="v128256", vocab=128256, tied_head=False, n_layers=1, exit_layers=()), id="v128256")]


@pytest.mark.parametrize("shape", VOCABS)
def test_sample_logits_matches_oracle(ad, shape):
    import torch
    V = shape.vocab
    g = ad.Model(shape, synth.make_weights(shape, seed=0), max_pos=8)
    rng = np.random.default_rng(V)
    n_cmp = 0
    for kind in ("flat", "peaked", "spike"):
        z = _logit_rows(rng, 6, V, kind)
        zg = torch.from_numpy(z).to("cuda:0")
        for r in range(6):
            for T, u in [(1.0, float(rng.random())), (0.3, float(rng.random())), (0.05, float(rng.random())), (1.0, 0.0),
                         (0.7, float(np.float32(1.0 - 2.0 ** -24)))]:
                u = float(np.float32(u))
                print(f"case V={V} {kind} row={r} T={T} u={u}", flush=True)
                p = orc.softmax_t(z[r].astype(np.float64), T)
                tok_o, margin = orc.sample_cdf(p, u)
                tok_g, prob_g = g.ad_sample_logits(zg[r], T, u)
                assert 0 <= tok_g < V
                if margin >= KERNEL_MARGIN:
                    assert tok_g == tok_o
                    assert abs(prob_g - p[tok_o]) <= 1e-4 * p[tok_o] + 1e-12
                    n_cmp += 1
                else:
                    # the draw sits on a boundary: the neighbouring token is as good; nothing of weight lies between
                    assert p[min(tok_g, tok_o) + 1:max(tok_g, tok_o)].sum() < 1e-4
    assert n_cmp >= 45
    # all logits equal: the uniform distribution, token floor(u * V)
    zg = torch.zeros(V, dtype=torch.float32, device="cuda:0")
    for u in (0.0, 0.25, 0.5 + 1.0 / (3 * V), 0.999):
        tok_g, prob_g = g.ad_sample_logits(zg, 1.0, u)
        assert abs(tok_g - int(u * V)) <= 1 and abs(prob_g * V - 1) < 1e-4
    # error paths: temperature and draw ranges are checked on the host
    for T, u in [(0.0, 0.5), (-1.0, 0.5), (1.0, 1.0), (1.0, -0.1)]:
        with pytest.raises(ad.AdError) as e:
            g.ad_sample_logits(zg, T, u)
        assert e.value.status == ad.AD_ERANGE
    g.close()


def _oracle_verify(zf, zq, draft, T, ua, ur, uf):
    """Eq. 2 over the rows with the oracle's building blocks: (n_accept, next, ratios, smallest margin)."""
    m = zf.shape[0]
    ratios = np.zeros(max(m - 1, 0))
    worst = 1.0
    for k in range(m - 1):
        p = orc.softmax_t(zf[k].astype(np.float64), T)
        q = orc.softmax_t(zq[k].astype(np.float64), T)
        acc, repl, ratio, mg = orc.accept_or_resample(p, q, int(draft[k]), float(ua[k]), float(ur[k]))
        ratios[k] = ratio
        worst = min(worst, mg)
        if not acc:
            return k, repl, ratios, worst
    p = orc.softmax_t(zf[m - 1].astype(np.float64), T)
    tok, mg = orc.sample_cdf(p, float(uf))
    return m - 1, tok, ratios, min(worst, mg)


@pytest.mark.parametrize("shape", VOCABS)
def test_verify_sampled_matches_oracle(ad, shape):
    import torch
    V = shape.vocab
    g = ad.Model(shape, synth.make_weights(shape, seed=0), max_pos=8)
    rng = np.random.default_rng(V + 1)
    n_cmp = n_rej = n_all = 0
    n_cases = 10 if V > 100000 else 40
    for case in range(n_cases):
        m = int(rng.integers(1, 9))
        kind = ("flat", "peaked", "spike")[case % 3]
        T = (1.0, 0.5, 0.1)[case % 3] if kind != "flat" else 0.05
        zf = _logit_rows(rng, m, V, kind)
        # drafts come from distributions close to the final ones (as a good exit head's would), some from unrelated ones
        noise = (0.0, 0.05, 0.3, 3.0)[case % 4]
        zq = (zf[:m - 1] + noise * rng.standard_normal((m - 1, V))).astype(np.float32)
        ua = rng.random(m - 1).astype(np.float32)
        ur = rng.random(m - 1).astype(np.float32)
        uf = float(np.float32(rng.random()))
        draft = np.array([orc.sample_cdf(orc.softmax_t(zq[k].astype(np.float64), T), float(rng.random()))[0] for k in range(m - 1)], dtype=np.int32)
        if case % 7 == 3 and m > 1:
            draft[m - 2] = rng.integers(0, V)                            # a token the draft distribution hardly supports
        print(f"case V={V} #{case} m={m} {kind} T={T} noise={noise}", flush=True)
        na_o, nx_o, ratios_o, margin = _oracle_verify(zf, zq, draft, T, ua, ur, uf)
        zfg = torch.from_numpy(zf).to("cuda:0")
        zqg = torch.from_numpy(zq).to("cuda:0") if m > 1 else None
        na_g, nx_g, ratios_g = g.ad_verify_sampled(zfg, zqg, draft, T, ua, ur, uf)
        assert 0 <= na_g <= m - 1 and 0 <= nx_g < V
        if margin >= KERNEL_MARGIN:
            assert (na_g, nx_g) == (na_o, nx_o)
            k = min(na_o + 1, m - 1)
            np.testing.assert_allclose(np.minimum(ratios_g[:k], 1e6), np.minimum(ratios_o[:k], 1e6), rtol=2e-4, atol=1e-30)
            assert np.all(ratios_g[k:] == 0)
            n_cmp += 1
            n_rej += na_o < m - 1
            n_all += na_o == m - 1 and m > 1
    assert n_cmp >= 0.8 * n_cases and n_rej >= 2 and n_all >= 2
    # identical distributions: every draft is accepted whatever the draws; one row: plain sampling of the next token
    zf = _logit_rows(rng, 5, V, "peaked")
    zfg = torch.from_numpy(zf).to("cuda:0")
    na, nx, ratios = g.ad_verify_sampled(zfg, zfg[:4].contiguous(), [1, 2, 3, 4], 0.5, [0.999] * 4, [0.5] * 4, 0.25)
    assert na == 4 and np.allclose(ratios, 1.0, rtol=1e-5)
    assert nx == orc.sample_cdf(orc.softmax_t(zf[4].astype(np.float64), 0.5), 0.25)[0]
    na, nx, _ = g.ad_verify_sampled(zfg[:1].contiguous(), None, [], 0.5, [], [], 0.25)
    assert na == 0 and nx == orc.sample_cdf(orc.softmax_t(zf[0].astype(np.float64), 0.5), 0.25)[0]
    with pytest.raises(ad.AdError) as e:
        g.ad_verify_sampled(zfg[:2].contiguous(), zfg[:1].contiguous(), [V], 0.5, [0.1], [0.1], 0.25)
    assert e.value.status == ad.AD_ERANGE
    g.close()


UNTIED = synth.TINY.with_(name="tiny-untied", tied_head=False, vocab=512, exit_layers=(1, 2, 3))


@pytest.mark.parametrize("shape", [UNTIED, synth.TINY_GQA.with_(name="tiny-gqa-untied", tied_head=False, vocab=640),
                                   UNTIED.with_(name="tiny-untied-bf16", dtype=synth.BF16),
                                   UNTIED.with_(name="tiny-untied-f16", dtype=synth.F16)], ids=lambda s: s.name)
def test_generate_sampled_matches_oracle_decisions(ad, shape):
    """Free runs of sampled Algorithm 1 on the GPU and in the oracle with the same draws: every decision of the whole
    run must agree, except draws that lie within the storage type's logit error of a boundary (the comparison then
    re-synchronises and continues; their number is bounded); exit heads with a random transform make the exit and
    final distributions differ, so that Eq. 2 rejects often."""
    from compare_runs import compare_sampled_runs
    w = synth.make_weights(shape, seed=0, with_T=True, T_std=0.03)
    max_pos = 128
    o = orc.Oracle(shape, w, max_pos=max_pos)
    g = ad.Model(shape, w, max_pos=max_pos)
    p = synth.make_prompt(shape, 0)
    agreed = total = tokens = rejections = early = 0
    lim = MAX_RESYNCS[shape.dtype]
    for seed, T, gamma, cap in [(0, 0.05, 0.3, 7), (1, 0.05, 0.0, 5), (2, 0.02, 0.5, 7), (3, 0.1, 0.0, 3), (4, 1.0, 0.0, 7)]:
        u = synth.make_uniforms(shape, seed, max_pos)
        print(f"case {shape.name} seed={seed} T={T} gamma={gamma} cap={cap}", flush=True)
        r = compare_sampled_runs(g, o, p, 48, gamma, cap, shape.dtype, T, u, max_resyncs=lim)
        agreed += r.agreed
        total += r.total
        tokens += r.tokens
        rejections += r.stats["rejections"]
        early += r.stats["early_preds"]
    assert early > 20 and rejections > 5
    # whole runs were compared (5 x 48 tokens), and all but the tolerated near-boundary draws agreed
    assert tokens == 5 * 48 and agreed >= total - 5 * lim and agreed >= 0.97 * total, (agreed, total, tokens)
    # forced schedules and scripted drafts with sampling
    forced = synth.make_forced_schedule(shape, 1, max_pos, probs=[0.6 / len(shape.exit_layers)] * len(shape.exit_layers))
    script = np.full(max_pos, -1, dtype=np.int32)
    script[[40, 47, 61]] = [1, 2, 3]
    u = synth.make_uniforms(shape, 9, max_pos)
    r = compare_sampled_runs(g, o, p, 48, 0.9, 5, shape.dtype, 0.05, u, max_resyncs=lim, forced_exit=forced, scripted_draft=script)
    assert r.tokens == 48 and r.agreed >= 0.97 * r.total
    g.close()


@pytest.mark.parametrize("shape", [synth.TINY, UNTIED.with_(name="tiny-untied-bf16", dtype=synth.BF16), synth.MINI8B],
                         ids=lambda s: s.name)
def test_low_temperature_limit_is_the_gpu_greedy_run(ad, shape):
    """At a temperature far below the smallest top-2 logit margin, sampling is argmax: the sampled run must emit the
    greedy run's tokens whatever the draws (a property that holds at any size)."""
    w = synth.make_weights(shape, seed=0)
    max_pos = 96
    g = ad.Model(shape, w, max_pos=max_pos)
    p = synth.make_prompt(shape, 0)[:16]
    n_new = 24
    greedy, _, _ = g.ad_generate(p, n_new, 1.0, 5)
    # margins of the greedy run on the GPU itself: recompute the final logits of each emitted token
    for seed, gamma, cap in [(0, 0.0, 7), (1, 0.6, 5)]:
        u = synth.make_uniforms(shape, seed, max_pos)
        toks, st, ev = g.ad_generate(p, n_new, gamma, cap, temperature=1e-6, uniforms=u)
        same = int(np.argmin(np.concatenate([toks == greedy, [False]])))
        if same < n_new:
            # a divergence is legitimate only at a near-tie of the greedy run (margin below 1e-2): check it on the oracle
            o = orc.Oracle(shape, w, max_pos=max_pos)
            _, margins = o.generate_greedy(p, same + 1)
            assert margins[same] < 1e-2, f"sampled run at T -> 0 leaves greedy at token {same} (margin {margins[same]})"
            o.close()
        assert st["tokens"] == n_new
        if gamma == 0.0 and shape.exit_layers:
            assert st["early_preds"] > 0
    g.close()
