"""Pins for the oracle's sampled decoding (Sec. 2.2: Eq. 1 with a sampled token, Eq. 2 in its general form).

1. softmax(z / T) against the library routine; inversion sampling against a library cumulative sum + search.
2. Eq. 2 for one draft: closed forms (identical distributions always accept; the ratio; the residual's support)
   and the textbook property of draft-accept-resample: the surviving token is distributed exactly like the
   final distribution, by Monte Carlo over the three uniform draws on a small vocabulary.
3. Algorithm 1 with sampling: the low-temperature limit is greedy decoding (already pinned); the law of the
   first generated token equals the final layer's distribution when every draft is taken (gamma = 0); the cache
   after a run equals a sequential forward over the emitted sequence; the bookkeeping identities hold.
"""
import numpy as np
import pytest
import scipy.special

from oracle import oracle as orc
from paper_2506_03700_amd import synth
from test_oracle_algorithm import check_bookkeeping

UNTIED = synth.TINY.with_(name="tiny-untied", tied_head=False, vocab=512, exit_layers=(1, 2, 3))


def test_softmax_with_temperature_is_the_library_softmax():
    rng = np.random.default_rng(0)
    for T in (0.05, 0.7, 1.0, 3.0):
        z = rng.standard_normal(301) * 4
        np.testing.assert_allclose(orc.softmax_t(z, T), scipy.special.softmax(z / T), rtol=1e-12, atol=0)
    # T -> 0 concentrates on the argmax, large T flattens
    z = np.array([0.1, 0.5, 0.3])
    assert np.argmax(orc.softmax_t(z, 1e-3)) == 1 and orc.softmax_t(z, 1e-3)[1] > 1 - 1e-12
    np.testing.assert_allclose(orc.softmax_t(z, 1e6), np.full(3, 1 / 3), atol=1e-6)


def test_inversion_sampling_matches_cumsum_search():
    rng = np.random.default_rng(1)
    for trial in range(200):
        n = int(rng.integers(1, 40))
        w = rng.random(n) ** 3
        w[rng.random(n) < 0.3] = 0.0              # zero-weight tokens are never drawn
        if w.sum() == 0:
            w[rng.integers(0, n)] = 1.0
        w *= rng.choice([1.0, 7.5, 1e-3])         # weights need not be normalised
        u = float(rng.random())
        tok, margin = orc.sample_cdf(w, u)
        c = np.cumsum(w)
        want = int(np.searchsorted(c, u * c[-1], side="right"))
        assert tok == want and w[tok] > 0
        lo = c[tok] - w[tok]
        assert margin == pytest.approx(min(u * c[-1] - lo, c[tok] - u * c[-1]) / c[-1], rel=1e-9, abs=1e-15)
    # edges: u = 0 gives the first token of positive weight; a one-hot vector gives its token for any u
    assert orc.sample_cdf([0.0, 0.0, 0.2, 0.8], 0.0)[0] == 2
    for u in (0.0, 0.3, 0.999999):
        assert orc.sample_cdf([0.0, 3.0, 0.0], u)[0] == 1
    # interval ends: token j owns [c_{j-1}, c_j)
    assert orc.sample_cdf([0.25, 0.25, 0.5], 0.25)[0] == 1
    assert orc.sample_cdf([0.25, 0.25, 0.5], 0.5)[0] == 2
    assert orc.sample_cdf([0.25, 0.25, 0.5], 0.4999)[0] == 1


def test_eq2_closed_forms():
    rng = np.random.default_rng(2)
    p = rng.dirichlet(np.ones(9))
    q = rng.dirichlet(np.ones(9))
    for t in range(9):
        for u in (0.0, 0.2, 0.6, 0.999):
            # identical distributions: ratio 1, always accepted
            acc, repl, ratio, mg = orc.accept_or_resample(p, p, t, u, 0.5)
            assert acc and ratio == 1.0
            acc, repl, ratio, mg = orc.accept_or_resample(p, q, t, u, 0.37)
            assert ratio == pytest.approx(p[t] / q[t], rel=1e-14)
            assert acc == (u < min(1.0, p[t] / q[t]))
            if not acc:
                res = np.maximum(p - q, 0)
                assert res[repl] > 0                   # the replacement comes from where p exceeds q
                assert res[t] == 0 and repl != t       # a rejected token has q > p, so it cannot come back
                c = np.cumsum(res)
                assert repl == int(np.searchsorted(c, 0.37 * c[-1], side="right"))
    # a token the draft distribution gives no mass to: accepted iff the final one gives it some
    assert orc.accept_or_resample([0.5, 0.5], [1.0, 0.0], 1, 0.99, 0.0)[0]
    acc, repl, ratio, _ = orc.accept_or_resample([1.0, 0.0], [0.5, 0.5], 1, 0.0, 0.3)
    assert not acc and repl == 0 and ratio == 0.0


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_draft_accept_resample_reproduces_the_final_distribution(seed):
    """Draft t ~ q, keep it with probability min(1, p(t)/q(t)), otherwise redraw from Normalize(max(0, p - q)):
    the result is distributed as p (the property Eq. 2 relies on).  Monte Carlo over the three draws."""
    rng = np.random.default_rng(seed)
    V, N = 6, 60000
    p = rng.dirichlet(np.ones(V) * 0.7)
    q = rng.dirichlet(np.ones(V) * 0.7)
    if seed == 2:
        q[1] = 0.0
        q /= q.sum()                                   # a token the draft never proposes
    u = rng.random((N, 3))
    counts = np.zeros(V)
    n_rej = 0
    for i in range(N):
        t, _ = orc.sample_cdf(q, u[i, 0])
        acc, repl, _, _ = orc.accept_or_resample(p, q, t, u[i, 1], u[i, 2])
        counts[t if acc else repl] += 1
        n_rej += not acc
    sigma = np.sqrt(N * p * (1 - p))
    assert np.all(np.abs(counts - N * p) < 5 * sigma + 1), (counts / N, p)
    # the rejection probability is the total-variation distance between q and p
    tv = 0.5 * np.abs(p - q).sum()
    assert abs(n_rej / N - tv) < 5 * np.sqrt(tv * (1 - tv) / N) + 1e-3


def _model(shape, seed=0, n_prompt=12, n_new=40):
    w = synth.make_weights(shape, seed)
    o = orc.Oracle(shape, w, max_pos=128)
    p = synth.make_prompt(shape, seed, n=n_prompt)
    g, margins = o.generate_greedy(p, n_new)
    return o, p, g, margins


@pytest.mark.parametrize("shape", [synth.TINY, UNTIED, synth.TINY_GQA], ids=lambda s: s.name)
def test_low_temperature_limit_is_greedy(shape):
    o, p, g, margins = _model(shape)
    assert margins.min() > 1e-3           # at T = 1e-5 a margin of 1e-3 leaves the runner-up a weight of e^-100
    for seed, gamma, cap in [(0, 0.0, 7), (1, 0.5, 5), (2, 0.999, 3), (3, 1.0, 5)]:
        u = synth.make_uniforms(shape, seed, 128)
        a, st, ev = o.generate_ada(p, 40, gamma, cap, temperature=1e-5, uniforms=u)
        np.testing.assert_array_equal(a, g)
        check_bookkeeping(shape, ev, st, len(p), cap)
        if gamma < 1.0:
            assert st["early_preds"] > 0
        else:
            assert st["early_preds"] == 0


def test_sampled_runs_keep_a_sequential_cache_and_are_reproducible():
    shape = UNTIED
    o, p, g, _ = _model(shape)
    for seed, T, gamma, cap in [(0, 0.05, 0.3, 7), (1, 0.05, 0.0, 5), (2, 1.0, 0.0, 7), (3, 0.02, 0.6, 3)]:
        u = synth.make_uniforms(shape, seed, 128)
        a, st, ev = o.generate_ada(p, 40, gamma, cap, temperature=T, uniforms=u)
        check_bookkeeping(shape, ev, st, len(p), cap)
        assert len(a) == 40
        kv = [o.kv_read(l, 0, len(p) + 39) for l in range(1, shape.n_layers + 1)]
        a2, st2, ev2 = o.generate_ada(p, 40, gamma, cap, temperature=T, uniforms=u)
        np.testing.assert_array_equal(a, a2)
        assert st == st2
        if gamma == 0.0:
            assert st["rejections"] > 0 and st["early_preds"] > st["rejections"]
        # a plain sequential forward over prompt + emitted tokens leaves the same cache (rollbacks included)
        o2 = orc.Oracle(shape, o.weights, max_pos=128)
        seq = np.concatenate([p, a])[:len(p) + 39]
        h = o2.embed(seq)
        for l in range(1, shape.n_layers + 1):
            h = o2.layer_step(l, h, np.arange(len(seq)))
            k2, v2 = o2.kv_read(l, 0, len(seq))
            np.testing.assert_allclose(kv[l - 1][0], k2, rtol=0, atol=1e-10)
            np.testing.assert_allclose(kv[l - 1][1], v2, rtol=0, atol=1e-10)
        o2.close()


def test_first_token_law_is_the_final_distribution_when_every_draft_is_taken():
    """gamma = 0: the first generated token is drafted at the first head, checked with Eq. 2 against the final
    layer and possibly replaced; over the uniform draws its law must be softmax(z* / T) of the prompt's last
    position, exactly what plain sampling from the full model would give."""
    shape = synth.TINY.with_(name="tiny-v8", vocab=8, n_layers=2, exit_layers=(1,), d_model=64, n_q_heads=1, n_kv_heads=1, d_ffn=64,
                             tied_head=False)
    # an untied head and a random transform T(i) = I + N(0, 0.1) at the exit head make the exit distribution
    # differ from the final one (total variation about 0.5), so that Eq. 2 rejects often
    w = synth.make_weights(shape, 3, with_T=True, T_std=0.1)
    o = orc.Oracle(shape, w, max_pos=16)
    p = synth.make_prompt(shape, 3, n=3)
    T = 0.1                                 # random-init logits are small: a low temperature makes the law uneven
    h = o.embed(p)
    for l in (1, 2):
        h = o.layer_step(l, h, np.arange(3))
    _, _, _, z = o.head(-1, h[-1], want_logits=True)
    want = orc.softmax_t(z, T)
    assert want.max() < 0.9 and (want > 0.02).sum() >= 3
    N = 4000
    rng = np.random.default_rng(0)
    counts = np.zeros(shape.vocab)
    n_rej = 0
    for i in range(N):
        u = rng.random((16, 4), dtype=np.float32)
        a, st, ev = o.generate_ada(p, 2, 0.0, 5, temperature=T, uniforms=u)
        assert st["early_preds"] == 1
        counts[a[0]] += 1
        n_rej += st["rejections"]
    sigma = np.sqrt(N * want * (1 - want))
    assert np.all(np.abs(counts - N * want) < 5 * sigma + 1), (counts / N, want)
    assert 0.3 * N < n_rej < 0.7 * N
    o.close()
