"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded inputs.

Tolerances (stated by the build's target): hidden states and KV entries within max relative error 1e-4
for fp32 models and 2e-2 for bf16 models, where the relative error of a tensor is max|gpu - oracle| /
max|oracle|; token ids and exit / verify decisions bit-exact except where the oracle's top-2 logit
margin is below 1e-2.  fp16 models (11 significant bits against bf16's 8) are held to the 16-bit bound
divided by 2^3: 2.5e-3.
"""
import numpy as np
import pytest

from oracle import oracle as orc
from paper_2506_03700_amd import synth
from tolerances import NEAR_TIE, REG, TOL, check_kv, check_rows, rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ad():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2506_03700_amd import binding
    binding.lib()          # fails loudly if the HIP library is missing
    return binding


def gpu_kv(model, layer, n):
    """K, V of one layer for positions [0, n) as float64 [n, Hkv, dh]."""
    return model.kv_read(layer, n)


def with_modes(shapes):
    """(shape, layer mode) cases: bf16 models run the layer step both as one kernel per phase (0) and as the
    fused persistent kernel (1); fp32 models have the per-phase kernels only."""
    return [pytest.param(s, m, id=f"{s.name}-{'fused' if m else 'kernels'}")
            for s in shapes for m in ((0, 1) if s.dtype == synth.BF16 else (0,))]


UNTIED = synth.TINY.with_(name="tiny-untied", tied_head=False, vocab=512, exit_layers=(1, 2, 3))
ODD = synth.TINY.with_(name="tiny-odd", n_q_heads=6, n_kv_heads=2, head_dim=64, d_model=208, d_ffn=200, vocab=301,
                       n_layers=3, exit_layers=(1,), rope_base=500000.0)


@pytest.mark.parametrize("shape,mode", with_modes([synth.TINY, synth.TINY_BF16, synth.TINY_GQA, ODD,
                                                    ODD.with_(name="tiny-odd-bf16", dtype=synth.BF16), synth.TINY_F16,
                                                    ODD.with_(name="tiny-odd-f16", dtype=synth.F16)]))
def test_layer_steps_ragged_small_models(ad, shape, mode):
    import torch
    print(f"case {shape.name} layer mode {mode}", flush=True)
    w = synth.make_weights(shape, seed=11, norm_jitter=0.2)
    T = 45
    toks = synth.make_prompt(shape, seed=5, n=T)
    o = orc.Oracle(shape, w, max_pos=64)
    g = ad.Model(shape, w, max_pos=64, layer_mode=mode)
    tol = TOL[shape.dtype]
    start = 0
    for m in [1, 3, 8, 1, 5, 2, 7, 4, 6, 8]:
        m = min(m, T - start)
        pos = np.arange(start, start + m)
        ho = o.embed(toks[start:start + m])
        hg = g.ad_embed(toks[start:start + m])
        np.testing.assert_array_equal(hg.cpu().numpy(), ho.astype(np.float32))
        for l in range(1, shape.n_layers + 1):
            ho = o.layer_step(l, ho, pos)
            g.ad_layer_step(l, hg, pos)
            check_rows(shape.dtype, hg.cpu().numpy(), ho, f"layer {l} rows {start}..{start + m - 1}")
        start += m
    assert start == T and g.kv_lens() == o.kv_lens() == [T] * shape.n_layers
    for l in range(1, shape.n_layers + 1):
        ko, vo = o.kv_read(l, 0, T)
        kg, vg = gpu_kv(g, l, T)
        check_kv(shape.dtype, kg, ko, f"K of layer {l}")
        check_kv(shape.dtype, vg, vo, f"V of layer {l}")
    # heads on the last rows: logits, greedy token, confidence
    layers = list(shape.exit_layers) + [shape.n_layers]
    for hi, layer in enumerate(layers):
        z = g.ad_head_logits(layer, hg).cpu().numpy()
        for r in range(hg.shape[0]):
            tok_o, conf_o, margin, zo = o.head(hi if layer != shape.n_layers else -1, ho[r], want_logits=True)
            check_rows(shape.dtype, z[r], zo, f"logits of the head at layer {layer}, row {r}")
            tok_g, conf_g = g.ad_exit_head(layer, hg[r])
            if margin >= NEAR_TIE:
                assert tok_g == tok_o
                assert abs(conf_g - conf_o) <= 5 * tol * conf_o + 1e-6
    g.close()


DEEP = synth.TINY_BF16.with_(name="tiny-bf16-6-layers", n_layers=6, exit_layers=(2, 4))


@pytest.mark.parametrize("shape,mode", with_modes([DEEP, synth.TINY_GQA, ODD.with_(name="tiny-odd-bf16", dtype=synth.BF16), synth.TINY,
                                                    DEEP.with_(name="tiny-f16-6-layers", dtype=synth.F16)]))
def test_layer_ranges_match_oracle(ad, shape, mode):
    """ad_layer_steps: the same rows through a stretch of consecutive layers in one call (one launch in the fused
    mode), for stretches of every length, against the oracle taken layer by layer."""
    print(f"case {shape.name} layer mode {mode}", flush=True)
    w = synth.make_weights(shape, seed=13, norm_jitter=0.2)
    L = shape.n_layers
    o = orc.Oracle(shape, w, max_pos=64)
    g = ad.Model(shape, w, max_pos=64, layer_mode=mode)
    tol = TOL[shape.dtype]
    toks = synth.make_prompt(shape, seed=6, n=40)
    # every way of cutting 1..L into at most two or three stretches gets its turn, row counts vary
    cuts = [[L], [1, L - 1], [L - 1, 1], [2, L - 2], [1, 1, L - 2], [L], [1] * L, [L]]
    start = 0
    for case, (m, cut) in enumerate(zip([1, 3, 8, 2, 5, 7, 4, 6], cuts)):
        pos = np.arange(start, start + m)
        ho = o.embed(toks[start:start + m])
        hg = g.ad_embed(toks[start:start + m])
        first = 1
        for n in cut:
            for l in range(first, first + n):
                ho = o.layer_step(l, ho, pos)
            g.ad_layer_steps(first, n, hg, pos)
            check_rows(shape.dtype, hg.cpu().numpy(), ho, f"case {case}: layers {first}..{first + n - 1}, rows {start}..{start + m - 1}")
            first += n
        assert first == L + 1
        start += m
    assert g.kv_lens() == o.kv_lens() == [start] * L
    for l in range(1, L + 1):
        ko, vo = o.kv_read(l, 0, start)
        kg, vg = gpu_kv(g, l, start)
        check_kv(shape.dtype, kg, ko, f"K of layer {l}")
        check_kv(shape.dtype, vg, vo, f"V of layer {l}")
    # error paths: a stretch that leaves the model, and one whose layers' caches end at different positions
    h = g.ad_embed(toks[:2])
    with pytest.raises(ad.AdError) as ei:
        g.ad_layer_steps(2, L, h, np.arange(start, start + 2))
    assert ei.value.status == ad.AD_ERANGE
    with pytest.raises(ad.AdError) as ei:
        g.ad_layer_steps(1, 0, h, np.arange(start, start + 2))
    assert ei.value.status == ad.AD_ERANGE
    g.ad_layer_steps(1, 1, h, np.arange(start, start + 2))
    with pytest.raises(ad.AdError) as ei:
        g.ad_layer_steps(1, 2, h, np.arange(start, start + 2))
    assert ei.value.status == ad.AD_ESTATE
    assert g.kv_lens() == [start + 2] + [start] * (L - 1)      # a refused call appends nothing
    g.close()


L13 = synth.LLAMA13B.with_(name="13b-layer", n_layers=1, exit_layers=(), vocab=256)
L8_F16 = synth.LLAMA8B_LAYER.with_(name="8b-layer-f16", dtype=synth.F16)
L13_F16 = L13.with_(name="13b-layer-f16", dtype=synth.F16)
L13_F32 = L13.with_(name="13b-layer-f32", dtype=synth.F32)
WIDE_BF16 = synth.WIDE_LAYER.with_(name="wide-layer-bf16", dtype=synth.BF16)
D6144 = synth.WIDE_LAYER.with_(name="d6144-layer", d_model=6144, n_q_heads=40, n_kv_heads=8, d_ffn=9992, dtype=synth.BF16)


@pytest.mark.parametrize("shape,ctx,mode", [(synth.LLAMA8B_LAYER, 4096, 0), (synth.LLAMA8B_LAYER, 4096, 1), (L13, 1000, 0), (L13, 1000, 1),
                                            (L8_F16, 4096, 0), (L13_F16, 1000, 0), (L13_F32, 300, 0),
                                            (synth.WIDE_LAYER, 2048, 0), (WIDE_BF16, 500, 0), (D6144, 300, 0),
                                            # more attention work items than compute units: the attention variant with
                                            # small workgroups (all m for 40 kv heads; m <= 4, two passes from m = 3, for the 8B shape)
                                            (L13, 2100, 0), (synth.LLAMA8B_LAYER, 8300, 0)],
                         ids=["8b-layer-kernels", "8b-layer-fused", "13b-layer-kernels", "13b-layer-fused",
                              "8b-layer-f16-kernels", "13b-layer-f16-kernels", "13b-layer-f32-kernels",
                              "wide-layer-f16-kernels", "wide-layer-bf16-kernels", "d6144-layer-bf16-kernels",
                              "13b-layer-many-items", "8b-layer-ctx8300"])
def test_layer_step_full_width_shapes(ad, shape, ctx, mode):
    """The single-layer microbenchmark workload: prefilled N(0,1) cache, N(0,1) hidden rows, m in {1,2,3,4,6,8}
    at positions ctx .. ctx+m-1, cache length reset before each call, hidden rows drawn afresh (their own seed) for
    every call.  The 8B shape, the one the benchmark times, gets the first 10 calls of every m; the other shapes 8
    calls in all."""
    import torch
    w = synth.make_weights(shape, seed=0)
    o = orc.Oracle(shape, w, max_pos=ctx + 8)
    g = ad.Model(shape, w, max_pos=ctx + 8, layer_mode=mode)
    k, v = synth.make_kv_prefill(shape, 0, 0, ctx)
    o.kv_write(1, 0, k.reshape(ctx, -1), v.reshape(ctx, -1))
    g.kv_fill(1, k, v)
    if shape is synth.LLAMA8B_LAYER and ctx == 4096:
        calls = [(m, c) for m in synth.MICRO_M for c in range(10)]
    else:
        calls = [(m, c) for c, m in enumerate([1, 2, 3, 4, 6, 8, 8, 1])]
    worst = worst_branch = 0.0
    for m, call in calls:
        print(f"case {shape.name} layer mode {mode} m={m} call={call}", flush=True)
        o.kv_set_len(1, ctx)
        g.kv_set_len(1, ctx)
        h = synth.make_hidden(shape, seed=synth.micro_call_seed(m, call), m=m)
        pos = np.arange(ctx, ctx + m)
        ho = o.layer_step(1, h, pos)
        hg = torch.from_numpy(h).to("cuda:0")
        g.ad_layer_step(1, hg, pos)
        worst = max(worst, check_rows(shape.dtype, hg.cpu().numpy(), ho, f"m={m} call={call}"))
        # the branch outputs themselves (y - x), which the residual otherwise dwarfs
        e2 = rel_err(hg.cpu().numpy() - h, ho - h)
        assert e2 <= TOL[shape.dtype] and e2 <= 4 * REG[shape.dtype], f"m={m}: branch rel err {e2}"
        worst_branch = max(worst_branch, e2)
        ko, vo = o.kv_read(1, ctx, m)
        kg, vg = gpu_kv(g, 1, ctx + m)
        check_kv(shape.dtype, kg[ctx:], ko, f"appended K, m={m}")
        check_kv(shape.dtype, vg[ctx:], vo, f"appended V, m={m}")
    print(f"    {shape.name} mode {mode}: {len(calls)} calls, largest rel err {worst:.3e}, of the branch output {worst_branch:.3e}", flush=True)
    g.close()


@pytest.mark.parametrize("shape,ctx", [(synth.LLAMA8B_LAYER, 4096), (synth.TINY_BF16.with_(name="tiny-bf16-6-layers", n_layers=6, exit_layers=(2, 4)), 0)],
                         ids=["8b-layer", "tiny-bf16-6-layers"])
def test_bf16_tensors_meet_the_stated_tolerance_against_an_unrounded_cache(ad, shape, ctx):
    """The oracle rounds stored K/V to the cache's 16-bit type because that rounding decides tokens (a quantisation
    step both sides must take alike).  The stated tensor tolerance does not depend on it: against an oracle that
    keeps its cache unrounded, hidden rows and cache entries of the bf16 GPU path stay within 2e-2."""
    import torch
    w = synth.make_weights(shape, seed=0, norm_jitter=0.1)
    T = 40
    o = orc.Oracle(shape, w, max_pos=ctx + 64, kv_dtype=synth.F32)
    g = ad.Model(shape, w, max_pos=ctx + 64)
    if ctx:
        k, v = synth.make_kv_prefill(shape, 0, 0, ctx)
        o.kv_write(1, 0, k.reshape(ctx, -1), v.reshape(ctx, -1))
        g.kv_fill(1, k, v)
        o.kv_set_len(1, ctx)
        g.kv_set_len(1, ctx)
    worst = 0.0
    start = ctx
    for call, m in enumerate([1, 3, 8, 2, 5, 7, 4, 6, 4]):
        h = synth.make_hidden(shape, seed=50 + call, m=m)
        pos = np.arange(start, start + m)
        ho = h.astype(np.float64)
        hg = torch.from_numpy(h).to("cuda:0")
        for l in range(1, shape.n_layers + 1):
            ho = o.layer_step(l, ho, pos)
            g.ad_layer_step(l, hg, pos)
            e = rel_err(hg.cpu().numpy(), ho)
            worst = max(worst, e)
            assert e <= TOL[shape.dtype], f"call {call} layer {l}: rel err {e}"
        start += m
    assert start == ctx + T
    for l in range(1, shape.n_layers + 1):
        ko, vo = o.kv_read(l, ctx, T)
        kg, vg = gpu_kv(g, l, ctx + T)
        ek, ev = rel_err(kg[ctx:], ko), rel_err(vg[ctx:], vo)
        worst = max(worst, ek, ev)
        assert ek <= TOL[shape.dtype] and ev <= TOL[shape.dtype], (l, ek, ev)
    print(f"    {shape.name}: largest rel err against the unrounded-cache oracle {worst:.3e}", flush=True)
    g.close()


def test_exit_head_with_transform_and_verify(ad):
    import torch
    shape = synth.TINY_GQA
    w = synth.make_weights(shape, seed=7, with_T=True, T_std=0.05, norm_jitter=0.1)
    o = orc.Oracle(shape, w, max_pos=8)
    g = ad.Model(shape, w, max_pos=8)
    rng = np.random.default_rng(5)      # a draw whose top-2 logit margins all exceed the near-tie threshold
    h = rng.standard_normal((5, shape.d_model)).astype(np.float32)
    hg = torch.from_numpy(h).to("cuda:0")
    for i, layer in enumerate(shape.exit_layers):
        z = g.ad_head_logits(layer, hg).cpu().numpy()
        for r in range(5):
            tok_o, conf_o, margin, zo = o.head(i, h[r], want_logits=True)
            assert rel_err(z[r], zo) <= 1e-4
            tok_g, conf_g = g.ad_exit_head(layer, hg[r])
            assert margin < NEAR_TIE or tok_g == tok_o
            assert abs(conf_g - conf_o) <= 1e-3 * conf_o
    # verification: drafts built from the oracle's own row argmaxes, then corrupted at each position
    n_acc, nxt, arg, mar = o.verify(h, [0, 0, 0, 0])
    assert mar.min() >= NEAR_TIE
    for bad in [None, 0, 1, 2, 3]:
        draft = [int(x) for x in arg[:4]]
        if bad is not None:
            draft[bad] = (draft[bad] + 1) % shape.vocab
        want = o.verify(h, draft)
        got = g.ad_verify(hg, draft)
        assert (got[0], got[1]) == (want[0], want[1]) and list(got[2]) == list(want[2])
    assert g.ad_verify(hg[:1], [])[:2] == o.verify(h[:1], [])[:2]
    g.close()


def test_argmax_tie_takes_lowest_id(ad):
    import torch
    shape = UNTIED
    w = dict(synth.make_weights(shape, seed=3))
    head = w["lm_head"].copy()
    head[400] = head[17]
    head[130] = head[17]            # three identical rows: exact three-way tie wherever row 17 wins
    w["lm_head"] = head
    g = ad.Model(shape, w, max_pos=8)
    o = orc.Oracle(shape, w, max_pos=8)
    h = (synth.as_f32(head[17]) * 40.0).astype(np.float32)          # makes row 17 (and its copies) the maximum
    tok_o, conf_o, margin = o.head(-1, h)
    assert tok_o == 17 and margin == 0.0
    tok_g, conf_g = g.ad_exit_head(shape.n_layers, torch.from_numpy(h).to("cuda:0"))
    assert tok_g == 17 and abs(conf_g - conf_o) <= 1e-3 * conf_o
    g.close()


# tolerated near-tie differences (each followed by a re-synchronisation on the oracle's output) per free run
MAX_RESYNCS = {synth.F32: 0, synth.BF16: 4, synth.F16: 2}


def compare_runs(shape, g, o, prompt, max_new, gamma, cap, **kw):
    """Whole-run comparison of decisions with the oracle; the run must be covered to its last token and all but
    the tolerated near ties (bounded in number, each checked against the oracle's margin) must agree."""
    from compare_runs import compare_runs as cmp
    r = cmp(g, o, prompt, max_new, gamma, cap, TOL[shape.dtype], max_resyncs=MAX_RESYNCS[shape.dtype], **kw)
    assert r.tokens == max_new and r.agreed >= r.total - MAX_RESYNCS[shape.dtype] and r.agreed >= 0.97 * r.total, str(r)
    return r


@pytest.mark.parametrize("shape,mode", with_modes([synth.TINY, UNTIED, synth.TINY_GQA, UNTIED.with_(name="tiny-untied-bf16", dtype=synth.BF16),
                                                    UNTIED.with_(name="tiny-untied-f16", dtype=synth.F16)]))
def test_generate_matches_oracle_decisions(ad, shape, mode):
    w = synth.make_weights(shape, seed=0)
    max_pos = 160
    o = orc.Oracle(shape, w, max_pos=max_pos)
    g = ad.Model(shape, w, max_pos=max_pos, layer_mode=mode)
    p = synth.make_prompt(shape, 0)
    greedy, margins = o.generate_greedy(p, 64)
    # the workload as stated (gamma 0.9), then thresholds at which exits actually happen, then forced schedules
    for gamma, cap in [(0.9, 7), (1.0, 5), (0.0, 5), (0.0045, 7), (0.05, 3)]:
        print(f"case {shape.name} layer mode {mode} gamma={gamma} cap={cap}", flush=True)
        compare_runs(shape, g, o, p, 64, gamma, cap)
    for seed in (1, 2):
        k = len(shape.exit_layers)
        forced = synth.make_forced_schedule(shape, seed, max_pos, probs=[0.6 / k] * k)
        script = np.full(max_pos, -1, dtype=np.int32)
        script[[40, 47, 61, 75]] = [1, 2, 3, 4]
        print(f"case {shape.name} forced seed={seed}", flush=True)
        compare_runs(shape, g, o, p, 64, 0.9, 7, forced_exit=forced)
        compare_runs(shape, g, o, p, 64, 0.9, 5, forced_exit=forced, scripted_draft=script)
    # output parity with plain greedy decoding on the GPU itself (gamma = 1 never exits)
    tg, _, _ = g.ad_generate(p, 64, 1.0, 5)
    if margins.min() >= NEAR_TIE:
        np.testing.assert_array_equal(tg, greedy)
    g.close()


@pytest.mark.parametrize("shape,mode", with_modes([UNTIED, UNTIED.with_(name="tiny-untied-bf16", dtype=synth.BF16)]))
def test_generate_edge_cases_match_oracle(ad, shape, mode):
    """Degenerate runs of Algorithm 1 against the oracle: a prompt of one token (no prefill, the first layer step
    runs on an empty cache), a budget of one token (nothing may be drafted), a cap of zero (plain decoding: no head
    is evaluated), a run that fills the cache to its last position with every token leaving early, and an
    end-of-sequence token that the last layer emits."""
    w = synth.make_weights(shape, seed=0)
    max_pos = 64
    o = orc.Oracle(shape, w, max_pos=max_pos)
    g = ad.Model(shape, w, max_pos=max_pos, layer_mode=mode)
    p = synth.make_prompt(shape, 5)
    k = len(shape.exit_layers)
    forced = synth.make_forced_schedule(shape, 4, max_pos, probs=[0.9 / k] * k)
    for what, prompt, n_new, gamma, cap, kw in [
            ("one-token prompt", p[:1], 24, 0.0045, 7, {}),
            ("one-token prompt, forced", p[:1], 24, 0.9, 7, dict(forced_exit=forced)),
            ("budget of one token", p[:9], 1, 0.0, 7, {}),
            ("budget of two tokens", p[:9], 2, 0.0, 7, {}),
            ("cap 0", p[:9], 24, 0.0, 0, {}),
            ("cap 1", p[:9], 24, 0.0, 1, {}),
            ("cache filled to the last position", p[:16], max_pos - 16, 0.9, 7, dict(forced_exit=forced)),
            ("cache filled to the last position, natural", p[:16], max_pos - 16, 0.0045, 7, {})]:
        print(f"case {shape.name} layer mode {mode}: {what}", flush=True)
        r = compare_runs(shape, g, o, prompt, n_new, gamma, cap, **kw)
        if what == "cap 0":
            assert r.stats["head_evals"] == 0 and r.stats["layer_steps"] == n_new * shape.n_layers
        if what == "budget of one token":
            assert r.stats["early_preds"] == 0
    # one position too many is refused before anything runs
    with pytest.raises(ad.AdError) as e:
        g.ad_generate(p[:16], max_pos - 15, 0.9, 7)
    assert e.value.status == ad.AD_ERANGE
    # end of sequence: the token the plain run emits 10th stops the run there, on both sides
    tg, _, _ = g.ad_generate(p[:9], 24, 0.0045, 7)
    to, _, _ = o.generate_ada(p[:9], 24, 0.0045, 7)
    eos = int(to[9])
    first = int(np.nonzero(to == eos)[0][0])
    print(f"case {shape.name} layer mode {mode}: end of sequence (token {eos}, first at {first})", flush=True)
    tg, sg, eg = g.ad_generate(p[:9], 24, 0.0045, 7, eos_id=eos)
    to2, so2, eo2 = o.generate_ada(p[:9], 24, 0.0045, 7, eos_id=eos)
    assert len(to2) == first + 1 and int(to2[-1]) == eos
    from compare_runs import events
    if events(eg) == events(eo2):
        np.testing.assert_array_equal(tg, to2)
    else:
        # a near tie may part the two runs (16-bit models); the GPU's run must still end with its first EOS
        assert shape.dtype != synth.F32
        assert int(tg[-1]) == eos and eos not in [int(t) for t in tg[:-1]]
    g.close()


@pytest.mark.parametrize("shape,mode", with_modes([synth.MINI8B, synth.MINI13B, synth.MINI8B.with_(name="8b-mini-f16", dtype=synth.F16),
                                                    synth.WIDE_MINI]))
def test_generate_full_width_reduced_depth(ad, shape, mode):
    """8B- and 13B-shaped layers (real d, heads, FFN), 4 layers and a reduced vocabulary so that the oracle
    finishes in seconds; forced schedules exercise ragged catch-up, scripted drafts force rejections."""
    w = synth.make_weights(shape, seed=0)
    max_pos = 64
    o = orc.Oracle(shape, w, max_pos=max_pos)
    g = ad.Model(shape, w, max_pos=max_pos, layer_mode=mode)
    p = synth.make_prompt(shape, 0)
    print(f"case {shape.name} layer mode {mode} natural", flush=True)
    compare_runs(shape, g, o, p, shape.gen_len, 0.9, 7)
    forced = synth.make_forced_schedule(shape, 1, max_pos, probs=[0.25] * len(shape.exit_layers))
    print(f"case {shape.name} forced", flush=True)
    compare_runs(shape, g, o, p, shape.gen_len, 0.9, 7, forced_exit=forced)
    script = np.full(max_pos, -1, dtype=np.int32)
    script[[shape.prompt_len + 2, shape.prompt_len + 7, shape.prompt_len + 16]] = [5, 6, 7]
    print(f"case {shape.name} forced+scripted", flush=True)
    compare_runs(shape, g, o, p, shape.gen_len, 0.9, 5, forced_exit=forced, scripted_draft=script)
    # cache parity after the run
    n = min(g.kv_lens())
    assert g.kv_lens() == o.kv_lens()
    for l in (1, shape.n_layers):
        ko, vo = o.kv_read(l, 0, n)
        kg, vg = gpu_kv(g, l, n)
        check_kv(shape.dtype, kg, ko, f"K of layer {l}")
        check_kv(shape.dtype, vg, vo, f"V of layer {l}")
    g.close()


def test_stream_probe_only_reads(ad):
    """The measurement aid reads a layer's weights and cache rows and changes nothing: a layer step gives the same
    bits before and after it, and arguments outside the model are refused."""
    import torch
    shape = synth.MINI8B
    w = synth.make_weights(shape, seed=0)
    g = ad.Model(shape, w, max_pos=64)
    h0 = synth.make_hidden(shape, 3, 5)

    def run():
        g.kv_truncate(0)
        h = torch.from_numpy(h0).to("cuda:0")
        for l in range(1, shape.n_layers + 1):
            g.ad_layer_step(l, h, np.arange(5))
        return h.cpu().numpy().copy(), [gpu_kv(g, l, 5) for l in (1, shape.n_layers)]

    a, kva = run()
    for mode in (ad.AD_PROBE_ONE_KERNEL, ad.AD_PROBE_PER_PHASE):
        for l in range(1, shape.n_layers + 1):
            for ctx in (0, 5, 64):
                g.ad_probe_stream(l, ctx, mode)
    torch.cuda.synchronize()
    kvb = [gpu_kv(g, l, 5) for l in (1, shape.n_layers)]
    b, _ = run()
    np.testing.assert_array_equal(a, b)
    for x, y in zip(kva, kvb):
        np.testing.assert_array_equal(x[0], y[0])
        np.testing.assert_array_equal(x[1], y[1])
    for bad in ((0, 4, 0), (shape.n_layers + 1, 4, 0), (1, 65, 0), (1, -1, 1), (1, 4, 2)):
        with pytest.raises(ad.AdError):
            g.ad_probe_stream(*bad)
    g.close()


def test_abi_error_paths(ad):
    import torch
    shape = synth.TINY
    w = synth.make_weights(shape, seed=1)
    g = ad.Model(shape, w, max_pos=8, m_max=4)
    h = g.ad_embed([1, 2])
    with pytest.raises(ad.AdError) as e:
        g.ad_layer_step(1, h, [1, 2])
    assert e.value.status == ad.AD_ESTATE
    with pytest.raises(ad.AdError) as e:
        g.ad_layer_step(1, h, [0, 2])
    assert e.value.status == ad.AD_ESTATE
    with pytest.raises(ad.AdError) as e:
        g.ad_layer_step(5, h, [0, 1])
    assert e.value.status == ad.AD_ERANGE
    with pytest.raises(ad.AdError) as e:
        g.ad_embed([1, 2, 3, 4, 5])                # m > m_max
    assert e.value.status == ad.AD_ERANGE
    with pytest.raises(ad.AdError) as e:
        g.ad_embed([shape.vocab])
    assert e.value.status == ad.AD_ERANGE
    with pytest.raises(ad.AdError) as e:
        g.ad_exit_head(1, h[0])                    # layer 1 has no head in this model
    assert e.value.status == ad.AD_ESTATE
    assert g.kv_lens() == [0, 0, 0, 0]             # failed calls leave the cache lengths unchanged
    g.ad_layer_step(1, h, [0, 1])
    assert g.kv_lens() == [2, 0, 0, 0]
    h7 = g.ad_embed([1, 2, 3, 4])
    with pytest.raises(ad.AdError) as e:
        g.ad_layer_step(1, h7, [5, 6, 7, 8])       # wrong start
    assert e.value.status == ad.AD_ESTATE
    g.kv_set_len(1, 6)
    with pytest.raises(ad.AdError) as e:
        g.ad_layer_step(1, h7, [6, 7, 8, 9])       # beyond max_pos
    assert e.value.status == ad.AD_ERANGE
    with pytest.raises(ad.AdError) as e:
        g.ad_generate([1, 2, 3], 8, 0.9, 2)        # prompt + max_new > max_pos
    assert e.value.status == ad.AD_ERANGE
    with pytest.raises(ad.AdError) as e:
        g.ad_generate([1, 2, 3], 4, 0.9, 4)        # cap needs more rows than m_max
    assert e.value.status == ad.AD_ERANGE
    with pytest.raises(ad.AdError) as e:
        g.ad_set_layer_mode(ad.AD_LAYER_FUSED)     # the fused layer step exists for bf16 models only
    assert e.value.status == ad.AD_ESTATE
    with pytest.raises(ad.AdError) as e:
        g.ad_set_layer_mode(7)
    assert e.value.status == ad.AD_EINVAL
    g.ad_set_layer_mode(ad.AD_LAYER_KERNELS)
    g.close()


def test_runs_are_reproducible(ad):
    import torch
    shape = synth.MINI8B
    w = synth.make_weights(shape, seed=0)
    g = ad.Model(shape, w, max_pos=64)
    h0 = synth.make_hidden(shape, 3, 8)
    outs = []
    for rep in range(3):
        g.kv_truncate(0)
        h = torch.from_numpy(h0).to("cuda:0")
        for l in range(1, shape.n_layers + 1):
            g.ad_layer_step(l, h, np.arange(8))
        outs.append((h.cpu().numpy().copy(), g.ad_head_logits(shape.n_layers, h).cpu().numpy().copy()))
    for a, b in outs[1:]:
        np.testing.assert_array_equal(a, outs[0][0])      # fixed-order reductions: bit-identical reruns
        np.testing.assert_array_equal(b, outs[0][1])
    g.close()


@pytest.mark.parametrize("shape", [UNTIED.with_(name="tiny-untied-bf16", dtype=synth.BF16), synth.MINI8B], ids=lambda s: s.name)
def test_work_issued_ahead_of_a_head_outcome_changes_nothing(ad, shape):
    """The first kernels of the expected continuation are issued behind a head evaluation before its outcome is
    known; with that switched off the run must be the same event for event, confidences bit for bit and the
    caches bit for bit: natural exits (expectation sometimes wrong), a forced schedule with scripted wrong drafts
    (rejections, roll-backs), and an end-of-sequence token (an early prediction that is not taken)."""
    from compare_runs import events
    w = synth.make_weights(shape, seed=0, with_T=(shape.name.startswith("tiny")), T_std=0.03)
    max_pos = 160
    g = ad.Model(shape, w, max_pos=max_pos)
    p = synth.make_prompt(shape, 1)
    forced = synth.make_forced_schedule(shape, 3, max_pos, probs=[0.25] * len(shape.exit_layers))
    script = np.full(max_pos, -1, dtype=np.int32)
    script[[len(p) + 3, len(p) + 11, len(p) + 30, len(p) + 41]] = [1, 2, 3, 4]
    # a threshold that about half of the head evaluations pass: the median confidence of a run without exits
    _, _, e = g.ad_generate(p, 96, 1.0, 5)
    natural = float(np.median(e[e["kind"] == ad.EV_HEAD]["conf"]))
    _, _, e = g.ad_generate(p, 96, natural, 5)
    taken = e[(e["kind"] == ad.EV_HEAD) & (e["flag"] == 1)]
    assert len(taken) > 8
    eos = int(taken[len(taken) // 2]["token"])          # ... and a token that an early prediction produces midway
    for kw in (dict(gamma=natural), dict(gamma=0.9, forced_exit=forced, scripted_draft=script), dict(gamma=natural, eos_id=eos)):
        gamma = kw.pop("gamma")
        print(f"case {shape.name} {sorted(kw)}", flush=True)
        t1, s1, e1 = g.ad_generate(p, 96, gamma, 5, **kw)
        lens1 = g.kv_lens()
        kv1 = [gpu_kv(g, l, min(lens1)) for l in (1, shape.n_layers)]
        t0, s0, e0 = g.ad_generate(p, 96, gamma, 5, no_issue_ahead=True, **kw)
        assert g.kv_lens() == lens1
        kv0 = [gpu_kv(g, l, min(lens1)) for l in (1, shape.n_layers)]
        np.testing.assert_array_equal(t1, t0)
        assert s1 == s0 and events(e1) == events(e0)
        np.testing.assert_array_equal(e1["conf"], e0["conf"])
        for a, b in zip(kv1, kv0):
            for x, y in zip(a, b):
                np.testing.assert_array_equal(x, y)
        if not kw:
            assert s1["early_preds"] > 8 and s1["head_evals"] > s1["early_preds"] + 8      # both outcomes occurred
        if "eos_id" in kw:
            assert t1[-1] == eos or len(t1) == 96
    g.close()


@pytest.mark.parametrize("shape", [UNTIED, UNTIED.with_(name="tiny-untied-bf16", dtype=synth.BF16)], ids=lambda s: s.name)
def test_ablation_switches_match_oracle(ad, shape):
    """The variants of Table 3 that are switches of the schedule: a single exit head (head_mask) and no
    verification, greedy and sampled, decision by decision against the oracle."""
    from compare_runs import compare_sampled_runs
    w = synth.make_weights(shape, seed=0, with_T=True, T_std=0.03)
    max_pos = 128
    o = orc.Oracle(shape, w, max_pos=max_pos)
    g = ad.Model(shape, w, max_pos=max_pos)
    p = synth.make_prompt(shape, 0)
    forced = synth.make_forced_schedule(shape, 2, max_pos, probs=[0.25, 0.25, 0.25])
    script = np.full(max_pos, -1, dtype=np.int32)
    script[[40, 47, 61, 75]] = [1, 2, 3, 4]
    for mask in (0b001, 0b010, 0b100, 0b101):
        print(f"case {shape.name} head_mask={mask:03b}", flush=True)
        compare_runs(shape, g, o, p, 48, 0.0045, 7, head_mask=mask)
        compare_runs(shape, g, o, p, 48, 0.9, 5, forced_exit=forced, scripted_draft=script, head_mask=mask)
    print(f"case {shape.name} no_verify", flush=True)
    compare_runs(shape, g, o, p, 48, 0.0045, 7, no_verify=True)
    compare_runs(shape, g, o, p, 48, 0.9, 5, forced_exit=forced, scripted_draft=script, no_verify=True)
    # an unverified wrong draft stays in the GPU's output
    tg, sg, _ = g.ad_generate(p, 48, 0.9, 5, forced_exit=forced, scripted_draft=script, no_verify=True)
    assert sg["rejections"] == 0 and sg["rolled_back"] == 0
    u = synth.make_uniforms(shape, 4, max_pos)
    print(f"case {shape.name} sampled no_verify / head_mask", flush=True)
    for kw in (dict(no_verify=True), dict(head_mask=0b010)):
        r = compare_sampled_runs(g, o, p, 48, 0.3, 7, shape.dtype, 0.05, u, max_resyncs=4, **kw)
        assert r.tokens == 48 and r.agreed >= 0.97 * r.total, str(r)
    g.close()


def test_caller_stream_and_two_models(ad):
    """Every entry point launches on the stream it is handed: a run on a caller-created stream (default priority),
    with a second model alive and used in between, gives the bits of the run on the default stream."""
    import torch
    shape = synth.TINY_BF16
    w = synth.make_weights(shape, seed=2, norm_jitter=0.1)
    w2 = synth.make_weights(shape, seed=3)
    g = ad.Model(shape, w, max_pos=64)
    g2 = ad.Model(shape, w2, max_pos=64)
    p = synth.make_prompt(shape, 2)[:12]
    h0 = synth.make_hidden(shape, 5, 4)

    def run():
        g.kv_truncate(0)
        h = torch.from_numpy(h0).to("cuda:0")
        for l in range(1, shape.n_layers + 1):
            g.ad_layer_step(l, h, np.arange(4))
            g2.kv_truncate(0)
            g2.ad_layer_step(l if l == 1 else 1, torch.from_numpy(h0).to("cuda:0"), np.arange(4))     # the other model, interleaved
        tok = g.ad_exit_head(shape.n_layers, h[3])
        toks, st, _ = g.ad_generate(p, 24, 0.0045, 5)
        torch.cuda.current_stream().synchronize()
        return h.cpu().numpy().copy(), tok, toks

    base = run()
    s = torch.cuda.Stream()            # default priority
    with torch.cuda.stream(s):
        other = run()
    s.synchronize()
    np.testing.assert_array_equal(base[0], other[0])
    assert base[1] == other[1]
    np.testing.assert_array_equal(base[2], other[2])
    g.close()
    g2.close()
