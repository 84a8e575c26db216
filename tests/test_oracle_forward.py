"""Pin for the oracle's decoder: its token-by-token, cache-based layer steps must equal a whole-sequence
causal forward written with library routines (torch fp64 matmul, softmax, scaled_dot_product_attention,
complex multiplication for the rotary embedding).  The two have different structure (full masked
attention over all positions at once vs. incremental rows against a cache), so a wrong index, sign,
transposed operand, dropped residual or wrong head grouping in the oracle shows up here.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import oracle as orc
from paper_2506_03700_amd import synth


def _t(w):
    return torch.from_numpy(synth.as_f32(w).astype(np.float64))


def _rms(x, w, eps):
    return x / torch.sqrt((x * x).mean(-1, keepdim=True) + eps) * w


def _rope_complex(x, base):
    """x: [T, H, dh]; pair (i, i + dh/2) taken as a complex number and multiplied by e^{i pos theta_i}."""
    T, H, dh = x.shape
    half = dh // 2
    theta = torch.tensor(base, dtype=torch.float64) ** (-torch.arange(half, dtype=torch.float64) * 2.0 / dh)
    ang = torch.arange(T, dtype=torch.float64)[:, None] * theta[None, :]
    rot = torch.polar(torch.ones_like(ang), ang)                     # [T, half]
    z = torch.complex(x[..., :half], x[..., half:]) * rot[:, None, :]
    return torch.cat([z.real, z.imag], dim=-1)


def library_forward(shape, w, tokens, T_index=None):
    """Returns (hidden after each layer [L+1][T, d], K [L][T,Hkv,dh], V, final logits [T, V])."""
    s = shape
    x = _t(w["embed"])[torch.from_numpy(np.asarray(tokens, dtype=np.int64))]
    T = x.shape[0]
    hs, Ks, Vs = [x], [], []
    for l in range(s.n_layers):
        p = f"layers.{l}."
        a = _rms(x, _t(w[p + "attn_norm"]), s.rms_eps)
        q = (a @ _t(w[p + "wq"]).T).view(T, s.n_q_heads, s.head_dim)
        k = (a @ _t(w[p + "wk"]).T).view(T, s.n_kv_heads, s.head_dim)
        v = (a @ _t(w[p + "wv"]).T).view(T, s.n_kv_heads, s.head_dim)
        q, k = _rope_complex(q, s.rope_base), _rope_complex(k, s.rope_base)
        if s.dtype == synth.BF16:      # a bf16 workload stores K and V in a bf16 cache (library rounding, RNE)
            k, v = k.float().bfloat16().double(), v.float().bfloat16().double()
        elif s.dtype == synth.F16:     # likewise an fp16 workload (the paper's inference precision, Sec. 4.2)
            k, v = k.float().half().double(), v.float().half().double()
        Ks.append(k)
        Vs.append(v)
        rep = s.n_q_heads // s.n_kv_heads
        o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.repeat_interleave(rep, dim=1).transpose(0, 1)[None],
                                           v.repeat_interleave(rep, dim=1).transpose(0, 1)[None], is_causal=True)[0]
        x = x + o.transpose(0, 1).reshape(T, -1) @ _t(w[p + "wo"]).T
        b = _rms(x, _t(w[p + "ffn_norm"]), s.rms_eps)
        x = x + (F.silu(b @ _t(w[p + "w_gate"]).T) * (b @ _t(w[p + "w_up"]).T)) @ _t(w[p + "w_down"]).T
        hs.append(x)
    n = _rms(x, _t(w["final_norm"]), s.rms_eps)
    if T_index is not None:
        n = n @ _t(w[f"exit_T.{T_index}"]).T
    return hs, Ks, Vs, n @ _t(w["lm_head"]).T


SHAPES = [synth.TINY, synth.TINY_BF16, synth.TINY_F16, synth.TINY_GQA.with_(name="tiny-gqa-f16", dtype=synth.F16), synth.TINY_GQA,
          synth.TINY.with_(name="tiny-odd", n_q_heads=6, n_kv_heads=2, head_dim=32, d_model=96, d_ffn=200, vocab=301,
                           n_layers=3, rope_base=500000.0)]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: s.name)
def test_incremental_steps_equal_whole_sequence_forward(shape):
    w = synth.make_weights(shape, seed=11, norm_jitter=0.2)
    T = 37
    toks = synth.make_prompt(shape, seed=5, n=T)
    hs, Ks, Vs, logits = library_forward(shape, w, toks)
    o = orc.Oracle(shape, w, max_pos=64)
    # ragged schedule of calls: 1 row, 3 rows, 8 rows, 1, 5, ... through every layer
    h_all = o.embed(toks)
    np.testing.assert_array_equal(h_all, hs[0].numpy())
    out = np.zeros_like(h_all)
    start = 0
    for m in [1, 3, 8, 1, 5, 2, 7, 4, 6]:
        m = min(m, T - start)
        pos = np.arange(start, start + m)
        h = h_all[start:start + m]
        for l in range(1, shape.n_layers + 1):
            h = o.layer_step(l, h, pos)
            np.testing.assert_allclose(h, hs[l][start:start + m].numpy(), rtol=0, atol=1e-11)
        out[start:start + m] = h
        start += m
    assert start == T and o.kv_lens() == [T] * shape.n_layers
    for l in range(shape.n_layers):
        k, v = o.kv_read(l + 1, 0, T)
        np.testing.assert_allclose(k, Ks[l].numpy(), rtol=0, atol=1e-11)
        np.testing.assert_allclose(v, Vs[l].numpy(), rtol=0, atol=1e-11)
    # final head: logits, argmax, confidence against library softmax
    for r in (0, T // 2, T - 1):
        tok, conf, margin, z = o.head(-1, out[r], want_logits=True)
        np.testing.assert_allclose(z, logits[r].numpy(), rtol=0, atol=1e-11)
        p = torch.softmax(logits[r], -1)
        assert tok == int(torch.argmax(logits[r])) and abs(conf - float(p.max())) < 1e-12
        top2 = torch.topk(logits[r], 2).values
        assert abs(margin - float(top2[0] - top2[1])) < 1e-10


def test_layer_step_argument_checks():
    shape = synth.TINY
    w = synth.make_weights(shape, seed=1)
    o = orc.Oracle(shape, w, max_pos=8)
    h = o.embed([1, 2])
    with pytest.raises(RuntimeError, match="rc=-2"):
        o.layer_step(1, h, [1, 2])            # cache is empty: must start at 0
    with pytest.raises(RuntimeError, match="rc=-2"):
        o.layer_step(1, h, [0, 2])            # gap
    with pytest.raises(RuntimeError, match="rc=-1"):
        o.layer_step(5, h, [0, 1])            # no such layer
    o.layer_step(1, h, [0, 1])
    assert o.kv_lens() == [2, 0, 0, 0]
    with pytest.raises(RuntimeError, match="rc=-3"):
        o.layer_step(1, o.embed(list(range(7))), list(range(2, 9)))    # beyond max_pos


def test_single_position_attention_returns_value_projection():
    # With one cached position the softmax is 1, so the attention output of every head is V itself and
    # x' = x + Wo (repeat of v per group).  Checked for a GQA shape, where the head -> group map matters.
    shape = synth.TINY_GQA.with_(n_layers=1, exit_layers=())
    w = synth.make_weights(shape, seed=3)
    # make the FFN a no-op so that the output is x' exactly
    w["layers.0.w_down"] = np.zeros_like(w["layers.0.w_down"])
    o = orc.Oracle(shape, w, max_pos=4)
    x = o.embed([123])
    y = o.layer_step(1, x, [0])[0]
    a = orc.rmsnorm(x[0], w["layers.0.attn_norm"], shape.rms_eps)
    v = w["layers.0.wv"].astype(np.float64) @ a                      # [Hkv*dh]
    rep = shape.n_q_heads // shape.n_kv_heads
    o_vec = np.concatenate([v.reshape(shape.n_kv_heads, shape.head_dim)[h // rep] for h in range(shape.n_q_heads)])
    np.testing.assert_allclose(y, x[0] + w["layers.0.wo"].astype(np.float64) @ o_vec, rtol=0, atol=1e-13)


def test_exit_head_with_transform_and_identity_special_case():
    # Sec. 2.1: E = E* T.  T = I must give the final head's result; a general T must equal the library
    # product E* (T n).
    shape = synth.TINY_GQA
    w = synth.make_weights(shape, seed=7, with_T=True, T_std=0.05, norm_jitter=0.1)
    o = orc.Oracle(shape, w, max_pos=4)
    h = np.random.default_rng(0).standard_normal(shape.d_model)
    n = _rms(torch.from_numpy(h), _t(w["final_norm"]), shape.rms_eps)
    for i in range(len(shape.exit_layers)):
        tok, conf, margin, z = o.head(i, h, want_logits=True)
        want = _t(w["lm_head"]) @ (_t(w[f"exit_T.{i}"]) @ n)
        np.testing.assert_allclose(z, want.numpy(), rtol=0, atol=1e-12)
    z_final = o.head(-1, h, want_logits=True)[3]
    np.testing.assert_allclose(z_final, (_t(w["lm_head"]) @ n).numpy(), rtol=0, atol=1e-12)
    w_id = dict(w)
    w_id["exit_T.0"] = np.eye(shape.d_model, dtype=np.float32)
    o2 = orc.Oracle(shape, w_id, max_pos=4)
    np.testing.assert_allclose(o2.head(0, h, want_logits=True)[3], z_final, rtol=0, atol=1e-13)


def test_verify_first_mismatch_rule():
    # Eq. 2 at temperature 0 on scripted logits: make the head an identity-like lookup so that each row's
    # argmax is known by construction, then check (n_accept, next_token) for every mismatch position.
    shape = synth.TINY.with_(vocab=256, d_model=256, tied_head=False)
    w = synth.make_weights(shape, seed=2)
    w["lm_head"] = np.eye(256, dtype=np.float32)               # logits = normalised hidden state
    o = orc.Oracle(shape, w, max_pos=4)
    picks = [5, 9, 200, 31, 77]
    hidden = np.full((5, 256), -1.0)
    for r, t in enumerate(picks):
        hidden[r, t] = 4.0                                     # row r's argmax is picks[r]
    # all drafts right: everything accepted, next token is the last row's argmax
    n_acc, nxt, arg, _ = o.verify(hidden, picks[:4])
    assert (n_acc, nxt) == (4, 77) and list(arg) == picks
    for bad in range(4):
        draft = list(picks[:4])
        draft[bad] = 0
        n_acc, nxt, _, _ = o.verify(hidden, draft)
        assert (n_acc, nxt) == (bad, picks[bad])               # accepted prefix, replacement = final argmax
    # a later mismatch does not matter once an earlier one is found
    assert o.verify(hidden, [5, 0, 0, 0])[:2] == (1, 9)
    # one row, no drafts: plain next-token prediction
    assert o.verify(hidden[:1], [])[:2] == (0, 5)


@pytest.mark.parametrize("shape", [synth.TINY, synth.TINY_GQA, synth.TINY_BF16,
                                   synth.TINY.with_(name="tiny-untied", tied_head=False, vocab=512, exit_layers=(1, 2, 3))],
                         ids=lambda s: s.name)
def test_greedy_generation_is_the_argmax_chain_of_the_whole_sequence_forward(shape):
    # Plain greedy decoding, pinned directly: feed prompt + output to the whole-sequence library forward (teacher
    # forcing); the final-layer argmax at every position from the last prompt token on must be the token the oracle
    # emitted next, and the margin it reports must be that position's top-2 logit gap.  Positions whose gap is within
    # the two implementations' rounding of zero could legitimately differ and are not expected with these seeds.
    w = synth.make_weights(shape, seed=0)
    prompt = synth.make_prompt(shape, 0)[:20]
    n_new = 24
    o = orc.Oracle(shape, w, max_pos=64)
    out, margins = o.generate_greedy(prompt, n_new)
    assert len(out) == n_new
    seq = np.concatenate([prompt, out])
    logits = library_forward(shape, w, seq[:-1])[3]
    M = len(prompt)
    for j in range(n_new):
        z = logits[M - 1 + j]
        top2 = torch.topk(z, 2)
        assert margins[j] > 1e-9, "an exact tie: pick another seed for this pin"
        assert int(top2.indices[0]) == int(out[j]), f"token {j}"
        assert abs(float(top2.values[0] - top2.values[1]) - margins[j]) < 1e-9
    # the end-of-sequence rule: generation stops after emitting eos_id
    out2, _ = o.generate_greedy(prompt, n_new, eos_id=int(out[5]))
    first = int(np.nonzero(out == out[5])[0][0])
    np.testing.assert_array_equal(out2, out[:first + 1])
