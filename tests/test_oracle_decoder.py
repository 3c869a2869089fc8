"""Pins for the CPU checker's decoder.

The checker evaluates the decoder with hand-written loops, one token at a time.  Here it is
compared with an independent whole-sequence evaluation assembled from library routines
(torch CPU, fp64: F.linear, F.rms_norm, F.scaled_dot_product_attention with is_causal, F.silu,
complex multiplication for the rotary embedding), with closed forms for the rotary convention,
and with the structural properties of a causal decoder.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
import synth

SMALL = synth.ModelShape(n_layers=2, hidden=64, n_q_heads=4, n_kv_heads=2, head_dim=16, ffn=96, vocab=50,
                         rms_eps=1e-6, rope_theta=1e4)


def _t(bits):
    return torch.from_numpy(synth.bf16_bits_to_f32(bits).astype(np.float64))


def torch_logits_all_positions(w, tokens):
    """[T, vocab] fp64 logits for every position, from library routines over the whole sequence."""
    s = w.shape
    T, d, half = len(tokens), s.head_dim, s.head_dim // 2
    x = F.embedding(torch.as_tensor(tokens, dtype=torch.long), _t(w.embed))
    inv_freq = torch.tensor(s.rope_theta, dtype=torch.float64) ** (-torch.arange(half, dtype=torch.float64) * 2 / d)
    ang = torch.arange(T, dtype=torch.float64)[:, None] * inv_freq[None, :]
    rot = torch.polar(torch.ones_like(ang), ang)                       # e^{i*angle}, [T, half]

    def rotary(v):                                                      # v [T, heads, d]; pair (i, i+half)
        z = torch.complex(v[..., :half], v[..., half:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    for L in w.layers:
        h = F.rms_norm(x, (s.hidden,), _t(L["norm1"]), eps=s.rms_eps)
        q = F.linear(h, _t(L["wq"]), _t(L["bq"])).view(T, s.n_q_heads, d)
        k = F.linear(h, _t(L["wk"]), _t(L["bk"])).view(T, s.n_kv_heads, d)
        v = F.linear(h, _t(L["wv"]), _t(L["bv"])).view(T, s.n_kv_heads, d)
        q, k = rotary(q), rotary(k)
        o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.transpose(0, 1)[None],
                                           v.transpose(0, 1)[None], is_causal=True, enable_gqa=True)
        o = o[0].transpose(0, 1).reshape(T, s.q_dim)
        x = x + F.linear(o, _t(L["wo"]))
        h = F.rms_norm(x, (s.hidden,), _t(L["norm2"]), eps=s.rms_eps)
        x = x + F.linear(F.silu(F.linear(h, _t(L["wg"]))) * F.linear(h, _t(L["wu"])), _t(L["wd"]))
    return F.linear(F.rms_norm(x, (s.hidden,), _t(w.final_norm), eps=s.rms_eps), _t(w.lm_head)).numpy()


@pytest.fixture(scope="module")
def small():
    # sigma 0.2 so that attention and the FFN are far from their linear regime
    w = synth.make_weights(SMALL, seed=11, sigma=0.2)
    rng = np.random.default_rng(0)
    for L in w.layers:           # non-trivial norm gains so that a dropped gain would be seen
        L["norm1"] = synth.f64_to_bf16_bits(rng.uniform(0.5, 1.5, SMALL.hidden))
        L["norm2"] = synth.f64_to_bf16_bits(rng.uniform(0.5, 1.5, SMALL.hidden))
    w.final_norm = synth.f64_to_bf16_bits(rng.uniform(0.5, 1.5, SMALL.hidden))
    return w


def test_decoder_matches_library_evaluation(small):
    tokens = synth.uniform_ids(23, 7, 99, SMALL.vocab)
    ref = torch_logits_all_positions(small, tokens)
    m = oracle.Model(small)
    seq = m.new_seq(64)
    for t, tok in enumerate(tokens):
        lg = seq.forward([tok])
        np.testing.assert_allclose(lg, ref[t], rtol=0, atol=1e-11)
    assert np.abs(ref).max() > 0.5           # the comparison is not vacuous


def test_chunked_equals_token_by_token_and_causal_prefix(small):
    tokens = synth.uniform_ids(20, 8, 100, SMALL.vocab)
    m = oracle.Model(small)
    a, b = m.new_seq(64), m.new_seq(64)
    la = a.forward(tokens[:12])
    for tok in tokens[:11]:
        b.forward([tok], want_logits=False)
    lb = b.forward([tokens[11]])
    assert np.array_equal(la, lb)
    # appending more tokens and rewinding does not change what position 11 predicted
    a.forward(tokens[12:])
    a.truncate(11)
    assert np.array_equal(a.forward([tokens[11]]), la)


def test_float_build_tracks_double_build(small):
    tokens = synth.uniform_ids(16, 9, 101, SMALL.vocab)
    ld = oracle.Model(small, "double").new_seq(32).forward(tokens)
    lf = oracle.Model(small, "float").new_seq(32).forward(tokens)
    assert lf.dtype == np.float32
    assert np.abs(ld - lf).max() < 1e-4
    assert oracle.argmax(ld)[0] == oracle.argmax(lf)[0]


def test_rope_convention_closed_forms():
    d, theta = 16, 1e6
    e0 = np.zeros(d); e0[0] = 1.0
    for pos in (0, 1, 7, 1000):
        r = oracle.rope_apply(e0, pos, theta)
        # pair (0, d/2) has frequency 1: rotation by exactly `pos` radians, counter-clockwise
        assert r[0] == pytest.approx(np.cos(pos)) and r[d // 2] == pytest.approx(np.sin(pos))
        assert np.count_nonzero(np.round(r, 15)) <= 2
    last = np.zeros(d); last[d // 2 - 1] = 1.0
    r = oracle.rope_apply(last, 12345, theta)
    ang = 12345 * theta ** (-(d - 2) / d)
    assert r[d // 2 - 1] == pytest.approx(np.cos(ang)) and r[d - 1] == pytest.approx(np.sin(ang))
    rng = np.random.default_rng(5)
    q, k = rng.standard_normal(d), rng.standard_normal(d)
    assert np.array_equal(oracle.rope_apply(q, 0, theta), q)
    np.testing.assert_allclose(oracle.rope_apply(oracle.rope_apply(q, 5, theta), 9, theta),
                               oracle.rope_apply(q, 14, theta), atol=1e-12)
    base = oracle.rope_apply(q, 40, theta) @ oracle.rope_apply(k, 33, theta)
    for shift in (1, 100, 4000):
        assert oracle.rope_apply(q, 40 + shift, theta) @ oracle.rope_apply(k, 33 + shift, theta) == \
            pytest.approx(base, abs=1e-9)
    half = d // 2
    rq = oracle.rope_apply(q, 77, theta)
    np.testing.assert_allclose(rq[:half] ** 2 + rq[half:] ** 2, q[:half] ** 2 + q[half:] ** 2, atol=1e-12)


def test_argmax_lowest_index_and_gap():
    lg = np.array([0.5, 2.0, -1.0, 2.0, 1.25])
    assert oracle.argmax(lg) == (1, 0.0)
    lg[3] = 1.5
    assert oracle.argmax(lg) == (1, 0.5)


def test_episode_accounting_and_identical_groups():
    """Gated rollout on the tiny shape: converging groups have S_K = 0 and leave at the gate turn;
    decoded-token count follows the step-token closed form n_seq*A*(T - f*(T-K)) (Table 1 caption)."""
    shape = synth.ModelShape(1, 32, 2, 1, 16, 48, 64)
    w = synth.make_weights(shape, seed=3, sigma=0.3)
    cfg = synth.EpisodeConfig("mini", 4, 3, 5, 4, 3, 2, 16, (2,), 0.3, 0.5)
    conv = synth.converging_groups(cfg, seed=1)
    assert conv.sum() == 2
    P = synth.prompts(cfg, shape.vocab, seed=1)
    rec = oracle.run_episode(oracle.Model(w), P, lambda t: synth.observations(cfg, shape.vocab, 1, t, conv),
                             cfg.G, cfg.turns, cfg.act_len, cfg.action_mod, cfg.gate_turns, cfg.threshold)
    gate = rec["gate"][2]
    assert gate["bound"] == oracle.gate_bound(0.3, 3, 2)
    for g in range(cfg.n_groups):
        if conv[g]:
            assert gate["sums"][g] == 0 and gate["cut"][g]
            acts = rec["actions"][g * cfg.G:(g + 1) * cfg.G]
            assert np.all(acts[:, :2] == acts[0, :2]) and np.all(acts[:, 2:] == -1)
    n_cut = sum(gate["cut"].values())
    f = n_cut / cfg.n_groups
    n_seq = cfg.n_groups * cfg.G
    assert rec["decoded_tokens"] == round(n_seq * cfg.act_len * (cfg.turns - f * (cfg.turns - 2)))
    assert rec["final_live_groups"] == [g for g in range(cfg.n_groups) if not gate["cut"][g]]


def test_episode_with_members_that_finish_early():
    """A member that ends after step K generates K*A tokens and nothing more; the others are unaffected (their
    tokens equal those of the run without finishers, since sequences do not interact); a group whose last
    member ends leaves un-cut; the gate sees the ended members' shorter prefixes and their count."""
    shape = synth.ModelShape(1, 32, 2, 1, 16, 48, 64)
    w = synth.make_weights(shape, seed=3, sigma=0.3)
    cfg = synth.EpisodeConfig("mini", 4, 3, 5, 4, 3, 2, 16, (3,), 0.3, 0.0)      # no converging groups
    conv = synth.converging_groups(cfg, seed=1)
    P = synth.prompts(cfg, shape.vocab, seed=1)
    obs = lambda t: synth.observations(cfg, shape.vocab, 1, t, conv)
    run = lambda **kw: oracle.run_episode(oracle.Model(w), P, obs, cfg.G, cfg.turns, cfg.act_len, cfg.action_mod,
                                          cfg.gate_turns, 0.0, **kw)               # d_L = 0: the d clause never fires
    base = run()
    ends = {0: 1, 4: 2, 6: 1, 7: 2, 8: 3, 11: 4}                                   # group 2 (rows 6..8) ends entirely
    rec = run(finish_fn=lambda K, r: ends.get(r) == K)
    n_seq, A, T = cfg.n_groups * cfg.G, cfg.act_len, cfg.turns
    assert rec["decoded_tokens"] == A * sum(min(ends.get(r, T), T) for r in range(n_seq))
    assert rec["live_rows"][3] == [1, 2, 3, 5, 9, 10, 11] and rec["live_groups"][3] == [0, 1, 3]
    for t in range(T):
        rows = rec["live_rows"][t]
        assert np.array_equal(rec["tokens"][t][:, rows], base["tokens"][t][:, rows])
    assert rec["gate"][3]["n_done"] == {0: 1, 1: 1, 3: 0} and not any(rec["gate"][3]["cut"].values())
    assert list(rec["end_step"][[0, 4, 8, 11]]) == [1, 2, 3, 4] and rec["end_step"][1] > T
    # the two-clause gate retires the groups of which at least a third has ended
    rec2 = run(finish_fn=lambda K, r: ends.get(r) == K, tau_H=1 / 3)
    assert rec2["gate"][3]["cut"] == {0: True, 1: True, 3: False} and rec2["final_live_groups"] == [3]


def test_sampler_draws_from_softmax():
    """Gumbel-max sampling with counter-based uniforms: empirical frequencies over many (sequence,
    position) keys match softmax(logits / T); draws are reproducible and keyed, not positional."""
    logits = np.array([1.0, 0.2, -0.5, 2.1, 0.0, 1.4])
    T = 0.7
    p = np.exp(logits / T) / np.exp(logits / T).sum()
    n = 40000
    counts = np.zeros(6)
    for i in range(n):
        tok, gap = oracle.sample(logits, T, 12345, i // 200, i % 200)
        counts[tok] += 1
        assert gap >= 0
    sigma = np.sqrt(n * p * (1 - p))
    assert np.all(np.abs(counts - n * p) < 4.5 * sigma), (counts / n, p)
    assert oracle.sample(logits, T, 1, 3, 7) == oracle.sample(logits, T, 1, 3, 7)
    draws = {oracle.sample(logits, T, 1, s, 7)[0] for s in range(50)}
    assert len(draws) > 2                                  # the sequence id matters
    assert oracle.sample(logits, 1e-3, 5, 0, 0)[0] == 3     # T -> 0 recovers the greedy choice
    flat = [oracle.sample(np.zeros(4), 1.0, 9, s, 0)[0] for s in range(4000)]
    assert np.all(np.abs(np.bincount(flat, minlength=4) - 1000) < 150)
