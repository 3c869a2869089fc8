"""Pins for the checker's "bf16 contract" mode.

The mode evaluates the decoder exactly (fp64) except that activations are rounded to bf16 at the
points where a bf16 matrix-core implementation has to round them.  The parity tests use its distance
from the exact evaluation as the measure of what bf16 operands cost at a given shape, so both the
rounding itself and the set of rounding points are fixed here by something other than the checker:

  - the rounding against hand-worked binary values (ties to even, a carry into the exponent, the
    intermediate single-precision step, negative values);
  - the set of points against a whole-sequence evaluation assembled from torch CPU routines in fp64
    with explicit `.to(float32).to(bfloat16)` casts (the library's own round-to-nearest-even) at the
    listed points -- and the same evaluation with any one point left out, with one point added, or with
    truncation instead of rounding must NOT match, so a mode that rounds more, less or differently than
    stated fails here.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
import synth

SMALL = synth.ModelShape(n_layers=2, hidden=64, n_q_heads=4, n_kv_heads=2, head_dim=16, ffn=96, vocab=50,
                         rms_eps=1e-6, rope_theta=1e4)

POINTS = ("norm", "q", "k", "v", "prob", "attn", "ffn")


def test_rounding_hand_worked_values():
    r = oracle.bf16_round
    # bf16 keeps 8 significant bits: the spacing in [1, 2) is 2^-7
    assert r(1.0) == 1.0 and r(0.0) == 0.0 and r(-2.5) == -2.5
    assert r(1 + 2 ** -7) == 1 + 2 ** -7                       # representable
    assert r(1 + 2 ** -8) == 1.0                               # tie: the even significand (…0) wins, downwards
    assert r(1 + 3 * 2 ** -8) == 1 + 2 ** -6                   # tie: the even significand wins, upwards
    assert r(1 + 2 ** -8 + 2 ** -20) == 1 + 2 ** -7            # just above the tie
    assert r(1 + 2 ** -8 - 2 ** -20) == 1.0                    # just below the tie
    assert r(2 - 2 ** -8) == 2.0                               # tie that carries into the exponent
    assert r(2 - 2 ** -8 - 2 ** -20) == 2 - 2 ** -7
    assert r(-(1 + 3 * 2 ** -8)) == -(1 + 2 ** -6)             # sign-symmetric
    assert r(3.0e-3) == pytest.approx(3.0e-3, rel=2 ** -8) and r(3.0e-3) != 3.0e-3
    # the value passes through single precision first: 2^-40 above a tie is lost there, so the tie rule applies
    assert r(1 + 2 ** -8 + 2 ** -40) == 1.0
    # truncation would give 1 + 2^-7 - ... -> 1.0 for everything below 1 + 2^-7; rounding does not
    assert r(1 + 2 ** -7 - 2 ** -12) == 1 + 2 ** -7
    # agreement with the library cast on a spread of magnitudes
    rng = np.random.default_rng(0)
    x = rng.standard_normal(4000) * np.exp(rng.uniform(-20, 20, 4000))
    want = torch.from_numpy(x).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(np.array([r(v) for v in x]), want)


def _t(bits):
    return torch.from_numpy(synth.bf16_bits_to_f32(bits).astype(np.float64))


def _rne(x):
    return x.to(torch.float32).to(torch.bfloat16).to(torch.float64)


def _trunc(x):
    bits = x.to(torch.float32).view(torch.int32) & -65536
    return bits.view(torch.float32).to(torch.float64)


def contract_logits(w, tokens, points=POINTS, rnd=_rne, extra=()):
    """[T, vocab] logits of the whole sequence with activations rounded at `points`:
    norm  output of every RMSNorm (the operand of the q/k/v, gate/up and LM-head projections)
    q     rotated queries                 k, v  rotated keys and the values, as stored
    prob  exp(score - row maximum), rounded BEFORE the division by the sum of the unrounded exponentials
    attn  per-head attention output (the operand of the output projection)
    ffn   silu(gate) * up (the operand of the down projection)
    `extra` names further places, used only to show that rounding there as well is detected."""
    s = w.shape
    T, d, half, rep = len(tokens), s.head_dim, s.head_dim // 2, s.n_q_heads // s.n_kv_heads
    R = lambda name, x: rnd(x) if (name in points or name in extra) else x
    x = F.embedding(torch.as_tensor(tokens, dtype=torch.long), _t(w.embed))
    inv_freq = torch.tensor(s.rope_theta, dtype=torch.float64) ** (-torch.arange(half, dtype=torch.float64) * 2 / d)
    ang = torch.arange(T, dtype=torch.float64)[:, None] * inv_freq[None, :]
    rot = torch.polar(torch.ones_like(ang), ang)

    def rotary(v):
        z = torch.complex(v[..., :half], v[..., half:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    causal = torch.ones(T, T, dtype=torch.bool).tril()
    for L in w.layers:
        h = R("norm", F.rms_norm(x, (s.hidden,), _t(L["norm1"]), eps=s.rms_eps))
        q = R("q", rotary(F.linear(h, _t(L["wq"]), _t(L["bq"])).view(T, s.n_q_heads, d)))
        k = R("k", rotary(F.linear(h, _t(L["wk"]), _t(L["bk"])).view(T, s.n_kv_heads, d)))
        v = R("v", F.linear(h, _t(L["wv"]), _t(L["bv"])).view(T, s.n_kv_heads, d))
        k, v = k.repeat_interleave(rep, dim=1), v.repeat_interleave(rep, dim=1)
        sc = R("score", torch.einsum("thd,uhd->htu", q, k) / np.sqrt(d)).masked_fill(~causal, -np.inf)
        e = torch.exp(sc - sc.max(dim=-1, keepdim=True).values)
        p = R("prob", e) / e.sum(dim=-1, keepdim=True)
        o = R("attn", torch.einsum("htu,uhd->thd", p, v)).reshape(T, s.q_dim)
        x = R("resid", x + F.linear(o, _t(L["wo"])))
        h = R("norm", F.rms_norm(x, (s.hidden,), _t(L["norm2"]), eps=s.rms_eps))
        a = R("ffn", F.silu(F.linear(h, _t(L["wg"]))) * F.linear(h, _t(L["wu"])))
        x = R("resid", x + F.linear(a, _t(L["wd"])))
    h = R("norm", F.rms_norm(x, (s.hidden,), _t(w.final_norm), eps=s.rms_eps))
    return F.linear(h, _t(w.lm_head)).numpy()


@pytest.fixture(scope="module")
def small():
    w = synth.make_weights(SMALL, seed=11, sigma=0.2)
    rng = np.random.default_rng(0)
    for L in w.layers:
        L["norm1"] = synth.f64_to_bf16_bits(rng.uniform(0.5, 1.5, SMALL.hidden))
        L["norm2"] = synth.f64_to_bf16_bits(rng.uniform(0.5, 1.5, SMALL.hidden))
    w.final_norm = synth.f64_to_bf16_bits(rng.uniform(0.5, 1.5, SMALL.hidden))
    return w


def _checker_contract_logits(w, tokens):
    m = oracle.Model(w)
    seq = m.new_seq(64)
    oracle.set_bf16_contract(True)
    try:
        return np.stack([seq.forward([t]) for t in tokens])
    finally:
        oracle.set_bf16_contract(False)


def test_contract_mode_rounds_exactly_at_the_listed_points(small):
    tokens = synth.uniform_ids(19, 4, 77, SMALL.vocab)
    got = _checker_contract_logits(small, tokens)
    want = contract_logits(small, tokens)
    # same values up to the order of fp64 additions
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-9)
    exact = contract_logits(small, tokens, points=())
    scale = np.abs(got - exact).max()
    assert scale > 1e-3                                         # the roundings are visible at this weight scale

    # every listed point matters, none may be missing
    for drop in POINTS:
        other = contract_logits(small, tokens, points=tuple(p for p in POINTS if p != drop))
        assert np.abs(other - got).max() > 1e-5, drop
    # and nothing else is rounded: the scores before the softmax, the residual stream
    for add in ("score", "resid"):
        other = contract_logits(small, tokens, extra=(add,))
        assert np.abs(other - got).max() > 1e-5, add
    # nearest-even, not truncation
    other = contract_logits(small, tokens, rnd=_trunc)
    assert np.abs(other - got).max() > 1e-4


def test_contract_mode_leaves_the_exact_mode_alone(small):
    tokens = synth.uniform_ids(12, 3, 55, SMALL.vocab)
    m = oracle.Model(small)
    exact = m.new_seq(32).forward(tokens)
    _checker_contract_logits(small, tokens)
    assert np.array_equal(exact, m.new_seq(32).forward(tokens))


def test_clone_continues_like_the_original(small):
    """Sequences do not interact: a copy taken after a common prefix continues bit for bit like a
    sequence that evaluated the prefix itself."""
    tokens = synth.uniform_ids(20, 5, 88, SMALL.vocab)
    m = oracle.Model(small)
    a = m.new_seq(32)
    a.forward(tokens[:11], want_logits=False)
    b = a.clone()
    c = m.new_seq(32)
    c.forward(tokens[:11], want_logits=False)
    assert len(b) == 11
    la, lb, lc = a.forward(tokens[11:]), b.forward(tokens[11:]), c.forward(tokens[11:])
    assert np.array_equal(la, lb) and np.array_equal(la, lc)
    a.forward([3])                                              # the copy is independent of the original
    assert len(b) == 20
