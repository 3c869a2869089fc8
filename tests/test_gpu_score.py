"""Teacher-forced log-likelihood pass and policy-gradient loss on the GPU vs the CPU checker.

The trajectories are the checker's own greedy rollout of the tiny episode; the GPU re-reads them through
sr_prefill_chunk (prompt, observations) and sr_score_chunk (action tokens).  Every per-token value
log softmax(logits)[token] differs from the fp64 checker by at most twice the logits bound (a logit and
the log-sum-exp each move by at most that bound), the per-sequence sums by that times the token count.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_05802_amd as sr
import synth
from paper_2605_05802_amd.runner import load_host_weights
from test_gpu_decoder import LOGIT_TOL, dev

pytestmark = pytest.mark.gpu

TOK_TOL = 2 * LOGIT_TOL


def oracle_rollout(shape, cfg, seed, sigma=0.02):
    w = synth.make_weights(shape, seed=0, sigma=sigma)
    conv = synth.converging_groups(cfg, seed)
    prompts = synth.prompts(cfg, shape.vocab, seed)
    obs_fn = lambda t: synth.observations(cfg, shape.vocab, seed, t, conv)
    rec = oracle.run_episode(oracle.Model(w), prompts, obs_fn, cfg.G, cfg.turns, cfg.act_len, cfg.action_mod,
                             (), cfg.threshold)                       # no gate: every trajectory runs to the end
    return w, prompts, obs_fn, rec


def oracle_scores(w, cfg, prompts, obs_fn, rec, mask_fn):
    """Per-turn per-token log-probabilities of the recorded action tokens, by the checker."""
    model = oracle.Model(w)
    n_seq = cfg.n_groups * cfg.G
    out = np.zeros((cfg.turns, n_seq, cfg.act_len))
    for r in range(n_seq):
        seq = model.new_seq(cfg.prompt_len + cfg.turns * (cfg.obs_len + cfg.act_len))
        last = seq.forward(prompts[r // cfg.G])
        for t in range(cfg.turns):
            last = seq.forward(obs_fn(t)[r])
            out[t, r], last = oracle.score(seq, last, rec["tokens"][t][:, r], mask_fn(t, r))
    return out


def gpu_scores(shape, cfg, w, prompts, obs_fn, rec, mask_fn, *, max_prefill_rows=0, page_tokens=32, rows=None):
    n_seq = cfg.n_groups * cfg.G
    rows = list(range(n_seq)) if rows is None else rows
    max_len = cfg.prompt_len + cfg.turns * (cfg.obs_len + cfg.act_len)
    ctx = sr.Context(shape, cfg.n_groups, cfg.G, cfg.threshold, page_tokens=page_tokens, max_seq_len=max_len,
                     max_turns=cfg.turns, action_mod=cfg.action_mod, max_prefill_rows=max_prefill_rows,
                     kv_pool_bytes=1 << 28)
    load_host_weights(ctx, w)
    ctx.sr_prefill_chunk(dev(prompts), True)
    out = np.zeros((cfg.turns, n_seq, cfg.act_len))
    tok_lp = torch.empty((n_seq, cfg.act_len), dtype=torch.float32, device="cuda")
    for t in range(cfg.turns):
        ctx.sr_prefill_chunk(dev(obs_fn(t)), False)
        acts = np.ascontiguousarray(rec["tokens"][t].T)               # [n_seq, act_len]
        mask = np.stack([np.asarray(mask_fn(t, r), dtype=np.uint8) for r in range(n_seq)])
        ctx.sr_score_chunk(dev(acts), dev(mask), tok_lp)
        torch.cuda.synchronize()
        out[t] = tok_lp.cpu().numpy()
    total = torch.empty(n_seq, dtype=torch.float64, device="cuda")
    ctx.sr_get_logprob(total)
    torch.cuda.synchronize()
    ctx.close()
    return out, total.cpu().numpy()


def test_tiny_episode_scores_match_the_checker():
    shape, cfg = synth.TINY, synth.TINY_EPISODE
    w, prompts, obs_fn, rec = oracle_rollout(shape, cfg, seed=0)
    rng = np.random.default_rng(0)
    masks = rng.random((cfg.turns, cfg.n_groups * cfg.G, cfg.act_len)) < 0.8
    mask_fn = lambda t, r: masks[t, r]
    ref = oracle_scores(w, cfg, prompts, obs_fn, rec, mask_fn)
    got, total = gpu_scores(shape, cfg, w, prompts, obs_fn, rec, mask_fn)
    err = np.abs(got - ref).max()
    print(f"per-token log-prob: worst error {err:.3e}; mean log-prob {ref[masks].mean():.3f}")
    assert err <= TOK_TOL
    assert (got[~masks] == 0).all()
    assert np.allclose(total, got.sum(axis=(0, 2)), rtol=0, atol=1e-4)          # the running sums are those tokens
    assert np.abs(total - ref.sum(axis=(0, 2))).max() <= TOK_TOL * masks.sum(axis=(0, 2)).max()
    # greedy tokens are the most likely ones: their log-probability beats the uniform one by a wide margin
    assert ref[masks].mean() > -np.log(shape.vocab)


def test_scoring_in_several_passes_gives_the_same_values():
    # a row cap below one chunk of the whole batch splits every call into several passes and LM-head blocks
    shape = synth.TINY
    cfg = synth.EpisodeConfig("score-long", 3, 4, 48, 2, 16, 40, 16, (), 0.3, 0.34)
    w, prompts, obs_fn, rec = oracle_rollout(shape, cfg, seed=1)
    mask_fn = lambda t, r: np.ones(cfg.act_len, dtype=bool)
    a, ta = gpu_scores(shape, cfg, w, prompts, obs_fn, rec, mask_fn)
    b, tb = gpu_scores(shape, cfg, w, prompts, obs_fn, rec, mask_fn, max_prefill_rows=256)
    assert np.abs(a - b).max() <= 1e-3 and np.abs(ta - tb).max() <= 1e-2
    ref = oracle_scores(w, cfg, prompts, obs_fn, rec, mask_fn)
    assert np.abs(a - ref).max() <= TOK_TOL and np.abs(b - ref).max() <= TOK_TOL


def test_running_sums_follow_their_sequences_through_compaction():
    shape, cfg = synth.TINY, synth.TINY_EPISODE
    w, prompts, obs_fn, rec = oracle_rollout(shape, cfg, seed=0)
    n_seq = cfg.n_groups * cfg.G
    ctx = sr.Context(shape, cfg.n_groups, cfg.G, cfg.threshold, page_tokens=32, max_seq_len=512, max_turns=cfg.turns,
                     action_mod=0, kv_pool_bytes=1 << 28)
    load_host_weights(ctx, w)
    ctx.sr_prefill_chunk(dev(prompts), True)
    ctx.sr_prefill_chunk(dev(obs_fn(0)), False)
    ctx.sr_score_chunk(dev(np.ascontiguousarray(rec["tokens"][0].T)))
    before = torch.empty(n_seq, dtype=torch.float64, device="cuda")
    ctx.sr_get_logprob(before)
    # retire the converging groups through the gate on identical / distinct action ids
    conv = synth.converging_groups(cfg, 0)
    ids = np.array([0 if conv[r // cfg.G] else r for r in range(n_seq)], dtype=np.int32)
    ctx.sr_set_actions(1, dev(ids))
    ctx.sr_gate(1)
    n_live = ctx.sr_retire_and_compact()
    keep = [r for r in range(n_seq) if not conv[r // cfg.G]]
    assert n_live * cfg.G == len(keep) and 0 < len(keep) < n_seq
    after = torch.empty(len(keep), dtype=torch.float64, device="cuda")
    ctx.sr_get_logprob(after)
    torch.cuda.synchronize()
    assert np.array_equal(after.cpu().numpy(), before.cpu().numpy()[keep])
    ctx.close()


def test_score_needs_a_context_and_rejects_bad_arguments():
    shape, cfg = synth.TINY, synth.TINY_EPISODE
    w = synth.make_weights(shape, seed=0)
    ctx = sr.Context(shape, cfg.n_groups, cfg.G, 0.3, page_tokens=32, max_seq_len=128, max_turns=4, kv_pool_bytes=1 << 27)
    load_host_weights(ctx, w)
    toks = torch.zeros((cfg.n_groups * cfg.G, 8), dtype=torch.int32, device="cuda")
    with pytest.raises(sr.SrError) as e:
        ctx.sr_score_chunk(toks)                                   # nothing predicts the first token yet
    assert e.value.status == sr.SR_E_STATE
    ctx.sr_prefill_chunk(dev(synth.prompts(cfg, shape.vocab, 0)), True)
    ctx.sr_score_chunk(toks)
    with pytest.raises(sr.SrError) as e:
        ctx.sr_score_chunk(torch.zeros((cfg.n_groups * cfg.G, 100), dtype=torch.int32, device="cuda"))
    assert e.value.status == sr.SR_E_ARG                           # beyond max_seq_len
    ctx.close()


def test_grpo_loss_matches_the_checker():
    rng = np.random.default_rng(3)
    n_groups, G = 37, 8
    lp = -rng.random(n_groups * G) * 300
    r = rng.integers(0, 2, size=n_groups * G).astype(np.float32)
    r[:3 * G] = 1.0                                                 # zero-variance groups
    r[3 * G:5 * G] = 0.0
    want_loss, want_A = oracle.grpo_loss(lp, r.astype(np.float64), G, 1e-6)
    adv = torch.empty(n_groups * G, dtype=torch.float32, device="cuda")
    scratch = torch.empty(n_groups, dtype=torch.float64, device="cuda")
    loss = torch.empty(1, dtype=torch.float64, device="cuda")
    sr.sr_grpo_loss(dev(lp), dev(r), G, 1e-6, adv, scratch, loss)
    torch.cuda.synchronize()
    A = adv.cpu().numpy()
    assert (A[:5 * G] == 0).all()                                   # exactly zero, not merely small
    assert np.allclose(A, want_A, rtol=1e-6, atol=1e-7)
    assert abs(loss.item() - want_loss) <= 1e-9 * max(1.0, abs(want_loss))


def test_scoring_a_few_hundred_rows_with_split_k_projections():
    """256 scored rows per call (64 sequences x 4 action tokens): between 129 and 1024 rows the thin projections
    are split along K, so the score path's final norm has partial sums to add; deep FFN so that the split is real."""
    shape = synth.ModelShape(1, 256, 4, 2, 64, 16896, 1024)
    cfg = synth.EpisodeConfig("score-mid", 8, 8, 16, 1, 4, 4, 16, (), 0.3, 0.4)
    w, prompts, obs_fn, rec = oracle_rollout(shape, cfg, seed=2)
    mask_fn = lambda t, r: np.ones(cfg.act_len, dtype=bool)
    ref = oracle_scores(w, cfg, prompts, obs_fn, rec, mask_fn)
    got, total = gpu_scores(shape, cfg, w, prompts, obs_fn, rec, mask_fn)
    err = np.abs(got - ref).max()
    print(f"mid-size scoring: worst per-token error {err:.3e}")
    assert err <= TOK_TOL
    assert np.abs(total - ref.sum(axis=(0, 2))).max() <= TOK_TOL * cfg.act_len
