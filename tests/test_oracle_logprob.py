"""Pins for the checker's teacher-forced log-likelihood (Appendix C.2) and policy-gradient loss (Section 2.1).

Expected values are closed forms, hand-worked numbers, or library routines (torch's log_softmax over the
whole-sequence logits assembled from torch ops in test_oracle_decoder) -- never the checker's own output.
"""
import math

import numpy as np
import torch
import torch.nn.functional as F

import oracle
import synth
from test_oracle_decoder import SMALL, torch_logits_all_positions


def test_logprob_closed_forms():
    V = 37
    assert abs(oracle.logprob(np.full(V, 3.25), 5) + math.log(V)) < 1e-15          # uniform: -ln V
    for x in (-4.0, 0.0, 0.5, 30.0):                                                # two classes: -log(1 + e^x)
        assert abs(oracle.logprob(np.array([0.0, x]), 0) + math.log1p(math.exp(x))) < 1e-12
    rng = np.random.default_rng(0)
    lg = rng.normal(0, 4, size=V)
    lps = np.array([oracle.logprob(lg, v) for v in range(V)])
    assert abs(np.exp(lps).sum() - 1.0) < 1e-13                                    # a probability distribution
    assert np.allclose(lps, [oracle.logprob(lg + 1000.0, v) for v in range(V)], rtol=0, atol=1e-10)  # shift invariant
    assert np.allclose(lps, F.log_softmax(torch.from_numpy(lg), dim=0).numpy(), rtol=0, atol=1e-13)
    assert oracle.logprob(np.array([0.0, 800.0]), 1) == 0.0                          # no overflow


def test_zero_lm_head_scores_minus_log_vocab_per_action_token():
    # a model whose LM head is all zeros assigns every token probability 1/V whatever the prefix
    w = synth.make_weights(SMALL, seed=3)
    w.lm_head[...] = 0
    seq = oracle.Model(w).new_seq(64)
    last = seq.forward([1, 2, 3])
    mask = [0, 1, 1, 0, 1, 0]
    lp, _ = oracle.score(seq, last, [7, 8, 9, 10, 11, 12], mask)
    assert np.allclose(lp, -math.log(SMALL.vocab) * np.array(mask), rtol=0, atol=1e-13)


def test_score_matches_library_log_softmax_with_the_one_position_shift():
    # the logits at position t-1 predict the token at position t; observation positions are masked out
    w = synth.make_weights(SMALL, seed=4, sigma=0.2)
    rng = np.random.default_rng(1)
    prompt = rng.integers(0, SMALL.vocab, size=5).astype(np.int32)
    traj = rng.integers(0, SMALL.vocab, size=12).astype(np.int32)
    mask = np.array([0, 0, 0, 1, 1, 0, 0, 0, 1, 1, 1, 1])
    full = np.concatenate([prompt, traj])
    ref_logits = torch.from_numpy(torch_logits_all_positions(w, full))
    ref_lsm = F.log_softmax(ref_logits, dim=-1).numpy()
    want = np.array([ref_lsm[len(prompt) + j - 1, traj[j]] for j in range(len(traj))]) * mask

    seq = oracle.Model(w).new_seq(64)
    last = seq.forward(prompt)
    lp, _ = oracle.score(seq, last, traj, mask)
    assert np.allclose(lp, want, rtol=0, atol=1e-9)
    assert (lp[mask == 0] == 0).all()
    # chunking the trajectory does not change the per-token values
    seq2 = oracle.Model(w).new_seq(64)
    last2 = seq2.forward(prompt)
    a, last2 = oracle.score(seq2, last2, traj[:7], mask[:7])
    b, _ = oracle.score(seq2, last2, traj[7:], mask[7:])
    assert np.allclose(np.concatenate([a, b]), lp, rtol=0, atol=1e-12)


def test_grpo_loss_hand_worked():
    # G = 2, rewards (1, 0): mean 1/2, population sigma 1/2 -> A = +-(1/2)/(1/2 + eps);
    # second group has equal rewards -> both advantages exactly 0 (Section 2.1)
    eps = 1e-6
    lp = np.array([-3.0, -5.0, -2.0, -7.0])
    r = np.array([1.0, 0.0, 0.3, 0.3])
    loss, A = oracle.grpo_loss(lp, r, 2, eps)
    a = 0.5 / (0.5 + eps)
    assert np.allclose(A, [a, -a, 0.0, 0.0], rtol=0, atol=1e-15) and A[2] == 0.0 and A[3] == 0.0
    assert abs(loss - (-(a * -3.0 + -a * -5.0) / 4)) < 1e-15
    # a batch of zero-variance groups has zero loss: nothing to learn from it
    assert oracle.grpo_loss(np.array([-1.0, -2.0, -3.0]), np.array([1.0, 1.0, 1.0]), 3)[0] == 0.0
    # advantages are invariant to shifting all rewards of a group; the loss flips sign with the rewards
    l1, A1 = oracle.grpo_loss(lp[:2], np.array([5.0, 4.0]), 2, eps)
    assert np.allclose(A1, [a, -a], rtol=0, atol=1e-12)
    l2, _ = oracle.grpo_loss(lp[:2], np.array([4.0, 5.0]), 2, eps)
    assert abs(l1 + l2) < 1e-15
