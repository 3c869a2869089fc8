"""GPU divergence signals and two-clause gate vs the CPU checker.

Integer outputs and decisions must be equal; d_K and the bigram Jaccard distance are sums of correctly
rounded quotients taken in the same pair order on both sides, so they must be equal bit for bit; the
entropy goes through each side's own logarithm and is compared to 1e-13.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_05802_amd as sr
import synth

pytestmark = pytest.mark.gpu

RUNNING = 10 ** 6
GPU_DTYPE = np.dtype([(f[0], f[1]) + tuple(f[2:]) for f in sr.SIGNALS_FIELDS], align=True)


def run_gpu(acts, lens, d_L, tau_H, obs=None, end=None):
    assert GPU_DTYPE.itemsize == sr.SIGNALS_BYTES
    a = torch.from_numpy(acts).cuda()
    o = None if obs is None else torch.from_numpy(obs).cuda()
    e = None if end is None else torch.from_numpy(end).cuda()
    out = torch.full((len(lens), acts.shape[0], sr.SIGNALS_BYTES), 0xAB, dtype=torch.uint8, device="cuda")
    sr.sr_signals_batch(a, lens, d_L, tau_H, out, obs=o, end_step=e)
    torch.cuda.synchronize()
    return out.cpu().numpy().view(GPU_DTYPE)[..., 0]


def check(acts, lens, d_L=0.3, tau_H=0.5, obs=None, end=None):
    got = run_gpu(acts, lens, d_L, tau_H, obs, end)
    ref = oracle.signals_batch(acts, lens, d_L, tau_H, obs=obs, end_step=end)
    for k in ("lev_scaled", "lev_sum", "unique_prefix", "n_at_step", "unique_action", "unique_obs", "n_done", "cut_d", "cut_or"):
        assert np.array_equal(got[k], ref[k]), k
    assert np.array_equal(got["d_K"], ref["d_K"])
    assert np.array_equal(got["bigram_jaccard"], ref["bigram_jaccard"])
    assert np.allclose(got["action_entropy"], ref["action_entropy"], rtol=0, atol=1e-13)
    return ref


def make(n_groups, G, stride, alphabet, seed, p_done=0.35):
    acts, _ = synth.gate_actions(n_groups, G, stride, alphabet, seed=seed)
    rng = np.random.default_rng(seed + 1)
    obs = rng.integers(0, 3, size=acts.shape).astype(np.int32)
    end = np.where(rng.random((n_groups, G)) < p_done, rng.integers(1, stride + 1, size=(n_groups, G)),
                   RUNNING).astype(np.int32)
    return acts, obs, end


@pytest.mark.parametrize("G", [2, 3, 5, 8, 11, 16])
@pytest.mark.parametrize("lens", [[1], [8], [3, 9, 16], [17, 24], [30], [32], [1, 2, 3, 4, 5, 6, 7, 8]])
def test_signal_shapes_with_early_finishers(G, lens):
    stride = max(lens) + (3 if max(lens) < 30 else 0)
    acts, obs, end = make(517, G, stride, 4, seed=G * 100 + len(lens))     # several workgroups, ragged tail
    check(acts, lens, d_L=0.25, tau_H=0.5, obs=obs, end=end)


def test_equal_lengths_agree_with_the_gate_kernel():
    acts, _ = synth.gate_actions(4096, 8, 30, 64, seed=0)
    lens = [5, 10, 15]
    ref = check(acts, lens, d_L=0.3, tau_H=2.0)
    a = torch.from_numpy(acts).cuda()
    retire = torch.zeros((3, 4096), dtype=torch.uint8, device="cuda")
    sr.sr_gate_batch(a, lens, 0.3, None, retire)
    assert np.array_equal(retire.cpu().numpy(), ref["cut_d"])
    assert np.array_equal(ref["cut_or"], ref["cut_d"])                     # tau_H > 1 switches the clause off


def test_signals_workload_full_size():
    """65536 groups x G=8 x length 30 over 64 symbols with early finishers; K = 5, 10, 15."""
    acts, obs, end = make(65536, 8, 30, 64, seed=0)
    ref = check(acts, [5, 10, 15], d_L=0.12, tau_H=0.5, obs=obs, end=end)
    assert 0 < ref["cut_or"][1].mean() < 1 and (ref["cut_or"] >= ref["cut_d"]).all()
    assert (ref["cut_or"] != ref["cut_d"]).any()                           # the backup clause does fire


def test_degenerate_groups():
    G, K = 8, 12
    same = np.tile(np.arange(K, dtype=np.int32), (G, 1))
    apart = (np.arange(G)[:, None] * 100 + np.arange(K)[None, :]).astype(np.int32)
    acts = np.stack([same, apart, same, apart])
    end = np.array([[RUNNING] * G, [RUNNING] * G, [1] * G, [0, 1, 2, 3, 4, 5, 6, 7]], dtype=np.int32)
    ref = check(acts, [1, 6, 12], d_L=0.3, tau_H=1.0, obs=acts, end=end)
    assert ref["d_K"][2, 0] == 0.0 and ref["d_K"][2, 1] == 1.0
    assert ref["n_done"][2, 2] == G and ref["cut_or"][2, 3] == 1 and ref["n_at_step"][2, 3] == 0


def test_threshold_edge_is_strict_on_the_gpu():
    acts = np.array([[[1, 2, 3, 9], [1, 2, 3, 4]]], dtype=np.int32)       # d_4 = 1/4 with lengths 3 and 4
    end = np.array([[3, RUNNING]], dtype=np.int32)
    assert run_gpu(acts, [4], 0.25, 2.0, end=end)["cut_d"][0, 0] == 0
    assert run_gpu(acts, [4], 0.250001, 2.0, end=end)["cut_d"][0, 0] == 1


def test_bad_arguments():
    a = torch.zeros((4, 8, 10), dtype=torch.int32, device="cuda")
    out = torch.zeros((1, 4, sr.SIGNALS_BYTES), dtype=torch.uint8, device="cuda")
    for lens in ([0], [11], [33]):
        with pytest.raises(sr.SrError):
            sr.sr_signals_batch(a, lens, 0.3, 0.5, out)
    with pytest.raises(sr.SrError):
        sr.sr_signals_batch(a, [5], 1.5, 0.5, out)
    with pytest.raises(sr.SrError):
        sr.sr_signals_batch(torch.zeros((4, 1, 10), dtype=torch.int32, device="cuda"), [5], 0.3, 0.5, out)
    sr.sr_signals_batch(a[:0], [5], 0.3, 0.5, out)                         # no groups: nothing to do
