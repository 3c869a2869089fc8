"""GPU gate vs the CPU checker: every pairwise-distance sum and every retire bit must be equal."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_05802_amd as sr
import synth

pytestmark = pytest.mark.gpu


def run_gpu(acts, lens, thr, fn=None):
    a = torch.from_numpy(acts).cuda()
    n_groups = acts.shape[0]
    sums = torch.full((len(lens), n_groups), -7, dtype=torch.int32, device="cuda")
    retire = torch.full((len(lens), n_groups), 9, dtype=torch.uint8, device="cuda")
    (fn or sr.sr_gate_batch)(a, lens, thr, sums, retire)
    torch.cuda.synchronize()
    return sums.cpu().numpy(), retire.cpu().numpy()


def check(acts, lens, thr):
    """Both decompositions of the gate (one lane per pair; one workgroup per group with anti-diagonals in LDS)
    against the checker: every sum and every decision equal."""
    s_ref, r_ref = oracle.gate_batch(acts, lens, thr)
    for fn in (sr.sr_gate_batch, sr.sr_gate_batch_antidiag):
        s_gpu, r_gpu = run_gpu(acts, lens, thr, fn)
        assert np.array_equal(s_gpu, s_ref), fn.__name__
        assert np.array_equal(r_gpu, r_ref), fn.__name__
    return s_ref, r_ref


def test_gate_workload_full_size():
    """65536 groups x G=8 x length 30 over 64 symbols; prefixes 5, 10, 15; threshold 0.3."""
    acts, pidx = synth.gate_actions(65536, 8, 30, 64, seed=0)
    sums, retire = check(acts, [5, 10, 15], 0.3)
    assert np.all(sums[:, pidx == 3] == 0) and np.all(retire[:, pidx == 3] == 1)
    assert 0.3 < retire[1].mean() < 0.8          # the workload straddles the threshold


@pytest.mark.parametrize("G", [2, 3, 5, 8, 11, 16])
@pytest.mark.parametrize("lens", [[1], [8], [3, 9, 16], [17, 24], [30], [32], [1, 2, 3, 4, 5, 6, 7, 8]])
def test_gate_shapes(G, lens):
    stride = max(lens) + (3 if max(lens) < 30 else 0)
    n_groups = 517                                  # several workgroups and a ragged tail
    acts, _ = synth.gate_actions(n_groups, G, stride, 5, seed=G * 100 + len(lens))
    check(acts, lens, 0.25)


def test_gate_adversarial_sequences():
    rng = np.random.default_rng(0)
    G, K = 8, 16
    cases = []
    base = rng.integers(0, 3, size=K)
    cases.append(np.tile(base, (G, 1)))                                           # identical
    cases.append(np.arange(G)[:, None] * 100 + np.arange(K)[None, :])             # nothing shared
    cases.append(np.stack([np.roll(base, s) for s in range(G)]))                  # shifts: insert+delete paths
    cases.append(np.stack([np.repeat(np.arange(K // 2), 2) if i % 2 else np.tile(np.arange(K // 2), 2)
                           for i in range(G)]))
    cases.append(np.stack([np.full(K, i % 2) for i in range(G)]))                 # two constant camps
    cases.append(rng.integers(-2**31, 2**31 - 1, size=(G, K)))                    # full int32 range
    acts = np.stack(cases).astype(np.int32)
    for thr in (0.0, 0.12, 0.3, 1.0):
        check(acts, [4, 10, 16], thr)


def test_gate_threshold_edge_is_strict():
    """One member differs in one step: S = G-1 = 7; choose d_L so that 7 sits exactly on the bound."""
    G, K = 8, 10
    acts = np.tile(np.arange(K, dtype=np.int32), (1, G, 1))
    acts[0, 3, 4] = 99
    s, r = check(acts, [K], 7 / 280)          # d_K == d_L: not cut
    assert s[0, 0] == 7 and r[0, 0] == 0
    s, r = check(acts, [K], 0.025001)
    assert r[0, 0] == 1


def test_gate_empty_batch_is_a_noop():
    a = torch.zeros((1, 8, 30), dtype=torch.int32, device="cuda")
    import ctypes
    lens = (ctypes.c_int * 1)(5)
    assert sr.lib().sr_gate_batch(a.data_ptr(), 0, 8, 30, lens, 1, 0.3, None, None, None) == 0


def test_device_weight_fill_matches_host_generator():
    """The device fill used for multi-gigabyte models is bit-identical to the host generator."""
    shape = synth.ModelShape(2, 128, 4, 2, 64, 256, 512)
    host = synth.make_weights(shape, seed=7)
    embed, lm, fn, layers = synth.make_weights_device(shape, seed=7)
    same = lambda t, a: np.array_equal(t.cpu().numpy().view(np.uint16), a)
    assert same(embed, host.embed) and same(lm, host.lm_head) and same(fn, host.final_norm)
    for l in range(2):
        for k, v in host.layers[l].items():
            assert same(layers[l][k], v), (l, k)
