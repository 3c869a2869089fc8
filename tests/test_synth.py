"""The seeded input generators: determinism, counter-based access, and the stated distributions."""
import numpy as np

import synth


def test_counter_based_and_deterministic():
    a = synth.fill_normal_bf16(1000, seed=0, stream=5)
    b = synth.fill_normal_bf16(1000, seed=0, stream=5)
    assert np.array_equal(a, b)
    assert np.array_equal(synth.fill_normal_bf16(100, 0, 5, first=300), a[300:400])
    assert not np.array_equal(synth.fill_normal_bf16(1000, 1, 5), a)
    assert not np.array_equal(synth.fill_normal_bf16(1000, 0, 6), a)


def test_splitmix64_published_vector():
    # first outputs of SplitMix64 seeded with 1234567 (reference implementation by Vigna)
    L = synth.lib()
    assert [L.srs_draw(1234567, i) for i in range(3)] == [6457827717110365317, 3203168211198807973,
                                                          9817491932198370423]


def test_weights_are_normal_0_02():
    x = synth.bf16_bits_to_f32(synth.fill_normal_bf16(1 << 20, 0, 17)).astype(np.float64)
    assert abs(x.mean()) < 1e-4
    assert abs(x.std() - 0.02) < 2e-4
    assert abs(np.mean(np.abs(x) < 0.02) - 0.6827) < 3e-3
    assert abs(np.mean(x ** 4) / x.var() ** 2 - 3.0) < 0.05
    w = synth.make_weights(synth.TINY)
    assert w.layers[1]["wd"].shape == (256, 688) and w.embed.shape == (1024, 256)
    assert np.all(w.layers[0]["norm1"] == 0x3F80)


def test_bf16_rounding_is_nearest_even():
    v = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -8 + 2 ** -20, -0.3])
    bits = synth.f64_to_bf16_bits(v)
    back = synth.bf16_bits_to_f32(bits)
    assert list(back[:4]) == [1.0, 1.0, 1.0 + 2 ** -6, 1.0 + 2 ** -7]
    assert abs(back[4] + 0.3) < 2 ** -9


def test_episode_inputs():
    cfg = synth.TINY_EPISODE
    conv = synth.converging_groups(cfg, 0)
    assert conv.sum() == 2
    assert synth.converging_groups(synth.C4_EPISODE, 0).sum() == 26
    obs = synth.observations(cfg, 1024, 0, 2, conv)
    assert obs.shape == (32, 16) and obs.min() >= 0 and obs.max() < 1024
    for g in range(cfg.n_groups):
        rows = obs[g * 8:(g + 1) * 8]
        assert bool(np.all(rows == rows[0])) == bool(conv[g])
    assert not np.array_equal(obs, synth.observations(cfg, 1024, 0, 3, conv))


def test_gate_workload_structure():
    acts, pidx = synth.gate_actions(4096, 8, 30, 64, seed=0)
    assert acts.shape == (4096, 8, 30) and acts.min() >= 0 and acts.max() < 64
    assert np.all(np.bincount(pidx, minlength=4) > 900)
    ident = np.all(acts == acts[:, :1, :], axis=(1, 2))
    assert np.all(ident[pidx == 3])                # p = 1.0: every member equals the leader
    agree = (acts == acts[:, :1, :]).mean(axis=(1, 2))
    assert agree[pidx == 0].mean() < agree[pidx == 1].mean() < agree[pidx == 2].mean() < 1.0
