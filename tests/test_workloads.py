"""The seeded input generators: deterministic, of the stated shapes and distributions."""
import numpy as np

import workloads as wl


def test_configs_shapes():
    c1, c2, c3, c4 = (wl.get_config(i) for i in (1, 2, 3, 4))
    assert (c1.P, c2.P, c3.P, c4.P) == (128, 384, 384, 384)
    assert wl.get_config(0).P == 12 and wl.get_config("c2").T == 8192 and c4.L == 26


def test_draws_are_deterministic_and_independent():
    c = wl.get_config(1).with_(H=64, I=16)
    a = wl.expert_weights(c, 3, 2, 1)
    b = wl.expert_weights(c, 3, 2, 1)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    assert not np.array_equal(a[0], wl.expert_weights(c, 3, 2, 0)[0])
    s = wl.stacked_expert_weights(c, 3, 2, 3)
    assert np.array_equal(s[0][1], a[0]) and s[0].dtype == np.uint16 and s[1].shape == (3, 64, 16)
    w = wl.bf16_bits_to_f32(s[0])
    assert abs(w.std() - 0.02) < 2e-3 and abs(w.mean()) < 2e-3


def test_tuned_sets_and_aid_distribution():
    c2 = wl.get_config(2)
    tuned = wl.tuned_sets(c2)
    assert len(tuned) == 20
    for J in tuned:
        assert 2 <= len(J) <= 16 and np.all(np.diff(J) > 0) and J.min() >= 0 and J.max() < 64
    assert tuned[0].tolist() != wl.tuned_sets(c2, layer=1)[0].tolist() or len(tuned[0]) != len(wl.tuned_sets(c2, 1)[0])
    aid = wl.adapter_ids(c2)
    assert aid.dtype == np.int32 and aid.min() == 0 and aid.max() <= 20
    frac0 = (aid == 0).mean()
    assert abs(frac0 - 0.31) < 0.03                                   # Zipf(1.1) over 21 classes: base ~31 %
    aid1 = wl.adapter_ids(wl.get_config(1), T=20000)
    assert np.all(np.abs(np.bincount(aid1, minlength=5) / 20000 - 0.2) < 0.02)


def test_distinct_topk_ids():
    c3 = wl.get_config(3)
    ids = wl.distinct_topk_ids(c3, T=4096)
    assert ids.shape == (4096, 6) and ids.dtype == np.int32 and ids.min() >= 0 and ids.max() < 64
    assert all(len(set(r)) == 6 for r in ids.tolist())
    assert np.all(np.abs(np.bincount(ids.reshape(-1), minlength=64) / ids.size - 1 / 64) < 0.004)


def test_bias_table():
    c2 = wl.get_config(2)
    tuned = wl.tuned_sets(c2)
    b = wl.logit_bias_table(c2, tuned)
    assert b.shape == (21, 64) and np.all(b[0] == 0)
    for a, J in enumerate(tuned, 1):
        assert np.nonzero(b[a])[0].tolist() == J.tolist() and np.all(b[a, J] == 2.0)


def test_powerlaw_adapter_popularity():
    """alpha = 1 is uniform over the adapters; alpha = 0.1 sends most requests to the first adapter; ids stay in 1..n."""
    c2 = wl.get_config(2)
    T = 40000
    for n in (5, 20):
        u = wl.adapter_ids_powerlaw(c2, T, n, 1.0)
        assert u.min() == 1 and u.max() == n and u.dtype == np.int32
        share = np.bincount(u, minlength=n + 1)[1:] / T
        assert np.abs(share - 1.0 / n).max() < 0.01
        sk = wl.adapter_ids_powerlaw(c2, T, n, 0.1)
        share = np.bincount(sk, minlength=n + 1)[1:] / T
        assert abs(share[0] - (1.0 / n) ** 0.1) < 0.01          # P(x < 1/n) = (1/n)^alpha
        assert np.all(np.diff(share) <= 0.005)                   # popularity falls with the adapter index
    assert np.array_equal(wl.adapter_ids_powerlaw(c2, 100, 5, 0.3), wl.adapter_ids_powerlaw(c2, 100, 5, 0.3))
