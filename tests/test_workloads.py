"""The seeded input generators: deterministic, right shapes, bf16-exact values."""
import numpy as np
import torch

import workloads as wl


def test_round_bf16_matches_torch():
    rng = np.random.default_rng(0)
    a = (rng.standard_normal(10000) * 10.0 ** rng.integers(-6, 6, size=10000)).astype(np.float32)
    a[:4] = [0.0, -0.0, 1.0, 3.140625]
    ref = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    got = wl.round_bf16(a)
    np.testing.assert_array_equal(got, ref)
    bits = wl.to_bf16_bits(got)
    back = (bits.astype(np.uint32) << 16).view(np.float32)
    np.testing.assert_array_equal(back, got)


def test_weights_deterministic_and_shaped():
    w1, w2 = wl.make_weights(wl.C0), wl.make_weights(wl.C0)
    assert set(w1) == set(wl.weight_shapes(wl.C0))
    for n, s in wl.weight_shapes(wl.C0).items():
        assert w1[n].shape == s and w1[n].dtype == np.float32
        np.testing.assert_array_equal(w1[n], w2[n])
    assert abs(w1["emb"].std() - 0.02) < 2e-3
    assert abs(w1["dec.0.ln1.g"].mean() - 1.0) < 2e-2
    small = wl.scaled(wl.C1, n_enc=1, n_dec=1, vocab=512, d_model=64, d_ff=128, n_heads=2)
    wb = wl.make_weights(small)
    for a in wb.values():
        np.testing.assert_array_equal(a, wl.round_bf16(a))


def test_sources_and_lengths():
    ids, n = wl.make_sources(wl.C0)
    assert ids.shape == (1, 16) and n.tolist() == [16] and ids.min() >= 3 and ids.max() < 256
    ids, n = wl.make_sources(wl.C3)
    assert ids.shape == (32, 128) and n.min() >= 1 and n.max() <= 128
    assert 15 < np.median(n) < 45
    for b in range(32):
        assert (ids[b, n[b]:] == 0).all() and ids[b, :n[b]].min() >= 3 and ids[b, :n[b]].max() < 32768
    ml = wl.make_max_len(wl.C3, n)
    assert ml.min() >= 1 and ml.max() <= 128 and len(set(ml.tolist())) > 4
    ids4, n4 = wl.make_sources(wl.C4)
    assert ids4.shape == (8, 192) and (n4 == 192).all() and ids4.min() >= 0 and ids4.max() < 256
    # Zipf: low ranks dominate
    big = wl._zipf_ids(np.random.default_rng(1), 20000, 32768)
    assert big.min() >= 3 and big.max() <= 32767 and (big < 100).mean() > 0.3


def test_schedules():
    for k, mean in [(8, 2), (8, 4), (10, 2), (10, 5), (10, 3), (10, 7)]:
        cfg = wl.scaled(wl.C3, k=k)
        s = wl.make_schedule(cfg, mean, 4000)
        assert s.shape == (4000, 32) and s.min() >= 1 and s.max() <= k
        assert abs(s.mean() - mean) < 0.05
    assert (wl.make_schedule(wl.C2, 1, 5) == 1).all()
    assert (wl.make_schedule(wl.C2, 10, 5) == 10).all()
    assert abs(wl.geometric_ratio(10, 3) - 0.69372) < 1e-4
    assert abs(wl.geometric_ratio(10, 7) - 1.21279) < 1e-4
