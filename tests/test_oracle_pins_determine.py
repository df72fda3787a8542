"""Pins for the oracle's Determine Sparse Pattern (Alg. 3): Jensen-Shannon distance, the
last-query-block estimate, the gate.  CPU only."""
from __future__ import annotations

import math

import numpy as np
import pytest
from scipy.spatial.distance import jensenshannon

import oracle
from synth import bf16_bits_to_f32, random_qkv


def _dist(rng, n, zeros=0.0):
    p = rng.random(n) ** 3
    p[rng.random(n) < zeros] = 0.0
    p[0] += 1e-3
    return (p / p.sum()).astype(np.float32)


def test_js_distance_matches_scipy():
    rng = np.random.default_rng(1)
    for n in (2, 7, 64, 1000):
        for zeros in (0.0, 0.5):
            p, q = _dist(rng, n, zeros), _dist(rng, n, zeros)
            want = jensenshannon(p.astype(np.float64), q.astype(np.float64))   # natural log, returns the sqrt
            assert abs(oracle.js_distance(p, q) - want) < 1e-6
            assert abs(oracle.js_distance(p, q) - oracle.js_distance(q, p)) < 1e-12   # symmetric


def test_js_distance_closed_forms():
    n = 16
    u = np.full(n, 1.0 / n, dtype=np.float32)
    assert oracle.js_distance(u, u) == 0.0
    a = np.zeros(n, dtype=np.float32)
    b = np.zeros(n, dtype=np.float32)
    a[:4] = 0.25
    b[8:12] = 0.25
    assert abs(oracle.js_distance(a, b) - math.sqrt(math.log(2.0))) < 1e-7       # disjoint supports: the maximum
    e0 = np.zeros(n, dtype=np.float32)
    e0[3] = 1.0
    # one-hot against uniform: KL(e||m) = ln(2n/(n+1)), KL(u||m) = ln(2/(n+1))/n + (n-1)/n ln 2
    jsd = 0.5 * math.log(2 * n / (n + 1)) + 0.5 * (math.log(2 / (n + 1)) / n + (n - 1) / n * math.log(2))
    assert abs(oracle.js_distance(e0, u) - math.sqrt(jsd)) < 1e-7
    # two-point distributions (t, 1-t) vs (1-t, t): direct evaluation of the definition by hand
    t = 0.25
    p = np.array([t, 1 - t], dtype=np.float32)
    q = np.array([1 - t, t], dtype=np.float32)
    kl = t * math.log(t / 0.5) + (1 - t) * math.log((1 - t) / 0.5)
    assert abs(oracle.js_distance(p, q) - math.sqrt(kl)) < 1e-7
    with pytest.raises(ValueError):
        oracle.js_distance(np.array([-0.1, 1.1], dtype=np.float32), q)


def test_last_row_estimate_is_last_row_of_the_score_map_and_special_cases():
    N, d, B = 256, 16, 32
    qb, kb, _ = random_qkv(41, N, 1, 1, d, 1.5)
    q, k = bf16_bits_to_f32(qb)[:, 0], bf16_bits_to_f32(kb)[:, 0]
    a = oracle.last_row_estimate(q, k, B)
    full = oracle.softmax_rows(oracle.mean_logit_rows(q, k, B))
    assert np.array_equal(a, full[-1]) and abs(a.sum() - 1.0) < 1e-6
    # materialised: pooled logits of the last B queries against every key block, causal inside the last block
    x = (q[-B:].astype(np.float64) @ k.astype(np.float64).T) / np.sqrt(d)
    keep = np.ones((B, N), dtype=bool)
    keep[:, N - B:] = np.tril(np.ones((B, B), dtype=bool))
    pooled = np.array([x[:, j * B:(j + 1) * B][keep[:, j * B:(j + 1) * B]].mean() for j in range(N // B)])
    e = np.exp(pooled - pooled.max())
    np.testing.assert_allclose(a, e / e.sum(), rtol=1e-5, atol=1e-9)
    # Q = 0: uniform estimate, distance 0 to uniform
    a0 = oracle.last_row_estimate(np.zeros_like(q), k, B)
    np.testing.assert_allclose(a0, 1.0 / (N // B), rtol=1e-6)
    assert oracle.determine_pattern(a0, None, 0.3, 0.2)[1] < 1e-6
    # keys of one block aligned with every query: the estimate concentrates there and the head reads as sparse
    q1 = np.ones_like(q)
    k1 = np.zeros_like(k)
    k1[2 * B:3 * B] = 8.0
    a1 = oracle.last_row_estimate(q1, k1, B)
    assert a1.argmax() == 2 and a1[2] > 0.999
    shared, d_sparse, _ = oracle.determine_pattern(a1, None, 0.3, 0.2)
    assert not shared and d_sparse > 0.6


def test_gate_thresholds_are_strict_and_both_must_hold():
    n = 8
    u = np.full(n, 1.0 / n, dtype=np.float32)
    near = u.copy()
    near[0] += 0.02
    near[1] -= 0.02
    far = np.zeros(n, dtype=np.float32)
    far[0] = 1.0
    d_near_u = oracle.js_distance(near, u)
    assert 0.0 < d_near_u < 0.1
    assert oracle.determine_pattern(near, u, 0.3, 0.2)[0]
    assert not oracle.determine_pattern(near, far, 0.3, 0.2)[0]              # similar enough to uniform, not to a~
    assert not oracle.determine_pattern(far, far, 0.3, 0.2)[0]               # identical to a~ but too sparse
    assert oracle.determine_pattern(far, far, 0.9, 0.2)[0]
    assert not oracle.determine_pattern(u, u, 0.3, 0.0)[0]                   # d_sim = 0 is not < 0: strict
    assert not oracle.determine_pattern(u, u, 0.0, 0.2)[0]
    assert not oracle.determine_pattern(near, u, d_near_u, 1.0)[0]           # equal to the threshold fails
    assert oracle.determine_pattern(near, u, np.nextafter(d_near_u, 1.0), 1.0)[0]
    assert oracle.determine_pattern(near, None, 0.3, 0.0)[0] is False        # no representative: d_sim := 0, still strict
    assert oracle.determine_pattern(near, None, 0.3, 1e-9)[0]


def test_prefill_layer_with_gate_is_the_composition():
    N, Hq, Hkv, d, B = 256, 4, 2, 16, 32
    qb, kb, vb = random_qkv(43, N, Hq, Hkv, d, 1.5)
    q, k, v = (bf16_bits_to_f32(a) for a in (qb, kb, vb))
    h2c, piv = [0, 0, 1, 1], [0, 2]
    est = [oracle.last_row_estimate(q[:, h], k[:, h // 2], B) for h in range(Hq)]
    d13 = oracle.js_distance(est[1], est[0]), oracle.js_distance(est[3], est[2])
    tau = 0.5 * (d13[0] + d13[1])                   # between the two similarity distances: exactly one head passes
    out = oracle.prefill_layer(q, k, v, B, h2c, piv, 0.9, gate=(1.0, tau))
    want = [True, d13[0] < tau, True, d13[1] < tau]
    assert list(out["shared"]) == want and sum(want) == 3
    assert abs(out["dist"][1, 1] - d13[0]) < 1e-12 and out["dist"][0, 1] == 0.0
    plain = oracle.prefill_layer(q, k, v, B, h2c, piv, 0.9)
    for h in (1, 3):
        if want[h]:
            assert np.array_equal(out["o"][:, h], plain["o"][:, h])
        else:
            dense, _, _ = oracle.dense_rows(q[:, h], k[:, h // 2], v[:, h // 2], B, want_scores=False)
            assert np.array_equal(out["o"][:, h], dense)
    forced = oracle.prefill_layer(q, k, v, B, h2c, piv, 0.9, shared=[True, False, True, False])
    assert list(forced["shared"]) == [True, False, True, False]
