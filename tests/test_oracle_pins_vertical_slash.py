"""Pins for the oracle's Search Vertical Slash Pattern (Alg. 5): vertical / slash sums, the
cumulative selection on a vector, the block lists.  CPU only."""
from __future__ import annotations

import itertools

import numpy as np
import pytest

import oracle
from synth import bf16_bits_to_f32, random_qkv
from tests.test_oracle_pins_paper_pattern import _quant, Q24


def _qk(seed, N, d, scale=1.0):
    q, k, _ = random_qkv(seed, N, 1, 1, d, scale)
    f = lambda a: bf16_bits_to_f32(a)[:, 0, :].astype(np.float64)
    return f(q), f(k)


@pytest.mark.parametrize("N,d,n_hat", [(96, 8, 32), (256, 16, 64), (200, 32, 200)])
def test_sums_match_materialised_numpy(N, d, n_hat):
    q, k = _qk(51, N, d, 1.5)
    x = (q @ k.T) / np.sqrt(d)
    x = np.where(np.tril(np.ones((N, N), dtype=bool)), x, -np.inf)[N - n_hat:]
    P = np.exp(x - x.max(axis=1, keepdims=True))
    P /= P.sum(axis=1, keepdims=True)
    want_v = P.sum(axis=0) / n_hat
    # slash o collects P[t][t-o]: the diagonals of the (n_hat x N) slab, counted from each row's own position
    want_s = np.zeros(N)
    for r in range(n_hat):
        t = N - n_hat + r
        want_s[:t + 1] += P[r, t::-1]
    want_s /= n_hat
    a_v, a_s = oracle.vertical_slash_sums(q, k, n_hat)
    np.testing.assert_allclose(a_v, want_v, rtol=2e-6, atol=1e-9)
    np.testing.assert_allclose(a_s, want_s, rtol=2e-6, atol=1e-9)
    assert abs(a_v.sum() - 1) < 1e-5 and abs(a_s.sum() - 1) < 1e-5


def test_sums_closed_form_for_zero_queries_and_a_dominant_key():
    N, d, n_hat = 64, 8, 16
    _, k = _qk(52, N, d)
    a_v, a_s = oracle.vertical_slash_sums(np.zeros((N, d)), k, n_hat)
    # uniform rows: query t spreads 1/(t+1) over keys 0..t, i.e. over offsets 0..t
    for s in (0, 10, N - n_hat, N - 3, N - 1):
        want = sum(1.0 / (t + 1) for t in range(max(s, N - n_hat), N)) / n_hat
        assert abs(a_v[s] - want) < 1e-7
    for o in (0, 5, N - n_hat, N - 2):
        want = sum(1.0 / (t + 1) for t in range(N - n_hat, N) if o <= t) / n_hat
        assert abs(a_s[o] - want) < 1e-7
    # one key that every query prefers: all vertical mass on it, the slash mass spread over n_hat offsets
    q1 = np.ones((N, d))
    k1 = np.zeros((N, d))
    k1[7] = 20.0
    a_v, a_s = oracle.vertical_slash_sums(q1, k1, n_hat)
    assert a_v[7] > 0.999 and a_v.argmax() == 7
    offs = np.array([t - 7 for t in range(N - n_hat, N)])
    np.testing.assert_allclose(a_s[offs], 1.0 / n_hat, rtol=1e-3)
    # a "slash" structure: query t matches the keys s with t - s = 3 (mod d), all with the same logit, so the
    # offsets 3, 3 + d, 3 + 2d, ... share the slash mass equally and the other offsets get almost none
    qs = np.zeros((N, d))
    ks = np.zeros((N, d))
    for t in range(N):
        qs[t, t % d] = 6.0
        ks[t, (t + 3) % d] = 6.0
    _, a_s2 = oracle.vertical_slash_sums(qs, ks, n_hat)
    assert abs(a_s2[3] - a_s2[3 + d]) < 1e-6 and a_s2[3] > 20 * a_s2[4]


def test_select_cumulative_hand_example_invariants_and_equivalence():
    v = np.array([0.125, 0.5, 0.0, 0.25, 0.125], dtype=np.float32)      # total 1
    keep, K = oracle.select_cumulative(v, 0.75)
    assert K == 2 and list(keep) == [0, 1, 0, 1, 0]                      # .5 + .25
    keep, K = oracle.select_cumulative(v, 0.8125)
    assert K == 3 and list(keep) == [1, 1, 0, 1, 0]                      # tie .125: lower index first
    keep, K = oracle.select_cumulative(v, 1.0)
    assert K == 4 and list(keep) == [1, 1, 0, 1, 1]                      # zeros are never needed
    assert oracle.select_cumulative(np.zeros(4, dtype=np.float32), 0.9)[1] == 0
    rng = np.random.default_rng(7)
    for n in (1, 5, 11):
        v = (rng.integers(0, 6, size=n) / 16.0).astype(np.float32)
        for gamma in (0.3, 0.9):
            keep, K = oracle.select_cumulative(v, gamma)
            u = [_quant(x) for x in v]
            tot, gq = sum(u), _quant(np.float32(gamma))
            if tot == 0:
                assert K == 0
                continue
            best = next(r for r in range(1, n + 1)
                        if any(sum(u[i] for i in c) * Q24 >= gq * tot for c in itertools.combinations(range(n), r)))
            assert K == best == int(keep.sum())
            assert sum(u[i] for i in range(n) if keep[i]) == sum(sorted(u, reverse=True)[:K])
    # a vector is a map with one non-empty row: the selection agrees with Alg. 2's global variant on it
    n = 24
    v = rng.random(n).astype(np.float32) ** 3
    m = np.zeros((n, n), dtype=np.float32)
    m[n - 1] = v
    idx, cnt, K2 = oracle.build_mask_global(m, 0.9, forced=False)
    keep, K = oracle.select_cumulative(v, 0.9)
    assert K == K2 and list(np.flatnonzero(keep)) == list(idx[n - 1, :cnt[n - 1]])


def test_block_lists_match_token_level_brute_force():
    rng = np.random.default_rng(8)
    N, B = 160, 32
    n = N // B
    for trial in range(6):
        kv = (rng.random(N) < [0.0, 0.02, 0.05, 0.0, 0.3, 0.01][trial]).astype(np.uint8)
        ks = (rng.random(N) < [0.0, 0.0, 0.03, 0.02, 0.1, 0.01][trial]).astype(np.uint8)
        if trial == 3:
            ks[:] = 0
            ks[B] = 1            # the single offset B: realised only by token pairs of blocks (i, i-1)
        t = np.arange(N)[:, None]
        s = np.arange(N)[None, :]
        tok = (s <= t) & ((kv[None, :] > 0) | (ks[np.clip(t - s, 0, N - 1)] > 0))
        blk = tok.reshape(n, B, n, B).any(axis=(1, 3))
        for forced in (False, True):
            idx, cnt = oracle.vs_block_lists(kv, ks, B, forced)
            for i in range(n):
                want = {j for j in range(i + 1) if blk[i, j]}
                if forced:
                    want |= {0, i}
                assert list(idx[i, :cnt[i]]) == sorted(want), (trial, forced, i)
                assert np.all(idx[i, cnt[i]:] == -1)


def test_vertical_slash_pattern_is_the_composition_of_its_stages():
    N, d, B = 256, 16, 32
    qb, kb, vb = random_qkv(53, N, 1, 1, d, 3.0)
    q, k, v = (bf16_bits_to_f32(a)[:, 0] for a in (qb, kb, vb))
    idx, cnt, a_v, a_s, keep_v, keep_s = oracle.vertical_slash_pattern(q, k, B, 0.6)
    av2, as2 = oracle.vertical_slash_sums(q, k, B)
    assert np.array_equal(a_v, av2) and np.array_equal(a_s, as2)
    assert np.array_equal(keep_v, oracle.select_cumulative(a_v, 0.6)[0])
    assert np.array_equal(keep_s, oracle.select_cumulative(a_s, 0.6)[0])
    i2, c2 = oracle.vs_block_lists(keep_v, keep_s, B, True)
    assert np.array_equal(idx, i2) and np.array_equal(cnt, c2)
    assert 0 < cnt.sum() <= (N // B) * (N // B + 1) // 2
    # kept offsets/keys reach gamma of their vectors
    assert a_v[keep_v > 0].sum() >= 0.6 - 1e-6 and a_s[keep_s > 0].sum() >= 0.6 - 1e-6


def test_layer_functions_route_failing_and_unclustered_heads_to_the_vertical_slash_pattern():
    N, Hq, Hkv, d, B = 256, 4, 2, 16, 32
    qb, kb, vb = random_qkv(54, N, Hq, Hkv, d, 3.0)
    q, k, v = (bf16_bits_to_f32(a) for a in (qb, kb, vb))
    out = oracle.prefill_layer(q, k, v, B, [0, 0, -1, 0], [0], 0.6, shared=[True, False, False, True],
                               fallback="vertical_slash")
    for h in (1, 2):        # head 1 fails the gate, head 2 has no cluster
        idx, cnt = oracle.vertical_slash_pattern(q[:, h], k[:, h // 2], B, 0.6)[:2]
        want = oracle.masked_rows(q[:, h], k[:, h // 2], v[:, h // 2], B, idx, cnt)
        assert np.array_equal(out["o"][:, h], want)
    want3 = oracle.masked_rows(q[:, 3], k[:, 1], v[:, 1], B, out["kb_idx"][0], out["kb_cnt"][0])
    assert np.array_equal(out["o"][:, 3], want3)
    layers = [{"q": q, "k": k, "v": v, "head_to_cluster": [0, 0, -1, 0]}]
    res, _ = oracle.prefill_layers_dict(layers, B, 0.6, 10.0, 0.0, fallback="vertical_slash")   # tau 0: nobody shares
    assert list(res[0]["role"]) == [-1, -1, -1, -1]
    for h in range(4):
        idx, cnt = oracle.vertical_slash_pattern(q[:, h], k[:, h // 2], B, 0.6)[:2]
        assert np.array_equal(res[0]["o"][:, h], oracle.masked_rows(q[:, h], k[:, h // 2], v[:, h // 2], B, idx, cnt))


# ---- attention over the token-level pattern (Alg. 5's mask under Sec. 5.1's A(Q,K,V,M)) ----------------------
def _token_brute(q, k, v, B, keep_v, keep_s, forced):
    """fp64 numpy on the materialised N x N boolean mask."""
    N, d = q.shape
    t, s = np.arange(N)[:, None], np.arange(N)[None, :]
    allow = (s <= t) & (keep_v.astype(bool)[None, :] | keep_s.astype(bool)[np.clip(t - s, 0, N - 1)])
    if forced:
        allow |= (s <= t) & ((s // B == 0) | (s // B == t // B))
    x = (q.astype(np.float64) @ k.astype(np.float64).T) / np.sqrt(d)
    x = np.where(allow, x, -np.inf)
    mx = np.where(np.isfinite(x.max(1, keepdims=True)), x.max(1, keepdims=True), 0.0)
    p = np.where(allow, np.exp(x - mx), 0.0)
    den = p.sum(1, keepdims=True)
    return np.where(den > 0, p / np.where(den > 0, den, 1.0), 0.0) @ v.astype(np.float64), allow


@pytest.mark.parametrize("forced", [True, False])
def test_token_pattern_attention_vs_materialised_mask(forced):
    rng = np.random.default_rng(31)
    N, d, B = 192, 32, 32
    q, k, v = (rng.standard_normal((N, d)).astype(np.float32) * 1.3 for _ in range(3))
    keep_v = (rng.random(N) < 0.08).astype(np.uint8)
    keep_s = (rng.random(N) < 0.05).astype(np.uint8)
    keep_s[0] = 0                       # without forced blocks some queries then have no allowed key at all
    want, allow = _token_brute(q, k, v, B, keep_v, keep_s, forced)
    got = oracle.vs_token_rows(q, k, v, B, keep_v, keep_s, forced)
    assert np.abs(got - want).max() <= 1e-5
    if not forced:
        empty = ~allow.any(1)
        assert empty.any() and np.all(got[empty] == 0.0)
    rows = [1, 4]
    sub = oracle.vs_token_rows(q, k, v, B, keep_v, keep_s, forced, rows=rows)
    assert np.array_equal(sub, np.concatenate([got[i * B:(i + 1) * B] for i in rows]))


def test_token_pattern_attention_special_cases():
    rng = np.random.default_rng(32)
    N, d, B = 128, 16, 32
    q, k, v = (rng.standard_normal((N, d)).astype(np.float32) for _ in range(3))
    zeros, ones = np.zeros(N, np.uint8), np.ones(N, np.uint8)
    dense, _, _ = oracle.dense_rows(q, k, v, B, want_scores=False)
    # every key kept, or every offset kept: the causal dense result
    assert np.abs(oracle.vs_token_rows(q, k, v, B, ones, zeros, False) - dense).max() <= 1e-6
    assert np.abs(oracle.vs_token_rows(q, k, v, B, zeros, ones, False) - dense).max() <= 1e-6
    # only offset 0: every query sees itself alone
    only0 = zeros.copy(); only0[0] = 1
    assert np.abs(oracle.vs_token_rows(q, k, v, B, zeros, only0, False) - v).max() <= 1e-6
    # one vertical line at s0: v[s0] from t = s0 on, nothing before
    s0 = 37
    one = zeros.copy(); one[s0] = 1
    got = oracle.vs_token_rows(q, k, v, B, one, zeros, False)
    assert np.all(got[:s0] == 0.0) and np.abs(got[s0:] - v[s0]).max() <= 1e-6
    # nothing kept but the forced blocks: the block pattern {0, i}
    idx, cnt = oracle.vs_block_lists(zeros, zeros, B, True)
    assert np.abs(oracle.vs_token_rows(q, k, v, B, zeros, zeros, True) - oracle.masked_rows(q, k, v, B, idx, cnt)).max() <= 1e-6
    # the token pattern never holds more than its block superset: a kept key in a block lists the whole block
    kv = zeros.copy(); kv[40] = 1
    idx, cnt = oracle.vs_block_lists(kv, zeros, B, True)
    tok = oracle.vs_token_rows(q, k, v, B, kv, zeros, True)
    blk = oracle.masked_rows(q, k, v, B, idx, cnt)
    assert np.abs(tok[:B] - blk[:B]).max() <= 1e-6 and np.abs(tok[2 * B:] - blk[2 * B:]).max() > 1e-3
