"""Pins for the oracle's paper-literal pattern construction (Sec. 5.2; Alg. 2 as printed):
block-mean logits, row softmax, one selection over the flattened map.  CPU only.

Each check ties the oracle to something other than itself: a materialised fp64 numpy
computation written differently (pooling identity, masked reshape), scipy's softmax,
closed forms, a hand-worked fixture, exhaustive subset search, and structural invariants.
"""
from __future__ import annotations

import itertools
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.special

import oracle
from synth import bf16_bits_to_f32, random_qkv

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
Q24 = 1 << 24


def _qk(seed, N, d, scale=1.0):
    q, k, _ = random_qkv(seed, N, 1, 1, d, scale)
    f = lambda a: bf16_bits_to_f32(a)[:, 0, :].astype(np.float64)
    return f(q), f(k)


# ---------------------------------------------------------------- block-mean logits

@pytest.mark.parametrize("N,d,B", [(64, 8, 16), (192, 16, 32), (256, 64, 64)])
def test_mean_logits_match_materialised_numpy(N, d, B):
    q, k = _qk(11, N, d)
    x = (q @ k.T) / np.sqrt(d)
    keep = np.tril(np.ones((N, N), dtype=bool))
    n = N // B
    num = np.where(keep, x, 0.0).reshape(n, B, n, B).sum(axis=(1, 3))
    cnt = keep.reshape(n, B, n, B).sum(axis=(1, 3))
    want = np.where(cnt > 0, num / np.maximum(cnt, 1), -np.inf)
    got = oracle.mean_logit_rows(q, k, B)
    assert np.all(np.isneginf(got[cnt == 0]))
    np.testing.assert_allclose(got[cnt > 0], want[cnt > 0], rtol=2e-6, atol=2e-6)
    # entry counts are what causality dictates
    assert cnt[0, 0] == B * (B + 1) // 2 and (n == 1 or cnt[1, 0] == B * B)


def test_mean_logits_full_blocks_equal_pooled_dot_product():
    """By linearity the average of q_t.k_s over a full block is (mean q).(mean k)."""
    N, d, B = 256, 32, 32
    q, k = _qk(12, N, d)
    n = N // B
    qb = q.reshape(n, B, d).mean(axis=1)
    kb = k.reshape(n, B, d).mean(axis=1)
    pooled = (qb @ kb.T) / np.sqrt(d)
    got = oracle.mean_logit_rows(q, k, B)
    for i in range(n):
        for j in range(i):
            assert abs(got[i, j] - pooled[i, j]) < 2e-6 * max(1.0, abs(pooled[i, j]))
    # the diagonal block is NOT the pooled product (only s <= t entries count)
    assert any(abs(got[i, i] - pooled[i, i]) > 1e-3 for i in range(n))


def test_mean_logits_row_subset_scale_and_swap_guard():
    N, d, B = 128, 16, 32
    q, k = _qk(13, N, d)
    full = oracle.mean_logit_rows(q, k, B)
    sub = oracle.mean_logit_rows(q, k, B, rows=[3, 1])
    assert np.array_equal(sub[0], full[3]) and np.array_equal(sub[1], full[1])
    twice = oracle.mean_logit_rows(q, k, B, scale=2.0 / np.sqrt(d))
    fin = np.isfinite(full)
    np.testing.assert_allclose(twice[fin], 2 * full[fin], rtol=1e-6, atol=1e-7)
    swapped = oracle.mean_logit_rows(k, q, B)
    assert np.abs(swapped[fin] - full[fin]).max() > 1e-3      # Q and K are not interchangeable
    # a constant added to every key along one direction shifts every block mean by the same amount
    e = np.zeros(d)
    e[0] = 1.0
    q1 = q.copy()
    q1[:, 0] = 1.0
    base = oracle.mean_logit_rows(q1, k, B)
    shifted = oracle.mean_logit_rows(q1, k + 3.0 * e, B)
    np.testing.assert_allclose(shifted[fin] - base[fin], 3.0 / np.sqrt(d), rtol=1e-5)


def test_zero_query_gives_uniform_rows():
    N, d, B = 160, 8, 32
    _, k = _qk(14, N, d)
    a = oracle.mean_logit_rows(np.zeros((N, d)), k, B)
    s = oracle.softmax_rows(a)
    for i in range(N // B):
        np.testing.assert_allclose(s[i, :i + 1], 1.0 / (i + 1), rtol=1e-6)
        assert np.all(s[i, i + 1:] == 0.0)


# ---------------------------------------------------------------- row softmax

def test_softmax_rows_matches_scipy_and_handles_minus_inf():
    rng = np.random.default_rng(3)
    a = (rng.standard_normal((9, 17)) * 5).astype(np.float32)
    a[np.triu_indices(9, 1, 17)] = -np.inf
    a[4, :] = -np.inf                                   # a row with nothing in it
    got = oracle.softmax_rows(a)
    want = scipy.special.softmax(a.astype(np.float64), axis=1)
    ok = [r for r in range(9) if r != 4]
    np.testing.assert_allclose(got[ok], want[ok], rtol=1e-6, atol=1e-12)
    assert np.all(got[4] == 0.0)
    assert np.all(got[np.isneginf(a)] == 0.0)
    np.testing.assert_allclose(got[ok].sum(axis=1), 1.0, rtol=1e-6)
    # shift invariance, and no overflow for large logits
    big = oracle.softmax_rows(a[ok] + np.float32(80.0))
    np.testing.assert_allclose(big, got[ok], rtol=2e-5, atol=1e-12)


# ---------------------------------------------------------------- global selection

def _read_global_fixture():
    lines = [l.strip() for l in open(os.path.join(GOLDEN, "mask_global_4x4.txt"))
             if l.strip() and not l.startswith("#")]
    a = lines.index("scores")
    first_case = next(n for n, l in enumerate(lines) if l.startswith("case"))
    sc = np.array([[float(x) for x in l.split()] for l in lines[a + 1:first_case]], dtype=np.float32)
    cases = []
    n = first_case
    while n < len(lines):
        _, gamma, _, K = lines[n].split()
        nr = sc.shape[0]
        assert lines[n + 1] == "lists" and lines[n + 2 + nr] == "forced"
        lists = [[int(x) for x in l.split()] for l in lines[n + 2:n + 2 + nr]]
        forced = [[int(x) for x in l.split()] for l in lines[n + 3 + nr:n + 3 + 2 * nr]]
        cases.append((float(gamma), int(K), lists, forced))
        n += 3 + 2 * nr
    return sc, cases


def test_global_mask_golden_hand_example():
    sc, cases = _read_global_fixture()
    assert len(cases) == 2
    for gamma, K, lists, forced in cases:
        for flag, want in ((False, lists), (True, forced)):
            idx, cnt, k = oracle.build_mask_global(sc, gamma, forced=flag)
            assert k == K
            for i, w in enumerate(want):
                assert list(idx[i, :cnt[i]]) == w
                assert np.all(idx[i, cnt[i]:] == -1)


def _quant(s):
    """Independent integer model of the 24-bit score: exact rationals, round half to even."""
    s = float(s)
    if not (s > 0.0):
        return 0
    s = min(s, 1.0)
    x = Fraction(s) * Q24
    fl = x.numerator // x.denominator
    rem = x - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    return fl


def _selected_set(idx, cnt):
    return {(i, int(j)) for i in range(len(cnt)) for j in idx[i, :cnt[i]]}


def _check_global_invariants(sc, gamma, idx, cnt, K):
    n = sc.shape[0]
    u = {(i, j): _quant(sc[i, j]) for i in range(n) for j in range(i + 1)}
    tot = sum(u.values())
    gq = _quant(np.float32(gamma))
    sel = _selected_set(idx, cnt)
    assert len(sel) == K == int(cnt.sum())
    for i in range(n):
        row = list(idx[i, :cnt[i]])
        assert row == sorted(set(row)) and all(0 <= j <= i for j in row)
    if tot == 0:
        assert K == 0
        return
    got = sum(u[e] for e in sel)
    assert got * Q24 >= gq * tot                                   # reaches gamma
    ranked = sorted(u.values(), reverse=True)
    assert sum(ranked[:K - 1]) * Q24 < gq * tot                    # no smaller set can
    assert got == sum(ranked[:K])                                  # it is a top-K set
    vmin = min(u[e] for e in sel)
    ties = sorted(e for e in u if u[e] == vmin)                    # row-major = flat order
    chosen = [e for e in ties if e in sel]
    assert chosen == ties[:len(chosen)]                            # lowest flat indices among equals
    assert all(e in sel for e in u if u[e] > vmin)


def test_global_mask_invariants_random_maps():
    rng = np.random.default_rng(5)
    for n in (1, 2, 7, 33):
        raw = np.tril(rng.random((n, n)) ** 5)
        sc = (raw / raw.sum(axis=1, keepdims=True)).astype(np.float32)
        sc[rng.random((n, n)) < 0.1] = 0.0
        for gamma in (0.3, 0.9, 0.95, 1.0):
            idx, cnt, K = oracle.build_mask_global(sc, gamma, forced=False)
            _check_global_invariants(sc, gamma, idx, cnt, K)
    # few distinct values: the tie rule decides most of the boundary
    sc = np.tril(rng.integers(0, 4, size=(12, 12)) / 8.0).astype(np.float32)
    for gamma in (0.25, 0.5, 0.77):
        idx, cnt, K = oracle.build_mask_global(sc, gamma, forced=False)
        _check_global_invariants(sc, gamma, idx, cnt, K)


def test_global_mask_minimal_by_exhaustive_subsets():
    rng = np.random.default_rng(6)
    n = 4
    cells = [(i, j) for i in range(n) for j in range(i + 1)]       # 10 cells, 1024 subsets
    for trial in range(6):
        sc = np.tril(rng.integers(0, 6, size=(n, n)) / 16.0).astype(np.float32)
        gamma = [0.4, 0.6, 0.75, 0.9, 0.95, 1.0][trial]
        u = {c: _quant(sc[c]) for c in cells}
        tot = sum(u.values())
        if tot == 0:
            continue
        gq = _quant(np.float32(gamma))
        best = None
        for r in range(1, len(cells) + 1):
            ok = [s for s in itertools.combinations(cells, r) if sum(u[c] for c in s) * Q24 >= gq * tot]
            if ok:
                best = r
                break
        idx, cnt, K = oracle.build_mask_global(sc, gamma, forced=False)
        assert K == best
        assert tuple(sorted(_selected_set(idx, cnt))) in {tuple(sorted(s)) for s in ok}


def test_global_mask_equal_scores_closed_form():
    """All causal entries equal: K = ceil(gamma_q * n / 2^24), the first K cells in flat order."""
    n = 9
    cells = [(i, j) for i in range(n) for j in range(i + 1)]
    sc = np.tril(np.full((n, n), 0.125, dtype=np.float32))
    for gamma in (0.1, 0.5, 0.95, 1.0):
        gq = _quant(np.float32(gamma))
        want_k = -(-gq * len(cells) // Q24)
        idx, cnt, K = oracle.build_mask_global(sc, gamma, forced=False)
        assert K == want_k
        assert sorted(_selected_set(idx, cnt)) == cells[:want_k]


def test_global_mask_uniform_rows_closed_form():
    """Rows uniform at 1/(i+1) (what Q = 0 gives), power-of-two rows only so values are exact:
    rows are consumed whole in order of increasing length."""
    n = 8
    sc = np.zeros((n, n), dtype=np.float32)
    for i in (0, 1, 3, 7):
        sc[i, :i + 1] = 1.0 / (i + 1)
    # total 4; gamma = 0.5 needs 2.0 = row 0 and row 1 exactly; gamma = 0.625 needs 2.5 = + two cells of row 3
    idx, cnt, K = oracle.build_mask_global(sc, 0.5, forced=False)
    assert K == 3 and list(cnt) == [1, 2, 0, 0, 0, 0, 0, 0]
    idx, cnt, K = oracle.build_mask_global(sc, 0.625, forced=False)
    assert K == 5 and list(cnt) == [1, 2, 0, 2, 0, 0, 0, 0] and list(idx[3, :2]) == [0, 1]


def test_global_mask_rows_are_row_prefixes_and_single_row_reduces_to_per_row():
    rng = np.random.default_rng(8)
    n = 24
    raw = np.tril(rng.random((n, n)) ** 4)
    sc = (raw / raw.sum(axis=1, keepdims=True)).astype(np.float32)
    idx, cnt, K = oracle.build_mask_global(sc, 0.9, forced=False)
    for i in range(n):
        order = sorted(range(i + 1), key=lambda j: (-_quant(sc[i, j]), j))
        assert set(idx[i, :cnt[i]]) == set(order[:cnt[i]])        # each row keeps a top-k of its own
    # a map with one non-empty row: the global rule and the per-row rule coincide on it
    one = np.zeros_like(sc)
    one[n - 1] = sc[n - 1]
    for gamma in (0.5, 0.9):
        gi, gc, gk = oracle.build_mask_global(one, gamma, forced=False)
        ri, rc, rk = oracle.build_mask_rows(one[n - 1:n], gamma, row_ids=[n - 1])
        assert gk == rk[0] and int(gc[:n - 1].sum()) == 0
        fi, fc, _ = oracle.build_mask_global(one, gamma, forced=True)
        assert list(fi[n - 1, :fc[n - 1]]) == list(ri[0, :rc[0]])  # per-row output carries the forced blocks


def test_global_mask_forced_monotone_and_bad_values():
    rng = np.random.default_rng(9)
    n = 16
    raw = np.tril(rng.random((n, n)) ** 3)
    sc = (raw / raw.sum(axis=1, keepdims=True)).astype(np.float32)
    prev = set()
    for gamma in (0.2, 0.5, 0.8, 0.95, 1.0):
        idx, cnt, K = oracle.build_mask_global(sc, gamma, forced=False)
        cur = _selected_set(idx, cnt)
        assert prev <= cur                                        # monotone in gamma
        prev = cur
        fi, fc, fk = oracle.build_mask_global(sc, gamma, forced=True)
        assert fk == K
        assert _selected_set(fi, fc) == cur | {(i, 0) for i in range(n)} | {(i, i) for i in range(n)}
    nz = {(i, j) for i in range(n) for j in range(i + 1) if _quant(sc[i, j]) > 0}
    assert prev == nz                                             # gamma = 1 keeps every non-zero cell
    # entries beyond the diagonal, NaN, negatives and values above 1 never break the rules
    bad = sc.copy()
    bad[np.triu_indices(n, 1)] = 0.9
    bad[3, 1] = np.nan
    bad[5, 2] = -1.0
    bad[6, 6] = 7.0
    ref = np.tril(bad)
    ref[3, 1] = 0.0
    ref[5, 2] = 0.0
    ref[6, 6] = 1.0
    a = oracle.build_mask_global(bad, 0.9, forced=False)
    b = oracle.build_mask_global(ref.astype(np.float32), 0.9, forced=False)
    assert a[2] == b[2] and np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    z = oracle.build_mask_global(np.zeros((5, 5), dtype=np.float32), 0.9, forced=False)
    assert z[2] == 0 and int(z[1].sum()) == 0
    with pytest.raises(ValueError):
        oracle.build_mask_global(sc, 0.0)
    with pytest.raises(ValueError):
        oracle.build_mask_global(sc, 1.5)


def test_prefill_layer_paper_pattern_is_the_composition_of_its_stages():
    N, Hq, Hkv, d, B = 256, 4, 2, 16, 32
    qb, kb, vb = random_qkv(21, N, Hq, Hkv, d, 1.5)
    q, k, v = (bf16_bits_to_f32(a) for a in (qb, kb, vb))
    h2c, piv = [0, 0, 1, 1], [0, 2]
    out = oracle.prefill_layer(q, k, v, B, h2c, piv, 0.9, paper_pattern=True)
    for c, p in enumerate(piv):
        s = oracle.softmax_rows(oracle.mean_logit_rows(q[:, p], k[:, p // 2], B))
        assert np.array_equal(out["scores"][c], s)
        idx, cnt, _ = oracle.build_mask_global(s, 0.9, forced=True)
        assert np.array_equal(out["kb_idx"][c], idx) and np.array_equal(out["kb_cnt"][c], cnt)
        o_dense, _, _ = oracle.dense_rows(q[:, p], k[:, p // 2], v[:, p // 2], B, want_scores=False)
        assert np.array_equal(out["o"][:, p], o_dense)
        h = p + 1
        o_sparse = oracle.masked_rows(q[:, h], k[:, h // 2], v[:, h // 2], B, idx, cnt)
        assert np.array_equal(out["o"][:, h], o_sparse)
