"""Pins for the CPU oracle: each check ties an oracle function to something other
than itself -- brute force in fp64 numpy on materialised N x N matrices, library
routines (torch SDPA, scipy softmax), closed forms, invariants and a hand-worked
fixture -- chosen so that a dropped term, a wrong sign or index, or a transposed
operand fails at least one of them.  CPU only.
"""
import itertools
import os

import numpy as np
import pytest

import oracle
from synth import bf16_bits_to_f32, random_qkv, make_layer, CONFIGS

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _qkv(seed, N, d, scale=1.0):
    q, k, v = random_qkv(seed, N, 1, 1, d, scale)
    f = lambda a: bf16_bits_to_f32(a)[:, 0, :].astype(np.float64)
    return f(q), f(k), f(v)


def _brute_P(q, k, allowed=None):
    """Materialised causal softmax in fp64 (Sec. 5.1: softmax(QK^T/sqrt(d) - c(1-M)))."""
    N, d = q.shape
    x = (q @ k.T) / np.sqrt(d)
    keep = np.tril(np.ones((N, N), dtype=bool))
    if allowed is not None:
        keep &= allowed
    x = np.where(keep, x, -np.inf)
    mx = x.max(axis=1, keepdims=True)
    mx = np.where(np.isfinite(mx), mx, 0.0)
    e = np.exp(x - mx)
    den = e.sum(axis=1, keepdims=True)
    return np.divide(e, den, out=np.zeros_like(e), where=den > 0)


def _brute_scores(P, B):
    N = P.shape[0]
    n = N // B
    return P.reshape(n, B, n, B).sum(axis=(1, 3)) / B


# ------------------------------------------------------------------ dense (O1-O2)
@pytest.mark.parametrize("N,d,B", [(64, 16, 16), (192, 32, 32), (256, 64, 64)])
def test_dense_matches_bruteforce(N, d, B):
    q, k, v = _qkv(1, N, d)
    o, sc, lse = oracle.dense_rows(q, k, v, B)
    P = _brute_P(q, k)
    np.testing.assert_allclose(o, P @ v, atol=1e-6)
    np.testing.assert_allclose(sc, _brute_scores(P, B), atol=1e-6)
    x = np.where(np.tril(np.ones((N, N), bool)), (q @ k.T) / np.sqrt(d), -np.inf)
    from scipy.special import logsumexp
    np.testing.assert_allclose(lse, logsumexp(x, axis=1), atol=1e-5)


def test_dense_matches_torch_sdpa_and_scipy():
    import torch
    from scipy.special import softmax
    N, d, B = 128, 32, 32
    q, k, v = _qkv(2, N, d)
    o, _, _ = oracle.dense_rows(q, k, v, B)
    tq, tk, tv = (torch.tensor(a, dtype=torch.float32)[None, None] for a in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0, 0].numpy()
    np.testing.assert_allclose(o, ref, atol=2e-5)
    x = np.where(np.tril(np.ones((N, N), bool)), (q @ k.T) / np.sqrt(d), -np.inf)
    np.testing.assert_allclose(o, softmax(x, axis=1) @ v, atol=1e-6)


def test_dense_row_subset_equals_full():
    N, d, B = 256, 32, 32
    q, k, v = _qkv(3, N, d)
    o, sc, lse = oracle.dense_rows(q, k, v, B)
    rows = [5, 0, 7]
    o2, sc2, lse2 = oracle.dense_rows(q, k, v, B, rows)
    for r, i in enumerate(rows):
        np.testing.assert_array_equal(o2[r * B:(r + 1) * B], o[i * B:(i + 1) * B])
        np.testing.assert_array_equal(sc2[r], sc[i])
        np.testing.assert_array_equal(lse2[r * B:(r + 1) * B], lse[i * B:(i + 1) * B])


def test_dense_zero_query_closed_form():
    """Q = 0: P[t][s] = 1/(t+1); O[t] is the prefix mean of V; the block scores are
    differences of harmonic numbers off the diagonal."""
    N, d, B = 192, 16, 32
    _, k, v = _qkv(4, N, d)
    q = np.zeros((N, d))
    o, sc, lse = oracle.dense_rows(q, k, v, B)
    prefix_mean = np.cumsum(v, axis=0) / np.arange(1, N + 1)[:, None]
    np.testing.assert_allclose(o, prefix_mean, atol=1e-6)
    np.testing.assert_allclose(lse, np.log(np.arange(1, N + 1)), atol=1e-6)
    H = np.concatenate([[0.0], np.cumsum(1.0 / np.arange(1, N + 1))])
    n = N // B
    for i in range(n):
        for j in range(n):
            if j < i:
                want = H[(i + 1) * B] - H[i * B]
            elif j == i:
                want = sum((r + 1) / (i * B + r + 1) for r in range(B)) / B
            else:
                want = 0.0
            assert abs(sc[i, j] - want) < 1e-6, (i, j)


def test_dense_invariants():
    N, d, B = 128, 32, 32
    q, k, v = _qkv(5, N, d)
    o, sc, _ = oracle.dense_rows(q, k, v, B)
    # rows of P sum to 1  <=>  V = 1 gives O = 1 ; rows of S sum to 1 ; S is lower triangular
    o1, _, _ = oracle.dense_rows(q, k, np.ones_like(v), B)
    np.testing.assert_allclose(o1, 1.0, atol=1e-6)
    np.testing.assert_allclose(sc.sum(axis=1), 1.0, atol=1e-5)
    assert np.all(np.triu(sc, 1) == 0)
    # adding the same vector w to every key shifts each row's logits by a constant
    w = np.linspace(-1, 1, d)
    o2, sc2, _ = oracle.dense_rows(q, k + w[None, :], v, B)
    np.testing.assert_allclose(o2, o, atol=1e-5)
    np.testing.assert_allclose(sc2, sc, atol=1e-6)
    # permuting keys (with their values) inside an off-diagonal block changes nothing for later blocks
    perm = np.arange(N)
    perm[B:2 * B] = perm[B:2 * B][::-1]
    o3, sc3, _ = oracle.dense_rows(q, k[perm], v[perm], B, rows=[2, 3])
    np.testing.assert_allclose(o3, o[2 * B:], atol=1e-6)
    np.testing.assert_allclose(sc3, sc[2:], atol=1e-6)
    # transposition guard: swapping the roles of Q and K must change the answer
    o4, _, _ = oracle.dense_rows(k, q, v, B)
    assert np.abs(o4 - o).max() > 1e-2


def test_scores_one_hot_for_huge_key():
    N, d, B = 128, 16, 32
    q, k, v = _qkv(6, N, d)
    q[:, 0] = 8.0
    k[:, 0] = 0.0
    s0 = 40
    k[s0, 0] = 50.0   # logit 8*50/4 = 100 above everything else
    _, sc, _ = oracle.dense_rows(q, k, v, B)
    for i in range(2, N // B):
        assert sc[i, s0 // B] > 1 - 1e-6
    # in the block that contains the key only queries t >= s0 see it
    frac = (2 * B - s0) / B
    assert abs(sc[1, 1] - frac) < 0.2 and sc[1, 1] > frac - 1e-6


def test_scale_argument():
    N, d, B = 64, 16, 16
    q, k, v = _qkv(7, N, d)
    o_a, _, _ = oracle.dense_rows(q, k, v, B, scale=0.5)
    o_b, _, _ = oracle.dense_rows(q * 2.0, k, v, B, scale=0.25)
    np.testing.assert_allclose(o_a, o_b, atol=1e-6)


# ------------------------------------------------------------------ mask (O4)
def _check_mask_invariants(scores_row, i, gamma, idx_row, cnt, kstar):
    u = np.rint(np.clip(np.nan_to_num(scores_row[: i + 1].astype(np.float32), nan=0.0), 0, 1)
                * np.float32(2 ** 24)).astype(np.int64)
    gq = int(np.rint(np.float32(gamma) * np.float32(2 ** 24)))
    tot = int(u.sum())
    R = list(idx_row[:cnt])
    assert all(idx_row[cnt:] == -1)
    assert R == sorted(set(R)) and all(0 <= j <= i for j in R)
    assert 0 in R and i in R
    order = sorted(range(i + 1), key=lambda j: (-u[j], j))
    T = order[:kstar]
    assert set(R) == set(T) | {0, i}
    if tot == 0:
        assert kstar == 0
        return
    sT = int(u[T].sum())
    assert sT * 2 ** 24 >= gq * tot            # reaches the threshold
    assert (sT - int(u[T[-1]])) * 2 ** 24 < gq * tot   # dropping the last element breaks it
    return u, gq, tot, T


def test_mask_golden_hand_example():
    lines = [l.strip() for l in open(os.path.join(GOLDEN, "mask_6x6.txt")) if l.strip() and not l.startswith("#")]
    gamma = float(lines[0].split()[1])
    a = lines.index("scores")
    b = next(n for n, l in enumerate(lines) if l.startswith("kstar"))
    sc = np.array([[float(x) for x in l.split()] for l in lines[a + 1:b]], dtype=np.float32)
    kstar = [int(x) for x in lines[b].split()[1:]]
    lists = [[int(x) for x in l.split()] for l in lines[b + 2:]]
    idx, cnt, ks = oracle.build_mask_rows(sc, gamma)
    assert list(ks) == kstar
    for i, want in enumerate(lists):
        assert list(idx[i, :cnt[i]]) == want
        assert all(idx[i, cnt[i]:] == -1)


def test_mask_invariants_random_and_synthetic():
    rng = np.random.default_rng(0)
    n = 48
    raw = rng.random((n, n)) ** 6
    raw = np.tril(raw)
    sc = (raw / raw.sum(axis=1, keepdims=True)).astype(np.float32)
    for gamma in (0.5, 0.9, 0.95, 1.0):
        idx, cnt, ks = oracle.build_mask_rows(sc, gamma)
        for i in range(n):
            _check_mask_invariants(sc[i], i, gamma, idx[i], cnt[i], ks[i])


def test_mask_minimal_by_exhaustive_subsets():
    """No subset smaller than k* reaches the threshold (nkb <= 12, all subsets)."""
    rng = np.random.default_rng(1)
    n = 12
    raw = np.tril(rng.random((n, n)) ** 3)
    raw[7, 2] = raw[7, 5]           # plant a tie
    sc = (raw / raw.sum(axis=1, keepdims=True)).astype(np.float32)
    gamma = 0.8
    idx, cnt, ks = oracle.build_mask_rows(sc, gamma)
    gq = int(np.rint(np.float32(gamma) * np.float32(2 ** 24)))
    for i in range(n):
        u = np.rint(sc[i, : i + 1] * np.float32(2 ** 24)).astype(np.int64)
        tot = int(u.sum())
        best = None
        for size in range(1, i + 2):
            if any(int(u[list(c)].sum()) * 2 ** 24 >= gq * tot for c in itertools.combinations(range(i + 1), size)):
                best = size
                break
        assert ks[i] == best, i


def test_mask_equal_scores_closed_form():
    n = 40
    sc = np.zeros((n, n), dtype=np.float32)
    for i in range(n):
        sc[i, : i + 1] = 1.0 / 64.0     # exactly representable, equal
    gamma = 0.7
    idx, cnt, ks = oracle.build_mask_rows(sc, gamma)
    gq = int(np.rint(np.float32(gamma) * np.float32(2 ** 24)))
    for i in range(n):
        want = -(-gq * (i + 1) // 2 ** 24)          # ceil(gq (i+1) / 2^24)
        assert ks[i] == want
        T = set(range(want))                         # ties -> lowest indices
        assert set(idx[i, :cnt[i]]) == T | {0, i}


def test_mask_monotone_in_gamma_and_extremes():
    L = make_layer(CONFIGS["tiny"])
    q, k, v = (bf16_bits_to_f32(L[x]) for x in "qkv")
    _, sc, _ = oracle.dense_rows(q[:, 0], k[:, 0], v[:, 0], 64)
    prev = None
    n = sc.shape[0]
    for gamma in (0.3, 0.6, 0.9, 0.99, 1.0):
        idx, cnt, ks = oracle.build_mask_rows(sc, gamma)
        cur = []
        for i in range(n):
            u = np.rint(sc[i, : i + 1] * np.float32(2 ** 24)).astype(np.int64)
            order = sorted(range(i + 1), key=lambda j: (-u[j], j))
            cur.append(order[: ks[i]])
            if gamma == 1.0:
                assert set(order[: ks[i]]) == {j for j in range(i + 1) if u[j] > 0}
        if prev is not None:
            for a, b in zip(prev, cur):
                assert b[: len(a)] == a          # T(g1) is a prefix of T(g2)
        prev = cur


def test_mask_one_hot_zero_nan_rows():
    n = 8
    sc = np.zeros((n, n), dtype=np.float32)
    sc[5, 3] = 1.0
    sc[6, :7] = np.nan
    sc[7, 2] = 2.5       # clamps to 1
    sc[7, 4] = -3.0      # clamps to 0
    idx, cnt, ks = oracle.build_mask_rows(sc, 0.9)
    assert list(idx[5, :cnt[5]]) == [0, 3, 5] and ks[5] == 1
    assert list(idx[4, :cnt[4]]) == [0, 4] and ks[4] == 0       # all-zero row: only forced blocks
    assert list(idx[6, :cnt[6]]) == [0, 6] and ks[6] == 0       # NaN -> 0
    assert list(idx[7, :cnt[7]]) == [0, 2, 7] and ks[7] == 1
    assert list(idx[0, :cnt[0]]) == [0]
    with pytest.raises(ValueError):
        oracle.build_mask_rows(sc, 0.0)
    with pytest.raises(ValueError):
        oracle.build_mask_rows(sc, 1.5)


# ------------------------------------------------------------------ masked (O5)
def _lists_to_allowed(idx, cnt, N, B):
    n = N // B
    blk = np.zeros((n, n), dtype=bool)
    for i in range(n):
        blk[i, idx[i, :cnt[i]]] = True
    return np.kron(blk, np.ones((B, B), dtype=bool))


def test_masked_all_ones_equals_dense():
    N, d, B = 192, 32, 32
    q, k, v = _qkv(8, N, d)
    n = N // B
    idx = np.full((n, n), -1, np.int32)
    cnt = np.zeros(n, np.int32)
    for i in range(n):
        idx[i, : i + 1] = np.arange(i + 1)
        cnt[i] = i + 1
    o_d, _, _ = oracle.dense_rows(q, k, v, B)
    o_m = oracle.masked_rows(q, k, v, B, idx, cnt)
    np.testing.assert_allclose(o_m, o_d, atol=1e-6)


@pytest.mark.parametrize("pattern", ["random", "sink_local"])
def test_masked_matches_bruteforce(pattern):
    N, d, B = 256, 32, 32
    q, k, v = _qkv(9, N, d)
    n = N // B
    rng = np.random.default_rng(2)
    idx = np.full((n, n), -1, np.int32)
    cnt = np.zeros(n, np.int32)
    for i in range(n):
        if pattern == "random":
            sel = sorted(set(rng.choice(i + 1, size=max(1, (i + 1) // 2), replace=False)) | {0, i})
        else:
            sel = sorted({0, i})
        idx[i, : len(sel)] = sel
        cnt[i] = len(sel)
    o = oracle.masked_rows(q, k, v, B, idx, cnt)
    P = _brute_P(q, k, _lists_to_allowed(idx, cnt, N, B))
    np.testing.assert_allclose(P.sum(axis=1), 1.0, atol=1e-12)
    np.testing.assert_allclose(o, P @ v, atol=1e-6)
    o1 = oracle.masked_rows(q, k, np.ones_like(v), B, idx, cnt)
    np.testing.assert_allclose(o1, 1.0, atol=1e-6)
    # row subset, with the lists given per listed row
    rows = [6, 1]
    o2 = oracle.masked_rows(q, k, v, B, idx[rows], cnt[rows], rows)
    for r, i in enumerate(rows):
        np.testing.assert_array_equal(o2[r * B:(r + 1) * B], o[i * B:(i + 1) * B])


def test_masked_block_beyond_diagonal_is_ignored_and_empty_row_is_zero():
    N, d, B = 64, 16, 16
    q, k, v = _qkv(10, N, d)
    n = N // B
    idx = np.full((n, n), -1, np.int32)
    cnt = np.zeros(n, np.int32)
    idx[1, :3] = [0, 1, 3]
    cnt[1] = 3
    idx[2, :1] = [3]          # only a future block: nothing admissible
    cnt[2] = 1
    o = oracle.masked_rows(q, k, v, B, idx[[1, 2]], cnt[[1, 2]], [1, 2])
    allowed = np.zeros((N, N), bool)
    allowed[B:2 * B, : 2 * B] = True
    P = _brute_P(q, k, allowed)
    np.testing.assert_allclose(o[:B], (P @ v)[B:2 * B], atol=1e-6)
    assert np.all(o[B:] == 0)


# ------------------------------------------------------------------ fused (O6)
def test_prefill_layer_is_the_composition_of_its_stages():
    L = make_layer(CONFIGS["tiny"], seq=512)
    q, k, v = (bf16_bits_to_f32(L[x]) for x in "qkv")
    B, gamma = 64, 0.9
    h2c, piv = L["head_to_cluster"], L["pivot_heads"]
    out = oracle.prefill_layer(q, k, v, B, h2c, piv, gamma)
    n = 512 // B
    for c, p in enumerate(piv):
        o_p, sc, _ = oracle.dense_rows(q[:, p], k[:, p], v[:, p], B)
        np.testing.assert_array_equal(out["o"][:, p], o_p)
        np.testing.assert_array_equal(out["scores"][c], sc)
        idx, cnt, _ = oracle.build_mask_rows(sc, gamma)
        np.testing.assert_array_equal(out["kb_idx"][c], idx)
        np.testing.assert_array_equal(out["kb_cnt"][c], cnt)
        for h in np.nonzero(h2c == c)[0]:
            if h == p:
                continue
            np.testing.assert_array_equal(out["o"][:, h], oracle.masked_rows(q[:, h], k[:, h], v[:, h], B, idx, cnt))
    # the shared pattern covers most of the *other* head's own attention mass (pattern similarity
    # inside a cluster is what the generator is built to have, Sec. 4 observation 1)
    _, sc_other, _ = oracle.dense_rows(q[:, 1], k[:, 1], v[:, 1], B)
    idx0, cnt0 = out["kb_idx"][0], out["kb_cnt"][0]
    cover = np.mean([sc_other[i, idx0[i, :cnt0[i]]].sum() for i in range(n)])
    assert cover > 0.85
    # a head outside every cluster runs dense
    h2c2 = h2c.copy()
    h2c2[1] = -1
    out2 = oracle.prefill_layer(q, k, v, B, h2c2, piv, gamma)
    o1, _, _ = oracle.dense_rows(q[:, 1], k[:, 1], v[:, 1], B)
    np.testing.assert_array_equal(out2["o"][:, 1], o1)
