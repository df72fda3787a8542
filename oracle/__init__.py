"""CPU oracle for the SharePrefill prefill hot path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes access to ``sp_oracle.c`` (plain C, fp64 arithmetic on fp32 inputs)
plus the per-layer composition of its stages.  Only the tests, the smoke check
and the benchmark's ``cpu_baseline`` leg may import this package; it shares no
code with the HIP path and never imports it.

Stages (one attention head at a time, arrays are float32 ``[N][d]``):

* ``dense_rows``      causal softmax attention + block-mass score rows
                      (Sec. 5.1 A(Q,K,V); Alg. 1 line 8 score map, mass reading)
* ``build_mask_rows`` Alg. 2 per query-block row in exact fixed point, plus the
                      forced sink and diagonal blocks
* ``masked_rows``     Sec. 5.1 A(Q,K,V,M) over the listed key blocks
* ``mean_logit_rows`` block-wise average of the scaled QK logits (Sec. 5.2, "Sparse
                      Attention Computation"), ``softmax_rows`` Alg. 2's first step,
                      ``build_mask_global`` Alg. 2 over the flattened map: the pattern
                      construction as the paper prints it
* ``js_distance``, ``last_row_estimate``, ``determine_pattern``
                      Alg. 3 (Determine Sparse Pattern): the last query block's
                      block-averaged attention estimate, its Jensen-Shannon distances to
                      the uniform distribution and to the pivot's representative, the gate
* ``vertical_slash_sums``, ``select_cumulative``, ``vs_block_lists``, ``vertical_slash_pattern``
                      Alg. 5 (Search Vertical Slash Pattern): vertical / slash sums of the last
                      query block's attention, the two cumulative selections, the block lists
* ``prefill_layers_dict`` Alg. 1 head by head, layer by layer, with the dynamic pivotal
                      pattern dictionary (Sec. 5.2): first qualifying head of a cluster runs
                      dense and installs the pattern, later heads, in this or later layers, share it
* ``prefill_layer``   Alg. 1 / Alg. 4 for one layer with given pivots: pivots run
                      dense, their score map becomes the cluster's pattern, all
                      other heads of the cluster run masked attention with it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sp_oracle.c")
_LIB = os.path.join(_HERE, "libsp_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile sp_oracle.c with gcc (OpenMP).  Returns the library path."""
    if force or (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        fp = ctypes.POINTER(ctypes.c_float)
        ip = ctypes.POINTER(ctypes.c_int32)
        L.spo_num_threads.restype = ctypes.c_int
        L.spo_dense_rows.restype = ctypes.c_int
        L.spo_dense_rows.argtypes = [fp, fp, fp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double,
                                     ip, ctypes.c_int, fp, fp, fp]
        L.spo_build_mask_rows.restype = ctypes.c_int
        L.spo_build_mask_rows.argtypes = [fp, ip, ctypes.c_int, ctypes.c_int, ctypes.c_float, ip, ip, ip]
        L.spo_masked_rows.restype = ctypes.c_int
        L.spo_masked_rows.argtypes = [fp, fp, fp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double,
                                      ip, ctypes.c_int, ip, ip, fp]
        L.spo_mean_logit_rows.restype = ctypes.c_int
        L.spo_mean_logit_rows.argtypes = [fp, fp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double,
                                          ip, ctypes.c_int, fp]
        L.spo_softmax_rows.restype = ctypes.c_int
        L.spo_softmax_rows.argtypes = [fp, ctypes.c_int, ctypes.c_int, fp]
        L.spo_build_mask_global.restype = ctypes.c_int
        L.spo_build_mask_global.argtypes = [fp, ctypes.c_int, ctypes.c_float, ctypes.c_int, ip, ip,
                                            ctypes.POINTER(ctypes.c_int64)]
        up = ctypes.POINTER(ctypes.c_ubyte)
        L.spo_vertical_slash_sums.restype = ctypes.c_int
        L.spo_vertical_slash_sums.argtypes = [fp, fp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double, fp, fp]
        L.spo_select_cumulative.restype = ctypes.c_int
        L.spo_select_cumulative.argtypes = [fp, ctypes.c_int64, ctypes.c_float, up, ctypes.POINTER(ctypes.c_int64)]
        L.spo_vs_block_lists.restype = ctypes.c_int
        L.spo_vs_block_lists.argtypes = [up, up, ctypes.c_int, ctypes.c_int, ctypes.c_int, ip, ip]
        L.spo_vs_token_rows.restype = ctypes.c_int
        L.spo_vs_token_rows.argtypes = [fp, fp, fp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double,
                                        ctypes.POINTER(ctypes.c_int), ctypes.c_int, up, up, ctypes.c_int, fp]
        L.spo_js_distance.restype = ctypes.c_int
        L.spo_js_distance.argtypes = [fp, fp, ctypes.c_int, ctypes.POINTER(ctypes.c_double)]
        _lib = L
    return _lib


def num_threads() -> int:
    return int(_load().spo_num_threads())


def _f(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _i(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _rows(rows, nqb):
    if rows is None:
        rows = np.arange(nqb, dtype=np.int32)
    return np.ascontiguousarray(rows, dtype=np.int32)


def dense_rows(q, k, v, block: int, rows: Optional[Sequence[int]] = None, scale: Optional[float] = None,
               want_scores: bool = True):
    """Dense causal attention of one head on the listed query-block rows.

    Returns (o [nrows*B][d], scores [nrows][nkb] or None, lse [nrows*B])."""
    q, qp = _f(q)
    k, kp = _f(k)
    v, vp = _f(v)
    N, d = q.shape
    assert k.shape == (N, d) and v.shape == (N, d)
    nkb = N // block
    rows = _rows(rows, nkb)
    nr = len(rows)
    scale = (1.0 / np.sqrt(d)) if scale is None else float(scale)
    o = np.empty((nr * block, d), dtype=np.float32)
    sc = np.empty((nr, nkb), dtype=np.float32) if want_scores else None
    lse = np.empty((nr * block,), dtype=np.float32)
    rc = _load().spo_dense_rows(qp, kp, vp, N, d, block, scale,
                                rows.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), nr,
                                o.ctypes.data_as(ctypes.POINTER(ctypes.c_float)),
                                sc.ctypes.data_as(ctypes.POINTER(ctypes.c_float)) if want_scores else None,
                                lse.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
    if rc:
        raise ValueError(f"spo_dense_rows failed ({rc})")
    return o, sc, lse


def build_mask_rows(scores, gamma: float, row_ids: Optional[Sequence[int]] = None):
    """Alg. 2 per row.  scores [nrows][nkb]; row r describes query block row_ids[r].

    Returns (kb_idx int32 [nrows][nkb] ascending, -1 tail; kb_cnt int32 [nrows];
    k_star int32 [nrows] = size of the thresholded set before forced blocks)."""
    scores, sp = _f(scores)
    nr, nkb = scores.shape
    if row_ids is None:
        assert nr == nkb
    row_ids = _rows(row_ids, nkb)
    assert len(row_ids) == nr
    idx = np.empty((nr, nkb), dtype=np.int32)
    cnt = np.empty((nr,), dtype=np.int32)
    ks = np.empty((nr,), dtype=np.int32)
    ip = ctypes.POINTER(ctypes.c_int32)
    rc = _load().spo_build_mask_rows(sp, row_ids.ctypes.data_as(ip), nr, nkb, ctypes.c_float(np.float32(gamma)),
                                     idx.ctypes.data_as(ip), cnt.ctypes.data_as(ip), ks.ctypes.data_as(ip))
    if rc:
        raise ValueError(f"spo_build_mask_rows failed ({rc})")
    return idx, cnt, ks


def masked_rows(q, k, v, block: int, kb_idx, kb_cnt, rows: Optional[Sequence[int]] = None,
                scale: Optional[float] = None):
    """Block-sparse causal attention of one head; kb_idx/kb_cnt are per listed row."""
    q, qp = _f(q)
    k, kp = _f(k)
    v, vp = _f(v)
    N, d = q.shape
    nkb = N // block
    rows = _rows(rows, nkb)
    nr = len(rows)
    kb_idx, xp = _i(kb_idx)
    kb_cnt, cp = _i(kb_cnt)
    assert kb_idx.shape == (nr, nkb) and kb_cnt.shape == (nr,)
    scale = (1.0 / np.sqrt(d)) if scale is None else float(scale)
    o = np.empty((nr * block, d), dtype=np.float32)
    rc = _load().spo_masked_rows(qp, kp, vp, N, d, block, scale,
                                 rows.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), nr, xp, cp,
                                 o.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
    if rc:
        raise ValueError(f"spo_masked_rows failed ({rc})")
    return o


def mean_logit_rows(q, k, block: int, rows: Optional[Sequence[int]] = None, scale: Optional[float] = None):
    """Block-wise average of the scaled causal logits of one head, [nrows][nkb], -inf beyond the diagonal."""
    q, qp = _f(q)
    k, kp = _f(k)
    N, d = q.shape
    nkb = N // block
    rows = _rows(rows, nkb)
    scale = (1.0 / np.sqrt(d)) if scale is None else float(scale)
    out = np.empty((len(rows), nkb), dtype=np.float32)
    rc = _load().spo_mean_logit_rows(qp, kp, N, d, block, scale,
                                     rows.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), len(rows),
                                     out.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
    if rc:
        raise ValueError(f"spo_mean_logit_rows failed ({rc})")
    return out


def softmax_rows(a):
    """Row softmax (fp64 inside); -inf entries become exactly 0."""
    a, ap = _f(a)
    out = np.empty_like(a)
    rc = _load().spo_softmax_rows(ap, a.shape[0], a.shape[1], out.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
    if rc:
        raise ValueError(f"spo_softmax_rows failed ({rc})")
    return out


def build_mask_global(scores, gamma: float, forced: bool = True):
    """Alg. 2 over the whole (square, causal) score map.  Returns (kb_idx, kb_cnt, K)."""
    scores, sp = _f(scores)
    nkb = scores.shape[0]
    assert scores.shape == (nkb, nkb)
    idx = np.empty((nkb, nkb), dtype=np.int32)
    cnt = np.empty((nkb,), dtype=np.int32)
    K = ctypes.c_int64(0)
    ip = ctypes.POINTER(ctypes.c_int32)
    rc = _load().spo_build_mask_global(sp, nkb, ctypes.c_float(np.float32(gamma)), int(bool(forced)),
                                       idx.ctypes.data_as(ip), cnt.ctypes.data_as(ip), ctypes.byref(K))
    if rc:
        raise ValueError(f"spo_build_mask_global failed ({rc})")
    return idx, cnt, int(K.value)


def js_distance(p, q) -> float:
    """sqrt of the Jensen-Shannon divergence (natural log) of two non-negative vectors."""
    p, pp = _f(p)
    q, qp = _f(q)
    assert p.shape == q.shape and p.ndim == 1
    out = ctypes.c_double(0.0)
    rc = _load().spo_js_distance(pp, qp, p.shape[0], ctypes.byref(out))
    if rc:
        raise ValueError(f"spo_js_distance failed ({rc})")
    return float(out.value)


def last_row_estimate(q, k, block: int, scale: Optional[float] = None):
    """a_hat of Alg. 3: softmax over key blocks of the pooled scaled logits of the last query block."""
    nkb = q.shape[0] // block
    return softmax_rows(mean_logit_rows(q, k, block, rows=[nkb - 1], scale=scale))[0]


def determine_pattern(a_hat, a_tilde, delta: float, tau: float):
    """Alg. 3's gate.  a_tilde None: no pivotal representative exists yet, only the sparsity test applies.
    Returns (shared: bool, d_sparse, d_sim)."""
    n = len(a_hat)
    d_sparse = js_distance(a_hat, np.full(n, 1.0 / n, dtype=np.float32))
    d_sim = 0.0 if a_tilde is None else js_distance(a_hat, a_tilde)
    return (d_sparse < delta) and (d_sim < tau), d_sparse, d_sim


def vertical_slash_sums(q, k, n_hat: int, scale: Optional[float] = None):
    """Alg. 5: normalised vertical sums a_v [N] and slash sums a_s [N] of the causal attention of the last
    n_hat queries."""
    q, qp = _f(q)
    k, kp = _f(k)
    N, d = q.shape
    scale = (1.0 / np.sqrt(d)) if scale is None else float(scale)
    a_v = np.empty(N, dtype=np.float32)
    a_s = np.empty(N, dtype=np.float32)
    fp = ctypes.POINTER(ctypes.c_float)
    rc = _load().spo_vertical_slash_sums(qp, kp, N, d, n_hat, scale, a_v.ctypes.data_as(fp), a_s.ctypes.data_as(fp))
    if rc:
        raise ValueError(f"spo_vertical_slash_sums failed ({rc})")
    return a_v, a_s


def select_cumulative(v, gamma: float):
    """Shortest descending prefix (ties: lower index) whose sum reaches gamma of the total: (keep uint8 [n], K)."""
    v, vp = _f(v)
    keep = np.zeros(v.shape[0], dtype=np.uint8)
    K = ctypes.c_int64(0)
    rc = _load().spo_select_cumulative(vp, v.shape[0], ctypes.c_float(np.float32(gamma)),
                                       keep.ctypes.data_as(ctypes.POINTER(ctypes.c_ubyte)), ctypes.byref(K))
    if rc:
        raise ValueError(f"spo_select_cumulative failed ({rc})")
    return keep, int(K.value)


def vs_block_lists(keep_v, keep_s, block: int, forced: bool = True):
    """Block lists (kb_idx [nkb][nkb], kb_cnt [nkb]) of the vertical-slash pattern with those kept keys / offsets."""
    keep_v = np.ascontiguousarray(keep_v, dtype=np.uint8)
    keep_s = np.ascontiguousarray(keep_s, dtype=np.uint8)
    N = keep_v.shape[0]
    assert keep_s.shape == (N,)
    nkb = N // block
    idx = np.empty((nkb, nkb), dtype=np.int32)
    cnt = np.empty((nkb,), dtype=np.int32)
    up, ip = ctypes.POINTER(ctypes.c_ubyte), ctypes.POINTER(ctypes.c_int32)
    rc = _load().spo_vs_block_lists(keep_v.ctypes.data_as(up), keep_s.ctypes.data_as(up), N, block,
                                    int(bool(forced)), idx.ctypes.data_as(ip), cnt.ctypes.data_as(ip))
    if rc:
        raise ValueError(f"spo_vs_block_lists failed ({rc})")
    return idx, cnt


def vs_token_rows(q, k, v, block: int, keep_v, keep_s, forced: bool = True, rows: Optional[Sequence[int]] = None,
                  scale: Optional[float] = None):
    """Attention over the token-level vertical-slash pattern (Alg. 5's mask; Sec. 5.1 A(Q,K,V,M)): key s <= t is
    allowed for query t iff keep_v[s] or keep_s[t - s] (or, forced, s lies in block 0 or in t's own block).
    Returns O [len(rows) * block][d]."""
    q, qp = _f(q)
    k, kp = _f(k)
    v, vp = _f(v)
    N, d = q.shape
    rows_a = _rows(rows, N // block)
    keep_v = np.ascontiguousarray(keep_v, dtype=np.uint8)
    keep_s = np.ascontiguousarray(keep_s, dtype=np.uint8)
    assert keep_v.shape == (N,) and keep_s.shape == (N,)
    scale = (1.0 / np.sqrt(d)) if scale is None else float(scale)
    o = np.empty((len(rows_a) * block, d), dtype=np.float32)
    up = ctypes.POINTER(ctypes.c_ubyte)
    rc = _load().spo_vs_token_rows(qp, kp, vp, N, d, block, scale, rows_a.ctypes.data_as(ctypes.POINTER(ctypes.c_int)),
                                   len(rows_a), keep_v.ctypes.data_as(up), keep_s.ctypes.data_as(up), int(bool(forced)),
                                   o.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
    if rc:
        raise ValueError(f"spo_vs_token_rows failed ({rc})")
    return o


def vertical_slash_pattern(q, k, block: int, gamma: float, scale: Optional[float] = None, forced: bool = True):
    """Alg. 5 for one head with Q_hat = the last `block` queries.  Returns (kb_idx, kb_cnt, a_v, a_s, keep_v, keep_s)."""
    a_v, a_s = vertical_slash_sums(q, k, block, scale)
    keep_v, _ = select_cumulative(a_v, gamma)
    keep_s, _ = select_cumulative(a_s, gamma)
    idx, cnt = vs_block_lists(keep_v, keep_s, block, forced)
    return idx, cnt, a_v, a_s, keep_v, keep_s


def prefill_layer(q, k, v, block: int, head_to_cluster, pivot_heads, gamma: float,
                  rows: Optional[Sequence[int]] = None, scale: Optional[float] = None,
                  masks=None, paper_pattern: bool = False, gate=None, shared=None, fallback: str = "dense"):
    """One layer of pattern sharing with given pivots (Alg. 1 / Alg. 2 / Alg. 4).

    q [N][Hq][d], k/v [N][Hkv][d] float32.  Returns a dict with
      o       [nrows*B][Hq][d] float32
      scores  [C][nrows][nkb]  float32 (pivot block-mass rows)
      kb_idx  [C][nrows][nkb], kb_cnt [C][nrows]
    Heads with cluster id -1 run dense.  `masks`, if given as (kb_idx, kb_cnt) with
    those shapes, replaces the oracle's own pattern for the non-pivot heads (used
    to check outputs against a pattern produced elsewhere).  `paper_pattern` swaps
    the pattern construction for the paper's printed one (row softmax of block-mean
    logits, one selection over the flattened map, forced sink/diagonal kept); it
    needs every row unless `masks` is given.  `gate` = (delta, tau) applies Alg. 3 to
    every clustered non-pivot head, the pivot's own estimate serving as the pivotal
    representative: heads that fail run dense (the stand-in for the fallback pattern);
    the result then also holds "shared" [Hq] bool and "dist" [Hq][2].  `shared`, if
    given, replaces the gate's decisions (to check outputs under decisions taken elsewhere).
    `fallback` = "vertical_slash" gives failing heads and heads without a cluster the
    pattern of Alg. 5 instead of dense attention (needs every row)."""
    q = np.asarray(q, dtype=np.float32)
    k = np.asarray(k, dtype=np.float32)
    v = np.asarray(v, dtype=np.float32)
    N, Hq, d = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    nkb = N // block
    rows = _rows(rows, nkb)
    nr = len(rows)
    C = len(pivot_heads)
    o = np.zeros((nr * block, Hq, d), dtype=np.float32)
    scores = np.zeros((C, nr, nkb), dtype=np.float32)
    kb_idx = np.full((C, nr, nkb), -1, dtype=np.int32)
    kb_cnt = np.zeros((C, nr), dtype=np.int32)
    for c, p in enumerate(pivot_heads):
        p = int(p)
        assert int(head_to_cluster[p]) == c
        g = p // G
        op, sc, _ = dense_rows(q[:, p], k[:, g], v[:, g], block, rows, scale, want_scores=not paper_pattern)
        o[:, p] = op
        if paper_pattern:
            sc = softmax_rows(mean_logit_rows(q[:, p], k[:, g], block, rows, scale))
            scores[c] = sc
            if masks is None:
                assert nr == nkb and np.array_equal(rows, np.arange(nkb)), "global selection needs the whole map"
                kb_idx[c], kb_cnt[c], _ = build_mask_global(sc, gamma, forced=True)
        else:
            scores[c] = sc
            kb_idx[c], kb_cnt[c], _ = build_mask_rows(sc, gamma, rows)
    if masks is not None:
        kb_idx, kb_cnt = masks
    pivots = {int(p) for p in pivot_heads}
    decided = np.ones(Hq, dtype=bool)
    dist = np.zeros((Hq, 2), dtype=np.float64)
    if gate is not None:
        est = {}
        for h in range(Hq):
            if int(head_to_cluster[h]) >= 0:
                est[h] = last_row_estimate(q[:, h], k[:, h // G], block, scale)
        for h in range(Hq):
            c = int(head_to_cluster[h])
            if c < 0:
                continue
            decided[h], dist[h, 0], dist[h, 1] = determine_pattern(est[h], est[int(pivot_heads[c])], gate[0], gate[1])
    if shared is not None:
        decided = np.asarray(shared, dtype=bool)
    for h in range(Hq):
        if h in pivots:
            continue
        c = int(head_to_cluster[h])
        g = h // G
        if (c < 0 or not decided[h]) and fallback == "vertical_slash":
            assert nr == nkb, "the vertical-slash lists are built for every row"
            vi, vc = vertical_slash_pattern(q[:, h], k[:, g], block, gamma, scale)[:2]
            o[:, h] = masked_rows(q[:, h], k[:, g], v[:, g], block, vi, vc, rows, scale)
        elif c < 0 or not decided[h]:
            o[:, h], _, _ = dense_rows(q[:, h], k[:, g], v[:, g], block, rows, scale, want_scores=False)
        else:
            o[:, h] = masked_rows(q[:, h], k[:, g], v[:, g], block, kb_idx[c], kb_cnt[c], rows, scale)
    return {"o": o, "scores": scores, "kb_idx": kb_idx, "kb_cnt": kb_cnt, "shared": decided, "dist": dist}


ROLE_FALLBACK, ROLE_PIVOT = -1, -2


def prefill_layers_dict(layers, block: int, gamma: float, delta: float, tau: float, paper_pattern: bool = False,
                        scale: Optional[float] = None, pattern_dict: Optional[dict] = None, fallback: str = "dense"):
    """Alg. 1 applied head by head (ascending head index), layer by layer, with the pivotal pattern
    dictionary of Sec. 5.2 carried across layers.

    `layers` is a list of dicts with q [N][Hq][d], k, v [N][Hkv][d] float32 and head_to_cluster [Hq]
    (cluster ids shared by all layers, -1 = no cluster).  For each head of a cluster c:
      Alg. 3 decides with the dictionary's representative a~ of c (no entry: only the sparsity test);
      shared_pivot and an entry exists  -> masked attention with the entry's lists (Alg. 4), role c;
      shared_pivot and no entry         -> dense attention (all-ones pattern), then Alg. 2 builds the
                                           lists and the entry (a~ = this head's estimate), role -2;
      otherwise                          -> the fallback pattern, role -1, no update: dense attention,
                                           or with fallback = "vertical_slash" the pattern of Alg. 5.
    Heads without a cluster take the fallback too (role -1).  Every row of every map is needed.

    Returns (results, pattern_dict): results[l] = {"o", "role" [Hq], "dist" [Hq][2]};
    pattern_dict[c] = {"a_tilde", "kb_idx", "kb_cnt", "scores", "layer", "head"}."""
    D = {} if pattern_dict is None else pattern_dict
    results = []
    for l, Lr in enumerate(layers):
        q = np.asarray(Lr["q"], dtype=np.float32)
        k = np.asarray(Lr["k"], dtype=np.float32)
        v = np.asarray(Lr["v"], dtype=np.float32)
        h2c = [int(x) for x in Lr["head_to_cluster"]]
        N, Hq, d = q.shape
        G = Hq // k.shape[1]
        o = np.zeros((N, Hq, d), dtype=np.float32)
        role = np.full(Hq, ROLE_FALLBACK, dtype=np.int32)
        dist = np.zeros((Hq, 2), dtype=np.float64)
        for h in range(Hq):
            c, g = h2c[h], h // G
            qh, kh, vh = q[:, h], k[:, g], v[:, g]
            shared = False
            if c >= 0:
                a_hat = last_row_estimate(qh, kh, block, scale)
                entry = D.get(c)
                shared, dist[h, 0], dist[h, 1] = determine_pattern(
                    a_hat, None if entry is None else entry["a_tilde"], delta, tau)
            if shared and entry is not None:
                o[:, h] = masked_rows(qh, kh, vh, block, entry["kb_idx"], entry["kb_cnt"], None, scale)
                role[h] = c
            elif shared:
                o[:, h], sc, _ = dense_rows(qh, kh, vh, block, None, scale, want_scores=not paper_pattern)
                if paper_pattern:
                    sc = softmax_rows(mean_logit_rows(qh, kh, block, None, scale))
                    idx, cnt, _ = build_mask_global(sc, gamma, forced=True)
                else:
                    idx, cnt, _ = build_mask_rows(sc, gamma)
                D[c] = {"a_tilde": a_hat, "kb_idx": idx, "kb_cnt": cnt, "scores": sc, "layer": l, "head": h}
                role[h] = ROLE_PIVOT
            elif fallback == "vertical_slash":
                vi, vc = vertical_slash_pattern(qh, kh, block, gamma, scale)[:2]
                o[:, h] = masked_rows(qh, kh, vh, block, vi, vc, None, scale)
            else:
                o[:, h], _, _ = dense_rows(qh, kh, vh, block, None, scale, want_scores=False)
        results.append({"o": o, "role": role, "dist": dist})
    return results, D
