"""Pins for the oracle's cross-layer pivotal pattern dictionary (Sec. 5.2; Alg. 1 with Alg. 2-4
head by head).  The stages it calls are pinned elsewhere; here the control flow is tied to
hand-derived role tables and to compositions written independently of it.  CPU only."""
from __future__ import annotations

import numpy as np

import oracle
from synth import CONFIGS, make_layer, bf16_bits_to_f32

B, GAMMA = 64, 0.9


def _layers(n, h2c=None, seq=512):
    out = []
    for l in range(n):
        L = make_layer(CONFIGS["tiny"], layer=l, seq=seq, structure_layer=0)
        d = {x: bf16_bits_to_f32(L[x]) for x in "qkv"}
        d["head_to_cluster"] = list(L["head_to_cluster"]) if h2c is None else h2c
        out.append(d)
    return out


def _head(Lr, h):
    g = h // (Lr["q"].shape[1] // Lr["k"].shape[1])       # tiny config: one KV head per query head
    return Lr["q"][:, h], Lr["k"][:, g], Lr["v"][:, g]


def test_open_gates_first_layer_elects_first_heads_second_layer_only_shares():
    Ls = _layers(2)
    res, D = oracle.prefill_layers_dict(Ls, B, GAMMA, 10.0, 10.0)
    # tiny config: clusters {0,1} and {2,3}; nothing in the dictionary -> heads 0 and 2 run dense and install
    assert list(res[0]["role"]) == [-2, 0, -2, 1]
    assert list(res[1]["role"]) == [0, 0, 1, 1]
    assert {c: (e["layer"], e["head"]) for c, e in D.items()} == {0: (0, 0), 1: (0, 2)}
    # layer 0 equals the single-layer composition with those pivots given
    ref = oracle.prefill_layer(Ls[0]["q"], Ls[0]["k"], Ls[0]["v"], B, [0, 0, 1, 1], [0, 2], GAMMA)
    assert np.array_equal(res[0]["o"], ref["o"])
    for c in (0, 1):
        assert np.array_equal(D[c]["kb_idx"], ref["kb_idx"][c]) and np.array_equal(D[c]["kb_cnt"], ref["kb_cnt"][c])
    # layer 1: every head attends through the lists built from layer 0's pivots
    for h in range(4):
        q, k, v = _head(Ls[1], h)
        want = oracle.masked_rows(q, k, v, B, D[h // 2]["kb_idx"], D[h // 2]["kb_cnt"])
        assert np.array_equal(res[1]["o"][:, h], want)
    # the representative is the pivot's own last-row estimate; a pivot's d_sim is 0 by definition
    q, k, _ = _head(Ls[0], 2)
    assert np.array_equal(D[1]["a_tilde"], oracle.last_row_estimate(q, k, B))
    assert res[0]["dist"][0, 1] == 0.0 and res[0]["dist"][2, 1] == 0.0 and res[0]["dist"][1, 1] > 0.0


def test_election_skips_heads_that_fail_the_sparsity_test():
    Ls = _layers(2)
    base, _ = oracle.prefill_layers_dict(Ls, B, GAMMA, 10.0, 10.0)
    ds0, ds1 = base[0]["dist"][:, 0], base[1]["dist"][:, 0]
    assert ds0[1] < ds0[0] < ds0[3] < ds0[2]              # what the thresholds below rely on
    delta = 0.5 * (ds0[0] + ds0[1])                       # head 1 passes, heads 0, 2, 3 do not
    res, D = oracle.prefill_layers_dict(Ls, B, GAMMA, delta, 10.0)
    assert list(res[0]["role"]) == [-1, -2, -1, -1]
    assert set(D) == {0} and (D[0]["layer"], D[0]["head"]) == (0, 1)
    want = [(0 if ds1[h] < delta else -1) for h in (0, 1)] + [-1 if ds1[h] >= delta else -2 for h in (2, 3)]
    if want[2] == -2 and want[3] == -2:
        want[3] = 1                                       # second qualifying head of cluster 1 shares
    assert list(res[1]["role"]) == want
    # fallback heads are plain dense attention and leave the dictionary alone
    q, k, v = _head(Ls[0], 0)
    dense, _, _ = oracle.dense_rows(q, k, v, B, want_scores=False)
    assert np.array_equal(res[0]["o"][:, 0], dense)


def test_similarity_test_uses_the_dictionary_entry_and_rejections_do_not_update_it():
    Ls = _layers(2)
    base, D0 = oracle.prefill_layers_dict(Ls, B, GAMMA, 10.0, 10.0)
    dm = base[1]["dist"][:, 1]                            # layer-1 heads against layer-0 representatives
    q, k, _ = _head(Ls[1], 0)
    assert abs(dm[0] - oracle.js_distance(oracle.last_row_estimate(q, k, B), D0[0]["a_tilde"])) < 1e-12
    order = np.argsort(dm)
    tau = 0.5 * (dm[order[1]] + dm[order[2]])             # the two most similar heads pass
    res, D = oracle.prefill_layers_dict(Ls[:1], B, GAMMA, 10.0, 10.0)
    snapshot = {c: (e["kb_idx"].copy(), e["kb_cnt"].copy(), e["a_tilde"].copy()) for c, e in D.items()}
    res1, D = oracle.prefill_layers_dict(Ls[1:], B, GAMMA, 10.0, tau, pattern_dict=D)   # continue with the same dict
    want = [(h // 2 if h in order[:2] else -1) for h in range(4)]
    assert list(res1[0]["role"]) == want
    for c, (i, n, a) in snapshot.items():
        assert np.array_equal(D[c]["kb_idx"], i) and np.array_equal(D[c]["kb_cnt"], n) and np.array_equal(D[c]["a_tilde"], a)
    # and continuing equals processing both layers in one call
    both, _ = oracle.prefill_layers_dict(Ls, B, GAMMA, 10.0, 10.0)
    again, Dx = oracle.prefill_layers_dict(Ls[:1], B, GAMMA, 10.0, 10.0)
    again1, _ = oracle.prefill_layers_dict(Ls[1:], B, GAMMA, 10.0, 10.0, pattern_dict=Dx)
    assert np.array_equal(both[1]["o"], again1[0]["o"]) and np.array_equal(both[0]["o"], again[0]["o"])


def test_unclustered_heads_and_printed_construction():
    Ls = _layers(2, h2c=[0, -1, 0, 5])
    res, D = oracle.prefill_layers_dict(Ls, B, GAMMA, 10.0, 10.0, paper_pattern=True)
    assert list(res[0]["role"]) == [-2, -1, 0, -2] and list(res[1]["role"]) == [0, -1, 0, 5]
    assert set(D) == {0, 5}
    q, k, v = _head(Ls[0], 1)
    dense, _, _ = oracle.dense_rows(q, k, v, B, want_scores=False)
    assert np.array_equal(res[0]["o"][:, 1], dense)
    q, k, _ = _head(Ls[0], 3)
    sc = oracle.softmax_rows(oracle.mean_logit_rows(q, k, B))
    idx, cnt, _ = oracle.build_mask_global(sc, GAMMA, forced=True)
    assert np.array_equal(D[5]["kb_idx"], idx) and np.array_equal(D[5]["kb_cnt"], cnt)
    assert np.array_equal(D[5]["a_tilde"], sc[-1])        # printed construction: a~ is the last row of the map
