"""GPU parity for Determine Sparse Pattern (Alg. 3): sp_determine_pattern,
sp_block_sparse_attn_gated and sp_prefill_layer_gated against the CPU oracle.

Bars.  Estimates a_hat: the score bar of the block-mean-logit map (relative 1e-4, absolute
1e-7).  Distances: |gpu - oracle| <= 2e-5 (both sum in fp64; what differs is the fp32
estimate they start from, relative 1e-6 or better, and d = sqrt(JSD) has slope 1/(2d) in JSD, so
the bar is checked where d >= 1e-3 and an absolute 1e-3 below that).  Decisions: equal to the
oracle's wherever both of its distances are farther than 1e-4 from their thresholds (the
thresholds reach both sides as the same fp32 numbers).  Outputs: max-abs 2e-2 / mean-abs 2e-3
against the oracle run with the GPU's own pattern and decisions."""
import numpy as np
import pytest

from tests.test_gpu_parity import _setup, OUT_MAX, OUT_MEAN
from tests.test_gpu_paper_pattern import _score_check

pytestmark = pytest.mark.gpu

D_TOL, MARGIN = 2e-5, 1e-4


def _f32(x):
    return float(np.float32(x))


def _oracle_gate(host, cfg, heads, ref_of, delta, tau):
    """Oracle estimates, distances and decisions for the listed heads (ref_of: head -> head or None)."""
    import oracle
    est = {h: oracle.last_row_estimate(host.head("q", h), host.head("k", h // cfg.group), cfg.block) for h in heads}
    out = {}
    for h in heads:
        ref = ref_of[h]
        out[h] = oracle.determine_pattern(est[h], None if ref is None else est[ref], _f32(delta), _f32(tau))
    return est, out


def _check_gate(est, gate, heads, a_hat_h, dist_h, pat_h, shared_map, delta, tau, label):
    n_border = 0
    worst_d = 0.0
    for n, h in enumerate(heads):
        _score_check(a_hat_h[n], est[h], f"{label} head {h} a_hat")
        shared, d_sparse, d_sim = gate[h]
        for got, want in ((dist_h[n, 0], d_sparse), (dist_h[n, 1], d_sim)):
            tol = D_TOL if want >= 1e-3 else 1e-3
            assert abs(got - want) <= tol, f"{label} head {h}: distance {got} vs {want}"
            worst_d = max(worst_d, abs(got - want))
        if abs(d_sparse - _f32(delta)) > MARGIN and abs(d_sim - _f32(tau)) > MARGIN:
            assert pat_h[h] == (shared_map[n] if shared else -1), f"{label} head {h}: decision differs"
        else:
            n_border += 1
    return worst_d, n_border


@pytest.mark.parametrize("name,seq", [("tiny", None), ("llama8b_32k", 4096), ("qwen7b_128k", 4096)])
def test_determine_pattern_matches_oracle(name, seq):
    import torch
    sp, cfg, L, dev, host = _setup(name, seq=seq)
    q, k = dev["q"], dev["k"]
    nqb, Hq = cfg.seq // cfg.block, cfg.n_q_heads
    shape = sp.shape_of(q, k, None, cfg.block)
    h2c, piv = [int(x) for x in L["head_to_cluster"]], [int(x) for x in L["pivot_heads"]]
    heads = list(range(Hq))[::-1]                     # listed in reverse: positions differ from head ids
    pos = {h: n for n, h in enumerate(heads)}
    # two heads get the representative of a *different* cluster, one has none
    ref_of = {h: piv[h2c[h]] for h in heads}
    ref_of[heads[0]] = piv[(h2c[heads[0]] + 1) % len(piv)]
    ref_of[heads[1]] = piv[(h2c[heads[1]] + 1) % len(piv)]
    ref_of[heads[2]] = None
    shared_map = [h2c[h] + 10 for h in heads]
    ws = torch.empty(sp.sp_score_workspace_bytes(shape, Hq), dtype=torch.uint8, device="cuda")
    a_hat = torch.full((1, Hq, nqb), -3.0, dtype=torch.float32, device="cuda")
    dist = torch.full((1, Hq, 2), -3.0, dtype=torch.float32, device="cuda")
    # first pass with thresholds that let everything through, to learn the distances
    est, gate = _oracle_gate(host, cfg, heads, ref_of, 10.0, 10.0)
    ds = sorted(g[1] for g in gate.values())
    dm = sorted(g[2] for g in gate.values() if g[2] > 0)
    delta = 0.5 * (ds[len(ds) // 2 - 1] + ds[len(ds) // 2])         # half the heads read as "highly sparse"
    tau = 0.5 * (dm[-2] + dm[-3]) if len(dm) >= 3 else 0.5 * dm[-1]  # the mismatched heads fail the similarity test
    for (dl, ta) in ((10.0, 10.0), (delta, tau), (0.3, 0.2)):
        pat = torch.full((1, Hq), -7, dtype=torch.int32, device="cuda")
        print(f"[determine {name}] launch delta={dl:.4f} tau={ta:.4f}", flush=True)
        sp.sp_determine_pattern(shape, q, k, heads, [(-1 if ref_of[h] is None else pos[ref_of[h]]) for h in heads],
                                shared_map, dl, ta, a_hat, dist, pat, ws)
        torch.cuda.synchronize()
        _, gate = _oracle_gate(host, cfg, heads, ref_of, dl, ta)
        worst, border = _check_gate(est, gate, heads, a_hat.cpu().numpy()[0], dist.cpu().numpy()[0],
                                    pat.cpu().numpy()[0], shared_map, dl, ta, name)
        n_shared = sum(1 for g in gate.values() if g[0])
        print(f"[determine {name}] delta={dl:.4f} tau={ta:.4f}: {n_shared}/{Hq} shared, distance err {worst:.2e}, "
              f"{border} borderline", flush=True)
        assert border == 0
        if (dl, ta) == (delta, tau):
            assert 0 < n_shared < Hq                 # both outcomes occur
    d_all = np.array([[g[1], g[2]] for g in gate.values()])
    print(f"[determine {name}] d_sparse {d_all[:, 0].min():.3f}..{d_all[:, 0].max():.3f}  d_sim(max) "
          f"{d_all[:, 1].max():.3f}", flush=True)


def _check_gated_layer(sp, cfg, L, dev, host, rows, delta, tau, label, h2c=None, check_heads=None, stages=True,
                       score_mode=0, select_mode=0):
    import torch
    import oracle
    from tests.gpu_util import alloc_layer, bf16_dev_to_f32, err_stats
    B, G = cfg.block, cfg.group
    nqb, Hq = cfg.seq // B, cfg.n_q_heads
    h2c = [int(x) for x in (L["head_to_cluster"] if h2c is None else h2c)]
    piv = [int(x) for x in L["pivot_heads"]]
    C = len(piv)
    q, k, v = dev["q"], dev["k"], dev["v"]
    shape, o, ws, scores, kb_idx, kb_cnt = alloc_layer(sp, cfg, q, k, C)
    a_hat = torch.empty((1, Hq, nqb), dtype=torch.float32, device="cuda")
    dist = torch.empty((1, Hq, 2), dtype=torch.float32, device="cuda")
    pat = torch.full((1, Hq), -7, dtype=torch.int32, device="cuda")
    o.zero_()
    print(f"[{label}] gated fused call delta={delta} tau={tau} N={cfg.seq}", flush=True)
    sp.sp_prefill_layer_gated(shape, q, k, v, h2c, piv, cfg.gamma, delta, tau, score_mode, select_mode, o, scores,
                              kb_idx, kb_cnt, a_hat, dist, pat, ws)
    torch.cuda.synchronize()
    pat_h = pat.cpu().numpy()[0]
    heads = list(range(Hq))
    ref_of = {h: (piv[h2c[h]] if h2c[h] >= 0 else None) for h in heads}
    est, gate = _oracle_gate(host, cfg, heads, ref_of, delta, tau)
    worst, border = _check_gate(est, gate, heads, a_hat.cpu().numpy()[0], dist.cpu().numpy()[0], pat_h,
                                h2c, delta, tau, label)
    assert border == 0
    for h in heads:
        if h2c[h] < 0:
            assert pat_h[h] == -1
    o_h = bf16_dev_to_f32(o)[0]
    idx_h, cnt_h = kb_idx.cpu().numpy()[0], kb_cnt.cpu().numpy()[0]
    rows = np.asarray(rows, dtype=np.int32)
    sel_t = np.concatenate([np.arange(i * B, (i + 1) * B) for i in rows])
    pivset = set(piv)
    n_dense = 0
    for h in (heads if check_heads is None else check_heads):
        g = h // G
        if h in pivset or pat_h[h] < 0:
            o_o, _, _ = oracle.dense_rows(host.head("q", h), host.head("k", g), host.head("v", g), B, rows,
                                          want_scores=False)
            n_dense += h not in pivset
        else:
            c = int(pat_h[h])
            assert c == h2c[h]
            o_o = oracle.masked_rows(host.head("q", h), host.head("k", g), host.head("v", g), B,
                                     idx_h[c][rows], cnt_h[c][rows], rows)
        emax, emean = err_stats(o_h[sel_t, h], o_o)
        assert emax <= OUT_MAX and emean <= OUT_MEAN, f"head {h}: out max-abs {emax}, mean-abs {emean}"
    n_shared = sum(1 for h in heads if h not in pivset and pat_h[h] >= 0)
    print(f"[{label}] {n_shared} heads share, {Hq - C - n_shared} fall back to dense ({n_dense} of them checked), "
          f"distance err {worst:.2e}", flush=True)
    if stages:      # determine -> pivots -> mask -> gated sparse reproduces the fused call bit for bit
        o2 = torch.zeros_like(o)
        sc2, idx2, cnt2 = torch.empty_like(scores), torch.empty_like(kb_idx), torch.empty_like(kb_cnt)
        a2, d2, p2 = torch.empty_like(a_hat), torch.empty_like(dist), torch.full_like(pat, -7)
        ws2 = torch.empty(sp.sp_score_workspace_bytes(shape, Hq), dtype=torch.uint8, device="cuda")
        sp.sp_determine_pattern(shape, q, k, heads, [(-1 if ref_of[h] is None else ref_of[h]) for h in heads], h2c,
                                delta, tau, a2, d2, p2, ws2)
        sp.sp_dense_attn_with_block_scores(shape, q, k, v, piv, o2, sc2, ws)
        free = [h for h in heads if h2c[h] < 0]
        if free:
            sp.sp_dense_attn_with_block_scores(shape, q, k, v, free, o2, None, ws)
        sp.sp_build_block_mask(sc2, C, nqb, nqb, cfg.gamma, idx2, cnt2)
        others = [h for h in heads if h2c[h] >= 0 and h not in pivset]
        sp.sp_block_sparse_attn_gated(shape, q, k, v, others, idx2, cnt2, C, p2, o2, ws)
        torch.cuda.synchronize()
        assert torch.equal(a2, a_hat) and torch.equal(d2, dist) and torch.equal(p2, pat)
        assert torch.equal(sc2, scores) and torch.equal(idx2, kb_idx) and torch.equal(cnt2, kb_cnt)
        assert torch.equal(o2.view(torch.int16), o.view(torch.int16))
    return pat_h, dist.cpu().numpy()[0]


@pytest.mark.parametrize("name,seq", [("tiny", None), ("llama8b_32k", 2048), ("qwen7b_128k", 4096)])
def test_gated_layer_small(name, seq):
    sp, cfg, L, dev, host = _setup(name, seq=seq)
    rows = np.arange(cfg.seq // cfg.block)
    # everything passes: identical to the ungated layer
    pat, dist = _check_gated_layer(sp, cfg, L, dev, host, rows, 10.0, 10.0, f"{name} open gate")
    assert np.all(pat >= 0)
    # a threshold between the heads' sparsity distances: some heads fall back to dense
    ds = np.sort(dist[:, 0])
    delta = float(0.5 * (ds[len(ds) // 2 - 1] + ds[len(ds) // 2]))
    pat, _ = _check_gated_layer(sp, cfg, L, dev, host, rows, delta, 10.0, f"{name} sparsity gate")
    assert np.any(pat < 0) and np.any(pat >= 0)
    # heads moved into a foreign cluster fail the similarity test; an unclustered head stays dense
    h2c = [int(x) for x in L["head_to_cluster"]]
    C = len(L["pivot_heads"])
    moved = [h for h in range(cfg.n_q_heads) if h not in set(int(p) for p in L["pivot_heads"])]
    h2c[moved[0]] = (h2c[moved[0]] + 1) % C
    if len(moved) > 2:
        h2c[moved[2]] = -1
    own = max(dist[h, 1] for h in range(cfg.n_q_heads))
    pat, dist2 = _check_gated_layer(sp, cfg, L, dev, host, rows, 10.0, float(own) + 0.02, f"{name} similarity gate",
                                    h2c=h2c, stages=False, score_mode=1, select_mode=1)
    assert pat[moved[0]] == -1, f"foreign head passed: d_sim {dist2[moved[0], 1]} vs own max {own}"


def test_llama8b_128k_gated_full_size():
    """Config 3 at full size with the paper's thresholds (delta 0.3, tau 0.2) and with an open sparsity gate."""
    from tests.test_gpu_full_size import _sample_rows, _sample_heads
    sp, cfg, L, dev, host = _setup("llama8b_128k")
    rows = _sample_rows(cfg.nqb, 9, extra=0)
    heads = _sample_heads(cfg, L, 1, clusters={0, 5})
    pat, dist = _check_gated_layer(sp, cfg, L, dev, host, rows, 0.3, 0.2, "cfg3 gate 0.3/0.2", check_heads=heads,
                                   stages=False)
    print(f"[cfg3 gate] d_sparse {dist[:, 0].min():.3f}..{dist[:, 0].max():.3f}, d_sim max {dist[:, 1].max():.3f}, "
          f"{int((pat >= 0).sum())} of {cfg.n_q_heads} heads pass the gate at delta 0.3 / tau 0.2", flush=True)
    _check_gated_layer(sp, cfg, L, dev, host, rows, 10.0, 0.2, "cfg3 gate open/0.2", check_heads=heads, stages=False)
