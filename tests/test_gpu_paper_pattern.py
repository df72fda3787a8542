"""GPU parity for the pattern construction as the paper prints it (Sec. 5.2; Alg. 2):
row softmax of block-mean logits and one selection over the flattened map, through
sp_block_mean_logit_scores / sp_build_block_mask_global / sp_prefill_layer_modes.

Bars.  Scores: |gpu - oracle| <= SC_ABS + SC_REL * oracle.  The GPU forms each block mean
from fp32 per-block sums (128 additions, then a 64- or 128-term dot product), the oracle in
fp64; with n = 256 rounding steps of relative size 2^-24 a logit of magnitude |x| <= 32 carries
an absolute error of about sqrt(n) * 2^-24 * |x| = 3e-5 (errors of mixed sign; 5e-4 if they all
lined up), which the softmax turns into the same *relative* error of a score: SC_REL = 1e-4,
with SC_ABS = 1e-7 covering scores that underflow towards 0 (measured: 4e-7 relative).  Lists and counts: bit-exact when the oracle's Alg. 2 is fed the GPU's own
score buffer.  Outputs: max-abs 2e-2 / mean-abs 2e-3 against the oracle run with the GPU's own
pattern."""
import numpy as np
import pytest

from tests.test_gpu_parity import _setup, OUT_MAX, OUT_MEAN

pytestmark = pytest.mark.gpu

SC_ABS, SC_REL = 1e-7, 1e-4


def _score_check(got, want, what):
    err = np.abs(got.astype(np.float64) - want.astype(np.float64))
    bound = SC_ABS + SC_REL * np.abs(want.astype(np.float64))
    worst = float((err / bound).max())
    assert worst <= 1.0, f"{what}: score error {worst:.2f}x the bound (max abs {err.max():.3e})"
    return float(err.max()), worst


@pytest.mark.parametrize("d,B,N", [(128, 128, 2048), (128, 64, 1024), (64, 128, 1152), (64, 64, 640)])
def test_mean_logit_scores_match_oracle(d, B, N):
    import torch
    import oracle
    import paper_2505_19578_amd as sp
    from synth import random_qkv, bf16_bits_to_f32
    from tests.gpu_util import to_dev
    Hq, Hkv = 4, 2
    qb, kb, _ = random_qkv(31, N, Hq, Hkv, d, 2.0)
    q, k = to_dev(qb), to_dev(kb)
    hq, hk = bf16_bits_to_f32(qb), bf16_bits_to_f32(kb)
    nqb = N // B
    shape = sp.shape_of(q, k, None, B)
    heads = [3, 0, 2]
    sc = torch.full((1, len(heads), nqb, nqb), -7.0, dtype=torch.float32, device="cuda")
    ws = torch.empty(sp.sp_score_workspace_bytes(shape, len(heads)), dtype=torch.uint8, device="cuda")
    print(f"[mean-logit d{d} B{B} N{N}] launch", flush=True)
    sp.sp_block_mean_logit_scores(shape, q, k, heads, sc, ws)
    torch.cuda.synchronize()
    sc_h = sc.cpu().numpy()[0]
    for n, h in enumerate(heads):
        want = oracle.softmax_rows(oracle.mean_logit_rows(hq[:, h], hk[:, h // 2], B))
        emax, worst = _score_check(sc_h[n], want, f"head {h}")
        assert np.all(np.triu(sc_h[n], 1) == 0)
        np.testing.assert_allclose(sc_h[n].sum(axis=-1), 1.0, atol=1e-5)
    print(f"[mean-logit d{d} B{B} N{N}] max abs {emax:.2e}, {worst:.3f} of the bound", flush=True)


def _maps_for_builder(rng, n_maps, n, kind):
    raw = np.tril(rng.random((n_maps, n, n)) ** 6)
    sc = raw / np.maximum(raw.sum(axis=-1, keepdims=True), 1e-30)
    if kind == "ties":
        sc = np.tril(rng.integers(0, 5, size=(n_maps, n, n)) / 16.0)
    elif kind == "sparse":
        sc[rng.random(sc.shape) < 0.7] = 0.0
    elif kind == "ones":        # one-hot rows: scores equal to 1.0 exactly (top histogram bin)
        sc = np.zeros((n_maps, n, n))
        for m in range(n_maps):
            for i in range(n):
                sc[m, i, rng.integers(0, i + 1)] = 1.0
    elif kind == "zero":
        sc = np.zeros((n_maps, n, n))
        if n_maps > 1:
            sc[1, n - 1, 0] = 0.25
    elif kind == "bad":
        sc[:, np.triu_indices(n, 1)[0], np.triu_indices(n, 1)[1]] = 0.5   # beyond the diagonal: ignored
        sc[0, n - 1, 0] = np.nan
        sc[0, n // 2, 0] = -3.0
        sc[0, n // 2, n // 2] = 9.0
    return sc.astype(np.float32)


@pytest.mark.parametrize("n", [1, 2, 3, 5, 64, 65, 257, 1024])
def test_global_mask_builder_bit_exact(n):
    import torch
    import oracle
    import paper_2505_19578_amd as sp
    rng = np.random.default_rng(100 + n)
    n_maps = 3
    ws = torch.empty(sp.sp_mask_workspace_bytes(n_maps, n), dtype=torch.uint8, device="cuda")
    idx = torch.empty((n_maps, n, n), dtype=torch.int32, device="cuda")
    cnt = torch.empty((n_maps, n), dtype=torch.int32, device="cuda")
    kinds = ["random", "ties", "sparse", "ones", "zero", "bad"] if n <= 257 else ["random", "ties"]
    for kind in kinds:
        sc = _maps_for_builder(rng, n_maps, n, kind)
        dev = torch.from_numpy(sc).cuda()
        for gamma, forced in ((0.9, True), (0.5, False), (1.0, False), (0.95, True)):
            idx.fill_(-5)
            cnt.fill_(-5)
            print(f"[global builder n={n} {kind} gamma={gamma} forced={forced}] launch", flush=True)
            sp.sp_build_block_mask_global(dev, n_maps, n, n, gamma, forced, idx, cnt, ws)
            torch.cuda.synchronize()
            idx_h, cnt_h = idx.cpu().numpy(), cnt.cpu().numpy()
            for m in range(n_maps):
                idx_o, cnt_o, _ = oracle.build_mask_global(sc[m], gamma, forced)
                assert np.array_equal(cnt_o, cnt_h[m]), f"{kind} map {m}: counts differ"
                assert np.array_equal(idx_o, idx_h[m]), f"{kind} map {m}: lists differ"


def _check_modes(sp, cfg, L, dev, host, rows, score_mode, select_mode, label, check_heads=None, stages=True):
    """Fused call in the given modes; scores / lists / outputs against the oracle on `rows`."""
    import torch
    import oracle
    from tests.gpu_util import alloc_layer, bf16_dev_to_f32, err_stats
    B, G = cfg.block, cfg.group
    nqb = cfg.seq // B
    h2c, piv = L["head_to_cluster"], L["pivot_heads"]
    C = len(piv)
    q, k, v = dev["q"], dev["k"], dev["v"]
    shape, o, ws, scores, kb_idx, kb_cnt = alloc_layer(sp, cfg, q, k, C)
    o.zero_()
    print(f"[{label}] fused call modes=({score_mode},{select_mode}) N={cfg.seq}", flush=True)
    sp.sp_prefill_layer_modes(shape, q, k, v, h2c, piv, cfg.gamma, score_mode, select_mode, o, scores, kb_idx,
                              kb_cnt, ws)
    torch.cuda.synchronize()
    o_h = bf16_dev_to_f32(o)[0]
    sc_h, idx_h, cnt_h = scores.cpu().numpy()[0], kb_idx.cpu().numpy()[0], kb_cnt.cpu().numpy()[0]
    rows = np.asarray(rows, dtype=np.int32)
    sel_t = np.concatenate([np.arange(i * B, (i + 1) * B) for i in rows])
    for c in range(C):      # lists bit-exact given the GPU's scores, all rows
        if select_mode == sp.SP_SELECT_GLOBAL:
            idx_o, cnt_o, _ = oracle.build_mask_global(sc_h[c], cfg.gamma, True)
        else:
            idx_o, cnt_o, _ = oracle.build_mask_rows(sc_h[c], cfg.gamma)
        assert np.array_equal(cnt_o, cnt_h[c]) and np.array_equal(idx_o, idx_h[c]), f"cluster {c}: lists differ"
    assert np.all(np.triu(sc_h, 1) == 0)
    heads = range(cfg.n_q_heads) if check_heads is None else check_heads
    pivset = {int(p) for p in piv}
    worst = [0.0, 0.0, 0.0]
    for h in heads:
        g, c = h // G, int(h2c[h])
        if h in pivset:
            o_o, sc_mass, _ = oracle.dense_rows(host.head("q", h), host.head("k", g), host.head("v", g), B, rows,
                                                want_scores=score_mode == sp.SP_SCORE_BLOCK_MASS)
            if score_mode == sp.SP_SCORE_MEAN_LOGIT:
                want = oracle.softmax_rows(oracle.mean_logit_rows(host.head("q", h), host.head("k", g), B, rows))
                worst[2] = max(worst[2], _score_check(sc_h[c][rows], want, f"head {h}")[1])
            else:
                assert err_stats(sc_h[c][rows], sc_mass)[0] <= 1e-3
        else:
            o_o = oracle.masked_rows(host.head("q", h), host.head("k", g), host.head("v", g), B,
                                     idx_h[c][rows], cnt_h[c][rows], rows)
        emax, emean = err_stats(o_h[sel_t, h], o_o)
        worst[0], worst[1] = max(worst[0], emax), max(worst[1], emean)
        assert emax <= OUT_MAX and emean <= OUT_MEAN, f"head {h}: out max-abs {emax}, mean-abs {emean}"
    dens = float(cnt_h.sum() / (C * nqb * (nqb + 1) / 2))
    print(f"[{label}] out max {worst[0]:.2e} mean {worst[1]:.2e} scores {worst[2]:.3f} of bound, "
          f"density {dens:.3f}", flush=True)
    if stages:      # the stage calls reproduce the fused call bit for bit
        o2, sc2, idx2, cnt2 = torch.zeros_like(o), torch.empty_like(scores), torch.empty_like(kb_idx), torch.empty_like(kb_cnt)
        if score_mode == sp.SP_SCORE_MEAN_LOGIT:
            sp.sp_dense_attn_with_block_scores(shape, q, k, v, list(piv), o2, None, ws)
            ws2 = torch.empty(sp.sp_score_workspace_bytes(shape, C), dtype=torch.uint8, device="cuda")
            sp.sp_block_mean_logit_scores(shape, q, k, list(piv), sc2, ws2)
        else:
            sp.sp_dense_attn_with_block_scores(shape, q, k, v, list(piv), o2, sc2, ws)
        if select_mode == sp.SP_SELECT_GLOBAL:
            ws3 = torch.empty(sp.sp_mask_workspace_bytes(C, nqb), dtype=torch.uint8, device="cuda")
            sp.sp_build_block_mask_global(sc2, C, nqb, nqb, cfg.gamma, True, idx2, cnt2, ws3)
        else:
            sp.sp_build_block_mask(sc2, C, nqb, nqb, cfg.gamma, idx2, cnt2)
        others = [h for h in range(cfg.n_q_heads) if h not in pivset]
        sp.sp_block_sparse_attn(shape, q, k, v, others, [int(h2c[h]) for h in others], idx2, cnt2, C, o2, ws)
        torch.cuda.synchronize()
        assert torch.equal(sc2, scores) and torch.equal(idx2, kb_idx) and torch.equal(cnt2, kb_cnt)
        assert torch.equal(o2.view(torch.int16), o.view(torch.int16))
    return dict(scores=scores, kb_idx=kb_idx, kb_cnt=kb_cnt, density=dens)


@pytest.mark.parametrize("name,seq", [("tiny", None), ("llama8b_32k", 2048), ("qwen7b_128k", 4096)])
def test_fused_paper_modes_small(name, seq):
    sp, cfg, L, dev, host = _setup(name, seq=seq)
    rows = np.arange(cfg.seq // cfg.block)
    _check_modes(sp, cfg, L, dev, host, rows, sp.SP_SCORE_MEAN_LOGIT, sp.SP_SELECT_GLOBAL, f"{name} paper")
    if name != "qwen7b_128k":       # the two mixed combinations
        _check_modes(sp, cfg, L, dev, host, rows, sp.SP_SCORE_BLOCK_MASS, sp.SP_SELECT_GLOBAL, f"{name} mass+global")
        _check_modes(sp, cfg, L, dev, host, rows, sp.SP_SCORE_MEAN_LOGIT, sp.SP_SELECT_PER_ROW, f"{name} logit+row")


def test_llama8b_128k_paper_modes_full_size_and_coverage():
    """Config 3 at full size in the paper's printed construction, on sampled rows; then the two
    constructions side by side on the same inputs: density, and how much true attention mass
    (the block-mass map of the pivot) each pattern covers."""
    import torch
    from tests.gpu_util import alloc_layer
    from tests.test_gpu_full_size import _sample_rows, _sample_heads
    sp, cfg, L, dev, host = _setup("llama8b_128k")
    rows = _sample_rows(cfg.nqb, 7)
    res = _check_modes(sp, cfg, L, dev, host, rows, sp.SP_SCORE_MEAN_LOGIT, sp.SP_SELECT_GLOBAL, "cfg3 paper",
                       check_heads=_sample_heads(cfg, L, 1), stages=False)
    shape, o, ws, mass, idx_r, cnt_r = alloc_layer(sp, cfg, dev["q"], dev["k"], cfg.n_clusters)
    sp.sp_prefill_layer(shape, dev["q"], dev["k"], dev["v"], L["head_to_cluster"], L["pivot_heads"], cfg.gamma, o,
                        mass, idx_r, cnt_r, ws)
    torch.cuda.synchronize()
    nqb = cfg.nqb

    def covered(idx, cnt):
        valid = torch.arange(nqb, device="cuda")[None, None, None, :] < cnt[..., None]
        hits = torch.zeros(mass.shape, dtype=torch.int32, device="cuda")
        hits.scatter_add_(-1, idx.clamp(min=0).long(), valid.to(torch.int32))   # the -1 tail adds 0 to block 0
        return (mass * (hits > 0)).sum(-1)                  # [1][C][nqb] covered mass per query-block row

    cov_row, cov_pap = covered(idx_r, cnt_r), covered(res["kb_idx"], res["kb_cnt"])
    tri = nqb * (nqb + 1) / 2 * cfg.n_clusters
    d_row, d_pap = float(cnt_r.sum()) / tri, float(res["kb_cnt"].sum()) / tri
    print(f"[cfg3 constructions] block-mass + per-row: density {d_row:.4f}, covered mass mean "
          f"{float(cov_row.mean()):.4f} min {float(cov_row.min()):.4f};  block-mean-logit + global: density "
          f"{d_pap:.4f}, covered mass mean {float(cov_pap.mean()):.4f} min {float(cov_pap.min()):.4f}", flush=True)
    assert float(cov_row.min()) >= cfg.gamma - 2e-3         # what the per-row reading guarantees by construction
    assert 0.0 < d_pap < 1.0
