"""GPU parity for Search Vertical Slash Pattern (Alg. 5): sp_search_vertical_slash and the
vertical-slash fallback of sp_prefill_layer_dict against the CPU oracle.

Bars.  Sums a_v / a_s: |gpu - oracle| <= 1e-8 + 1e-4 * oracle.  A logit is a 64- or 128-term fp32
sum of exact bf16 products (absolute error about 1e-5 at |x| ~ 30), the exponential carries that as a
relative error of the same size, the row normaliser averages it out and a sum adds `block` such terms;
measured relative errors are below 1e-6.  Lists and counts: bit-exact when the oracle's selection and
block conversion are fed the GPU's own sums.  Outputs: max-abs 2e-2 / mean-abs 2e-3 against the oracle
run with the GPU's lists."""
import numpy as np
import pytest

from tests.test_gpu_parity import OUT_MAX, OUT_MEAN, _LazyHost

pytestmark = pytest.mark.gpu

S_ABS, S_REL = 1e-8, 1e-4


def _sum_check(got, want, what):
    err = np.abs(got.astype(np.float64) - want.astype(np.float64))
    bound = S_ABS + S_REL * np.abs(want.astype(np.float64))
    worst = float((err / bound).max())
    assert worst <= 1.0, f"{what}: {worst:.2f}x the bound (max abs {err.max():.3e})"
    return worst


def _search(sp, q, k, B, heads, gamma, forced):
    import torch
    shape = sp.shape_of(q, k, None, B)
    N = q.shape[1]
    nkb = N // B
    n = len(heads)
    ws = torch.empty(sp.sp_vs_workspace_bytes(shape, n), dtype=torch.uint8, device="cuda")
    sums = torch.full((1, n, 2, N), -1.0, dtype=torch.float32, device="cuda")
    idx = torch.full((1, n, nkb, nkb), -5, dtype=torch.int32, device="cuda")
    cnt = torch.full((1, n, nkb), -5, dtype=torch.int32, device="cuda")
    sp.sp_search_vertical_slash(shape, q, k, heads, gamma, forced, sums, idx, cnt, ws)
    torch.cuda.synchronize()
    return shape, sums.cpu().numpy()[0], idx, cnt


def _check_lists(oracle, sums_h, idx_h, cnt_h, B, gamma, forced, what):
    for n in range(sums_h.shape[0]):
        keep_v, _ = oracle.select_cumulative(sums_h[n, 0], gamma)
        keep_s, _ = oracle.select_cumulative(sums_h[n, 1], gamma)
        idx_o, cnt_o = oracle.vs_block_lists(keep_v, keep_s, B, forced)
        assert np.array_equal(cnt_o, cnt_h[n]), f"{what} head #{n}: counts differ"
        assert np.array_equal(idx_o, idx_h[n]), f"{what} head #{n}: lists differ"


@pytest.mark.parametrize("d,B,N", [(128, 128, 2048), (128, 64, 1024), (64, 128, 1152), (64, 64, 640)])
def test_vertical_slash_random_inputs(d, B, N):
    import oracle
    import paper_2505_19578_amd as sp
    from synth import random_qkv, bf16_bits_to_f32
    from tests.gpu_util import to_dev
    qb, kb, _ = random_qkv(61, N, 4, 2, d, 2.5)
    q, k = to_dev(qb), to_dev(kb)
    hq, hk = bf16_bits_to_f32(qb), bf16_bits_to_f32(kb)
    heads = [3, 0]
    for gamma, forced in ((0.5, True), (0.9, False), (0.2, False)):
        print(f"[vs random d{d} B{B} N{N}] gamma {gamma} forced {forced}", flush=True)
        _, sums_h, idx, cnt = _search(sp, q, k, B, heads, gamma, forced)
        worst = 0.0
        for n, h in enumerate(heads):
            a_v, a_s = oracle.vertical_slash_sums(hq[:, h], hk[:, h // 2], B)
            worst = max(worst, _sum_check(sums_h[n, 0], a_v, f"head {h} a_v"), _sum_check(sums_h[n, 1], a_s, f"head {h} a_s"))
        _check_lists(oracle, sums_h, idx.cpu().numpy()[0], cnt.cpu().numpy()[0], B, gamma, forced, f"gamma {gamma}")
    print(f"[vs random d{d} B{B} N{N}] sums at {worst:.3f} of the bound", flush=True)


@pytest.mark.parametrize("name,seq", [("tiny", None), ("llama8b_32k", 4096)])
def test_vertical_slash_synthetic_and_attention_over_its_lists(name, seq):
    import torch
    import oracle
    import paper_2505_19578_amd as sp
    from synth import CONFIGS, make_layer
    from tests.gpu_util import to_dev, bf16_dev_to_f32, err_stats
    L = make_layer(CONFIGS[name], seq=seq)
    cfg = L["cfg"]
    host = _LazyHost(L)
    q, k, v = (to_dev(L[x]) for x in "qkv")
    B, G = cfg.block, cfg.group
    nkb = cfg.seq // B
    heads = [1, cfg.n_q_heads - 1, 2]
    shape, sums_h, idx, cnt = _search(sp, q, k, B, heads, cfg.gamma, True)
    idx_h, cnt_h = idx.cpu().numpy()[0], cnt.cpu().numpy()[0]
    worst = 0.0
    for n, h in enumerate(heads):
        a_v, a_s = oracle.vertical_slash_sums(host.head("q", h), host.head("k", h // G), B)
        worst = max(worst, _sum_check(sums_h[n, 0], a_v, f"head {h} a_v"), _sum_check(sums_h[n, 1], a_s, f"head {h} a_s"))
    _check_lists(oracle, sums_h, idx_h, cnt_h, B, cfg.gamma, True, name)
    dens = float(cnt_h.sum() / (len(heads) * nkb * (nkb + 1) / 2))
    # block-sparse attention over the lists
    o = torch.zeros_like(q)
    ws = torch.empty(sp.sp_workspace_bytes(shape, 0), dtype=torch.uint8, device="cuda")
    sp.sp_block_sparse_attn(shape, q, k, v, heads, list(range(len(heads))), idx, cnt, len(heads), o, ws)
    torch.cuda.synchronize()
    o_h = bf16_dev_to_f32(o)[0]
    for n, h in enumerate(heads):
        o_o = oracle.masked_rows(host.head("q", h), host.head("k", h // G), host.head("v", h // G), B, idx_h[n], cnt_h[n])
        emax, emean = err_stats(o_h[:, h], o_o)
        assert emax <= OUT_MAX and emean <= OUT_MEAN, f"head {h}: {emax} / {emean}"
    print(f"[vs {name}] sums at {worst:.3f} of the bound, block density {dens:.3f}", flush=True)


def test_dict_layer_with_vertical_slash_fallback():
    """Two layers through the dictionary with a sparsity threshold that sends part of the heads to the
    fallback, plus a head without a cluster: their lists equal a stand-alone search, their outputs the
    oracle's masked attention over those lists; roles equal the oracle's own run."""
    import torch
    import oracle
    import paper_2505_19578_amd as sp
    from synth import CONFIGS, make_layer, bf16_bits_to_f32
    from tests.gpu_util import to_dev, bf16_dev_to_f32, err_stats
    from tests.test_gpu_dict import _Dict
    from tests.test_gpu_determine import _f32, MARGIN
    Ls = [make_layer(CONFIGS["llama8b_32k"], layer=l, seq=2048, structure_layer=0) for l in range(2)]
    cfg = Ls[0]["cfg"]
    B, G, Hq, C = cfg.block, cfg.group, cfg.n_q_heads, cfg.n_clusters
    nqb = cfg.seq // B
    h2c = [int(x) for x in Ls[0]["head_to_cluster"]]
    h2c[6] = -1
    # d_sparse does not depend on the thresholds: take it from the oracle and cut at a wide gap
    ds = np.sort(np.array([oracle.determine_pattern(
        oracle.last_row_estimate(bf16_bits_to_f32(L["q"][:, h]), bf16_bits_to_f32(L["k"][:, h // G]), B), None, 10, 10)[1]
        for L in Ls for h in range(Hq)]))
    lo, hi = len(ds) // 4, 3 * len(ds) // 4
    i = lo + int(np.argmax(ds[lo + 1:hi + 1] - ds[lo:hi]))
    delta = float(0.5 * (ds[i] + ds[i + 1]))
    assert ds[i + 1] - ds[i] > 4 * MARGIN
    D = _Dict(sp, 1, C, nqb)
    vs_idx = torch.full((1, Hq, nqb, nqb), -3, dtype=torch.int32, device="cuda")
    vs_cnt = torch.full((1, Hq, nqb), -3, dtype=torch.int32, device="cuda")
    roles = []
    for l, L in enumerate(Ls):
        q, k, v = (to_dev(L[x]) for x in "qkv")
        host = _LazyHost(L)
        shape = sp.shape_of(q, k, None, B)
        slots = sorted({c for c in h2c if c >= 0})
        ws = torch.empty(sp.sp_workspace_bytes(shape, len(slots)) + sp.sp_vs_workspace_bytes(shape, Hq),
                         dtype=torch.uint8, device="cuda")
        o = torch.zeros_like(q)
        scores = torch.empty((1, len(slots), nqb, nqb), dtype=torch.float32, device="cuda")
        role = torch.full((1, Hq), -7, dtype=torch.int32, device="cuda")
        a_hat = torch.empty((1, Hq, nqb), dtype=torch.float32, device="cuda")
        dist = torch.empty((1, Hq, 2), dtype=torch.float32, device="cuda")
        vs_idx.fill_(-3)
        vs_cnt.fill_(-3)
        print(f"[dict + vs] layer {l} delta {delta:.4f}", flush=True)
        sp.sp_prefill_layer_dict(shape, q, k, v, h2c, cfg.gamma, delta, 10.0, 0, 0, D.c, o, scores, role, a_hat, dist, ws,
                                 fallback_mode=sp.SP_FALLBACK_VERTICAL_SLASH, vs_idx=vs_idx, vs_cnt=vs_cnt)
        torch.cuda.synchronize()
        role_h = role.cpu().numpy()[0]
        fb = [h for h in range(Hq) if role_h[h] == -1]
        assert 6 in fb and len(fb) > 1 and (role_h >= 0).any()
        # fallback heads: lists equal a stand-alone search of exactly those heads; other heads' lists untouched
        _, _, idx2, cnt2 = _search(sp, q, k, B, fb, cfg.gamma, True)
        vi, vc = vs_idx.cpu().numpy()[0], vs_cnt.cpu().numpy()[0]
        for n, h in enumerate(fb):
            assert np.array_equal(vi[h], idx2.cpu().numpy()[0, n]) and np.array_equal(vc[h], cnt2.cpu().numpy()[0, n])
        for h in range(Hq):
            if h not in fb:
                assert np.all(vc[h] == -3)
        o_h = bf16_dev_to_f32(o)[0]
        didx, dcnt = D.kb_idx.cpu().numpy()[0], D.kb_cnt.cpu().numpy()[0]
        for h in range(Hq):
            g = h // G
            qh, kh, vh = host.head("q", h), host.head("k", g), host.head("v", g)
            if role_h[h] == -1:
                o_o = oracle.masked_rows(qh, kh, vh, B, vi[h], vc[h])
            elif role_h[h] >= 0:
                o_o = oracle.masked_rows(qh, kh, vh, B, didx[role_h[h]], dcnt[role_h[h]])
            else:
                o_o, _, _ = oracle.dense_rows(qh, kh, vh, B, want_scores=False)
            emax, emean = err_stats(o_h[:, h], o_o)
            assert emax <= OUT_MAX and emean <= OUT_MEAN, f"layer {l} head {h} role {role_h[h]}: {emax} / {emean}"
        dens = float(sum(vc[h].sum() for h in fb) / (len(fb) * nqb * (nqb + 1) / 2))
        print(f"[dict + vs] layer {l}: roles {[int(x) for x in role_h]}; {len(fb)} heads on vertical-slash lists, "
              f"block density {dens:.3f}", flush=True)
        roles.append(role_h)
    o_layers = [{x: bf16_bits_to_f32(L[x]) for x in "qkv"} | {"head_to_cluster": h2c} for L in Ls]
    res, _ = oracle.prefill_layers_dict(o_layers, B, cfg.gamma, _f32(delta), 10.0, fallback="vertical_slash")
    for l in range(2):
        assert list(res[l]["role"]) == list(roles[l])


def test_vertical_slash_llama8b_128k_full_size():
    import torch
    import oracle
    import paper_2505_19578_amd as sp
    from synth import CONFIGS, make_layer
    from tests.gpu_util import to_dev, bf16_dev_to_f32, err_stats
    from tests.test_gpu_full_size import _sample_rows
    L = make_layer(CONFIGS["llama8b_128k"])
    cfg = L["cfg"]
    host = _LazyHost(L)
    q, k, v = (to_dev(L[x]) for x in "qkv")
    B, G = cfg.block, cfg.group
    nkb = cfg.nqb
    heads = [5, 30]
    print("[vs cfg3] search", flush=True)
    shape, sums_h, idx, cnt = _search(sp, q, k, B, heads, cfg.gamma, True)
    idx_h, cnt_h = idx.cpu().numpy()[0], cnt.cpu().numpy()[0]
    worst = 0.0
    for n, h in enumerate(heads):
        a_v, a_s = oracle.vertical_slash_sums(host.head("q", h), host.head("k", h // G), B)
        worst = max(worst, _sum_check(sums_h[n, 0], a_v, f"head {h} a_v"), _sum_check(sums_h[n, 1], a_s, f"head {h} a_s"))
    _check_lists(oracle, sums_h, idx_h, cnt_h, B, cfg.gamma, True, "cfg3")
    dens = float(cnt_h.sum() / (len(heads) * nkb * (nkb + 1) / 2))
    o = torch.zeros_like(q)
    ws = torch.empty(sp.sp_workspace_bytes(shape, 0), dtype=torch.uint8, device="cuda")
    sp.sp_block_sparse_attn(shape, q, k, v, heads, [0, 1], idx, cnt, 2, o, ws)
    torch.cuda.synchronize()
    rows = np.asarray(_sample_rows(nkb, 13, extra=0), dtype=np.int32)
    sel_t = np.concatenate([np.arange(i * B, (i + 1) * B) for i in rows])
    o_h = bf16_dev_to_f32(o[:, :, heads])[0]
    for n, h in enumerate(heads):
        o_o = oracle.masked_rows(host.head("q", h), host.head("k", h // G), host.head("v", h // G), B,
                                 idx_h[n][rows], cnt_h[n][rows], rows)
        emax, emean = err_stats(o_h[sel_t, n], o_o)
        assert emax <= OUT_MAX and emean <= OUT_MEAN, f"head {h}: {emax} / {emean}"
    print(f"[vs cfg3] sums at {worst:.3f} of the bound, block density of the vertical-slash lists {dens:.3f}", flush=True)
