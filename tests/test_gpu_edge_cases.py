"""GPU edge cases of the C-ABI calls against the CPU oracle: batch > 1, strided (interleaved QKV) layouts,
a caller-given softmax scale, caller-made key-block lists (all-ones = dense, sink + diagonal only, empty),
heads outside every cluster, the bitmask output, every mask-kernel code path (rows in registers / re-read
rows / nkb not a multiple of 64), special score values, and run-to-run determinism."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

OUT_MAX, OUT_MEAN = 2e-2, 2e-3


def _dev(bits):
    import torch
    return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()


def _f32(bits):
    from synth import bf16_bits_to_f32
    return bf16_bits_to_f32(bits)


def _err(got, want):
    d = np.abs(got.astype(np.float64) - want.astype(np.float64))
    return float(d.max()), float(d.mean())


def test_batch2_interleaved_qkv_and_custom_scale():
    """Q, K, V are slices of one [b][t][Hq+2Hkv][d] tensor (non-trivial strides), batch 2, scale 0.2."""
    import torch
    import oracle
    import paper_2505_19578_amd as sp
    from synth import random_qkv
    N, Hq, Hkv, d, B, scale = 512, 4, 2, 64, 64, 0.2
    packs = []
    for bb in range(2):
        q, k, v = random_qkv(20 + bb, N, Hq, Hkv, d)
        packs.append(np.concatenate([q, k, v], axis=1))
    qkv = _dev(np.stack(packs))                        # [2][N][Hq+2Hkv][d]
    q, k, v = qkv[:, :, :Hq], qkv[:, :, Hq:Hq + Hkv], qkv[:, :, Hq + Hkv:]
    o_full = torch.zeros((2, N, Hq + 1, d), dtype=torch.bfloat16, device="cuda")   # padded head stride
    o = o_full[:, :, :Hq]
    shape = sp.shape_of(q, k, o, B, softmax_scale=scale)
    nqb = N // B
    ws = torch.empty(sp.sp_workspace_bytes(shape, 2), dtype=torch.uint8, device="cuda")
    sc = torch.empty((2, 2, nqb, nqb), dtype=torch.float32, device="cuda")
    idx = torch.empty((2, 2, nqb, nqb), dtype=torch.int32, device="cuda")
    cnt = torch.empty((2, 2, nqb), dtype=torch.int32, device="cuda")
    h2c, piv, gamma = [0, 1, 0, 1], [0, 1], 0.7
    sp.sp_prefill_layer(shape, q, k, v, h2c, piv, gamma, o, sc, idx, cnt, ws)
    torch.cuda.synchronize()
    assert torch.all(o_full[:, :, Hq] == 0)            # the padding head slot is never written
    for bb in range(2):
        hq, hk, hv = (_f32(packs[bb][:, a:b]) for a, b in ((0, Hq), (Hq, Hq + Hkv), (Hq + Hkv, Hq + 2 * Hkv)))
        idx_h, cnt_h = idx[bb].cpu().numpy(), cnt[bb].cpu().numpy()
        ref = oracle.prefill_layer(hq, hk, hv, B, h2c, piv, gamma, scale=scale, masks=(idx_h, cnt_h))
        assert np.abs(sc[bb].cpu().numpy() - ref["scores"]).max() <= 1e-3
        for c in range(2):
            i2, c2, _ = oracle.build_mask_rows(sc[bb, c].cpu().numpy(), gamma)
            assert np.array_equal(i2, idx_h[c]) and np.array_equal(c2, cnt_h[c])
        e = _err(o[bb].float().cpu().numpy(), ref["o"])
        assert e[0] <= OUT_MAX and e[1] <= OUT_MEAN, e


def test_sparse_call_with_caller_lists_and_unclustered_heads():
    import torch
    import oracle
    import paper_2505_19578_amd as sp
    from synth import random_qkv
    N, Hq, Hkv, d, B = 1024, 4, 2, 128, 128
    qb, kb, vb = random_qkv(31, N, Hq, Hkv, d)
    q, k, v = (_dev(x).unsqueeze(0) for x in (qb, kb, vb))
    hq, hk, hv = _f32(qb), _f32(kb), _f32(vb)
    nqb = N // B
    shape = sp.shape_of(q, k, None, B)
    ws = torch.empty(sp.sp_workspace_bytes(shape, Hq), dtype=torch.uint8, device="cuda")
    # three maps: all-ones, sink + diagonal, empty
    idx = np.full((3, nqb, nqb), -1, np.int32)
    cnt = np.zeros((3, nqb), np.int32)
    for i in range(nqb):
        idx[0, i, : i + 1] = np.arange(i + 1)
        cnt[0, i] = i + 1
        sel = sorted({0, i})
        idx[1, i, : len(sel)] = sel
        cnt[1, i] = len(sel)
    o = torch.full_like(q, 7.0)
    sp.sp_block_sparse_attn(shape, q, k, v, [3, 0, 2], [0, 1, 2], torch.from_numpy(idx).cuda().unsqueeze(0),
                            torch.from_numpy(cnt).cuda().unsqueeze(0), 3, o, ws)
    torch.cuda.synchronize()
    og = o.float().cpu().numpy()[0]
    assert np.all(og[:, 1] == 7.0)                                       # head 1 not listed: untouched
    assert np.all(og[:, 2] == 0.0)                                       # empty lists: zeros
    dense3, _, _ = oracle.dense_rows(hq[:, 3], hk[:, 1], hv[:, 1], B)
    e = _err(og[:, 3], dense3)
    assert e[0] <= OUT_MAX and e[1] <= OUT_MEAN                          # all-ones pattern == dense attention
    ref0 = oracle.masked_rows(hq[:, 0], hk[:, 0], hv[:, 0], B, idx[1], cnt[1])
    e = _err(og[:, 0], ref0)
    assert e[0] <= OUT_MAX and e[1] <= OUT_MEAN
    # the dense call on the same head gives the same bits as the all-ones sparse call? not required; but
    # a head outside every cluster must come out dense in the fused call
    o2 = torch.zeros_like(q)
    sc = torch.empty((1, 1, nqb, nqb), dtype=torch.float32, device="cuda")
    ix = torch.empty((1, 1, nqb, nqb), dtype=torch.int32, device="cuda")
    ct = torch.empty((1, 1, nqb), dtype=torch.int32, device="cuda")
    sp.sp_prefill_layer(shape, q, k, v, [0, 0, -1, -1], [0], 0.9, o2, sc, ix, ct, ws)
    torch.cuda.synchronize()
    o2h = o2.float().cpu().numpy()[0]
    for h in (2, 3):
        dn, _, _ = oracle.dense_rows(hq[:, h], hk[:, h // 2], hv[:, h // 2], B)
        e = _err(o2h[:, h], dn)
        assert e[0] <= OUT_MAX and e[1] <= OUT_MEAN
    m1 = oracle.masked_rows(hq[:, 1], hk[:, 0], hv[:, 0], B, ix.cpu().numpy()[0, 0], ct.cpu().numpy()[0, 0])
    e = _err(o2h[:, 1], m1)
    assert e[0] <= OUT_MAX and e[1] <= OUT_MEAN


@pytest.mark.parametrize("nkb,n_maps", [(1, 2), (7, 3), (64, 2), (200, 2), (256, 1), (257, 2), (1000, 1), (1024, 1),
                                        (1500, 1), (4096, 1)])
def test_mask_builder_all_paths_bit_exact(nkb, n_maps):
    """Random, tied, one-hot, zero, NaN, negative and > 1 scores; every register / re-read code path."""
    import torch
    import oracle
    import paper_2505_19578_amd as sp
    rng = np.random.default_rng(nkb)
    sc = np.tril(rng.random((n_maps, nkb, nkb)).astype(np.float32) ** 8)
    sc /= np.maximum(sc.sum(-1, keepdims=True), 1e-30)
    sc = sc.astype(np.float32)
    if nkb >= 7:
        sc[0, 3, :4] = 0.25                       # exact four-way tie
        sc[0, 4, :5] = 0.0                        # all-zero row
        sc[0, 5, :6] = [0, 0, 1.0, 0, 0, 0]       # one-hot
        sc[0, 6, :7] = [np.nan, -1.0, 2.0, 0.125, 0.125, np.inf, 0.0625]
    if nkb >= 200:
        sc[-1, 150, :151] = np.float32(1.0 / 256)  # 151-way tie
    for gamma in (0.5, 0.9, 1.0):
        dsc = torch.from_numpy(sc).cuda()
        idx = torch.empty((n_maps, nkb, nkb), dtype=torch.int32, device="cuda")
        cnt = torch.empty((n_maps, nkb), dtype=torch.int32, device="cuda")
        bm = torch.empty((n_maps, nkb, (nkb + 63) // 64), dtype=torch.int64, device="cuda")
        sp.sp_build_block_mask(dsc, n_maps, nkb, nkb, gamma, idx, cnt, bm)
        torch.cuda.synchronize()
        idx_h, cnt_h, bm_h = idx.cpu().numpy(), cnt.cpu().numpy(), bm.cpu().numpy().view(np.uint64)
        for mm in range(n_maps):
            i2, c2, _ = oracle.build_mask_rows(sc[mm], gamma)
            assert np.array_equal(c2, cnt_h[mm]), (nkb, gamma, mm)
            assert np.array_equal(i2, idx_h[mm]), (nkb, gamma, mm)
        # bitmask == the lists, bit j % 64 of word j / 64
        rows = rng.integers(0, nkb, size=min(nkb, 16))
        for i in rows:
            bits = np.zeros(((nkb + 63) // 64) * 64, dtype=bool)
            bits[idx_h[0, i, : cnt_h[0, i]]] = True
            words = np.packbits(bits.reshape(-1, 64)[:, ::-1], axis=1).view(">u8").reshape(-1)
            assert np.array_equal(words.astype(np.uint64), bm_h[0, i])


def test_run_to_run_determinism():
    import torch
    import paper_2505_19578_amd as sp
    from synth import CONFIGS, make_layer
    L = make_layer(CONFIGS["llama8b_32k"], seq=4096)
    cfg = L["cfg"]
    q, k, v = (_dev(L[x]).unsqueeze(0) for x in "qkv")
    nqb, C = cfg.seq // cfg.block, cfg.n_clusters
    shape = sp.shape_of(q, k, None, cfg.block)
    ws = torch.empty(sp.sp_workspace_bytes(shape, C), dtype=torch.uint8, device="cuda")
    outs = []
    for _ in range(3):
        o = torch.zeros_like(q)
        sc = torch.empty((1, C, nqb, nqb), dtype=torch.float32, device="cuda")
        idx = torch.empty((1, C, nqb, nqb), dtype=torch.int32, device="cuda")
        cnt = torch.empty((1, C, nqb), dtype=torch.int32, device="cuda")
        ws.random_(0, 255)                                  # stale workspace contents must not matter
        sp.sp_prefill_layer(shape, q, k, v, L["head_to_cluster"], L["pivot_heads"], cfg.gamma, o, sc, idx, cnt, ws)
        torch.cuda.synchronize()
        outs.append((o.view(torch.int16).clone(), sc.clone(), idx.clone(), cnt.clone()))
    for a in outs[1:]:
        for x, y in zip(outs[0], a):
            assert torch.equal(x, y)


def test_pattern_calls_batch2_interleaved_qkv_and_custom_scale():
    """The printed score map, Alg. 3's gate and Alg. 5's search on a batch of two prompts whose Q, K, V are
    slices of one interleaved tensor (non-trivial strides), with a caller-given softmax scale."""
    import torch
    import oracle
    import paper_2505_19578_amd as sp
    from synth import random_qkv
    N, Hq, Hkv, d, B, scale = 640, 4, 2, 64, 64, 0.2
    packs = []
    for bb in range(2):
        q, k, v = random_qkv(70 + bb, N, Hq, Hkv, d, 1.5)
        packs.append(np.concatenate([q, k, v], axis=1))
    qkv = _dev(np.stack(packs))                        # [2][N][Hq+2Hkv][d]
    q, k = qkv[:, :, :Hq], qkv[:, :, Hq:Hq + Hkv]
    shape = sp.shape_of(q, k, None, B, softmax_scale=scale)
    nqb = N // B
    heads = [2, 0, 3]
    ws = torch.empty(sp.sp_score_workspace_bytes(shape, len(heads)), dtype=torch.uint8, device="cuda")
    sc = torch.full((2, len(heads), nqb, nqb), -1.0, dtype=torch.float32, device="cuda")
    sp.sp_block_mean_logit_scores(shape, q, k, heads, sc, ws)
    a_hat = torch.empty((2, len(heads), nqb), dtype=torch.float32, device="cuda")
    dist = torch.empty((2, len(heads), 2), dtype=torch.float32, device="cuda")
    pat = torch.full((2, Hq), -7, dtype=torch.int32, device="cuda")
    sp.sp_determine_pattern(shape, q, k, heads, [0, 0, -1], [5, 6, 7], 10.0, 10.0, a_hat, dist, pat, ws)
    wv = torch.empty(sp.sp_vs_workspace_bytes(shape, len(heads)), dtype=torch.uint8, device="cuda")
    sums = torch.empty((2, len(heads), 2, N), dtype=torch.float32, device="cuda")
    vidx = torch.empty((2, len(heads), nqb, nqb), dtype=torch.int32, device="cuda")
    vcnt = torch.empty((2, len(heads), nqb), dtype=torch.int32, device="cuda")
    sp.sp_search_vertical_slash(shape, q, k, heads, 0.6, True, sums, vidx, vcnt, wv)
    torch.cuda.synchronize()
    assert list(pat[0].cpu().numpy()) == [6, -7, 5, 7] and list(pat[1].cpu().numpy()) == [6, -7, 5, 7]
    for bb in range(2):
        hq, hk = _f32(packs[bb][:, :Hq]), _f32(packs[bb][:, Hq:Hq + Hkv])
        est = []
        for n, h in enumerate(heads):
            want = oracle.softmax_rows(oracle.mean_logit_rows(hq[:, h], hk[:, h // 2], B, scale=scale))
            got = sc[bb, n].cpu().numpy()
            assert np.abs(got - want).max() <= 1e-7 + 1e-4 * want.max()
            assert np.abs(a_hat[bb, n].cpu().numpy() - want[-1]).max() <= 1e-7 + 1e-4 * want[-1].max()
            est.append(want[-1])
            a_v, a_s = oracle.vertical_slash_sums(hq[:, h], hk[:, h // 2], B, scale=scale)
            s_h = sums[bb, n].cpu().numpy()
            assert np.abs(s_h[0] - a_v).max() <= 1e-8 + 1e-4 * a_v.max() and np.abs(s_h[1] - a_s).max() <= 1e-8 + 1e-4 * a_s.max()
            kv, _ = oracle.select_cumulative(s_h[0], 0.6)
            ks, _ = oracle.select_cumulative(s_h[1], 0.6)
            i2, c2 = oracle.vs_block_lists(kv, ks, B, True)
            assert np.array_equal(i2, vidx[bb, n].cpu().numpy()) and np.array_equal(c2, vcnt[bb, n].cpu().numpy())
        d_h = dist[bb].cpu().numpy()
        u = np.full(nqb, 1.0 / nqb, dtype=np.float32)
        for n in range(len(heads)):
            assert abs(d_h[n, 0] - oracle.js_distance(est[n], u)) <= 2e-5
        assert abs(d_h[1, 1] - oracle.js_distance(est[1], est[0])) <= 2e-5 and d_h[0, 1] == 0.0 and d_h[2, 1] == 0.0


@pytest.mark.parametrize("N,B,d", [(128, 128, 128), (128, 64, 64), (384, 128, 64), (192, 64, 64), (320, 64, 128)])
def test_shortest_sequences_through_every_layer_call(N, B, d):
    """One, two, three and five query blocks (two lengths are multiples of block = 64 but not of 128): the printed construction, the gate, the dictionary over two layers and
    the vertical-slash fallback all against the oracle's own runs (every row, every head)."""
    import torch
    import oracle
    import paper_2505_19578_amd as sp
    from synth import random_qkv
    Hq, Hkv, gamma = 4, 2, 0.8
    nqb = N // B
    h2c, piv = [0, 0, 1, 1], [0, 2]
    layers = [random_qkv(90 + l, N, Hq, Hkv, d, 1.5) for l in range(2)]
    dev = [[_dev(x[None]) for x in L] for L in layers]
    host = [[_f32(x) for x in L] for L in layers]
    q, k, v = dev[0]
    shape = sp.shape_of(q, k, None, B)
    ws = torch.empty(sp.sp_workspace_bytes(shape, 2) + sp.sp_vs_workspace_bytes(shape, Hq), dtype=torch.uint8, device="cuda")
    sc = torch.empty((1, 2, nqb, nqb), dtype=torch.float32, device="cuda")
    idx = torch.empty((1, 2, nqb, nqb), dtype=torch.int32, device="cuda")
    cnt = torch.empty((1, 2, nqb), dtype=torch.int32, device="cuda")

    def check_out(o, ref_o, what):
        emax, emean = _err(o[0].float().cpu().numpy(), ref_o)
        assert emax <= OUT_MAX and emean <= OUT_MEAN, f"{what}: {emax} / {emean}"

    # printed construction (mean-logit scores, one selection over the map)
    o = torch.zeros_like(q)
    sp.sp_prefill_layer_modes(shape, q, k, v, h2c, piv, gamma, 1, 1, o, sc, idx, cnt, ws)
    torch.cuda.synchronize()
    idx_h, cnt_h = idx[0].cpu().numpy(), cnt[0].cpu().numpy()
    ref = oracle.prefill_layer(*host[0], B, h2c, piv, gamma, masks=(idx_h, cnt_h), paper_pattern=True)
    assert np.abs(sc[0].cpu().numpy() - ref["scores"]).max() <= 1e-6 + 1e-4 * ref["scores"].max()
    for c in range(2):
        i2, c2, _ = oracle.build_mask_global(sc[0, c].cpu().numpy(), gamma, True)
        assert np.array_equal(i2, idx_h[c]) and np.array_equal(c2, cnt_h[c])
    check_out(o, ref["o"], "printed construction")
    # dictionary over two layers, open gate, then with everything sent to the vertical-slash fallback
    for delta, fallback in ((10.0, sp.SP_FALLBACK_DENSE), (0.0, sp.SP_FALLBACK_VERTICAL_SLASH)):
        valid = torch.zeros((1, 2), dtype=torch.int32, device="cuda")
        a_t = torch.zeros((1, 2, nqb), dtype=torch.float32, device="cuda")
        didx = torch.full((1, 2, nqb, nqb), -9, dtype=torch.int32, device="cuda")
        dcnt = torch.full((1, 2, nqb), -9, dtype=torch.int32, device="cuda")
        pd = sp.pattern_dict_of(valid, a_t, didx, dcnt)
        vidx = torch.full((1, Hq, nqb, nqb), -3, dtype=torch.int32, device="cuda")
        vcnt = torch.full((1, Hq, nqb), -3, dtype=torch.int32, device="cuda")
        for l in range(2):
            ql, kl, vl = dev[l]
            o = torch.zeros_like(ql)
            role = torch.full((1, Hq), -7, dtype=torch.int32, device="cuda")
            a_hat = torch.empty((1, Hq, nqb), dtype=torch.float32, device="cuda")
            dist = torch.empty((1, Hq, 2), dtype=torch.float32, device="cuda")
            sp.sp_prefill_layer_dict(shape, ql, kl, vl, h2c, gamma, delta, 10.0, 0, 0, pd, o, sc, role, a_hat, dist, ws,
                                     fallback_mode=fallback, vs_idx=vidx, vs_cnt=vcnt)
            torch.cuda.synchronize()
            role_h = role[0].cpu().numpy()
            want_roles = ([-2, 0, -2, 1] if l == 0 else [0, 0, 1, 1]) if delta > 0 else [-1] * 4
            assert list(role_h) == want_roles, (l, delta, list(role_h))
            hq, hk, hv = host[l]
            for h in range(Hq):
                g = h // 2
                if role_h[h] >= 0:
                    c = int(role_h[h])
                    ref_o = oracle.masked_rows(hq[:, h], hk[:, g], hv[:, g], B, didx[0, c].cpu().numpy(), dcnt[0, c].cpu().numpy())
                elif role_h[h] == -1 and fallback == sp.SP_FALLBACK_VERTICAL_SLASH:
                    ref_o = oracle.masked_rows(hq[:, h], hk[:, g], hv[:, g], B, vidx[0, h].cpu().numpy(), vcnt[0, h].cpu().numpy())
                    assert np.all(vcnt[0, h].cpu().numpy() >= 1)
                else:
                    ref_o, _, _ = oracle.dense_rows(hq[:, h], hk[:, g], hv[:, g], B, want_scores=False)
                emax, emean = _err(o[0, :, h].float().cpu().numpy(), ref_o)
                assert emax <= OUT_MAX and emean <= OUT_MEAN, f"layer {l} head {h} role {role_h[h]}: {emax} / {emean}"


def test_fused_layer_without_returned_scores():
    """block_scores = NULL: the score maps stay in the workspace; lists, counts and outputs are the same bits."""
    import torch
    import paper_2505_19578_amd as sp
    from synth import CONFIGS, make_layer
    from tests.gpu_util import to_dev, alloc_layer
    L = make_layer(CONFIGS["llama8b_32k"], seq=1024)
    cfg = L["cfg"]
    q, k, v = (to_dev(L[x]) for x in "qkv")
    C = cfg.n_clusters
    shape, o, ws, scores, kb_idx, kb_cnt = alloc_layer(sp, cfg, q, k, C)
    sp.sp_prefill_layer(shape, q, k, v, L["head_to_cluster"], L["pivot_heads"], cfg.gamma, o, scores, kb_idx, kb_cnt, ws)
    o2, idx2, cnt2 = torch.zeros_like(o), torch.full_like(kb_idx, -5), torch.full_like(kb_cnt, -5)
    sp.sp_prefill_layer(shape, q, k, v, L["head_to_cluster"], L["pivot_heads"], cfg.gamma, o2, None, idx2, cnt2, ws)
    torch.cuda.synchronize()
    assert torch.equal(idx2, kb_idx) and torch.equal(cnt2, kb_cnt)
    assert torch.equal(o2.view(torch.int16), o.view(torch.int16))
