"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs.  Bars: block scores max-abs <= 1e-3 and row sums within
1e-3; key-block lists and counts bit-exact when the oracle's Alg. 2 is fed the
GPU's own score buffer; outputs max-abs <= 2e-2 and mean-abs <= 2e-3 against the
oracle run with the GPU's own pattern."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

OUT_MAX, OUT_MEAN, SC_MAX = 2e-2, 2e-3, 1e-3


class _LazyHost:
    """fp32 views of one head at a time (keeps host memory small at 128K)."""

    def __init__(self, L):
        self.L = L

    def head(self, x, h):
        from synth import bf16_bits_to_f32
        return bf16_bits_to_f32(self.L[x][:, h])


def _setup(name, seq=None, layer=0):
    import paper_2505_19578_amd as sp
    from synth import CONFIGS, make_layer, bf16_bits_to_f32
    from tests.gpu_util import to_dev
    L = make_layer(CONFIGS[name], layer=layer, seq=seq)
    cfg = L["cfg"]
    dev = {x: to_dev(L[x]) for x in "qkv"}
    host = _LazyHost(L)
    return sp, cfg, L, dev, host


def _check_layer(sp, cfg, L, dev, host, rows, check_heads=None, label="", stages=True, bufs=None):
    """Run the fused call and its three stages; compare on the listed query-block rows."""
    import torch
    import oracle
    from tests.gpu_util import alloc_layer, bf16_dev_to_f32, err_stats
    B, G = cfg.block, cfg.group
    nqb = cfg.seq // B
    h2c, piv = L["head_to_cluster"], L["pivot_heads"]
    C = len(piv)
    q, k, v = dev["q"], dev["k"], dev["v"]
    if bufs is None:
        shape, o, ws, scores, kb_idx, kb_cnt = alloc_layer(sp, cfg, q, k, C)
        o.zero_()
        print(f"[{label}] fused call N={cfg.seq} Hq={cfg.n_q_heads} C={C}", flush=True)
        sp.sp_prefill_layer(shape, q, k, v, h2c, piv, cfg.gamma, o, scores, kb_idx, kb_cnt, ws)
        torch.cuda.synchronize()
    else:       # results of a fused call the caller already ran
        shape, o, ws, scores, kb_idx, kb_cnt = bufs
    o_h = bf16_dev_to_f32(o)[0]
    sc_h = scores.cpu().numpy()[0]
    idx_h = kb_idx.cpu().numpy()[0]
    cnt_h = kb_cnt.cpu().numpy()[0]
    rows = np.asarray(rows, dtype=np.int32)
    sel_t = np.concatenate([np.arange(i * B, (i + 1) * B) for i in rows])

    # -- stage 2 everywhere: lists bit-exact given the GPU's scores (all rows, all clusters)
    for c in range(C):
        idx_o, cnt_o, _ = oracle.build_mask_rows(sc_h[c], cfg.gamma)
        assert np.array_equal(cnt_o, cnt_h[c]), f"cluster {c}: counts differ"
        assert np.array_equal(idx_o, idx_h[c]), f"cluster {c}: lists differ"
    np.testing.assert_allclose(sc_h.sum(axis=-1), 1.0, atol=SC_MAX)
    assert np.all(np.triu(sc_h, 1) == 0)

    heads = range(cfg.n_q_heads) if check_heads is None else check_heads
    pivset = {int(p) for p in piv}
    worst = [0.0, 0.0, 0.0]
    jac = []
    for h in heads:
        g = h // G
        c = int(h2c[h])
        if h in pivset:
            o_o, sc_o, _ = oracle.dense_rows(host.head("q", h), host.head("k", g), host.head("v", g), B, rows)
            smax, _ = err_stats(sc_h[c][rows], sc_o)
            worst[2] = max(worst[2], smax)
            assert smax <= SC_MAX, f"head {h}: block scores max-abs {smax}"
            idx_o, cnt_o, _ = oracle.build_mask_rows(sc_o, cfg.gamma, rows)
            for r, i in enumerate(rows):
                a, b = set(idx_o[r, :cnt_o[r]]), set(idx_h[c][i, :cnt_h[c][i]])
                jac.append(len(a & b) / len(a | b))
        else:
            o_o = oracle.masked_rows(host.head("q", h), host.head("k", g), host.head("v", g), B,
                                     idx_h[c][rows], cnt_h[c][rows], rows)
        emax, emean = err_stats(o_h[sel_t, h], o_o)
        worst[0], worst[1] = max(worst[0], emax), max(worst[1], emean)
        assert emax <= OUT_MAX and emean <= OUT_MEAN, f"head {h}: out max-abs {emax}, mean-abs {emean}"
        rms = float(np.sqrt(np.mean(o_o.astype(np.float64) ** 2)))
        assert rms > 0.05, "outputs too small for the absolute tolerance to mean anything"
    dens = float(cnt_h.sum() / (C * nqb * (nqb + 1) / 2))
    print(f"[{label}] out max {worst[0]:.2e} mean {worst[1]:.2e} scores max {worst[2]:.2e} "
          f"jaccard(min) {min(jac) if jac else 1:.3f} density {dens:.3f}", flush=True)

    if not stages:
        return dens
    # -- the three stage calls reproduce the fused call bit for bit
    o2 = torch.zeros_like(o)
    sc2 = torch.empty_like(scores)
    idx2 = torch.empty_like(kb_idx)
    cnt2 = torch.empty_like(kb_cnt)
    sp.sp_dense_attn_with_block_scores(shape, q, k, v, list(piv), o2, sc2, ws)
    sp.sp_build_block_mask(sc2, C, nqb, nqb, cfg.gamma, idx2, cnt2)
    others = [h for h in range(cfg.n_q_heads) if h not in pivset]
    sp.sp_block_sparse_attn(shape, q, k, v, others, [int(h2c[h]) for h in others], idx2, cnt2, C, o2, ws)
    torch.cuda.synchronize()
    assert torch.equal(sc2, scores) and torch.equal(idx2, kb_idx) and torch.equal(cnt2, kb_cnt)
    assert torch.equal(o2.view(torch.int16), o.view(torch.int16))
    return dens


def test_tiny_config_full():
    sp, cfg, L, dev, host = _setup("tiny")
    _check_layer(sp, cfg, L, dev, host, np.arange(cfg.seq // cfg.block), label="tiny")


def test_d128_b128_2k_full():
    sp, cfg, L, dev, host = _setup("llama8b_32k", seq=2048)
    _check_layer(sp, cfg, L, dev, host, np.arange(cfg.seq // cfg.block), label="llama8b@2k")


def test_qwen_shape_permuted_clusters_4k():
    sp, cfg, L, dev, host = _setup("qwen7b_128k", seq=4096)
    _check_layer(sp, cfg, L, dev, host, np.arange(cfg.seq // cfg.block), label="qwen7b@4k")


@pytest.mark.parametrize("d,B", [(128, 64), (64, 128)])
def test_mixed_dim_block(d, B):
    """The two remaining (head_dim, block) instantiations, on plain N(0,1) inputs."""
    import torch
    import oracle
    import paper_2505_19578_amd as sp
    from synth import random_qkv, bf16_bits_to_f32
    from tests.gpu_util import to_dev, bf16_dev_to_f32, err_stats
    N, Hq, Hkv = 1024, 4, 2
    qb, kb, vb = random_qkv(11, N, Hq, Hkv, d)
    q, k, v = to_dev(qb), to_dev(kb), to_dev(vb)
    hq, hk, hv = (bf16_bits_to_f32(x) for x in (qb, kb, vb))
    nqb = N // B
    shape = sp.shape_of(q, k, None, B)
    o = torch.zeros_like(q)
    ws = torch.empty(sp.sp_workspace_bytes(shape, 2), dtype=torch.uint8, device="cuda")
    sc = torch.empty((1, 2, nqb, nqb), dtype=torch.float32, device="cuda")
    idx = torch.empty((1, 2, nqb, nqb), dtype=torch.int32, device="cuda")
    cnt = torch.empty((1, 2, nqb), dtype=torch.int32, device="cuda")
    sp.sp_prefill_layer(shape, q, k, v, [0, 0, 1, 1], [0, 2], 0.8, o, sc, idx, cnt, ws)
    torch.cuda.synchronize()
    o_h, sc_h, idx_h, cnt_h = bf16_dev_to_f32(o)[0], sc.cpu().numpy()[0], idx.cpu().numpy()[0], cnt.cpu().numpy()[0]
    for c, p in enumerate([0, 2]):
        o_o, sc_o, _ = oracle.dense_rows(hq[:, p], hk[:, p // 2], hv[:, p // 2], B)
        assert err_stats(sc_h[c], sc_o)[0] <= SC_MAX
        e = err_stats(o_h[:, p], o_o)
        assert e[0] <= OUT_MAX and e[1] <= OUT_MEAN
        idx_o, cnt_o, _ = oracle.build_mask_rows(sc_h[c], 0.8)
        assert np.array_equal(idx_o, idx_h[c]) and np.array_equal(cnt_o, cnt_h[c])
        hh = p + 1
        o_m = oracle.masked_rows(hq[:, hh], hk[:, hh // 2], hv[:, hh // 2], B, idx_h[c], cnt_h[c])
        e = err_stats(o_h[:, hh], o_m)
        assert e[0] <= OUT_MAX and e[1] <= OUT_MEAN
