"""GPU parity for attention over the token-level vertical-slash pattern (Alg. 5's mask under Sec. 5.1's
A(Q,K,V,M)): sp_vertical_slash_attn and the token-level fallback of sp_prefill_layer_dict against the CPU oracle.

The kept keys / offsets the call reports must be, bit for bit, the oracle's selection fed the GPU's own sums (the
sums themselves are held to the search test's bar there); outputs: max-abs 2e-2 / mean-abs 2e-3 against the
oracle's token-level attention run with the GPU's kept sets; the reported pair count is exact."""
import numpy as np
import pytest

from tests.test_gpu_parity import OUT_MAX, OUT_MEAN, _LazyHost

pytestmark = pytest.mark.gpu


def _bits_to_keep(words, N):
    return np.unpackbits(np.ascontiguousarray(words).view(np.uint8), bitorder="little")[:N].astype(np.uint8)


def _run(sp, q, k, v, B, heads, gamma, forced):
    import torch
    shape = sp.shape_of(q, k, None, B)
    N, n = q.shape[1], len(heads)
    ws = torch.empty(sp.sp_vs_token_workspace_bytes(shape, n), dtype=torch.uint8, device="cuda")
    o = torch.zeros_like(q)
    bits = torch.zeros((1, n, 2, N // 64), dtype=torch.int64, device="cuda")
    pairs = torch.full((1, n), -1, dtype=torch.int64, device="cuda")
    sp.sp_vertical_slash_attn(shape, q, k, v, heads, gamma, forced, o, bits, pairs, ws)
    torch.cuda.synchronize()
    return shape, o, bits.cpu().numpy()[0].view(np.uint64), pairs.cpu().numpy()[0]


def _pair_count(keep_v, keep_s, B, forced):
    N = len(keep_v)
    total = 0
    cs = np.concatenate([[0], np.cumsum(keep_s.astype(np.int64))])
    for t in range(N):
        s = np.arange(t + 1)
        allow = keep_v[:t + 1].astype(bool) | keep_s[t - s].astype(bool)
        if forced:
            allow |= (s // B == 0) | (s // B == t // B)
        total += int(allow.sum())
    return total


@pytest.mark.parametrize("d,B,N,forced,gamma", [(128, 128, 1024, True, 0.5), (128, 128, 1024, False, 0.5),
                                                (128, 64, 576, True, 0.5), (64, 128, 768, True, 0.5),
                                                (64, 64, 448, False, 0.5),
                                                # nearly everything kept (long runs of full gathered items, every
                                                # band), and nearly nothing
                                                (128, 128, 1536, True, 0.98), (64, 64, 640, False, 0.98),
                                                (128, 128, 1024, False, 0.02), (128, 64, 576, True, 0.02)])
def test_token_attention_random_inputs(d, B, N, forced, gamma):
    import torch
    import oracle
    import paper_2505_19578_amd as sp
    from synth import random_qkv, bf16_bits_to_f32
    from tests.gpu_util import to_dev, err_stats
    qb, kb, _ = random_qkv(71, N, 4, 2, d, 2.0)
    _, _, vb = random_qkv(72, N, 4, 2, d, 1.0)     # |V| < 8: output rounding alone stays under the absolute bar
    q, k, v = to_dev(qb), to_dev(kb), to_dev(vb)
    hq, hk, hv = (bf16_bits_to_f32(x) for x in (qb, kb, vb))
    heads = [0, 3, 2]
    print(f"[vs token] d{d} B{B} N{N} forced {forced} gamma {gamma}", flush=True)
    shape, o, bits, pairs = _run(sp, q, k, v, B, heads, gamma, forced)
    # the search's own sums on the same inputs (bit-identical run to run): what the kept sets must follow from
    ws = torch.empty(sp.sp_vs_workspace_bytes(shape, len(heads)), dtype=torch.uint8, device="cuda")
    sums = torch.empty((1, len(heads), 2, N), dtype=torch.float32, device="cuda")
    nkb = N // B
    idx = torch.empty((1, len(heads), nkb, nkb), dtype=torch.int32, device="cuda")
    cnt = torch.empty((1, len(heads), nkb), dtype=torch.int32, device="cuda")
    sp.sp_search_vertical_slash(shape, q, k, heads, gamma, forced, sums, idx, cnt, ws)
    torch.cuda.synchronize()
    sums_h = sums.cpu().numpy()[0]
    o_h = o.float().cpu().numpy()[0]
    for n, h in enumerate(heads):
        keep_v, keep_s = _bits_to_keep(bits[n, 0], N), _bits_to_keep(bits[n, 1], N)
        kv_o, _ = oracle.select_cumulative(sums_h[n, 0], gamma)
        ks_o, _ = oracle.select_cumulative(sums_h[n, 1], gamma)
        assert np.array_equal(keep_v, kv_o) and np.array_equal(keep_s, ks_o), f"head {h}: kept sets differ"
        assert 0 < keep_v.sum() < N and 0 < keep_s.sum() < N
        ref = oracle.vs_token_rows(hq[:, h], hk[:, h // 2], hv[:, h // 2], B, keep_v, keep_s, forced)
        emax, emean = err_stats(o_h[:, h], ref)
        assert emax <= OUT_MAX and emean <= OUT_MEAN, f"head {h}: {emax} / {emean}"
        assert int(pairs[n]) == _pair_count(keep_v, keep_s, B, forced), f"head {h}: pair count"
    assert np.all(o_h[:, 1] == 0)          # a head that was not listed is not written


def test_token_attention_structured_2k_and_dictionary_fallback():
    """The structured workload at 2K: the stand-alone call on every head, then one dictionary layer in which every
    head falls back (delta = 0) to the token-level pattern: same bits as the stand-alone call."""
    import torch
    import oracle
    import paper_2505_19578_amd as sp
    from synth import CONFIGS, make_layer
    from tests.gpu_util import to_dev, err_stats
    L = make_layer(CONFIGS["llama8b_32k"], seq=2048)
    cfg = L["cfg"]
    B, Hq, G, N = cfg.block, cfg.n_q_heads, cfg.group, cfg.seq
    q, k, v = (to_dev(L[x]) for x in "qkv")
    host = _LazyHost(L)
    heads = list(range(Hq))
    shape, o, bits, pairs = _run(sp, q, k, v, B, heads, cfg.gamma, True)
    o_h = o.float().cpu().numpy()[0]
    dens = []
    for h in [0, 5, 14, 31]:
        keep_v, keep_s = _bits_to_keep(bits[h, 0], N), _bits_to_keep(bits[h, 1], N)
        ref = oracle.vs_token_rows(host.head("q", h), host.head("k", h // G), host.head("v", h // G), B, keep_v, keep_s, True)
        emax, emean = err_stats(o_h[:, h], ref)
        assert emax <= OUT_MAX and emean <= OUT_MEAN, f"head {h}: {emax} / {emean}"
        dens.append(pairs[h] / (N * (N + 1) / 2))
    print(f"[vs token] llama8b@2k kept-pair fraction of sampled heads: {np.round(dens, 3)}", flush=True)
    nqb = N // B
    C = cfg.n_clusters
    valid = torch.zeros((1, C), dtype=torch.int32, device="cuda")
    a_t = torch.zeros((1, C, nqb), dtype=torch.float32, device="cuda")
    didx = torch.full((1, C, nqb, nqb), -9, dtype=torch.int32, device="cuda")
    dcnt = torch.full((1, C, nqb), -9, dtype=torch.int32, device="cuda")
    pd = sp.pattern_dict_of(valid, a_t, didx, dcnt)
    ws = torch.empty(sp.sp_workspace_bytes(shape, C) + sp.sp_vs_token_workspace_bytes(shape, Hq), dtype=torch.uint8, device="cuda")
    sc = torch.empty((1, C, nqb, nqb), dtype=torch.float32, device="cuda")
    role = torch.full((1, Hq), -7, dtype=torch.int32, device="cuda")
    a_hat = torch.empty((1, Hq, nqb), dtype=torch.float32, device="cuda")
    dist = torch.empty((1, Hq, 2), dtype=torch.float32, device="cuda")
    o2 = torch.zeros_like(q)
    sp.sp_prefill_layer_dict(shape, q, k, v, [int(c) for c in L["head_to_cluster"]], cfg.gamma, 0.0, 0.2, 0, 0, pd, o2,
                             sc, role, a_hat, dist, ws, fallback_mode=sp.SP_FALLBACK_VERTICAL_SLASH_TOKEN)
    torch.cuda.synchronize()
    assert np.all(role.cpu().numpy() == -1)
    assert torch.equal(o2.view(torch.int16), o.view(torch.int16))


def test_token_attention_llama8b_128k_sampled_rows():
    """Full size: two heads, outputs on sampled query-block rows, kept-pair fraction next to the block superset's."""
    import torch
    import oracle
    import paper_2505_19578_amd as sp
    from synth import CONFIGS, make_layer
    from tests.gpu_util import to_dev, err_stats
    from tests.test_gpu_full_size import _sample_rows
    L = make_layer(CONFIGS["llama8b_128k"])
    cfg = L["cfg"]
    B, G, N = cfg.block, cfg.group, cfg.seq
    q, k, v = (to_dev(L[x]) for x in "qkv")
    host = _LazyHost(L)
    heads = [1, 22]
    shape, o, bits, pairs = _run(sp, q, k, v, B, heads, cfg.gamma, True)
    o_h = o.float().cpu().numpy()[0]
    rows = _sample_rows(cfg.nqb, 77, extra=1)
    sel_t = np.concatenate([np.arange(i * B, (i + 1) * B) for i in rows])
    for n, h in enumerate(heads):
        keep_v, keep_s = _bits_to_keep(bits[n, 0], N), _bits_to_keep(bits[n, 1], N)
        ref = oracle.vs_token_rows(host.head("q", h), host.head("k", h // G), host.head("v", h // G), B, keep_v, keep_s,
                                   True, rows=rows)
        emax, emean = err_stats(o_h[sel_t, h], ref)
        assert emax <= OUT_MAX and emean <= OUT_MEAN, f"head {h}: {emax} / {emean}"
        idx_b, cnt_b = oracle.vs_block_lists(keep_v, keep_s, B, True)
        frac_tok = pairs[n] / (N * (N + 1) / 2)
        frac_blk = cnt_b.sum() / (cfg.nqb * (cfg.nqb + 1) / 2)
        print(f"[vs token] cfg3 head {h}: kept keys {int(keep_v.sum())}, kept offsets {int(keep_s.sum())}, "
              f"pairs {frac_tok:.4f} of causal, block superset {frac_blk:.4f} of causal blocks", flush=True)
        assert frac_tok <= frac_blk + 1e-9
