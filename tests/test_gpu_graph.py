"""The layer calls enqueue kernels only (no allocation, no memset node, no host synchronisation, every
decision that depends on the data stays on the device), so a whole stack of layers can be captured
into one HIP graph.  Each replay must reproduce the eager results bit for bit, also with other work
and synchronisations between replays."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _layers(n, seq):
    from synth import CONFIGS, make_layer
    from tests.gpu_util import to_dev
    Ls = [make_layer(CONFIGS["tiny"], layer=l, seq=seq, structure_layer=0) for l in range(n)]
    return Ls, [{x: to_dev(L[x]) for x in "qkv"} for L in Ls]


def test_fused_layer_call_in_a_graph():
    import torch
    import paper_2505_19578_amd as sp
    Ls, dev = _layers(1, 1024)
    cfg = Ls[0]["cfg"]
    q, k, v = dev[0]["q"], dev[0]["k"], dev[0]["v"]
    nqb, C = cfg.seq // cfg.block, cfg.n_clusters
    h2c, piv = [int(x) for x in Ls[0]["head_to_cluster"]], [int(x) for x in Ls[0]["pivot_heads"]]
    shape = sp.shape_of(q, k, None, cfg.block)
    ws = torch.empty(sp.sp_workspace_bytes(shape, C), dtype=torch.uint8, device="cuda")
    bufs = lambda: (torch.zeros_like(q), torch.zeros((1, C, nqb, nqb), dtype=torch.float32, device="cuda"),
                    torch.zeros((1, C, nqb, nqb), dtype=torch.int32, device="cuda"),
                    torch.zeros((1, C, nqb), dtype=torch.int32, device="cuda"))
    o_e, sc_e, idx_e, cnt_e = bufs()
    sp.sp_prefill_layer(shape, q, k, v, h2c, piv, cfg.gamma, o_e, sc_e, idx_e, cnt_e, ws)
    torch.cuda.synchronize()
    o_g, sc_g, idx_g, cnt_g = bufs()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):       # warm-up on the capture stream, as torch's capture protocol asks
        sp.sp_prefill_layer(shape, q, k, v, h2c, piv, cfg.gamma, o_g, sc_g, idx_g, cnt_g, ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        sp.sp_prefill_layer(shape, q, k, v, h2c, piv, cfg.gamma, o_g, sc_g, idx_g, cnt_g, ws)
    for rep in range(3):
        for t in (o_g, sc_g, idx_g, cnt_g):
            t.fill_(7)
        print(f"[graph] fused layer replay {rep}", flush=True)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(o_g, o_e) and torch.equal(sc_g, sc_e) and torch.equal(idx_g, idx_e) and torch.equal(cnt_g, cnt_e)
        junk = torch.randn(1 << 16, device="cuda").sum().item()    # unrelated eager work and a sync in between
        assert np.isfinite(junk)


@pytest.mark.parametrize("token_level", [False, True])
def test_three_dictionary_layers_in_one_graph(token_level):
    """Pivot election, sharing and the vertical-slash fallback (block superset or token level) are decided on the
    device: three layers of one prompt, dictionary reset included, replay as one graph."""
    import torch
    import paper_2505_19578_amd as sp
    Ls, dev = _layers(3, 1024)
    cfg = Ls[0]["cfg"]
    B, Hq, C = cfg.block, cfg.n_q_heads, cfg.n_clusters
    nqb = cfg.seq // B
    h2c = [int(x) for x in Ls[0]["head_to_cluster"]]
    shape = sp.shape_of(dev[0]["q"], dev[0]["k"], None, B)
    vs_bytes = sp.sp_vs_token_workspace_bytes(shape, Hq) if token_level else sp.sp_vs_workspace_bytes(shape, Hq)
    ws = torch.empty(sp.sp_workspace_bytes(shape, C) + vs_bytes, dtype=torch.uint8, device="cuda")
    mode = dict(fallback_mode=sp.SP_FALLBACK_VERTICAL_SLASH_TOKEN) if token_level else \
        dict(fallback_mode=sp.SP_FALLBACK_VERTICAL_SLASH, vs_idx=None, vs_cnt=None)
    valid = torch.zeros((1, C), dtype=torch.int32, device="cuda")
    a_t = torch.zeros((1, C, nqb), dtype=torch.float32, device="cuda")
    didx = torch.zeros((1, C, nqb, nqb), dtype=torch.int32, device="cuda")
    dcnt = torch.zeros((1, C, nqb), dtype=torch.int32, device="cuda")
    pd = sp.pattern_dict_of(valid, a_t, didx, dcnt)
    vidx = torch.zeros((1, Hq, nqb, nqb), dtype=torch.int32, device="cuda")
    vcnt = torch.zeros((1, Hq, nqb), dtype=torch.int32, device="cuda")
    scores = torch.zeros((1, C, nqb, nqb), dtype=torch.float32, device="cuda")
    a_hat = torch.zeros((1, Hq, nqb), dtype=torch.float32, device="cuda")
    dist = torch.zeros((1, Hq, 2), dtype=torch.float32, device="cuda")
    outs = [torch.zeros_like(d["q"]) for d in dev]
    roles = [torch.zeros((1, Hq), dtype=torch.int32, device="cuda") for _ in dev]
    delta = 0.05        # between the heads' sparsity distances at this length: some fall back, some elect / share
    if not token_level:
        mode.update(vs_idx=vidx, vs_cnt=vcnt)

    def prefill():
        valid.zero_()
        for l, d in enumerate(dev):
            sp.sp_prefill_layer_dict(shape, d["q"], d["k"], d["v"], h2c, cfg.gamma, delta, 10.0, 0, 0, pd, outs[l],
                                     scores, roles[l], a_hat, dist, ws, **mode)

    prefill()
    torch.cuda.synchronize()
    want = [t.clone() for t in outs + roles + [valid, didx, dcnt]]
    r0 = roles[0].cpu().numpy()[0]
    assert (r0 == -1).any() and (r0 == -2).any(), r0
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        prefill()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        prefill()
    for rep in range(3):
        for t in outs + roles:
            t.fill_(3)
        valid.fill_(1)          # a stale dictionary: the graph's own reset has to clear it
        print(f"[graph] dictionary prefill replay {rep}", flush=True)
        graph.replay()
        torch.cuda.synchronize()
        for got, w in zip(outs + roles + [valid, didx, dcnt], want):
            assert torch.equal(got, w)
        junk = torch.randn(1 << 16, device="cuda").sum().item()
        assert np.isfinite(junk)
