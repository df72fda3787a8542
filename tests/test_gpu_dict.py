"""GPU parity for the cross-layer pivotal pattern dictionary (Sec. 5.2; Alg. 1 with Alg. 2-4):
sp_prefill_layer_dict over several layers of one prompt against the CPU oracle.

What is compared, layer by layer: the roles (election / sharing / fallback) with the oracle's own
head-by-head run wherever its distances are farther than 1e-4 from the thresholds; estimates and
distances to the bars of the Alg. 3 tests; the lists an elected pivot installs, bit for bit, with
the oracle's Alg. 2 fed the GPU's score map; that entries, once installed, never change; and every
head's output (max-abs 2e-2 / mean-abs 2e-3) against the oracle stage its role calls for, run with
the dictionary lists the GPU used."""
import numpy as np
import pytest

from tests.test_gpu_parity import OUT_MAX, OUT_MEAN, _LazyHost
from tests.test_gpu_determine import _f32, MARGIN

pytestmark = pytest.mark.gpu


class _Dict:
    def __init__(self, sp, batch, n_clusters, nqb):
        import torch
        self.valid = torch.zeros((batch, n_clusters), dtype=torch.int32, device="cuda")
        self.a_tilde = torch.full((batch, n_clusters, nqb), -1.0, dtype=torch.float32, device="cuda")
        self.kb_idx = torch.full((batch, n_clusters, nqb, nqb), -9, dtype=torch.int32, device="cuda")
        self.kb_cnt = torch.full((batch, n_clusters, nqb), -9, dtype=torch.int32, device="cuda")
        self.c = sp.pattern_dict_of(self.valid, self.a_tilde, self.kb_idx, self.kb_cnt)

    def snapshot(self):
        return [t.cpu().numpy().copy() for t in (self.valid, self.a_tilde, self.kb_idx, self.kb_cnt)]


def _layers(name, n_layers, seq):
    from synth import CONFIGS, make_layer
    return [make_layer(CONFIGS[name], layer=l, seq=seq, structure_layer=0) for l in range(n_layers)]


def _run_and_check(name, seq, n_layers, delta, tau, modes=(0, 0), h2c_of_layer=None, n_clusters=None, rows=None,
                   check_heads=None, full_oracle=True, label=""):
    import torch
    import oracle
    import paper_2505_19578_amd as sp
    from synth import bf16_bits_to_f32
    from tests.gpu_util import to_dev, bf16_dev_to_f32, err_stats
    Ls = _layers(name, n_layers, seq)
    cfg = Ls[0]["cfg"]
    B, G, Hq = cfg.block, cfg.group, cfg.n_q_heads
    nqb = cfg.seq // B
    C = cfg.n_clusters if n_clusters is None else n_clusters
    D = _Dict(sp, 1, C, nqb)
    rows = np.arange(nqb) if rows is None else np.asarray(rows, dtype=np.int32)
    sel_t = np.concatenate([np.arange(i * B, (i + 1) * B) for i in rows])
    gpu_layers, prev = [], D.snapshot()
    for l, L in enumerate(Ls):
        h2c = [int(x) for x in (L["head_to_cluster"] if h2c_of_layer is None else h2c_of_layer(l, L))]
        slots = sorted({c for c in h2c if c >= 0})
        dev = {x: to_dev(L[x]) for x in "qkv"}
        q, k, v = dev["q"], dev["k"], dev["v"]
        shape = sp.shape_of(q, k, None, B)
        o = torch.zeros_like(q)
        ws = torch.empty(sp.sp_workspace_bytes(shape, len(slots)), dtype=torch.uint8, device="cuda")
        scores = torch.full((1, max(len(slots), 1), nqb, nqb), float("nan"), dtype=torch.float32, device="cuda")
        role = torch.full((1, Hq), -7, dtype=torch.int32, device="cuda")
        a_hat = torch.empty((1, Hq, nqb), dtype=torch.float32, device="cuda")
        dist = torch.empty((1, Hq, 2), dtype=torch.float32, device="cuda")
        print(f"[{label}] layer {l}: sp_prefill_layer_dict N={cfg.seq} slots={slots}", flush=True)
        sp.sp_prefill_layer_dict(shape, q, k, v, h2c, cfg.gamma, delta, tau, modes[0], modes[1], D.c, o, scores, role,
                                 a_hat, dist, ws)
        torch.cuda.synchronize()
        now = D.snapshot()
        role_h = role.cpu().numpy()[0]
        host = _LazyHost(L)
        # -- dictionary bookkeeping
        for c in range(C):
            pivots = [h for h in range(Hq) if h2c[h] == c and role_h[h] == -2]
            if prev[0][0, c]:                                   # an entry never changes, and elects nobody
                assert not pivots and now[0][0, c] == 1
                for a, b_ in zip(prev[1:], now[1:]):
                    assert np.array_equal(a[0, c], b_[0, c]), f"layer {l}: entry {c} changed"
            elif pivots:                                        # installed now
                assert len(pivots) == 1 and now[0][0, c] == 1
                p = pivots[0]
                assert np.array_equal(now[1][0, c], a_hat.cpu().numpy()[0, p])
                sc = scores.cpu().numpy()[0, slots.index(c)]
                if modes[1] == 1:
                    idx_o, cnt_o, _ = oracle.build_mask_global(sc, cfg.gamma, True)
                else:
                    idx_o, cnt_o, _ = oracle.build_mask_rows(sc, cfg.gamma)
                same = np.array_equal(idx_o, now[2][0, c]) and np.array_equal(cnt_o, now[3][0, c])
                assert same, f"layer {l}: lists of new entry {c} differ"
            else:
                assert now[0][0, c] == 0
        # -- outputs by role, with the lists the GPU used
        o_h = bf16_dev_to_f32(o)[0]
        worst = 0.0
        for h in (range(Hq) if check_heads is None else check_heads):
            g = h // G
            if role_h[h] >= 0:
                c = int(role_h[h])
                assert c == h2c[h] and now[0][0, c] == 1
                o_o = oracle.masked_rows(host.head("q", h), host.head("k", g), host.head("v", g), B,
                                         now[2][0, c][rows], now[3][0, c][rows], rows)
            else:
                o_o, _, _ = oracle.dense_rows(host.head("q", h), host.head("k", g), host.head("v", g), B, rows,
                                              want_scores=False)
            emax, emean = err_stats(o_h[sel_t, h], o_o)
            worst = max(worst, emax)
            assert emax <= OUT_MAX and emean <= OUT_MEAN, f"layer {l} head {h} role {role_h[h]}: {emax} / {emean}"
        gpu_layers.append(dict(role=role_h, dist=dist.cpu().numpy()[0], a_hat=a_hat.cpu().numpy()[0], h2c=h2c))
        print(f"[{label}] layer {l}: roles {[int(x) for x in role_h]} out max {worst:.2e}", flush=True)
        prev = now
    if full_oracle:     # the oracle's own head-by-head run: roles and distances
        o_layers = []
        for l, L in enumerate(Ls):
            o_layers.append({x: bf16_bits_to_f32(L[x]) for x in "qkv"} | {"head_to_cluster": gpu_layers[l]["h2c"]})
        res, _ = oracle.prefill_layers_dict(o_layers, B, cfg.gamma, _f32(delta), _f32(tau), paper_pattern=modes[0] == 1)
        for l, (r, gl) in enumerate(zip(res, gpu_layers)):
            for h in range(Hq):
                if gl["h2c"][h] < 0:
                    continue            # Alg. 3 is not evaluated for heads without a cluster
                ds, dm = r["dist"][h]
                assert abs(gl["dist"][h, 0] - ds) <= 2e-5 and abs(gl["dist"][h, 1] - dm) <= (2e-5 if dm >= 1e-3 else 1e-3)
                assert abs(ds - _f32(delta)) > MARGIN and abs(dm - _f32(tau)) > MARGIN, "borderline case in the test data"
            assert list(r["role"]) == list(gl["role"]), f"layer {l}: roles {list(gl['role'])} vs oracle {list(r['role'])}"
    return gpu_layers


def test_dict_open_gates_three_layers():
    g = _run_and_check("tiny", None, 3, 10.0, 10.0, label="tiny open")
    assert list(g[0]["role"]) == [-2, 0, -2, 1] and list(g[1]["role"]) == [0, 0, 1, 1] == list(g[2]["role"])
    g = _run_and_check("llama8b_32k", 2048, 3, 10.0, 10.0, modes=(1, 1), label="llama8b@2k open, printed construction")
    assert sum(1 for r in g[0]["role"] if r == -2) == 8 and all(r >= 0 for r in g[1]["role"])


def test_dict_sparsity_gate_delays_election():
    # learn the spread of d_sparse over all three layers (it does not depend on the thresholds), then put
    # delta into the widest gap of its lower half: some clusters cannot elect in layer 0
    g = _run_and_check("llama8b_32k", 2048, 3, 10.0, 10.0, full_oracle=False, label="probe")
    ds = np.sort(np.concatenate([x["dist"][:, 0] for x in g]))
    lo, hi = len(ds) // 5, len(ds) // 2
    i = lo + int(np.argmax(ds[lo + 1:hi + 1] - ds[lo:hi]))
    delta = float(0.5 * (ds[i] + ds[i + 1]))
    assert ds[i + 1] - ds[i] > 4e-4
    g = _run_and_check("llama8b_32k", 2048, 3, delta, 10.0, label="llama8b@2k sparsity gate")
    roles = np.array([x["role"] for x in g])
    assert (roles == -1).any() and (roles == -2).any() and (roles >= 0).any()


def test_dict_new_clusters_unclustered_heads_and_similarity_rejection():
    def h2c_of_layer(l, L):
        h2c = [int(x) for x in L["head_to_cluster"]]
        if l >= 1:
            h2c[1] = 9          # a cluster id that first appears in layer 1
            h2c[5] = 9
            h2c[6] = -1         # no cluster
            h2c[9] = (h2c[9] + 1) % 8   # planted into a foreign cluster: must fail the similarity test
        return h2c
    g = _run_and_check("llama8b_32k", 2048, 1, 10.0, 10.0, full_oracle=False, label="probe")
    tau = float(g[0]["dist"][:, 1].max()) + 0.05
    g = _run_and_check("llama8b_32k", 2048, 3, 10.0, tau, h2c_of_layer=h2c_of_layer, n_clusters=12,
                       label="llama8b@2k new clusters")
    assert g[1]["role"][1] == -2 and g[1]["role"][6] == -1 and g[2]["role"][1] == 9
    assert g[1]["role"][9] == -1, f"foreign head shared: d_sim {g[1]['dist'][9, 1]} tau {tau}"


def test_dict_llama8b_128k_three_layers_full_size():
    from tests.test_gpu_full_size import _sample_rows
    rows = _sample_rows(1024, 11, extra=0)
    g = _run_and_check("llama8b_128k", None, 3, 10.0, 0.2, rows=rows, check_heads=[0, 1, 13, 30], full_oracle=False,
                       label="cfg3 x3 layers")
    assert sum(1 for r in g[0]["role"] if r == -2) == 8
    assert all(r >= 0 for r in g[1]["role"]) and all(r >= 0 for r in g[2]["role"])


def test_dict_batch_of_two_prompts_equals_two_single_runs():
    """Batch entries are independent prefills with their own dictionaries: a batch of two prompts gives, bit for
    bit, what each prompt gives alone (roles, dictionary, outputs), also with the vertical-slash fallback."""
    import torch
    import paper_2505_19578_amd as sp
    from synth import CONFIGS, make_layer
    from tests.gpu_util import to_dev
    cfg = CONFIGS["tiny"]
    B, Hq, C = cfg.block, cfg.n_q_heads, cfg.n_clusters
    prompts = [[make_layer(cfg, layer=l, structure_layer=s0) for l in (s0, s0 + 1)] for s0 in (0, 20)]
    nqb = prompts[0][0]["cfg"].seq // B
    h2c = [int(x) for x in prompts[0][0]["head_to_cluster"]]
    for fallback, delta in ((sp.SP_FALLBACK_DENSE, 10.0), (sp.SP_FALLBACK_VERTICAL_SLASH, 0.05),
                            (sp.SP_FALLBACK_VERTICAL_SLASH_TOKEN, 0.05)):
        def run(batch_prompts):
            nb = len(batch_prompts)
            D = _Dict(sp, nb, C, nqb)
            vs_idx = torch.full((nb, Hq, nqb, nqb), -3, dtype=torch.int32, device="cuda")
            vs_cnt = torch.full((nb, Hq, nqb), -3, dtype=torch.int32, device="cuda")
            outs = []
            for l in range(2):
                q, k, v = (torch.cat([to_dev(p[l][x]) for p in batch_prompts], dim=0) for x in "qkv")
                shape = sp.shape_of(q, k, None, B)
                ws = torch.empty(sp.sp_workspace_bytes(shape, C) + max(sp.sp_vs_workspace_bytes(shape, Hq),
                                                                         sp.sp_vs_token_workspace_bytes(shape, Hq)),
                                 dtype=torch.uint8, device="cuda")
                o = torch.zeros_like(q)
                scores = torch.zeros((nb, C, nqb, nqb), dtype=torch.float32, device="cuda")
                role = torch.full((nb, Hq), -7, dtype=torch.int32, device="cuda")
                a_hat = torch.empty((nb, Hq, nqb), dtype=torch.float32, device="cuda")
                dist = torch.empty((nb, Hq, 2), dtype=torch.float32, device="cuda")
                print(f"[dict batch {nb}] layer {l} fallback {fallback}", flush=True)
                lists = {} if fallback == sp.SP_FALLBACK_VERTICAL_SLASH_TOKEN else dict(vs_idx=vs_idx, vs_cnt=vs_cnt)
                sp.sp_prefill_layer_dict(shape, q, k, v, h2c, cfg.gamma, delta, 10.0, 0, 0, D.c, o, scores, role, a_hat,
                                         dist, ws, fallback_mode=fallback, **lists)
                torch.cuda.synchronize()
                outs.append((o.clone(), role.clone(), dist.clone(), a_hat.clone()))
            return outs, D
        both, Db = run(prompts)
        for n, p in enumerate(prompts):
            single, Ds = run([p])
            for l in range(2):
                for tb, ts in zip(both[l], single[l]):
                    assert torch.equal(tb[n:n + 1], ts), (n, l)
            assert torch.equal(Db.valid[n], Ds.valid[0])
            for c in range(C):
                if int(Ds.valid[0, c]):
                    assert torch.equal(Db.kb_idx[n, c], Ds.kb_idx[0, c]) and torch.equal(Db.kb_cnt[n, c], Ds.kb_cnt[0, c])
                    assert torch.equal(Db.a_tilde[n, c], Ds.a_tilde[0, c])
        roles = both[0][1].cpu().numpy()
        print(f"[dict batch 2] fallback {fallback}: layer-0 roles {roles.tolist()}", flush=True)
        if fallback != sp.SP_FALLBACK_DENSE:
            assert (roles == -1).any()


def test_dict_permuted_clusters_with_fallbacks():
    """Clusters that straddle KV heads (a seeded permutation of the heads): the slot table of the role-driven
    launches is then not in head order, which the device-side compaction of sharing / falling-back heads has to
    follow.  Open gates, then a sparsity threshold that sends part of the heads to the dense fallback."""
    g = _run_and_check("qwen7b_128k", 4096, 2, 10.0, 10.0, label="qwen7b@4k open")
    assert sum(1 for r in g[0]["role"] if r == -2) == 7 and all(r >= 0 for r in g[1]["role"])
    ds = np.sort(np.concatenate([x["dist"][:, 0] for x in g]))
    lo, hi = len(ds) // 4, 3 * len(ds) // 4
    i = lo + int(np.argmax(ds[lo + 1:hi + 1] - ds[lo:hi]))
    assert ds[i + 1] - ds[i] > 4e-4
    g = _run_and_check("qwen7b_128k", 4096, 2, float(0.5 * (ds[i] + ds[i + 1])), 10.0, label="qwen7b@4k sparsity gate")
    roles = np.array([x["role"] for x in g])
    assert (roles == -1).any() and (roles >= 0).any()


def test_dict_paper_thresholds_on_the_spread_workload():
    """The thresholds the paper states (Sec. 6.1 "Implementation Details": gamma 0.9, tau 0.2, delta 0.3) on the
    workload whose heads spread in sparsity: every layer has heads that share, heads that fall back because they
    are highly sparse or not similar enough, and the first layer elects the pivots; roles, distances, dictionary
    and outputs against the oracle's head-by-head run."""
    g = _run_and_check("llama8b_128k_regime", 4096, 2, 0.3, 0.2, label="regime@4k paper thresholds")
    roles = np.array([x["role"] for x in g])
    assert (roles[0] == -2).sum() >= 6 and (roles[0] >= 0).any() and (roles[0] == -1).any()
    assert (roles[1] >= 0).sum() > (roles[1] == -1).sum() > 0
    ds = g[0]["dist"][:, 0]
    assert ds.min() < 0.3 < ds.max(), "the workload must straddle the sparsity threshold"
