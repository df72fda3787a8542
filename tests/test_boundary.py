"""CPU-only checks of the boundary: the library loads, exports every symbol the
header declares, and rejects bad arguments synchronously without a GPU."""
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _shape(sp, **kw):
    s = sp.SpShape()
    s.batch, s.seq, s.n_q_heads, s.n_kv_heads, s.head_dim, s.block = 1, 1024, 4, 4, 64, 64
    for f in ("q", "kv", "o"):
        setattr(s, f + "_stride_b", 1024 * 256)
        setattr(s, f + "_stride_t", 256)
        setattr(s, f + "_stride_h", 64)
    for k, v in kw.items():
        setattr(s, k, v)
    return s


def test_header_symbols_are_exported():
    import paper_2505_19578_amd as sp
    hdr = open(os.path.join(ROOT, "include", "shareprefill.h")).read()
    declared = set(re.findall(r"\b(sp_[a-z_]+)\s*\(", hdr))
    assert declared == set(sp.EXPORTED_SYMBOLS)
    L = sp.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert L.sp_status_string(0) == b"SP_OK"


def test_workspace_bytes_and_shape_validation():
    import paper_2505_19578_amd as sp
    s = _shape(sp)
    pack = 1 * 4 * 1024 * 64 * 2 * 2
    def score_ws(n):    # key sums of every KV head, query sums + diagonal sums of n heads
        return 4 * 16 * 64 * 4 + n * 16 * 64 * 4 + 256

    def mask_ws(n):     # two histograms + state + per-row counters, per map
        return -(-(n * (2 * 4104 * 8 + 64 + 256)) // 256) * 256

    assert sp.sp_score_workspace_bytes(s, 2) == score_ws(2)
    assert sp.sp_mask_workspace_bytes(2, 16) == mask_ws(2)
    # the attention calls' workspace also covers the gate, which pools all 4 heads
    tables = 256        # elected pivots and list routing of the dictionary call, 2 x batch x heads int32
    assert sp.sp_workspace_bytes(s, 0) == pack + score_ws(4) + mask_ws(4) + tables
    # scored heads add their block log-sum-exps (causal half: nqb(nqb+1)/2 key-block slots of `block` floats per
    # head) and room for the score maps of a call that does not return them
    lse, maps = 2 * (16 * 17 // 2) * 64 * 4, 2 * 16 * 16 * 4
    assert sp.sp_workspace_bytes(s, 2) == pack + lse + score_ws(4) + mask_ws(4) + tables + maps
    with pytest.raises(sp.SpError):
        sp.sp_mask_workspace_bytes(0, 16)
    with pytest.raises(sp.SpError):
        sp.sp_mask_workspace_bytes(1, 40000)
    with pytest.raises(sp.SpError):
        sp.sp_score_workspace_bytes(s, 5)
    for bad, status in [
        (dict(seq=1000), "SP_ERR_UNSUPPORTED"),
        (dict(seq=960, block=128), "SP_ERR_UNSUPPORTED"),
        (dict(head_dim=96), "SP_ERR_UNSUPPORTED"),
        (dict(block=32), "SP_ERR_UNSUPPORTED"),
        (dict(n_kv_heads=3), "SP_ERR_INVALID_ARG"),
        (dict(q_stride_t=260), "SP_ERR_INVALID_ARG"),
        (dict(batch=0), "SP_ERR_INVALID_ARG"),
        (dict(softmax_scale=-1.0), "SP_ERR_INVALID_ARG"),
    ]:
        with pytest.raises(sp.SpError) as e:
            sp.sp_workspace_bytes(_shape(sp, **bad), 1)
        assert e.value.status_name == status, bad
    with pytest.raises(sp.SpError):
        sp.sp_workspace_bytes(s, 5)
    assert sp.sp_workspace_bytes(_shape(sp, seq=960), 1) > 0       # a multiple of block = 64, not of 128


def test_calls_reject_bad_arguments_without_launching():
    """Null / misaligned pointers, bad ids, bad gamma, missing workspace: all rejected on the host."""
    import ctypes
    import paper_2505_19578_amd as sp
    L = sp.lib()
    s = _shape(sp)
    ids = (ctypes.c_int32 * 4)(0, 1, 2, 3)
    fake = ctypes.c_void_p(4096)     # never dereferenced: validation fails first
    rc = L.sp_dense_attn_with_block_scores(ctypes.byref(s), None, fake, fake, ids, 1, fake, None, None, 0, None)
    assert L.sp_status_string(rc) == b"SP_ERR_INVALID_ARG" and b"q is NULL" in L.sp_last_error()
    rc = L.sp_dense_attn_with_block_scores(ctypes.byref(s), ctypes.c_void_p(4100), fake, fake, ids, 1, fake, None,
                                           None, 0, None)
    assert L.sp_status_string(rc) == b"SP_ERR_INVALID_ARG"
    rc = L.sp_dense_attn_with_block_scores(ctypes.byref(s), fake, fake, fake, ids, 1, fake, None, None, 0, None)
    assert L.sp_status_string(rc) == b"SP_ERR_WORKSPACE"
    bad = (ctypes.c_int32 * 2)(1, 1)
    rc = L.sp_dense_attn_with_block_scores(ctypes.byref(s), fake, fake, fake, bad, 2, fake, None, fake, 1 << 30, None)
    assert L.sp_status_string(rc) == b"SP_ERR_INVALID_ARG" and b"twice" in L.sp_last_error()
    rc = L.sp_build_block_mask(fake, 1, 16, 16, ctypes.c_float(0.0), fake, fake, None, None)
    assert L.sp_status_string(rc) == b"SP_ERR_INVALID_ARG"
    rc = L.sp_build_block_mask(fake, 1, 16, 8, ctypes.c_float(0.9), fake, fake, None, None)
    assert L.sp_status_string(rc) == b"SP_ERR_INVALID_ARG"
    rc = L.sp_build_block_mask(fake, 1, 40000, 40000, ctypes.c_float(0.9), fake, fake, None, None)
    assert L.sp_status_string(rc) == b"SP_ERR_UNSUPPORTED"
    hm = (ctypes.c_int32 * 1)(3)
    rc = L.sp_block_sparse_attn(ctypes.byref(s), fake, fake, fake, ids, hm, 1, fake, fake, 2, fake, fake, 1 << 30, None)
    assert L.sp_status_string(rc) == b"SP_ERR_INVALID_ARG" and b"head_map" in L.sp_last_error()
    h2c = (ctypes.c_int32 * 4)(0, 0, 1, 1)
    piv = (ctypes.c_int32 * 2)(0, 1)     # head 1 is not in cluster 1
    rc = L.sp_prefill_layer(ctypes.byref(s), fake, fake, fake, h2c, piv, 2, ctypes.c_float(0.9), fake, fake, fake,
                            fake, fake, 1 << 30, None)
    assert L.sp_status_string(rc) == b"SP_ERR_INVALID_ARG" and b"lies in cluster" in L.sp_last_error()
    piv = (ctypes.c_int32 * 2)(0, 2)
    rc = L.sp_prefill_layer(ctypes.byref(s), fake, fake, fake, h2c, piv, 2, ctypes.c_float(0.9), fake, fake, fake,
                            fake, fake, 16, None)
    assert L.sp_status_string(rc) == b"SP_ERR_WORKSPACE"
    # pattern construction as printed: scores, global selection, fused call with modes
    rc = L.sp_block_mean_logit_scores(ctypes.byref(s), fake, None, ids, 1, fake, fake, 1 << 30, None)
    assert L.sp_status_string(rc) == b"SP_ERR_INVALID_ARG" and b"k is NULL" in L.sp_last_error()
    rc = L.sp_block_mean_logit_scores(ctypes.byref(s), fake, fake, ids, 1, None, fake, 1 << 30, None)
    assert L.sp_status_string(rc) == b"SP_ERR_INVALID_ARG"
    rc = L.sp_block_mean_logit_scores(ctypes.byref(s), fake, fake, ids, 1, fake, fake, 64, None)
    assert L.sp_status_string(rc) == b"SP_ERR_WORKSPACE"
    rc = L.sp_build_block_mask_global(fake, 1, 16, 16, ctypes.c_float(1.5), 1, fake, fake, fake, 1 << 30, None)
    assert L.sp_status_string(rc) == b"SP_ERR_INVALID_ARG"
    rc = L.sp_build_block_mask_global(fake, 1, 16, 8, ctypes.c_float(0.9), 1, fake, fake, fake, 1 << 30, None)
    assert L.sp_status_string(rc) == b"SP_ERR_INVALID_ARG"
    rc = L.sp_build_block_mask_global(fake, 70000, 16, 16, ctypes.c_float(0.9), 1, fake, fake, fake, 1 << 40, None)
    assert L.sp_status_string(rc) == b"SP_ERR_UNSUPPORTED"
    rc = L.sp_build_block_mask_global(fake, 1, 16, 16, ctypes.c_float(0.9), 1, fake, fake, fake, 1024, None)
    assert L.sp_status_string(rc) == b"SP_ERR_WORKSPACE"
    rc = L.sp_build_block_mask_global(fake, 1, 16, 16, ctypes.c_float(0.9), 1, fake, fake, None, 0, None)
    assert L.sp_status_string(rc) == b"SP_ERR_WORKSPACE"
    rc = L.sp_prefill_layer_modes(ctypes.byref(s), fake, fake, fake, h2c, piv, 2, ctypes.c_float(0.9), 2, 0, fake,
                                  fake, fake, fake, fake, 1 << 30, None)
    assert L.sp_status_string(rc) == b"SP_ERR_INVALID_ARG" and b"score_mode" in L.sp_last_error()
    rc = L.sp_prefill_layer_modes(ctypes.byref(s), fake, fake, fake, h2c, piv, 2, ctypes.c_float(0.9), 1, 1, fake,
                                  fake, fake, fake, fake, 16, None)
    assert L.sp_status_string(rc) == b"SP_ERR_WORKSPACE"
    # Alg. 3 gate
    ref = (ctypes.c_int32 * 4)(0, 0, 2, 9)
    rc = L.sp_determine_pattern(ctypes.byref(s), fake, fake, ids, 4, ref, h2c, ctypes.c_float(0.3),
                                ctypes.c_float(0.2), fake, fake, fake, fake, 1 << 30, None)
    assert L.sp_status_string(rc) == b"SP_ERR_INVALID_ARG" and b"ref_pos" in L.sp_last_error()
    ref = (ctypes.c_int32 * 4)(0, 0, 2, 2)
    rc = L.sp_determine_pattern(ctypes.byref(s), fake, fake, ids, 4, ref, h2c, ctypes.c_float(-0.3),
                                ctypes.c_float(0.2), fake, fake, fake, fake, 1 << 30, None)
    assert L.sp_status_string(rc) == b"SP_ERR_INVALID_ARG" and b"delta" in L.sp_last_error()
    rc = L.sp_determine_pattern(ctypes.byref(s), fake, fake, ids, 4, ref, h2c, ctypes.c_float(0.3),
                                ctypes.c_float(0.2), fake, None, fake, fake, 1 << 30, None)
    assert L.sp_status_string(rc) == b"SP_ERR_INVALID_ARG"
    rc = L.sp_determine_pattern(ctypes.byref(s), fake, fake, ids, 4, ref, h2c, ctypes.c_float(0.3),
                                ctypes.c_float(0.2), fake, fake, fake, fake, 128, None)
    assert L.sp_status_string(rc) == b"SP_ERR_WORKSPACE"
    rc = L.sp_block_sparse_attn_gated(ctypes.byref(s), fake, fake, fake, ids, 4, fake, fake, 2, None, fake, fake,
                                      1 << 30, None)
    assert L.sp_status_string(rc) == b"SP_ERR_INVALID_ARG" and b"head_pattern" in L.sp_last_error()
    rc = L.sp_prefill_layer_gated(ctypes.byref(s), fake, fake, fake, h2c, piv, 2, ctypes.c_float(0.9),
                                  ctypes.c_float(0.3), ctypes.c_float(0.2), 0, 0, fake, fake, fake, fake, fake, None,
                                  fake, fake, 1 << 30, None)
    assert L.sp_status_string(rc) == b"SP_ERR_INVALID_ARG" and b"dist" in L.sp_last_error()
    # dictionary call
    d = sp.SpPatternDict()
    d.n_clusters, d.valid, d.a_tilde, d.kb_idx, d.kb_cnt = 2, 4096, 4096, 4096, 4096
    args = lambda dd, hc, ws_bytes, fb=0, vsp=None: (
        ctypes.byref(s), fake, fake, fake, hc, ctypes.c_float(0.9), ctypes.c_float(0.3), ctypes.c_float(0.2), 0, 0, fb,
        dd, fake, fake, fake, fake, fake, vsp, vsp, fake, ws_bytes, None)
    rc = L.sp_prefill_layer_dict(*args(None, h2c, 1 << 30))
    assert L.sp_status_string(rc) == b"SP_ERR_INVALID_ARG"
    bad_c = (ctypes.c_int32 * 4)(0, 0, 1, 2)          # cluster 2 does not exist in a 2-cluster dictionary
    rc = L.sp_prefill_layer_dict(*args(ctypes.byref(d), bad_c, 1 << 30))
    assert L.sp_status_string(rc) == b"SP_ERR_INVALID_ARG" and b"head_to_cluster[3]" in L.sp_last_error()
    rc = L.sp_prefill_layer_dict(*args(ctypes.byref(d), h2c, 64))
    assert L.sp_status_string(rc) == b"SP_ERR_WORKSPACE"
    rc = L.sp_prefill_layer_dict(*args(ctypes.byref(d), h2c, 1 << 30, fb=1))      # vertical-slash fallback needs its lists
    assert L.sp_status_string(rc) == b"SP_ERR_INVALID_ARG" and b"vs_idx" in L.sp_last_error()
    rc = L.sp_prefill_layer_dict(*args(ctypes.byref(d), h2c, 1 << 30, fb=7, vsp=fake))
    assert L.sp_status_string(rc) == b"SP_ERR_INVALID_ARG" and b"fallback_mode" in L.sp_last_error()
    d.kb_cnt = None
    rc = L.sp_prefill_layer_dict(*args(ctypes.byref(d), h2c, 1 << 30))
    assert L.sp_status_string(rc) == b"SP_ERR_INVALID_ARG" and b"dict" in L.sp_last_error()
    # Alg. 5
    rc = L.sp_search_vertical_slash(ctypes.byref(s), fake, fake, ids, 2, ctypes.c_float(0.9), 1, None, fake, None,
                                    fake, 1 << 40, None)
    assert L.sp_status_string(rc) == b"SP_ERR_INVALID_ARG" and b"kb_cnt" in L.sp_last_error()
    rc = L.sp_search_vertical_slash(ctypes.byref(s), fake, fake, ids, 2, ctypes.c_float(0.0), 1, None, fake, fake,
                                    fake, 1 << 40, None)
    assert L.sp_status_string(rc) == b"SP_ERR_INVALID_ARG" and b"gamma" in L.sp_last_error()
    rc = L.sp_search_vertical_slash(ctypes.byref(s), fake, fake, ids, 2, ctypes.c_float(0.9), 1, None, fake, fake,
                                    fake, 4096, None)
    assert L.sp_status_string(rc) == b"SP_ERR_WORKSPACE"
    # slab of raw logits (block x seq fp32 per head) dominates the search's workspace
    assert sp.sp_vs_workspace_bytes(s, 2) >= 2 * 64 * 1024 * 4 + 2 * 2 * 1024 * 4
    # attention over the token-level pattern of Alg. 5
    tok = lambda gamma, bits, ws_bytes, o=fake: L.sp_vertical_slash_attn(
        ctypes.byref(s), fake, fake, fake, ids, 2, ctypes.c_float(gamma), 1, o, bits, None, fake, ws_bytes, None)
    rc = tok(1.5, None, 1 << 40)
    assert L.sp_status_string(rc) == b"SP_ERR_INVALID_ARG" and b"gamma" in L.sp_last_error()
    rc = tok(0.9, 4100, 1 << 40)                       # a bitmap pointer that is not 8-byte aligned
    assert L.sp_status_string(rc) == b"SP_ERR_INVALID_ARG" and b"keep_bits" in L.sp_last_error()
    rc = tok(0.9, None, 1 << 40, o=None)
    assert L.sp_status_string(rc) == b"SP_ERR_INVALID_ARG"
    rc = tok(0.9, None, 4096)
    assert L.sp_status_string(rc) == b"SP_ERR_WORKSPACE"
    # on top of the search's workspace: bitmaps, ranks of the kept keys (seq ints) and one more packed K/V copy per head
    extra = sp.sp_vs_token_workspace_bytes(s, 2) - sp.sp_vs_workspace_bytes(s, 2)
    assert extra >= 2 * (2 * (s.seq // 8) + s.seq * 4 + s.seq * s.head_dim * 2 * 2)
    assert sp.sp_vs_token_workspace_bytes(s, 4) > sp.sp_vs_token_workspace_bytes(s, 2)


def test_generator_is_deterministic_and_bf16_round_trip():
    import numpy as np
    from synth import CONFIGS, make_layer, f32_to_bf16_bits, bf16_bits_to_f32
    a = make_layer(CONFIGS["tiny"], seq=256)
    b = make_layer(CONFIGS["tiny"], seq=256)
    for x in "qkv":
        assert np.array_equal(a[x], b[x])
    assert list(a["head_to_cluster"]) == [0, 0, 1, 1] and list(a["pivot_heads"]) == [0, 2]
    c = make_layer(CONFIGS["tiny"], layer=1, seq=256)
    assert not np.array_equal(a["q"], c["q"])
    # layers of one prompt: structure (clusters, heavy positions) from layer 0, projections / noise of their own
    p0 = make_layer(CONFIGS["qwen7b_128k"], layer=0, seq=512)
    p1 = make_layer(CONFIGS["qwen7b_128k"], layer=1, seq=512, structure_layer=0)
    own = make_layer(CONFIGS["qwen7b_128k"], layer=1, seq=512)
    assert np.array_equal(p0["head_to_cluster"], p1["head_to_cluster"]) and np.array_equal(p0["heavy"], p1["heavy"])
    assert not np.array_equal(p0["head_to_cluster"], own["head_to_cluster"])
    assert not np.array_equal(p0["q"], p1["q"]) and p1["seed"] == own["seed"]
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.0e38], dtype=np.float32)
    bits = f32_to_bf16_bits(x)
    # 1 + 2^-8 is a tie -> even (1.0); 1 + 3*2^-8 is a tie -> even (1 + 2^-6)
    assert list(bf16_bits_to_f32(bits)[:4]) == [1.0, 1.0, 1.015625, -2.5]
    import torch
    t = torch.tensor(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, t)
    q = make_layer(CONFIGS["qwen7b_128k"], seq=512)
    assert sorted(np.bincount(q["head_to_cluster"])) == [4] * 7
    assert all(q["head_to_cluster"][p] == c for c, p in enumerate(q["pivot_heads"]))


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                         text=True, timeout=120)
    assert res.returncode != 0
    assert "single-GPU" in res.stderr and res.stdout.strip() == ""
