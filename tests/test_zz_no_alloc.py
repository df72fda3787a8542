"""The entry point that allocates nothing (sp_build_block_mask_global_static: selection scratch in a static
device array inside the library) against sp_build_block_mask_global with a caller workspace: same lists and
counts, bit for bit, on two calls in a row, the second on a smaller input; the size limit is an error."""
import numpy as np
import pytest


def _scores(n_maps, nqb, seed):
    """Row-stochastic lower-triangular maps with ties, zeros and a heavy column (inputs only)."""
    rng = np.random.default_rng(seed)
    s = rng.random((n_maps, nqb, nqb), dtype=np.float32) ** 4
    s[:, :, 0] += 0.5
    s[rng.random(s.shape) < 0.2] = 0.0
    s[:, :, 3 % nqb] = np.float32(0.25)            # ties down a column
    s = np.tril(s)
    s /= np.maximum(s.sum(-1, keepdims=True), np.float32(1e-30))
    return s.astype(np.float32)


@pytest.mark.gpu
def test_static_scratch_call_matches_workspace_call_twice():
    import torch
    import paper_2505_19578_amd as sp
    for call, (n_maps, nqb, gamma, forced) in enumerate([(7, 256, 0.9, True), (3, 40, 0.95, False)]):
        print(f"[no-alloc] call {call}: n_maps {n_maps} nqb {nqb}", flush=True)
        sc = torch.from_numpy(_scores(n_maps, nqb, 100 + call)).cuda()
        ws = torch.empty(sp.sp_mask_workspace_bytes(n_maps, nqb), dtype=torch.uint8, device="cuda")
        idx_a = torch.full((n_maps, nqb, nqb), -7, dtype=torch.int32, device="cuda")
        cnt_a = torch.full((n_maps, nqb), -7, dtype=torch.int32, device="cuda")
        idx_b, cnt_b = idx_a.clone(), cnt_a.clone()
        sp.sp_build_block_mask_global(sc, n_maps, nqb, nqb, gamma, forced, idx_a, cnt_a, ws)
        sp.sp_build_block_mask_global_static(sc, n_maps, nqb, nqb, gamma, forced, idx_b, cnt_b)
        torch.cuda.synchronize()
        assert torch.equal(cnt_a, cnt_b) and torch.equal(idx_a, idx_b)
        assert int(cnt_a.min()) >= 0 and int(cnt_a.sum()) > 0


def test_static_scratch_limit_is_an_error():
    """Argument and size checks come before any device call: runs without a GPU."""
    import ctypes
    import paper_2505_19578_amd as sp
    L = sp.lib()
    dummy = ctypes.c_void_p(256)
    nqb = 1024
    per_map = 2 * 4096 * 8 + 256 * ((8 * nqb + 255) // 256)     # lower bound of the scratch of one map
    too_many = sp.SP_STATIC_SCRATCH_BYTES // per_map + 1
    rc = L.sp_build_block_mask_global_static(dummy, too_many, nqb, nqb, ctypes.c_float(0.9), 1, dummy, dummy, None)
    assert L.sp_status_string(rc) == b"SP_ERR_UNSUPPORTED" and b"static" in L.sp_last_error()
    rc = L.sp_build_block_mask_global_static(None, 1, nqb, nqb, ctypes.c_float(0.9), 1, dummy, dummy, None)
    assert L.sp_status_string(rc) == b"SP_ERR_INVALID_ARG"
