"""The entry point that allocates nothing (bsga_sparse_attn_noalloc, for callers that cannot call
hipMalloc) against bsga_sparse_attn on the same inputs, through the raw C ABI: two calls in a row on
the library's built-in scratch, the second with a smaller input.  Both entry points run the same
kernels in the same launch order, so the outputs must be identical bit for bit."""
import ctypes

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _raw():
    import paper_2509_07120_amd as pkg
    lib = ctypes.CDLL(pkg.LIB_PATH)
    vp, ci, c64, cf, csz = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t
    lib.bsga_sparse_attn.restype = ci
    lib.bsga_sparse_attn.argtypes = [vp, vp, vp, ci, ci, c64, ci, ci, cf, vp, vp, ci, vp, vp, vp, csz, vp]
    lib.bsga_sparse_attn_noalloc.restype = ci
    lib.bsga_sparse_attn_noalloc.argtypes = [vp, vp, vp, ci, ci, c64, ci, ci, cf, vp, vp, ci, vp, vp, vp]
    lib.bsga_noalloc_scratch_bytes.restype = csz
    lib.bsga_noalloc_scratch_bytes.argtypes = []
    lib.bsga_attn_workspace_bytes.restype = csz
    lib.bsga_attn_workspace_bytes.argtypes = [ci, ci, c64, ci]
    lib.bsga_last_error.restype = ctypes.c_char_p
    return lib


def _case(H, N, b, seed, density):
    g = torch.Generator().manual_seed(seed)
    q, k, v = (torch.randn(H, N, 64, generator=g).to(torch.bfloat16).cuda() for _ in range(3))
    nb = -(-N // b)
    rng = np.random.default_rng(seed)
    mask = rng.random((H, nb, nb)) < density
    mask[:, ::7, :] = True                       # some rows keep everything: the launch order matters
    mask[:, :, 0] = True
    cnt = mask.sum(-1).astype(np.int32)
    idx = np.zeros((H, nb, nb), np.int32)
    for h in range(H):
        for I in range(nb):
            js = np.flatnonzero(mask[h, I])
            idx[h, I, :js.size] = js
    return q, k, v, torch.from_numpy(idx).cuda(), torch.from_numpy(cnt).cuda(), nb


def test_noalloc_matches_workspace_entry_point_twice():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    lib = _raw()
    st = torch.cuda.current_stream().cuda_stream
    assert lib.bsga_noalloc_scratch_bytes() == 2 << 20
    # first call: 8 heads x 160 query blocks = 1280 rows (launch order active); second: a smaller input
    for H, N, b, seed, density in [(8, 160 * 128 - 37, 128, 1, 0.1), (4, 700, 128, 2, 0.5), (2, 64 * 9 + 5, 64, 3, 0.5)]:
        q, k, v, idx, cnt, nb = _case(H, N, b, seed, density)
        need = lib.bsga_attn_workspace_bytes(0, H, N, 64)
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        want = torch.empty_like(q); want_lse = torch.empty(H, N, dtype=torch.float32, device="cuda")
        got = torch.full_like(q, float("nan")); got_lse = torch.full_like(want_lse, float("nan"))
        rc = lib.bsga_sparse_attn(q.data_ptr(), k.data_ptr(), v.data_ptr(), 0, H, N, 64, b, 0.125, idx.data_ptr(),
                                  cnt.data_ptr(), nb, want.data_ptr(), want_lse.data_ptr(), ws.data_ptr(), need, st)
        assert rc == 0, lib.bsga_last_error()
        rc = lib.bsga_sparse_attn_noalloc(q.data_ptr(), k.data_ptr(), v.data_ptr(), 0, H, N, 64, b, 0.125,
                                          idx.data_ptr(), cnt.data_ptr(), nb, got.data_ptr(), got_lse.data_ptr(), st)
        assert rc == 0, lib.bsga_last_error()
        torch.cuda.synchronize()
        assert torch.equal(got, want) and torch.equal(got_lse, want_lse), (H, N, b)
        assert torch.isfinite(got.float()).all()


def test_noalloc_rejects_shapes_beyond_its_scratch():
    lib = _raw()
    a = 0x1000
    # 4096 heads x 2^20 tokens would need 4096 * (16384 + 1 + 32) * 4 bytes > 2 MiB; refused before any GPU work
    rc = lib.bsga_sparse_attn_noalloc(a, a, a, 0, 4096, 1 << 20, 64, 128, 0.125, a, a, 1 << 14, a, None, None)
    assert rc == 2 and b"scratch" in lib.bsga_last_error()
    rc = lib.bsga_sparse_attn_noalloc(a, a, a, 0, 4, 1000, 64, 128, 0.125, None, a, 8, a, None, None)
    assert rc == 1
