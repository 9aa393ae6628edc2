"""Out-of-bounds canaries: every output of every entry point is placed in the middle of a larger
buffer filled with a sentinel; after the call the guard regions must be untouched and the outputs
finite.  Shapes have ragged tails so that the last block / last tile paths run."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

GUARD = 4096  # bytes on each side


@pytest.fixture(scope="module")
def B():
    import paper_2509_07120_amd as pkg
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return pkg


class Guarded:
    """A tensor view of `shape` / `dtype` with GUARD bytes of 0xA5 before and after it."""

    def __init__(self, shape, dtype):
        n = int(np.prod(shape)) * torch.empty((), dtype=dtype).element_size()
        self.raw = torch.full((n + 2 * GUARD,), 0xA5, dtype=torch.uint8, device="cuda")
        self.view = self.raw[GUARD:GUARD + n].view(dtype).view(*shape)
        self.n = n

    def intact(self):
        return bool((self.raw[:GUARD] == 0xA5).all() and (self.raw[GUARD + self.n:] == 0xA5).all())


@pytest.mark.parametrize("dtype,block,N", [(torch.bfloat16, 128, 1000), (torch.bfloat16, 64, 333), (torch.float32, 64, 200),
                                           (torch.bfloat16, 128, 129)])
def test_no_entry_point_writes_outside_its_outputs(B, dtype, block, N):
    H = 3
    g = torch.Generator(device="cuda").manual_seed(N)
    q, k, v = (torch.randn((H, N, 64), device="cuda", generator=g).to(dtype) for _ in range(3))
    L, st = B.lib, torch.cuda.current_stream().cuda_stream
    code = 0 if dtype == torch.bfloat16 else 1
    nb = -(-N // block)
    words = -(-nb // 32)

    q_pool, k_pool = Guarded((H, nb, 64), torch.float64), Guarded((H, nb, 64), torch.float64)
    assert L.bsga_pool_qk(q.data_ptr(), k.data_ptr(), code, H, N, 64, block, q_pool.view.data_ptr(),
                          k_pool.view.data_ptr(), st) == 0

    bits, idx, cnt = Guarded((H, nb, words), torch.int32), Guarded((H, nb, nb), torch.int32), Guarded((H, nb), torch.int32)
    sel_ws = Guarded((B.bsga_select_workspace_bytes(H, nb, nb),), torch.uint8)
    assert L.bsga_select_blocks(q_pool.view.data_ptr(), k_pool.view.data_ptr(), H, nb, nb, 64, 0.125, 0.7, 0.9, None, None,
                                bits.view.data_ptr(), idx.view.data_ptr(), cnt.view.data_ptr(), nb,
                                sel_ws.view.data_ptr(), sel_ws.n, st) == 0

    out, lse = Guarded((H, N, 64), dtype), Guarded((H, N), torch.float32)
    att_ws = Guarded((max(B.bsga_attn_workspace_bytes(dtype, H, N), 16),), torch.uint8)
    assert L.bsga_sparse_attn(q.data_ptr(), k.data_ptr(), v.data_ptr(), code, H, N, 64, block, 0.125, idx.view.data_ptr(),
                              cnt.view.data_ptr(), nb, out.view.data_ptr(), lse.view.data_ptr(), att_ws.view.data_ptr(),
                              att_ws.n, st) == 0
    dout, dlse = Guarded((H, N, 64), dtype), Guarded((H, N), torch.float32)
    assert L.bsga_dense_attn(q.data_ptr(), k.data_ptr(), v.data_ptr(), code, H, N, 64, 0.125, dout.view.data_ptr(),
                             dlse.view.data_ptr(), None, 0, st) == 0

    index = torch.randperm(N, device="cuda", generator=g).to(torch.int32)[: N - 7].contiguous()
    gath = Guarded((H, N - 7, 64), dtype)
    assert L.bsga_gather_tokens(q.data_ptr(), code, H, N, 64, index.data_ptr(), N - 7, gath.view.data_ptr(), st) == 0
    torch.cuda.synchronize()

    for name, gbuf in [("q_pool", q_pool), ("k_pool", k_pool), ("mask_bits", bits), ("kv_idx", idx), ("kv_cnt", cnt),
                       ("select workspace", sel_ws), ("out", out), ("lse", lse), ("attention workspace", att_ws),
                       ("dense out", dout), ("dense lse", dlse), ("gather dst", gath)]:
        assert gbuf.intact(), f"{name}: guard bytes were overwritten"
    for t in (q_pool.view, k_pool.view, out.view.float(), lse.view, dout.view.float(), dlse.view, gath.view.float()):
        assert torch.isfinite(t).all()
    c = cnt.view
    assert int(c.min()) >= 1 and int(c.max()) <= nb


def test_half_tile_key_blocks_stay_in_bounds(B):
    H, N = 2, 777
    g = torch.Generator(device="cuda").manual_seed(1)
    q, k, v = (torch.randn((H, N, 64), device="cuda", generator=g).to(torch.bfloat16) for _ in range(3))
    nbq, nbk = -(-N // 128), -(-N // 64)
    keep = torch.rand((H, nbq, nbk), device="cuda", generator=g) < 0.5
    keep[..., -1] = True
    cnt = keep.sum(-1).to(torch.int32)
    idx = torch.argsort((~keep).to(torch.int8), dim=-1, stable=True).to(torch.int32).contiguous()
    out, lse = Guarded((H, N, 64), torch.bfloat16), Guarded((H, N), torch.float32)
    st = torch.cuda.current_stream().cuda_stream
    assert B.lib.bsga_sparse_attn_qk(q.data_ptr(), k.data_ptr(), v.data_ptr(), 0, H, N, 64, 128, 64, 0.125, idx.data_ptr(),
                                     cnt.data_ptr(), nbk, out.view.data_ptr(), lse.view.data_ptr(), None, 0, st) == 0
    torch.cuda.synchronize()
    assert out.intact() and lse.intact()
    assert torch.isfinite(out.view.float()).all() and torch.isfinite(lse.view).all()


def test_mfma_probe_runs_and_reports_a_plausible_rate(B):
    """The instruction-rate probe: finishes, and its rates are ordered as the hardware dictates (zero
    operands are not slower than random ones; extra vector work does not make the MFMAs faster)."""
    zero = B.bsga_probe_mfma(0, 0, iters=2000, repeats=2)
    rand = B.bsga_probe_mfma(1, 0, iters=2000, repeats=2)
    mix = min(B.bsga_probe_mfma(1, 1, iters=2000, repeats=2), B.bsga_probe_mfma(1, 2, iters=2000, repeats=2))
    print(f"mfma probe: zero {zero:.0f}, random {rand:.0f}, random + softmax arithmetic {mix:.0f} TFLOP/s")
    assert 300.0 < mix <= rand * 1.05 and rand <= zero * 1.05 and zero < 2600.0
