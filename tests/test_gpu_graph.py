"""The whole layer under HIP graph capture.  The library allocates nothing, never synchronises and
records no memset, so a caller with preallocated buffers can capture pool -> select -> block-sparse
attention (Sec. 4.1) once and replay it.  The graph is replayed several times, with eager work and
synchronisations in between and with new contents in the input buffers, and every replay must
reproduce the eager results bit for bit."""
import numpy as np
import pytest
import torch

from workload import CONFIGS, generate
from tests.helpers import to_device

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import paper_2509_07120_amd as pkg
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return pkg


def _buffers(B, q, nb):
    H, N, d = q.shape
    t = torch
    return {
        "pool": (t.empty((H, nb, d), dtype=t.float64, device="cuda"), t.empty((H, nb, d), dtype=t.float64, device="cuda")),
        "sel_ws": t.empty(B.bsga_select_workspace_bytes(H, nb, nb), dtype=t.uint8, device="cuda"),
        "sel": (t.empty((H, nb, (nb + 31) // 32), dtype=t.int32, device="cuda"),
                t.empty((H, nb, nb), dtype=t.int32, device="cuda"), t.empty((H, nb), dtype=t.int32, device="cuda")),
        "ws": t.empty(max(B.bsga_attn_workspace_bytes(q.dtype, H, N, d), 16), dtype=t.uint8, device="cuda"),
        "out": t.empty_like(q),
        "out2": t.empty_like(q),
    }


@pytest.mark.parametrize("use_noalloc", [False, True])
def test_layer_replays_from_a_graph(B, use_noalloc):
    cfg = CONFIGS[3]                                   # 32 frames, block 128; 4 heads x 344 blocks: launch order in use
    data = [tuple(to_device(x, cfg.dtype) for x in generate(cfg, base_seed=s, heads=4)) for s in (0, 7)]
    q, k, v = (x.clone() for x in data[0])             # the buffers the graph reads
    buf = _buffers(B, q, cfg.n_blocks)
    tau = 0.9

    def layer(out):
        qp, kp = B.bsga_pool_qk(q, k, cfg.block, out=buf["pool"])
        bits, idx, cnt = B.bsga_select_blocks(qp, kp, tau, 1.0, workspace=buf["sel_ws"], out=buf["sel"])
        if use_noalloc:
            B.bsga_sparse_attn_noalloc(q, k, v, cfg.block, idx, cnt, out)
        else:
            B.bsga_sparse_attn(q, k, v, cfg.block, idx, cnt, out=out, workspace=buf["ws"])

    def eager(inputs):
        for dst, src in zip((q, k, v), inputs):
            dst.copy_(src)
        layer(buf["out2"])
        torch.cuda.synchronize()
        return buf["out2"].clone(), buf["sel"][0].clone(), buf["sel"][2].clone()

    want = [eager(d) for d in data]                    # also the library's one-time set-up, outside the capture
    assert not torch.equal(want[0][0], want[1][0])
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        layer(buf["out"])
    for rep, which in enumerate((0, 1, 1, 0, 1)):
        for dst, src in zip((q, k, v), data[which]):
            dst.copy_(src)
        buf["out"].fill_(float("nan"))
        buf["sel"][2].zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        out_w, bits_w, cnt_w = want[which]
        assert torch.equal(buf["sel"][0], bits_w), rep
        assert torch.equal(buf["sel"][2], cnt_w), rep
        assert torch.equal(buf["out"], out_w), rep
        # eager work between replays (another stream of launches through the same library state)
        B.bsga_dense_attn(q[:1, :4096], k[:1, :4096], v[:1, :4096])
        torch.cuda.synchronize()
