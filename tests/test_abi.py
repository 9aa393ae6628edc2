"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header
declares, and rejects bad arguments before touching a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "bsga.h")


@pytest.fixture(scope="module")
def B():
    import paper_2509_07120_amd as pkg
    return pkg


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bsga_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_are_exported(B):
    names = _declared_functions()
    assert set(names) == set(B.EXPORTED_SYMBOLS)
    raw = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(raw, n), n
    assert B.lib.bsga_version() == 3


def test_header_compiles_as_plain_c(tmp_path):
    src = tmp_path / "t.c"
    src.write_text('#include "bsga.h"\nint main(void){return BSGA_OK;}\n')
    import subprocess
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), "-c", str(src),
                    "-o", str(tmp_path / "t.o")], check=True)


def _err(B):
    return B.lib.bsga_last_error().decode()


A = 0x1000  # a fake, 16-byte aligned, non-null pointer; validation must fail before it is used


def test_pool_argument_errors(B):
    L = B.lib
    assert L.bsga_pool_qk(None, None, 0, 16, 100, 64, 64, None, None, None) == 1 and "nothing to pool" in _err(B)
    assert L.bsga_pool_qk(A, A, 7, 16, 100, 64, 64, A, A, None) == 1 and "dtype" in _err(B)
    assert L.bsga_pool_qk(A, A, 0, 0, 100, 64, 64, A, A, None) == 1 and "heads" in _err(B)
    assert L.bsga_pool_qk(A, A, 0, 16, 0, 64, 64, A, A, None) == 1 and "n_tokens" in _err(B)
    assert L.bsga_pool_qk(A, A, 0, 16, 100, 128, 64, A, A, None) == 2 and "head_dim" in _err(B)
    assert L.bsga_pool_qk(A, A, 0, 16, 100, 64, 32, A, A, None) == 2 and "block" in _err(B)
    assert L.bsga_pool_qk(A, A, 0, 16, 100, 64, 64, None, A, None) == 1 and "output" in _err(B)
    assert L.bsga_pool_qk(A + 4, A, 0, 16, 100, 64, 64, A, A, None) == 1 and "aligned" in _err(B)


def test_select_argument_errors(B):
    L = B.lib
    ok = dict(h=16, nbq=10, nbk=10, d=64, s=0.125, tau=0.9, rho=1.0)

    def call(q=A, k=A, h=16, nbq=10, nbk=10, d=64, s=0.125, tau=0.9, rho=1.0, bits=A, idx=A, cnt=A, stride=10, ws=A,
             wsb=1 << 30):
        return L.bsga_select_blocks(q, k, h, nbq, nbk, d, s, tau, rho, None, None, bits, idx, cnt, stride, ws, wsb,
                                    None)

    assert call(q=None) == 1
    assert call(nbk=0) == 1 and "nb_k" in _err(B)
    assert call(nbk=8193, stride=8193) == 2 and "8192" in _err(B)
    assert call(d=32) == 2
    assert call(tau=-0.1) == 1 and "tau" in _err(B)
    assert call(tau=float("nan")) == 1
    assert call(rho=1.5) == 1 and "rho" in _err(B)
    assert call(s=float("inf")) == 1
    assert call(stride=9) == 1 and "idx_stride" in _err(B)
    assert call(bits=None, idx=None, cnt=None) == 1 and "no output" in _err(B)
    assert call(ws=None) == 3 and "workspace" in _err(B)
    assert call(wsb=16 * 10 * 10 * 8 - 1) == 3 and "12800 needed" in _err(B)


def test_gather_argument_errors(B):
    L = B.lib
    assert L.bsga_gather_tokens(None, 0, 16, 100, 64, A, 100, A, None) == 1
    assert L.bsga_gather_tokens(A, 0, 16, 100, 64, None, 100, A, None) == 1 and "index" in _err(B)
    assert L.bsga_gather_tokens(A, 2, 16, 100, 64, A, 100, A, None) == 1 and "dtype" in _err(B)
    assert L.bsga_gather_tokens(A, 0, 16, 100, 32, A, 100, A, None) == 2
    assert L.bsga_gather_tokens(A, 0, 16, 0, 64, A, 100, A, None) == 1 and "n_src" in _err(B)
    assert L.bsga_gather_tokens(A, 0, 16, 100, 64, A, -1, A, None) == 1 and "n_dst" in _err(B)
    assert L.bsga_gather_tokens(A, 0, 16, 100, 64, A, 0, A, None) == 0  # nothing to do, nothing launched


def test_attention_argument_errors(B):
    L = B.lib

    def sparse(q=A, k=A, v=A, dt=0, h=16, n=1000, d=64, b=128, sc=0.125, idx=A, cnt=A, stride=8, out=A, ws=A,
               wsb=1 << 30):
        return L.bsga_sparse_attn(q, k, v, dt, h, n, d, b, sc, idx, cnt, stride, out, None, ws, wsb, None)

    assert sparse(idx=None) == 1 and "kv_idx" in _err(B)
    assert sparse(v=None) == 1
    assert sparse(b=32) == 2
    assert sparse(sc=0.0) == 1 and "softmax_scale" in _err(B)
    assert sparse(stride=7) == 1 and "idx_stride" in _err(B)
    assert sparse(n=(1 << 24) + 1, stride=1 << 20) == 2
    assert L.bsga_dense_attn(A, A, A, 0, 16, 1000, 64, 0.125, None, None, A, 1 << 30, None) == 1
    assert L.bsga_dense_attn(A, A, A, 3, 16, 1000, 64, 0.125, A, None, A, 1 << 30, None) == 1


def test_workspace_size(B):
    """Attention keeps every intermediate on chip; the sparse bf16 kernel wants 4 bytes per query block."""
    import torch
    assert B.bsga_attn_workspace_bytes(torch.bfloat16, 16, 137400) == (16 * (2147 + 1) + 32 * 16 + 4) * 4  # one spare block for a split sequence
    assert B.bsga_attn_workspace_bytes(torch.float32, 16, 137400) == 0
    # selection keeps the float64 block logits between its two kernels
    assert B.bsga_select_workspace_bytes(16, 1074, 1074) == 16 * 1074 * 1074 * 8
    assert B.bsga_select_workspace_bytes(0, 10, 10) == 0
    assert B.bsga_attn_workspace_bytes(torch.float32, 16, 2748) == 0
    assert B.lib.bsga_attn_workspace_bytes(0, 0, 100, 64) == 0


def test_split_argument_errors(B):
    L = B.lib
    assert L.bsga_pool_qk_split(A, A, 0, 16, 100, 101, 64, 64, A, A, None) == 1 and "n_first" in _err(B)
    assert L.bsga_pool_qk_split(A, A, 0, 16, 100, -1, 64, 64, A, A, None) == 1 and "n_first" in _err(B)
    args = (A, A, A, 0, 16, 1000)
    assert L.bsga_sparse_attn_split(*args, 1001, 64, 128, 128, 0.125, A, A, 16, A, None, None, 0, None) == 1
    assert "n_first" in _err(B)
    # 1000 tokens split at 130: key blocks of 128 -> 2 + 7 = 9 blocks, so a stride of 8 is too short
    assert L.bsga_sparse_attn_split(*args, 130, 64, 128, 128, 0.125, A, A, 8, A, None, None, 0, None) == 1
    assert "idx_stride" in _err(B)
    assert L.bsga_sparse_attn_split(*args, 130, 64, 64, 128, 0.125, A, A, 16, A, None, None, 0, None) == 2
    assert L.bsga_sparse_attn_split(*args, 130, 64, 128, 128, 0.125, None, A, 16, A, None, None, 0, None) == 1


def test_probe_argument_errors(B):
    L = B.lib
    assert L.bsga_probe_mfma(2, 0, 10, A, 1 << 20, None, None) == 1 and "operands" in _err(B)
    assert L.bsga_probe_mfma(0, 0, 0, A, 1 << 20, None, None) == 1 and "iters" in _err(B)
    assert L.bsga_probe_mfma(0, 0, 10, None, 1 << 20, None, None) == 1 and "sink" in _err(B)
