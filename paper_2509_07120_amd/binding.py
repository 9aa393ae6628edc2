"""ctypes binding of libbsga.so: argument marshalling only.

Every function here forwards to the C-ABI entry point of the same name with
device pointers taken from torch tensors and the current torch HIP stream.
Outputs and workspaces are torch tensors (torch is the device allocator and
stream provider, nothing else); all arithmetic happens in the HIP kernels.
There is no fallback path: if the library is missing or a call fails, an
exception is raised.
"""
from __future__ import annotations

import ctypes
import math
import os
from typing import Optional, Tuple

import torch

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG_DIR, "libbsga.so")

BSGA_OK = 0
BSGA_ERR_INVALID_ARG = 1
BSGA_ERR_UNSUPPORTED = 2
BSGA_ERR_WORKSPACE = 3
BSGA_ERR_HIP = 4
BSGA_BF16 = 0
BSGA_FP32 = 1

EXPORTED_SYMBOLS = (
    "bsga_version",
    "bsga_last_error",
    "bsga_pool_qk",
    "bsga_pool_qk_split",
    "bsga_select_workspace_bytes",
    "bsga_select_blocks",
    "bsga_gather_tokens",
    "bsga_attn_workspace_bytes",
    "bsga_sparse_attn",
    "bsga_sparse_attn_noalloc",
    "bsga_noalloc_scratch_bytes",
    "bsga_sparse_attn_qk",
    "bsga_sparse_attn_split",
    "bsga_dense_attn",
    "bsga_probe_mfma",
)


class BsgaError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"bsga error {code}: {message}")
        self.code = code
        self.message = message


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'` "
            "or `python paper_2509_07120_amd/build.py` first (there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    c_void_p, c_int, c_int64, c_double, c_float, c_size_t = (
        ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_double, ctypes.c_float, ctypes.c_size_t)
    lib.bsga_version.restype = c_int
    lib.bsga_version.argtypes = []
    lib.bsga_last_error.restype = ctypes.c_char_p
    lib.bsga_last_error.argtypes = []
    lib.bsga_pool_qk.restype = c_int
    lib.bsga_pool_qk.argtypes = [c_void_p, c_void_p, c_int, c_int, c_int64, c_int, c_int, c_void_p, c_void_p, c_void_p]
    lib.bsga_pool_qk_split.restype = c_int
    lib.bsga_pool_qk_split.argtypes = [c_void_p, c_void_p, c_int, c_int, c_int64, c_int64, c_int, c_int, c_void_p,
                                       c_void_p, c_void_p]
    lib.bsga_select_blocks.restype = c_int
    lib.bsga_select_blocks.argtypes = [c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_double, c_double, c_double,
                                       c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_void_p, c_size_t,
                                       c_void_p]
    lib.bsga_select_workspace_bytes.restype = c_size_t
    lib.bsga_select_workspace_bytes.argtypes = [c_int, c_int, c_int]
    lib.bsga_gather_tokens.restype = c_int
    lib.bsga_gather_tokens.argtypes = [c_void_p, c_int, c_int, c_int64, c_int, c_void_p, c_int64, c_void_p, c_void_p]
    lib.bsga_attn_workspace_bytes.restype = c_size_t
    lib.bsga_attn_workspace_bytes.argtypes = [c_int, c_int, c_int64, c_int]
    lib.bsga_sparse_attn.restype = c_int
    lib.bsga_sparse_attn.argtypes = [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int64, c_int, c_int, c_float,
                                     c_void_p, c_void_p, c_int, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
    lib.bsga_sparse_attn_noalloc.restype = c_int
    lib.bsga_sparse_attn_noalloc.argtypes = [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int64, c_int, c_int, c_float,
                                             c_void_p, c_void_p, c_int, c_void_p, c_void_p, c_void_p]
    lib.bsga_noalloc_scratch_bytes.restype = c_size_t
    lib.bsga_noalloc_scratch_bytes.argtypes = []
    lib.bsga_sparse_attn_qk.restype = c_int
    lib.bsga_sparse_attn_qk.argtypes = [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int64, c_int, c_int, c_int, c_float,
                                        c_void_p, c_void_p, c_int, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
    lib.bsga_sparse_attn_split.restype = c_int
    lib.bsga_sparse_attn_split.argtypes = [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int64, c_int64, c_int, c_int,
                                           c_int, c_float, c_void_p, c_void_p, c_int, c_void_p, c_void_p, c_void_p,
                                           c_size_t, c_void_p]
    lib.bsga_dense_attn.restype = c_int
    lib.bsga_dense_attn.argtypes = [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int64, c_int, c_float,
                                    c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
    lib.bsga_probe_mfma.restype = c_int
    lib.bsga_probe_mfma.argtypes = [c_int, c_int, c_int, c_void_p, c_size_t, ctypes.POINTER(c_double), c_void_p]
    return lib


lib = _load()


def _check(rc: int) -> None:
    if rc != BSGA_OK:
        raise BsgaError(rc, lib.bsga_last_error().decode())


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(t: torch.Tensor) -> int:
    return torch.cuda.current_stream(t.device).cuda_stream


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return BSGA_BF16
    if t.dtype == torch.float32:
        return BSGA_FP32
    raise TypeError(f"unsupported dtype {t.dtype}: bsga takes bfloat16 or float32")


def _require(t: torch.Tensor, name: str, dtype=None) -> None:
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")


def num_blocks(n_tokens: int, block: int) -> int:
    return (n_tokens + block - 1) // block


def bsga_pool_qk(q: torch.Tensor, k: torch.Tensor, block: int,
                 out: Optional[Tuple[torch.Tensor, torch.Tensor]] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """q, k [H, N, 64] -> (q_pool, k_pool) [H, ceil(N/block), 64] float64 (written into `out` if given)."""
    _require(q, "q"); _require(k, "k", q.dtype)
    if q.shape != k.shape or q.dim() != 3:
        raise ValueError("q and k must both be [heads, n_tokens, head_dim]")
    H, N, d = q.shape
    nb = num_blocks(N, block)
    if out is None:
        q_pool = torch.empty((H, nb, d), dtype=torch.float64, device=q.device)
        k_pool = torch.empty_like(q_pool)
    else:
        q_pool, k_pool = out
        for t in (q_pool, k_pool):
            _require(t, "out", torch.float64)
            if tuple(t.shape) != (H, nb, d):
                raise ValueError(f"out tensors must be {(H, nb, d)}")
    _check(lib.bsga_pool_qk(_ptr(q), _ptr(k), _dtype_code(q), H, N, d, block, _ptr(q_pool), _ptr(k_pool), _stream(q)))
    return q_pool, k_pool


def split_blocks(n_tokens: int, n_first: int, block: int) -> int:
    """Blocks of a sequence whose parts [0, n_first) and [n_first, n_tokens) are blocked separately."""
    return num_blocks(n_first, block) + num_blocks(n_tokens - n_first, block)


def bsga_pool_qk_split(q: torch.Tensor, k: torch.Tensor, block: int, n_first: int,
                       out: Optional[Tuple[torch.Tensor, torch.Tensor]] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """As bsga_pool_qk for a sequence split at token n_first: no block crosses n_first."""
    _require(q, "q"); _require(k, "k", q.dtype)
    if q.shape != k.shape or q.dim() != 3:
        raise ValueError("q and k must both be [heads, n_tokens, head_dim]")
    H, N, d = q.shape
    nb = split_blocks(N, n_first, block) if 0 <= n_first <= N else 1
    if out is None:
        q_pool = torch.empty((H, nb, d), dtype=torch.float64, device=q.device)
        k_pool = torch.empty_like(q_pool)
    else:
        q_pool, k_pool = out
        for t in (q_pool, k_pool):
            _require(t, "out", torch.float64)
            if tuple(t.shape) != (H, nb, d):
                raise ValueError(f"out tensors must be {(H, nb, d)}")
    _check(lib.bsga_pool_qk_split(_ptr(q), _ptr(k), _dtype_code(q), H, N, n_first, d, block, _ptr(q_pool),
                                  _ptr(k_pool), _stream(q)))
    return q_pool, k_pool


def bsga_pool(x: torch.Tensor, block: int) -> torch.Tensor:
    """x [H, N, 64] -> block means [H, ceil(N/block), 64] float64 (one tensor; for separate q / k block sizes)."""
    _require(x, "x")
    H, N, d = x.shape
    pooled = torch.empty((H, num_blocks(N, block), d), dtype=torch.float64, device=x.device)
    _check(lib.bsga_pool_qk(_ptr(x), None, _dtype_code(x), H, N, d, block, _ptr(pooled), None, _stream(x)))
    return pooled


def bsga_select_blocks(q_pool: torch.Tensor, k_pool: torch.Tensor, tau: float, rho: float = 1.0,
                       score_scale: Optional[float] = None, force_q: Optional[torch.Tensor] = None,
                       force_k: Optional[torch.Tensor] = None, want_bits: bool = True,
                       workspace: Optional[torch.Tensor] = None, out=None):
    """Pooled Q/K -> (mask_bits [H,nbq,ceil(nbk/32)] uint32-as-int32, kv_idx [H,nbq,nbk] int32, kv_cnt [H,nbq] int32).
    `workspace`: optional device byte buffer of bsga_select_workspace_bytes(H, nbq, nbk) bytes (allocated if absent).
    `out`: optional (mask_bits or None, kv_idx, kv_cnt) tensors of those shapes to write into."""
    _require(q_pool, "q_pool", torch.float64); _require(k_pool, "k_pool", torch.float64)
    H, nbq, d = q_pool.shape
    nbk = k_pool.shape[1]
    if score_scale is None:
        score_scale = 1.0 / math.sqrt(d)
    dev = q_pool.device
    words = (nbk + 31) // 32
    if out is None:
        # every word of every row is written by the kernel, so nothing needs to be cleared
        mask_bits = torch.empty((H, nbq, words), dtype=torch.int32, device=dev) if want_bits else None
        kv_idx = torch.empty((H, nbq, nbk), dtype=torch.int32, device=dev)
        kv_cnt = torch.empty((H, nbq), dtype=torch.int32, device=dev)
    else:
        mask_bits, kv_idx, kv_cnt = out
        for t, shape, name in ((mask_bits, (H, nbq, words), "mask_bits"), (kv_idx, (H, nbq, nbk), "kv_idx"),
                               (kv_cnt, (H, nbq), "kv_cnt")):
            if t is None and name == "mask_bits":
                continue
            _require(t, name, torch.int32)
            if tuple(t.shape) != shape:
                raise ValueError(f"{name} must be {shape}, got {tuple(t.shape)}")
    if force_q is not None:
        _require(force_q, "force_q", torch.uint8)
    if force_k is not None:
        _require(force_k, "force_k", torch.uint8)
    if workspace is None:
        workspace = torch.empty(bsga_select_workspace_bytes(H, nbq, nbk), dtype=torch.uint8, device=dev)
    ws_bytes = workspace.numel() * workspace.element_size()
    _check(lib.bsga_select_blocks(_ptr(q_pool), _ptr(k_pool), H, nbq, nbk, d, float(score_scale), float(tau),
                                  float(rho), _ptr(force_q), _ptr(force_k), _ptr(mask_bits), _ptr(kv_idx),
                                  _ptr(kv_cnt), nbk, _ptr(workspace), ws_bytes, _stream(q_pool)))
    return mask_bits, kv_idx, kv_cnt


def bsga_select_workspace_bytes(heads: int, nb_q: int, nb_k: int) -> int:
    return int(lib.bsga_select_workspace_bytes(heads, nb_q, nb_k))


def bsga_attn_workspace_bytes(dtype: torch.dtype, heads: int, n_tokens: int, head_dim: int = 64) -> int:
    code = BSGA_BF16 if dtype == torch.bfloat16 else BSGA_FP32
    return int(lib.bsga_attn_workspace_bytes(code, heads, n_tokens, head_dim))


def _workspace(q: torch.Tensor, workspace: Optional[torch.Tensor]) -> Tuple[Optional[torch.Tensor], int]:
    H, N, d = q.shape
    need = bsga_attn_workspace_bytes(q.dtype, H, N, d)
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    return workspace, nbytes


def bsga_sparse_attn(q, k, v, block: int, kv_idx: torch.Tensor, kv_cnt: torch.Tensor,
                     softmax_scale: Optional[float] = None, return_lse: bool = False,
                     out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                     ordered: bool = True, block_k: Optional[int] = None):
    """Attention of each query block over its kept key blocks; returns O (and lse).
    ordered = False passes no workspace: rows are launched in index order, not heaviest first.
    block_k: size of the key blocks the lists refer to when it differs from the query block size."""
    _require(q, "q"); _require(k, "k", q.dtype); _require(v, "v", q.dtype)
    _require(kv_idx, "kv_idx", torch.int32); _require(kv_cnt, "kv_cnt", torch.int32)
    H, N, d = q.shape
    if softmax_scale is None:
        softmax_scale = 1.0 / math.sqrt(d)
    if out is None:
        out = torch.empty_like(q)
    lse = torch.empty((H, N), dtype=torch.float32, device=q.device) if return_lse else None
    workspace, ws_bytes = _workspace(q, workspace) if ordered else (None, 0)
    if block_k is None or block_k == block:
        _check(lib.bsga_sparse_attn(_ptr(q), _ptr(k), _ptr(v), _dtype_code(q), H, N, d, block, float(softmax_scale),
                                    _ptr(kv_idx), _ptr(kv_cnt), kv_idx.shape[-1], _ptr(out), _ptr(lse),
                                    _ptr(workspace), ws_bytes, _stream(q)))
    else:
        _check(lib.bsga_sparse_attn_qk(_ptr(q), _ptr(k), _ptr(v), _dtype_code(q), H, N, d, block, block_k,
                                       float(softmax_scale), _ptr(kv_idx), _ptr(kv_cnt), kv_idx.shape[-1], _ptr(out),
                                       _ptr(lse), _ptr(workspace), ws_bytes, _stream(q)))
    return (out, lse) if return_lse else out


def bsga_noalloc_scratch_bytes() -> int:
    return int(lib.bsga_noalloc_scratch_bytes())


def bsga_sparse_attn_noalloc(q, k, v, block: int, kv_idx: torch.Tensor, kv_cnt: torch.Tensor, out: torch.Tensor,
                             softmax_scale: Optional[float] = None, lse: Optional[torch.Tensor] = None):
    """bsga_sparse_attn on the library's built-in scratch: nothing is allocated here either (the
    caller passes `out`, and `lse` [H, N] float32 if wanted)."""
    _require(q, "q"); _require(k, "k", q.dtype); _require(v, "v", q.dtype); _require(out, "out", q.dtype)
    _require(kv_idx, "kv_idx", torch.int32); _require(kv_cnt, "kv_cnt", torch.int32)
    H, N, d = q.shape
    if softmax_scale is None:
        softmax_scale = 1.0 / math.sqrt(d)
    _check(lib.bsga_sparse_attn_noalloc(_ptr(q), _ptr(k), _ptr(v), _dtype_code(q), H, N, d, block, float(softmax_scale),
                                        _ptr(kv_idx), _ptr(kv_cnt), kv_idx.shape[-1], _ptr(out), _ptr(lse), _stream(q)))
    return out


def bsga_sparse_attn_split(q, k, v, block: int, n_first: int, kv_idx: torch.Tensor, kv_cnt: torch.Tensor,
                           softmax_scale: Optional[float] = None, return_lse: bool = False,
                           out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                           block_k: Optional[int] = None):
    """As bsga_sparse_attn for a sequence split at token n_first (blocks as in bsga_pool_qk_split)."""
    _require(q, "q"); _require(k, "k", q.dtype); _require(v, "v", q.dtype)
    _require(kv_idx, "kv_idx", torch.int32); _require(kv_cnt, "kv_cnt", torch.int32)
    H, N, d = q.shape
    if softmax_scale is None:
        softmax_scale = 1.0 / math.sqrt(d)
    if out is None:
        out = torch.empty_like(q)
    lse = torch.empty((H, N), dtype=torch.float32, device=q.device) if return_lse else None
    workspace, ws_bytes = _workspace(q, workspace)
    _check(lib.bsga_sparse_attn_split(_ptr(q), _ptr(k), _ptr(v), _dtype_code(q), H, N, n_first, d, block,
                                      block if block_k is None else block_k, float(softmax_scale), _ptr(kv_idx),
                                      _ptr(kv_cnt), kv_idx.shape[-1], _ptr(out), _ptr(lse), _ptr(workspace), ws_bytes,
                                      _stream(q)))
    return (out, lse) if return_lse else out


def bsga_dense_attn(q, k, v, softmax_scale: Optional[float] = None, return_lse: bool = False,
                    out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                    balanced: bool = True):
    """Dense softmax attention baseline; returns O (and lse).
    balanced = False passes no workspace: every row is then computed by the workgroup of its number
    instead of the last rows being handed out at run time."""
    _require(q, "q"); _require(k, "k", q.dtype); _require(v, "v", q.dtype)
    H, N, d = q.shape
    if softmax_scale is None:
        softmax_scale = 1.0 / math.sqrt(d)
    if out is None:
        out = torch.empty_like(q)
    lse = torch.empty((H, N), dtype=torch.float32, device=q.device) if return_lse else None
    workspace, ws_bytes = _workspace(q, workspace) if balanced else (None, 0)
    _check(lib.bsga_dense_attn(_ptr(q), _ptr(k), _ptr(v), _dtype_code(q), H, N, d, float(softmax_scale),
                               _ptr(out), _ptr(lse), _ptr(workspace), ws_bytes, _stream(q)))
    return (out, lse) if return_lse else out


def sparse_global_attention(q, k, v, block: int, tau: float, rho: float = 1.0,
                            score_scale: Optional[float] = None, softmax_scale: Optional[float] = None,
                            workspace: Optional[torch.Tensor] = None):
    """The whole layer: pool -> select -> block-sparse attention.  Returns (O, kv_idx, kv_cnt, mask_bits)."""
    q_pool, k_pool = bsga_pool_qk(q, k, block)
    mask_bits, kv_idx, kv_cnt = bsga_select_blocks(q_pool, k_pool, tau, rho, score_scale)
    out = bsga_sparse_attn(q, k, v, block, kv_idx, kv_cnt, softmax_scale, workspace=workspace)
    return out, kv_idx, kv_cnt, mask_bits


def bsga_gather_tokens(x: torch.Tensor, index: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """out[h, i] = x[h, index[i]] for x [H, N, 64] and an int32 device index [n_out]."""
    _require(x, "x"); _require(index, "index", torch.int32)
    H, N, d = x.shape
    n_out = index.numel()
    if out is None:
        out = torch.empty((H, n_out, d), dtype=x.dtype, device=x.device)
    _check(lib.bsga_gather_tokens(_ptr(x), _dtype_code(x), H, N, d, _ptr(index), n_out, _ptr(out), _stream(x)))
    return out


class SpecialTokenPlan:
    """Index bookkeeping for the special-token split (Sec. 4.2), built once per sequence layout.

    The working order puts the patch tokens X_p first (in their original order) and the special
    tokens X_s last, and the two parts are blocked separately (the *_split entry points with
    n_first = N_p): blocks 0 .. n_patch_blocks-1, n_patch_blocks = ceil(N_p / block), hold every patch
    token and nothing else (the last of them may be ragged); they are the blocks the map is predicted
    on.  The blocks after them hold the special tokens, which attend and are attended densely:
    force_q = 1, force_k = 2 (kept, not ranked)."""

    def __init__(self, special: torch.Tensor, block: int, device):
        special = torch.as_tensor(special, dtype=torch.bool).cpu()
        n = special.numel()
        order = torch.cat([torch.nonzero(~special).flatten(), torch.nonzero(special).flatten()])
        inverse = torch.empty_like(order)
        inverse[order] = torch.arange(n)
        self.n_tokens = n
        self.block = block
        self.n_patch = int((~special).sum())
        self.n_patch_blocks = num_blocks(self.n_patch, block)
        nb = split_blocks(n, self.n_patch, block)
        self.n_blocks = nb
        dense = torch.arange(nb) >= self.n_patch_blocks
        self.perm = order.to(torch.int32).to(device)
        self.inverse = inverse.to(torch.int32).to(device)
        self.force_q = dense.to(torch.uint8).to(device)
        self.force_k = (dense.to(torch.uint8) * 2).to(device)


def sparse_global_attention_special(q, k, v, plan: SpecialTokenPlan, tau: float, rho: float = 1.0,
                                    score_scale: Optional[float] = None, softmax_scale: Optional[float] = None):
    """The layer with the special-token split: gather into the working order, pool, select on the
    patch blocks only, block-sparse attention, gather back.  Returns (O in the caller's token order,
    kv_idx, kv_cnt, mask_bits); the lists refer to blocks of the working order."""
    qw, kw, vw = (bsga_gather_tokens(x, plan.perm) for x in (q, k, v))
    q_pool, k_pool = bsga_pool_qk_split(qw, kw, plan.block, plan.n_patch)
    mask_bits, kv_idx, kv_cnt = bsga_select_blocks(q_pool, k_pool, tau, rho, score_scale, force_q=plan.force_q,
                                                   force_k=plan.force_k)
    ow = bsga_sparse_attn_split(qw, kw, vw, plan.block, plan.n_patch, kv_idx, kv_cnt, softmax_scale)
    return bsga_gather_tokens(ow, plan.inverse), kv_idx, kv_cnt, mask_bits


def bsga_probe_mfma(operands: int, softmax_mix: int, iters: int = 20000, repeats: int = 3) -> float:
    """Sustained TFLOP/s of the attention kernels' MFMA instruction with no memory traffic (see
    bsga_probe_mfma in the header).  Times `repeats` launches with events and returns the best."""
    dev = torch.device("cuda", torch.cuda.current_device())
    sink = torch.empty(2 * torch.cuda.get_device_properties(dev).multi_processor_count * 256, dtype=torch.float32, device=dev)
    flops = ctypes.c_double(0.0)
    stream = torch.cuda.current_stream(dev).cuda_stream
    best = 0.0
    for r in range(repeats + 1):  # the first launch is a warm-up
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        _check(lib.bsga_probe_mfma(int(operands), int(softmax_mix), int(iters), _ptr(sink), sink.numel() * 4,
                                   ctypes.byref(flops), stream))
        e1.record()
        torch.cuda.synchronize(dev)
        if r > 0:
            best = max(best, flops.value / (e0.elapsed_time(e1) * 1e-3) / 1e12)
    return best
