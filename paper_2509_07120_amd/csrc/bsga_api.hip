// C-ABI entry points of libbsga: argument validation and dispatch to the kernel launchers.
// Validation runs before any HIP call, so argument errors are reported on machines without a GPU.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>

#include <mutex>

#include "bsga_internal.h"

// Scratch of bsga_sparse_attn_noalloc: the launch order of the (head, query block) rows and the
// class table that builds it.  Every GPU the library runs on holds its own copy for the life of the
// process; host code reaches it only through the per-device address taken below, never by name.
constexpr size_t kStaticScratchBytes = size_t(2) << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace bsga {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

void clear_error() { g_err[0] = '\0'; }

int check_hip(hipError_t e, const char* what) {
  if (e == hipSuccess) return BSGA_OK;
  return fail(BSGA_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static int check_shape(const char* fn, int dtype, int heads, int64_t n_tokens, int head_dim) {
  if (dtype != BSGA_BF16 && dtype != BSGA_FP32)
    return fail(BSGA_ERR_INVALID_ARG, "%s: dtype must be BSGA_BF16 (0) or BSGA_FP32 (1), got %d", fn, dtype);
  if (heads < 1 || heads > 65535)
    return fail(BSGA_ERR_INVALID_ARG, "%s: heads must be in [1, 65535], got %d", fn, heads);
  if (n_tokens < 1) return fail(BSGA_ERR_INVALID_ARG, "%s: n_tokens must be >= 1, got %lld", fn, (long long)n_tokens);
  if (n_tokens > (int64_t(1) << 24))
    return fail(BSGA_ERR_UNSUPPORTED, "%s: n_tokens above 2^24 is not supported, got %lld", fn, (long long)n_tokens);
  if (head_dim != 64) return fail(BSGA_ERR_UNSUPPORTED, "%s: head_dim must be 64, got %d", fn, head_dim);
  return BSGA_OK;
}

static int check_block(const char* fn, int block) {
  if (block != 64 && block != 128)
    return fail(BSGA_ERR_UNSUPPORTED, "%s: block must be 64 or 128, got %d", fn, block);
  return BSGA_OK;
}

static size_t attn_workspace(int dtype, int heads, int64_t n_tokens) {
  // Q, K and V are read in place and every intermediate stays on chip; the only scratch is the
  // launch order of the (head, query block) rows of the sparse bf16 kernel: one int32 per row, sized
  // for the smaller block size (plus one block for a split sequence), plus a [32 classes][heads] table.
  if (dtype != BSGA_BF16) return 0;
  return (static_cast<size_t>(heads) * static_cast<size_t>(ceil_div(n_tokens, 64) + 1) + 32u * static_cast<size_t>(heads) + 4u) *
         sizeof(int32_t);
}

static int attn_common(const char* fn, const void* q, const void* k, const void* v, int dtype, int heads,
                       int64_t n_tokens, int64_t n_first, int head_dim, int block, int block_k, float softmax_scale,
                       const int32_t* kv_idx, const int32_t* kv_cnt, int idx_stride, void* out, float* lse,
                       void* workspace, size_t workspace_bytes, void* stream) {
  clear_error();
  if (int rc = check_shape(fn, dtype, heads, n_tokens, head_dim)) return rc;
  if (int rc = check_block(fn, block)) return rc;
  if (n_first < 0 || n_first > n_tokens)
    return fail(BSGA_ERR_INVALID_ARG, "%s: n_first must be in [0, n_tokens], got %lld", fn, (long long)n_first);
  if (block_k != block) {
    if (!(block == 128 && block_k == 64))
      return fail(BSGA_ERR_UNSUPPORTED, "%s: key blocks must have the query block size, or 64 with query blocks of 128 (got %d / %d)",
                  fn, block, block_k);
    if (dtype != BSGA_BF16)
      return fail(BSGA_ERR_UNSUPPORTED, "%s: separate query / key block sizes are implemented for bf16 only", fn);
  }
  if (!q || !k || !v || !out) return fail(BSGA_ERR_INVALID_ARG, "%s: q, k, v and out must be non-null", fn);
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out))
    return fail(BSGA_ERR_INVALID_ARG, "%s: q, k, v and out must be 16-byte aligned", fn);
  if (!(softmax_scale > 0.0f) || !isfinite(softmax_scale))
    return fail(BSGA_ERR_INVALID_ARG, "%s: softmax_scale must be finite and > 0", fn);
  const int64_t nb = split_blocks(n_tokens, n_first, block_k);
  if (kv_idx || kv_cnt) {
    if (!kv_idx || !kv_cnt) return fail(BSGA_ERR_INVALID_ARG, "%s: kv_idx and kv_cnt must both be given", fn);
    if (idx_stride < nb)
      return fail(BSGA_ERR_INVALID_ARG, "%s: idx_stride (%d) must be >= number of key blocks (%lld)", fn, idx_stride,
                  (long long)nb);
  }
  const size_t need = kv_idx ? attn_workspace(dtype, heads, n_tokens) : 0;  // the dense kernel needs none
  if (need > 0 && workspace) {  // without a workspace the rows are launched in index order
    if (workspace_bytes < need)
      return fail(BSGA_ERR_WORKSPACE, "%s: workspace has %zu bytes, %zu needed", fn, workspace_bytes, need);
    if (!aligned16(workspace)) return fail(BSGA_ERR_INVALID_ARG, "%s: workspace must be 16-byte aligned", fn);
  }
  // the dense kernel uses a workspace, if it gets one, for one counter (balancing rows across the XCDs)
  if (!kv_idx && workspace && (workspace_bytes < 16 || !aligned16(workspace))) workspace = nullptr;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (dtype == BSGA_BF16)
    return launch_attn_bf16(q, k, v, heads, n_tokens, n_first, block, block_k, softmax_scale, kv_idx, kv_cnt, idx_stride, out, lse,
                            workspace, s);
  return launch_attn_fp32(static_cast<const float*>(q), static_cast<const float*>(k), static_cast<const float*>(v),
                          heads, n_tokens, n_first, block, softmax_scale, kv_idx, kv_cnt, idx_stride,
                          static_cast<float*>(out), lse, s);
}

// Device address of `scratch` on the current device, looked up once per device.
static int static_scratch(const char* fn, void** ptr) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* addr[kMaxDevices] = {};
  int dev = -1;
  if (int rc = check_hip(hipGetDevice(&dev), "hipGetDevice")) return rc;
  if (dev < 0 || dev >= kMaxDevices)
    return fail(BSGA_ERR_UNSUPPORTED, "%s: device ordinal %d is outside [0, %d)", fn, dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(mu);
  if (addr[dev] == nullptr) {
    void* p = nullptr;
    if (int rc = check_hip(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)")) return rc;
    if (p == nullptr) return fail(BSGA_ERR_HIP, "%s: hipGetSymbolAddress returned a null address", fn);
    addr[dev] = p;
  }
  *ptr = addr[dev];
  return BSGA_OK;
}

}  // namespace bsga

using namespace bsga;

extern "C" {

int bsga_version(void) { return 3; }

const char* bsga_last_error(void) { return g_err; }

static int pool_common(const char* fn, const void* q, const void* k, int dtype, int heads, int64_t n_tokens,
                       int64_t n_first, int head_dim, int block, double* q_pool, double* k_pool, void* stream) {
  clear_error();
  if (int rc = check_shape(fn, dtype, heads, n_tokens, head_dim)) return rc;
  if (int rc = check_block(fn, block)) return rc;
  if (n_first < 0 || n_first > n_tokens)
    return fail(BSGA_ERR_INVALID_ARG, "%s: n_first must be in [0, n_tokens], got %lld", fn, (long long)n_first);
  if ((q == nullptr) != (q_pool == nullptr) || (k == nullptr) != (k_pool == nullptr))
    return fail(BSGA_ERR_INVALID_ARG, "%s: each input must come with its output (q with q_pool, k with k_pool)", fn);
  if (!q && !k) return fail(BSGA_ERR_INVALID_ARG, "%s: nothing to pool (q and k are both null)", fn);
  if ((q && !aligned16(q)) || (k && !aligned16(k)) || (q_pool && !aligned16(q_pool)) || (k_pool && !aligned16(k_pool)))
    return fail(BSGA_ERR_INVALID_ARG, "%s: pointers must be 16-byte aligned", fn);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (q)
    if (int rc = launch_pool(q, dtype, heads, n_tokens, n_first, block, q_pool, s)) return rc;
  if (k)
    if (int rc = launch_pool(k, dtype, heads, n_tokens, n_first, block, k_pool, s)) return rc;
  return BSGA_OK;
}

int bsga_pool_qk(const void* q, const void* k, int dtype, int heads, int64_t n_tokens, int head_dim, int block,
                 double* q_pool, double* k_pool, void* stream) {
  return pool_common("bsga_pool_qk", q, k, dtype, heads, n_tokens, n_tokens, head_dim, block, q_pool, k_pool, stream);
}

int bsga_pool_qk_split(const void* q, const void* k, int dtype, int heads, int64_t n_tokens, int64_t n_first,
                       int head_dim, int block, double* q_pool, double* k_pool, void* stream) {
  return pool_common("bsga_pool_qk_split", q, k, dtype, heads, n_tokens, n_first, head_dim, block, q_pool, k_pool,
                     stream);
}

size_t bsga_select_workspace_bytes(int heads, int nb_q, int nb_k) {
  if (heads < 1 || nb_q < 1 || nb_k < 1) return 0;
  return select_workspace_bytes(heads, nb_q, nb_k);
}

int bsga_select_blocks(const double* q_pool, const double* k_pool, int heads, int nb_q, int nb_k, int head_dim,
                       double score_scale, double tau, double rho, const uint8_t* force_q, const uint8_t* force_k,
                       uint32_t* mask_bits, int32_t* kv_idx, int32_t* kv_cnt, int idx_stride, void* workspace,
                       size_t workspace_bytes, void* stream) {
  const char* fn = "bsga_select_blocks";
  clear_error();
  if (!q_pool || !k_pool) return fail(BSGA_ERR_INVALID_ARG, "%s: q_pool and k_pool must be non-null", fn);
  if (!aligned16(q_pool) || !aligned16(k_pool))
    return fail(BSGA_ERR_INVALID_ARG, "%s: q_pool and k_pool must be 16-byte aligned", fn);
  if (heads < 1 || heads > 65535) return fail(BSGA_ERR_INVALID_ARG, "%s: heads must be in [1, 65535], got %d", fn, heads);
  if (head_dim != 64) return fail(BSGA_ERR_UNSUPPORTED, "%s: head_dim must be 64, got %d", fn, head_dim);
  if (nb_q < 1 || nb_q > (1 << 18))
    return fail(BSGA_ERR_INVALID_ARG, "%s: nb_q must be in [1, 2^18], got %d", fn, nb_q);
  if (nb_k < 1) return fail(BSGA_ERR_INVALID_ARG, "%s: nb_k must be >= 1, got %d", fn, nb_k);
  if (nb_k > 8192) return fail(BSGA_ERR_UNSUPPORTED, "%s: nb_k above 8192 is not supported, got %d", fn, nb_k);
  if (!isfinite(score_scale)) return fail(BSGA_ERR_INVALID_ARG, "%s: score_scale must be finite", fn);
  if (!(tau >= 0.0)) return fail(BSGA_ERR_INVALID_ARG, "%s: tau must be >= 0", fn);
  if (!(rho >= 0.0 && rho <= 1.0)) return fail(BSGA_ERR_INVALID_ARG, "%s: rho must be in [0, 1]", fn);
  if (kv_idx && idx_stride < nb_k)
    return fail(BSGA_ERR_INVALID_ARG, "%s: idx_stride (%d) must be >= nb_k (%d)", fn, idx_stride, nb_k);
  if (!mask_bits && !kv_idx && !kv_cnt) return fail(BSGA_ERR_INVALID_ARG, "%s: no output requested", fn);
  const size_t need = select_workspace_bytes(heads, nb_q, nb_k);
  if (!workspace) return fail(BSGA_ERR_WORKSPACE, "%s: workspace is null, %zu bytes needed", fn, need);
  if (workspace_bytes < need)
    return fail(BSGA_ERR_WORKSPACE, "%s: workspace has %zu bytes, %zu needed", fn, workspace_bytes, need);
  if (!aligned16(workspace)) return fail(BSGA_ERR_INVALID_ARG, "%s: workspace must be 16-byte aligned", fn);
  return launch_select(q_pool, k_pool, heads, nb_q, nb_k, score_scale, tau, 1.0 - rho, force_q, force_k, mask_bits,
                       kv_idx, kv_cnt, idx_stride, workspace, static_cast<hipStream_t>(stream));
}

int bsga_gather_tokens(const void* src, int dtype, int heads, int64_t n_src, int head_dim, const int32_t* index,
                       int64_t n_dst, void* dst, void* stream) {
  const char* fn = "bsga_gather_tokens";
  clear_error();
  if (!src || !dst || !index) return fail(BSGA_ERR_INVALID_ARG, "%s: src, index and dst must be non-null", fn);
  if (!aligned16(src) || !aligned16(dst)) return fail(BSGA_ERR_INVALID_ARG, "%s: src and dst must be 16-byte aligned", fn);
  if (dtype != BSGA_BF16 && dtype != BSGA_FP32) return fail(BSGA_ERR_INVALID_ARG, "%s: unknown dtype %d", fn, dtype);
  if (heads < 1 || heads > 65535) return fail(BSGA_ERR_INVALID_ARG, "%s: heads must be in [1, 65535], got %d", fn, heads);
  if (head_dim != 64) return fail(BSGA_ERR_UNSUPPORTED, "%s: head_dim must be 64, got %d", fn, head_dim);
  if (n_src < 1 || n_src > (int64_t(1) << 24))
    return fail(BSGA_ERR_INVALID_ARG, "%s: n_src must be in [1, 2^24], got %lld", fn, static_cast<long long>(n_src));
  if (n_dst < 0 || n_dst > (int64_t(1) << 24))
    return fail(BSGA_ERR_INVALID_ARG, "%s: n_dst must be in [0, 2^24], got %lld", fn, static_cast<long long>(n_dst));
  if (n_dst == 0) return BSGA_OK;
  return launch_gather(src, dtype, heads, n_src, index, n_dst, dst, static_cast<hipStream_t>(stream));
}

size_t bsga_attn_workspace_bytes(int dtype, int heads, int64_t n_tokens, int head_dim) {
  if ((dtype != BSGA_BF16 && dtype != BSGA_FP32) || heads < 1 || n_tokens < 1 || head_dim != 64) return 0;
  return attn_workspace(dtype, heads, n_tokens);
}

int bsga_sparse_attn(const void* q, const void* k, const void* v, int dtype, int heads, int64_t n_tokens,
                     int head_dim, int block, float softmax_scale, const int32_t* kv_idx, const int32_t* kv_cnt,
                     int idx_stride, void* out, float* lse, void* workspace, size_t workspace_bytes, void* stream) {
  if (!kv_idx || !kv_cnt) {
    clear_error();
    return fail(BSGA_ERR_INVALID_ARG, "bsga_sparse_attn: kv_idx and kv_cnt must be non-null");
  }
  return attn_common("bsga_sparse_attn", q, k, v, dtype, heads, n_tokens, n_tokens, head_dim, block, block, softmax_scale,
                     kv_idx, kv_cnt, idx_stride, out, lse, workspace, workspace_bytes, stream);
}

size_t bsga_noalloc_scratch_bytes(void) { return kStaticScratchBytes; }

int bsga_sparse_attn_noalloc(const void* q, const void* k, const void* v, int dtype, int heads, int64_t n_tokens,
                             int head_dim, int block, float softmax_scale, const int32_t* kv_idx,
                             const int32_t* kv_cnt, int idx_stride, void* out, float* lse, void* stream) {
  const char* fn = "bsga_sparse_attn_noalloc";
  clear_error();
  if (!kv_idx || !kv_cnt) return fail(BSGA_ERR_INVALID_ARG, "%s: kv_idx and kv_cnt must be non-null", fn);
  if (int rc = check_shape(fn, dtype, heads, n_tokens, head_dim)) return rc;
  const size_t need = attn_workspace(dtype, heads, n_tokens);
  if (need > kStaticScratchBytes)
    return fail(BSGA_ERR_UNSUPPORTED,
                "%s: this shape needs %zu bytes of scratch, the built-in buffer holds %zu (about heads * "
                "(ceil(n_tokens / 64) + 33) <= %zu); use bsga_sparse_attn with a workspace",
                fn, need, kStaticScratchBytes, kStaticScratchBytes / sizeof(int32_t));
  void* ws = nullptr;
  if (need > 0)
    if (int rc = static_scratch(fn, &ws)) return rc;
  return attn_common(fn, q, k, v, dtype, heads, n_tokens, n_tokens, head_dim, block, block, softmax_scale, kv_idx,
                     kv_cnt, idx_stride, out, lse, ws, ws ? kStaticScratchBytes : 0, stream);
}

int bsga_sparse_attn_qk(const void* q, const void* k, const void* v, int dtype, int heads, int64_t n_tokens,
                        int head_dim, int block_q, int block_k, float softmax_scale, const int32_t* kv_idx,
                        const int32_t* kv_cnt, int idx_stride, void* out, float* lse, void* workspace,
                        size_t workspace_bytes, void* stream) {
  if (!kv_idx || !kv_cnt) {
    clear_error();
    return fail(BSGA_ERR_INVALID_ARG, "bsga_sparse_attn_qk: kv_idx and kv_cnt must be non-null");
  }
  return attn_common("bsga_sparse_attn_qk", q, k, v, dtype, heads, n_tokens, n_tokens, head_dim, block_q, block_k,
                     softmax_scale, kv_idx, kv_cnt, idx_stride, out, lse, workspace, workspace_bytes, stream);
}

int bsga_sparse_attn_split(const void* q, const void* k, const void* v, int dtype, int heads, int64_t n_tokens,
                           int64_t n_first, int head_dim, int block_q, int block_k, float softmax_scale,
                           const int32_t* kv_idx, const int32_t* kv_cnt, int idx_stride, void* out, float* lse,
                           void* workspace, size_t workspace_bytes, void* stream) {
  if (!kv_idx || !kv_cnt) {
    clear_error();
    return fail(BSGA_ERR_INVALID_ARG, "bsga_sparse_attn_split: kv_idx and kv_cnt must be non-null");
  }
  return attn_common("bsga_sparse_attn_split", q, k, v, dtype, heads, n_tokens, n_first, head_dim, block_q, block_k,
                     softmax_scale, kv_idx, kv_cnt, idx_stride, out, lse, workspace, workspace_bytes, stream);
}

int bsga_probe_mfma(int operands, int softmax_mix, int iters, void* sink, size_t sink_bytes, double* flops,
                    void* stream) {
  const char* fn = "bsga_probe_mfma";
  clear_error();
  if (operands != 0 && operands != 1) return fail(BSGA_ERR_INVALID_ARG, "%s: operands must be 0 (zeros) or 1 (random)", fn);
  if (softmax_mix < 0 || softmax_mix > 2) return fail(BSGA_ERR_INVALID_ARG, "%s: softmax_mix must be 0, 1 or 2", fn);
  if (iters < 1 || iters > (1 << 24)) return fail(BSGA_ERR_INVALID_ARG, "%s: iters must be in [1, 2^24], got %d", fn, iters);
  if (!sink) return fail(BSGA_ERR_INVALID_ARG, "%s: sink must be non-null", fn);
  return launch_probe_mfma(operands, softmax_mix, iters, static_cast<float*>(sink), sink_bytes, flops,
                           static_cast<hipStream_t>(stream));
}

int bsga_dense_attn(const void* q, const void* k, const void* v, int dtype, int heads, int64_t n_tokens,
                    int head_dim, float softmax_scale, void* out, float* lse, void* workspace,
                    size_t workspace_bytes, void* stream) {
  const int block = (dtype == BSGA_FP32) ? 64 : 128;
  return attn_common("bsga_dense_attn", q, k, v, dtype, heads, n_tokens, n_tokens, head_dim, block, block, softmax_scale, nullptr,
                     nullptr, 0, out, lse, workspace, workspace_bytes, stream);
}

}  // extern "C"
