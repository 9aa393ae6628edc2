// Host-side check of the C-ABI glue (argument validation, block arithmetic, workspace sizing, error
// strings) under AddressSanitizer / UndefinedBehaviorSanitizer.  The kernel launchers are replaced
// by the stubs below, which only check the invariants the real launchers rely on, so the program
// runs on a machine without a GPU.  Built and run by tests/test_hostglue_sanitized.py.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include <string>

#include "bsga.h"
#include "bsga_internal.h"

static int g_calls = 0;
static int g_fail = 0;
#define CHECK(cond)                                                        \
  do {                                                                     \
    if (!(cond)) {                                                         \
      fprintf(stderr, "FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond);    \
      ++g_fail;                                                            \
    }                                                                      \
  } while (0)

namespace bsga {
// ---- stubs: the launchers' preconditions, as the API layer must establish them -------------------
int launch_pool(const void* x, int dtype, int heads, int64_t n_tokens, int64_t n_first, int block, double* pooled,
                hipStream_t) {
  ++g_calls;
  CHECK(x && pooled && heads >= 1 && n_tokens >= 1 && n_first >= 0 && n_first <= n_tokens);
  CHECK((block == 64 || block == 128) && (dtype == BSGA_BF16 || dtype == BSGA_FP32));
  return BSGA_OK;
}
size_t select_workspace_bytes(int heads, int nb_q, int nb_k) { return size_t(heads) * nb_q * nb_k * sizeof(double); }
int launch_select(const double* q_pool, const double* k_pool, int heads, int nb_q, int nb_k, double, double tau,
                  double one_minus_rho, const uint8_t*, const uint8_t*, uint32_t* mask_bits, int32_t* kv_idx,
                  int32_t* kv_cnt, int idx_stride, void* workspace, hipStream_t) {
  ++g_calls;
  CHECK(q_pool && k_pool && workspace && heads >= 1 && nb_q >= 1 && nb_k >= 1 && nb_k <= 8192);
  CHECK(tau >= 0.0 && one_minus_rho >= 0.0 && one_minus_rho <= 1.0);
  CHECK(mask_bits || kv_idx || kv_cnt);
  CHECK(!kv_idx || idx_stride >= nb_k);
  return BSGA_OK;
}
int launch_gather(const void* src, int, int heads, int64_t n_src, const int32_t* index, int64_t n_dst, void* dst,
                  hipStream_t) {
  ++g_calls;
  CHECK(src && index && dst && heads >= 1 && n_src >= 1 && n_dst >= 1);
  return BSGA_OK;
}
static void check_attn(int heads, int64_t n_tokens, int64_t n_first, int block, int block_k, const int32_t* kv_idx,
                       const int32_t* kv_cnt, int idx_stride) {
  CHECK(heads >= 1 && n_tokens >= 1 && n_first >= 0 && n_first <= n_tokens);
  CHECK((kv_idx == nullptr) == (kv_cnt == nullptr));
  CHECK(!kv_idx || idx_stride >= split_blocks(n_tokens, n_first, block_k));
  CHECK(block == block_k || (block == 128 && block_k == 64));
}
int launch_attn_bf16(const void* q, const void* k, const void* v, int heads, int64_t n_tokens, int64_t n_first, int block,
                     int block_k, float scale, const int32_t* kv_idx, const int32_t* kv_cnt, int idx_stride, void* out,
                     float*, void* workspace, hipStream_t) {
  ++g_calls;
  CHECK(q && k && v && out && scale > 0.f);
  check_attn(heads, n_tokens, n_first, block, block_k, kv_idx, kv_cnt, idx_stride);
  if (workspace) {  // the launch order needs one word per query block plus the class table: touch it all
    const size_t words = size_t(heads) * split_blocks(n_tokens, n_first, block) + 32u * heads + 1;
    memset(workspace, 0, words * sizeof(int32_t));  // ASan faults here if the API sized the workspace too small
  }
  return BSGA_OK;
}
int launch_attn_fp32(const float* q, const float* k, const float* v, int heads, int64_t n_tokens, int64_t n_first,
                     int block, float scale, const int32_t* kv_idx, const int32_t* kv_cnt, int idx_stride, float* out,
                     float*, hipStream_t) {
  ++g_calls;
  CHECK(q && k && v && out && scale > 0.f);
  check_attn(heads, n_tokens, n_first, block, block, kv_idx, kv_cnt, idx_stride);
  return BSGA_OK;
}
int launch_probe_mfma(int pattern, int mix, int iters, float* sink, size_t, double* flops, hipStream_t) {
  ++g_calls;
  CHECK((pattern == 0 || pattern == 1) && mix >= 0 && mix <= 2 && iters >= 1 && sink);
  if (flops) *flops = 1.0;
  return BSGA_OK;
}
}  // namespace bsga

static bool err_has(const char* what) { return strstr(bsga_last_error(), what) != nullptr; }

int main() {
  alignas(16) static unsigned char buf[1 << 16];
  void* A = buf;  // a real, 16-byte aligned host buffer standing in for device memory (never dereferenced
                  // by the API layer; the stubs only touch the workspace)
  CHECK(bsga_version() == 3);
  CHECK(strlen(bsga_last_error()) == 0);

  // ---- pooling
  CHECK(bsga_pool_qk(A, A, 0, 16, 1000, 64, 128, (double*)A, (double*)A, nullptr) == BSGA_OK);
  CHECK(bsga_pool_qk(A, nullptr, 0, 16, 1000, 64, 128, (double*)A, nullptr, nullptr) == BSGA_OK);
  CHECK(bsga_pool_qk(nullptr, nullptr, 0, 16, 1000, 64, 128, nullptr, nullptr, nullptr) == BSGA_ERR_INVALID_ARG && err_has("nothing"));
  CHECK(bsga_pool_qk(A, A, 9, 16, 1000, 64, 128, (double*)A, (double*)A, nullptr) == BSGA_ERR_INVALID_ARG && err_has("dtype"));
  CHECK(bsga_pool_qk(A, A, 0, 16, 1000, 64, 96, (double*)A, (double*)A, nullptr) == BSGA_ERR_UNSUPPORTED && err_has("block"));
  CHECK(bsga_pool_qk(buf + 4, A, 0, 16, 1000, 64, 64, (double*)A, (double*)A, nullptr) == BSGA_ERR_INVALID_ARG && err_has("aligned"));
  CHECK(bsga_pool_qk(A, A, 0, 16, (int64_t(1) << 24) + 1, 64, 64, (double*)A, (double*)A, nullptr) == BSGA_ERR_UNSUPPORTED);
  CHECK(bsga_pool_qk_split(A, A, 0, 16, 1000, 0, 64, 64, (double*)A, (double*)A, nullptr) == BSGA_OK);
  CHECK(bsga_pool_qk_split(A, A, 0, 16, 1000, 1000, 64, 64, (double*)A, (double*)A, nullptr) == BSGA_OK);
  CHECK(bsga_pool_qk_split(A, A, 0, 16, 1000, 1001, 64, 64, (double*)A, (double*)A, nullptr) == BSGA_ERR_INVALID_ARG && err_has("n_first"));
  CHECK(bsga_pool_qk_split(A, A, 0, 16, 1000, -1, 64, 64, (double*)A, (double*)A, nullptr) == BSGA_ERR_INVALID_ARG);

  // ---- selection: workspace sizing at the edges
  CHECK(bsga_select_workspace_bytes(16, 1074, 1074) == size_t(16) * 1074 * 1074 * 8);
  CHECK(bsga_select_workspace_bytes(0, 1, 1) == 0 && bsga_select_workspace_bytes(1, -1, 1) == 0);
  CHECK(bsga_select_workspace_bytes(65535, 1 << 18, 8192) == size_t(65535) * (size_t(1) << 18) * 8192 * 8);  // no 32-bit overflow
  const size_t sel_ws = bsga_select_workspace_bytes(2, 9, 9);
  CHECK(bsga_select_blocks((double*)A, (double*)A, 2, 9, 9, 64, 0.125, 0.9, 1.0, nullptr, nullptr, (uint32_t*)A,
                           (int32_t*)A, (int32_t*)A, 9, A, sel_ws, nullptr) == BSGA_OK);
  CHECK(bsga_select_blocks((double*)A, (double*)A, 2, 9, 9, 64, 0.125, 0.9, 1.0, nullptr, nullptr, (uint32_t*)A,
                           (int32_t*)A, (int32_t*)A, 9, A, sel_ws - 1, nullptr) == BSGA_ERR_WORKSPACE);
  CHECK(bsga_select_blocks((double*)A, (double*)A, 2, 9, 9, 64, 0.125, 0.9, 1.0, nullptr, nullptr, (uint32_t*)A,
                           (int32_t*)A, (int32_t*)A, 8, A, sel_ws, nullptr) == BSGA_ERR_INVALID_ARG && err_has("idx_stride"));
  CHECK(bsga_select_blocks((double*)A, (double*)A, 2, 9, 9, 64, 0.125, -0.1, 1.0, nullptr, nullptr, (uint32_t*)A,
                           (int32_t*)A, (int32_t*)A, 9, A, sel_ws, nullptr) == BSGA_ERR_INVALID_ARG && err_has("tau"));
  CHECK(bsga_select_blocks((double*)A, (double*)A, 2, 9, 9, 64, 0.125, 0.9, 1.5, nullptr, nullptr, (uint32_t*)A,
                           (int32_t*)A, (int32_t*)A, 9, A, sel_ws, nullptr) == BSGA_ERR_INVALID_ARG && err_has("rho"));
  CHECK(bsga_select_blocks((double*)A, (double*)A, 2, 9, 8193, 64, 0.125, 0.9, 1.0, nullptr, nullptr, (uint32_t*)A,
                           (int32_t*)A, (int32_t*)A, 8193, A, size_t(1) << 40, nullptr) == BSGA_ERR_UNSUPPORTED);
  CHECK(bsga_select_blocks((double*)A, (double*)A, 2, 9, 9, 64, 0.125, 0.9, 1.0, nullptr, nullptr, nullptr, nullptr,
                           nullptr, 9, A, sel_ws, nullptr) == BSGA_ERR_INVALID_ARG && err_has("no output"));
  const double nan = __builtin_nan("");
  CHECK(bsga_select_blocks((double*)A, (double*)A, 2, 9, 9, 64, nan, 0.9, 1.0, nullptr, nullptr, (uint32_t*)A,
                           (int32_t*)A, (int32_t*)A, 9, A, sel_ws, nullptr) == BSGA_ERR_INVALID_ARG);
  CHECK(bsga_select_blocks((double*)A, (double*)A, 2, 9, 9, 64, 0.125, nan, 1.0, nullptr, nullptr, (uint32_t*)A,
                           (int32_t*)A, (int32_t*)A, 9, A, sel_ws, nullptr) == BSGA_ERR_INVALID_ARG);

  // ---- gather
  CHECK(bsga_gather_tokens(A, 0, 3, 100, 64, (int32_t*)A, 50, A, nullptr) == BSGA_OK);
  CHECK(bsga_gather_tokens(A, 0, 3, 100, 64, (int32_t*)A, 0, A, nullptr) == BSGA_OK);
  CHECK(bsga_gather_tokens(A, 0, 3, 0, 64, (int32_t*)A, 5, A, nullptr) == BSGA_ERR_INVALID_ARG);
  CHECK(bsga_gather_tokens(nullptr, 0, 3, 100, 64, (int32_t*)A, 5, A, nullptr) == BSGA_ERR_INVALID_ARG);

  // ---- attention: the workspace the API asks for must cover what the launcher writes, for every
  // shape class (uniform, split with one more block, block 64, block 128)
  for (int64_t n : {1LL, 63LL, 64LL, 129LL, 1000LL, 137400LL}) {
    for (int heads : {1, 16}) {
      const size_t need = bsga_attn_workspace_bytes(BSGA_BF16, heads, n, 64);
      CHECK(need >= (size_t(heads) * ((n + 63) / 64) + 32u * heads + 1) * 4);
      unsigned char* ws = new unsigned char[need + 16];  // exact size: an overrun is an ASan report
      void* wsa = ws + ((16 - (reinterpret_cast<uintptr_t>(ws) & 15)) & 15);
      for (int block : {64, 128}) {
        const int stride = int((n + block - 1) / block) + 1;
        CHECK(bsga_sparse_attn(A, A, A, 0, heads, n, 64, block, 0.125f, (int32_t*)A, (int32_t*)A, stride, A, nullptr, wsa,
                               need, nullptr) == BSGA_OK);
        for (int64_t n_first : {int64_t(0), n / 3, n}) {
          CHECK(bsga_sparse_attn_split(A, A, A, 0, heads, n, n_first, 64, block, block, 0.125f, (int32_t*)A, (int32_t*)A,
                                       stride + 1, A, nullptr, wsa, need, nullptr) == BSGA_OK);
        }
      }
      CHECK(bsga_sparse_attn_qk(A, A, A, 0, heads, n, 64, 128, 64, 0.125f, (int32_t*)A, (int32_t*)A, int((n + 63) / 64), A,
                                nullptr, wsa, need, nullptr) == BSGA_OK);
      if (need > 16)
        CHECK(bsga_sparse_attn(A, A, A, 0, heads, n, 64, 128, 0.125f, (int32_t*)A, (int32_t*)A, 1 << 20, A, nullptr, wsa,
                               need - 16, nullptr) == BSGA_ERR_WORKSPACE);
      CHECK(bsga_dense_attn(A, A, A, 0, heads, n, 64, 0.125f, A, nullptr, nullptr, 0, nullptr) == BSGA_OK);
      CHECK(bsga_dense_attn(A, A, A, 1, heads, n, 64, 0.125f, A, nullptr, nullptr, 0, nullptr) == BSGA_OK);
      delete[] ws;
    }
  }
  CHECK(bsga_attn_workspace_bytes(BSGA_FP32, 16, 1000, 64) == 0 && bsga_attn_workspace_bytes(0, 0, 1000, 64) == 0);
  CHECK(bsga_sparse_attn(A, A, A, 0, 4, 1000, 64, 128, 0.125f, nullptr, (int32_t*)A, 8, A, nullptr, nullptr, 0, nullptr) == BSGA_ERR_INVALID_ARG);
  CHECK(bsga_sparse_attn(A, A, A, 0, 4, 1000, 64, 128, 0.125f, (int32_t*)A, (int32_t*)A, 7, A, nullptr, nullptr, 0, nullptr) == BSGA_ERR_INVALID_ARG && err_has("idx_stride"));
  CHECK(bsga_sparse_attn(A, A, A, 0, 4, 1000, 64, 128, 0.f, (int32_t*)A, (int32_t*)A, 8, A, nullptr, nullptr, 0, nullptr) == BSGA_ERR_INVALID_ARG && err_has("softmax_scale"));
  CHECK(bsga_sparse_attn(A, A, A, 0, 4, 1000, 32, 128, 0.125f, (int32_t*)A, (int32_t*)A, 8, A, nullptr, nullptr, 0, nullptr) == BSGA_ERR_UNSUPPORTED);
  CHECK(bsga_sparse_attn_qk(A, A, A, 0, 4, 1000, 64, 64, 128, 0.125f, (int32_t*)A, (int32_t*)A, 16, A, nullptr, nullptr, 0, nullptr) == BSGA_ERR_UNSUPPORTED);
  CHECK(bsga_sparse_attn_qk(A, A, A, 1, 4, 1000, 64, 128, 64, 0.125f, (int32_t*)A, (int32_t*)A, 16, A, nullptr, nullptr, 0, nullptr) == BSGA_ERR_UNSUPPORTED);
  CHECK(bsga_sparse_attn_split(A, A, A, 0, 4, 1000, 1001, 64, 128, 128, 0.125f, (int32_t*)A, (int32_t*)A, 16, A, nullptr, nullptr, 0, nullptr) == BSGA_ERR_INVALID_ARG);

  // ---- the entry point on built-in scratch: size limit is checked before any device call; on a
  // machine without a GPU a fitting shape ends in a HIP error, never in a launch
  CHECK(bsga_noalloc_scratch_bytes() == (size_t(2) << 20));
  CHECK(bsga_sparse_attn_noalloc(A, A, A, 0, 4096, 1 << 20, 64, 128, 0.125f, (int32_t*)A, (int32_t*)A, 1 << 14, A, nullptr, nullptr) == BSGA_ERR_UNSUPPORTED && err_has("scratch"));
  CHECK(bsga_sparse_attn_noalloc(A, A, A, 0, 4, 1000, 64, 128, 0.125f, nullptr, (int32_t*)A, 8, A, nullptr, nullptr) == BSGA_ERR_INVALID_ARG);
  {
    const int before = g_calls;
    const int rc = bsga_sparse_attn_noalloc(A, A, A, 0, 4, 1000, 64, 128, 0.125f, (int32_t*)A, (int32_t*)A, 8, A, nullptr, nullptr);
    CHECK(rc == BSGA_ERR_HIP || rc == BSGA_OK);
    CHECK(rc == BSGA_OK || g_calls == before);
  }

  // ---- probe
  double flops = 0.0;
  CHECK(bsga_probe_mfma(1, 2, 10, A, sizeof(buf), &flops, nullptr) == BSGA_OK && flops == 1.0);
  CHECK(bsga_probe_mfma(3, 0, 10, A, sizeof(buf), nullptr, nullptr) == BSGA_ERR_INVALID_ARG);
  CHECK(bsga_probe_mfma(0, 3, 10, A, sizeof(buf), nullptr, nullptr) == BSGA_ERR_INVALID_ARG);

  // ---- error strings never overflow their buffer
  CHECK(bsga_pool_qk(A, A, 0, 2147483647, 1000, 64, 128, (double*)A, (double*)A, nullptr) == BSGA_ERR_INVALID_ARG);
  CHECK(strlen(bsga_last_error()) < 512);

  printf("hostglue: %d stub launches, %d failed checks\n", g_calls, g_fail);
  return g_fail == 0 ? 0 : 1;
}
