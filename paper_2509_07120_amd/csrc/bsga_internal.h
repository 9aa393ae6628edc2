// Internal declarations shared by the bsga translation units (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "bsga.h"

namespace bsga {

// Records a message for bsga_last_error() and returns `code`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();

// Turns a HIP status into a bsga return code (records the HIP error string).
int check_hip(hipError_t e, const char* what);

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Number of blocks when tokens [0, n_first) and [n_first, n_tokens) are cut into blocks separately
// (no block crosses n_first).  n_first = n_tokens or 0 gives ceil(n_tokens / block).
inline int64_t split_blocks(int64_t n_tokens, int64_t n_first, int64_t block) {
  return ceil_div(n_first, block) + ceil_div(n_tokens - n_first, block);
}

// Kernel launchers.  Arguments are already validated.
int launch_pool(const void* x, int dtype, int heads, int64_t n_tokens, int64_t n_first, int block, double* pooled,
                hipStream_t stream);

int launch_select(const double* q_pool, const double* k_pool, int heads, int nb_q, int nb_k,
                  double score_scale, double tau, double one_minus_rho, const uint8_t* force_q,
                  const uint8_t* force_k, uint32_t* mask_bits, int32_t* kv_idx, int32_t* kv_cnt,
                  int idx_stride, void* workspace, hipStream_t stream);
size_t select_workspace_bytes(int heads, int nb_q, int nb_k);

int launch_gather(const void* src, int dtype, int heads, int64_t n_src, const int32_t* index,
                  int64_t n_dst, void* dst, hipStream_t stream);

int launch_attn_bf16(const void* q, const void* k, const void* v, int heads, int64_t n_tokens, int64_t n_first,
                     int block, int block_k, float softmax_scale, const int32_t* kv_idx, const int32_t* kv_cnt,
                     int idx_stride, void* out, float* lse, void* workspace, hipStream_t stream);

int launch_attn_fp32(const float* q, const float* k, const float* v, int heads, int64_t n_tokens, int64_t n_first,
                     int block, float softmax_scale, const int32_t* kv_idx, const int32_t* kv_cnt,
                     int idx_stride, float* out, float* lse, hipStream_t stream);

int launch_probe_mfma(int pattern, int mix, int iters, float* sink, size_t sink_bytes, double* flops,
                      hipStream_t stream);

}  // namespace bsga
