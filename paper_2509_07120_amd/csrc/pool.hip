// Block average pooling P^b(x) (Sec. 4.1, "Predicting Block Masks").
//
// One workgroup per (head, block): 256 threads stream the block's b x 64 elements with 16-byte
// loads (a block is one contiguous run of memory), add them up in float64 and write the 64
// block means.  The kernel is bound by HBM reads: 2 bytes (bf16) or 4 bytes (fp32) per element,
// each read exactly once.
#include "bsga_internal.h"

namespace bsga {
namespace {

constexpr int kThreads = 256;
constexpr int kD = 64;

__device__ inline void widen8(const uint4& raw, double* acc) {
  // eight bf16 values packed in 16 bytes -> added into acc[0..7]
  const unsigned w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    acc[2 * i] += static_cast<double>(__uint_as_float(w[i] << 16));
    acc[2 * i + 1] += static_cast<double>(__uint_as_float(w[i] & 0xffff0000u));
  }
}

__device__ inline void widen4(const uint4& raw, double* acc) {
  acc[0] += static_cast<double>(__uint_as_float(raw.x));
  acc[1] += static_cast<double>(__uint_as_float(raw.y));
  acc[2] += static_cast<double>(__uint_as_float(raw.z));
  acc[3] += static_cast<double>(__uint_as_float(raw.w));
}

// ELEM_BYTES: 2 = bf16, 4 = fp32.
template <int ELEM_BYTES, int B>
__global__ __launch_bounds__(kThreads) void pool_kernel(const uint4* __restrict__ x, double* __restrict__ pooled,
                                                        int64_t n_tokens, int64_t n_first, int nb1, int nb) {
  constexpr int E = 16 / ELEM_BYTES;     // elements per 16-byte chunk
  constexpr int CH = kD / E;             // chunks per token row
  constexpr int TL = kThreads / CH;      // tokens covered per pass
  constexpr int PASSES = B / TL;
  __shared__ double red[TL][kD + 1];

  const int I = blockIdx.x;
  const int h = blockIdx.y;
  const int t = threadIdx.x;
  const int cg = t % CH;
  const int tl = t / CH;
  // blocks 0 .. nb1-1 tile tokens [0, n_first), the others tokens [n_first, n_tokens)
  const int64_t tok0 = I < nb1 ? int64_t(I) * B : n_first + int64_t(I - nb1) * B;
  const int valid = static_cast<int>(min<int64_t>(B, (I < nb1 ? n_first : n_tokens) - tok0));
  const uint4* base = x + (int64_t(h) * n_tokens + tok0) * CH;

  double acc[E];
#pragma unroll
  for (int e = 0; e < E; ++e) acc[e] = 0.0;

  uint4 raw[PASSES];
#pragma unroll
  for (int p = 0; p < PASSES; ++p) {
    const int tok = tl + p * TL;
    raw[p] = make_uint4(0, 0, 0, 0);
    if (tok < valid) raw[p] = base[int64_t(tok) * CH + cg];
  }
#pragma unroll
  for (int p = 0; p < PASSES; ++p) {
    if constexpr (ELEM_BYTES == 2) widen8(raw[p], acc); else widen4(raw[p], acc);
  }
#pragma unroll
  for (int e = 0; e < E; ++e) red[tl][cg * E + e] = acc[e];
  __syncthreads();
  if (t < kD) {
    double s = 0.0;
#pragma unroll 8
    for (int r = 0; r < TL; ++r) s += red[r][t];
    pooled[(int64_t(h) * nb + I) * kD + t] = s / static_cast<double>(valid);
  }
}

}  // namespace

int launch_pool(const void* x, int dtype, int heads, int64_t n_tokens, int64_t n_first, int block, double* pooled,
                hipStream_t stream) {
  const int nb = static_cast<int>(split_blocks(n_tokens, n_first, block));
  const int nb1 = static_cast<int>(ceil_div(n_first, block));
  dim3 grid(nb, heads), blk(kThreads);
  const uint4* xp = static_cast<const uint4*>(x);
  if (dtype == BSGA_BF16) {
    if (block == 64) hipLaunchKernelGGL((pool_kernel<2, 64>), grid, blk, 0, stream, xp, pooled, n_tokens, n_first, nb1, nb);
    else hipLaunchKernelGGL((pool_kernel<2, 128>), grid, blk, 0, stream, xp, pooled, n_tokens, n_first, nb1, nb);
  } else {
    if (block == 64) hipLaunchKernelGGL((pool_kernel<4, 64>), grid, blk, 0, stream, xp, pooled, n_tokens, n_first, nb1, nb);
    else hipLaunchKernelGGL((pool_kernel<4, 128>), grid, blk, 0, stream, xp, pooled, n_tokens, n_first, nb1, nb);
  }
  return check_hip(hipGetLastError(), "bsga_pool_qk launch");
}

}  // namespace bsga
