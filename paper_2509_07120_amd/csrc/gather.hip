// Token gather: dst[h, i, :] = src[h, index[i], :] (Sec. 4.2: the tokens are split into patch
// tokens and special tokens; this reorders a [heads, n, 64] tensor so that each kind is contiguous,
// and back).  HBM-bound: every row (128 B in bf16, 256 B in fp32) is read once and written once,
// 16 bytes per lane, so consecutive lanes cover whole rows and both sides move full cache lines.
#include "bsga_internal.h"

namespace bsga {
namespace {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

template <int CHUNKS>  // 16-byte chunks per row
__global__ __launch_bounds__(256) void gather_kernel(const u32x4* __restrict__ src, const int32_t* __restrict__ index,
                                                     u32x4* __restrict__ dst, int64_t n_src, int64_t n_dst) {
  const int64_t t = int64_t(blockIdx.x) * 256 + threadIdx.x;
  const int64_t i = t / CHUNKS;
  const int c = static_cast<int>(t % CHUNKS);
  if (i >= n_dst) return;
  int64_t j = index[i];
  j = j < 0 ? 0 : (j >= n_src ? n_src - 1 : j);  // an out-of-range index cannot read outside the tensor
  const int64_t h = blockIdx.y;
  dst[(h * n_dst + i) * CHUNKS + c] = src[(h * n_src + j) * CHUNKS + c];
}

}  // namespace

int launch_gather(const void* src, int dtype, int heads, int64_t n_src, const int32_t* index, int64_t n_dst,
                  void* dst, hipStream_t stream) {
  const int chunks = dtype == BSGA_BF16 ? 8 : 16;
  const dim3 grid(static_cast<unsigned>(ceil_div(n_dst * chunks, 256)), heads);
  const u32x4* s = static_cast<const u32x4*>(src);
  u32x4* d = static_cast<u32x4*>(dst);
  if (dtype == BSGA_BF16) {
    hipLaunchKernelGGL(gather_kernel<8>, grid, dim3(256), 0, stream, s, index, d, n_src, n_dst);
  } else {
    hipLaunchKernelGGL(gather_kernel<16>, grid, dim3(256), 0, stream, s, index, d, n_src, n_dst);
  }
  return check_hip(hipGetLastError(), "bsga_gather_tokens launch");
}

}  // namespace bsga
