// fp32 attention over kept key blocks (Sec. 4.1, Eq. (2); Eq. (1) when no index list is given).
//
// Correctness path for fp32 tensors, not a tuned one: one thread per query row keeps q and the
// output accumulator in registers, key/value blocks are staged through LDS and read as
// wave-wide broadcasts, and the softmax is the usual online form (running max m, running sum l,
// rescale when m grows), all in fp32.
#include "bsga_internal.h"

namespace bsga {
namespace {

constexpr int kD = 64;

template <int B>
__global__ __launch_bounds__(B) void attn_fp32_kernel(const float* __restrict__ q, const float* __restrict__ k,
                                                      const float* __restrict__ v, int64_t n_tokens,
                                                      int64_t n_first, int nb1, int nb,
                                                      float scale_log2, const int32_t* __restrict__ kv_idx,
                                                      const int32_t* __restrict__ kv_cnt, int idx_stride,
                                                      float* __restrict__ out, float* __restrict__ lse) {
  __shared__ __align__(16) float ks[B][kD];
  __shared__ __align__(16) float vs[B][kD];
  const int I = blockIdx.x;
  const int h = blockIdx.y;
  const int t = threadIdx.x;
  const int64_t head_off = int64_t(h) * n_tokens * kD;
  // blocks 0 .. nb1-1 tile tokens [0, n_first), the others tokens [n_first, n_tokens)
  auto block_start = [&](int J) { return J < nb1 ? int64_t(J) * B : n_first + int64_t(J - nb1) * B; };
  auto block_count = [&](int J) {
    return static_cast<int>(min<int64_t>(B, (J < nb1 ? n_first : n_tokens) - block_start(J)));
  };
  const int64_t qi = block_start(I) + t;
  const bool qvalid = t < block_count(I);

  float qr[kD], o[kD];
#pragma unroll
  for (int d = 0; d < kD; d += 4) {
    float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
    if (qvalid) x = *reinterpret_cast<const float4*>(q + head_off + qi * kD + d);
    qr[d] = x.x * scale_log2; qr[d + 1] = x.y * scale_log2; qr[d + 2] = x.z * scale_log2; qr[d + 3] = x.w * scale_log2;
    o[d] = o[d + 1] = o[d + 2] = o[d + 3] = 0.f;
  }
  float m = -INFINITY, l = 0.f;

  const bool dense = kv_idx == nullptr;
  const int64_t row = int64_t(h) * nb + I;
  const int count = dense ? nb : min(max(kv_cnt[row], 0), nb);
  for (int it = 0; it < count; ++it) {
    int J = dense ? it : kv_idx[row * idx_stride + it];
    J = min(max(J, 0), nb - 1);
    const int64_t key0 = block_start(J);
    const int valid = block_count(J);
    __syncthreads();
    for (int c = t; c < B * (kD / 4); c += B) {
      const int r = c / (kD / 4), d4 = c % (kD / 4);
      float4 kk = make_float4(0.f, 0.f, 0.f, 0.f), vv = kk;
      if (r < valid) {
        kk = *reinterpret_cast<const float4*>(k + head_off + (key0 + r) * kD + d4 * 4);
        vv = *reinterpret_cast<const float4*>(v + head_off + (key0 + r) * kD + d4 * 4);
      }
      *reinterpret_cast<float4*>(&ks[r][d4 * 4]) = kk;
      *reinterpret_cast<float4*>(&vs[r][d4 * 4]) = vv;
    }
    __syncthreads();
    for (int j = 0; j < valid; ++j) {
      float s = 0.f;
#pragma unroll
      for (int d = 0; d < kD; ++d) s = fmaf(qr[d], ks[j][d], s);  // log2-domain logit
      if (s > m) {
        const float a = exp2f(m - s);  // exp2f(-inf) = 0 on the first key
        l *= a;
#pragma unroll
        for (int d = 0; d < kD; ++d) o[d] *= a;
        m = s;
      }
      const float p = exp2f(s - m);
      l += p;
#pragma unroll
      for (int d = 0; d < kD; ++d) o[d] = fmaf(p, vs[j][d], o[d]);
    }
  }
  if (qvalid) {
    const float inv = l > 0.f ? 1.f / l : 0.f;
#pragma unroll
    for (int d = 0; d < kD; d += 4) {
      *reinterpret_cast<float4*>(out + head_off + qi * kD + d) =
          make_float4(o[d] * inv, o[d + 1] * inv, o[d + 2] * inv, o[d + 3] * inv);
    }
    if (lse != nullptr) lse[int64_t(h) * n_tokens + qi] = (l > 0.f) ? (m + log2f(l)) * 0.6931471805599453f : -INFINITY;
  }
}

}  // namespace

int launch_attn_fp32(const float* q, const float* k, const float* v, int heads, int64_t n_tokens, int64_t n_first,
                     int block, float softmax_scale, const int32_t* kv_idx, const int32_t* kv_cnt, int idx_stride, float* out,
                     float* lse, hipStream_t stream) {
  const int nb = static_cast<int>(split_blocks(n_tokens, n_first, block));
  const int nb1 = static_cast<int>(ceil_div(n_first, block));
  const float scale_log2 = softmax_scale * 1.4426950408889634f;
  dim3 grid(nb, heads);
  if (block == 64)
    hipLaunchKernelGGL((attn_fp32_kernel<64>), grid, dim3(64), 0, stream, q, k, v, n_tokens, n_first, nb1, nb, scale_log2, kv_idx,
                       kv_cnt, idx_stride, out, lse);
  else
    hipLaunchKernelGGL((attn_fp32_kernel<128>), grid, dim3(128), 0, stream, q, k, v, n_tokens, n_first, nb1, nb, scale_log2,
                       kv_idx, kv_cnt, idx_stride, out, lse);
  return check_hip(hipGetLastError(), "bsga fp32 attention launch");
}

}  // namespace bsga
