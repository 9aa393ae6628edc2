// Instruction-rate probe: what the matrix pipe of this GPU sustains on the attention kernel's MFMA
// (v_mfma_f32_32x32x16_bf16) with nothing else in the way -- no LDS, no global memory -- for a given
// operand bit pattern and with or without the attention kernel's softmax arithmetic beside it
// (Sec. 4.1, Eq. (2) at head dim 64 costs, per 32 x 32 x 16 product, two exp2, one pack to bf16 and
// the row sum of two weights: mix 1 takes the row sums with two fp32 adds, mix 2 the way the
// attention kernel does, with one small 16x16x32 MFMA per four products).  The part lowers its clock with the switching activity of
// the operands, so the sustained rate on random values, not the nominal peak, is what bounds any
// bf16 kernel on real data; the benchmark reports this figure beside the attention kernel's.
//
// Every workgroup (4 waves, two workgroups per CU, the attention kernel's occupancy) runs `iters`
// rounds of 8 MFMAs over 8 operand pairs held in registers, so consecutive MFMAs see different
// operands, as they do in the attention kernel.
#include "bsga_internal.h"

namespace bsga {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ unsigned hash32(unsigned x) {  // a fixed integer mixer (no state)
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}

// bf16 bit pattern of a roughly unit-normal value: sum of four uniform bytes, centred and scaled
__device__ __forceinline__ unsigned short normal_bf16(unsigned seed) {
  const unsigned h = hash32(seed);
  const float s = static_cast<float>((h & 255u) + ((h >> 8) & 255u) + ((h >> 16) & 255u) + (h >> 24));
  const float v = (s - 510.0f) * (1.0f / 147.8f);  // mean 510, standard deviation 147.8
  return static_cast<unsigned short>(__float_as_uint(v) >> 16);
}

__device__ __forceinline__ unsigned pack_bf16(float a, float b) {
  const f32x2 two = {a, b};
  return __builtin_bit_cast(unsigned, __builtin_convertvector(two, bf16x2));
}

template <int MIX>
__global__ __launch_bounds__(256, 2) void probe_kernel(int pattern, int iters, float* __restrict__ sink) {
  bf16x8 a[8], b[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    u32x4 wa, wb;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const unsigned seed = ((blockIdx.x * 256u + threadIdx.x) * 8u + i) * 8u + e;
      unsigned lo_a = 0, hi_a = 0, lo_b = 0, hi_b = 0;
      if (pattern == 1) {
        lo_a = normal_bf16(seed * 4u); hi_a = normal_bf16(seed * 4u + 1u);
        lo_b = normal_bf16(seed * 4u + 2u); hi_b = normal_bf16(seed * 4u + 3u);
      }
      wa[e] = lo_a | (hi_a << 16);
      wb[e] = lo_b | (hi_b << 16);
    }
    a[i] = __builtin_bit_cast(bf16x8, wa);
    b[i] = __builtin_bit_cast(bf16x8, wb);
  }
  f32x16 c[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) c[j][e] = 0.f;
  // softmax-like side work: 16 "scores" per MFMA pair, exponentiated, summed and packed
  float s[16], l = 0.f;
  unsigned w[8] = {};
#pragma unroll
  for (int e = 0; e < 16; ++e) s[e] = pattern == 1 ? -0.125f * static_cast<float>((threadIdx.x + 5 * e) & 31) : 0.f;
  // mix 2: a selector A operand that makes a 16x16x32 MFMA add each lane's own eight B values into one
  // accumulator register (ones where row%4 == 0 and the lane's k group equals row/4)
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  f32x4 lacc = {0.f, 0.f, 0.f, 0.f};
  const unsigned lane = threadIdx.x & 63u;
  const unsigned sel1 = ((lane & 3u) == 0u && (lane >> 4) == ((lane & 15u) >> 2)) ? 0x3F803F80u : 0u;
  const bf16x8 sel = __builtin_bit_cast(bf16x8, u32x4{sel1, sel1, sel1, sel1});
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      c[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[i], c[i & 3], 0, 0, 0);
      if constexpr (MIX != 0) {
        asm volatile("" : "+v"(s[2 * i]), "+v"(s[2 * i + 1]));  // opaque: recomputed every round
        const float e0 = __builtin_amdgcn_exp2f(s[2 * i]), e1 = __builtin_amdgcn_exp2f(s[2 * i + 1]);
        if constexpr (MIX == 1) l += e0 + e1;
        w[i] = pack_bf16(e0, e1);
        // the packed weights go into the B operand of this pair's next MFMA, as in attention
        u32x4 bw = __builtin_bit_cast(u32x4, b[i]);
        bw[0] = w[i];
        b[i] = __builtin_bit_cast(bf16x8, bw);
        if constexpr (MIX == 2) {
          if ((i & 3) == 3) lacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(sel, b[i], lacc, 0, 0, 0);
        }
      }
    }
  }
  float total = l + lacc[0] + lacc[1] + lacc[2] + lacc[3];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) total += c[j][e];
#pragma unroll
  for (int i = 0; i < 8; ++i) total += __uint_as_float(w[i] << 16);
  sink[blockIdx.x * 256 + threadIdx.x] = total;
}

}  // namespace

int launch_probe_mfma(int pattern, int mix, int iters, float* sink, size_t sink_bytes, double* flops, hipStream_t stream) {
  int dev = 0, cus = 0;
  if (int rc = check_hip(hipGetDevice(&dev), "hipGetDevice")) return rc;
  if (int rc = check_hip(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev), "hipDeviceGetAttribute"))
    return rc;
  const int grid = 2 * cus;
  if (sink_bytes < size_t(grid) * 256 * sizeof(float))
    return fail(BSGA_ERR_WORKSPACE, "bsga_probe_mfma: sink has %zu bytes, %zu needed", sink_bytes,
                size_t(grid) * 256 * sizeof(float));
  if (mix == 2) hipLaunchKernelGGL(probe_kernel<2>, dim3(grid), dim3(256), 0, stream, pattern, iters, sink);
  else if (mix == 1) hipLaunchKernelGGL(probe_kernel<1>, dim3(grid), dim3(256), 0, stream, pattern, iters, sink);
  else hipLaunchKernelGGL(probe_kernel<0>, dim3(grid), dim3(256), 0, stream, pattern, iters, sink);
  if (flops) *flops = double(grid) * 4.0 * double(iters) * 8.0 * (2.0 * 32 * 32 * 16);
  return check_hip(hipGetLastError(), "bsga_probe_mfma launch");
}

}  // namespace bsga
