// Block scores, block softmax and block selection (Sec. 4.1, "Predicting Block Masks" and
// "Selecting Blocks"), all in float64.
//
// One workgroup of 256 threads handles R consecutive query-block rows of one head:
//   1. logits[r][J] = scale * <q_pool[I+r], k_pool[J]>  four lanes share one J (16 dims each); every
//      k_pool element is loaded once and used for all R rows (k_pool of a head is re-read by every
//      workgroup from L2, which is what bounds this kernel, hence R rows per workgroup)
// then, row by row:
//   2. p = softmax(logits)                          block-wide max and sum
//   3. rank: bitonic sort in LDS by (p descending, J ascending)
//   4. inclusive scan of p in rank order; n_cdf = 1 + first rank whose running sum reaches tau
//   5. keep the first n = min(nb_k, max(n_cdf, k, 1)) ranks, OR the forced rows/columns in
//   6. emit bit mask words, the ascending index list and the count
// Nothing but the outputs goes to HBM.
#include "bsga_internal.h"

namespace bsga {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kD = 64;

__device__ inline double wave_max(double v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v = fmax(v, __shfl_xor(v, o));
  return v;
}
__device__ inline double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// rank order: larger p first, equal p by smaller block index
__device__ inline bool ranks_before(double pa, int ia, double pb, int ib) {
  return pa > pb || (pa == pb && ia < ib);
}

template <int R>
__global__ __launch_bounds__(kThreads) void select_kernel(
    const double* __restrict__ q_pool, const double* __restrict__ k_pool, int nb_q, int nb_k, int nbp,
    double score_scale, double tau, int k_floor, const uint8_t* __restrict__ force_q,
    const uint8_t* __restrict__ force_k, uint32_t* __restrict__ mask_bits, int32_t* __restrict__ kv_idx,
    int32_t* __restrict__ kv_cnt, int idx_stride) {
  extern __shared__ __align__(16) unsigned char smem[];
  double* val = reinterpret_cast<double*>(smem);                 // [nbp] p of the current row -> sorted p
  int* idx = reinterpret_cast<int*>(smem + size_t(nbp) * 8);     // [nbp] block index per rank
  double* logit = reinterpret_cast<double*>(smem + size_t(nbp) * 12);  // [R][nb_k] logits of all rows
  __shared__ double red[kWaves];
  __shared__ double red2[kWaves];
  __shared__ int wave_cnt[kWaves];
  __shared__ int first_rank;

  const int I0 = blockIdx.x * R;
  const int h = blockIdx.y;
  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = t >> 6;

  // ---- 1. logits of R rows ----------------------------------------------------------------------
  // lane quarter qd of a group of four handles the 16-byte chunks qd, qd+4, ..., qd+28 of a row
  const int qd = t & 3;
  double2 qv[R][8];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int I = min(I0 + r, nb_q - 1);  // rows past the end repeat the last row and are not emitted
    const double2* qrow = reinterpret_cast<const double2*>(q_pool + (int64_t(h) * nb_q + I) * kD);
#pragma unroll
    for (int i = 0; i < 8; ++i) qv[r][i] = qrow[4 * i + qd];
  }
  const double2* kbase = reinterpret_cast<const double2*>(k_pool + int64_t(h) * nb_k * kD);
  for (int j0 = 0; j0 < nb_k; j0 += kThreads / 4) {
    const int J = j0 + (t >> 2);
    double acc[R];
#pragma unroll
    for (int r = 0; r < R; ++r) acc[r] = 0.0;
    if (J < nb_k) {
      const double2* krow = kbase + int64_t(J) * (kD / 2);
      double2 kv[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) kv[i] = krow[4 * i + qd];
#pragma unroll
      for (int r = 0; r < R; ++r)
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[r] = fma(qv[r][i].x, kv[i].x, fma(qv[r][i].y, kv[i].y, acc[r]));
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
      acc[r] += __shfl_xor(acc[r], 1);
      acc[r] += __shfl_xor(acc[r], 2);
      if (qd == 0 && J < nb_k) logit[r * nb_k + J] = score_scale * acc[r];
    }
  }
  __syncthreads();

  for (int rr = 0; rr < R; ++rr) {
  const int I = I0 + rr;
  if (I >= nb_q) break;  // uniform
  const double* lrow = logit + rr * nb_k;
  // ---- 2. softmax -------------------------------------------------------------------------
  double m = -INFINITY;
  for (int J = t; J < nb_k; J += kThreads) m = fmax(m, lrow[J]);
  m = wave_max(m);
  if (lane == 0) red[wave] = m;
  __syncthreads();
  m = fmax(fmax(red[0], red[1]), fmax(red[2], red[3]));
  double z = 0.0;
  for (int J = t; J < nb_k; J += kThreads) {
    const double e = exp(lrow[J] - m);
    val[J] = e;
    z += e;
  }
  z = wave_sum(z);
  if (lane == 0) red2[wave] = z;
  __syncthreads();
  z = (red2[0] + red2[1]) + (red2[2] + red2[3]);
  for (int J = t; J < nbp; J += kThreads) {
    val[J] = (J < nb_k) ? val[J] / z : -1.0;  // padding ranks after every real block
    idx[J] = J;
  }
  if (t == 0) first_rank = nbp;
  __syncthreads();

  // ---- 3. bitonic sort into rank order ---------------------------------------------------
  for (int k = 2; k <= nbp; k <<= 1) {
    for (int j = k >> 1; j >= 1; j >>= 1) {
      for (int i = t; i < (nbp >> 1); i += kThreads) {
        const int a = ((i / j) * (j << 1)) + (i % j);
        const int b = a + j;
        const double pa = val[a], pb = val[b];
        const int ia = idx[a], ib = idx[b];
        const bool up = (a & k) == 0;  // this sub-sequence must end in rank order
        const bool swap = up ? ranks_before(pb, ib, pa, ia) : ranks_before(pa, ia, pb, ib);
        if (swap) {
          val[a] = pb; val[b] = pa;
          idx[a] = ib; idx[b] = ia;
        }
      }
      __syncthreads();
    }
  }

  // ---- 4. cumulative mass in rank order ---------------------------------------------------
  const int seg = nbp / kThreads;  // nbp is a multiple of 256
  const int r0 = t * seg;
  double local = 0.0;
  for (int r = r0; r < r0 + seg; ++r) local += (r < nb_k) ? val[r] : 0.0;
  // exclusive scan of the 256 per-thread totals
  double incl = local;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const double up = __shfl_up(incl, o);
    if (lane >= o) incl += up;
  }
  if (lane == 63) red[wave] = incl;
  __syncthreads();
  double offset = incl - local;
  for (int w = 0; w < wave; ++w) offset += red[w];
  if (tau < 1.0) {
    double run = offset;
    for (int r = r0; r < r0 + seg && r < nb_k; ++r) {
      run += val[r];
      if (run >= tau) {
        atomicMin(&first_rank, r);
        break;
      }
    }
  }
  __syncthreads();
  const int n_cdf = (first_rank < nb_k) ? first_rank + 1 : nb_k;
  const int n_keep = min(nb_k, max(max(n_cdf, k_floor), 1));
  const bool whole_row = force_q != nullptr && force_q[I] != 0;
  __syncthreads();

  // ---- 5. keep flags (val is reused as the flag array; ranks are read from idx) ------------
  unsigned char* keep = reinterpret_cast<unsigned char*>(val);
  for (int J = t; J < nbp; J += kThreads) keep[J] = 0;
  __syncthreads();
  for (int r = t; r < n_keep; r += kThreads) keep[idx[r]] = 1;
  __syncthreads();

  // ---- 6. emit -----------------------------------------------------------------------------
  const int words = (nb_k + 31) >> 5;
  const int64_t row = int64_t(h) * nb_q + I;
  int running = 0;
  for (int j0 = 0; j0 < nb_k; j0 += kThreads) {
    const int J = j0 + t;
    bool f = false;
    if (J < nb_k) f = whole_row || keep[J] != 0 || (force_k != nullptr && force_k[J] != 0);
    const unsigned long long bal = __ballot(f);
    if (lane == 0) {
      wave_cnt[wave] = __popcll(bal);
      if (mask_bits != nullptr) {
        const int w0 = (j0 >> 5) + 2 * wave;
        if (w0 < words) mask_bits[row * words + w0] = static_cast<uint32_t>(bal);
        if (w0 + 1 < words) mask_bits[row * words + w0 + 1] = static_cast<uint32_t>(bal >> 32);
      }
    }
    __syncthreads();
    int pos = running;
    for (int w = 0; w < wave; ++w) pos += wave_cnt[w];
    pos += __popcll(bal & ((1ull << lane) - 1ull));
    if (f && kv_idx != nullptr) kv_idx[row * idx_stride + pos] = J;
    running += wave_cnt[0] + wave_cnt[1] + wave_cnt[2] + wave_cnt[3];
    __syncthreads();
  }
  if (t == 0 && kv_cnt != nullptr) kv_cnt[row] = running;
  __syncthreads();  // val / idx / first_rank are reused by the next row
  }
}

template <int R>
static int launch_rows(const double* q_pool, const double* k_pool, int heads, int nb_q, int nb_k, int nbp,
                       size_t smem, double score_scale, double tau, int k_floor, const uint8_t* force_q,
                       const uint8_t* force_k, uint32_t* mask_bits, int32_t* kv_idx, int32_t* kv_cnt, int idx_stride,
                       hipStream_t stream) {
  if (smem > 64 * 1024) {
    if (int rc = check_hip(hipFuncSetAttribute(reinterpret_cast<const void*>(&select_kernel<R>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(smem)),
                           "bsga_select_blocks: raising the dynamic LDS limit"))
      return rc;
  }
  dim3 grid((nb_q + R - 1) / R, heads), blk(kThreads);
  hipLaunchKernelGGL(select_kernel<R>, grid, blk, smem, stream, q_pool, k_pool, nb_q, nb_k, nbp, score_scale, tau,
                     k_floor, force_q, force_k, mask_bits, kv_idx, kv_cnt, idx_stride);
  return check_hip(hipGetLastError(), "bsga_select_blocks launch");
}

}  // namespace

int launch_select(const double* q_pool, const double* k_pool, int heads, int nb_q, int nb_k, double score_scale,
                  double tau, int k_floor, const uint8_t* force_q, const uint8_t* force_k, uint32_t* mask_bits,
                  int32_t* kv_idx, int32_t* kv_cnt, int idx_stride, hipStream_t stream) {
  int nbp = kThreads;
  while (nbp < nb_k) nbp <<= 1;
  // LDS: sort arrays (12 bytes per padded rank) + R rows of logits; up to 96 KB so two workgroups fit a CU
  auto bytes = [&](int rows) { return size_t(nbp) * 12 + size_t(rows) * nb_k * 8; };
  if (nb_q >= 4 && bytes(4) <= 96 * 1024)
    return launch_rows<4>(q_pool, k_pool, heads, nb_q, nb_k, nbp, bytes(4), score_scale, tau, k_floor, force_q,
                          force_k, mask_bits, kv_idx, kv_cnt, idx_stride, stream);
  if (nb_q >= 2 && bytes(2) <= 96 * 1024)
    return launch_rows<2>(q_pool, k_pool, heads, nb_q, nb_k, nbp, bytes(2), score_scale, tau, k_floor, force_q,
                          force_k, mask_bits, kv_idx, kv_cnt, idx_stride, stream);
  return launch_rows<1>(q_pool, k_pool, heads, nb_q, nb_k, nbp, bytes(1), score_scale, tau, k_floor, force_q,
                        force_k, mask_bits, kv_idx, kv_cnt, idx_stride, stream);
}

}  // namespace bsga
