// Block scores, block softmax and block selection (Sec. 4.1, "Predicting Block Masks" and
// "Selecting Blocks"), all in float64.  Two kernels:
//
// logits_kernel: one workgroup computes R consecutive query-block rows of one head,
//     logits[I][J] = scale * <q_pool[I], k_pool[J]>,
//   four lanes sharing one J (16 dims each).  Every k_pool element is loaded once per workgroup and
//   used for all R rows: k_pool of a head is re-read by every workgroup from L2, and that traffic is
//   what bounds this step.  The logits go to a caller-provided workspace [heads, nb_q, nb_k].
//
// select_kernel: one WAVE per row, the whole row in registers (lane l holds blocks l, l+64, ...),
//   no LDS and no barriers.  The ranked prefix the method keeps is found without sorting:
//   with key(p) = the bit pattern of p (monotone for p >= 0) and, for a threshold key C,
//       M(C) = sum of p over {key >= C},   cnt(C) = number of blocks with key >= C,
//   the block at which the ranked cumulative mass first reaches tau is the one with key
//       T = max{C : cnt(C) >= 1 and M(C) >= tau},
//   found by bisection over the key range [key(p_min), key(p_max)] (each step one wave-wide sum);
//   the bisection stops as soon as one block is left in the window.  Blocks above T are kept;
//   blocks that tie with T are kept in ascending block order while the running mass is below tau.
//   The top-k floor is the same search with the predicate cnt(C) >= k.  The sums are taken in a
//   fixed order (lane-local in ascending block order, then a butterfly), so results are
//   deterministic; adding non-negative terms in a fixed order is monotone, which the bisection needs.
#include "bsga_internal.h"

namespace bsga {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kD = 64;

template <int R>
__global__ __launch_bounds__(kThreads) void logits_kernel(const double* __restrict__ q_pool,
                                                          const double* __restrict__ k_pool, int nb_q, int nb_k,
                                                          double score_scale, double* __restrict__ logits) {
  const int I0 = blockIdx.x * R;
  const int h = blockIdx.y;
  const int t = threadIdx.x;
  // lane quarter qd of a group of four handles the 16-byte chunks qd, qd+4, ..., qd+28 of a row
  const int qd = t & 3;
  double2 qv[R][8];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int I = min(I0 + r, nb_q - 1);  // rows past the end repeat the last row and are not stored
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
      if (qd == 0 && J < nb_k && I0 + r < nb_q)
        logits[(int64_t(h) * nb_q + I0 + r) * nb_k + J] = score_scale * acc[r];
    }
  }
}

__device__ inline double wave_sum_all(double v) {
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) v += __shfl_xor(v, o);
  return v;  // the butterfly leaves the same bits in every lane
}
__device__ inline int wave_sum_all(int v) {
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) v += __shfl_xor(v, o);
  return v;
}
__device__ inline uint64_t uniform64(uint64_t v) {
  const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v));
  const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v >> 32));
  return (uint64_t(hi) << 32) | lo;
}

// Threshold search.  MASS: largest C with cnt(C) >= 1 and M(C) >= tau; otherwise largest C with
// cnt(C) >= k_target.  Requires the predicate to hold at key_min.  Returns the threshold key T and
// n_gt = cnt(T+1), mass_gt = M(T+1), ties = number of blocks whose key equals T.
template <int E, bool MASS>
__device__ inline uint64_t find_threshold(const double (&p)[E], uint64_t key_min, uint64_t key_max, int nb_k,
                                          double tau, int k_target, int& n_gt, double& mass_gt, int& ties) {
  uint64_t lo = key_min, hi = key_max + 1;
  int cnt_lo = nb_k, cnt_hi = 0;
  double mass_hi = 0.0;
  while (cnt_lo - cnt_hi > 1 && hi - lo > 1) {
    const uint64_t mid = lo + ((hi - lo) >> 1);
    double s = 0.0;
    int c = 0;
#pragma unroll
    for (int r = 0; r < E; ++r) {
      const bool ge = static_cast<uint64_t>(__double_as_longlong(p[r])) >= mid;  // padding has key 0 < mid
      s += ge ? p[r] : 0.0;
      c += ge ? 1 : 0;
    }
    c = __builtin_amdgcn_readfirstlane(wave_sum_all(c));
    const double m = wave_sum_all(s);
    const bool holds = MASS ? (c >= 1 && m >= tau) : (c >= k_target);
    if (__builtin_amdgcn_readfirstlane(holds ? 1 : 0)) {
      lo = mid;
      cnt_lo = c;
    } else {
      hi = mid;
      cnt_hi = c;
      mass_hi = m;
    }
  }
  uint64_t T = lo;
  if (hi - lo > 1) {  // one block left in [lo, hi): its key is the threshold
    uint64_t best = 0;
#pragma unroll
    for (int r = 0; r < E; ++r) {
      const uint64_t key = static_cast<uint64_t>(__double_as_longlong(p[r]));
      if (key >= lo && key < hi) best = key;
    }
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const uint64_t other = static_cast<uint64_t>(__shfl_xor(static_cast<long long>(best), o));
      best = best > other ? best : other;
    }
    T = uniform64(best);
  }
  n_gt = cnt_hi;
  mass_gt = mass_hi;
  ties = cnt_lo - cnt_hi;
  return T;
}

template <int E>
__global__ __launch_bounds__(kThreads) void select_kernel(
    const double* __restrict__ logits, int nb_q, int nb_k, int64_t rows, double tau, double one_minus_rho,
    const uint8_t* __restrict__ force_q, const uint8_t* __restrict__ force_k, uint32_t* __restrict__ mask_bits,
    int32_t* __restrict__ kv_idx, int32_t* __restrict__ kv_cnt, int idx_stride) {
  const int lane = threadIdx.x & 63;
  const int64_t row = int64_t(blockIdx.x) * kWaves + (threadIdx.x >> 6);  // = head * nb_q + I
  if (row >= rows) return;  // whole wave; the kernel has no barriers
  const int I = static_cast<int>(row % nb_q);
  const double* lrow = logits + row * nb_k;

  // ---- softmax over the ranked blocks: p[r] belongs to block J = 64 r + lane.  Padding (J >= nb_k)
  // and blocks with force_k[J] == 2 (always kept, not ranked) get p = 0 and take no part below.
  double p[E];
  unsigned long long ranked[(E + 63) / 64] = {};  // bit r: block 64 r + lane is ranked
  double mx = -INFINITY;
#pragma unroll
  for (int r = 0; r < E; ++r) {
    const int J = r * 64 + lane;
    bool rk = J < nb_k;
    if (rk && force_k != nullptr) rk = force_k[J] != 2;
    if (rk) ranked[r >> 6] |= 1ull << (r & 63);
    p[r] = rk ? lrow[J] : -INFINITY;
    mx = fmax(mx, p[r]);
  }
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) mx = fmax(mx, __shfl_xor(mx, o));
  int my_ranked = 0;
#pragma unroll
  for (int w = 0; w < (E + 63) / 64; ++w) my_ranked += __popcll(ranked[w]);
  const int nb_ranked = __builtin_amdgcn_readfirstlane(wave_sum_all(my_ranked));
  double z = 0.0;
#pragma unroll
  for (int r = 0; r < E; ++r) {
    p[r] = ((ranked[r >> 6] >> (r & 63)) & 1) ? exp(p[r] - mx) : 0.0;
    z += p[r];
  }
  z = wave_sum_all(z);
  double total = 0.0;
#pragma unroll
  for (int r = 0; r < E; ++r) {
    p[r] = ((ranked[r >> 6] >> (r & 63)) & 1) ? p[r] / z : 0.0;
    total += p[r];
  }
  total = wave_sum_all(total);
  // smallest and largest key among the ranked blocks: the range the bisection works on
  uint64_t key_min = ~0ull, key_max = 0;
#pragma unroll
  for (int r = 0; r < E; ++r) {
    const uint64_t key = static_cast<uint64_t>(__double_as_longlong(p[r]));
    if ((ranked[r >> 6] >> (r & 63)) & 1) {
      key_min = key < key_min ? key : key_min;
      key_max = key > key_max ? key : key_max;
    }
  }
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint64_t a = static_cast<uint64_t>(__shfl_xor(static_cast<long long>(key_min), o));
    const uint64_t b = static_cast<uint64_t>(__shfl_xor(static_cast<long long>(key_max), o));
    key_min = a < key_min ? a : key_min;
    key_max = b > key_max ? b : key_max;
  }
  key_min = uniform64(key_min);
  key_max = uniform64(key_max);

  // ---- threshold ----------------------------------------------------------------------------
  // k = floor(B (1 - rho)) in binary64 as the definition is written, B = number of ranked blocks
  const int k_floor = static_cast<int>(floor(static_cast<double>(nb_ranked) * one_minus_rho));
  const int k_target = min(nb_ranked, max(k_floor, 1));
  // tau >= 1 keeps every block by definition (the summed mass may round to 1.0 before blocks of
  // negligible mass are counted); so does a mass that never gets to tau, and a row with nothing ranked
  const bool keep_all = tau >= 1.0 || !(total >= tau) || nb_ranked == 0;
  uint64_t T = 0;
  int n_ties = 0;
  if (!keep_all) {
    int n_gt, ties;
    double mass_gt;
    int n_cdf = 1;  // tau <= 0: the first ranked block already covers it (top-k only selection)
    if (tau > 0.0) {
      T = find_threshold<E, true>(p, key_min, key_max, nb_ranked, tau, 0, n_gt, mass_gt, ties);
      const double pt = __longlong_as_double(static_cast<long long>(T));
      double run = mass_gt;
      n_ties = 0;
      do {
        run += pt;
        ++n_ties;
      } while (run < tau && n_ties < ties);
      n_cdf = n_gt + n_ties;
    }
    if (n_cdf < k_target || !(tau > 0.0)) {  // the top-k floor decides
      T = find_threshold<E, false>(p, key_min, key_max, nb_ranked, tau, k_target, n_gt, mass_gt, ties);
      n_ties = k_target - n_gt;
    }
  }
  const bool whole_row = force_q != nullptr && force_q[I] != 0;

  // ---- emit: 64 blocks per step = two mask words; ties are ranked by block index ---------------
  const int words = (nb_k + 31) >> 5;
  const unsigned long long below = (1ull << lane) - 1ull;
  int running = 0, tie_run = 0;
#pragma unroll
  for (int r = 0; r < E; ++r) {
    if (r * 64 < nb_k) {  // uniform
      const int J = r * 64 + lane;
      const bool valid = J < nb_k;
      const uint64_t key = static_cast<uint64_t>(__double_as_longlong(p[r]));
      const bool rk = (ranked[r >> 6] >> (r & 63)) & 1;
      const bool tied = rk && key == T;
      const unsigned long long tb = __ballot(tied);
      const int tie_idx = tie_run + __popcll(tb & below);
      bool f = rk && (keep_all || key > T || (tied && tie_idx < n_ties));
      f = f || whole_row;
      if (valid && force_k != nullptr) f = f || force_k[J] != 0;
      f = f && valid;
      const unsigned long long bal = __ballot(f);
      if (mask_bits != nullptr && lane < 2 && 2 * r + lane < words)
        mask_bits[row * words + 2 * r + lane] = static_cast<uint32_t>(lane == 0 ? bal : (bal >> 32));
      if (f && kv_idx != nullptr) kv_idx[row * idx_stride + running + __popcll(bal & below)] = J;
      running += __popcll(bal);
      tie_run += __popcll(tb);
    }
  }
  if (lane == 0 && kv_cnt != nullptr) kv_cnt[row] = running;
}

template <int E>
void launch_select_rows(const double* logits, int heads, int nb_q, int nb_k, double tau, double one_minus_rho,
                        const uint8_t* force_q, const uint8_t* force_k, uint32_t* mask_bits, int32_t* kv_idx,
                        int32_t* kv_cnt, int idx_stride, hipStream_t stream) {
  const int64_t rows = int64_t(heads) * nb_q;
  hipLaunchKernelGGL(select_kernel<E>, dim3(static_cast<unsigned>((rows + kWaves - 1) / kWaves)), dim3(kThreads), 0,
                     stream, logits, nb_q, nb_k, rows, tau, one_minus_rho, force_q, force_k, mask_bits, kv_idx, kv_cnt,
                     idx_stride);
}

}  // namespace

size_t select_workspace_bytes(int heads, int nb_q, int nb_k) {
  return size_t(heads) * size_t(nb_q) * size_t(nb_k) * sizeof(double);
}

int launch_select(const double* q_pool, const double* k_pool, int heads, int nb_q, int nb_k, double score_scale,
                  double tau, double one_minus_rho, const uint8_t* force_q, const uint8_t* force_k, uint32_t* mask_bits,
                  int32_t* kv_idx, int32_t* kv_cnt, int idx_stride, void* workspace, hipStream_t stream) {
  double* logits = static_cast<double*>(workspace);
  constexpr int R = 4;
  hipLaunchKernelGGL(logits_kernel<R>, dim3((nb_q + R - 1) / R, heads), dim3(kThreads), 0, stream, q_pool, k_pool,
                     nb_q, nb_k, score_scale, logits);
  if (int rc = check_hip(hipGetLastError(), "bsga_select_blocks (logits) launch")) return rc;
  // per-lane register tile: the smallest instantiation that holds ceil(nb_k / 64) blocks per lane
  const int e = (nb_k + 63) / 64;
#define BSGA_SELECT_CASE(E_)                                                                                     \
  if (e <= E_) {                                                                                                 \
    launch_select_rows<E_>(logits, heads, nb_q, nb_k, tau, one_minus_rho, force_q, force_k, mask_bits, kv_idx, kv_cnt, \
                           idx_stride, stream);                                                                  \
  } else
  BSGA_SELECT_CASE(4)
  BSGA_SELECT_CASE(8)
  BSGA_SELECT_CASE(12)
  BSGA_SELECT_CASE(20)
  BSGA_SELECT_CASE(28)
  BSGA_SELECT_CASE(40)
  BSGA_SELECT_CASE(52)
  BSGA_SELECT_CASE(64)
  BSGA_SELECT_CASE(96)
  BSGA_SELECT_CASE(128) { return fail(BSGA_ERR_UNSUPPORTED, "bsga_select_blocks: nb_k = %d exceeds 8192", nb_k); }
#undef BSGA_SELECT_CASE
  return check_hip(hipGetLastError(), "bsga_select_blocks launch");
}

}  // namespace bsga
