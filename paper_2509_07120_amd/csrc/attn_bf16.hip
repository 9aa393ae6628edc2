// bf16 flash-style attention over kept key blocks for gfx950 (Sec. 4.1, Eq. (2); Eq. (1) when no
// index list is given).  bf16 MFMA (32x32x16) for both products, fp32 accumulation, fp32 online
// softmax in the log2 domain.
//
// Work split.  One workgroup per (head, query block of B rows); it walks the row's kept key
// blocks (tiles of B keys).  Waves are arranged WQ x 2: wave (qi, kh) owns 64 query rows
// (qi) and one half of every key tile (kh), so each K/V^T operand fetched from LDS feeds two
// MFMAs.  The two key halves keep independent softmax states that are merged once at the end.
//
// Register layouts.  Scores are produced transposed, S^T = K Q^T (M = keys, N = queries): in the
// 32x32 accumulator layout lane (n = lane%32, g = lane/32) then holds, for query n, the keys
// 8*r4 + 4*g + r (register 4*r4 + r).  A lane therefore owns whole query columns: row max/sum
// need one cross-lane step (lane ^ 32), and after exponentiation the same registers are, without
// any data movement, the B operand of O^T += V^T P^T provided the contraction index ("slot")
// is permuted as  slot 16c + 8g + 4t + r  <->  key 16c + 8t + 4g + r.  V is repacked once per call
// into that slot order, transposed to [dim][slot] per key tile and pre-swizzled for
// conflict-free 16-byte LDS reads, so that a key tile of V^T is one contiguous 64 x B block.
#include "bsga_internal.h"

namespace bsga {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

constexpr int kD = 64;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kLog2e = 1.4426950408889634f;

// 16-byte chunk swizzles (chunk index within a row of the LDS tile)
__device__ __host__ inline int swz_k(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }
template <int B>
__device__ __host__ inline int swz_v(int row, int chunk) {
  return (B == 128) ? (chunk ^ (row & 15)) : (chunk ^ ((row >> 1) & 7));
}
// contraction slot -> key offset inside a key tile
__device__ __host__ inline int slot_to_key(int s) {
  return (s & ~15) | ((s & 4) << 1) | ((s & 8) >> 1) | (s & 3);
}

// ---------------------------------------------------------------------------------------------
// V repack: V [H, N, 64] -> workspace [H, NB, 64 dims, B slots] (slot-permuted, chunk-swizzled,
// keys past N zero-filled).
template <int B>
__global__ __launch_bounds__(256) void repack_v_kernel(const uint4* __restrict__ v, uint4* __restrict__ vt,
                                                       int64_t n_tokens, int nb) {
  constexpr int PITCH = kD + 2;  // ushorts per staged key row (odd dword pitch)
  __shared__ unsigned short tile[B * PITCH];
  const int J = blockIdx.x;
  const int h = blockIdx.y;
  const int t = threadIdx.x;
  const int64_t key0 = int64_t(J) * B;
  const int valid = static_cast<int>(min<int64_t>(B, n_tokens - key0));
  const uint4* src = v + (int64_t(h) * n_tokens + key0) * 8;
  for (int c = t; c < B * 8; c += 256) {
    const int r = c >> 3, d8 = c & 7;
    uint4 x = make_uint4(0, 0, 0, 0);
    if (r < valid) x = src[c];
    unsigned* dst = reinterpret_cast<unsigned*>(&tile[r * PITCH + d8 * 8]);
    dst[0] = x.x; dst[1] = x.y; dst[2] = x.z; dst[3] = x.w;
  }
  __syncthreads();
  constexpr int CPR = B / 8;  // 16-byte chunks per output row
  uint4* dstt = vt + (int64_t(h) * nb + J) * (kD * CPR);
  for (int p = t; p < kD * CPR; p += 256) {
    const int row = p / CPR, pc = p % CPR;
    const int cc = swz_v<B>(row, pc);  // XOR swizzle is its own inverse
    unsigned short e[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) e[i] = tile[slot_to_key(cc * 8 + i) * PITCH + row];
    uint4 o;
    o.x = e[0] | (unsigned(e[1]) << 16); o.y = e[2] | (unsigned(e[3]) << 16);
    o.z = e[4] | (unsigned(e[5]) << 16); o.w = e[6] | (unsigned(e[7]) << 16);
    dstt[p] = o;
  }
}

// global -> registers for key tile J: K rows in swizzled chunk order (rows past the end read as
// zero), the V^T tile as a straight copy.  Thread `tid` of 2B owns chunks tid, tid + 2B, ...
template <int B>
__device__ __forceinline__ void fetch_tile(const u32x4* __restrict__ k, const u32x4* __restrict__ vt,
                                           int64_t head_chunks, int h, int nb, int tail, int J, int tid,
                                           u32x4 (&sk)[4], u32x4 (&sv)[4]) {
  const int64_t key0 = int64_t(J) * B;
  const int valid = (J == nb - 1) ? tail : B;
  const u32x4* vsrc = vt + (int64_t(h) * nb + J) * (B * 8);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int p = tid + i * 2 * B;
    const int r = p >> 3, pc = p & 7;
    const int rr = min(r, valid - 1);
    u32x4 x = k[head_chunks + (key0 + rr) * 8 + swz_k(r, pc)];
    if (r >= valid) x = u32x4{0u, 0u, 0u, 0u};
    sk[i] = x;
    sv[i] = vsrc[p];
  }
}
// registers -> LDS buffer (K tile followed by V^T tile)
template <int B>
__device__ __forceinline__ void commit_tile(unsigned char* buf, int tid, const u32x4 (&sk)[4],
                                            const u32x4 (&sv)[4]) {
  u32x4* kd = reinterpret_cast<u32x4*>(buf);
  u32x4* vd = reinterpret_cast<u32x4*>(buf + B * 128);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    kd[tid + i * 2 * B] = sk[i];
    vd[tid + i * 2 * B] = sv[i];
  }
}

// ---------------------------------------------------------------------------------------------
template <int B>
__global__ __launch_bounds__(2 * B) void attn_bf16_kernel(
    const u32x4* __restrict__ q, const u32x4* __restrict__ k, const u32x4* __restrict__ vt,
    unsigned short* __restrict__ out, float* __restrict__ lse, const int32_t* __restrict__ kv_idx,
    const int32_t* __restrict__ kv_cnt, int idx_stride, int64_t n_tokens, int nb, float scale_log2) {
  constexpr int WQ = B / 64;        // waves along queries
  constexpr int KW = B / 2;         // keys per wave per tile
  constexpr int MB = KW / 32;       // 32-key MFMA row blocks per wave
  constexpr int KC = KW / 16;       // 16-slot contraction chunks per wave in P V
  constexpr int THREADS = 2 * B;
  constexpr int TILE_BYTES = B * 128;
  constexpr int CHUNKS = B * 8;     // 16-byte chunks per tile
  constexpr int CPT = CHUNKS / THREADS;  // = 4 chunks per thread per tensor
  extern __shared__ __align__(16) unsigned char smem[];  // [2 buffers][K tile | V^T tile]

  const int tid = threadIdx.x;
  const int wave = tid >> 6;
  const int lane = tid & 63;
  const int n = lane & 31;
  const int g = lane >> 5;
  const int qi = wave % WQ;
  const int kh = wave / WQ;
  const int I = blockIdx.x;
  const int h = blockIdx.y;
  const int64_t head_chunks = int64_t(h) * n_tokens * 8;  // 16-byte chunks before this head in Q/K
  const int64_t rowid = int64_t(h) * nb + I;

  // ---- Q fragments (B operand of S^T = K Q^T): lane (n, g) holds dims 16c + 8g .. +7 of its row
  bf16x8 qf[2][4];
#pragma unroll
  for (int b2 = 0; b2 < 2; ++b2) {
    const int64_t row = int64_t(I) * B + qi * 64 + b2 * 32 + n;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      u32x4 x = u32x4{0u, 0u, 0u, 0u};
      if (row < n_tokens) x = q[head_chunks + row * 8 + 2 * c + g];
      qf[b2][c] = __builtin_bit_cast(bf16x8, x);
    }
  }

  f32x16 o[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b2 = 0; b2 < 2; ++b2)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[a][b2][i] = 0.f;
  float m_run[2] = {-INFINITY, -INFINITY};
  float l_run[2] = {0.f, 0.f};

  const bool dense = kv_idx == nullptr;
  const int count = dense ? nb : min(max(kv_cnt[rowid], 0), nb);
  const int32_t* my_idx = dense ? nullptr : kv_idx + rowid * idx_stride;
  const int tail = static_cast<int>(n_tokens - int64_t(nb - 1) * B);  // valid keys in the last tile

  u32x4 stage_k[CPT], stage_v[CPT];
  auto block_at = [&](int it) {
    int J = dense ? it : my_idx[it];
    return min(max(J, 0), nb - 1);
  };

  if (count > 0) {
    fetch_tile<B>(k, vt, head_chunks, h, nb, tail, block_at(0), tid, stage_k, stage_v);
    commit_tile<B>(smem, tid, stage_k, stage_v);
  }
  __syncthreads();

  for (int it = 0; it < count; ++it) {
    const int buf = it & 1;
    const int J = block_at(it);
    const bool more = it + 1 < count;
    if (more) fetch_tile<B>(k, vt, head_chunks, h, nb, tail, block_at(it + 1), tid, stage_k, stage_v);

    const unsigned char* kt = smem + buf * 2 * TILE_BYTES;
    const unsigned char* vtile = kt + TILE_BYTES;

    // ---- S^T = K Q^T ------------------------------------------------------------------------
    f32x16 s[MB][2];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int b2 = 0; b2 < 2; ++b2)
#pragma unroll
        for (int i = 0; i < 16; ++i) s[mb][b2][i] = 0.f;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const int r = kh * KW + mb * 32 + n;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(kt + r * 128 + (swz_k(r, 2 * c + g) << 4));
#pragma unroll
        for (int b2 = 0; b2 < 2; ++b2)
          s[mb][b2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[b2][c], s[mb][b2], 0, 0, 0);
      }
    }
    if (J == nb - 1 && tail < B) {  // ragged last key block: keys past the end get -inf
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int key = kh * KW + mb * 32 + 8 * (i >> 2) + 4 * g + (i & 3);
          if (key >= tail) {
            s[mb][0][i] = -INFINITY;
            s[mb][1][i] = -INFINITY;
          }
        }
    }

    // ---- online softmax (log2 domain), per query column ----------------------------------------
    bf16x8 pf[2][KC];
#pragma unroll
    for (int b2 = 0; b2 < 2; ++b2) {
      float tmax = -INFINITY;
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int i = 0; i < 16; ++i) tmax = fmaxf(tmax, s[mb][b2][i]);
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
      const float m_new = fmaxf(m_run[b2], tmax * scale_log2);
      const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
      const float alpha = exp2f(m_run[b2] - m_use);
      float rowsum = 0.f;
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float p = exp2f(fmaf(s[mb][b2][i], scale_log2, -m_use));
          s[mb][b2][i] = p;
          rowsum += p;
        }
      l_run[b2] = l_run[b2] * alpha + rowsum;
      m_run[b2] = m_new;
      if (__any(alpha != 1.f)) {
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
          for (int i = 0; i < 16; ++i) o[db][b2][i] *= alpha;
      }
#pragma unroll
      for (int kc = 0; kc < KC; ++kc) {
        const int mb = kc >> 1, cp = kc & 1;
        unsigned w[4];
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
          for (int r2 = 0; r2 < 2; ++r2) {
            const int i0 = 4 * (2 * cp + t2) + 2 * r2;
            const f32x2 two = {s[mb][b2][i0], s[mb][b2][i0 + 1]};
            w[2 * t2 + r2] = __builtin_bit_cast(unsigned, __builtin_convertvector(two, bf16x2));
          }
        const u32x4 pk = u32x4{w[0], w[1], w[2], w[3]};
        pf[b2][kc] = __builtin_bit_cast(bf16x8, pk);
      }
    }

    // ---- O^T += V^T P^T -----------------------------------------------------------------------
#pragma unroll
    for (int db = 0; db < 2; ++db) {
      const int row = db * 32 + n;
#pragma unroll
      for (int kc = 0; kc < KC; ++kc) {
        const int cc = (kh * KW + kc * 16 + g * 8) >> 3;
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(vtile + row * (2 * B) + (swz_v<B>(row, cc) << 4));
#pragma unroll
        for (int b2 = 0; b2 < 2; ++b2)
          o[db][b2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[b2][kc], o[db][b2], 0, 0, 0);
      }
    }

    if (more) commit_tile<B>(smem + (buf ^ 1) * 2 * TILE_BYTES, tid, stage_k, stage_v);
    __syncthreads();
  }

  // ---- merge the two key halves and write ---------------------------------------------------
  // wave (qi, 1) parks its state in LDS as [qi][68 values][64 lanes]; wave (qi, 0) folds it in.
  float* park = reinterpret_cast<float*>(smem) + qi * 68 * 64;
  if (kh == 1) {
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int b2 = 0; b2 < 2; ++b2)
#pragma unroll
        for (int i = 0; i < 16; ++i) park[((db * 2 + b2) * 16 + i) * 64 + lane] = o[db][b2][i];
#pragma unroll
    for (int b2 = 0; b2 < 2; ++b2) {
      park[(64 + b2) * 64 + lane] = m_run[b2];
      park[(66 + b2) * 64 + lane] = l_run[b2];
    }
  }
  __syncthreads();
  if (kh == 0) {
#pragma unroll
    for (int b2 = 0; b2 < 2; ++b2) {
      const float m1 = park[(64 + b2) * 64 + lane];
      const float l1 = park[(66 + b2) * 64 + lane];
      const float m0 = m_run[b2];
      const float mt = fmaxf(m0, m1);
      const float mu = (mt == -INFINITY) ? 0.f : mt;
      const float a0 = exp2f(m0 - mu), a1 = exp2f(m1 - mu);
      float lt = l_run[b2] * a0 + l1 * a1;
      lt += __shfl_xor(lt, 32);
      const float inv = lt > 0.f ? 1.f / lt : 0.f;
      const int64_t row = int64_t(I) * B + qi * 64 + b2 * 32 + n;
      if (row < n_tokens) {
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
          for (int r4 = 0; r4 < 4; ++r4) {
            float x[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const int i = 4 * r4 + r;
              x[r] = (o[db][b2][i] * a0 + park[((db * 2 + b2) * 16 + i) * 64 + lane] * a1) * inv;
            }
            const f32x2 lo = {x[0], x[1]}, hi = {x[2], x[3]};
            const bf16x2 blo = __builtin_convertvector(lo, bf16x2), bhi = __builtin_convertvector(hi, bf16x2);
            uint2 w;
            w.x = __builtin_bit_cast(unsigned, blo);
            w.y = __builtin_bit_cast(unsigned, bhi);
            *reinterpret_cast<uint2*>(out + (int64_t(h) * n_tokens + row) * kD + db * 32 + 8 * r4 + 4 * g) = w;
          }
        if (lse != nullptr && g == 0)
          lse[int64_t(h) * n_tokens + row] = lt > 0.f ? (mt + log2f(lt)) * kLn2 : -INFINITY;
      }
    }
  }
}

}  // namespace

int launch_attn_bf16(const void* q, const void* k, const void* v, int heads, int64_t n_tokens, int block,
                     float softmax_scale, const int32_t* kv_idx, const int32_t* kv_cnt, int idx_stride, void* out,
                     float* lse, void* workspace, hipStream_t stream) {
  const int nb = static_cast<int>(ceil_div(n_tokens, block));
  const float scale_log2 = softmax_scale * kLog2e;
  dim3 grid(nb, heads);
  const u32x4* qp = static_cast<const u32x4*>(q);
  const u32x4* kp = static_cast<const u32x4*>(k);
  u32x4* vt = static_cast<u32x4*>(workspace);
  unsigned short* op = static_cast<unsigned short*>(out);
  if (block == 64) {
    hipLaunchKernelGGL((repack_v_kernel<64>), grid, dim3(256), 0, stream, static_cast<const uint4*>(v), reinterpret_cast<uint4*>(vt), n_tokens, nb);
    hipLaunchKernelGGL((attn_bf16_kernel<64>), grid, dim3(128), 4 * 64 * 128, stream, qp, kp, vt, op, lse, kv_idx,
                       kv_cnt, idx_stride, n_tokens, nb, scale_log2);
  } else {
    hipLaunchKernelGGL((repack_v_kernel<128>), grid, dim3(256), 0, stream, static_cast<const uint4*>(v), reinterpret_cast<uint4*>(vt), n_tokens, nb);
    hipLaunchKernelGGL((attn_bf16_kernel<128>), grid, dim3(256), 4 * 128 * 128, stream, qp, kp, vt, op, lse, kv_idx,
                       kv_cnt, idx_stride, n_tokens, nb, scale_log2);
  }
  return check_hip(hipGetLastError(), "bsga bf16 attention launch");
}

}  // namespace bsga
