// bf16 flash-style attention over kept key blocks for gfx950 (Sec. 4.1, Eq. (2); Eq. (1) when no
// index list is given).  bf16 MFMA (32x32x16) for both products, fp32 accumulation, fp32 online
// softmax in the log2 domain.
//
// Work split.  One workgroup per (head, query block of B rows); it walks the row's kept key
// blocks (tiles of B keys).  Waves are arranged WQ x 2: wave (qi, kh) owns 64 query rows (qi)
// and one half of every key tile (kh), so each K/V operand fetched from LDS feeds two MFMAs.
// The two key halves keep independent softmax states that are merged once at the end.  Two
// workgroups share a CU (two waves per SIMD), so one wave's softmax VALU work overlaps the
// other's MFMAs.
//
// Data movement.  K and V tiles go HBM/L2 -> LDS with direct-to-LDS loads (16 bytes per lane, no
// staging registers), double buffered: the loads of tile t+1 are in flight while tile t is
// computed.  Tiles stay row-major [key][64]; only the order of the eight 16-byte chunks inside a
// row is permuted (XOR swizzle, chosen per tensor) so the operand reads below are conflict free.
//
// Register layouts.  Scores are produced transposed, S^T = K Q^T (M = keys, N = queries): in the
// 32x32 accumulator layout lane (n = lane%32, g = lane/32) holds, for query n, the keys
// 8*r4 + 4*g + r (register 4*r4 + r).  A lane owns whole query columns, so row max/sum need one
// cross-lane step (lane ^ 32), and after exponentiation the same registers are, with no data
// movement, the B operand of O^T += V^T P^T if the contraction index is taken in the order the
// accumulator holds the keys.  The matching A operand (V^T: 32 dims x 16 keys) is read from the
// row-major V tile with the LDS transpose read (ds_read_b64_tr_b16): each 16-lane group names four
// keys and gets, per lane, those four keys' values of one dim.
//
// Softmax.  Q is pre-multiplied by softmax_scale*log2(e) when it is loaded, and the accumulator
// of the score MFMA is initialised to -m_ref (the lane's reference maximum), so the MFMA result
// is already the exponent of exp2.  m_ref is raised only when a tile exceeds it by more than
// 2^8 (the weights then stay <= 256, harmless in fp32/bf16); the final O / l is exact for any
// reference, so this only skips rescaling work.  Row sums are taken from the bf16-rounded
// weights (dot2 with ones), i.e. from exactly what multiplies V.
#include <stdio.h>
#include <stdlib.h>

#include <type_traits>

#include "bsga_internal.h"

namespace bsga {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

#define LDS_PTR(T, p) ((const T __attribute__((address_space(3)))*)(p))

constexpr int kD = 64;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kRaise = 8.0f;  // raise the reference maximum when a tile exceeds it by 2^8

// chunk swizzles: 16-byte chunk c of tile row r is stored at chunk position c ^ swz(r)
__device__ __forceinline__ int swz_k(int row) { return (row ^ (row >> 3)) & 7; }
__device__ __forceinline__ int swz_v(int row) { return (row & 3) << 1; }

__device__ __forceinline__ unsigned pack_bf16(float a, float b) {
  const f32x2 two = {a, b};
  return __builtin_bit_cast(unsigned, __builtin_convertvector(two, bf16x2));
}

__device__ __forceinline__ float xor32(float x) { return __shfl_xor(x, 32); }

typedef int i32x4 __attribute__((ext_vector_type(4)));

// 16 bytes per lane from a raw buffer straight into LDS (buffer_load_dwordx4 ... lds): lane i's
// data lands at LDS byte address lds_addr + 16 i.  voff is the per-lane byte offset, soff a
// wave-uniform one; reads past the buffer's size return 0.  Written as inline assembly on purpose:
// the compiler then does not count these loads as LDS writes and so does not make later LDS reads
// of the *other* buffer wait for them; the kernel orders them itself (s_waitcnt vmcnt + barrier).
__device__ __forceinline__ void dma16(i32x4 rsrc, unsigned voff, unsigned soff, unsigned lds_addr) {
  unsigned saved_m0;  // M0 (the LDS base of the load) is put back, so the statement has no side effect on it
  asm volatile(
      "s_mov_b32 %0, m0\n\t"
      "s_mov_b32 m0, %1\n\t"
      "buffer_load_dwordx4 %2, %3, %4 offen lds\n\t"
      "s_mov_b32 m0, %0"
      : "=&s"(saved_m0)
      : "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff)
      : "memory");
}

// raw buffer descriptor over [base, base + bytes): stride 0, 32-bit element data format
__device__ __forceinline__ i32x4 make_rsrc(const void* base, unsigned bytes) {
  const unsigned long long a = reinterpret_cast<unsigned long long>(base);
  const i32x4 r = {__builtin_amdgcn_readfirstlane(static_cast<int>(static_cast<unsigned>(a))),
                   __builtin_amdgcn_readfirstlane(static_cast<int>(static_cast<unsigned>(a >> 32) & 0xffffu)),
                   __builtin_amdgcn_readfirstlane(static_cast<int>(bytes)), 0x00020000};
  return r;
}

template <int B>
__global__ __launch_bounds__(2 * B, 2) void attn_bf16_kernel(
    const unsigned char* __restrict__ q, const unsigned char* __restrict__ k, const unsigned char* __restrict__ v,
    unsigned short* __restrict__ out, float* __restrict__ lse, const int32_t* __restrict__ kv_idx,
    const int32_t* __restrict__ kv_cnt, int idx_stride, int64_t n_tokens, int nb, float scale_log2) {
  constexpr int WQ = B / 64;              // waves along queries
  constexpr int KW = B / 2;               // keys per wave per tile
  constexpr int MB = KW / 32;             // 32-key MFMA row blocks per wave
  constexpr int KC = KW / 16;             // 16-key contraction chunks per wave in P V
  constexpr int NW = B / 32;              // waves per workgroup
  constexpr int TILE_BYTES = B * 128;     // one K or V tile
  constexpr int BUF_BYTES = 2 * TILE_BYTES;
  extern __shared__ __align__(1024) unsigned char smem[];  // [2 buffers][K tile | V tile]

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int n = lane & 31;
  const int g = lane >> 5;
  const int qi = wave % WQ;
  const int kh = wave / WQ;
  const int I = blockIdx.x;
  const int h = blockIdx.y;
  const int64_t head_bytes = int64_t(h) * n_tokens * 128;
  const int64_t rowid = int64_t(h) * nb + I;
  // raw buffer views of this head's K and V (byte-addressed, bounds-checked by the hardware)
  const unsigned head_size = static_cast<unsigned>(n_tokens * 128);
  const i32x4 krsrc = make_rsrc(k + head_bytes, head_size);
  const i32x4 vrsrc = make_rsrc(v + head_bytes, head_size);
  const unsigned smem_addr =
      static_cast<unsigned>(reinterpret_cast<size_t>((__attribute__((address_space(3))) unsigned char*)smem));

  // ---- Q fragments (B operand of S^T = K Q^T), pre-scaled: lane (n, g) holds dims 16c + 8g .. +7
  bf16x8 qf[2][4];
#pragma unroll
  for (int b2 = 0; b2 < 2; ++b2) {
    const int64_t row = int64_t(I) * B + qi * 64 + b2 * 32 + n;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      u32x4 x = {0u, 0u, 0u, 0u};
      if (row < n_tokens) x = *reinterpret_cast<const u32x4*>(q + head_bytes + row * 128 + (2 * c + g) * 16);
      u32x4 y;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float lo = __uint_as_float(x[e] << 16) * scale_log2;
        const float hi = __uint_as_float(x[e] & 0xffff0000u) * scale_log2;
        y[e] = pack_bf16(lo, hi);
      }
      qf[b2][c] = __builtin_bit_cast(bf16x8, y);
    }
  }

  // ---- per-lane constants -------------------------------------------------------------------------
  // direct-to-LDS loads: wave-load j covers LDS bytes [1024 j, 1024 j + 1024) of a tile; this wave
  // issues j = wave + NW*i, i = 0..3, for the K tile and for the V tile.  Lane -> LDS position
  // p = 64 j + lane -> (row p/8, chunk position p%8) -> global chunk (p%8) ^ swz(row).  Row r_i is
  // r_0 + 8 NW i with r_0 < 8 NW, so swz_k(r_i) = swz_k(r_0) ^ swz_k(8 NW i) and swz_v(r_i) =
  // swz_v(r_0): the K offsets repeat with period KN in i up to a multiple of 1024 NW (which goes
  // into the wave-uniform offset), the V offsets differ by that multiple only.
  constexpr int KN = (B == 128) ? 2 : 4;
  const int dma_r0 = wave * 8 + (lane >> 3);
  const int dma_pc = lane & 7;
  unsigned koff[KN];
#pragma unroll
  for (int i = 0; i < KN; ++i) {
    const int r = dma_r0 + 8 * NW * i;
    koff[i] = r * 128 + ((dma_pc ^ swz_k(r)) << 4);
  }
  const unsigned voff = dma_r0 * 128 + ((dma_pc ^ swz_v(dma_r0)) << 4);
  // K operand reads (ds_read_b128): row r = kh*KW + mb*32 + n, logical chunk 2c + g.  Since
  // swz_k(r + 32) = swz_k(r) ^ 4, block mb = 1 reads chunk c where block 0 reads chunk c ^ 2.
  unsigned kaddr[4];
  {
    const int r = kh * KW + n;
#pragma unroll
    for (int c = 0; c < 4; ++c) kaddr[c] = r * 128 + (((2 * c + g) ^ swz_k(r)) << 4);
  }
  // V operand reads (transpose read, 8 bytes per lane): 16-lane group G = lane/16 covers dims
  // db*32 + 16*(G&1) .. +15 for key-slot half g = G/2; inside the group lane i names key
  // m = i/4 of the four and the dim quad j = i%4.
  unsigned vaddr[2];
  {
    const int i16 = lane & 15, m = i16 >> 2, j = i16 & 3, G = lane >> 4;
    const int keyl = kh * KW + 4 * g + m;  // + 16*kc + 8*t added as an immediate
#pragma unroll
    for (int db = 0; db < 2; ++db) {
      const int cc = db * 4 + 2 * (G & 1) + (j >> 1);
      vaddr[db] = TILE_BYTES + keyl * 128 + ((cc ^ swz_v(keyl)) << 4) + (j & 1) * 8;
    }
  }

  f32x16 o[2][2];
  float m_ref[2];  // reference maximum per query column (log2 domain); unused by the fast pass
  float l_run[2];  // this lane's share of the row sum

  const bool dense = kv_idx == nullptr;
  const int count = dense ? nb : min(max(kv_cnt[rowid], 0), nb);
  const int32_t* my_idx = dense ? nullptr : kv_idx + rowid * idx_stride;
  const int tail = static_cast<int>(n_tokens - int64_t(nb - 1) * B);  // valid keys in the last tile

  // The row's key-block list is read 64 entries at a time, one per lane, and handed out with
  // readlane; the next 64 are already in flight while the current ones are consumed.
  int idx_cur = 0, idx_next = 0;
  auto load_idx = [&](int first) {
    const int t = first + lane;
    return (!dense && t < count) ? my_idx[t] : 0;
  };
  auto block_at = [&](int it) {  // must be called with it = 0, 1, 2, ... in order
    if (dense) return it;
    if (it > 0 && (it & 63) == 0) {
      idx_cur = idx_next;
      idx_next = load_idx(it + 64);
    }
    const int J = __builtin_amdgcn_readlane(idx_cur, it & 63);
    return min(max(J, 0), nb - 1);
  };
  // Direct-to-LDS load number i (0..7) of key tile J into buffer `buf`: even i moves 1 KB of the K
  // tile, odd i 1 KB of the V tile.  The eight loads of a tile are issued one at a time between
  // MFMAs so that they never queue up in front of the LDS reads.  Rows of a ragged last tile that
  // lie past the end of the head's buffer are out of range for the hardware bounds check, which
  // makes the load write zeros for them.
  auto issue_part = [&](int J, int buf, int i2) {
    const int i = i2 >> 1;
    const bool is_v = (i2 & 1) != 0;
    const unsigned soff = static_cast<unsigned>(J) * TILE_BYTES;
    const unsigned dst = smem_addr + buf * BUF_BYTES + wave * 1024 + (is_v ? TILE_BYTES : 0) + NW * i * 1024;
    if (is_v) {
      dma16(vrsrc, voff, soff + i * NW * 1024, dst);
    } else {
      dma16(krsrc, koff[i % KN], soff + (i / KN) * KN * NW * 1024, dst);
    }
  };
  auto issue = [&](int J, int buf) {
#pragma unroll
    for (int i2 = 0; i2 < 8; ++i2) issue_part(J, buf, i2);
  };

  // K operands (A of S^T = K Q^T) of 32-key sub-tile mb from the tile in buffer `buf`.  Chunk c of
  // sub-tile 1 sits where chunk c ^ 2 of sub-tile 0 does (swz_k(r + 32) = swz_k(r) ^ 4).
  bf16x8 ka[4];
  auto read_k = [&](int buf, int mb) {
#pragma unroll
    for (int c = 0; c < 4; ++c)
      ka[c] = *LDS_PTR(bf16x8, smem + buf * BUF_BYTES + kaddr[(mb & 1) ? (c ^ 2) : c] + mb * 4096);
  };

  // One key tile, software pipelined against its neighbours.  On entry the tile's data is in
  // buffer BUF, visible to every wave, and ka holds the K operands of its first sub-tile.  Per
  // 32-key sub-tile: scores (8 MFMAs) -> weights (VALU) -> O update (8 MFMAs).  Before the last O
  // update the workgroup synchronises: from then on nobody reads buffer BUF any more, so the loads
  // of tile it+2 are started into it, and tile it+1 (in the other buffer) is known to have landed,
  // so its first K operands are fetched while the last 8 MFMAs run.
  //
  // SAFE = false (fast pass): weights are exp2 of the raw scaled logits, i.e. the softmax reference
  // is 0 for every row.  Any reference gives the same O / l; the choice only matters for range, and
  // the caller checks the range afterwards.  No maximum is tracked and nothing is subtracted.
  // SAFE = true: classic online softmax.  The accumulator of the score MFMA starts at -m_ref so the
  // MFMA result is already relative to the reference, and m_ref is raised only when a tile exceeds
  // it by more than 2^kRaise.
  auto step = [&](auto bufc, auto safec, int it, bool ragged, int J_next2) {
    constexpr int buf = decltype(bufc)::value;
    constexpr bool SAFE = decltype(safec)::value;
    const unsigned char* tile = smem + buf * BUF_BYTES;

#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const bool last = (mb == MB - 1);
      // V^T operands of this sub-tile: [dim block][16-key chunk] = two 4-key transpose reads each
      bf16x8 va[2][2];
#pragma unroll
      for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int cp = 0; cp < 2; ++cp) {
          const int key0 = (2 * mb + cp) * 16;
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (s16x4 __attribute__((address_space(3)))*)(tile + vaddr[db] + key0 * 128));
          const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (s16x4 __attribute__((address_space(3)))*)(tile + vaddr[db] + (key0 + 8) * 128));
          const u32x2 lo2 = __builtin_bit_cast(u32x2, lo), hi2 = __builtin_bit_cast(u32x2, hi);
          const u32x4 av = {lo2[0], lo2[1], hi2[0], hi2[1]};
          va[db][cp] = __builtin_bit_cast(bf16x8, av);
        }

      // ---- S^T = K Q^T (- m_ref) for 32 keys x 64 queries ------------------------------------------
      float base[2] = {0.f, 0.f};
      f32x16 sc[2];
#pragma unroll
      for (int b2 = 0; b2 < 2; ++b2) {
        if constexpr (SAFE) base[b2] = (m_ref[b2] == -INFINITY) ? 0.f : m_ref[b2];
#pragma unroll
        for (int i = 0; i < 16; ++i) sc[b2][i] = SAFE ? -base[b2] : 0.f;
      }
#pragma unroll
      for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int b2 = 0; b2 < 2; ++b2)
          sc[b2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[c], qf[b2][c], sc[b2], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if (!last) read_k(buf, mb + 1);  // lands while the weights below are computed
      if constexpr (SAFE) {
        // Ragged last key block: its rows past the end were loaded as zeros (score 0, value 0).
        // The running-max form masks them out; the fast pass instead lets each contribute a weight
        // of exactly 2^0 = 1 to the row sum and nothing to O, and subtracts their count at the end.
        if (ragged) {
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int key = kh * KW + mb * 32 + 8 * (i >> 2) + 4 * g + (i & 3);
            if (key >= tail) {
              sc[0][i] = -INFINITY;
              sc[1][i] = -INFINITY;
            }
          }
        }
      }

      // ---- softmax weights, per query column -----------------------------------------------------
      bf16x8 pf[2][2];
#pragma unroll
      for (int b2 = 0; b2 < 2; ++b2) {
        if constexpr (SAFE) {
          float tmax = -INFINITY;
#pragma unroll
          for (int i = 0; i < 16; ++i) tmax = fmaxf(tmax, sc[b2][i]);
          tmax = fmaxf(tmax, xor32(tmax));
          const bool unset = m_ref[b2] == -INFINITY;
          const bool raise = unset ? (tmax > -INFINITY) : (tmax > kRaise);
          if (__any(raise)) {  // rare after the first tile
            const float shift = raise ? tmax : 0.f;
            const float alpha = unset ? 1.f : exp2f(-shift);  // nothing accumulated yet while unset
            if (raise) m_ref[b2] = base[b2] + shift;
            l_run[b2] *= alpha;
#pragma unroll
            for (int db = 0; db < 2; ++db)
#pragma unroll
              for (int i = 0; i < 16; ++i) o[db][b2][i] *= alpha;
#pragma unroll
            for (int i = 0; i < 16; ++i) sc[b2][i] -= shift;
          }
        }
        const bf16x2 ones = {static_cast<__bf16>(1.0f), static_cast<__bf16>(1.0f)};
        float rowsum = l_run[b2];
#pragma unroll
        for (int cp = 0; cp < 2; ++cp) {
          u32x4 w;
#pragma unroll
          for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
            for (int r2 = 0; r2 < 2; ++r2) {
              const int i0 = 4 * (2 * cp + t2) + 2 * r2;
              const unsigned pk = pack_bf16(__builtin_amdgcn_exp2f(sc[b2][i0]), __builtin_amdgcn_exp2f(sc[b2][i0 + 1]));
              rowsum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk), ones, rowsum, false);
              w[2 * t2 + r2] = pk;
            }
          pf[b2][cp] = __builtin_bit_cast(bf16x8, w);
        }
        l_run[b2] = rowsum;
      }
      __builtin_amdgcn_sched_barrier(0);

      if (last) {
        // every LDS read of this tile has been issued; once all waves are here the buffer is free
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's share of tile it+1 has landed
        __syncthreads();
        if (it + 1 < count) read_k(buf ^ 1, 0);
        __builtin_amdgcn_sched_barrier(0);
      }

      // ---- O^T += V^T P^T, with the loads of tile it+2 slotted between the last MFMAs -------------
#pragma unroll
      for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int cp = 0; cp < 2; ++cp)
#pragma unroll
          for (int b2 = 0; b2 < 2; ++b2) {
            o[db][b2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[db][cp], pf[b2][cp], o[db][b2], 0, 0, 0);
            if (last) {
              if (it + 2 < count) issue_part(J_next2, buf, (db * 2 + cp) * 2 + b2);
              __builtin_amdgcn_sched_barrier(0);
            }
          }
    }
  };

  // A whole pass over the row's key tiles, then the merge of the two key halves: wave (qi, 1)
  // parks its state in LDS as [qi][68 values][64 lanes] and wave (qi, 0) folds it in.  Returns
  // true (to every thread of the workgroup) if the pass must be repeated in SAFE mode because a
  // row sum or an output left the range in which the reference-free weights are trustworthy:
  // a weight 2^s overflows for s >= 128 (the sum then exceeds the upper limit or O is not finite),
  // and weights below 2^-126 flush to zero, which is harmless as long as the row sum is at least
  // 2^-80 (at most 2^24 keys x 2^-126 lost, a relative error under 2^-22 ... 2^-29).
  auto pass = [&](auto safec) -> bool {
    constexpr bool SAFE = decltype(safec)::value;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b2 = 0; b2 < 2; ++b2)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[a][b2][i] = 0.f;
    m_ref[0] = m_ref[1] = -INFINITY;
    l_run[0] = l_run[1] = 0.f;
    idx_cur = load_idx(0);
    idx_next = load_idx(64);
    // prologue: tile 0 -> buffer 0, wait for it, tile 1 -> buffer 1, first K operands
    int J_cur = 0, J_nxt = 0;
    if (count > 0) {
      J_cur = block_at(0);
      issue(J_cur, 0);
      if (count > 1) J_nxt = block_at(1);
      __builtin_amdgcn_s_waitcnt(0x0F70);
      __syncthreads();
      if (count > 1) issue(J_nxt, 1);
      read_k(0, 0);
    }
    int pad_keys = 0;  // zero-filled keys past the end that the fast pass has summed as weight 1
    auto tile_step = [&](auto bufc, int it, int J, int J_next2) {
      const bool ragged = (J == nb - 1 && tail < B);
      if (ragged) pad_keys += B - tail;
      step(bufc, safec, it, ragged, J_next2);
    };
    for (int it = 0; it < count; it += 2) {
      int J2 = (it + 2 < count) ? block_at(it + 2) : 0;
      tile_step(std::integral_constant<int, 0>{}, it, J_cur, J2);
      if (it + 1 >= count) break;
      const int J3 = (it + 3 < count) ? block_at(it + 3) : 0;
      tile_step(std::integral_constant<int, 1>{}, it + 1, J_nxt, J3);
      J_cur = J2;
      J_nxt = J3;
    }
    __syncthreads();  // every wave is done reading the tiles: LDS can be reused

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
        park[(64 + b2) * 64 + lane] = m_ref[b2];
        park[(66 + b2) * 64 + lane] = l_run[b2];
      }
    }
    __syncthreads();
    bool bad = false;
    float lt[2], mt[2];
    if (kh == 0) {
#pragma unroll
      for (int b2 = 0; b2 < 2; ++b2) {
        const float l1 = park[(66 + b2) * 64 + lane];
        float a0 = 1.f, a1 = 1.f;
        mt[b2] = 0.f;
        if constexpr (SAFE) {
          const float m1 = park[(64 + b2) * 64 + lane];
          const float m0 = m_ref[b2];
          mt[b2] = fmaxf(m0, m1);
          const float mu = (mt[b2] == -INFINITY) ? 0.f : mt[b2];
          a0 = exp2f(m0 - mu);  // exp2f(-inf) = 0 for a half that saw nothing
          a1 = exp2f(m1 - mu);
        }
        float l = l_run[b2] * a0 + l1 * a1;
        l += xor32(l);
        if constexpr (!SAFE) l -= static_cast<float>(pad_keys);
        lt[b2] = l;
        if constexpr (!SAFE) bad = bad || !(l >= 0x1p-80f && l <= 0x1p100f);
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            o[db][b2][i] = o[db][b2][i] * a0 + park[((db * 2 + b2) * 16 + i) * 64 + lane] * a1;
            if constexpr (!SAFE) bad = bad || !(fabsf(o[db][b2][i]) < INFINITY);
          }
      }
    }
    if constexpr (!SAFE) {
      if (__syncthreads_or(bad)) return true;
    }
    if (kh == 0) {
#pragma unroll
      for (int b2 = 0; b2 < 2; ++b2) {
        const float inv = lt[b2] > 0.f ? 1.f / lt[b2] : 0.f;
        const int64_t row = int64_t(I) * B + qi * 64 + b2 * 32 + n;
        if (row < n_tokens) {
#pragma unroll
          for (int db = 0; db < 2; ++db)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
              const f32x16& x = o[db][b2];
              const int i = 4 * r4;
              const u32x2 w = {pack_bf16(x[i] * inv, x[i + 1] * inv), pack_bf16(x[i + 2] * inv, x[i + 3] * inv)};
              *reinterpret_cast<u32x2*>(out + (int64_t(h) * n_tokens + row) * kD + db * 32 + 8 * r4 + 4 * g) = w;
            }
          if (lse != nullptr && g == 0)
            lse[int64_t(h) * n_tokens + row] = lt[b2] > 0.f ? (mt[b2] + log2f(lt[b2])) * kLn2 : -INFINITY;
        }
      }
    }
    return false;
  };

  if (pass(std::false_type{})) {
    __syncthreads();  // the parked state has been read by everyone: LDS is free for tiles again
    pass(std::true_type{});
  }
}

}  // namespace

int launch_attn_bf16(const void* q, const void* k, const void* v, int heads, int64_t n_tokens, int block,
                     float softmax_scale, const int32_t* kv_idx, const int32_t* kv_cnt, int idx_stride, void* out,
                     float* lse, void* workspace, hipStream_t stream) {
  (void)workspace;
  const int nb = static_cast<int>(ceil_div(n_tokens, block));
  const float scale_log2 = softmax_scale * kLog2e;
  dim3 grid(nb, heads);
  const unsigned char* qp = static_cast<const unsigned char*>(q);
  const unsigned char* kp = static_cast<const unsigned char*>(k);
  const unsigned char* vp = static_cast<const unsigned char*>(v);
  unsigned short* op = static_cast<unsigned short*>(out);
  if (getenv("BSGA_DEBUG") != nullptr) {
    int n64 = -1, n128 = -1;
    (void)hipOccupancyMaxActiveBlocksPerMultiprocessor(&n64, attn_bf16_kernel<64>, 128, 4 * 64 * 128);
    (void)hipOccupancyMaxActiveBlocksPerMultiprocessor(&n128, attn_bf16_kernel<128>, 256, 4 * 128 * 128);
    fprintf(stderr, "[bsga] attention occupancy (workgroups per CU): block 64 -> %d, block 128 -> %d\n", n64, n128);
  }
  if (block == 64) {
    hipLaunchKernelGGL((attn_bf16_kernel<64>), grid, dim3(128), 4 * 64 * 128, stream, qp, kp, vp, op, lse, kv_idx,
                       kv_cnt, idx_stride, n_tokens, nb, scale_log2);
  } else {
    hipLaunchKernelGGL((attn_bf16_kernel<128>), grid, dim3(256), 4 * 128 * 128, stream, qp, kp, vp, op, lse, kv_idx,
                       kv_cnt, idx_stride, n_tokens, nb, scale_log2);
  }
  return check_hip(hipGetLastError(), "bsga bf16 attention launch");
}

}  // namespace bsga
