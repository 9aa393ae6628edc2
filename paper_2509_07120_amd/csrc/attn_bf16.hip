// bf16 flash-style attention over kept key blocks for gfx950 (Sec. 4.1, Eq. (2); Eq. (1) when no
// index list is given).  bf16 MFMA (32x32x16) for both products, fp32 accumulation, fp32 softmax
// weights in the log2 domain.
//
// Work split.  One workgroup per (head, query block of B rows); it walks the row's kept key
// blocks (tiles of B keys; with key blocks of B/2 keys a tile is two consecutive list entries).
// Blocks are those of a sequence cut in two separately blocked parts (Sec. 4.2; n_first = n_tokens
// is the plain blocking).  Waves are arranged WQ x 2: wave (qi, kh) owns 64 query rows (qi)
// and one half of every key tile (kh), so each K/V operand fetched from LDS into registers feeds
// two MFMAs (register-file traffic, not LDS bandwidth, is what this saves: LDS read data and MFMA
// operands share the VGPR ports).  The two key halves keep independent softmax states that are
// merged once at the end.  Two workgroups share a CU (two waves per SIMD).
// Which workgroup computes which row: see the top of the kernel (launch order, 64 consecutive rows
// per XCD, the last eighth of a large launch handed out at run time).
//
// Data movement.  K and V tiles go HBM/L2 -> LDS with direct-to-LDS loads (16 bytes per lane, no
// staging registers), double buffered, with one workgroup barrier per tile.  Tiles stay row-major
// [key][64]; only the order of the eight 16-byte chunks inside a row is permuted (XOR swizzle,
// chosen per tensor) so the operand reads below are bank-conflict free.
//
// Register layouts.  Scores are produced transposed, S^T = K Q^T (M = keys, N = queries): in the
// 32x32 accumulator layout lane (n = lane%32, g = lane/32) holds, for query n, the keys
// 8*r4 + 4*g + r (register 4*r4 + r).  A lane owns a whole query column, so row sums need one
// cross-lane step (lane ^ 32) at the very end, and after exponentiation the same registers are,
// with no data movement, the B operand of O^T += V^T P^T if the contraction index is taken in the
// order the accumulator holds the keys.  The matching A operand (V^T: 32 dims x 16 keys) is read
// from the row-major V tile with the LDS transpose read (ds_read_b64_tr_b16): each 16-lane group
// names four keys and gets, per lane, those four keys' values of one dim.
//
// Softmax.  Q is pre-multiplied by softmax_scale*log2(e) when it is loaded.  The fast pass takes
// the weights as exp2 of the raw scaled logits, i.e. with reference 0 for every row: any reference
// gives the same O / l, the choice only matters for range, and the range is checked afterwards
// (see pass()).  Only if that check fails is the workgroup repeated with a running reference
// maximum (SAFE pass).  V is multiplied by the bf16 roundings of the weights.  The pipelined loop
// sums those same bf16 weights (on the matrix pipe, see fast_loop), so numerator and denominator
// agree exactly; the plain tile code sums the fp32 weights, which differ from the bf16 ones by at
// most one rounding (2^-9 relative), the size of rounding the output itself.
//
// Tile rows that are not keys of the listed block (past the end of a ragged block, or the absent
// second half of a tile of half-size key blocks) get weight exactly 0: their scores are set to -inf
// before they are exponentiated.  Only the plain tile code masks; the pipelined loop runs over the
// row's leading full tiles and hands the rest of the row to the plain code.
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
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

#define LDS_PTR(T, p) ((const T __attribute__((address_space(3)))*)(p))

constexpr int kD = 64;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kRaise = 8.0f;  // SAFE pass: raise the reference maximum when a tile exceeds it by 2^8

template <int V>
using Int = std::integral_constant<int, V>;

// chunk swizzles: 16-byte chunk c of tile row r is stored at chunk position c ^ swz(r)
__device__ __forceinline__ int swz_k(int row) { return (row ^ (row >> 3)) & 7; }
__device__ __forceinline__ int swz_v(int row) { return (row & 3) << 1; }

__device__ __forceinline__ unsigned pack_bf16(float a, float b) {
  const f32x2 two = {a, b};
  return __builtin_bit_cast(unsigned, __builtin_convertvector(two, bf16x2));
}

__device__ __forceinline__ float xor32(float x) { return __shfl_xor(x, 32); }

// 16 bytes per lane from a raw buffer straight into LDS (buffer_load_dwordx4 ... lds): lane i's
// data lands at LDS byte address lds_base + lds_imm + 16 i.  voff is the per-lane byte offset, soff a
// wave-uniform one; lanes whose offset is past the buffer's size get zeros.  Written as inline
// assembly on purpose: the compiler then does not count these loads as LDS writes and so does not
// make later LDS reads of the *other* buffer wait for them; the kernel orders them itself
// (s_waitcnt vmcnt + barrier).  M0 (the LDS base of the load) is declared clobbered; nothing else in
// these kernels uses it.
template <unsigned LDS_IMM>
__device__ __forceinline__ void dma16(i32x4 rsrc, unsigned voff, unsigned soff, unsigned lds_base) {
  asm volatile(
      "s_add_u32 m0, %0, %4\n\t"
      "s_nop 0\n\t"  // one wait state between a scalar write of M0 and an LDS-DMA instruction that reads it
      "buffer_load_dwordx4 %1, %2, %3 offen lds"
      :
      : "s"(lds_base), "v"(voff), "s"(rsrc), "s"(soff), "n"(LDS_IMM)
      : "memory", "m0", "scc");
}

// raw buffer descriptor over [base, base + bytes): stride 0, 32-bit element data format
__device__ __forceinline__ i32x4 make_rsrc(const void* base, unsigned bytes) {
  const unsigned long long a = reinterpret_cast<unsigned long long>(base);
  const i32x4 r = {__builtin_amdgcn_readfirstlane(static_cast<int>(static_cast<unsigned>(a))),
                   __builtin_amdgcn_readfirstlane(static_cast<int>(static_cast<unsigned>(a >> 32) & 0xffffu)),
                   __builtin_amdgcn_readfirstlane(static_cast<int>(bytes)), 0x00020000};
  return r;
}

// Launch order of the (head, query block) rows.  Rows much longer than the average (more kept key
// blocks) go first, longest first, so that they do not end up alone at the end of the grid; all
// other rows keep the natural order (head-major), because workgroups of equal length that start
// together walk the keys together and share the K/V tiles in L2, and reordering rows of nearly
// equal length would only break that up.  Counting sort by kOrderClasses classes of kept count /
// nb; the classes whose lower bound is below 1.4 x the mean count are merged into one.  Four small
// kernels: per-head class histogram -> merge -> exclusive scan of the [class][head] table ->
// placement.  The rows of the merged class keep their natural order inside a head (neighbouring
// query blocks tend to keep similar key blocks); rows of one of the longer (class, head) groups come
// out in arbitrary order, which only changes which workgroup computes which row.
constexpr int kOrderClasses = 32;

__device__ __forceinline__ int order_class(int cnt, int nb) {  // class 0 holds the longest rows
  const int c = min(max(cnt, 0), nb);
  return (kOrderClasses - 1) - static_cast<int>((int64_t(c) * (kOrderClasses - 1)) / nb);
}

__global__ __launch_bounds__(256) void order_hist_kernel(const int32_t* __restrict__ kv_cnt, int nb, int nbk,
                                                         int heads, int32_t* __restrict__ table) {
  __shared__ int bins[kOrderClasses];
  const int h = blockIdx.x;
  const int t = threadIdx.x;
  if (t < kOrderClasses) bins[t] = 0;
  __syncthreads();
  for (int I = t; I < nb; I += 256) atomicAdd(&bins[order_class(kv_cnt[int64_t(h) * nb + I], nbk)], 1);
  __syncthreads();
  if (t < kOrderClasses) table[int64_t(t) * heads + h] = bins[t];
}

// One workgroup.  Finds the first class c_bulk whose lower bound (31 - c) / 31 is below 1.4 x the
// mean kept fraction, folds every lighter class into it (table rows c > c_bulk are added to row
// c_bulk and zeroed) and leaves c_bulk in table[kOrderClasses * heads].
__global__ __launch_bounds__(256) void order_merge_kernel(int32_t* __restrict__ table, int heads) {
  __shared__ long long total[kOrderClasses];
  __shared__ int c_bulk;
  const int t = threadIdx.x;
  if (t < kOrderClasses) total[t] = 0;
  __syncthreads();
  for (int64_t i = t; i < int64_t(kOrderClasses) * heads; i += 256)
    atomicAdd(reinterpret_cast<unsigned long long*>(&total[i / heads]), static_cast<unsigned long long>(table[i]));
  __syncthreads();
  if (t == 0) {
    double rows = 0.0, mass = 0.0;  // mass: kept fraction at the middle of each class
    for (int c = 0; c < kOrderClasses; ++c) {
      rows += static_cast<double>(total[c]);
      mass += static_cast<double>(total[c]) * (kOrderClasses - 1 - c + 0.5) / (kOrderClasses - 1);
    }
    const double mean = rows > 0.0 ? mass / rows : 1.0;
    int c = 0;
    while (c < kOrderClasses - 1 && static_cast<double>(kOrderClasses - 1 - c) / (kOrderClasses - 1) >= 1.4 * mean) ++c;
    c_bulk = c;
    table[int64_t(kOrderClasses) * heads] = c;
    table[int64_t(kOrderClasses) * heads + 1] = 0;  // the attention kernel's counter of rows handed out at run time
  }
  __syncthreads();
  const int cb = c_bulk;
  for (int h = t; h < heads; h += 256) {
    int sum = 0;
    for (int c = cb; c < kOrderClasses; ++c) {
      sum += table[int64_t(c) * heads + h];
      table[int64_t(c) * heads + h] = 0;
    }
    table[int64_t(cb) * heads + h] = sum;
  }
}

// in-place exclusive scan of table[0 .. n) by one workgroup
__global__ __launch_bounds__(1024) void order_scan_kernel(int32_t* __restrict__ table, int64_t n) {
  __shared__ int part[1024];
  __shared__ int carry;
  const int t = threadIdx.x;
  if (t == 0) carry = 0;
  __syncthreads();
  for (int64_t base = 0; base < n; base += 1024) {
    const int64_t i = base + t;
    const int x = i < n ? table[i] : 0;
    part[t] = x;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {
      const int add = t >= o ? part[t - o] : 0;
      __syncthreads();
      part[t] += add;
      __syncthreads();
    }
    const int before = carry;
    if (i < n) table[i] = before + part[t] - x;
    __syncthreads();
    if (t == 1023) carry = before + part[1023];
    __syncthreads();
  }
}

__global__ __launch_bounds__(256) void order_place_kernel(const int32_t* __restrict__ kv_cnt, int nb, int nbk,
                                                          int heads, const int32_t* __restrict__ table,
                                                          int32_t* __restrict__ order) {
  __shared__ int next[kOrderClasses];
  __shared__ int wave_bulk[4];
  const int h = blockIdx.x;
  const int t = threadIdx.x;
  if (t < kOrderClasses) next[t] = table[int64_t(t) * heads + h];
  const int c_bulk = table[int64_t(kOrderClasses) * heads];
  __syncthreads();
  int bulk_next = next[c_bulk];  // every thread keeps its own copy of the bulk group's fill position
  for (int base = 0; base < nb; base += 256) {
    const int I = base + t;
    const int cls = I < nb ? min(order_class(kv_cnt[int64_t(h) * nb + I], nbk), c_bulk) : -1;
    // the bulk group keeps the natural order of its rows: rank of this row among the chunk's bulk rows
    const bool bulk = cls == c_bulk;
    const unsigned long long vote = __ballot(bulk);
    const int below = __popcll(vote & ((1ull << (t & 63)) - 1ull));
    if ((t & 63) == 0) wave_bulk[t >> 6] = __popcll(vote);
    __syncthreads();
    int before = 0, chunk = 0;
    for (int w = 0; w < 4; ++w) {
      before += w < (t >> 6) ? wave_bulk[w] : 0;
      chunk += wave_bulk[w];
    }
    if (bulk) order[bulk_next + before + below] = h * nb + I;
    else if (cls >= 0) order[atomicAdd(&next[cls], 1)] = h * nb + I;
    bulk_next += chunk;
    __syncthreads();
  }
}

__global__ void zero_word_kernel(int* __restrict__ word) {
  if (threadIdx.x == 0) *word = 0;
}

// Token blocks.  The sequence is two segments, tokens [0, n_first) and [n_first, n_tokens), each cut
// into blocks of its own (Sec. 4.2 keeps the patch tokens and the special tokens in separate blocks);
// nbq1 / nbk1 = number of query / key blocks of the first segment.  n_first = n_tokens is the plain
// single-segment blocking.
struct Segments {
  int n_first, nbq1, nbk1;
};

// A key tile of B keys in LDS.  With key blocks of B keys it is one listed block (a); with key blocks
// of B/2 keys it is two consecutive entries of the row's list, one per half (b < 0: the list ended,
// the second half is empty).
struct Tile {
  int a, b;
  unsigned oa, ob;  // byte offsets of the blocks' first keys inside the head (filled in by fix())
};

// B: query rows per workgroup = keys per LDS tile.  KB: size of the key blocks the index list refers
// to, B or B/2.
template <int B, int KB>
__global__ __launch_bounds__(2 * B, 2) void attn_bf16_kernel(
    const unsigned char* __restrict__ q, const unsigned char* __restrict__ k, const unsigned char* __restrict__ v,
    unsigned short* __restrict__ out, float* __restrict__ lse, const int32_t* __restrict__ kv_idx,
    const int32_t* __restrict__ kv_cnt, const int32_t* __restrict__ order, int idx_stride, int64_t n_tokens, int nb,
    int nbk, float scale_log2, Segments seg, int heads, int64_t n_static, int* __restrict__ next_row) {
  static_assert(KB == B || (2 * KB == B && B == 128), "key blocks are whole tiles or half tiles of 128");
  constexpr bool HALF = KB != B;          // two listed key blocks per tile
  constexpr int WQ = B / 64;              // waves along queries (64 rows each)
  constexpr int KW = B / 2;               // keys per wave per tile
  constexpr int NH = KW / 32;             // 32-key sub-tiles per wave per tile
  constexpr int NW = B / 32;              // waves per workgroup
  constexpr int TILE_BYTES = B * 128;     // one K or V tile
  constexpr int V_BASE = 2 * TILE_BYTES;  // LDS layout: K buffers 0, 1, then V buffers 0, 1
  extern __shared__ __align__(16) unsigned char smem[];

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int n = lane & 31;
  const int g = lane >> 5;
  const int qi = wave % WQ;
  const int kh = wave / WQ;
  // Which (head, query block) row this workgroup computes.  Workgroup number w of the grid runs on
  // XCD w % 8, whatever the XCDs' speeds, and the chip holds 512 workgroups at a time, 64 per XCD.
  //  - The first n_static workgroups take positions of the launch order by their number.  Inside each
  //    full group of 512 consecutive workgroups the positions are dealt out so that an XCD gets 64
  //    consecutive ones: rows that are neighbours in the order, whose lists tend to overlap, then
  //    share one L2 instead of being spread over all eight.
  //  - The other workgroups (there are more of them than rows left) take the remaining positions
  //    first come, first served, through one atomic counter, and leave at once when none is left.
  //    Under load the XCDs of a part run at clocks that differ by several per cent; an XCD that is
  //    through with its static share early thus takes more of the remaining rows than a slow one.
  const int64_t total = int64_t(heads) * nb;
  const int64_t w = int64_t(blockIdx.y) * nb + blockIdx.x;
  int64_t pos;
  if (w < n_static) {
    const int r = static_cast<int>(w & 511);
    pos = (w - r) + 512 <= n_static ? (w - r) + (r & 7) * 64 + (r >> 3) : w;
  } else {
    int* slot = reinterpret_cast<int*>(smem);
    if (tid == 0) *slot = atomicAdd(next_row, 1);
    __syncthreads();
    const int t = __builtin_amdgcn_readfirstlane(*slot);
    __syncthreads();  // the slot lies where the first K tile goes
    if (t >= total - n_static) return;  // the whole workgroup leaves, before any other barrier
    pos = n_static + t;
  }
  const int64_t row = order != nullptr ? int64_t(__builtin_amdgcn_readfirstlane(order[pos])) : pos;
  const int h = static_cast<int>(min(max(row / nb, int64_t(0)), int64_t(heads - 1)));
  const int I = static_cast<int>(min(max(row - int64_t(h) * nb, int64_t(0)), int64_t(nb - 1)));
  const int64_t head_bytes = int64_t(h) * n_tokens * 128;
  const int64_t rowid = int64_t(h) * nb + I;
  // this query block: first token and number of tokens (a block never crosses the segment boundary)
  const int n_tok = static_cast<int>(n_tokens);
  const int q_start = I < seg.nbq1 ? I * B : seg.n_first + (I - seg.nbq1) * B;
  const int q_valid = min(B, (I < seg.nbq1 ? seg.n_first : n_tok) - q_start);
  // raw buffer views of this head's K and V (byte-addressed, bounds-checked by the hardware)
  const unsigned head_size = static_cast<unsigned>(n_tokens * 128);
  const i32x4 krsrc = make_rsrc(k + head_bytes, head_size);
  const i32x4 vrsrc = make_rsrc(v + head_bytes, head_size);
  const unsigned smem_addr =
      static_cast<unsigned>(reinterpret_cast<size_t>((__attribute__((address_space(3))) unsigned char*)smem));

  // ---- Q fragments (B operand of S^T = K Q^T), pre-scaled: [query half][16-dim chunk]; lane (n, g)
  // holds dims 16c + 8g .. +7 of query row 32 b + n of the wave's 64
  bf16x8 qf[2][4];
#pragma unroll
  for (int b2 = 0; b2 < 2; ++b2) {
    const int64_t row = int64_t(q_start) + qi * 64 + b2 * 32 + n;  // rows past q_valid are computed, not stored
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
  // K operand reads (ds_read_b128) of the wave's sub-tile u: row r = kh*KW + 32u + n, logical chunk
  // 2c + g.  Since swz_k(r + 32) = swz_k(r) ^ 4, sub-tile 1 reads chunk c where sub-tile 0 reads c ^ 2.
  unsigned kaddr[4];
  {
    const int r = kh * KW + n;
#pragma unroll
    for (int c = 0; c < 4; ++c) kaddr[c] = r * 128 + (((2 * c + g) ^ swz_k(r)) << 4);
  }
  // V operand reads (transpose read, 8 bytes per lane): 16-lane group G = lane/16 covers dims
  // db*32 + 16*(G&1) .. +15 for key-slot half g = G/2; inside the group lane i names key
  // m = i/4 of the four and the dim quad j = i%4.  Key = kh*KW + 32u + 16cp + 8t + 4g + m.
  unsigned vaddr[2];
  {
    const int i16 = lane & 15, m = i16 >> 2, j = i16 & 3, G = lane >> 4;
    const int keyl = kh * KW + 4 * g + m;
#pragma unroll
    for (int db = 0; db < 2; ++db) {
      const int cc = db * 4 + 2 * (G & 1) + (j >> 1);
      vaddr[db] = V_BASE + keyl * 128 + ((cc ^ swz_v(keyl)) << 4) + (j & 1) * 8;
    }
  }

  f32x16 o[2][2];  // O^T accumulators: [dim block][query half], this lane's query column
  float m_ref[2];  // SAFE pass: reference maximum per query column (log2 domain)
  float l_run[2];  // this lane's share of the row sums

  const bool dense = kv_idx == nullptr;
  const int count = dense ? nbk : min(max(kv_cnt[rowid], 0), nbk);  // listed key blocks
  const int ntiles = HALF ? (count + 1) >> 1 : count;
  const int32_t* my_idx = dense ? nullptr : kv_idx + rowid * idx_stride;
  // key block J: first token and number of tokens.  Blocks of the first segment (J < nbk1) tile
  // tokens [0, n_first), the others tokens [n_first, n_tokens); the last block of each may be ragged.
  auto key_start = [&](int J) { return J < seg.nbk1 ? J * KB : seg.n_first + (J - seg.nbk1) * KB; };
  auto key_count = [&](int J) { return min(KB, (J < seg.nbk1 ? seg.n_first : n_tok) - key_start(J)); };

  // The row's key-block list is the same for the whole workgroup, so its entries are fetched with
  // scalar loads (the list is read through a constant-address-space pointer: it is never written
  // while the kernel runs), which do not count as vector memory operations: the waits on the
  // direct-to-LDS loads (vmcnt) stay exact.  raw_at(it) only issues the loads of tile `it` (any it;
  // past the end it repeats the last tile) and hands back the unchecked entries; the caller keeps
  // them for a tile before fix() turns them into block numbers, so nothing waits for the load.
  typedef const int32_t __attribute__((address_space(4))) * const_idx_ptr;
  const const_idx_ptr cidx = (const_idx_ptr)my_idx;
  auto raw_at = [&](int it) -> Tile {
    if (dense) return Tile{min(it, nbk - 1), -1, 0u, 0u};
    constexpr int PER = HALF ? 2 : 1;  // list entries per tile
    const int e = min(it, ntiles - 1) * PER;
    Tile t{cidx[e], -1, 0u, 0u};
    if constexpr (HALF) t.b = cidx[min(e + 1, count - 1)];
    return t;
  };
  // An absent second half gets an offset past the end of the head's buffer: the bounds check of
  // the loads then zero-fills it.
  auto fix = [&](const Tile& r, int it) -> Tile {  // r = raw_at(it)
    Tile t{r.a, -1, 0u, head_size};
    if (!dense) {
      t.a = min(max(r.a, 0), nbk - 1);
      if constexpr (HALF) {
        if (min(it, ntiles - 1) * 2 + 1 < count) t.b = min(max(r.b, 0), nbk - 1);
      }
    }
    t.oa = static_cast<unsigned>(key_start(t.a)) * 128u;
    if constexpr (HALF) {
      if (t.b >= 0) t.ob = static_cast<unsigned>(key_start(t.b)) * 128u;
    }
    return t;
  };
  auto block_at = [&](int it) -> Tile { return fix(raw_at(it), it); };
  // The offsets are operands of scalar type in the load instructions.  A tile description that has
  // been carried around a loop may live in vector registers (the same value in every lane): this
  // moves the offsets back.
  auto scalar = [&](Tile t) -> Tile {
    t.oa = static_cast<unsigned>(__builtin_amdgcn_readfirstlane(static_cast<int>(t.oa)));
    t.ob = static_cast<unsigned>(__builtin_amdgcn_readfirstlane(static_cast<int>(t.ob)));
    return t;
  };
  // This wave's keys of a tile are the tile rows [kh*KW, (kh+1)*KW).  wave_limit(t) is the first of
  // them that is not a key of the listed block (a ragged block, or an absent second half): rows at
  // or past it hold zeros or tokens of another block, and their scores are masked before they are
  // exponentiated.  A full tile gives (kh+1)*KW.
  auto wave_limit = [&](const Tile& t) {
    const int J = (HALF && kh == 1) ? t.b : t.a;
    const int cnt = J < 0 ? 0 : key_count(J);
    return HALF ? kh * KW + cnt : min(cnt, (kh + 1) * KW);
  };
  // scores of the wave's 32-key sub-tile u: keys at or past `limit` (tile row numbers) get weight 0
  // (register i of the lane is tile row kh*KW + 32u + 8(i/4) + 4g + i%4).  Runs for the few ragged
  // tiles only; the lane number is taken afresh through an opaque instruction, so that nothing of
  // this is computed ahead and kept in registers across the tile loops.
  auto mask_keys = [&](f32x16& sc, int u, int limit) {
    int l;
    asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(l));
    const int t = limit - kh * KW - u * 32 - ((l >> 5) << 2);  // row 8(i/4) + i%4 is masked iff it is >= t
#pragma unroll
    for (int i = 0; i < 16; ++i) sc[i] = (8 * (i >> 2) + (i & 3) >= t) ? -INFINITY : sc[i];
  };
  // Does the tile hold rows that are not keys of its listed block(s)?  The same answer in every wave
  // of the workgroup (the pipelined loop below leaves such tiles to the plain tile code, and all
  // waves must agree on that).  Only the last block of each segment can be short.
  const int short_a = (seg.n_first % KB) != 0 ? seg.nbk1 - 1 : -1;
  const int short_b = ((n_tok - seg.n_first) % KB) != 0 ? nbk - 1 : -1;
  auto tile_ragged = [&](const Tile& t) {
    bool r = t.a == short_a || t.a == short_b;
    if constexpr (HALF) r = r || t.b < 0 || t.b == short_a || t.b == short_b;
    return r;
  };
  // Direct-to-LDS load number i2 (0..7) of key tile J into buffer pair `buf`: even i2 moves 1 KB of
  // the K tile, odd i2 1 KB of the V tile.  Rows that lie past the end of the head's buffer fail
  // the hardware bounds check, which makes the load write zeros for them (so V rows past the end
  // are finite; rows past a ragged block inside the sequence hold the following tokens).
  // With half-tile key blocks, loads i = 0, 1 fill tile rows 0..63 from block a and i = 2, 3 rows
  // 64..127 from block b (an absent b: zero-filled, see fix()).
  const unsigned dma_base = smem_addr + wave * 1024;  // this wave's 1 KB slice of every 4 KB (8 KB) group
  auto issue_part = [&](const Tile& J, auto bufc, auto i2c) {
    constexpr int buf = decltype(bufc)::value, i2 = decltype(i2c)::value;
    constexpr int i = i2 >> 1;
    constexpr bool is_v = (i2 & 1) != 0;
    constexpr unsigned dst = NW * i * 1024 + (is_v ? V_BASE : 0) + buf * TILE_BYTES;
    if constexpr (HALF) {
      const unsigned soff = (i >> 1) ? J.ob : J.oa;
      if (is_v) {
        dma16<dst>(vrsrc, voff, soff + (i & 1) * NW * 1024, dma_base);
      } else {
        dma16<dst>(krsrc, koff[i % KN], soff, dma_base);
      }
    } else {
      const unsigned soff = J.oa;
      if (is_v) {
        dma16<dst>(vrsrc, voff, soff + i * NW * 1024, dma_base);
      } else {
        dma16<dst>(krsrc, koff[i % KN], soff + (i / KN) * KN * NW * 1024, dma_base);
      }
    }
  };
  auto issue = [&](const Tile& J, auto bufc) {
    issue_part(J, bufc, Int<0>{}); issue_part(J, bufc, Int<1>{}); issue_part(J, bufc, Int<2>{}); issue_part(J, bufc, Int<3>{});
    issue_part(J, bufc, Int<4>{}); issue_part(J, bufc, Int<5>{}); issue_part(J, bufc, Int<6>{}); issue_part(J, bufc, Int<7>{});
  };
  auto issue_rt = [&](const Tile& J, int buf) {  // buffer known at run time only
    if (buf) issue(J, Int<1>{});
    else issue(J, Int<0>{});
  };

  // K operands (A of S^T = K Q^T) of the wave's 32-key sub-tile u; boff = byte offset of the buffer
  auto read_k = [&](bf16x8 (&ka)[4], unsigned boff, int u) {
#pragma unroll
    for (int c = 0; c < 4; ++c) ka[c] = *LDS_PTR(bf16x8, smem + boff + kaddr[(u & 1) ? (c ^ 2) : c] + u * 4096);
  };
  // V^T operands (A of O^T += V^T P^T) of sub-tile u: [dim block][16-key chunk]
  auto read_v = [&](bf16x8 (&va)[2][2], unsigned boff, int u) {
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int cp = 0; cp < 2; ++cp) {
        const unsigned char* p = smem + boff + vaddr[db] + (32 * u + 16 * cp) * 128;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p));
        const s16x4 hi =
            __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p + 8 * 128));
        const u32x2 lo2 = __builtin_bit_cast(u32x2, lo), hi2 = __builtin_bit_cast(u32x2, hi);
        const u32x4 av = {lo2[0], lo2[1], hi2[0], hi2[1]};
        va[db][cp] = __builtin_bit_cast(bf16x8, av);
      }
  };

  // weights of key pair j (registers 2j, 2j+1) of a score block: exp2, add to the row sum, round to
  // bf16, store as word j of the two B operands.  The row sum takes the fp32 weights with two plain
  // adds: on this part a dot2 of the packed pair costs four times as much as an add and, unlike the
  // exp2 and the adds, does not run beside the matrix pipe.
  auto weigh_pair = [&](const f32x16& sc, u32x4 (&w)[2], float& lsum, int j) {
    const float e0 = __builtin_amdgcn_exp2f(sc[2 * j]), e1 = __builtin_amdgcn_exp2f(sc[2 * j + 1]);
    lsum += e0 + e1;
    w[j >> 2][j & 3] = pack_bf16(e0, e1);
  };

  // ---------------------------------------------------------------------------------------------
  // One tile, plain form: per (32-key sub-tile, query half) scores (4 MFMAs) -> weights -> O update
  // (4 MFMAs), from the tile buffers at byte offset boff.  `limit` = wave_limit of the tile.
  //   SAFE = true: online softmax.  The accumulator of the score MFMA starts at -m_ref, so the MFMA
  //   result is already relative to the reference, and m_ref is raised only when a sub-tile exceeds
  //   it by more than 2^kRaise.
  //   SAFE = false: reference 0, no maximum.
  // In both forms the scores of tile rows that are not keys of the listed block are masked.
  // after_reads() runs once every LDS read of the tile has been consumed.
  // ka, va, sc, w: working registers (the pipelined loop lends its own, which are free between runs).
  auto compute_tile = [&](auto safec, unsigned boff, int limit, auto&& after_reads, bf16x8 (&ka)[4],
                          bf16x8 (&va)[2][2], f32x16 (&sc)[2], u32x4 (&w)[2][2]) {
    constexpr bool SAFE = decltype(safec)::value;
    const bool ragged = limit < (kh + 1) * KW;
#pragma unroll
    for (int u = 0; u < NH; ++u) {
      read_k(ka, boff, u);
      read_v(va, boff, u);
      // the scores of both query halves first (eight MFMAs in a row), so that the weights of the
      // first half are computed while the matrix pipe still works on the second, and the O update
      // of the first half runs under the weights of the second
      float base[2];
#pragma unroll
      for (int b2 = 0; b2 < 2; ++b2) {
        base[b2] = (SAFE && m_ref[b2] != -INFINITY) ? m_ref[b2] : 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) sc[b2][i] = -base[b2];
#pragma unroll
        for (int c = 0; c < 4; ++c) sc[b2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[c], qf[b2][c], sc[b2], 0, 0, 0);
      }
      if (ragged) {
        mask_keys(sc[0], u, limit);
        mask_keys(sc[1], u, limit);
      }
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
#pragma unroll
        for (int j = 0; j < 8; ++j) weigh_pair(sc[b2], w[b2], l_run[b2], j);
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
          for (int cp = 0; cp < 2; ++cp)
            o[db][b2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[db][cp], __builtin_bit_cast(bf16x8, w[b2][cp]),
                                                                o[db][b2], 0, 0, 0);
      }
      if (u == NH - 1) after_reads();
    }
  };

  // Plain tile loop: compute_tile per tile, one barrier per tile, the next tile's loads in flight
  // meanwhile.  Used for the SAFE pass and for block 64.
  auto plain_loop = [&](auto safec) {
    if (ntiles <= 0) return;
    Tile J_cur = block_at(0);
    issue(J_cur, Int<0>{});
    Tile J_pre = raw_at(1);  // list entries are fetched a tile before they are used
    bf16x8 ka[4], va[2][2];
    f32x16 sc[2];
    u32x4 w[2][2];
    for (int it = 0; it < ntiles; ++it) {
      const int buf = it & 1;
      const Tile J_next = (it + 1 < ntiles) ? fix(J_pre, it + 1) : Tile{0, -1, 0u, 0u};
      __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's share of tile `it` has landed
      __syncthreads();                     // ... and so has everyone else's; buffer buf^1 is free
      if (it + 1 < ntiles) issue_rt(scalar(J_next), buf ^ 1);
      // The list entries of the tile after next.  Scalar loads return out of order with LDS reads, so
      // a wait for LDS data would also wait for them: they are issued where every LDS read of the
      // tile has been consumed, and used at the top of the next tile.
      compute_tile(safec, buf * TILE_BYTES, wave_limit(J_cur), [&]() { J_pre = raw_at(it + 2); }, ka, va, sc, w);
      J_cur = J_next;
    }
  };

  // ---------------------------------------------------------------------------------------------
  // Fast pass for block 128: the same arithmetic as compute_tile<SAFE = false>, software pipelined
  // inside the wave.  A unit is (32-key sub-tile u, query half b): scores QK (4 MFMAs into 16
  // registers), weights W (16 exp2, 8 packs, 16 adds), O update PV (4 MFMAs).  A tile has four units
  // n = 0..3 = (u0,b0), (u0,b1), (u1,b0), (u1,b1).  While the VALU works on W(n) the matrix pipe gets
  // QK(n+1) and PV(n-1), one MFMA per four VALU instructions, so the wave's VALU and MFMA streams
  // overlap instead of waiting for each other.  K operands of a sub-tile serve two units, V operands
  // likewise; they are fetched from LDS at least half a unit ahead of their first use.  By the end
  // of unit 1 every LDS read of the tile has been issued, so at the start of unit 2 the workgroup
  // synchronises once: the next tile is known to have landed (its first K operands are read right
  // after the last score MFMA of this tile) and the current buffers are free, so the eight loads of
  // the tile after next are issued into them, one after each of the following MFMAs.
  //
  // The pipelined code has no masking in it (a conditional in the slot sequence costs 5 %): it runs
  // over the row's leading full tiles.  From the first tile with rows that are not keys (a short
  // block, an absent half) the remaining tiles go through compute_tile, which masks.  With ascending
  // lists that is the row's last tile, or, for a split sequence with the short first segment's
  // blocks listed last but a few, the last few tiles.  Either way a tile costs every wave exactly
  // one barrier, and the loads stay two tiles ahead.
  auto fast_loop = [&]() {
    if (ntiles <= 0) return;
    f32x16 sc[2];        // scores: [query half]
    u32x4 pw[2][2];      // weights as packed bf16 pairs: [query half][16-key chunk]
    bf16x8 ka[4];        // K operands of the sub-tile whose scores are computed next
    bf16x8 va[2][2][2];  // V^T operands: [sub-tile][dim block][16-key chunk]
    float ex[2][2];      // exponentiated scores of the key pair that is packed in the next slot
    // Row sums on the matrix pipe.  In v_mfma_f32_16x16x32_bf16 lane l supplies, as B operand, eight
    // bf16 values B[k][j] of column j = l%16 with k = 8(l/16) .. 8(l/16)+7, supplies row l%16 of A for
    // the same eight k, and receives D[4(l/16) + r][l%16] in accumulator register r = 0..3.  With
    //   A_h[i][k] = 1 if i%4 == h and k/8 == i/4, else 0
    // the product D = A_h B puts, in register h of every lane, the sum of that lane's own eight B
    // values, and nothing in the other registers.  The B operand is the very register tuple of packed
    // weights that the O update multiplies with V, so two such instructions per unit (h = the query
    // half) sum the sixteen weights a lane holds: they replace sixteen fp32 adds per unit (64 cycles
    // of vector issue in a loop whose vector and matrix pipes are both saturated) by 32 cycles of
    // matrix pipe, and the sums are over the bf16 weights, exactly the values that multiply V.
    f32x4 lacc = {0.f, 0.f, 0.f, 0.f};
    bf16x8 row_sel[2];
#pragma unroll
    for (int h2 = 0; h2 < 2; ++h2) {
      const bool on = (lane & 3) == h2 && (lane >> 4) == ((lane & 15) >> 2);
      const unsigned w1 = on ? 0x3F803F80u : 0u;  // two bf16 ones
      row_sel[h2] = __builtin_bit_cast(bf16x8, u32x4{w1, w1, w1, w1});
    }
    auto add_weights = [&](auto hc, const u32x4& words) {
      lacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(row_sel[decltype(hc)::value], __builtin_bit_cast(bf16x8, words), lacc, 0,
                                                      0, 0);
    };

    // one unit N = (sub-tile N/2, query half N%2).  Slots 0..3: MFMA of QK(N+1) + one weight pair;
    // slots 4..7: MFMA of PV(N-1) + one weight pair.  mid(slot) places LDS reads, the barrier and
    // loads after that slot's MFMA.
    auto unit = [&](auto nc, auto&& mid) {
      constexpr int N = decltype(nc)::value;
      constexpr int BQ = N & 1;                 // query half whose weights are computed
      constexpr int BN = (N + 1) & 1;           // query half of QK(N+1)
      constexpr int BP = (N + 3) & 1;           // query half of PV(N-1)
      constexpr int UP = ((N + 3) & 3) >> 1;    // sub-tile of PV(N-1)
#define BSGA_SLOT(S_)                                                                                          \
  {                                                                                                            \
    if constexpr ((S_) < 4) {                                                                                  \
      if constexpr ((S_) == 0) {                                                                               \
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};   \
        sc[BN] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[0], qf[BN][0], zero, 0, 0, 0);                     \
      } else {                                                                                                 \
        sc[BN] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[(S_) & 3], qf[BN][(S_) & 3], sc[BN], 0, 0, 0);      \
      }                                                                                                        \
    } else {                                                                                                   \
      /* the two dim blocks alternate: consecutive MFMAs are independent and share the weights  */         \
      o[(S_) & 1][BP] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                                               \
          va[UP][(S_) & 1][((S_) >> 1) & 1], __builtin_bit_cast(bf16x8, pw[BP][((S_) >> 1) & 1]), o[(S_) & 1][BP], 0, \
          0, 0);                                                                                               \
    }                                                                                                          \
    /* weights, staggered by one slot so that no instruction waits for the one just before it:   */          \
    /* pack pair S_ (exponentiated in the previous slot), exponentiate the next pair, then sum   */          \
    /* pair S_ (two fp32 adds).                                                                  */          \
    {                                                                                                          \
      const unsigned pk = pack_bf16(ex[(S_) & 1][0], ex[(S_) & 1][1]);                                         \
      if constexpr ((S_) < 7) {                                                                                \
        ex[((S_) + 1) & 1][0] = __builtin_amdgcn_exp2f(sc[BQ][2 * (S_) + 2]);                                  \
        ex[((S_) + 1) & 1][1] = __builtin_amdgcn_exp2f(sc[BQ][2 * (S_) + 3]);                                  \
      } else {                                                                                                 \
        ex[0][0] = __builtin_amdgcn_exp2f(sc[BN][0]);                                                          \
        ex[0][1] = __builtin_amdgcn_exp2f(sc[BN][1]);                                                          \
      }                                                                                                        \
      __builtin_amdgcn_sched_barrier(0);                                                                       \
      /* row sums: the previous unit's second group of weights in slot 1, this unit's first in slot 5 */    \
      if constexpr ((S_) == 1) add_weights(Int<BP>{}, pw[BP][1]);                                              \
      if constexpr ((S_) == 5) add_weights(Int<BQ>{}, pw[BQ][0]);                                              \
      pw[BQ][(S_) >> 2][(S_) & 3] = pk;                                                                        \
    }                                                                                                          \
    mid(Int<(S_)>{});                                                                                          \
    __builtin_amdgcn_sched_barrier(0);                                                                         \
  }
      BSGA_SLOT(0) BSGA_SLOT(1) BSGA_SLOT(2) BSGA_SLOT(3) BSGA_SLOT(4) BSGA_SLOT(5) BSGA_SLOT(6) BSGA_SLOT(7)
#undef BSGA_SLOT
    };

    // a whole (full) tile in buffer pair `buf` (byte offset boff; the other pair is at boff ^ TILE_BYTES).
    // On entry: sc[0] = QK(0) of this tile, ka = K operands of sub-tile 0, pw[1] / va[1] = weights /
    // V operands of the previous tile's unit 3 (zeros at the start of a run).  What it prepares for
    // the following tile (K operands and first scores from the other buffer) goes unused when the run
    // ends here.
    auto tile = [&](const Tile& J_next2, auto bufc) {
      constexpr int buf = decltype(bufc)::value;
      constexpr unsigned boff = buf * TILE_BYTES;
      unit(Int<0>{}, [&](auto slot) {  // QK(1); K(u1); PV(previous 3); V(u0)
        constexpr int S = decltype(slot)::value;
        if constexpr (S == 0) read_v(va[0], boff, 0);
        if constexpr (S == 3) read_k(ka, boff, 1);
      });
      unit(Int<1>{}, [&](auto slot) {  // QK(2); PV(0); V(u1)
        constexpr int S = decltype(slot)::value;
        if constexpr (S == 0) read_v(va[1], boff, 1);
      });
      unit(Int<2>{}, [&](auto slot) {  // synchronise; QK(3); K(next tile u0); PV(1) + loads 0..3
        constexpr int S = decltype(slot)::value;
        if constexpr (S == 0) {
          __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's share of the next tile has landed
          __syncthreads();                     // every read of this tile is complete in every wave
        }
        if constexpr (S == 3) read_k(ka, boff ^ TILE_BYTES, 0);
        if constexpr (S >= 4) issue_part(J_next2, bufc, Int<S - 4>{});
      });
      unit(Int<3>{}, [&](auto slot) {  // QK(next tile's unit 0); PV(2) + loads 4..7
        constexpr int S = decltype(slot)::value;
        if constexpr (S >= 4) issue_part(J_next2, bufc, slot);
      });
    };

    // ---- tiles 0 and 1 on their way ----------------------------------------------------------------
    Tile J_cur = block_at(0);
    issue(J_cur, Int<0>{});
    Tile J_nxt = J_cur;
    if (ntiles > 1) {
      J_nxt = block_at(1);
      issue(J_nxt, Int<1>{});
    }
    Tile J_pre = raw_at(2);  // fetched one tile before it becomes "the tile after next"
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    // Invariant at the top of the loop: tile T lies in buffer T&1 and every wave knows it; the loads
    // of tile T+1 into the other buffer have been issued; J_cur / J_nxt are tiles T / T+1 and J_pre
    // holds the raw list entries of tile T+2.
    int T = 0;
    if (!tile_ragged(J_cur)) {
      // ---- the run of full tiles: K operands of sub-tile 0, QK(0), nothing pending for the O update --
      read_k(ka, 0u, 0);
#pragma unroll
      for (int cp = 0; cp < 2; ++cp) {
        pw[1][cp] = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
        for (int db = 0; db < 2; ++db) va[1][db][cp] = __builtin_bit_cast(bf16x8, u32x4{0u, 0u, 0u, 0u});
      }
      {
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        sc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[0], qf[0][0], zero, 0, 0, 0);
#pragma unroll
        for (int c = 1; c < 4; ++c) sc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[c], qf[0][c], sc[0], 0, 0, 0);
      }
      ex[0][0] = __builtin_amdgcn_exp2f(sc[0][0]);
      ex[0][1] = __builtin_amdgcn_exp2f(sc[0][1]);
      __builtin_amdgcn_sched_barrier(0);
      // two tiles per round, so that every LDS address is a constant of the code (even tiles lie in
      // buffer pair 0, odd ones in pair 1)
      auto step = [&](auto bufc) {
        // the tile after next; at the end of the list one more (harmless) load of a valid tile
        const Tile J2 = scalar((T + 2 < ntiles) ? fix(J_pre, T + 2) : J_cur);
        J_pre = raw_at(T + 3);
        tile(J2, bufc);
        J_cur = J_nxt;
        J_nxt = J2;
        ++T;
        return T < ntiles && !tile_ragged(J_cur);
      };
      while (step(Int<0>{}) && step(Int<1>{})) {
      }
      // ---- the O update and the last row-sum step of the run's last unit ------------------------------
#pragma unroll
      for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int cp = 0; cp < 2; ++cp)
          o[db][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[1][db][cp], __builtin_bit_cast(bf16x8, pw[1][cp]),
                                                             o[db][1], 0, 0, 0);
      add_weights(Int<1>{}, pw[1][1]);
      l_run[0] += lacc[0];
      l_run[1] += lacc[1];
    }
    // ---- from the first ragged tile on: plain tiles (the same buffers and the same one barrier per
    // tile; the loads stay two tiles ahead) ------------------------------------------------------------
    for (; T < ntiles; ++T) {
      compute_tile(std::false_type{}, (T & 1) * TILE_BYTES, wave_limit(J_cur), []() {}, ka, va[0], sc, pw);
      const Tile J2 = scalar((T + 2 < ntiles) ? fix(J_pre, T + 2) : J_cur);
      J_pre = raw_at(T + 3);
      __builtin_amdgcn_s_waitcnt(0x0F70);  // this wave's share of tile T+1 has landed
      __syncthreads();                     // ... everyone's has, and nobody still reads tile T
      issue_rt(J2, T & 1);
      J_cur = J_nxt;
      J_nxt = J2;
    }
  };

  // A whole pass over the row's key tiles, then the merge of the two key halves (wave (qi, 1) parks
  // its state in LDS as [qi][68 values][64 lanes] and wave (qi, 0) folds it in) and the output.
  // Returns true (to every thread of the workgroup) if the fast pass must be repeated in SAFE mode
  // because a row sum or an output left the range in which reference-free weights are trustworthy:
  // a weight 2^s overflows for s >= 128 (the row sum then exceeds the upper limit, or O is not
  // finite), and weights below 2^-126 flush to zero, which is harmless as long as the row sum is at
  // least 2^-80 (at most 2^24 keys x 2^-126 lost: a relative error under 2^-22).
  auto pass = [&](auto safec) -> bool {
    constexpr bool SAFE = decltype(safec)::value;
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int b2 = 0; b2 < 2; ++b2)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][b2][i] = 0.f;
    m_ref[0] = m_ref[1] = -INFINITY;
    l_run[0] = l_run[1] = 0.f;
    if constexpr (!SAFE && B == 128) fast_loop();
    else plain_loop(safec);
    __builtin_amdgcn_s_waitcnt(0x0F70);  // no direct-to-LDS load may still be in flight
    __syncthreads();                     // ... in any wave: LDS can be reused

    float* park = reinterpret_cast<float*>(smem) + 16 + qi * 68 * 64;
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
    volatile int* flag = reinterpret_cast<volatile int*>(smem);  // workgroup-wide OR of `bad`
    if (tid == 0) *flag = 0;
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
        if constexpr (!SAFE) bad = bad || !(l >= 0x1p-80f && l <= 0x1p100f);
        lt[b2] = l;
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
      if (count <= 0) bad = false;  // an empty row is zeros by definition, not a range problem
      if (bad) *flag = 1;
      __syncthreads();
      const bool any_bad = *flag != 0;
      __syncthreads();
      if (any_bad) return true;
    }
    if (kh == 0) {
#pragma unroll
      for (int b2 = 0; b2 < 2; ++b2) {
        const float inv = lt[b2] > 0.f ? 1.f / lt[b2] : 0.f;
        const int lrow = qi * 64 + b2 * 32 + n;
        const int64_t row = int64_t(q_start) + lrow;
        if (lrow < q_valid) {
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
    pass(std::true_type{});
  }
}

}  // namespace

int launch_attn_bf16(const void* q, const void* k, const void* v, int heads, int64_t n_tokens, int64_t n_first,
                     int block, int block_k, float softmax_scale, const int32_t* kv_idx, const int32_t* kv_cnt,
                     int idx_stride, void* out, float* lse, void* workspace, hipStream_t stream) {
  const int nb = static_cast<int>(split_blocks(n_tokens, n_first, block));     // query blocks
  const int nbk = static_cast<int>(split_blocks(n_tokens, n_first, block_k));  // key blocks the lists refer to
  const Segments seg = {static_cast<int>(n_first), static_cast<int>(ceil_div(n_first, block)),
                        static_cast<int>(ceil_div(n_first, block_k))};
  const int32_t* order = nullptr;
  const int64_t rows = int64_t(heads) * nb;
  int64_t n_static = rows;  // without a workspace every row is taken by workgroup number
  int extra = 0;                          // workgroups beyond one per row
  int* next_row = nullptr;
  // ordering and balancing matter only when the grid does not fit the chip at once
  // (and only while the extra workgroups fit the grid's second dimension)
  const bool big = workspace != nullptr && rows >= 1024 && rows < (int64_t(1) << 30) &&
                   heads + ceil_div(rows / 16 + 1024, nb) <= 65535;
  if (big) {
    // The last eighth of the rows is handed out at run time; half as many workgroups again as that
    // are launched for it, so that an XCD can take up to 1.5 times its even share of those rows.
    const int64_t dynamic = rows / 8;
    n_static = (rows - dynamic) / 512 * 512;
    extra = static_cast<int>((rows - n_static) / 2 + 512);
  }
  if (big && kv_idx == nullptr) {
    // dense: the workspace holds the counter only
    next_row = static_cast<int*>(workspace);
    hipLaunchKernelGGL(zero_word_kernel, dim3(1), dim3(64), 0, stream, next_row);
  }
  if (big && kv_idx != nullptr) {
    // workspace: [heads * nb] launch order, then the [classes][heads] table, the number of the merged
    // class and the counter of the rows handed out at run time (cleared by order_merge_kernel)
    int32_t* ord = static_cast<int32_t*>(workspace);
    int32_t* table = ord + int64_t(heads) * nb;
    next_row = table + int64_t(kOrderClasses) * heads + 1;
    hipLaunchKernelGGL(order_hist_kernel, dim3(heads), dim3(256), 0, stream, kv_cnt, nb, nbk, heads, table);
    hipLaunchKernelGGL(order_merge_kernel, dim3(1), dim3(256), 0, stream, table, heads);
    hipLaunchKernelGGL(order_scan_kernel, dim3(1), dim3(1024), 0, stream, table, int64_t(kOrderClasses) * heads);
    hipLaunchKernelGGL(order_place_kernel, dim3(heads), dim3(256), 0, stream, kv_cnt, nb, nbk, heads, table, ord);
    if (int rc = check_hip(hipGetLastError(), "bsga bf16 attention (launch order)")) return rc;
    order = ord;
  }
  const float scale_log2 = softmax_scale * kLog2e;
  dim3 grid(nb, heads + static_cast<int>(ceil_div(extra, nb)));
  const unsigned char* qp = static_cast<const unsigned char*>(q);
  const unsigned char* kp = static_cast<const unsigned char*>(k);
  const unsigned char* vp = static_cast<const unsigned char*>(v);
  unsigned short* op = static_cast<unsigned short*>(out);
  // LDS: two K and two V tile buffers (64 KB for block 128); block 64 also needs room for the
  // parked accumulators of the end merge (17 KB + 64 B), which 32 KB covers
  const size_t lds64 = 4 * 64 * 128, lds128 = 4 * 128 * 128;
  if (getenv("BSGA_DEBUG") != nullptr) {
    int n64 = -1, n128 = -1;
    (void)hipOccupancyMaxActiveBlocksPerMultiprocessor(&n64, attn_bf16_kernel<64, 64>, 128, lds64);
    (void)hipOccupancyMaxActiveBlocksPerMultiprocessor(&n128, attn_bf16_kernel<128, 128>, 256, lds128);
    fprintf(stderr, "[bsga] attention occupancy (workgroups per CU): block 64 -> %d, block 128 -> %d\n", n64, n128);
  }
  if (block == 64) {
    hipLaunchKernelGGL((attn_bf16_kernel<64, 64>), grid, dim3(128), lds64, stream, qp, kp, vp, op, lse, kv_idx,
                       kv_cnt, order, idx_stride, n_tokens, nb, nbk, scale_log2, seg, heads, n_static, next_row);
  } else if (block_k == 128) {
    hipLaunchKernelGGL((attn_bf16_kernel<128, 128>), grid, dim3(256), lds128, stream, qp, kp, vp, op, lse, kv_idx,
                       kv_cnt, order, idx_stride, n_tokens, nb, nbk, scale_log2, seg, heads, n_static, next_row);
  } else {
    hipLaunchKernelGGL((attn_bf16_kernel<128, 64>), grid, dim3(256), lds128, stream, qp, kp, vp, op, lse, kv_idx,
                       kv_cnt, order, idx_stride, n_tokens, nb, nbk, scale_log2, seg, heads, n_static, next_row);
  }
  return check_hip(hipGetLastError(), "bsga bf16 attention launch");
}

}  // namespace bsga
