// Device-side shared definitions for the gfx950 kernels (not part of the public ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/palu.h"

namespace palu {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));
typedef uint32_t uint2v __attribute__((ext_vector_type(2)));

constexpr int kDHead = PALU_D_HEAD;        // 128
constexpr int kHalf = kDHead / 2;          // 64 rotation pairs
constexpr int kTile = 32;                  // tokens per MFMA tile (N of the 32x32x16 instruction)

// Layer metadata passed by value in the kernel arguments.  Heads are QUERY heads:
// with grouped-query attention (qpk query heads per key/value head) head_off counts
// qpk heads per key/value head of the descriptor, and bk_off / bv_off are the
// offsets of per-query-head data laid out like the weights (the folded queries);
// the weights themselves have one column block per key/value head, see weight_block.
struct Meta {
  int n_heads;
  int n_groups;
  int qpk;                   // heads per key/value head: the model's query heads per key/value head times nq
  int nq;                    // queries per sequence in this call (1 for plain decode); see q_row

  int head_off[PALU_MAX_GROUPS + 1];
  int k_off[PALU_MAX_GROUPS + 1];
  int v_off[PALU_MAX_GROUPS + 1];
  int bk_off[PALU_MAX_GROUPS + 1];   // element offset of group j inside the concatenated B_k
  int bv_off[PALU_MAX_GROUPS + 1];
  uint8_t group_of_head[PALU_MAX_HEADS];
};

// Storage type helpers: the activation dtype is either IEEE half or bfloat16,
// both 16 bits wide; kernels are templated on a tag.
struct F16 {
  using vec8 = half8;
  static __device__ __forceinline__ float to_float(uint16_t bits) {
    return (float)__builtin_bit_cast(_Float16, bits);
  }
  static __device__ __forceinline__ uint16_t from_float(float v) {
    return __builtin_bit_cast(uint16_t, (_Float16)v);
  }
  static __device__ __forceinline__ float16v mfma(vec8 a, vec8 b, float16v c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
  }
};

struct BF16 {
  using vec8 = bf16x8;
  static __device__ __forceinline__ float to_float(uint16_t bits) {
    return __builtin_bit_cast(float, (uint32_t)bits << 16);
  }
  static __device__ __forceinline__ uint16_t from_float(float v) {   // round to nearest even
    uint32_t u = __builtin_bit_cast(uint32_t, v);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
  }
  static __device__ __forceinline__ float16v mfma(vec8 a, vec8 b, float16v c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
  }
};

// A constant in a vector register that the compiler takes for a per-lane value.  (x & mask) | c becomes one
// v_and_or_b32 only if at most one of its operands is uniform: with two constants the compiler emits v_and + v_or.
// The statement emits no instruction, so the compiler still sees, and spaces, everything around the matrix instructions.
__device__ __forceinline__ uint32_t per_lane_constant(uint32_t c) {
  asm volatile("" : "+v"(c));
  return c;
}
// Four 4-bit codes of each of two 16-bit halves of w (code u of a half in its bits 4u .. 4u+3) as four fp16
// pairs: pair u holds code u of the low half and code u of the high half, each in mantissa bits 4 .. 7 of
// 0x3c00, i.e. the exact fp16 numbers 1 + c/64.  one = per_lane_constant(0x3c003c00), made once by the caller.
struct NibblePairs {
  uint32_t p[4];
};
__device__ __forceinline__ NibblePairs nibbles_to_fp16_pairs(uint32_t w, uint32_t one) {
  constexpr uint32_t kNib = 0x00f000f0u;
  NibblePairs r;
  r.p[0] = ((w << 4) & kNib) | one;
  r.p[1] = (w & kNib) | one;
  r.p[2] = ((w >> 4) & kNib) | one;
  r.p[3] = ((w >> 8) & kNib) | one;
  return r;
}

// Dequantization of the 8 codes of a 32-bit word (code u in bits 4u .. 4u+3) to fp16, (c - z) * scale with one
// rounding, in channel order.  Packed form: a code c in the low mantissa bits of 0x6400 is the fp16 number 1024 + c;
// with an integer zero-point |z| <= 1000 the difference (1024 + c) - (1024 + z) is the exact integer c - z, and its
// fp16 product with the scale is rounded once: the same number as ((float)c - z) * scale rounded to fp16.  Codes u and
// u + 4 are 16 bits apart, i.e. in the two halves of one register: one shift and one masked merge per pair, two
// packed operations, then four byte permutes back to channel order.  k1024 = per_lane_constant(0x64006400).
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ bool zero_point_is_small_integer(uint16_t z16) {
  const float zf = F16::to_float(z16);
  return fabsf(zf) <= 1000.f && zf == rintf(zf);
}
__device__ __forceinline__ uint4v dequant8_packed(uint32_t w, uint16_t s16, uint16_t z16, uint32_t k1024) {
  constexpr uint32_t kNib = 0x000f000fu;
  const uint32_t zz = (uint32_t)z16 | ((uint32_t)z16 << 16), ss = (uint32_t)s16 | ((uint32_t)s16 << 16);
  const half2v zc = __builtin_bit_cast(half2v, zz) + __builtin_bit_cast(half2v, (uint32_t)0x64006400u);     // 1024 + z, exact
  const half2v sc = __builtin_bit_cast(half2v, ss);
  uint32_t p[4];                                              // pair u: channels u and u + 4
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const uint32_t c = ((w >> (4 * u)) & kNib) | k1024;       // (1024 + c_u, 1024 + c_{u+4})
    const half2v d = (__builtin_bit_cast(half2v, c) - zc) * sc;
    p[u] = __builtin_bit_cast(uint32_t, d);
  }
  uint4v out;                                                 // perm: selector bytes 0-3 pick from the second operand
  out.x = __builtin_amdgcn_perm(p[1], p[0], 0x05040100u);     // channels 0, 1
  out.y = __builtin_amdgcn_perm(p[3], p[2], 0x05040100u);     // 2, 3
  out.z = __builtin_amdgcn_perm(p[1], p[0], 0x07060302u);     // 4, 5
  out.w = __builtin_amdgcn_perm(p[3], p[2], 0x07060302u);     // 6, 7
  return out;
}
__device__ __forceinline__ uint4v dequant8_float(uint32_t w, uint16_t s16, uint16_t z16) {
  const float sc = F16::to_float(s16), zf = F16::to_float(z16);
  auto pair = [&](int e) __attribute__((always_inline)) {
    const float lo = ((float)((w >> (8 * e)) & 15u) - zf) * sc;
    const float hi = ((float)((w >> (8 * e + 4)) & 15u) - zf) * sc;
    return (uint32_t)F16::from_float(lo) | ((uint32_t)F16::from_float(hi) << 16);
  };
  return uint4v{pair(0), pair(1), pair(2), pair(3)};
}

// 2- and 3-bit latents (the low-bit settings of Sec. 4.4): eight channels' codes, stored as 16 bits of
// two-bit fields (channel u in bits 2u, 2u+1) and, for 3 bits, 8 third bits (channel u in bit u), spread
// into the 4-bit layout the kernels work on (channel u in bits 4u .. 4u+3).
__device__ __forceinline__ uint32_t expand_low_bits(uint32_t lo16, uint32_t hi8, bool three) {
  uint32_t x = lo16 & 0xffffu;
  x = (x | (x << 8)) & 0x00ff00ffu;
  x = (x | (x << 4)) & 0x0f0f0f0fu;
  x = (x | (x << 2)) & 0x33333333u;
  if (three) {
    uint32_t y = hi8 & 0xffu;
    y = (y | (y << 12)) & 0x000f000fu;
    y = (y | (y << 6)) & 0x03030303u;
    y = (y | (y << 3)) & 0x11111111u;
    x |= y << 2;
  }
  return x;
}

// Position of accumulator element i of a 32x32 MFMA tile: the lane holds
// column n = lane % 32 and rows 8*(i/4) + 4*(lane/32) + (i%4), i = 0..15.
__device__ __forceinline__ int mfma_row(int i, int lane_hi) { return 8 * (i >> 2) + 4 * lane_hi + (i & 3); }

// RoPE angle table, in tiles of 32 positions (tile T = positions 32T .. 32T+31), each tile two parts:
//  (1) float32 [pair f 0..63][cos | sin][position j 0..31], 16 KiB, so that a lane that owns
//      one rotation pair finds the angles of consecutive positions contiguously;
//  (2) float16 rows [position j][128] in rope_slot order, 8 KiB, read by the shared-key score form.
// Positions are rounded up to whole tiles.
constexpr int kRopeTilePos = 32;
constexpr int kRopeTileBytes = kHalf * 2 * kRopeTilePos * 4;      // 16384: part (1) of a tile
constexpr int kRopeRowsBytes = kRopeTilePos * kDHead * 2;         //  8192: part (2) of a tile
constexpr int kRopeTableStride = kRopeTileBytes + kRopeRowsBytes; // the table keeps both parts of a tile together
__host__ __device__ __forceinline__ size_t rope_tiles(long long n_pos) { return (size_t)((n_pos + kRopeTilePos - 1) / kRopeTilePos); }
// float index of (position p, pair f, cs = 0 cos / 1 sin) in tiles `stride` bytes apart
__host__ __device__ __forceinline__ size_t rope_f32_index(long long p, int f, int cs, int stride) {
  return (size_t)(p >> 5) * (stride / 4) + (size_t)((f * 2 + cs) * kRopeTilePos) + (size_t)(p & 31);
}

// Index of feature c' (0..127: 0..63 pair with cos, 64..127 with sin) inside a
// row of part (2), arranged so that lane-half `hi` of a wave finds the 64
// values its accumulators need contiguously: [hi][row tile][i].
__host__ __device__ __forceinline__ int rope_slot(int cprime) {
  const int rt = cprime >> 5, rr = cprime & 31;
  const int hi = (rr >> 2) & 1;
  const int i = ((rr >> 3) << 2) | (rr & 3);
  return hi * 64 + rt * 16 + i;
}

// A work unit of the score kernel: `nh` consecutive heads starting at h0, taken
// from one group or from 2 / 4 adjacent groups of equal rank and `s` heads each.
// Everything a wavefront needs about its head follows from these six numbers.
struct ScoreUnit {
  int h0, nh;
  int s;                     // heads per group inside the unit
  int head_off0;             // first head of the unit's first group
  int k_off0;                // first latent column the unit stages (group start + rank slice)
  int bk_off0;               // element offset of the unit's first head's folded weights (+ rank slice)
  int head_stride;           // elements between the folded weights of consecutive heads (rank * 128)
  int part0;                 // first partial-score plane the unit writes (2 per rank slice)
};
constexpr int kMaxScoreUnits = 64;      // per launch
constexpr int kMaxMixClasses = 7;       // ranks 64, 96, .. 256
struct ScoreMix {
  int n_cls;
  int first[kMaxMixClasses];            // first workgroup of the class
  int n_chunks[kMaxMixClasses];         // sequence chunks per (unit, sequence)
  int chunk_tokens[kMaxMixClasses];     // tokens per chunk (multiple of kTile)
  int unit0[kMaxMixClasses];            // the class's units: unit0 .. unit0 + n_units - 1 of ScoreArgs.units
  int n_units[kMaxMixClasses];
  int nk[kMaxMixClasses];               // rank / 32
};
struct ScoreUnits {
  int n_units;
  ScoreUnit u[kMaxScoreUnits];
};

struct ScoreArgs {
  const void* hk;            // latents or packed codes
  const uint16_t* hk_scale;  // fp16 bits (int4 only)
  const uint16_t* hk_zero;
  const uint16_t* mfold;     // B_k transposed, in matrix-core operand order (fold_kernel); per batch stride mfold_bstride elements
  const void* rope_rows;     // angles of the cached tokens in tiles of 32 tokens, rope_tile_stride bytes apart (the table
                             // itself, or tiles gathered by k_pos): float32 parts (1) for the one-query form, float16 rows (2)
                             // for the shared-key form
  const uint16_t* q;         // one-query form: the queries before RoPE [batch, heads, 128] (see q_row) ...
  const int32_t* q_pos;      // ... and their positions [batch * nq]
  const int32_t* seq_lens;
  float* scores;             // [parts][batch][n_heads][lpad]
  long long mfold_bstride;
  long long row_elems;       // R_k: elements per latent row
  long long max_seq;
  int seq_len;
  int lpad;                  // row pitch of the score buffer (floats)
  int batch;
  int chunk_tokens;          // tokens per workgroup (multiple of kTile)
  int n_chunks;
  int n_heads;
  int n_blocks_q;            // R_k / quant_block (int4 only)
  int quant_block;
  int bits;                  // quantized latents: 4, 3 or 2 bits per code
  float scale;               // log2(e) / sqrt(d_h)
  // shared-key form (grouped-query attention): units count key/value heads, n_heads the query heads
  const uint16_t* qfrag;     // rotated queries as contraction operands, see qfrag_kernel
  int qpk;                   // query heads per key/value head
  int n_kv;                  // key/value heads
  const float* w_scale;      // 8-bit weights (score8_kernel): the power-of-two scale of every feature column [heads][128]
  int m_qpk, m_nq;           // one-query form: Meta::qpk and Meta::nq of the call (layout of q, see q_row)
  int sk_row0, sk_rows;      // exact shared-key form: the query rows of every key/value head this launch takes
  ScoreMix mix;              // one launch over several rank classes (score16_mixed_kernel)
  int rope_tile_stride;
  float rev_hi[kHalf];       // theta^(-2f/128) / (2 pi) from the host's float64 value, as a float pair hi + lo
  float rev_lo[kHalf];
  ScoreUnits units;
};

struct RopeGatherArgs {
  const void* table;         // the part of the table that is gathered
  const int32_t* k_pos;      // [k_pos_len]
  void* rows;                // tiles over token indices 0 .. n-1 (n a multiple of 32): float16 rows (8 KiB per tile) or float32 parts (16 KiB)
  int n;
  int k_pos_len;
  int table_len;
};

// Rotated queries of the shared-key score form as A operands of its query contractions.
struct QfragArgs {
  const uint16_t* q;         // [batch, n_kv * qpk, 128]
  const int32_t* q_pos;
  uint16_t* qfrag;           // [batch][n_kv][2 feature halves][8 steps][2 lane halves][16 queries] 16-byte entries
  float theta;
  float rev_hi[kHalf];
  float rev_lo[kHalf];
  int n_kv, qpk;
  int nq;                    // queries per sequence; q_pos has batch * nq entries
  int n_heads;               // n_kv * qpk
  int small;                 // 1: qpk <= 4, operands of the 4x4x4 form
};

struct FoldArgs {
  const uint16_t* Bk;
  uint16_t* mfold;           // B_k transposed per head, in matrix-core operand order
  float rev_hi[kHalf];       // theta^(-2f/128) / (2 pi) from the host's float64 value, as a float pair hi + lo
  float rev_lo[kHalf];       // (read by the query items that ride in the same launch, see qfrag_body)
  int layout16;              // score16_kernel's operand order for: 1 = heads of rank 64 .. 256 and above 512 (slices of 256); 2 = every head of rank 64 and more
  Meta meta;
};

struct CombineArgs {
  const float* o_part;
  const float* ml_part;
  const uint16_t* Bv;
  const int32_t* seq_lens;
  float* out;                // [batch, n_heads, 128]
  float* out_latent;         // non-NULL: write the normalised latent output [batch, o_stride] instead and skip B_v
  int n_split;
  int split_tokens;
  int seq_len;
  int o_stride;
  Meta meta;
};

// Where query head h of group j finds its 128 columns inside the concatenated
// reconstruction matrices: `off` is bk_off[j] or bv_off[j]; *width receives the
// row pitch of the group's matrix (key/value heads of the group times 128).
__device__ __forceinline__ int weight_block(const Meta& m, int j, int h, int off, int* width) {
  const int s_q = m.head_off[j + 1] - m.head_off[j];
  if (m.qpk == 1) {
    *width = s_q * kDHead;
    return off + (h - m.head_off[j]) * kDHead;
  }
  *width = s_q / m.qpk * kDHead;
  return off / m.qpk + (h - m.head_off[j]) / m.qpk * kDHead;
}

// With nq > 1 queries per sequence, head h of the kernels is (key/value head, query j, model
// head of that key/value head): h = kv * qpk + j * (qpk / nq) + qh, so that all rows
// that share a key/value head are adjacent.  The caller's q and out are laid out
// [batch, nq, model query heads, 128]: q_row gives the row of head h there, q_token the query j.
__device__ __forceinline__ int q_token(const Meta& m, int h) {
  return m.nq == 1 ? 0 : (h % m.qpk) / (m.qpk / m.nq);
}
__device__ __forceinline__ size_t q_row(const Meta& m, int b, int h) {
  if (m.nq == 1) return (size_t)b * m.n_heads + h;
  const int per = m.qpk / m.nq;                     // model query heads per key/value head
  const int kv = h / m.qpk, x = h - kv * m.qpk;
  const int j = x / per, qh = x - j * per;
  return ((size_t)b * m.nq + j) * (m.n_heads / m.nq) + kv * per + qh;
}

// Group of head h, read as the word that holds its byte: for a workgroup-uniform h that is a scalar load
// from the kernel arguments, where indexing the byte array is always a vector load (a memory round trip
// ahead of whatever needs the group).
__device__ __forceinline__ int group_of(const Meta& m, int h) {
  return (int)((reinterpret_cast<const uint32_t*>(m.group_of_head)[h >> 2] >> (8 * (h & 3))) & 0xffu);
}

// Per-head offset of its value-latent accumulator inside an o_part row:
// heads are laid out in order, head h taking r_v(group(h)) floats.
__device__ __forceinline__ int o_head_off(const Meta& m, int h) {
  const int j = group_of(m, h);
  // heads before group j take sum_{i<j} s_i r_i floats = bv_off[j] / 128
  return m.bv_off[j] / kDHead + (h - m.head_off[j]) * (m.v_off[j + 1] - m.v_off[j]);
}

}  // namespace palu
