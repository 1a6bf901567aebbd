// Fused key reconstruction + RoPE + query product (Sec. 3.1.2, Appendix B):
//   score[b,i,t] = RoPE(q_i) . RoPE(H_k[b,t] B_k)_i * log2(e)/sqrt(d_h)
// The keys K = H_k B_k are rebuilt on the matrix cores from the 16-bit latents and
// weights as they are (float32 accumulation), exist only as MFMA accumulators, and
// are rotated and multiplied by the rotated query in float32 on the vector ALU:
//   q' . RoPE(k, t) = sum_f k_f (c_f q'_f + s_f q'_{f+64}) + k_{f+64} (c_f q'_{f+64} - s_f q'_f)
// with c_f, s_f the float32 cos / sin of the position's angle, read from the table.
// Nothing on the way is rounded to 16 bits, so the logit error does not grow with the logit.
//
// Design for gfx950 (not the paper's one-thread-block-per-tile Triton layout):
//   * weight-stationary: each wavefront keeps its slice of B_k^T (128 x r per head,
//     laid out by fold_kernel) in registers for the lifetime of the workgroup, so the
//     only operand that moves per token tile is the latent tile;
//   * a workgroup covers up to 4 heads that read the same (or adjacent) latent
//     columns and walks a chunk of the sequence in tiles of 32 tokens; each tile
//     (and its 32 cos/sin rows) is fetched once, several tiles ahead of its use.
//     fp16 latents go from global memory straight into LDS (LDS-direct loads,
//     no staging registers, waits counted by hand); bf16 and int4 latents are
//     parked in registers, converted, and stored to LDS;
//   * accumulators are tokens x features: a lane owns one feature (one rotation pair's
//     half) of 16 tokens, so the rotated query enters as two registers per 32 features
//     and the angles of consecutive tokens are one 16-byte LDS read; the sum over
//     the features of a token is a halving exchange between lanes (DPP), 15 adds for
//     16 tokens.  (The shared-key form below keeps the transposed layout, features x tokens.);
//   * with 8 wavefronts (two per SIMD) the two wavefronts of a SIMD run half a
//     tile out of phase ("ping-pong"): while one issues its MFMAs the other does
//     its RoPE epilogue and queues loads, so the matrix pipe never waits for them.

#include <type_traits>

#pragma once
#include "palu_dev.h"

namespace palu {

// x[lane] + x[lane ^ 32] in every lane, on the VALU (no LDS crossbar round trip).
__device__ __forceinline__ float sum_across_halves(float x) {
  unsigned a = __builtin_bit_cast(unsigned, x), b = a;
  // swaps lanes 32..63 of the first register with lanes 0..31 of the second:
  // afterwards a holds the low half twice, b the high half twice
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
  return __builtin_bit_cast(float, a) + __builtin_bit_cast(float, b);
}

// A wavefront-uniform pointer, made scalar for the compiler too (operands of "s" asm constraints).
__device__ __forceinline__ const unsigned char* uniform_ptr(const unsigned char* p) {
  const uint64_t v = (uint64_t)p;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return (const unsigned char*)(((uint64_t)hi << 32) | lo);
}

// s_waitcnt immediate that waits only for the vector-memory counter (gfx9 layout:
// vmcnt in bits 3:0 and 15:14, expcnt 6:4 and lgkmcnt 11:8 left at "no wait").
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0F70; }

constexpr int kRowPad = 16;                      // bytes of padding per LDS latent row: 16-byte column reads hit distinct banks
constexpr int kRopeTileB = kTile * kDHead * 2;   // shared-key form: float16 cos/sin rows of one tile in LDS (unpadded, XOR-swizzled)
constexpr int kLdsBudget = 160 * 1024 - 1024;    // LDS of one CU, less a little slack

// LDS layout, shared with the host for the launch.
// One-query form (`exact`): a ring of latent tiles, then a ring of float32 angle tiles (kRopeTileBytes each).
// With the ping-pong schedule a wavefront reads a tile's angles one barrier phase after the tile's
// latents were last read, so that ring is one tile longer than the latent ring.
// Shared-key form: one ring of (latent tile + float16 angle rows), then the query operands.
constexpr int score_tile_bytes(int width) { return kTile * (width * 2 + kRowPad); }
constexpr int score_qf_bytes() { return 8 * 4096; }      // shared-key form: query operands of 8 wavefronts
constexpr int score_num_bufs(int width, bool dma, bool exact, bool pingpong) {
  if (!dma) return 2;
  if (!exact) return 4 * (score_tile_bytes(width) + kRopeTileB) <= kLdsBudget ? 4 : 3;
  for (int n = 4; n > 2; --n)
    if (n * score_tile_bytes(width) + (n + (pingpong ? 1 : 0)) * kRopeTileBytes <= kLdsBudget) return n;
  return 2;
}
constexpr int score_angle_bufs(int width, bool dma, bool exact, bool pingpong) {
  if (!exact) return 0;
  if (!dma) return pingpong ? 3 : 2;
  return score_num_bufs(width, dma, exact, pingpong) + (pingpong ? 1 : 0);
}
constexpr int score_lds_bytes(int width, bool dma, bool exact, bool pingpong) {
  return exact ? score_num_bufs(width, dma, true, pingpong) * score_tile_bytes(width) +
                     score_angle_bufs(width, dma, true, pingpong) * kRopeTileBytes
               : score_num_bufs(width, dma, false, pingpong) * (score_tile_bytes(width) + kRopeTileB) + score_qf_bytes();
}

template <int CTRL>
__device__ __forceinline__ float dpp_lane_move(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}

// p[i], i = 4a + b, belongs to token 8a + 4 (lane / 32) + b of a 32-token tile and to the feature this lane
// owns.  Returns the sum over the 32 lanes of the wavefront half of ONE of the lane's 16 tokens:
//   token 16 L2 + 8 L0 + 4 (lane / 32) + 2 L1 + L3     (Lk = bit k of the lane number)
// Four halving exchanges (a lane keeps the half of its values that its partner sends it the other half
// of): 8 + 4 + 2 + 1 adds instead of 16 x 5.  Partners: 7 - l inside 8 lanes (any pairing serves while all
// lanes hold all tokens), then lane ^ 1, lane ^ 2 and lane ^ 8, each agreeing on the bits that chose earlier
// halves; the last step adds lane ^ 16.
__device__ __forceinline__ float sum_tokens_over_features(const float (&p)[16], int lane) {
  const bool l0 = lane & 1, l1 = lane & 2, l2 = lane & 4, l3 = lane & 8;
  float v8[8], v4[4], v2[2];
#pragma unroll
  for (int j = 0; j < 8; ++j) v8[j] = (l2 ? p[8 + j] : p[j]) + dpp_lane_move<0x141>(l2 ? p[j] : p[8 + j]);       // row_half_mirror
#pragma unroll
  for (int j = 0; j < 4; ++j) v4[j] = (l0 ? v8[4 + j] : v8[j]) + dpp_lane_move<0xB1>(l0 ? v8[j] : v8[4 + j]);   // quad_perm [1,0,3,2]
#pragma unroll
  for (int j = 0; j < 2; ++j) v2[j] = (l1 ? v4[2 + j] : v4[j]) + dpp_lane_move<0x4E>(l1 ? v4[j] : v4[2 + j]);   // quad_perm [2,3,0,1]
  const float v1 = (l3 ? v2[1] : v2[0]) + dpp_lane_move<0x128>(l3 ? v2[0] : v2[1]);                              // row_ror 8
  return v1 + __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v1), 0x401F));       // lane ^ 16
}
__device__ __forceinline__ int summed_token_of_lane(int lane) {
  return 16 * ((lane >> 2) & 1) + 8 * (lane & 1) + 4 * (lane >> 5) + 2 * ((lane >> 1) & 1) + ((lane >> 3) & 1);
}

// T:    storage type of the weights and of unquantized latents; the matrix instruction is
//       the one of that type (fp16 or bf16 inputs as they are, float32 accumulation).
// NKS:  k-steps of 16: the rank of every head in the workgroup is exactly 16*NKS
// RT:   32-feature tiles per wavefront: 4 = a whole head, 2 = half a head: features
//       0..63 (the k_f of the identity above) or 64..127 (the k_{f+64}); the two halves
//       of a head write separate partial scores
// G:    groups spanned by the workgroup's heads (1, 2 or 4 adjacent groups of
//       equal rank): the staged latent row is G*16*NKS columns wide
// NW:   wavefronts per workgroup.  4: one per SIMD (RT = 4: four heads, RT = 2:
//       two heads).  8: two per SIMD, RT = 2, four heads, ping-pong schedule:
//       wavefronts 0-3 own features 0..63, 4-7 features 64..127.
// I4:   latents are packed codes (4 bits; 3 or 2 with LB) with per-(token, block) scale and zero
// QP:   0: one query per head, float32 rotation and query product as described above.
//       1, 2: shared-key form, for up to 4 (QP = 1) or 16 (QP = 2) queries per key/value
//       head (the query heads of grouped-query attention, several query tokens per
//       sequence, or both).  Faster per query, but the rebuilt key, the angles and their
//       products are rounded to fp16 on the way into the query contraction: its logit
//       error grows with the logit (about 4e-4 of it).
//       The accumulators are the key K[feature][token], rebuilt once for all queries
//       that share it.  With q' a
//       rotated query, its score is the contraction over f < 64 of
//         K_f (cos_f q'_f + sin_f q'_{f+64})  +  K_{f+64} (cos_f q'_{f+64} - sin_f q'_f):
//       a wavefront owns one half of the features (K_f or K_{f+64}), scales its
//       accumulators by the position's cos and sin (packed fp16), and contracts the
//       128 products per token with the queries in 8 further 32x32x16 MFMAs whose B
//       operand is what the lane already holds (its token, its 8 values per step) and
//       whose A operand (queries x the same values' query entries, written by
//       qfrag_kernel) sits in 4 KiB of LDS per wavefront.  Rows of the result are
//       queries; the two lane halves' features are summed by the contraction itself.
//       With at most 4 queries (QP = 1) the query contraction runs on
//       v_mfma_f32_4x4x4_16B_f16 instead (16 blocks of 4 queries x 4 tokens: a lane feeds
//       its own token's 4 values per step and collects that token's four scores, the two
//       lane halves are then added): 16 short instructions take less of the matrix pipe
//       than 8 full-size ones with 28 of 32 rows empty.
// LB:   quantized latents of 3 or 2 bits (a.bits) instead of 4: the codes are spread into the
//       4-bit layout while they are staged
template <typename T, int NKS, int RT, int G, int NW, bool I4, int QP = 0, bool LB = false>
__global__ __launch_bounds__(NW * 64) void score_kernel(ScoreArgs a) {
  static_assert(!LB || I4, "low-bit codes are quantized latents");
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  static_assert(NW == 4 || (NW == 8 && RT == 2), "8 wavefronts only as half-head ping-pong");
  constexpr bool kIsBf16 = !__is_same(T, F16);
  constexpr bool kExact = QP == 0;                              // one-query form
  constexpr bool kDma = !I4;                                    // unquantized latents: global -> LDS without registers
  static_assert(QP == 0 || (NW == 8 && G == 1 && kDma && !kIsBf16), "shared-key form: fp16 latents, ping-pong schedule, one group");
  static_assert(!I4 || !kIsBf16, "quantized latents are dequantized to fp16");
  constexpr bool kPingPong = NW == 8;
  using Vec = typename T::vec8;
  constexpr int kRank = NKS * 16;
  constexpr int kWidth = G * kRank;                             // staged columns per token
  static_assert(kWidth <= 512, "latent tile row too wide");
  constexpr int kCpr = kWidth / 8;                              // 16-byte chunks per tile row
  constexpr int kChunks = kTile * kCpr;                         // chunks per tile
  constexpr int kThreads = NW * 64;
  // register staging: a thread takes kCh neighbouring chunks per pass (2- and 3-bit codes: two, i.e. 4 bytes of two-bit
  // fields and 2 bytes of third bits per request instead of 2 and 1: requests cost per instruction, not per byte)
  constexpr int kCh = LB ? 2 : 1;
  static_assert(kCpr % (2 * kCh) == 0, "neighbouring threads stage chunks of one row and quantization block");
  constexpr int kPass = (kChunks / kCh + kThreads - 1) / kThreads;    // loads per thread and tile
  constexpr int kCsPass = (kExact ? kRopeTileBytes / 16 : kTile * 16) / kThreads;   // register staging: angle chunks per thread and tile
  constexpr int kRowB = kWidth * 2 + kRowPad;                   // LDS row pitch in bytes
  constexpr int kTileB = kTile * kRowB;                         // latent tile bytes
  constexpr int kBufB = kExact ? kTileB : kTileB + kRopeTileB;  // pitch of the latent ring (shared-key form: + the tile's cos/sin rows)
  constexpr int kBufs = score_num_bufs(kWidth, kDma, kExact, kPingPong);      // latent tiles resident in LDS
  constexpr int kCsBufs = kExact ? score_angle_bufs(kWidth, kDma, true, kPingPong) : 1;   // one-query form: angle tiles resident in LDS ...
  constexpr int kCsRing = kBufs * kBufB;                        // ... in a ring of their own behind the latent ring
  // LDS-direct: loop position k requests tile k + kAhead into the buffer that tile k-1
  // (whose last reader has passed a barrier) occupied; kBufs-2 requested tiles may
  // still be in flight when tile k+1 is needed
  constexpr int kAheadTiles = kBufs - 1;
  constexpr int kInFlight = kBufs - 2;
  // LDS-direct loads per wavefront and tile: one per latent row it owns, one per 4 cos/sin rows
  // A masked LDS-direct load (fewer than 64 active lanes) costs about 50 cycles of
  // issue, a full one about 6.  Rows of 32 chunks (512 bytes) are therefore requested
  // two per instruction: the pair lies contiguously in LDS (pitch 2*512+32 bytes) and
  // the odd row is stored rotated by one chunk, which keeps the 16-byte column reads
  // of 16 consecutive tokens on distinct banks.
  constexpr bool kPair = kDma && kCpr == 32;
  constexpr int kPairB = 2 * kWidth * 2 + 2 * kRowPad;           // = 2 * kRowB: same tile size as the padded layout
  constexpr int kRowsPerWave = kTile / NW;
  constexpr int kRowOps = kPair ? kRowsPerWave / 2 : kRowsPerWave;
  constexpr int kCsPerWave = kExact ? kRopeTileBytes / 1024 / NW : kTile / 4 / NW;
  constexpr int kDmaOps = kRowOps + kCsPerWave;

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);    // scalar: everything derived from it is uniform
  const int lane = tid & 63;
  const int lane_lo = lane & 31, lane_hi = lane >> 5;

  // grid (sequence chunks, units, batch): the indices come straight from the workgroup
  // id registers, so the unit descriptor and the other arguments are fetched by
  // independent scalar loads (one round trip, not a chain through index arithmetic).
  // Chunk fastest: neighbouring workgroups (dealt to the 8 XCDs round-robin) work on
  // different sequence chunks of the same heads.
  const int chunk = blockIdx.x, unit = blockIdx.y, b = blockIdx.z;
  const ScoreUnit u = a.units.u[unit];
  // have them all in registers here: the loads are issued together and waited for once
  asm volatile("" :: "s"(a.seq_lens), "s"(a.seq_len), "s"(a.chunk_tokens), "s"(a.hk), "s"(a.rope_rows), "s"(a.row_elems),
               "s"(a.max_seq), "s"(a.mfold), "s"(a.mfold_bstride), "s"(a.scores), "s"(a.lpad), "s"(a.batch), "s"(a.n_heads));
  asm volatile("" :: "s"(u.h0), "s"(u.nh), "s"(u.s), "s"(u.head_off0), "s"(u.k_off0), "s"(u.bk_off0), "s"(u.head_stride),
               "s"(u.part0));

  const int L = a.seq_lens ? min(a.seq_lens[b], a.seq_len) : a.seq_len;
  const int t_begin = chunk * a.chunk_tokens;
  if (t_begin >= L) return;                                     // uniform for the workgroup
  const int t_end = min(t_begin + a.chunk_tokens, L);
  const int n_tiles = (t_end - t_begin + kTile - 1) / kTile;
  const int last_tile = n_tiles - 1;
  const int rel_last = L - 1 - t_begin;                         // last attendable row, relative to the chunk

  // ---- addressing: a uniform 64-bit base (first row of this workgroup's sequence
  // chunk) plus 32-bit byte offsets (the host keeps a chunk of the cache below 2^31 bytes)
  const int c_lo = u.k_off0;                                    // first latent column staged by the workgroup
  const size_t seq_base = (size_t)b * a.max_seq;
  // quantized latents: 4-bit codes, or 2-bit fields followed (3 bits) by a plane of third bits at R/4 bytes
  const int bits = I4 ? (LB ? a.bits : 4) : 16;
  const unsigned row_bytes = (unsigned)a.row_elems * (unsigned)bits / 8u;
  const unsigned char* hk_base = (const unsigned char*)a.hk + (seq_base + t_begin) * row_bytes +
                                 (I4 ? (bits == 4 ? c_lo / 2 : c_lo / 4) : c_lo * 2);
  const unsigned hi_plane = (unsigned)a.row_elems / 4u + (unsigned)c_lo / 8u - (unsigned)c_lo / 4u;   // from hk_base to the third bits
  // angles of the chunk's first token: float32 tiles of 32 tokens (t_begin is a multiple of 32), or float16 rows
  const unsigned char* rope_base = (const unsigned char*)a.rope_rows + (size_t)(t_begin >> 5) * a.rope_tile_stride;
  const unsigned char* rope_base_u = uniform_ptr(rope_base);
  const unsigned lds_base = (unsigned)(size_t)lds;

  // =========================== staging, LDS-direct (fp16) ===========================
  // Each load instruction moves 16 bytes per active lane to LDS address
  // M0 + 16*lane.  A latent row (<= 1 KiB) is one instruction with kCpr active
  // lanes; four cos/sin rows (4 x 256 B, stored without padding but with their
  // 16-byte pieces XOR-swizzled by the row number) are one instruction.
  // Loads are issued unconditionally (tiles past the end of the chunk re-read its
  // last tile) so that the number of loads in flight at every wait is a constant.
  // Per-wavefront constants of its share of a tile, so that one request costs a
  // handful of scalar instructions: byte offsets of its rows inside a tile and,
  // per lane, of its pieces of the cos/sin rows.
  unsigned dma_row_off[kRowOps];                                // scalar (one row per request) or per lane (pairs)
  unsigned dma_pair_col = 0;
#pragma unroll
  for (int x = 0; x < kRowOps; ++x) {
    if (kPair) dma_row_off[x] = (unsigned)(2 * (wave * kRowOps + x) + (lane >> 5)) * row_bytes;
    else dma_row_off[x] = (unsigned)(wave * kRowsPerWave + x) * row_bytes;
  }
  if (kPair) dma_pair_col = (unsigned)((lane + (lane >> 5)) & 31) * 16u;     // odd row: LDS slot j holds chunk j+1
  // One-query form: an angle tile is 64 rows (rotation pairs) of 256 bytes: 8 pieces of cos, 8 of sin, 4 tokens
  // each; in LDS piece P of row f sits at slot P ^ (f & 15), so that the 16-byte reads of 16 lanes that own
  // consecutive pairs fall on distinct banks.  One request moves 4 rows: lane = (row, slot).
  unsigned dma_cs_off[kCsPerWave], dma_cs_swz[kCsPerWave];
#pragma unroll
  for (int x = 0; x < kCsPerWave; ++x) {
    const int row = 4 * (wave * kCsPerWave + x) + (lane >> 4);
    dma_cs_off[x] = (unsigned)row * (kDHead * 2u);
    dma_cs_swz[x] = (unsigned)(((lane & 15) ^ (row & 15)) * 16);
  }
  // what all requests of one tile share; rows past the last attendable one re-read it
  struct DmaTile {
    const unsigned char* src;    // first latent row of the tile
    unsigned lim;                // byte offset of the last attendable row inside the tile
    unsigned cs_base, cs_lim;    // the same for the cos/sin rows (32-bit offsets from rope_base); one-query form: the angle tile
    unsigned m0;                 // LDS address of the tile's buffer
    unsigned m0cs;               // one-query form: LDS address of the tile's angle buffer
  };
  auto dma_tile = [&](int tile_unclamped) __attribute__((always_inline)) {
    DmaTile d;
    const int r0 = min(tile_unclamped, last_tile) * kTile;
    d.src = uniform_ptr(hk_base + (size_t)((unsigned)r0 * row_bytes));
    d.lim = (unsigned)(rel_last - r0) * row_bytes;
    d.cs_base = (unsigned)(r0 >> 5) * (unsigned)a.rope_tile_stride;      // the tile's angles (float32 tile, or 32 float16 rows)
    d.cs_lim = (unsigned)(rel_last - r0) * (kDHead * 2u);
    d.m0 = __builtin_amdgcn_readfirstlane(lds_base + (unsigned)((tile_unclamped % kBufs) * kBufB));
    d.m0cs = __builtin_amdgcn_readfirstlane(lds_base + (unsigned)(kCsRing + (tile_unclamped % kCsBufs) * kRopeTileBytes));
    return d;
  };
  // op x of a tile: x < kRowOps a latent row (or pair of rows), else a quad of cos/sin rows
  auto dma_issue_op = [&](const DmaTile& d, int x) __attribute__((always_inline)) {
    if (x < kRowOps) {
      if constexpr (kPair) {
        const unsigned voff = min(dma_row_off[x], d.lim) + dma_pair_col;
        const unsigned m0v = d.m0 + (unsigned)((wave * kRowOps + x) * kPairB);
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" :: "s"(m0v), "v"(voff), "s"(d.src) : "memory");
      } else {
        const unsigned char* src = d.src + min(dma_row_off[x], d.lim);        // scalar address
        const unsigned m0v = d.m0 + (unsigned)((wave * kRowsPerWave + x) * kRowB);
        const unsigned voff = (unsigned)lane * 16u;
        if (kCpr == 64 || lane < kCpr)
          asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" :: "s"(m0v), "v"(voff), "s"(src) : "memory");
      }
    } else if constexpr (kExact) {
      const int y = x - kRowOps;
      const unsigned voff = d.cs_base + dma_cs_off[y] + dma_cs_swz[y];      // whole tiles exist in the table: no clamping
      const unsigned m0v = d.m0cs + (unsigned)((wave * kCsPerWave + y) * 1024);
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" :: "s"(m0v), "v"(voff), "s"(rope_base_u) : "memory");
    } else {
      const int y = x - kRowOps;
      const unsigned voff = d.cs_base + min(dma_cs_off[y], d.cs_lim) + dma_cs_swz[y];
      const unsigned m0v = d.m0 + (unsigned)(kTileB + (wave * kCsPerWave + y) * 4 * kDHead * 2);
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" :: "s"(m0v), "v"(voff), "s"(rope_base_u) : "memory");
    }
  };
  auto dma_issue = [&](int tile_unclamped) __attribute__((always_inline)) {
    const DmaTile d = dma_tile(tile_unclamped);
#pragma unroll
    for (int x = 0; x < kDmaOps; ++x) dma_issue_op(d, x);
  };
  // wait until at most `tiles_in_flight` tiles' worth of this wavefront's LDS-direct loads are outstanding
  auto dma_wait = [&](auto tiles_in_flight) {
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(decltype(tiles_in_flight)::value * kDmaOps));
  };

  // =========================== staging through registers (bf16, int4) ===========================
  const uint32_t k1024 = per_lane_constant(0x64006400u);
  int st_row[kPass], st_col[kPass];
#pragma unroll
  for (int p = 0; p < kPass; ++p) {
    const int id = min(p * kThreads + tid, kChunks / kCh - 1);  // surplus threads repeat the last chunk (pair)
    st_row[p] = id / (kCpr / kCh);
    st_col[p] = (id - st_row[p] * (kCpr / kCh)) * kCh;
  }
  // the angle tile's 1024 chunks, chunk x * kThreads + tid per pass (row = chunk / 16, piece = chunk % 16)
  struct Stage {
    uint4v h[kPass];
    uint4v cs[kCsPass];
  };
  Stage st[2];
  auto issue_loads = [&](Stage& s, int tile_unclamped) {
    const int r0 = min(tile_unclamped, last_tile) * kTile;
    if constexpr (kExact) {                              // (the shared-key form never stages through registers)
      const uint4v* rp = reinterpret_cast<const uint4v*>(rope_base + (size_t)(r0 >> 5) * a.rope_tile_stride) + tid;
#pragma unroll
      for (int x = 0; x < kCsPass; ++x) s.cs[x] = rp[x * kThreads];
    }
#pragma unroll
    for (int p = 0; p < kPass; ++p) {
      const unsigned rel = (unsigned)min(r0 + st_row[p], rel_last);
      if (!I4) {
        const unsigned off = __umul24(rel, row_bytes) + (unsigned)st_col[p] * 16u;
        s.h[p] = *reinterpret_cast<const uint4v*>(hk_base + off);
      } else {
        const size_t sb = (seq_base + t_begin + rel) * a.n_blocks_q + (c_lo + st_col[p] * 8) / a.quant_block;
        if constexpr (!LB) {
          const unsigned off = __umul24(rel, row_bytes) + (unsigned)st_col[p] * 4u;
          s.h[p].x = *reinterpret_cast<const uint32_t*>(hk_base + off);
        } else {
          const unsigned off = __umul24(rel, row_bytes) + (unsigned)st_col[p] * 2u;
          s.h[p].x = *reinterpret_cast<const uint32_t*>(hk_base + off);                                          // chunks st_col, st_col + 1
          if (bits == 3) s.h[p].z = *reinterpret_cast<const uint16_t*>(hk_base + off + hi_plane - (unsigned)st_col[p]);
        }
        // threads 2k and 2k + 1 hold chunks of the same row and quantization block: one requests the scale, one the
        // zero-point (a 2-byte request costs the memory pipeline as much as the code request), swapped in store_stage
        s.h[p].y = ((tid & 1) ? a.hk_zero : a.hk_scale)[sb];
      }
    }
  };
  // tile: the tile the stage holds (its angles go to buffer tile % kCsBufs of their own ring)
  auto store_stage = [&](Stage& s, int buf, int tile) {
    unsigned char* base = lds + (size_t)buf * kBufB;
    if constexpr (kExact) {
      unsigned char* cb = lds + kCsRing + (size_t)(tile % kCsBufs) * kRopeTileBytes;
#pragma unroll
      for (int x = 0; x < kCsPass; ++x) {
        const int id = x * kThreads + tid, f = id >> 4, piece = id & 15;
        *reinterpret_cast<uint4v*>(cb + f * 256 + ((piece ^ (f & 15)) * 16)) = s.cs[x];
      }
    }
    // quantized latents: (code - zero) * scale, one rounding to fp16.  With integer zero-points of magnitude up to
    // 1000 (what the quantizer produces for latents that are not far off centre) the packed fp16 form gives the same
    // numbers in half the operations; the whole wavefront takes the float32 form for a tile in which any of its
    // zero-points is something else (a uniform branch around two straight-line bodies).
    bool packed = I4;
    if constexpr (I4) {
#pragma unroll
      for (int p = 0; p < kPass; ++p) {
        const uint32_t own = s.h[p].y & 0xffffu;
        const uint32_t other = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)own, 0xB1, 0xf, 0xf, false) & 0xffffu;   // quad_perm [1,0,3,2]
        s.h[p].y = (tid & 1) ? (other | (own << 16)) : (own | (other << 16));                 // scale | zero-point << 16
        packed = packed && zero_point_is_small_integer((uint16_t)(s.h[p].y >> 16));
      }
      packed = __builtin_amdgcn_ballot_w64(!packed) == 0;
    }
    if (packed) {
#pragma unroll
      for (int p = 0; p < kPass; ++p) {
#pragma unroll
        for (int c = 0; c < kCh; ++c) {
          const uint32_t codes = !LB ? s.h[p].x : expand_low_bits(s.h[p].x >> (16 * c), s.h[p].z >> (8 * c), bits == 3);
          const uint4v v = dequant8_packed(codes, (uint16_t)(s.h[p].y & 0xffffu), (uint16_t)(s.h[p].y >> 16), k1024);
          if (p * kThreads + tid < kChunks / kCh) *reinterpret_cast<uint4v*>(base + st_row[p] * kRowB + (st_col[p] + c) * 16) = v;
        }
      }
    } else {
#pragma unroll
      for (int p = 0; p < kPass; ++p) {
#pragma unroll
        for (int c = 0; c < kCh; ++c) {
          uint4v v = s.h[p];
          if (I4) {
            const uint32_t codes = !LB ? v.x : expand_low_bits(v.x >> (16 * c), v.z >> (8 * c), bits == 3);
            v = dequant8_float(codes, (uint16_t)(v.y & 0xffffu), (uint16_t)(v.y >> 16));
          }
          if (p * kThreads + tid < kChunks / kCh) *reinterpret_cast<uint4v*>(base + st_row[p] * kRowB + (st_col[p] + c) * 16) = v;
        }
      }
    }
  };

  // ---- the first latent tiles go out before the (larger) weight fetch so that
  // their HBM latency overlaps it
  if constexpr (QP > 0) {
    // shared-key form: this wavefront's query operands (4 KiB) go first, straight into LDS.  Being the oldest
    // requests of the wavefront they have landed whenever one of the counted waits below has been passed.
    const int hq = u.h0 + ((wave & 3) < u.nh ? (wave & 3) : 0);
    const unsigned char* src = uniform_ptr(reinterpret_cast<const unsigned char*>(a.qfrag) +
                                           (((size_t)b * a.n_kv + hq) * 2 + (wave >> 2)) * 4096);
#pragma unroll
    for (int x = 0; x < (QP == 1 ? 1 : 4); ++x) {      // QP = 1: 1 KiB of operands
      const unsigned m0v = __builtin_amdgcn_readfirstlane(lds_base + (unsigned)(kBufs * kBufB) + (unsigned)(wave * 4096 + x * 1024));
      const unsigned voff = (unsigned)lane * 16u + (unsigned)x * 1024u;
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" :: "s"(m0v), "v"(voff), "s"(src) : "memory");
    }
  }
  if (kDma) {
#pragma unroll
    for (int x = 0; x < kAheadTiles; ++x) dma_issue(x);
  } else {
    issue_loads(st[0], 0);
  }

  // ---- which head / feature rows this wavefront owns
  // wsel: head of the unit; hh: which half of it (RT = 2).  Shared-key form: the half is features 0..63 or
  // 64..127 (feature tiles 2 hh, 2 hh + 1).  One-query form: the half is rotation pairs 0..31 or 32..63 with
  // both of their features, k_f and k_{f+64} (feature tiles hh and hh + 2), so that a wavefront reads the
  // angles of its pairs once for both.
  int wsel, hh;
  if (kPingPong)    { wsel = wave & 3; hh = wave >> 2; }
  else if (RT == 4) { wsel = wave; hh = 0; }
  else              { wsel = wave >> 1; hh = wave & 1; }
  const int rt0 = 2 * hh;                                       // shared-key form: first feature tile
  auto feature_tile = [&](int rt) __attribute__((always_inline)) { return (kExact && RT == 2) ? hh + 2 * rt : rt0 + rt; };
  const bool active = wsel < u.nh;
  const int hsel = active ? wsel : 0;                           // idle wavefronts mirror head h0: same values, same stores
  const int hc = u.h0 + hsel;
  // group of the head relative to the unit's first group (groups in a unit have equal rank and size)
  const int g_rel = G == 1 ? 0 : (u.s == 1 ? (hc - u.head_off0) : ((hc - u.head_off0) >> 1));
  const int u_in_g = hc - u.head_off0 - g_rel * u.s;
  const int kbase_b = g_rel * kRank * 2;                        // this head's first column inside the tile row, bytes
  // B operand of k-step ks (8 latent values of token lane_lo, k-octet lane_hi) sits at
  // tile + h_off + 32*ks; in the paired layout the odd rows are rotated by one chunk,
  // which wraps for the very first chunk of the row only: k-step 0 has its own offset.
  int h_off, h_off0;
  if (kPair) {
    const int odd = lane_lo & 1;
    const int rowb = (lane_lo >> 1) * kPairB + odd * (kWidth * 2);
    h_off = rowb + kbase_b + (lane_hi - odd) * 16;
    h_off0 = rowb + (((kbase_b >> 4) + lane_hi - odd) & 31) * 16;
  } else {
    h_off = lane_lo * kRowB + kbase_b + lane_hi * 16;
    h_off0 = h_off;
  }
  auto h_ptr = [&](const unsigned char* tile, int ks) __attribute__((always_inline)) {
    return reinterpret_cast<const Vec*>(tile + (ks == 0 ? h_off0 : h_off + ks * 32));
  };

  // ---- stationary operand: B_k^T of the head, feature tiles feature_tile(0 .. RT-1)
  Vec W[NKS][RT];
  // shared-key form: the query operands of this wavefront's key/value head and feature half,
  // [8 steps][2 lane halves][16 queries] x 16 bytes, behind the tile buffers
  constexpr int kQfBytes = 4096;
  const unsigned qf_off = (unsigned)(kBufs * kBufB) + (unsigned)wave * kQfBytes;
  // QP = 2: [8 steps][2 lane halves][16 queries] x 16 bytes.  QP = 1: [16 steps][2 lane halves][4 queries] x 8 bytes.
  const unsigned char* qf_lds = lds + qf_off + (QP == 1 ? (lane_hi * 4 + (lane & 3)) * 8 : (lane_hi * 16 + (lane_lo & 15)) * 16);
  auto load_weights = [&]() __attribute__((always_inline)) {
    const uint16_t* mf = a.mfold + (size_t)b * a.mfold_bstride + u.bk_off0 +
                         ((size_t)g_rel * u.s + u_in_g) * u.head_stride;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
      for (int rt = 0; rt < RT; ++rt)
        W[ks][rt] = *reinterpret_cast<const Vec*>(mf + ((size_t)(ks * 4 + feature_tile(rt)) * 64 + lane) * 8);
  };
  // Ping-pong with LDS-direct loads: the wavefronts that run the first MFMA phase fetch their
  // weights now; the others only after the first barrier, so that the barrier does not wait
  // for the issue of their 32 KiB each and their fetch overlaps the first phase.
  // one-query form with LDS-direct staging: every wavefront runs the software-pipelined loop below by itself (two to a
  // SIMD with 8 wavefronts: the matrix instructions of the two interleave, which hides the issue gap between
  // back-to-back matrix instructions of one wavefront); the phase-alternating ping-pong remains for the other forms
  constexpr bool kPipelined = kExact && kDma && NKS >= 4 && kBufs >= 3;
  constexpr bool kSplitStart = kPingPong && kDma && !kPipelined;
  if (!kSplitStart || wave < 4) load_weights();

  const int part_idx = u.part0 + (RT == 2 ? hh : 0);
  // row of head hc; in the shared-key form hc is a key/value head and its query heads' rows follow each other
  float* out_row = a.scores + ((size_t)part_idx * a.batch + b) * a.n_heads * (size_t)a.lpad +
                   (size_t)hc * (QP > 0 ? a.qpk : 1) * a.lpad;

  // MFMA phase of one tile: accumulators (features x tokens) and the tile's cos/sin weights
  struct TileAcc {
    float16v acc[RT];                // one-query form: K[token][feature]; shared-key form: K[feature][token]
    half8 cs[QP > 0 ? RT : 1][2];    // shared-key form: cs = cos, sn = sin of the accumulators' rotation pairs
    half8 sn[QP > 0 ? RT : 1][2];
  };
  auto mfma_phase = [&](TileAcc& r, int tile) {
    const unsigned char* base = lds + (size_t)(tile % kBufs) * kBufB;
    // shared-key form: acc[rt][i] is feature 32*(rt0+rt) + mfma_row(i) of token lane_lo; the cos/sin of its pair are
    // halves of the token's table row, in 16-byte pieces stored at piece ^ (row & 15)
    const unsigned char* crow = base + kTileB + lane_lo * (kDHead * 2);
    // B operand of k-step ks: 8 latent values of token lane_lo; fetched two steps ahead of its MFMAs
    constexpr int kAhead = 2;
    Vec hf[kAhead + 1];
#pragma unroll
    for (int x = 0; x < kAhead && x < NKS; ++x) hf[x] = *h_ptr(base, x);
    if constexpr (QP > 0) {
#pragma unroll
      for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int hx = 0; hx < 2; ++hx) {
          // accumulator row 32 (rt0 + rt) + x is feature f or f + 64 of pair f = 32 rt + x: the table row
          // keeps cos_f at slot(f) and sin_f at slot(f + 64)
          const int pc = lane_hi * 8 + rt * 2 + hx, ps = lane_hi * 8 + (rt + 2) * 2 + hx;
          r.cs[rt][hx] = *reinterpret_cast<const half8*>(crow + ((pc ^ (lane_lo & 15)) * 16));
          r.sn[rt][hx] = *reinterpret_cast<const half8*>(crow + ((ps ^ (lane_lo & 15)) * 16));
        }
    }
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      if (ks + kAhead < NKS)
        hf[(ks + kAhead) % (kAhead + 1)] = *h_ptr(base, ks + kAhead);
      const Vec hfrag = hf[ks % (kAhead + 1)];
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        float16v prev;
        if (ks == 0) {
#pragma unroll
          for (int i = 0; i < 16; ++i) prev[i] = 0.f;
        } else {
          prev = r.acc[rt];
        }
        // one-query form: rows = the tile's tokens (latents), columns = features (weights); shared-key form: transposed
        r.acc[rt] = kExact ? T::mfma(hfrag, W[ks][rt], prev) : T::mfma(W[ks][rt], hfrag, prev);
      }
      __builtin_amdgcn_sched_barrier(0);        // keep the fetch-ahead order: nothing moves across a k-step
    }
  };

  // ---- one-query form: the rotated query of this wavefront's head, as the two factors of
  // the identity at the top of the file for each of the lane's RT features, scaled by
  // log2(e) / sqrt(d_h): score += K[t][feature] * (cos * qa + sin * qb).
  // Feature 32 R + lane_lo, R = feature_tile(rt), is k_f (R < 2: qa = q'_f, qb = q'_{f+64}) or
  // k_{f+64} (R >= 2: qa = q'_{f+64}, qb = -q'_f) of pair f = 32 (R & 1) + lane_lo.
  float qa[RT], qb[RT];
  // (requested here, next to the weights; rotated after the start-up barrier, when they have long arrived)
  uint16_t q_raw[RT][2];
  float q_rev[RT][2];
  int q_position = 0;
  if constexpr (kExact) {
    Meta mq;                                            // only the fields q_row and q_token read
    mq.n_heads = a.n_heads; mq.qpk = a.m_qpk; mq.nq = a.m_nq;
    const uint16_t* qp = a.q + q_row(mq, b, hc) * kDHead;
    q_position = a.q_pos[b * a.m_nq + q_token(mq, hc)];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      const int f = 32 * (feature_tile(rt) & 1) + lane_lo;
      q_raw[rt][0] = qp[f];
      q_raw[rt][1] = qp[f + kHalf];
      q_rev[rt][0] = a.rev_hi[f];
      q_rev[rt][1] = a.rev_lo[f];
    }
  }
  auto rotate_query = [&]() __attribute__((always_inline)) {
    const float pos = (float)q_position;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      const int R = feature_tile(rt);
      const float x0 = T::to_float(q_raw[rt][0]), x1 = T::to_float(q_raw[rt][1]);
      // angle = pos * w_f in revolutions, w_f / 2 pi given as a float pair (hi, lo) from the host's
      // float64 value: ~1e-7 absolute accuracy for positions up to 2^24
      const float ph = pos * q_rev[rt][0];
      const float pe = fmaf(pos, q_rev[rt][0], -ph);
      const float rev = (ph - floorf(ph)) + (pe + pos * q_rev[rt][1]);
      const float sn = __builtin_amdgcn_sinf(rev), cn = __builtin_amdgcn_cosf(rev);
      const float q0 = x0 * cn - x1 * sn, q1 = x1 * cn + x0 * sn;       // q'_f, q'_{f+64}
      qa[rt] = (R < 2 ? q0 : q1) * a.scale;
      qb[rt] = (R < 2 ? q1 : -q0) * a.scale;
    }
  };
  // angle tile in LDS: pair f at row f (256 bytes), piece P (cos: 2a + lane_hi, sin: 8 + 2a + lane_hi, each the
  // four tokens 8a + 4 lane_hi + 0..3) at slot P ^ (f & 15)
  // A wavefront works on kPairBlocks blocks of 32 pairs: block pb holds pairs 32 rp + lane_lo, rp = hh (RT = 2) or pb
  // (RT = 4), and the accumulators of their two features: acc[pair_acc(pb, 0)] = k_f, acc[pair_acc(pb, 1)] = k_{f+64}.
  constexpr int kPairBlocks = RT / 2;
  auto pair_acc = [&](int pb, int h2) __attribute__((always_inline)) { return RT == 2 ? h2 : pb + 2 * h2; };
  const unsigned cs_lane_off = (unsigned)((RT == 2 ? 32 * hh : 0) + lane_lo) * 256u;
  const unsigned cs_fx = (unsigned)(lane_lo & 15);
  auto angle_piece = [&](const unsigned char* cst, int pb, int piece) __attribute__((always_inline)) {
    return *reinterpret_cast<const float4v*>(cst + cs_lane_off + (RT == 2 ? 0 : pb) * (32 * 256) + (((unsigned)(piece + lane_hi) ^ cs_fx) * 16u));
  };
  auto angle_tile = [&](int tile) __attribute__((always_inline)) {
    return lds + kCsRing + (size_t)(tile % kCsBufs) * kRopeTileBytes;
  };
  // part[4 a4 + bb] += contribution of both features of pair block pb, token bb of token quad a4
  auto rotate_dot = [&](const float16v (&acc)[RT], float (&part)[16], int pb, int a4, int bb, const float4v& c, const float4v& s)
      __attribute__((always_inline)) {
    const int i = 4 * a4 + bb;
#pragma unroll
    for (int h2 = 0; h2 < 2; ++h2) {
      const int rt = pair_acc(pb, h2);
      const float coef = fmaf(s[bb], qb[rt], c[bb] * qa[rt]);
      part[i] = fmaf(acc[rt][i], coef, part[i]);
    }
  };
  auto exact_epilogue = [&](const float16v (&acc)[RT], int tile) __attribute__((always_inline)) {
    const unsigned char* cst = angle_tile(tile);
    float part[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) part[i] = 0.f;
#pragma unroll
    for (int pb = 0; pb < kPairBlocks; ++pb)
#pragma unroll
      for (int a4 = 0; a4 < 4; ++a4) {
        const float4v c = angle_piece(cst, pb, 2 * a4), s = angle_piece(cst, pb, 8 + 2 * a4);
#pragma unroll
        for (int bb = 0; bb < 4; ++bb) rotate_dot(acc, part, pb, a4, bb, c, s);
      }
    const float sum = sum_tokens_over_features(part, lane);
    // Unconditional store (a constant number of memory operations in flight): lanes l and l ^ 16 hold the
    // same sum, idle wavefronts duplicate head h0's values, and rows past the end of the sequence fall into
    // the padding of the score buffer (its pitch is a multiple of the tile), which nobody reads.
    out_row[t_begin + tile * kTile + summed_token_of_lane(lane)] = sum;
  };
  // RoPE-weighted feature sum of one tile and the score store
  auto epilogue = [&](const TileAcc& r, int tile) {
    const int t0 = t_begin + tile * kTile;
    if constexpr (QP > 0) {
      typedef _Float16 half2f __attribute__((ext_vector_type(2)));
      typedef float float2f __attribute__((ext_vector_type(2)));
      // Step N of the contraction takes the accumulators e = 4N .. 4N+3 (e = 16 rt + i), rounded to fp16 and
      // multiplied by the position's cos and sin as packed fp16, in the order
      // (K cos)(e), (K cos)(e+1), (K sin)(e), (K sin)(e+1), then the same for e+2, e+3.
      if constexpr (QP == 1) {
        // at most 4 queries: step n = 8 rt + ip takes accumulators 2ip, 2ip+1 as (cos, cos, sin, sin) products;
        // two independent accumulation chains
        float4v s4[2] = {float4v{0.f, 0.f, 0.f, 0.f}, float4v{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
          for (int ip = 0; ip < 8; ++ip) {
            const int n = 8 * rt + ip;
            const float2f kf = {r.acc[rt][2 * ip], r.acc[rt][2 * ip + 1]};
            const half2f kk = __builtin_convertvector(kf, half2f);
            const uint4v cw = __builtin_bit_cast(uint4v, r.cs[rt][ip >> 2]), sw = __builtin_bit_cast(uint4v, r.sn[rt][ip >> 2]);
            const uint32_t cb = cw[ip & 3], sb = sw[ip & 3];
            const half2f pc = kk * __builtin_bit_cast(half2f, cb), ps = kk * __builtin_bit_cast(half2f, sb);
            const uint2v bq = {__builtin_bit_cast(uint32_t, pc), __builtin_bit_cast(uint32_t, ps)};
            const uint2v aq = *reinterpret_cast<const uint2v*>(qf_lds + n * 64);
            s4[n & 1] = __builtin_amdgcn_mfma_f32_4x4x4f16(__builtin_bit_cast(half4, aq), __builtin_bit_cast(half4, bq), s4[n & 1], 0, 0, 0);
          }
        // entry i: query i, this lane's token, this lane half's features.  Each lane half stores two of the queries.
        const float s0 = sum_across_halves(s4[0][0] + s4[1][0]), s1 = sum_across_halves(s4[0][1] + s4[1][1]);
        const float s2 = sum_across_halves(s4[0][2] + s4[1][2]), s3 = sum_across_halves(s4[0][3] + s4[1][3]);
        const int hq = 2 * lane_hi;
        float* row = out_row + (size_t)hq * a.lpad + t0 + lane_lo;
        if (hq < a.qpk) row[0] = (lane_hi ? s2 : s0) * a.scale;
        if (hq + 1 < a.qpk) row[a.lpad] = (lane_hi ? s3 : s1) * a.scale;
        return;
      }
      float16v sc;
#pragma unroll
      for (int i = 0; i < 16; ++i) sc[i] = 0.f;
#pragma unroll
      for (int N = 0; N < 4 * RT; ++N) {
        uint4v bw;
#pragma unroll
        for (int y = 0; y < 2; ++y) {
          const int e = 4 * N + 2 * y, rt = e >> 4, ip = (e & 15) >> 1;
          const float2f kf = {r.acc[rt][2 * ip], r.acc[rt][2 * ip + 1]};
          const half2f kk = __builtin_convertvector(kf, half2f);
          const uint4v cw = __builtin_bit_cast(uint4v, r.cs[rt][ip >> 2]), sw = __builtin_bit_cast(uint4v, r.sn[rt][ip >> 2]);
          const uint32_t cb = cw[ip & 3], sb = sw[ip & 3];
          const half2f pc = kk * __builtin_bit_cast(half2f, cb), ps = kk * __builtin_bit_cast(half2f, sb);
          bw[2 * y] = __builtin_bit_cast(uint32_t, pc);
          bw[2 * y + 1] = __builtin_bit_cast(uint32_t, ps);
        }
        const half8 aq = *reinterpret_cast<const half8*>(qf_lds + N * 512);
        sc = F16::mfma(aq, __builtin_bit_cast(half8, bw), sc);
      }
      // sc[i]: query 8 (i / 4) + 4 lane_hi + i % 4 of this lane's token, i < 8 (queries 16.. are not kept)
      float* row = out_row + t0 + lane_lo;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int qi = 8 * (i >> 2) + 4 * lane_hi + (i & 3);
        if (qi < a.qpk) row[(size_t)qi * a.lpad] = sc[i] * a.scale;
      }
      return;
    }
    exact_epilogue(r.acc, tile);
  };

  // ---- start-up
  if (kDma) {
    // tiles 0 .. kAheadTiles-1 are in flight; tile 0 must have landed before the first MFMA phase.
    // Where the weight loads were issued after them, those stay outstanding as well: the first
    // phase begins with the first k-steps' weights (the compiler waits per k-step from there on).
    constexpr int kStartWait = kInFlight * kDmaOps + NKS * RT;
    static_assert(!kSplitStart || kStartWait <= 63, "start-up wait exceeds the counter");
    if (kSplitStart && wave < 4) __builtin_amdgcn_s_waitcnt(vmcnt_imm(kStartWait <= 63 ? kStartWait : 0));
    else dma_wait(std::integral_constant<int, kInFlight>{});
  } else {
    // tile 0 into LDS, tiles 1 and 2 in flight.  The explicit wait (vmcnt = 0) lets
    // the loop start from the same set of pending loads as every later iteration.
    store_stage(st[0], 0, 0);
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    issue_loads(st[1], 1);
    issue_loads(st[0], 2);
  }
  __syncthreads();
  if (kSplitStart && wave >= 4) load_weights();
  if constexpr (kExact) rotate_query();

  if constexpr (kPipelined) {
    // One wavefront per SIMD, software-pipelined: while the matrix pipe works on
    // tile k, the vector ALU does the cos/sin-weighted sums of tile k-1 (whose
    // accumulators sit in a second register set) in the shadow of the MFMAs of
    // the first half of the k-steps.  In the middle of the tile: make sure tile
    // k+1 has landed, one barrier, request tile k+3 into the buffer of tile k-1
    // (all its readers are past the barrier).  The last k-steps already fetch the
    // first operands of tile k+1, so the pipe does not drain at the tile boundary.
    constexpr int kHalfK = NKS / 2 > 0 ? NKS / 2 : 1;
    // the previous tile's rotation and query product, in items: item e = (pair block pb, token quad a4, token bb)
    // handles accumulator 4 a4 + bb of both features of the block's pairs
    constexpr int kItems = 16 * kPairBlocks;
    float16v acc[2][RT];
    // latent operands are fetched kOpAhead k-steps ahead (two wavefronts to a SIMD: one is enough and saves registers)
    constexpr int kOpAhead = NW == 8 ? 1 : 2;
    Vec hf[kOpAhead + 1], hn[kOpAhead];                  // latent operands of this tile (ring) and the next tile's first ones
    auto tile_of = [&](int tile) { return lds + (size_t)(tile % kBufs) * kBufB; };
    // `cur`: accumulator set of tile k; with_epi: tile k-1's sums are formed on the way.
    // Every MFMA is followed by its share of the other work and a scheduling fence, so
    // that the vector and memory instructions issue in the shadow of that MFMA.
    constexpr int kEpiPer = (kItems + kHalfK * RT - 1) / (kHalfK * RT);   // items per MFMA of the first half
    auto body = [&](auto cur_c, auto epi_c, int k) {
      constexpr int cur = decltype(cur_c)::value;
      constexpr bool with_epi = decltype(epi_c)::value;
      const unsigned char* hrow = tile_of(k);
      const unsigned char* hnext = tile_of(k + 1);
      const unsigned char* cst = angle_tile(k - 1);
      float part[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) part[i] = 0.f;
      float4v csr[2][2];                                 // [ring][cos | sin] of the token quad being worked on and the next
      DmaTile nxt;
      if (with_epi) {
        csr[0][0] = angle_piece(cst, 0, 0);
        csr[0][1] = angle_piece(cst, 0, 8);
      }
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) {
        if (ks == kHalfK) {
          if (with_epi) {
            const float sum = sum_tokens_over_features(part, lane);
            out_row[t_begin + (k - 1) * kTile + summed_token_of_lane(lane)] = sum;
          }
          dma_wait(std::integral_constant<int, kAheadTiles - 2>{});   // tile k+1 has landed (this wavefront's share)
          __syncthreads();
          nxt = dma_tile(k + kAheadTiles);
          __builtin_amdgcn_sched_barrier(0);
        }
        // latent operand kOpAhead k-steps ahead; the last steps fetch tile k+1's first operands
        if (ks + kOpAhead < NKS) hf[(ks + kOpAhead) % (kOpAhead + 1)] = *h_ptr(hrow, ks + kOpAhead);
        else hn[ks + kOpAhead - NKS] = *h_ptr(hnext, ks + kOpAhead - NKS);
        const Vec hfrag = hf[ks % (kOpAhead + 1)];
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
          if (ks == 0) {
            float16v zero;
#pragma unroll
            for (int i = 0; i < 16; ++i) zero[i] = 0.f;
            acc[cur][rt] = T::mfma(hfrag, W[ks][rt], zero);
          } else {
            acc[cur][rt] = T::mfma(hfrag, W[ks][rt], acc[cur][rt]);
          }
          if (ks < kHalfK) {
            if (with_epi) {
#pragma unroll
              for (int j = 0; j < kEpiPer; ++j) {
                const int e = (ks * RT + rt) * kEpiPer + j;      // item of tile k-1
                if (e >= kItems) continue;
                const int g = e >> 2, bb = e & 3, pb = g >> 2, a4 = g & 3;
                if (bb == 0 && g + 1 < 4 * kPairBlocks) {        // the next token quad's angles
                  csr[(g + 1) & 1][0] = angle_piece(cst, (g + 1) >> 2, 2 * ((g + 1) & 3));
                  csr[(g + 1) & 1][1] = angle_piece(cst, (g + 1) >> 2, 8 + 2 * ((g + 1) & 3));
                }
                rotate_dot(acc[cur ^ 1], part, pb, a4, bb, csr[g & 1][0], csr[g & 1][1]);
              }
            }
          } else {
            const int x = (ks - kHalfK) * RT + rt;               // request tile k+3 into the buffer tile k-1 occupied
            if (x < kDmaOps) dma_issue_op(nxt, x);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
#pragma unroll
      for (int x = (NKS - kHalfK) * RT; x < kDmaOps; ++x) dma_issue_op(nxt, x);   // few k-steps: the rest of the requests
#pragma unroll
      for (int x = 0; x < kOpAhead; ++x) hf[x] = hn[x];
    };
    using C0 = std::integral_constant<int, 0>;
    using C1 = std::integral_constant<int, 1>;
#pragma unroll
    for (int x = 0; x < kOpAhead; ++x) hf[x] = *h_ptr(tile_of(0), x);
    body(C0{}, std::false_type{}, 0);
    int k = 1;
    for (; k + 1 < n_tiles; k += 2) {
      body(C1{}, std::true_type{}, k);
      body(C0{}, std::true_type{}, k + 1);
    }
    // the last tile's sums (its accumulator set: parity of n_tiles - 1)
    auto tail = [&](auto set_c, int tile) {
      constexpr int set = decltype(set_c)::value;
      exact_epilogue(acc[set], tile);
    };
    if (k < n_tiles) {
      body(C1{}, std::true_type{}, k);
      tail(C1{}, k);
    } else {
      tail(C0{}, k - 1);
    }
  } else if (!kPingPong) {
    // one wavefront per SIMD: compute tile k, then publish tile k+1
    TileAcc r;
    for (int k = 0; k < n_tiles; k += 2) {
      mfma_phase(r, k);
      epilogue(r, k);
      if (kDma) { dma_issue(k + kAheadTiles); dma_wait(std::integral_constant<int, kInFlight>{}); }
      else      { store_stage(st[1], 1, k + 1); issue_loads(st[1], k + 3); }
      __syncthreads();
      if (k + 1 >= n_tiles) break;
      mfma_phase(r, k + 1);
      epilogue(r, k + 1);
      if (kDma) { dma_issue(k + 1 + kAheadTiles); dma_wait(std::integral_constant<int, kInFlight>{}); }
      else      { store_stage(st[0], 0, k + 2); issue_loads(st[0], k + 4); }
      __syncthreads();
    }
  } else {
    // Ping-pong: phases alternate between barriers.  In even phases wavefronts
    // 0-3 (group A) run the MFMAs of a tile while 4-7 (group B) do everything
    // else (RoPE epilogue of their previous tile, staging); in odd phases the
    // roles swap.  Both groups execute the same loop - an aux step, a barrier,
    // an MFMA step, a barrier - and group A simply enters it one MFMA step
    // early, so group B computes tile k-1 where A computes tile k.  At loop
    // position k every thread makes sure its share of tile k+1 is in LDS and
    // requests a later tile into the buffer whose last reader (tile k-1) has
    // passed a barrier: a tile is complete one barrier before either group
    // reads it.
    const int grp = wave >> 2;                       // uniform
    const int n_iter = n_tiles + grp;
    TileAcc r;
    bool have = false;
    int tile_done = 0;
    if (grp == 0) {
      mfma_phase(r, 0);
      have = true;
      __syncthreads();
    }
    auto position = [&](int k, Stage& s) {
      if (kDma) {
        if (have) epilogue(r, tile_done);
        dma_issue(k + kAheadTiles);                  // into the buffer tile k-1 occupied
        dma_wait(std::integral_constant<int, kInFlight>{});   // everything up to tile k+1 has landed
      } else {
        // past the last tile this publishes a duplicate of it into the buffer nobody reads any more
        store_stage(s, (k + 1) & 1, k + 1);
        if (have) epilogue(r, tile_done);
        issue_loads(s, k + 3);
      }
      __syncthreads();
      const int t = k + 1 - grp;
      have = t < n_tiles;
      if (have) {
        mfma_phase(r, t);
        tile_done = t;
      }
      if (grp == 0 || k + 1 < n_iter) __syncthreads();   // group B's last position has no partner phase
    };
    for (int k = 0; k < n_iter; k += 2) {
      position(k, st[1]);
      if (k + 1 >= n_iter) break;
      position(k + 1, st[0]);
    }
  }
  if (kDma) __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));   // no LDS-direct load may outlive the workgroup's LDS allocation
}

}  // namespace palu
