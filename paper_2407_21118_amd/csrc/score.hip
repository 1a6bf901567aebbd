// Fused key reconstruction + RoPE + query product (Sec. 3.1.2, Appendix B):
//   score[b,i,t] = RoPE(q_i) . RoPE(H_k[b,t] B_k)_i * log2(e)/sqrt(d_h)
// computed as the contraction H_k . M_i on the matrix cores, where M_i is the
// query-folded reconstruction matrix (see rope_fold.hip), followed by one
// cos/sin-weighted sum per position in registers.  Reconstructed keys exist
// only as MFMA accumulators.
//
// Design for gfx950 (not the paper's one-thread-block-per-tile Triton layout):
//   * weight-stationary: each wavefront keeps its slice of M_i (r x 128 fp16 per
//     head) in registers for the lifetime of the workgroup, so the only operand
//     that moves per token tile is the latent tile;
//   * a workgroup covers up to 4 heads that read the same (or adjacent) latent
//     columns and walks a chunk of the sequence in tiles of 32 tokens; each tile
//     (and its 32 cos/sin rows) is fetched once, several tiles ahead of its use.
//     fp16 latents go from global memory straight into LDS (LDS-direct loads,
//     no staging registers, waits counted by hand); bf16 and int4 latents are
//     parked in registers, converted, and stored to LDS;
//   * accumulators are computed transposed (features x tokens) so that the sum
//     over the features of a token is an in-lane sum plus one cross-half exchange;
//   * with 8 wavefronts (two per SIMD) the two wavefronts of a SIMD run half a
//     tile out of phase ("ping-pong"): while one issues its MFMAs the other does
//     its RoPE epilogue and queues loads, so the matrix pipe never waits for them.

#include <type_traits>

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
constexpr int kRopeTileB = kTile * kDHead * 2;   // cos/sin rows of one tile in LDS (unpadded, XOR-swizzled)
constexpr int kLdsBudget = 160 * 1024 - 1024;    // LDS of one CU, less a little slack

// LDS bytes per buffered tile and number of buffers, shared with the host for the launch
constexpr int score_buf_bytes(int width) { return kTile * (width * 2 + kRowPad) + kRopeTileB; }
constexpr int score_qf_bytes() { return 8 * 4096; }      // shared-key form: query operands of 8 wavefronts
constexpr int score_num_bufs(int width, bool dma) {
  return !dma ? 2 : (4 * score_buf_bytes(width) <= kLdsBudget ? 4 : 3);
}

// T:    storage type of unquantized latents.  The contraction itself always
//       runs in fp16 with float32 accumulation: bfloat16 latents are converted
//       while they are staged (exact for magnitudes in [2^-14, 65504],
//       saturating above, truncating below), because a bfloat16 copy of the
//       folded weights alone would cost 2^-9 relative error per element, more
//       than the whole error budget.
// NKS:  k-steps of 16: the rank of every head in the workgroup is exactly 16*NKS
// RT:   32-row feature tiles per wavefront: 4 = a whole head, 2 = half a head
//       (the two halves of a head write separate partial scores)
// G:    groups spanned by the workgroup's heads (1, 2 or 4 adjacent groups of
//       equal rank): the staged latent row is G*16*NKS columns wide
// NW:   wavefronts per workgroup.  4: one per SIMD (RT = 4: four heads, RT = 2:
//       two heads).  8: two per SIMD, RT = 2, four heads, ping-pong schedule:
//       wavefronts 0-3 own the cos halves, 4-7 the sin halves.
// I4:   latents are packed codes (4 bits; 3 or 2 with LB) with per-(token, block) scale and zero
// QP:   0: one query per key/value head, folded into the weights as described above.
//       1, 2: shared-key form, for up to 4 (QP = 1) or 16 (QP = 2) queries per key/value
//       head (the query heads of grouped-query attention, several query tokens per
//       sequence, or both).
//       The stationary operand is B_k itself (transposed), so the accumulators are the
//       key K[feature][token], rebuilt once for all queries that share it.  With q' a
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
  constexpr bool kDma = !I4 && !kIsBf16;                        // fp16 latents: global -> LDS without registers
  static_assert(QP == 0 || (NW == 8 && G == 1 && kDma), "shared-key form: fp16 latents, ping-pong schedule, one group");
  constexpr bool kPingPong = NW == 8;
  constexpr int kRank = NKS * 16;
  constexpr int kWidth = G * kRank;                             // staged columns per token
  static_assert(kWidth <= 512, "latent tile row too wide");
  constexpr int kCpr = kWidth / 8;                              // 16-byte chunks per tile row
  constexpr int kChunks = kTile * kCpr;                         // chunks per tile
  constexpr int kThreads = NW * 64;
  constexpr int kPass = (kChunks + kThreads - 1) / kThreads;    // register staging: loads per thread and tile
  constexpr int kCsPass = (kTile * 16) / kThreads;              // register staging: cos/sin chunks per thread and tile
  constexpr int kRowB = kWidth * 2 + kRowPad;                   // LDS row pitch in bytes
  constexpr int kTileB = kTile * kRowB;                         // latent tile bytes
  constexpr int kBufB = score_buf_bytes(kWidth);                // + its cos/sin rows
  constexpr int kBufs = score_num_bufs(kWidth, kDma);           // tiles resident in LDS
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
  constexpr int kCsPerWave = kTile / 4 / NW;
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
  const unsigned char* rope_base = (const unsigned char*)(a.rope_rows + (size_t)t_begin * kDHead);
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
    unsigned cs_base, cs_lim;    // the same for the cos/sin rows (32-bit offsets from rope_base)
    unsigned m0;                 // LDS address of the tile's buffer
  };
  auto dma_tile = [&](int tile_unclamped) __attribute__((always_inline)) {
    DmaTile d;
    const int r0 = min(tile_unclamped, last_tile) * kTile;
    d.src = uniform_ptr(hk_base + (size_t)((unsigned)r0 * row_bytes));
    d.lim = (unsigned)(rel_last - r0) * row_bytes;
    d.cs_base = (unsigned)r0 * (kDHead * 2u);
    d.cs_lim = (unsigned)(rel_last - r0) * (kDHead * 2u);
    d.m0 = __builtin_amdgcn_readfirstlane(lds_base + (unsigned)((tile_unclamped % kBufs) * kBufB));
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
  int st_row[kPass], st_col[kPass];
#pragma unroll
  for (int p = 0; p < kPass; ++p) {
    const int id = min(p * kThreads + tid, kChunks - 1);        // surplus threads repeat the last chunk
    st_row[p] = id / kCpr;
    st_col[p] = id - st_row[p] * kCpr;
  }
  // cos/sin rows: 16 chunks of 16 bytes per token, 512 chunks per tile, kCsPass adjacent ones per thread
  const int rope_row = (tid * kCsPass) >> 4, rope_col = (tid * kCsPass) & 15;
  struct Stage {
    uint4v h[kPass];
    uint4v cs[kCsPass];
  };
  Stage st[2];
  auto issue_loads = [&](Stage& s, int tile_unclamped) {
    const int r0 = min(tile_unclamped, last_tile) * kTile;
    {
      const unsigned rel = (unsigned)min(r0 + rope_row, rel_last);
      const uint4v* rp = reinterpret_cast<const uint4v*>(rope_base + rel * (kDHead * 2u) + rope_col * 16u);
#pragma unroll
      for (int x = 0; x < kCsPass; ++x) s.cs[x] = rp[x];
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
          s.h[p].x = *reinterpret_cast<const uint16_t*>(hk_base + off);
          if (bits == 3) s.h[p].z = hk_base[off + hi_plane - (unsigned)st_col[p]];
        }
        s.h[p].y = (uint32_t)a.hk_scale[sb] | ((uint32_t)a.hk_zero[sb] << 16);
      }
    }
  };
  auto store_stage = [&](Stage& s, int buf) {
    unsigned char* base = lds + (size_t)buf * kBufB;
#pragma unroll
    for (int x = 0; x < kCsPass; ++x) {
      const int c = rope_col + x;
      *reinterpret_cast<uint4v*>(base + kTileB + rope_row * (kDHead * 2) + ((c ^ (rope_row & 15)) * 16)) = s.cs[x];
    }
#pragma unroll
    for (int p = 0; p < kPass; ++p) {
      uint4v v = s.h[p];
      if (I4) {            // dequantize: (code - zero) * scale in float32, one rounding to fp16
        const uint32_t codes = !LB ? v.x : expand_low_bits(v.x, v.z, bits == 3);
        const float sc = F16::to_float((uint16_t)(v.y & 0xffffu));
        const float z = F16::to_float((uint16_t)(v.y >> 16));
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float lo = ((float)((codes >> (8 * e)) & 15u) - z) * sc;
          const float hi = ((float)((codes >> (8 * e + 4)) & 15u) - z) * sc;
          v[e] = (uint32_t)F16::from_float(lo) | ((uint32_t)F16::from_float(hi) << 16);
        }
      } else if (kIsBf16) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float lo = __builtin_bit_cast(float, v[e] << 16);
          const float hi = __builtin_bit_cast(float, v[e] & 0xffff0000u);
          v[e] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(lo, hi));
        }
      }
      if (p * kThreads + tid < kChunks) *reinterpret_cast<uint4v*>(base + st_row[p] * kRowB + st_col[p] * 16) = v;
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
  int wsel, rt0;
  if (kPingPong)    { wsel = wave & 3; rt0 = (wave >> 2) * 2; }
  else if (RT == 4) { wsel = wave; rt0 = 0; }
  else              { wsel = wave >> 1; rt0 = (wave & 1) * 2; }
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
    return reinterpret_cast<const half8*>(tile + (ks == 0 ? h_off0 : h_off + ks * 32));
  };

  // ---- stationary operand: folded weights of (b, head), rows [32*rt0, 32*(rt0+RT))
  half8 W[NKS][RT];
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
        W[ks][rt] = *reinterpret_cast<const half8*>(mf + ((size_t)(ks * 4 + rt0 + rt) * 64 + lane) * 8);
  };
  // Ping-pong with LDS-direct loads: the wavefronts that run the first MFMA phase fetch their
  // weights now; the others only after the first barrier, so that the barrier does not wait
  // for the issue of their 32 KiB each and their fetch overlaps the first phase.
  constexpr bool kSplitStart = kPingPong && kDma;
  if (!kSplitStart || wave < 4) load_weights();

  const int part_idx = u.part0 + (RT == 2 ? (rt0 >> 1) : 0);
  // row of head hc; in the shared-key form hc is a key/value head and its query heads' rows follow each other
  float* out_row = a.scores + ((size_t)part_idx * a.batch + b) * a.n_heads * (size_t)a.lpad +
                   (size_t)hc * (QP > 0 ? a.qpk : 1) * a.lpad;

  // MFMA phase of one tile: accumulators (features x tokens) and the tile's cos/sin weights
  struct TileAcc {
    float16v acc[RT];
    half8 cs[RT][2];
    half8 sn[QP > 0 ? RT : 1][2];    // shared-key form: cs = cos, sn = sin of the accumulators' rotation pairs
  };
  auto mfma_phase = [&](TileAcc& r, int tile) {
    const unsigned char* base = lds + (size_t)(tile % kBufs) * kBufB;
    // acc[rt][i] is feature 32*(rt0+rt) + mfma_row(i) of token lane_lo; its cos/sin weight is
    // half (rt0+rt)*16 + i of the token's table row half lane_hi, i.e. 16-byte piece
    // lane_hi*8 + (rt0+rt)*2 + i/8, stored at piece ^ (row & 15)
    const unsigned char* crow = base + kTileB + lane_lo * (kDHead * 2);
    // B operand of k-step ks: 8 latent values of token lane_lo; fetched two steps ahead of its MFMAs
    constexpr int kAhead = 2;
    half8 hf[kAhead + 1];
#pragma unroll
    for (int x = 0; x < kAhead && x < NKS; ++x) hf[x] = *h_ptr(base, x);
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
      for (int hx = 0; hx < 2; ++hx) {
        if constexpr (QP > 0) {
          // accumulator row 32 (rt0 + rt) + x is feature f or f + 64 of pair f = 32 rt + x: cos_f sits in
          // the table row where the folded form keeps the weight of row f, sin_f where it keeps that of row f + 64
          const int pc = lane_hi * 8 + rt * 2 + hx, ps = lane_hi * 8 + (rt + 2) * 2 + hx;
          r.cs[rt][hx] = *reinterpret_cast<const half8*>(crow + ((pc ^ (lane_lo & 15)) * 16));
          r.sn[rt][hx] = *reinterpret_cast<const half8*>(crow + ((ps ^ (lane_lo & 15)) * 16));
        } else {
          const int piece = lane_hi * 8 + (rt0 + rt) * 2 + hx;
          r.cs[rt][hx] = *reinterpret_cast<const half8*>(crow + ((piece ^ (lane_lo & 15)) * 16));
        }
      }
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      if (ks + kAhead < NKS)
        hf[(ks + kAhead) % (kAhead + 1)] = *h_ptr(base, ks + kAhead);
      const half8 hfrag = hf[ks % (kAhead + 1)];
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        if (ks == 0) {
          float16v zero;
#pragma unroll
          for (int i = 0; i < 16; ++i) zero[i] = 0.f;
          r.acc[rt] = F16::mfma(W[ks][rt], hfrag, zero);
        } else {
          r.acc[rt] = F16::mfma(W[ks][rt], hfrag, r.acc[rt]);
        }
      }
      __builtin_amdgcn_sched_barrier(0);        // keep the fetch-ahead order: nothing moves across a k-step
    }
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
    float part[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
#pragma unroll
      for (int i = 0; i < 8; ++i) part[i & 3] = fmaf(r.acc[rt][i], (float)r.cs[rt][0][i], part[i & 3]);
#pragma unroll
      for (int i = 0; i < 8; ++i) part[i & 3] = fmaf(r.acc[rt][8 + i], (float)r.cs[rt][1][i], part[i & 3]);
    }
    const float sum = sum_across_halves((part[0] + part[1]) + (part[2] + part[3]));
    // Unconditional store (a constant number of memory operations in flight): both
    // lane halves hold the same sum, idle wavefronts duplicate head h0's values,
    // and rows past the end of the sequence fall into the padding of the score
    // buffer (its pitch is a multiple of the tile), which nobody reads.
    out_row[t0 + lane_lo] = sum * a.scale;
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
    store_stage(st[0], 0);
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    issue_loads(st[1], 1);
    issue_loads(st[0], 2);
  }
  __syncthreads();
  if (kSplitStart && wave >= 4) load_weights();

  if constexpr (!kPingPong && kDma && NKS >= 4) {
    // One wavefront per SIMD, software-pipelined: while the matrix pipe works on
    // tile k, the vector ALU does the cos/sin-weighted sums of tile k-1 (whose
    // accumulators sit in a second register set) in the shadow of the MFMAs of
    // the first half of the k-steps.  In the middle of the tile: make sure tile
    // k+1 has landed, one barrier, request tile k+3 into the buffer of tile k-1
    // (all its readers are past the barrier).  The last k-steps already fetch the
    // first operands of tile k+1, so the pipe does not drain at the tile boundary.
    constexpr int kHalfK = NKS / 2 > 0 ? NKS / 2 : 1;
    constexpr int kGroups = 2 * RT;                      // epilogue groups of 8 accumulators
    float16v acc[2][RT];
    half8 hf[3], hn[2];                                  // B operands of this tile (ring) and the next tile's first two
    auto tile_of = [&](int tile) { return lds + (size_t)(tile % kBufs) * kBufB; };
    auto cs_piece = [&](int tile, int g) {               // cos/sin halves of accumulators 8*(g&1) .. +7 of row tile g>>1
      const unsigned char* crow = lds + (size_t)(tile % kBufs) * kBufB + kTileB + lane_lo * (kDHead * 2);
      const int piece = lane_hi * 8 + (rt0 + (g >> 1)) * 2 + (g & 1);
      return *reinterpret_cast<const half8*>(crow + ((piece ^ (lane_lo & 15)) * 16));
    };
    // `cur`: accumulator set of tile k; with_epi: tile k-1's sums are formed on the way.
    // Every MFMA is followed by its share of the other work and a scheduling fence, so
    // that the vector and memory instructions issue in the shadow of that MFMA.
    constexpr int kEpiPer = (16 + kHalfK - 1) / kHalfK;  // previous tile's accumulators handled per MFMA of the first half
    auto body = [&](auto cur_c, auto epi_c, int k) {
      constexpr int cur = decltype(cur_c)::value;
      constexpr bool with_epi = decltype(epi_c)::value;
      const unsigned char* hrow = tile_of(k);
      const unsigned char* hnext = tile_of(k + 1);
      float part[4] = {0.f, 0.f, 0.f, 0.f};
      half8 csr[2];
      DmaTile nxt;
      if (with_epi) csr[0] = cs_piece(k - 1, 0);
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) {
        if (ks == kHalfK) {
          if (with_epi) {
            const float sum = sum_across_halves((part[0] + part[1]) + (part[2] + part[3]));
            out_row[t_begin + (k - 1) * kTile + lane_lo] = sum * a.scale;
          }
          dma_wait(std::integral_constant<int, kAheadTiles - 2>{});   // tile k+1 has landed (this wavefront's share)
          __syncthreads();
          nxt = dma_tile(k + kAheadTiles);
          __builtin_amdgcn_sched_barrier(0);
        }
        // B operand two k-steps ahead; the last two steps fetch tile k+1's first operands
        if (ks + 2 < NKS) hf[(ks + 2) % 3] = *h_ptr(hrow, ks + 2);
        else hn[ks + 2 - NKS] = *h_ptr(hnext, ks + 2 - NKS);
        const half8 hfrag = hf[ks % 3];
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
          if (ks == 0) {
            float16v zero;
#pragma unroll
            for (int i = 0; i < 16; ++i) zero[i] = 0.f;
            acc[cur][rt] = F16::mfma(W[ks][rt], hfrag, zero);
          } else {
            acc[cur][rt] = F16::mfma(W[ks][rt], hfrag, acc[cur][rt]);
          }
          if (ks < kHalfK) {
            if (with_epi) {
#pragma unroll
              for (int j = 0; j < kEpiPer; ++j) {
                const int e = (ks * RT + rt) * kEpiPer + j;      // accumulator e = 16 * row tile + i of tile k-1
                if (e >= 16 * RT) continue;
                const int g = e >> 3;
                if ((e & 7) == 0 && g + 1 < kGroups) csr[(g + 1) & 1] = cs_piece(k - 1, g + 1);
                part[e & 3] = fmaf(acc[cur ^ 1][e >> 4][e & 15], (float)csr[g & 1][e & 7], part[e & 3]);
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
      hf[0] = hn[0];
      hf[1] = hn[1];
    };
    using C0 = std::integral_constant<int, 0>;
    using C1 = std::integral_constant<int, 1>;
    hf[0] = *h_ptr(tile_of(0), 0);
    hf[1] = *h_ptr(tile_of(0), 1);
    body(C0{}, std::false_type{}, 0);
    int k = 1;
    for (; k + 1 < n_tiles; k += 2) {
      body(C1{}, std::true_type{}, k);
      body(C0{}, std::true_type{}, k + 1);
    }
    // the last tile's sums (its accumulator set: parity of n_tiles - 1)
    TileAcc r;
    auto tail = [&](auto set_c, int tile) {
      constexpr int set = decltype(set_c)::value;
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        r.acc[rt] = acc[set][rt];
        r.cs[rt][0] = cs_piece(tile, 2 * rt);
        r.cs[rt][1] = cs_piece(tile, 2 * rt + 1);
      }
      epilogue(r, tile);
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
      else      { store_stage(st[1], 1); issue_loads(st[1], k + 3); }
      __syncthreads();
      if (k + 1 >= n_tiles) break;
      mfma_phase(r, k + 1);
      epilogue(r, k + 1);
      if (kDma) { dma_issue(k + 1 + kAheadTiles); dma_wait(std::integral_constant<int, kInFlight>{}); }
      else      { store_stage(st[0], 0); issue_loads(st[0], k + 4); }
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
        store_stage(s, (k + 1) & 1);
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
