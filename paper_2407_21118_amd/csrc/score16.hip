// The score kernel of score.hip (key reconstruction + RoPE + query product in float32, Sec. 3.1.2,
// Sec. 2.1 Eq. 2, Appendix B) for its most common case: unquantized fp16 / bf16 latents, ranks up
// to 256, one query per head.  Same LDS layout and LDS-direct staging; a different use of the CU:
//
//   * four wavefronts, one per SIMD, each owning ONE WHOLE HEAD: B_k^T of the head (128 x r) stays in
//     its registers (256 at rank 256).  A head's two features of a rotation pair sit in the same lane,
//     so a wavefront reads the angles of a (token, pair) once for both, sums a token's 128 products
//     with ONE lane exchange sequence per head (the half-head wavefronts of score.hip: two), and each
//     16-byte latent read from LDS feeds 8 matrix instructions (there: 2 of twice the size);
//   * v_mfma_f32_16x16x32: 16 tokens x 16 features per instruction.  An accumulator set of a 16-token
//     sub-tile is 32 registers, so two sets fit beside the weights: the vector ALU rotates and
//     multiplies sub-tile s-1 (6 operations per token and pair, dealt out between the matrix
//     instructions of sub-tile s) while the matrix pipe works on s.  The lane exchange that sums a
//     token's products runs inside the 16 lanes of a DPP row: 11 operations for the 4 tokens a lane holds.
//
// Per 32-token tile and CU this moves 160 KiB through the LDS where the ping-pong schedule moves 225,
// and issues 0.75 as many vector instructions.
//
// Several queries per key/value head (grouped-query layers, several query tokens per sequence; NQ = 2, 4, 8, other
// counts in passes with idle rows): the
// wavefront's head is a key/value head; its key tile is rebuilt once, each key pair rotated once in float32 and
// multiplied by each of the NQ rotated queries (4 + 2 NQ operations per token and pair instead of 6 NQ), then one
// lane exchange and one score row per query.

#pragma once
#include <type_traits>

#include "score.hip"

namespace palu {

// LDS bytes of score16_kernel for a staged row of `width` columns (shared with the host)
constexpr int score16_lds_bytes(int width) { return score_lds_bytes(width, true, true, false); }

// part[j], j = 0..3, belongs to token 4 (lane / 16) + j of a 16-token sub-tile and to the feature this lane
// owns (lane % 16).  Returns the sum over the 16 lanes of the row of ONE of the lane's tokens:
//   token 4 (lane / 16) + 2 L2 + L0    (Lk = bit k of the lane number),
// the same value in the four lanes that differ in bits 1 and 3.
__device__ __forceinline__ float sum_quad_over_row(const float (&p)[4], int lane) {
  const bool l0 = lane & 1, l2 = lane & 4;
  float v2[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) v2[j] = (l2 ? p[2 + j] : p[j]) + dpp_lane_move<0x141>(l2 ? p[j] : p[2 + j]);      // row_half_mirror
  float v = (l0 ? v2[1] : v2[0]) + dpp_lane_move<0xB1>(l0 ? v2[0] : v2[1]);                                     // quad_perm [1,0,3,2]
  v += dpp_lane_move<0x4E>(v);                                                                                  // quad_perm [2,3,0,1]
  return v + dpp_lane_move<0x128>(v);                                                                           // row_ror 8
}

// T:  storage type of the weights and latents (the matrix instruction of that type)
// NK: k-steps of 32: the rank of every head of the workgroup is 32 * NK (NK <= 8)
// G:  groups spanned by the workgroup's heads (1, 2 or 4 adjacent groups of equal rank): the staged
//     latent row is G * 32 * NK columns wide
// grid (sequence chunks, units, batch), 256 threads.  a.mfold: B_k^T in the operand order of
// fold_body's 16-feature layout.
// NQ: queries that share the wavefront's key/value head (grouped-query layers, several query tokens per sequence):
//     the unit's heads are then key/value heads with a.m_qpk query rows each; this launch takes rows a.sk_row0 ..
//     + a.sk_rows - 1 (at most NQ) of every key/value head: the key tile is rebuilt once, rotated once in float32
//     and multiplied by each rotated query (NQ = 1: the head's own query)
// QB: 4: the key latents are 4-bit codes (Sec. 3.4, Appendix A; fp16 layers).  Their tiles then go through registers:
//     codes, scales and zero-points are requested a tile ahead, dequantized to fp16 at the tile hand-over ((code -
//     zero) * scale, one rounding; see dequant8_packed) and written to LDS in the layout the matrix instructions
//     read; only the angle tiles stay LDS-direct.  The hand-over's vector work is not hidden by matrix instructions,
//     which is why this form is used where several queries share the key tile (NQ > 1) and score_kernel elsewhere.
// The body takes its place in the launch as arguments (sequence chunk of chunk_tokens tokens, unit, sequence), so
// that a launch over several rank classes can hand each workgroup the body of its unit's class.
template <typename T, int NK, int G, int NQ = 1, int QB = 0>
__device__ __forceinline__ void score16_body(const ScoreArgs& a, const int chunk, const int unit, const int b, const int chunk_tokens) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  using Vec = typename T::vec8;
  constexpr bool kStaged = QB != 0;
  static_assert(QB == 0 || (QB == 4 && __is_same(T, F16)), "quantized keys: 4-bit codes dequantized to fp16");
  constexpr int kRank = NK * 32;
  constexpr int kWidth = G * kRank;
  static_assert(kWidth <= 512 && NK >= 2 && NK <= 8, "latent tile row too wide / rank outside 64 .. 256");
  static_assert(NQ == 1 || G == 1, "shared keys: one group per workgroup");
  constexpr int kCpr = kWidth / 8;                              // 16-byte chunks per tile row
  constexpr int kRowB = kWidth * 2 + kRowPad;
  constexpr int kTileB = kTile * kRowB;
  // staged tiles: three buffers (tile k+1 is written while stragglers may still read tile k-1)
  constexpr int kBufs = kStaged ? 3 : score_num_bufs(kWidth, true, true, false);
  constexpr int kCsRing = kBufs * kTileB;                       // the angle tiles' ring behind the latent ring, kBufs tiles too
  constexpr int kAheadTiles = kBufs - 1;
  static_assert(kBufs >= 3, "the schedule keeps at least one tile in flight beyond the next");
  constexpr bool kPair = !kStaged && kCpr == 32;                // rows of 512 bytes are requested two per instruction (see score.hip)
  constexpr int kPairB = 2 * kWidth * 2 + 2 * kRowPad;
  constexpr int kRowsPerWave = kTile / 4;
  constexpr int kRowOps = kStaged ? 0 : (kPair ? kRowsPerWave / 2 : kRowsPerWave);   // LDS-direct row requests per wavefront and tile
  constexpr int kCsPerWave = kRopeTileBytes / 1024 / 4;
  constexpr int kDmaOps = kRowOps + kCsPerWave;
  constexpr int kMfmas = NK * 8;                                // matrix instructions per 16-token sub-tile

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int n16 = lane & 15, kq = lane >> 4;                    // feature column (B, D) or token row (A); k-octet (A, B) or token quad (D)

  const ScoreUnit u = a.units.u[unit];
  asm volatile("" :: "s"(a.seq_lens), "s"(a.seq_len), "s"(chunk_tokens), "s"(a.hk), "s"(a.rope_rows), "s"(a.row_elems),
               "s"(a.max_seq), "s"(a.mfold), "s"(a.scores), "s"(a.lpad), "s"(a.batch), "s"(a.n_heads), "s"(a.q), "s"(a.q_pos));
  asm volatile("" :: "s"(u.h0), "s"(u.nh), "s"(u.s), "s"(u.head_off0), "s"(u.k_off0), "s"(u.bk_off0), "s"(u.head_stride),
               "s"(u.part0));

  const int L = a.seq_lens ? min(a.seq_lens[b], a.seq_len) : a.seq_len;
  const int t_begin = chunk * chunk_tokens;
  if (t_begin >= L) return;                                     // uniform for the workgroup
  const int t_end = min(t_begin + chunk_tokens, L);
  const int n_tiles = (t_end - t_begin + kTile - 1) / kTile;
  const int last_tile = n_tiles - 1;
  const int rel_last = L - 1 - t_begin;

  const unsigned row_bytes = kStaged ? (unsigned)a.row_elems / 2u : (unsigned)a.row_elems * 2u;
  const size_t row0 = (size_t)b * a.max_seq + t_begin;
  const unsigned char* hk_base = (const unsigned char*)a.hk + row0 * row_bytes + (kStaged ? u.k_off0 / 2 : u.k_off0 * 2);
  const unsigned char* rope_base_u = uniform_ptr((const unsigned char*)a.rope_rows + (size_t)(t_begin >> 5) * a.rope_tile_stride);
  const unsigned lds_base = (unsigned)(size_t)lds;

  // ---- staging: LDS-direct requests, as in score_kernel (rows past the last attendable one re-read it, tiles past
  // the end of the chunk re-read its last tile, so that the number of requests in flight at every wait is a constant)
  unsigned dma_row_off[kRowOps > 0 ? kRowOps : 1];
  unsigned dma_pair_col = 0;
#pragma unroll
  for (int x = 0; x < kRowOps; ++x) {
    if (kPair) dma_row_off[x] = (unsigned)(2 * (wave * kRowOps + x) + (lane >> 5)) * row_bytes;
    else dma_row_off[x] = (unsigned)(wave * kRowsPerWave + x) * row_bytes;
  }
  if (kPair) dma_pair_col = (unsigned)((lane + (lane >> 5)) & 31) * 16u;
  unsigned dma_cs_off[kCsPerWave];
#pragma unroll
  for (int x = 0; x < kCsPerWave; ++x) {
    const int row = 4 * (wave * kCsPerWave + x) + (lane >> 4);  // pair; piece P of its 256-byte row goes to slot P ^ (row & 15)
    dma_cs_off[x] = (unsigned)row * 256u + (unsigned)(((lane & 15) ^ (row & 15)) * 16);
  }
  struct DmaTile {
    const unsigned char* src;
    unsigned lim, cs_base, m0, m0cs;
  };
  auto dma_tile = [&](int tile_unclamped) __attribute__((always_inline)) {
    DmaTile d;
    const int r0 = min(tile_unclamped, last_tile) * kTile;
    d.src = uniform_ptr(hk_base + (size_t)((unsigned)r0 * row_bytes));
    d.lim = (unsigned)(rel_last - r0) * row_bytes;
    d.cs_base = (unsigned)(r0 >> 5) * (unsigned)a.rope_tile_stride;
    d.m0 = __builtin_amdgcn_readfirstlane(lds_base + (unsigned)((tile_unclamped % kBufs) * kTileB));
    d.m0cs = __builtin_amdgcn_readfirstlane(lds_base + (unsigned)(kCsRing + (tile_unclamped % kBufs) * kRopeTileBytes));
    return d;
  };
  auto dma_issue_op = [&](const DmaTile& d, int x) __attribute__((always_inline)) {
    if (x < kRowOps) {
      if constexpr (kPair) {
        const unsigned voff = min(dma_row_off[x], d.lim) + dma_pair_col;
        const unsigned m0v = d.m0 + (unsigned)((wave * kRowOps + x) * kPairB);
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" :: "s"(m0v), "v"(voff), "s"(d.src) : "memory");
      } else {
        const unsigned char* src = d.src + min(dma_row_off[x], d.lim);
        const unsigned m0v = d.m0 + (unsigned)((wave * kRowsPerWave + x) * kRowB);
        const unsigned voff = (unsigned)lane * 16u;
        if (kCpr == 64 || lane < kCpr)
          asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" :: "s"(m0v), "v"(voff), "s"(src) : "memory");
      }
    } else {
      const int y = x - kRowOps;
      const unsigned voff = d.cs_base + dma_cs_off[y];
      const unsigned m0v = d.m0cs + (unsigned)((wave * kCsPerWave + y) * 1024);
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" :: "s"(m0v), "v"(voff), "s"(rope_base_u) : "memory");
    }
  };
  auto dma_issue = [&](int tile_unclamped) __attribute__((always_inline)) {
    const DmaTile d = dma_tile(tile_unclamped);
#pragma unroll
    for (int x = 0; x < kDmaOps; ++x) dma_issue_op(d, x);
  };

  // ---- quantized keys: a tile's codes, scales and zero-points through registers (rows past the last attendable one
  // re-read it); chunk = 8 channels of one token = 4 bytes of codes -> 16 bytes of fp16 in LDS
  constexpr int kChunks = kTile * kCpr;
  constexpr int kPass = kStaged ? (kChunks + 255) / 256 : 1;     // chunks per thread and tile
  struct Staged {
    uint32_t codes;
    uint16_t scale, zero;
  };
  Staged stage[kPass];
  int st_row[kPass], st_col[kPass], st_blk[kPass];
  uint32_t k1024 = 0;
  if constexpr (kStaged) {
    k1024 = per_lane_constant(0x64006400u);
#pragma unroll
    for (int p = 0; p < kPass; ++p) {
      const int id = min(p * 256 + tid, kChunks - 1);           // surplus threads repeat the last chunk
      st_row[p] = id / kCpr;
      st_col[p] = id - st_row[p] * kCpr;
      st_blk[p] = (u.k_off0 + st_col[p] * 8) / a.quant_block;   // quantization block of the chunk's 8 channels
    }
  }
  auto latent_loads = [&](int tile_unclamped) __attribute__((always_inline)) {
    const int r0 = min(tile_unclamped, last_tile) * kTile;
#pragma unroll
    for (int p = 0; p < kPass; ++p) {
      const unsigned rel = (unsigned)min(r0 + st_row[p], rel_last);
      stage[p].codes = *reinterpret_cast<const uint32_t*>(hk_base + (size_t)rel * row_bytes + (unsigned)st_col[p] * 4u);
      const size_t sb = (row0 + rel) * a.n_blocks_q + st_blk[p];
      stage[p].scale = a.hk_scale[sb];
      stage[p].zero = a.hk_zero[sb];
    }
  };
  // the whole wavefront takes the float32 form for a tile in which any of its zero-points is not a small integer
  // (a uniform branch around two straight-line bodies)
  auto latent_store = [&](int tile) __attribute__((always_inline)) {
    unsigned char* base = lds + (size_t)(tile % kBufs) * kTileB;
    bool small = true;
#pragma unroll
    for (int p = 0; p < kPass; ++p) small = small && zero_point_is_small_integer(stage[p].zero);
    if (__builtin_amdgcn_ballot_w64(!small) == 0) {
#pragma unroll
      for (int p = 0; p < kPass; ++p) {
        const uint4v v = dequant8_packed(stage[p].codes, stage[p].scale, stage[p].zero, k1024);
        if (p * 256 + tid < kChunks) *reinterpret_cast<uint4v*>(base + st_row[p] * kRowB + st_col[p] * 16) = v;
      }
    } else {
#pragma unroll
      for (int p = 0; p < kPass; ++p) {
        const uint4v v = dequant8_float(stage[p].codes, stage[p].scale, stage[p].zero);
        if (p * 256 + tid < kChunks) *reinterpret_cast<uint4v*>(base + st_row[p] * kRowB + st_col[p] * 16) = v;
      }
    }
  };

  // ---- this wavefront's head
  const bool active = wave < u.nh;
  const int hc = u.h0 + (active ? wave : 0);                    // idle wavefronts mirror head h0: same values, same stores
  const int g_rel = G == 1 ? 0 : (u.s == 1 ? (hc - u.head_off0) : ((hc - u.head_off0) >> 1));
  const int u_in_g = hc - u.head_off0 - g_rel * u.s;
  const int kbase_b = g_rel * kRank * 2;                        // the head's first column inside the tile row, bytes

  // the first tile's requests, then the query and the weights (everything the first sub-tile waits for), then the other tiles
  dma_issue(0);
  if constexpr (kStaged) latent_loads(0);
  uint16_t q_raw[NQ][4][2];
  float q_rev[4][2];
  int q_position[NQ];
  {
    Meta mq;                                                    // only the fields q_row and q_token read
    mq.n_heads = a.n_heads; mq.qpk = a.m_qpk; mq.nq = a.m_nq;
#pragma unroll
    for (int i = 0; i < NQ; ++i) {
      // the query row (NQ = 1: the head itself); rows past the launch's share re-read its last row and count as zero
      const int hq = NQ == 1 ? hc : hc * a.m_qpk + a.sk_row0 + min(i, a.sk_rows - 1);
      const uint16_t* qp = a.q + q_row(mq, b, hq) * kDHead;
      q_position[i] = a.q_pos[b * a.m_nq + q_token(mq, hq)];
#pragma unroll
      for (int pb = 0; pb < 4; ++pb) {
        const int f = 16 * pb + n16;
        q_raw[i][pb][0] = qp[f];
        q_raw[i][pb][1] = qp[f + kHalf];
      }
    }
#pragma unroll
    for (int pb = 0; pb < 4; ++pb) {
      const int f = 16 * pb + n16;
      q_rev[pb][0] = a.rev_hi[f];
      q_rev[pb][1] = a.rev_lo[f];
    }
  }
  // stationary operand: B_k^T of the head; W[ks][ct]: k = 32 ks + 8 kq .. + 7 of feature 16 ct + n16
  Vec W[NK][8];
  {
    const uint16_t* mf = a.mfold + u.bk_off0 + ((size_t)g_rel * u.s + u_in_g) * u.head_stride;
#pragma unroll
    for (int ks = 0; ks < NK; ++ks)
#pragma unroll
      for (int ct = 0; ct < 8; ++ct) W[ks][ct] = *reinterpret_cast<const Vec*>(mf + ((size_t)(ks * 8 + ct) * 64 + lane) * 8);
  }
#pragma unroll
  for (int x = 1; x < kAheadTiles; ++x) dma_issue(x);

  // A operand of k-step ks of sub-tile tt: token 16 tt + n16, k-octet 4 ks + kq of the head's columns.  In the paired
  // layout the odd rows are rotated by one chunk, which wraps for the first chunk of the row only.
  int a_off[2], a_off0[2];
#pragma unroll
  for (int tt = 0; tt < 2; ++tt) {
    const int tok = 16 * tt + n16;
    if (kPair) {
      const int odd = tok & 1;
      const int rowb = (tok >> 1) * kPairB + odd * (kWidth * 2);
      a_off[tt] = rowb + kbase_b + (kq - odd) * 16;
      a_off0[tt] = rowb + (((kbase_b >> 4) + kq - odd) & 31) * 16;
    } else {
      a_off[tt] = tok * kRowB + kbase_b + kq * 16;
      a_off0[tt] = a_off[tt];
    }
  }
  auto a_ptr = [&](const unsigned char* tile, int tt, int ks) __attribute__((always_inline)) {
    return reinterpret_cast<const Vec*>(tile + (ks == 0 ? a_off0[tt] : a_off[tt] + ks * 64));
  };
  auto tile_of = [&](int tile) __attribute__((always_inline)) { return lds + (size_t)(tile % kBufs) * kTileB; };

  // angles: pair f = 16 pb + n16 at row f of the angle tile; piece P (cos: 4 tt + kq, sin: 8 + 4 tt + kq: the four tokens
  // 16 tt + 4 kq + 0..3) at slot P ^ (f & 15)
  auto angle_piece = [&](const unsigned char* cst, int pb, int piece) __attribute__((always_inline)) {
    return *reinterpret_cast<const float4v*>(cst + (16 * pb + n16) * 256 + (((unsigned)(piece + kq) ^ (unsigned)n16) * 16u));
  };
  auto angle_tile = [&](int tile) __attribute__((always_inline)) { return lds + kCsRing + (size_t)(tile % kBufs) * kRopeTileBytes; };

  // the score row of the wavefront's first query row (the others follow, lpad floats apart)
  float* out_row = a.scores + ((size_t)u.part0 * a.batch + b) * a.n_heads * (size_t)a.lpad +
                   (size_t)(NQ == 1 ? hc : hc * a.m_qpk + a.sk_row0) * a.lpad + t_begin;
  const int tok_of_lane = 4 * kq + 2 * ((lane >> 2) & 1) + (lane & 1);      // see sum_quad_over_row

  // ---- start-up: tile 0, the query and the weights have landed; tiles 1 .. kAheadTiles-1 stay in flight
  __builtin_amdgcn_s_waitcnt(vmcnt_imm((kAheadTiles - 1) * kDmaOps));
  if constexpr (kStaged) {                                      // tile 0 goes to LDS, tile 1 into the staging registers
    latent_store(0);
    latent_loads(1);
  }
  __syncthreads();
  // the rotated query, scaled by log2(e) / sqrt(d_h): qa = q'_f, qb = q'_{f+64} of pair f = 16 pb + n16
  float qa[NQ][4], qb[NQ][4];
#pragma unroll
  for (int i = 0; i < NQ; ++i) {
    const float pos = (float)q_position[i];
#pragma unroll
    for (int pb = 0; pb < 4; ++pb) {
      const float x0 = T::to_float(q_raw[i][pb][0]), x1 = T::to_float(q_raw[i][pb][1]);
      const float ph = pos * q_rev[pb][0];
      const float pe = fmaf(pos, q_rev[pb][0], -ph);
      const float rev = (ph - floorf(ph)) + (pe + pos * q_rev[pb][1]);          // the angle in revolutions, see score.hip
      const float sn = __builtin_amdgcn_sinf(rev), cn = __builtin_amdgcn_cosf(rev);
      const float on = (NQ == 1 || i < a.sk_rows) ? a.scale : 0.f;
      qa[i][pb] = (x0 * cn - x1 * sn) * on;
      qb[i][pb] = (x1 * cn + x0 * sn) * on;
    }
  }

  float4v acc[2][8];                                            // [sub-tile parity][16-feature tile]: tokens 4 kq + 0..3 of feature 16 ct + n16
  Vec af[3], an[2];                                             // A operands of this sub-tile (ring) and the next sub-tile's first two

  // The rotation and query product of a sub-tile in 32 half-items of three vector operations: pair block pb
  // (features 16 pb + n16 and + 64), token j, feature half h2:
  //   score += k_f (c qa + s qb)   (h2 = 0),     score += k_{f+64} (c qb - s qa)   (h2 = 1)
  auto half_item = [&](const float4v (&ac)[8], float (&part)[4], int e2, const float4v& c, const float4v& s)
      __attribute__((always_inline)) {
    const int pb = e2 >> 3, j = (e2 >> 1) & 3, h2 = e2 & 1;
    const float coef = h2 == 0 ? fmaf(s[j], qb[0][pb], c[j] * qa[0][pb]) : fmaf(-s[j], qa[0][pb], c[j] * qb[0][pb]);
    part[j] = fmaf(ac[pb + 4 * h2][j], coef, part[j]);
  };
  // Shared keys (NQ > 1): pair block pb, token j in 1 + NQ / 2 steps of four operations: step 0 rotates the key pair,
  //   r0 = k_f c - k_{f+64} s,  r1 = k_{f+64} c + k_f s,   step x > 0 adds r0 q'_f + r1 q'_{f+64} for queries 2x-2 and 2x-1
  constexpr int kPairSteps = 1 + NQ / 2;
  auto pair_step = [&](const float4v (&ac)[8], float (&part)[NQ][4], float (&rot)[2], int st, const float4v& c, const float4v& s)
      __attribute__((always_inline)) {
    const int it = st / kPairSteps, x = st % kPairSteps, pb = it >> 2, j = it & 3;
    if (x == 0) {
      const float kf = ac[pb][j], kg = ac[pb + 4][j];
      rot[0] = fmaf(-kg, s[j], kf * c[j]);
      rot[1] = fmaf(kf, s[j], kg * c[j]);
    } else {
#pragma unroll
      for (int i = 0; i < NQ; ++i)
        if (i / 2 == x - 1) part[i][j] = fmaf(rot[1], qb[i][pb], fmaf(rot[0], qa[i][pb], part[i][j]));
    }
  };
  // the sum over the features of the 4 tokens a lane holds (sum_quad_over_row) in four steps of at most three operations
  struct RowSum {
    float v2[2], v;
  };
  auto row_sum_step = [&](RowSum& r, const float (&p)[4], int step) __attribute__((always_inline)) {
    const bool l0 = lane & 1, l2 = lane & 4;
    if (step == 0) r.v2[0] = (l2 ? p[2] : p[0]) + dpp_lane_move<0x141>(l2 ? p[0] : p[2]);
    if (step == 1) r.v2[1] = (l2 ? p[3] : p[1]) + dpp_lane_move<0x141>(l2 ? p[1] : p[3]);
    if (step == 2) r.v = (l0 ? r.v2[1] : r.v2[0]) + dpp_lane_move<0xB1>(l0 ? r.v2[0] : r.v2[1]);
    if (step == 3) {
      r.v += dpp_lane_move<0x4E>(r.v);
      r.v += dpp_lane_move<0x128>(r.v);
    }
  };
  // the whole of it at once (the last sub-tile of the chunk)
  auto finish = [&](const float4v (&ac)[8], int tile, int tt) __attribute__((always_inline)) {
    const unsigned char* cst = angle_tile(tile);
    if constexpr (NQ == 1) {
      float part[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int pb = 0; pb < 4; ++pb) {
        const float4v c = angle_piece(cst, pb, 4 * tt), s = angle_piece(cst, pb, 8 + 4 * tt);
#pragma unroll
        for (int x = 0; x < 8; ++x) half_item(ac, part, 8 * pb + x, c, s);
      }
      out_row[tile * kTile + 16 * tt + tok_of_lane] = sum_quad_over_row(part, lane);
    } else {
      float part[NQ][4];
      float rot[2];
#pragma unroll
      for (int i = 0; i < NQ; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) part[i][j] = 0.f;
#pragma unroll
      for (int pb = 0; pb < 4; ++pb) {
        const float4v c = angle_piece(cst, pb, 4 * tt), s = angle_piece(cst, pb, 8 + 4 * tt);
#pragma unroll
        for (int x = 0; x < 4 * kPairSteps; ++x) pair_step(ac, part, rot, 4 * kPairSteps * pb + x, c, s);
      }
#pragma unroll
      for (int i = 0; i < NQ; ++i) {
        const float v = sum_quad_over_row(part[i], lane);
        if (i < a.sk_rows) out_row[(size_t)i * a.lpad + tile * kTile + 16 * tt + tok_of_lane] = v;
      }
    }
  };

  // Sub-tile tt of tile k: its matrix instructions, each followed by at most a few vector operations of the previous
  // sub-tile (one wavefront per SIMD issues in order: more than three between two matrix instructions leave the
  // matrix pipe idle): the 32 half-items over the first three quarters of the instructions, the lane exchange over the
  // last quarter; in the second sub-tile of a tile also the tile hand-over: wait for this wavefront's share of tile
  // k+1, one barrier, request tile k + kAheadTiles into the buffers tile k-1 occupied (every reader of tile k-1, its
  // last sub-tile's items included, is past that barrier).
  constexpr int kTail = 5 * NQ;                                 // per query: four lane-exchange steps and the store ...
  constexpr int kSumSlot0 = kMfmas - kTail >= kMfmas / 2 ? kMfmas - kTail : kMfmas / 2;   // ... one per slot where the slots suffice
  constexpr int kTailSlots = kMfmas - kSumSlot0;
  constexpr int kItemSlots = kMfmas * 3 / 4 < kSumSlot0 ? kMfmas * 3 / 4 : kSumSlot0;
  constexpr int kSteps = NQ == 1 ? 32 : 16 * kPairSteps;        // half-items, or steps of the shared-key pairs, per sub-tile
  static_assert(kItemSlots <= kSumSlot0, "the lane exchange follows the last half-item");
  // k-step before which the hand-over happens: the middle of the sub-tile where its last two k-steps (which already
  // read tile k+1) come after it, else its start
  constexpr int kHandK = NK >= 4 ? NK / 2 : 0;
  constexpr int kAfterHand = kMfmas - kHandK * 8;              // matrix instructions after the hand-over
  constexpr int kDmaStep = kAfterHand / kDmaOps > 0 ? kAfterHand / kDmaOps : 1;
  auto body = [&](auto tt_c, int k, bool have_prev) __attribute__((always_inline)) {
    constexpr int tt = decltype(tt_c)::value;
    const unsigned char* hrow = tile_of(k);
    const unsigned char* hnext = tile_of(tt == 0 ? k : k + 1);
    // the previous sub-tile: (k, 0) for tt = 1, (k - 1, 1) for tt = 0
    const int ptile = tt == 0 ? k - 1 : k;
    constexpr int ptt = 1 - tt;
    const unsigned char* cst = angle_tile(have_prev ? ptile : k);
    float part[NQ][4];
    float rot[2];
#pragma unroll
    for (int i = 0; i < NQ; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) part[i][j] = 0.f;
    float4v csr[2][2];
    RowSum rs;
    DmaTile nxt;
    if (have_prev) {
      csr[0][0] = angle_piece(cst, 0, 4 * ptt);
      csr[0][1] = angle_piece(cst, 0, 8 + 4 * ptt);
    }
#pragma unroll
    for (int ks = 0; ks < NK; ++ks) {
      if (tt == 1 && ks == kHandK) {
        __builtin_amdgcn_s_waitcnt(vmcnt_imm((kAheadTiles - 2) * kDmaOps));         // tile k+1 has landed (this wavefront's share)
        if constexpr (kStaged) latent_store(k + 1);             // ... in the staging registers: dequantized into buffer (k+1) % 3
        __syncthreads();
        if constexpr (kStaged) latent_loads(k + 2);
        nxt = dma_tile(k + kAheadTiles);
        __builtin_amdgcn_sched_barrier(0);
      }
      // A operand two k-steps ahead; the last two steps fetch the next sub-tile's first operands
      if (ks + 2 < NK) af[(ks + 2) % 3] = *a_ptr(hrow, tt, ks + 2);
      else an[ks + 2 - NK] = *a_ptr(hnext, 1 - tt, ks + 2 - NK);
      const Vec afrag = af[ks % 3];
#pragma unroll
      for (int ct = 0; ct < 8; ++ct) {
        const int mi = ks * 8 + ct;
        float4v prev;
        if (ks == 0) prev = float4v{0.f, 0.f, 0.f, 0.f};
        else prev = acc[tt][ct];
        if constexpr (__is_same(T, F16)) acc[tt][ct] = __builtin_amdgcn_mfma_f32_16x16x32_f16(afrag, W[ks][ct], prev, 0, 0, 0);
        else acc[tt][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(afrag, W[ks][ct], prev, 0, 0, 0);
        if (have_prev) {
          if (mi < kItemSlots) {
            // steps [mi * kSteps / kItemSlots, (mi + 1) * kSteps / kItemSlots); a quarter of them per pair block
#pragma unroll
            for (int e2 = mi * kSteps / kItemSlots; e2 < (mi + 1) * kSteps / kItemSlots; ++e2) {
              const int pb = e2 / (kSteps / 4);
              if (e2 % (kSteps / 4) == 0 && pb + 1 < 4) {       // the next pair block's angles
                csr[(pb + 1) & 1][0] = angle_piece(cst, pb + 1, 4 * ptt);
                csr[(pb + 1) & 1][1] = angle_piece(cst, pb + 1, 8 + 4 * ptt);
              }
              if constexpr (NQ == 1) half_item(acc[ptt], part[0], e2, csr[pb & 1][0], csr[pb & 1][1]);
              else pair_step(acc[ptt], part, rot, e2, csr[pb & 1][0], csr[pb & 1][1]);
            }
          } else if (mi >= kSumSlot0) {
#pragma unroll
            for (int ts = (mi - kSumSlot0) * kTail / kTailSlots; ts < (mi - kSumSlot0 + 1) * kTail / kTailSlots; ++ts) {
              const int i = ts / 5, x = ts % 5;                                // query, step
              if (x < 4) row_sum_step(rs, part[i], x);
              else if (NQ == 1 || i < a.sk_rows) out_row[(size_t)i * a.lpad + ptile * kTile + 16 * ptt + tok_of_lane] = rs.v;
            }
          }
        }
        if (tt == 1 && ks >= kHandK) {
          const int y = mi - kHandK * 8;                         // the requests, spread over the instructions after the hand-over
          if (y % kDmaStep == 0 && y / kDmaStep < kDmaOps) dma_issue_op(nxt, y / kDmaStep);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    if (tt == 1) {
#pragma unroll
      for (int x = (kAfterHand + kDmaStep - 1) / kDmaStep; x < kDmaOps; ++x) dma_issue_op(nxt, x);   // few matrix instructions: the rest of the requests
    }
    af[0] = an[0];
    af[1] = an[1];
  };

  af[0] = *a_ptr(tile_of(0), 0, 0);
  if (NK > 1) af[1] = *a_ptr(tile_of(0), 0, 1);
  for (int k = 0; k < n_tiles; ++k) {
    body(std::integral_constant<int, 0>{}, k, k > 0);
    body(std::integral_constant<int, 1>{}, k, true);
  }
  finish(acc[1], last_tile, 1);
  __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));     // no LDS-direct load may outlive the workgroup's LDS allocation
}

// grid (sequence chunks, units, batch), 256 threads: every unit of the launch has rank 32 * NK
template <typename T, int NK, int G, int NQ = 1, int QB = 0>
__global__ __launch_bounds__(256) void score16_kernel(ScoreArgs a) {
  score16_body<T, NK, G, NQ, QB>(a, blockIdx.x, blockIdx.y, blockIdx.z, a.chunk_tokens);
}

// One launch for a layer whose groups have different ranks (the ranks a search assigns per group, Sec. 3.3):
// a.mix lists the rank classes, heaviest first, each with its own chunk length (chosen by the host so that
// workgroups of different classes take about as long) and its units, which lie side by side in a.units.
// grid (sum over classes of chunks x units x batch), 256 threads; the workgroups of a class are consecutive.
template <typename T>
__global__ __launch_bounds__(256) void score16_mixed_kernel(ScoreArgs a) {
  int c = 0;
#pragma unroll
  for (int i = 1; i < kMaxMixClasses; ++i)
    if (i < a.mix.n_cls && (int)blockIdx.x >= a.mix.first[i]) c = i;
  const int local = (int)blockIdx.x - a.mix.first[c];
  const int n_chunks = a.mix.n_chunks[c], n_units = a.mix.n_units[c];
  const int chunk = local % n_chunks, rest = local / n_chunks;
  const int unit = a.mix.unit0[c] + rest % n_units, b = rest / n_units;
  const int ct = a.mix.chunk_tokens[c];
  switch (a.mix.nk[c]) {
    case 2: score16_body<T, 2, 1>(a, chunk, unit, b, ct); break;
    case 3: score16_body<T, 3, 1>(a, chunk, unit, b, ct); break;
    case 4: score16_body<T, 4, 1>(a, chunk, unit, b, ct); break;
    case 5: score16_body<T, 5, 1>(a, chunk, unit, b, ct); break;
    case 6: score16_body<T, 6, 1>(a, chunk, unit, b, ct); break;
    case 7: score16_body<T, 7, 1>(a, chunk, unit, b, ct); break;
    default: score16_body<T, 8, 1>(a, chunk, unit, b, ct); break;
  }
}

}  // namespace palu
