// Low-precision key reconstruction (Sec. 4.5.2, last paragraph: the decomposed weight matrices quantized
// further so that low-precision matrix hardware rebuilds the keys).  Opt-in variant of score16_kernel:
//   * B_k as 8-bit floats (OCP E4M3) with one power-of-two scale per feature column, made per call by
//     fold8_kernel:  B8[k, f] = round(B[k, f] / e_f),  e_f the smallest power of two with max_k |B[k, f]| / e_f <= 448;
//   * fp16 key latents rounded to E4M3 while they are staged (clamped to +-448, no scale);
//   * K[t, f] = e_f sum_k H8[t, k] B8[k, f] on the 8-bit matrix instructions (products of 8-bit floats are exact
//     in float32, float32 accumulation): v_mfma_f32_16x16x128_f8f6f4 at rank 256 (128 k per instruction, the
//     form that runs at twice the fp16 rate), v_mfma_f32_16x16x32_fp8_fp8 at the other ranks; e_f rides in the
//     rotated-query factors, so the epilogue is unchanged: RoPE and the query product in float32.
// The result is attention over keys rebuilt from the rounded operands, a different numeric contract
// from the default path (about 3 % noise on every key entry).  Weights take half the registers (128 at
// rank 256), the latent tile half the LDS bytes.
// Same workgroup shape as score16_kernel (one whole head per wavefront, two accumulator sets, the previous
// sub-tile's vector work between the matrix instructions); the latent tile goes through registers (it is
// converted on the way), the angle tiles stay LDS-direct.

#include <type_traits>

#include "score16.hip"

namespace palu {

// ---- B_k -> E4M3 in operand order, and its column scales ----------------------------------------
typedef int int8v __attribute__((ext_vector_type(8)));

struct Fold8Args {
  const uint16_t* Bk;
  unsigned char* w8;         // per head r * 128 bytes at byte offset (bk_off[group] + head in group * r * 128)
  float* scale;              // [n_heads][128]
  Meta meta;
};

// two floats -> two E4M3 bytes in the low half of the result (round to nearest even; inputs within +-448)
__device__ __forceinline__ uint32_t cvt2_e4m3(float a, float b) {
  return (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(a, b, 0, false) & 0xffffu;
}

// grid (n_heads, 4), 256 threads: a workgroup does 32 feature columns of one head.  Column maxima first (the scale
// needs all rows; thread = (column, one of 8 row classes)), then the rounded values in operand order of
// v_mfma_f32_16x16x32_fp8_fp8's B operand: per k-step of 32 rows, 512 words of 8 bytes: word (feature tile ct, lane) =
// rows 8 (lane / 16) .. + 7 of feature 16 ct + lane % 16.  Heads of rank 256 are laid out for
// v_mfma_f32_16x16x128_f8f6f4 instead: per k-step of 128 rows, 512 words of 32 bytes: word (ct, lane) = rows
// 32 (lane / 16) .. + 31 of that feature.  (Which k of a step a lane's byte stands for is the kernel's choice, as
// long as both operands agree: the sum runs over all of them.)
template <typename T>
__global__ __launch_bounds__(256) void fold8_kernel(Fold8Args a) {
  __shared__ float cmax[8][32];
  __shared__ float cscale[32];
  const int tid = threadIdx.x, h = blockIdx.x, q4 = blockIdx.y;
  const Meta& m = a.meta;
  const int j = group_of(m, h);
  const int u = h - m.head_off[j];
  const int r = m.k_off[j + 1] - m.k_off[j];
  int width;
  const uint16_t* B = a.Bk + weight_block(m, j, h, m.bk_off[j], &width) + 32 * q4;
  {
    const int col = tid & 31, rl = tid >> 5;
    float mx = 0.f;
    for (int k0 = rl; k0 < r; k0 += 64) {                        // 8 independent loads per batch (ranks are multiples of 32)
      uint16_t raw[8];
#pragma unroll
      for (int x = 0; x < 8; ++x) raw[x] = B[(size_t)min(k0 + 8 * x, r - 8 + rl) * width + col];
#pragma unroll
      for (int x = 0; x < 8; ++x) mx = fmaxf(mx, fabsf(T::to_float(raw[x])));
    }
    cmax[rl][col] = mx;
  }
  __syncthreads();
  if (tid < 32) {
    float mm = 0.f;
#pragma unroll
    for (int x = 0; x < 8; ++x) mm = fmaxf(mm, cmax[x][tid]);
    // smallest power of two e with mm / e <= 448: e = 2^ceil(log2(mm / 448))
    float e = 1.f;
    if (mm > 0.f) {
      int ex;
      const float fr = frexpf(mm * (1.f / 448.f), &ex);          // mm / 448 = fr * 2^ex, fr in [0.5, 1); that division is not exact,
      e = ldexpf(1.f, fr == 0.5f ? ex - 1 : ex);                  // so the boundary is settled on the exact products below
      if (mm > 448.f * e) e *= 2.f;
      else if (mm <= 224.f * e) e *= 0.5f;
    }
    cscale[tid] = e;
    a.scale[(size_t)h * kDHead + 32 * q4 + tid] = e;
  }
  __syncthreads();
  unsigned char* out = a.w8 + m.bk_off[j] + (size_t)u * r * kDHead;
  const bool wide = r == 256;
  // items of 8 rows of one feature: (k-step, feature tile 2 q4 + ctl, lane[, quarter of the 32-byte word])
  const int n_items = wide ? (r >> 7) * 2 * 64 * 4 : (r >> 5) * 2 * 64;
  for (int w = tid; w < n_items; w += 256) {
    int ks, ctl, lane, k0;
    size_t dst;
    if (wide) {
      const int quarter = w & 3, word = w >> 2;
      ks = word >> 7; ctl = (word >> 6) & 1; lane = word & 63;
      k0 = 128 * ks + 32 * (lane >> 4) + 8 * quarter;
      dst = ((size_t)(ks * 8 + 2 * q4 + ctl) * 64 + lane) * 32 + quarter * 8;
    } else {
      ks = w >> 7; ctl = (w >> 6) & 1; lane = w & 63;
      k0 = 32 * ks + 8 * (lane >> 4);
      dst = ((size_t)(ks * 8 + 2 * q4 + ctl) * 64 + lane) * 8;
    }
    const int c = 16 * ctl + (lane & 15);                         // column inside this workgroup's 32
    const float inv = 1.f / cscale[c];                            // a power of two: exact
    uint16_t raw[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) raw[e] = B[(size_t)(k0 + e) * width + c];
    float v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = T::to_float(raw[e]) * inv;
    uint2v pk;
    pk.x = cvt2_e4m3(v[0], v[1]) | (cvt2_e4m3(v[2], v[3]) << 16);
    pk.y = cvt2_e4m3(v[4], v[5]) | (cvt2_e4m3(v[6], v[7]) << 16);
    *reinterpret_cast<uint2v*>(out + dst) = pk;
  }
}

constexpr int kRowPad8 = 16;      // bytes of padding per LDS row of the 8-bit latent tile
constexpr int score8_lds_bytes(int width) { return 3 * kTile * (width + kRowPad8) + 3 * kRopeTileBytes; }

// NK: k-steps of 32: the rank of every head of the workgroup is 32 * NK (2 <= NK <= 8)
// G:  groups spanned by the workgroup's heads, see score16_kernel
// a.mfold: fold8_kernel's bytes; a.w_scale: its column scales.  fp16 latents and queries.
template <int NK, int G>
__global__ __launch_bounds__(256) void score8_kernel(ScoreArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  using T = F16;
  constexpr int kRank = NK * 32;
  constexpr int kWidth = G * kRank;
  static_assert(kWidth <= 512 && NK >= 2 && NK <= 8, "latent tile row too wide / rank outside 64 .. 256");
  constexpr int kCpr = kWidth / 8;                              // 8-element chunks per tile row: 16 bytes in memory, 8 in LDS
  constexpr int kChunks = kTile * kCpr;
  constexpr int kPass = (kChunks + 255) / 256;                  // chunks per thread and tile
  constexpr int kRowB = kWidth + kRowPad8;
  constexpr int kTileB = kTile * kRowB;
  constexpr int kBufs = 3;                                      // latent tiles: tile k+1 is written while stragglers may still read tile k-1
  constexpr int kCsBufs = 3;                                    // angle tiles: k (read), k+1 (landed), k+2 (in flight)
  constexpr int kCsRing = kBufs * kTileB;
  constexpr int kCsPerWave = kRopeTileBytes / 1024 / 4;
  // rank 256: two k-steps of 128 on v_mfma_f32_16x16x128_f8f6f4 (operands of 32 bytes); else NK k-steps of 32 (8 bytes)
  constexpr bool kWide = NK == 8;
  constexpr int NS = kWide ? NK / 4 : NK;                       // k-steps
  constexpr int kStepB = kWide ? 128 : 32;                      // bytes of a latent row per k-step
  using Frag = typename std::conditional<kWide, int8v, long>::type;
  constexpr int kMfmas = NS * 8;

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int n16 = lane & 15, kq = lane >> 4;

  const int chunk = blockIdx.x, unit = blockIdx.y, b = blockIdx.z;
  const ScoreUnit u = a.units.u[unit];
  const int L = a.seq_lens ? min(a.seq_lens[b], a.seq_len) : a.seq_len;
  const int t_begin = chunk * a.chunk_tokens;
  if (t_begin >= L) return;                                     // uniform for the workgroup
  const int t_end = min(t_begin + a.chunk_tokens, L);
  const int n_tiles = (t_end - t_begin + kTile - 1) / kTile;
  const int last_tile = n_tiles - 1;
  const int rel_last = L - 1 - t_begin;

  const unsigned row_bytes = (unsigned)a.row_elems * 2u;
  const unsigned char* hk_base = (const unsigned char*)a.hk + ((size_t)b * a.max_seq + t_begin) * row_bytes + u.k_off0 * 2;
  const unsigned char* rope_base_u = uniform_ptr((const unsigned char*)a.rope_rows + (size_t)(t_begin >> 5) * a.rope_tile_stride);
  const unsigned lds_base = (unsigned)(size_t)lds;

  // ---- angle tiles: LDS-direct, 4 requests per wavefront and tile (as in score16_kernel)
  unsigned dma_cs_off[kCsPerWave];
#pragma unroll
  for (int x = 0; x < kCsPerWave; ++x) {
    const int row = 4 * (wave * kCsPerWave + x) + (lane >> 4);
    dma_cs_off[x] = (unsigned)row * 256u + (unsigned)(((lane & 15) ^ (row & 15)) * 16);
  }
  auto angle_dma = [&](int tile_unclamped) __attribute__((always_inline)) {
    const unsigned cs_base = (unsigned)min(tile_unclamped, last_tile) * (unsigned)a.rope_tile_stride;
    const unsigned m0 = __builtin_amdgcn_readfirstlane(lds_base + (unsigned)(kCsRing + (tile_unclamped % kCsBufs) * kRopeTileBytes));
#pragma unroll
    for (int y = 0; y < kCsPerWave; ++y) {
      const unsigned voff = cs_base + dma_cs_off[y];
      const unsigned m0v = m0 + (unsigned)((wave * kCsPerWave + y) * 1024);
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" :: "s"(m0v), "v"(voff), "s"(rope_base_u) : "memory");
    }
  };

  // ---- latent tiles: through registers, rounded to E4M3 on the way (rows past the last attendable one re-read it)
  int st_row[kPass], st_col[kPass];
#pragma unroll
  for (int p = 0; p < kPass; ++p) {
    const int id = min(p * 256 + tid, kChunks - 1);             // surplus threads repeat the last chunk
    st_row[p] = id / kCpr;
    st_col[p] = id - st_row[p] * kCpr;
  }
  uint4v stage[kPass];
  auto latent_loads = [&](int tile_unclamped) __attribute__((always_inline)) {
    const int r0 = min(tile_unclamped, last_tile) * kTile;
#pragma unroll
    for (int p = 0; p < kPass; ++p) {
      const unsigned rel = (unsigned)min(r0 + st_row[p], rel_last);
      stage[p] = *reinterpret_cast<const uint4v*>(hk_base + (size_t)rel * row_bytes + (unsigned)st_col[p] * 16u);
    }
  };
  auto latent_store = [&](int tile) __attribute__((always_inline)) {
    unsigned char* base = lds + (size_t)(tile % kBufs) * kTileB;
#pragma unroll
    for (int p = 0; p < kPass; ++p) {
      float f[8];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        f[2 * e] = F16::to_float((uint16_t)(stage[p][e] & 0xffffu));
        f[2 * e + 1] = F16::to_float((uint16_t)(stage[p][e] >> 16));
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) f[e] = __builtin_amdgcn_fmed3f(f[e], -448.f, 448.f);
      uint2v pk;
      pk.x = cvt2_e4m3(f[0], f[1]) | (cvt2_e4m3(f[2], f[3]) << 16);
      pk.y = cvt2_e4m3(f[4], f[5]) | (cvt2_e4m3(f[6], f[7]) << 16);
      if (p * 256 + tid < kChunks) *reinterpret_cast<uint2v*>(base + st_row[p] * kRowB + st_col[p] * 8) = pk;
    }
  };

  // ---- this wavefront's head
  const bool active = wave < u.nh;
  const int hc = u.h0 + (active ? wave : 0);                    // idle wavefronts mirror head h0
  const int g_rel = G == 1 ? 0 : (u.s == 1 ? (hc - u.head_off0) : ((hc - u.head_off0) >> 1));
  const int u_in_g = hc - u.head_off0 - g_rel * u.s;
  const int kbase_b = g_rel * kRank;                            // the head's first column inside the tile row, bytes

  latent_loads(0);
  angle_dma(0);
  angle_dma(1);
  uint16_t q_raw[4][2];
  float q_rev[4][2], w_sc[4][2];
  int q_position;
  {
    Meta mq;
    mq.n_heads = a.n_heads; mq.qpk = a.m_qpk; mq.nq = a.m_nq;
    const uint16_t* qp = a.q + q_row(mq, b, hc) * kDHead;
    q_position = a.q_pos[b * a.m_nq + q_token(mq, hc)];
#pragma unroll
    for (int pb = 0; pb < 4; ++pb) {
      const int f = 16 * pb + n16;
      q_raw[pb][0] = qp[f];
      q_raw[pb][1] = qp[f + kHalf];
      q_rev[pb][0] = a.rev_hi[f];
      q_rev[pb][1] = a.rev_lo[f];
      w_sc[pb][0] = a.w_scale[(size_t)hc * kDHead + f];
      w_sc[pb][1] = a.w_scale[(size_t)hc * kDHead + f + kHalf];
    }
  }
  // stationary operand: W[ks][ct]: the k of lane group kq of k-step ks (8 or 32 rows), feature 16 ct + n16
  Frag W[NS][8];
  {
    const unsigned char* mf = reinterpret_cast<const unsigned char*>(a.mfold) + u.bk_off0 + ((size_t)g_rel * u.s + u_in_g) * (size_t)(kRank * kDHead);
#pragma unroll
    for (int ks = 0; ks < NS; ++ks)
#pragma unroll
      for (int ct = 0; ct < 8; ++ct) W[ks][ct] = *reinterpret_cast<const Frag*>(mf + ((size_t)(ks * 8 + ct) * 64 + lane) * sizeof(Frag));
  }

  // A operand of k-step ks of sub-tile tt: token 16 tt + n16, the same k of the head's columns (bytes of its LDS row)
  int a_off[2];
#pragma unroll
  for (int tt = 0; tt < 2; ++tt) a_off[tt] = (16 * tt + n16) * kRowB + kbase_b + kq * (int)sizeof(Frag);
  auto a_ptr = [&](const unsigned char* tile, int tt, int ks) __attribute__((always_inline)) {
    return reinterpret_cast<const Frag*>(tile + a_off[tt] + ks * kStepB);
  };
  auto tile_of = [&](int tile) __attribute__((always_inline)) { return lds + (size_t)(tile % kBufs) * kTileB; };
  auto angle_piece = [&](const unsigned char* cst, int pb, int piece) __attribute__((always_inline)) {
    return *reinterpret_cast<const float4v*>(cst + (16 * pb + n16) * 256 + (((unsigned)(piece + kq) ^ (unsigned)n16) * 16u));
  };
  auto angle_tile = [&](int tile) __attribute__((always_inline)) { return lds + kCsRing + (size_t)(tile % kCsBufs) * kRopeTileBytes; };

  float* out_row = a.scores + ((size_t)u.part0 * a.batch + b) * a.n_heads * (size_t)a.lpad + (size_t)hc * a.lpad + t_begin;
  const int tok_of_lane = 4 * kq + 2 * ((lane >> 2) & 1) + (lane & 1);

  // ---- start-up: everything requested so far has landed; tile 0 goes to LDS, tile 1 into the staging registers
  __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
  latent_store(0);
  latent_loads(1);
  __syncthreads();
  // the rotated query times log2(e) / sqrt(d_h) and the column scales: factors of k_f (x0, y0) and of k_{f+64} (x1, y1):
  //   score += K8_f (c x0 + s y0) + K8_{f+64} (c x1 + s y1)
  float x0[4], y0[4], x1[4], y1[4];
  {
    const float pos = (float)q_position;
#pragma unroll
    for (int pb = 0; pb < 4; ++pb) {
      const float r0 = T::to_float(q_raw[pb][0]), r1 = T::to_float(q_raw[pb][1]);
      const float ph = pos * q_rev[pb][0];
      const float pe = fmaf(pos, q_rev[pb][0], -ph);
      const float rev = (ph - floorf(ph)) + (pe + pos * q_rev[pb][1]);
      const float sn = __builtin_amdgcn_sinf(rev), cn = __builtin_amdgcn_cosf(rev);
      const float qa = (r0 * cn - r1 * sn) * a.scale, qb = (r1 * cn + r0 * sn) * a.scale;
      x0[pb] = qa * w_sc[pb][0];
      y0[pb] = qb * w_sc[pb][0];
      x1[pb] = qb * w_sc[pb][1];
      y1[pb] = -qa * w_sc[pb][1];
    }
  }

  float4v acc[2][8];
  Frag af[3], an[2];

  auto half_item = [&](const float4v (&ac)[8], float (&part)[4], int e2, const float4v& c, const float4v& s)
      __attribute__((always_inline)) {
    const int pb = e2 >> 3, j = (e2 >> 1) & 3, h2 = e2 & 1;
    const float coef = h2 == 0 ? fmaf(s[j], y0[pb], c[j] * x0[pb]) : fmaf(s[j], y1[pb], c[j] * x1[pb]);
    part[j] = fmaf(ac[pb + 4 * h2][j], coef, part[j]);
  };
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
  auto finish = [&](const float4v (&ac)[8], int tile, int tt) __attribute__((always_inline)) {
    const unsigned char* cst = angle_tile(tile);
    float part[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int pb = 0; pb < 4; ++pb) {
      const float4v c = angle_piece(cst, pb, 4 * tt), s = angle_piece(cst, pb, 8 + 4 * tt);
#pragma unroll
      for (int x = 0; x < 8; ++x) half_item(ac, part, 8 * pb + x, c, s);
    }
    out_row[tile * kTile + 16 * tt + tok_of_lane] = sum_quad_over_row(part, lane);
  };

  // Sub-tile tt of tile k, as in score16_kernel.  The tile hand-over (second sub-tile, before k-step kHandK):
  // everything this wavefront requested has landed (tile k+1's latents in the staging registers, its
  // angles in LDS); the latents go to LDS rounded (buffer (k+1) % 3: its previous tile, k-2, was finished
  // by every wavefront before the previous barrier); one barrier; tile k+2 is requested.
  constexpr int kSumSlot0 = kMfmas - 5;
  constexpr int kItemSlots = kMfmas * 3 / 4 < kSumSlot0 ? kMfmas * 3 / 4 : kSumSlot0;
  constexpr int kHandK = NS >= 4 ? NS / 2 : 0;
  auto body = [&](auto tt_c, int k, bool have_prev) __attribute__((always_inline)) {
    constexpr int tt = decltype(tt_c)::value;
    const unsigned char* hrow = tile_of(k);
    const unsigned char* hnext = tile_of(tt == 0 ? k : k + 1);
    const int ptile = tt == 0 ? k - 1 : k;
    constexpr int ptt = 1 - tt;
    const unsigned char* cst = angle_tile(have_prev ? ptile : k);
    float part[4] = {0.f, 0.f, 0.f, 0.f};
    float4v csr[2][2];
    RowSum rs;
    if (have_prev) {
      csr[0][0] = angle_piece(cst, 0, 4 * ptt);
      csr[0][1] = angle_piece(cst, 0, 8 + 4 * ptt);
    }
#pragma unroll
    for (int ks = 0; ks < NS; ++ks) {
      if (tt == 1 && ks == kHandK) {
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
        latent_store(k + 1);
        __syncthreads();
        latent_loads(k + 2);
        angle_dma(k + 2);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (ks + 2 < NS) af[(ks + 2) % 3] = *a_ptr(hrow, tt, ks + 2);
      else an[ks + 2 - NS] = *a_ptr(hnext, 1 - tt, ks + 2 - NS);
      const Frag afrag = af[ks % 3];
#pragma unroll
      for (int ct = 0; ct < 8; ++ct) {
        const int mi = ks * 8 + ct;
        float4v prev;
        if (ks == 0) prev = float4v{0.f, 0.f, 0.f, 0.f};
        else prev = acc[tt][ct];
        if constexpr (kWide) acc[tt][ct] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(afrag, W[ks][ct], prev, 0, 0, 0, 0, 0, 0);
        else acc[tt][ct] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(afrag, W[ks][ct], prev, 0, 0, 0);
        if (have_prev) {
          if (mi < kItemSlots) {
#pragma unroll
            for (int e2 = mi * 32 / kItemSlots; e2 < (mi + 1) * 32 / kItemSlots; ++e2) {
              const int pb = e2 >> 3;
              if ((e2 & 7) == 0 && pb + 1 < 4) {
                csr[(pb + 1) & 1][0] = angle_piece(cst, pb + 1, 4 * ptt);
                csr[(pb + 1) & 1][1] = angle_piece(cst, pb + 1, 8 + 4 * ptt);
              }
              half_item(acc[ptt], part, e2, csr[pb & 1][0], csr[pb & 1][1]);
            }
          } else if (mi >= kSumSlot0 && mi < kSumSlot0 + 4) {
            row_sum_step(rs, part, mi - kSumSlot0);
          } else if (mi == kSumSlot0 + 4) {
            out_row[ptile * kTile + 16 * ptt + tok_of_lane] = rs.v;
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    af[0] = an[0];
    af[1] = an[1];
  };

  af[0] = *a_ptr(tile_of(0), 0, 0);
  af[1] = *a_ptr(tile_of(0), 0, 1);
  for (int k = 0; k < n_tiles; ++k) {
    body(std::integral_constant<int, 0>{}, k, k > 0);
    body(std::integral_constant<int, 1>{}, k, true);
  }
  finish(acc[1], last_tile, 1);
  __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));     // no LDS-direct load may outlive the workgroup's LDS allocation
}

}  // namespace palu
