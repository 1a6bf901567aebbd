// Softmax partials and the value contraction in latent space on the matrix cores
// (Eq. 4: softmax(q K^T) (H_v B_v) evaluated as (p H_v) B_v; Sec. 3.1.1):
//   per (sequence, split of the sequence, unit of heads x latent columns)
//     p_t = exp2(score_t - m),  l = sum_t p_t,  o[c] = sum_t p_t H_v[t, c].
//
// One wavefront owns one split and shares nothing with the others: no workgroup
// barrier anywhere.  It walks its tokens in sets of 32 with an online softmax
// (running maximum m, accumulators rescaled when m grows) and contracts each
// set with v_mfma_f32_16x16x32_f16: A = probabilities (rows = heads, k = tokens),
// B = latents (k = tokens, columns = latent channels).  The cache is token-major,
// so a 16-byte load brings 8 channels of one token, while the matrix cores want
// 8 tokens of one channel per lane: each lane loads the same 8-channel chunk of
// 8 consecutive tokens and transposes the 8x8 block in registers with byte
// permutes (one per operand register); channel e of every chunk then forms the
// B operand of the e-th of 8 accumulator sets.  The vector ALU only does the
// softmax (a few operations per token and head) and the transposes, so the
// kernel stays bound by the latent stream for every head-group size (a latent
// shared by all 32 heads goes in two blocks of 16 heads, side by side in a
// workgroup, so that the second read of a row comes from the cache).
//
// 4-bit latents: while transposing, a code c is masked in place into the low mantissa bits of an fp16 zero,
// i.e. becomes the subnormal number c 2^-24 (codes in bits 0 .. 3) or c 2^-20 (bits 4 .. 7): the matrix cores
// take subnormal fp16 operands exactly, so one AND per operand register (and one shift per four) dequantizes.
// The per-(token, 128-channel block) scale is folded into the probabilities (one probability tile per block,
// a = p s), the power of two into the write-out, and the zero-points into one scalar per (head, block):
// sum_t a (c - z) = 2^24 sum_t a (c 2^-24) - sum_t a z.
//
// The running maximum is lazy: it only rises (and the accumulators are only rescaled) when a set's maximum
// exceeds it by more than 8 (scores are base-2 logarithms), so probabilities reach 256 at most; the (max, sum)
// pair a split reports is consistent with its accumulators, which is all the combination needs.

#include "palu_dev.h"

#ifndef PALU_PV_PAIR_DEPTH
#define PALU_PV_PAIR_DEPTH 2
#endif

namespace palu {

struct PvUnit {
  int32_t c0;         // first column of the value-latent row
  uint16_t h0;        // first head
  uint16_t ncols;     // columns (multiple of 32, at most 128 * NG)
  uint8_t nh;         // heads (at most 16 in the built forms); a head only keeps the columns of its own group
  uint8_t write_ml;   // this unit stores the (max, sum) pair of its heads
};
constexpr int kMaxPvUnits = 128;
struct PvUnits {
  int n_units;
  PvUnit u[kMaxPvUnits];
};

struct PvArgs {
  const void* hv;
  const uint16_t* hv_scale;
  const uint16_t* hv_zero;
  const float* scores;       // [parts][batch][n_heads][lpad]; planes 0 and 1 are read
  const int32_t* seq_lens;
  const int32_t* q_len;      // several queries per sequence: rows attended by query j of sequence b at [b * nq + j]; or NULL
  float* o_part;             // [batch][n_split][o_stride]
  float* ml_part;            // [batch][n_split][n_heads][2]
  long long row_elems;       // R_v
  long long max_seq;
  long long part_stride;
  int seq_len;
  int lpad;
  int batch;
  int split_tokens;          // tokens per wavefront (multiple of 32)
  int n_split;
  int o_stride;
  int n_blocks_q;
  int units_per_wg;          // 1, 2 or 4: the wavefronts of a workgroup take this many units of the same splits
  uint8_t n_parts[PALU_MAX_HEADS];   // 1 or 2 score planes per head
  Meta meta;
  PvUnits units;
};

struct PlaneSumArgs {
  float* scores;
  long long part_stride;
  int lpad;
  int seq_len;
  int n_heads;
  uint8_t n_parts[PALU_MAX_HEADS];
};

// scores[0] += scores[1] + ... + scores[n_parts-1] for heads with more than two
// partial planes (ranks contracted in slices); the value kernel then reads one.
__global__ __launch_bounds__(256) void plane_sum_kernel(PlaneSumArgs a) {
  const int h = blockIdx.y, b = blockIdx.z;
  const int np = a.n_parts[h];
  if (np <= 2) return;
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t >= a.seq_len) return;
  float* p = a.scores + ((size_t)b * a.n_heads + h) * a.lpad + t;
  float s = p[0];
  for (int pl = 1; pl < np; ++pl) s += p[(size_t)pl * a.part_stride];
  p[0] = s;
}

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}
// lane ^ 16 inside each half of the wavefront
__device__ __forceinline__ float swap16(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v), 0x401F));
}
// Maximum over the 32 lanes of a wavefront half; the result is in all 32 lanes.  The numbers (no NaN among
// them) are compared as integers of the same order (negative floats have their low 31 bits inverted): an
// integer maximum with its lane move is one instruction, where fmaxf() of a moved float takes four (the move
// and its initial value, and one per operand to quiet signalling NaNs).
__device__ __forceinline__ int float_order(int b) { return b ^ ((b >> 31) & 0x7fffffff); }     // its own inverse
template <int CTRL>
__device__ __forceinline__ int dpp_peek(int v) {          // every lane has a source lane under these controls: no old value to keep
  return __builtin_amdgcn_update_dpp((int)0x80000000, v, CTRL, 0xf, 0xf, false);
}
__device__ __forceinline__ float half_wave_max(float f) {
  int v = float_order(__builtin_bit_cast(int, f));
  v = max(v, dpp_peek<0xB1>(v));      // quad_perm [1,0,3,2]
  v = max(v, dpp_peek<0x4E>(v));      // quad_perm [2,3,0,1]
  v = max(v, dpp_peek<0x141>(v));     // row_half_mirror
  v = max(v, dpp_peek<0x140>(v));     // row_mirror
  v = max(v, __builtin_amdgcn_ds_swizzle(v, 0x401F));
  return __builtin_bit_cast(float, float_order(v));
}
__device__ __forceinline__ float half_wave_sum(float v) {
  v += dpp_move<0xB1>(v);
  v += dpp_move<0x4E>(v);
  v += dpp_move<0x141>(v);
  v += dpp_move<0x140>(v);
  return v + swap16(v);
}

// LDS written by some lanes of this wavefront is read by others: the hardware keeps
// a wavefront's LDS operations in order, this keeps the compiler from moving them
__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

// T:  storage type of unquantized latents (bfloat16 is converted to fp16 in registers: exact in the fp16 range)
// HS: score slots per lane: the unit has at most 2*HS heads (built: 2 and 8; above 8 the code takes two 16-row tiles)
// NG: 128-column blocks per unit (16 lanes x 8 channels each)
// QB: latents are QB-bit codes (4, 3 or 2; 0: unquantized); every 128-column block of the unit is one
//     quantization block.  In the body I4 = "quantized": 3- and 2-bit codes are spread into the
//     4-bit register layout when they are consumed and then follow the 4-bit arithmetic.
// TWO: some head of the launch has two score planes (the kernel then requests both planes of every head; with one
//     plane everywhere the second request, an instruction per head slot and set, is left out)
template <typename T, int HS, int NG, int QB, bool TWO>
__global__ __launch_bounds__(256, (QB != 0 && HS <= 2) ? 2 : 1) void pv_kernel(PvArgs a) {
  constexpr bool I4 = QB != 0;
  constexpr bool kIsBf16 = !__is_same(T, F16);
  constexpr int MT = HS > 8 ? 2 : 1;
  constexpr int NA = I4 ? NG : 1;                  // scaled probabilities: one set per quantization block
  // Quantized latents, four heads, two blocks: a lane takes two neighbouring 8-channel chunks with one load (8 bytes
  // of 4-bit codes: a load instruction then covers whole 128-byte rows; 4 bytes of 2-bit fields, plus 2 bytes of
  // third bits), and a set needs half the requests.  The chunks of lanes
  // n < 8 lie in block 0 and those of lanes n >= 8 in block 1, so one matrix instruction serves both blocks:
  // the probability tile has rows (block, head) - 8 of its 16 - and a lane keeps the rows of its own block.
  constexpr bool kPair = I4 && NG == 2 && HS == 2;
  constexpr int NT = kPair ? 1 : NA;               // probability tiles
  constexpr int kPitch = 40;                       // halfs per head row: 80-byte pitch, 16-byte reads of 16 rows hit distinct banks
  __shared__ __attribute__((aligned(16))) _Float16 p_lds[4][NT][MT * 16 * kPitch];
  __shared__ __attribute__((aligned(16))) float x_lds[4][MT * 16 * NA];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n = lane & 15, kq = lane >> 4;         // matrix-core roles: column (B, D) or head row (A); token quarter
  const int tl = lane & 31, hp = lane >> 5;        // softmax roles: token of the set; head parity
  const Meta& m = a.meta;

  // grid (groups of units_per_wg units, groups of 4 / units_per_wg splits, batch); the wavefronts of a
  // workgroup take neighbouring units of the same split first: they read neighbouring columns of the same
  // rows, and the scales and zero-points of a token's blocks, which lie side by side, come into this
  // compute unit's cache once instead of once per unit.
  const int upw = a.units_per_wg;
  const int unit = blockIdx.x * upw + (wave & (upw - 1)), b = blockIdx.z;
  const int split = blockIdx.y * (4 / upw) + wave / upw;
  if (unit >= a.units.n_units) return;             // whole wavefront; nothing below synchronises wavefronts
  const int L = a.seq_lens ? min(a.seq_lens[b], a.seq_len) : a.seq_len;
  const int s0 = split * a.split_tokens;
  if (split >= a.n_split || s0 >= L) return;       // whole wavefront; nothing below synchronises wavefronts
  const int ntok = min(a.split_tokens, L - s0);
  const int n_sets = (ntok + 31) >> 5;
  const int last = ntok - 1;

  const PvUnit u = a.units.u[unit];
  asm volatile("" :: "s"(a.hv), "s"(a.scores), "s"(a.seq_lens), "s"(a.o_part), "s"(a.ml_part), "s"(a.row_elems), "s"(a.max_seq),
               "s"(a.part_stride), "s"(a.seq_len), "s"(a.lpad), "s"(a.split_tokens), "s"(a.n_split), "s"(a.o_stride),
               "s"(u.c0), "s"((int)u.h0), "s"((int)u.ncols), "s"((int)u.nh));      // all in registers here: one round trip
  const int h0 = u.h0, nh = u.nh, c0 = u.c0;
  const int lpt = u.ncols >> 3;                    // 8-channel chunks per row of the unit

  const size_t row0 = (size_t)b * a.max_seq + s0;
  // quantized latents: 4-bit codes, or 2-bit fields followed (3 bits) by a plane of third bits at R/4 bytes
  constexpr int bits = I4 ? QB : 16;
  const unsigned row_bytes = (unsigned)a.row_elems * (unsigned)bits / 8u;
  const unsigned char* base = (const unsigned char*)a.hv + row0 * row_bytes + (I4 ? (bits == 4 ? c0 / 2 : c0 / 4) : c0 * 2);
  const unsigned hi_plane = (unsigned)a.row_elems / 4u + (unsigned)c0 / 8u - (unsigned)c0 / 4u;   // from `base` to the third bits
  unsigned coff[NG];
#pragma unroll
  for (int ng = 0; ng < NG; ++ng) coff[ng] = (unsigned)min(ng * 16 + n, lpt - 1) * (I4 ? (bits == 4 ? 4u : 2u) : 16u);
  if constexpr (kPair) coff[0] = (unsigned)min(n, (lpt >> 1) - 1) * (bits == 4 ? 8u : 4u);      // chunks 2n and 2n + 1 (a unit has a multiple of 4 chunks)
  // byte offset of the row of the lane's token j in set 0; a set further on is 32 rows further, clamped to the last row
  unsigned roff[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) roff[j] = (unsigned)(8 * kq + j) * row_bytes;
  const unsigned last_off = (unsigned)last * row_bytes, set_bytes = 32u * row_bytes;

  const float* sc_ptr[HS];
  bool two[HS];
  int lim[HS];                                     // tokens of this split the head's query attends (its own row limit)
#pragma unroll
  for (int i = 0; i < HS; ++i) {
    const int h = h0 + min(hp + 2 * i, nh - 1);
    sc_ptr[i] = a.scores + ((size_t)b * m.n_heads + h) * a.lpad + s0;
    two[i] = a.n_parts[h] > 1;
    lim[i] = a.q_len ? a.q_len[b * m.nq + q_token(m, h)] - s0 : 0x7fffffff;
  }
  const size_t sz_idx0 = I4 ? row0 * a.n_blocks_q + (c0 >> 7) : 0;
  const int n_blk = (u.ncols + 127) >> 7;          // 128-column blocks the unit really has

  struct Blk {
    uint32_t h[8][I4 ? (QB == 3 ? 2 : 1) : 4];     // [token j of the lane's quarter][dword]; quantized: codes, third bits (3-bit only)
  };
  struct Set {
    Blk blk[NG];
    float sc[HS][TWO ? 2 : 1];
    uint16_t sz[NA];                               // quantized: scales (lanes 0 .. 31) or zero-points (32 .. 63) of the lane's softmax token, as loaded
  };

  // every load is unconditional and in bounds (clamped to the last token / chunk / head);
  // what a clamped load returns is given zero weight or never stored
  auto issue = [&](Set& st, int k) {
    const int tb = k * 32;
#pragma unroll
    for (int ng = 0; ng < (kPair ? 1 : NG); ++ng) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const unsigned char* p = base + (size_t)(min(roff[j] + (unsigned)k * set_bytes, last_off) + coff[ng]);
        if constexpr (kPair && bits == 4) {
          const uint2v v = *reinterpret_cast<const uint2v*>(p);
          st.blk[0].h[j][0] = v.x;
          st.blk[1].h[j][0] = v.y;
        } else if constexpr (kPair) {
          const uint32_t v = *reinterpret_cast<const uint32_t*>(p);                 // two chunks' two-bit fields
          st.blk[0].h[j][0] = v;
          st.blk[1].h[j][0] = v >> 16;
          if constexpr (QB == 3) {
            const uint32_t pl = *reinterpret_cast<const uint16_t*>(p + hi_plane - (coff[0] >> 1));   // their two bytes of third bits
            st.blk[0].h[j][1] = pl;
            st.blk[1].h[j][1] = pl >> 8;
          }
        } else if constexpr (I4) {
          if constexpr (bits == 4) {
            st.blk[ng].h[j][0] = *reinterpret_cast<const uint32_t*>(p);
          } else {
            st.blk[ng].h[j][0] = *reinterpret_cast<const uint16_t*>(p);
            if constexpr (QB == 3) st.blk[ng].h[j][1] = p[hi_plane - (coff[ng] >> 1)];      // the chunk's byte of the third-bit plane
          }
        } else {
          const uint4v v = *reinterpret_cast<const uint4v*>(p);
          st.blk[ng].h[j][0] = v.x; st.blk[ng].h[j][1] = v.y; st.blk[ng].h[j][2] = v.z; st.blk[ng].h[j][3] = v.w;
        }
      }
    }
    const int ts = min(tb + tl, last);
#pragma unroll
    for (int i = 0; i < HS; ++i) {
      st.sc[i][0] = sc_ptr[i][ts];
      if constexpr (TWO) st.sc[i][1] = sc_ptr[i][ts + a.part_stride];
    }
    if constexpr (I4) {
      // the two lanes of a token split its scales and zero-points (2-byte requests cost the memory pipeline as much
      // as the 8-byte latent ones) and swap them in process()
      const uint16_t* arr = hp ? a.hv_zero : a.hv_scale;
#pragma unroll
      for (int ng = 0; ng < NG; ++ng)
        st.sz[ng] = arr[sz_idx0 + (size_t)ts * a.n_blocks_q + min(ng, n_blk - 1)];     // a narrow unit's idle block re-reads block 0
    }
  };

  constexpr float kLazy = 8.f;
  float mx[HS], lsum[HS], lz[HS][NA];
#pragma unroll
  for (int i = 0; i < HS; ++i) {
    mx[i] = -INFINITY;
    lsum[i] = 0.f;
#pragma unroll
    for (int g = 0; g < NA; ++g) lz[i][g] = 0.f;
  }
  float4v acc[MT][NG][8];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int ng = 0; ng < NG; ++ng)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[mt][ng][e] = float4v{0.f, 0.f, 0.f, 0.f};

  _Float16* pw = &p_lds[wave][0][0];
  float* xw = &x_lds[wave][0];

  auto process = [&](Set& st, int k) {
    const bool tok_ok = k * 32 + tl < ntok;
    // ---- online softmax statistics of the 32 tokens
    float s[HS], bm[HS];
    bool grew = false;
    // lazy maximum: probabilities up to 2^kLazy.  Quantized latents carry the scale in the fp16 weights a = p s:
    // with a scale above 128 somewhere in the set the maximum is exact (p <= 1) and a stays in range as before.
    float lazy = kLazy;
    uint16_t qs[NA], qz[NA];                                   // scales and zero-points of the lane's token
    if constexpr (I4) {
      uint32_t own = st.sz[0];
      if constexpr (NA > 1) own |= (uint32_t)st.sz[1] << 16;
      const uint32_t other = (uint32_t)__builtin_amdgcn_ds_bpermute((lane ^ 32) * 4, (int)own);
      const uint32_t sv = hp ? other : own, zv = hp ? own : other;
      bool big = false;
#pragma unroll
      for (int g = 0; g < NA; ++g) {
        qs[g] = (uint16_t)(sv >> (16 * g));
        qz[g] = (uint16_t)(zv >> (16 * g));
        big |= qs[g] > (uint16_t)0x5800;                       // fp16 bits of 128 (a negative or NaN scale also lands here)
      }
      if (__builtin_amdgcn_ballot_w64(big) != 0) lazy = 0.f;
    }
#pragma unroll
    for (int i = 0; i < HS; ++i) {
      float v = st.sc[i][0];
      if constexpr (TWO) v += two[i] ? st.sc[i][1] : 0.f;
      s[i] = (tok_ok && hp + 2 * i < nh && k * 32 + tl < lim[i]) ? v : -INFINITY;
      bm[i] = half_wave_max(s[i]);
      grew |= bm[i] > mx[i] + lazy;
    }
    if (__builtin_amdgcn_ballot_w64(grew) != 0) {             // uniform: some head's running maximum rises
#pragma unroll
      for (int i = 0; i < HS; ++i) {
        const float mn = fmaxf(mx[i], bm[i]);
        const float al = mx[i] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mx[i] - mn);
        mx[i] = mn;
        lsum[i] *= al;
#pragma unroll
        for (int g = 0; g < NA; ++g) lz[i][g] *= al;
        if (tl == 0) {
          xw[hp + 2 * i] = al;
          if constexpr (kPair) xw[4 + hp + 2 * i] = al;       // rows 4 .. 7: the same heads under block 1
        }
      }
      wave_lds_fence();
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const float4v al = *reinterpret_cast<const float4v*>(xw + mt * 16 + 4 * kq);   // accumulator rows 4*kq + 0..3
#pragma unroll
        for (int ng = 0; ng < NG; ++ng)
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[mt][ng][e] *= al;
      }
      wave_lds_fence();
    }
#pragma unroll
    for (int i = 0; i < HS; ++i) {
      const float p = s[i] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(s[i] - mx[i]);
      const int slot = (hp + 2 * i) * kPitch + tl;
      if constexpr (!I4) {
        const _Float16 ph = (_Float16)p;
        lsum[i] += (float)ph;                                  // the weights that enter the contraction
        pw[slot] = ph;
      } else {
        lsum[i] += p;
#pragma unroll
        for (int g = 0; g < NA; ++g) {
          const float sc = F16::to_float(qs[g]);
          const float zp = F16::to_float(qz[g]);
          const _Float16 ah = (_Float16)(p * sc);
          lz[i][g] = fmaf((float)ah, zp, lz[i][g]);
          pw[kPair ? slot + g * 4 * kPitch : g * (MT * 16 * kPitch) + slot] = ah;
        }
      }
    }
    wave_lds_fence();
    half8 pa[NT][MT];
#pragma unroll
    for (int g = 0; g < NT; ++g)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        pa[g][mt] = *reinterpret_cast<const half8*>(pw + g * (MT * 16 * kPitch) + (mt * 16 + n) * kPitch + 8 * kq);
    wave_lds_fence();

    // ---- transposed latents as B operands, 8 accumulator sets per 128-column block
#pragma unroll
    for (int ng = 0; ng < NG; ++ng) {
      const Blk& bl = st.blk[ng];
      uint32_t o[8][4];                                        // [channel e of the chunk][token pair]
#pragma unroll
      for (int jp = 0; jp < 4; ++jp) {
        if constexpr (!I4) {
#pragma unroll
          for (int d = 0; d < 4; ++d) {
            // perm(hi_src, lo_src, sel): selector bytes 0-3 pick from lo_src, 4-7 from hi_src
            uint32_t lo = __builtin_amdgcn_perm(bl.h[2 * jp + 1][d], bl.h[2 * jp][d], 0x05040100u);
            uint32_t hi = __builtin_amdgcn_perm(bl.h[2 * jp + 1][d], bl.h[2 * jp][d], 0x07060302u);
            if constexpr (kIsBf16) {
              lo = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(__builtin_bit_cast(float, lo << 16),
                                                                           __builtin_bit_cast(float, lo & 0xffff0000u)));
              hi = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(__builtin_bit_cast(float, hi << 16),
                                                                           __builtin_bit_cast(float, hi & 0xffff0000u)));
            }
            o[2 * d][jp] = lo;
            o[2 * d + 1][jp] = hi;
          }
        } else {
          uint32_t ca = bl.h[2 * jp][0], cb = bl.h[2 * jp + 1][0];
          if constexpr (bits != 4) {
            ca = expand_low_bits(ca, bl.h[2 * jp][QB == 3 ? 1 : 0], QB == 3);
            cb = expand_low_bits(cb, bl.h[2 * jp + 1][QB == 3 ? 1 : 0], QB == 3);
          }
          // Four channels of both tokens side by side (token a's 16 bits of codes below token b's): the codes of
          // channel u of the two tokens are then 16 bits apart, i.e. in the two halves of one operand register.
          // Masked in place they are the subnormal fp16 numbers c 2^-24 (channels 0 and 2 of the four, after a
          // shift by 8 for the latter) and c 2^-20 (channels 1 and 3); the powers of two are undone at the write-out.
#pragma unroll
          for (int half = 0; half < 2; ++half) {
            const uint32_t x = __builtin_amdgcn_perm(cb, ca, half ? 0x07060302u : 0x05040100u), x8 = x >> 8;
            o[4 * half + 0][jp] = x & 0x000f000fu;
            o[4 * half + 1][jp] = x & 0x00f000f0u;
            o[4 * half + 2][jp] = x8 & 0x000f000fu;
            o[4 * half + 3][jp] = x8 & 0x00f000f0u;
          }
        }
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const uint4v bw = {o[e][0], o[e][1], o[e][2], o[e][3]};
        const half8 bop = __builtin_bit_cast(half8, bw);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          acc[mt][ng][e] = __builtin_amdgcn_mfma_f32_16x16x32_f16(pa[NT > 1 ? ng : 0][mt], bop, acc[mt][ng][e], 0, 0, 0);
      }
    }
  };

  // ---- kDepth register sets in turn: the loads of the next kDepth - 1 sets are in flight while one is
  // consumed.  Every request is unconditional (past the last set the clamped addresses re-read the last
  // token, and nothing consumes them): with a request under a branch the wait in front of process() would
  // have to cover both ways of reaching it, i.e. every load in flight, and nothing would be prefetched.
  // (Three and four sets for quantized latents, whose sets are a quarter of the bytes, measured 5 - 10 % slower,
  // and 2-bit codes take as long as 4-bit ones: that kernel is bound by its instruction stream, not by bytes in flight.)
  constexpr int kDepth = kPair ? PALU_PV_PAIR_DEPTH : 2;
  Set ring[kDepth];
#pragma unroll
  for (int d = 0; d < kDepth - 1; ++d) issue(ring[d], d);
  for (int k = 0; k < n_sets; k += kDepth) {
#pragma unroll
    for (int d = 0; d < kDepth; ++d) {
      issue(ring[(d + kDepth - 1) % kDepth], k + d + kDepth - 1);
      if (d == 0 || k + d < n_sets) process(ring[d], k + d);      // uniform
    }
  }

  // ---- results of the split
#pragma unroll
  for (int i = 0; i < HS; ++i) {
    const float ls = half_wave_sum(lsum[i]);
    const int hh = hp + 2 * i;
    if (tl == 0 && hh < nh && u.write_ml) {
      float* ml = a.ml_part + (((size_t)b * a.n_split + split) * m.n_heads + h0 + hh) * 2;
      ml[0] = mx[i];
      ml[1] = ls;
    }
    if constexpr (I4) {
#pragma unroll
      for (int g = 0; g < NA; ++g) {
        const float zs = half_wave_sum(lz[i][g]);
        if (tl == 0) xw[hh * NA + g] = zs;
      }
    }
  }
  if constexpr (I4) wave_lds_fence();

  float* op = a.o_part + ((size_t)b * a.n_split + split) * a.o_stride;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      if (kPair && kq != (n >> 3)) continue;                  // rows 4 kq + r: block kq's scale; the lane's chunks are in block n / 8
      const int hh = kPair ? r : mt * 16 + 4 * kq + r;        // accumulator row = head of the unit
      if (hh >= nh) continue;
      const int h = h0 + hh;
      const int j = group_of(m, h);
      const int lo = m.v_off[j], hi = m.v_off[j + 1];
      float* oh = op + o_head_off(m, h) - lo;
#pragma unroll
      for (int ng = 0; ng < NG; ++ng) {
        const int chunk = kPair ? 2 * n + ng : ng * 16 + n;
        const int col = c0 + chunk * 8;
        if (chunk >= lpt || col < lo || col >= hi) continue;   // a head keeps the columns of its own group
        // quantized: acc = sum a c 2^-24 (even channels of the chunk) or sum a c 2^-20 (odd), zt = sum a z
        const float zt = I4 ? xw[hh * NA + (kPair ? n >> 3 : ng)] : 0.f;
        const float g0 = I4 ? 16777216.f : 1.f, g1 = I4 ? 1048576.f : 1.f;
        float4v v0, v1;
        v0.x = fmaf(g0, acc[mt][ng][0][r], -zt); v0.y = fmaf(g1, acc[mt][ng][1][r], -zt);
        v0.z = fmaf(g0, acc[mt][ng][2][r], -zt); v0.w = fmaf(g1, acc[mt][ng][3][r], -zt);
        v1.x = fmaf(g0, acc[mt][ng][4][r], -zt); v1.y = fmaf(g1, acc[mt][ng][5][r], -zt);
        v1.z = fmaf(g0, acc[mt][ng][6][r], -zt); v1.w = fmaf(g1, acc[mt][ng][7][r], -zt);
        *reinterpret_cast<float4v*>(oh + col) = v0;
        *reinterpret_cast<float4v*>(oh + col + 4) = v1;
      }
    }
  }
}

#define PALU_PV_INST2(T, I4, TWO)                                      \
  template __global__ void pv_kernel<T, 2, 1, I4, TWO>(PvArgs);         \
  template __global__ void pv_kernel<T, 2, 2, I4, TWO>(PvArgs);         \
  template __global__ void pv_kernel<T, 8, 1, I4, TWO>(PvArgs);         \
  template __global__ void pv_kernel<T, 8, 2, I4, TWO>(PvArgs);
#define PALU_PV_INST(T, I4) PALU_PV_INST2(T, I4, true) PALU_PV_INST2(T, I4, false)
PALU_PV_INST(F16, 0)
PALU_PV_INST(BF16, 0)
PALU_PV_INST(F16, 4)
PALU_PV_INST(F16, 3)
PALU_PV_INST(F16, 2)

}  // namespace palu
