// Fused key reconstruction + RoPE + query product (Sec. 3.1.2, Appendix B):
//   score[b,i,t] = RoPE(q_i) . RoPE(H_k[b,t] B_k)_i * log2(e)/sqrt(d_h)
// computed as the contraction H_k . M_i on the matrix cores, where M_i is the
// query-folded reconstruction matrix (see rope_fold.hip), followed by one
// cos/sin-weighted sum per position in registers.  Reconstructed keys exist
// only as MFMA accumulators.
//
// Design for gfx950 (not the paper's one-thread-block-per-tile Triton layout):
//   * weight-stationary: each wavefront keeps its head's whole M_i (r x 128
//     fp16, up to 256 registers) resident for the lifetime of the workgroup, so
//     the only operand that moves per token tile is the latent tile;
//   * a workgroup = 4 wavefronts = up to 4 heads that read the same (or
//     adjacent) latent columns; it walks a chunk of the sequence in tiles of
//     32 tokens; each tile (and its 32 cos/sin rows) is fetched once with
//     coalesced 16-byte loads issued two tiles ahead, parked in registers, and
//     published through a double-buffered LDS tile;
//   * accumulators are computed transposed (features x tokens) so that the
//     sum over the 128 features of a token is an in-lane sum plus one
//     cross-half exchange.

#include "palu_dev.h"

namespace palu {

constexpr int kRowPad = 16;                    // bytes of padding per LDS row: keeps 16-byte column reads conflict-free
constexpr int kRopeRowB = kDHead * 2 + kRowPad;  // LDS pitch of one cos/sin row

// T:    storage type of unquantized latents.  The contraction itself always
//       runs in fp16 with float32 accumulation: bfloat16 latents are converted
//       while they are staged (exact for magnitudes in [2^-14, 65504],
//       saturating above, truncating below), because a bfloat16 copy of the
//       folded weights alone would cost 2^-9 relative error per element, more
//       than the whole error budget.
// NKS:  k-steps of 16: the rank of every head in the workgroup is exactly 16*NKS
// RT:   32-row feature tiles per wavefront: 4 = a whole head, 2 = half a head
//       (two wavefronts per head, each writing its own partial score)
// G:    groups spanned by the workgroup's heads (1, 2 or 4 adjacent groups of
//       equal rank): the staged latent row is G*16*NKS columns wide
// I4:   latents are packed 4-bit codes with per-(token, block) scale and zero
template <typename T, int NKS, int RT, int G, bool I4>
__global__ __launch_bounds__(256, 1) void score_kernel(ScoreArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  constexpr bool kIsBf16 = !__is_same(T, F16);
  constexpr int kRank = NKS * 16;
  constexpr int kWidth = G * kRank;                             // staged columns per token
  static_assert(kWidth <= 512, "latent tile row too wide");
  constexpr int kCpr = kWidth / 8;                              // 16-byte chunks per tile row
  constexpr int kChunks = kTile * kCpr;                         // chunks per tile
  constexpr int kPass = (kChunks + 255) / 256;                  // staging loads per thread and tile
  constexpr int kRowB = kWidth * 2 + kRowPad;                   // LDS row pitch in bytes
  constexpr int kTileB = kTile * kRowB;                         // latent tile bytes
  constexpr int kBufB = kTileB + kTile * kRopeRowB;             // + its cos/sin rows

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);        // scalar: everything derived from it is uniform
  const int lane = tid & 63;
  const int lane_lo = lane & 31, lane_hi = lane >> 5;
  const Meta& m = a.meta;

  int wg = blockIdx.x;
  const int unit = wg % a.units.n_units;
  wg /= a.units.n_units;
  const int chunk = wg % a.n_chunks;
  const int b = wg / a.n_chunks;

  const int L = a.seq_lens ? min(a.seq_lens[b], a.seq_len) : a.seq_len;
  const int t_begin = chunk * a.chunk_tokens;
  if (t_begin >= L) return;                                   // uniform for the workgroup
  const int t_end = min(t_begin + a.chunk_tokens, L);
  const int n_tiles = (t_end - t_begin + kTile - 1) / kTile;

  // ---- which head / feature rows this wavefront owns
  const int h0 = a.units.h0[unit], nh = a.units.nh[unit];
  int head, rt0;
  if (RT == 4) { head = h0 + wave; rt0 = 0; }
  else         { head = h0 + (wave >> 1); rt0 = (wave & 1) * 2; }
  const bool active = head < h0 + nh;
  const int hc = active ? head : h0;                           // idle wavefronts mirror head h0 but never store
  const int j = m.group_of_head[hc];
  // first column of the latent row staged by the workgroup (the groups of heads h0 .. h0+nh-1)
  const int c_lo = m.k_off[m.group_of_head[h0]];
  const int kbase_b = (m.k_off[j] - c_lo) * 2;                 // this head's first column inside the tile row

  // ---- stationary operand: folded weights of (b, head), rows [32*rt0, 32*(rt0+RT))
  half8 W[NKS][RT];
  {
    const uint16_t* mf = a.mfold + (size_t)b * a.mfold_bstride + m.bk_off[j] +
                         (size_t)(hc - m.head_off[j]) * kRank * kDHead;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
      for (int rt = 0; rt < RT; ++rt)
        W[ks][rt] = *reinterpret_cast<const half8*>(mf + ((size_t)(ks * 4 + rt0 + rt) * 64 + lane) * 8);
  }

  // ---- staging geometry: chunk id = p*256 + tid -> (row, 16-byte column) of the tile
  // cos/sin rows: 16 chunks of 16 bytes per token, 512 chunks per tile, two per thread
  const int rope_row = tid >> 3, rope_col = (tid & 7) * 2;
  const size_t seq_base = (size_t)b * a.max_seq;

  struct Stage {
    uint4v h[kPass];
    uint4v cs[2];
  };
  Stage st[2];

  auto issue_loads = [&](Stage& s, int tile) {
    const int t0 = t_begin + tile * kTile;
    {
      const int t = min(t0 + rope_row, L - 1);
      int pos = a.k_pos ? a.k_pos[t] : t;
      pos = max(0, min(pos, a.rope_len - 1));
      const uint4v* rp = reinterpret_cast<const uint4v*>(a.rope + (size_t)pos * kDHead) + rope_col;
      s.cs[0] = rp[0];
      s.cs[1] = rp[1];
    }
#pragma unroll
    for (int p = 0; p < kPass; ++p) {
      const int id = min(p * 256 + tid, kChunks - 1);          // surplus threads repeat the last chunk
      const int rr = id / kCpr, col = id - rr * kCpr;
      const int t = min(t0 + rr, L - 1);
      if (!I4) {
        const uint16_t* src = (const uint16_t*)a.hk + (seq_base + t) * a.row_elems + c_lo + col * 8;
        s.h[p] = *reinterpret_cast<const uint4v*>(src);
      } else {
        const int c = c_lo + col * 8;
        const uint8_t* src = (const uint8_t*)a.hk + ((seq_base + t) * a.row_elems + c) / 2;
        const size_t sb = (seq_base + t) * a.n_blocks_q + c / a.quant_block;
        s.h[p].x = *reinterpret_cast<const uint32_t*>(src);
        s.h[p].y = (uint32_t)a.hk_scale[sb] | ((uint32_t)a.hk_zero[sb] << 16);
      }
    }
  };
  auto store_stage = [&](Stage& s, int buf) {
    unsigned char* base = lds + (size_t)buf * kBufB;
    *reinterpret_cast<uint4v*>(base + kTileB + rope_row * kRopeRowB + rope_col * 16) = s.cs[0];
    *reinterpret_cast<uint4v*>(base + kTileB + rope_row * kRopeRowB + rope_col * 16 + 16) = s.cs[1];
#pragma unroll
    for (int p = 0; p < kPass; ++p) {
      const int id = p * 256 + tid;
      const int rr = id / kCpr, col = id - rr * kCpr;
      uint4v v = s.h[p];
      if (I4) {            // dequantize: (code - zero) * scale in float32, one rounding to fp16
        const uint32_t codes = v.x;
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
      if (id < kChunks) *reinterpret_cast<uint4v*>(base + rr * kRowB + col * 16) = v;
    }
  };

  float* out_row = a.scores + ((size_t)(RT == 2 ? (wave & 1) : 0) * a.batch + b) * m.n_heads * (size_t)a.lpad +
                   (size_t)hc * a.lpad;

  auto compute_tile = [&](int tile) {
    const int t0 = t_begin + tile * kTile;
    const unsigned char* base = lds + (size_t)(tile & 1) * kBufB;
    const unsigned char* hrow = base + lane_lo * kRowB + kbase_b + lane_hi * 16;
    const unsigned char* crow = base + kTileB + lane_lo * kRopeRowB + (lane_hi * 64 + rt0 * 16) * 2;
    // B operand of k-step ks: 8 latent values of token lane_lo; fetched two steps ahead of its MFMAs
    constexpr int kAhead = 2;
    half8 hf[kAhead + 1];
#pragma unroll
    for (int x = 0; x < kAhead && x < NKS; ++x) hf[x] = *reinterpret_cast<const half8*>(hrow + x * 32);
    float16v acc[RT];
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      if (ks + kAhead < NKS)
        hf[(ks + kAhead) % (kAhead + 1)] = *reinterpret_cast<const half8*>(hrow + (ks + kAhead) * 32);
      const half8 hfrag = hf[ks % (kAhead + 1)];
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        if (ks == 0) {
          float16v zero;
#pragma unroll
          for (int i = 0; i < 16; ++i) zero[i] = 0.f;
          acc[rt] = F16::mfma(W[ks][rt], hfrag, zero);
        } else {
          acc[rt] = F16::mfma(W[ks][rt], hfrag, acc[rt]);
        }
      }
      __builtin_amdgcn_sched_barrier(0);        // keep the fetch-ahead order: nothing moves across a k-step
    }
    // RoPE-weighted feature sum: acc[rt][i] is feature 32*(rt0+rt) + mfma_row(i) of token lane_lo;
    // its cos/sin weight sits at slot lane_hi*64 + (rt0+rt)*16 + i of the token's table row.
    float part = 0.f;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      const half8 c0 = *reinterpret_cast<const half8*>(crow + rt * 32);
      const half8 c1 = *reinterpret_cast<const half8*>(crow + rt * 32 + 16);
#pragma unroll
      for (int i = 0; i < 8; ++i) part = fmaf(acc[rt][i], (float)c0[i], part);
#pragma unroll
      for (int i = 0; i < 8; ++i) part = fmaf(acc[rt][8 + i], (float)c1[i], part);
    }
    part += __shfl_xor(part, 32, 64);
    if (active && lane_hi == 0 && t0 + lane_lo < t_end) out_row[t0 + lane_lo] = part * a.scale;
  };

  // ---- pipeline: loads for tile i+2 are in flight while tile i is computed
  issue_loads(st[0], 0);
  if (n_tiles > 1) issue_loads(st[1], 1);
  store_stage(st[0], 0);
  __syncthreads();

  for (int tile = 0; tile < n_tiles; tile += 2) {
    // even tile: stage set 0 is free (tile was stored), set 1 holds tile+1
    if (tile + 2 < n_tiles) issue_loads(st[0], tile + 2);
    compute_tile(tile);
    if (tile + 1 < n_tiles) store_stage(st[1], 1);
    __syncthreads();
    if (tile + 1 >= n_tiles) break;
    // odd tile
    if (tile + 3 < n_tiles) issue_loads(st[1], tile + 3);
    compute_tile(tile + 1);
    if (tile + 2 < n_tiles) store_stage(st[0], 0);
    __syncthreads();
  }
}

}  // namespace palu
