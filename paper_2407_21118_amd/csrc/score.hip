// Fused key reconstruction + RoPE + query product (Sec. 3.1.2, Appendix B):
//   score[b,i,t] = RoPE(q_i) . RoPE(H_k[b,t] B_k)_i * log2(e)/sqrt(d_h)
// computed as the contraction H_k . M_i on the matrix cores, where M_i is the
// query-folded reconstruction matrix (see rope_fold.hip), followed by one
// cos/sin-weighted sum per position in registers.  Reconstructed keys exist
// only as MFMA accumulators.
//
// Design for gfx950 (not the paper's one-thread-block-per-tile Triton layout):
//   * weight-stationary: each wavefront keeps its head's whole M_i (r x 128
//     fp16, up to 256 VGPRs) in registers for the lifetime of the workgroup,
//     so the only operand that moves per token tile is the latent tile;
//   * a workgroup = 4 wavefronts = up to 4 heads that read the same (or
//     adjacent) latent columns; it walks a chunk of the sequence in tiles of
//     32 tokens, staging each tile once in LDS with coalesced 16-byte loads;
//   * accumulators are computed transposed (features x tokens) so that the
//     sum over the 128 features of a token is an in-lane sum plus one
//     cross-half exchange.

#include "palu_dev.h"

namespace palu {

constexpr int kRowPad = 16;   // bytes of padding per LDS row: keeps 16-byte column reads conflict-free

template <int N>
struct StaticFor {
  template <typename F>
  static __device__ __forceinline__ void run(F&& f) {
    StaticFor<N - 1>::run(f);
    f(N - 1);
  }
};
template <>
struct StaticFor<0> {
  template <typename F>
  static __device__ __forceinline__ void run(F&&) {}
};

// KS_MAX: k-steps of 16 held in registers (rank <= 16*KS_MAX)
// RT:     32-row feature tiles per wavefront: 4 = a whole head, 2 = half a head
// I4:     latents are packed 4-bit codes with per-(token, block) scale and zero
template <typename T, int KS_MAX, int RT, bool I4>
__global__ __launch_bounds__(256, 1) void score_kernel(ScoreArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  using vec8 = typename T::vec8;

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
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
  const int r = m.k_off[j + 1] - m.k_off[j];
  const int nks = r >> 4;
  // column range of the latent row staged by the workgroup
  const int jl = m.group_of_head[h0], jh = m.group_of_head[h0 + nh - 1];
  const int c_lo = m.k_off[jl], c_hi = m.k_off[jh + 1];
  const int width = c_hi - c_lo;                               // elements, multiple of 32
  const int row_b = width * 2 + kRowPad;                       // LDS row pitch in bytes
  const int kbase_b = (m.k_off[j] - c_lo) * 2;                 // this head's first column inside the tile row

  // ---- stationary operand: folded weights of (b, head), rows [32*rt0, 32*(rt0+RT))
  vec8 W[KS_MAX][RT];
  {
    const uint16_t* mf = a.mfold + (size_t)b * a.mfold_bstride + m.bk_off[j] +
                         (size_t)(hc - m.head_off[j]) * r * kDHead;
    StaticFor<KS_MAX>::run([&](int ks) {
      if (ks < nks) {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
          W[ks][rt] = *reinterpret_cast<const vec8*>(mf + ((size_t)(ks * 4 + rt0 + rt) * 64 + lane) * 8);
      }
    });
  }

  // ---- staging geometry: 16-byte chunks of a tile row, `cpr` per row
  const int cpr = width >> 3;
  const int rows_pp = 256 / cpr;                               // rows per pass
  const int my_row = tid / cpr, my_col = tid - my_row * cpr;
  const bool stager = my_row < rows_pp;
  const int n_pass = (kTile + rows_pp - 1) / rows_pp;          // <= 8 because width <= 512
  constexpr int kMaxPass = 8;

  const size_t seq_base = (size_t)b * a.max_seq;
  uint4v stage[kMaxPass];

  auto issue_loads = [&](int tile) {
    const int t0 = t_begin + tile * kTile;
    StaticFor<kMaxPass>::run([&](int p) {
      if (p < n_pass) {
        const int rr = p * rows_pp + my_row;
        if (stager && rr < kTile) {
          const int t = min(t0 + rr, L - 1);
          if (!I4) {
            const uint16_t* src = (const uint16_t*)a.hk + (seq_base + t) * a.row_elems + c_lo + my_col * 8;
            stage[p] = *reinterpret_cast<const uint4v*>(src);
          } else {
            const int c = c_lo + my_col * 8;
            const uint8_t* src = (const uint8_t*)a.hk + ((seq_base + t) * a.row_elems + c) / 2;
            const uint32_t codes = *reinterpret_cast<const uint32_t*>(src);
            const size_t sb = (seq_base + t) * a.n_blocks_q + c / a.quant_block;
            const float s = F16::to_float(a.hk_scale[sb]);
            const float z = F16::to_float(a.hk_zero[sb]);
            uint32_t o[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float lo = ((float)((codes >> (8 * e)) & 15u) - z) * s;
              const float hi = ((float)((codes >> (8 * e + 4)) & 15u) - z) * s;
              o[e] = (uint32_t)T::from_float(lo) | ((uint32_t)T::from_float(hi) << 16);
            }
            stage[p] = uint4v{o[0], o[1], o[2], o[3]};
          }
        }
      }
    });
  };
  auto store_stage = [&](int buf) {
    unsigned char* base = lds + (size_t)buf * kTile * row_b;
    StaticFor<kMaxPass>::run([&](int p) {
      if (p < n_pass) {
        const int rr = p * rows_pp + my_row;
        if (stager && rr < kTile) *reinterpret_cast<uint4v*>(base + rr * row_b + my_col * 16) = stage[p];
      }
    });
  };

  issue_loads(0);
  store_stage(0);
  __syncthreads();

  const uint16_t* rope_base = a.rope + lane_hi * 64 + rt0 * 16;
  float* out_row = a.scores + ((size_t)(RT == 2 ? (wave & 1) : 0) * a.batch + b) * m.n_heads * (size_t)a.lpad +
                   (size_t)hc * a.lpad;

  for (int tile = 0; tile < n_tiles; ++tile) {
    const int t0 = t_begin + tile * kTile;
    if (tile + 1 < n_tiles) issue_loads(tile + 1);

    // cos/sin row of this lane's token (the lane's token is column lane_lo of the tile)
    const int t_mine = min(t0 + lane_lo, L - 1);
    int pos = a.k_pos ? a.k_pos[t_mine] : t_mine;
    pos = max(0, min(pos, a.rope_len - 1));
    const uint4v* rp = reinterpret_cast<const uint4v*>(a.rope + (size_t)pos * kDHead + (rope_base - a.rope));
    uint4v cs[RT * 2];
#pragma unroll
    for (int x = 0; x < RT * 2; ++x) cs[x] = rp[x];

    float16v acc[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[rt][i] = 0.f;

    const unsigned char* tile_base = lds + (size_t)(tile & 1) * kTile * row_b + lane_lo * row_b + kbase_b + lane_hi * 16;
    StaticFor<KS_MAX>::run([&](int ks) {
      if (ks < nks) {
        const vec8 hfrag = *reinterpret_cast<const vec8*>(tile_base + ks * 32);
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) acc[rt] = T::mfma(W[ks][rt], hfrag, acc[rt]);
      }
    });

    // RoPE-weighted feature sum: acc[rt][i] is feature 32*(rt0+rt) + mfma_row(i) of token lane_lo
    float part = 0.f;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const uint32_t wrd = cs[rt * 2 + (i >> 3)][(i >> 1) & 3];
        const uint16_t bits = (i & 1) ? (uint16_t)(wrd >> 16) : (uint16_t)(wrd & 0xffffu);
        part = fmaf(acc[rt][i], F16::to_float(bits), part);
      }
    }
    part += __shfl_xor(part, 32, 64);
    if (active && lane_hi == 0 && t0 + lane_lo < t_end) out_row[t0 + lane_lo] = part * a.scale;

    if (tile + 1 < n_tiles) store_stage((tile + 1) & 1);
    __syncthreads();
  }
}

#define PALU_SCORE_INST(T, KS, RT, I4) template __global__ void score_kernel<T, KS, RT, I4>(ScoreArgs);
PALU_SCORE_INST(F16, 4, 4, false)
PALU_SCORE_INST(F16, 8, 4, false)
PALU_SCORE_INST(F16, 16, 4, false)
PALU_SCORE_INST(F16, 32, 2, false)
PALU_SCORE_INST(F16, 4, 4, true)
PALU_SCORE_INST(F16, 8, 4, true)
PALU_SCORE_INST(F16, 16, 4, true)
PALU_SCORE_INST(F16, 32, 2, true)
PALU_SCORE_INST(BF16, 4, 4, false)
PALU_SCORE_INST(BF16, 8, 4, false)
PALU_SCORE_INST(BF16, 16, 4, false)
PALU_SCORE_INST(BF16, 32, 2, false)

}  // namespace palu
