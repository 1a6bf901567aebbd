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

// Columns a latent tile row takes in LDS: the rows of unquantized latents (at most 256 columns: groups x rank) are
// laid out in the 32 slots of a 256-column row, whatever their width, and requested two per instruction.
constexpr int score16_lds_width(int width, bool staged) { return staged ? width : 256; }
// LDS bytes of score16_kernel for unquantized latents (shared with the host)
constexpr int score16_lds_bytes(int width) { return score_lds_bytes(score16_lds_width(width, false), true, true, false); }

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
template <typename T, int NK, int G, int NQ = 1, int QB = 0>
__global__ __launch_bounds__(256) void score16_kernel(ScoreArgs a) {
  const int chunk = blockIdx.x, unit = blockIdx.y, b = blockIdx.z;
  const int chunk_tokens = a.chunk_tokens;
#include "score16_body.inc"
}

// The same body with its place in the launch as arguments (sequence chunk of chunk_tokens tokens, unit, sequence), so
// that a launch over several rank classes can hand each workgroup the body of its unit's class.
template <typename T, int NK, int G, int NQ = 1, int QB = 0>
__device__ __forceinline__ void score16_body(const ScoreArgs& a, const int chunk, const int unit, const int b, const int chunk_tokens) {
#include "score16_body.inc"
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
