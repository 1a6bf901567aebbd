// RoPE angle table, and B_k laid out as the stationary operand of the score kernel.
//
// The score path rebuilds the key of every cached position, K[t] = H_k[t] B_k
// (Sec. 3.2.3), on the matrix cores from the exact 16-bit inputs with float32
// accumulation, rotates it (RoPE pairs feature f with f + 64, angle
// phi_f(t) = pos_t * theta^(-2f/128); Sec. 3.1.2) and multiplies by the rotated query
// q' in float32 (Sec. 2.1 Eq. 2).  With k = K[t], c = cos phi_f(t), s = sin phi_f(t):
//   q' . RoPE(k, t) = sum_f  k_f (c q'_f + s q'_{f+64})  +  k_{f+64} (c q'_{f+64} - s q'_f).
// fold_kernel writes B_k^T per head (128 x r) in the register layout of the matrix
// instruction's operand; that layout does not depend on the query or the sequence.

#include "palu_dev.h"

namespace palu {

// One (position, pair) per thread; positions 0 .. 32 * ceil(n_pos / 32) - 1 (whole tiles); layout in palu_dev.h.
__global__ __launch_bounds__(256) void rope_table_kernel(unsigned char* table, int n_pos_padded, float theta) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  const int p = idx >> 6, f = idx & 63;
  if (p >= n_pos_padded) return;
  double c = 1.0, s = 0.0;
  if (theta > 0.f) {
    const double w = pow((double)theta, -2.0 * (double)f / (double)kDHead);
    sincos((double)p * w, &s, &c);
  }
  float* f32 = reinterpret_cast<float*>(table);
  f32[rope_f32_index(p, f, 0, kRopeTableStride)] = (float)c;
  f32[rope_f32_index(p, f, 1, kRopeTableStride)] = (float)s;
  uint16_t* row = reinterpret_cast<uint16_t*>(table + (size_t)(p >> 5) * kRopeTableStride + kRopeTileBytes) + (size_t)(p & 31) * kDHead;
  row[rope_slot(f)] = F16::from_float((float)c);
  row[rope_slot(f + kHalf)] = F16::from_float((float)s);
}

// rows[t] = table[clamp(k_pos[t])] for the float16 rows: lets the shared-key score form address
// cos/sin rows by cached-token index.  One thread per 16-byte piece of a row.
__global__ __launch_bounds__(256) void rope_gather_kernel(RopeGatherArgs a) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  const int t = idx >> 4, c = idx & 15;
  if (t >= a.n) return;
  const int pos = max(0, min(a.k_pos[min(t, a.k_pos_len - 1)], a.table_len - 1));
  const unsigned char* src = static_cast<const unsigned char*>(a.table) + (size_t)(pos >> 5) * kRopeTableStride + kRopeTileBytes;
  reinterpret_cast<uint4v*>(a.rows)[(size_t)t * 16 + c] = reinterpret_cast<const uint4v*>(src)[(size_t)(pos & 31) * 16 + c];
}

// The same for the float32 tiles: the angles of cached token t (position k_pos[t]) at token
// index t of the output tiles.  One thread per (token, pair); a.n is a multiple of 32 and
// token indices past the end of k_pos repeat its last entry (they are never attended).
__global__ __launch_bounds__(256) void rope_gather_tiles_kernel(RopeGatherArgs a) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  const int t = idx & 31, f = (idx >> 5) & 63, tile = idx >> 11;     // token fastest: coalesced stores
  const int tok = tile * 32 + t;
  if (tok >= a.n) return;
  const int pos = max(0, min(a.k_pos[min(tok, a.k_pos_len - 1)], a.table_len - 1));
  const float* src = static_cast<const float*>(a.table);
  float* dst = static_cast<float*>(a.rows);
  dst[rope_f32_index(tok, f, 0, kRopeTileBytes)] = src[rope_f32_index(pos, f, 0, kRopeTableStride)];
  dst[rope_f32_index(tok, f, 1, kRopeTileBytes)] = src[rope_f32_index(pos, f, 1, kRopeTableStride)];
}

// grid (max k-steps of any head, n_heads), 256 threads: one workgroup lays out one
// k-step (16 rows of B_k) of one head.  The 16 x 128 block of B_k is fetched
// with coalesced 16-byte loads, transposed through LDS, and written as 256
// 16-byte words in operand order: word (row tile rt, lane) = 8 consecutive k of
// feature 32 rt + lane % 32, k-octet lane / 32.  The 16-bit values are copied as they are.
// Heads of rank 64 and more are laid out for score16_kernel instead when a.layout16 is set (16-feature
// operands of v_mfma_f32_16x16x32): per k-step of 32 rows, 512 words: word (feature tile ct, lane) =
// 8 consecutive k (k-octet lane / 16 of the 32) of feature 16 ct + lane % 16; the workgroups of even ks
// do two 16-row steps each.
// (ks, h): the workgroup's position in that grid.
__device__ __forceinline__ void fold_body(const FoldArgs& a, int ks, int h) {
  __shared__ __attribute__((aligned(16))) uint16_t Bs[32][kDHead + 8];
  const int tid = threadIdx.x;
  const Meta& m = a.meta;
  const int j = group_of(m, h);
  const int u = h - m.head_off[j];
  const int r = m.k_off[j + 1] - m.k_off[j];
  if (ks >= (r >> 4)) return;
  int width;
  // ranks above 256 are contracted in slices of up to 256 rows (layout16 == 1: only those above 512, the others by score_kernel)
  if (a.layout16 && r >= 64 && (a.layout16 == 2 || r <= 256 || r > 512)) {
    if (ks & 1) return;
    const uint16_t* B = a.Bk + weight_block(m, j, h, m.bk_off[j], &width);
    const int lrow = tid >> 3, lcol = (tid & 7) * 16;             // thread = (row of 32, 16-column piece)
    const uint16_t* src = B + (size_t)(16 * ks + lrow) * width + lcol;
    *reinterpret_cast<uint4v*>(&Bs[lrow][lcol]) = *reinterpret_cast<const uint4v*>(src);
    *reinterpret_cast<uint4v*>(&Bs[lrow][lcol + 8]) = *reinterpret_cast<const uint4v*>(src + 8);
    __syncthreads();
    uint16_t* out = a.mfold + m.bk_off[j] + (size_t)u * r * kDHead + (size_t)(ks >> 1) * 512 * 8;
#pragma unroll
    for (int x = 0; x < 2; ++x) {
      const int w = tid + 256 * x, ct = w >> 6, lane = w & 63;
      const int col = 16 * ct + (lane & 15), k0 = 8 * (lane >> 4);
      uint16_t v[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = Bs[k0 + e][col];
      uint4v pk;
      pk.x = v[0] | ((uint32_t)v[1] << 16);
      pk.y = v[2] | ((uint32_t)v[3] << 16);
      pk.z = v[4] | ((uint32_t)v[5] << 16);
      pk.w = v[6] | ((uint32_t)v[7] << 16);
      *reinterpret_cast<uint4v*>(out + (size_t)w * 8) = pk;
    }
    return;
  }

  // rows 16*ks .. 16*ks+15 of this head's 128 columns: thread = (row, 8-column piece)
  const uint16_t* B = a.Bk + weight_block(m, j, h, m.bk_off[j], &width);
  const int lrow = tid >> 4, lcol = (tid & 15) * 8;
  *reinterpret_cast<uint4v*>(&Bs[lrow][lcol]) = *reinterpret_cast<const uint4v*>(B + (size_t)(16 * ks + lrow) * width + lcol);
  __syncthreads();

  const int lane = tid & 63, rt = tid >> 6;
  const int cp = 32 * rt + (lane & 31);
  const int k0 = 8 * (lane >> 5);
  uint16_t v[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = Bs[k0 + e][cp];
  uint4v pk;
  pk.x = v[0] | ((uint32_t)v[1] << 16);
  pk.y = v[2] | ((uint32_t)v[3] << 16);
  pk.z = v[4] | ((uint32_t)v[5] << 16);
  pk.w = v[6] | ((uint32_t)v[7] << 16);
  uint16_t* out = a.mfold + m.bk_off[j] + (size_t)u * r * kDHead;
  *reinterpret_cast<uint4v*>(out + ((size_t)ks * 256 + tid) * 8) = pk;
}

__global__ __launch_bounds__(256) void fold_kernel(FoldArgs a) {
  fold_body(a, blockIdx.x, blockIdx.y);
}

// Shared-key form of the score kernel: the rotated queries q' = RoPE(q, position of
// the query) of the (up to 16) queries of one key/value head, as A operands of its 8
// query contractions (v_mfma_f32_32x32x16: row = query, k-octet = lane half).  Step N
// of lane half `hi` covers the accumulators e = 4N .. 4N+3 (e = 16 rt + i: rotation
// pair f = 32 rt + mfma_row(i, hi)) as K cos_f and K sin_f in the order (cos e, cos
// e+1, sin e, sin e+1, cos e+2, cos e+3, sin e+2, sin e+3); the matching query
// entries are q'_f for cos and q'_{f+64} for sin where the wavefront holds K_f, and
// q'_{f+64} and -q'_f where it holds K_{f+64}.  Rows of absent queries are zero.
// Layout [batch][kv head][feature half][step 8][lane half 2][query 16] x 16 bytes (4 KiB per feature half); with at
// most 4 queries (`small`) the 4x4x4 form's operands instead, see below.
// grid (key/value heads, batch), 256 threads.
// (kvh, b): the workgroup's position in that grid.
// A: QfragArgs, or anything with the same members (the fused first launch of a decode step passes a view of its own arguments).
template <typename T, typename A>
__device__ __forceinline__ void qfrag_body(const A& a, int kvh, int b) {
  __shared__ float qr[16][kDHead];
  const int tid = threadIdx.x;
  Meta m;                                             // only the fields q_row and q_token read
  m.n_heads = a.n_heads; m.qpk = a.qpk; m.nq = a.nq;
  for (int h0 = 0; h0 < a.qpk; h0 += 4) {
    const int hq = h0 + (tid >> 6), f = tid & 63;
    if (hq >= a.qpk) continue;
    const int h = kvh * a.qpk + hq;
    const uint16_t* qp = a.q + q_row(m, b, h) * kDHead;
    const float x0 = T::to_float(qp[f]);
    const float x1 = T::to_float(qp[f + kHalf]);
    const float pos = (float)a.q_pos[b * a.nq + q_token(m, h)];
    const float p = pos * a.rev_hi[f];
    const float e = fmaf(pos, a.rev_hi[f], -p);
    const float rev = (p - floorf(p)) + (e + pos * a.rev_lo[f]);      // angle in revolutions: ~1e-7 absolute accuracy for positions up to 2^24
    const float s = __builtin_amdgcn_sinf(rev), c = __builtin_amdgcn_cosf(rev);
    qr[hq][f] = x0 * c - x1 * s;
    qr[hq][f + kHalf] = x1 * c + x0 * s;
  }
  __syncthreads();
  if (a.small) {
    // at most 4 queries, contracted on 4x4x4 blocks: [feature half][step n 16][lane half 2][query 4] x 8 bytes, step n
    // covering the accumulators e = 2n, 2n+1 in the order (cos e, cos e+1, sin e, sin e+1); 4 KiB apart per feature half
    uint2v* out2 = reinterpret_cast<uint2v*>(a.qfrag) + ((size_t)b * a.n_kv + kvh) * 1024;
    {
      const int item = tid;                               // 2 x 16 x 2 x 4 = 256 entries
      const int row = item & 3, hi = (item >> 2) & 1, n = (item >> 3) & 15, half = item >> 7;
      uint16_t v[4];
#pragma unroll
      for (int y = 0; y < 2; ++y) {
        const int e = 2 * n + y;
        const int f = 32 * (e >> 4) + mfma_row(e & 15, hi);
        float qc = 0.f, qs = 0.f;
        if (row < a.qpk) {
          qc = half ? qr[row][f + kHalf] : qr[row][f];
          qs = half ? -qr[row][f] : qr[row][f + kHalf];
        }
        v[y] = F16::from_float(qc);
        v[2 + y] = F16::from_float(qs);
      }
      uint2v pk;
      pk.x = v[0] | ((uint32_t)v[1] << 16);
      pk.y = v[2] | ((uint32_t)v[3] << 16);
      out2[half * 512 + (item & 127)] = pk;
    }
    return;
  }
  uint4v* out = reinterpret_cast<uint4v*>(a.qfrag) + ((size_t)b * a.n_kv + kvh) * 512;
  for (int item = tid; item < 512; item += 256) {
    const int row = item & 15, hi = (item >> 4) & 1, N = (item >> 5) & 7, half = item >> 8;
    uint16_t v[8];
#pragma unroll
    for (int y = 0; y < 4; ++y) {
      const int e = 4 * N + y;
      const int f = 32 * (e >> 4) + mfma_row(e & 15, hi);
      float qc = 0.f, qs = 0.f;
      if (row < a.qpk) {
        qc = half ? qr[row][f + kHalf] : qr[row][f];
        qs = half ? -qr[row][f] : qr[row][f + kHalf];
      }
      // accumulators e = 4N + y: y = 0, 1 fill entries (0, 1) with cos parts and (2, 3) with sin parts; y = 2, 3 entries 4 .. 7
      v[4 * (y >> 1) + (y & 1)] = F16::from_float(qc);
      v[4 * (y >> 1) + 2 + (y & 1)] = F16::from_float(qs);
    }
    uint4v pk;
    pk.x = v[0] | ((uint32_t)v[1] << 16);
    pk.y = v[2] | ((uint32_t)v[3] << 16);
    pk.z = v[4] | ((uint32_t)v[5] << 16);
    pk.w = v[6] | ((uint32_t)v[7] << 16);
    out[item] = pk;
  }
}

template <typename T>
__global__ __launch_bounds__(256) void qfrag_kernel(QfragArgs a) {
  qfrag_body<T>(a, blockIdx.x, blockIdx.y);
}

template __global__ void qfrag_kernel<F16>(QfragArgs);

}  // namespace palu
