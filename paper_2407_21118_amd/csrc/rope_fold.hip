// RoPE angle table and the per-step fold of the rotated query into B_k.
//
// Score identity used by the whole score path (RoPE pairs feature f with
// f + 64, angle phi_f(t) = pos_t * theta^(-2f/128); Sec. 3.1.2):
//   q' . RoPE(k, t) = sum_f cos(phi_f(t)) (q'_f k_f + q'_{f+64} k_{f+64})
//                         + sin(phi_f(t)) (q'_{f+64} k_f - q'_f k_{f+64})
// and with k = h B (Sec. 3.2.3) every bracket is h . (a column built from q' and B):
//   u_f = q'_f B[:,f] + q'_{f+64} B[:,f+64],   w_f = q'_{f+64} B[:,f] - q'_f B[:,f+64].
// The fold kernel writes M = [u_0..u_63 | w_0..w_63] (r x 128 per head, fp16) in the
// register layout of the MFMA A operand, so that the score kernel's contraction
// H_k . M is the reconstruction GEMM itself (same r x 128 MACs per token and
// head) and RoPE reduces to one cos/sin-weighted sum per accumulator.

#include "palu_dev.h"

namespace palu {

// table[p][slot(c')] = fp16(cos(p w_c')) for c' < 64, fp16(sin(p w_{c'-64})) otherwise.
__global__ __launch_bounds__(256) void rope_table_kernel(uint16_t* table, int n_pos, float theta) {
  const int idx = blockIdx.x * 256 + threadIdx.x;      // one (position, pair) per thread
  const int p = idx >> 6, f = idx & 63;
  if (p >= n_pos) return;
  double c = 1.0, s = 0.0;
  if (theta > 0.f) {
    const double w = pow((double)theta, -2.0 * (double)f / (double)kDHead);
    sincos((double)p * w, &s, &c);
  }
  uint16_t* row = table + (size_t)p * kDHead;
  row[rope_slot(f)] = F16::from_float((float)c);
  row[rope_slot(f + kHalf)] = F16::from_float((float)s);
}

// rows[t] = table[clamp(k_pos[t])]: lets the score kernel address cos/sin rows by
// cached-token index without a dependent position load in its inner loop.
// One thread per 16-byte piece of a row.
__global__ __launch_bounds__(256) void rope_gather_kernel(RopeGatherArgs a) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  const int t = idx >> 4, c = idx & 15;
  if (t >= a.n) return;
  const int pos = max(0, min(a.k_pos[t], a.table_len - 1));
  reinterpret_cast<uint4v*>(a.rows)[(size_t)t * 16 + c] = reinterpret_cast<const uint4v*>(a.table)[(size_t)pos * 16 + c];
}

// grid (max k-steps of any head, n_heads, batch), 256 threads: one workgroup folds
// one k-step (16 rows of B_k) of one head.  The 16 x 128 block of B_k is fetched
// with coalesced 16-byte loads, transposed through LDS, and written as 256
// 16-byte words in MFMA operand order.
// (ks, h, b): the workgroup's position in that grid.
template <typename T>
__device__ __forceinline__ void fold_body(const FoldArgs& a, int ks, int h, int b) {
  __shared__ float qr[kDHead];
  __shared__ __attribute__((aligned(16))) uint16_t Bs[16][kDHead + 8];
  const int tid = threadIdx.x;
  const Meta& m = a.meta;
  const int j = group_of(m, h);
  const int u = h - m.head_off[j];
  const int r = m.k_off[j + 1] - m.k_off[j];
  if (ks >= (r >> 4)) return;
  int width;

  // rows 16*ks .. 16*ks+15 of this head's 128 columns: thread = (row, 8-column piece)
  const uint16_t* B = a.Bk + weight_block(m, j, h, m.bk_off[j], &width);
  const int lrow = tid >> 4, lcol = (tid & 15) * 8;
  const uint4v raw = *reinterpret_cast<const uint4v*>(B + (size_t)(16 * ks + lrow) * width + lcol);

  if (tid < kHalf && !a.plain) {
    // rotate the query: angle = pos * w_f with w_f / 2pi given as a float pair
    // (hi, lo) from the host's float64 value, so that the angle in revolutions
    // keeps ~1e-7 absolute accuracy for positions up to 2^24
    const uint16_t* qp = a.q + q_row(m, b, h) * kDHead;
    const float x0 = T::to_float(qp[tid]);
    const float x1 = T::to_float(qp[tid + kHalf]);
    float c = 1.f, s = 0.f;
    if (a.theta > 0.f) {
      const float pos = (float)a.q_pos[b * m.nq + q_token(m, h)];
      const float p = pos * a.rev_hi[tid];
      const float e = fmaf(pos, a.rev_hi[tid], -p);
      const float rev = (p - floorf(p)) + (e + pos * a.rev_lo[tid]);
      s = __builtin_amdgcn_sinf(rev);
      c = __builtin_amdgcn_cosf(rev);
    }
    qr[tid] = x0 * c - x1 * s;
    qr[tid + kHalf] = x1 * c + x0 * s;
  }
  *reinterpret_cast<uint4v*>(&Bs[lrow][lcol]) = raw;
  __syncthreads();

  // one item = (row tile rt, lane) = 8 consecutive k of feature row c' = 32*rt + lane%32
  const int lane = tid & 63, rt = tid >> 6;
  const int cp = 32 * rt + (lane & 31);
  const int f = cp & 63;
  const bool is_w = cp >= kHalf;
  const float qa = a.plain ? 0.f : qr[f], qb = a.plain ? 0.f : qr[f + kHalf];
  const int k0 = 8 * (lane >> 5);
  uint16_t v[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const float b1 = T::to_float(Bs[k0 + e][f]);
    const float b2 = T::to_float(Bs[k0 + e][f + kHalf]);
    const float val = a.plain ? (is_w ? b2 : b1) : (is_w ? (qb * b1 - qa * b2) : (qa * b1 + qb * b2));
    v[e] = F16::from_float(val);       // the score kernel always contracts in fp16
  }
  uint4v pk;
  pk.x = v[0] | ((uint32_t)v[1] << 16);
  pk.y = v[2] | ((uint32_t)v[3] << 16);
  pk.z = v[4] | ((uint32_t)v[5] << 16);
  pk.w = v[6] | ((uint32_t)v[7] << 16);
  uint16_t* out = a.mfold + (size_t)b * a.mfold_bstride + m.bk_off[j] + (size_t)u * r * kDHead;
  *reinterpret_cast<uint4v*>(out + ((size_t)ks * 256 + tid) * 8) = pk;
}

template <typename T>
__global__ __launch_bounds__(256) void fold_kernel(FoldArgs a) {
  fold_body<T>(a, blockIdx.x, blockIdx.y, blockIdx.z);
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
    const float rev = (p - floorf(p)) + (e + pos * a.rev_lo[f]);      // angle in revolutions, as in fold_kernel
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
template __global__ void fold_kernel<F16>(FoldArgs);
template __global__ void fold_kernel<BF16>(FoldArgs);

}  // namespace palu
