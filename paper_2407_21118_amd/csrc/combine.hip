// Split merge, normalisation and the B_v up-projection (Eq. 4: (p H_v) B_v), after
// the per-split softmax partials of pv.hip:
//   combine_kernel merges the partials (m, l, o) of a head over the splits of its
//   sequence, divides by l and multiplies by the head's block of B_v.

#include "palu_dev.h"

namespace palu {

constexpr int kMaxSplits = 1024;    // splits per sequence the combine kernel accepts

template <int HB>
__device__ __forceinline__ void block_reduce(float (&v)[HB], float* scratch, bool is_max) {
  // 256 threads = 4 wavefronts; result broadcast to all threads
#pragma unroll
  for (int h = 0; h < HB; ++h) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      const float o = __shfl_xor(v[h], off, 64);
      v[h] = is_max ? fmaxf(v[h], o) : v[h] + o;
    }
  }
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  __syncthreads();
  if (lane == 0) {
#pragma unroll
    for (int h = 0; h < HB; ++h) scratch[wave * HB + h] = v[h];
  }
  __syncthreads();
#pragma unroll
  for (int h = 0; h < HB; ++h) {
    float r = scratch[h];
#pragma unroll
    for (int w = 1; w < 4; ++w) r = is_max ? fmaxf(r, scratch[w * HB + h]) : r + scratch[w * HB + h];
    v[h] = r;
  }
}

// grid (n_heads * 4, batch), 256 threads: a workgroup produces 32 of the 128
// output columns of one head (the merge of the splits is repeated by the four
// workgroups of a head; it is small and this keeps the kernel to one launch).
// Small and latency-bound: every phase spreads its loads over all 256 threads
// and keeps them independent.
template <typename T>
__global__ __launch_bounds__(256) void combine_kernel(CombineArgs a) {
  __shared__ float w[kMaxSplits];
  __shared__ __attribute__((aligned(16))) float olat[PALU_MAX_RANK];
  __shared__ __attribute__((aligned(16))) float part[1024];              // phase 2: [4 split groups][64 k-quads][4]; phase 3: [8 k parts][32 column quads][4]
  __shared__ float red[4];
  const int tid = threadIdx.x;
  const Meta& m = a.meta;
  const int h = blockIdx.x >> 2, quarter = blockIdx.x & 3, b = blockIdx.y;
  const int L = a.seq_lens ? min(a.seq_lens[b], a.seq_len) : a.seq_len;
  const int nsp = L > 0 ? (L + a.split_tokens - 1) / a.split_tokens : 0;
  const int j = group_of(m, h);
  const int rv = m.v_off[j + 1] - m.v_off[j];
  int width;
  const int bv_blk = weight_block(m, j, h, m.bv_off[j], &width);

  // ---- softmax merge weights of the splits
  const float* ml = a.ml_part + ((size_t)b * a.n_split * m.n_heads + h) * 2;
  const size_t ml_stride = (size_t)m.n_heads * 2;
  float mx[1] = {-INFINITY};
  for (int c = tid; c < nsp; c += 256) mx[0] = fmaxf(mx[0], ml[c * ml_stride]);
  block_reduce<1>(mx, red, true);
  float sum[1] = {0.f};
  for (int c = tid; c < nsp; c += 256) {
    const float wc = mx[0] == -INFINITY ? 0.f : exp2f(ml[c * ml_stride] - mx[0]);     // no split saw an attended row: all weights 0
    w[c] = wc;
    sum[0] += wc * ml[c * ml_stride + 1];
  }
  block_reduce<1>(sum, red, false);      // barriers publish w[]

  // ---- o_lat[k] = sum_c w_c o_c[k]: thread = (split group sg of 4, k-quad kq of 64), 16-byte loads
  const float* op = a.o_part + (size_t)b * a.n_split * a.o_stride + o_head_off(m, h);
  const int sg = tid >> 6, kq = tid & 63;
  for (int kb = 0; kb < rv; kb += 256) {
    const int k = kb + kq * 4;
    float4v acc = {0.f, 0.f, 0.f, 0.f};
    if (k < rv) {
      // 16 independent loads per batch: the merge is a chain of L2 latencies otherwise
      for (int c0 = sg; c0 < nsp; c0 += 64) {
        float4v v[16];
#pragma unroll
        for (int x = 0; x < 16; ++x) {
          const int c = min(c0 + 4 * x, nsp - 1);
          v[x] = *reinterpret_cast<const float4v*>(op + (size_t)c * a.o_stride + k);
        }
#pragma unroll
        for (int x = 0; x < 16; ++x) {
          const int c = c0 + 4 * x;
          const float wc = c < nsp ? w[c] : 0.f;
          acc.x = fmaf(wc, v[x].x, acc.x);
          acc.y = fmaf(wc, v[x].y, acc.y);
          acc.z = fmaf(wc, v[x].z, acc.z);
          acc.w = fmaf(wc, v[x].w, acc.w);
        }
      }
    }
    *reinterpret_cast<float4v*>(part + (sg * 64 + kq) * 4) = acc;
    __syncthreads();
    if (tid < 64 && k < rv) {
      float4v s = *reinterpret_cast<const float4v*>(part + kq * 4);
#pragma unroll
      for (int g = 1; g < 4; ++g) {
        const float4v o = *reinterpret_cast<const float4v*>(part + (g * 64 + kq) * 4);
        s.x += o.x; s.y += o.y; s.z += o.z; s.w += o.w;
      }
      *reinterpret_cast<float4v*>(olat + k) = s;
    }
    __syncthreads();
  }

  if (a.out_latent) {          // output stays in the latent space: this workgroup writes its quarter of the head's r_v values
    float* ol = a.out_latent + (size_t)b * a.o_stride + o_head_off(m, h);
    const int per = ((rv >> 2) + 3) & ~3;
    for (int k = quarter * per + tid; k < min(rv, (quarter + 1) * per); k += 256) ol[k] = sum[0] > 0.f ? olat[k] / sum[0] : 0.f;
    return;
  }

  // ---- out = o_lat . B_v[:, 32 of the head's columns] / l: thread = (k part kp of 32, column quad cq of 8), 8-byte loads
  const int kp = tid >> 3, cq = tid & 7;
  const uint16_t* Bv = a.Bv + bv_blk + quarter * 32 + cq * 4;
  const int k_per = rv >> 5;                       // rank is a multiple of 32
  float4v o = {0.f, 0.f, 0.f, 0.f};
  for (int k0 = 0; k0 < k_per; k0 += 8) {          // 8 independent loads per batch
    uint2v raw[8];
#pragma unroll
    for (int x = 0; x < 8; ++x) raw[x] = *reinterpret_cast<const uint2v*>(Bv + (size_t)(kp * k_per + min(k0 + x, k_per - 1)) * width);
#pragma unroll
    for (int x = 0; x < 8; ++x) {
      const float ol = k0 + x < k_per ? olat[kp * k_per + k0 + x] : 0.f;
      o.x = fmaf(ol, T::to_float((uint16_t)(raw[x].x & 0xffffu)), o.x);
      o.y = fmaf(ol, T::to_float((uint16_t)(raw[x].x >> 16)), o.y);
      o.z = fmaf(ol, T::to_float((uint16_t)(raw[x].y & 0xffffu)), o.z);
      o.w = fmaf(ol, T::to_float((uint16_t)(raw[x].y >> 16)), o.w);
    }
  }
  *reinterpret_cast<float4v*>(part + (kp * 8 + cq) * 4) = o;
  __syncthreads();
  if (tid < 32) {
    const int c4 = tid >> 2, e = tid & 3;
    float s = 0.f;
#pragma unroll
    for (int g = 0; g < 32; ++g) s += part[(g * 8 + c4) * 4 + e];
    a.out[q_row(m, b, h) * kDHead + quarter * 32 + tid] = sum[0] > 0.f ? s / sum[0] : 0.f;   // no row attended: zeros
  }
}

template __global__ void combine_kernel<F16>(CombineArgs);
template __global__ void combine_kernel<BF16>(CombineArgs);

}  // namespace palu
