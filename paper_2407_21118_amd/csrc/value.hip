// Softmax and the value side, contracted in latent space (Eq. 4: (p H_v) B_v):
//   value_kernel   per (sequence, group, split of the sequence): p = exp2(score - max),
//                  l = sum p, o = sum_t p_t H_v[t, group columns]   (split-K partials)
//   combine_kernel merges the partials of a head, normalises, applies B_v.
// The P.H_v contraction has only s (heads per group) FLOP per latent element,
// so it is HBM-bound: plain float32 FMAs on coalesced 16-byte loads, no matrix
// cores and no LDS staging of the latents.

#include "palu_dev.h"

namespace palu {

constexpr int kSplitMax = 1024;     // tokens per split kept as probabilities in LDS
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

// HB: heads of one group handled per workgroup (1, 2 or 4); all read the same latent columns.
template <typename T, int HB, bool I4>
__global__ __launch_bounds__(256) void value_kernel(ValueArgs a) {
  __shared__ __attribute__((aligned(16))) float sh[256 * HB * 8];   // probabilities, then the reduction buffer
  __shared__ float red[4 * HB];
  static_assert(256 * HB * 8 >= kSplitMax * HB, "probability buffer too small");

  const int tid = threadIdx.x;
  const Meta& m = a.meta;
  int wg = blockIdx.x;
  const int unit = wg % a.units.n_units;
  wg /= a.units.n_units;
  const int split = wg % a.n_split;
  const int b = wg / a.n_split;

  const int L = a.seq_lens ? min(a.seq_lens[b], a.seq_len) : a.seq_len;
  const int s0 = split * a.split_tokens;
  if (s0 >= L) return;
  const int ntok = min(a.split_tokens, L - s0);

  const int h0 = a.units.h0[unit], nh = a.units.nh[unit];
  const int j = m.group_of_head[h0];
  const int v0 = m.v_off[j];
  const int rv = m.v_off[j + 1] - v0;

  // ---- thread = (token in pass, 8-channel chunk) of the value-latent stream
  const int lpt = rv >> 3;                       // 16-byte chunks per token row of this group
  const int tpp = 256 / lpt;                     // tokens per pass
  const int my_tok = tid / lpt, my_ch = tid - my_tok * lpt;
  const bool worker = my_tok < tpp;
  const size_t row0 = (size_t)b * a.max_seq + s0;
  constexpr int U = 8;                           // loads in flight per thread
  const unsigned row_bytes = I4 ? (unsigned)a.row_elems / 2u : (unsigned)a.row_elems * 2u;
  const unsigned char* hv_base = (const unsigned char*)a.hv +
                                 (I4 ? (row0 * a.row_elems + v0 + my_ch * 8) / 2 : (row0 * a.row_elems + v0 + my_ch * 8) * 2);
  const size_t sb_base = row0 * a.n_blocks_q + (v0 + my_ch * 8) / a.quant_block;     // int4: scale / zero index of row 0

  // raw latents (and int4 scale/zero) of U tokens: my_tok + tb, my_tok + tb + tpp, ...
  struct Batch {
    uint4v h[U];
  };
  auto load_batch = [&](Batch& bt, int tb) {
#pragma unroll
    for (int x = 0; x < U; ++x) {
      const int tc = min(tb + x * tpp, ntok - 1);          // clamped: the weight of an out-of-range token is zero
      if (!I4) {
        bt.h[x] = *reinterpret_cast<const uint4v*>(hv_base + (size_t)tc * row_bytes);
      } else {
        bt.h[x].x = *reinterpret_cast<const uint32_t*>(hv_base + (size_t)tc * row_bytes);
        const size_t sb = sb_base + (size_t)tc * a.n_blocks_q;
        bt.h[x].y = (uint32_t)a.hv_scale[sb] | ((uint32_t)a.hv_zero[sb] << 16);
      }
    }
  };
  // the first batch goes out before the softmax prologue: HBM latency overlaps it
  Batch cur;
  if (worker) load_batch(cur, my_tok);

  // ---- scores of the split -> LDS, running max per head
  float mx[HB], sum[HB];
#pragma unroll
  for (int hh = 0; hh < HB; ++hh) { mx[hh] = -INFINITY; sum[hh] = 0.f; }
#pragma unroll
  for (int hh = 0; hh < HB; ++hh) {
    if (hh < nh) {
      const int h = h0 + hh;
      const float* s0p = a.scores + ((size_t)b * m.n_heads + h) * a.lpad + s0;
      const int np = a.n_parts[h];
      for (int t = tid; t < ntok; t += 256) {
        float s = s0p[t];
        for (int pl = 1; pl < np; ++pl) s += s0p[pl * a.part_stride + t];
        sh[t * HB + hh] = s;
        mx[hh] = fmaxf(mx[hh], s);
      }
    }
  }
  block_reduce<HB>(mx, red, true);
#pragma unroll
  for (int hh = 0; hh < HB; ++hh) {
    for (int t = tid; t < ntok; t += 256) {
      const float p = hh < nh ? exp2f(sh[t * HB + hh] - mx[hh]) : 0.f;
      sh[t * HB + hh] = p;
      sum[hh] += p;
    }
  }
  block_reduce<HB>(sum, red, false);     // its barriers also publish the probabilities

  // ---- stream the value latents
  float acc[HB][8];
#pragma unroll
  for (int hh = 0; hh < HB; ++hh)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[hh][e] = 0.f;

  if (worker) {
    for (int tb = my_tok; tb < ntok; tb += tpp * U) {
      Batch nxt;
      load_batch(nxt, tb + tpp * U);               // next batch in flight while this one is consumed
#pragma unroll
      for (int x = 0; x < U; ++x) {
        const int t = tb + x * tpp;
        const bool ok = t < ntok;
        const int tc = ok ? t : ntok - 1;
        float hvf[8];
        float pw[HB];
        if (!I4) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            hvf[2 * e] = T::to_float((uint16_t)(cur.h[x][e] & 0xffffu));
            hvf[2 * e + 1] = T::to_float((uint16_t)(cur.h[x][e] >> 16));
          }
#pragma unroll
          for (int hh = 0; hh < HB; ++hh) pw[hh] = ok ? sh[tc * HB + hh] : 0.f;
        } else {
          const uint32_t codes = cur.h[x].x;
          const float s = F16::to_float((uint16_t)(cur.h[x].y & 0xffffu));
          const float z = F16::to_float((uint16_t)(cur.h[x].y >> 16));
#pragma unroll
          for (int e = 0; e < 8; ++e) hvf[e] = (float)((codes >> (4 * e)) & 15u) - z;
#pragma unroll
          for (int hh = 0; hh < HB; ++hh) pw[hh] = ok ? sh[tc * HB + hh] * s : 0.f;
        }
#pragma unroll
        for (int hh = 0; hh < HB; ++hh)
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[hh][e] = fmaf(pw[hh], hvf[e], acc[hh][e]);
      }
      cur = nxt;
    }
  }

  // ---- reduce over the tokens-in-pass dimension and write the partial
  __syncthreads();                               // everyone is done reading probabilities
  if (worker) {
#pragma unroll
    for (int hh = 0; hh < HB; ++hh)
#pragma unroll
      for (int e = 0; e < 8; ++e) sh[(hh * 8 + e) * 256 + tid] = acc[hh][e];
  }
  __syncthreads();
  float* op = a.o_part + ((size_t)b * a.n_split + split) * a.o_stride;
  for (int idx = tid; idx < nh * rv; idx += 256) {
    const int hh = idx / rv, c = idx - hh * rv;
    const int ch = c >> 3, e = c & 7;
    float s = 0.f;
    for (int tp = 0; tp < tpp; ++tp) s += sh[(hh * 8 + e) * 256 + tp * lpt + ch];
    op[o_head_off(m, h0 + hh) + c] = s;
  }
  if (tid < nh) {
    float* ml = a.ml_part + (((size_t)b * a.n_split + split) * m.n_heads + h0 + tid) * 2;
    float mv = 0.f, sv = 0.f;
#pragma unroll
    for (int hh = 0; hh < HB; ++hh)
      if (hh == tid) { mv = mx[hh]; sv = sum[hh]; }
    ml[0] = mv;
    ml[1] = sv;
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
  const int nsp = (L + a.split_tokens - 1) / a.split_tokens;
  const int j = m.group_of_head[h];
  const int u = h - m.head_off[j];
  const int rv = m.v_off[j + 1] - m.v_off[j];
  const int width = (m.head_off[j + 1] - m.head_off[j]) * kDHead;

  // ---- softmax merge weights of the splits
  const float* ml = a.ml_part + ((size_t)b * a.n_split * m.n_heads + h) * 2;
  const size_t ml_stride = (size_t)m.n_heads * 2;
  float mx[1] = {-INFINITY};
  for (int c = tid; c < nsp; c += 256) mx[0] = fmaxf(mx[0], ml[c * ml_stride]);
  block_reduce<1>(mx, red, true);
  float sum[1] = {0.f};
  for (int c = tid; c < nsp; c += 256) {
    const float wc = exp2f(ml[c * ml_stride] - mx[0]);
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
#pragma unroll 4
      for (int c = sg; c < nsp; c += 4) {
        const float4v v = *reinterpret_cast<const float4v*>(op + (size_t)c * a.o_stride + k);
        const float wc = w[c];
        acc.x = fmaf(wc, v.x, acc.x);
        acc.y = fmaf(wc, v.y, acc.y);
        acc.z = fmaf(wc, v.z, acc.z);
        acc.w = fmaf(wc, v.w, acc.w);
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

  // ---- out = o_lat . B_v[:, 32 of the head's columns] / l: thread = (k part kp of 32, column quad cq of 8), 8-byte loads
  const int kp = tid >> 3, cq = tid & 7;
  const uint16_t* Bv = a.Bv + m.bv_off[j] + u * kDHead + quarter * 32 + cq * 4;
  const int k_per = rv >> 5;                       // rank is a multiple of 32
  float4v o = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
  for (int kk = 0; kk < k_per; ++kk) {
    const int k = kp * k_per + kk;
    const uint2v raw = *reinterpret_cast<const uint2v*>(Bv + (size_t)k * width);
    const float ol = olat[k];
    o.x = fmaf(ol, T::to_float((uint16_t)(raw.x & 0xffffu)), o.x);
    o.y = fmaf(ol, T::to_float((uint16_t)(raw.x >> 16)), o.y);
    o.z = fmaf(ol, T::to_float((uint16_t)(raw.y & 0xffffu)), o.z);
    o.w = fmaf(ol, T::to_float((uint16_t)(raw.y >> 16)), o.w);
  }
  *reinterpret_cast<float4v*>(part + (kp * 8 + cq) * 4) = o;
  __syncthreads();
  if (tid < 32) {
    const int c4 = tid >> 2, e = tid & 3;
    float s = 0.f;
#pragma unroll
    for (int g = 0; g < 32; ++g) s += part[(g * 8 + c4) * 4 + e];
    a.out[((size_t)b * m.n_heads + h) * kDHead + quarter * 32 + tid] = s / sum[0];
  }
}

#define PALU_VALUE_INST(T, HB, I4) template __global__ void value_kernel<T, HB, I4>(ValueArgs);
PALU_VALUE_INST(F16, 1, false)
PALU_VALUE_INST(F16, 2, false)
PALU_VALUE_INST(F16, 4, false)
PALU_VALUE_INST(F16, 1, true)
PALU_VALUE_INST(F16, 2, true)
PALU_VALUE_INST(F16, 4, true)
PALU_VALUE_INST(BF16, 1, false)
PALU_VALUE_INST(BF16, 2, false)
PALU_VALUE_INST(BF16, 4, false)
template __global__ void combine_kernel<F16>(CombineArgs);
template __global__ void combine_kernel<BF16>(CombineArgs);

}  // namespace palu
