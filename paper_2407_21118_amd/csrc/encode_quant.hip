// Cache-append side: down-projection h = x A (Sec. 3.1) for a handful of new
// tokens, and the 4-bit asymmetric quantizer of Appendix A.
//
// At decode time the projection reads all of A (d x R) for n_tok = batch
// tokens: a weight-streaming problem (HBM-bound, 2*n_tok FLOP per weight
// element), so it is a split-K float32 FMA kernel on 16-byte coalesced loads
// followed by a small reduction that rounds once and scatters the rows.

#pragma once

#include "palu_dev.h"

namespace palu {

constexpr int kEncRows = 64;      // rows of A per workgroup (16 per wavefront)
constexpr int kEncCols = 512;     // columns of A per workgroup (8 per lane)
constexpr int kEncTokMax = 8;     // most tokens accumulated per pass over the weights

struct EncodeSide {
  const uint16_t* A;       // [d, R]
  float* partial;          // [k_splits][n_tok][R]
  uint16_t* latent;
  long long row_stride;
  int R;
  uint8_t* codes;          // fused quantization (GEMM path only): packed codes, rows of R/2 bytes ...
  uint16_t* scale;         // ... and the fp16 (scale, zero) pairs, rows of R/128
  uint16_t* zero;
};
struct EncodeArgs {
  const uint16_t* x;       // [n_tok, d]
  const int32_t* dst_row;
  EncodeSide side[2];      // key and value caches; blockIdx.z selects (one launch may cover both)
  int n_tok, d, k_splits;
};

// The prompt-sized projection (encode_gemm.hip, compiled on its own): C[n_tok, R] = X A on the matrix
// cores for the one or two sides of `a`, quantized in place of stored when `quant`.
// tile_opt: token rows per workgroup (0 = by the number of tokens); n_cu: compute units of the device.
int launch_encode_gemm_tiles(int act, const EncodeArgs& a, int max_R, int n_sides, bool quant, int tile_opt, int n_cu,
                             hipStream_t s);

// grid (ceil(max R / 512), d / 64, sides), 256 threads.
// kEncTok: tokens accumulated per pass over the weights (1, 2, 4 or 8: a decode
// step of one sequence should not pay for eight).
// (bx, by, bz): the workgroup's position in that grid (the kernel below passes blockIdx; the fused
// first launch of a decode step runs the same body next to the query fold)
// while_loading(): work of the whole workgroup that is independent of the projection, run after the
// weight loads have been issued, in the shadow of their latency (the fused decode step folds the query there)
struct NoExtraWork {
  __device__ __forceinline__ void operator()() const {}
};
template <typename T, int kEncTok, typename Extra = NoExtraWork>
__device__ __forceinline__ void encode_partial_body(const EncodeArgs& a, int bx, int by, int bz, Extra while_loading = Extra{}) {
  __shared__ float xs[kEncTok][kEncRows];
  __shared__ float red[3][kEncTok][kEncCols];     // wavefronts 1..3 hand their sums to wavefront 0
  const EncodeSide sd = a.side[bz];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int c0 = bx * kEncCols + lane * 8;
  const int k0 = by * kEncRows;
  const bool col_ok = c0 < sd.R;                  // R is a multiple of 32, so 8 columns are all in or all out
  if (bx * kEncCols >= sd.R) {                    // uniform
    while_loading();
    return;
  }

  // the weight rows go out first: they are the long-latency HBM stream and do
  // not depend on the activations
  uint4v wraw[16];
#pragma unroll
  for (int kk = 0; kk < 16; ++kk) {
    const int k = wave * 16 + kk;
    wraw[kk] = col_ok ? *reinterpret_cast<const uint4v*>(sd.A + (size_t)(k0 + k) * sd.R + c0) : uint4v{0, 0, 0, 0};
  }
  while_loading();

  for (int tb = 0; tb < a.n_tok; tb += kEncTok) {
    const int nt = min(kEncTok, a.n_tok - tb);
    __syncthreads();
    for (int i = tid; i < kEncTok * kEncRows; i += 256) {
      const int t = i / kEncRows, k = i - t * kEncRows;
      xs[t][k] = t < nt ? T::to_float(a.x[(size_t)(tb + t) * a.d + k0 + k]) : 0.f;
    }
    __syncthreads();
    float acc[kEncTok][8];
#pragma unroll
    for (int t = 0; t < kEncTok; ++t)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[t][e] = 0.f;
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      const int k = wave * 16 + kk;
      float wv[8];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        wv[2 * e] = T::to_float((uint16_t)(wraw[kk][e] & 0xffffu));
        wv[2 * e + 1] = T::to_float((uint16_t)(wraw[kk][e] >> 16));
      }
#pragma unroll
      for (int t = 0; t < kEncTok; ++t) {
        const float xv = xs[t][k];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[t][e] = fmaf(xv, wv[e], acc[t][e]);
      }
    }
    if (wave > 0) {
#pragma unroll
      for (int t = 0; t < kEncTok; ++t)
#pragma unroll
        for (int e = 0; e < 8; ++e) red[wave - 1][t][e * 64 + lane] = acc[t][e];
    }
    __syncthreads();
    if (wave == 0 && col_ok) {
#pragma unroll
      for (int t = 0; t < kEncTok; ++t) {
        if (t >= nt) break;
        float* dst = sd.partial + ((size_t)by * a.n_tok + tb + t) * sd.R + c0;
        float4v o0, o1;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float s = acc[t][e] + red[0][t][e * 64 + lane] + red[1][t][e * 64 + lane] + red[2][t][e * 64 + lane];
          if (e < 4) o0[e] = s; else o1[e - 4] = s;
        }
        *reinterpret_cast<float4v*>(dst) = o0;
        *reinterpret_cast<float4v*>(dst + 4) = o1;
      }
    }
  }
}

template <typename T, int kEncTok>
__global__ __launch_bounds__(256) void encode_partial_kernel(EncodeArgs a) {
  encode_partial_body<T, kEncTok>(a, blockIdx.x, blockIdx.y, blockIdx.z);
}

// Sums the split-K partials in a fixed order, rounds once, scatters the rows.
// Workgroup = 64 columns of one token; thread = (quarter of the splits, column).
// grid (ceil(max R / 64), n_tok, sides), 256 threads.
template <typename T>
__global__ __launch_bounds__(256) void encode_finish_kernel(EncodeArgs a) {
  __shared__ float part[4][64];
  const EncodeSide sd = a.side[blockIdx.z];
  if ((int)blockIdx.x * 64 >= sd.R) return;       // uniform
  const int tid = threadIdx.x;
  const int c = blockIdx.x * 64 + (tid & 63), t = blockIdx.y, sub = tid >> 6;
  const int per = (a.k_splits + 3) / 4;
  float s = 0.f;
  if (c < sd.R) {
    const float* p = sd.partial + (size_t)t * sd.R + c;
#pragma unroll 8
    for (int ks = sub * per; ks < min((sub + 1) * per, a.k_splits); ++ks) s += p[(size_t)ks * a.n_tok * sd.R];
  }
  part[sub][tid & 63] = s;
  __syncthreads();
  if (tid < 32 && (int)blockIdx.x * 64 + tid * 2 < sd.R) {
    const int cc = tid * 2;
    const float s0 = (part[0][cc] + part[1][cc]) + (part[2][cc] + part[3][cc]);
    const float s1 = (part[0][cc + 1] + part[1][cc + 1]) + (part[2][cc + 1] + part[3][cc + 1]);
    const long long row = a.dst_row ? a.dst_row[t] : t;
    uint32_t* dst = reinterpret_cast<uint32_t*>(sd.latent + row * sd.row_stride + blockIdx.x * 64 + cc);
    *dst = (uint32_t)T::from_float(s0) | ((uint32_t)T::from_float(s1) << 16);
  }
}

// ---- the same projection from transposed weights At [R, d] (column c of A contiguous): a wavefront owns
// kTCols columns and all of k, so a column's sum is finished inside the wavefront, in one launch, with no
// partial sums in memory.  Workgroup = 4 wavefronts = 4 kTCols columns of one side; every weight load of
// the wavefront (kTCols x 8 chunks of 1 KiB) goes out before anything else.
constexpr int kTCols = 2;          // columns per wavefront (4 for passes of 4 or 8 tokens was slower: half the workgroups)
constexpr int kTBlock = 4096;      // k per batch of loads: 8 chunks of 64 lanes x 8
struct EncodeTArgs {
  const uint16_t* x;               // [n_tok, d]
  const int32_t* dst_row;
  const uint16_t* At[2];           // [R, d]
  uint16_t* latent[2];
  long long row_stride[2];
  int R[2];
  int n_tok, d, wg_side1;          // workgroups below wg_side1 work on side 0
};
// acc + sum of the 8 products of two packed 16-byte operands
template <typename T>
__device__ __forceinline__ float dot8(const uint4v& w, const uint4v& x, float acc) {
  if constexpr (__is_same(T, F16)) {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t we = w[e], xe = x[e];                       // named copies: a bit cast applied to a vector element reads element 0
      acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(h2, we), __builtin_bit_cast(h2, xe), acc, false);
    }
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      acc = fmaf(T::to_float((uint16_t)(x[e] & 0xffffu)), T::to_float((uint16_t)(w[e] & 0xffffu)), acc);
      acc = fmaf(T::to_float((uint16_t)(x[e] >> 16)), T::to_float((uint16_t)(w[e] >> 16)), acc);
    }
  }
  return acc;
}

// wg_id: the workgroup's index in the projection's grid of wg_side1 + ceil(R_v / (4 kTCols)) workgroups
// while_loading(): as for encode_partial_body
template <typename T, int TOK, typename Extra = NoExtraWork>
__device__ __forceinline__ void encode_t_body(const EncodeTArgs& a, int wg_id, Extra while_loading = Extra{}) {
  extern __shared__ __attribute__((aligned(16))) unsigned char enct_lds[];
  uint16_t* xs = reinterpret_cast<uint16_t*>(enct_lds);          // [TOK][d]
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int side = wg_id >= a.wg_side1 ? 1 : 0;
  const int wg = wg_id - (side ? a.wg_side1 : 0);
  const int R = a.R[side];
  const int c0 = (wg * 4 + wave) * kTCols;                       // R is a multiple of 32: a wavefront's columns are all in or all out
  const bool cols_ok = c0 < R;
  const uint16_t* At = a.At[side] + (size_t)min(c0, R - kTCols) * a.d;
  for (int tb = 0; tb < a.n_tok; tb += TOK) {
    float acc[kTCols][TOK];
#pragma unroll
    for (int c = 0; c < kTCols; ++c)
#pragma unroll
      for (int t = 0; t < TOK; ++t) acc[c][t] = 0.f;
    for (int kb = 0; kb < a.d; kb += kTBlock) {
      // One or two tokens: a lane needs only its own k of x, the same for every column, and takes them straight
      // from memory ahead of the weights (loads return in order: behind the weights they would cost a second
      // round trip).  More tokens would not fit the registers and go through LDS.
      constexpr bool kDirect = TOK <= 2;
      uint4v xd[kDirect ? TOK : 1][8];
      if constexpr (kDirect) {
#pragma unroll
        for (int t = 0; t < TOK; ++t)
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            const int k = kb + (i * 64 + lane) * 8;
            xd[t][i] = (k < a.d && tb + t < a.n_tok) ? *reinterpret_cast<const uint4v*>(a.x + (size_t)(tb + t) * a.d + k) : uint4v{0, 0, 0, 0};
          }
      }
      uint4v w[kTCols][8];
#pragma unroll
      for (int c = 0; c < kTCols; ++c)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int k = kb + (i * 64 + lane) * 8;
          w[c][i] = k < a.d ? *reinterpret_cast<const uint4v*>(At + (size_t)c * a.d + k) : uint4v{0, 0, 0, 0};
        }
      if (kb == 0) {
        if (tb == 0) while_loading();
        if constexpr (!kDirect) {
          __syncthreads();                                       // the previous pass has read xs
          const int nt = min(TOK, a.n_tok - tb);
          for (int i = tid; i < TOK * (a.d >> 3); i += 256) {
            const int t = i / (a.d >> 3), k8 = i - t * (a.d >> 3);
            reinterpret_cast<uint4v*>(xs)[i] = t < nt ? reinterpret_cast<const uint4v*>(a.x + (size_t)(tb + t) * a.d)[k8] : uint4v{0, 0, 0, 0};
          }
          __syncthreads();
        }
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int k = kb + (i * 64 + lane) * 8;
        if (k >= a.d) continue;
#pragma unroll
        for (int t = 0; t < TOK; ++t) {
          uint4v xv;
          if constexpr (kDirect) xv = xd[t][i];
          else xv = *reinterpret_cast<const uint4v*>(xs + (size_t)t * a.d + k);
#pragma unroll
          for (int c = 0; c < kTCols; ++c) acc[c][t] = dot8<T>(w[c][i], xv, acc[c][t]);
        }
      }
    }
#pragma unroll
    for (int c = 0; c < kTCols; ++c)
#pragma unroll
      for (int t = 0; t < TOK; ++t) {
        float v = acc[c][t];
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
        if (lane == 0 && cols_ok && tb + t < a.n_tok) {
          const long long row = a.dst_row ? a.dst_row[tb + t] : tb + t;
          a.latent[side][row * a.row_stride[side] + c0 + c] = T::from_float(v);
        }
      }
  }
}

template <typename T, int TOK>
__global__ __launch_bounds__(256) void encode_t_kernel(EncodeTArgs a) {
  encode_t_body<T, TOK>(a, blockIdx.x);
}

// The quantizer of Appendix A with B = 4 (s = (max-min)/(2^B-1), z = round(-min/s),
// code = clamp(round(x/s) + z, 0, 2^B-1)) for one (token, 128-channel block).
// Every arithmetic step is a single IEEE float32 operation so the integer codes are
// reproducible bit for bit; scale and zero are stored as fp16 and used as stored.
struct QuantParams {
  float sf, zf, top;
  uint16_t s16, z16;
};
// top = 2^B - 1: 15 for the 4-bit cache, 7 and 3 for the 3- and 2-bit settings of Sec. 4.4
__device__ __forceinline__ QuantParams quant_params(float mn, float mx, float top = 15.0f) {
  QuantParams p;
  p.top = top;
  const float s32 = __fdiv_rn(__fsub_rn(mx, mn), top);
  p.s16 = F16::from_float(s32);
  if ((p.s16 & 0x7fffu) == 0) p.s16 = 0x3c00u;                  // s == 0 -> 1
  p.sf = F16::to_float(p.s16);
  float z = rintf(__fdiv_rn(-mn, p.sf));
  z = fminf(fmaxf(z, -65504.0f), 65504.0f);
  p.z16 = F16::from_float(z);
  p.zf = F16::to_float(p.z16);
  return p;
}
__device__ __forceinline__ uint32_t quant_code(float x, const QuantParams& p) {
  return (uint32_t)fminf(fmaxf(__fadd_rn(rintf(__fdiv_rn(x, p.sf)), p.zf), 0.0f), p.top);
}

struct QuantArgs {
  const uint16_t* latent;
  uint8_t* codes;
  uint16_t* scale;
  uint16_t* zero;
  const int32_t* dst_row;     // output row of token t (NULL: t)
  long long row_stride;
  int n_tok, R, n_blocks;     // n_blocks = R / 128
  int bits;                   // 4, 3 or 2
};

// One wavefront per (token, 128-channel block); lane l owns channels 2l, 2l+1.
template <typename T>
__global__ __launch_bounds__(256) void quant_kernel(QuantArgs a) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const long long item = (long long)blockIdx.x * 4 + wave;
  if (item >= (long long)a.n_tok * a.n_blocks) return;
  const int t = (int)(item / a.n_blocks), blk = (int)(item - (long long)t * a.n_blocks);
  const uint32_t raw = *reinterpret_cast<const uint32_t*>(a.latent + (size_t)t * a.row_stride + blk * 128 + lane * 2);
  const float x0 = T::to_float((uint16_t)(raw & 0xffffu));
  const float x1 = T::to_float((uint16_t)(raw >> 16));
  float mn = fminf(x0, x1), mx = fmaxf(x0, x1);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    mn = fminf(mn, __shfl_xor(mn, off, 64));
    mx = fmaxf(mx, __shfl_xor(mx, off, 64));
  }
  const QuantParams qp = quant_params(mn, mx, (float)((1 << a.bits) - 1));
  const size_t orow = a.dst_row ? (size_t)a.dst_row[t] : (size_t)t;
  const uint32_t c0 = quant_code(x0, qp), c1 = quant_code(x1, qp);
  if (a.bits == 4) {
    a.codes[orow * (a.R / 2) + blk * 64 + lane] = (uint8_t)(c0 | (c1 << 4));
  } else {
    // 2 bits: byte k of a row holds channels 4k .. 4k+3 (lanes 2k, 2k+1).  3 bits: the low two bits of every
    // code in that layout, then the third bits, byte k holding channels 8k .. 8k+7 (lanes 4k .. 4k+3).
    uint8_t* row = a.codes + orow * (size_t)(a.R * a.bits / 8);
    const uint32_t lo = (c0 & 3u) | ((c1 & 3u) << 2);
    const uint32_t lo_n = __shfl_xor(lo, 1, 64);
    if ((lane & 1) == 0) row[blk * 32 + (lane >> 1)] = (uint8_t)(lo | (lo_n << 4));
    if (a.bits == 3) {
      uint32_t hi = (c0 >> 2) | ((c1 >> 2) << 1);                  // 2 bits: this lane's channels
      hi |= __shfl_xor(hi, 1, 64) << 2;                            // even lanes: 4 bits
      hi |= __shfl_xor(hi, 2, 64) << 4;                            // lanes 4k: 8 bits
      if ((lane & 3) == 0) row[a.R / 4 + blk * 16 + (lane >> 2)] = (uint8_t)hi;
    }
  }
  if (lane == 0) {
    a.scale[orow * a.n_blocks + blk] = qp.s16;
    a.zero[orow * a.n_blocks + blk] = qp.z16;
  }
}

}  // namespace palu
