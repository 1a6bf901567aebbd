// Scores without positional rotation (Sec. 3.1.2, Eq. 5): with no RoPE between
// the reconstruction and the query product, B_k moves to the query side,
//   q K^T = q (H_k B_k)^T = (q B_k^T) H_k^T,
// so the keys are never rebuilt: one small kernel folds the query into the
// latent space and the score is a matrix-vector product over the latents,
// bound by the latent stream alone (2 FLOP per latent element and head).
//
//   qfold_kernel  qt[b, unit][head, column] = q[b, head] . B_k[column, head's 128 features]
//                 for the columns of the head's own group, 0 elsewhere; kept as a pair of fp16
//                 numbers hi + lo (lo = the rounding error of hi), so that the folded query
//                 carries ~22 bits into the matrix cores and the logit error stays far below
//                 the tolerance for logits of any size (one fp16 number alone: ~3e-4 of the logit)
//   qk_kernel     scores[b, head, t] = H_k[b, t, unit columns] . qt[b, unit][head, :] * log2(e)/sqrt(d_h)
//
// qk_kernel: one wavefront owns a range of tokens of one (sequence, unit) and
// shares nothing with the others after the folded query has been staged in
// LDS.  v_mfma_f32_16x16x32_f16 with A = folded queries (rows = heads) and
// B = latents (k = latent channels, columns = 16 tokens): the contraction runs
// over the contiguous dimension of the cache, so a lane's 16-byte load is its
// operand as it stands.  Units are the value kernel's: up to 256 latent columns
// of up to 4 heads from adjacent small groups (the folded query is then block
// diagonal), or one whole group of up to 32 heads, walked in chunks of 256 columns.
//
// 4-bit latents: a lane's 16-byte load holds the 32 codes of a quarter of a
// quantization block; a code c enters the matrix cores as the exact fp16 number
// 1 + c/64 and the scale, zero-point and offset are applied to the block's sum per token:
//   sum_k s (c_k - z) qt_k = s (64 sum_k (1 + c_k/64) qt_k - (64 + z) sum_k qt_k).

#include "palu_dev.h"

namespace palu {

struct QkUnit {
  int32_t c0;          // first latent column
  int32_t q_off;       // element offset of the unit's [2][nh][wpad] folded-query matrices, hi then lo (per sequence)
  int32_t qs_off;      // float offset of its [nh][wpad / 128] block sums (int4)
  uint16_t h0;
  uint16_t ncols;      // multiple of 32
  uint16_t wpad;       // ncols rounded up to a multiple of 256: columns of the staged matrix
  uint8_t nh;          // at most 32
  uint8_t use_lo;      // unquantized latents: the score kernel also contracts the lo part (its staging fits the LDS)
};
constexpr int kMaxQkUnits = 64;
struct QkUnits {
  int n_units;
  QkUnit u[kMaxQkUnits];
};

struct QfoldArgs {
  const uint16_t* q;         // [batch, n_heads, 128]
  const uint16_t* Bk;
  uint16_t* qt;              // fp16 folded queries, per sequence stride qt_bstride
  float* qsum;               // per sequence stride qs_bstride
  long long qt_bstride, qs_bstride;
  int batch;
  int head0;                              // first head of this launch (blockIdx.y = head - head0)
  uint8_t unit_of_head[PALU_MAX_HEADS];   // index into units
  Meta meta;
  QkUnits units;
};

struct QkArgs {
  const void* hk;
  const uint16_t* hk_scale;
  const uint16_t* hk_zero;
  const uint16_t* qt;
  const float* qsum;
  const int32_t* seq_lens;
  float* scores;             // plane 0: [batch][n_heads][lpad]
  long long qt_bstride, qs_bstride;
  long long row_elems;       // R_k
  long long max_seq;
  int seq_len;
  int lpad;
  int batch;
  int n_heads;
  int split_tokens;          // tokens per wavefront (multiple of 32)
  int n_split;
  int n_blocks_q;
  int units_per_wg;          // 1, 2 or 4: the wavefronts of a workgroup take this many units of the same token ranges
  int lds_unit_stride;       // bytes of LDS per staged unit
  float scale;               // log2(e) / sqrt(d_h)
  QkUnits units;
};

// grid (wpad_max / 128, heads of the launch, batch / 4), 256 threads: a workgroup fills
// 128 columns of one head's row for four sequences; thread = (column, half of the
// features).  The B_k values are loaded once and reused for the four.
// (bx, by, bz): the workgroup's position in that grid.
template <typename T>
__device__ __forceinline__ void qfold_body(const QfoldArgs& a, int bx, int by, int bz) {
  __shared__ float blk[4][4];
  const Meta& m = a.meta;
  const int h = a.head0 + by;
  const QkUnit u = a.units.u[a.unit_of_head[h]];
  const int hh = h - u.h0;
  const int col0 = bx * 128;
  if (col0 >= u.wpad) return;
  const int tid = threadIdx.x, wave = tid >> 6;
  const int c = col0 + (tid >> 1);               // column inside the unit
  const int fh = (tid & 1) * 64;                  // first of this thread's 64 features
  const int cabs = u.c0 + c;                      // latent column
  const int j = group_of(m, h);
  const bool mine = c < u.ncols && cabs >= m.k_off[j] && cabs < m.k_off[j + 1];   // the same for both threads of a column
  uint4v bw[8];
#pragma unroll
  for (int x = 0; x < 8; ++x) bw[x] = uint4v{0, 0, 0, 0};
  if (mine) {
    int width;
    const int blk = weight_block(m, j, h, m.bk_off[j], &width);
    const uint16_t* Brow = a.Bk + blk + (size_t)(cabs - m.k_off[j]) * width + fh;
#pragma unroll
    for (int x = 0; x < 8; ++x) bw[x] = *reinterpret_cast<const uint4v*>(Brow + 8 * x);
  }
  // four sequences per workgroup, their query loads issued together
  const int b0 = bz * 4;
  const int nb = min(4, a.batch - b0);
  uint4v qw[4][8];
#pragma unroll
  for (int bb = 0; bb < 4; ++bb) {
    if (bb >= nb) break;                             // uniform
    const uint16_t* qp = a.q + q_row(m, b0 + bb, h) * kDHead + fh;
#pragma unroll
    for (int x = 0; x < 8; ++x) qw[bb][x] = *reinterpret_cast<const uint4v*>(qp + 8 * x);
  }
#pragma unroll
  for (int bb = 0; bb < 4; ++bb) {
    if (bb >= nb) break;                             // uniform: fewer than four sequences left
    float s = 0.f;
#pragma unroll
    for (int x = 0; x < 8; ++x) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        s = fmaf(T::to_float((uint16_t)(qw[bb][x][e] & 0xffffu)), T::to_float((uint16_t)(bw[x][e] & 0xffffu)), s);
        s = fmaf(T::to_float((uint16_t)(qw[bb][x][e] >> 16)), T::to_float((uint16_t)(bw[x][e] >> 16)), s);
      }
    }
    s += __shfl_xor(s, 1, 64);
    const uint16_t hv = F16::from_float(s);        // the contraction runs in fp16 whatever the storage type
    if ((tid & 1) == 0 && bb < nb) {
      uint16_t* dst = a.qt + (size_t)(b0 + bb) * a.qt_bstride + u.q_off + (size_t)hh * u.wpad + c;
      dst[0] = hv;
      dst[(size_t)u.nh * u.wpad] = F16::from_float(s - F16::to_float(hv));
    }
    // sum of the rounded values over this 128-column block (int4 zero-point term)
    float r = (tid & 1) == 0 ? F16::to_float(hv) : 0.f;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) r += __shfl_xor(r, off, 64);
    if ((tid & 63) == 0) blk[bb][wave] = r;
  }
  __syncthreads();
  if (tid < nb)
    a.qsum[(size_t)(b0 + tid) * a.qs_bstride + u.qs_off + (size_t)hh * (u.wpad >> 7) + bx] =
        (blk[tid][0] + blk[tid][1]) + (blk[tid][2] + blk[tid][3]);
}

template <typename T>
__global__ __launch_bounds__(256) void qfold_kernel(QfoldArgs a) {
  qfold_body<T>(a, blockIdx.x, blockIdx.y, blockIdx.z);
}

// T:  storage type of unquantized latents (bfloat16 converted to fp16 in registers)
// MT: 16-row head tiles (1: up to 16 heads, 2: up to 32)
// QB: latents are QB-bit codes (4, 3 or 2; 0: unquantized); I4 below means "quantized"
template <typename T, int MT, int QB>
__global__ __launch_bounds__(256, 2) void qk_kernel(QkArgs a) {
  constexpr bool I4 = QB != 0;                   // QB: bits per code of quantized latents (4, 3, 2), 0 for fp16 / bf16
  extern __shared__ __attribute__((aligned(16))) unsigned char qk_lds_all[];
  constexpr bool kIsBf16 = !__is_same(T, F16);
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 15, kq = lane >> 4;       // token column (B, D) or head row (A); quarter of the 32 channels of a k-step

  // grid (groups of units_per_wg units, groups of 4 / units_per_wg token ranges, batch); the wavefronts of a
  // workgroup take neighbouring units of the same token range first: they read neighbouring columns of the
  // same rows, and the scales and zero-points of a token's blocks, which lie side by side, come into this
  // compute unit's cache once instead of once per unit.
  const int upw = a.units_per_wg, b = blockIdx.z;
  const int unit = blockIdx.x * upw + (wave & (upw - 1));
  const bool has_unit = unit < a.units.n_units;                       // wavefront-uniform
  const QkUnit u = a.units.u[min(unit, a.units.n_units - 1)];
  asm volatile("" :: "s"(a.hk), "s"(a.qt), "s"(a.seq_lens), "s"(a.scores), "s"(a.qt_bstride), "s"(a.row_elems), "s"(a.max_seq),
               "s"(a.seq_len), "s"(a.lpad), "s"(a.n_heads), "s"(a.split_tokens), "s"(a.n_split), "s"(u.c0), "s"(u.q_off),
               "s"((int)u.h0), "s"((int)u.ncols), "s"((int)u.wpad), "s"((int)u.nh));   // all in registers here: one round trip
  const int nh = u.nh, wpad = u.wpad;
  const int pitch = wpad + 8;                    // halfs per staged row: 16 bytes of padding keep the 16 head rows on distinct banks
  const bool use_lo = !I4 && u.use_lo;           // uniform
  const int lo_rows = nh * pitch * 2;            // byte offset of the lo rows behind the hi rows
  unsigned char* const qk_lds = qk_lds_all + (wave & (upw - 1)) * a.lds_unit_stride;   // this wavefront's unit

  // ---- folded queries of the workgroup's units -> LDS (rows of heads beyond nh are never read: their lanes re-read row nh-1)
  for (int j = 0; j < upw; ++j) {
    const int uj = blockIdx.x * upw + j;
    if (uj >= a.units.n_units) break;              // uniform
    const QkUnit& v_u = a.units.u[uj];
    const int j_wpad = v_u.wpad, j_nh = v_u.nh, j_pitch = j_wpad + 8;
    const int j_rows = ((!I4 && v_u.use_lo) ? 2 : 1) * j_nh;
    const uint16_t* src = a.qt + (size_t)b * a.qt_bstride + v_u.q_off;
    unsigned char* dst = qk_lds_all + j * a.lds_unit_stride;
    const int cpr = j_wpad >> 3;                   // 16-byte chunks per row
    for (int i = tid; i < j_rows * cpr; i += 256) {
      const int r = i / cpr, cc = i - r * cpr;
      uint4v v = *reinterpret_cast<const uint4v*>(src + (size_t)r * j_wpad + cc * 8);
      if constexpr (I4) {
        // channels (0 .. 7) of a chunk in the order 0 4 1 5 2 6 3 7: the order in which the codes of one
        // 32-bit word leave the dequantizer below (perm: selector bytes 0-3 pick from the second operand)
        v = uint4v{__builtin_amdgcn_perm(v.z, v.x, 0x05040100u), __builtin_amdgcn_perm(v.z, v.x, 0x07060302u),
                   __builtin_amdgcn_perm(v.w, v.y, 0x05040100u), __builtin_amdgcn_perm(v.w, v.y, 0x07060302u)};
      }
      *reinterpret_cast<uint4v*>(dst + ((size_t)r * j_pitch + cc * 8) * 2) = v;
    }
    if constexpr (I4) {
      // the block sums [nh][wpad / 128] of the folded query behind its rows: read from LDS in the loop, they are
      // not in the queue of the memory loads (which return in order, so a wait for a value requested after
      // the next step's latents would wait for those latents too)
      const float* qs_src = a.qsum + (size_t)b * a.qs_bstride + v_u.qs_off;
      float* qs_dst = reinterpret_cast<float*>(dst + (size_t)j_nh * j_pitch * 2);
      for (int i = tid; i < j_nh * (j_wpad >> 7); i += 256) qs_dst[i] = qs_src[i];
    }
  }
  __syncthreads();
  if (!has_unit) return;                         // whole wavefront; no barrier below

  const int split = blockIdx.y * (4 / upw) + wave / upw;
  const int L = a.seq_lens ? min(a.seq_lens[b], a.seq_len) : a.seq_len;
  const int s0 = split * a.split_tokens;
  if (split >= a.n_split || s0 >= L) return;     // whole wavefront; no barrier below
  const int ntok = min(a.split_tokens, L - s0);
  const int n_sets = (ntok + 31) >> 5;           // 32 tokens: two tiles of 16
  const int last = ntok - 1;
  const int n_chunks = wpad >> 8;                // chunks of 256 columns
  const int ncols = u.ncols;

  const size_t row0 = (size_t)b * a.max_seq + s0;
  // quantized latents: 4-bit codes, or 2-bit fields followed (3 bits) by a plane of third bits at R/4 bytes
  constexpr int bits = I4 ? QB : 16;
  const unsigned row_bytes = (unsigned)a.row_elems * (unsigned)bits / 8u;
  const unsigned char* base = (const unsigned char*)a.hk + row0 * row_bytes + (I4 ? (bits == 4 ? u.c0 / 2 : u.c0 / 4) : u.c0 * 2);
  const unsigned hi_plane = (unsigned)a.row_elems / 4u + (unsigned)u.c0 / 8u - (unsigned)u.c0 / 4u;    // from `base` to the third bits
  const size_t sz_idx0 = I4 ? row0 * a.n_blocks_q + (u.c0 >> 7) : 0;
  const int n_blk = (ncols + 127) >> 7;

  constexpr int NL = I4 ? 2 : 8;                 // 16-byte loads per tile and chunk: int4 one per 128-column block, else one per 32 columns
  struct Step {
    uint4v h[2][NL];
    uint16_t sz[2];            // quantized: the lane's share of the step's scales and zero-points, as loaded (see issue())
  };
  // loads of (set, chunk); clamped to the last token / last valid columns (whose folded query is zero-padded)
  auto issue = [&](Step& st, int set, int chunk) {
    if constexpr (I4) {
      // Scales and zero-points of the step's 32 tokens x 2 blocks: the four lanes that share a token column split
      // them (lane quarter kq: tile kq / 2, scales or zero-points by kq % 2; both blocks), two 2-byte requests per
      // lane instead of eight, and hand them round in process().  These requests, 16 rows of 2 bytes each,
      // cost the memory pipeline as much as a 16-byte-per-lane latent request: eight of them per step made the
      // kernel half as slow again as the latent stream alone.
      const unsigned t = (unsigned)min(set * 32 + (kq >> 1) * 16 + n, last);
      const uint16_t* arr = (kq & 1) ? a.hk_zero : a.hk_scale;
#pragma unroll
      for (int x = 0; x < 2; ++x)
        st.sz[x] = arr[sz_idx0 + (size_t)t * a.n_blocks_q + min(chunk * 2 + x, n_blk - 1)];
    }
#pragma unroll
    for (int tau = 0; tau < 2; ++tau) {
      const unsigned t = (unsigned)min(set * 32 + tau * 16 + n, last);
#pragma unroll
      for (int x = 0; x < NL; ++x) {
        unsigned off;
        if (I4) {
          const int blkc = min(chunk * 2 + x, n_blk - 1);
          off = (unsigned)blkc * 64u + (unsigned)kq * 16u;
        } else {
          const int col = min(chunk * 256 + x * 32 + kq * 8, ncols - 8);
          off = (unsigned)col * 2u;
        }
        if constexpr (!I4 || bits == 4) {
          st.h[tau][x] = *reinterpret_cast<const uint4v*>(base + (size_t)(t * row_bytes + off));
        } else {
          // the lane's 32 codes: 8 bytes of two-bit fields (half the 4-bit offset), 4 bytes of third bits (a quarter)
          const unsigned char* p = base + (size_t)(t * row_bytes);
          const uint2v lo = *reinterpret_cast<const uint2v*>(p + (off >> 1));
          st.h[tau][x].x = lo.x;
          st.h[tau][x].y = lo.y;
          if constexpr (bits == 3) st.h[tau][x].z = *reinterpret_cast<const uint32_t*>(p + hi_plane + (off >> 2));
        }
      }
    }
  };

  const uint32_t fp16_ones = per_lane_constant(0x3c003c00u);
  float4v acc[MT][2];
  int qrow[MT];                                  // byte offset of this lane's head row in the staged matrix
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) qrow[mt] = min(mt * 16 + n, nh - 1) * pitch * 2;
  const float* qs_base = reinterpret_cast<const float*>(qk_lds + (size_t)nh * pitch * 2);     // staged block sums (quantized latents)

  auto process = [&](Step& st, int set, int chunk) {
    if (chunk == 0) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int tau = 0; tau < 2; ++tau) acc[mt][tau] = float4v{0.f, 0.f, 0.f, 0.f};
    }
    if constexpr (!I4) {
#pragma unroll
      for (int x = 0; x < 8; ++x) {
        half8 af[MT], al[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          af[mt] = *reinterpret_cast<const half8*>(qk_lds + qrow[mt] + (chunk * 256 + x * 32 + kq * 8) * 2);
          if (use_lo) al[mt] = *reinterpret_cast<const half8*>(qk_lds + lo_rows + qrow[mt] + (chunk * 256 + x * 32 + kq * 8) * 2);
        }
#pragma unroll
        for (int tau = 0; tau < 2; ++tau) {
          uint4v hw = st.h[tau][x];
          if constexpr (kIsBf16) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              hw[e] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(__builtin_bit_cast(float, hw[e] << 16),
                                                                              __builtin_bit_cast(float, hw[e] & 0xffff0000u)));
          }
          const half8 bop = __builtin_bit_cast(half8, hw);
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            acc[mt][tau] = __builtin_amdgcn_mfma_f32_16x16x32_f16(af[mt], bop, acc[mt][tau], 0, 0, 0);
            if (use_lo) acc[mt][tau] = __builtin_amdgcn_mfma_f32_16x16x32_f16(al[mt], bop, acc[mt][tau], 0, 0, 0);
          }
        }
      }
    } else {
      // the step's scales and zero-points from the four lanes of this token column: [2 tau + (0: scales, 1: zero-points)],
      // block x in bits 16 x .. 16 x + 15
      uint32_t szv[4];
      {
        const int own = (int)((uint32_t)st.sz[0] | ((uint32_t)st.sz[1] << 16));
#pragma unroll
        for (int k4 = 0; k4 < 4; ++k4) szv[k4] = (uint32_t)__builtin_amdgcn_ds_bpermute((n + 16 * k4) * 4, own);
      }
#pragma unroll
      for (int x = 0; x < 2; ++x) {                // quantization block chunk*2 + x
        const int blkc = min(chunk * 2 + x, n_blk - 1);
        half8 af[MT][4];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int jj = 0; jj < 4; ++jj)            // lane's codes 8jj .. 8jj+7 are channels blk*128 + kq*32 + 8jj ..
            af[mt][jj] = *reinterpret_cast<const half8*>(qk_lds + qrow[mt] + ((chunk * 2 + x) * 128 + kq * 32 + jj * 8) * 2);
        float4v qs[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int r = 0; r < 4; ++r)
            qs[mt][r] = qs_base[(size_t)min(mt * 16 + 4 * kq + r, nh - 1) * (wpad >> 7) + blkc];
#pragma unroll
        for (int tau = 0; tau < 2; ++tau) {
          float4v d[MT];
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) d[mt] = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) {
            uint32_t w = st.h[tau][x][jj];
            if constexpr (bits != 4)
              w = expand_low_bits(st.h[tau][x][jj >> 1] >> (16 * (jj & 1)), st.h[tau][x][2] >> (8 * jj), bits == 3);
            // code c of channel u sits in bits 4u .. 4u+3; moved to mantissa bits 4 .. 7 of 0x3c00 it is the fp16
            // number 1 + c/64 (exact).  Channels u and u + 4 are 16 bits apart, i.e. already in the two halves of
            // one operand register: one shift and one masked merge per register, and the k order 0 4 1 5 2 6 3 7,
            // which is the order the folded query was staged in.  The offset is undone on the block's sum below.
            const NibblePairs np = nibbles_to_fp16_pairs(w, fp16_ones);
            const uint4v bw = {np.p[0], np.p[1], np.p[2], np.p[3]};
            const half8 bop = __builtin_bit_cast(half8, bw);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) d[mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(af[mt][jj], bop, d[mt], 0, 0, 0);
          }
          const float sc = chunk * 2 + x < n_blk ? F16::to_float((uint16_t)(szv[2 * tau] >> (16 * x))) : 0.f;
          const float zp = F16::to_float((uint16_t)(szv[2 * tau + 1] >> (16 * x)));
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 4; ++r)      // d = sum qt (1 + c/64): sum qt (c - z) = 64 d - (64 + z) sum qt
              acc[mt][tau][r] = fmaf(sc, fmaf(-(zp + 64.f), qs[mt][r], 64.f * d[mt][r]), acc[mt][tau][r]);
        }
      }
    }
    if (chunk == n_chunks - 1) {
      // accumulator row 4*kq + r (+16 per tile of heads) = head of the unit, column n = token of the tile
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int hh = mt * 16 + 4 * kq + r;
          if (hh >= nh) continue;
          float* row = a.scores + ((size_t)b * a.n_heads + u.h0 + hh) * a.lpad + s0 + set * 32 + n;
          row[0] = acc[mt][0][r] * a.scale;         // tokens past the end fall into the padding of the score row
          row[16] = acc[mt][1][r] * a.scale;
        }
    }
  };

  // steps (set, chunk) in order, kDepth register sets in turn: the loads of the next kDepth - 1 steps are in
  // flight while one is consumed (four steps deep measured slower for quantized latents).  Every request is
  // unconditional (past the last step the clamped addresses re-read the last token, and nothing consumes
  // them): with a request under a branch the wait in front of process() would have to cover both ways of
  // reaching it, i.e. every load in flight, and nothing would be prefetched.
  const int n_steps = n_sets * n_chunks;
  auto next = [&](int& set, int& chunk) { if (++chunk == n_chunks) { chunk = 0; ++set; } };
  constexpr int kDepth = 2;
  Step ring[kDepth];
  int is = 0, ic = 0, ps = 0, pc = 0;            // next step to request / to consume
#pragma unroll
  for (int d = 0; d < kDepth - 1; ++d) { issue(ring[d], is, ic); next(is, ic); }
  for (int k = 0; k < n_steps; k += kDepth) {
#pragma unroll
    for (int d = 0; d < kDepth; ++d) {
      issue(ring[(d + kDepth - 1) % kDepth], is, ic); next(is, ic);
      __builtin_amdgcn_sched_barrier(0);           // the requests stay in front of the work that hides them
      if (d == 0 || k + d < n_steps) { process(ring[d], ps, pc); next(ps, pc); }     // uniform
    }
  }
}

template __global__ void qfold_kernel<F16>(QfoldArgs);
template __global__ void qfold_kernel<BF16>(QfoldArgs);
#define PALU_QK_INST(T, I4)                                   \
  template __global__ void qk_kernel<T, 1, I4>(QkArgs);       \
  template __global__ void qk_kernel<T, 2, I4>(QkArgs);
PALU_QK_INST(F16, 0)
PALU_QK_INST(BF16, 0)
PALU_QK_INST(F16, 4)
PALU_QK_INST(F16, 3)
PALU_QK_INST(F16, 2)

}  // namespace palu
