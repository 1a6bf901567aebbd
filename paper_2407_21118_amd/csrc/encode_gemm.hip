// Cache-append side for many tokens at once: the prompt-sized down-projection
// h = x A (Sec. 3.1), optionally quantized as it is stored (Sec. 3.4, Appendix A).
//
// This file is a translation unit of its own: encode_gemm_kernel keeps up to 256
// accumulators per lane in the accumulation registers, while the rest of the library is
// compiled with the matrix instructions writing ordinary vector registers, an option that
// applies to a whole compilation and that this kernel does not fit.

#include "encode_quant.hip"

namespace palu {

// A tiled GEMM on the matrix cores, C[n_tok, R] = X[n_tok, d] A[d, R].  Workgroup = TM x 256 outputs (TM = 256, or
// 128 / 64 for shorter prompts), four wavefronts of TM/2 x 128 (TM/64 x 4 tiles of
// v_mfma_f32_32x32x16), one per SIMD with up to 256 accumulator registers.  k advances
// in stages of 64 through two LDS buffers: while a stage is multiplied, the next one
// (already in registers) is written to the other buffer and the one after it is
// requested from memory, so a stage's loads have a whole stage of matrix work to
// arrive and there is one barrier per stage.  X is k-contiguous, which is what an MFMA
// operand wants; A is column-contiguous, so each thread loads one 8-column chunk of 8
// consecutive k and transposes the 8 x 8 block in registers (one byte permute per
// operand register) on its way to LDS.  The finished tile goes through LDS once more,
// so that rows leave in 16-byte pieces (or as codes, QUANT).
//
// Workgroups are numbered so that each of the 8 XCDs (workgroup id mod 8) owns a
// contiguous range of the tiles, columns fastest: the column tiles of a token row share
// their X rows through that XCD's L2.
// output columns per workgroup: 256, or 128 with the 64-row tile where even that leaves compute units idle
constexpr int kGemmK = 64;                     // k per stage
constexpr int kGemmPitch = kGemmK + 8;         // halfs per LDS row: 16-byte reads of 16 consecutive rows hit distinct banks
// token rows per workgroup: 256, or 128 / 64 while the taller tile would leave compute units without a workgroup

constexpr size_t gemm_lds_bytes(int tm, int tn) {
  const size_t stages = (size_t)2 * (tm + tn) * kGemmPitch * 2, out = (size_t)tm * (tn + 8) * 2;
  return stages > out ? stages : out;
}

struct GemmGrid {
  int n_col_tiles, n_row_tiles, n_tiles, per_xcd;     // tiles: sides x row tiles x column tiles
};

// QUANT: every 128 columns of the tile are exactly one quantization block per token, so the
// workgroup quantizes its rounded outputs in place of storing them (Sec. 3.4 applied
// while the cache is filled): codes, scales and zero-points are the ones quant_kernel
// gives for the latents the plain kernel stores.
// grid (8 * per_xcd), 256 threads, gemm_lds_bytes(TM, TN) of LDS.
template <typename T, bool QUANT, int TM, int TN>
__global__ __launch_bounds__(256) void encode_gemm_kernel(EncodeArgs a, GemmGrid gg) {
  extern __shared__ __attribute__((aligned(16))) unsigned char gemm_lds[];
  constexpr int MI = TM / 64;                                            // 32-row tiles of a wavefront
  constexpr int XC = TM / 32;                                            // 16-byte X chunks per thread and stage
  constexpr int NJ = TN / 64;                                            // 32-column tiles of a wavefront
  constexpr int kOutPitch = TN + 8;                                      // halfs per row of the output tile
  constexpr int kAL = TN == 256 ? 8 : 4;                                 // 16-byte A loads per thread and stage
  constexpr int kBufHalfs = (TM + TN) * kGemmPitch;
  uint16_t* lds16 = reinterpret_cast<uint16_t*>(gemm_lds);

  const int tile = (blockIdx.x & 7) * gg.per_xcd + (blockIdx.x >> 3);
  if ((int)(blockIdx.x >> 3) >= gg.per_xcd || tile >= gg.n_tiles) return;          // uniform
  const int per_side = gg.n_col_tiles * gg.n_row_tiles;
  const int side = tile / per_side, in_side = tile - side * per_side;
  const int row_tile = in_side / gg.n_col_tiles, col_tile = in_side - row_tile * gg.n_col_tiles;
  const EncodeSide sd = a.side[side];
  const int n0 = col_tile * TN, m0 = row_tile * TM;
  if (n0 >= sd.R) return;                                                // uniform
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lane_lo = lane & 31, lane_hi = lane >> 5;
  const int wm = (wave >> 1) * (TM / 2), wn = (wave & 1) * (TN / 2);     // this wavefront's corner of the tile

  // staging roles.  X: 16-byte piece lane % 8 of the stage's 64 k of row x_row(i) (i < XC): the 16 lanes of a store
  // pass hold rows r and r + 8, whose pieces lie 32 banks apart with this pitch (neighbouring rows overlap by 4 banks).
  // A, 256 columns: one (k-octet oct, 8-column chunk cc) item per thread: rows k0 + 8 oct + j (j < 8), columns
  // n0 + 8 cc ..; 128 columns: half an octet per thread (quad = tid / 16: rows k0 + 4 quad + j, j < 4).
  const int quad = tid >> 4;
  const int oct = TN == 256 ? tid >> 5 : quad >> 1, cc = TN == 256 ? tid & 31 : tid & 15;
  const int a_col = min(n0 + cc * 8, sd.R - 8);                          // R is a multiple of 32: clamped chunks are never stored
  const uint16_t* x_base = a.x + (size_t)m0 * a.d;
  unsigned x_off[XC];                                                    // rows past the last token re-read it; they are never stored
  auto x_row = [&](int i) { return 16 * (wave + 4 * (i >> 1)) + 4 * (i & 1) + (lane >> 4) + 8 * ((lane >> 3) & 1); };
#pragma unroll
  for (int i = 0; i < XC; ++i)
    x_off[i] = (unsigned)min(x_row(i), a.n_tok - 1 - m0) * (unsigned)a.d + (unsigned)(lane & 7) * 8u;
  const uint16_t* a_src = sd.A + (size_t)(TN == 256 ? oct * 8 : quad * 4) * sd.R + a_col;
  // the stage after the one being multiplied waits in these registers; the one after that is requested as
  // soon as they have been written to LDS
  uint4v xr[XC], ar[kAL];
  auto fetch_x = [&](int stage) {
#pragma unroll
    for (int i = 0; i < XC; ++i) xr[i] = *reinterpret_cast<const uint4v*>(x_base + x_off[i] + stage * kGemmK);
  };
  auto fetch_a = [&](int stage) {
#pragma unroll
    for (int j = 0; j < kAL; ++j) ar[j] = *reinterpret_cast<const uint4v*>(a_src + (size_t)(stage * kGemmK + j) * sd.R);
  };
  auto stash_x = [&](int buf) {
    uint16_t* Xs = lds16 + buf * kBufHalfs;
#pragma unroll
    for (int i = 0; i < XC; ++i) *reinterpret_cast<uint4v*>(Xs + x_row(i) * kGemmPitch + (lane & 7) * 8) = xr[i];
  };
  auto stash_a = [&](int buf) {
    uint16_t* As = lds16 + buf * kBufHalfs + TM * kGemmPitch;
    // 8 x 8 transpose: column e of the chunk over the 8 k rows, as four (k, k+1) pairs
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      uint4v t;
#pragma unroll
      for (int jp = 0; jp < kAL / 2; ++jp)
        t[jp] = __builtin_amdgcn_perm(ar[2 * jp + 1][e >> 1], ar[2 * jp][e >> 1], (e & 1) ? 0x07060302u : 0x05040100u);
      // the 16-byte k-octets of a row are stored XOR-swizzled by bits 3..5 of the row number (its chunk
      // number): the lanes of a store pass (chunks, rows 8 apart) would otherwise share two bank groups
      uint16_t* dst = As + (cc * 8 + e) * kGemmPitch + ((oct ^ cc) & 7) * 8;
      if constexpr (TN == 256) *reinterpret_cast<uint4v*>(dst) = t;
      else *reinterpret_cast<uint2v*>(dst + (quad & 1) * 4) = uint2v{t[0], t[1]};
    }
  };
  // read side of the swizzle: k-step ks reads octet 2 ks + lane_hi of row n, stored at octet ^ ((n >> 3) & 7)
  int a_row[NJ], a_swz[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int n = wn + 32 * j + lane_lo;
    a_row[j] = n * kGemmPitch;
    a_swz[j] = (n >> 3) & 7;
  }

  float16v acc[MI][NJ];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // operand registers of one k-step (16 k); two sets, so that a k-step's reads are in flight
  // while the previous one is multiplied (one wavefront per SIMD: nobody else hides them)
  typename T::vec8 xa[2][MI], ab[2][NJ];
  auto read_step = [&](int set, int buf, int ks) {
    const uint16_t* Xs = lds16 + buf * kBufHalfs;
    const uint16_t* As = Xs + TM * kGemmPitch;
#pragma unroll
    for (int i = 0; i < MI; ++i)
      xa[set][i] = *reinterpret_cast<const typename T::vec8*>(Xs + (wm + 32 * i + lane_lo) * kGemmPitch + ks * 16 + lane_hi * 8);
#pragma unroll
    for (int j = 0; j < NJ; ++j)
      ab[set][j] = *reinterpret_cast<const typename T::vec8*>(As + a_row[j] + (((2 * ks + lane_hi) ^ a_swz[j]) * 8));
  };

  auto multiply = [&](int set) {
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < NJ; ++j) acc[i][j] = T::mfma(xa[set][i], ab[set][j], acc[i][j]);
  };
  // One stage: four k-steps, each with the next step's operand reads in flight.  The first writes the X rows of
  // stage s + 1 from their registers to the other LDS buffer (last read before the previous barrier), the second
  // requests those of stage s + 2 into the same registers; the third and fourth do the same for A.  The
  // scheduling barriers keep this order (left alone, the compiler sinks the loads to the end of the stage and
  // hoists their use to its start), and inside a k-step the other work is dealt out one piece per matrix
  // instruction: a wavefront is alone on its SIMD, so whatever it issues in a row between two of them leaves
  // the matrix pipe idle.  Past the end of k the last stage is fetched and stored again, into the buffer nobody
  // reads any more.
  const int n_stages = a.d / kGemmK;
  constexpr int kMma = MI * NJ, kRd = MI + NJ;   // matrix instructions and operand reads of a k-step
  constexpr int kHalf = kMma / 2, kRdPer = (kRd + kHalf - 1) / kHalf;
  constexpr int kXwPer = (XC + kHalf - 1) / kHalf, kAwPer = (8 + kHalf - 1) / kHalf, kLdPerMma = (kAL + kMma - 1) / kMma;
  fetch_x(0);
  fetch_a(0);
  stash_x(0);
  stash_a(0);
  fetch_x(min(1, n_stages - 1));
  fetch_a(min(1, n_stages - 1));
  __syncthreads();
  read_step(0, 0, 0);
  for (int s = 0; s < n_stages; ++s) {
    const int buf = s & 1, next = min(s + 2, n_stages - 1);
    read_step(1, buf, 1);
    multiply(0);
    stash_x(buf ^ 1);
#pragma unroll
    for (int i = 0; i < kMma; ++i) {             // LDS accesses keep their program order: reads first
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      if (i < kHalf && i * kRdPer < kRd) __builtin_amdgcn_sched_group_barrier(0x100, kRdPer, 0);
      if (i >= kHalf && (i - kHalf) * kXwPer < XC) __builtin_amdgcn_sched_group_barrier(0x200, kXwPer, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    read_step(0, buf, 2);
    multiply(1);
    fetch_x(next);
#pragma unroll
    for (int i = 0; i < kMma; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      if (i < kRd) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      if (i < XC) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    read_step(1, buf, 3);
    multiply(0);
    stash_a(buf ^ 1);
#pragma unroll
    for (int i = 0; i < kMma; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      if (i < kHalf && i * kRdPer < kRd) __builtin_amdgcn_sched_group_barrier(0x100, kRdPer, 0);
      if (i >= kHalf && (i - kHalf) * kAwPer < 8) __builtin_amdgcn_sched_group_barrier(0x200, kAwPer, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    multiply(1);
    fetch_a(next);
#pragma unroll
    for (int i = 0; i < kMma; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      if (i * kLdPerMma < kAL) __builtin_amdgcn_sched_group_barrier(0x020, kLdPerMma, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();                             // the next stage is in LDS; this one has been read
    read_step(0, buf ^ 1, 0);                    // (after the last stage: unused)
    __builtin_amdgcn_sched_barrier(0);
  }

  // accumulator element e of tile (i, j): token m0 + wm + 32 i + mfma_row(e), column n0 + wn + 32 j + lane_lo.
  // Every stage has been read (barrier above): LDS becomes the rounded output tile [TM][kOutPitch].
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e)
#pragma unroll
      for (int j = 0; j < NJ; ++j)
        lds16[(wm + 32 * i + mfma_row(e, lane_hi)) * kOutPitch + wn + 32 * j + lane_lo] = T::from_float(acc[i][j][e]);
  __syncthreads();

  if constexpr (QUANT) {
    // two threads per (token, 128-column block), 64 channels each
    const int n_blocks = sd.R / 128;
    constexpr int NB = TN / 128;                     // quantization blocks per token in the tile
#pragma unroll 1
    for (int item = tid; item < TM * NB * 2; item += 256) {
      const int tr = item / (NB * 2), bl = (item >> 1) % NB, hf = item & 1;
      uint4v v[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = *reinterpret_cast<const uint4v*>(lds16 + tr * kOutPitch + bl * 128 + hf * 64 + i * 8);
      float mn = T::to_float((uint16_t)(v[0][0] & 0xffffu)), mx = mn;
#pragma unroll
      for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const float x0 = T::to_float((uint16_t)(v[i][w] & 0xffffu)), x1 = T::to_float((uint16_t)(v[i][w] >> 16));
          mn = fminf(mn, fminf(x0, x1));
          mx = fmaxf(mx, fmaxf(x0, x1));
        }
      mn = fminf(mn, __shfl_xor(mn, 1, 64));
      mx = fmaxf(mx, __shfl_xor(mx, 1, 64));
      const int t = m0 + tr, blk = col_tile * NB + bl;
      if (t >= a.n_tok || blk >= n_blocks) continue;
      const QuantParams qp = quant_params(mn, mx);
      const size_t orow = a.dst_row ? (size_t)a.dst_row[t] : (size_t)t;
      uint4v* dst = reinterpret_cast<uint4v*>(sd.codes + orow * (size_t)(sd.R / 2) + blk * 64 + hf * 32);
#pragma unroll
      for (int o = 0; o < 2; ++o) {
        uint4v pk;
#pragma unroll
        for (int w = 0; w < 4; ++w) {           // output word w of this store: channels 8 (4 o + w) .. + 7 of the thread's 64
          uint32_t word = 0;
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const uint32_t pr = v[4 * o + w][c];
            word |= (quant_code(T::to_float((uint16_t)(pr & 0xffffu)), qp) | (quant_code(T::to_float((uint16_t)(pr >> 16)), qp) << 4)) << (8 * c);
          }
          pk[w] = word;
        }
        dst[o] = pk;
      }
      if (hf == 0) {
        sd.scale[orow * n_blocks + blk] = qp.s16;
        sd.zero[orow * n_blocks + blk] = qp.z16;
      }
    }
    return;
  }
  // rows leave in 16-byte pieces where the destination allows it (4-byte alignment is all the interface asks for)
  const bool wide = ((reinterpret_cast<uintptr_t>(sd.latent) & 15) == 0) && ((sd.row_stride & 7) == 0);
#pragma unroll 4
  for (int id = tid; id < TM * (TN / 8); id += 256) {
    const int tr = id / (TN / 8), c8 = (id % (TN / 8)) * 8;
    const int t = m0 + tr;
    if (t >= a.n_tok || n0 + c8 >= sd.R) continue;
    const uint4v v = *reinterpret_cast<const uint4v*>(lds16 + tr * kOutPitch + c8);
    const long long row = a.dst_row ? a.dst_row[t] : t;
    uint16_t* dst = sd.latent + row * sd.row_stride + n0 + c8;
    if (wide) {
      *reinterpret_cast<uint4v*>(dst) = v;
    } else {
      uint32_t* d32 = reinterpret_cast<uint32_t*>(dst);
      d32[0] = v[0]; d32[1] = v[1]; d32[2] = v[2]; d32[3] = v[3];
    }
  }
}

namespace {

template <typename K>
int allow_gemm_lds(K kernel, size_t bytes) {
  if (bytes <= 64 * 1024) return PALU_OK;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)bytes) == hipSuccess ? PALU_OK : PALU_ERR_HIP;
}

// Tile height by the number of tokens, tiles dealt to the XCDs in contiguous ranges.
template <typename T, bool Q>
int launch_gemm_t(const EncodeArgs& a, int max_R, int n_sides, int tile_opt, int n_cu, hipStream_t s) {
  auto ceil_div = [](int x, int y) { return (x + y - 1) / y; };
  // the largest tile that still gives most compute units (7 of 10: measured at 512 .. 4096 tokens) a workgroup:
  // 256 or 128 token rows of 256 columns; below that 64 rows of 128 columns, two workgroups to a compute unit
  int tm = 256, tn = 256;
  auto tiles = [&]() { return ceil_div(max_R, tn) * ceil_div(a.n_tok, tm) * n_sides; };
  while (tm > 64 && tiles() * 10 < n_cu * 7) tm >>= 1;
  if (tm == 64) tn = 128;
  if (tile_opt > 0) {
    tm = tile_opt == 32 ? 64 : tile_opt;     // 32: the narrow tile
    tn = tile_opt == 32 ? 128 : 256;
  }
  GemmGrid gg;
  gg.n_col_tiles = ceil_div(max_R, tn);
  gg.n_row_tiles = ceil_div(a.n_tok, tm);
  gg.n_tiles = gg.n_col_tiles * gg.n_row_tiles * n_sides;
  gg.per_xcd = ceil_div(gg.n_tiles, 8);
  const size_t lds = gemm_lds_bytes(tm, tn);
  auto fn = tn == 128 ? encode_gemm_kernel<T, Q, 64, 128>
                      : tm == 256 ? encode_gemm_kernel<T, Q, 256, 256> : tm == 128 ? encode_gemm_kernel<T, Q, 128, 256> : encode_gemm_kernel<T, Q, 64, 256>;
  if (allow_gemm_lds(fn, lds) != PALU_OK) return PALU_ERR_HIP;
  hipLaunchKernelGGL(fn, dim3((unsigned)(8 * gg.per_xcd)), dim3(256), lds, s, a, gg);
  return hipGetLastError() == hipSuccess ? PALU_OK : PALU_ERR_HIP;
}

}  // namespace

int launch_encode_gemm_tiles(int act, const EncodeArgs& a, int max_R, int n_sides, bool quant, int tile_opt, int n_cu,
                             hipStream_t s) {
  if (act == PALU_F16) {
    return quant ? launch_gemm_t<F16, true>(a, max_R, n_sides, tile_opt, n_cu, s)
                 : launch_gemm_t<F16, false>(a, max_R, n_sides, tile_opt, n_cu, s);
  }
  return quant ? launch_gemm_t<BF16, true>(a, max_R, n_sides, tile_opt, n_cu, s)
               : launch_gemm_t<BF16, false>(a, max_R, n_sides, tile_opt, n_cu, s);
}

}  // namespace palu
