/*
 * palu.h - C ABI of the MI355X (gfx950) decode-attention library for a
 * low-rank latent KV-cache (Palu, arXiv 2407.21118).
 *
 * Notation follows the paper: n heads of width d_h, groups of s heads
 * (Sec. 3.2.3); per group j a down-projection A_gj in R^{d x r_j} and a
 * reconstruction matrix B_gj in R^{r_j x (s_j d_h)}; the cache holds latents
 * h = x A (Sec. 3.1) instead of keys and values; row-vector convention
 * (h = x A, y = h B) throughout.
 *
 * Conventions common to every entry point
 *   - plain C, every function returns a status (PALU_OK or a negative code),
 *     never throws, never aborts;
 *   - pointers marked DEVICE are HBM addresses on the current HIP device and
 *     stay owned by the caller; pointers marked HOST are ordinary memory read
 *     during the call;
 *   - work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and the call returns without synchronising;
 *   - the library allocates no device memory: scratch space comes from a
 *     caller-provided workspace whose size is obtained from the matching
 *     *_workspace_bytes query;
 *   - arguments are validated on the host before anything is launched; on an
 *     error nothing is enqueued and outputs are untouched.
 */
#ifndef PALU_H
#define PALU_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  PALU_OK = 0,
  PALU_ERR_INVALID_ARG = -1,        /* NULL / negative / inconsistent argument            */
  PALU_ERR_UNSUPPORTED = -2,        /* valid request this build has no kernel for         */
  PALU_ERR_WORKSPACE_TOO_SMALL = -3,
  PALU_ERR_HIP = -4                 /* a HIP runtime call failed (launch, attribute query) */
};

/* PALU_I4, PALU_I3, PALU_I2: latents quantized to 4, 3 or 2 bits (Appendix A; Sec. 4.4) */
enum { PALU_F16 = 0, PALU_BF16 = 1, PALU_I4 = 2, PALU_I3 = 3, PALU_I2 = 4 };

/* Limits of this build. */
enum {
  PALU_MAX_HEADS = 256,
  PALU_MAX_GROUPS = 64,
  PALU_D_HEAD = 128,          /* only head width supported                                */
  PALU_RANK_MULTIPLE = 32,    /* every group rank must be a multiple of this              */
  PALU_MAX_RANK = 2048        /* per group                                                */
};

/*
 * One compressed attention layer (Sec. 3.2.3, G-LRD; group size 1 is M-LRD,
 * one group of all heads is J-LRD).
 *   group j owns heads  [group_head_off[j], group_head_off[j+1])  - contiguous -
 *   and latent columns  [k_rank_off[j], k_rank_off[j+1]) of a key-latent row,
 *                       [v_rank_off[j], v_rank_off[j+1]) of a value-latent row.
 *   Head u of group j (u counted inside the group) owns columns
 *   [u d_h, (u+1) d_h) of B_gj.
 * The three offset arrays are HOST arrays of n_groups+1 int32, starting at 0.
 *
 * Grouped-query attention (the Llama-3 and Mistral models of Sec. 4.1): the
 * decomposition covers the key and value projections, so n_heads,
 * group_head_off and the B matrices count KEY/VALUE heads; there are
 * n_heads*q_per_kv query heads, query head i attends key/value head
 * i / q_per_kv, and wherever an argument below is shaped by heads (q, out, the
 * latent output, the width n_heads*d_head of x) the heads are the query heads.
 * n_heads*q_per_kv <= PALU_MAX_HEADS.  Several queries per sequence at one position
 * (parallel samples over a shared prefix) are the same thing: multiply q_per_kv by
 * the number of queries and lay q out as [batch, key/value head, query, head of the
 * key/value head, d_head].
 */
typedef struct palu_layer_desc {
  int32_t n_heads;
  int32_t d_head;
  int32_t n_groups;
  const int32_t* group_head_off;   /* HOST [n_groups+1] */
  const int32_t* k_rank_off;       /* HOST [n_groups+1] */
  const int32_t* v_rank_off;       /* HOST [n_groups+1] */
  int32_t act_dtype;               /* PALU_F16 | PALU_BF16: q, x, A, B_k, B_v, unquantized latents */
  int32_t k_latent_dtype;          /* act_dtype, PALU_I4, PALU_I3 or PALU_I2 */
  int32_t v_latent_dtype;          /* act_dtype, PALU_I4, PALU_I3 or PALU_I2 */
  int32_t quant_block;             /* channels per (scale, zero) pair; 128 */
  float rope_theta;                /* RoPE base, e.g. 10000; <= 0: no rotation */
  int32_t q_per_kv;                /* grouped-query attention: query heads per key/value head; 0 or 1 = multi-head */
} palu_layer_desc;

/* Human-readable text for a status code (static storage, never NULL). */
const char* palu_status_string(int status);

/* Library version, major*10000 + minor*100 + patch. */
int palu_version(void);

/*
 * Process-wide tuning knobs for experiments; every default (0, where not stated otherwise) lets the library
 * choose.  Not thread-safe against concurrent decode calls.
 *   "score_waves"         4 or 8 wavefronts per score workgroup for ranks <= 256
 *   "score_chunks"        sequence chunks per (sequence, head block) in the score kernel
 *   "score_mixed"         default 1: a layer whose groups have different ranks (all 64 .. 256 after slicing, fp16 or
 *                         bf16 latents, one query per head) gets ONE score launch over all rank classes; 0: one
 *                         launch per rank class
 *   "value_split_tokens"  tokens per sequence split in the value kernel (multiple of 32, <= 4096)
 *   "score_fp8"           1: low-precision key reconstruction (Sec. 4.5.2, last paragraph), for fp16 layers with RoPE,
 *                         unquantized key latents and ranks 64 .. 256: B_k is rounded to 8-bit floats (OCP E4M3)
 *                         with one power-of-two scale per feature column, the key latents are rounded to E4M3
 *                         (clamped to +-448, no scale), and the keys are rebuilt on the 8-bit matrix
 *                         instructions; rotation, scores, softmax and values as in the default path.  The
 *                         result is exact attention over keys rebuilt from the rounded operands (about 3 % noise
 *                         per key entry): a different numeric contract, 1.2x faster scores on a 7B-shaped layer.
 *                         Set it before querying the workspace size (it adds a region).  Default 0.
 *   "shared_key_fp16"     1: with 2 .. 16 queries per key/value head (grouped-query heads, several queries per
 *                         sequence), fp16 latents and ranks <= 256, rebuild each key once for the queries that
 *                         share it and contract it with them on the matrix cores after rounding the key and
 *                         its cos / sin products to fp16.  About 1.5x faster scores on a 4:1 grouped-query layer
 *                         than the default, but the logit error is about 4e-4 of the logit (output error 2e-3
 *                         reached at logits of about +-25).  Default 0: keys are rebuilt and rotated in float32,
 *                         once per key/value head and pass of up to 8 of its queries where every key rank of
 *                         the layer is 64 .. 512 (4-bit keys: 128 or 256), else once per query head.
 *   "encode_tile_rows"    token rows per workgroup of the prompt-sized projection (64, 128 or 256, each
 *                         with 256 columns; 32 selects the narrow tile of 64 rows x 128 columns)
 * Unknown names and out-of-range values return PALU_ERR_INVALID_ARG.  Set
 * value_split_tokens before querying the workspace size: a smaller split needs
 * more workspace, and palu_attn_decode reports a shortfall.
 */
int palu_set_option(const char* name, int value);

/*
 * Device probes for benchmarking (not part of the method): what this GPU sustains
 * on a bare matrix-core loop and on a bare streaming read, so that kernel rates can
 * be quoted against measured ceilings as well as against the data-sheet peaks.
 *   palu_probe_mfma  every SIMD issues iters*4*2 independent v_mfma_f32_32x32x16_f16;
 *                    *out_flops (HOST, may be NULL) receives the FLOPs of the launch
 *   palu_probe_read  reads `bytes` bytes (multiple of 16) at src (DEVICE, 16-byte aligned) once
 *   sink             DEVICE float[1]; practically never written
 * Time the launches with events on `stream`.
 */
int palu_probe_mfma(int32_t iters, float* sink, void* stream, double* out_flops);
int palu_probe_read(const void* src, size_t bytes, float* sink, void* stream);

/*
 * RoPE angle table (Sec. 3.1.2: RoPE acts on queries and keys before their
 * product).  For position p and pair f < d_h/2 the table stores cos(p w_f) and
 * sin(p w_f) with w_f = theta^(-2f/d_h): as float32 (read by the default score
 * kernels) and, beside them, as float16 (read by the opt-in shared-key form).
 * The angle is reduced in revolutions with float32 pair arithmetic from the
 * host's float64 frequencies (about 1e-7 absolute for positions up to 2^24);
 * the pairing is (f, f + d_h/2) as in the Huggingface Llama implementation the
 * paper builds on (Sec. 4.1).  The layout (tiles of 32 positions) is private to
 * the library; its size is palu_rope_table_bytes.  One table serves every layer
 * and step of a model; build it once for the longest position that will occur.
 * theta <= 0 fills the table with cos = 1, sin = 0.
 *   n_pos     number of positions 0 .. n_pos-1
 *   table     DEVICE, palu_rope_table_bytes(...) bytes, 256-byte aligned
 */
int palu_rope_table_bytes(int32_t d_head, int32_t n_pos, size_t* out_bytes);
int palu_rope_table_init(float rope_theta, int32_t d_head, int32_t n_pos, void* table, void* stream);

/*
 * Down-projection h = x A of new tokens into the latent cache (Sec. 3.1,
 * first display; grouped A of Sec. 3.2.3: group j is columns rank_off[j].. of
 * A, so all groups are one product).
 *   which       0 = key side (k_rank_off), 1 = value side (v_rank_off); the workspace
 *               query also accepts 2 = both sides, for palu_encode_kv
 *   x           DEVICE [n_tok, n_heads*d_head] act_dtype, row-major
 *   A           DEVICE [n_heads*d_head, R] act_dtype, row-major, R = rank_off[n_groups]
 *   latent      DEVICE base of the cache, act_dtype; token t is written to
 *               latent + dst_row[t]*row_stride_elems, R contiguous elements
 *   dst_row     DEVICE int32 [n_tok] row index per token (lets several
 *               sequences append in one call), or NULL for row t
 *   workspace   DEVICE scratch of palu_encode_workspace_bytes(...) bytes
 * Accumulates in float32, rounds once to act_dtype.  Writes only the rows named.
 */
int palu_encode_workspace_bytes(const palu_layer_desc* desc, int which, int32_t n_tok, size_t* out_bytes);
int palu_encode(const palu_layer_desc* desc, int which, const void* x, int32_t n_tok, const void* A,
                void* latent, int64_t row_stride_elems, const int32_t* dst_row,
                void* workspace, size_t workspace_bytes, void* stream);

/*
 * Both down-projections of the same tokens in one pass (h_k = x A_k into the key
 * cache, h_v = x A_v into the value cache; Sec. 3.1, Fig. 2): the same result as
 * palu_encode(which = 0) followed by palu_encode(which = 1), with half the
 * launches.  Arguments as for palu_encode; workspace of
 * palu_encode_workspace_bytes(desc, 2, n_tok) bytes.
 */
int palu_encode_kv(const palu_layer_desc* desc, const void* x, int32_t n_tok, const void* Ak, const void* Av,
                   void* hk, int64_t hk_row_stride_elems, void* hv, int64_t hv_row_stride_elems,
                   const int32_t* dst_row, void* workspace, size_t workspace_bytes, void* stream);

/*
 * palu_encode_kv from transposed weights: Akt = A_k^T [R_k, n_heads*d_head] and
 * Avt = A_v^T [R_v, n_heads*d_head], row-major, so that the weights of one latent
 * channel are contiguous (h = x A of Sec. 3.1 with A stored column by column; the
 * projection matrices are fixed after the decomposition, so this layout is made once,
 * offline).  A wavefront then owns whole columns and finishes their sums by itself:
 * one launch, no workspace, no partial sums in memory.  It pays for one or two tokens
 * per call (a decode step of one or two sequences: one launch instead of two, about
 * 3 us less on a 7B-shaped layer); from about four tokens on the row-major form is
 * the faster one.
 *   n_tok       1 <= n_tok < 64 (a prompt goes through palu_encode / palu_encode_kv)
 *   hk, hv      DEVICE caches, act_dtype; 2-byte aligned, any row stride >= R
 * Everything else as for palu_encode_kv.  Accumulates in float32, rounds once to
 * act_dtype; the order of the sum differs from palu_encode_kv, so the two can differ
 * in the last bit of a latent.  PALU_ERR_UNSUPPORTED for quantized caches and for
 * n_tok >= 64.
 */
int palu_encode_kv_t(const palu_layer_desc* desc, const void* x, int32_t n_tok, const void* Akt, const void* Avt,
                     void* hk, int64_t hk_row_stride_elems, void* hv, int64_t hv_row_stride_elems,
                     const int32_t* dst_row, void* stream);

/*
 * Asymmetric uniform B-bit quantization of latent rows (Appendix A), one (scale, zero)
 * pair per token per quant_block channels; B = 4, 3 or 2 as the side's latent dtype
 * says (PALU_I4 / PALU_I3 / PALU_I2; 4 where the side is not declared quantized):
 *     s = fp16((max - min) / (2^B - 1)), s == 0 -> 1;   z = fp16(clamp(rint(-min / s), +-65504));
 *     code = clamp(rint(x / s) + z, 0, 2^B - 1)         (float32 arithmetic, ties to even)
 *   latent      DEVICE act_dtype, token t at latent + t*row_stride_elems, R elements
 *   codes       DEVICE uint8 rows of R*B/8 bytes.  4 bits: byte c/2 holds channel c (c even)
 *               in its low nibble and channel c+1 in its high nibble.  2 bits: byte k holds
 *               channels 4k .. 4k+3, channel 4k+u in bits 2u, 2u+1.  3 bits: the low two bits
 *               of every code in the 2-bit layout (R/4 bytes), then the third bits, byte k
 *               holding channels 8k .. 8k+7, channel 8k+u in bit u (R/8 bytes).  The same
 *               layouts are what palu_attn_decode reads.
 *   scale,zero  DEVICE float16 rows of R/quant_block
 *   dst_row     DEVICE int32 [n_tok]: token t is written to row dst_row[t] of codes,
 *               scale and zero (appending to several sequences of a cache at once),
 *               or NULL for row t
 * R must be a multiple of quant_block.
 */
int palu_quant_latent(const palu_layer_desc* desc, int which, const void* latent, int64_t row_stride_elems,
                      int32_t n_tok, uint8_t* codes, void* scale, void* zero, const int32_t* dst_row,
                      void* stream);

/*
 * Down-projection and 4-bit quantization of new tokens in one kernel, for filling
 * a quantized cache from a prompt (Sec. 3.1 first display, then Appendix A with
 * B = 4, Sec. 3.4): the unquantized latents never reach memory.  The bytes written
 * are those of palu_encode (its many-token form, n_tok >= 64) followed by
 * palu_quant_latent: the product is accumulated in float32, rounded once to
 * act_dtype, and quantized from that rounded value.  Works for any n_tok >= 1 but
 * computes in tiles of 128 tokens, so for a handful of tokens the two-call form
 * is cheaper.
 *   which       0 = key side, 1 = value side; R = rank_off[n_groups] must be a multiple of 128
 *   x, A        as for palu_encode (16-byte aligned)
 *   codes       DEVICE uint8 rows of R/2 bytes, 16-byte aligned, layout as palu_quant_latent
 *   scale,zero  DEVICE float16 rows of R/128
 *   dst_row     DEVICE int32 [n_tok] output row per token, or NULL for row t
 * Needs no workspace.  Writes only the rows named.
 */
int palu_encode_quant(const palu_layer_desc* desc, int which, const void* x, int32_t n_tok, const void* A,
                      uint8_t* codes, void* scale, void* zero, const int32_t* dst_row, void* stream);

/*
 * One decode step of attention over the latent cache for `batch` sequences
 * (Sec. 2.1 Eq. 2 with K = RoPE(H_k B_k) rebuilt on the fly, Sec. 3.1.2 and
 * Appendix B; values contracted in latent space first, (p H_v) B_v, Eq. 4):
 *     out[b,i] = softmax_t( RoPE(q[b,i], q_pos[b]) . RoPE(H_k[b,t] B_k, k_pos[t])_i / sqrt(d_h) ) H_v[b] B_v |_i
 * over t in [0, seq_lens[b]).  No causal mask: every cached row is attended.
 * With desc->rope_theta <= 0 there is no rotation and the non-RoPE form of
 * Sec. 3.1.2 (Eq. 5) is used: the query is multiplied by B_k^T once and the
 * scores are (q B_k^T) H_k^T, without rebuilding any key; q_pos, k_pos and the
 * table are then not read (a valid table pointer is still required).
 *
 *   q          DEVICE [batch, n_heads, d_head] act_dtype, before RoPE (Sec. 4.5.2)
 *   q_pos      DEVICE int32 [batch] position of each query token
 *   hk, hv     DEVICE latents [batch, max_seq, R] act_dtype, or packed codes
 *              [batch, max_seq, R*B/8] uint8 when the side is PALU_I4 / I3 / I2 (layouts
 *              under palu_quant_latent); sequence b starts at b*max_seq rows
 *   h*_scale, h*_zero   DEVICE float16 [batch, max_seq, R/quant_block] (quantized side), else NULL
 *   k_pos      DEVICE int32 [max_seq] position of cached row t, or NULL (row t is position t).
 *              Positions must lie in [0, rope_table_len); the kernels clamp to that
 *              range to stay in bounds, results for out-of-range positions are undefined
 *   seq_lens   DEVICE int32 [batch] rows to attend per sequence, each in [0, seq_len],
 *              or NULL (all seq_len rows).  A sequence with 0 rows (an idle slot of the
 *              batch) reads nothing from the caches and gets an output row of zeros
 *   seq_len    upper bound of rows attended (1 <= seq_len <= max_seq)
 *   Bk, Bv     DEVICE act_dtype; group j at element offset sum_{i<j} r_i s_i d_h,
 *              row-major [r_j, s_j d_h]
 *   rope_table DEVICE table from palu_rope_table_init (same theta, d_head),
 *              rope_table_len positions; with k_pos == NULL needs rope_table_len >= seq_len
 *   out        DEVICE float32 [batch, n_heads, d_head]
 *   workspace  DEVICE scratch, at least palu_attn_decode_workspace_bytes(desc, batch, max_seq)
 *              bytes, 256-byte aligned; contents need not be preserved between calls.
 *              Calls sharing a workspace must be ordered on one stream.
 *
 * Arithmetic.  Keys are rebuilt on the matrix cores from the 16-bit latents and B_k as they are (fp16 or
 * bf16 instruction of act_dtype, float32 accumulation), rotated and multiplied by the rotated query in
 * float32 with float32 cos / sin: the logit error does not grow with the logit.  The value side contracts
 * fp16 numbers: probabilities exp(score - running max) rounded to fp16 (float32 row sums of the rounded
 * values), latents in fp16.  The non-RoPE form contracts the key latents in fp16 with q B_k^T kept as an
 * fp16 pair hi + lo.  Quantized latents are dequantized to fp16 ((code - zero) * scale, one rounding).
 *
 * bfloat16 layers: on the RoPE score path bf16 key latents and B_k enter the bf16 matrix instruction
 * unchanged.  bf16 VALUE latents, and bf16 KEY latents of the non-RoPE form, are converted to fp16 before
 * their contraction: exact for 2^-17 <= |h| <= 65504 (every bf16 number in that range is an fp16 number);
 * larger magnitudes are clamped to +-65504 (infinities stay infinite), smaller ones are truncated toward
 * zero to the fp16 subnormal grid (multiples of 2^-24; below 2^-24: zero).  No error is reported for
 * latents outside that range; a cache that holds such values should be stored as fp16 with its own scaling.
 */
int palu_attn_decode_workspace_bytes(const palu_layer_desc* desc, int32_t batch, int32_t max_seq, size_t* out_bytes);
int palu_attn_decode(const palu_layer_desc* desc, int32_t batch, int32_t seq_len, int32_t max_seq,
                     const void* q, const int32_t* q_pos,
                     const void* hk, const void* hk_scale, const void* hk_zero,
                     const void* hv, const void* hv_scale, const void* hv_zero,
                     const int32_t* k_pos, const int32_t* seq_lens,
                     const void* Bk, const void* Bv,
                     const void* rope_table, int32_t rope_table_len,
                     float* out, void* workspace, size_t workspace_bytes, void* stream);

/*
 * palu_attn_decode for callers that cannot allocate device memory or carry a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, same kernels and same results as palu_attn_decode, without
 * the workspace: the scratch is a static device array of PALU_NOALLOC_SCRATCH_BYTES inside
 * the library (each GPU the library is used on holds that much until the process ends).
 * The call allocates nothing; the first call on a device looks up the array's address
 * there.  PALU_ERR_WORKSPACE_TOO_SMALL when palu_attn_decode_workspace_bytes(desc, batch,
 * max_seq) exceeds PALU_NOALLOC_SCRATCH_BYTES (nothing is enqueued).  All calls on one GPU
 * share the array, which keeps the previous call's contents (no call relies on them):
 * calls that overlap on one GPU, on different streams or from different threads, race;
 * order them on one stream.
 */
enum { PALU_NOALLOC_SCRATCH_BYTES = 32 * 1024 * 1024 };
int palu_attn_decode_noalloc(const palu_layer_desc* desc, int32_t batch, int32_t seq_len, int32_t max_seq,
                             const void* q, const int32_t* q_pos,
                             const void* hk, const void* hk_scale, const void* hk_zero,
                             const void* hv, const void* hv_scale, const void* hv_zero,
                             const int32_t* k_pos, const int32_t* seq_lens,
                             const void* Bk, const void* Bv,
                             const void* rope_table, int32_t rope_table_len,
                             float* out, void* stream);

/*
 * The same decode step with the output left in the value latent space
 * (Sec. 3.1.1: B_v is absorbed into the output projection W_o offline, so the
 * attention module returns (p H_v) and never multiplies by B_v):
 *     out_latent[b, off(i) .. off(i) + r_v(g(i))) = softmax_t(...) H_v[b][:, columns of group g(i)]
 * with off(i) = sum over heads i' < i of r_v(g(i')).  Arguments as for
 * palu_attn_decode, without Bv;
 *   out_latent DEVICE float32 [batch, sum_i r_v(g(i))]
 * Uses the same workspace size as palu_attn_decode.
 */
int palu_attn_decode_latent(const palu_layer_desc* desc, int32_t batch, int32_t seq_len, int32_t max_seq,
                            const void* q, const int32_t* q_pos,
                            const void* hk, const void* hk_scale, const void* hk_zero,
                            const void* hv, const void* hv_scale, const void* hv_zero,
                            const int32_t* k_pos, const int32_t* seq_lens,
                            const void* Bk,
                            const void* rope_table, int32_t rope_table_len,
                            float* out_latent, void* workspace, size_t workspace_bytes, void* stream);

/*
 * One whole decode step in one call: append the new token of every sequence to both
 * caches (h = x A, Sec. 3.1) and attend (palu_attn_decode).  Same results, bit for
 * bit, as palu_encode_kv followed by palu_attn_decode; where the step folds the
 * query into B_k (RoPE, fp16 / bf16 latents, one query per key/value head, fewer
 * than 64 sequences) the projection's first launch and the fold, which do not depend
 * on each other, share one grid, so the step has one launch less.
 *   x            DEVICE [batch, n_heads*q_per_kv*d_head] act_dtype: the new tokens' activations
 *   Ak, Av       as for palu_encode_kv
 *   dst_row      DEVICE int32 [batch]: row of hk / hv (counted over all batch*max_seq rows)
 *                that receives sequence b's new latent; it must be one of the rows attended
 *   encode_workspace  of palu_encode_workspace_bytes(desc, 2, batch) bytes
 *   hk, hv       DEVICE caches [batch, max_seq, R] act_dtype (quantized caches: PALU_ERR_UNSUPPORTED,
 *                use the separate calls with palu_quant_latent in between)
 *   the rest     as for palu_attn_decode
 */
int palu_decode_step(const palu_layer_desc* desc, int32_t batch, int32_t seq_len, int32_t max_seq,
                     const void* x, const void* Ak, const void* Av, const int32_t* dst_row,
                     void* encode_workspace, size_t encode_workspace_bytes,
                     const void* q, const int32_t* q_pos, void* hk, void* hv,
                     const int32_t* k_pos, const int32_t* seq_lens,
                     const void* Bk, const void* Bv,
                     const void* rope_table, int32_t rope_table_len,
                     float* out, void* workspace, size_t workspace_bytes, void* stream);

/*
 * palu_decode_step from transposed weights (palu_encode_kv_t followed by
 * palu_attn_decode, in one call): the projection is one launch, and where the step
 * folds the query into B_k that fold rides in the projection's workgroups, so the
 * whole append costs one launch.  No encode workspace.  Arguments as for
 * palu_decode_step with Akt, Avt as for palu_encode_kv_t; batch < 64.
 */
int palu_decode_step_t(const palu_layer_desc* desc, int32_t batch, int32_t seq_len, int32_t max_seq,
                       const void* x, const void* Akt, const void* Avt, const int32_t* dst_row,
                       const void* q, const int32_t* q_pos, void* hk, void* hv,
                       const int32_t* k_pos, const int32_t* seq_lens,
                       const void* Bk, const void* Bv,
                       const void* rope_table, int32_t rope_table_len,
                       float* out, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Several new query tokens per sequence in one call (a block of a chunked prompt,
 * or a speculative-decoding check): each query is an ordinary decode step of Sec. 2.1
 * Eq. 2 over the latent cache, with its own position and its own number of cached
 * rows, so a causal block over rows that were appended first is
 * q_len[b, j] = seq_lens[b] - n_q + j + 1.  Same result as n_q calls of
 * palu_attn_decode with seq_lens = q_len[:, j]; the latents are read once and, for
 * fp16 latents with RoPE and q_per_kv * n_q <= 16, each key is rebuilt once for all
 * queries of its key/value head.
 *   n_q        queries per sequence, n_heads * q_per_kv * n_q <= PALU_MAX_HEADS
 *   q          DEVICE [batch, n_q, n_heads*q_per_kv, d_head] act_dtype, before RoPE
 *   q_pos      DEVICE int32 [batch, n_q]
 *   q_len      DEVICE int32 [batch, n_q] rows attended by each query, in [0, seq_lens[b]]
 *              (seq_len where seq_lens is NULL), or NULL: every query attends all rows.
 *              A query with 0 rows gets zeros
 *   out        DEVICE float32 [batch, n_q, n_heads*q_per_kv, d_head]
 *   workspace  of palu_attn_decode_multi_workspace_bytes(desc, batch, n_q, max_seq) bytes
 * Everything else as for palu_attn_decode.
 */
int palu_attn_decode_multi_workspace_bytes(const palu_layer_desc* desc, int32_t batch, int32_t n_q, int32_t max_seq,
                                           size_t* out_bytes);
int palu_attn_decode_multi(const palu_layer_desc* desc, int32_t batch, int32_t n_q, int32_t seq_len, int32_t max_seq,
                           const void* q, const int32_t* q_pos, const int32_t* q_len,
                           const void* hk, const void* hk_scale, const void* hk_zero,
                           const void* hv, const void* hv_scale, const void* hv_zero,
                           const int32_t* k_pos, const int32_t* seq_lens,
                           const void* Bk, const void* Bv,
                           const void* rope_table, int32_t rope_table_len,
                           float* out, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Same call with per-stage timing hooks, for benchmarks that price each
 * stage against its own roofline.  The decode step runs as PALU_DECODE_STAGES
 * stages (0 fold the rotated query into B_k, 1 scores = reconstruction + RoPE +
 * query product, 2 softmax partials and P H_v per sequence split, 3 merge
 * splits and apply B_v).  `stage_events` is a HOST array of
 * PALU_DECODE_STAGES + 1 hipEvent_t handles created by the caller (each passed
 * as void*): event i is recorded on `stream` before stage i is enqueued, the
 * last one after the final stage.  NULL disables the hooks (then identical to
 * palu_attn_decode).  Recording events between the stages inserts queue
 * barriers, so a step timed this way is slower than an unhooked one.
 */
enum { PALU_DECODE_STAGES = 4 };
int palu_attn_decode_staged(const palu_layer_desc* desc, int32_t batch, int32_t seq_len, int32_t max_seq,
                            const void* q, const int32_t* q_pos,
                            const void* hk, const void* hk_scale, const void* hk_zero,
                            const void* hv, const void* hv_scale, const void* hv_zero,
                            const int32_t* k_pos, const int32_t* seq_lens,
                            const void* Bk, const void* Bv,
                            const void* rope_table, int32_t rope_table_len,
                            float* out, void* workspace, size_t workspace_bytes, void* stream,
                            void* const* stage_events);

#ifdef __cplusplus
}
#endif
#endif /* PALU_H */
