"""CPU oracle for decode attention over a low-rank latent KV-cache (Palu).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain, obviously-correct
definition that the HIP kernels are checked against.  Only the tests, the
smoke check and the benchmark's CPU-baseline leg may import it; the product
package never does, and nothing here imports the product package.

Everything is numpy in float64 except the quantizer, which the paper defines
as an integer-valued function and which is therefore evaluated in IEEE float32
so that its integer decisions are reproducible bit for bit.

Conventions (row-vector form used by the paper everywhere except one display):
    h = x . A          latent, A in R^{d x r}               (Sec. 3.1)
    y = h . B          reconstruction, B in R^{r x (s*d_h)} (Sec. 3.2.3)
    head u of group j owns columns [u*d_h, (u+1)*d_h) of y.

Parity status of each function is given in its docstring.  The paper prints no
worked numeric example of latents, scores or outputs, so the attention output
values themselves are pinned only through special cases, identities and brute
force (see tests/test_oracle_pins.py), not through printed numbers.
"""

from __future__ import annotations

import numpy as np

__all__ = [
    "rope_inv_freq", "rope_rotate", "unpack_int4", "pack_int4",
    "dequant_latent", "quant_latent", "encode", "reconstruct",
    "attn_decode", "attn_decode_scores", "softmax_rows",
    "storage_ratio", "kv_cache_bytes", "reconstruction_macs_per_token",
    "fp8_e4m3_value", "fp8_e4m3_round", "fp8_weight_scales", "fp8_keys", "attn_decode_fp8_keys",
]


# --------------------------------------------------------------------------
# RoPE (Sec. 3.1.2 says only "RoPE"; the model family is Llama via the
# Huggingface library (Sec. 4.1), whose convention pairs feature f with
# feature f + d_h/2 and uses frequency theta^(-2f/d_h)).
# --------------------------------------------------------------------------

def rope_inv_freq(d_head: int, theta: float) -> np.ndarray:
    """Angular frequency of pair f, f = 0 .. d_head/2 - 1 (float64)."""
    f = np.arange(d_head // 2, dtype=np.float64)
    return np.float64(theta) ** (-2.0 * f / np.float64(d_head))


def rope_rotate(x: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Rotate the last axis of x (length d_head) by the angles of `pos`.

    x   [..., d_head] float64
    pos broadcastable to x.shape[:-1], integer positions
    Pair (x[f], x[f + d_head/2]) is rotated by angle pos * inv_freq[f].
    theta <= 0 disables the rotation (non-RoPE attention, Sec. 3.1.2 last
    paragraph).
    """
    x = np.asarray(x, dtype=np.float64)
    if theta <= 0:
        return x.copy()
    d = x.shape[-1]
    half = d // 2
    phi = np.asarray(pos, dtype=np.float64)[..., None] * rope_inv_freq(d, theta)
    c, s = np.cos(phi), np.sin(phi)
    lo, hi = x[..., :half], x[..., half:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


# --------------------------------------------------------------------------
# int4 latents (Appendix A: asymmetric uniform quantization, B = 4 bits)
# --------------------------------------------------------------------------

def unpack_int4(packed: np.ndarray) -> np.ndarray:
    """[..., n] uint8 -> [..., 2n] uint8 codes; low nibble = even channel."""
    packed = np.asarray(packed, dtype=np.uint8)
    out = np.empty(packed.shape[:-1] + (packed.shape[-1] * 2,), dtype=np.uint8)
    out[..., 0::2] = packed & 0x0F
    out[..., 1::2] = packed >> 4
    return out


def pack_int4(codes: np.ndarray) -> np.ndarray:
    """[..., 2n] codes in 0..15 -> [..., n] uint8; low nibble = even channel."""
    codes = np.asarray(codes, dtype=np.uint8)
    assert codes.shape[-1] % 2 == 0
    assert codes.max(initial=0) <= 15
    return (codes[..., 0::2] | (codes[..., 1::2] << 4)).astype(np.uint8)


def pack_codes(codes: np.ndarray, bits: int) -> np.ndarray:
    """Storage format of B-bit codes (Sec. 4.4 quantizes the latents to 4, 3 and 2 bits;
    the byte layouts are this build's):
      4 bits: byte k holds channel 2k in its low nibble, channel 2k+1 in its high nibble;
      2 bits: byte k holds channels 4k .. 4k+3, channel 4k+u in bits 2u, 2u+1;
      3 bits: the low two bits of every code in the 2-bit layout (R/4 bytes), followed by
              the third bits, byte k holding channels 8k .. 8k+7, channel 8k+u in bit u
              (R/8 bytes): 3R/8 bytes per row."""
    codes = np.asarray(codes, dtype=np.uint8)
    R = codes.shape[-1]
    assert codes.max(initial=0) < (1 << bits)
    if bits == 4:
        return pack_int4(codes)
    assert R % 8 == 0
    lo = codes & 3
    low_plane = (lo[..., 0::4] | (lo[..., 1::4] << 2) | (lo[..., 2::4] << 4) | (lo[..., 3::4] << 6)).astype(np.uint8)
    if bits == 2:
        return low_plane
    assert bits == 3
    hi = (codes >> 2) & 1
    high_plane = np.zeros(codes.shape[:-1] + (R // 8,), dtype=np.uint8)
    for u in range(8):
        high_plane |= (hi[..., u::8] << u).astype(np.uint8)
    return np.concatenate([low_plane, high_plane], axis=-1)


def unpack_codes(packed: np.ndarray, bits: int) -> np.ndarray:
    """Inverse of pack_codes: [..., R*bits/8] uint8 -> [..., R] uint8 codes."""
    packed = np.asarray(packed, dtype=np.uint8)
    if bits == 4:
        return unpack_int4(packed)
    nb = packed.shape[-1]
    R = nb * 4 if bits == 2 else nb * 8 // 3
    low = packed[..., :R // 4]
    out = np.empty(packed.shape[:-1] + (R,), dtype=np.uint8)
    for u in range(4):
        out[..., u::4] = (low >> (2 * u)) & 3
    if bits == 3:
        high = packed[..., R // 4:]
        for u in range(8):
            out[..., u::8] |= (((high >> u) & 1) << 2).astype(np.uint8)
    return out


def dequant_latent(packed, scale, zero, block: int = 128, bits: int = 4) -> np.ndarray:
    """Dequantize packed B-bit latents to float64.

    packed [..., R*bits/8] uint8 (pack_codes), scale/zero [..., R/block] (float16 values).
    h[c] = (code[c] - zero[c // block]) * scale[c // block], evaluated in
    float64 from the stored float16 scale and zero-point (Appendix A read
    backwards; the benchmark configuration fixes one (scale, zero) per token
    per `block` channels).
    """
    codes = unpack_codes(packed, bits).astype(np.float64)
    s = np.repeat(np.asarray(scale, dtype=np.float64), block, axis=-1)
    z = np.repeat(np.asarray(zero, dtype=np.float64), block, axis=-1)
    return (codes - z) * s


def quant_latent(h: np.ndarray, block: int = 128, bits: int = 4):
    """Asymmetric uniform B-bit quantization of latents (Appendix A; B = 4 below, and
    the 3- and 2-bit settings of Sec. 4.4 with 15 replaced by 2^B - 1).

    h [..., R] with values exactly representable in float16/bfloat16 (they are
    converted to float32 exactly).  Per (row, block of `block` channels):

        s  = (max - min) / 15                  float32, then rounded to float16
             (s == 0 -> s = 1: a constant block quantizes to code 0 + z)
        z  = round(-min / s)                   round-half-even, float32 divide,
             clamped to +-65504 and rounded to float16 (the storage format);
             the *stored* z is the one used for the codes
        q  = clamp(round(x / s) + z, 0, 15)

    Returns (packed [..., R/2] uint8, scale [..., R/block] float16,
             zero [..., R/block] float16).
    Every step is a single correctly-rounded IEEE float32 operation, so a GPU
    doing the same steps in float32 must agree bit for bit.
    """
    h32 = np.asarray(h, dtype=np.float32)
    R = h32.shape[-1]
    assert R % block == 0 and block % 2 == 0
    hb = h32.reshape(h32.shape[:-1] + (R // block, block))
    mn = hb.min(axis=-1)
    mx = hb.max(axis=-1)
    top = np.float32((1 << bits) - 1)
    s32 = (mx - mn) / top
    s16 = s32.astype(np.float16)
    s16 = np.where(s16 == 0, np.float16(1.0), s16).astype(np.float16)
    sf = s16.astype(np.float32)
    z = np.rint((-mn) / sf)
    z = np.clip(z, np.float32(-65504.0), np.float32(65504.0))
    z16 = z.astype(np.float16)
    zf = z16.astype(np.float32)
    q = np.rint(hb / sf[..., None]) + zf[..., None]
    q = np.clip(q, np.float32(0.0), top)
    codes = q.astype(np.uint8).reshape(h32.shape)
    return pack_codes(codes, bits), s16, z16


# --------------------------------------------------------------------------
# Encode: h = x . A  (Sec. 3.1, first display; Sec. 3.2.3 for the grouped A)
# --------------------------------------------------------------------------

def encode(x: np.ndarray, A: np.ndarray) -> np.ndarray:
    """Latent h = x . A in float64 (the caller rounds to the cache dtype).

    x [T, d], A [d, R]; group j's A_gj occupies columns rank_off[j]..rank_off[j+1]
    of A, so the grouped down-projection is a single matrix product.
    """
    return np.asarray(x, dtype=np.float64) @ np.asarray(A, dtype=np.float64)


# --------------------------------------------------------------------------
# Reconstruction y = h . B  (Sec. 3.2.3 display) and attention (Sec. 2.1)
# --------------------------------------------------------------------------

def _group_matrix(B_flat, j, group_head_off, rank_off, d_head):
    """View of group j's reconstruction matrix [r_j, s_j*d_head] inside the
    concatenated buffer (group j starts at sum_{i<j} r_i*s_i*d_head)."""
    off = 0
    for i in range(j):
        off += (rank_off[i + 1] - rank_off[i]) * (group_head_off[i + 1] - group_head_off[i]) * d_head
    r = rank_off[j + 1] - rank_off[j]
    w = (group_head_off[j + 1] - group_head_off[j]) * d_head
    return np.asarray(B_flat).reshape(-1)[off:off + r * w].reshape(r, w)


def reconstruct(H: np.ndarray, B_flat, group_head_off, rank_off, d_head: int) -> np.ndarray:
    """Full-width states from latents: [y_{j,1} .. y_{j,s}] = h_gj . B_gj.

    H [L, R] float64 latents of one sequence, returns [L, n_heads*d_head].
    """
    H = np.asarray(H, dtype=np.float64)
    n_groups = len(group_head_off) - 1
    n_heads = group_head_off[-1]
    Y = np.empty((H.shape[0], n_heads * d_head), dtype=np.float64)
    for j in range(n_groups):
        Bj = _group_matrix(B_flat, j, group_head_off, rank_off, d_head).astype(np.float64)
        cols = slice(rank_off[j], rank_off[j + 1])
        h0, h1 = group_head_off[j], group_head_off[j + 1]
        Y[:, h0 * d_head:h1 * d_head] = H[:, cols] @ Bj
    return Y


def softmax_rows(s: np.ndarray) -> np.ndarray:
    """Softmax over the last axis, max-subtracted, float64.  Over an empty axis
    (a sequence with no cached row: the sums of Eq. 2 are empty) the result is
    empty and every product with it is the empty sum, zero."""
    s = np.asarray(s, dtype=np.float64)
    if s.shape[-1] == 0:
        return np.zeros_like(s)
    e = np.exp(s - s.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def attn_decode_scores(q, q_pos, Hk, Bk, group_head_off, k_rank_off, d_head,
                       rope_theta, k_pos=None, seq_lens=None, q_per_kv: int = 1):
    """Pre-softmax scores q'_i . K'_{i,t} / sqrt(d_h) as a list over batch of
    [n_heads, L_b] float64 arrays (Eq. 2 numerator with RoPE on q and K,
    Sec. 3.1.2).  With grouped-query attention (the Llama-3 / Mistral models of
    Sec. 4.1) the decomposition covers the key/value heads only and query head
    i reads key/value head i // q_per_kv: the rebuilt heads are repeated."""
    q = np.asarray(q, dtype=np.float64)
    Bsz, n_heads, _ = q.shape
    n_kv = int(group_head_off[-1])
    assert n_heads == n_kv * q_per_kv
    out = []
    for b in range(Bsz):
        L = int(seq_lens[b]) if seq_lens is not None else Hk.shape[1]
        pos = np.arange(L) if k_pos is None else np.asarray(k_pos)[:L]
        K = reconstruct(np.asarray(Hk[b, :L], dtype=np.float64), Bk, group_head_off, k_rank_off, d_head)
        K = np.repeat(K.reshape(L, n_kv, d_head), q_per_kv, axis=1)                   # [L, n, d_h]
        K = rope_rotate(K, pos[:, None], rope_theta)
        qr = rope_rotate(q[b], np.full((n_heads,), int(np.asarray(q_pos)[b])), rope_theta)  # [n, d_h]
        out.append(np.einsum("lnd,nd->nl", K, qr) / np.sqrt(np.float64(d_head)))
    return out


def attn_decode(q, q_pos, Hk, Hv, Bk, Bv, group_head_off, k_rank_off, v_rank_off,
                d_head: int, rope_theta: float, k_pos=None, seq_lens=None, q_per_kv: int = 1) -> np.ndarray:
    """One decode step of attention over the latent cache, by the definition.

    q   [B, n_heads, d_head]  pre-RoPE query (Sec. 4.5.2 times the kernel from
        the pre-RoPE query)
    q_pos [B] position of the query token
    Hk  [B, Lmax, R_k], Hv [B, Lmax, R_v]  latents (already dequantized when
        the cache is int4: the caller passes dequant_latent(...))
    Bk, Bv  concatenated per-group reconstruction matrices
    k_pos [Lmax] or None (token t sits at position t)
    seq_lens [B] or None (all Lmax rows are attended)

    Steps, in the paper's order: K = H_k B_k and V = H_v B_v fully materialised
    (Sec. 3.2.3), RoPE on K rows and on q (Sec. 3.1.2), p = softmax(q K^T /
    sqrt(d_h)), a = p V (Eq. 2).  Returns [B, n_heads, d_head] float64.
    No causal mask: every cached row up to seq_lens[b] is attended.
    q_per_kv > 1 is grouped-query attention: group_head_off counts key/value
    heads, q has q_per_kv times as many, and query head i uses key/value head
    i // q_per_kv.
    """
    q = np.asarray(q, dtype=np.float64)
    Bsz, n_heads, _ = q.shape
    scores = attn_decode_scores(q, q_pos, Hk, Bk, group_head_off, k_rank_off, d_head,
                                rope_theta, k_pos, seq_lens, q_per_kv)
    out = np.empty((Bsz, n_heads, d_head), dtype=np.float64)
    for b in range(Bsz):
        L = scores[b].shape[1]
        V = reconstruct(np.asarray(Hv[b, :L], dtype=np.float64), Bv, group_head_off, v_rank_off, d_head)
        V = np.repeat(V.reshape(L, n_heads // q_per_kv, d_head), q_per_kv, axis=1)
        p = softmax_rows(scores[b])                       # [n, L]
        out[b] = np.einsum("nl,lnd->nd", p, V)
    return out


def attn_decode_latent(q, q_pos, Hk, Hv, Bk, group_head_off, k_rank_off, v_rank_off,
                       d_head: int, rope_theta: float, k_pos=None, seq_lens=None, q_per_kv: int = 1) -> np.ndarray:
    """Attention output left in the value latent space (Sec. 3.1.1, Eq. 4 before
    the multiplication by B_v, which the paper absorbs into the output
    projection W_o offline): for head i of group j, a^lat_i = p_i H_v[:, columns of j],
    with p_i the same softmax as attn_decode.  Returns [B, sum_i r_v(group(i))]
    float64, heads in order, head i occupying r_v(group(i)) entries.  With
    q_per_kv > 1 the heads are the query heads, q_per_kv per key/value head."""
    q = np.asarray(q, dtype=np.float64)
    Bsz, n_heads, _ = q.shape
    scores = attn_decode_scores(q, q_pos, Hk, Bk, group_head_off, k_rank_off, d_head,
                                rope_theta, k_pos, seq_lens, q_per_kv)
    widths = []
    for j in range(len(group_head_off) - 1):
        widths += [v_rank_off[j + 1] - v_rank_off[j]] * ((group_head_off[j + 1] - group_head_off[j]) * q_per_kv)
    out = np.empty((Bsz, int(sum(widths))), dtype=np.float64)
    for b in range(Bsz):
        L = scores[b].shape[1]
        p = softmax_rows(scores[b])                       # [n, L]
        H = np.asarray(Hv[b, :L], dtype=np.float64)
        at = 0
        for j in range(len(group_head_off) - 1):
            Hj = H[:, v_rank_off[j]:v_rank_off[j + 1]]    # [L, r_j]
            for i in range(group_head_off[j] * q_per_kv, group_head_off[j + 1] * q_per_kv):
                out[b, at:at + Hj.shape[1]] = p[i] @ Hj
                at += Hj.shape[1]
    return out


def attn_decode_multi(q, q_pos, q_len, Hk, Hv, Bk, Bv, group_head_off, k_rank_off, v_rank_off,
                      d_head: int, rope_theta: float, k_pos=None, q_per_kv: int = 1) -> np.ndarray:
    """Several new query tokens per sequence: query j of sequence b is its own
    decode step (Sec. 2.1 Eq. 2 on the rebuilt keys and values) at position
    q_pos[b, j] over the first q_len[b, j] cached rows.  q [B, n_q, n, d_head];
    returns [B, n_q, n, d_head] float64."""
    q = np.asarray(q, dtype=np.float64)
    out = np.empty_like(q)
    for j in range(q.shape[1]):
        out[:, j] = attn_decode(q[:, j], np.asarray(q_pos)[:, j], Hk, Hv, Bk, Bv, group_head_off, k_rank_off,
                                v_rank_off, d_head, rope_theta, k_pos, np.asarray(q_len)[:, j], q_per_kv)
    return out


# --------------------------------------------------------------------------
# Closed forms the paper prints (used as pins and by the benchmark's counters)
# --------------------------------------------------------------------------

def storage_ratio(m: float, n: float, r: float) -> float:
    """(m r + r n) / (m n): size of A and B relative to W (Sec. 2.2)."""
    return (m * r + r * n) / (m * n)


def kv_cache_bytes(n_layers: int, seq_len: int, hidden: int, keep_fraction: float, bits: float) -> float:
    """Bytes of K plus V cache: 2 * layers * L * (hidden * keep) * bits / 8
    (Table 2's size column; scale and zero-point overhead not counted)."""
    return 2.0 * n_layers * seq_len * hidden * keep_fraction * bits / 8.0


def reconstruction_macs_per_token(group_head_off, rank_off, d_head: int) -> int:
    """Multiply-accumulates to rebuild all heads of one token:
    sum_j r_j * s_j * d_h  (Sec. 3.2.2 'High Inference Overhead', Sec. 3.2.3)."""
    total = 0
    for j in range(len(group_head_off) - 1):
        total += (rank_off[j + 1] - rank_off[j]) * (group_head_off[j + 1] - group_head_off[j]) * d_head
    return int(total)


# --------------------------------------------------------------------------
# Low-precision key reconstruction (Sec. 4.5.2, last paragraph: the decomposed
# weight matrices quantized further so that low-precision matrix hardware does
# the online reconstruction).  The paper names the idea and fixes no format;
# this build's reading, which the kernels follow and this section defines:
#   * format: 8-bit float E4M3 of the OCP 8-bit floating point specification
#     (1 sign, 4 exponent bits with bias 7, 3 mantissa bits; no infinities;
#     exponent 15 with mantissa 7 is NaN; largest finite 448; subnormals are
#     multiples of 2^-9), round to nearest even, magnitudes above 448 saturate;
#   * B_k: every column (one feature of one head) has a power-of-two scale e,
#     the smallest with max |B[:, f]| / e <= 448 (e = 1 for a zero column), and
#     is stored as round(B[:, f] / e): the division is exact;
#   * key latents: round(h), no scale;
#   * the key is K[t, f] = e_f sum_k round(h[t, k]) round(B[k, f] / e_f), and
#     everything after it (RoPE, scores, softmax, values) is unchanged.
# Parity status: fp8_e4m3_value / fp8_e4m3_round are pinned by the format's
# definition (all 256 codes, ties, saturation, subnormals) in
# tests/test_oracle_pins.py; attn_decode_fp8_keys is attn_decode on the rounded
# operands and is pinned through it.  What the rounding does to model accuracy
# is the paper's open question, not measured here.
# --------------------------------------------------------------------------

def fp8_e4m3_value(code) -> np.ndarray:
    """Value of an E4M3 byte (float64; NaN for 0x7f / 0xff)."""
    code = np.asarray(code, dtype=np.int64)
    sign = np.where(code & 0x80, -1.0, 1.0)
    e = (code >> 3) & 0xF
    m = (code & 7).astype(np.float64)
    val = np.where(e == 0, m / 8.0 * 2.0 ** -6, (1.0 + m / 8.0) * 2.0 ** (e.astype(np.float64) - 7.0))
    return np.where((e == 15) & ((code & 7) == 7), np.nan, sign * val)


def fp8_e4m3_round(x) -> np.ndarray:
    """Nearest E4M3 value (ties to the even mantissa), as float64; magnitudes
    above 448 (and infinities) give +-448."""
    x = np.asarray(x, dtype=np.float64)
    a = np.minimum(np.abs(x), 448.0)
    # spacing of the grid at a: 2^(floor(log2 a) - 3) in the normal range, 2^-9 below 2^-6
    with np.errstate(divide="ignore"):
        ex = np.floor(np.log2(np.where(a > 0, a, 1.0)))
    step = 2.0 ** (np.maximum(ex, -6.0) - 3.0)
    q = np.rint(a / step) * step                 # a / step is exact (power of two); rint rounds half to even
    return np.copysign(np.minimum(q, 448.0), x)


def fp8_weight_scales(Bj: np.ndarray) -> np.ndarray:
    """Power-of-two scale of every column of one group's reconstruction matrix [r, s*d_head]."""
    m = np.abs(np.asarray(Bj, dtype=np.float64)).max(axis=0)
    with np.errstate(divide="ignore"):
        e = 2.0 ** np.ceil(np.log2(np.where(m > 0, m, 448.0) / 448.0))
    return e


def fp8_keys(Hk, Bk, group_head_off, k_rank_off, d_head):
    """The operands of the low-precision reconstruction as float64 arrays: rounded latents, and
    the concatenated B_k with every column replaced by e_f * round(B[:, f] / e_f)."""
    H8 = fp8_e4m3_round(Hk)
    B8 = np.array(np.asarray(Bk, dtype=np.float64).reshape(-1), copy=True)
    off = 0
    for j in range(len(group_head_off) - 1):
        r = k_rank_off[j + 1] - k_rank_off[j]
        w = (group_head_off[j + 1] - group_head_off[j]) * d_head
        Bj = B8[off:off + r * w].reshape(r, w)
        e = fp8_weight_scales(Bj)
        Bj[:] = fp8_e4m3_round(Bj / e) * e
        off += r * w
    return H8, B8


def attn_decode_fp8_keys(q, q_pos, Hk, Hv, Bk, Bv, group_head_off, k_rank_off, v_rank_off,
                         d_head: int, rope_theta: float, k_pos=None, seq_lens=None, q_per_kv: int = 1) -> np.ndarray:
    """attn_decode with the keys rebuilt from E4M3-rounded latents and weights (see above)."""
    H8, B8 = fp8_keys(Hk, Bk, group_head_off, k_rank_off, d_head)
    return attn_decode(q, q_pos, H8, Hv, B8, Bv, group_head_off, k_rank_off, v_rank_off, d_head, rope_theta,
                       k_pos, seq_lens, q_per_kv)
