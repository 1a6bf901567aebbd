"""Pins for the CPU oracle: every check here compares oracle/ against something
other than itself — a textbook special case written independently, brute force
in pure Python, an algebraic identity the paper states, or a number the paper
prints (tests/golden/paper_values.json)."""

import cmath
import json
import math
import os

import numpy as np
import pytest

from oracle import palu_oracle as O
from workloads import synth

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.json")))


# ----------------------------------------------------------------- helpers

def textbook_rope_mha(q, q_pos, K, V, k_pos, theta):
    """Independent RoPE multi-head attention on full keys/values (Sec. 2.1,
    Eq. 2), RoPE written as complex multiplication of (x_f + i x_{f+d/2}) by
    exp(i pos theta^(-2f/d)).  q [n,d], K,V [L,n,d]."""
    n, d = q.shape
    half = d // 2
    w = np.array([theta ** (-2.0 * f / d) for f in range(half)])

    def rot(x, pos):
        z = (x[..., :half] + 1j * x[..., half:]) * np.exp(1j * np.multiply.outer(pos, w))
        return np.concatenate([z.real, z.imag], axis=-1)

    out = np.zeros((n, d))
    for i in range(n):
        qi = rot(q[i], np.float64(q_pos))
        Ki = rot(K[:, i, :], np.asarray(k_pos, dtype=np.float64))
        s = Ki @ qi / math.sqrt(d)
        e = np.exp(s - s.max())
        out[i] = (e / e.sum()) @ V[:, i, :]
    return out


def brute_force(q, q_pos, Hk, Hv, Bk_groups, Bv_groups, heads_per_group, d, theta, k_pos):
    """Pure-Python triple loops, scalar math only."""
    L = len(Hk)
    n = len(q)
    half = d // 2
    out = [[0.0] * d for _ in range(n)]
    for i in range(n):
        j, u = divmod(i, heads_per_group)
        Bk, Bv = Bk_groups[j], Bv_groups[j]
        rk, rv = len(Bk), len(Bv)
        k0 = sum(len(Bk_groups[g]) for g in range(j))
        v0 = sum(len(Bv_groups[g]) for g in range(j))

        def rope(vec, pos):
            o = [0.0] * d
            for f in range(half):
                ang = pos * theta ** (-2.0 * f / d)
                z = complex(vec[f], vec[f + half]) * cmath.exp(1j * ang)
                o[f], o[f + half] = z.real, z.imag
            return o

        qi = rope(q[i], q_pos)
        scores = []
        vals = []
        for t in range(L):
            k = [sum(Hk[t][k0 + a] * Bk[a][u * d + c] for a in range(rk)) for c in range(d)]
            v = [sum(Hv[t][v0 + a] * Bv[a][u * d + c] for a in range(rv)) for c in range(d)]
            k = rope(k, k_pos[t])
            scores.append(sum(qi[c] * k[c] for c in range(d)) / math.sqrt(d))
            vals.append(v)
        m = max(scores)
        e = [math.exp(s - m) for s in scores]
        z = sum(e)
        for t in range(L):
            for c in range(d):
                out[i][c] += e[t] / z * vals[t][c]
    return np.array(out)


def small_problem(seed=0, B=2, n=4, s=2, d=8, rk=(3, 5), rv=(4, 2), L=7):
    rng = np.random.default_rng(seed)
    gho = [j * s for j in range(n // s + 1)]
    kro = [0] + list(np.cumsum(rk))
    vro = [0] + list(np.cumsum(rv))
    Hk = rng.standard_normal((B, L, kro[-1]))
    Hv = rng.standard_normal((B, L, vro[-1]))
    Bk = [rng.standard_normal((rk[j], s * d)) for j in range(len(rk))]
    Bv = [rng.standard_normal((rv[j], s * d)) for j in range(len(rv))]
    q = rng.standard_normal((B, n, d))
    q_pos = np.array([L + 3, L - 1][:B])
    k_pos = np.arange(L) * 2 + 1
    return dict(gho=gho, kro=kro, vro=vro, Hk=Hk, Hv=Hv, Bk=Bk, Bv=Bv, q=q, q_pos=q_pos, k_pos=k_pos,
                d=d, s=s, L=L, B=B, n=n,
                Bk_flat=np.concatenate([b.reshape(-1) for b in Bk]),
                Bv_flat=np.concatenate([b.reshape(-1) for b in Bv]))


def run_oracle(p, theta=10000.0, **over):
    a = dict(p)
    a.update(over)
    return O.attn_decode(a["q"], a["q_pos"], a["Hk"], a["Hv"], a["Bk_flat"], a["Bv_flat"],
                         a["gho"], a["kro"], a["vro"], a["d"], theta, a.get("k_pos"), a.get("seq_lens"))


# ------------------------------------------------------- whole-pipeline pins

def test_brute_force_tiny():
    p = small_problem()
    got = run_oracle(p)
    for b in range(p["B"]):
        want = brute_force(p["q"][b].tolist(), int(p["q_pos"][b]), p["Hk"][b].tolist(), p["Hv"][b].tolist(),
                           [m.tolist() for m in p["Bk"]], [m.tolist() for m in p["Bv"]], p["s"], p["d"],
                           10000.0, p["k_pos"].tolist())
        np.testing.assert_allclose(got[b], want, rtol=1e-11, atol=1e-12)


@pytest.mark.parametrize("s,n", [(1, 4), (2, 4), (4, 4)])
def test_full_rank_orthogonal_equals_textbook_mha(s, n):
    """r = s*d_h with square orthogonal B: H = Y B^T reconstructs Y exactly, so
    the latent-cache attention must equal standard MHA on (K, V)."""
    d, L, B = 16, 37, 2
    rng = np.random.default_rng(5)
    ng = n // s
    w = s * d
    K = rng.standard_normal((B, L, n, d))
    V = rng.standard_normal((B, L, n, d))
    Bk = [np.linalg.qr(rng.standard_normal((w, w)))[0] for _ in range(ng)]
    Bv = [np.linalg.qr(rng.standard_normal((w, w)))[0] for _ in range(ng)]
    Hk = np.concatenate([K.reshape(B, L, ng, w)[:, :, j] @ Bk[j].T for j in range(ng)], axis=-1)
    Hv = np.concatenate([V.reshape(B, L, ng, w)[:, :, j] @ Bv[j].T for j in range(ng)], axis=-1)
    q = rng.standard_normal((B, n, d))
    q_pos = np.array([L - 1, L + 10])
    k_pos = np.arange(L)
    off = [j * w for j in range(ng + 1)]
    got = O.attn_decode(q, q_pos, Hk, Hv, np.concatenate([b.reshape(-1) for b in Bk]),
                        np.concatenate([b.reshape(-1) for b in Bv]),
                        [j * s for j in range(ng + 1)], off, off, d, 10000.0, k_pos)
    for b in range(B):
        want = textbook_rope_mha(q[b], q_pos[b], K[b], V[b], k_pos, 10000.0)
        np.testing.assert_allclose(got[b], want, rtol=1e-10, atol=1e-12)


def test_seq_lens_and_default_positions():
    p = small_problem()
    lens = np.array([4, 7])
    got = run_oracle(p, k_pos=None, seq_lens=lens)
    for b in range(2):
        L = lens[b]
        want = brute_force(p["q"][b].tolist(), int(p["q_pos"][b]), p["Hk"][b, :L].tolist(), p["Hv"][b, :L].tolist(),
                           [m.tolist() for m in p["Bk"]], [m.tolist() for m in p["Bv"]], p["s"], p["d"],
                           10000.0, list(range(L)))
        np.testing.assert_allclose(got[b], want, rtol=1e-11, atol=1e-12)


# ------------------------------------------------------------- factorisation

def test_svd_factor_reconstructs_and_eckart_young():
    rng = np.random.default_rng(1)
    W = rng.standard_normal((40, 24))
    A, Bm = synth.svd_factor(W, 24)
    assert np.linalg.norm(W - A @ Bm) <= 1e-13 * np.linalg.norm(W)
    sv = np.linalg.svd(W, compute_uv=False)
    for r in (4, 11, 20):
        A, Bm = synth.svd_factor(W, r)
        assert A.shape == (40, r) and Bm.shape == (r, 24)
        np.testing.assert_allclose(np.linalg.norm(W - A @ Bm), math.sqrt((sv[r:] ** 2).sum()), rtol=1e-10)
        # Sec. 2.2: A = U sqrt(S), B = sqrt(S) V^T  => A^T A = B B^T = diag(S_r)
        np.testing.assert_allclose(A.T @ A, np.diag(sv[:r]), atol=1e-10)
        np.testing.assert_allclose(Bm @ Bm.T, np.diag(sv[:r]), atol=1e-10)


def test_reconstruct_equals_factored_matrix():
    """K from the oracle equals x.W when A.B = W exactly (Sec. 3.1: y = x A B)."""
    rng = np.random.default_rng(2)
    d_model, d, s, ng, L = 24, 4, 2, 3, 9
    gho = [j * s for j in range(ng + 1)]
    ranks = [s * d] * ng
    ro = [0] + list(np.cumsum(ranks))
    Ws = [rng.standard_normal((d_model, s * d)) for _ in range(ng)]
    fac = [synth.svd_factor(W, s * d) for W in Ws]
    A = np.concatenate([f[0] for f in fac], axis=1)
    Bflat = np.concatenate([f[1].reshape(-1) for f in fac])
    x = rng.standard_normal((L, d_model))
    H = O.encode(x, A)
    Y = O.reconstruct(H, Bflat, gho, ro, d)
    np.testing.assert_allclose(Y, x @ np.concatenate(Ws, axis=1), rtol=1e-10, atol=1e-11)


def test_fused_vo_identity():
    """(p H_v) B_v == p (H_v B_v) (Eq. 4): contract in latent space first,
    then apply B_v, against the oracle's materialised-V order."""
    p = small_problem(seed=3)
    got = run_oracle(p)
    scores = O.attn_decode_scores(p["q"], p["q_pos"], p["Hk"], p["Bk_flat"], p["gho"], p["kro"], p["d"],
                                  10000.0, p["k_pos"])
    for b in range(p["B"]):
        P = O.softmax_rows(scores[b])
        for i in range(p["n"]):
            j, u = divmod(i, p["s"])
            o_lat = P[i] @ p["Hv"][b][:, p["vro"][j]:p["vro"][j + 1]]
            want = o_lat @ p["Bv"][j][:, u * p["d"]:(u + 1) * p["d"]]
            np.testing.assert_allclose(got[b, i], want, rtol=1e-10, atol=1e-12)


def test_latent_output_times_b_v_is_the_attention_output():
    """attn_decode_latent leaves the output in the value latent space (Sec. 3.1.1);
    multiplying head i's slice by its block of B_v must give attn_decode's output,
    and with L = 1 the latent output is the single value latent row itself."""
    p = small_problem(seed=5)
    full = run_oracle(p)
    lat = O.attn_decode_latent(p["q"], p["q_pos"], p["Hk"], p["Hv"], p["Bk_flat"], p["gho"], p["kro"], p["vro"],
                               p["d"], 10000.0, p["k_pos"])
    at = 0
    for i in range(p["n"]):
        j, u = divmod(i, p["s"])
        r = p["vro"][j + 1] - p["vro"][j]
        for b in range(p["B"]):
            np.testing.assert_allclose(lat[b, at:at + r] @ p["Bv"][j][:, u * p["d"]:(u + 1) * p["d"]], full[b, i],
                                       rtol=1e-10, atol=1e-12)
        at += r
    assert at == lat.shape[1]
    one = O.attn_decode_latent(p["q"], p["q_pos"], p["Hk"][:, :1], p["Hv"][:, :1], p["Bk_flat"], p["gho"], p["kro"],
                               p["vro"], p["d"], 10000.0)
    at = 0
    for i in range(p["n"]):
        j = i // p["s"]
        r = p["vro"][j + 1] - p["vro"][j]
        np.testing.assert_allclose(one[:, at:at + r], p["Hv"][:, 0, p["vro"][j]:p["vro"][j + 1]], rtol=1e-12)
        at += r


@pytest.mark.parametrize("qpk", [2, 4])
def test_grouped_query_reduces_to_one_query_per_kv_head(qpk):
    """Grouped-query attention (q_per_kv query heads share a key/value head): taking
    every q_per_kv-th query head, starting at w, leaves one query per key/value head,
    which is the multi-head case pinned above; heads i = kv * q_per_kv + w must agree.
    A head map of i % n_kv instead of i // q_per_kv fails this."""
    p = small_problem(seed=9)
    rng = np.random.default_rng(90)
    q = rng.standard_normal((p["B"], p["n"] * qpk, p["d"]))
    got = O.attn_decode(q, p["q_pos"], p["Hk"], p["Hv"], p["Bk_flat"], p["Bv_flat"], p["gho"], p["kro"], p["vro"],
                        p["d"], 10000.0, p["k_pos"], None, qpk)
    lat = O.attn_decode_latent(q, p["q_pos"], p["Hk"], p["Hv"], p["Bk_flat"], p["gho"], p["kro"], p["vro"],
                               p["d"], 10000.0, p["k_pos"], None, qpk)
    assert got.shape == (p["B"], p["n"] * qpk, p["d"])
    for w in range(qpk):
        want = run_oracle(p, q=q[:, w::qpk])
        np.testing.assert_allclose(got[:, w::qpk], want, rtol=1e-11, atol=1e-13)
    at = 0
    for i in range(p["n"] * qpk):
        j, u = divmod(i // qpk, p["s"])
        r = p["vro"][j + 1] - p["vro"][j]
        np.testing.assert_allclose(lat[:, at:at + r] @ p["Bv"][j][:, u * p["d"]:(u + 1) * p["d"]], got[:, i],
                                   rtol=1e-10, atol=1e-12)
        at += r
    assert at == lat.shape[1]


def test_several_queries_are_independent_decode_steps():
    """attn_decode_multi against a hand-rolled causal block: with the new tokens' rows
    appended, query j must equal textbook softmax attention over rows [0, L - n_q + j]
    of the rebuilt K and V (a dropped '+ 1' in the row count or a shared position fails)."""
    p = small_problem(seed=12, L=9)
    n_q, L, d = 3, p["L"], p["d"]
    rng = np.random.default_rng(120)
    q = rng.standard_normal((p["B"], n_q, p["n"], d))
    q_len = np.array([[L - n_q + j + 1 for j in range(n_q)]] * p["B"])
    q_pos = q_len - 1
    got = O.attn_decode_multi(q, q_pos, q_len, p["Hk"], p["Hv"], p["Bk_flat"], p["Bv_flat"], p["gho"], p["kro"],
                              p["vro"], d, 10000.0)
    for b in range(p["B"]):
        K = O.reconstruct(p["Hk"][b], p["Bk_flat"], p["gho"], p["kro"], d).reshape(L, p["n"], d)
        V = O.reconstruct(p["Hv"][b], p["Bv_flat"], p["gho"], p["vro"], d).reshape(L, p["n"], d)
        Kr = O.rope_rotate(K, np.arange(L)[:, None], 10000.0)
        for j in range(n_q):
            n_rows = L - n_q + j + 1
            for i in range(p["n"]):
                qr = O.rope_rotate(q[b, j, i][None], np.array([n_rows - 1]), 10000.0)[0]
                sc = Kr[:n_rows, i] @ qr / math.sqrt(d)
                w = np.exp(sc - sc.max())
                want = (w / w.sum()) @ V[:n_rows, i]
                np.testing.assert_allclose(got[b, j, i], want, rtol=1e-10, atol=1e-12)


def test_zero_positions_equal_fused_qk_form():
    """With every position 0 RoPE is the identity and the score must equal
    (q B_k^T) H_k^T / sqrt(d_h) (Eq. 5)."""
    p = small_problem(seed=4)
    L = p["L"]
    sc = O.attn_decode_scores(p["q"], np.zeros(p["B"], int), p["Hk"], p["Bk_flat"], p["gho"], p["kro"], p["d"],
                              10000.0, np.zeros(L, int))
    for b in range(p["B"]):
        for i in range(p["n"]):
            j, u = divmod(i, p["s"])
            qt = p["q"][b, i] @ p["Bk"][j][:, u * p["d"]:(u + 1) * p["d"]].T
            want = p["Hk"][b][:, p["kro"][j]:p["kro"][j + 1]] @ qt / math.sqrt(p["d"])
            np.testing.assert_allclose(sc[b][i], want, rtol=1e-11, atol=1e-12)
    # and theta <= 0 (non-RoPE attention) gives the same thing at any position
    sc2 = O.attn_decode_scores(p["q"], p["q_pos"], p["Hk"], p["Bk_flat"], p["gho"], p["kro"], p["d"],
                               0.0, p["k_pos"])
    for b in range(p["B"]):
        np.testing.assert_allclose(sc2[b], sc[b], rtol=1e-12)


# ----------------------------------------------------------------------- RoPE

def test_rope_properties():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((5, 3, 16))
    pos = np.array([0, 1, 77, 4095, 65535])[:, None]
    y = O.rope_rotate(x, pos, 10000.0)
    np.testing.assert_allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-12)
    np.testing.assert_allclose(y[..., :8] ** 2 + y[..., 8:] ** 2, x[..., :8] ** 2 + x[..., 8:] ** 2, rtol=1e-10)
    np.testing.assert_array_equal(y[0], x[0])                       # position 0 is the identity
    # frequency of pair f is theta^(-2f/d): pair 0 turns by exactly pos radians,
    # the last pair by pos * theta^(-(d-2)/d)
    e = np.zeros((1, 16))
    e[0, 0] = 1.0
    r = O.rope_rotate(e, np.array([3]), 10000.0)
    np.testing.assert_allclose([r[0, 0], r[0, 8]], [math.cos(3.0), math.sin(3.0)], rtol=1e-14)
    e = np.zeros((1, 16))
    e[0, 7] = 1.0
    r = O.rope_rotate(e, np.array([1000]), 10000.0)
    ang = 1000 * 10000.0 ** (-14.0 / 16.0)
    np.testing.assert_allclose([r[0, 7], r[0, 15]], [math.cos(ang), math.sin(ang)], rtol=1e-12)
    # composition: rotating by a then b equals rotating by a + b
    z = O.rope_rotate(O.rope_rotate(x[:1], np.array([[11]]), 10000.0), np.array([[31]]), 10000.0)
    np.testing.assert_allclose(z, O.rope_rotate(x[:1], np.array([[42]]), 10000.0), rtol=1e-10, atol=1e-12)


def test_output_depends_only_on_relative_position():
    p = small_problem(seed=7)
    a = run_oracle(p)
    b = run_oracle(p, q_pos=p["q_pos"] + 1000, k_pos=p["k_pos"] + 1000)
    np.testing.assert_allclose(a, b, rtol=1e-8, atol=1e-10)


# -------------------------------------------------------------------- softmax

def test_softmax_pins():
    p = small_problem(seed=8)
    sc = O.attn_decode_scores(p["q"], p["q_pos"], p["Hk"], p["Bk_flat"], p["gho"], p["kro"], p["d"],
                              10000.0, p["k_pos"])
    P = O.softmax_rows(sc[0])
    np.testing.assert_allclose(P.sum(axis=-1), 1.0, rtol=1e-14)
    np.testing.assert_allclose(O.softmax_rows(sc[0] + 123.0), P, rtol=1e-10)
    np.testing.assert_allclose(O.softmax_rows(np.log(np.array([[1.0, 2.0, 5.0]]))), [[0.125, 0.25, 0.625]], rtol=1e-14)
    # L = 1: the output is the single value row
    one = run_oracle(p, Hk=p["Hk"][:, :1], Hv=p["Hv"][:, :1], k_pos=p["k_pos"][:1])
    V = O.reconstruct(p["Hv"][0, :1], p["Bv_flat"], p["gho"], p["vro"], p["d"])
    np.testing.assert_allclose(one[0].reshape(-1), V[0], rtol=1e-12)
    # identical key latents at identical positions: uniform attention -> mean of V
    Hk = np.repeat(p["Hk"][:, :1], p["L"], axis=1)
    same = run_oracle(p, Hk=Hk, k_pos=np.full(p["L"], 5))
    V = O.reconstruct(p["Hv"][1], p["Bv_flat"], p["gho"], p["vro"], p["d"])
    np.testing.assert_allclose(same[1].reshape(-1), V.mean(axis=0), rtol=1e-10, atol=1e-12)


def test_split_k_combine_equals_unsplit():
    """Merging per-chunk (m, l, o) partials reproduces the full softmax-weighted
    sum for any partition of the sequence."""
    p = small_problem(seed=9, L=23)
    full = run_oracle(p)
    sc = O.attn_decode_scores(p["q"], p["q_pos"], p["Hk"], p["Bk_flat"], p["gho"], p["kro"], p["d"],
                              10000.0, p["k_pos"])
    cuts = [0, 5, 6, 17, 23]
    for b in range(p["B"]):
        V = O.reconstruct(p["Hv"][b], p["Bv_flat"], p["gho"], p["vro"], p["d"]).reshape(23, p["n"], p["d"])
        for i in range(p["n"]):
            parts = []
            for a, z in zip(cuts[:-1], cuts[1:]):
                s = sc[b][i, a:z]
                m = s.max()
                e = np.exp(s - m)
                parts.append((m, e.sum(), e @ V[a:z, i]))
            M = max(m for m, _, _ in parts)
            num = sum(math.exp(m - M) * o for m, _, o in parts)
            den = sum(math.exp(m - M) * l for m, l, _ in parts)
            np.testing.assert_allclose(num / den, full[b, i], rtol=1e-10, atol=1e-12)


# ------------------------------------------------------------------- Hadamard

def test_hadamard_fold_changes_nothing():
    R = synth.hadamard(16)
    np.testing.assert_allclose(R @ R.T, np.eye(16), atol=1e-14)
    np.testing.assert_allclose(R, R.T)
    assert set(np.unique(np.round(np.abs(R) * 4, 12))) == {1.0}
    layer = synth.uniform_layer(4, 2, 16, d_head=8)
    Ak, Bk = synth.make_factors(layer, 0, "k", d_model=32)
    Av, Bv = synth.make_factors(layer, 0, "v", d_model=32)
    Akr, Bkr = synth.make_factors(layer, 0, "k", d_model=32, rotate=True)
    Avr, Bvr = synth.make_factors(layer, 0, "v", d_model=32, rotate=True)
    rng = np.random.default_rng(0)
    x = rng.standard_normal((1, 12, 32))
    q = rng.standard_normal((1, 4, 8))
    a = O.attn_decode(q, [11], O.encode(x, Ak), O.encode(x, Av), Bk, Bv, layer.group_head_off,
                      layer.k_rank_off, layer.v_rank_off, 8, 10000.0)
    b = O.attn_decode(q, [11], O.encode(x, Akr), O.encode(x, Avr), Bkr, Bvr, layer.group_head_off,
                      layer.k_rank_off, layer.v_rank_off, 8, 10000.0)
    np.testing.assert_allclose(a, b, rtol=1e-9, atol=1e-12)
    assert np.abs(O.encode(x, Ak) - O.encode(x, Akr)).max() > 1e-3       # the latents themselves do change


# ------------------------------------------------------------------ quantizer

def test_pack_unpack_roundtrip_all_bytes():
    allb = np.arange(256, dtype=np.uint8)
    codes = O.unpack_int4(allb)
    np.testing.assert_array_equal(codes[0::2], allb & 15)
    np.testing.assert_array_equal(codes[1::2], allb >> 4)
    np.testing.assert_array_equal(O.pack_int4(codes), allb)
    rng = np.random.default_rng(0)
    c = rng.integers(0, 16, size=(7, 64)).astype(np.uint8)
    np.testing.assert_array_equal(O.unpack_int4(O.pack_int4(c)), c)
    assert O.pack_int4(np.array([3, 10], np.uint8))[0] == 0xA3          # low nibble = even channel


def test_quantizer_hand_examples():
    # values 0..15 repeated: s = 1, z = 0, codes = values (Appendix A with B = 4)
    x = np.tile(np.arange(16, dtype=np.float32), 8)[None, :]
    packed, s, z = O.quant_latent(x, block=128)
    assert s.dtype == np.float16 and z.dtype == np.float16
    assert float(s[0, 0]) == 1.0 and float(z[0, 0]) == 0.0
    np.testing.assert_array_equal(O.unpack_int4(packed)[0], x[0].astype(np.uint8))
    # shift by -4 and scale by 0.5: min = -2, s = 0.5, z = round(2 / 0.5) = 4, codes unchanged
    x2 = (x - 4.0) * 0.5
    packed2, s2, z2 = O.quant_latent(x2, block=128)
    assert float(s2[0, 0]) == 0.5 and float(z2[0, 0]) == 4.0
    np.testing.assert_array_equal(packed2, packed)
    np.testing.assert_array_equal(O.dequant_latent(packed2, s2, z2), x2.astype(np.float64))
    # all-positive block: the zero-point is negative and is not clamped
    x3 = x + 32.0
    _, s3, z3 = O.quant_latent(x3, block=128)
    assert float(s3[0, 0]) == 1.0 and float(z3[0, 0]) == -32.0
    # constant block: s := 1, every code equals round(c) + z = 0
    x4 = np.full((1, 128), 3.0, np.float32)
    p4, s4, z4 = O.quant_latent(x4, block=128)
    assert float(s4[0, 0]) == 1.0 and float(z4[0, 0]) == -3.0 and not p4.any()
    # ties round to even: x/s = 0.5 -> 0, 1.5 -> 2, 2.5 -> 2
    x5 = np.zeros((1, 128), np.float32)
    x5[0, :5] = [0.0, 15.0, 0.5, 1.5, 2.5]
    p5, s5, z5 = O.quant_latent(x5, block=128)
    np.testing.assert_array_equal(O.unpack_int4(p5)[0, :5], [0, 15, 0, 2, 2])
    # two blocks are independent
    x6 = np.concatenate([x, x2], axis=1)
    p6, s6, z6 = O.quant_latent(x6, block=128)
    np.testing.assert_array_equal(s6[0], [1.0, 0.5])
    np.testing.assert_array_equal(z6[0], [0.0, 4.0])


@pytest.mark.parametrize("bits", [2, 3])
def test_low_bit_formats_and_quantizer(bits):
    """2- and 3-bit latents (Sec. 4.4): byte layouts spelled out by hand, round trip over random
    codes, hand examples of Appendix A with 2^B - 1 levels, and the half-step error bound."""
    top = (1 << bits) - 1
    # layout, by hand: channels 0..7 = 1, 2, 3, 0, 3, 3, 0, 1 (2 bits) / 5, 2, 7, 0, 3, 6, 4, 1 (3 bits)
    if bits == 2:
        c = np.array([[1, 2, 3, 0, 3, 3, 0, 1]], np.uint8)
        want = [1 | 2 << 2 | 3 << 4 | 0 << 6, 3 | 3 << 2 | 0 << 4 | 1 << 6]
    else:
        c = np.array([[5, 2, 7, 0, 3, 6, 4, 1]], np.uint8)
        low = [1 | 2 << 2 | 3 << 4 | 0 << 6, 3 | 2 << 2 | 0 << 4 | 1 << 6]
        high = [1 << 0 | 0 << 1 | 1 << 2 | 0 << 3 | 0 << 4 | 1 << 5 | 1 << 6 | 0 << 7]
        want = low + high
    np.testing.assert_array_equal(O.pack_codes(c, bits)[0], np.array(want, np.uint8))
    rng = np.random.default_rng(bits)
    codes = rng.integers(0, top + 1, size=(5, 256)).astype(np.uint8)
    packed = O.pack_codes(codes, bits)
    assert packed.shape == (5, 256 * bits // 8)
    np.testing.assert_array_equal(O.unpack_codes(packed, bits), codes)
    # values 0..top repeated: s = 1, z = 0, codes = values; shifted and scaled: same codes
    x = np.tile(np.arange(top + 1, dtype=np.float32), 128 // (top + 1))[None, :]
    pk, sc, zp = O.quant_latent(x, bits=bits)
    assert float(sc[0, 0]) == 1.0 and float(zp[0, 0]) == 0.0
    np.testing.assert_array_equal(O.unpack_codes(pk, bits)[0], x[0].astype(np.uint8))
    x2 = (x - 1.0) * 0.25
    pk2, sc2, zp2 = O.quant_latent(x2, bits=bits)
    assert float(sc2[0, 0]) == 0.25 and float(zp2[0, 0]) == 1.0
    np.testing.assert_array_equal(pk2, pk)
    np.testing.assert_array_equal(O.dequant_latent(pk2, sc2, zp2, bits=bits), x2.astype(np.float64))
    # random rows: every code within range, error at most half a step (plus the fp16 rounding of s and z)
    h = (rng.standard_normal((20, 256)) * rng.uniform(0.1, 10, size=(20, 1))).astype(np.float16).astype(np.float32)
    pk3, sc3, zp3 = O.quant_latent(h, bits=bits)
    assert O.unpack_codes(pk3, bits).max() <= top
    err = np.abs(O.dequant_latent(pk3, sc3, zp3, bits=bits) - h)
    step = np.repeat(sc3.astype(np.float64), 128, axis=-1)
    assert (err <= 0.51 * step + 1e-3 * np.abs(h).max()).all()
    # 4 bits through the same entry points is the int4 format
    np.testing.assert_array_equal(O.pack_codes(codes & 3, 4), O.pack_int4(codes & 3))


def test_quantizer_properties_random():
    rng = np.random.default_rng(11)
    x = (rng.standard_normal((64, 512)) * rng.uniform(0.01, 30, size=(64, 1))).astype(np.float16).astype(np.float32)
    x[:8] += 5.0
    packed, s, z = O.quant_latent(x, block=128)
    codes = O.unpack_int4(packed)
    assert codes.max() <= 15
    xb = x.reshape(64, 4, 128)
    cb = codes.reshape(64, 4, 128)
    amin = xb.argmin(axis=-1)
    np.testing.assert_array_equal(np.take_along_axis(cb, amin[..., None], -1)[..., 0], 0)   # min -> code 0
    deq = O.dequant_latent(packed, s, z).reshape(64, 4, 128)
    sf = s.astype(np.float64)[..., None]
    err = np.abs(deq - xb)
    unclamped = cb < 15
    # |x - dequant| <= s/2 when not clamped (plus float32 rounding of x/s), <= 1.5 s at the top code
    assert (err[unclamped] <= (0.5 + 1e-3) * np.broadcast_to(sf, err.shape)[unclamped]).all()
    assert (err <= 1.5 * sf + 1e-6).all()
    # z is an integer and s is the float16 rounding of range/15
    assert (z.astype(np.float64) == np.rint(z.astype(np.float64))).all()
    rng_ = (xb.max(-1) - xb.min(-1)).astype(np.float64)
    np.testing.assert_allclose(s.astype(np.float64), rng_ / 15.0, rtol=2 ** -10)


def test_attention_on_dequantized_latents_close_to_unquantized():
    """4-bit latents with the Hadamard fold perturb the output only mildly
    (sanity that dequantization and the fold are wired the right way round)."""
    layer = synth.uniform_layer(4, 2, 128, d_head=64)
    case = synth.make_case_svd(layer, 1, 64, seed=1, rotate=True, d_model=256)
    pk, sk, zk = O.quant_latent(case.Hk)
    pv, sv, zv = O.quant_latent(case.Hv)
    args = (layer.group_head_off, layer.k_rank_off, layer.v_rank_off, 64, 10000.0)
    ref = O.attn_decode(case.q, case.q_pos, case.Hk, case.Hv, case.Bk, case.Bv, *args)
    got = O.attn_decode(case.q, case.q_pos, O.dequant_latent(pk, sk, zk), O.dequant_latent(pv, sv, zv),
                        case.Bk, case.Bv, *args)
    assert np.abs(got - ref).max() < 0.25 * np.abs(ref).max()
    assert np.abs(got - ref).max() > 0


# --------------------------------------------------------- printed closed forms

def test_storage_ratio_printed_values():
    for row in GOLD["storage_ratio"]:
        assert O.storage_ratio(row["m"], row["n"], row["r"]) == pytest.approx(row["value"], rel=1e-12)


def test_kv_cache_size_table():
    g = GOLD["kv_size_GB_at_128K_llama2_7b"]
    base = None
    for row in g["rows"]:
        gb = O.kv_cache_bytes(g["layers"], g["seq"], g["hidden"], row["keep"], row["bits"]) / 2 ** 30
        assert gb == pytest.approx(row["GB"], abs=0.05)
        if base is None:
            base = gb
        if "rate_pct" in row:
            assert 100.0 * (1.0 - gb / base) == pytest.approx(row["rate_pct"], abs=0.0051)


def test_reconstruction_cost_ratios():
    g = GOLD["reconstruction_cost_ratio"]
    for spec in (g, g["fig3"]):
        n, s = spec["n_heads"], spec["group_size"]
        total = 64 * n                        # same total latent size for all three schemes
        def macs(gs):
            layer = synth.uniform_layer(n, gs, total // (n // gs))
            return O.reconstruction_macs_per_token(layer.group_head_off, layer.k_rank_off, layer.d_head)
        assert macs(n) == spec["joint_over_multi"] * macs(1)
        assert macs(s) == spec["group_over_multi"] * macs(1)
        assert macs(n) == (n // s) * macs(s)


# ---------------------------------------------- the pins bite: planted mistakes

@pytest.mark.parametrize("mutation", ["rope_sign", "no_scale", "transposed_B", "wrong_head_slice", "interleaved_rope"])
def test_planted_mistake_is_caught(monkeypatch, mutation):
    """Plant one plausible mistake in the oracle and check that the textbook
    special case no longer matches."""
    if mutation == "rope_sign":
        orig = O.rope_rotate
        monkeypatch.setattr(O, "rope_rotate", lambda x, pos, th: orig(x, -np.asarray(pos), th) if np.ndim(x) == 3 else orig(x, pos, th))
    elif mutation == "no_scale":
        orig_s = O.attn_decode_scores
        monkeypatch.setattr(O, "attn_decode_scores", lambda *a, **k: [s * math.sqrt(a[6]) for s in orig_s(*a, **k)])
    elif mutation == "transposed_B":
        orig_g = O._group_matrix
        monkeypatch.setattr(O, "_group_matrix", lambda *a: orig_g(*a).T.copy().reshape(orig_g(*a).shape))
    elif mutation == "wrong_head_slice":
        orig_r = O.reconstruct
        monkeypatch.setattr(O, "reconstruct", lambda *a: np.roll(orig_r(*a), a[4], axis=1))
    elif mutation == "interleaved_rope":
        def inter(x, pos, theta):
            x = np.asarray(x, float)
            d = x.shape[-1]
            phi = np.asarray(pos, float)[..., None] * O.rope_inv_freq(d, theta)
            c, s = np.cos(phi), np.sin(phi)
            y = np.empty_like(x)
            y[..., 0::2] = x[..., 0::2] * c - x[..., 1::2] * s
            y[..., 1::2] = x[..., 1::2] * c + x[..., 0::2] * s
            return y
        monkeypatch.setattr(O, "rope_rotate", inter)
    with pytest.raises(AssertionError):
        test_full_rank_orthogonal_equals_textbook_mha(2, 4)


def test_empty_sequence_is_the_empty_sum():
    """A sequence with no cached row: every sum of Eq. 2 is empty, the output is zero, and the
    other sequences of the batch are what they are alone."""
    layer = synth.Layer(4, 128, [0, 2, 4], [0, 128, 256], [0, 128, 192])
    case = synth.make_case_orthonormal(layer, 2, 40, seed=3)
    args = (layer.group_head_off, layer.k_rank_off, layer.v_rank_off, 128, 10000.0)
    both = O.attn_decode(case.q, [0, 39], case.Hk, case.Hv, case.Bk, case.Bv, *args, None, np.array([0, 40]))
    alone = O.attn_decode(case.q[1:], [39], case.Hk[1:], case.Hv[1:], case.Bk, case.Bv, *args, None, None)
    assert not both[0].any()
    np.testing.assert_array_equal(both[1], alone[0])
    assert O.softmax_rows(np.zeros((3, 0))).shape == (3, 0)


# --------------------------------------------------------------------------
# 8-bit float operands of the low-precision key reconstruction (Sec. 4.5.2, last paragraph)
# --------------------------------------------------------------------------

def _e4m3_table():
    """All finite E4M3 values written out from the format's definition, independently of the oracle."""
    vals = []
    for code in range(256):
        s, e, m = code >> 7, (code >> 3) & 15, code & 7
        if e == 15 and m == 7:
            continue
        v = (m / 8) * 2.0 ** -6 if e == 0 else (1 + m / 8) * 2.0 ** (e - 7)
        vals.append(-v if s else v)
    return np.array(sorted(set(vals)))


def test_fp8_e4m3_codes_and_rounding():
    tab = _e4m3_table()
    assert tab.max() == 448.0 and tab.min() == -448.0 and len(tab) == 253        # 254 finite codes, +0 and -0 coincide
    assert np.abs(tab[tab != 0]).min() == 2.0 ** -9
    # every code decodes to its table value; every table value rounds to itself
    dec = O.fp8_e4m3_value(np.arange(256))
    assert np.isnan(dec[0x7f]) and np.isnan(dec[0xff]) and np.isnan(dec).sum() == 2
    assert set(dec[~np.isnan(dec)].tolist()) == set(tab.tolist())
    np.testing.assert_array_equal(O.fp8_e4m3_round(tab), tab)
    # hand examples: 1.0625 is halfway between 1.0 (mantissa 0, even) and 1.125 (mantissa 1): down; 1.1875 between
    # 1.125 (odd) and 1.25 (even): up; 17 -> 16 (tie, even), 19 -> 20 (tie: 18 has mantissa 1, 20 mantissa 2)
    np.testing.assert_array_equal(O.fp8_e4m3_round([1.0625, 1.1875, 17.0, 19.0, 0.3, -5.3, 1e9, -np.inf, 460.0, 2.0 ** -10, 3 * 2.0 ** -10]),
                                  [1.0, 1.25, 16.0, 20.0, 0.3125, -5.5, 448.0, -448.0, 448.0, 0.0, 2.0 ** -8])
    # brute force: nearest table value for random inputs, ties excluded
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(4000) * 3, rng.standard_normal(2000) * 200, rng.standard_normal(2000) * 0.01])
    d = np.abs(x[:, None] - tab[None, :])
    near = tab[np.argmin(d, axis=1)]
    srt = np.sort(d, axis=1)
    clear = srt[:, 1] - srt[:, 0] > 1e-12
    np.testing.assert_array_equal(O.fp8_e4m3_round(x)[clear], np.clip(near, -448, 448)[clear])
    # half-ulp bound in the normal range: relative error at most 2^-4
    xn = x[(np.abs(x) >= 2.0 ** -6) & (np.abs(x) <= 448)]
    assert (np.abs(O.fp8_e4m3_round(xn) - xn) <= np.abs(xn) * 2.0 ** -4).all()


def test_fp8_weight_scales_and_key_operands():
    rng = np.random.default_rng(1)
    B = rng.standard_normal((64, 256)) * rng.uniform(1e-3, 50.0, size=(1, 256))
    B[:, 5] = 0.0
    e = O.fp8_weight_scales(B)
    assert e[5] == 1.0
    assert (np.log2(e) == np.round(np.log2(e))).all()                       # powers of two
    m = np.abs(B).max(axis=0)
    nz = m > 0
    assert ((m[nz] / e[nz] <= 448) & (m[nz] / e[nz] > 224)).all()           # the smallest such power of two
    # multiplying a column by a power of two changes its scale, not its codes: the operands scale exactly
    layer = ([0, 2], [0, 64], 128)
    H = rng.standard_normal((1, 9, 64))
    H8, B8 = O.fp8_keys(H, B.reshape(-1), layer[0], layer[1], layer[2])
    B2 = B.copy()
    B2[:, 7] *= 2.0 ** 5
    _, B8b = O.fp8_keys(H, B2.reshape(-1), layer[0], layer[1], layer[2])
    np.testing.assert_array_equal(B8b.reshape(64, 256)[:, 7], B8.reshape(64, 256)[:, 7] * 2.0 ** 5)
    # operands are on the grid: latents as they are, weights after division by their scale
    np.testing.assert_array_equal(O.fp8_e4m3_round(H8), H8)
    np.testing.assert_array_equal(O.fp8_e4m3_round(B8.reshape(64, 256) / e), B8.reshape(64, 256) / e)
    assert np.abs(B8.reshape(64, 256) - B).max() <= (np.abs(B) * 2.0 ** -4 + e * 2.0 ** -10).max()


def test_attn_decode_fp8_keys_is_attention_on_the_rounded_operands():
    rng = np.random.default_rng(2)
    gho, kro, vro, d = [0, 2], [0, 32], [0, 32], 8
    q = rng.standard_normal((2, 2, d))
    Hk, Hv = rng.standard_normal((2, 11, 32)) * 2, rng.standard_normal((2, 11, 32))
    Bk, Bv = rng.standard_normal(32 * 2 * d), rng.standard_normal(32 * 2 * d)
    got = O.attn_decode_fp8_keys(q, [10, 4], Hk, Hv, Bk, Bv, gho, kro, vro, d, 10000.0)
    H8, B8 = O.fp8_keys(Hk, Bk, gho, kro, d)
    np.testing.assert_array_equal(got, O.attn_decode(q, [10, 4], H8, Hv, B8, Bv, gho, kro, vro, d, 10000.0))
    # operands already on the grid (small integers, columns whose largest entry is a power of two <= 448): nothing changes
    Hi = rng.integers(-8, 9, size=(2, 11, 32)).astype(np.float64)
    Bi = rng.integers(-4, 5, size=(32, 2 * d)).astype(np.float64)
    Bi[0, :] = 4.0
    np.testing.assert_allclose(O.attn_decode_fp8_keys(q, [10, 4], Hi, Hv, Bi.reshape(-1), Bv, gho, kro, vro, d, 10000.0),
                               O.attn_decode(q, [10, 4], Hi, Hv, Bi.reshape(-1), Bv, gho, kro, vro, d, 10000.0), rtol=0, atol=1e-13)
