"""Pins for the CPU oracle: it is checked here against things other than itself.

Each test names the passage of the paper, or the piece of mathematics, that fixes the expected
value.  The independent references in this file are written differently from the oracle on
purpose: the RoPElite score equation is evaluated in its RELATIVE form (Section 2.2 eq. 1b and
the Section 3.1 score equation) from un-rotated full keys with explicit 2x2 matrices; ordinary
RoPE attention uses complex multiplication; the brute force uses Python floats and loops only.
"""
import cmath
import math
import os

import numpy as np
import pytest

import elitekv_synth as synth
from oracle import elitekv_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
TOL = 1e-11


# ----------------------------------------------------------------------------------------------
# independent references (none of them calls the oracle)
# ----------------------------------------------------------------------------------------------
def _theta_plain(d_h, base):
    return [base ** (-(2.0 * i) / d_h) for i in range(d_h // 2)]


def _rot_matrix(a):
    # row-vector convention: (u, v) R(a) = (u cos a - v sin a, u sin a + v cos a)
    return np.array([[math.cos(a), math.sin(a)], [-math.sin(a), math.cos(a)]])


def ropelite_attention_relative(q, q_pos, k_raw, v, k_pos, elite_sets, base):
    """Section 3.1 score equation, relative form, then Section 2.1 softmax attention.

    q [n_h, d_h]; k_raw, v [S, n_h, d_h] un-rotated full keys / values; k_pos [S];
    elite_sets: list of per-head iterables of chunk indices.
    """
    S, n_h, d_h = k_raw.shape
    th = _theta_plain(d_h, base)
    out = np.zeros((n_h, d_h))
    for h in range(n_h):
        elite = set(int(i) for i in elite_sets[h])
        s = []
        for j in range(S):
            acc = 0.0
            for i in range(d_h // 2):
                qi = q[h, 2 * i:2 * i + 2]
                ki = k_raw[j, h, 2 * i:2 * i + 2]
                if i in elite:
                    acc += float(qi @ _rot_matrix((int(q_pos) - int(k_pos[j])) * th[i]) @ ki)
                else:
                    acc += float(qi @ ki)
            s.append(acc / math.sqrt(d_h))
        mx = max(s)
        e = [math.exp(t - mx) for t in s]
        z = sum(e)
        for j in range(S):
            out[h] += (e[j] / z) * v[j, h]
    return out


def rope_attention_complex(q, q_pos, k_raw, v, k_pos, base):
    """Ordinary RoPE attention, absolute form (Section 2.2 eq. 1a), via complex numbers."""
    S, n_h, d_h = k_raw.shape
    th = _theta_plain(d_h, base)
    out = np.zeros((n_h, d_h))
    for h in range(n_h):
        qc = [complex(q[h, 2 * i], q[h, 2 * i + 1]) * cmath.exp(1j * int(q_pos) * th[i])
              for i in range(d_h // 2)]
        s = []
        for j in range(S):
            kc = [complex(k_raw[j, h, 2 * i], k_raw[j, h, 2 * i + 1])
                  * cmath.exp(1j * int(k_pos[j]) * th[i]) for i in range(d_h // 2)]
            # real inner product of the two 2-vectors = Re(q * conj(k))
            s.append(sum((a * b.conjugate()).real for a, b in zip(qc, kc)) / math.sqrt(d_h))
        mx = max(s)
        e = [math.exp(t - mx) for t in s]
        z = sum(e)
        for j in range(S):
            out[h] += (e[j] / z) * v[j, h]
    return out


def exact_elitekv_weights(rng, Wk, Wv, elite_idx):
    """Lossless J-LRD factors of [W^k_ehat, W^v] with d_c = d (Section 3.2): A = random
    orthogonal, B = A^T [W^k_ehat, W^v]."""
    d, n_h, d_h = Wk.shape
    r = elite_idx.shape[1]
    W_ke = np.zeros((d, n_h, 2 * r))
    ne_cols = []
    for h in range(n_h):
        el = set()
        for j in range(r):
            i = int(elite_idx[h, j])
            W_ke[:, h, 2 * j] = Wk[:, h, 2 * i]
            W_ke[:, h, 2 * j + 1] = Wk[:, h, 2 * i + 1]
            el.update((2 * i, 2 * i + 1))
        ne_cols.append(Wk[:, h, [t for t in range(d_h) if t not in el]])
    M = np.concatenate(ne_cols + [Wv[:, h, :] for h in range(n_h)], axis=1)
    A, _ = np.linalg.qr(rng.standard_normal((d, d)))
    Bm = A.T @ M
    n_ne = n_h * (d_h - 2 * r)
    W_uk = Bm[:, :n_ne].reshape(d, n_h, d_h - 2 * r)
    W_uv = Bm[:, n_ne:].reshape(d, n_h, d_h)
    return W_ke, A, W_uk, W_uv


def _full_model(seed, d, n_h, d_h, r, S):
    rng = np.random.default_rng(seed)
    Wk = rng.standard_normal((d, n_h, d_h)) / math.sqrt(d)
    Wv = rng.standard_normal((d, n_h, d_h)) / math.sqrt(d)
    idx = synth.draw_elite_idx(rng, n_h, d_h, r) if r else np.zeros((n_h, 0), dtype=np.int32)
    x = rng.standard_normal((S, d))
    q = rng.standard_normal((1, n_h, d_h))
    pos = rng.permutation(5 * S)[:S].astype(np.int64)       # arbitrary distinct positions
    q_pos = int(5 * S + 3)
    return rng, Wk, Wv, idx, x, q, pos, q_pos


def _oracle_end_to_end(W_ke, W_dkv, W_uk, W_uv, idx, x, pos, q, q_pos, d_h, base):
    ke, c = orc.append(x, pos, W_ke, W_dkv, idx, d_h, base)
    return orc.decode_attn(q, [q_pos], ke[None], c[None], [x.shape[0]], W_uk, W_uv, idx, d_h, base)[0]


# ----------------------------------------------------------------------------------------------
# P1: r = d_h/2 and exact factors  ==>  ordinary RoPE attention
# (Section 3.1: the elite set then is all of I; Table 2's caption: r = 64 is the original model)
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("seed", [1, 2])
def test_p1_full_rope_equals_standard_attention(seed):
    d, n_h, d_h, S, base = 24, 3, 8, 7, 10000.0
    rng, Wk, Wv, idx, x, q, pos, q_pos = _full_model(seed, d, n_h, d_h, d_h // 2, S)
    W_ke, A, W_uk, W_uv = exact_elitekv_weights(rng, Wk, Wv, idx)
    assert W_uk.shape[2] == 0
    got = _oracle_end_to_end(W_ke, A, W_uk, W_uv, idx, x, pos, q, q_pos, d_h, base)
    k_raw = np.einsum("sd,dhe->she", x, Wk)
    v = np.einsum("sd,dhe->she", x, Wv)
    ref = rope_attention_complex(q[0], q_pos, k_raw, v, pos, base)
    assert np.max(np.abs(got - ref)) < TOL


# ----------------------------------------------------------------------------------------------
# P2: any r, exact factors ==> the RoPElite score equation evaluated directly (Section 3.1)
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("r", [1, 2, 3])
def test_p2_matches_ropelite_equation_relative_form(r):
    d, n_h, d_h, S, base = 30, 3, 8, 6, 500.0
    rng, Wk, Wv, idx, x, q, pos, q_pos = _full_model(10 + r, d, n_h, d_h, r, S)
    W_ke, A, W_uk, W_uv = exact_elitekv_weights(rng, Wk, Wv, idx)
    got = _oracle_end_to_end(W_ke, A, W_uk, W_uv, idx, x, pos, q, q_pos, d_h, base)
    k_raw = np.einsum("sd,dhe->she", x, Wk)
    v = np.einsum("sd,dhe->she", x, Wv)
    ref = ropelite_attention_relative(q[0], q_pos, k_raw, v, pos, idx, base)
    assert np.max(np.abs(got - ref)) < TOL


# ----------------------------------------------------------------------------------------------
# P3: r = 0 ==> position-free attention with K = c W_uk, V = c W_uv
# ----------------------------------------------------------------------------------------------
def test_p3_no_elite_chunks_is_position_free_low_rank_attention():
    d, n_h, d_h, S, d_c = 12, 2, 4, 5, 3
    rng = np.random.default_rng(3)
    idx = np.zeros((n_h, 0), dtype=np.int32)
    W_ke = np.zeros((d, n_h, 0))
    W_dkv = rng.standard_normal((d, d_c))
    W_uk = rng.standard_normal((d_c, n_h, d_h))
    W_uv = rng.standard_normal((d_c, n_h, d_h))
    x = rng.standard_normal((S, d))
    q = rng.standard_normal((1, n_h, d_h))
    got = _oracle_end_to_end(W_ke, W_dkv, W_uk, W_uv, idx, x, np.arange(S), q, 77, d_h, 10000.0)
    got2 = _oracle_end_to_end(W_ke, W_dkv, W_uk, W_uv, idx, x, np.arange(S) * 13 + 5, q, 2, d_h, 10000.0)
    assert np.array_equal(got, got2)               # positions cannot matter
    for h in range(n_h):
        c = x @ W_dkv
        K = c @ W_uk[:, h, :]
        V = c @ W_uv[:, h, :]
        s = K @ q[0, h] / 2.0                      # sqrt(d_h) = 2
        p = np.exp(s - s.max())
        p /= p.sum()
        assert np.max(np.abs(got[h] - p @ V)) < TOL


# ----------------------------------------------------------------------------------------------
# P4: R(0) = I  (Section 2.2): at position 0 the cached elite keys are x W_ke bit for bit
# ----------------------------------------------------------------------------------------------
def test_p4_position_zero_is_identity():
    cfg = synth.CONFIGS["tiny_fp32"]
    p = synth.problem(cfg, tokens=9)
    ke, c = orc.append(p["x"], np.zeros(9, dtype=np.int64), p["W_ke"], p["W_dkv"], p["elite_idx"],
                       cfg.head_dim, cfg.rope_base)
    raw = p["x"] @ p["W_ke"].reshape(cfg.d_model, -1)
    assert np.array_equal(ke.reshape(9, -1), raw)
    assert np.array_equal(c, p["x"] @ p["W_dkv"])


# ----------------------------------------------------------------------------------------------
# hand-computed rotations: theta_1 = 10000^(-2/4) = 0.01 exactly, so pos = 100 gives an angle of
# exactly 1 rad; (1, 0) -> (cos 1, sin 1), (0, 1) -> (-sin 1, cos 1).  Fixes the sense of R, the
# exponent of theta, and which position multiplies which frequency.
# ----------------------------------------------------------------------------------------------
def test_hand_computed_rotation_golden():
    vals = {}
    with open(os.path.join(GOLDEN, "rotation_by_one_radian.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, v = line.split()
            vals[k] = float(v)
    d_h = 4
    W_ke = np.zeros((2, 1, 2))
    W_ke[0, 0, 0] = 1.0
    W_ke[1, 0, 1] = 1.0                              # key pair = (x0, x1)
    x = np.array([[1.0, 0.0], [0.0, 1.0], [1.0, 0.0]])
    pos = np.array([100, 100, 0])
    ke, _ = orc.append(x, pos, W_ke, np.zeros((2, 1)), np.array([[1]]), d_h, 10000.0)
    assert abs(orc.rope_theta(4, 10000.0)[1] - 0.01) < 1e-18
    assert abs(ke[0, 0, 0] - vals["cos1"]) < 1e-15 and abs(ke[0, 0, 1] - vals["sin1"]) < 1e-15
    assert abs(ke[1, 0, 0] + vals["sin1"]) < 1e-15 and abs(ke[1, 0, 1] - vals["cos1"]) < 1e-15
    assert ke[2, 0, 0] == 1.0 and ke[2, 0, 1] == 0.0
    # chunk 0 has theta = 1: pos 1 also turns by one radian
    ke0, _ = orc.append(x[:1], np.array([1]), W_ke, np.zeros((2, 1)), np.array([[0]]), d_h, 10000.0)
    assert abs(ke0[0, 0, 0] - vals["cos1"]) < 1e-15 and abs(ke0[0, 0, 1] - vals["sin1"]) < 1e-15


# ----------------------------------------------------------------------------------------------
# P5: eq. 1a = eq. 1b: shifting every position (cache and query) by the same amount changes nothing
# ----------------------------------------------------------------------------------------------
def test_p5_shift_invariance():
    cfg = synth.CONFIGS["tiny_fp32"]
    p = synth.problem(cfg, tokens=17)
    args = (p["W_ke"], p["W_dkv"], p["W_uk"], p["W_uv"], p["elite_idx"], p["x"])
    a = _oracle_end_to_end(*args, np.arange(17), p["q"], 16, cfg.head_dim, cfg.rope_base)
    b = _oracle_end_to_end(*args, np.arange(17) + 1000, p["q"], 1016, cfg.head_dim, cfg.rope_base)
    c = _oracle_end_to_end(*args, np.arange(17), p["q"], 17, cfg.head_dim, cfg.rope_base)
    assert np.max(np.abs(a - b)) < 1e-10
    assert np.max(np.abs(a - c)) > 1e-6             # and the query position does matter


# P6: a rotation preserves the norm of every pair
def test_p6_rotation_preserves_pair_norms():
    cfg = synth.CONFIGS["tiny_fp32"]
    p = synth.problem(cfg, tokens=11)
    pos = np.arange(11) * 37 + 1
    ke, _ = orc.append(p["x"], pos, p["W_ke"], p["W_dkv"], p["elite_idx"], cfg.head_dim, cfg.rope_base)
    raw = (p["x"] @ p["W_ke"].reshape(cfg.d_model, -1)).reshape(11, cfg.n_heads, cfg.r, 2)
    n0 = np.sum(raw ** 2, axis=-1)
    n1 = np.sum(ke.reshape(11, cfg.n_heads, cfg.r, 2) ** 2, axis=-1)
    assert np.max(np.abs(n0 - n1)) < 1e-12
    assert np.max(np.abs(ke.reshape(raw.shape) - raw)) > 1e-3


# ----------------------------------------------------------------------------------------------
# P7: closed forms of the softmax (Section 2.1)
# ----------------------------------------------------------------------------------------------
def test_p7_single_token_and_zero_query_closed_forms():
    cfg = synth.CONFIGS["tiny_fp32"]
    p = synth.problem(cfg, tokens=6)
    ke, c = orc.append(p["x"], np.arange(6), p["W_ke"], p["W_dkv"], p["elite_idx"], cfg.head_dim,
                       cfg.rope_base)
    o1 = orc.decode_attn(p["q"], [5], ke[None], c[None], [1], p["W_uk"], p["W_uv"], p["elite_idx"],
                         cfg.head_dim, cfg.rope_base)[0]
    for h in range(cfg.n_heads):
        assert np.max(np.abs(o1[h] - c[0] @ p["W_uv"][:, h, :])) < TOL
    o0 = orc.decode_attn(np.zeros_like(p["q"]), [5], ke[None], c[None], [6], p["W_uk"], p["W_uv"],
                         p["elite_idx"], cfg.head_dim, cfg.rope_base)[0]
    for h in range(cfg.n_heads):
        assert np.max(np.abs(o0[h] - c.mean(axis=0) @ p["W_uv"][:, h, :])) < TOL
    # an empty context gives a zero row (reading: no NaN)
    oz = orc.decode_attn(p["q"], [5], ke[None], c[None], [0], p["W_uk"], p["W_uv"], p["elite_idx"],
                         cfg.head_dim, cfg.rope_base)
    assert np.all(oz == 0.0)


# ----------------------------------------------------------------------------------------------
# P8: the score is a sum over a set of chunks and over cached tokens: orders do not matter
# ----------------------------------------------------------------------------------------------
def test_p8_permutation_invariances():
    cfg = synth.CONFIGS["tiny_fp32"]
    p = synth.problem(cfg, tokens=10)
    rng = np.random.default_rng(8)
    pos = np.arange(10)
    base_out = _oracle_end_to_end(p["W_ke"], p["W_dkv"], p["W_uk"], p["W_uv"], p["elite_idx"], p["x"],
                                  pos, p["q"], 9, cfg.head_dim, cfg.rope_base)
    perm = rng.permutation(10)
    out_rows = _oracle_end_to_end(p["W_ke"], p["W_dkv"], p["W_uk"], p["W_uv"], p["elite_idx"],
                                  p["x"][perm], pos[perm], p["q"], 9, cfg.head_dim, cfg.rope_base)
    assert np.max(np.abs(base_out - out_rows)) < 1e-12
    # reverse each head's slot order; W_ke's slot columns move with it
    idx2 = p["elite_idx"][:, ::-1].copy()
    W_ke2 = p["W_ke"].reshape(cfg.d_model, cfg.n_heads, cfg.r, 2)[:, :, ::-1, :].reshape(p["W_ke"].shape)
    out_slots = _oracle_end_to_end(W_ke2, p["W_dkv"], p["W_uk"], p["W_uv"], idx2, p["x"], pos, p["q"],
                                   9, cfg.head_dim, cfg.rope_base)
    assert np.max(np.abs(base_out - out_slots)) < 1e-12
    # but pairing a slot with the wrong frequency does change the result
    out_bad = _oracle_end_to_end(p["W_ke"], p["W_dkv"], p["W_uk"], p["W_uv"], idx2, p["x"], pos, p["q"],
                                 9, cfg.head_dim, cfg.rope_base)
    assert np.max(np.abs(base_out - out_bad)) > 1e-6


# ----------------------------------------------------------------------------------------------
# P9: brute force in Python floats on a tiny shape
# ----------------------------------------------------------------------------------------------
def _brute_force(x, pos, W_ke, W_dkv, W_uk, W_uv, idx, q, q_pos, d_h, base):
    S, d = len(x), len(x[0])
    n_h, r = len(idx), len(idx[0])
    d_c = len(W_dkv[0])
    th = _theta_plain(d_h, base)
    out = [[0.0] * d_h for _ in range(n_h)]
    lat = [[sum(x[t][a] * W_dkv[a][k] for a in range(d)) for k in range(d_c)] for t in range(S)]
    for h in range(n_h):
        elite = [i for i in idx[h]]
        el_dims = set()
        for i in elite:
            el_dims.update((2 * i, 2 * i + 1))
        ne = [t for t in range(d_h) if t not in el_dims]
        scores = []
        for t in range(S):
            s = 0.0
            for j, i in enumerate(elite):
                ku = sum(x[t][a] * W_ke[a][h][2 * j] for a in range(d))
                kv = sum(x[t][a] * W_ke[a][h][2 * j + 1] for a in range(d))
                a_k = pos[t] * th[i]
                ku, kv = ku * math.cos(a_k) - kv * math.sin(a_k), ku * math.sin(a_k) + kv * math.cos(a_k)
                a_q = q_pos * th[i]
                qu, qv = q[h][2 * i], q[h][2 * i + 1]
                qu, qv = qu * math.cos(a_q) - qv * math.sin(a_q), qu * math.sin(a_q) + qv * math.cos(a_q)
                s += qu * ku + qv * kv
            for m, dim in enumerate(ne):
                kd = sum(lat[t][k] * W_uk[k][h][m] for k in range(d_c))
                s += q[h][dim] * kd
            scores.append(s / math.sqrt(d_h))
        mx = max(scores)
        e = [math.exp(s - mx) for s in scores]
        z = sum(e)
        for t in range(S):
            for o in range(d_h):
                vd = sum(lat[t][k] * W_uv[k][h][o] for k in range(d_c))
                out[h][o] += e[t] / z * vd
    return np.array(out)


@pytest.mark.parametrize("r", [0, 1, 2])
def test_p9_brute_force_tiny(r):
    d, n_h, d_h, d_c, S, base = 5, 2, 6, 3, 4, 100.0
    rng = np.random.default_rng(90 + r)
    idx = synth.draw_elite_idx(rng, n_h, d_h, r) if r else np.zeros((n_h, 0), dtype=np.int32)
    W_ke, W_dkv, W_uk, W_uv = synth.draw_weights(rng, d, n_h, d_h, r, d_c)
    x = rng.standard_normal((S, d))
    q = rng.standard_normal((1, n_h, d_h))
    pos = [3, 0, 7, 2]
    got = _oracle_end_to_end(W_ke, W_dkv, W_uk, W_uv, idx, x, np.array(pos), q, 9, d_h, base)
    ref = _brute_force(x.tolist(), pos, W_ke.tolist(), W_dkv.tolist(), W_uk.tolist(), W_uv.tolist(),
                       idx.tolist(), q[0].tolist(), 9, d_h, base)
    assert np.max(np.abs(got - ref)) < 1e-12


# ----------------------------------------------------------------------------------------------
# P10: cache-size and parameter-count formulas (Section 3.2, J-LRD) and Table 1's "Cache" column
# ----------------------------------------------------------------------------------------------
def test_p10_cache_ratio_golden_and_param_count():
    rows = []
    with open(os.path.join(GOLDEN, "cache_ratios.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, ratio = line.split()
            rows.append((name, float(ratio)))
    for name, ratio in rows:
        cfg = synth.CONFIGS[name]
        full = 2 * cfg.head_dim * cfg.n_heads           # Section 3.2: d_h per head for K, same for V
        assert abs(100.0 * orc.cache_row_elems(cfg.n_heads, cfg.r, cfg.d_c) / full - ratio) < 1e-9
        p = synth.problem(cfg, tokens=1, batch=1) if cfg.d_model <= 128 else None
        n_w = (cfg.d_model * cfg.n_heads * 2 * cfg.r + cfg.d_model * cfg.d_c
               + cfg.d_c * cfg.n_heads * (cfg.head_dim - 2 * cfg.r) + cfg.d_c * cfg.n_heads * cfg.head_dim)
        assert orc.param_count(cfg.d_model, cfg.n_heads, cfg.head_dim, cfg.r, cfg.d_c) == n_w
        if p is not None:
            assert sum(p[k].size for k in ("W_ke", "W_dkv", "W_uk", "W_uv")) == n_w
        if cfg.dtype == "bf16":
            # Appendix C: d_c a multiple of 128, and no more parameters than W^k plus W^v
            assert cfg.d_c % 128 == 0
            assert n_w <= 2 * cfg.d_model * cfg.n_heads * cfg.head_dim


# ----------------------------------------------------------------------------------------------
# the comparator oracle (ordinary RoPE decode) against the complex-number reference
# ----------------------------------------------------------------------------------------------
def test_mha_decode_matches_complex_reference():
    rng = np.random.default_rng(5)
    S, n_h, d_h, base = 6, 2, 8, 10000.0
    k_raw = rng.standard_normal((S, n_h, d_h))
    v = rng.standard_normal((S, n_h, d_h))
    q = rng.standard_normal((1, n_h, d_h))
    pos = np.arange(S) + 4
    th = orc.rope_theta(d_h, base)
    K_rot = np.empty_like(k_raw)
    for j in range(S):
        for h in range(n_h):
            for i in range(d_h // 2):
                z = complex(k_raw[j, h, 2 * i], k_raw[j, h, 2 * i + 1]) * cmath.exp(1j * int(pos[j]) * th[i])
                K_rot[j, h, 2 * i], K_rot[j, h, 2 * i + 1] = z.real, z.imag
    got = orc.mha_decode(q, [11], K_rot[None], v[None], [S], base)[0]
    ref = rope_attention_complex(q[0], 11, k_raw, v, pos, base)
    assert np.max(np.abs(got - ref)) < TOL


# ----------------------------------------------------------------------------------------------
# the pins bite: plant one mistake at a time in the oracle and require some pin to fail
# ----------------------------------------------------------------------------------------------
# ----------------------------------------------------------------------------------------------
# Several queries per sequence: against causal attention written as one masked score matrix over
# un-rotated full keys (relative form of Section 2.2 eq. 1b; Section 2.1 for the softmax)
# ----------------------------------------------------------------------------------------------
def test_multiquery_equals_masked_causal_attention():
    d, n_h, d_h, r, S, T, base = 20, 2, 8, 2, 9, 4, 1000.0
    rng, Wk, Wv, idx, x, _, _, _ = _full_model(71, d, n_h, d_h, r, S)
    W_ke, A, W_uk, W_uv = exact_elitekv_weights(rng, Wk, Wv, idx)
    pos = np.arange(S)
    ke, c = orc.append(x, pos, W_ke, A, idx, d_h, base)
    q = rng.standard_normal((1, T, n_h, d_h))
    q_pos = np.arange(S - T, S)[None]                     # the last T tokens of the sequence are the queries
    got = orc.multiquery_attn(q, q_pos, [ke], [c], q_pos + 1, W_uk, W_uv, idx, d_h, base)[0]
    # reference: one [T, S] score matrix per head from full keys, relative rotations, causal mask
    k_raw = np.einsum("sd,dhe->she", x, Wk)
    v = np.einsum("sd,dhe->she", x, Wv)
    th = _theta_plain(d_h, base)
    for h in range(n_h):
        elite = set(int(i) for i in idx[h])
        s = np.full((T, S), -np.inf)
        for t in range(T):
            for j in range(S):
                if j > q_pos[0, t]:
                    continue                               # the mask: no later token is visible
                acc = 0.0
                for i in range(d_h // 2):
                    qi, ki = q[0, t, h, 2 * i:2 * i + 2], k_raw[j, h, 2 * i:2 * i + 2]
                    acc += float(qi @ _rot_matrix((int(q_pos[0, t]) - j) * th[i]) @ ki) if i in elite else float(qi @ ki)
                s[t, j] = acc / math.sqrt(d_h)
        p = np.exp(s - s.max(axis=1, keepdims=True))
        p /= p.sum(axis=1, keepdims=True)
        assert np.max(np.abs(got[:, h, :] - p @ v[:, h, :])) < TOL


def _pins():
    return [lambda: test_p1_full_rope_equals_standard_attention(1),
            lambda: test_p2_matches_ropelite_equation_relative_form(2),
            test_p3_no_elite_chunks_is_position_free_low_rank_attention,
            test_hand_computed_rotation_golden,
            test_p7_single_token_and_zero_query_closed_forms,
            lambda: test_p9_brute_force_tiny(2)]


def _some_pin_fails():
    for pin in _pins():
        try:
            pin()
        except AssertionError:
            return True
    return False


def test_pins_pass_unmutated():
    assert not _some_pin_fails()


@pytest.mark.parametrize("mutation", ["rot_sense", "theta_exponent", "nonelite_order", "elite_pair_swap",
                                      "scale", "softmax_no_norm", "half_split_pairs"])
def test_planted_mistakes_are_caught(monkeypatch, mutation):
    if mutation == "rot_sense":
        real = orc.rotate_pairs
        monkeypatch.setattr(orc, "rotate_pairs", lambda p, a: real(p, -a))
    elif mutation == "theta_exponent":
        monkeypatch.setattr(orc, "rope_theta",
                            lambda d_h, b: np.power(float(b), -np.arange(d_h // 2) / float(d_h)))
    elif mutation == "nonelite_order":
        real = orc.nonelite_dims
        monkeypatch.setattr(orc, "nonelite_dims", lambda i, d: real(i, d)[::-1])
    elif mutation == "elite_pair_swap":
        real = orc.elite_dims
        def swapped(i):
            e = real(i).reshape(-1, 2)[:, ::-1]
            return e.reshape(-1)
        monkeypatch.setattr(orc, "elite_dims", swapped)
    elif mutation == "scale":
        real = orc.softmax_attention
        monkeypatch.setattr(orc, "softmax_attention", lambda q, K, V, d_h: real(q, K, V, 1))
    elif mutation == "softmax_no_norm":
        def bad(q, K, V, d_h):
            s = K @ q / np.sqrt(d_h)
            return np.exp(s - s.max()) @ V
        monkeypatch.setattr(orc, "softmax_attention", bad)
    elif mutation == "half_split_pairs":
        def half(i):
            return np.array([[int(t), int(t) + 4] for t in np.asarray(i).tolist()]).reshape(-1)
        monkeypatch.setattr(orc, "elite_dims", half)
    assert _some_pin_fails()


def _metric_cases():
    rows = []
    for line in open(os.path.join(GOLDEN, "max_abs_rel_cases.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        got, ref, want = (part.split() for part in line.split(";"))
        rows.append((np.array(got, dtype=float), np.array(ref, dtype=float), float(want[0])))
    return rows


def _metric_pin():
    rows = _metric_cases()
    assert len(rows) == 6
    for got, ref, want in rows:
        assert abs(orc.max_abs_rel(got, ref) - want) <= 1e-12 * max(want, 1.0), (got, ref, want)
    # shape does not matter, one tensor = one number; an empty tensor has no error
    assert abs(orc.max_abs_rel(np.array([[1.25, 2.0], [3.0, 11.0]]), np.array([[1.0, 2.0], [3.0, 10.0]])) - 0.1) < 1e-15
    assert orc.max_abs_rel(np.zeros((0, 3)), np.zeros((0, 3))) == 0.0
    # the metric of the parity gates is scale-free and not symmetric in its arguments
    assert abs(orc.max_abs_rel(3.0 * np.array([1.5, -6.0]), 3.0 * np.array([1.0, -4.0])) - 0.5) < 1e-15
    assert abs(orc.max_abs_rel(np.array([1.0, -4.0]), np.array([1.5, -6.0])) - 1.0 / 3.0) < 1e-15
    # a NaN anywhere in the result must not pass a gate of the form  err <= tol
    assert not (orc.max_abs_rel(np.array([1.0, np.nan]), np.array([1.0, 2.0])) <= 1.0)


def test_max_abs_rel_hand_computed_cases():
    """The metric every GPU parity gate uses, on hand-computed cases (tests/golden/max_abs_rel_cases.txt):
    normalised by the largest |ref| (not |got|), absolute values on both the difference and the
    normaliser, zero reference floored at 1e-30, empty tensors, NaN results."""
    _metric_pin()


@pytest.mark.parametrize("mutation", ["normalise_by_got", "no_abs_on_difference", "signed_normaliser", "mean_not_max",
                                      "nan_ignored"])
def test_planted_metric_mistakes_are_caught(monkeypatch, mutation):
    bad = {
        "normalise_by_got": lambda g, r: float(np.max(np.abs(np.asarray(g) - np.asarray(r)))) / max(float(np.max(np.abs(g))), 1e-30),
        "no_abs_on_difference": lambda g, r: float(np.max(np.asarray(g) - np.asarray(r))) / max(float(np.max(np.abs(r))), 1e-30),
        "signed_normaliser": lambda g, r: float(np.max(np.abs(np.asarray(g) - np.asarray(r)))) / max(float(np.max(r)), 1e-30),
        "mean_not_max": lambda g, r: float(np.mean(np.abs(np.asarray(g) - np.asarray(r)))) / max(float(np.max(np.abs(r))), 1e-30),
        "nan_ignored": lambda g, r: float(np.nanmax(np.abs(np.asarray(g) - np.asarray(r)))) / max(float(np.max(np.abs(r))), 1e-30),
    }[mutation]
    monkeypatch.setattr(orc, "max_abs_rel", lambda g, r: 0.0 if np.asarray(r).size == 0 else bad(g, r))
    with pytest.raises(AssertionError):
        _metric_pin()
