"""Pins for the S-LRD functions of the CPU oracle (Section 3.2, "Separated Low-Rank Decomposition").

Independent references: the RoPElite score equation in relative form and the Python-float brute
force (neither calls the oracle), the joint-variant oracle (pinned on its own in
test_oracle_pins.py) through the block embedding, closed forms, and the paper's size formulas.
"""
import math

import numpy as np
import pytest

import elitekv_synth as synth
from oracle import elitekv_oracle as orc

from test_oracle_pins import _full_model, _theta_plain, ropelite_attention_relative

TOL = 1e-11


def _exact_slrd_weights(rng, Wk, Wv, idx):
    """W_ke gathered from Wk; A_k, A_v two DIFFERENT orthogonal bases with B = A^T W, so that
    A^k B^k_S and A^v B^v_S reproduce the non-elite key block and the value block exactly."""
    d, n_h, d_h = Wk.shape
    r = idx.shape[1]
    W_ke = np.zeros((d, n_h, 2 * r))
    ne_cols = []
    for h in range(n_h):
        el = set()
        for j, i in enumerate(idx[h]):
            W_ke[:, h, 2 * j] = Wk[:, h, 2 * i]
            W_ke[:, h, 2 * j + 1] = Wk[:, h, 2 * i + 1]
            el.update((2 * int(i), 2 * int(i) + 1))
        ne_cols.append(Wk[:, h, [t for t in range(d_h) if t not in el]])
    A_k, _ = np.linalg.qr(rng.standard_normal((d, d)))
    A_v, _ = np.linalg.qr(rng.standard_normal((d, d)))
    B_k = (A_k.T @ np.concatenate(ne_cols, axis=1)).reshape(d, n_h, d_h - 2 * r)
    B_v = (A_v.T @ Wv.reshape(d, n_h * d_h)).reshape(d, n_h, d_h)
    return W_ke, A_k, A_v, B_k, B_v


def _slrd_end_to_end(W_ke, A_k, A_v, B_k, B_v, idx, x, pos, q, q_pos, d_h, base):
    ke, ck, cv = orc.slrd_append(x, pos, W_ke, A_k, A_v, idx, d_h, base)
    return orc.slrd_decode_attn(q, [q_pos], ke[None], ck[None], cv[None], [x.shape[0]], B_k, B_v, idx, d_h, base)[0]


@pytest.mark.parametrize("r", [1, 2, 4])
def test_s1_exact_separate_factors_match_ropelite_equation(r):
    """Exact factors of both blocks => the Section 3.1 score equation with full keys and values
    (r = d_h/2 is ordinary RoPE attention)."""
    d, n_h, d_h, S, base = 30, 3, 8, 6, 500.0
    rng, Wk, Wv, idx, x, q, pos, q_pos = _full_model(20 + r, d, n_h, d_h, r, S)
    W_ke, A_k, A_v, B_k, B_v = _exact_slrd_weights(rng, Wk, Wv, idx)
    got = _slrd_end_to_end(W_ke, A_k, A_v, B_k, B_v, idx, x, pos, q, q_pos, d_h, base)
    k_raw = np.einsum("sd,dhe->she", x, Wk)
    v = np.einsum("sd,dhe->she", x, Wv)
    ref = ropelite_attention_relative(q[0], q_pos, k_raw, v, pos, idx, base)
    assert np.max(np.abs(got - ref)) < TOL


def _brute_force_slrd(x, pos, W_ke, A_k, A_v, B_k, B_v, idx, q, q_pos, d_h, base):
    S, d = len(x), len(x[0])
    n_h, r = len(idx), len(idx[0])
    d_ck, d_cv = len(A_k[0]), len(A_v[0])
    th = _theta_plain(d_h, base)
    out = [[0.0] * d_h for _ in range(n_h)]
    lat_k = [[sum(x[t][a] * A_k[a][k] for a in range(d)) for k in range(d_ck)] for t in range(S)]
    lat_v = [[sum(x[t][a] * A_v[a][k] for a in range(d)) for k in range(d_cv)] for t in range(S)]
    for h in range(n_h):
        elite = list(idx[h])
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
                s += q[h][dim] * sum(lat_k[t][k] * B_k[k][h][m] for k in range(d_ck))
            scores.append(s / math.sqrt(d_h))
        mx = max(scores)
        e = [math.exp(s - mx) for s in scores]
        z = sum(e)
        for t in range(S):
            for o in range(d_h):
                out[h][o] += e[t] / z * sum(lat_v[t][k] * B_v[k][h][o] for k in range(d_cv))
    return np.array(out)


def _draw_slrd(rng, d, n_h, d_h, r, d_ck, d_cv):
    W_ke, A_k, B_k, _ = synth.draw_weights(rng, d, n_h, d_h, r, d_ck)
    _, A_v, _, B_v = synth.draw_weights(rng, d, n_h, d_h, r, d_cv)
    return W_ke, A_k, A_v, B_k, B_v


def _check_brute_force(r, d_ck, d_cv):
    d, n_h, d_h, S, base = 5, 2, 6, 4, 100.0
    rng = np.random.default_rng(190 + r)
    idx = synth.draw_elite_idx(rng, n_h, d_h, r) if r else np.zeros((n_h, 0), dtype=np.int32)
    W_ke, A_k, A_v, B_k, B_v = _draw_slrd(rng, d, n_h, d_h, r, d_ck, d_cv)
    x = rng.standard_normal((S, d))
    q = rng.standard_normal((1, n_h, d_h))
    pos = [3, 0, 7, 2]
    got = _slrd_end_to_end(W_ke, A_k, A_v, B_k, B_v, idx, x, np.array(pos), q, 9, d_h, base)
    ref = _brute_force_slrd(x.tolist(), pos, W_ke.tolist(), A_k.tolist(), A_v.tolist(), B_k.tolist(), B_v.tolist(),
                            idx.tolist(), q[0].tolist(), 9, d_h, base)
    assert np.max(np.abs(got - ref)) < 1e-12


@pytest.mark.parametrize("r", [0, 1, 2])
def test_s2_brute_force_tiny(r):
    _check_brute_force(r, 3, 4)
    _check_brute_force(r, 4, 4)


def test_s3_embedding_into_the_joint_variant():
    """S-LRD is J-LRD with the latent [c^k | c^v], A^{kv} = [A^k | A^v] and block-zero
    up-projections B^k_J = [B^k_S; 0], B^v_J = [0; B^v_S] (Section 3.2, both definitions)."""
    d, n_h, d_h, r, d_ck, d_cv, S, base = 16, 3, 8, 2, 5, 7, 9, 10000.0
    rng = np.random.default_rng(33)
    idx = synth.draw_elite_idx(rng, n_h, d_h, r)
    W_ke, A_k, A_v, B_k, B_v = _draw_slrd(rng, d, n_h, d_h, r, d_ck, d_cv)
    x = rng.standard_normal((S, d))
    q = rng.standard_normal((2, n_h, d_h))
    pos = np.arange(S)
    ke, ck, cv = orc.slrd_append(x, pos, W_ke, A_k, A_v, idx, d_h, base)
    got = orc.slrd_decode_attn(q, [S - 1, 4], [ke, ke], [ck, ck], [cv, cv], [S, 5], B_k, B_v, idx, d_h, base)
    A_kv = np.concatenate([A_k, A_v], axis=1)
    Bk_J = np.concatenate([B_k, np.zeros((d_cv, n_h, d_h - 2 * r))], axis=0)
    Bv_J = np.concatenate([np.zeros((d_ck, n_h, d_h)), B_v], axis=0)
    ke_j, c_j = orc.append(x, pos, W_ke, A_kv, idx, d_h, base)
    assert np.array_equal(ke_j, ke) and np.max(np.abs(c_j - np.concatenate([ck, cv], axis=1))) < 1e-13
    ref = orc.decode_attn(q, [S - 1, 4], [ke_j, ke_j], [c_j, c_j], [S, 5], Bk_J, Bv_J, idx, d_h, base)
    assert np.max(np.abs(got - ref)) < TOL


def test_s4_closed_forms():
    """One cached token: o = c^v_0 B^v_h.  Zero query: o = mean_j(c^v_j) B^v_h.  (Section 2.1)"""
    d, n_h, d_h, r, d_ck, d_cv, S = 10, 2, 8, 1, 4, 6, 5
    rng = np.random.default_rng(44)
    idx = synth.draw_elite_idx(rng, n_h, d_h, r)
    W_ke, A_k, A_v, B_k, B_v = _draw_slrd(rng, d, n_h, d_h, r, d_ck, d_cv)
    x = rng.standard_normal((S, d))
    ke, ck, cv = orc.slrd_append(x, np.arange(S), W_ke, A_k, A_v, idx, d_h, 10000.0)
    q = rng.standard_normal((1, n_h, d_h))
    one = orc.slrd_decode_attn(q, [0], ke[None], ck[None], cv[None], [1], B_k, B_v, idx, d_h, 10000.0)[0]
    zero = orc.slrd_decode_attn(np.zeros_like(q), [S], ke[None], ck[None], cv[None], [S], B_k, B_v, idx, d_h,
                                10000.0)[0]
    for h in range(n_h):
        assert np.max(np.abs(one[h] - (x[0] @ A_v) @ B_v[:, h, :])) < TOL
        assert np.max(np.abs(zero[h] - (x @ A_v).mean(axis=0) @ B_v[:, h, :])) < TOL


def test_s6_several_queries_equal_masked_causal_attention():
    """Exact separate factors, the last T tokens as queries: one masked [T, S] score matrix per head
    from un-rotated full keys with relative rotations on the elite chunks (Section 2.2 eq. 1b,
    Section 2.1 for the softmax), values from the full value projection."""
    d, n_h, d_h, r, S, T, base = 20, 2, 8, 2, 9, 4, 1000.0
    rng, Wk, Wv, idx, x, _, _, _ = _full_model(81, d, n_h, d_h, r, S)
    W_ke, A_k, A_v, B_k, B_v = _exact_slrd_weights(rng, Wk, Wv, idx)
    ke, ck, cv = orc.slrd_append(x, np.arange(S), W_ke, A_k, A_v, idx, d_h, base)
    q = rng.standard_normal((1, T, n_h, d_h))
    q_pos = np.arange(S - T, S)[None]
    got = orc.slrd_multiquery_attn(q, q_pos, [ke], [ck], [cv], q_pos + 1, B_k, B_v, idx, d_h, base)[0]
    k_raw = np.einsum("sd,dhe->she", x, Wk)
    v = np.einsum("sd,dhe->she", x, Wv)
    th = _theta_plain(d_h, base)
    for h in range(n_h):
        elite = set(int(i) for i in idx[h])
        s = np.full((T, S), -np.inf)
        for t in range(T):
            for j in range(int(q_pos[0, t]) + 1):          # the mask: no later token is visible
                acc = 0.0
                for i in range(d_h // 2):
                    qa, qb = q[0, t, h, 2 * i], q[0, t, h, 2 * i + 1]
                    ka, kb = k_raw[j, h, 2 * i], k_raw[j, h, 2 * i + 1]
                    if i in elite:
                        # (R(m th) q) . (R(n th) k) = q^T R((n - m) th) k, R(a) = [[cos a, -sin a], [sin a, cos a]]
                        a = (j - int(q_pos[0, t])) * th[i]
                        acc += (qa * ka + qb * kb) * math.cos(a) + (qb * ka - qa * kb) * math.sin(a)
                    else:
                        acc += qa * ka + qb * kb
                s[t, j] = acc / math.sqrt(d_h)
        p = np.exp(s - s.max(axis=1, keepdims=True))
        p /= p.sum(axis=1, keepdims=True)
        assert np.max(np.abs(got[:, h, :] - p @ v[:, h, :])) < TOL
    # a query that sees nothing returns zeros; visibility is per query, not per sequence
    z = orc.slrd_multiquery_attn(q, q_pos, [ke], [ck], [cv], np.array([[0, 1, 0, S]]), B_k, B_v, idx, d_h, base)[0]
    assert np.all(z[0] == 0.0) and np.all(z[2] == 0.0)
    assert np.max(np.abs(z[1] - np.einsum("d,dhe->he", x[0], Wv))) < TOL
    assert np.max(np.abs(z[3] - got[3])) == 0.0


def test_s5_size_formulas():
    """Section 3.2: cache 2 r n_h + d_ck + d_cv per token; with d = d_h n_h the storage cost
    simplifies to (2 d_ck + 2 d_cv + 2 r n_h) d - 2 d_ck r n_h."""
    for d_h, n_h, r, d_ck, d_cv in [(128, 32, 8, 576, 960), (128, 40, 8, 768, 1152), (64, 8, 4, 64, 192)]:
        d = d_h * n_h
        assert orc.slrd_param_count(d, n_h, d_h, r, d_ck, d_cv) == (2 * d_ck + 2 * d_cv + 2 * r * n_h) * d - 2 * d_ck * r * n_h
        assert orc.slrd_cache_row_elems(n_h, r, d_ck, d_cv) == 2 * r * n_h + d_ck + d_cv
    # 7B shape: 512 elite + 576 + 960 = 2048 = a quarter of the 2 * 32 * 128 elements of the full cache
    assert orc.slrd_cache_row_elems(32, 8, 576, 960) * 4 == 2 * 32 * 128


@pytest.mark.parametrize("mutation", ["value_latent_from_key_basis", "keys_from_value_latent",
                                      "values_from_key_latent"])
def test_planted_slrd_mistakes_are_caught(monkeypatch, mutation):
    """A plausible mix-up of the two latents (shapes agree when d_ck == d_cv) must make a pin fail."""
    if mutation == "value_latent_from_key_basis":
        real_append = orc.slrd_append
        monkeypatch.setattr(orc, "slrd_append",
                            lambda x, pos, W_ke, A_k, A_v, *a: real_append(x, pos, W_ke, A_k, A_k, *a))
    else:
        real = orc.slrd_decode_attn

        def bad(q, q_pos, ke, c_k, c_v, *a, **kw):
            if mutation == "keys_from_value_latent":
                return real(q, q_pos, ke, c_v, c_v, *a, **kw)
            return real(q, q_pos, ke, c_k, c_k, *a, **kw)
        monkeypatch.setattr(orc, "slrd_decode_attn", bad)
    with pytest.raises(AssertionError):
        _check_brute_force(1, 4, 4)
