"""Pins of the oracle's whole-block decode step (`attention_block_step`: q = x W^q, append, attention
over the compressed cache, output projection; Section 2.1 for the projections, Section 3 for the
rest) against things other than itself:
  B1  r = d_h/2 with exact factors: the block equals an ordinary RoPE multi-head attention block
      computed from the un-factorised W^k, W^v with complex rotations and explicit loops;
  B2  an empty cache: softmax over the single new token is 1, so y = sum_h (x W_dkv W_uv,h) W^o_h
      whatever W^q is (closed form);
  B3  y is linear in W^o and the sequences of a batch do not interact;
  B4  planted mistakes (W^o indexed [d_h, n_h], W^q's head and dim axes swapped, the new token left
      out of the attended set, the new token appended at the wrong position) each fail a pin.
The separated variant (`slrd_attention_block_step`, Section 3.2 S-LRD) has the same pins with two different
exact bases for keys and values (SB1: ordinary RoPE block at r = d_h/2, and the RoPElite equation in relative
form for smaller r; SB2: empty cache closed form through A^v, B^v only; SB3: linearity and row independence)
and planted mix-ups of the two latents.
"""
import cmath
import math

import numpy as np
import pytest

import elitekv_synth as synth
from oracle import elitekv_oracle as orc
from test_oracle_pins import exact_elitekv_weights, ropelite_attention_relative
from test_oracle_slrd_pins import _exact_slrd_weights

TOL = 1e-10


def _mha_block_reference(x_all, pos_all, Wq, Wk, Wv, Wo, base):
    """Textbook block for ONE sequence: tokens x_all [S, d] at positions pos_all, the last one is the
    query.  RoPE on all chunks by complex multiplication (Section 2.2 eq. 1a), softmax attention per
    head (Section 2.1), heads concatenated, times W^o."""
    S, d = x_all.shape
    _, n_h, d_h = Wq.shape
    th = [base ** (-2.0 * i / d_h) for i in range(d_h // 2)]
    y = np.zeros(d)
    for h in range(n_h):
        qv = x_all[-1] @ Wq[:, h, :]
        qc = [complex(qv[2 * i], qv[2 * i + 1]) * cmath.exp(1j * int(pos_all[-1]) * th[i]) for i in range(d_h // 2)]
        s, vs = [], []
        for j in range(S):
            kv = x_all[j] @ Wk[:, h, :]
            kc = [complex(kv[2 * i], kv[2 * i + 1]) * cmath.exp(1j * int(pos_all[j]) * th[i]) for i in range(d_h // 2)]
            s.append(sum((a * b.conjugate()).real for a, b in zip(qc, kc)) / math.sqrt(d_h))
            vs.append(x_all[j] @ Wv[:, h, :])
        mx = max(s)
        e = [math.exp(t - mx) for t in s]
        z = sum(e)
        o_h = sum((e[j] / z) * vs[j] for j in range(S))
        y += o_h @ Wo[h]
    return y


def _model(seed, d=20, n_h=3, d_h=8, r=4, lens=(5, 0, 3)):
    rng = np.random.default_rng(seed)
    Wq = rng.standard_normal((d, n_h, d_h)) / math.sqrt(d)
    Wk = rng.standard_normal((d, n_h, d_h)) / math.sqrt(d)
    Wv = rng.standard_normal((d, n_h, d_h)) / math.sqrt(d)
    Wo = rng.standard_normal((n_h, d_h, d)) / math.sqrt(n_h * d_h)
    idx = synth.draw_elite_idx(rng, n_h, d_h, r)
    W_ke, A, W_uk, W_uv = exact_elitekv_weights(rng, Wk, Wv, idx)
    hist = [rng.standard_normal((L, d)) for L in lens]                  # earlier tokens of every sequence
    hpos = [np.sort(rng.permutation(40)[:L]).astype(np.int64) for L in lens]
    x = rng.standard_normal((len(lens), d))
    pos = np.array([int(p[-1]) + 2 if len(p) else 7 for p in hpos], dtype=np.int64)
    return rng, Wq, Wk, Wv, Wo, idx, W_ke, A, W_uk, W_uv, hist, hpos, x, pos


def _block(m, d_h=8, base=10000.0, Wq=None, Wo=None):
    rng, Wq0, Wk, Wv, Wo0, idx, W_ke, A, W_uk, W_uv, hist, hpos, x, pos = m
    old = [orc.append(hist[b], hpos[b], W_ke, A, idx, d_h, base) if len(hpos[b]) else
           (np.zeros((0,) + W_ke.shape[1:]), np.zeros((0, A.shape[1]))) for b in range(len(hist))]
    return orc.attention_block_step(x, pos, [o[0] for o in old], [o[1] for o in old], Wq0 if Wq is None else Wq, W_ke, A,
                                    W_uk, W_uv, Wo0 if Wo is None else Wo, idx, d_h, base)


def pin_b1_full_rope_block():
    m = _model(11)
    rng, Wq, Wk, Wv, Wo, idx, W_ke, A, W_uk, W_uv, hist, hpos, x, pos = m
    y, _, _ = _block(m)
    for b in range(x.shape[0]):
        x_all = np.concatenate([hist[b], x[b:b + 1]], axis=0)
        pos_all = np.concatenate([hpos[b], pos[b:b + 1]])
        ref = _mha_block_reference(x_all, pos_all, Wq, Wk, Wv, Wo, 10000.0)
        assert np.max(np.abs(y[b] - ref)) < TOL, b


def pin_b2_empty_cache_closed_form():
    m = _model(12, r=2, lens=(0, 0))
    rng, Wq, Wk, Wv, Wo, idx, W_ke, A, W_uk, W_uv, hist, hpos, x, pos = m
    y, ke_new, c_new = _block(m)
    ref = np.zeros_like(y)
    for b in range(x.shape[0]):
        c = x[b] @ A
        for h in range(Wo.shape[0]):
            ref[b] += (c @ W_uv[:, h, :]) @ Wo[h]
    assert np.max(np.abs(y - ref)) < TOL
    assert np.max(np.abs(c_new - x @ A)) < TOL
    y2, _, _ = _block(m, Wq=3.0 * Wq[::-1].copy())                       # any other W^q
    assert np.max(np.abs(y2 - y)) < TOL


def pin_b3_linear_in_wo_and_rows_independent():
    m = _model(13, r=1)
    rng, Wq, Wk, Wv, Wo, idx, W_ke, A, W_uk, W_uv, hist, hpos, x, pos = m
    Wo2 = rng.standard_normal(Wo.shape)
    ya, _, _ = _block(m)
    yb, _, _ = _block(m, Wo=Wo2)
    yc, _, _ = _block(m, Wo=2.0 * Wo - 0.5 * Wo2)
    assert np.max(np.abs(yc - (2.0 * ya - 0.5 * yb))) < 1e-9
    # a sequence alone gives the same row as inside the batch
    for b in range(x.shape[0]):
        mb = (rng, Wq, Wk, Wv, Wo, idx, W_ke, A, W_uk, W_uv, [hist[b]], [hpos[b]], x[b:b + 1], pos[b:b + 1])
        y1, _, _ = _block(mb)
        assert np.max(np.abs(y1[0] - ya[b])) < TOL


PINS = (pin_b1_full_rope_block, pin_b2_empty_cache_closed_form, pin_b3_linear_in_wo_and_rows_independent)


@pytest.mark.parametrize("pin", PINS, ids=lambda f: f.__name__)
def test_block_pins(pin):
    pin()


def _some_pin_fails():
    for pin in PINS:
        try:
            pin()
        except AssertionError:
            return True
        except Exception:
            return True
    return False


@pytest.mark.parametrize("mutation", ["wo_axes", "wq_axes", "new_token_not_attended", "new_token_position"])
def test_planted_mistakes_in_the_block_are_caught(monkeypatch, mutation):
    real = orc.attention_block_step
    if mutation == "wo_axes":
        def bad(x, pos, ke_old, c_old, W_q, W_ke, W_dkv, W_uk, W_uv, W_o, *a, **k):
            W_o = np.asarray(W_o)
            n_h, d_h, d = W_o.shape
            return real(x, pos, ke_old, c_old, W_q, W_ke, W_dkv, W_uk, W_uv,
                        W_o.reshape(d_h, n_h, d).transpose(1, 0, 2), *a, **k)
    elif mutation == "wq_axes":
        def bad(x, pos, ke_old, c_old, W_q, *a, **k):
            W_q = np.asarray(W_q)
            d, n_h, d_h = W_q.shape
            return real(x, pos, ke_old, c_old, W_q.reshape(d, d_h, n_h).transpose(0, 2, 1), *a, **k)
    elif mutation == "new_token_not_attended":
        def bad(x, pos, ke_old, c_old, W_q, W_ke, W_dkv, W_uk, W_uv, W_o, idx, d_h, base):
            y, ke_new, c_new = real(x, pos, ke_old, c_old, W_q, W_ke, W_dkv, W_uk, W_uv, W_o, idx, d_h, base)
            q = np.einsum("bd,dhj->bhj", np.asarray(x, dtype=np.float64), np.asarray(W_q, dtype=np.float64))
            seq = [np.asarray(k).shape[0] for k in ke_old]
            o = orc.decode_attn(q, pos, ke_old, c_old, seq, W_uk, W_uv, idx, d_h, base)
            return np.einsum("bhj,hjd->bd", o, np.asarray(W_o, dtype=np.float64)), ke_new, c_new
    else:
        def bad(x, pos, *a, **k):
            return real(x, np.asarray(pos) + 1, *a, **k)
    monkeypatch.setattr(orc, "attention_block_step", bad)
    assert _some_pin_fails()


# ---------------------------------------------------------------------------------------------
# separated latents
# ---------------------------------------------------------------------------------------------
def _slrd_model(seed, d=20, n_h=3, d_h=8, r=4, lens=(5, 0, 3)):
    rng = np.random.default_rng(seed)
    Wq = rng.standard_normal((d, n_h, d_h)) / math.sqrt(d)
    Wk = rng.standard_normal((d, n_h, d_h)) / math.sqrt(d)
    Wv = rng.standard_normal((d, n_h, d_h)) / math.sqrt(d)
    Wo = rng.standard_normal((n_h, d_h, d)) / math.sqrt(n_h * d_h)
    idx = synth.draw_elite_idx(rng, n_h, d_h, r)
    W_ke, A_k, A_v, B_k, B_v = _exact_slrd_weights(rng, Wk, Wv, idx)
    hist = [rng.standard_normal((L, d)) for L in lens]
    hpos = [np.sort(rng.permutation(40)[:L]).astype(np.int64) for L in lens]
    x = rng.standard_normal((len(lens), d))
    pos = np.array([int(p[-1]) + 2 if len(p) else 7 for p in hpos], dtype=np.int64)
    return dict(rng=rng, Wq=Wq, Wk=Wk, Wv=Wv, Wo=Wo, idx=idx, W_ke=W_ke, A_k=A_k, A_v=A_v, B_k=B_k, B_v=B_v, hist=hist,
                hpos=hpos, x=x, pos=pos)


def _slrd_block(m, d_h=8, base=10000.0, **over):
    g = dict(m, **over)
    d_ck, d_cv = g["A_k"].shape[1], g["A_v"].shape[1]
    old = [orc.slrd_append(g["hist"][b], g["hpos"][b], g["W_ke"], g["A_k"], g["A_v"], g["idx"], d_h, base)
           if len(g["hpos"][b]) else (np.zeros((0,) + g["W_ke"].shape[1:]), np.zeros((0, d_ck)), np.zeros((0, d_cv)))
           for b in range(len(g["hist"]))]
    return orc.slrd_attention_block_step(g["x"], g["pos"], [o[0] for o in old], [o[1] for o in old], [o[2] for o in old],
                                         g["Wq"], g["W_ke"], g["A_k"], g["A_v"], g["B_k"], g["B_v"], g["Wo"], g["idx"],
                                         d_h, base)


def pin_sb1_exact_factors_give_the_ropelite_block():
    # r = d_h/2: an ordinary RoPE multi-head block from the un-factorised weights (complex rotations)
    m = _slrd_model(21)
    y = _slrd_block(m)[0]
    for b in range(m["x"].shape[0]):
        x_all = np.concatenate([m["hist"][b], m["x"][b:b + 1]], axis=0)
        pos_all = np.concatenate([m["hpos"][b], m["pos"][b:b + 1]])
        ref = _mha_block_reference(x_all, pos_all, m["Wq"], m["Wk"], m["Wv"], m["Wo"], 10000.0)
        assert np.max(np.abs(y[b] - ref)) < TOL, b
    # r < d_h/2: the Section 3.1 score equation in its relative form from full keys and values
    m = _slrd_model(22, r=1)
    y = _slrd_block(m)[0]
    for b in range(m["x"].shape[0]):
        x_all = np.concatenate([m["hist"][b], m["x"][b:b + 1]], axis=0)
        pos_all = np.concatenate([m["hpos"][b], m["pos"][b:b + 1]])
        q = m["x"][b] @ m["Wq"].reshape(m["x"].shape[1], -1)
        k_raw = np.einsum("sd,dhe->she", x_all, m["Wk"])
        v = np.einsum("sd,dhe->she", x_all, m["Wv"])
        o = ropelite_attention_relative(q.reshape(m["Wq"].shape[1:]), int(m["pos"][b]), k_raw, v, pos_all, m["idx"], 10000.0)
        ref = sum(o[h] @ m["Wo"][h] for h in range(m["Wo"].shape[0]))
        assert np.max(np.abs(y[b] - ref)) < TOL, b


def pin_sb2_empty_cache_closed_form():
    m = _slrd_model(23, r=2, lens=(0, 0))
    y, ke_new, ck_new, cv_new = _slrd_block(m)
    ref = np.zeros_like(y)
    for b in range(m["x"].shape[0]):
        cv = m["x"][b] @ m["A_v"]
        for h in range(m["Wo"].shape[0]):
            ref[b] += (cv @ m["B_v"][:, h, :]) @ m["Wo"][h]
    assert np.max(np.abs(y - ref)) < TOL
    assert np.max(np.abs(ck_new - m["x"] @ m["A_k"])) < TOL and np.max(np.abs(cv_new - m["x"] @ m["A_v"])) < TOL
    y2 = _slrd_block(m, Wq=3.0 * m["Wq"][::-1].copy(), B_k=2.0 * m["B_k"])[0]   # neither W^q nor B^k matters here
    assert np.max(np.abs(y2 - y)) < TOL


def pin_sb3_linear_in_wo_and_rows_independent():
    m = _slrd_model(24, r=1)
    Wo2 = m["rng"].standard_normal(m["Wo"].shape)
    ya = _slrd_block(m)[0]
    yb = _slrd_block(m, Wo=Wo2)[0]
    yc = _slrd_block(m, Wo=2.0 * m["Wo"] - 0.5 * Wo2)[0]
    assert np.max(np.abs(yc - (2.0 * ya - 0.5 * yb))) < 1e-9
    for b in range(m["x"].shape[0]):
        y1 = _slrd_block(m, hist=[m["hist"][b]], hpos=[m["hpos"][b]], x=m["x"][b:b + 1], pos=m["pos"][b:b + 1])[0]
        assert np.max(np.abs(y1[0] - ya[b])) < TOL


SLRD_PINS = (pin_sb1_exact_factors_give_the_ropelite_block, pin_sb2_empty_cache_closed_form,
             pin_sb3_linear_in_wo_and_rows_independent)


@pytest.mark.parametrize("pin", SLRD_PINS, ids=lambda f: f.__name__)
def test_slrd_block_pins(pin):
    pin()


@pytest.mark.parametrize("mutation", ["values_from_key_latent", "keys_from_value_latent", "new_token_not_attended",
                                      "wo_axes"])
def test_planted_mistakes_in_the_slrd_block_are_caught(monkeypatch, mutation):
    real = orc.slrd_attention_block_step
    if mutation == "values_from_key_latent":
        def bad(x, pos, ke_old, ck_old, cv_old, W_q, W_ke, A_k, A_v, B_k, B_v, *a):
            return real(x, pos, ke_old, ck_old, ck_old, W_q, W_ke, A_k, A_k, B_k, B_v, *a)
    elif mutation == "keys_from_value_latent":
        def bad(x, pos, ke_old, ck_old, cv_old, W_q, W_ke, A_k, A_v, B_k, B_v, *a):
            return real(x, pos, ke_old, cv_old, cv_old, W_q, W_ke, A_v, A_v, B_k, B_v, *a)
    elif mutation == "new_token_not_attended":
        def bad(x, pos, ke_old, ck_old, cv_old, W_q, W_ke, A_k, A_v, B_k, B_v, W_o, idx, d_h, base):
            out = real(x, pos, ke_old, ck_old, cv_old, W_q, W_ke, A_k, A_v, B_k, B_v, W_o, idx, d_h, base)
            q = np.einsum("bd,dhj->bhj", np.asarray(x, dtype=np.float64), np.asarray(W_q, dtype=np.float64))
            seq = [np.asarray(k).shape[0] for k in ke_old]
            o = orc.slrd_decode_attn(q, pos, ke_old, ck_old, cv_old, seq, B_k, B_v, idx, d_h, base)
            return (np.einsum("bhj,hjd->bd", o, np.asarray(W_o, dtype=np.float64)),) + tuple(out[1:])
    else:
        def bad(x, pos, ke_old, ck_old, cv_old, W_q, W_ke, A_k, A_v, B_k, B_v, W_o, *a):
            W_o = np.asarray(W_o)
            n_h, d_h, d = W_o.shape
            return real(x, pos, ke_old, ck_old, cv_old, W_q, W_ke, A_k, A_v, B_k, B_v,
                        W_o.reshape(d_h, n_h, d).transpose(1, 0, 2), *a)
    monkeypatch.setattr(orc, "slrd_attention_block_step", bad)
    failed = False
    for pin in SLRD_PINS:
        try:
            pin()
        except Exception:
            failed = True
    assert failed
