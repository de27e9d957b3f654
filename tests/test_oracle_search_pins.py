"""Pins for the RoPElite search of the CPU oracle (Section 3.1, Algorithm 1).

The references here do not call the oracle: the brute force evaluates the Section 3.1 score
equation in its relative form with Python floats; the other tests use properties that the
mathematics fixes (all chunks selected => distance 0; the dominant chunk goes first; scale
invariance; a permutation when r = d_h/2)."""
import math

import numpy as np
import pytest

from oracle import elitekv_oracle as orc

from test_oracle_pins import _rot_matrix, _theta_plain


def _scores_relative(q, k, pos, rotated, d_h, base):
    """s[t][j] for j <= t with R((t - j) theta_i) on the chunks in `rotated` only (Section 3.1)."""
    T = len(q)
    th = _theta_plain(d_h, base)
    s = [[0.0] * T for _ in range(T)]
    for t in range(T):
        for j in range(t + 1):
            acc = 0.0
            for i in range(d_h // 2):
                qi, ki = np.array(q[t][2 * i:2 * i + 2]), np.array(k[j][2 * i:2 * i + 2])
                acc += float(qi @ _rot_matrix((pos[t] - pos[j]) * th[i]) @ ki) if i in rotated else float(qi @ ki)
            s[t][j] = acc / math.sqrt(d_h)
    return s


def _brute_search(q, k, pos, r, d_h, base):
    T = len(q)
    full = _scores_relative(q, k, pos, set(range(d_h // 2)), d_h, base)
    e, dists = [], []
    for _ in range(r):
        best, best_d = -1, float("inf")
        for c in range(d_h // 2):
            if c in e:
                continue
            tr = _scores_relative(q, k, pos, set(e + [c]), d_h, base)
            dd = sum(abs(full[t][j] - tr[t][j]) for t in range(T) for j in range(t + 1))
            if dd < best_d:
                best, best_d = c, dd
        e.append(best)
        dists.append(best_d)
    return e, dists


@pytest.mark.parametrize("seed", [0, 1])
def test_search_matches_brute_force_in_relative_form(seed):
    T, n_h, d_h, r, base = 6, 2, 8, 3, 50.0
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((T, n_h, d_h))
    k = rng.standard_normal((T, n_h, d_h))
    pos = np.array([0, 1, 3, 4, 7, 9])
    elite, dist = orc.ropelite_search(q, k, pos, r, d_h, base)
    for h in range(n_h):
        e, dd = _brute_search(q[:, h].tolist(), k[:, h].tolist(), pos.tolist(), r, d_h, base)
        assert elite[h].tolist() == e
        assert np.max(np.abs(dist[h] - np.array(dd))) < 1e-11


def test_all_chunks_selected_is_a_permutation_with_zero_final_distance():
    T, n_h, d_h, base = 9, 2, 8, 100.0
    rng = np.random.default_rng(5)
    q, k = rng.standard_normal((T, n_h, d_h)), rng.standard_normal((T, n_h, d_h))
    elite, dist = orc.ropelite_search(q, k, np.arange(T), d_h // 2, d_h, base)
    for h in range(n_h):
        assert sorted(elite[h].tolist()) == list(range(d_h // 2))
        assert abs(dist[h, -1]) < 1e-12                    # every chunk rotated: the scores ARE the full-RoPE scores
        assert np.all(np.diff(dist[h]) <= 1e-12)           # each round can only come closer


def test_dominant_chunk_goes_first_and_scale_does_not_matter():
    """A chunk that carries far more of q and k than the others causes most of the difference between
    rotated and un-rotated scores, so the greedy choice takes it first; multiplying q by a constant
    multiplies every distance by it and changes no choice."""
    T, d_h, base = 24, 8, 10.0
    rng = np.random.default_rng(9)
    q, k = rng.standard_normal((T, 1, d_h)), rng.standard_normal((T, 1, d_h))
    for big, nxt in ((2, 0), (0, 1)):
        qs, ks = q.copy(), k.copy()
        qs[:, 0, 2 * big:2 * big + 2] *= 30.0
        ks[:, 0, 2 * big:2 * big + 2] *= 30.0
        qs[:, 0, 2 * nxt:2 * nxt + 2] *= 5.0
        ks[:, 0, 2 * nxt:2 * nxt + 2] *= 5.0
        e1, d1 = orc.ropelite_search(qs, ks, np.arange(T), 2, d_h, base)
        assert e1[0].tolist() == [big, nxt]
        e2, d2 = orc.ropelite_search(3.0 * qs, ks, np.arange(T), 2, d_h, base)
        assert e2[0].tolist() == [big, nxt]
        assert np.max(np.abs(d2 - 3.0 * d1)) < 1e-9 * np.max(d1)


def test_one_round_distances_agree_with_the_search():
    T, n_h, d_h, base = 7, 2, 8, 100.0
    rng = np.random.default_rng(11)
    q, k = rng.standard_normal((T, n_h, d_h)), rng.standard_normal((T, n_h, d_h))
    elite, dist = orc.ropelite_search(q, k, np.arange(T), 2, d_h, base)
    for h in range(n_h):
        d0 = orc.ropelite_distances(q, k, np.arange(T), [], h, d_h, base)
        assert int(np.argmin(d0)) == elite[h, 0] and abs(d0.min() - dist[h, 0]) < 1e-12
        d1 = orc.ropelite_distances(q, k, np.arange(T), [elite[h, 0]], h, d_h, base)
        assert np.isinf(d1[elite[h, 0]]) and int(np.argmin(d1)) == elite[h, 1]


@pytest.mark.parametrize("mutation", ["no_causal_mask", "rotate_keys_only"])
def test_planted_search_mistakes_are_caught(monkeypatch, mutation):
    if mutation == "no_causal_mask":
        monkeypatch.setattr(orc, "causal_scores", lambda qh, kh, d_h: (qh @ kh.T) / np.sqrt(d_h))
    else:
        real = orc.rope_on_chunks
        calls = {"n": 0}

        def bad(x, pos, chunks, d_h, base):                # every other call (the query side) is left un-rotated
            calls["n"] += 1
            return real(x, pos, chunks if calls["n"] % 2 == 0 else [], d_h, base)
        monkeypatch.setattr(orc, "rope_on_chunks", bad)
    with pytest.raises(AssertionError):
        test_search_matches_brute_force_in_relative_form(0)
