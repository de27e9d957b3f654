"""CPU oracle for the EliteKV decode hot path (RoPElite + joint low-rank decomposition).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, float64 statement of
what the path computes.  Only the tests, the smoke check and the benchmark's
`cpu_baseline` leg may import it; the product (the HIP library and its Python
binding) never does, and this file imports nothing from the product.

What is computed, and where the paper defines it:

* Cache append (Section 3.1, the expression for what enters the KV cache at
  step t of a RoPElite model; Section 3.2 "Joint Low-Rank Decomposition",
  c = x A^{kv}; Section 3.2's definition of W^k_{e,h}, the d x 2r block of the
  key projection that serves head h's elite chunks): the elite chunks of each
  head's key are stored rotated by R(t * theta_i); the rest of the key and the
  whole value are represented by the shared latent c_t = x_t W_dkv.

* Decode attention (Section 3.1, the RoPElite score equation; Section 2.1, the
  softmax attention equations; Section 3.2, B^{kv} = [B^k_J, B^v_J]): given
  the four weight blocks and the index sets, the method's result IS textbook
  softmax attention over the reconstructed keys
      k_j = [ rotated elite dims | c_j W_uk,h ]   and values   v_j = c_j W_uv,h.
  Absorbing W_uk into the query, online softmax, split-K and accumulating in
  latent space are exact algebraic rearrangements of this, so the oracle writes
  out the definition itself: reconstruct, then plain attention.  No blocking,
  no absorption, no running maximum.

Readings of points the paper leaves open (all listed again in the design notes):
  - theta_i = base^(-2i/d_h) (RoFormer's frequencies; the paper only cites it);
  - chunks are ADJACENT dims [2i, 2i+1] (Section 2.2, the definition of I);
  - R(a) acts on a row pair as (u, v) -> (u cos a - v sin a, u sin a + v cos a);
  - positions are explicit integers, no implicit origin;
  - the softmax scale stays 1/sqrt(d_h) with the original d_h (Section 2.1);
  - column order inside a head: elite slots in the caller's I_h order, each as
    (lane 0, lane 1); non-elite dims in ascending original index;
  - a batch row with seq_len 0 gives a zero output row.

Pins (tests/test_oracle_pins.py): equality with ordinary RoPE attention when
r = d_h/2 and the factors are exact; equality with the RoPElite score equation
evaluated in its relative form from full keys for any r; the r = 0 case;
R(0) = identity; shift invariance; norm preservation; the closed forms for one
cached token and for q = 0; permutation invariances; triple-loop brute force;
hand-computed rotations; the cache-size and parameter-count formulas.

The separated variant (S-LRD, two latents per token) has its own functions at the end of this
file and its own pins (tests/test_oracle_slrd_pins.py): exact separate factors against the
RoPElite score equation, brute force, the embedding into the joint variant with block-zero
up-projections, closed forms, and the Section 3.2 size formulas.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def rope_theta(head_dim: int, rope_base: float) -> np.ndarray:
    """theta_i = base^(-2i/d_h), i = 0 .. d_h/2 - 1 (Section 2.2; RoFormer's choice)."""
    i = np.arange(head_dim // 2, dtype=F64)
    return np.power(F64(rope_base), -2.0 * i / F64(head_dim))


def rotate_pairs(pairs: np.ndarray, alpha: np.ndarray) -> np.ndarray:
    """Apply the 2-D rotation R(alpha) to row pairs (Section 2.2, eq. 1a).

    pairs: [..., 2], alpha: [...] ->  (u cos a - v sin a, u sin a + v cos a).
    """
    u = pairs[..., 0]
    v = pairs[..., 1]
    ca = np.cos(alpha)
    sa = np.sin(alpha)
    return np.stack([u * ca - v * sa, u * sa + v * ca], axis=-1)


def nonelite_dims(elite_idx_h: np.ndarray, head_dim: int) -> np.ndarray:
    """Original head dims that are NOT in head h's elite chunks, ascending."""
    elite = set()
    for i in np.asarray(elite_idx_h).tolist():
        elite.add(2 * i)
        elite.add(2 * i + 1)
    return np.array([t for t in range(head_dim) if t not in elite], dtype=np.int64)


def elite_dims(elite_idx_h: np.ndarray) -> np.ndarray:
    """Original head dims of head h's elite chunks in slot order: (2i, 2i+1) per slot."""
    out = []
    for i in np.asarray(elite_idx_h).tolist():
        out += [2 * i, 2 * i + 1]
    return np.array(out, dtype=np.int64)


def cache_row_elems(n_heads: int, r: int, d_c: int) -> int:
    """KV-cache elements per token per layer: 2 r n_h + d_c (Section 3.2, J-LRD)."""
    return 2 * r * n_heads + d_c


def param_count(d_model: int, n_heads: int, head_dim: int, r: int, d_c: int) -> int:
    """Parameters of RoPElite + J-LRD: 2 r n_h d + d_c (d + 2 d_h n_h - 2 r n_h) (Section 3.2)."""
    return 2 * r * n_heads * d_model + d_c * (d_model + 2 * head_dim * n_heads - 2 * r * n_heads)


def append(x, pos, W_ke, W_dkv, elite_idx, head_dim: int, rope_base: float):
    """Cache rows for T tokens.

    x [T, d]; pos [T] ints; W_ke [d, n_h, 2r]; W_dkv [d, d_c]; elite_idx [n_h, r].
    Returns (ke [T, n_h, 2r] rotated elite keys, c [T, d_c] latent), float64.
    """
    x = np.asarray(x, dtype=F64)
    W_ke = np.asarray(W_ke, dtype=F64)
    W_dkv = np.asarray(W_dkv, dtype=F64)
    elite_idx = np.asarray(elite_idx)
    pos = np.asarray(pos)
    T, d = x.shape
    n_h, r = elite_idx.shape
    theta = rope_theta(head_dim, rope_base)

    c = x @ W_dkv                                            # c_t = x_t A^{kv}
    raw = (x @ W_ke.reshape(d, n_h * 2 * r)).reshape(T, n_h, r, 2)   # x_t W^k_{e,h}
    ke = np.empty_like(raw)
    for h in range(n_h):
        for j in range(r):
            alpha = pos.astype(F64) * theta[int(elite_idx[h, j])]    # t * theta_i
            ke[:, h, j, :] = rotate_pairs(raw[:, h, j, :], alpha)
    return ke.reshape(T, n_h, 2 * r), c


def softmax_attention(q_vec, K, V, head_dim: int):
    """Section 2.1: s = q K^T, p = softmax(s / sqrt(d_h)), o = p V.  q [D], K [S, D], V [S, Dv]."""
    s = K @ q_vec / np.sqrt(F64(head_dim))
    p = np.exp(s - np.max(s))
    p = p / np.sum(p)
    return p @ V


def decode_attn(q, q_pos, ke, c, seq_len, W_uk, W_uv, elite_idx, head_dim: int,
                rope_base: float, heads=None):
    """Single-token decode attention over the compressed cache.

    q [B, n_h, d_h] un-rotated, original dim order; q_pos [B]; ke[b] [>=S_b, n_h, 2r] and
    c[b] [>=S_b, d_c] (indexable by b: an array with a leading batch axis or a list);
    seq_len [B]; W_uk [d_c, n_h, d_h-2r]; W_uv [d_c, n_h, d_h]; elite_idx [n_h, r].
    heads: optional list of head indices to compute (others left zero).
    Returns o [B, n_h, d_h] float64.
    """
    q = np.asarray(q, dtype=F64)
    W_uk = np.asarray(W_uk, dtype=F64)
    W_uv = np.asarray(W_uv, dtype=F64)
    elite_idx = np.asarray(elite_idx)
    B, n_h, d_h = q.shape
    assert d_h == head_dim
    r = elite_idx.shape[1]
    theta = rope_theta(head_dim, rope_base)
    out = np.zeros((B, n_h, d_h), dtype=F64)
    head_list = range(n_h) if heads is None else heads
    for b in range(B):
        S = int(seq_len[b])
        if S == 0:
            continue
        ke_b = np.asarray(ke[b], dtype=F64)[:S]
        c_b = np.asarray(c[b], dtype=F64)[:S]
        for h in head_list:
            idx_h = elite_idx[h]
            # the query: elite chunks rotated at the query's position, the rest as is
            q_e = q[b, h, elite_dims(idx_h)].reshape(r, 2)
            alpha = F64(int(q_pos[b])) * theta[idx_h.astype(np.int64)] if r else np.zeros(0)
            q_e = rotate_pairs(q_e, alpha).reshape(2 * r)
            q_ne = q[b, h, nonelite_dims(idx_h, d_h)]
            q_hat = np.concatenate([q_e, q_ne])
            # reconstructed keys and values of every cached token
            K_full = np.concatenate([ke_b[:, h, :], c_b @ W_uk[:, h, :]], axis=1)
            V_full = c_b @ W_uv[:, h, :]
            out[b, h] = softmax_attention(q_hat, K_full, V_full, d_h)
    return out


# ----------------------------------------------------------------------------------------------
# The whole attention block of one decode step (Section 2.1: q_t = x_t W^q per head, the heads'
# outputs concatenated and multiplied by W^o; Section 3: everything in between as above).  The
# step's token is appended to the cache first and is the last token its query attends to.
# ----------------------------------------------------------------------------------------------
def attention_block_step(x, pos, ke_old, c_old, W_q, W_ke, W_dkv, W_uk, W_uv, W_o, elite_idx,
                         head_dim: int, rope_base: float):
    """One decode step of the attention block for B independent sequences.

    x [B, d] hidden states of the new tokens; pos [B] their positions; ke_old[b] [S_b, n_h, 2r] and
    c_old[b] [S_b, d_c] the rows cached so far (lists: S_b may differ, may be 0);
    W_q [d, n_h, d_h]; W_o [n_h, d_h, d]; the other weights as in append / decode_attn.
    Returns (y [B, d], ke_new [B, n_h, 2r], c_new [B, d_c]), float64.
    """
    x = np.asarray(x, dtype=F64)
    W_q = np.asarray(W_q, dtype=F64)
    W_o = np.asarray(W_o, dtype=F64)
    B = x.shape[0]
    q = np.einsum("bd,dhj->bhj", x, W_q)                                  # q_t = x_t W^q, head by head
    ke_new, c_new = append(x, pos, W_ke, W_dkv, elite_idx, head_dim, rope_base)
    ke_all = [np.concatenate([np.asarray(ke_old[b], dtype=F64), ke_new[b:b + 1]], axis=0) for b in range(B)]
    c_all = [np.concatenate([np.asarray(c_old[b], dtype=F64), c_new[b:b + 1]], axis=0) for b in range(B)]
    seq = [ke_all[b].shape[0] for b in range(B)]
    o = decode_attn(q, pos, ke_all, c_all, seq, W_uk, W_uv, elite_idx, head_dim, rope_base)
    y = np.einsum("bhj,hjd->bd", o, W_o)                                  # [o_0, ..., o_{n_h-1}] W^o
    return y, ke_new, c_new


# ----------------------------------------------------------------------------------------------
# Separated low-rank decomposition (Section 3.2, "Separated Low-Rank Decomposition"): the
# non-elite key block and the value block are factorised separately,
#     W^k_{e^,0:n_h-1} ~ A^k B^k_S,   W^v_{0:n_h-1} ~ A^v B^v_S,
# so a token caches two latents, c^k = x A^k (d_ck wide) and c^v = x A^v (d_cv wide), next to
# its rotated elite keys.  Everything else is as in the joint variant.
# ----------------------------------------------------------------------------------------------
def slrd_cache_row_elems(n_heads: int, r: int, d_ck: int, d_cv: int) -> int:
    """KV-cache elements per token per layer with S-LRD: 2 r n_h + d_ck + d_cv (Section 3.2)."""
    return 2 * r * n_heads + d_ck + d_cv


def slrd_param_count(d_model: int, n_heads: int, head_dim: int, r: int, d_ck: int, d_cv: int) -> int:
    """Section 3.2, storage cost of RoPElite with S-LRD:
    2 r n_h d + d_ck (d + d_h n_h - 2 r n_h) + d_cv (d + d_h n_h)."""
    return (2 * r * n_heads * d_model + d_ck * (d_model + head_dim * n_heads - 2 * r * n_heads)
            + d_cv * (d_model + head_dim * n_heads))


def slrd_append(x, pos, W_ke, A_k, A_v, elite_idx, head_dim: int, rope_base: float):
    """Cache rows for T tokens of an S-LRD model.

    x [T, d]; W_ke [d, n_h, 2r]; A_k [d, d_ck]; A_v [d, d_cv]; elite_idx [n_h, r].
    Returns (ke [T, n_h, 2r] rotated elite keys, c_k [T, d_ck], c_v [T, d_cv]), float64.
    """
    x = np.asarray(x, dtype=F64)
    ke, c_k = append(x, pos, W_ke, A_k, elite_idx, head_dim, rope_base)   # elite keys do not depend on the latent
    c_v = x @ np.asarray(A_v, dtype=F64)                                   # c^v_t = x_t A^v
    return ke, c_k, c_v


def slrd_decode_attn(q, q_pos, ke, c_k, c_v, seq_len, B_k, B_v, elite_idx, head_dim: int,
                     rope_base: float, heads=None):
    """Single-token decode attention of an S-LRD model: textbook attention (Section 2.1) over
        k_j = [ rotated elite dims | c^k_j B^k_S,h ]   and   v_j = c^v_j B^v_S,h.

    ke[b] [>=S_b, n_h, 2r]; c_k[b] [>=S_b, d_ck]; c_v[b] [>=S_b, d_cv];
    B_k [d_ck, n_h, d_h-2r]; B_v [d_cv, n_h, d_h].  Other arguments as decode_attn.
    """
    q = np.asarray(q, dtype=F64)
    B_k = np.asarray(B_k, dtype=F64)
    B_v = np.asarray(B_v, dtype=F64)
    elite_idx = np.asarray(elite_idx)
    B, n_h, d_h = q.shape
    assert d_h == head_dim
    r = elite_idx.shape[1]
    theta = rope_theta(head_dim, rope_base)
    out = np.zeros((B, n_h, d_h), dtype=F64)
    head_list = range(n_h) if heads is None else heads
    for b in range(B):
        S = int(seq_len[b])
        if S == 0:
            continue
        ke_b = np.asarray(ke[b], dtype=F64)[:S]
        ck_b = np.asarray(c_k[b], dtype=F64)[:S]
        cv_b = np.asarray(c_v[b], dtype=F64)[:S]
        for h in head_list:
            idx_h = elite_idx[h]
            q_e = q[b, h, elite_dims(idx_h)].reshape(r, 2)
            alpha = F64(int(q_pos[b])) * theta[idx_h.astype(np.int64)] if r else np.zeros(0)
            q_e = rotate_pairs(q_e, alpha).reshape(2 * r)
            q_hat = np.concatenate([q_e, q[b, h, nonelite_dims(idx_h, d_h)]])
            K_full = np.concatenate([ke_b[:, h, :], ck_b @ B_k[:, h, :]], axis=1)   # keys from c^k only
            V_full = cv_b @ B_v[:, h, :]                                             # values from c^v only
            out[b, h] = softmax_attention(q_hat, K_full, V_full, d_h)
    return out


def slrd_attention_block_step(x, pos, ke_old, ck_old, cv_old, W_q, W_ke, A_k, A_v, B_k, B_v, W_o, elite_idx,
                              head_dim: int, rope_base: float):
    """One decode step of the attention block of an S-LRD model (Section 2.1 for the projections
    q_t = x_t W^q and [o_0 .. o_{n_h-1}] W^o, Section 3.2 "Separated Low-Rank Decomposition" for what is
    cached and attended): the step's tokens are appended first and are the last tokens attended to.

    x [B, d]; pos [B]; ke_old[b] [S_b, n_h, 2r], ck_old[b] [S_b, d_ck], cv_old[b] [S_b, d_cv] (lists; S_b may
    be 0); W_q [d, n_h, d_h]; W_o [n_h, d_h, d]; the other weights as in slrd_append / slrd_decode_attn.
    Returns (y [B, d], ke_new [B, n_h, 2r], ck_new [B, d_ck], cv_new [B, d_cv]), float64.
    """
    x = np.asarray(x, dtype=F64)
    W_q = np.asarray(W_q, dtype=F64)
    W_o = np.asarray(W_o, dtype=F64)
    B = x.shape[0]
    q = np.einsum("bd,dhj->bhj", x, W_q)                                  # q_t = x_t W^q, head by head
    ke_new, ck_new, cv_new = slrd_append(x, pos, W_ke, A_k, A_v, elite_idx, head_dim, rope_base)
    cat = lambda old, new, b: np.concatenate([np.asarray(old[b], dtype=F64), new[b:b + 1]], axis=0)
    ke_all = [cat(ke_old, ke_new, b) for b in range(B)]
    ck_all = [cat(ck_old, ck_new, b) for b in range(B)]
    cv_all = [cat(cv_old, cv_new, b) for b in range(B)]
    seq = [ke_all[b].shape[0] for b in range(B)]
    o = slrd_decode_attn(q, pos, ke_all, ck_all, cv_all, seq, B_k, B_v, elite_idx, head_dim, rope_base)
    y = np.einsum("bhj,hjd->bd", o, W_o)                                  # [o_0, ..., o_{n_h-1}] W^o
    return y, ke_new, ck_new, cv_new


# ----------------------------------------------------------------------------------------------
# Several queries per sequence (a prefill chunk, or the verification of drafted tokens): every
# query is one more instance of the decode attention above, over the rows of its own sequence that
# it may see.  Section 2.1 builds K_t, V_t from the tokens up to t: a query at step t attends to the
# cache rows of steps <= t, which the caller states as a visible-row count per query.
# ----------------------------------------------------------------------------------------------
def multiquery_attn(q, q_pos, ke, c, kv_len, W_uk, W_uv, elite_idx, head_dim: int, rope_base: float):
    """q [B, T, n_h, d_h]; q_pos [B, T]; ke[b], c[b]: the planes of sequence b; kv_len [B, T] rows of
    sequence b visible to query (b, t) (causal decoding: position + 1).  Returns o [B, T, n_h, d_h]."""
    q = np.asarray(q, dtype=F64)
    B, T = q.shape[:2]
    out = np.zeros_like(q)
    for b in range(B):
        for t in range(T):
            out[b, t] = decode_attn(q[b, t][None], [int(q_pos[b][t])], [ke[b]], [c[b]], [int(kv_len[b][t])],
                                    W_uk, W_uv, elite_idx, head_dim, rope_base)[0]
    return out


def slrd_multiquery_attn(q, q_pos, ke, c_k, c_v, kv_len, B_k, B_v, elite_idx, head_dim: int, rope_base: float):
    """Several queries per sequence of an S-LRD model (Section 3.2): query (b, t) is one instance of
    slrd_decode_attn over the first kv_len[b][t] rows of sequence b.  Shapes as multiquery_attn, with
    the two latents c_k[b], c_v[b] and their up-projections B_k, B_v in place of c, W_uk, W_uv."""
    q = np.asarray(q, dtype=F64)
    B, T = q.shape[:2]
    out = np.zeros_like(q)
    for b in range(B):
        for t in range(T):
            out[b, t] = slrd_decode_attn(q[b, t][None], [int(q_pos[b][t])], [ke[b]], [c_k[b]], [c_v[b]],
                                         [int(kv_len[b][t])], B_k, B_v, elite_idx, head_dim, rope_base)[0]
    return out


# ----------------------------------------------------------------------------------------------
# RoPElite search (Section 3.1, Algorithm 1): the greedy choice of each head's elite chunks.
# Round after round, every chunk that is not yet elite is tried as the one additional rotated chunk;
# the chunk whose scores come closest (L1) to the scores of full RoPE is appended.
# Readings: "attn_score" is the pre-softmax score s of Section 2.1 (the quantity the Section 3.1 score
# equation rewrites), over the causal pairs (a query sees the keys up to its own step); ties go to
# the lowest chunk index.
# ----------------------------------------------------------------------------------------------
def rope_on_chunks(x, pos, chunks, head_dim: int, rope_base: float):
    """x [T, d_h] with only the listed chunks rotated by R(pos * theta_i) (Section 2.2, eq. 1a)."""
    x = np.array(x, dtype=F64, copy=True)
    theta = rope_theta(head_dim, rope_base)
    for i in chunks:
        i = int(i)
        x[:, 2 * i:2 * i + 2] = rotate_pairs(x[:, 2 * i:2 * i + 2], np.asarray(pos, dtype=F64) * theta[i])
    return x


def causal_scores(q_h, k_h, head_dim: int):
    """s[t, j] = q_t . k_j / sqrt(d_h) for j <= t, 0 elsewhere (Section 2.1, before the softmax)."""
    s = (q_h @ k_h.T) / np.sqrt(F64(head_dim))
    return np.tril(s)


def ropelite_search(q, k, pos, r: int, head_dim: int, rope_base: float):
    """q, k [T, n_h, d_h] un-rotated queries and keys of one layer; pos [T].
    Returns (elite [n_h, r] int32 in selection order, dist [n_h, r] the winning L1 distances)."""
    q = np.asarray(q, dtype=F64)
    k = np.asarray(k, dtype=F64)
    T, n_h, d_h = q.shape
    all_chunks = list(range(d_h // 2))
    elite = np.zeros((n_h, r), dtype=np.int32)
    dist_out = np.zeros((n_h, r), dtype=F64)
    for h in range(n_h):
        s_full = causal_scores(rope_on_chunks(q[:, h], pos, all_chunks, d_h, rope_base),
                               rope_on_chunks(k[:, h], pos, all_chunks, d_h, rope_base), d_h)
        e = []
        for i in range(r):
            best, best_d = -1, np.inf
            for j in all_chunks:
                if j in e:
                    continue
                s_try = causal_scores(rope_on_chunks(q[:, h], pos, e + [j], d_h, rope_base),
                                      rope_on_chunks(k[:, h], pos, e + [j], d_h, rope_base), d_h)
                dj = float(np.sum(np.abs(s_full - s_try)))
                if dj < best_d:                       # strict: the lowest index wins a tie
                    best, best_d = j, dj
            e.append(best)
            elite[h, i] = best
            dist_out[h, i] = best_d
    return elite, dist_out


def ropelite_distances(q, k, pos, elite_h, head, head_dim: int, rope_base: float):
    """L1 distance to the full-RoPE scores of head `head` for every chunk tried as the one addition
    to the elite list `elite_h` (np.inf for chunks already in it): one round of Algorithm 1."""
    q = np.asarray(q, dtype=F64)
    k = np.asarray(k, dtype=F64)
    d_h = q.shape[2]
    all_chunks = list(range(d_h // 2))
    e = [int(i) for i in elite_h]
    s_full = causal_scores(rope_on_chunks(q[:, head], pos, all_chunks, d_h, rope_base),
                           rope_on_chunks(k[:, head], pos, all_chunks, d_h, rope_base), d_h)
    out = np.full(d_h // 2, np.inf)
    for j in all_chunks:
        if j in e:
            continue
        s_try = causal_scores(rope_on_chunks(q[:, head], pos, e + [j], d_h, rope_base),
                              rope_on_chunks(k[:, head], pos, e + [j], d_h, rope_base), d_h)
        out[j] = float(np.sum(np.abs(s_full - s_try)))
    return out


def mha_decode(q, q_pos, K_rot, V, seq_len, rope_base: float):
    """Comparator: ordinary RoPE multi-head decode attention (Sections 2.1 and 2.2).

    q [B, n_h, d_h] un-rotated; K_rot[b] [>=S_b, n_h, d_h] keys already rotated at their
    own positions (what a RoPE model caches); V[b] [>=S_b, n_h, d_h].
    Every chunk of q is rotated at q_pos[b]; then textbook attention.
    """
    q = np.asarray(q, dtype=F64)
    B, n_h, d_h = q.shape
    theta = rope_theta(d_h, rope_base)
    out = np.zeros((B, n_h, d_h), dtype=F64)
    for b in range(B):
        S = int(seq_len[b])
        if S == 0:
            continue
        K_b = np.asarray(K_rot[b], dtype=F64)[:S]
        V_b = np.asarray(V[b], dtype=F64)[:S]
        alpha = F64(int(q_pos[b])) * theta
        for h in range(n_h):
            q_rot = rotate_pairs(q[b, h].reshape(d_h // 2, 2), alpha).reshape(d_h)
            out[b, h] = softmax_attention(q_rot, K_b[:, h, :], V_b[:, h, :], d_h)
    return out


def max_abs_rel(got, ref) -> float:
    """Error metric of the parity gates: max|got - ref| / max|ref| over one tensor."""
    got = np.asarray(got, dtype=F64)
    ref = np.asarray(ref, dtype=F64)
    denom = max(float(np.max(np.abs(ref))) if ref.size else 0.0, 1e-30)
    return float(np.max(np.abs(got - ref))) / denom if ref.size else 0.0
