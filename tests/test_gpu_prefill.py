"""GPU parity of attention with MANY queries per sequence (elitekv_prefill_attn: keys and values
rebuilt once per cached row, then flash attention) against the float64 oracle, through the C ABI.
The oracle computes every query by the decode definition (reconstructed keys and values, textbook
attention), so it is run on a seeded sample of the queries (all heads of each); every query is also
compared with the library's own absorbed-form path (elitekv_multiquery_attn), which has its own
oracle test.  Bound: 2e-2 (bf16), max-abs-rel."""
import numpy as np
import pytest
import torch

import paper_2503_01586_amd as ekv
from oracle import elitekv_oracle as orc

from gpu_util import DEV, TOL, dev, dims_of, host64, i32
from test_gpu_parity import _draw, shape

pytestmark = pytest.mark.gpu

CASES = {
    # name: (shape, cached rows per sequence, T, kind of visibility, sampled queries per sequence)
    # causal: the T queries are the last T tokens of the sequence; random: any visible length, zeros included
    "small_two_seqs_causal": (shape(64, 8, 128, 8, 256, "bf16"), [300, 191], 150, "causal", 24),
    "small_three_blocks_random": (shape(64, 8, 128, 8, 256, "bf16"), [333], 300, "random", 32),
    "small_full_prefill_r4": (shape(64, 8, 128, 4, 384, "bf16"), [257, 129], 129, "causal", 20),
    "7b_full_prefill": (shape(64, 32, 128, 8, 1536, "bf16"), [200], 200, "causal", 10),
    "7b_12pct_chunk_over_context": (shape(64, 32, 128, 4, 768, "bf16"), [130, 257], 70, "causal", 6),
    "13b_full_prefill": (shape(64, 40, 128, 8, 1920, "bf16"), [97], 97, "causal", 6),
    # more work-groups than compute units, three sequences, five query blocks (an unpaired middle one)
    "many_work_groups": (shape(64, 32, 128, 8, 256, "bf16"), [700, 650, 720], 640, "causal", 5),
    # the sequences lie back to back in the planes (stride == max_seq_len): one rebuild launch for all of them
    "back_to_back": (shape(64, 8, 128, 8, 256, "bf16"), [300, 130, 257], 130, "causal", 8),
}
PAD = {"back_to_back": 0}        # plane rows between the longest sequence's end and the next sequence's start (default 3)


def _run(name):
    sh, rows, T, kind, n_sample = CASES[name]
    dt = sh["dtype"]
    B, stride, S = len(rows), max(rows) + PAD.get(name, 3), max(rows)
    n_h, d_h = sh["n_heads"], sh["head_dim"]
    rng, idx, W_ke, W_dkv, W_uk, W_uv, x, _ = _draw(sh, B * stride, B, 4200 + len(name))
    q = rng.standard_normal((B, T, n_h, d_h))
    dims = dims_of(sh)
    pos = np.tile(np.arange(stride), B)
    ke64, c64 = orc.append(x, pos, W_ke, W_dkv, idx, d_h, sh["rope_base"])
    # rows a sequence does not own yet hold NaN: nothing may read them into a result
    # (the rebuild does read the first S latent rows of every sequence; what it makes of them is never used)
    for b, n in enumerate(rows):
        ke64[b * stride + n:(b + 1) * stride] = np.nan
        c64[b * stride + n:(b + 1) * stride] = np.nan
    ked, cd = dev(ke64, dt), dev(c64, dt)
    qd, Wukd, Wuvd = dev(q, dt), dev(W_uk, dt), dev(W_uv, dt)
    if kind == "causal":
        q_pos = np.array([[max(n - T + t, 0) for t in range(T)] for n in rows])
        kv_len = np.array([[max(n - T + t + 1, 0) for t in range(T)] for n in rows])
    else:
        kv_len = np.stack([rng.integers(0, n + 1, size=T) for n in rows])
        kv_len[:, ::17] = 0
        kv_len[:, 5] = np.array(rows)
        q_pos = np.maximum(kv_len - 1, 0)
    out = torch.full((B, T, n_h, d_h), float("nan"), dtype=ekv.torch_dtype(dims), device=DEV)
    nws = ekv.elitekv_prefill_attn_workspace_bytes(dims, B, T, S)
    assert nws > 0
    ws = torch.full((nws,), 0xFF, dtype=torch.uint8, device=DEV)      # poisoned: nothing may depend on old contents
    ekv.elitekv_prefill_attn(dims, qd, i32(q_pos.reshape(-1)), i32(kv_len.reshape(-1)), S, stride, Wukd, Wuvd,
                             i32(idx), ked, cd, out, ws)
    torch.cuda.synchronize()
    o = host64(out)
    assert np.all(np.isfinite(o)), name
    assert np.all(o[kv_len == 0] == 0.0)
    return sh, rows, T, B, stride, rng, idx, qd, q_pos, kv_len, ked, cd, Wukd, Wuvd, dims, o, n_sample, S


@pytest.mark.parametrize("name", list(CASES))
def test_prefill_matches_oracle_on_sampled_queries(name):
    sh, rows, T, B, stride, rng, idx, qd, q_pos, kv_len, ked, cd, Wukd, Wuvd, dims, o, n_sample, S = _run(name)
    n_h, d_h = sh["n_heads"], sh["head_dim"]
    # first, last, block edges and random queries
    pick = sorted(set([0, T - 1, min(127, T - 1), min(128, T - 1)] + list(rng.choice(T, size=n_sample, replace=False))))
    ke_h = np.nan_to_num(host64(ked)).reshape(B, stride, n_h, -1)
    c_h = np.nan_to_num(host64(cd)).reshape(B, stride, -1)
    ref = orc.multiquery_attn(host64(qd)[:, pick], q_pos[:, pick], ke_h, c_h, kv_len[:, pick], host64(Wukd),
                              host64(Wuvd), idx, d_h, sh["rope_base"])
    assert orc.max_abs_rel(o[:, pick], ref) <= TOL["bf16"]


@pytest.mark.parametrize("name", ["small_two_seqs_causal", "small_three_blocks_random", "7b_full_prefill",
                                  "many_work_groups", "back_to_back"])
def test_prefill_agrees_with_the_absorbed_form_on_every_query(name):
    sh, rows, T, B, stride, rng, idx, qd, q_pos, kv_len, ked, cd, Wukd, Wuvd, dims, o, n_sample, S = _run(name)
    out2 = torch.full_like(torch.empty(B, T, sh["n_heads"], sh["head_dim"], dtype=torch.bfloat16, device=DEV), float("nan"))
    ws = torch.empty(ekv.elitekv_multiquery_workspace_bytes(dims, B, T, S), dtype=torch.uint8, device=DEV)
    ked2, cd2 = torch.nan_to_num(ked), torch.nan_to_num(cd)
    ekv.elitekv_multiquery_attn(dims, qd, i32(q_pos.reshape(-1)), i32(kv_len.reshape(-1)), S, stride, Wukd, Wuvd,
                                i32(idx), ked2, cd2, out2, ws)
    torch.cuda.synchronize()
    o2 = host64(out2)
    # two bf16 computations of the same quantity, each within 2e-2 of the exact result
    scale = np.max(np.abs(o2))
    assert np.max(np.abs(o - o2)) <= 2 * TOL["bf16"] * scale


def test_prefill_is_repeatable_bit_for_bit():
    a = _run("small_three_blocks_random")[15]
    b = _run("small_three_blocks_random")[15]
    assert np.array_equal(a, b)


def test_other_shapes_take_the_decode_kernels():
    """head_dim 64 is outside the flash kernel: the call is served query by query and still matches."""
    sh = shape(64, 4, 64, 4, 128, "bf16")
    rows, T = [90], 20
    B, stride = 1, 95
    rng, idx, W_ke, W_dkv, W_uk, W_uv, x, _ = _draw(sh, stride, B, 77)
    q = rng.standard_normal((B, T, 4, 64))
    dims = dims_of(sh)
    ke64, c64 = orc.append(x, np.arange(stride), W_ke, W_dkv, idx, 64, sh["rope_base"])
    ked, cd, qd, Wukd, Wuvd = dev(ke64, "bf16"), dev(c64, "bf16"), dev(q, "bf16"), dev(W_uk, "bf16"), dev(W_uv, "bf16")
    q_pos = np.array([[90 - T + t for t in range(T)]])
    kv_len = q_pos + 1
    out = torch.full((B, T, 4, 64), float("nan"), dtype=torch.bfloat16, device=DEV)
    ws = torch.empty(ekv.elitekv_prefill_attn_workspace_bytes(dims, B, T, 90), dtype=torch.uint8, device=DEV)
    ekv.elitekv_prefill_attn(dims, qd, i32(q_pos.reshape(-1)), i32(kv_len.reshape(-1)), 90, stride, Wukd, Wuvd, i32(idx),
                             ked, cd, out, ws)
    torch.cuda.synchronize()
    ref = orc.multiquery_attn(host64(qd), q_pos, host64(ked).reshape(B, stride, 4, -1), host64(cd).reshape(B, stride, -1),
                              kv_len, host64(Wukd), host64(Wuvd), idx, 64, sh["rope_base"])
    assert orc.max_abs_rel(host64(out), ref) <= TOL["bf16"]


def test_prefill_with_scores_that_keep_rising():
    """The running maximum of a query has to be raised many times along the keys (and is lowered never):
    the latent rows are multiples g(j) of one direction, so a head's score is g(j) times a per-(query, head)
    constant, rising for some and falling for others, far beyond the kernel's slack of 8 (log2 domain)."""
    import elitekv_synth as synth
    sh = shape(64, 8, 128, 8, 256, "bf16")
    S, T, n_h, d_c = 500, 200, 8, 256
    rng, idx, _, _, W_uk, W_uv, _, _ = _draw(sh, 1, 1, 78)
    ke64, c64 = synth.draw_cache_planes(rng, S, n_h, sh["r"], d_c)
    v = rng.standard_normal(d_c)
    g = np.linspace(0.0, 15.0, S) + 0.3 * np.sin(np.arange(S))
    c64 = 0.05 * c64 + g[:, None] * v[None, :]
    q = rng.standard_normal((1, T, n_h, 128))
    dims = dims_of(sh)
    ked, cd, qd, Wukd, Wuvd = dev(ke64, "bf16"), dev(c64, "bf16"), dev(q, "bf16"), dev(W_uk, "bf16"), dev(W_uv, "bf16")
    q_pos = np.arange(S - T, S)[None]
    kv_len = q_pos + 1
    q64, Wuk64, c_r = host64(qd)[0], host64(Wukd), host64(cd)
    rise = []
    for h in range(n_h):
        qt = q64[:, h][:, orc.nonelite_dims(idx[h], 128)] @ Wuk64[:, h, :].T           # [T, d_c]
        s = (qt @ c_r.T) * np.log2(np.e) / np.sqrt(128.0)
        rise.append(s[:, S - T] - s[:, 0])
    rise = np.concatenate(rise)
    assert rise.max() > 24.0 and rise.min() < -24.0
    out = torch.full((1, T, n_h, 128), float("nan"), dtype=torch.bfloat16, device=DEV)
    ws = torch.empty(ekv.elitekv_prefill_attn_workspace_bytes(dims, 1, T, S), dtype=torch.uint8, device=DEV)
    ekv.elitekv_prefill_attn(dims, qd, i32(q_pos.reshape(-1)), i32(kv_len.reshape(-1)), S, S, Wukd, Wuvd, i32(idx),
                             ked, cd, out, ws)
    torch.cuda.synchronize()
    o = host64(out)
    assert np.all(np.isfinite(o))
    pick = list(range(0, T, 9)) + [T - 1]
    ref = orc.multiquery_attn(host64(qd)[:, pick], q_pos[:, pick], host64(ked).reshape(1, S, n_h, -1),
                              c_r.reshape(1, S, -1), kv_len[:, pick], Wuk64, host64(Wuvd), idx, 128, sh["rope_base"])
    assert orc.max_abs_rel(o[:, pick], ref) <= TOL["bf16"]


# ----------------------------------------------------------------------------------------------
# Separated latents (Section 3.2, S-LRD): keys rebuilt from c^k, values from c^v
# ----------------------------------------------------------------------------------------------
from test_gpu_slrd import _draw as _draw_slrd, shape as slrd_shape   # noqa: E402

SLRD_CASES = {
    # name: (shape, cached rows per sequence, T, kind of visibility, sampled queries per sequence)
    "7b_576_960_two_seqs_causal": (slrd_shape(64, 32, 128, 8, 576, 960, "bf16"), [300, 191], 150, "causal", 8),
    "7b_768_768_random": (slrd_shape(64, 32, 128, 8, 768, 768, "bf16"), [333], 300, "random", 10),
    "7b_192_1344_full_prefill": (slrd_shape(64, 32, 128, 8, 192, 1344, "bf16"), [200], 200, "causal", 8),
    "7b_12pct_384_384": (slrd_shape(64, 32, 128, 4, 384, 384, "bf16"), [130, 257], 70, "causal", 6),
    "13b_960_960": (slrd_shape(64, 40, 128, 8, 960, 960, "bf16"), [97], 97, "causal", 6),
    "small_8_heads_160_96": (slrd_shape(64, 8, 128, 8, 160, 96, "bf16"), [700, 650, 720], 640, "causal", 6),
    # d_ck not a multiple of 32: served query by query through the decode kernels
    "7b_576_960_back_to_back": (slrd_shape(64, 32, 128, 8, 576, 960, "bf16"), [200, 120], 100, "causal", 6),
    "7b_d_ck_72_handed_over": (slrd_shape(64, 32, 128, 8, 72, 56, "bf16"), [90], 50, "causal", 6),
}


@pytest.mark.parametrize("name", list(SLRD_CASES))
def test_slrd_prefill_matches_oracle_and_the_absorbed_form(name):
    sh, rows, T, kind, n_sample = SLRD_CASES[name]
    dt, d_ck = sh["dtype"], sh["d_ck"]
    B, stride, S = len(rows), max(rows) + (0 if name.endswith("back_to_back") else 3), max(rows)
    n_h, d_h = sh["n_heads"], sh["head_dim"]
    rng, idx, W_ke, A_k, A_v, B_k, B_v, x, _ = _draw_slrd(sh, B * stride, B, 5200 + len(name))
    q = rng.standard_normal((B, T, n_h, d_h))
    dims = dims_of(sh)
    pos = np.tile(np.arange(stride), B)
    ke64, ck64, cv64 = orc.slrd_append(x, pos, W_ke, A_k, A_v, idx, d_h, sh["rope_base"])
    c64 = np.concatenate([ck64, cv64], axis=1)
    for b, n in enumerate(rows):                   # rows a sequence does not own yet: nothing may read them into a result
        ke64[b * stride + n:(b + 1) * stride] = np.nan
        c64[b * stride + n:(b + 1) * stride] = np.nan
    ked, cd = dev(ke64, dt), dev(c64, dt)
    qd, Bkd, Bvd = dev(q, dt), dev(B_k, dt), dev(B_v, dt)
    if kind == "causal":
        q_pos = np.array([[max(n - T + t, 0) for t in range(T)] for n in rows])
        kv_len = np.array([[max(n - T + t + 1, 0) for t in range(T)] for n in rows])
    else:
        kv_len = np.stack([rng.integers(0, n + 1, size=T) for n in rows])
        kv_len[:, ::17] = 0
        kv_len[:, 5] = np.array(rows)
        q_pos = np.maximum(kv_len - 1, 0)
    out = torch.full((B, T, n_h, d_h), float("nan"), dtype=torch.bfloat16, device=DEV)
    nws = ekv.elitekv_slrd_prefill_attn_workspace_bytes(dims, d_ck, B, T, S)
    assert nws > 0
    ws = torch.full((nws,), 0xFF, dtype=torch.uint8, device=DEV)
    ekv.elitekv_slrd_prefill_attn(dims, d_ck, qd, i32(q_pos.reshape(-1)), i32(kv_len.reshape(-1)), S, stride, Bkd, Bvd,
                                  i32(idx), ked, cd, out, ws)
    torch.cuda.synchronize()
    o = host64(out)
    assert np.all(np.isfinite(o)), name
    assert np.all(o[kv_len == 0] == 0.0)
    # the oracle on sampled queries (first, last, block edges, random)
    pick = sorted(set([0, T - 1, min(127, T - 1), min(128, T - 1)] + list(rng.choice(T, size=n_sample, replace=False))))
    ke_h = np.nan_to_num(host64(ked)).reshape(B, stride, n_h, -1)
    c_h = np.nan_to_num(host64(cd)).reshape(B, stride, -1)
    ref = orc.slrd_multiquery_attn(host64(qd)[:, pick], q_pos[:, pick], ke_h, c_h[:, :, :d_ck], c_h[:, :, d_ck:],
                                   kv_len[:, pick], host64(Bkd), host64(Bvd), idx, d_h, sh["rope_base"])
    assert orc.max_abs_rel(o[:, pick], ref) <= TOL["bf16"]
    # every query against the absorbed form (two bf16 computations, each within 2e-2 of the exact result)
    out2 = torch.full_like(out, float("nan"))
    ws2 = torch.empty(ekv.elitekv_slrd_multiquery_workspace_bytes(dims, d_ck, B, T, S), dtype=torch.uint8, device=DEV)
    ekv.elitekv_slrd_multiquery_attn(dims, d_ck, qd, i32(q_pos.reshape(-1)), i32(kv_len.reshape(-1)), S, stride, Bkd,
                                     Bvd, i32(idx), torch.nan_to_num(ked), torch.nan_to_num(cd), out2, ws2)
    torch.cuda.synchronize()
    o2 = host64(out2)
    assert np.max(np.abs(o - o2)) <= 2 * TOL["bf16"] * np.max(np.abs(o2))
