"""GPU parity of the separated low-rank variant (Section 3.2, S-LRD; two latents per token stored
side by side in one latent-plane row) against the float64 oracle, through the C ABI.
Bounds as for the joint variant: max-abs-rel <= 1e-5 (fp32), 2e-2 (bf16)."""
import numpy as np
import pytest
import torch

import elitekv_synth as synth
import paper_2503_01586_amd as ekv
from oracle import elitekv_oracle as orc

from gpu_util import DEV, TOL, dev, dims_of, host64, i32, i64

pytestmark = pytest.mark.gpu


def shape(d_model, n_heads, head_dim, r, d_ck, d_cv, dtype, rope_base=10000.0):
    return dict(d_model=d_model, n_heads=n_heads, head_dim=head_dim, r=r, d_c=d_ck + d_cv, d_ck=d_ck, d_cv=d_cv,
                dtype=dtype, rope_base=rope_base)


def _draw(sh, T, B, seed):
    rng = np.random.default_rng(seed)
    n_h, d_h, r, d = sh["n_heads"], sh["head_dim"], sh["r"], sh["d_model"]
    idx = synth.draw_elite_idx(rng, n_h, d_h, r) if r else np.zeros((n_h, 0), dtype=np.int32)
    W_ke, A_k, B_k, _ = synth.draw_weights(rng, d, n_h, d_h, r, sh["d_ck"])
    _, A_v, _, B_v = synth.draw_weights(rng, d, n_h, d_h, r, sh["d_cv"])
    x = synth.draw_hidden(rng, T, d)
    q = synth.draw_query(rng, B, n_h, d_h)
    return rng, idx, W_ke, A_k, A_v, B_k, B_v, x, q


def gpu_slrd_append(dims, d_ck, x, pos, slot, W_ke, A_k, A_v, idx, rows):
    dt = ekv.torch_dtype(dims)
    ke = torch.zeros(rows, dims.n_heads, 2 * dims.r, dtype=dt, device=DEV)
    c = torch.zeros(rows, dims.d_c, dtype=dt, device=DEV)
    ws = torch.empty(max(ekv.elitekv_slrd_append_workspace_bytes(dims, d_ck, x.shape[0]), 16), dtype=torch.uint8,
                     device=DEV)
    ekv.elitekv_slrd_append(dims, d_ck, x, pos, slot, W_ke, A_k, A_v, idx, ke, c, ws=ws)
    torch.cuda.synchronize()
    return ke, c


def gpu_slrd_decode(dims, d_ck, q, q_pos, seq_len, max_seq, stride, B_k, B_v, idx, ke, c, n_splits=0):
    B = q.shape[0]
    out = torch.full((B, dims.n_heads, dims.head_dim), float("nan"), dtype=ekv.torch_dtype(dims), device=DEV)
    nws = ekv.elitekv_slrd_decode_workspace_bytes(dims, d_ck, B, max_seq, n_splits)
    assert nws > 0
    ws = torch.full((nws,), 0xFF, dtype=torch.uint8, device=DEV)     # nothing may depend on old contents
    ekv.elitekv_slrd_decode_attn(dims, d_ck, q, q_pos, seq_len, max_seq, stride, B_k, B_v, idx, ke, c, out, ws,
                                 n_splits=n_splits)
    torch.cuda.synchronize()
    return out


APPEND_CASES = {
    # name: (shape, T)   -- generic fp32, few-token VALU, split-K MFMA, MFMA GEMM
    "fp32_tiny": (shape(96, 3, 16, 2, 24, 40, "fp32"), 21),
    "bf16_7b_one_token": (shape(4096, 32, 128, 8, 576, 960, "bf16"), 1),
    "bf16_7b_batch_16": (shape(4096, 32, 128, 8, 576, 960, "bf16"), 16),
    "bf16_7b_300_tokens": (shape(4096, 32, 128, 8, 640, 896, "bf16"), 300),
    "bf16_7b_300_tokens_576": (shape(4096, 32, 128, 8, 576, 960, "bf16"), 300),      # boundary inside a 128-column block
    "bf16_unaligned_split": (shape(512, 8, 64, 4, 72, 56, "bf16"), 40),       # falls to the generic kernel
}


@pytest.mark.parametrize("name", list(APPEND_CASES))
def test_slrd_append_matches_oracle(name):
    sh, T = APPEND_CASES[name]
    dt, d_ck = sh["dtype"], sh["d_ck"]
    rng, idx, W_ke, A_k, A_v, _, _, x, _ = _draw(sh, T, 1, 300 + len(name))
    dims = dims_of(sh)
    pos = rng.integers(0, 5000, size=T)
    rows = T + 4
    slot = rng.permutation(rows)[:T]
    xd, Wked, Akd, Avd = dev(x, dt), dev(W_ke, dt), dev(A_k, dt), dev(A_v, dt)
    ke, c = gpu_slrd_append(dims, d_ck, xd, i32(pos), i64(slot), Wked, Akd, Avd, i32(idx), rows)
    ke_ref, ck_ref, cv_ref = orc.slrd_append(host64(xd), pos, host64(Wked), host64(Akd), host64(Avd), idx,
                                             sh["head_dim"], sh["rope_base"])
    c_g = host64(c)
    assert orc.max_abs_rel(c_g[slot][:, :d_ck], ck_ref) <= TOL[dt]
    assert orc.max_abs_rel(c_g[slot][:, d_ck:], cv_ref) <= TOL[dt]
    assert orc.max_abs_rel(host64(ke)[slot], ke_ref) <= TOL[dt]
    untouched = np.setdiff1d(np.arange(rows), slot)
    assert np.all(c_g[untouched] == 0.0)


DECODE_CASES = {
    # name: (shape, seq_len per batch row, splits)
    "fp32_tiny": (shape(64, 3, 24, 5, 20, 37, "fp32"), [0, 1, 63, 130], [0, 1, 3]),
    "bf16_7b_576_960": (shape(64, 32, 128, 8, 576, 960, "bf16"), [300, 1, 257], [0, 1, 4]),
    "bf16_7b_192_1344": (shape(64, 32, 128, 8, 192, 1344, "bf16"), [97], [0, 3]),
    "bf16_7b_1344_192": (shape(64, 32, 128, 8, 1344, 192, "bf16"), [150], [0, 2]),
    "bf16_7b_batch_768_768": (shape(64, 32, 128, 8, 768, 768, "bf16"), [0, 1, 15, 16, 17, 250, 33, 48, 100], [0, 3]),
    "bf16_7b_12pct_384_384": (shape(64, 32, 128, 4, 384, 384, "bf16"), [130, 64], [0, 3]),
    "bf16_small_heads_64_192": (shape(64, 8, 64, 4, 64, 192, "bf16"), [70, 33], [0, 2]),
    "bf16_13b_960_960": (shape(64, 40, 128, 8, 960, 960, "bf16"), [97, 40], [0, 2]),      # generic kernels
    "bf16_448_448_one_wave_per_simd": (shape(64, 32, 128, 8, 448, 448, "bf16"), [150, 33], [0, 2]),   # 224-column wave slices
    "bf16_r16_448_448": (shape(64, 32, 128, 16, 448, 448, "bf16"), [150, 33], [0, 2]),    # generic kernels (32 elite values beside 224-column slices)
    "bf16_r32_512_512": (shape(64, 32, 128, 32, 512, 512, "bf16"), [97, 16], [0, 2]),     # generic kernels (64 elite values per head)
}


@pytest.mark.parametrize("name", list(DECODE_CASES))
def test_slrd_decode_matches_oracle_on_same_planes(name):
    sh, seqs, splits = DECODE_CASES[name]
    dt, d_ck = sh["dtype"], sh["d_ck"]
    B, stride = len(seqs), max(seqs) + 3
    rng, idx, W_ke, A_k, A_v, B_k, B_v, x, q = _draw(sh, B * stride, B, 400 + len(name))
    dims = dims_of(sh)
    pos = np.tile(np.arange(stride), B)
    ke64, ck64, cv64 = orc.slrd_append(x, pos, W_ke, A_k, A_v, idx, sh["head_dim"], sh["rope_base"])
    ked, cd = dev(ke64, dt), dev(np.concatenate([ck64, cv64], axis=1), dt)
    qd, Bkd, Bvd = dev(q, dt), dev(B_k, dt), dev(B_v, dt)
    q_pos = np.array([max(s - 1, 0) for s in seqs])
    c_h = host64(cd).reshape(B, stride, -1)
    ref = orc.slrd_decode_attn(host64(qd), q_pos, host64(ked).reshape(B, stride, sh["n_heads"], -1),
                               c_h[:, :, :d_ck], c_h[:, :, d_ck:], seqs, host64(Bkd), host64(Bvd), idx,
                               sh["head_dim"], sh["rope_base"])
    outs = []
    for ns in splits:
        o = host64(gpu_slrd_decode(dims, d_ck, qd, i32(q_pos), i32(seqs), max(seqs), stride, Bkd, Bvd, i32(idx),
                                   ked, cd, n_splits=ns))
        assert np.all(np.isfinite(o))
        err = orc.max_abs_rel(o, ref)
        assert err <= TOL[dt], "n_splits=%d err=%g" % (ns, err)
        for b, s in enumerate(seqs):
            if s == 0:
                assert np.all(o[b] == 0.0)
        outs.append(o)
    for o in outs[1:]:
        assert orc.max_abs_rel(o, outs[0]) <= TOL[dt]


MULTIQUERY_CASES = {
    # name: (shape, cached rows per sequence, T, splits)
    "fp32_tiny": (shape(64, 3, 24, 5, 20, 37, "fp32"), [40, 7, 130], 5, [0, 2]),
    "bf16_7b_576_960_chunk_of_4": (shape(64, 32, 128, 8, 576, 960, "bf16"), [300, 65], 4, [0, 3]),
    "bf16_7b_768_768_chunk_of_16": (shape(64, 32, 128, 8, 768, 768, "bf16"), [200], 16, [0]),
    "bf16_12pct_384_384_chunk_of_9": (shape(64, 32, 128, 4, 384, 384, "bf16"), [130], 9, [0]),
    "bf16_13b_960_960_chunk_of_3": (shape(64, 40, 128, 8, 960, 960, "bf16"), [97, 160], 3, [0, 2]),
}


@pytest.mark.parametrize("name", list(MULTIQUERY_CASES))
def test_slrd_multiquery_matches_oracle(name):
    """The queries are the last T tokens of each sequence; a sequence shorter than the chunk leaves
    its first queries with nothing to see (zeros)."""
    sh, rows, T, splits = MULTIQUERY_CASES[name]
    dt, d_ck = sh["dtype"], sh["d_ck"]
    n_h, d_h = sh["n_heads"], sh["head_dim"]
    B, stride = len(rows), max(rows) + 2
    rng, idx, W_ke, A_k, A_v, B_k, B_v, x, _ = _draw(sh, B * stride, B, 700 + len(name))
    q = rng.standard_normal((B, T, n_h, d_h))
    dims = dims_of(sh)
    pos = np.tile(np.arange(stride), B)
    ke64, ck64, cv64 = orc.slrd_append(x, pos, W_ke, A_k, A_v, idx, d_h, sh["rope_base"])
    ked, cd = dev(ke64, dt), dev(np.concatenate([ck64, cv64], axis=1), dt)
    qd, Bkd, Bvd = dev(q, dt), dev(B_k, dt), dev(B_v, dt)
    q_pos = np.array([[max(n - T + t, 0) for t in range(T)] for n in rows])
    kv_len = np.array([[max(n - T + t + 1, 0) for t in range(T)] for n in rows])
    c_h = host64(cd).reshape(B, stride, -1)
    ref = orc.slrd_multiquery_attn(host64(qd), q_pos, host64(ked).reshape(B, stride, n_h, -1), c_h[:, :, :d_ck],
                                   c_h[:, :, d_ck:], kv_len, host64(Bkd), host64(Bvd), idx, d_h, sh["rope_base"])
    for ns in splits:
        out = torch.full((B, T, n_h, d_h), float("nan"), dtype=ekv.torch_dtype(dims), device=DEV)
        nws = ekv.elitekv_slrd_multiquery_workspace_bytes(dims, d_ck, B, T, max(rows), ns)
        assert nws > 0
        ws = torch.full((nws,), 0xFF, dtype=torch.uint8, device=DEV)
        ekv.elitekv_slrd_multiquery_attn(dims, d_ck, qd, i32(q_pos.reshape(-1)), i32(kv_len.reshape(-1)), max(rows),
                                         stride, Bkd, Bvd, i32(idx), ked, cd, out, ws, n_splits=ns)
        torch.cuda.synchronize()
        o = host64(out)
        assert np.all(np.isfinite(o))
        assert orc.max_abs_rel(o, ref) <= TOL[dt], "n_splits=%d" % ns
        assert np.all(o[kv_len == 0] == 0.0)


def test_slrd_one_query_per_sequence_is_the_decode_call():
    sh = shape(64, 32, 128, 8, 576, 960, "bf16")
    rows, B, stride = [120, 77], 2, 125
    rng, idx, _, _, _, B_k, B_v, _, q = _draw(sh, 1, B, 19)
    dims, d_ck = dims_of(sh), sh["d_ck"]
    ke64, c64 = synth.draw_cache_planes(rng, B * stride, 32, 8, 1536)
    ked, cd, qd, Bkd, Bvd = (dev(a, "bf16") for a in (ke64, c64, q, B_k, B_v))
    q_pos, seq = i32([r - 1 for r in rows]), i32(rows)
    a = gpu_slrd_decode(dims, d_ck, qd, q_pos, seq, max(rows), stride, Bkd, Bvd, i32(idx), ked, cd)
    out = torch.empty(B, 1, 32, 128, dtype=torch.bfloat16, device=DEV)
    ws = torch.empty(ekv.elitekv_slrd_multiquery_workspace_bytes(dims, d_ck, B, 1, max(rows)), dtype=torch.uint8,
                     device=DEV)
    ekv.elitekv_slrd_multiquery_attn(dims, d_ck, qd.reshape(B, 1, 32, 128), q_pos, seq, max(rows), stride, Bkd, Bvd,
                                     i32(idx), ked, cd, out, ws)
    torch.cuda.synchronize()
    assert torch.equal(out.reshape(B, 32, 128), a)


def test_slrd_end_to_end_and_repeatable():
    sh, S = shape(256, 32, 128, 8, 576, 960, "bf16"), 333
    _, idx, W_ke, A_k, A_v, B_k, B_v, x, q = _draw(sh, S, 1, 51)
    dims, d_ck = dims_of(sh), sh["d_ck"]
    pos = np.arange(S)
    xd, Wked, Akd, Avd, Bkd, Bvd, qd = (dev(a, "bf16") for a in (x, W_ke, A_k, A_v, B_k, B_v, q))
    ke, c = gpu_slrd_append(dims, d_ck, xd, i32(pos), i64(pos), Wked, Akd, Avd, i32(idx), S)
    out = gpu_slrd_decode(dims, d_ck, qd, i32([S - 1]), i32([S]), S, S, Bkd, Bvd, i32(idx), ke, c)
    again = gpu_slrd_decode(dims, d_ck, qd, i32([S - 1]), i32([S]), S, S, Bkd, Bvd, i32(idx), ke, c)
    assert torch.equal(out, again)
    ke_r, ck_r, cv_r = orc.slrd_append(host64(xd), pos, host64(Wked), host64(Akd), host64(Avd), idx, 128, 10000.0)
    ref = orc.slrd_decode_attn(host64(qd), [S - 1], ke_r[None], ck_r[None], cv_r[None], [S], host64(Bkd), host64(Bvd),
                               idx, 128, 10000.0)
    assert orc.max_abs_rel(host64(out), ref) <= TOL["bf16"]


def test_slrd_argument_errors():
    sh = shape(64, 32, 128, 8, 576, 960, "bf16")
    dims = dims_of(sh)
    assert ekv.elitekv_slrd_decode_workspace_bytes(dims, 0, 1, 128) == 0          # d_ck must be inside (0, d_c)
    assert ekv.elitekv_slrd_decode_workspace_bytes(dims, 1536, 1, 128) == 0
    assert ekv.elitekv_slrd_param_count(dims, 576) == orc.slrd_param_count(64, 32, 128, 8, 576, 960)
    with pytest.raises(ekv.EliteKVError):
        ekv.elitekv_slrd_param_count(dims, 1536)
