"""A seeded sweep of the decode attention over drawn batch sizes, sequence lengths (tile edges and
empty sequences included), plane strides, split counts and latent widths, against the float64
oracle through the C ABI: the joint latent and the separated latents, the single-query call and the
several-queries call.  Bounds: 2e-2 (bf16), max-abs-rel."""
import numpy as np
import pytest
import torch

import elitekv_synth as synth
import paper_2503_01586_amd as ekv
from oracle import elitekv_oracle as orc

from gpu_util import DEV, TOL, dev, dims_of, gpu_decode, host64, i32

pytestmark = pytest.mark.gpu

# (n_heads, r, d_c): 7B at 25 % and 12.5 %, the 13B shape (two head groups), a narrow latent
SHAPES = [(32, 8, 1536), (32, 4, 768), (40, 8, 1920), (32, 8, 512)]
EDGE_LENGTHS = [0, 1, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 128, 129]


def _case(seed):
    rng = np.random.default_rng(9000 + seed)
    n_h, r, d_c = SHAPES[seed % len(SHAPES)]
    B = int(rng.integers(1, 10))
    lens = [int(rng.choice(EDGE_LENGTHS)) if rng.random() < 0.5 else int(rng.integers(1, 420)) for _ in range(B)]
    if max(lens) == 0:
        lens[0] = 37
    stride = max(lens) + int(rng.integers(0, 6))
    n_splits = int(rng.choice([0, 0, 1, 2, 3, 5, 7]))
    return rng, n_h, r, d_c, B, lens, stride, n_splits


@pytest.mark.parametrize("seed", range(12))
def test_decode_sweep_joint(seed):
    rng, n_h, r, d_c, B, lens, stride, n_splits = _case(seed)
    d_h = 128
    idx = synth.draw_elite_idx(rng, n_h, d_h, r)
    _, _, W_uk, W_uv = synth.draw_weights(rng, 64, n_h, d_h, r, d_c)
    ke64, c64 = synth.draw_cache_planes(rng, B * stride, n_h, r, d_c)
    q = synth.draw_query(rng, B, n_h, d_h)
    dims = ekv.make_dims(64, n_h, d_h, r, d_c, "bf16", 10000.0)
    ked, cd, qd, Wukd, Wuvd = (dev(a, "bf16") for a in (ke64, c64, q, W_uk, W_uv))
    q_pos = np.array([max(n - 1, 0) for n in lens])
    out = host64(gpu_decode(dims, qd, i32(q_pos), i32(lens), max(lens), stride, Wukd, Wuvd, i32(idx), ked, cd,
                            n_splits=n_splits))
    ref = orc.decode_attn(host64(qd), q_pos, host64(ked).reshape(B, stride, n_h, -1), host64(cd).reshape(B, stride, -1),
                          lens, host64(Wukd), host64(Wuvd), idx, d_h, 10000.0)
    assert np.all(np.isfinite(out))
    assert orc.max_abs_rel(out, ref) <= TOL["bf16"], (n_h, r, d_c, B, lens, stride, n_splits)
    for b, n in enumerate(lens):
        if n == 0:
            assert np.all(out[b] == 0.0)


@pytest.mark.parametrize("seed", range(8))
def test_decode_sweep_separated_and_several_queries(seed):
    rng, n_h, r, d_c, B, lens, stride, n_splits = _case(100 + seed)
    if n_h == 40:
        n_h, d_c = 32, 1536                                   # separated latents at 40 heads take the generic kernels
    d_h = 128
    d_ck = int(rng.choice([d_c // 4, d_c // 2, 3 * d_c // 4]))
    T = int(rng.integers(1, 5))
    idx = synth.draw_elite_idx(rng, n_h, d_h, r)
    _, _, B_k, _ = synth.draw_weights(rng, 64, n_h, d_h, r, d_ck)
    _, _, _, B_v = synth.draw_weights(rng, 64, n_h, d_h, r, d_c - d_ck)
    ke64, c64 = synth.draw_cache_planes(rng, B * stride, n_h, r, d_c)
    q = rng.standard_normal((B, T, n_h, d_h))
    dims = ekv.make_dims(64, n_h, d_h, r, d_c, "bf16", 10000.0)
    ked, cd, qd, Bkd, Bvd = (dev(a, "bf16") for a in (ke64, c64, q, B_k, B_v))
    # query t of sequence b sees the rows up to its own position; the last query sees the whole sequence
    kv_len = np.array([[max(n - (T - 1 - t), 0) for t in range(T)] for n in lens])
    q_pos = np.maximum(kv_len - 1, 0)
    out = torch.full((B, T, n_h, d_h), float("nan"), dtype=torch.bfloat16, device=DEV)
    nws = ekv.elitekv_slrd_multiquery_workspace_bytes(dims, d_ck, B, T, max(lens), n_splits)
    assert nws > 0
    ws = torch.full((nws,), 0xFF, dtype=torch.uint8, device=DEV)
    ekv.elitekv_slrd_multiquery_attn(dims, d_ck, qd, i32(q_pos.reshape(-1)), i32(kv_len.reshape(-1)), max(lens), stride,
                                     Bkd, Bvd, i32(idx), ked, cd, out, ws, n_splits=n_splits)
    torch.cuda.synchronize()
    o = host64(out)
    c_h = host64(cd).reshape(B, stride, -1)
    ref = orc.slrd_multiquery_attn(host64(qd), q_pos, host64(ked).reshape(B, stride, n_h, -1), c_h[:, :, :d_ck],
                                   c_h[:, :, d_ck:], kv_len, host64(Bkd), host64(Bvd), idx, d_h, 10000.0)
    assert np.all(np.isfinite(o))
    assert orc.max_abs_rel(o, ref) <= TOL["bf16"], (n_h, r, d_c, d_ck, B, T, lens, stride, n_splits)
    assert np.all(o[kv_len == 0] == 0.0)
