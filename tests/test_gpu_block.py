"""GPU parity of the whole-block decode step (q = x W^q, append, attention over the compressed cache,
W^o; one call) against the float64 oracle `attention_block_step`, through the C ABI.  Inputs are
rounded once to bf16 and go to both sides; the GPU additionally rounds the query and the attention
output to bf16 as a model would hold them.  Bound: max-abs-rel <= 2e-2 (bf16)."""
import numpy as np
import pytest
import torch

import elitekv_synth as synth
import paper_2503_01586_amd as ekv
from oracle import elitekv_oracle as orc

from gpu_util import DEV, TOL, dev, dims_of, host64, i32, i64
from test_gpu_parity import _draw, shape
from test_gpu_slrd import _draw as _draw_slrd, shape as slrd_shape

pytestmark = pytest.mark.gpu

BLOCK_CASES = {
    "bf16_7b_one_sequence": (shape(4096, 32, 128, 8, 1536, "bf16"), [120]),
    "bf16_7b_three_sequences": (shape(4096, 32, 128, 8, 1536, "bf16"), [1, 64, 33]),
    "bf16_7b_seven_sequences": (shape(4096, 32, 128, 8, 1536, "bf16"), [5, 17, 16, 48, 2, 31, 90]),
    "bf16_13b_two_sequences": (shape(5120, 40, 128, 8, 1920, "bf16"), [70, 9]),
    "bf16_7b_12pct_one_sequence": (shape(4096, 32, 128, 4, 768, "bf16"), [55]),
    "bf16_small_hidden_head_dim_64": (shape(768, 16, 64, 8, 512, "bf16"), [40, 3]),
    # eight sequences and more: the composed form (projections around the decode step's kernels)
    "bf16_7b_eight_sequences": (shape(4096, 32, 128, 8, 1536, "bf16"), [9, 40, 3, 77, 120, 16, 15, 64]),
    "bf16_13b_sixteen_sequences": (shape(5120, 40, 128, 8, 1920, "bf16"), [10 + 5 * i for i in range(16)]),
    "bf16_7b_12pct_forty_sequences": (shape(4096, 32, 128, 4, 768, "bf16"), [3 + (7 * i) % 90 for i in range(40)]),
    "bf16_7b_sixty_four_sequences": (shape(4096, 32, 128, 8, 1536, "bf16"), [1 + (11 * i) % 70 for i in range(64)]),
    "bf16_generic_latent_width_two_sequences": (shape(1024, 8, 64, 4, 320, "bf16"), [33, 50]),   # generic decode kernels
}


@pytest.mark.parametrize("name", list(BLOCK_CASES))
def test_block_step_matches_oracle(name):
    sh, seqs = BLOCK_CASES[name]
    n_h, d_h, d, r, d_c = sh["n_heads"], sh["head_dim"], sh["d_model"], sh["r"], sh["d_c"]
    B, stride = len(seqs), max(seqs) + 2
    rng, idx, W_ke, W_dkv, W_uk, W_uv, x, _ = _draw(sh, B, B, 600 + len(name))
    W_q = rng.standard_normal((d, n_h, d_h)) / np.sqrt(d)
    W_o = rng.standard_normal((n_h, d_h, d)) / np.sqrt(n_h * d_h)
    dims = dims_of(sh)
    ke64, c64 = synth.draw_cache_planes(rng, B * stride, n_h, r, d_c)
    ke, c = dev(ke64, "bf16"), dev(c64, "bf16")
    ke_before, c_before = host64(ke).reshape(B, stride, n_h, -1), host64(c).reshape(B, stride, -1)
    pos = np.array(seqs) - 1
    slot = np.arange(B) * stride + pos
    xd, Wqd, Wked, Wdkvd, Wukd, Wuvd, Wod = (dev(a, "bf16") for a in (x, W_q, W_ke, W_dkv, W_uk, W_uv, W_o))
    y = torch.full((B, d), float("nan"), dtype=torch.bfloat16, device=DEV)
    nws = ekv.elitekv_block_step_workspace_bytes(dims, B, max(seqs))
    assert nws > 0
    ws = torch.full((nws,), 0xFF, dtype=torch.uint8, device=DEV)     # nothing may depend on old contents
    ekv.elitekv_block_step(dims, xd, i32(pos), i64(slot), i32(seqs), max(seqs), stride, Wqd, Wked, Wdkvd, Wukd, Wuvd,
                           Wod, i32(idx), ke, c, y, ws)
    torch.cuda.synchronize()
    y_ref, ke_ref, c_ref = orc.attention_block_step(
        host64(xd), pos, [ke_before[b, :seqs[b] - 1] for b in range(B)], [c_before[b, :seqs[b] - 1] for b in range(B)],
        host64(Wqd), host64(Wked), host64(Wdkvd), host64(Wukd), host64(Wuvd), host64(Wod), idx, d_h, sh["rope_base"])
    yg = host64(y)
    assert np.all(np.isfinite(yg))
    assert orc.max_abs_rel(yg, y_ref) <= TOL["bf16"]
    # the appended rows, and nothing else, changed
    ke_g, c_g = host64(ke).reshape(B * stride, n_h, -1), host64(c)
    assert orc.max_abs_rel(c_g[slot], c_ref) <= TOL["bf16"]
    assert orc.max_abs_rel(ke_g[slot], ke_ref) <= TOL["bf16"]
    other = np.setdiff1d(np.arange(B * stride), slot)
    assert np.array_equal(c_g[other], c_before.reshape(B * stride, -1)[other])


def test_block_step_equals_projections_around_the_decode_step():
    """y of the block = (decode step fed with bf16(x W_q)) W_o, both computed on the GPU."""
    sh, seqs = shape(4096, 32, 128, 8, 1536, "bf16"), [77, 20]
    B, stride, d, n_h, d_h = 2, 80, 4096, 32, 128
    rng, idx, W_ke, W_dkv, W_uk, W_uv, x, _ = _draw(sh, B, B, 91)
    W_q = rng.standard_normal((d, n_h, d_h)) / np.sqrt(d)
    W_o = rng.standard_normal((n_h, d_h, d)) / np.sqrt(n_h * d_h)
    dims = dims_of(sh)
    ke64, c64 = synth.draw_cache_planes(rng, B * stride, n_h, 8, 1536)
    ke, c = dev(ke64, "bf16"), dev(c64, "bf16")
    ke2, c2 = ke.clone(), c.clone()
    pos = np.array(seqs) - 1
    slot = np.arange(B) * stride + pos
    xd, Wqd, Wked, Wdkvd, Wukd, Wuvd, Wod = (dev(a, "bf16") for a in (x, W_q, W_ke, W_dkv, W_uk, W_uv, W_o))
    y = torch.zeros(B, d, dtype=torch.bfloat16, device=DEV)
    ws = torch.empty(ekv.elitekv_block_step_workspace_bytes(dims, B, max(seqs)), dtype=torch.uint8, device=DEV)
    ekv.elitekv_block_step(dims, xd, i32(pos), i64(slot), i32(seqs), max(seqs), stride, Wqd, Wked, Wdkvd, Wukd, Wuvd,
                           Wod, i32(idx), ke, c, y, ws)
    q = (xd.float() @ Wqd.float().reshape(d, n_h * d_h)).to(torch.bfloat16).reshape(B, n_h, d_h).contiguous()
    out = torch.zeros(B, n_h, d_h, dtype=torch.bfloat16, device=DEV)
    sws = torch.empty(ekv.elitekv_decode_step_workspace_bytes(dims, B, max(seqs)), dtype=torch.uint8, device=DEV)
    ekv.elitekv_decode_step(dims, xd, q, i32(pos), i64(slot), i32(seqs), max(seqs), stride, Wked, Wdkvd, Wukd, Wuvd,
                            i32(idx), ke2, c2, out, sws)
    y2 = out.float().reshape(B, n_h * d_h) @ Wod.float().reshape(n_h * d_h, d)
    torch.cuda.synchronize()
    assert orc.max_abs_rel(host64(y), host64(y2)) <= 1e-2
    assert torch.equal(c, c2) and torch.equal(ke, ke2)      # the same append arithmetic: identical rows


def test_block_step_argument_errors():
    big = ekv.make_dims(4096, 32, 128, 8, 1536, "bf16")
    assert ekv.elitekv_block_step_workspace_bytes(big, 1, 4096) > ekv.elitekv_decode_step_workspace_bytes(big, 1, 4096)
    assert ekv.elitekv_block_step_workspace_bytes(big, 8, 4096) > 0            # eight sequences: the composed form
    assert ekv.elitekv_block_step_workspace_bytes(big, 65, 4096) == 0          # more than 64 sequences: not covered
    tiny = ekv.make_dims(128, 4, 32, 2, 64, "fp32")
    assert ekv.elitekv_block_step_workspace_bytes(tiny, 1, 128) == 0           # fp32: not covered


SLRD_BLOCK_CASES = {
    "bf16_7b_one_sequence": (slrd_shape(4096, 32, 128, 8, 576, 960, "bf16"), [260]),
    "bf16_7b_four_sequences": (slrd_shape(4096, 32, 128, 8, 576, 960, "bf16"), [31, 100, 2, 65]),
    "bf16_7b_even_split_twelve_sequences": (slrd_shape(4096, 32, 128, 8, 768, 768, "bf16"), [7 + 9 * i for i in range(12)]),
}


@pytest.mark.parametrize("name", list(SLRD_BLOCK_CASES))
def test_slrd_block_step_matches_oracle(name):
    """elitekv_slrd_block_step against the oracle's slrd_attention_block_step (Section 2.1 projections around
    Section 3.2's separated decomposition), one to twelve sequences."""
    sh, seqs = SLRD_BLOCK_CASES[name]
    n_h, d_h, d, r, d_c, d_ck = sh["n_heads"], sh["head_dim"], sh["d_model"], sh["r"], sh["d_c"], sh["d_ck"]
    B, stride = len(seqs), max(seqs) + 2
    rng, idx, W_ke, A_k, A_v, B_k, B_v, x, _ = _draw_slrd(sh, B, B, 700 + len(name))
    W_q = rng.standard_normal((d, n_h, d_h)) / np.sqrt(d)
    W_o = rng.standard_normal((n_h, d_h, d)) / np.sqrt(n_h * d_h)
    dims = dims_of(sh)
    ke64, c64 = synth.draw_cache_planes(rng, B * stride, n_h, r, d_c)
    ke, c = dev(ke64, "bf16"), dev(c64, "bf16")
    ke_before, c_before = host64(ke).reshape(B, stride, n_h, -1), host64(c).reshape(B, stride, -1)
    pos = np.array(seqs) - 1
    slot = np.arange(B) * stride + pos
    xd, Wqd, Wked, Akd, Avd, Bkd, Bvd, Wod = (dev(a, "bf16") for a in (x, W_q, W_ke, A_k, A_v, B_k, B_v, W_o))
    y = torch.full((B, d), float("nan"), dtype=torch.bfloat16, device=DEV)
    nws = ekv.elitekv_slrd_block_step_workspace_bytes(dims, d_ck, B, max(seqs))
    assert nws > 0
    ws = torch.full((nws,), 0xFF, dtype=torch.uint8, device=DEV)
    ekv.elitekv_slrd_block_step(dims, d_ck, xd, i32(pos), i64(slot), i32(seqs), max(seqs), stride, Wqd, Wked, Akd, Avd,
                                Bkd, Bvd, Wod, i32(idx), ke, c, y, ws)
    torch.cuda.synchronize()
    old = lambda a, lo, hi: [a[b, :seqs[b] - 1, ..., lo:hi] if a.ndim == 3 else a[b, :seqs[b] - 1] for b in range(B)]
    y_ref, ke_ref, ck_ref, cv_ref = orc.slrd_attention_block_step(
        host64(xd), pos, old(ke_before, 0, None), old(c_before, 0, d_ck), old(c_before, d_ck, None), host64(Wqd),
        host64(Wked), host64(Akd), host64(Avd), host64(Bkd), host64(Bvd), host64(Wod), idx, d_h, sh["rope_base"])
    yg = host64(y)
    assert np.all(np.isfinite(yg))
    assert orc.max_abs_rel(yg, y_ref) <= TOL["bf16"]
    ke_g, c_g = host64(ke).reshape(B * stride, n_h, -1), host64(c)
    assert orc.max_abs_rel(c_g[slot][:, :d_ck], ck_ref) <= TOL["bf16"]
    assert orc.max_abs_rel(c_g[slot][:, d_ck:], cv_ref) <= TOL["bf16"]
    assert orc.max_abs_rel(ke_g[slot], ke_ref) <= TOL["bf16"]
    other = np.setdiff1d(np.arange(B * stride), slot)
    assert np.array_equal(c_g[other], c_before.reshape(B * stride, -1)[other])
