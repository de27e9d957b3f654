"""GPU parity of the fused decode step (append of the step's tokens + attention in one call) against
the float64 oracle, through the C ABI.  The step must give what elitekv_append followed by
elitekv_decode_attn give: the appended cache rows are compared with the oracle's append, and the
attention output with the oracle's decode over the planes as they stand on the device after the step
(old rows + the new rows as stored).  Bounds: max-abs-rel <= 1e-5 (fp32), 2e-2 (bf16)."""
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

# name: (shape, cached tokens per sequence INCLUDING the new one)
STEP_CASES = {
    "bf16_7b_one_sequence": (shape(4096, 32, 128, 8, 1536, "bf16"), [301]),
    "bf16_7b_two_sequences": (shape(4096, 32, 128, 8, 1536, "bf16"), [17, 130]),
    "bf16_7b_three_sequences": (shape(4096, 32, 128, 8, 1536, "bf16"), [1, 64, 97]),
    "bf16_7b_five_sequences": (shape(4096, 32, 128, 8, 1536, "bf16"), [33, 1, 16, 250, 47]),
    "bf16_7b_seven_sequences": (shape(4096, 32, 128, 8, 1536, "bf16"), [5, 6, 7, 8, 100, 31, 32]),
    "bf16_7b_eight_sequences": (shape(4096, 32, 128, 8, 1536, "bf16"), [9, 40, 3, 77, 120, 16, 15, 64]),
    "bf16_7b_sixteen_sequences": (shape(4096, 32, 128, 8, 1536, "bf16"), list(range(20, 36))),
    "bf16_7b_12pct_forty_sequences": (shape(4096, 32, 128, 4, 768, "bf16"), [3 + (7 * i) % 90 for i in range(40)]),
    "bf16_7b_sixty_four_sequences": (shape(4096, 32, 128, 8, 1536, "bf16"), [1 + (11 * i) % 70 for i in range(64)]),
    "bf16_13b_sixteen_sequences": (shape(5120, 40, 128, 8, 1920, "bf16"), [10 + 5 * i for i in range(16)]),
    "bf16_13b_one_sequence": (shape(5120, 40, 128, 8, 1920, "bf16"), [200]),
    "bf16_13b_four_sequences": (shape(5120, 40, 128, 8, 1920, "bf16"), [18, 90, 1, 33]),
    "bf16_7b_12pct_two_sequences": (shape(4096, 32, 128, 4, 768, "bf16"), [70, 71]),
    "bf16_odd_hidden_one_sequence": (shape(1000, 32, 128, 8, 1536, "bf16"), [50]),
    "bf16_narrow_hidden_one_sequence": (shape(64, 32, 128, 8, 512, "bf16"), [40]),
    "bf16_small_heads_two_waves": (shape(512, 8, 64, 4, 128, "bf16"), [77, 16]),          # d_c = 128: two-wave attention
    "bf16_forty_heads_r4": (shape(1024, 40, 128, 4, 256, "bf16"), [40, 41, 1]),             # two head groups, 2r = 8
    "bf16_head_dim_64_five_sequences": (shape(768, 16, 64, 8, 512, "bf16"), [9, 100, 33, 64, 2]),
    "bf16_r16_one_sequence": (shape(4096, 32, 128, 16, 1792, "bf16"), [301]),                 # 2r = 32 elite values per head
    "bf16_r16_three_sequences": (shape(4096, 32, 128, 16, 1024, "bf16"), [1, 64, 97]),
    "bf16_r16_twelve_sequences": (shape(4096, 32, 128, 16, 1792, "bf16"), [7 + 13 * i for i in range(12)]),
    "bf16_r32_one_sequence": (shape(4096, 32, 128, 32, 1024, "bf16"), [301]),                 # 2r = 64 elite values per head
    "bf16_r32_twelve_sequences": (shape(4096, 32, 128, 32, 1152, "bf16"), [7 + 13 * i for i in range(12)]),
    "fp32_tiny_three_sequences": (synth.CONFIGS["tiny_fp32"].as_dict(), [129, 5, 60]),
}


def _planes(rng, B, stride, n_h, r, d_c, dt):
    ke64, c64 = synth.draw_cache_planes(rng, B * stride, n_h, r, d_c)
    return dev(ke64, dt), dev(c64, dt)


@pytest.mark.parametrize("name", list(STEP_CASES))
def test_step_matches_oracle(name):
    sh, seqs = STEP_CASES[name]
    dt, n_h, d_h = sh["dtype"], sh["n_heads"], sh["head_dim"]
    B, stride = len(seqs), max(seqs) + 2
    rng, idx, W_ke, W_dkv, W_uk, W_uv, x, q = _draw(sh, B, B, 300 + len(name))
    dims = dims_of(sh)
    ke, c = _planes(rng, B, stride, n_h, sh["r"], sh["d_c"], dt)
    ke0, c0 = ke.clone(), c.clone()
    pos = np.array(seqs) - 1
    slot = np.arange(B) * stride + pos
    xd, qd, Wked, Wdkvd, Wukd, Wuvd = (dev(a, dt) for a in (x, q, W_ke, W_dkv, W_uk, W_uv))
    out = torch.full((B, n_h, d_h), float("nan"), dtype=ekv.torch_dtype(dims), device=DEV)
    nws = ekv.elitekv_decode_step_workspace_bytes(dims, B, max(seqs))
    assert nws > 0
    ws = torch.full((nws,), 0xFF, dtype=torch.uint8, device=DEV)     # nothing may depend on old contents
    ekv.elitekv_decode_step(dims, xd, qd, i32(pos), i64(slot), i32(seqs), max(seqs), stride, Wked, Wdkvd, Wukd, Wuvd,
                            i32(idx), ke, c, out, ws)
    torch.cuda.synchronize()
    # (1) the appended rows
    ke_ref, c_ref = orc.append(host64(xd), pos, host64(Wked), host64(Wdkvd), idx, d_h, sh["rope_base"])
    ke_g, c_g = host64(ke).reshape(B * stride, n_h, -1), host64(c)
    assert orc.max_abs_rel(c_g[slot], c_ref) <= TOL[dt]
    if sh["r"]:
        assert orc.max_abs_rel(ke_g[slot], ke_ref) <= TOL[dt]
    # (2) every other row is as it was
    other = np.setdiff1d(np.arange(B * stride), slot)
    assert np.array_equal(c_g[other], host64(c0)[other])
    assert np.array_equal(ke_g[other], host64(ke0).reshape(B * stride, n_h, -1)[other])
    # (3) the attention output over the planes as they now stand
    ref = orc.decode_attn(host64(qd), pos, ke_g.reshape(B, stride, n_h, -1), c_g.reshape(B, stride, -1), seqs,
                          host64(Wukd), host64(Wuvd), idx, d_h, sh["rope_base"])
    o = host64(out)
    assert np.all(np.isfinite(o))
    assert orc.max_abs_rel(o, ref) <= TOL[dt]


def test_step_agrees_with_the_two_calls_and_skips_out_of_range_slots():
    sh, seqs = shape(4096, 32, 128, 8, 1536, "bf16"), [90, 41, 64]
    B, stride = 3, 100
    rng, idx, W_ke, W_dkv, W_uk, W_uv, x, q = _draw(sh, B, B, 77)
    dims = dims_of(sh)
    ke, c = _planes(rng, B, stride, 32, 8, 1536, "bf16")
    ke2, c2, c_before = ke.clone(), c.clone(), c.clone()
    pos = np.array(seqs) - 1
    slot = np.arange(B) * stride + pos
    slot[1] = -1                                         # this token is not stored (its attention output is unspecified)
    xd, qd, Wked, Wdkvd, Wukd, Wuvd = (dev(a, "bf16") for a in (x, q, W_ke, W_dkv, W_uk, W_uv))
    out = torch.zeros(B, 32, 128, dtype=torch.bfloat16, device=DEV)
    out2 = torch.zeros_like(out)
    ws = torch.empty(ekv.elitekv_decode_step_workspace_bytes(dims, B, max(seqs)), dtype=torch.uint8, device=DEV)
    ekv.elitekv_decode_step(dims, xd, qd, i32(pos), i64(slot), i32(seqs), max(seqs), stride, Wked, Wdkvd, Wukd, Wuvd,
                            i32(idx), ke, c, out, ws)
    slot2 = slot
    aws = torch.empty(max(ekv.elitekv_append_workspace_bytes(dims, B), 16), dtype=torch.uint8, device=DEV)
    ekv.elitekv_append(dims, xd, i32(pos), i64(slot2), Wked, Wdkvd, i32(idx), ke2, c2, ws=aws)
    dws = torch.empty(ekv.elitekv_decode_workspace_bytes(dims, B, max(seqs)), dtype=torch.uint8, device=DEV)
    ekv.elitekv_decode_attn(dims, qd, i32(pos), i32(seqs), max(seqs), stride, Wukd, Wuvd, i32(idx), ke2, c2, out2, dws)
    torch.cuda.synchronize()
    assert orc.max_abs_rel(host64(out)[[0, 2]], host64(out2)[[0, 2]]) <= TOL["bf16"]
    stored = [int(slot[0]), int(slot[2])]
    assert orc.max_abs_rel(host64(c)[stored], host64(c2)[stored]) <= 2.0 ** -8    # one bf16 rounding of differently ordered sums
    assert orc.max_abs_rel(host64(ke)[stored], host64(ke2)[stored]) <= 2.0 ** -8
    row = stride + pos[1]                                # the row of the token that was not stored is untouched
    assert torch.equal(c[row], c_before[row])


@pytest.mark.parametrize("B", [2, 9])
def test_step_with_a_sequence_that_attends_to_nothing(B):
    """seq_len = 0 for the first sequence: its output row is zero, its token is stored all the same."""
    sh = shape(4096, 32, 128, 8, 1536, "bf16")
    seqs = [0] + [20 + 3 * i for i in range(B - 1)]
    stride = 64
    rng, idx, W_ke, W_dkv, W_uk, W_uv, x, q = _draw(sh, B, B, 5 + B)
    dims = dims_of(sh)
    ke, c = _planes(rng, B, stride, 32, 8, 1536, "bf16")
    pos = np.maximum(np.array(seqs) - 1, 0)
    slot = np.arange(B) * stride + pos
    slot[0] = 7                                          # in range, although sequence 0 attends to nothing
    xd, qd, Wked, Wdkvd, Wukd, Wuvd = (dev(a, "bf16") for a in (x, q, W_ke, W_dkv, W_uk, W_uv))
    out = torch.full((B, 32, 128), float("nan"), dtype=torch.bfloat16, device=DEV)
    ws = torch.full((ekv.elitekv_decode_step_workspace_bytes(dims, B, max(seqs)),), 0xFF, dtype=torch.uint8, device=DEV)
    ekv.elitekv_decode_step(dims, xd, qd, i32(pos), i64(slot), i32(seqs), max(seqs), stride, Wked, Wdkvd, Wukd, Wuvd,
                            i32(idx), ke, c, out, ws)
    torch.cuda.synchronize()
    o = host64(out)
    assert np.all(o[0] == 0.0) and np.all(np.isfinite(o))
    ke_ref, c_ref = orc.append(host64(xd), pos, host64(Wked), host64(Wdkvd), idx, 128, sh["rope_base"])
    assert orc.max_abs_rel(host64(c)[slot], c_ref) <= TOL["bf16"]
    assert orc.max_abs_rel(host64(ke).reshape(B * stride, 32, -1)[slot], ke_ref) <= TOL["bf16"]
    ke_g, c_g = host64(ke).reshape(B, stride, 32, -1), host64(c).reshape(B, stride, -1)
    ref = orc.decode_attn(host64(qd)[1:], pos[1:], ke_g[1:], c_g[1:], seqs[1:], host64(Wukd), host64(Wuvd), idx, 128,
                          sh["rope_base"])
    assert orc.max_abs_rel(o[1:], ref) <= TOL["bf16"]


# (shape, cached tokens per sequence including the new one, sequence splits): splits of several tiles, so the owner
# work-group of a new row stores it while its earlier tiles stream and requests the row's tile last
LONG_SPLIT_CASES = {
    "bf16_7b_one_sequence_two_splits": (shape(4096, 32, 128, 8, 1536, "bf16"), [301], 2),
    "bf16_7b_one_sequence_one_split": (shape(4096, 32, 128, 8, 1536, "bf16"), [130], 1),
    "bf16_7b_three_tiles_exactly": (shape(4096, 32, 128, 8, 1536, "bf16"), [48], 1),
    "bf16_7b_three_sequences_three_splits": (shape(4096, 32, 128, 8, 1536, "bf16"), [100, 250, 49], 3),
    "bf16_7b_nine_sequences_two_splits": (shape(4096, 32, 128, 8, 1536, "bf16"), [300, 17, 64, 129, 255, 33, 97, 48, 200], 2),
    "bf16_7b_12pct_sixteen_sequences": (shape(4096, 32, 128, 4, 768, "bf16"), [40 + 13 * i for i in range(16)], 2),
    "bf16_13b_one_sequence_two_splits": (shape(5120, 40, 128, 8, 1920, "bf16"), [200], 2),
    "bf16_13b_eight_sequences_one_split": (shape(5120, 40, 128, 8, 1920, "bf16"), [50 + 21 * i for i in range(8)], 1),
}


@pytest.mark.parametrize("name", list(LONG_SPLIT_CASES))
def test_step_reads_back_the_rows_it_stores_in_long_splits(name):
    """The slots of the new rows hold NaN before the step: an attention tile that was requested before the step's
    own row had reached it would carry the NaN into the output."""
    sh, seqs, n_splits = LONG_SPLIT_CASES[name]
    dt, n_h, d_h = sh["dtype"], sh["n_heads"], sh["head_dim"]
    B, stride = len(seqs), max(seqs) + 2
    rng, idx, W_ke, W_dkv, W_uk, W_uv, x, q = _draw(sh, B, B, 900 + len(name))
    dims = dims_of(sh)
    ke, c = _planes(rng, B, stride, n_h, sh["r"], sh["d_c"], dt)
    pos = np.array(seqs) - 1
    slot = np.arange(B) * stride + pos
    ke[i64(slot)] = float("nan")
    c[i64(slot)] = float("nan")
    xd, qd, Wked, Wdkvd, Wukd, Wuvd = (dev(a, dt) for a in (x, q, W_ke, W_dkv, W_uk, W_uv))
    out = torch.full((B, n_h, d_h), float("nan"), dtype=ekv.torch_dtype(dims), device=DEV)
    ws = torch.full((ekv.elitekv_decode_step_workspace_bytes(dims, B, max(seqs), n_splits),), 0xFF, dtype=torch.uint8,
                    device=DEV)
    for rep in range(3):                                  # the second and third step find warm caches: other timing
        if rep:
            ke[i64(slot)] = float("nan")
            c[i64(slot)] = float("nan")
        ekv.elitekv_decode_step(dims, xd, qd, i32(pos), i64(slot), i32(seqs), max(seqs), stride, Wked, Wdkvd, Wukd, Wuvd,
                                i32(idx), ke, c, out, ws, n_splits=n_splits)
        torch.cuda.synchronize()
        ke_g, c_g = host64(ke).reshape(B * stride, n_h, -1), host64(c)
        ke_ref, c_ref = orc.append(host64(xd), pos, host64(Wked), host64(Wdkvd), idx, d_h, sh["rope_base"])
        assert orc.max_abs_rel(c_g[slot], c_ref) <= TOL[dt]
        assert orc.max_abs_rel(ke_g[slot], ke_ref) <= TOL[dt]
        ref = orc.decode_attn(host64(qd), pos, ke_g.reshape(B, stride, n_h, -1), c_g.reshape(B, stride, -1), seqs,
                              host64(Wukd), host64(Wuvd), idx, d_h, sh["rope_base"])
        o = host64(out)
        assert np.all(np.isfinite(o)), "step %d: NaN from a new row's slot reached the output" % rep
        assert orc.max_abs_rel(o, ref) <= TOL[dt]


def test_step_argument_errors():
    sh = shape(4096, 32, 128, 8, 1536, "bf16")
    dims = dims_of(sh)
    B, S = 1, 64
    z = lambda *s: torch.zeros(*s, dtype=torch.bfloat16, device=DEV)
    x, q, W_ke, W_dkv, W_uk, W_uv = z(1, 4096), z(1, 32, 128), z(4096, 512), z(4096, 1536), z(1536, 32, 112), z(1536, 32, 128)
    ke, c, out = z(S, 32, 16), z(S, 1536), z(1, 32, 128)
    idx = i32(np.tile(np.arange(8), (32, 1)))
    need = ekv.elitekv_decode_step_workspace_bytes(dims, B, S)
    small = torch.empty(need - 256, dtype=torch.uint8, device=DEV)
    with pytest.raises(ekv.EliteKVError, match="workspace"):
        ekv.elitekv_decode_step(dims, x, q, i32([S - 1]), i64([S - 1]), i32([S]), S, S, W_ke, W_dkv, W_uk, W_uv, idx,
                                ke, c, out, small)
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    with pytest.raises(ekv.EliteKVError, match="NULL"):
        ekv.elitekv_decode_step(dims, None, q, i32([S - 1]), i64([S - 1]), i32([S]), S, S, W_ke, W_dkv, W_uk, W_uv,
                                idx, ke, c, out, ws)


SLRD_STEP_CASES = {
    "bf16_7b_one_sequence": (slrd_shape(4096, 32, 128, 8, 576, 960, "bf16"), [260]),
    "bf16_7b_four_sequences": (slrd_shape(4096, 32, 128, 8, 576, 960, "bf16"), [31, 100, 2, 65]),
    "bf16_7b_even_split_eight_sequences": (slrd_shape(4096, 32, 128, 8, 768, 768, "bf16"), [30, 31, 32, 33, 1, 90, 16, 48]),
    "fp32_tiny_two_sequences": (slrd_shape(96, 3, 16, 2, 24, 40, "fp32"), [20, 7]),
}


@pytest.mark.parametrize("name", list(SLRD_STEP_CASES))
def test_slrd_step_matches_oracle(name):
    sh, seqs = SLRD_STEP_CASES[name]
    dt, n_h, d_h, d_ck = sh["dtype"], sh["n_heads"], sh["head_dim"], sh["d_ck"]
    B, stride = len(seqs), max(seqs) + 2
    rng, idx, W_ke, A_k, A_v, B_k, B_v, x, q = _draw_slrd(sh, B, B, 400 + len(name))
    dims = dims_of(sh)
    ke, c = _planes(rng, B, stride, n_h, sh["r"], sh["d_c"], dt)
    pos = np.array(seqs) - 1
    slot = np.arange(B) * stride + pos
    xd, qd, Wked, Akd, Avd, Bkd, Bvd = (dev(a, dt) for a in (x, q, W_ke, A_k, A_v, B_k, B_v))
    out = torch.full((B, n_h, d_h), float("nan"), dtype=ekv.torch_dtype(dims), device=DEV)
    nws = ekv.elitekv_slrd_decode_step_workspace_bytes(dims, d_ck, B, max(seqs))
    assert nws > 0
    ws = torch.full((nws,), 0xFF, dtype=torch.uint8, device=DEV)
    ekv.elitekv_slrd_decode_step(dims, d_ck, xd, qd, i32(pos), i64(slot), i32(seqs), max(seqs), stride, Wked, Akd,
                                 Avd, Bkd, Bvd, i32(idx), ke, c, out, ws)
    torch.cuda.synchronize()
    ke_ref, ck_ref, cv_ref = orc.slrd_append(host64(xd), pos, host64(Wked), host64(Akd), host64(Avd), idx, d_h,
                                             sh["rope_base"])
    ke_g, c_g = host64(ke).reshape(B * stride, n_h, -1), host64(c)
    assert orc.max_abs_rel(c_g[slot][:, :d_ck], ck_ref) <= TOL[dt]
    assert orc.max_abs_rel(c_g[slot][:, d_ck:], cv_ref) <= TOL[dt]
    if sh["r"]:
        assert orc.max_abs_rel(ke_g[slot], ke_ref) <= TOL[dt]
    cb = c_g.reshape(B, stride, -1)
    ref = orc.slrd_decode_attn(host64(qd), pos, ke_g.reshape(B, stride, n_h, -1), cb[:, :, :d_ck], cb[:, :, d_ck:],
                               seqs, host64(Bkd), host64(Bvd), idx, d_h, sh["rope_base"])
    o = host64(out)
    assert np.all(np.isfinite(o))
    assert orc.max_abs_rel(o, ref) <= TOL[dt]
