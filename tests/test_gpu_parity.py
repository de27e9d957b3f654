"""GPU parity: the HIP path, called through the C ABI, against the float64 CPU oracle, element by
element on the same seeded inputs.  Bounds: max|gpu - ref| / max|ref| <= 1e-5 (fp32) or 2e-2 (bf16).
"""
import numpy as np
import pytest
import torch

import elitekv_synth as synth
import paper_2503_01586_amd as ekv
from oracle import elitekv_oracle as orc

from gpu_util import DEV, TOL, dev, dims_of, gpu_append, gpu_decode, host64, i32, i64

pytestmark = pytest.mark.gpu


def shape(d_model, n_heads, head_dim, r, d_c, dtype, rope_base=10000.0):
    return dict(d_model=d_model, n_heads=n_heads, head_dim=head_dim, r=r, d_c=d_c, dtype=dtype,
                rope_base=rope_base)


TINY = synth.CONFIGS["tiny_fp32"].as_dict()

APPEND_CASES = {
    # name: (shape, T, max position)
    "tiny_fp32": (TINY, 129, 128),
    "fp32_ragged_dims": (shape(200, 3, 24, 5, 37, "fp32"), 37, 5000),
    "fp32_no_elite": (shape(96, 2, 16, 0, 40, "fp32"), 9, 10),
    "fp32_all_elite": (shape(64, 2, 16, 8, 24, "fp32"), 21, 300),
    "bf16_7b_rows": (shape(4096, 32, 128, 8, 1536, "bf16"), 70, 32767),
    "bf16_7b_12pct": (shape(4096, 32, 128, 4, 768, "bf16"), 33, 2047),
    "bf16_13b_rows": (shape(5120, 40, 128, 8, 1920, "bf16"), 19, 8191),
    "bf16_one_token": (shape(512, 8, 64, 4, 128, "bf16"), 1, 77),
    "bf16_7b_decode_step": (shape(4096, 32, 128, 8, 1536, "bf16"), 8, 32767),
    "bf16_7b_64_tokens": (shape(4096, 32, 128, 8, 1536, "bf16"), 64, 4095),
    "bf16_odd_hidden": (shape(1000, 32, 128, 8, 1536, "bf16"), 5, 100),
    "bf16_odd_hidden_batch": (shape(1000, 32, 128, 8, 1536, "bf16"), 24, 100),
    "bf16_13b_batch_16": (shape(5120, 40, 128, 8, 1920, "bf16"), 16, 8191),
    "bf16_7b_12pct_batch_64": (shape(4096, 32, 128, 4, 768, "bf16"), 64, 2047),
    "bf16_7b_batch_40": (shape(4096, 32, 128, 8, 1536, "bf16"), 40, 4095),
    "bf16_7b_300_tokens": (shape(4096, 32, 128, 8, 1536, "bf16"), 300, 32767),
    "bf16_13b_200_tokens": (shape(5120, 40, 128, 8, 1920, "bf16"), 200, 8191),
    "bf16_12pct_odd_hidden_130": (shape(1000, 32, 128, 4, 768, "bf16"), 130, 2047),
    "bf16_half_block_boundary_200": (shape(1024, 24, 64, 4, 320, "bf16"), 200, 999),   # 2 r n_h = 192
    "bf16_7b_2100_tokens": (shape(4096, 32, 128, 8, 1536, "bf16"), 2100, 32767),   # about one 128 x 128 tile per compute unit
    "bf16_r16_one_token": (shape(4096, 32, 128, 16, 1792, "bf16"), 1, 32767),
    "bf16_r16_batch_16": (shape(4096, 32, 128, 16, 1792, "bf16"), 16, 4095),
    "bf16_r16_300_tokens": (shape(4096, 32, 128, 16, 1792, "bf16"), 300, 8191),
    "bf16_r32_one_token": (shape(4096, 32, 128, 32, 1024, "bf16"), 1, 32767),
    "bf16_r32_batch_16": (shape(4096, 32, 128, 32, 1152, "bf16"), 16, 4095),
    "bf16_r32_300_tokens": (shape(4096, 32, 128, 32, 1024, "bf16"), 300, 8191),
}


def _draw(sh, T, B, seed):
    rng = np.random.default_rng(seed)
    idx = (synth.draw_elite_idx(rng, sh["n_heads"], sh["head_dim"], sh["r"]) if sh["r"]
           else np.zeros((sh["n_heads"], 0), dtype=np.int32))
    W_ke, W_dkv, W_uk, W_uv = synth.draw_weights(rng, sh["d_model"], sh["n_heads"], sh["head_dim"], sh["r"],
                                                 sh["d_c"])
    x = synth.draw_hidden(rng, T, sh["d_model"])
    q = synth.draw_query(rng, B, sh["n_heads"], sh["head_dim"])
    return rng, idx, W_ke, W_dkv, W_uk, W_uv, x, q


@pytest.mark.parametrize("name", list(APPEND_CASES))
def test_append_matches_oracle(name):
    sh, T, max_pos = APPEND_CASES[name]
    dt = sh["dtype"]
    rng, idx, W_ke, W_dkv, _, _, x, _ = _draw(sh, T, 1, 100 + len(name))
    dims = dims_of(sh)
    pos = rng.integers(0, max_pos + 1, size=T)
    pos[0] = max_pos
    rows = T + 5
    slot = rng.permutation(rows)[:T]                      # scattered destination rows
    xd, Wked, Wdkvd = dev(x, dt), dev(W_ke, dt), dev(W_dkv, dt)
    ke, c = gpu_append(dims, xd, i32(pos), i64(slot), Wked, Wdkvd, i32(idx), rows)
    ke_ref, c_ref = orc.append(host64(xd), pos, host64(Wked), host64(Wdkvd), idx, sh["head_dim"],
                               sh["rope_base"])
    ke_g, c_g = host64(ke), host64(c)
    assert orc.max_abs_rel(c_g[slot], c_ref) <= TOL[dt]
    if sh["r"]:
        assert orc.max_abs_rel(ke_g[slot], ke_ref) <= TOL[dt]
    untouched = np.setdiff1d(np.arange(rows), slot)
    assert np.all(c_g[untouched] == 0.0) and np.all(ke_g[untouched] == 0.0)


def test_append_out_of_range_slots_are_skipped_and_rows_overwritten():
    sh = TINY
    rng, idx, W_ke, W_dkv, _, _, x, _ = _draw(sh, 6, 1, 7)
    dims = dims_of(sh)
    xd, Wked, Wdkvd = dev(x, "fp32"), dev(W_ke, "fp32"), dev(W_dkv, "fp32")
    slot = np.array([0, -1, 9, 2, 4, 3])                 # plane has 4 rows: -1, 9 and 4 are no-ops
    pos = np.arange(6)
    ke0 = torch.full((4, sh["n_heads"], 2 * sh["r"]), 7.0, dtype=torch.float32, device=DEV)
    c0 = torch.full((4, sh["d_c"]), 7.0, dtype=torch.float32, device=DEV)
    ke, c = gpu_append(dims, xd, i32(pos), i64(slot), Wked, Wdkvd, i32(idx), 4, ke=ke0, c=c0)
    ke_ref, c_ref = orc.append(host64(xd), pos, host64(Wked), host64(Wdkvd), idx, sh["head_dim"], 10000.0)
    c_g = host64(c)
    for t, s in enumerate(slot):
        if 0 <= s < 4:
            assert orc.max_abs_rel(c_g[s], c_ref[t]) <= 1e-5
            assert orc.max_abs_rel(host64(ke)[s], ke_ref[t]) <= 1e-5
    assert np.all(c_g[1] == 7.0)                          # row 1 was never a destination


DECODE_CASES = {
    # name: (shape, seq_len per batch row, splits to try)
    "tiny_fp32": (TINY, [129], [0, 1, 2, 5]),
    "fp32_ragged_batch": (shape(64, 3, 24, 5, 37, "fp32"), [0, 1, 63, 64, 65, 200], [0, 1, 3]),
    "fp32_no_elite": (shape(32, 2, 16, 0, 40, "fp32"), [50, 7], [0, 2]),
    "fp32_all_elite": (shape(32, 2, 16, 8, 24, "fp32"), [33], [0, 2]),
    "fp32_wide_latent": (shape(32, 2, 32, 3, 700, "fp32"), [150], [0, 4]),
    "bf16_7b": (shape(64, 32, 128, 8, 1536, "bf16"), [300, 1, 257], [0, 1, 4]),
    "bf16_7b_12pct": (shape(64, 32, 128, 4, 768, "bf16"), [130, 64], [0, 3]),
    "bf16_13b": (shape(64, 40, 128, 8, 1920, "bf16"), [97, 160], [0, 2]),
    "bf16_13b_ragged_batch": (shape(64, 40, 128, 8, 1920, "bf16"), [0, 1, 15, 16, 17, 250, 33, 48, 100], [0, 3, 5]),
    "bf16_13b_r4": (shape(64, 40, 128, 4, 1920, "bf16"), [130, 31], [0, 2]),
    "bf16_small_heads": (shape(64, 8, 64, 4, 128, "bf16"), [70], [0, 2]),
    "bf16_few_heads_256": (shape(64, 8, 64, 4, 256, "bf16"), [70, 33, 0], [0, 2]),
    "bf16_two_head_groups": (shape(64, 40, 128, 8, 1536, "bf16"), [97, 160], [0, 2]),
    "bf16_7b_longer": (shape(64, 32, 128, 8, 1536, "bf16"), [1500], [0, 1, 7, 47]),
}


# every latent width the matrix-core attention kernel is compiled for (multiples of 128 up to 2048)
for _dc in (128, 384, 512, 640, 896, 1024, 1152, 1280, 1408, 1664, 1792, 2048):
    DECODE_CASES["bf16_latent_%d" % _dc] = (shape(64, 32, 128, 8 if _dc % 256 else 4, _dc, "bf16"), [150, 33, 16],
                                            [0, 3])
# r = 16 elite chunks per head (Table 2's RoPElite setting; 34.4 % of the full cache at the 7B shape with d_c 1792)
DECODE_CASES["bf16_r16_latent_1792"] = (shape(64, 32, 128, 16, 1792, "bf16"), [300, 1, 257, 16], [0, 1, 4])
DECODE_CASES["bf16_r16_latent_1024_batch_9"] = (shape(64, 32, 128, 16, 1024, "bf16"),
                                                [0, 1, 15, 16, 17, 250, 33, 48, 100], [0, 3])
DECODE_CASES["bf16_r16_latent_1536_40_heads"] = (shape(64, 40, 128, 16, 1536, "bf16"), [97, 160], [0, 2])
DECODE_CASES["bf16_r16_latent_896_one_wave_per_simd"] = (shape(64, 32, 128, 16, 896, "bf16"), [150, 33, 16], [0, 3])
DECODE_CASES["bf16_r16_small_heads"] = (shape(64, 8, 64, 16, 256, "bf16"), [70, 33], [0, 2])
# r = 32 elite chunks per head (Table 2's largest RoPElite setting; 37.5 % of the full cache at the 7B shape with d_c 1024)
DECODE_CASES["bf16_r32_latent_1024"] = (shape(64, 32, 128, 32, 1024, "bf16"), [300, 1, 257, 16], [0, 1, 4])
DECODE_CASES["bf16_r32_latent_1152_batch_9"] = (shape(64, 32, 128, 32, 1152, "bf16"),
                                                [0, 1, 15, 16, 17, 250, 33, 48, 100], [0, 3])
DECODE_CASES["bf16_r32_latent_768_40_heads"] = (shape(64, 40, 128, 32, 768, "bf16"), [97, 160], [0, 2])
DECODE_CASES["bf16_r32_eight_heads"] = (shape(64, 8, 128, 32, 256, "bf16"), [70, 33], [0, 2])
DECODE_CASES["bf16_latent_2048_40_heads"] = (shape(64, 40, 128, 8, 2048, "bf16"), [97, 160], [0, 2])
DECODE_CASES["bf16_latent_1024_batch_9"] = (shape(64, 32, 128, 8, 1024, "bf16"), [0, 1, 15, 16, 17, 250, 33, 48, 100],
                                            [0, 3])


@pytest.mark.parametrize("name", list(DECODE_CASES))
def test_decode_matches_oracle_on_same_planes(name):
    sh, seqs, splits = DECODE_CASES[name]
    dt = sh["dtype"]
    B, stride = len(seqs), max(seqs) + 3
    rng, idx, W_ke, W_dkv, W_uk, W_uv, x, q = _draw(sh, B * stride, B, 200 + len(name))
    dims = dims_of(sh)
    pos = np.tile(np.arange(stride), B)
    # cache rows from the oracle's append, rounded once to the cache dtype; both sides read these
    ke64, c64 = orc.append(x, pos, W_ke, W_dkv, idx, sh["head_dim"], sh["rope_base"])
    ked, cd = dev(ke64, dt), dev(c64, dt)
    qd, Wukd, Wuvd = dev(q, dt), dev(W_uk, dt), dev(W_uv, dt)
    q_pos = np.array([max(s - 1, 0) for s in seqs])
    ref = orc.decode_attn(host64(qd), q_pos, host64(ked).reshape(B, stride, sh["n_heads"], -1),
                          host64(cd).reshape(B, stride, -1), seqs, host64(Wukd), host64(Wuvd), idx,
                          sh["head_dim"], sh["rope_base"])
    outs = []
    for ns in splits:
        out = gpu_decode(dims, qd, i32(q_pos), i32(seqs), max(seqs), stride, Wukd, Wuvd, i32(idx), ked, cd,
                         n_splits=ns)
        o = host64(out)
        assert np.all(np.isfinite(o))
        err = orc.max_abs_rel(o, ref)
        assert err <= TOL[dt], "n_splits=%d err=%g" % (ns, err)
        for b, s in enumerate(seqs):
            if s == 0:
                assert np.all(o[b] == 0.0)
        outs.append(o)
    # the split count changes rounding only
    for o in outs[1:]:
        assert orc.max_abs_rel(o, outs[0]) <= TOL[dt]


@pytest.mark.parametrize("name", ["bf16_7b", "bf16_13b_ragged_batch", "bf16_7b_12pct", "bf16_r32_latent_1024", "fp32_ragged_batch"])
def test_rows_beyond_a_sequence_never_reach_the_result(name):
    """max_seq_len is only a host-side bound: the kernels may read a sequence's rows up to it before seq_len[b] has
    arrived on the device (the split attention kernel requests its first tile at once).  Whatever those rows hold
    must not matter: the planes beyond every seq_len[b] are filled with NaN, max_seq_len is the whole stride, and
    the result has to be finite and equal to the oracle's, with few and with many splits."""
    sh, seqs, _ = DECODE_CASES[name]
    dt = sh["dtype"]
    B, stride = len(seqs), max(seqs) + 40
    rng, idx, W_ke, W_dkv, W_uk, W_uv, x, q = _draw(sh, B * stride, B, 900 + len(name))
    dims = dims_of(sh)
    pos = np.tile(np.arange(stride), B)
    ke64, c64 = orc.append(x, pos, W_ke, W_dkv, idx, sh["head_dim"], sh["rope_base"])
    ked, cd = dev(ke64, dt), dev(c64, dt)
    qd, Wukd, Wuvd = dev(q, dt), dev(W_uk, dt), dev(W_uv, dt)
    q_pos = np.array([max(s - 1, 0) for s in seqs])
    ref = orc.decode_attn(host64(qd), q_pos, host64(ked).reshape(B, stride, sh["n_heads"], -1),
                          host64(cd).reshape(B, stride, -1), seqs, host64(Wukd), host64(Wuvd), idx,
                          sh["head_dim"], sh["rope_base"])
    for b, s in enumerate(seqs):                      # poison what no query may see
        ked[b * stride + s:(b + 1) * stride] = float("nan")
        cd[b * stride + s:(b + 1) * stride] = float("nan")
    for ns in (0, 1, 7):
        out = host64(gpu_decode(dims, qd, i32(q_pos), i32(seqs), stride, stride, Wukd, Wuvd, i32(idx), ked, cd,
                                n_splits=ns))
        assert np.all(np.isfinite(out)), "n_splits=%d" % ns
        assert orc.max_abs_rel(out, ref) <= TOL[dt], "n_splits=%d" % ns


@pytest.mark.parametrize("d_c,n_heads", [(1536, 32), (768, 32), (1920, 40)])
def test_decode_with_scores_that_keep_rising(d_c, n_heads):
    """The running maximum of the online softmax has to be raised many times along the sequence:
    the latent rows are multiples g(j) of one direction, so every head's score is g(j) times a
    per-head constant (rising for some heads, falling for the others)."""
    sh = shape(64, n_heads, 128, 8, d_c, "bf16")
    S = 700
    rng, idx, _, _, W_uk, W_uv, _, q = _draw(sh, 1, 1, 77)
    ke64, c64 = synth.draw_cache_planes(rng, S, n_heads, sh["r"], d_c)
    v = rng.standard_normal(d_c)
    g = np.linspace(0.0, 15.0, S) + 0.3 * np.sin(np.arange(S))
    c64 = 0.05 * c64 + g[:, None] * v[None, :]
    dims = dims_of(sh)
    ked, cd, qd, Wukd, Wuvd = dev(ke64, "bf16"), dev(c64, "bf16"), dev(q, "bf16"), dev(W_uk, "bf16"), dev(W_uv, "bf16")
    ref = orc.decode_attn(host64(qd), [S - 1], host64(ked).reshape(1, S, n_heads, -1), host64(cd).reshape(1, S, -1),
                          [S], host64(Wukd), host64(Wuvd), idx, 128, sh["rope_base"])
    # the scores of the test really span far more than the rescale slack
    q64, Wuk64, c_r = host64(qd)[0], host64(Wukd), host64(cd)
    rise = []
    for h in range(n_heads):
        qt_h = Wuk64[:, h, :] @ q64[h, orc.nonelite_dims(idx[h], 128)]
        s_h = (c_r @ qt_h) * np.log2(np.e) / np.sqrt(128.0)
        rise.append(s_h[-1] - s_h[0])
    assert max(rise) > 24.0 and min(rise) < -24.0          # in the log2 domain; the kernels' slack is 8
    for ns in (1, 3):
        out = host64(gpu_decode(dims, qd, i32([S - 1]), i32([S]), S, S, Wukd, Wuvd, i32(idx), ked, cd, n_splits=ns))
        assert np.all(np.isfinite(out))
        assert orc.max_abs_rel(out, ref) <= TOL["bf16"], "n_splits=%d" % ns


def test_decode_is_bitwise_repeatable():
    sh, seqs, _ = DECODE_CASES["bf16_7b"]
    B, stride = len(seqs), max(seqs)
    rng, idx, _, _, W_uk, W_uv, _, q = _draw(sh, 1, B, 5)
    ke64, c64 = synth.draw_cache_planes(rng, B * stride, sh["n_heads"], sh["r"], sh["d_c"])
    dims = dims_of(sh)
    args = (dims, dev(q, "bf16"), i32([s - 1 for s in seqs]), i32(seqs), max(seqs), stride, dev(W_uk, "bf16"),
            dev(W_uv, "bf16"), i32(idx), dev(ke64, "bf16"), dev(c64, "bf16"))
    a = gpu_decode(*args)
    b = gpu_decode(*args)
    assert torch.equal(a, b)


@pytest.mark.parametrize("name", ["tiny_fp32", "bf16_mid"])
def test_end_to_end_append_then_decode(name):
    if name == "tiny_fp32":
        cfg = synth.CONFIGS["tiny_fp32"]
        sh, S, p = cfg.as_dict(), cfg.context, synth.problem(cfg)
        idx, W_ke, W_dkv, W_uk, W_uv, x, q = (p[k] for k in ("elite_idx", "W_ke", "W_dkv", "W_uk", "W_uv", "x", "q"))
    else:
        sh, S = shape(256, 32, 128, 8, 1536, "bf16"), 333
        _, idx, W_ke, W_dkv, W_uk, W_uv, x, q = _draw(sh, S, 1, 31)
    dt = sh["dtype"]
    dims = dims_of(sh)
    pos = np.arange(S)
    xd, Wked, Wdkvd, Wukd, Wuvd, qd = (dev(a, dt) for a in (x, W_ke, W_dkv, W_uk, W_uv, q))
    ke, c = gpu_append(dims, xd, i32(pos), i64(pos), Wked, Wdkvd, i32(idx), S)
    out = gpu_decode(dims, qd, i32([S - 1]), i32([S]), S, S, Wukd, Wuvd, i32(idx), ke, c)
    # the oracle runs the whole chain in float64 from the same rounded inputs
    ke_ref, c_ref = orc.append(host64(xd), pos, host64(Wked), host64(Wdkvd), idx, sh["head_dim"], sh["rope_base"])
    ref = orc.decode_attn(host64(qd), [S - 1], ke_ref[None], c_ref[None], [S], host64(Wukd), host64(Wuvd), idx,
                          sh["head_dim"], sh["rope_base"])
    assert orc.max_abs_rel(host64(out), ref) <= TOL[dt]


def test_shift_invariance_on_gpu():
    """Section 2.2 eq. 1a = 1b: shifting cache and query positions together changes nothing."""
    cfg = synth.CONFIGS["tiny_fp32"]
    p = synth.problem(cfg, tokens=40)
    dims = dims_of(cfg)
    S = 40
    dv = lambda k: dev(p[k], "fp32")
    outs = []
    for shift in (0, 20000):
        pos = np.arange(S) + shift
        ke, c = gpu_append(dims, dv("x"), i32(pos), i64(np.arange(S)), dv("W_ke"), dv("W_dkv"), i32(p["elite_idx"]), S)
        outs.append(host64(gpu_decode(dims, dv("q"), i32([S - 1 + shift]), i32([S]), S, S, dv("W_uk"), dv("W_uv"),
                                      i32(p["elite_idx"]), ke, c)))
    assert orc.max_abs_rel(outs[1], outs[0]) <= 1e-5


MHA_CASES = {"fp32": (2, 32, [77, 5], "fp32"), "bf16": (32, 128, [300, 129], "bf16")}


@pytest.mark.parametrize("name", list(MHA_CASES))
def test_mha_comparator_matches_oracle(name):
    n_h, d_h, seqs, dt = MHA_CASES[name]
    rng = np.random.default_rng(17)
    B, stride = len(seqs), max(seqs)
    K = rng.standard_normal((B * stride, n_h, d_h))
    V = rng.standard_normal((B * stride, n_h, d_h))
    q = rng.standard_normal((B, n_h, d_h))
    dims = ekv.make_dims(n_h * d_h, n_h, d_h, 0, 8, dt)
    Kd, Vd, qd = dev(K, dt), dev(V, dt), dev(q, dt)
    q_pos = [s - 1 for s in seqs]
    ref = orc.mha_decode(host64(qd), q_pos, host64(Kd).reshape(B, stride, n_h, d_h),
                         host64(Vd).reshape(B, stride, n_h, d_h), seqs, 10000.0)
    for ns in (0, 1, 3):
        out = torch.empty(B, n_h, d_h, dtype=ekv.torch_dtype(dims), device=DEV)
        ws = torch.empty(ekv.elitekv_mha_decode_workspace_bytes(dims, B, stride, ns), dtype=torch.uint8, device=DEV)
        ekv.elitekv_mha_decode(dims, qd, i32(q_pos), i32(seqs), stride, stride, Kd, Vd, out, ws, n_splits=ns)
        torch.cuda.synchronize()
        assert orc.max_abs_rel(host64(out), ref) <= TOL[dt]


def test_stream_read_probe_runs():
    src = torch.arange(1 << 20, dtype=torch.int32, device=DEV)
    sink = torch.zeros(4096, dtype=torch.int32, device=DEV)
    ekv.elitekv_stream_read(src, sink)
    torch.cuda.synchronize()
    # xor of all words read must equal the xor of the buffer
    want = int(np.bitwise_xor.reduce(np.arange(1 << 20, dtype=np.uint32)))
    got = int(np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32)))
    assert got == want


def test_stream_read_by_load_kind():
    """Loads into registers (plain, non-temporal) fold every word read; the direct global->LDS forms read
    whole 16 MiB units and report how many bytes that was."""
    n_words = 9 << 20                                            # 36 MiB: two units and a remainder
    src = torch.arange(n_words, dtype=torch.int32, device=DEV)
    want = int(np.bitwise_xor.reduce(np.arange(n_words, dtype=np.uint32)))
    for mode in (0, 1):
        sink = torch.zeros(4096, dtype=torch.int32, device=DEV)
        assert ekv.elitekv_stream_read_mode(src, sink, mode) == 4 * n_words
        torch.cuda.synchronize()
        assert int(np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32))) == want
    for mode in (2, 3):
        sink = torch.zeros(4096, dtype=torch.int32, device=DEV)
        assert ekv.elitekv_stream_read_mode(src, sink, mode) == 32 << 20
        assert ekv.elitekv_stream_read_mode(src, sink, mode, nbytes=8 << 20) == 0     # less than one unit: no launch
        torch.cuda.synchronize()
