"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times (automatic
split count, same strides): the planes are built by the library's own append from seeded hidden
states; whole append calls are checked row by row against the oracle's append, and EVERY
(batch row, head) output of the decode is checked against the float64 oracle on exactly the planes
the GPU reads, for a flat and for a peaked softmax; then one decode step through the single-call
entry point is checked the same way.
"""
import numpy as np
import pytest
import torch

import elitekv_synth as synth
import paper_2503_01586_amd as ekv
from oracle import elitekv_oracle as orc

from gpu_util import DEV, TOL, dev, dims_of, gpu_decode, host64, i32, i64, parity_report

pytestmark = pytest.mark.gpu

# workload -> (batch row, first token) of the append calls checked row by row, tokens appended per call
# (7b_12: the 2048-token prefill of a sequence is one call; every row of three sequences is checked)
CHECKED_APPENDS = {
    "7b_25_b8_s4096": ([(5, 0)], 4096),
    "7b_25_b1_s32768": ([(0, 8192)], 8192),
    "13b_25_b16_s8192": ([(15, 0)], 8192),
    "7b_12_b64_s2048": ([(0, 0), (41, 0), (63, 0)], 2048),
}
ROW_TOL = 5e-2          # sanity bound on the max-abs-rel of every single row / (batch row, head) output vector (observed: up to 1.8e-2 with a peaked softmax)


@pytest.mark.parametrize("name", list(CHECKED_APPENDS))
def test_full_size_append_and_decode(name):
    """One benchmark workload at full size, in the launch configuration bench.py times.
    append: EVERY row of the checked calls against the oracle's append of the same hidden states (so
    the decode checks below do not rest on rows nobody looked at), and three sampled rows of every
    other call; decode: EVERY (batch row, head) output vector against the oracle on exactly the planes
    the GPU reads -- with the recipe's query (logits ~ N(0, 1), a nearly flat softmax over thousands of
    tokens) and with the query scaled by 4 (logits ~ N(0, 16): a few tokens carry the sum, so a lost or
    mis-masked tile moves the output by far more than the bound); then one decode step through the
    single-call entry point, again every output vector."""
    cfg = synth.CONFIGS[name]
    checked, t_call = CHECKED_APPENDS[name]
    B, S, n_h, d_h, r, d_c, d = cfg.batch, cfg.context, cfg.n_heads, cfg.head_dim, cfg.r, cfg.d_c, cfg.d_model
    dt = cfg.dtype
    dims = dims_of(cfg)
    rng = synth.rng_for(cfg.index)
    idx = synth.draw_elite_idx(rng, n_h, d_h, r)
    W_ke, W_dkv, W_uk, W_uv = synth.draw_weights(rng, d, n_h, d_h, r, d_c)
    q = synth.draw_query(rng, B, n_h, d_h)
    Wked, Wdkvd, Wukd, Wuvd, qd = (dev(a, dt) for a in (W_ke, W_dkv, W_uk, W_uv, q))
    idxd = i32(idx)
    Wke64, Wdkv64 = host64(Wked), host64(Wdkvd)

    ke = torch.zeros(B * S, n_h, 2 * r, dtype=ekv.torch_dtype(dims), device=DEV)
    c = torch.zeros(B * S, d_c, dtype=ekv.torch_dtype(dims), device=DEV)
    ws = torch.empty(max(ekv.elitekv_append_workspace_bytes(dims, t_call), 16), dtype=torch.uint8, device=DEV)
    kept = {}                                       # sampled hidden rows of the calls not checked in full
    full = {}                                       # hidden states of the calls checked in full
    xrng = synth.rng_for(cfg.index, stream=7)
    for b in range(B):
        for t0 in range(0, S, t_call):
            x = xrng.standard_normal((t_call, d), dtype=np.float32)
            xd = torch.from_numpy(x).to(ekv.torch_dtype(dims)).to(DEV)
            pos = torch.arange(t0, t0 + t_call, dtype=torch.int32, device=DEV)
            slot = torch.arange(b * S + t0, b * S + t0 + t_call, dtype=torch.int64, device=DEV)
            ekv.elitekv_append(dims, xd, pos, slot, Wked, Wdkvd, idxd, ke, c, ws=ws)
            if (b, t0) in checked:
                full[(b, t0)] = host64(xd)
            else:
                for tt in (0, t_call // 2 + 1, t_call - 1):
                    kept[(b, t0 + tt)] = host64(xd[tt:tt + 1])
    torch.cuda.synchronize()

    # append: every row of the checked calls, sampled rows of the others
    for (b, t0), x64 in full.items():
        print("append check: %s sequence %d tokens %d..%d" % (name, b, t0, t0 + t_call - 1), flush=True)
        ke_ref, c_ref = orc.append(x64, np.arange(t0, t0 + t_call), Wke64, Wdkv64, idx, d_h, cfg.rope_base)
        lo = b * S + t0
        e_c, r_c = parity_report("%s append latent rows" % name, host64(c[lo:lo + t_call]), c_ref, TOL[dt])
        e_k, r_k = parity_report("%s append elite rows" % name, host64(ke[lo:lo + t_call]).reshape(t_call, -1),
                                 ke_ref.reshape(t_call, -1), TOL[dt])
        assert max(e_c, e_k) <= TOL[dt] and max(r_c, r_k) <= ROW_TOL
    for (b, t), x64 in kept.items():
        ke_ref, c_ref = orc.append(x64, np.array([t]), Wke64, Wdkv64, idx, d_h, cfg.rope_base)
        assert orc.max_abs_rel(host64(c[b * S + t]), c_ref[0]) <= TOL[dt]
        assert orc.max_abs_rel(host64(ke[b * S + t]), ke_ref[0]) <= TOL[dt]

    # decode in the benchmark's launch configuration (automatic splits): every batch row, every head
    q_pos = np.full(B, S - 1)
    seq = np.full(B, S)
    Wuk64, Wuv64 = host64(Wukd), host64(Wuvd)
    ke64 = host64(ke).reshape(B, S, n_h, 2 * r)
    c64 = host64(c).reshape(B, S, d_c)

    def decode_case(label, q_dev):
        out = host64(gpu_decode(dims, q_dev, i32(q_pos), i32(seq), S, S, Wukd, Wuvd, idxd, ke, c, n_splits=0))
        assert np.all(np.isfinite(out))
        ref = orc.decode_attn(host64(q_dev), q_pos, ke64, c64, seq, Wuk64, Wuv64, idx, d_h, cfg.rope_base)
        err, row_err = parity_report("%s decode, %s" % (name, label), out, ref, TOL[dt])
        assert err <= TOL[dt], "%s: max-abs-rel %g" % (label, err)
        assert row_err <= ROW_TOL, "%s: worst (batch row, head) max-abs-rel %g" % (label, row_err)
        return ref

    decode_case("recipe query", qd)
    ref_peaked = decode_case("query x 4 (peaked softmax)", dev(4.0 * host64(qd), dt))
    # the peaked case really is peaked: the output is far from the mean of the values
    assert np.max(np.abs(ref_peaked)) > 3 * np.max(np.abs(orc.decode_attn(0 * host64(qd[:1]), q_pos[:1], ke64[:1], c64[:1],
                                                                          seq[:1], Wuk64, Wuv64, idx, d_h, cfg.rope_base,
                                                                          heads=[0])))

    # one decode step through the single-call entry point, as bench.py times it: a new token per
    # sequence replaces the last cached row and the query attends to all S tokens
    x_new = synth.draw_hidden(synth.rng_for(cfg.index, stream=9), B, d)
    xnd = dev(x_new, dt)
    slot_new = np.arange(B) * S + (S - 1)
    out2 = torch.full((B, n_h, d_h), float("nan"), dtype=ekv.torch_dtype(dims), device=DEV)
    sws = torch.full((ekv.elitekv_decode_step_workspace_bytes(dims, B, S),), 0xFF, dtype=torch.uint8, device=DEV)
    ekv.elitekv_decode_step(dims, xnd, qd, i32(q_pos), i64(slot_new), i32(seq), S, S, Wked, Wdkvd, Wukd, Wuvd, idxd,
                            ke, c, out2, sws)
    torch.cuda.synchronize()
    out2 = host64(out2)
    assert np.all(np.isfinite(out2))
    ke_ref, c_ref = orc.append(host64(xnd), np.full(B, S - 1), Wke64, Wdkv64, idx, d_h, cfg.rope_base)
    rows_t = torch.tensor(slot_new, device=DEV)
    e_c, _ = parity_report("%s step: new latent rows" % name, host64(c[rows_t]), c_ref, TOL[dt])
    e_k, _ = parity_report("%s step: new elite rows" % name, host64(ke[rows_t]).reshape(B, -1), ke_ref.reshape(B, -1),
                           TOL[dt])
    assert max(e_c, e_k) <= TOL[dt]
    ke64 = host64(ke).reshape(B, S, n_h, 2 * r)
    c64 = host64(c).reshape(B, S, d_c)
    ref = orc.decode_attn(host64(qd), q_pos, ke64, c64, seq, Wuk64, Wuv64, idx, d_h, cfg.rope_base)
    err, row_err = parity_report("%s decode step" % name, out2, ref, TOL[dt])
    assert err <= TOL[dt], "decode step: max-abs-rel %g" % err
    assert row_err <= ROW_TOL, "decode step: worst (batch row, head) max-abs-rel %g" % row_err


@pytest.mark.parametrize("name,T", [("7b_12_b64_s2048", 33100), ("7b_25_b1_s32768", 16500),
                                    ("13b_25_b16_s8192", 13100)])
def test_prefill_append_with_wide_token_tiles(name, T):
    """Appends large enough for the widest tiles of the GEMM path (256 tokens x 256 columns; token
    counts that are not a multiple of any tile): sampled rows against the oracle -- every 32-token
    sub-tile of the first and of the ragged last tile, and rows around tile borders -- and the rows
    around the destination range stay untouched."""
    cfg = synth.CONFIGS[name]
    n_h, d_h, r, d_c, d = cfg.n_heads, cfg.head_dim, cfg.r, cfg.d_c, cfg.d_model
    dims = dims_of(cfg)
    guard = 7
    rng = synth.rng_for(cfg.index, stream=11)
    idx = synth.draw_elite_idx(rng, n_h, d_h, r)
    W_ke, W_dkv, _, _ = synth.draw_weights(rng, d, n_h, d_h, r, d_c)
    Wked, Wdkvd = dev(W_ke, "bf16"), dev(W_dkv, "bf16")
    xd = torch.from_numpy(rng.standard_normal((T, d), dtype=np.float32)).to(torch.bfloat16).to(DEV)
    pos_h = rng.integers(0, 4096, size=T)
    slot_h = np.arange(T) + guard
    ke = torch.full((T + 2 * guard, n_h, 2 * r), 3.0, dtype=torch.bfloat16, device=DEV)
    c = torch.full((T + 2 * guard, d_c), 3.0, dtype=torch.bfloat16, device=DEV)
    ws = torch.empty(max(ekv.elitekv_append_workspace_bytes(dims, T), 16), dtype=torch.uint8, device=DEV)
    ekv.elitekv_append(dims, xd, i32(pos_h), i64(slot_h), Wked, Wdkvd, i32(idx), ke, c, ws=ws)
    torch.cuda.synchronize()
    assert bool((ke[:guard] == 3.0).all()) and bool((ke[T + guard:] == 3.0).all())
    assert bool((c[:guard] == 3.0).all()) and bool((c[T + guard:] == 3.0).all())
    Wke64, Wdkv64 = host64(Wked), host64(Wdkvd)
    last0 = (T - 1) // 256 * 256
    rows = sorted(set(list(range(0, 256, 19)) + [1, 31, 32, 127, 128, 255, 256, 257, 2047, 2048, 12345 % T, T // 2]
                      + list(range(last0, T, 13)) + [T - 2, T - 1]))
    rows_t = torch.tensor(rows, device=DEV)
    ke_ref, c_ref = orc.append(host64(xd[rows_t]), pos_h[rows], Wke64, Wdkv64, idx, d_h, cfg.rope_base)
    srows = torch.tensor(slot_h[rows], device=DEV)
    for i, t in enumerate(rows):
        assert orc.max_abs_rel(host64(c[srows[i]]), c_ref[i]) <= TOL["bf16"], "latent row %d" % t
        assert orc.max_abs_rel(host64(ke[srows[i]]), ke_ref[i]) <= TOL["bf16"], "elite row %d" % t


def test_slrd_prefill_append_with_wide_tiles():
    """S-LRD prefill through the widest GEMM tiles, with the A^k / A^v boundary (column 512 + 576)
    inside a 256-column tile: sampled rows against the oracle."""
    d, n_h, d_h, r, d_ck, d_cv, T = 4096, 32, 128, 8, 576, 960, 16500
    dims = ekv.make_dims(d, n_h, d_h, r, d_ck + d_cv, "bf16", 10000.0)
    rng = np.random.default_rng(20250)
    idx = synth.draw_elite_idx(rng, n_h, d_h, r)
    W_ke = rng.standard_normal((d, n_h, 2 * r)) / np.sqrt(d)
    A_k = rng.standard_normal((d, d_ck)) / np.sqrt(d)
    A_v = rng.standard_normal((d, d_cv)) / np.sqrt(d)
    Wked, Akd, Avd = dev(W_ke, "bf16"), dev(A_k, "bf16"), dev(A_v, "bf16")
    xd = torch.from_numpy(rng.standard_normal((T, d), dtype=np.float32)).to(torch.bfloat16).to(DEV)
    pos_h = rng.integers(0, 4096, size=T)
    slot_h = rng.permutation(T + 5)[:T]
    ke = torch.full((T + 5, n_h, 2 * r), 3.0, dtype=torch.bfloat16, device=DEV)
    c = torch.full((T + 5, d_ck + d_cv), 3.0, dtype=torch.bfloat16, device=DEV)
    ws = torch.empty(max(ekv.elitekv_slrd_append_workspace_bytes(dims, d_ck, T), 16), dtype=torch.uint8, device=DEV)
    ekv.elitekv_slrd_append(dims, d_ck, xd, i32(pos_h), i64(slot_h), Wked, Akd, Avd, i32(idx), ke, c, ws=ws)
    torch.cuda.synchronize()
    untouched = torch.tensor(np.setdiff1d(np.arange(T + 5), slot_h), device=DEV)
    assert bool((c[untouched] == 3.0).all()) and bool((ke[untouched] == 3.0).all())
    rows = sorted(set(list(range(0, 256, 23)) + [255, 256, 8191, 8192, 16383, 16384] + list(range(16384, T, 11))))
    ke_ref, ck_ref, cv_ref = orc.slrd_append(host64(xd[torch.tensor(rows, device=DEV)]), pos_h[rows], host64(Wked),
                                             host64(Akd), host64(Avd), idx, d_h, 10000.0)
    srows = torch.tensor(slot_h[rows], device=DEV)
    c_g, ke_g = host64(c[srows]), host64(ke[srows])
    assert orc.max_abs_rel(c_g[:, :d_ck], ck_ref) <= TOL["bf16"]
    assert orc.max_abs_rel(c_g[:, d_ck:], cv_ref) <= TOL["bf16"]
    assert orc.max_abs_rel(ke_g, ke_ref) <= TOL["bf16"]


@pytest.mark.parametrize("name,T", [("7b_25_b1_s32768", 2048), ("7b_12_b64_s2048", 2048), ("13b_25_b16_s8192", 2048),
                                    ("7b_25_b1_s32768", 4500)])
def test_full_size_prefill_attention(name, T):
    """elitekv_prefill_attn in the configuration bench.py times (one sequence, the T-token prompt attends
    causally to its own T cache rows; 4500 tokens: two work-groups per compute unit, a ragged last block):
    the planes come from the library's append of seeded hidden states; sampled (query, head) outputs are
    computed one by one by the float64 oracle from exactly the planes the GPU reads."""
    cfg = synth.CONFIGS[name]
    n_h, d_h, r, d_c, d = cfg.n_heads, cfg.head_dim, cfg.r, cfg.d_c, cfg.d_model
    dims = dims_of(cfg)
    rng = synth.rng_for(cfg.index, stream=13)
    idx = synth.draw_elite_idx(rng, n_h, d_h, r)
    W_ke, W_dkv, W_uk, W_uv = synth.draw_weights(rng, d, n_h, d_h, r, d_c)
    Wked, Wdkvd, Wukd, Wuvd = (dev(a, "bf16") for a in (W_ke, W_dkv, W_uk, W_uv))
    idxd = i32(idx)
    xd = torch.from_numpy(rng.standard_normal((T, d), dtype=np.float32)).to(torch.bfloat16).to(DEV)
    qd = torch.from_numpy(rng.standard_normal((1, T, n_h, d_h), dtype=np.float32)).to(torch.bfloat16).to(DEV)
    ke = torch.zeros(T, n_h, 2 * r, dtype=torch.bfloat16, device=DEV)
    c = torch.zeros(T, d_c, dtype=torch.bfloat16, device=DEV)
    ws = torch.empty(max(ekv.elitekv_append_workspace_bytes(dims, T), 16), dtype=torch.uint8, device=DEV)
    pos = torch.arange(T, dtype=torch.int32, device=DEV)
    ekv.elitekv_append(dims, xd, pos, torch.arange(T, dtype=torch.int64, device=DEV), Wked, Wdkvd, idxd, ke, c, ws=ws)
    out = torch.full((1, T, n_h, d_h), float("nan"), dtype=torch.bfloat16, device=DEV)
    pws = torch.full((ekv.elitekv_prefill_attn_workspace_bytes(dims, 1, T, T),), 0xFF, dtype=torch.uint8, device=DEV)
    ekv.elitekv_prefill_attn(dims, qd, pos, pos + 1, T, T, Wukd, Wuvd, idxd, ke, c, out, pws)
    torch.cuda.synchronize()
    o = host64(out)
    assert np.all(np.isfinite(o))
    heads_s = [0, n_h // 2 + 1, n_h - 1]
    queries = sorted(set([0, 1, 63, 64, 127, 128, 129, T // 2 + 7, T - 129, T - 2, T - 1]))
    ke64, c64, q64 = host64(ke), host64(c), host64(qd)
    Wuk64, Wuv64 = host64(Wukd), host64(Wuvd)
    refs, gots = [], []
    for t in queries:
        ref = orc.decode_attn(q64[0, t:t + 1], [t], [ke64], [c64], [t + 1], Wuk64, Wuv64, idx, d_h, cfg.rope_base,
                              heads=heads_s)
        for h in heads_s:
            refs.append(ref[0, h])
            gots.append(o[0, t, h])
    err = orc.max_abs_rel(np.stack(gots), np.stack(refs))
    assert err <= TOL["bf16"], "max-abs-rel %g" % err


def test_full_size_slrd_prefill_attention():
    """elitekv_slrd_prefill_attn at the 7B shape with the paper's 25 % S-LRD split sizes (d_ck 576, d_cv 960),
    one 2048-token prompt attending causally to its own rows (the 256 x 256 tile of the rebuild GEMM with a
    different contraction slice per column block): planes from the library's own S-LRD append; sampled
    (query, head) outputs one by one from the float64 oracle on exactly the planes the GPU reads."""
    cfg = synth.CONFIGS["7b_25_b1_s32768"]
    n_h, d_h, r, d_c, d, T = cfg.n_heads, cfg.head_dim, cfg.r, cfg.d_c, cfg.d_model, 2048
    d_ck = 576
    dims = dims_of(cfg)
    rng = synth.rng_for(cfg.index, stream=17)
    idx = synth.draw_elite_idx(rng, n_h, d_h, r)
    W_ke, A_k, B_k, _ = synth.draw_weights(rng, d, n_h, d_h, r, d_ck)
    _, A_v, _, B_v = synth.draw_weights(rng, d, n_h, d_h, r, d_c - d_ck)
    Wked, Akd, Avd, Bkd, Bvd = (dev(a, "bf16") for a in (W_ke, A_k, A_v, B_k, B_v))
    idxd = i32(idx)
    xd = torch.from_numpy(rng.standard_normal((T, d), dtype=np.float32)).to(torch.bfloat16).to(DEV)
    qd = torch.from_numpy(rng.standard_normal((1, T, n_h, d_h), dtype=np.float32)).to(torch.bfloat16).to(DEV)
    ke = torch.zeros(T, n_h, 2 * r, dtype=torch.bfloat16, device=DEV)
    c = torch.zeros(T, d_c, dtype=torch.bfloat16, device=DEV)
    ws = torch.empty(max(ekv.elitekv_slrd_append_workspace_bytes(dims, d_ck, T), 16), dtype=torch.uint8, device=DEV)
    pos = torch.arange(T, dtype=torch.int32, device=DEV)
    ekv.elitekv_slrd_append(dims, d_ck, xd, pos, torch.arange(T, dtype=torch.int64, device=DEV), Wked, Akd, Avd, idxd,
                            ke, c, ws=ws)
    out = torch.full((1, T, n_h, d_h), float("nan"), dtype=torch.bfloat16, device=DEV)
    pws = torch.full((ekv.elitekv_slrd_prefill_attn_workspace_bytes(dims, d_ck, 1, T, T),), 0xFF, dtype=torch.uint8,
                     device=DEV)
    ekv.elitekv_slrd_prefill_attn(dims, d_ck, qd, pos, pos + 1, T, T, Bkd, Bvd, idxd, ke, c, out, pws)
    torch.cuda.synchronize()
    o = host64(out)
    assert np.all(np.isfinite(o))
    heads_s = [0, n_h // 2 + 1, n_h - 1]
    queries = sorted(set([0, 1, 63, 64, 127, 128, 129, T // 2 + 7, T - 129, T - 2, T - 1]))
    ke64, c64, q64 = host64(ke), host64(c), host64(qd)
    Bk64, Bv64 = host64(Bkd), host64(Bvd)
    refs, gots = [], []
    for t in queries:
        ref = orc.slrd_decode_attn(q64[0, t:t + 1], [t], [ke64], [c64[:, :d_ck]], [c64[:, d_ck:]], [t + 1], Bk64, Bv64,
                                   idx, d_h, cfg.rope_base, heads=heads_s)
        for h in heads_s:
            refs.append(ref[0, h])
            gots.append(o[0, t, h])
    err = orc.max_abs_rel(np.stack(gots), np.stack(refs))
    assert err <= TOL["bf16"], "max-abs-rel %g" % err
