"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and every validation path returns its error code before any launch."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import elitekv_synth as synth
import paper_2503_01586_amd as ekv
from oracle import elitekv_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
lib = ekv.raw()
FAKE = 0x10000  # a non-NULL, 16-byte aligned address that is never dereferenced on these paths


def _dims(**kw):
    base = dict(d_model=128, n_heads=4, head_dim=32, r=2, d_c=64, dtype="fp32", rope_base=10000.0)
    base.update(kw)
    return ekv.make_dims(**base)


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "elitekv.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(elitekv_[a-z0-9_]+)\s*\(", hdr))
    assert declared, "no declarations parsed"
    for name in declared:
        assert hasattr(lib, name), "library does not export %s" % name
    assert declared == set(ekv.EXPORTS), (declared ^ set(ekv.EXPORTS))


def test_strerror_names_every_code():
    seen = set()
    for code in range(0, -8, -1):
        s = ekv.elitekv_strerror(code)
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 8
    assert ekv.elitekv_strerror(-99) == "unknown status"


@pytest.mark.parametrize("name", list(synth.CONFIGS))
def test_cache_row_and_param_formulas_match_oracle(name):
    cfg = synth.CONFIGS[name]
    d = ekv.make_dims(cfg.d_model, cfg.n_heads, cfg.head_dim, cfg.r, cfg.d_c, cfg.dtype)
    ke, c = ekv.elitekv_cache_row_elems(d)
    assert ke + c == orc.cache_row_elems(cfg.n_heads, cfg.r, cfg.d_c)
    assert (ke, c) == (2 * cfg.r * cfg.n_heads, cfg.d_c)
    assert ekv.elitekv_param_count(d) == orc.param_count(cfg.d_model, cfg.n_heads, cfg.head_dim, cfg.r, cfg.d_c)


@pytest.mark.parametrize("bad", [dict(head_dim=31), dict(r=-1), dict(r=17), dict(d_c=0), dict(n_heads=0),
                                 dict(d_model=0), dict(dtype=7), dict(rope_base=0.0), dict(rope_base=-3.0)])
def test_bad_dims_are_einval(bad):
    d = _dims(**bad)
    ke, c = C.c_int64(), C.c_int64()
    assert lib.elitekv_cache_row_elems(C.byref(d), C.byref(ke), C.byref(c)) == ekv.EINVAL
    assert ekv.elitekv_decode_workspace_bytes(d, 1, 128) == 0
    assert ekv.elitekv_append_workspace_bytes(d, 1) == 0
    assert lib.elitekv_append(C.byref(d), FAKE, FAKE, FAKE, 4, FAKE, FAKE, FAKE, FAKE, FAKE, 16, None, 0,
                              None) == ekv.EINVAL
    assert lib.elitekv_decode_attn(C.byref(d), FAKE, FAKE, FAKE, 1, 16, 16, FAKE, FAKE, FAKE, FAKE, FAKE,
                                   16, FAKE, FAKE, 1 << 20, 0, None) == ekv.EINVAL


def test_validate_elite_idx():
    d = _dims()
    good = np.array([[0, 15], [3, 4], [7, 1], [9, 2]], dtype=np.int32)
    assert ekv.elitekv_validate_elite_idx(d, good) == ekv.OK
    for bad in ([[0, 16]], [[-1, 2]], [[5, 5]]):
        arr = good.copy()
        arr[2] = bad[0]
        assert ekv.elitekv_validate_elite_idx(d, arr) == ekv.EINDEX
    assert lib.elitekv_validate_elite_idx(C.byref(d), None) == ekv.ENULL
    assert lib.elitekv_validate_elite_idx(C.byref(_dims(r=0)), None) == ekv.OK
    cfg = synth.CONFIGS["7b_25_b1_s32768"]
    idx = synth.draw_elite_idx(synth.rng_for(2), cfg.n_heads, cfg.head_dim, cfg.r)
    assert ekv.elitekv_validate_elite_idx(ekv.make_dims(4096, 32, 128, 8, 1536, "bf16"), idx) == ekv.OK


def _append(d, x=FAKE, pos=FAKE, slot=FAKE, T=4, W_ke=FAKE, W_dkv=FAKE, idx=FAKE, ke=FAKE, c=FAKE,
            rows=16, ws=None, ws_bytes=0):
    return lib.elitekv_append(C.byref(d), x, pos, slot, T, W_ke, W_dkv, idx, ke, c, rows, ws, ws_bytes, None)


def test_append_argument_errors():
    d = _dims()
    assert _append(d, T=0) == ekv.OK                      # empty call is a no-op
    assert _append(d, T=-1) == ekv.EINVAL
    assert _append(d, rows=-1) == ekv.EINVAL
    for k in ("x", "pos", "slot", "W_ke", "W_dkv", "idx", "ke", "c"):
        assert _append(d, **{k: None}) == ekv.ENULL, k
    for k in ("x", "W_ke", "W_dkv", "ke", "c"):
        assert _append(d, **{k: FAKE + 4}) == ekv.EALIGN, k
    d0 = _dims(r=0)                                        # no elite part: its pointers may be NULL
    assert _append(d0, T=0, W_ke=None, idx=None, ke=None) == ekv.OK


def _decode(d, q=FAKE, q_pos=FAKE, seq=FAKE, B=1, max_seq=128, stride=128, W_uk=FAKE, W_uv=FAKE, idx=FAKE,
            ke=FAKE, c=FAKE, rows=128, out=FAKE, ws=FAKE, ws_bytes=1 << 30, n_splits=0):
    return lib.elitekv_decode_attn(C.byref(d), q, q_pos, seq, B, max_seq, stride, W_uk, W_uv, idx, ke, c,
                                   rows, out, ws, ws_bytes, n_splits, None)


def test_decode_argument_errors():
    d = _dims()
    assert _decode(d, B=0) == ekv.OK
    assert _decode(d, B=-1) == ekv.EINVAL
    assert _decode(d, max_seq=-1) == ekv.EINVAL
    assert _decode(d, stride=-1) == ekv.EINVAL
    assert _decode(d, n_splits=-1) == ekv.EINVAL
    assert _decode(d, n_splits=4096) == ekv.EUNSUPPORTED
    assert _decode(_dims(d_c=8192)) == ekv.EUNSUPPORTED
    for k in ("q", "q_pos", "seq", "W_uk", "W_uv", "idx", "ke", "c", "out", "ws"):
        assert _decode(d, **{k: None}) == ekv.ENULL, k
    for k in ("q", "W_uk", "W_uv", "ke", "c", "out", "ws"):
        assert _decode(d, **{k: FAKE + 8}) == ekv.EALIGN, k
    need = ekv.elitekv_decode_workspace_bytes(d, 1, 128)
    assert need > 0
    assert _decode(d, ws_bytes=need - 1) == ekv.EWORKSPACE


def test_workspace_grows_with_batch_and_splits():
    d = ekv.make_dims(4096, 32, 128, 8, 1536, "bf16")
    a = ekv.elitekv_decode_workspace_bytes(d, 1, 32768, 16)
    b = ekv.elitekv_decode_workspace_bytes(d, 2, 32768, 16)
    c = ekv.elitekv_decode_workspace_bytes(d, 1, 32768, 32)
    assert 0 < a < b and a < c
    ns = ekv.elitekv_decode_auto_splits(d, 1, 32768)
    assert 1 <= ns <= 1024
    assert ekv.elitekv_decode_workspace_bytes(d, 1, 32768, 0) == ekv.elitekv_decode_workspace_bytes(d, 1, 32768, ns)
    assert ekv.elitekv_decode_auto_splits(d, 1, 1) == 1


def test_mha_and_stream_argument_errors():
    d = _dims()
    need = ekv.elitekv_mha_decode_workspace_bytes(d, 2, 256)
    assert need > 0
    f = lambda **kw: lib.elitekv_mha_decode(C.byref(d), kw.get("q", FAKE), FAKE, FAKE, kw.get("B", 2), 256, 256,
                                            kw.get("k", FAKE), FAKE, 512, FAKE, FAKE, kw.get("wsb", need), 0, None)
    assert f(B=0) == ekv.OK
    assert f(q=None) == ekv.ENULL
    assert f(k=FAKE + 2) == ekv.EALIGN
    assert f(wsb=need - 1) == ekv.EWORKSPACE
    assert ekv.elitekv_mha_decode_workspace_bytes(_dims(head_dim=36), 1, 64) == 0   # 36/4 lanes: not a power of two
    assert lib.elitekv_stream_read(None, 16, FAKE, None) == ekv.ENULL
    assert lib.elitekv_stream_read(FAKE, 24, FAKE, None) == ekv.EALIGN
    assert lib.elitekv_stream_read(FAKE, 0, FAKE, None) == ekv.OK
    n = C.c_size_t(7)
    assert lib.elitekv_stream_read_mode(FAKE, 32, FAKE, 4, C.byref(n), None) == ekv.EINVAL
    assert lib.elitekv_stream_read_mode(FAKE, 32, FAKE, -1, None, None) == ekv.EINVAL
    assert lib.elitekv_stream_read_mode(None, 32, FAKE, 0, None, None) == ekv.ENULL
    assert lib.elitekv_stream_read_mode(FAKE, 24, FAKE, 3, None, None) == ekv.EALIGN
    assert lib.elitekv_stream_read_mode(FAKE, 0, FAKE, 3, C.byref(n), None) == ekv.OK and n.value == 0


def test_slrd_argument_errors():
    d = _dims()
    dc = d.d_c
    slrd = lambda d_ck, **kw: lib.elitekv_slrd_decode_attn(
        C.byref(d), d_ck, kw.get("q", FAKE), FAKE, FAKE, kw.get("B", 1), 128, 128, FAKE, kw.get("B_v", FAKE), FAKE,
        FAKE, FAKE, 128, FAKE, FAKE, kw.get("wsb", 1 << 30), 0, None)
    assert slrd(0) == ekv.EINVAL and slrd(dc) == ekv.EINVAL and slrd(-3) == ekv.EINVAL    # 0 < d_ck < d_c
    assert slrd(dc // 2, B=0) == ekv.OK
    assert slrd(dc // 2, q=None) == ekv.ENULL
    assert slrd(dc // 2, B_v=FAKE + 4) == ekv.EALIGN
    need = ekv.elitekv_slrd_decode_workspace_bytes(d, dc // 2, 1, 128)
    assert need > 0 and slrd(dc // 2, wsb=need - 1) == ekv.EWORKSPACE
    assert ekv.elitekv_slrd_decode_workspace_bytes(d, 0, 1, 128) == 0
    app = lambda d_ck, **kw: lib.elitekv_slrd_append(C.byref(d), d_ck, FAKE, FAKE, FAKE, kw.get("T", 1), FAKE, FAKE,
                                                     kw.get("A_v", FAKE), FAKE, FAKE, FAKE, 16, FAKE, 1 << 30, None)
    assert app(0) == ekv.EINVAL and app(dc) == ekv.EINVAL
    assert app(dc // 2, T=0) == ekv.OK
    assert app(dc // 2, A_v=None) == ekv.ENULL
    # Section 3.2, S-LRD storage cost, against the oracle's statement of the same formula
    big = ekv.make_dims(4096, 32, 128, 8, 1536, "bf16")
    assert ekv.elitekv_slrd_param_count(big, 576) == orc.slrd_param_count(4096, 32, 128, 8, 576, 960)
    # the separated latents at the 7B shape take the matrix-core path only for whole wave slices
    assert ekv.elitekv_slrd_decode_workspace_bytes(big, 576, 1, 4096) < ekv.elitekv_decode_workspace_bytes(big, 1, 4096)


def test_multiquery_argument_errors():
    d = _dims()
    mq = lambda **kw: lib.elitekv_multiquery_attn(C.byref(d), kw.get("q", FAKE), FAKE, FAKE, kw.get("B", 2),
                                                  kw.get("T", 3), 128, 128, FAKE, FAKE, FAKE, FAKE, FAKE, 256, FAKE,
                                                  FAKE, kw.get("wsb", 1 << 30), 0, None)
    assert mq(T=0) == ekv.EINVAL and mq(B=-1) == ekv.EINVAL
    assert mq(B=0) == ekv.OK
    assert mq(B=300, T=300) == ekv.EUNSUPPORTED
    assert mq(q=None) == ekv.ENULL
    need = ekv.elitekv_multiquery_workspace_bytes(d, 2, 3, 128)
    assert need == ekv.elitekv_decode_workspace_bytes(d, 6, 128)       # B*T query rows
    assert mq(wsb=need - 1) == ekv.EWORKSPACE


def test_slrd_multiquery_argument_errors():
    d = _dims()
    dc = d.d_c
    mq = lambda d_ck, **kw: lib.elitekv_slrd_multiquery_attn(
        C.byref(d), d_ck, kw.get("q", FAKE), FAKE, FAKE, kw.get("B", 2), kw.get("T", 3), 128, 128, FAKE, FAKE, FAKE,
        FAKE, FAKE, 256, FAKE, FAKE, kw.get("wsb", 1 << 30), 0, None)
    assert mq(0) == ekv.EINVAL and mq(dc) == ekv.EINVAL                                  # 0 < d_ck < d_c
    assert mq(dc // 2, T=0) == ekv.EINVAL and mq(dc // 2, B=-1) == ekv.EINVAL
    assert mq(dc // 2, B=0) == ekv.OK
    assert mq(dc // 2, B=300, T=300) == ekv.EUNSUPPORTED
    assert mq(dc // 2, q=None) == ekv.ENULL
    need = ekv.elitekv_slrd_multiquery_workspace_bytes(d, dc // 2, 2, 3, 128)
    assert need == ekv.elitekv_slrd_decode_workspace_bytes(d, dc // 2, 6, 128)           # B*T query rows
    assert need > 0 and mq(dc // 2, wsb=need - 1) == ekv.EWORKSPACE
    assert ekv.elitekv_slrd_multiquery_workspace_bytes(d, 0, 2, 3, 128) == 0
    assert lib.elitekv_slrd_multiquery_attn(None, 4, FAKE, FAKE, FAKE, 1, 1, 128, 128, FAKE, FAKE, FAKE, FAKE, FAKE,
                                            256, FAKE, FAKE, 1 << 30, 0, None) == ekv.ENULL


def test_prefill_argument_errors():
    big = ekv.make_dims(4096, 32, 128, 8, 1536, "bf16")
    pf = lambda **kw: lib.elitekv_prefill_attn(C.byref(kw.get("dims", big)), kw.get("q", FAKE), FAKE, FAKE, kw.get("B", 2),
                                               kw.get("T", 300), kw.get("S", 512), 512, FAKE, kw.get("W_uv", FAKE), FAKE,
                                               FAKE, FAKE, 1024, FAKE, FAKE, kw.get("wsb", 1 << 40), None)
    assert pf(T=0) == ekv.EINVAL and pf(B=-1) == ekv.EINVAL and pf(S=-1) == ekv.EINVAL
    assert pf(B=0) == ekv.OK
    assert pf(q=None) == ekv.ENULL
    assert pf(W_uv=FAKE + 2) == ekv.EALIGN
    assert pf(B=1 << 20, T=1 << 10) == ekv.EUNSUPPORTED
    need = ekv.elitekv_prefill_attn_workspace_bytes(big, 2, 300, 512)
    # the rebuilt keys and values of 2 x 512 rows dominate: n_h (2 d_h - 2 r) bf16 elements per row
    rebuilt = 2 * 512 * 32 * (2 * 128 - 16) * 2
    assert rebuilt <= need <= rebuilt + 2 * 300 * 32 * 128 * 2 + 512 * 12 + 4 * 256
    assert pf(wsb=need - 1) == ekv.EWORKSPACE
    # shapes outside the flash path (fp32, short caches) are the several-queries call, with its limits
    d = _dims()
    assert ekv.elitekv_prefill_attn_workspace_bytes(d, 2, 3, 128) == ekv.elitekv_multiquery_workspace_bytes(d, 2, 3, 128)
    assert ekv.elitekv_prefill_attn_workspace_bytes(big, 2, 300, 64) == ekv.elitekv_multiquery_workspace_bytes(big, 2, 300, 64)
    assert pf(dims=d, B=300, T=300) == ekv.EUNSUPPORTED
    # few queries per sequence: the absorbed form is the cheaper order, the call is the several-queries call
    assert ekv.elitekv_prefill_attn_workspace_bytes(big, 2, 8, 512) == ekv.elitekv_multiquery_workspace_bytes(big, 2, 8, 512)


def test_decode_step_argument_errors():
    d = _dims()
    step = lambda **kw: lib.elitekv_decode_step(
        C.byref(d), kw.get("x", FAKE), kw.get("q", FAKE), FAKE, kw.get("slot", FAKE), FAKE, kw.get("B", 1), 128, 128,
        FAKE, FAKE, FAKE, kw.get("W_uv", FAKE), FAKE, FAKE, FAKE, 128, FAKE, FAKE, kw.get("wsb", 1 << 30), 0, None)
    assert step(B=0) == ekv.OK
    assert step(B=-1) == ekv.EINVAL
    assert step(x=None) == ekv.ENULL and step(q=None) == ekv.ENULL and step(slot=None) == ekv.ENULL
    assert step(W_uv=FAKE + 4) == ekv.EALIGN
    need = ekv.elitekv_decode_step_workspace_bytes(d, 1, 128)
    assert need > 0 and step(wsb=need - 1) == ekv.EWORKSPACE
    # the step's workspace holds the attention's and what the append needs on top
    big = ekv.make_dims(4096, 32, 128, 8, 1536, "bf16")
    for B in (1, 4, 8, 64):
        assert ekv.elitekv_decode_step_workspace_bytes(big, B, 4096) >= ekv.elitekv_decode_workspace_bytes(big, B, 4096)
    dc = d.d_c
    sstep = lambda d_ck, **kw: lib.elitekv_slrd_decode_step(
        C.byref(d), d_ck, FAKE, FAKE, FAKE, FAKE, FAKE, kw.get("B", 1), 128, 128, FAKE, FAKE, kw.get("A_v", FAKE), FAKE,
        FAKE, FAKE, FAKE, FAKE, 128, FAKE, FAKE, 1 << 30, 0, None)
    assert sstep(0) == ekv.EINVAL and sstep(dc) == ekv.EINVAL
    assert sstep(dc // 2, B=0) == ekv.OK
    assert sstep(dc // 2, A_v=None) == ekv.ENULL
    assert ekv.elitekv_slrd_decode_step_workspace_bytes(d, 0, 1, 128) == 0


def test_block_step_argument_errors():
    big = ekv.make_dims(4096, 32, 128, 8, 1536, "bf16")
    blk = lambda **kw: lib.elitekv_block_step(
        C.byref(kw.get("dims", big)), kw.get("x", FAKE), FAKE, FAKE, FAKE, kw.get("B", 1), 128, 128,
        kw.get("W_q", FAKE), FAKE, FAKE, FAKE, FAKE, kw.get("W_o", FAKE), FAKE, FAKE, FAKE, 128, FAKE, FAKE,
        kw.get("wsb", 1 << 30), 0, None)
    assert blk(B=0) == ekv.OK
    assert blk(x=None) == ekv.ENULL and blk(W_q=None) == ekv.ENULL and blk(W_o=None) == ekv.ENULL
    assert blk(W_o=FAKE + 8) == ekv.EALIGN
    need = ekv.elitekv_block_step_workspace_bytes(big, 1, 128)
    assert need > 0 and blk(wsb=need - 1) == ekv.EWORKSPACE
    # eight to 64 sequences take the composed form (projections around the decode step): same validation
    need8 = ekv.elitekv_block_step_workspace_bytes(big, 8, 128)
    assert need8 > ekv.elitekv_decode_step_workspace_bytes(big, 8, 128)
    assert blk(B=8, x=None) == ekv.ENULL and blk(B=8, W_o=None) == ekv.ENULL
    assert blk(B=8, W_q=FAKE + 8) == ekv.EALIGN
    assert blk(B=8, wsb=need8 - 1) == ekv.EWORKSPACE
    assert blk(B=65) == ekv.EUNSUPPORTED and ekv.elitekv_block_step_workspace_bytes(big, 65, 128) == 0
    assert blk(dims=_dims()) == ekv.EUNSUPPORTED                      # fp32
    # separated latents
    sblk = lambda d_ck, **kw: lib.elitekv_slrd_block_step(
        C.byref(big), d_ck, kw.get("x", FAKE), FAKE, FAKE, FAKE, kw.get("B", 2), 128, 128, FAKE, FAKE, FAKE,
        kw.get("A_v", FAKE), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 256, FAKE, FAKE, kw.get("wsb", 1 << 30), 0, None)
    assert sblk(0) == ekv.EINVAL and sblk(1536) == ekv.EINVAL
    assert sblk(576, B=0) == ekv.OK
    assert sblk(576, x=None) == ekv.ENULL and sblk(576, A_v=None) == ekv.ENULL
    needs = ekv.elitekv_slrd_block_step_workspace_bytes(big, 576, 2, 128)
    assert needs > 0 and sblk(576, wsb=needs - 1) == ekv.EWORKSPACE
    assert ekv.elitekv_slrd_block_step_workspace_bytes(big, 0, 2, 128) == 0


def test_slrd_prefill_argument_errors():
    big = ekv.make_dims(4096, 32, 128, 8, 1536, "bf16")
    pf = lambda d_ck, **kw: lib.elitekv_slrd_prefill_attn(
        C.byref(kw.get("dims", big)), d_ck, kw.get("q", FAKE), FAKE, FAKE, kw.get("B", 2), kw.get("T", 300),
        kw.get("S", 512), 512, FAKE, kw.get("B_v", FAKE), FAKE, FAKE, FAKE, 1024, FAKE, FAKE, kw.get("wsb", 1 << 40), None)
    assert pf(0) == ekv.EINVAL and pf(1536) == ekv.EINVAL
    assert pf(576, T=0) == ekv.EINVAL and pf(576, B=-1) == ekv.EINVAL
    assert pf(576, B=0) == ekv.OK
    assert pf(576, q=None) == ekv.ENULL
    assert pf(576, B_v=FAKE + 2) == ekv.EALIGN
    need = ekv.elitekv_slrd_prefill_attn_workspace_bytes(big, 576, 2, 300, 512)
    assert need == ekv.elitekv_prefill_attn_workspace_bytes(big, 2, 300, 512)             # the same rebuilt rows
    assert pf(576, wsb=need - 1) == ekv.EWORKSPACE
    assert ekv.elitekv_slrd_prefill_attn_workspace_bytes(big, 0, 2, 300, 512) == 0
    # a d_ck that is not a multiple of 32, few queries, or 12.5 % at 40 heads (n_h (d_h - 2r) not a multiple of 128):
    # the call is the several-queries call
    for dims_, d_ck, T in [(big, 584, 300), (big, 576, 8), (ekv.make_dims(5120, 40, 128, 4, 960, "bf16"), 480, 300)]:
        assert ekv.elitekv_slrd_prefill_attn_workspace_bytes(dims_, d_ck, 1, T, 512) == \
            ekv.elitekv_slrd_multiquery_workspace_bytes(dims_, d_ck, 1, T, 512)


def test_noalloc_entry_point_rejects_oversized_calls_on_the_host():
    """The scratch-size check comes before anything touches a device: a call whose workspace exceeds the
    built-in buffer is refused with ESCRATCH (no GPU needed), and bad dims keep their own codes."""
    import ctypes as C
    dims = ekv.make_dims(4096, 32, 128, 8, 1536, "bf16")
    assert ekv.elitekv_decode_workspace_bytes(dims, 1, 32768, 512) > ekv.NOALLOC_SCRATCH_BYTES
    p = 4096   # never dereferenced
    st = ekv.raw().elitekv_decode_attn_noalloc(C.byref(dims), p, p, p, 1, 32768, 32768, p, p, p, p, p, 32768, p, 512,
                                               None)
    assert st == ekv.ESCRATCH
    assert "scratch" in ekv.elitekv_strerror(st)
    bad = ekv.make_dims(4096, 32, 127, 8, 1536, "bf16")
    st = ekv.raw().elitekv_decode_attn_noalloc(C.byref(bad), p, p, p, 1, 64, 64, p, p, p, p, p, 64, p, 0, None)
    assert st == ekv.EINVAL


def test_append_rejects_head_dims_beyond_the_rope_table():
    """head_dim > 256 would index past the 128 chunk frequencies the append kernels are given:
    refused on the host (EUNSUPPORTED, the limit the decode path has), also through the S-LRD append
    and the decode step."""
    import ctypes as C
    dims = ekv.make_dims(1024, 2, 512, 4, 128, "bf16")
    p = 4096   # never dereferenced
    lib = ekv.raw()
    assert lib.elitekv_append(C.byref(dims), p, p, p, 3, p, p, p, p, p, 16, p, 1 << 20, None) == ekv.EUNSUPPORTED
    assert lib.elitekv_slrd_append(C.byref(dims), 64, p, p, p, 3, p, p, p, p, p, p, 16, p, 1 << 20, None) == ekv.EUNSUPPORTED
    assert lib.elitekv_decode_step(C.byref(dims), p, p, p, p, p, 1, 16, 16, p, p, p, p, p, p, p, 16, p, p, 1 << 20, 0,
                                   None) == ekv.EUNSUPPORTED
    ok = ekv.make_dims(1024, 2, 256, 4, 128, "bf16")
    assert lib.elitekv_append(C.byref(ok), p, p, p, 0, p, p, p, p, p, 16, p, 1 << 20, None) == ekv.OK


def test_decode_path_query_names_the_kernels_a_shape_runs():
    """elitekv_decode_path: the paper's RoPElite settings r = 4, 8, 16, 32 at hardware-friendly latent widths take
    the matrix-core kernels; fp32, other r, other widths and r = 16 with rows too wide for the LDS take the
    generic ones -- visibly, not silently (r = 32: up to d_c 1152)."""
    mk = lambda r, d_c, dt="bf16", n_h=32, d_h=128: ekv.make_dims(4096, n_h, d_h, r, d_c, dt)
    MC, GEN = ekv.PATH_MATRIX_CORE, ekv.PATH_GENERIC
    assert ekv.elitekv_decode_path(mk(8, 1536)) == MC
    assert ekv.elitekv_decode_path(mk(4, 768)) == MC
    assert ekv.elitekv_decode_path(mk(16, 1792)) == MC          # 34.4 % of the full cache at the 7B shape
    assert ekv.elitekv_decode_path(mk(16, 1024)) == MC
    assert ekv.elitekv_decode_path(mk(8, 1920, n_h=40)) == MC
    assert ekv.elitekv_decode_path(mk(16, 2048)) == GEN         # tiles + 32 elite values per head exceed the LDS
    assert ekv.elitekv_decode_path(mk(32, 1024)) == MC          # r = 32: 37.5 % of the full cache
    assert ekv.elitekv_decode_path(mk(32, 1152)) == MC
    assert ekv.elitekv_decode_path(mk(32, 2048)) == GEN         # r = 32 at 50 % cache: tiles + 64 elite values per head exceed the LDS
    assert ekv.elitekv_decode_path(mk(32, 1280)) == GEN
    assert ekv.elitekv_decode_path(mk(8, 1500)) == GEN
    assert ekv.elitekv_decode_path(mk(8, 1536, "fp32")) == GEN
    assert ekv.elitekv_decode_path(mk(8, 1536), 576) == MC      # separated latents, whole wave slices
    assert ekv.elitekv_decode_path(mk(8, 1536), 500) == GEN
    with pytest.raises(ekv.EliteKVError):
        ekv.elitekv_decode_path(mk(8, 1536, n_h=32, d_h=127))
