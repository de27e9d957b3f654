"""elitekv_decode_attn_noalloc (the entry point for callers that cannot allocate): through the C ABI, against
elitekv_decode_attn on the same inputs, bit for bit (same kernels, same split plan), and against the CPU
oracle within the parity bound.  Two calls in a row share the built-in scratch buffer, the second with a
smaller input, so stale contents of the first call would show."""
import ctypes as C

import numpy as np
import pytest
import torch

import elitekv_synth as synth
import paper_2503_01586_amd as ekv
from oracle import elitekv_oracle as orc

from gpu_util import DEV, TOL, dev, dims_of, gpu_decode, host64, i32

pytestmark = pytest.mark.gpu

SHAPE = dict(d_model=256, n_heads=32, head_dim=128, r=8, d_c=1536, dtype="bf16", rope_base=10000.0)


def _case(seed, B, lens, stride):
    rng = np.random.default_rng(seed)
    sh = SHAPE
    idx = synth.draw_elite_idx(rng, sh["n_heads"], sh["head_dim"], sh["r"])
    _, _, W_uk, W_uv = synth.draw_weights(rng, sh["d_model"], sh["n_heads"], sh["head_dim"], sh["r"], sh["d_c"])
    ke, c = synth.draw_cache_planes(rng, B * stride, sh["n_heads"], sh["r"], sh["d_c"])
    q = synth.draw_query(rng, B, sh["n_heads"], sh["head_dim"])
    return idx, W_uk, W_uv, ke, c, q, np.asarray(lens, dtype=np.int32)


def _run_both(seed, B, lens, stride):
    dims = dims_of(SHAPE)
    idx, W_uk, W_uv, ke, c, q, lens = _case(seed, B, lens, stride)
    dt = "bf16"
    d = dict(q=dev(q, dt), W_uk=dev(W_uk, dt), W_uv=dev(W_uv, dt), ke=dev(ke, dt), c=dev(c, dt))
    idx_d, len_d, pos_d = i32(idx), i32(lens), i32(np.maximum(lens - 1, 0))
    max_seq = int(lens.max())
    assert 0 < ekv.elitekv_decode_workspace_bytes(dims, B, max_seq) <= ekv.NOALLOC_SCRATCH_BYTES
    print("no-alloc case: seed %d B %d lens %s" % (seed, B, lens.tolist()), flush=True)
    out_na = torch.full((B, SHAPE["n_heads"], SHAPE["head_dim"]), float("nan"), dtype=torch.bfloat16, device=DEV)
    ekv.elitekv_decode_attn_noalloc(dims, d["q"], pos_d, len_d, max_seq, stride, d["W_uk"], d["W_uv"], idx_d,
                                    d["ke"], d["c"], out_na)
    torch.cuda.synchronize()
    out_ws = gpu_decode(dims, d["q"], pos_d, len_d, max_seq, stride, d["W_uk"], d["W_uv"], idx_d, d["ke"], d["c"])
    assert torch.equal(out_na.view(torch.int16), out_ws.view(torch.int16)), "differs from elitekv_decode_attn"
    ref = orc.decode_attn(host64(d["q"]), np.maximum(lens - 1, 0),
                          host64(d["ke"]).reshape(B, stride, SHAPE["n_heads"], 2 * SHAPE["r"]),
                          host64(d["c"]).reshape(B, stride, SHAPE["d_c"]), lens, host64(d["W_uk"]),
                          host64(d["W_uv"]), idx, SHAPE["head_dim"], SHAPE["rope_base"])
    err = orc.max_abs_rel(host64(out_na), ref)
    assert err <= TOL["bf16"], err


def test_noalloc_two_calls_second_smaller():
    # first call: three sequences, several tiles and a ragged tail each, many splits in the scratch;
    # second call: one short sequence (fewer splits, fewer rows): it must not see the first call's partials
    _run_both(7001, 3, [700, 333, 1], 704)
    _run_both(7002, 1, [45], 48)


def test_noalloc_rejects_what_does_not_fit():
    dims = dims_of(SHAPE)
    B, S, splits = 1, 32768, 512        # 512 splits x 98 KB of partials: beyond the built-in buffer
    assert ekv.elitekv_decode_workspace_bytes(dims, B, S, splits) > ekv.NOALLOC_SCRATCH_BYTES
    p = torch.zeros(16, dtype=torch.uint8, device=DEV).data_ptr()
    st = ekv.raw().elitekv_decode_attn_noalloc(C.byref(dims), p, p, p, B, S, S, p, p, p, p, p, B * S, p, splits, None)
    assert st == ekv.ESCRATCH
