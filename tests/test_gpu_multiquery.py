"""GPU parity of attention with several queries per sequence (a prefill chunk / drafted tokens)
against the float64 oracle, through the C ABI.  Bounds: 1e-5 (fp32), 2e-2 (bf16), max-abs-rel."""
import numpy as np
import pytest
import torch

import elitekv_synth as synth
import paper_2503_01586_amd as ekv
from oracle import elitekv_oracle as orc

from gpu_util import DEV, TOL, dev, dims_of, gpu_decode, host64, i32
from test_gpu_parity import _draw, shape

pytestmark = pytest.mark.gpu

CASES = {
    # name: (shape, per sequence: cached rows, T, splits)
    "fp32_tiny": (shape(64, 3, 24, 5, 37, "fp32"), [40, 7, 130], 5, [0, 2]),
    "bf16_7b_chunk_of_4": (shape(64, 32, 128, 8, 1536, "bf16"), [300, 65], 4, [0, 3]),
    "bf16_7b_chunk_of_16": (shape(64, 32, 128, 8, 1536, "bf16"), [200], 16, [0]),
    "bf16_13b_chunk_of_3": (shape(64, 40, 128, 8, 1920, "bf16"), [97, 160], 3, [0, 2]),
    "bf16_12pct_chunk_of_9": (shape(64, 32, 128, 4, 768, "bf16"), [130], 9, [0]),
}


@pytest.mark.parametrize("name", list(CASES))
def test_multiquery_matches_oracle(name):
    sh, rows, T, splits = CASES[name]
    dt = sh["dtype"]
    B, stride = len(rows), max(rows) + 2
    rng, idx, W_ke, W_dkv, W_uk, W_uv, x, _ = _draw(sh, B * stride, B, 600 + len(name))
    q = rng.standard_normal((B, T, sh["n_heads"], sh["head_dim"]))
    dims = dims_of(sh)
    pos = np.tile(np.arange(stride), B)
    ke64, c64 = orc.append(x, pos, W_ke, W_dkv, idx, sh["head_dim"], sh["rope_base"])
    ked, cd = dev(ke64, dt), dev(c64, dt)
    qd, Wukd, Wuvd = dev(q, dt), dev(W_uk, dt), dev(W_uv, dt)
    # the queries are the last T tokens of each sequence (fewer visible rows for the earlier ones);
    # a sequence shorter than the chunk leaves its first queries with nothing to see
    q_pos = np.array([[max(n - T + t, 0) for t in range(T)] for n in rows])
    kv_len = np.array([[max(n - T + t + 1, 0) for t in range(T)] for n in rows])
    ref = orc.multiquery_attn(host64(qd), q_pos, host64(ked).reshape(B, stride, sh["n_heads"], -1),
                              host64(cd).reshape(B, stride, -1), kv_len, host64(Wukd), host64(Wuvd), idx,
                              sh["head_dim"], sh["rope_base"])
    for ns in splits:
        out = torch.full((B, T, sh["n_heads"], sh["head_dim"]), float("nan"), dtype=ekv.torch_dtype(dims), device=DEV)
        nws = ekv.elitekv_multiquery_workspace_bytes(dims, B, T, max(rows), ns)
        assert nws > 0
        ws = torch.full((nws,), 0xFF, dtype=torch.uint8, device=DEV)
        ekv.elitekv_multiquery_attn(dims, qd, i32(q_pos.reshape(-1)), i32(kv_len.reshape(-1)), max(rows), stride, Wukd,
                                    Wuvd, i32(idx), ked, cd, out, ws, n_splits=ns)
        torch.cuda.synchronize()
        o = host64(out)
        assert np.all(np.isfinite(o))
        assert orc.max_abs_rel(o, ref) <= TOL[dt], "n_splits=%d" % ns
        assert np.all(o[kv_len == 0] == 0.0)


def test_one_query_per_sequence_is_the_decode_call():
    sh = shape(64, 32, 128, 8, 1536, "bf16")
    rows = [120, 77]
    B, stride = 2, 125
    rng, idx, W_ke, W_dkv, W_uk, W_uv, x, q = _draw(sh, B * stride, B, 9)
    dims = dims_of(sh)
    ke64, c64 = synth.draw_cache_planes(rng, B * stride, 32, 8, 1536)
    ked, cd, qd, Wukd, Wuvd = dev(ke64, "bf16"), dev(c64, "bf16"), dev(q, "bf16"), dev(W_uk, "bf16"), dev(W_uv, "bf16")
    q_pos, seq = i32([r - 1 for r in rows]), i32(rows)
    a = gpu_decode(dims, qd, q_pos, seq, max(rows), stride, Wukd, Wuvd, i32(idx), ked, cd)
    out = torch.empty(B, 1, 32, 128, dtype=torch.bfloat16, device=DEV)
    ws = torch.empty(ekv.elitekv_multiquery_workspace_bytes(dims, B, 1, max(rows)), dtype=torch.uint8, device=DEV)
    ekv.elitekv_multiquery_attn(dims, qd.reshape(B, 1, 32, 128), q_pos, seq, max(rows), stride, Wukd, Wuvd, i32(idx),
                                ked, cd, out, ws)
    torch.cuda.synchronize()
    assert torch.equal(out.reshape(B, 32, 128), a)
