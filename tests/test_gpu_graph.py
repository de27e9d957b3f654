"""The library only enqueues kernels on the caller's stream (no allocation, no synchronisation, no
memset), so a decode step can be captured into a HIP graph and replayed.  The graph is replayed
several times with eager work and synchronisations in between, and every replay is checked
against the eager result."""
import numpy as np
import pytest
import torch

import elitekv_synth as synth
import paper_2503_01586_amd as ekv

from gpu_util import DEV, dev, dims_of, i32, i64
from test_gpu_parity import _draw, shape

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("B,fused", [(1, False), (8, False), (1, True), (3, True), (8, True)])
def test_append_and_decode_replay_from_a_graph(B, fused):
    sh, S = shape(512, 32, 128, 8, 1536, "bf16"), 700
    rng, idx, W_ke, W_dkv, W_uk, W_uv, x, q = _draw(sh, B, B, 123 + B)
    dims = dims_of(sh)
    ke64, c64 = synth.draw_cache_planes(rng, B * S, 32, 8, 1536)
    ke, c = dev(ke64, "bf16"), dev(c64, "bf16")
    xd, qd, Wked, Wdkvd, Wukd, Wuvd = (dev(a, "bf16") for a in (x, q, W_ke, W_dkv, W_uk, W_uv))
    idxd = i32(idx)
    pos = torch.full((B,), S - 1, dtype=torch.int32, device=DEV)
    slot = torch.arange(B, dtype=torch.int64, device=DEV) * S + (S - 1)
    seq = torch.full((B,), S, dtype=torch.int32, device=DEV)
    out = torch.zeros(B, 32, 128, dtype=torch.bfloat16, device=DEV)
    ws = torch.empty(ekv.elitekv_decode_workspace_bytes(dims, B, S), dtype=torch.uint8, device=DEV)
    aws = torch.empty(max(ekv.elitekv_append_workspace_bytes(dims, B), 16), dtype=torch.uint8, device=DEV)

    sws = torch.empty(ekv.elitekv_decode_step_workspace_bytes(dims, B, S), dtype=torch.uint8, device=DEV)

    def step(stream):
        if fused:
            ekv.elitekv_decode_step(dims, xd, qd, pos, slot, seq, S, S, Wked, Wdkvd, Wukd, Wuvd, idxd, ke, c, out, sws,
                                    stream=stream)
            return
        ekv.elitekv_append(dims, xd, pos, slot, Wked, Wdkvd, idxd, ke, c, ws=aws, stream=stream)
        ekv.elitekv_decode_attn(dims, qd, pos, seq, S, S, Wukd, Wuvd, idxd, ke, c, out, ws, stream=stream)

    step(torch.cuda.current_stream().cuda_stream)          # eager (also the first-launch set-up of the kernels)
    torch.cuda.synchronize()
    want = out.clone()

    side = torch.cuda.Stream()                             # default priority
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step(side.cuda_stream)                             # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step(torch.cuda.current_stream().cuda_stream)
    for rep in range(4):
        out.fill_(float("nan"))                            # eager work between the replays
        ws.fill_(0xFF)
        sws.fill_(0xFF)
        c[slot] = 0
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want), "replay %d differs from the eager step" % rep


def test_prefill_attention_replays_from_a_graph():
    """The prefill call is launches only (one GEMM per sequence + the flash kernel): captured and replayed."""
    sh, rows, T = shape(64, 8, 128, 8, 256, "bf16"), [300, 260], 200
    B, stride, S = 2, 310, 300
    rng, idx, _, _, W_uk, W_uv, _, _ = _draw(sh, 1, 1, 321)
    dims = dims_of(sh)
    ke64, c64 = synth.draw_cache_planes(rng, B * stride, 8, 8, 256)
    ke, c = dev(ke64, "bf16"), dev(c64, "bf16")
    qd = dev(rng.standard_normal((B, T, 8, 128)), "bf16")
    Wukd, Wuvd, idxd = dev(W_uk, "bf16"), dev(W_uv, "bf16"), i32(idx)
    q_pos = i32(np.concatenate([np.arange(n - T, n) for n in rows]))
    kv_len = q_pos + 1
    out = torch.zeros(B, T, 8, 128, dtype=torch.bfloat16, device=DEV)
    ws = torch.empty(ekv.elitekv_prefill_attn_workspace_bytes(dims, B, T, S), dtype=torch.uint8, device=DEV)

    def call(stream):
        ekv.elitekv_prefill_attn(dims, qd, q_pos, kv_len, S, stride, Wukd, Wuvd, idxd, ke, c, out, ws, stream=stream)

    call(torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    want = out.clone()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        call(side.cuda_stream)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            call(torch.cuda.current_stream().cuda_stream)
    for rep in range(3):
        out.fill_(float("nan"))
        ws.fill_(0xFF)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want), "replay %d differs from the eager call" % rep
