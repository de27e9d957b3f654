"""Helpers of the GPU parity tests: move seeded arrays to the device in the I/O dtype, call the
library through its binding, and bring results back as float64 for the oracle comparison."""
import numpy as np
import torch

import paper_2503_01586_amd as ekv

DEV = "cuda:0"
TOL = {"fp32": 1e-5, "bf16": 2e-2}   # max-abs-rel bounds of the parity gates


def tdtype(name):
    return {"fp32": torch.float32, "bf16": torch.bfloat16}[name]


def dev(arr, dtype):
    """float64 numpy -> device tensor in the I/O dtype (one rounding, round-to-nearest-even)."""
    return torch.from_numpy(np.ascontiguousarray(arr)).to(tdtype(dtype)).to(DEV).contiguous()


def host64(t):
    """device tensor -> float64 numpy of exactly the stored values."""
    return t.detach().to("cpu").to(torch.float64).numpy()


def i32(a):
    return torch.as_tensor(np.asarray(a), dtype=torch.int32).to(DEV)


def i64(a):
    return torch.as_tensor(np.asarray(a), dtype=torch.int64).to(DEV)


def dims_of(cfg_or_dict, dtype=None):
    c = cfg_or_dict
    if isinstance(c, dict):
        return ekv.make_dims(c["d_model"], c["n_heads"], c["head_dim"], c["r"], c["d_c"],
                             dtype or c["dtype"], c.get("rope_base", 10000.0))
    return ekv.make_dims(c.d_model, c.n_heads, c.head_dim, c.r, c.d_c, dtype or c.dtype, c.rope_base)


def gpu_append(dims, x, pos, slot, W_ke, W_dkv, idx, plane_rows, ke=None, c=None):
    dt = ekv.torch_dtype(dims)
    if ke is None:
        ke = torch.zeros(plane_rows, dims.n_heads, 2 * dims.r, dtype=dt, device=DEV)
    if c is None:
        c = torch.zeros(plane_rows, dims.d_c, dtype=dt, device=DEV)
    nws = ekv.elitekv_append_workspace_bytes(dims, x.shape[0])
    ws = torch.empty(max(nws, 16), dtype=torch.uint8, device=DEV)
    ekv.elitekv_append(dims, x, pos, slot, W_ke, W_dkv, idx, ke, c, ws=ws)
    torch.cuda.synchronize()
    return ke, c


def gpu_decode(dims, q, q_pos, seq_len, max_seq, stride, W_uk, W_uv, idx, ke, c, n_splits=0):
    B = q.shape[0]
    out = torch.full((B, dims.n_heads, dims.head_dim), float("nan"), dtype=ekv.torch_dtype(dims), device=DEV)
    nws = ekv.elitekv_decode_workspace_bytes(dims, B, max_seq, n_splits)
    assert nws > 0
    # poison the workspace: nothing may depend on its previous contents
    ws = torch.full((nws,), 0xFF, dtype=torch.uint8, device=DEV)
    ekv.elitekv_decode_attn(dims, q, q_pos, seq_len, max_seq, stride, W_uk, W_uv, idx, ke, c, out, ws,
                            n_splits=n_splits)
    torch.cuda.synchronize()
    return out


def parity_report(name, got, ref, tol, per_row_axes=None):
    """The parity gate of one output tensor plus what the benchmark definition asks to be logged next to it:
    returns max|got - ref| / max|ref| over the tensor (the gated metric, oracle.max_abs_rel) and prints
    the largest ELEMENT-WISE relative error among the elements with |ref| > 1e-3 max|ref|, and the worst
    max-abs-rel of any single row (leading axes = rows, e.g. one (batch row, head) output vector each), so
    that a row of small magnitude cannot hide behind a large one in the same tensor."""
    from oracle import elitekv_oracle as orc
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    err = orc.max_abs_rel(got, ref)
    big = np.abs(ref) > 1e-3 * np.max(np.abs(ref)) if ref.size else np.zeros(ref.shape, dtype=bool)
    elem = float(np.max(np.abs(got - ref)[big] / np.abs(ref)[big])) if big.any() else 0.0
    rows_g, rows_r = got.reshape(-1, got.shape[-1]), ref.reshape(-1, ref.shape[-1])
    row_err = max((orc.max_abs_rel(g, r) for g, r in zip(rows_g, rows_r)), default=0.0)
    print("parity %-44s max-abs-rel %.3e (bound %.0e)  worst row %.3e  max element-wise rel (|ref| > 1e-3 max) %.3e"
          % (name, err, tol, row_err, elem), flush=True)
    return err, row_err
