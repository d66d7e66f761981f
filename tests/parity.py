"""Helpers shared by the GPU parity tests: move seeded inputs to the device, compare with the
fp64 oracle.  Tolerances (normalised by the sum of absolute terms of each output element):
2e-3 for 16-bit inputs, 1e-5 for fp32 inputs."""
import numpy as np
import torch

from paper_2412_12218_amd import binding as B

TOL = {torch.float32: 1e-5, torch.float16: 2e-3, torch.bfloat16: 2e-3}
# half an ulp of a 16-bit output, relative to the value itself
OUT_ROUND = {torch.float32: 0.0, torch.float16: 2.0 ** -11, torch.bfloat16: 2.0 ** -8}
# ... and half the spacing of fp16 subnormals for outputs below the smallest normal fp16 number
OUT_ROUND_ABS = {torch.float32: 0.0, torch.float16: 2.0 ** -25, torch.bfloat16: 0.0}


def dev_graph(g):
    return B.Graph.from_numpy(g.row_ptr, g.col_idx)


def quantise(x32, dtype):
    """float32 numpy -> (torch tensor of `dtype` on the GPU, exact fp64 numpy of the rounded values)"""
    t = torch.from_numpy(np.ascontiguousarray(x32)).to(dtype)
    return t.cuda(), t.double().numpy()


def norm_err(got, ref, ab, out_dtype=torch.float32):
    """max |got - ref| / (abs-sum of terms), after removing the output rounding allowance."""
    got = got.detach().cpu().double().numpy()
    diff = np.abs(got - ref) - np.maximum(OUT_ROUND[out_dtype] * np.abs(ref), OUT_ROUND_ABS[out_dtype])
    scale = np.where(ab > 0, ab, 1.0)
    # where no term contributes the result must be exactly zero
    assert np.all(got[ab == 0] == 0)
    return float(np.max(np.maximum(diff, 0) / scale)) if diff.size else 0.0


def rel_err(got, ref):
    got = got.detach().cpu().double().numpy()
    return float(np.max(np.abs(got - ref) / np.abs(ref))) if ref.size else 0.0


def check_windows(win, ref):
    assert np.array_equal(win.edge_to_row.cpu().numpy(), ref["edge_to_row"])
    assert np.array_equal(win.edge_to_col.cpu().numpy(), ref["edge_to_col"])
    assert np.array_equal(win.block_partition.cpu().numpy(), ref["block_partition"])
    assert np.array_equal(win.win_col_ptr.cpu().numpy(), ref["win_col_ptr"])
    su = win.summary.cpu().numpy()
    assert np.array_equal(su, ref["summary"])
    assert np.array_equal(win.win_cols.cpu().numpy()[:int(su[0])], ref["win_cols"])
