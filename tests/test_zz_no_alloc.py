"""mx_linear_static_workspace (the entry point that allocates nothing) against mx_linear, through the C ABI."""
import numpy as np
import pytest
import torch

from paper_2307_15517_amd import inputs, mx

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def run_pair(M, K, N, block, wx, ww, seed):
    """The same call through both entry points; returns (mx_linear's Y, the static-workspace entry point's Y)."""
    rng = np.random.default_rng(seed)
    x = torch.from_numpy(rng.standard_normal((M, K)).astype(np.float32)).to(DEV)
    wt = torch.from_numpy((rng.standard_normal((N, K)) * 0.02).astype(np.float32)).to(DEV)
    fa, fb = mx.fmt(block, wx), mx.fmt(block, ww)
    B = mx.quantize_pack(wt, fb, mx.MX_LAYOUT_FRAGMENT)
    ws = mx.linear_workspace(M, K, N, fa, fb, DEV)
    y_ref = torch.full((M, N), 3.0, dtype=torch.float32, device=DEV)
    y_new = torch.full((M, N), 5.0, dtype=torch.float32, device=DEV)
    mx.mx_linear(x, M, K, K, fa, ws, B, N, fb, mx.MX_LAYOUT_FRAGMENT, y_ref, N)
    mx.mx_linear_static_workspace(x, M, K, K, fa, B, N, fb, mx.MX_LAYOUT_FRAGMENT, y_new, N)
    torch.cuda.synchronize()
    return y_ref, y_new


def test_static_workspace_entry_point_matches_mx_linear_on_two_calls_in_a_row():
    """Two calls in a row share the library's one device array, the second with a smaller input: each must give
    the bits of mx_linear with a caller-owned workspace (same kernels, same order of additions).  Then the other
    routes of mx_linear (one row: no exchange between workgroups; unaligned rows: two launches) and the rejection
    of a shape whose workspace exceeds the array."""
    assert mx.mx_linear_static_workspace_max() == 8 << 20
    for (M, K, N) in ((8, 5120, 5120), (4, 1024, 300)):                       # K slices of several workgroups; smaller
        y_ref, y_new = run_pair(M, K, N, 16, 8, 4, seed=M)
        assert torch.equal(y_ref, y_new), (M, K, N)
    for (M, K, N, block) in ((1, 2048, 512, 16), (6, 32 * 40, 200, 32)):
        y_ref, y_new = run_pair(M, K, N, block, 8, 4, seed=10 + M)
        assert torch.equal(y_ref, y_new), (M, K, N)
    # rows that are not 16-byte aligned take the two-launch form, whose packed activations live in the array too
    rng = np.random.default_rng(5)
    xp = torch.from_numpy(rng.standard_normal((5, 640 + 4)).astype(np.float32)).to(DEV)
    wt = torch.from_numpy((rng.standard_normal((96, 640)) * 0.02).astype(np.float32)).to(DEV)
    fa, fb = mx.fmt(16, 8), mx.fmt(16, 4)
    B = mx.quantize_pack(wt, fb, mx.MX_LAYOUT_FRAGMENT)
    ws = mx.linear_workspace(5, 640, 96, fa, fb, DEV)
    ya = torch.zeros((5, 96), dtype=torch.float32, device=DEV)
    yb = torch.ones((5, 96), dtype=torch.float32, device=DEV)
    mx.mx_linear(xp[:, 1:641], 5, 640, 644, fa, ws, B, 96, fb, mx.MX_LAYOUT_FRAGMENT, ya, 96)
    mx.mx_linear_static_workspace(xp[:, 1:641], 5, 640, 644, fa, B, 96, fb, mx.MX_LAYOUT_FRAGMENT, yb, 96)
    torch.cuda.synchronize()
    assert torch.equal(ya, yb)
    # a shape that needs more than the array: refused before any launch (pointers are never dereferenced)
    big_n = 131072
    assert mx.mx_linear_workspace_bytes(8, 16384, big_n, fa, fb) > mx.mx_linear_static_workspace_max()
    assert mx.mx_linear_static_workspace(256, 8, 16384, 16384, fa, 512, big_n, fb, mx.MX_LAYOUT_FRAGMENT, 1024, big_n,
                                         check=False) == mx.MX_ERR_UNSUPPORTED
    assert mx.mx_linear_static_workspace(0, 8, 1024, 1024, fa, 512, 64, fb, mx.MX_LAYOUT_FRAGMENT, 1024, 64,
                                         check=False) == mx.MX_ERR_BAD_ARG
