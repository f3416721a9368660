"""The entry point that allocates nothing (dp_norms_multi_static) against dp_norms_multi, which
takes the same kernels through a caller-provided workspace: same bits, on two calls in a row, the
second on a smaller stack, so that what the first call left in the library's static array cannot
leak into the second."""
import ctypes

import numpy as np
import pytest

import synth_inputs as si
from oracle import bk_oracle as o

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def dev(x):
    return torch.from_numpy(x.view(np.int16) if x.dtype == np.uint16 else x).cuda()


def stack(dp, B, T, dims, seed):
    w = si.small_workload("na", si.BF16, B, T, dims, data_seed=seed)
    layers = [si.gen_layer(w, l) for l in range(w.L)]
    desc = [(dev(a), dev(g), T, d, p, dp.dp_choose_path(T, d, p)) for (a, g), (d, p) in zip(layers, dims)]
    return layers, desc


def test_static_scratch_entry_point_matches_workspace_entry_point():
    import paper_2311_11822_amd.binding as dp
    # first call: ghost norm on large and small tiles and the instantiated norm, 3 samples;
    # second call: fewer, smaller layers and 2 samples
    calls = [(3, 320, [(384, 1280), (136, 264), (264, 72), (256, 640)], 7),
             (2, 96, [(128, 320), (72, 24)], 8)]
    for B, T, dims, seed in calls:
        layers, desc = stack(dp, B, T, dims, seed)
        arr = dp.layer_array(desc)
        nbytes = dp.dp_norms_multi_workspace_bytes(arr, dp.DP_BF16, B)
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        want = torch.full((len(dims), B), -1.0, dtype=torch.float32, device="cuda")
        dp.dp_norms_multi(arr, dp.DP_BF16, B, want, ws)
        got = torch.full((len(dims), B), -2.0, dtype=torch.float32, device="cuda")
        # straight through the C ABI
        st = dp.lib.dp_norms_multi_static(arr, len(arr), dp.DP_BF16, B, got.data_ptr(),
                                          torch.cuda.current_stream().cuda_stream)
        assert st == dp.DP_OK
        torch.cuda.synchronize()
        assert torch.equal(got, want)                      # same kernels, same order: same bits
        ref = np.stack([o.perex_sqnorm(si.to_f64(a), si.to_f64(g)) for a, g in layers])
        assert np.max(np.abs(got.cpu().numpy() - ref) / ref) <= 2e-3


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    import paper_2311_11822_amd.binding as dp
    x = torch.zeros(64, dtype=torch.float32, device="cuda")
    p = x.data_ptr()
    # 300000 samples x 1 tile > 262144 partial sums; refused on the host, nothing is launched
    arr = dp.layer_array([(p, p, 8, 8, 8, 0)])
    assert dp.dp_norms_multi_workspace_bytes(arr, dp.DP_BF16, 300000) > (1 << 20)
    assert dp.lib.dp_norms_multi_static(arr, 1, dp.DP_BF16, 300000, p, None) == dp.DP_ERR_WORKSPACE
    many = dp.layer_array([(p, p, 8, 8, 8, 0)] * 1025)
    assert dp.lib.dp_norms_multi_static(many, 1025, dp.DP_BF16, 1, p, None) == dp.DP_ERR_WORKSPACE
    assert dp.lib.dp_norms_multi_static(None, 1, dp.DP_BF16, 1, p, None) == dp.DP_ERR_INVALID_ARG
    assert dp.lib.dp_norms_multi_static(arr, 1, dp.DP_BF16, 1, None, None) == dp.DP_ERR_INVALID_ARG
    torch.cuda.synchronize()
    assert not x.any()
