"""Host-only checks of the C-ABI library (no GPU): it loads, exports every symbol the header
declares, and its pure host functions and argument validation behave as documented."""
import os
import re

import numpy as np
import pytest

import synth_inputs as si
from oracle import bk_oracle as o

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def dp():
    import paper_2311_11822_amd.binding as b
    return b


def declared_functions():
    text = open(os.path.join(ROOT, "include", "dp_bk.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dp_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(dp):
    names = declared_functions()
    assert {"dp_ghost_norm", "dp_perex_norm", "dp_clip_factors", "dp_clipped_grad", "dp_add_noise"} <= set(names)
    for name in names:
        assert hasattr(dp.lib, name), name
    assert sorted(dp.EXPORTS) == names          # the binding covers the whole header


def test_status_strings(dp):
    seen = {dp.lib.dp_status_string(s) for s in range(5)}
    assert len(seen) == 5 and all(seen)
    assert dp.dp_version() >= 100


def test_path_rule_matches_oracle_reading(dp):
    for w in si.WORKLOADS.values():
        for d, p in w.layers:
            assert dp.dp_choose_path(w.T, d, p) == o.choose_path(w.T, d, p)
    for T, d, p in [(8, 16, 8), (8, 16, 7), (1, 1, 2), (1, 1, 1), (3037000500, 2 ** 31, 2 ** 31), (2 ** 31, 2 ** 31, 2 ** 31)]:
        assert dp.dp_choose_path(T, d, p) == o.choose_path(T, d, p), (T, d, p)


def test_workspace_sizes(dp):
    assert dp.dp_norm_workspace_bytes(0, 1, 16, 256, 768, 2304) >= 16 * 4      # at least one partial per sample
    assert dp.dp_norm_workspace_bytes(0, 1, 0, 256, 768, 2304) == 0
    assert dp.dp_norm_workspace_bytes(0, 1, 1, 256, 12, 8) == 0       # bf16 row not a multiple of 16 B
    assert dp.dp_norm_workspace_bytes(1, 0, 4, 8, 16, 16) > 0
    layers = [(None, None, 256, 768, 768, 0), (None, None, 256, 768, 3072, 1)]
    both = dp.dp_norms_multi_workspace_bytes(layers, 1, 16)
    assert both == sum(dp.dp_norm_workspace_bytes(path, 1, 16, T, d, p) for _, _, T, d, p, path in layers)


def test_validation_refuses_before_any_launch(dp):
    lib, INV = dp.lib, dp.DP_ERR_INVALID_ARG
    fake = 0x1000                     # never dereferenced: every call below fails validation
    assert lib.dp_ghost_norm(None, fake, 1, 1, 8, 8, 8, fake, fake, 64, None) == INV
    assert lib.dp_perex_norm(fake, fake, 1, 1, 8, 8, 8, None, fake, 64, None) == INV
    assert lib.dp_ghost_norm(fake, fake, 1, 1, 8, 8, 8, fake, None, 0, None) == dp.DP_ERR_WORKSPACE
    assert lib.dp_clip_factors(fake, 0, 1, 0, 1.0, 0.01, fake, None, None) == INV
    assert lib.dp_clip_factors(fake, 1, 1, 0, -1.0, 0.01, fake, None, None) == INV
    assert lib.dp_clipped_grad(fake, fake, 1, 1, 8, 8, 8, fake, None, 0, None) == INV
    assert lib.dp_add_noise(fake, 0, 16, float("nan"), 1.0, 0, 0, None) == INV
    assert lib.dp_add_noise(fake, 0, 16, 0.0, float("inf"), 0, 0, None) == dp.DP_OK   # sigma = 0: no-op
    assert lib.dp_philox_blocks(None, 0, 4, 0, 0, None) == INV
    with pytest.raises(dp.DpError):
        dp.dp_clip_factors(fake, 1, 1, 5, 1.0, 0.01, fake, stream=0)


def test_validation_of_the_later_entry_points(dp):
    import ctypes as C
    lib, INV = dp.lib, dp.DP_ERR_INVALID_ARG
    fake = 0x1000                     # never dereferenced: every call below fails validation
    arr = dp.layer_array([(fake, fake, 8, 8, 8, 0)])
    gp = (C.c_void_p * 1)(fake)
    offs = (C.c_uint64 * 1)(0)
    # fp16 is a storage type like bf16: rows must be multiples of 16 bytes
    assert dp.dp_norm_workspace_bytes(0, dp.DP_F16, 4, 256, 768, 768) == dp.dp_norm_workspace_bytes(0, dp.DP_BF16, 4, 256, 768, 768)
    assert dp.dp_norm_workspace_bytes(0, dp.DP_F16, 1, 256, 12, 8) == 0
    assert dp.dp_norm_workspace_bytes(0, 3, 4, 256, 768, 768) == 0                   # unknown dtype
    # gradients with noise
    assert lib.dp_clipped_grad_noise_multi(arr, 1, 1, 1, fake, gp, None, 0, 0, 16, 1.0, 1.0, 0, 0, None) == INV
    assert lib.dp_clipped_grad_noise_multi(arr, 1, 1, 1, fake, gp, offs, 0, 0, 16, float("nan"), 1.0, 0, 0, None) == INV
    assert lib.dp_clipped_grad_noise_multi(arr, 1, 1, 1, fake, gp, offs, 0, 0, 16, 1.0, 0.0, 0, 0, None) == INV
    assert lib.dp_clipped_grad_noise_multi(arr, 1, 1, 1, fake, gp, offs, 0, 2 ** 64 - 1, 2, 1.0, 1.0, 0, 0, None) == INV
    assert lib.dp_clipped_grad_noise_multi(arr, 1, 1, 0, fake, gp, offs, 0, 0, 16, 1.0, 1.0, 0, 0, None) == INV   # B = 0
    # group-wise clipping
    begin, R = (C.c_int32 * 3)(0, 1, 2), (C.c_float * 2)(1.0, 1.0)
    assert lib.dp_clip_factors_grouped(fake, 2, 4, begin, 2, R, 0, 0.01, None, None, None) == INV
    assert lib.dp_clip_factors_grouped(fake, 2, 4, None, 2, R, 0, 0.01, fake, None, None) == INV
    bad_begin = (C.c_int32 * 3)(0, 2, 1)                                            # not monotone
    assert lib.dp_clip_factors_grouped(fake, 2, 4, bad_begin, 2, R, 0, 0.01, fake, None, None) == INV
    bad_R = (C.c_float * 2)(1.0, -1.0)
    assert lib.dp_clip_factors_grouped(fake, 2, 4, begin, 2, bad_R, 0, 0.01, fake, None, None) == INV
    gol = (C.c_int32 * 1)(3)                                                         # group out of range
    assert lib.dp_clipped_grad_grouped(arr, 1, 1, 1, fake, gol, 2, gp, 0, None) == INV
    assert dp.dp_group_noise_threshold([3.0, 4.0]) == 5.0
    # bias
    assert lib.dp_bias_norm(None, 1, 1, 8, 8, fake, fake, None) == INV
    assert lib.dp_bias_norm(fake, 1, 1, 8, 12, fake, fake, None) == INV             # 16-bit row not 16 B
    assert lib.dp_clipped_bias_grad(fake, 1, 8, None, fake, 0, None) == INV
    assert lib.dp_clipped_bias_grad(fake, 1, 8, fake, fake, 2, None) == INV


# ----------------------------------------------------------------------------
# tile orders of the large-tile kernels: every tile exactly once, for any shape
# ----------------------------------------------------------------------------

GRAD_SHAPES = sorted({(d, p) for w in si.WORKLOADS.values() for d, p in w.layers if d >= 128} |
                     {(136, 264), (4360, 3848), (1800, 1544), (256, 256), (257, 255), (12288, 256), (256, 49152),
                      (4352, 8448), (8704, 4352), (17 * 256, 33 * 256), (70 * 256 - 8, 41 * 256 + 8)})


@pytest.mark.parametrize("d,p", GRAD_SHAPES)
def test_gradient_tile_order_is_a_bijection(dp, d, p):
    r, c = dp.dp_clipped_grad_tile_order(d, p)
    tiles_m, tiles_n = -(-d // 256), -(-p // 256)
    assert len(r) == tiles_m * tiles_n
    assert np.all(r % 256 == 0) and np.all(c % 256 == 0)
    seen = np.zeros((tiles_m, tiles_n), dtype=np.int64)
    np.add.at(seen, (r // 256, c // 256), 1)
    assert np.all(seen == 1)


def test_gradient_tile_order_keeps_patches_together(dp):
    # the 32 tiles one XCD takes in a round (workgroups x, x + 8, ... of a run of 256) form a
    # patch of at most 4 tile rows x 8 tile columns
    r, c = dp.dp_clipped_grad_tile_order(12288, 36864)
    for base in (0, 256, 256 * 13):
        for x in range(8):
            ids = base + x + 8 * np.arange(32)
            rows, cols = np.unique(r[ids] // 256), np.unique(c[ids] // 256)
            assert len(rows) <= 4 and len(cols) <= 8 and len(rows) * len(cols) == 32


@pytest.mark.parametrize("T,B", [(2048, 4), (512, 8), (256, 16), (96, 3), (130, 2), (300, 2), (1024, 3), (1025, 3),
                                 (1152, 2), (2049, 1), (3000, 2), (4096, 2), (5000, 1), (8192, 1), (2304, 5)])
def test_ghost_tile_order_is_a_bijection(dp, T, B):
    sample, r0, c0, slot = dp.dp_ghost_tile_order(T, B)
    nj, ni = -(-T // 128), -(-T // 256)
    tps = sum(nj - 2 * I for I in range(ni))
    assert len(sample) == B * tps
    I, J = r0 // 256, c0 // 128
    assert np.all((sample >= 0) & (sample < B) & (I >= 0) & (I < ni) & (J >= 2 * I) & (J < nj))
    seen = np.zeros((B, ni, nj), dtype=np.int64)
    np.add.at(seen, (sample, I, J), 1)
    want = np.zeros((ni, nj), dtype=np.int64)
    for i in range(ni):
        want[i, 2 * i:] = 1
    assert np.all(seen == want[None])
    # partial-sum slots: each used once, and a sample's slots are contiguous
    assert sorted(slot.tolist()) == list(range(B * tps))
    assert np.all(slot // tps == sample)
