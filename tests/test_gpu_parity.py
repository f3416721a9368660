"""GPU parity: every C-ABI entry point against the CPU oracle on the same seeded inputs.

Tolerances (stated by the task's acceptance rule): Philox integers bit-exact; fp32 paths 1e-5
relative; bf16-in/fp32-accumulate 2e-3 relative on norms and 1e-2 relative Frobenius on gradients
(measured before noise); normals |z_gpu - z_ref| <= 1e-5 max(1, |z_ref|).
"""
import math

import numpy as np
import pytest

import synth_inputs as si
from oracle import bk_oracle as o

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

TOL_F32 = 1e-5
TOL_BF16_NORM = 2e-3
TOL_BF16_GRAD = 1e-2
TOL_Z = 1e-5


@pytest.fixture(scope="module")
def dp():
    import paper_2311_11822_amd.binding as b
    return b


@pytest.fixture(scope="module")
def Pipe():
    from paper_2311_11822_amd.pipeline import BkPipeline
    return BkPipeline


def dev(x: np.ndarray):
    if x.dtype == np.uint16:
        return torch.from_numpy(x.view(np.int16)).cuda()
    return torch.from_numpy(x).cuda()


def dt_of(dp, dtype):
    return {si.F32: dp.DP_F32, si.BF16: dp.DP_BF16, si.F16: dp.DP_F16}[dtype]


HALF_TYPES = [si.BF16, si.F16]


def host(t) -> np.ndarray:
    torch.cuda.synchronize()
    return t.detach().cpu().numpy()


def rel(got, want):
    got, want = np.asarray(got, dtype=np.float64), np.asarray(want, dtype=np.float64)
    return np.max(np.abs(got - want) / np.maximum(np.abs(want), 1e-300))


def frob(got, want):
    got, want = np.asarray(got, dtype=np.float64), np.asarray(want, dtype=np.float64)
    return np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300)


def gen(w):
    return [si.gen_layer(w, l) for l in range(w.L)]


# ----------------------------------------------------------------------------
# noise generator
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("seed,step,first,n", [
    (1, 0, 0, 100000),
    (0, 0, 0, 1),
    (0xDEADBEEFCAFEF00D, 7, 12345, 4099),
    (3, (1 << 40) + 5, (1 << 32) - 1000, 2000),       # block index crosses 2^32
    (2 ** 64 - 1, 2 ** 64 - 1, 2 ** 40 + 1, 513),
])
def test_philox_stream_bit_exact(dp, seed, step, first, n):
    out = torch.zeros(4 * n, dtype=torch.int32, device="cuda")
    dp.dp_philox_blocks(out, first, n, seed, step)
    got = host(out).view(np.uint32).reshape(n, 4)
    np.testing.assert_array_equal(got, o.philox_blocks(seed, step, first, n))


@pytest.mark.parametrize("offset,count,pad", [
    (0, 1 << 20, 0), (0, 4, 0), (5, 1, 3), (3, 1021, 1), (1 << 34, 4096, 0), (7, 65537, 2), (1, 2, 0),
])
def test_normals_match_oracle_and_stay_in_slice(dp, offset, count, pad):
    # A zero buffer with sigma*R = 1 returns z itself.  `pad` shifts the slice's address so both
    # the float4 and the scalar kernels are exercised.
    guard = 8
    buf = torch.zeros(count + 2 * guard + pad, dtype=torch.float32, device="cuda")
    view = buf[guard + pad: guard + pad + count]
    dp.dp_add_noise(view, offset, count, 0.5, 2.0, 1, 0)
    got = host(buf)
    want = o.normals(1, 0, offset, count)
    z = got[guard + pad: guard + pad + count].astype(np.float64)
    assert np.all(np.abs(z - want) <= TOL_Z * np.maximum(1.0, np.abs(want)))
    assert np.all(got[:guard + pad] == 0) and np.all(got[guard + pad + count:] == 0)


def test_noise_adds_with_level_and_splits(dp):
    n = 100003
    base = np.random.default_rng(3).standard_normal(n).astype(np.float32)
    one = dev(base.copy())
    dp.dp_add_noise(one, 40, n, 0.8, 1.5, 9, 2)
    two = dev(base.copy())
    k = 33333
    dp.dp_add_noise(two, 40, k, 0.8, 1.5, 9, 2)
    dp.dp_add_noise(two.data_ptr() + 4 * k, 40 + k, n - k, 0.8, 1.5, 9, 2)
    a, b = host(one), host(two)
    np.testing.assert_array_equal(a, b)                  # any split draws the same noise
    want = o.add_noise(base, 40, 0.8, 1.5, 9, 2)
    assert np.all(np.abs(a.astype(np.float64) - want) <= 1.2 * TOL_Z * np.maximum(1.0, np.abs(want)))
    # sigma = 0 is the non-private case: untouched, even with R = inf
    three = dev(base.copy())
    dp.dp_add_noise(three, 0, n, 0.0, math.inf, 9, 2)
    np.testing.assert_array_equal(host(three), base)


def test_noise_statistics_large(dp):
    n = 1 << 24
    buf = torch.zeros(n, dtype=torch.float32, device="cuda")
    dp.dp_add_noise(buf, 0, n, 1.0, 1.0, 1, 0)
    m, v = float(buf.double().mean()), float(buf.double().var())
    assert abs(m) < 5 / math.sqrt(n) and abs(v - 1) < 5 * math.sqrt(2 / n)
    assert float(buf.abs().max()) <= 5.78


# ----------------------------------------------------------------------------
# clip factors
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("L,B", [(1, 1), (5, 9), (144, 16), (3, 700)])
def test_clip_factors(dp, mode, L, B):
    rng = np.random.default_rng(L * 1000 + B)
    sqn = rng.uniform(0, 4.0 / L, size=(L, B)).astype(np.float32)
    sqn[:, 0] = 0.0
    if B > 2:
        sqn[:, 1] = 1e-9
        sqn[0, 2] = -1e-3 if L == 1 else sqn[0, 2]
    for R in (0.7, 1.0, math.inf):
        if mode == 1 and math.isinf(R):
            continue
        Cd = torch.zeros(B, dtype=torch.float32, device="cuda")
        nd = torch.zeros(B, dtype=torch.float32, device="cuda")
        dp.dp_clip_factors(dev(sqn), L, B, mode, R, 0.01, Cd, nd)
        C, norm = o.clip_factors(sqn.astype(np.float64), mode, R, 0.01)
        np.testing.assert_allclose(host(nd), norm, rtol=TOL_F32, atol=1e-30)
        np.testing.assert_allclose(host(Cd), C, rtol=TOL_F32)


# ----------------------------------------------------------------------------
# fp32 kernels (cfg0 and ragged shapes)
# ----------------------------------------------------------------------------

F32_SHAPES = [(4, 8, 16, 16), (1, 1, 1, 1), (3, 5, 7, 11), (2, 37, 50, 13), (5, 17, 3, 64)]


@pytest.mark.parametrize("B,T,d,p", F32_SHAPES)
def test_fp32_entry_points(dp, B, T, d, p):
    w = si.small_workload("f32", si.F32, B, T, [(d, p)])
    a, g = si.gen_layer(w, 0)
    a64, g64 = si.to_f64(a), si.to_f64(g)
    ad, gd = dev(a), dev(g)
    want = o.perex_sqnorm(a64, g64)
    for fn in (dp.dp_ghost_norm, dp.dp_perex_norm):
        out = torch.zeros(B, dtype=torch.float32, device="cuda")
        fn(ad, gd, dp.DP_F32, B, T, d, p, out, None)
        assert rel(host(out), want) <= TOL_F32
    C = np.random.default_rng(1).uniform(0.0, 1.0, B)
    C[0] = 0.0
    grad = torch.full((d, p), 7.0, dtype=torch.float32, device="cuda")
    Cd = dev(C.astype(np.float32))
    dp.dp_clipped_grad(ad, gd, dp.DP_F32, B, T, d, p, Cd, grad, 0)
    G = o.clipped_grad(a64, g64, C.astype(np.float32).astype(np.float64))
    assert frob(host(grad), G) <= TOL_F32
    dp.dp_clipped_grad(ad, gd, dp.DP_F32, B, T, d, p, Cd, grad, 1)
    assert frob(host(grad), 2 * G) <= TOL_F32


def test_cfg0_pipeline_both_paths(dp, Pipe):
    w = si.WORKLOADS["cfg0"]
    layers = gen(w)
    l64 = [(si.to_f64(a), si.to_f64(g)) for a, g in layers]
    off, cnt = w.noise_range()
    Cs = []
    for path in (dp.DP_PATH_GHOST, dp.DP_PATH_PEREX):
        ref = o.private_gradient(l64, w.clip_mode, w.R, w.sigma, w.stability, w.noise_seed,
                                 w.noise_step, off, cnt, force_path=path)
        pipe = Pipe([(dev(a), dev(g)) for a, g in layers], paths=[path])
        pipe.norms()
        pipe.clip(w.clip_mode, w.R, w.stability)
        pipe.grad()
        assert rel(host(pipe.sqnorm), ref["sqnorm"]) <= TOL_F32
        assert rel(host(pipe.C), ref["C"]) <= TOL_F32
        assert frob(host(pipe.grads[0]), ref["grads"][0]) <= TOL_F32
        pipe.noise(w.sigma, w.R, w.noise_seed, w.noise_step, off, cnt)
        np.testing.assert_allclose(host(pipe.flat), ref["flat"], rtol=0, atol=2e-5)
        Cs.append(host(pipe.C))
    np.testing.assert_allclose(Cs[0], Cs[1], rtol=TOL_F32)


# ----------------------------------------------------------------------------
# bf16 matrix-core kernels: small ragged shapes spanning several tiles
# ----------------------------------------------------------------------------

BF16_SHAPES = [
    (2, 8, 16, 16),          # far smaller than one tile
    (3, 130, 72, 264),       # ragged T, widths not multiples of the k-step
    (2, 300, 136, 520),      # 3 token tiles, tile edges inside d and p
    (1, 257, 8, 8),          # minimum widths
    (5, 64, 392, 24),
    (2, 513, 256, 256),      # exact tile multiples plus one token
    # T a multiple of 32 and widths >= 128: the large-tile gradient kernels
    (3, 160, 136, 264),      # 2 tiles, all computed as 64 x 64 sub-tiles; edges inside sub-tiles
    (2, 96, 392, 520),       # 6 tiles (sub-tile kernel), sub-tiles wholly past the edge
    (2, 64, 1800, 1544),     # 56 tiles: one short round of 256 x 256 tiles, ragged edges
    (2, 32, 4360, 3848),     # 288 tiles: a full round of large tiles plus 32 tiles of sub-tiles
    # 129 .. 256 tokens and widths that are multiples of 64: the ghost norm with one workgroup per sample
    (3, 200, 128, 320),      # ragged T: token rows 200 .. 255 are zero-filled
    (2, 256, 64, 64),        # one k-block per operand
    (2, 129, 192, 448),      # one token past the single-tile case
]


@pytest.mark.parametrize("dtype", HALF_TYPES)
@pytest.mark.parametrize("B,T,d,p", BF16_SHAPES)
def test_bf16_norms(dp, B, T, d, p, dtype):
    w = si.small_workload("b", dtype, B, T, [(d, p)])
    DT = dt_of(dp, dtype)
    a, g = si.gen_layer(w, 0)
    a64, g64 = si.to_f64(a), si.to_f64(g)
    want = o.perex_sqnorm(a64, g64)
    np.testing.assert_allclose(o.ghost_sqnorm(a64, g64), want, rtol=1e-9)
    ad, gd = dev(a), dev(g)
    for path, fn in ((dp.DP_PATH_GHOST, dp.dp_ghost_norm), (dp.DP_PATH_PEREX, dp.dp_perex_norm)):
        nbytes = dp.dp_norm_workspace_bytes(path, DT, B, T, d, p)
        assert nbytes > 0
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        out = torch.full((B,), -1.0, dtype=torch.float32, device="cuda")
        fn(ad, gd, DT, B, T, d, p, out, ws)
        assert rel(host(out), want) <= TOL_BF16_NORM, (path, host(out), want)
        first = host(out).copy()
        fn(ad, gd, DT, B, T, d, p, out, ws)
        np.testing.assert_array_equal(host(out), first)       # deterministic


@pytest.mark.parametrize("dtype", HALF_TYPES)
@pytest.mark.parametrize("B,T,d,p", BF16_SHAPES)
def test_bf16_clipped_grad(dp, B, T, d, p, dtype):
    w = si.small_workload("b", dtype, B, T, [(d, p)])
    DT = dt_of(dp, dtype)
    a, g = si.gen_layer(w, 0)
    a64, g64 = si.to_f64(a), si.to_f64(g)
    C = np.random.default_rng(2).uniform(1e-3, 1.0, B).astype(np.float32)
    if B > 2:
        C[1] = 0.0                       # a masked sample
        C[2] = 1.0
    ad, gd, Cd = dev(a), dev(g), dev(C)
    grad = torch.full((d, p), 3.0, dtype=torch.float32, device="cuda")
    dp.dp_clipped_grad(ad, gd, DT, B, T, d, p, Cd, grad, 0)
    G = o.clipped_grad(a64, g64, C.astype(np.float64))
    assert frob(host(grad), G) <= TOL_BF16_GRAD
    assert frob(host(grad), G) <= 1e-5          # products are exact: only fp32 summation differs
    dp.dp_clipped_grad(ad, gd, DT, B, T, d, p, Cd, grad, 1)
    assert frob(host(grad), 2 * G) <= 1e-5
    # all factors zero: the gradient is zero (overwrite) and unchanged (accumulate)
    Z = torch.zeros(B, dtype=torch.float32, device="cuda")
    before = host(grad).copy()
    dp.dp_clipped_grad(ad, gd, DT, B, T, d, p, Z, grad, 1)
    np.testing.assert_array_equal(host(grad), before)
    dp.dp_clipped_grad(ad, gd, DT, B, T, d, p, Z, grad, 0)
    assert not host(grad).any()


@pytest.mark.parametrize("B,T,d,p", [(4, 64, 264, 136), (4, 32, 1800, 1544), (5, 50, 72, 264)])
@pytest.mark.parametrize("pattern", ["first_zero", "last_zero", "one_left", "all_equal", "two_equal_runs"])
def test_weight_patterns(dp, B, T, d, p, pattern):
    # zero weights skip their samples (also at the ends of the batch); equal consecutive weights
    # take the path that leaves the accumulator as it is
    w = si.small_workload("wp", si.BF16, B, T, [(d, p)])
    a, g = si.gen_layer(w, 0)
    C = np.random.default_rng(3).uniform(0.05, 1.0, B).astype(np.float32)
    if pattern == "first_zero":
        C[0] = 0.0
    elif pattern == "last_zero":
        C[-1] = 0.0
    elif pattern == "one_left":
        C[:] = 0.0
        C[B // 2] = 0.37
    elif pattern == "all_equal":
        C[:] = 0.61
    else:
        C[: B // 2] = 1.0
        C[B // 2:] = 0.25
    grad = torch.full((d, p), -2.0, dtype=torch.float32, device="cuda")
    dp.dp_clipped_grad(dev(a), dev(g), dp.DP_BF16, B, T, d, p, dev(C), grad, 0)
    G = o.clipped_grad(si.to_f64(a), si.to_f64(g), C.astype(np.float64))
    assert frob(host(grad), G) <= 1e-5


@pytest.mark.parametrize("B,T,d,p", [(3, 96, 392, 520), (2, 32, 4360, 3848), (3, 50, 72, 264)])
def test_gradient_is_reproducible_bit_for_bit(dp, B, T, d, p):
    # no atomics and a fixed summation order in every gradient kernel: two runs give the same bits
    w = si.small_workload("det", si.BF16, B, T, [(d, p)])
    a, g = si.gen_layer(w, 0)
    ad, gd = dev(a), dev(g)
    Cd = dev(np.random.default_rng(9).uniform(0.1, 1.0, B).astype(np.float32))
    runs = []
    for _ in range(2):
        grad = torch.zeros((d, p), dtype=torch.float32, device="cuda")
        dp.dp_clipped_grad(ad, gd, dp.DP_BF16, B, T, d, p, Cd, grad, 0)
        runs.append(grad)
    assert torch.equal(runs[0], runs[1])


def test_bf16_unclipped_is_plain_product(dp):
    # C = 1: the standard gradient a^T g over all B*T rows.
    B, T, d, p = 3, 200, 264, 136
    w = si.small_workload("b", si.BF16, B, T, [(d, p)])
    a, g = si.gen_layer(w, 0)
    ones = torch.ones(B, dtype=torch.float32, device="cuda")
    grad = torch.zeros((d, p), dtype=torch.float32, device="cuda")
    dp.dp_clipped_grad(dev(a), dev(g), dp.DP_BF16, B, T, d, p, ones, grad, 0)
    want = si.to_f64(a).reshape(-1, d).T @ si.to_f64(g).reshape(-1, p)
    assert frob(host(grad), want) <= 1e-5


@pytest.mark.parametrize("keep", [False, True])
@pytest.mark.parametrize("dtype", HALF_TYPES)
def test_multi_layer_stack_mixed_paths(dp, Pipe, dtype, keep):
    # A stack whose layers take different norm paths and shapes, in one grouped launch each;
    # with `keep`, the instantiated layers' gradients come from the kept per-sample gradients.
    dims = [(72, 264), (264, 72), (8, 8), (136, 136), (520, 16)]
    w = si.small_workload("m", dtype, 3, 150, dims, clip_mode=si.CLIP_AUTOMATIC)
    layers = gen(w)
    l64 = [(si.to_f64(a), si.to_f64(g)) for a, g in layers]
    paths = [0, 1, 1, 0, 1]
    pipe = Pipe([(dev(a), dev(g)) for a, g in layers], paths=paths, keep_instantiated=keep)
    assert pipe.any_kept == keep
    pipe.norms()
    pipe.clip(w.clip_mode, w.R, w.stability)
    pipe.grad()
    want = np.stack([o.perex_sqnorm(a, g) for a, g in l64])
    assert rel(host(pipe.sqnorm), want) <= TOL_BF16_NORM
    C, _ = o.clip_factors(want, w.clip_mode, w.R, w.stability)
    assert rel(host(pipe.C), C) <= TOL_BF16_NORM
    for l, (a, g) in enumerate(l64):
        assert frob(host(pipe.grads[l]), o.clipped_grad(a, g, C)) <= 1e-4


def test_standard_clipping_takes_both_branches(dp, Pipe):
    # Output gradients small enough that some samples fall below R (C_i = 1) while others are
    # clipped (C_i < 1): per-sample scales spread the norms around R.
    dims = [(136, 264), (264, 136)]
    B, T = 6, 96
    w = si.small_workload("both", si.BF16, B, T, dims, g_std=1e-2)
    layers = gen(w)
    scale = np.array([1e-3, 3.0, 1e-2, 1.0, 1e-4, 10.0], dtype=np.float32)    # applied in fp32, rounded again
    layers = [(a, si.f32_to_bf16_bits(si.bf16_bits_to_f32(g) * scale[:, None, None])) for a, g in layers]
    l64 = [(si.to_f64(a), si.to_f64(g)) for a, g in layers]
    pipe = Pipe([(dev(a), dev(g)) for a, g in layers])
    pipe.norms()
    pipe.clip(dp.DP_CLIP_STANDARD, 1.0)
    pipe.grad()
    sqn = np.stack([o.ghost_sqnorm(a, g) for a, g in l64])
    C, norm = o.clip_factors(sqn, o.CLIP_STANDARD, 1.0, 0.01)
    assert (C == 1.0).sum() >= 2 and (C < 1.0).sum() >= 2
    got = host(pipe.C)
    assert np.array_equal(got == 1.0, C == 1.0)
    assert rel(got, C) <= TOL_BF16_NORM
    for l, (a, g) in enumerate(l64):
        assert frob(host(pipe.grads[l]), o.clipped_grad(a, g, C)) <= 1e-4


@pytest.mark.parametrize("with_wide_layer", [False, True])
def test_stack_with_three_sequence_lengths(dp, Pipe, with_wide_layer):
    # T is a per-layer quantity (section 3: a_l in R^{B x T_l x d_l}); one grouped launch holds
    # layers of different T.  Ghost norm: the T = 96 layer rides in a large-tile launch that takes
    # the general plan because of the T = 320 layer, the T = 256 layer takes the whole-sample
    # kernel; one layer takes the instantiated norm.
    # Gradient: 19 tiles (all computed as sub-tiles) or, with the wide T = 64 layer, 75 tiles
    # (all computed as 256 x 256 tiles), k extents 64 to 320 in one launch.
    dims = [(128, 320), (256, 640), (384, 1280), (264, 392)] + ([(1800, 1544)] if with_wide_layer else [])
    Ts = [96, 256, 320, 256] + ([64] if with_wide_layer else [])
    B = 3
    layers = []
    for l, ((d, p), T) in enumerate(zip(dims, Ts)):
        w = si.small_workload("mt", si.BF16, B, T, [(d, p)], data_seed=100 + l)
        layers.append(si.gen_layer(w, 0))
    l64 = [(si.to_f64(a), si.to_f64(g)) for a, g in layers]
    pipe = Pipe([(dev(a), dev(g)) for a, g in layers])
    assert [T for T, _, _ in pipe.dims] == Ts
    assert pipe.paths[:4] == [0, 0, 0, 1]
    pipe.norms()
    pipe.clip(dp.DP_CLIP_AUTOMATIC, 1.0, 0.01)
    pipe.grad()
    sqn = np.stack([o.perex_sqnorm(a, g) for a, g in l64])
    assert rel(host(pipe.sqnorm), sqn) <= TOL_BF16_NORM
    C, _ = o.clip_factors(sqn, o.CLIP_AUTOMATIC, 1.0, 0.01)
    assert rel(host(pipe.C), C) <= TOL_BF16_NORM
    Cg = host(pipe.C).astype(np.float64)              # the weights the kernels actually used
    clean = []
    for l, (a, g) in enumerate(l64):
        G = o.clipped_grad(a, g, Cg)
        assert frob(host(pipe.grads[l]), G) <= 1e-5
        clean.append(G)
    # the same stack with the noise added in the gradient pass
    sigma, R, seed, step = 0.5, 1.0, 17, 3
    two_pass = pipe.flat.clone()
    dp.dp_add_noise(two_pass, 0, pipe.psi, sigma, R, seed, step)
    pipe.flat.fill_(1.0)
    pipe.grad_noise(sigma, R, seed, step, 0, pipe.psi)
    assert torch.equal(pipe.flat, two_pass)
    z = o.normals(seed, step, 0, pipe.psi)
    want = np.concatenate([G.reshape(-1) for G in clean]) + sigma * R * z
    have = host(pipe.flat).astype(np.float64)
    assert np.all(np.abs(have - want) <= 2e-5 * sigma * R * np.maximum(1.0, np.abs(z)) + 1e-4 * np.abs(want - sigma * R * z))


@pytest.mark.parametrize("d", [465920, 524288])
def test_sample_slabs_at_the_addressing_limit(dp, d):
    # The kernels that load through buffer descriptors address a sample's [T, d] slab with 32-bit
    # byte offsets.  d = 465920: (T + 256) d 2 bytes lies just below 2^31, the largest slab those
    # kernels take; d = 524288: T d 2 = 2^31 exactly, so every kernel falls back to its 64-bit
    # form.  Two samples, so that the second slab starts 2 GiB into the array.  Inputs are drawn
    # on the device (seeded; a ~ N(0,1), g ~ N(0, 1e-4) as in the workloads) and the oracle runs on
    # column chunks of a: rows of G and the sum of squares split exactly over them.
    B, T, p = 2, 2048, 128
    gen_ = torch.Generator(device="cuda").manual_seed(d)
    a = torch.randn(B, T, d, device="cuda", generator=gen_).to(torch.bfloat16)
    g = (torch.randn(B, T, p, device="cuda", generator=gen_) * 1e-2).to(torch.bfloat16)
    C = np.array([0.75, 0.031], dtype=np.float32)
    g64 = g.float().cpu().numpy().astype(np.float64)
    want_sq = np.zeros(B)
    want_G = np.empty((d, p))
    step = 16384
    for j0 in range(0, d, step):
        a64 = a[:, :, j0:j0 + step].float().cpu().numpy().astype(np.float64)
        want_sq += o.perex_sqnorm(a64, g64)
        want_G[j0:j0 + step] = o.clipped_grad(a64, g64, C.astype(np.float64))
    for path, fn in ((dp.DP_PATH_GHOST, dp.dp_ghost_norm), (dp.DP_PATH_PEREX, dp.dp_perex_norm)):
        ws = torch.empty(dp.dp_norm_workspace_bytes(path, dp.DP_BF16, B, T, d, p), dtype=torch.uint8, device="cuda")
        out = torch.full((B,), -1.0, dtype=torch.float32, device="cuda")
        fn(a, g, dp.DP_BF16, B, T, d, p, out, ws)
        assert rel(host(out), want_sq) <= TOL_BF16_NORM, (path, host(out), want_sq)
    grad = torch.full((d, p), 3.0, dtype=torch.float32, device="cuda")
    dp.dp_clipped_grad(a, g, dp.DP_BF16, B, T, d, p, dev(C), grad, 0)
    assert frob(host(grad), want_G) <= 1e-5


def random_stack(seed):
    """A seeded stack of four layers whose (T, d, p) are drawn so that the sweep reaches every
    16-bit kernel: whole and ragged k-blocks, widths from 8 up, both norm paths."""
    rng = np.random.default_rng(seed)
    B = int(rng.integers(1, 6))
    dims, Ts = [], []
    for _ in range(4):
        kind = int(rng.integers(0, 4))
        if kind == 0:        # whole 32-token blocks and wide layers: large-tile kernels
            T = 32 * int(rng.integers(1, 11))
            d, p = (8 * int(rng.integers(16, 90)) for _ in range(2))
        elif kind == 1:      # widths that are multiples of 64: large-tile / whole-sample ghost norm
            T = int(rng.integers(96, 330))
            d, p = (64 * int(rng.integers(1, 9)) for _ in range(2))
        elif kind == 2:      # anything goes
            T = int(rng.integers(1, 300))
            d, p = (8 * int(rng.integers(1, 60)) for _ in range(2))
        else:                # long samples, narrow layers: the instantiated path
            T = int(rng.integers(200, 700))
            d, p = (8 * int(rng.integers(1, 40)) for _ in range(2))
        dims.append((d, p))
        Ts.append(T)
    return B, Ts, dims


@pytest.mark.parametrize("dtype", HALF_TYPES)
@pytest.mark.parametrize("seed", range(16))
def test_random_stacks(dp, Pipe, seed, dtype):
    B, Ts, dims = random_stack(seed)
    layers = []
    for l, ((d, p), T) in enumerate(zip(dims, Ts)):
        w = si.small_workload("rs", dtype, B, T, [(d, p)], data_seed=1000 * seed + l)
        layers.append(si.gen_layer(w, 0))
    l64 = [(si.to_f64(a), si.to_f64(g)) for a, g in layers]
    sqn = np.stack([o.perex_sqnorm(a, g) for a, g in l64])
    for keep in (True, False):
        pipe = Pipe([(dev(a), dev(g)) for a, g in layers], keep_instantiated=keep)
        assert pipe.paths == [o.choose_path(T, d, p) for T, (d, p) in zip(Ts, dims)]
        pipe.norms()
        pipe.clip(dp.DP_CLIP_AUTOMATIC, 1.0, 0.01)
        pipe.flat.fill_(7.0)
        pipe.grad()
        assert rel(host(pipe.sqnorm), sqn) <= TOL_BF16_NORM, (B, Ts, dims)
        C, _ = o.clip_factors(sqn, o.CLIP_AUTOMATIC, 1.0, 0.01)
        assert rel(host(pipe.C), C) <= TOL_BF16_NORM
        Cg = host(pipe.C).astype(np.float64)
        for l, (a, g) in enumerate(l64):
            assert frob(host(pipe.grads[l]), o.clipped_grad(a, g, Cg)) <= 1e-5, (l, B, Ts, dims)
        # no atomics anywhere: the same call gives the same bits
        first = pipe.flat.clone()
        sq_first = pipe.sqnorm.clone()
        pipe.norms()
        pipe.flat.fill_(-1.0)
        pipe.grad()
        assert torch.equal(pipe.flat, first) and torch.equal(pipe.sqnorm, sq_first)
        # noise in the gradient pass = gradient pass + noise pass, on a shard inside the stack
        lo, cnt = pipe.psi // 7, pipe.psi // 2
        two_pass = pipe.flat.clone()
        dp.dp_add_noise(two_pass[lo:], lo, cnt, 0.7, 1.0, 5 + seed, 2)
        pipe.flat.fill_(-3.0)
        pipe.grad_noise(0.7, 1.0, 5 + seed, 2, lo, cnt)
        assert torch.equal(pipe.flat, two_pass)
    # layer-wise clipping pass by pass against the oracle's grouped definition
    L = len(dims)
    R = [0.3, 1.0, 0.1, 2.0]
    pipe.set_groups(list(range(L)), R)
    pipe.flat.fill_(2.0)
    pipe.layerwise_step(dp.DP_CLIP_STANDARD, 0.01, 0.0, 1, 1, 0, pipe.psi)
    ref = o.private_gradient_grouped(l64, list(range(L)), R, o.CLIP_STANDARD, 0.0, 0.01, 1, 1, 0, 0)
    assert rel(host(pipe.sqnorm), ref["sqnorm"]) <= TOL_BF16_NORM
    Cl = host(pipe.C_groups).astype(np.float64)
    assert rel(Cl, ref["C"]) <= TOL_BF16_NORM
    for l, (a, g) in enumerate(l64):
        assert frob(host(pipe.grads[l]), o.clipped_grad(a, g, Cl[l])) <= 1e-5, (l, B, Ts, dims)


@pytest.mark.parametrize("B,T,d,p", [
    (6, 64, 1800, 1544),     # one short round of 256 x 256 tiles
    (6, 96, 392, 520),       # sub-tile kernel only
    (6, 50, 136, 264),       # T not a multiple of 32: the 8-wave kernel
    (6, 32, 4360, 3848),     # a full round of large tiles plus sub-tiles
])
def test_weight_ratios_across_ten_decades(dp, B, T, d, p):
    # The kernels hold one accumulator in units of the current sample's weight and multiply it by
    # C_i / C_{i+1} between samples: ratios from 1e-10 to 1e10 in one batch, in both directions
    w = si.small_workload("wr", si.BF16, B, T, [(d, p)])
    a, g = si.gen_layer(w, 0)
    a64, g64 = si.to_f64(a), si.to_f64(g)
    for C in ([1e-8, 1e2, 1e-8, 3e-3, 1e2, 1.0], [1e2, 1e-8, 1e2, 1.0, 1e-8, 1e-8], [1e-8] * 6, [-1.0, 1e2, 0.0, -1e-8, 1.0, 1e2]):
        C = np.array(C, dtype=np.float32)
        grad = torch.full((d, p), 5.0, dtype=torch.float32, device="cuda")
        dp.dp_clipped_grad(dev(a), dev(g), dp.DP_BF16, B, T, d, p, dev(C), grad, 0)
        G = o.clipped_grad(a64, g64, C.astype(np.float64))
        got = host(grad)
        assert np.all(np.isfinite(got))
        assert frob(got, G) <= 1e-5, C


def test_calls_on_a_side_stream(dp, Pipe):
    # every entry point enqueues on the stream it is given: the whole path on a non-default
    # stream, with the default stream kept busy on an unrelated buffer
    w = si.small_workload("st", si.BF16, 3, 160, [(136, 264), (392, 520), (264, 72)], clip_mode=si.CLIP_AUTOMATIC)
    layers = gen(w)
    l64 = [(si.to_f64(a), si.to_f64(g)) for a, g in layers]
    pipe = Pipe([(dev(a), dev(g)) for a, g in layers])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())          # inputs were uploaded on the current stream
    busy = torch.zeros(1 << 24, device="cuda")
    for _ in range(8):
        busy.add_(1.0)                                     # default-stream work in flight meanwhile
    off, cnt = 0, pipe.psi
    pipe.step(w.clip_mode, w.R, 0.5, w.stability, 5, 1, off, cnt, stream=side, fused=False)
    side.synchronize()
    ref = o.private_gradient(l64, w.clip_mode, w.R, 0.5, w.stability, 5, 1, off, cnt)
    assert rel(pipe.C.cpu().numpy(), ref["C"]) <= TOL_BF16_NORM
    np.testing.assert_allclose(pipe.flat.cpu().numpy(), ref["flat"], rtol=0, atol=1e-4)
    two = pipe.flat.clone()
    pipe.step(w.clip_mode, w.R, 0.5, w.stability, 5, 1, off, cnt, stream=side, fused=True)
    side.synchronize()
    assert torch.equal(pipe.flat, two)
    torch.cuda.synchronize()
    assert float(busy[0]) == 8.0


def test_clip_factor_corner_values_on_device(dp):
    # zero norm without a stability constant -> 0; NaN squared norm -> NaN factor in both modes;
    # infinite norm -> factor 0
    sqn = np.array([[0.0, 4.0, np.nan, np.inf, -1e-9]], dtype=np.float32)
    for mode, stab in ((0, 0.01), (1, 0.0), (1, 0.01)):
        Cd = torch.zeros(5, dtype=torch.float32, device="cuda")
        nd = torch.zeros(5, dtype=torch.float32, device="cuda")
        dp.dp_clip_factors(dev(sqn), 1, 5, mode, 1.0, stab, Cd, nd)
        C, norm = o.clip_factors(sqn.astype(np.float64), mode, 1.0, stab)
        got = host(Cd)
        assert np.isnan(got[2]) and np.isnan(C[2]) and got[3] == 0.0 and C[3] == 0.0
        np.testing.assert_allclose(got[[0, 1, 4]], C[[0, 1, 4]], rtol=TOL_F32)
        Cg = torch.zeros((1, 5), dtype=torch.float32, device="cuda")
        dp.dp_clip_factors_grouped(dev(sqn), 1, 5, [0, 1], [1.0], mode, stab, Cg)
        np.testing.assert_array_equal(host(Cg)[0], got)


# ----------------------------------------------------------------------------
# full-size workloads
# ----------------------------------------------------------------------------

def sampled_grad_check(w, layers, C, pipe, full_layers=(), n_samples=2048, seed=5):
    """Gradient before noise: whole matrix for `full_layers`, else seeded random entries plus
    the four corners' neighbourhoods, each entry computed on its own by the oracle."""
    worst = 0.0
    rng = np.random.default_rng(seed)
    for l, (a, g) in enumerate(layers):
        d, p = w.layers[l]
        got = pipe.grads[l]
        if l in full_layers:
            G = o.clipped_grad(si.to_f64(a), si.to_f64(g), C)
            worst = max(worst, frob(host(got), G))
            # every 64 x 64 block on its own too: the smallest unit one workgroup writes
            have = host(got).astype(np.float64)
            for r0 in range(0, d, 64):
                for c0 in range(0, p, 64):
                    worst = max(worst, frob(have[r0:r0 + 64, c0:c0 + 64], G[r0:r0 + 64, c0:c0 + 64]))
            continue
        rows = np.concatenate([rng.integers(0, d, n_samples), [0, 0, d - 1, d - 1]])
        cols = np.concatenate([rng.integers(0, p, n_samples), [0, p - 1, 0, p - 1]])
        ur, ri = np.unique(rows, return_inverse=True)
        uc, ci = np.unique(cols, return_inverse=True)
        a_sel = si.to_f64(np.ascontiguousarray(a[:, :, ur]))
        g_sel = si.to_f64(np.ascontiguousarray(g[:, :, uc]))
        want = o.clipped_grad_entries(a_sel, g_sel, C, ri, ci)
        idx = torch.from_numpy(rows * p + cols).cuda()
        have = host(got.reshape(-1)[idx])
        worst = max(worst, frob(have, want))
    return worst


def block_grid_check(w, layers, C, pipe, seed=11):
    """Gradient before noise, one seeded entry in every 64 x 64 block of every layer (64 x 64 is
    the smallest unit a workgroup of any gradient kernel writes): one row index per 64-row band,
    one column index per 64-column band; those columns of a and g are gathered and the oracle's
    clip-weighted gradient of the gathered operands is the grid of expected entries."""
    worst = 0.0
    rng = np.random.default_rng(seed)
    for l, (a, g) in enumerate(layers):
        d, p = w.layers[l]
        rows = np.array([r0 + rng.integers(0, min(64, d - r0)) for r0 in range(0, d, 64)])
        cols = np.array([c0 + rng.integers(0, min(64, p - c0)) for c0 in range(0, p, 64)])
        want = o.clipped_grad(si.to_f64(np.ascontiguousarray(a[:, :, rows])),
                              si.to_f64(np.ascontiguousarray(g[:, :, cols])), C)
        have = host(pipe.grads[l][torch.from_numpy(rows).cuda()][:, torch.from_numpy(cols).cuda()])
        assert have.shape == want.shape
        worst = max(worst, frob(have, want))
        # entry by entry too: one wrong or unwritten block must not hide in the Frobenius norm
        scale = np.sqrt(np.mean(want * want))
        assert np.max(np.abs(have - want)) <= 1e-3 * scale, (l, float(np.max(np.abs(have - want))), scale)
    return worst


def run_workload(dp, Pipe, name, full_layers=()):
    w = si.WORKLOADS[name]
    layers = gen(w)
    pipe = Pipe([(dev(a), dev(g)) for a, g in layers])
    # the logged path choice is the paper's rule, as the oracle reads it
    assert pipe.paths == [o.choose_path(w.T, d, p) for d, p in w.layers]
    pipe.norms()
    pipe.clip(w.clip_mode, w.R, w.stability)
    pipe.grad()
    sqn = np.stack([
        (o.ghost_sqnorm if path == o.PATH_GHOST else o.perex_sqnorm)(si.to_f64(a), si.to_f64(g))
        for (a, g), path in zip(layers, pipe.paths)])
    assert rel(host(pipe.sqnorm), sqn) <= TOL_BF16_NORM
    C, norm = o.clip_factors(sqn, w.clip_mode, w.R, w.stability)
    assert rel(host(pipe.norm), norm) <= TOL_BF16_NORM
    assert rel(host(pipe.C), C) <= TOL_BF16_NORM
    assert sampled_grad_check(w, layers, C, pipe, full_layers) <= TOL_BF16_GRAD
    assert block_grid_check(w, layers, C, pipe) <= TOL_BF16_GRAD
    # noise on the rank's shard only; checked on the head, the tail and a window inside
    off, cnt = w.noise_range()
    before = pipe.flat.clone()
    pipe.noise(w.sigma, w.R, w.noise_seed, w.noise_step, off, cnt)
    std = w.sigma * w.R
    for lo in (off, off + cnt // 2 - 1001, off + cnt - 4096):
        hi = min(lo + 4096, off + cnt)
        z = (host(pipe.flat[lo:hi]).astype(np.float64) - host(before[lo:hi])) / std
        ref = o.normals(w.noise_seed, w.noise_step, lo, hi - lo)
        assert np.all(np.abs(z - ref) <= 2e-5 * np.maximum(1.0, np.abs(ref)))   # fp32 add of grad + noise
    if off > 0:
        assert torch.equal(pipe.flat[:off], before[:off])
    if off + cnt < w.psi:
        assert torch.equal(pipe.flat[off + cnt:], before[off + cnt:])
        delta = (pipe.flat[off:off + cnt] - before[off:off + cnt]).double()
        assert abs(float(delta.std()) / std - 1) < 1e-3
    # the same step with the noise added in the gradient kernels' epilogue: value for value
    two_pass = pipe.flat.clone()
    pipe.flat.fill_(7.0)
    pipe.grad_noise(w.sigma, w.R, w.noise_seed, w.noise_step, off, cnt)
    assert torch.equal(pipe.flat, two_pass)
    return pipe


def test_cfg1_gpt2_small_full(dp, Pipe):
    # layer 47 holds the launch's last tiles, which the sub-tile kernel computes
    run_workload(dp, Pipe, "cfg1", full_layers=(0, 1, 2, 3, 47))


def test_cfg3_long_sequence_full(dp, Pipe):
    pipe = run_workload(dp, Pipe, "cfg3", full_layers=(0, 1, 2, 3))
    assert pipe.paths == [dp.DP_PATH_PEREX] * 4


def test_cfg2_gpt2_large_full(dp, Pipe):
    # the last layer of each launch of 48 holds the tiles the sub-tile kernel computes
    run_workload(dp, Pipe, "cfg2", full_layers=(47, 95, 143))


def test_cfg4_wide_block_shard(dp, Pipe):
    import dataclasses
    # the 12288 x 12288 layer is compared in full (every element, and every 64 x 64 block on its
    # own); the wider ones on one entry per 64 x 64 block and on random entries
    pipe = run_workload(dp, Pipe, "cfg4", full_layers=(1,))
    # the shard of rank 2 of 8 crosses the boundary between the second and the third layer
    w = dataclasses.replace(si.WORKLOADS["cfg4"], shard_rank=2)
    off, cnt = w.noise_range()
    edge = w.layer_offsets()[2]
    assert off < edge < off + cnt
    pipe.grad()
    before = pipe.flat.clone()
    pipe.noise(w.sigma, w.R, w.noise_seed, w.noise_step, off, cnt)
    std = w.sigma * w.R
    for lo in (off, edge - 2048, off + cnt - 4096):
        z = (host(pipe.flat[lo:lo + 4096]).astype(np.float64) - host(before[lo:lo + 4096])) / std
        ref = o.normals(w.noise_seed, w.noise_step, lo, 4096)
        assert np.all(np.abs(z - ref) <= 2e-5 * np.maximum(1.0, np.abs(ref)))
    assert torch.equal(pipe.flat[:off], before[:off])
    assert torch.equal(pipe.flat[off + cnt:], before[off + cnt:])
    two_pass = pipe.flat.clone()
    del before
    pipe.flat.fill_(-3.0)
    pipe.grad_noise(w.sigma, w.R, w.noise_seed, w.noise_step, off, cnt)
    assert torch.equal(pipe.flat, two_pass)


# ----------------------------------------------------------------------------
# group-wise clipping (eq. (1), M groups) and bias gradients (appendix A.1)
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("mode", [0, 1])
def test_grouped_clip_factors(dp, mode):
    rng = np.random.default_rng(31)
    L, B = 11, 37
    sqn = rng.uniform(0, 2, size=(L, B)).astype(np.float32)
    begin = [0, 3, 3, 4, 11]                          # group 1 is empty
    R = [0.5, 1.0, 2.0, 1e3]
    group_of_row = [0, 0, 0, 2, 3, 3, 3, 3, 3, 3, 3]
    Cd = torch.zeros((4, B), dtype=torch.float32, device="cuda")
    nd = torch.zeros((4, B), dtype=torch.float32, device="cuda")
    dp.dp_clip_factors_grouped(dev(sqn), L, B, begin, R, mode, 0.01, Cd, nd)
    C, norm = o.clip_factors_grouped(sqn.astype(np.float64), group_of_row, R, mode, 0.01)
    np.testing.assert_allclose(host(nd), norm, rtol=TOL_F32, atol=1e-30)
    np.testing.assert_allclose(host(Cd), C, rtol=TOL_F32)
    assert dp.dp_group_noise_threshold([3.0, 4.0]) == 5.0


@pytest.mark.parametrize("dtype,B,T,p", [(si.F32, 3, 5, 7), (si.BF16, 2, 300, 520), (si.BF16, 8, 512, 5120),
                                         (si.BF16, 1, 1, 8), (si.F32, 4, 8, 16), (si.F16, 2, 300, 520),
                                         (si.F16, 3, 64, 8)])
def test_bias_norm_and_clipped_bias_grad(dp, dtype, B, T, p):
    w = si.small_workload("bias", dtype, B, T, [(8, p)])
    g = si.gen_tensor(w, 0, 1)
    g64 = si.to_f64(g)
    dt = dt_of(dp, dtype)
    colsum = torch.full((B, p), -1.0, dtype=torch.float32, device="cuda")
    sq = torch.full((B,), -1.0, dtype=torch.float32, device="cuda")
    dp.dp_bias_norm(dev(g), dt, B, T, p, colsum, sq)
    tol = TOL_F32 if dtype == si.F32 else TOL_BF16_NORM
    assert frob(host(colsum), o.bias_per_sample_grad(g64)) <= 1e-5
    assert rel(host(sq), o.bias_sqnorm(g64)) <= tol
    C = np.random.default_rng(4).uniform(0, 1, B).astype(np.float32)
    C[0] = 0.0
    gb = torch.full((p,), 2.0, dtype=torch.float32, device="cuda")
    dp.dp_clipped_bias_grad(colsum, B, p, dev(C), gb, 0)
    want = o.clipped_bias_grad(g64, C.astype(np.float64))
    assert frob(host(gb), want) <= 1e-5 or np.linalg.norm(want) == 0
    dp.dp_clipped_bias_grad(colsum, B, p, dev(C), gb, 1)
    assert frob(host(gb), 2 * want) <= 1e-5 or np.linalg.norm(want) == 0


@pytest.mark.parametrize("dtype", [si.F32, si.BF16, si.F16])
def test_layerwise_clipping_with_biases(dp, dtype):
    # The paper's default setting: one clipping group per layer (weight + bias), noise level
    # sigma * ||R||_2; flattened result [W_0, b_0, W_1, b_1, ...].
    dims = [(72, 264), (264, 136), (136, 16)] if dtype != si.F32 else [(4, 8), (8, 4), (4, 12)]
    B, T = (3, 150) if dtype != si.F32 else (4, 6)
    w = si.small_workload("lw", dtype, B, T, dims, g_std=1e-2 if dtype != si.F32 else 1.0)
    layers = gen(w)
    l64 = [(si.to_f64(a), si.to_f64(g)) for a, g in layers]
    dt = dt_of(dp, dtype)
    L, M = len(dims), len(dims)
    R = [0.05, 0.2, 1e3]
    sigma = 0.3
    dlayers = [(dev(a), dev(g)) for a, g in layers]
    # rows of sqnorm: W_0, b_0, W_1, b_1, ...
    sqn = torch.zeros((2 * L, B), dtype=torch.float32, device="cuda")
    colsums, paths = [], []
    for l, ((a, g), (d, p)) in enumerate(zip(dlayers, dims)):
        path = dp.dp_choose_path(T, d, p)
        paths.append(path)
        nbytes = dp.dp_norm_workspace_bytes(path, dt, B, T, d, p)
        ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device="cuda")
        fn = dp.dp_ghost_norm if path == dp.DP_PATH_GHOST else dp.dp_perex_norm
        fn(a, g, dt, B, T, d, p, sqn[2 * l], ws)
        cs = torch.zeros((B, p), dtype=torch.float32, device="cuda")
        dp.dp_bias_norm(g, dt, B, T, p, cs, sqn[2 * l + 1])
        colsums.append(cs)
    Cd = torch.zeros((M, B), dtype=torch.float32, device="cuda")
    dp.dp_clip_factors_grouped(sqn, 2 * L, B, [0, 2, 4, 6], R, dp.DP_CLIP_STANDARD, 0.01, Cd)
    psi = sum(d * p + p for d, p in dims)
    flat = torch.zeros(psi, dtype=torch.float32, device="cuda")
    wg, bg, off = [], [], 0
    for d, p in dims:
        wg.append(flat[off:off + d * p].view(d, p))
        off += d * p
        bg.append(flat[off:off + p])
        off += p
    desc = [(a, g, T, d, p, path) for (a, g), (d, p), path in zip(dlayers, dims, paths)]
    if any(x.data_ptr() % 16 for x in wg):
        pytest.skip("flattened layout not 16-byte aligned for this shape")
    dp.dp_clipped_grad_grouped(desc, dt, B, Cd, [0, 1, 2], M, wg, 0)
    for l, (d, p) in enumerate(dims):
        dp.dp_clipped_bias_grad(colsums[l], B, p, Cd[l], bg[l], 0)
    ref = o.private_gradient_grouped(l64, [0, 1, 2], R, o.CLIP_STANDARD, 0.0, 0.01, 1, 0, 0, 0, with_bias=True)
    tol = TOL_F32 if dtype == si.F32 else TOL_BF16_NORM
    assert rel(host(sqn), ref["sqnorm"]) <= tol
    assert rel(host(Cd), ref["C"]) <= tol
    assert np.all(host(Cd)[2] == 1.0) and np.all(host(Cd)[0] < 1.0)
    assert frob(host(flat), ref["flat"]) <= (1e-5 if dtype == si.F32 else 1e-4)
    clean = host(flat).copy()
    thr = dp.dp_group_noise_threshold(R)
    dp.dp_add_noise(flat, 0, psi, sigma, thr, 1, 0)
    z = (host(flat).astype(np.float64) - clean) / o.group_noise_std(sigma, R)
    want = o.normals(1, 0, 0, psi)
    assert np.all(np.abs(z - want) <= 2e-5 * np.maximum(1.0, np.abs(want)))


# ----------------------------------------------------------------------------
# error paths: every refusal happens on the host, nothing is launched
# ----------------------------------------------------------------------------

def test_layerwise_normalising_variant(dp, Pipe):
    # Appendix on the hook-free implementation: per layer, a_i^T g_i divided by its own norm,
    # i.e. layer-wise automatic clipping with R = 1 and no stability constant.
    dims = [(136, 264), (264, 136), (72, 24)]
    w = si.small_workload("nv", si.BF16, 4, 96, dims)
    layers = gen(w)
    l64 = [(si.to_f64(a), si.to_f64(g)) for a, g in layers]
    pipe = Pipe([(dev(a), dev(g)) for a, g in layers])
    pipe.set_groups([0, 1, 2], [1.0, 1.0, 1.0])
    pipe.norms()
    pipe.clip_grouped(dp.DP_CLIP_AUTOMATIC, 0.0)
    pipe.grad_grouped()
    for l, (a, g) in enumerate(l64):
        want = np.zeros(dims[l])
        for i in range(w.B):
            Gi = a[i].T @ g[i]
            want += Gi / np.linalg.norm(Gi)             # every sample enters with unit norm
        assert frob(host(pipe.grads[l]), want) <= 5e-3  # bf16-path norms: 2e-3 on each weight
    ref = o.private_gradient_grouped(l64, [0, 1, 2], [1.0] * 3, o.CLIP_AUTOMATIC, 0.0, 0.0, 1, 0, 0, 0)
    assert rel(host(pipe.C_groups), ref["C"]) <= TOL_BF16_NORM


def test_pipeline_layerwise_step(dp, Pipe):
    # the sequence bench.py --clipping layer-wise times, against the oracle's group-wise path
    dims = [(136, 264), (264, 136), (136, 136), (392, 24)]
    w = si.small_workload("plw", si.BF16, 3, 96, dims)
    layers = gen(w)
    l64 = [(si.to_f64(a), si.to_f64(g)) for a, g in layers]
    R = [0.02, 0.5, 0.1, 1e3]
    sigma, seed, step = 0.4, 11, 2
    pipe = Pipe([(dev(a), dev(g)) for a, g in layers])
    pipe.set_groups([0, 1, 2, 3], R)
    pipe.norms()
    pipe.clip_grouped(dp.DP_CLIP_STANDARD, 0.01)
    pipe.grad_grouped()
    ref = o.private_gradient_grouped(l64, [0, 1, 2, 3], R, o.CLIP_STANDARD, 0.0, 0.01, seed, step, 0, 0)
    assert rel(host(pipe.C_groups), ref["C"]) <= TOL_BF16_NORM
    assert frob(host(pipe.flat), ref["flat"]) <= 1e-4
    clean = host(pipe.flat).copy()
    pipe.noise_grouped(sigma, seed, step, 0, pipe.psi)
    z = (host(pipe.flat).astype(np.float64) - clean) / o.group_noise_std(sigma, R)
    want = o.normals(seed, step, 0, pipe.psi)
    assert np.all(np.abs(z - want) <= 2e-5 * np.maximum(1.0, np.abs(want)))


# ----------------------------------------------------------------------------
# instantiated layers with their per-sample gradients kept (dp_norms_multi_keep,
# dp_clipped_grad_kept_multi)
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("dtype", HALF_TYPES)
def test_kept_per_sample_gradients(dp, dtype):
    # three layers on the instantiated path (several tiles with ragged edges; one tile; tiny) and
    # one on the ghost path; offsets chosen so that one kept layer starts off a generator block
    B, T = 4, 264
    dims = [(264, 392), (136, 72), (8, 16), (392, 520)]
    gaps = [0, 2, 0, 6]
    w = si.small_workload("kp", dtype, B, T, dims)
    layers = gen(w)
    l64 = [(si.to_f64(a), si.to_f64(g)) for a, g in layers]
    DT = dt_of(dp, dtype)
    paths = [dp.dp_choose_path(T, d, p) for d, p in dims]
    assert paths == [1, 1, 1, 0]
    desc = dp.layer_array([(dev(a), dev(g), T, d, p, path) for (a, g), (d, p), path in zip(layers, dims, paths)])
    keep_alive = [(dev(a), dev(g)) for a, g in layers]
    desc = dp.layer_array([(a, g, T, d, p, path) for (a, g), (d, p), path in zip(keep_alive, dims, paths)])
    L = len(dims)
    kept = [torch.full((B, d, p), 7.0, dtype=torch.float32, device="cuda") if path == 1 else None
            for (d, p), path in zip(dims, paths)]
    ws = torch.empty(dp.dp_norms_multi_workspace_bytes(desc, DT, B), dtype=torch.uint8, device="cuda")
    sqn = torch.zeros((L, B), dtype=torch.float32, device="cuda")
    dp.dp_norms_multi_keep(desc, DT, B, sqn, kept, ws)
    plain = torch.zeros((L, B), dtype=torch.float32, device="cuda")
    dp.dp_norms_multi(desc, DT, B, plain, ws)
    assert torch.equal(sqn, plain)                                   # keeping does not change the norms
    want_sqn = np.stack([o.perex_sqnorm(a, g) for a, g in l64])
    assert rel(host(sqn), want_sqn) <= TOL_BF16_NORM
    for l, (a, g) in enumerate(l64):
        if kept[l] is None:
            continue
        got = host(kept[l])
        for i in range(B):
            assert frob(got[i], a[i].T @ g[i]) <= 1e-5, (l, i)      # the instantiated per-sample gradient
    C = np.array([0.3, 0.0, 1.0, 1e-3], dtype=np.float32)
    Cd = dev(C)
    offs, acc = [], 10 ** 9
    for (d, p), gap in zip(dims, gaps):
        acc += gap
        offs.append(acc)
        acc += d * p
    total_lo, total_hi = offs[0], acc
    sigma, R, seed, step = 0.7, 1.3, 99, 6
    grads = lambda fill: [torch.full((d, p), fill, dtype=torch.float32, device="cuda") for d, p in dims]
    for accumulate in (0, 1):
        for lo, cnt in ((total_lo, total_hi - total_lo), (offs[0] + 1001, 50000), (offs[1] + 3, 8), (0, 0)):
            ref = grads(0.5)
            dp.dp_clipped_grad_multi(desc, DT, B, Cd, ref, accumulate)
            for l, (d, p) in enumerate(dims):
                x0, x1 = max(offs[l], lo), min(offs[l] + d * p, lo + cnt)
                if x0 < x1:
                    dp.dp_add_noise(ref[l].view(-1).data_ptr() + 4 * (x0 - offs[l]), x0, x1 - x0, sigma, R, seed, step)
            got = grads(0.5)
            dp.dp_clipped_grad_kept_multi(desc, DT, B, Cd, kept, got, offs, accumulate, lo, cnt, sigma, R, seed, step)
            for l in range(L):
                if kept[l] is None:
                    assert torch.equal(got[l], ref[l])               # same kernels as without kept layers
                else:                                                # other summation order, same noise values
                    G = o.clipped_grad(l64[l][0], l64[l][1], C.astype(np.float64))
                    scale = np.sqrt(np.mean(G * G))
                    assert np.max(np.abs(host(got[l]) - host(ref[l]))) <= 2e-5 * scale + 1e-6 * (sigma * R if cnt else 0) * 6
    # against the oracle, no noise
    got = grads(-1.0)
    dp.dp_clipped_grad_kept_multi(desc, DT, B, Cd, kept, got, None, 0, 0, 0, 0.0, 1.0, 0, 0)
    for l, (a, g) in enumerate(l64):
        assert frob(host(got[l]), o.clipped_grad(a, g, C.astype(np.float64))) <= 1e-5
    # refusals: a kept buffer for a ghost-path layer; fp32 storage
    bad = list(kept)
    bad[3] = torch.zeros((B, 392, 520), dtype=torch.float32, device="cuda")
    with pytest.raises(dp.DpError) as err:
        dp.dp_norms_multi_keep(desc, DT, B, sqn, bad, ws)
    assert err.value.status == dp.DP_ERR_INVALID_ARG


def test_kept_gradients_whole_pipeline_cfg3_noise_is_bit_identical(dp, Pipe):
    # cfg3 with kept gradients: gradient + noise in one call equals gradient, then dp_add_noise
    w = si.WORKLOADS["cfg3"]
    layers = gen(w)
    pipe = Pipe([(dev(a), dev(g)) for a, g in layers])
    assert pipe.any_kept and all(k is not None for k in pipe.kept)
    pipe.norms()
    pipe.clip(w.clip_mode, w.R, w.stability)
    off, cnt = 1000, w.psi - 3000
    pipe.grad()
    pipe.noise(w.sigma, w.R, w.noise_seed, w.noise_step, off, cnt)
    two = pipe.flat.clone()
    pipe.flat.fill_(4.0)
    pipe.grad_noise(w.sigma, w.R, w.noise_seed, w.noise_step, off, cnt)
    assert torch.equal(pipe.flat, two)
    # and the GEMM path on the same layers agrees to rounding
    gemm = Pipe([(dev(a), dev(g)) for a, g in layers], keep_instantiated=False)
    gemm.norms()
    gemm.clip(w.clip_mode, w.R, w.stability)
    gemm.grad()
    pipe.grad()
    assert torch.equal(gemm.C, pipe.C)
    assert frob(host(pipe.flat), host(gemm.flat)) <= 1e-5


# ----------------------------------------------------------------------------
# layer-wise clipping without book-keeping (dp_layerwise_clipped_grad)
# ----------------------------------------------------------------------------

LAYERWISE_STACK = [(72, 24), (128, 128), (392, 24), (24, 392), (136, 264), (392, 520), (16, 8), (104, 128)]


@pytest.mark.parametrize("dtype", HALF_TYPES)
@pytest.mark.parametrize("mode,stability", [(0, 0.01), (1, 0.01), (1, 0.0)])
def test_layerwise_without_book_keeping(dp, Pipe, dtype, mode, stability):
    # Small layers on the instantiated path (the first four and the last two fit one workgroup
    # tile: norm, factor and weighted sum in one kernel), a larger one on it, and one on the
    # ghost path; five samples so that the sample chunks of the one-pass kernel are uneven.
    dims, B, T = LAYERWISE_STACK, 5, 200
    w = si.small_workload("lw1", dtype, B, T, dims)
    layers = gen(w)
    # per-sample scales so that standard clipping takes both branches in most layers
    scale = np.array([1e-3, 1.0, 3e-2, 10.0, 0.3], dtype=np.float32)
    if dtype == si.BF16:
        layers = [(a, si.f32_to_bf16_bits(si.bf16_bits_to_f32(g) * scale[:, None, None])) for a, g in layers]
    else:
        layers = [(a, (g.astype(np.float32) * scale[:, None, None]).astype(np.float16)) for a, g in layers]
    l64 = [(si.to_f64(a), si.to_f64(g)) for a, g in layers]
    L = len(dims)
    R = [0.05, 0.5, 0.02, 0.1, 0.3, 1.0, 0.01, 0.2]
    sigma, seed, step = 0.6, 21, 4
    pipe = Pipe([(dev(a), dev(g)) for a, g in layers])
    assert pipe.paths == [o.choose_path(T, d, p) for d, p in dims] == [1, 1, 1, 1, 1, 0, 1, 1]
    pipe.set_groups(list(range(L)), R)
    psi = pipe.psi
    ref = o.private_gradient_grouped(l64, list(range(L)), R, mode, 0.0, stability, seed, step, 0, 0)
    pipe.flat.fill_(9.0)
    pipe.layerwise_step(mode, stability, 0.0, seed, step, 0, psi)
    assert rel(host(pipe.sqnorm), ref["sqnorm"]) <= TOL_BF16_NORM
    assert rel(host(pipe.C_groups), ref["C"]) <= TOL_BF16_NORM
    if mode == 0:
        assert (ref["C"] == 1.0).sum() >= L and (ref["C"] < 1.0).sum() >= L
        assert np.array_equal(host(pipe.C_groups) == 1.0, ref["C"] == 1.0)
    # the gradient against the oracle's definition with the weights the kernels used
    Cg = host(pipe.C_groups).astype(np.float64)
    clean = host(pipe.flat).copy()
    for l, (a, g) in enumerate(l64):
        assert frob(host(pipe.grads[l]), o.clipped_grad(a, g, Cg[l])) <= 1e-5, l
    assert frob(clean, ref["flat"]) <= 2 * TOL_BF16_NORM      # weights differ by the norms' rounding
    # the same bits whatever the pass size
    for per_pass in (1, 3):
        pipe.flat.fill_(-1.0)
        pipe.layerwise_step(mode, stability, 0.0, seed, step, 0, psi, layers_per_pass=per_pass)
        np.testing.assert_array_equal(host(pipe.flat), clean)
    # the ghost-path layer gives the bits of the two-pass sequence (layer 4, on the instantiated
    # path, is the weighted sum of its kept per-sample gradients here and a second contraction there)
    pipe.norms()
    pipe.clip_grouped(mode, stability)
    pipe.flat.fill_(3.0)
    pipe.grad_grouped()
    for l in (5,):
        np.testing.assert_array_equal(host(pipe.grads[l]).reshape(-1), clean[sum(d * p for d, p in dims[:l]):][:dims[l][0] * dims[l][1]])
    # accumulate, and noise of level sigma ||R||_2 on a shard that starts and ends inside layers
    lo, cnt = 1000, psi - 1500
    pipe.flat.copy_(torch.from_numpy(clean).cuda())
    pipe.layerwise_step(mode, stability, sigma, seed, step, lo, cnt, accumulate=1)
    got = host(pipe.flat).astype(np.float64)
    z = np.zeros(psi)
    z[lo:lo + cnt] = o.normals(seed, step, lo, cnt)
    std = o.group_noise_std(sigma, R)
    want = 2.0 * clean.astype(np.float64) + std * z
    assert np.all(np.abs(got - want) <= 2e-5 * std * np.maximum(1.0, np.abs(z)) + 1e-5 * np.abs(clean))
    assert np.array_equal(got[:lo], 2.0 * clean[:lo].astype(np.float64))


def test_layerwise_without_book_keeping_fp32(dp, Pipe):
    dims, B, T = [(4, 8), (8, 4), (4, 12)], 4, 6
    w = si.small_workload("lw32", si.F32, B, T, dims, g_std=1.0)
    layers = gen(w)
    l64 = [(si.to_f64(a), si.to_f64(g)) for a, g in layers]
    R = [0.5, 2.0, 1e3]
    pipe = Pipe([(dev(a), dev(g)) for a, g in layers])
    pipe.set_groups([0, 1, 2], R)
    pipe.layerwise_step(dp.DP_CLIP_STANDARD, 0.01, 0.4, 3, 1, 0, pipe.psi)
    ref = o.private_gradient_grouped(l64, [0, 1, 2], R, o.CLIP_STANDARD, 0.4, 0.01, 3, 1, 0, pipe.psi)
    assert rel(host(pipe.C_groups), ref["C"]) <= TOL_F32
    np.testing.assert_allclose(host(pipe.flat), ref["flat"], rtol=TOL_F32, atol=2e-5)


def test_layerwise_argument_errors(dp):
    import ctypes
    x = torch.zeros(4096, dtype=torch.float32, device="cuda")
    p = x.data_ptr()
    lib, INV = dp.lib, dp.DP_ERR_INVALID_ARG
    arr = dp.layer_array([(p, p, 8, 8, 8, 1)])
    gp = (ctypes.c_void_p * 1)(p + 8192)
    offs = (ctypes.c_uint64 * 1)(0)
    R = (ctypes.c_float * 1)(1.0)
    bad_R = (ctypes.c_float * 1)(0.0)
    n = dp.dp_layerwise_workspace_bytes(arr, dp.DP_BF16, 1)
    assert n > 0
    call = lambda *a: lib.dp_layerwise_clipped_grad(*a)
    ok = [arr, 1, 1, 1, R, 0, 0.01, gp, offs, 0, 0, 16, 1.0, 0, 0, p, p + 4096, p + 1024, n, 0, None]
    def with_(i, v):
        a = list(ok)
        a[i] = v
        return a
    assert call(*with_(4, bad_R)) == INV
    assert call(*with_(5, 2)) == INV
    assert call(*with_(8, None)) == INV                   # noise asked for, no offsets
    assert call(*with_(12, -1.0)) == INV
    assert call(*with_(15, None)) == INV
    assert call(*with_(18, 0)) == dp.DP_ERR_WORKSPACE
    assert call(*with_(19, -1)) == INV
    torch.cuda.synchronize()
    assert not host(x).any()


# ----------------------------------------------------------------------------
# gradient + noise in one pass (dp_clipped_grad_noise_multi)
# ----------------------------------------------------------------------------

FUSED_CASES = [
    # dtype, B, T, dims, gaps (elements skipped before each layer in the flattened model), base offset
    (si.BF16, 3, 96, [(136, 264), (264, 136), (392, 520), (8, 16)], [0, 0, 0, 0], 0),
    (si.BF16, 3, 96, [(136, 264), (264, 136), (392, 520), (8, 16)], [0, 3, 0, 8], 1 << 34),   # 2nd, 3rd start off a block
    (si.F16, 2, 64, [(1800, 1544), (128, 128)], [4, 0], 12),
    (si.BF16, 2, 32, [(4360, 3848)], [0], 0),                    # large tiles and sub-tiles in one launch
    (si.BF16, 2, 50, [(136, 264), (264, 136)], [0, 0], 0),       # T not a multiple of 32: small-layer kernel
    (si.F32, 3, 5, [(8, 12), (12, 4)], [0, 1], 0),
]


@pytest.mark.parametrize("accumulate", [0, 1])
@pytest.mark.parametrize("dtype,B,T,dims,gaps,base", FUSED_CASES)
def test_fused_noise_equals_two_passes(dp, dtype, B, T, dims, gaps, base, accumulate):
    w = si.small_workload("fz", dtype, B, T, dims)
    layers = gen(w)
    dt = dt_of(dp, dtype)
    desc = [(dev(a), dev(g), T, d, p, dp.dp_choose_path(T, d, p)) for (a, g), (d, p) in zip(layers, dims)]
    C = np.random.default_rng(8).uniform(0.1, 1.0, B).astype(np.float32)
    if B > 2:
        C[1] = 0.0
    Cd = dev(C)
    offs, acc = [], 0
    for (d, p), gap in zip(dims, gaps):
        acc += gap
        offs.append(acc)
        acc += d * p
    total = acc
    sigma, R, seed, step = 0.7, 1.5, 0xABCDEF0123, 5

    def buffers():
        # device layout: one 16-byte aligned buffer per layer, whatever its global offset
        return [torch.full((d, p), 0.25, dtype=torch.float32, device="cuda") for d, p in dims]

    shards = [(0, total), (1001 % total, max(1, total // 3)), (total - 1, 1), (total + 5, 10), (3, 0)]
    for s_off, s_cnt in shards:
        lo, hi = base + s_off, base + s_off + s_cnt
        ref = buffers()
        dp.dp_clipped_grad_multi(desc, dt, B, Cd, ref, accumulate)
        for (d, p), o_l, buf in zip(dims, offs, ref):
            b0, b1 = base + o_l, base + o_l + d * p
            x0, x1 = max(b0, lo), min(b1, hi)
            if x0 < x1:
                flat = buf.view(-1)
                dp.dp_add_noise(flat.data_ptr() + 4 * (x0 - b0), x0, x1 - x0, sigma, R, seed, step)
        got = buffers()
        dp.dp_clipped_grad_noise_multi(desc, dt, B, Cd, got, [base + o_l for o_l in offs], accumulate,
                                       lo, s_cnt, sigma, R, seed, step)
        for l, (x, y) in enumerate(zip(got, ref)):
            assert torch.equal(x, y), (l, s_off, s_cnt, float((x - y).abs().max()))
    # and against the oracle: noise values at the global indices, gradient from the definition
    l64 = [(si.to_f64(a), si.to_f64(g)) for a, g in layers]
    got = buffers()
    dp.dp_clipped_grad_noise_multi(desc, dt, B, Cd, got, [base + o_l for o_l in offs], 0, base, total,
                                   sigma, R, seed, step)
    for (a, g), (d, p), o_l, buf in zip(l64, dims, offs, got):
        G = o.clipped_grad(a, g, C.astype(np.float64))
        n_chk = min(d * p, 5000)
        z = o.normals(seed, step, base + o_l, n_chk)
        want = G.reshape(-1)[:n_chk] + sigma * R * z
        have = host(buf).reshape(-1)[:n_chk]
        assert np.all(np.abs(have - want) <= 2e-5 * sigma * R * np.maximum(1.0, np.abs(z)) + 1e-4 * np.abs(G.reshape(-1)[:n_chk]))


# ----------------------------------------------------------------------------
# gradient stored in the 16-bit type of the operands (dp_clipped_grad_noise_multi_h16)
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("accumulate", [0, 1])
@pytest.mark.parametrize("dims", [[(392, 520), (1800, 1544), (128, 136)],      # 63 tiles: 256 x 256-tile kernel
                                  [(392, 520), (136, 264)]])                    # 8 tiles: sub-tile kernel
@pytest.mark.parametrize("dtype", HALF_TYPES)
def test_half_precision_gradient_output(dp, dtype, dims, accumulate):
    B, T = 3, 96
    w = si.small_workload("h16", dtype, B, T, dims)
    layers = gen(w)
    l64 = [(si.to_f64(a), si.to_f64(g)) for a, g in layers]
    DT = dt_of(dp, dtype)
    tdt = torch.bfloat16 if dtype == si.BF16 else torch.float16
    keep = [(dev(a), dev(g)) for a, g in layers]
    desc = dp.layer_array([(a, g, T, d, p, 0) for (a, g), (d, p) in zip(keep, dims)])
    C = np.array([0.7, 0.0, 0.05], dtype=np.float32)
    Cd = dev(C)
    offs, acc = [], 4 * 10 ** 8
    for d, p in dims:
        offs.append(acc)
        acc += d * p + 8
    sigma, R, seed, step = 0.01, 2.0, 5, 9                       # noise of the gradient's own size
    lo, cnt = offs[0] + 1002, acc - offs[0] - 5000
    old16 = [(torch.randn(d, p, device="cuda") * 0.05).to(tdt) for d, p in dims]
    ref32 = [x.float().clone() for x in old16]
    dp.dp_clipped_grad_noise_multi(desc, DT, B, Cd, ref32, offs, accumulate, lo, cnt, sigma, R, seed, step)
    got16 = [x.clone() for x in old16]
    dp.dp_clipped_grad_noise_multi_h16(desc, DT, B, Cd, got16, offs, accumulate, lo, cnt, sigma, R, seed, step)
    torch.cuda.synchronize()
    ulp = 2.0 ** -8 if dtype == si.BF16 else 2.0 ** -11       # unit roundoff: largest relative error of one rounding
    for l, ((a, g), (d, p)) in enumerate(zip(l64, dims)):
        # the same fp32 value, rounded once to nearest even
        assert torch.equal(got16[l].view(torch.int16), ref32[l].to(tdt).view(torch.int16)), l
        # and against the definition: within one unit in the last place of the 16-bit type
        want = o.clipped_grad(a, g, C.astype(np.float64))
        if accumulate:
            want = want + old16[l].float().cpu().numpy().astype(np.float64)
        z = np.zeros(d * p)
        x0, x1 = max(offs[l], lo), min(offs[l] + d * p, lo + cnt)
        z[x0 - offs[l]:x1 - offs[l]] = o.normals(seed, step, x0, x1 - x0)
        want = want + sigma * R * z.reshape(d, p)
        have = got16[l].float().cpu().numpy().astype(np.float64)
        assert np.all(np.abs(have - want) <= ulp * np.abs(want) + 1e-7)
    # no noise: plain 16-bit weighted gradient
    plain = [torch.zeros((d, p), dtype=tdt, device="cuda") for d, p in dims]
    dp.dp_clipped_grad_noise_multi_h16(desc, DT, B, Cd, plain, None, 0, 0, 0, 0.0, 1.0, 0, 0)
    for l, (a, g) in enumerate(l64):
        want = o.clipped_grad(a, g, C.astype(np.float64))
        # (a value next to a rounding boundary may go to the other neighbour: still half a spacing away)
        # fp16 values below 6.1e-5 are subnormal: spacing 2^-24 whatever their size
        atol = 1e-9 if dtype == si.BF16 else 2.0 ** -24
        assert np.all(np.abs(plain[l].float().cpu().numpy() - want) <= ulp * (1 + 1e-3) * np.abs(want) + atol)


def test_half_precision_gradient_output_refusals(dp):
    B, T = 2, 96
    x = torch.zeros(1 << 20, dtype=torch.int16, device="cuda")
    p = x.data_ptr()
    out = torch.zeros(1 << 18, dtype=torch.int16, device="cuda")
    UNS = dp.DP_ERR_UNSUPPORTED
    def status(dims, dt, offs, sigma, T=T):
        desc = dp.layer_array([(p, p, T, d, q, 0) for d, q in dims])
        try:
            dp.dp_clipped_grad_noise_multi_h16(desc, dt, B, p, [out] * len(dims), offs, 0, 0, 1 << 30, sigma, 1.0, 0, 0)
        except dp.DpError as e:
            return e.status
        return dp.DP_OK
    assert status([(72, 264)], dp.DP_BF16, [0], 0.0) == UNS              # narrower than a large tile
    assert status([(128, 128)], dp.DP_BF16, [0], 0.0, T=50) == UNS       # T not a multiple of 32
    assert status([(128, 128)], dp.DP_F32, [0], 0.0) == UNS
    assert status([(128, 128)], dp.DP_F16, [2], 1.0) == UNS              # noise that does not start on a generator block
    assert status([(128, 128), (72, 264)], dp.DP_BF16, [0, 1 << 20], 1.0) == UNS
    torch.cuda.synchronize()
    assert not out.any()


# ----------------------------------------------------------------------------
# fp16 inputs without loss scaling (section 3.4 and the loss-scaling table)
# ----------------------------------------------------------------------------

def fp16_path_check(dp, Pipe, w, tol_norm=TOL_BF16_NORM):
    layers = gen(w)
    l64 = [(si.to_f64(a), si.to_f64(g)) for a, g in layers]
    pipe = Pipe([(dev(a), dev(g)) for a, g in layers])
    assert pipe.dt == dp.DP_F16
    pipe.norms()
    pipe.clip(w.clip_mode, w.R, w.stability)
    pipe.grad()
    sqn = np.stack([(o.ghost_sqnorm if path == o.PATH_GHOST else o.perex_sqnorm)(a, g)
                    for (a, g), path in zip(l64, pipe.paths)])
    assert np.all(np.isfinite(host(pipe.sqnorm)))
    assert rel(host(pipe.sqnorm), sqn) <= tol_norm
    C, _ = o.clip_factors(sqn, w.clip_mode, w.R, w.stability)
    assert rel(host(pipe.C), C) <= tol_norm
    for l, (a, g) in enumerate(l64):
        assert frob(host(pipe.grads[l]), o.clipped_grad(a, g, C)) <= 1e-4
    return pipe, l64, sqn


def test_fp16_gpt_block_stack(dp, Pipe):
    # one GPT-shaped block (d = 256) at T = 256: large-tile gradient kernel, whole-sample ghost norm,
    # and the instantiated norm on the square layer
    w = si.small_workload("h", si.F16, 4, 256, [(256, 768), (256, 256), (256, 1024), (1024, 256)],
                          clip_mode=si.CLIP_AUTOMATIC)
    pipe, _, _ = fp16_path_check(dp, Pipe, w)
    assert pipe.paths == [o.choose_path(w.T, d, p) for d, p in w.layers] == [0, 1, 0, 0]


def test_fp16_underflow_range_is_honoured(dp, Pipe):
    # Output gradients of 1e-6 are subnormal in fp16 (below 6.1e-5; spacing 6e-8), the low end of
    # the range the loss-scaling table lists for training without a loss scale.  They must reach
    # the sums as they are stored, not as zeros.
    w = si.small_workload("u", si.F16, 3, 160, [(136, 264), (264, 72)], g_std=1e-6,
                          clip_mode=si.CLIP_AUTOMATIC)
    g = si.gen_tensor(w, 0, 1)
    assert np.all(np.abs(g.astype(np.float64)) < 6.2e-5) and (g != 0).mean() > 0.9     # all subnormal
    pipe, _, sqn = fp16_path_check(dp, Pipe, w)
    assert np.all(sqn > 0) and np.all(host(pipe.sqnorm) > 0)


def test_fp16_large_range_does_not_overflow(dp, Pipe):
    # Activations of order 1e2 and a loss-scaled output gradient of order 10: Gram entries reach
    # 1e6 and above, beyond fp16's largest number (65504), the overflow the loss-scaling table
    # marks.  They are formed and summed in fp32 here, so the norms stay finite and correct.
    w = si.small_workload("o", si.F16, 2, 300, [(136, 264), (264, 136)], g_std=10.0, a_std=100.0)
    a = si.to_f64(si.gen_tensor(w, 0, 0))
    assert np.max(a[0] @ a[0].T) > 65504.0
    pipe, _, sqn = fp16_path_check(dp, Pipe, w)
    assert np.all(host(pipe.C) < 1e-6)                 # clipping does the scaling down


def test_argument_errors(dp):
    x = torch.zeros(4096, dtype=torch.float32, device="cuda")
    lib = dp.lib
    p = x.data_ptr()
    INV, WSP = dp.DP_ERR_INVALID_ARG, dp.DP_ERR_WORKSPACE
    assert lib.dp_ghost_norm(None, p, 1, 1, 8, 8, 8, p, p, 64, None) == INV
    assert lib.dp_ghost_norm(p, p, 1, 1, 8, 12, 8, p, p, 64, None) == INV      # bf16 row not 16 B
    assert lib.dp_ghost_norm(p, p, 1, 0, 8, 8, 8, p, p, 64, None) == INV
    assert lib.dp_ghost_norm(p, p, 7, 1, 8, 8, 8, p, p, 64, None) == INV       # bad dtype
    assert lib.dp_ghost_norm(p, p, 2, 1, 8, 12, 8, p, p, 64, None) == INV      # fp16 row not 16 B
    assert lib.dp_ghost_norm(p + 2, p, 1, 1, 8, 8, 8, p, p, 64, None) == INV   # misaligned
    assert lib.dp_ghost_norm(p, p, 1, 1, 8, 8, 8, p, None, 0, None) == WSP
    assert lib.dp_perex_norm(p, p, 1, 1, 8, 8, 8, p, p, 2, None) == WSP
    assert lib.dp_clip_factors(p, 1, 1, 0, 0.0, 0.01, p, None, None) == INV
    assert lib.dp_clip_factors(p, 1, 1, 0, float("nan"), 0.01, p, None, None) == INV
    assert lib.dp_clip_factors(p, 1, 1, 2, 1.0, 0.01, p, None, None) == INV
    assert lib.dp_clip_factors(p, 1, 1, 1, 1.0, -1.0, p, None, None) == INV
    assert lib.dp_clipped_grad(p, p, 1, 1, 8, 8, 8, None, p, 0, None) == INV
    assert lib.dp_clipped_grad(p, p, 1, 1, 8, 8, 8, p, p, 2, None) == INV
    assert lib.dp_add_noise(p, 0, 16, -1.0, 1.0, 0, 0, None) == INV
    assert lib.dp_add_noise(p, 0, 16, 1.0, float("inf"), 0, 0, None) == INV
    assert lib.dp_add_noise(p + 1, 0, 16, 1.0, 1.0, 0, 0, None) == INV
    assert lib.dp_add_noise(None, 0, 16, 1.0, 1.0, 0, 0, None) == INV
    assert lib.dp_add_noise(p, 2 ** 64 - 4, 16, 1.0, 1.0, 0, 0, None) == INV
    assert lib.dp_add_noise(p, 0, 0, 1.0, 1.0, 0, 0, None) == dp.DP_OK
    import ctypes
    arr = dp.layer_array([(p, p, 8, 8, 8, 0)])
    gp = (ctypes.c_void_p * 1)(p + 8192)
    offs = (ctypes.c_uint64 * 1)(0)
    assert lib.dp_clipped_grad_noise_multi(arr, 1, 1, 1, p, gp, None, 0, 0, 16, 1.0, 1.0, 0, 0, None) == INV
    assert lib.dp_clipped_grad_noise_multi(arr, 1, 1, 1, p, gp, offs, 0, 0, 16, -1.0, 1.0, 0, 0, None) == INV
    assert lib.dp_clipped_grad_noise_multi(arr, 1, 1, 1, p, gp, offs, 0, 2 ** 64 - 4, 16, 1.0, 1.0, 0, 0, None) == INV
    assert lib.dp_clipped_grad_noise_multi(arr, 1, 1, 1, p, gp, offs, 0, 0, 16, 1.0, float("inf"), 0, 0, None) == INV
    torch.cuda.synchronize()
    assert not host(x).any()
