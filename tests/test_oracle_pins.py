"""Pins of the CPU oracle against things other than itself (CPU only).

Each test names the passage of the paper, or the piece of mathematics, that
fixes the expected value.  Brute-force references below are pure-Python loops
over scalars, written from the definition, not calls back into the oracle.
"""
import math
import os
import subprocess
import sys

import numpy as np
import pytest

from oracle import bk_oracle as o
import synth_inputs as si


# ----------------------------------------------------------------------------
# helpers: scalar brute force from the definitions
# ----------------------------------------------------------------------------

def brute_per_sample_grad(a_i, g_i):
    """a_i [T][d], g_i [T][p] -> nested list [d][p] of sum_t a[t][j] g[t][k]."""
    T, d, p = len(a_i), len(a_i[0]), len(g_i[0])
    return [[math.fsum(a_i[t][j] * g_i[t][k] for t in range(T)) for k in range(p)]
            for j in range(d)]


def brute_sqnorm(a_i, g_i):
    G = brute_per_sample_grad(a_i, g_i)
    return math.fsum(x * x for row in G for x in row)


def rand_ag(seed, B, T, d, p):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((B, T, d)), rng.standard_normal((B, T, p))


SHAPES = [(1, 1, 1, 1), (2, 1, 3, 5), (3, 4, 2, 7), (4, 8, 16, 16), (2, 7, 5, 3), (1, 6, 1, 4)]


# ----------------------------------------------------------------------------
# P1 / P2: per-sample squared norms (appendix A.1, eq. mixed ghost norm)
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("B,T,d,p", SHAPES)
def test_norms_equal_brute_force_frobenius(B, T, d, p):
    a, g = rand_ag(10 + T, B, T, d, p)
    want = np.array([brute_sqnorm(a[i].tolist(), g[i].tolist()) for i in range(B)])
    np.testing.assert_allclose(o.perex_sqnorm(a, g), want, rtol=1e-12)
    np.testing.assert_allclose(o.ghost_sqnorm(a, g), want, rtol=1e-11)


def test_cfg0_ghost_equals_instantiated():
    w = si.WORKLOADS["cfg0"]
    a, g = (si.to_f64(x) for x in si.gen_layer(w, 0))
    want = np.array([brute_sqnorm(a[i].tolist(), g[i].tolist()) for i in range(w.B)])
    np.testing.assert_allclose(o.ghost_sqnorm(a, g), want, rtol=1e-12)
    np.testing.assert_allclose(o.perex_sqnorm(a, g), want, rtol=1e-12)


def test_norms_match_library_routine():
    a, g = rand_ag(3, 3, 9, 6, 4)
    want = np.linalg.norm(np.einsum("itj,itk->ijk", a, g).reshape(3, -1), axis=1) ** 2
    np.testing.assert_allclose(o.perex_sqnorm(a, g), want, rtol=1e-12)
    np.testing.assert_allclose(o.ghost_sqnorm(a, g), want, rtol=1e-12)


def test_norm_closed_form_single_token():
    # T = 1: the per-sample gradient is an outer product, so its squared norm is |a|^2 |g|^2.
    a, g = rand_ag(4, 5, 1, 6, 3)
    want = np.sum(a[:, 0] ** 2, axis=1) * np.sum(g[:, 0] ** 2, axis=1)
    np.testing.assert_allclose(o.perex_sqnorm(a, g), want, rtol=1e-12)
    np.testing.assert_allclose(o.ghost_sqnorm(a, g), want, rtol=1e-12)


def test_norm_closed_form_repeated_activation_row():
    # Every token has the same activation v: a^T g = v (sum_t g_t)^T, norm^2 = |v|^2 |sum_t g_t|^2.
    rng = np.random.default_rng(5)
    v = rng.standard_normal(7)
    a = np.broadcast_to(v, (2, 5, 7)).copy()
    g = rng.standard_normal((2, 5, 4))
    want = np.sum(v ** 2) * np.sum(g.sum(axis=1) ** 2, axis=1)
    np.testing.assert_allclose(o.perex_sqnorm(a, g), want, rtol=1e-12)
    np.testing.assert_allclose(o.ghost_sqnorm(a, g), want, rtol=1e-12)


def test_norm_closed_form_one_hot_activations():
    # Orthonormal one-hot activation rows: a a^T = I, so norm^2 = sum_t |g_t|^2.
    rng = np.random.default_rng(6)
    T, d, p = 4, 6, 3
    a = np.zeros((1, T, d))
    a[0, np.arange(T), [5, 0, 3, 2]] = 1.0
    g = rng.standard_normal((1, T, p))
    want = np.array([np.sum(g ** 2)])
    np.testing.assert_allclose(o.perex_sqnorm(a, g), want, rtol=1e-12)
    np.testing.assert_allclose(o.ghost_sqnorm(a, g), want, rtol=1e-12)


def test_norm_is_not_symmetric_in_token_pairing():
    # A transposed operand or a mismatched token index must show: permuting the tokens of
    # g alone changes the answer, permuting a and g together does not.
    a, g = rand_ag(7, 1, 6, 4, 5)
    perm = np.array([3, 0, 5, 1, 4, 2])
    base = o.ghost_sqnorm(a, g)
    np.testing.assert_allclose(o.ghost_sqnorm(a[:, perm], g[:, perm]), base, rtol=1e-12)
    np.testing.assert_allclose(o.perex_sqnorm(a[:, perm], g[:, perm]), base, rtol=1e-12)
    assert abs(o.ghost_sqnorm(a, g[:, perm])[0] - base[0]) > 1e-3 * base[0]
    assert abs(o.perex_sqnorm(a, g[:, perm])[0] - base[0]) > 1e-3 * base[0]


# ----------------------------------------------------------------------------
# P5: path rule (appendix A.1: "the cheaper of two techniques at each layer")
# ----------------------------------------------------------------------------

def test_path_rule_on_workloads():
    for name, w in si.WORKLOADS.items():
        for d, p in w.layers:
            want = o.PATH_PEREX if name == "cfg3" else o.PATH_GHOST
            assert o.choose_path(w.T, d, p) == want, (name, d, p)


def test_path_rule_boundary():
    assert o.choose_path(8, 16, 8) == o.PATH_GHOST          # 2*64 == 128: tie -> ghost
    assert o.choose_path(8, 16, 7) == o.PATH_PEREX          # 128 > 112
    assert o.choose_path(4096, 768, 768) == o.PATH_PEREX    # long sequence
    assert o.choose_path(1, 1, 2) == o.PATH_GHOST


# ----------------------------------------------------------------------------
# P3: clip factors (section 2.1, eq. (1): ||C_i g_i|| <= R)
# ----------------------------------------------------------------------------

def test_clip_bound_and_values():
    rng = np.random.default_rng(8)
    sqn = rng.uniform(0.0, 4.0, size=(5, 9))
    sqn[:, 0] = 1e-6                                    # a sample well inside the ball
    n = np.sqrt(sqn.sum(axis=0))
    for R in (0.5, 1.0, 3.0):
        C, norm = o.clip_factors(sqn, o.CLIP_STANDARD, R)
        np.testing.assert_allclose(norm, n, rtol=1e-14)
        assert np.all(C * n <= R * (1 + 1e-12))
        clipped = n > R
        np.testing.assert_allclose((C * n)[clipped], R, rtol=1e-12)    # lands on the sphere
        assert np.all(C[~clipped] == 1.0)                               # untouched inside
        assert C[0] == 1.0
        Ca, _ = o.clip_factors(sqn, o.CLIP_AUTOMATIC, R)
        np.testing.assert_allclose(Ca * n, R * n / (n + 0.01), rtol=1e-12)
        assert np.all(Ca * n < R)


def test_clip_cross_layer_accumulation_is_sum_of_squares():
    # Hand-computed: layers contribute 9 and 16 -> norm 5.
    C, norm = o.clip_factors(np.array([[9.0], [16.0]]), o.CLIP_STANDARD, 1.0)
    assert norm[0] == 5.0 and C[0] == 0.2
    C, _ = o.clip_factors(np.array([[9.0], [16.0]]), o.CLIP_AUTOMATIC, 2.0)
    assert C[0] == pytest.approx(2.0 / 5.01, rel=1e-15)


def test_clip_degenerate_cases():
    C, norm = o.clip_factors(np.array([[0.0, -1e-12, 4.0]]), o.CLIP_STANDARD, 1.0)
    assert list(norm) == [0.0, 0.0, 2.0]
    assert list(C) == [1.0, 1.0, 0.5]                   # zero gradient is left alone
    C, _ = o.clip_factors(np.array([[0.0, 4.0]]), o.CLIP_STANDARD, math.inf)
    assert list(C) == [1.0, 1.0]                        # R = inf: nothing is clipped
    C, _ = o.clip_factors(np.array([[0.0]]), o.CLIP_AUTOMATIC, 1.0)
    assert C[0] == pytest.approx(100.0)
    # no stability constant (the normalising form of the hook-free appendix): every non-zero
    # gradient comes out with norm R exactly; a zero gradient gets factor 0, not R/0
    C, norm = o.clip_factors(np.array([[0.0, 4.0, 1e-30]]), o.CLIP_AUTOMATIC, 3.0, 0.0)
    assert C[0] == 0.0
    np.testing.assert_allclose((C * norm)[1:], 3.0, rtol=1e-15)
    # a gradient that is not a number shows in its factor in both modes
    for mode in (o.CLIP_STANDARD, o.CLIP_AUTOMATIC):
        C, norm = o.clip_factors(np.array([[np.nan, 4.0]]), mode, 1.0)
        assert np.isnan(C[0]) and np.isnan(norm[0]) and np.isfinite(C[1])


def test_standard_clipping_scale_invariance():
    # Once clipped, C_i g_i does not depend on the scale of g (it is R g_i/|g_i|).
    sqn = np.array([[4.0, 25.0], [5.0, 11.0]])
    C1, n1 = o.clip_factors(sqn, o.CLIP_STANDARD, 1.0)
    C2, n2 = o.clip_factors(sqn * 49.0, o.CLIP_STANDARD, 1.0)
    np.testing.assert_allclose(C1 * n1, C2 * n2, rtol=1e-14)
    np.testing.assert_allclose(C2, C1 / 7.0, rtol=1e-14)


# ----------------------------------------------------------------------------
# P4: clip-weighted gradient (section 3, DP gradient; C = 1, sigma = 0 is the standard one)
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("B,T,d,p", SHAPES)
def test_clipped_grad_equals_brute_force(B, T, d, p):
    a, g = rand_ag(20 + d, B, T, d, p)
    C = np.random.default_rng(1).uniform(0.1, 2.0, B)
    want = np.zeros((d, p))
    for i in range(B):
        want += C[i] * np.array(brute_per_sample_grad(a[i].tolist(), g[i].tolist()))
    np.testing.assert_allclose(o.clipped_grad(a, g, C), want, rtol=1e-12, atol=1e-13)


def test_unclipped_reduces_to_plain_matrix_product():
    # R -> infinity, sigma = 0: the private gradient is the ordinary a^T g over all B*T rows.
    w = si.WORKLOADS["cfg0"]
    a, g = (si.to_f64(x) for x in si.gen_layer(w, 0))
    res = o.private_gradient([(a, g)], o.CLIP_STANDARD, math.inf, 0.0, 0.01, 1, 0, 0, 256)
    assert np.all(res["C"] == 1.0)
    want = a.reshape(-1, 16).T @ g.reshape(-1, 16)
    np.testing.assert_allclose(res["grads"][0], want, rtol=1e-13, atol=1e-13)
    np.testing.assert_array_equal(res["flat"], want.reshape(-1).astype(np.float32))


def test_one_hot_clip_factor_selects_per_sample_gradient():
    a, g = rand_ag(9, 3, 5, 4, 6)
    for i in range(3):
        C = np.zeros(3)
        C[i] = 1.0
        want = np.array(brute_per_sample_grad(a[i].tolist(), g[i].tolist()))
        np.testing.assert_allclose(o.clipped_grad(a, g, C), want, rtol=1e-12, atol=1e-13)


def test_clipped_grad_entries_match_full():
    a, g = rand_ag(11, 3, 6, 5, 7)
    C = np.array([0.3, 1.0, 0.01])
    full = o.clipped_grad(a, g, C)
    rows = np.array([0, 4, 2, 2])
    cols = np.array([6, 0, 3, 3])
    np.testing.assert_allclose(o.clipped_grad_entries(a, g, C, rows, cols), full[rows, cols], rtol=1e-13)


def test_private_gradient_norm_bounds():
    # Each clipped per-sample gradient has norm <= R over the whole group, so the sum of B of
    # them has norm <= B R (eq. (1)); checked with per-sample gradients built by brute force.
    rng = np.random.default_rng(12)
    B, T = 4, 5
    dims = [(3, 4), (4, 2), (2, 6)]
    layers = [(rng.standard_normal((B, T, d)), rng.standard_normal((B, T, p))) for d, p in dims]
    for mode in (o.CLIP_STANDARD, o.CLIP_AUTOMATIC):
        res = o.private_gradient(layers, mode, 1.5, 0.0, 0.01, 0, 0, 0, 0)
        for i in range(B):
            sq = sum(brute_sqnorm(a[i].tolist(), g[i].tolist()) for a, g in layers)
            assert res["C"][i] * math.sqrt(sq) <= 1.5 * (1 + 1e-12)
            np.testing.assert_allclose(res["norm"][i], math.sqrt(sq), rtol=1e-12)
        total = math.sqrt(sum(np.sum(G ** 2) for G in res["grads"]))
        assert total <= B * 1.5


def test_mixed_clipped_and_unclipped_samples():
    # Output gradients of two samples are tiny, so the min(1, .) branch is taken for them.
    w = si.WORKLOADS["cfg0"]
    a, g = (si.to_f64(x) for x in si.gen_layer(w, 0))
    g[1] *= 1e-6
    g[3] *= 1e-6
    res = o.private_gradient([(a, g)], o.CLIP_STANDARD, 1.0, 0.0, 0.01, 0, 0, 0, 0)
    assert res["C"][1] == 1.0 and res["C"][3] == 1.0
    assert res["C"][0] < 1.0 and res["C"][2] < 1.0


def test_paths_agree_on_cfg0_pipeline():
    w = si.WORKLOADS["cfg0"]
    a, g = (si.to_f64(x) for x in si.gen_layer(w, 0))
    r0 = o.private_gradient([(a, g)], w.clip_mode, w.R, w.sigma, w.stability, 1, 0, 0, 256,
                            force_path=o.PATH_GHOST)
    r1 = o.private_gradient([(a, g)], w.clip_mode, w.R, w.sigma, w.stability, 1, 0, 0, 256,
                            force_path=o.PATH_PEREX)
    np.testing.assert_allclose(r0["C"], r1["C"], rtol=1e-12)
    np.testing.assert_allclose(r0["flat"], r1["flat"], rtol=1e-6, atol=1e-7)


# ----------------------------------------------------------------------------
# P6: Philox4x32-10 integers
# ----------------------------------------------------------------------------

def _mulhilo(a, b):
    prod = a * b
    return prod >> 32, prod & 0xFFFFFFFF


def philox_python_ints(ctr, key):
    """Independent scalar implementation on Python integers (SC'11 paper, section 3.3:
    two 32x32->64 multiplies, xor with the neighbours and the key, Weyl key schedule)."""
    c = list(ctr)
    k = list(key)
    for _ in range(10):
        hi0, lo0 = _mulhilo(0xD2511F53, c[0])
        hi1, lo1 = _mulhilo(0xCD9E8D57, c[2])
        c = [hi1 ^ c[1] ^ k[0], lo1, hi0 ^ c[3] ^ k[1], lo0]
        k = [(k[0] + 0x9E3779B9) & 0xFFFFFFFF, (k[1] + 0xBB67AE85) & 0xFFFFFFFF]
    return c


def test_philox_matches_python_integer_implementation():
    rng = np.random.default_rng(13)
    cases = rng.integers(0, 2 ** 32, size=(200, 6), dtype=np.uint64)
    for row in cases:
        c = [int(x) for x in row[:4]]
        k = [int(x) for x in row[4:]]
        got = o.philox4x32_10(*[np.array([x], dtype=np.uint32) for x in c], k[0], k[1])
        assert [int(x[0]) for x in got] == philox_python_ints(c, k)


@pytest.fixture(scope="module")
def library_engine(tmp_path_factory):
    """The Philox4x32-10 engine in the installed PyTorch headers, built as a host program."""
    import torch
    inc = os.path.join(os.path.dirname(torch.__file__), "include")
    if not os.path.exists(os.path.join(inc, "ATen/core/PhiloxRNGEngine.h")):
        pytest.skip("library Philox header not installed")
    exe = str(tmp_path_factory.mktemp("philox") / "engine")
    src = os.path.join(os.path.dirname(__file__), "philox_library_engine.cpp")
    subprocess.run(["g++", "-O1", "-std=c++17", "-I", inc, src, "-o", exe], check=True)

    def run(seed, subseq, offset, n):
        out = subprocess.run([exe, str(seed), str(subseq), str(offset), str(n)],
                             check=True, capture_output=True, text=True).stdout
        return np.array([[int(x, 16) for x in line.split()] for line in out.splitlines()],
                        dtype=np.uint32)
    return run


@pytest.mark.parametrize("seed,step,first,n", [
    (0, 0, 0, 64),
    (1, 0, 0, 1000),
    (0xDEADBEEFCAFEF00D, 7, 12345, 257),
    (3, (1 << 40) + 5, (1 << 32) - 3, 16),          # block index crosses 2^32
    (2 ** 64 - 1, 2 ** 64 - 1, 2 ** 33 + 1, 8),
])
def test_philox_matches_library_engine(library_engine, seed, step, first, n):
    # The library engine's (seed, subsequence, offset) are key, counter words 2-3, and
    # counter words 0-1: the same assignment as this build's (seed, step, block).
    want = library_engine(seed, step, first, n)
    np.testing.assert_array_equal(o.philox_blocks(seed, step, first, n), want)


def test_philox_avalanche():
    # Flipping any single counter or key bit changes about half of the 128 output bits.
    base_c = [0x12345678, 0x9ABCDEF0, 0x0F1E2D3C, 0x4B5A6978]
    base_k = [0xA5A5A5A5, 0x3C3C3C3C]
    ref = philox_python_ints(base_c, base_k)
    flips = []
    for word in range(6):
        for bit in range(32):
            c, k = list(base_c), list(base_k)
            if word < 4:
                c[word] ^= 1 << bit
            else:
                k[word - 4] ^= 1 << bit
            got = o.philox4x32_10(*[np.array([x], dtype=np.uint32) for x in c], k[0], k[1])
            flips.append(sum(bin(int(x[0]) ^ y).count("1") for x, y in zip(got, ref)))
    flips = np.array(flips)
    assert flips.min() >= 35 and flips.max() <= 93
    assert abs(flips.mean() - 64.0) < 3.0


def test_philox_is_a_bijection_on_counters():
    x = o.philox_blocks(5, 0, 0, 1 << 16)
    packed = x.astype(np.uint64)
    keys = (packed[:, 0] << np.uint64(32) | packed[:, 1]), (packed[:, 2] << np.uint64(32) | packed[:, 3])
    assert len(set(zip(keys[0].tolist(), keys[1].tolist()))) == 1 << 16


# ----------------------------------------------------------------------------
# P7: normals (eq. (1): the noise is N(0, I))
# ----------------------------------------------------------------------------

def test_uniform_map_range_and_exactness():
    u = o.uniforms_from_bits(np.array([0, 0x1FF, 0x200, 0xFFFFFFFF], dtype=np.uint32))
    assert u[0] == 2.0 ** -24 and u[1] == 2.0 ** -24
    assert u[2] == 1.5 * 2.0 ** -23
    assert u[3] == 1.0 - 2.0 ** -24
    assert np.all(u.astype(np.float32).astype(np.float64) == u)     # representable in float32


def test_box_muller_known_angles():
    # u_b = 0, 1/4, 1/2 give the axes; u_a = exp(-1/2) gives radius 1.
    ua = np.full(3, math.exp(-0.5))
    z0, z1 = o.box_muller(ua, np.array([0.0, 0.25, 0.5]))
    np.testing.assert_allclose(z0, [1.0, 0.0, -1.0], atol=1e-15)
    np.testing.assert_allclose(z1, [0.0, 1.0, 0.0], atol=1e-15)
    z0, z1 = o.box_muller(np.array([math.exp(-2.0)]), np.array([0.125]))
    np.testing.assert_allclose([z0[0], z1[0]], [math.sqrt(2.0), math.sqrt(2.0)], rtol=1e-15)


def test_normals_pairing_with_raw_stream():
    # z_{4k}^2 + z_{4k+1}^2 = -2 ln u(x0) and the angle comes from x1; same for (x2, x3).
    x = o.philox_blocks(1, 0, 10, 50)
    z = o.normals(1, 0, 40, 200).reshape(50, 4)
    for col in (0, 2):
        ua = ((x[:, col] >> 9).astype(np.float64) + 0.5) / 2 ** 23
        ub = ((x[:, col + 1] >> 9).astype(np.float64) + 0.5) / 2 ** 23
        np.testing.assert_allclose(z[:, col] ** 2 + z[:, col + 1] ** 2, -2 * np.log(ua), rtol=1e-12)
        ang = np.mod(np.arctan2(z[:, col + 1], z[:, col]) / (2 * np.pi), 1.0)
        np.testing.assert_allclose(ang, ub, atol=1e-12)


def test_normals_distribution():
    from scipy import stats
    n = 1 << 20
    z = o.normals(1, 0, 0, n)
    assert abs(z.mean()) < 5 / math.sqrt(n)
    assert abs(z.var() - 1.0) < 5 * math.sqrt(2.0 / n)
    assert np.max(np.abs(z)) <= math.sqrt(-2 * math.log(2.0 ** -24)) + 1e-12
    for lag in (1, 2, 3, 4):
        assert abs(np.mean(z[:-lag] * z[lag:])) < 5 / math.sqrt(n)
    assert abs(stats.kurtosis(z)) < 0.03 and abs(stats.skew(z)) < 0.02
    assert stats.kstest(z[: 1 << 17], "norm").pvalue > 1e-3
    # another seed and step are independent streams
    z2 = o.normals(2, 0, 0, n)
    z3 = o.normals(1, 1, 0, n)
    assert abs(np.mean(z * z2)) < 5 / math.sqrt(n)
    assert abs(np.mean(z * z3)) < 5 / math.sqrt(n)


def test_normals_range_split_and_unaligned_offsets():
    full = o.normals(9, 3, 0, 103)
    for off, cnt in [(0, 40), (40, 63), (1, 5), (3, 1), (7, 96), (102, 1)]:
        np.testing.assert_array_equal(o.normals(9, 3, off, cnt), full[off:off + cnt])
    assert o.normals(9, 3, 5, 0).size == 0


# ----------------------------------------------------------------------------
# P8: noise placement and level (eq. (1): sigma * R * N(0, I) on the rank's slice)
# ----------------------------------------------------------------------------

def test_noise_level_and_placement():
    n = 1 << 18
    base = np.random.default_rng(14).standard_normal(n).astype(np.float32)
    out = o.add_noise(base[1000:1000 + 65536], 1000, 0.5, 3.0, 1, 0)
    delta = out.astype(np.float64) - base[1000:1000 + 65536]
    assert abs(delta.std() - 1.5) < 1.5 * 5 * math.sqrt(1.0 / 65536)
    np.testing.assert_allclose(delta, 1.5 * o.normals(1, 0, 1000, 65536), atol=2e-6)
    # sigma = 0 with R = inf leaves the gradient untouched
    np.testing.assert_array_equal(o.add_noise(base[:8], 0, 0.0, math.inf, 1, 0), base[:8])


def test_noise_only_touches_the_shard():
    rng = np.random.default_rng(15)
    B, T = 2, 3
    layers = [(rng.standard_normal((B, T, 4)), rng.standard_normal((B, T, 5))),
              (rng.standard_normal((B, T, 5)), rng.standard_normal((B, T, 4)))]
    clean = o.private_gradient(layers, o.CLIP_STANDARD, 1.0, 0.0, 0.01, 1, 0, 0, 0)["flat"]
    noisy = o.private_gradient(layers, o.CLIP_STANDARD, 1.0, 0.7, 0.01, 1, 0, 16, 12)["flat"]
    np.testing.assert_array_equal(noisy[:16], clean[:16])
    np.testing.assert_array_equal(noisy[28:], clean[28:])
    want = clean[16:28].astype(np.float64) + 0.7 * o.normals(1, 0, 16, 12)   # crosses the layer boundary at 20
    np.testing.assert_allclose(noisy[16:28], want, rtol=1e-6)


# ----------------------------------------------------------------------------
# input generator sanity (value ranges quoted in the paper's loss-scaling table)
# ----------------------------------------------------------------------------

def test_bf16_rounding_helper():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.3895314e38, 1e-40], dtype=np.float32)
    b = si.f32_to_bf16_bits(x)
    back = si.bf16_bits_to_f32(b)
    assert back[0] == 1.0 and back[3] == -2.5
    assert back[1] == 1.0                       # tie -> even mantissa
    assert back[2] == np.float32(1.015625)      # tie -> even (up)
    assert np.all(np.abs(back[:4] - x[:4]) <= np.abs(x[:4]) * 2.0 ** -8)


def test_synthetic_ranges_and_determinism():
    w = si.WORKLOADS["cfg1"]
    a1 = si.gen_tensor(w, 1, 0)
    a2 = si.gen_tensor(w, 1, 0)
    np.testing.assert_array_equal(a1, a2)
    a = si.bf16_bits_to_f32(a1)
    g = si.bf16_bits_to_f32(si.gen_tensor(w, 1, 1))
    assert 0.99 < a.std() < 1.01 and np.abs(a).max() < 1e2
    s = si.layer_g_scale(w, 1)
    assert 0.5 <= s < 2.0
    assert abs(g.std() / (1e-2 * s) - 1.0) < 0.01 and np.abs(g).max() < 1e1
    assert si.WORKLOADS["cfg4"].noise_range() == (0, 226492416)
    assert si.WORKLOADS["cfg1"].psi == 84934656 and si.WORKLOADS["cfg2"].psi == 707788800


# ----------------------------------------------------------------------------
# group-wise clipping (eq. (1) with M groups; section 2.1) and bias gradients (appendix A.1)
# ----------------------------------------------------------------------------

def test_grouped_clipping_one_group_is_all_layer():
    rng = np.random.default_rng(21)
    sqn = rng.uniform(0, 3, size=(4, 6))
    for mode in (o.CLIP_STANDARD, o.CLIP_AUTOMATIC):
        C1, n1 = o.clip_factors(sqn, mode, 1.3)
        Cg, ng = o.clip_factors_grouped(sqn, [0, 0, 0, 0], [1.3], mode)
        np.testing.assert_array_equal(Cg[0], C1)
        np.testing.assert_array_equal(ng[0], n1)


def test_grouped_clipping_hand_values():
    # layers 0 and 2 form group 0 (9 + 16 -> norm 5), layer 1 is group 1 (norm 2)
    sqn = np.array([[9.0], [4.0], [16.0]])
    C, norm = o.clip_factors_grouped(sqn, [0, 1, 0], [1.0, 4.0], o.CLIP_STANDARD)
    assert norm[0, 0] == 5.0 and norm[1, 0] == 2.0
    assert C[0, 0] == 0.2 and C[1, 0] == 1.0           # group 1 is inside its ball (R = 4)
    C, _ = o.clip_factors_grouped(sqn, [0, 1, 0], [1.0, 4.0], o.CLIP_AUTOMATIC)
    assert C[0, 0] == pytest.approx(1 / 5.01) and C[1, 0] == pytest.approx(4 / 2.01)


def test_layerwise_clipping_bounds_every_group():
    # ||C_{m,i} g_{[m],i}|| <= R_m for every group m and sample i, from brute-force gradients
    rng = np.random.default_rng(22)
    B, T = 3, 4
    dims = [(3, 4), (4, 2), (2, 5)]
    layers = [(rng.standard_normal((B, T, d)), rng.standard_normal((B, T, p))) for d, p in dims]
    R = [0.5, 2.0, 1e3]
    res = o.private_gradient_grouped(layers, [0, 1, 2], R, o.CLIP_STANDARD, 0.0, 0.01, 0, 0, 0, 0)
    for m, (a, g) in enumerate(layers):
        for i in range(B):
            n = math.sqrt(brute_sqnorm(a[i].tolist(), g[i].tolist()))
            assert res["C"][m, i] * n <= R[m] * (1 + 1e-12)
            np.testing.assert_allclose(res["norm"][m, i], n, rtol=1e-12)
        assert np.all(res["C"][2] == 1.0)               # R = 1000: nothing clipped in group 2
        want = sum(res["C"][m, i] * np.array(brute_per_sample_grad(a[i].tolist(), g[i].tolist())) for i in range(B))
        np.testing.assert_allclose(res["grads"][m], want, rtol=1e-12, atol=1e-13)


def test_group_noise_level():
    assert o.group_noise_std(0.5, [3.0, 4.0]) == 2.5
    assert o.group_noise_std(2.0, [1.5]) == 3.0
    rng = np.random.default_rng(23)
    layers = [(rng.standard_normal((2, 3, 64)), rng.standard_normal((2, 3, 512))) for _ in range(2)]
    clean = o.private_gradient_grouped(layers, [0, 1], [3.0, 4.0], o.CLIP_STANDARD, 0.0, 0.01, 1, 0, 0, 65536)["flat"]
    noisy = o.private_gradient_grouped(layers, [0, 1], [3.0, 4.0], o.CLIP_STANDARD, 0.5, 0.01, 1, 0, 0, 65536)["flat"]
    delta = noisy.astype(np.float64) - clean
    assert abs(delta.std() / 2.5 - 1) < 5 / math.sqrt(2 * 65536)
    np.testing.assert_allclose(delta, 2.5 * o.normals(1, 0, 0, 65536), atol=1e-5)


def test_bias_gradient_brute_force_and_closed_forms():
    rng = np.random.default_rng(24)
    g = rng.standard_normal((3, 5, 4))
    want = np.array([[math.fsum(g[i, t, k] for t in range(5)) for k in range(4)] for i in range(3)])
    np.testing.assert_allclose(o.bias_per_sample_grad(g), want, rtol=1e-14, atol=1e-15)
    np.testing.assert_allclose(o.bias_sqnorm(g), np.sum(want ** 2, axis=1), rtol=1e-13)
    # one token: the bias gradient is that row
    np.testing.assert_array_equal(o.bias_per_sample_grad(g[:, :1]), g[:, 0])
    # unit weights: the plain bias gradient, column sums over all B*T rows (library routine)
    np.testing.assert_allclose(o.clipped_bias_grad(g, np.ones(3)), g.reshape(-1, 4).sum(axis=0), rtol=1e-13)
    C = np.array([0.5, 0.0, 2.0])
    np.testing.assert_allclose(o.clipped_bias_grad(g, C), 0.5 * want[0] + 2.0 * want[2], rtol=1e-13)
    # rows that cancel: zero bias gradient whatever the weight gradient is
    g2 = np.stack([np.concatenate([g[0], -g[0]])])
    assert np.all(np.abs(o.bias_sqnorm(g2)) < 1e-28)


def test_bias_joins_the_group_norm():
    rng = np.random.default_rng(25)
    B, T = 2, 3
    layers = [(rng.standard_normal((B, T, 3)), rng.standard_normal((B, T, 4)))]
    res = o.private_gradient_grouped(layers, [0], [1.0], o.CLIP_STANDARD, 0.0, 0.01, 0, 0, 0, 0, with_bias=True)
    a, g = layers[0]
    for i in range(B):
        total = brute_sqnorm(a[i].tolist(), g[i].tolist()) + float(np.sum(g[i].sum(axis=0) ** 2))
        np.testing.assert_allclose(res["norm"][0, i], math.sqrt(total), rtol=1e-12)
        assert res["C"][0, i] * math.sqrt(total) <= 1.0 + 1e-12
    assert res["flat"].size == 3 * 4 + 4
    np.testing.assert_allclose(res["flat"][12:], res["bias_grads"][0], rtol=1e-6)


# ----------------------------------------------------------------------------
# fixtures under tests/golden/
# ----------------------------------------------------------------------------

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [line.split() for line in f if line.strip() and not line.startswith("#")]


def test_synthetic_inputs_lie_in_the_ranges_the_paper_prints():
    # Loss-scaling table of section 3.4, row "DP w/o scaling".  Typical magnitudes (1st percentile
    # to maximum of the absolute values) of the synthetic activations and output gradients must lie
    # inside the printed ranges; Gram diagonals within a decade of theirs (the table is for one
    # model, the stand-in layers are 768 to 3072 wide).
    rng = {r[0]: (float(r[1]), float(r[2])) for r in _rows("loss_scaling_table_ranges.txt")}
    w = si.WORKLOADS["cfg1"]
    w = si.small_workload("ranges", w.dtype, 2, w.T, w.layers[:4], g_std=w.g_std, g_layer_scale=True)
    for l in range(w.L):
        a, g = (si.to_f64(x) for x in si.gen_layer(w, l))
        for x, key in ((a, "activation"), (g, "output_grad")):
            mag = np.abs(x[x != 0])
            lo, hi = rng[key]
            assert np.percentile(mag, 1) >= lo and mag.max() <= hi, (l, key)
        for x, key in ((a, "gram_activation"), (g, "gram_output_grad")):
            diag = np.einsum("itk,itk->it", x, x)
            lo, hi = rng[key]
            assert diag.min() >= lo / 10 and diag.max() <= hi * 10, (l, key, diag.min(), diag.max())
