"""Plain CPU oracle of the Book-Keeping (BK) per-sample clipped gradient.

TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Everything is float64 numpy written
straight from the definitions in the paper; nothing here is blocked, fused or
tuned, and nothing is shared with the HIP kernels.  Inputs are the same stored
values the GPU consumes (float32, or bfloat16 widened exactly to float64 by the
caller), so the two sides differ only by summation order and rounding.

Pins (tests/test_oracle_pins.py): brute-force Python loops on tiny inputs, closed
forms, the clipping bound, the reduction to a plain matrix product, an
independent library Philox engine, and distribution tests of the normals.
Every function here has at least one such pin; none is "parity unpinned" except
that the paper itself names no random generator, so the generator's layout
(counter/key assignment, uniform map, Box-Muller pairing) is this build's own
convention and is pinned only against the published Philox4x32-10 definition.

Notation follows the paper: a_l [B,T,d], g_l = dL/ds_l [B,T,p], per-sample weight
gradient a_{l,i}^T g_{l,i} [d,p], clip factor C_i, threshold R, noise level sigma.
"""
from __future__ import annotations

import numpy as np

PATH_GHOST = 0
PATH_PEREX = 1
CLIP_STANDARD = 0
CLIP_AUTOMATIC = 1


# ----------------------------------------------------------------------------
# Mixed ghost norm (appendix A.1, eq. "mixed ghost norm")
# ----------------------------------------------------------------------------

def choose_path(T: int, d: int, p: int) -> int:
    """Cheaper of the two norm techniques for one layer (appendix A.1, last paragraph).

    The paper only says "the cheaper"; the cost figures it attributes to the
    mixed-ghost-norm analysis are 2T^2 space for the two Gram matrices against
    p*d space for an instantiated per-sample gradient.  Reading taken: ghost norm
    iff 2*T^2 <= p*d, ties to ghost.
    """
    return PATH_GHOST if 2 * T * T <= d * p else PATH_PEREX


def perex_sqnorm(a: np.ndarray, g: np.ndarray) -> np.ndarray:
    """||a_i^T g_i||_F^2 by instantiating each per-sample gradient (eq. mixed ghost
    norm, left equality).  a [B,T,d], g [B,T,p] float64 -> [B] float64."""
    B = a.shape[0]
    out = np.empty(B, dtype=np.float64)
    for i in range(B):
        Gi = a[i].T @ g[i]                      # [d, p]
        out[i] = np.sum(Gi * Gi)
    return out


def ghost_sqnorm(a: np.ndarray, g: np.ndarray) -> np.ndarray:
    """vec(g_i g_i^T) . vec(a_i a_i^T) (eq. mixed ghost norm, right equality)."""
    B = a.shape[0]
    out = np.empty(B, dtype=np.float64)
    for i in range(B):
        gram_a = a[i] @ a[i].T                  # [T, T]
        gram_g = g[i] @ g[i].T                  # [T, T]
        out[i] = np.sum(gram_a * gram_g)
    return out


# ----------------------------------------------------------------------------
# Clip factors (section 2.1, "Per-sample gradient clipping"; eq. (1) with M = 1)
# ----------------------------------------------------------------------------

def clip_factors(sqnorm: np.ndarray, mode: int, R: float, stability: float = 0.01):
    """All-layer clipping: one group holding every layer's weights.

    sqnorm [L,B]: squared per-sample norms of each layer.  Returns (C [B], norm [B]).
    Standard: C_i = min(R/||g_i||, 1).  Automatic: C_i = R/(||g_i|| + stability)
    (the paper prints the R = 1 case with stability 0.01; with stability 0 a zero norm
    gives C_i = 0).  A squared norm that rounding pushed below zero counts as zero; a NaN
    norm gives a NaN factor in both modes.
    """
    total = np.sum(np.asarray(sqnorm, dtype=np.float64), axis=0)
    norm = np.sqrt(np.maximum(total, 0.0))
    if mode == CLIP_STANDARD:
        with np.errstate(divide="ignore"):
            C = np.minimum(np.float64(R) / norm, 1.0)
    elif mode == CLIP_AUTOMATIC:
        # A zero gradient with no stability constant is 0/0 in the paper's normalising form
        # (hook-free appendix: a_i^T g_i divided by its own norm).  Reading: its factor is 0 --
        # the sample adds nothing under any finite weight.
        den = norm + stability
        with np.errstate(divide="ignore", invalid="ignore"):
            C = np.where(den > 0, np.float64(R) / den, np.where(np.isnan(den), den, 0.0))
    else:
        raise ValueError("unknown clip mode")
    return C, norm


def clip_factors_grouped(sqnorm: np.ndarray, group_of_layer, R, mode: int, stability: float = 0.01):
    """Group-wise clipping (eq. (1) with M groups; section 2.1, "Mathematical gradient
    partition"): layer l belongs to group group_of_layer[l]; group m has its own threshold
    R[m] and its own per-sample norm over the group's layers.  Layer-wise clipping is one
    group per layer, all-layer clipping one group in all.  Returns (C [M,B], norm [M,B])."""
    sqnorm = np.asarray(sqnorm, dtype=np.float64)
    R = np.asarray(R, dtype=np.float64)
    M, B = len(R), sqnorm.shape[1]
    C = np.empty((M, B), dtype=np.float64)
    norm = np.empty((M, B), dtype=np.float64)
    for m in range(M):
        rows = [l for l, gm in enumerate(group_of_layer) if gm == m]
        if rows:
            C[m], norm[m] = clip_factors(sqnorm[rows], mode, R[m], stability)
        else:                                   # an empty group has zero gradient
            C[m], norm[m] = clip_factors(np.zeros((1, B)), mode, R[m], stability)
    return C, norm


def group_noise_std(sigma: float, R) -> float:
    """Standard deviation of the noise in eq. (1): sigma_DP * ||[R_1, ..., R_M]||_2."""
    return float(sigma) * float(np.sqrt(np.sum(np.asarray(R, dtype=np.float64) ** 2)))


# ----------------------------------------------------------------------------
# Bias (appendix A.1, last paragraph): dL_i/db = 1^T dL/ds_i, norm by instantiation
# ----------------------------------------------------------------------------

def bias_per_sample_grad(g: np.ndarray) -> np.ndarray:
    """Per-sample bias gradient: the sum of g[i] over its T token rows.  [B,T,p] -> [B,p]."""
    B, T, p = g.shape
    out = np.zeros((B, p), dtype=np.float64)
    for i in range(B):
        for t in range(T):
            out[i] += g[i, t]
    return out


def bias_sqnorm(g: np.ndarray) -> np.ndarray:
    """|| 1^T g_i ||^2 per sample."""
    bg = bias_per_sample_grad(g)
    return np.sum(bg * bg, axis=1)


def clipped_bias_grad(g: np.ndarray, C: np.ndarray) -> np.ndarray:
    """sum_i C_i 1^T g_i -> [p]."""
    bg = bias_per_sample_grad(g)
    out = np.zeros(g.shape[2], dtype=np.float64)
    for i in range(g.shape[0]):
        out += C[i] * bg[i]
    return out


# ----------------------------------------------------------------------------
# Clip-weighted gradient (section 3, "DP gradient": a^T diag(C_1..C_B) dL/ds)
# ----------------------------------------------------------------------------

def clipped_grad(a: np.ndarray, g: np.ndarray, C: np.ndarray) -> np.ndarray:
    """sum_i C_i a_i^T g_i -> [d, p] float64; C_i scales all T rows of sample i."""
    B, _, d = a.shape
    p = g.shape[2]
    G = np.zeros((d, p), dtype=np.float64)
    for i in range(B):
        G += C[i] * (a[i].T @ g[i])
    return G


def clipped_grad_entries(a, g, C, rows: np.ndarray, cols: np.ndarray) -> np.ndarray:
    """Selected entries G[rows[k], cols[k]] of clipped_grad, each computed on its own
    as sum_i C_i sum_t a[i,t,row] g[i,t,col].  `a`, `g` may be any dtype that widens
    exactly to float64 via the supplied arrays (callers pass float64 columns)."""
    B = a.shape[0]
    out = np.zeros(len(rows), dtype=np.float64)
    for i in range(B):
        out += C[i] * np.einsum("tk,tk->k", a[i][:, rows], g[i][:, cols])
    return out


# ----------------------------------------------------------------------------
# Gaussian noise: Philox4x32-10 counter-based generator + Box-Muller
# (eq. (1): the additive term sigma_DP * ||[R_1..R_M]|| * N(0, I), M = 1)
# ----------------------------------------------------------------------------

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK = np.uint64(0xFFFFFFFF)
_S32 = np.uint64(32)


def philox4x32_10(c0, c1, c2, c3, k0: int, k1: int):
    """Ten rounds of the Philox-4x32 bijection (Salmon et al., SC'11, section 3.3).

    c0..c3: uint32 arrays (the 128-bit counter, one per block); k0, k1: the 64-bit
    key as two Python ints.  Returns four uint32 arrays.
    """
    c0 = np.asarray(c0, dtype=np.uint64)
    c1 = np.asarray(c1, dtype=np.uint64)
    c2 = np.asarray(c2, dtype=np.uint64)
    c3 = np.asarray(c3, dtype=np.uint64)
    for rnd in range(10):
        key0 = np.uint64((k0 + rnd * _W0) & 0xFFFFFFFF)
        key1 = np.uint64((k1 + rnd * _W1) & 0xFFFFFFFF)
        prod0 = _M0 * c0                       # 32x32 -> 64, exact in uint64
        prod1 = _M1 * c2
        hi0, lo0 = prod0 >> _S32, prod0 & _MASK
        hi1, lo1 = prod1 >> _S32, prod1 & _MASK
        c0, c1, c2, c3 = hi1 ^ c1 ^ key0, lo1, hi0 ^ c3 ^ key1, lo0
    return (c0.astype(np.uint32), c1.astype(np.uint32),
            c2.astype(np.uint32), c3.astype(np.uint32))


def philox_blocks(seed: int, step: int, first_block: int, n_blocks: int) -> np.ndarray:
    """Raw generator output for blocks first_block .. first_block+n_blocks-1.

    Convention of this build: block k of the element stream has counter
    (k mod 2^32, k >> 32, step mod 2^32, step >> 32) and key (seed mod 2^32,
    seed >> 32).  Returns uint32 [n_blocks, 4].
    """
    k = np.arange(first_block, first_block + n_blocks, dtype=np.uint64)
    n = len(k)
    x = philox4x32_10(k & _MASK, k >> _S32,
                      np.full(n, step & 0xFFFFFFFF, dtype=np.uint64),
                      np.full(n, (step >> 32) & 0xFFFFFFFF, dtype=np.uint64),
                      seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    return np.stack(x, axis=1)


def uniforms_from_bits(x: np.ndarray) -> np.ndarray:
    """u = ((x >> 9) + 1/2) * 2^-23, strictly inside (0, 1) and exact in float32."""
    return ((np.asarray(x, dtype=np.uint32) >> np.uint32(9)).astype(np.float64) + 0.5) * 2.0 ** -23


def box_muller(u_a: np.ndarray, u_b: np.ndarray):
    """Two independent N(0,1) from two uniforms: r = sqrt(-2 ln u_a),
    (r cos 2 pi u_b, r sin 2 pi u_b)."""
    r = np.sqrt(-2.0 * np.log(u_a))
    ang = 2.0 * np.pi * u_b
    return r * np.cos(ang), r * np.sin(ang)


def normals(seed: int, step: int, offset: int, count: int) -> np.ndarray:
    """z_e for global elements e in [offset, offset+count), float64.

    Element e lives in block e >> 2; the block's outputs (x0,x1,x2,x3) give
    (z_{4k}, z_{4k+1}) from the uniform pair (x0, x1) and (z_{4k+2}, z_{4k+3}) from
    (x2, x3).
    """
    if count == 0:
        return np.zeros(0, dtype=np.float64)
    first = offset >> 2
    last = (offset + count - 1) >> 2
    x = philox_blocks(seed, step, first, last - first + 1)
    u = uniforms_from_bits(x)
    z = np.empty((len(x), 4), dtype=np.float64)
    z[:, 0], z[:, 1] = box_muller(u[:, 0], u[:, 1])
    z[:, 2], z[:, 3] = box_muller(u[:, 2], u[:, 3])
    z = z.reshape(-1)
    lead = offset - 4 * first
    return z[lead:lead + count]


def add_noise(grad_slice: np.ndarray, global_offset: int, sigma: float, R: float,
              seed: int, step: int) -> np.ndarray:
    """grad[e] + sigma*R*z_e on a contiguous slice starting at global element
    `global_offset`; float32 in, float32 out (sum formed in float64, rounded once).
    sigma == 0 means non-private: the slice is returned unchanged and sigma*R is
    never formed, so R may be infinite."""
    grad_slice = np.asarray(grad_slice, dtype=np.float32)
    if sigma == 0:
        return grad_slice.copy()
    z = normals(seed, step, global_offset, grad_slice.size).reshape(grad_slice.shape)
    return (grad_slice.astype(np.float64) + (float(sigma) * float(R)) * z).astype(np.float32)


# ----------------------------------------------------------------------------
# Whole path on one micro-batch (section 3, flowchart: output gradient ->
# clipping factor -> parameter gradient -> noising)
# ----------------------------------------------------------------------------

def private_gradient_grouped(layers, group_of_layer, R, mode: int, sigma: float, stability: float,
                             seed: int, step: int, noise_offset: int, noise_count: int,
                             with_bias: bool = False):
    """Group-wise form of private_gradient (eq. (1), M groups).  With `with_bias`, every layer
    also has a bias whose per-sample gradient 1^T g_i joins the layer's group; the flattened
    result is then [W_0, b_0, W_1, b_1, ...].  Noise level sigma * ||R||_2 on the given range."""
    L = len(layers)
    B = layers[0][0].shape[0]
    rows, row_group = [], []
    for l, (a, g) in enumerate(layers):
        path = choose_path(a.shape[1], a.shape[2], g.shape[2])
        rows.append(ghost_sqnorm(a, g) if path == PATH_GHOST else perex_sqnorm(a, g))
        row_group.append(group_of_layer[l])
        if with_bias:
            rows.append(bias_sqnorm(g))
            row_group.append(group_of_layer[l])
    sqn = np.stack(rows)
    C, norm = clip_factors_grouped(sqn, row_group, R, mode, stability)
    pieces, grads, bias_grads = [], [], []
    for l, (a, g) in enumerate(layers):
        G = clipped_grad(a, g, C[group_of_layer[l]])
        grads.append(G)
        pieces.append(G.reshape(-1))
        if with_bias:
            bgrad = clipped_bias_grad(g, C[group_of_layer[l]])
            bias_grads.append(bgrad)
            pieces.append(bgrad)
    flat = np.concatenate(pieces).astype(np.float32)
    if noise_count and sigma != 0:
        std = group_noise_std(sigma, R)
        sl = slice(noise_offset, noise_offset + noise_count)
        z = normals(seed, step, noise_offset, noise_count)
        flat[sl] = (flat[sl].astype(np.float64) + std * z).astype(np.float32)
    return dict(sqnorm=sqn, C=C, norm=norm, grads=grads, bias_grads=bias_grads, flat=flat)


def private_gradient(layers, mode: int, R: float, sigma: float, stability: float,
                     seed: int, step: int, noise_offset: int, noise_count: int,
                     force_path=None):
    """layers: list of (a [B,T,d], g [B,T,p]) float64 pairs.

    Returns dict with per-layer squared norms [L,B], chosen paths, C [B], the
    per-layer clipped gradients before noise (float64) and the flattened float32
    gradient after noise on [noise_offset, noise_offset+noise_count).
    """
    L = len(layers)
    B = layers[0][0].shape[0]
    sqn = np.empty((L, B), dtype=np.float64)
    paths = []
    for l, (a, g) in enumerate(layers):
        path = choose_path(a.shape[1], a.shape[2], g.shape[2]) if force_path is None else force_path
        paths.append(path)
        sqn[l] = ghost_sqnorm(a, g) if path == PATH_GHOST else perex_sqnorm(a, g)
    C, norm = clip_factors(sqn, mode, R, stability)
    grads = [clipped_grad(a, g, C) for a, g in layers]
    flat = np.concatenate([G.reshape(-1) for G in grads]).astype(np.float32)
    if noise_count:
        sl = slice(noise_offset, noise_offset + noise_count)
        flat[sl] = add_noise(flat[sl], noise_offset, sigma, R, seed, step)
    return dict(sqnorm=sqn, paths=paths, C=C, norm=norm, grads=grads, flat=flat)
