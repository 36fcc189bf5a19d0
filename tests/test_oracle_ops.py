"""Pins for the oracle's operators: each is checked against something other than itself --
a library routine for the same textbook layer (torch CPU fp64 / numpy / scipy), closed
forms, invariants, and hand-computed small cases."""
import math

import numpy as np
import pytest
import scipy.special
import torch
import torch.nn.functional as F

from oracle import ops

RNG = np.random.default_rng(12345)
T64 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float64))


def close(a, b, tol=1e-12):
    a, b = np.asarray(a), np.asarray(b)
    assert a.shape == b.shape, (a.shape, b.shape)
    err = np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-300)
    assert err <= tol, err


# ---------------------------------------------------------------- patch embed
def test_patch_embed_matches_library_strided_conv():
    img = RNG.normal(size=(3, 42, 56))
    w = RNG.normal(size=(16, 3, 14, 14))
    b = RNG.normal(size=16)
    got = ops.patch_embed(img, w, b)
    ref = F.conv2d(T64(img)[None], T64(w), T64(b), stride=14)[0]          # [D][3][4]
    close(got, ref.permute(1, 2, 0).reshape(12, 16).numpy())


def test_patch_embed_one_hot_kernel_picks_pixel():
    # kernel that is 1 at (c=1,u=3,v=5) for d=0 and zero elsewhere: output = that pixel of each patch
    img = RNG.normal(size=(3, 28, 28))
    w = np.zeros((2, 3, 14, 14))
    w[0, 1, 3, 5] = 1.0
    out = ops.patch_embed(img, w, np.array([0.0, 7.0]))
    exp = np.array([img[1, 14 * i + 3, 14 * j + 5] for i in range(2) for j in range(2)])
    close(out[:, 0], exp)
    close(out[:, 1], np.full(4, 7.0))


# ---------------------------------------------------------------- layernorm
def test_layernorm_matches_library():
    x = RNG.normal(size=(7, 48)) * 3 + 1
    g, b = RNG.normal(size=48), RNG.normal(size=48)
    close(ops.layernorm(x, g, b, 1e-6), F.layer_norm(T64(x), (48,), T64(g), T64(b), 1e-6).numpy())


def test_layernorm_unit_affine_gives_zero_mean_and_known_variance():
    x = RNG.normal(size=(5, 64)) * 2.5
    eps = 1e-6
    y = ops.layernorm(x, np.ones(64), np.zeros(64), eps)
    assert np.max(np.abs(y.mean(axis=1))) < 1e-14
    var_in = x.var(axis=1)
    close(y.var(axis=1), var_in / (var_in + eps), 1e-12)


def test_layernorm_eps_matters_for_small_variance():
    x = np.array([[1e-3, -1e-3, 1e-3, -1e-3]])
    y = ops.layernorm(x, np.ones(4), np.zeros(4), 1e-6)
    close(y, x / math.sqrt(1e-6 + 1e-6))


# ---------------------------------------------------------------- linear
def test_linear_matches_matmul_and_is_not_transposed():
    x, w, b = RNG.normal(size=(5, 7)), RNG.normal(size=(7, 3)), RNG.normal(size=3)
    close(ops.linear(x, w, b), x @ w + b)
    close(ops.linear(x, w), x @ w)


# ---------------------------------------------------------------- attention
def _sdpa(qkv, nh, dh):
    N = qkv.shape[0]
    D = nh * dh
    q, k, v = (T64(qkv[:, i * D:(i + 1) * D]).reshape(N, nh, dh).permute(1, 0, 2) for i in range(3))
    return F.scaled_dot_product_attention(q, k, v).permute(1, 0, 2).reshape(N, D).numpy()


@pytest.mark.parametrize("N,nh,dh", [(5, 1, 8), (37, 3, 16), (70, 2, 64)])
def test_attention_matches_library(N, nh, dh):
    qkv = RNG.normal(size=(N, 3 * nh * dh))
    close(ops.attention(qkv, nh, dh), _sdpa(qkv, nh, dh), 1e-12)


def test_attention_rows_sum_to_one_and_scale_is_inverse_sqrt_dh():
    N, nh, dh = 9, 2, 16
    qkv = RNG.normal(size=(N, 3 * nh * dh))
    out, probs = ops.attention(qkv, nh, dh, return_probs=True)
    close(probs.sum(axis=2), np.ones((nh, N)), 1e-14)
    D = nh * dh
    q, k = qkv[:, :dh], qkv[:, D:D + dh]                      # head 0
    s = q @ k.T / math.sqrt(dh)
    e = np.exp(s - s.max(axis=1, keepdims=True))
    close(probs[0], e / e.sum(axis=1, keepdims=True), 1e-13)


def test_attention_identical_tokens_give_uniform_weights():
    N, nh, dh = 11, 2, 8
    row = RNG.normal(size=(1, 3 * nh * dh))
    out, probs = ops.attention(np.repeat(row, N, 0), nh, dh, return_probs=True)
    close(probs, np.full((nh, N, N), 1.0 / N), 1e-14)
    close(out, np.repeat(row[:, 2 * nh * dh:], N, 0), 1e-14)


def test_attention_equal_values_pass_through():
    N, nh, dh = 6, 2, 8
    D = nh * dh
    qkv = RNG.normal(size=(N, 3 * D))
    qkv[:, 2 * D:] = qkv[0, 2 * D:]
    close(ops.attention(qkv, nh, dh), np.repeat(qkv[:1, 2 * D:], N, 0), 1e-14)


def test_attention_heads_do_not_mix():
    # changing head 1's q/k/v leaves head 0's output columns untouched
    N, nh, dh = 7, 2, 8
    D = nh * dh
    a = RNG.normal(size=(N, 3 * D))
    b = a.copy()
    for third in range(3):
        b[:, third * D + dh:third * D + 2 * dh] = RNG.normal(size=(N, dh))
    oa, ob = ops.attention(a, nh, dh), ops.attention(b, nh, dh)
    close(oa[:, :dh], ob[:, :dh], 0.0)
    assert np.max(np.abs(oa[:, dh:] - ob[:, dh:])) > 1e-3


# ---------------------------------------------------------------- activations
def test_gelu_is_the_erf_form():
    x = np.linspace(-6, 6, 241)
    close(ops.gelu(x), 0.5 * x * (1 + scipy.special.erf(x / np.sqrt(2))), 1e-15)
    close(ops.gelu(x), F.gelu(T64(x)).numpy(), 1e-14)
    assert ops.gelu(np.zeros(1))[0] == 0.0
    assert np.max(np.abs(ops.gelu(x) - ops.gelu(-x) - x)) < 1e-15
    # the tanh approximation is measurably different, so this pin tells the two apart
    assert np.max(np.abs(ops.gelu(x) - F.gelu(T64(x), approximate="tanh").numpy())) > 1e-4


def test_swiglu_matches_library_and_reduces_to_silu():
    h = RNG.normal(size=(4, 10))
    a, b = T64(h[:, :5]), T64(h[:, 5:])
    close(ops.swiglu(h), (F.silu(a) * b).numpy(), 1e-14)
    h1 = h.copy()
    h1[:, 5:] = 1.0
    close(ops.swiglu(h1), F.silu(a).numpy(), 1e-14)
    # gate and linear halves are not interchangeable
    assert np.max(np.abs(ops.swiglu(h) - ops.swiglu(np.concatenate([h[:, 5:], h[:, :5]], 1)))) > 1e-3


def test_scale_residual():
    x, m, g = RNG.normal(size=(3, 4)), RNG.normal(size=(3, 4)), RNG.normal(size=4)
    close(ops.scale_residual(x, m, g), x + g[None, :] * m, 1e-15)


# ---------------------------------------------------------------- convolutions
@pytest.mark.parametrize("relu", [False, True])
def test_conv3x3_matches_library(relu):
    x, w, b = RNG.normal(size=(5, 6, 9)), RNG.normal(size=(4, 5, 3, 3)), RNG.normal(size=4)
    ref = F.conv2d(T64(x)[None], T64(w), T64(b), padding=1)[0]
    if relu:
        ref = F.relu(ref)
    close(ops.conv3x3(x, w, b, relu), ref.numpy(), 1e-13)


def test_conv3x3_centred_delta_is_identity_and_shift_pads_with_zero():
    x = RNG.normal(size=(2, 4, 5))
    w = np.zeros((2, 2, 3, 3))
    w[0, 0, 1, 1] = w[1, 1, 1, 1] = 1.0
    close(ops.conv3x3(x, w, np.zeros(2)), x, 0.0)
    # kernel 1 at (ky=0,kx=1): out[y][x] = in[y-1][x]; first row sees the zero padding
    w = np.zeros((1, 1, 3, 3))
    w[0, 0, 0, 1] = 1.0
    x1 = RNG.normal(size=(1, 3, 3))
    out = ops.conv3x3(x1, w, None)
    close(out[0, 1:], x1[0, :-1], 0.0)
    close(out[0, 0], np.zeros(3), 0.0)
    # kernel 1 at (ky=1,kx=2): out[y][x] = in[y][x+1]; last column is padding
    w = np.zeros((1, 1, 3, 3))
    w[0, 0, 1, 2] = 1.0
    out = ops.conv3x3(x1, w, None)
    close(out[0, :, :-1], x1[0, :, 1:], 0.0)
    close(out[0, :, -1], np.zeros(3), 0.0)


def test_conv3x3_all_ones_counts_neighbours_on_3x3():
    out = ops.conv3x3(np.ones((1, 3, 3)), np.ones((1, 1, 3, 3)), np.array([0.5]))
    close(out[0], np.array([[4, 6, 4], [6, 9, 6], [4, 6, 4]]) + 0.5, 0.0)


def test_conv1x1_is_per_pixel_matmul():
    x, w, b = RNG.normal(size=(6, 4, 5)), RNG.normal(size=(3, 6)), RNG.normal(size=3)
    close(ops.conv1x1(x, w, b), np.einsum("oc,chw->ohw", w, x) + b[:, None, None], 1e-14)


# ---------------------------------------------------------------- bilinear
@pytest.mark.parametrize("h,w,H,W", [(3, 4, 6, 8), (3, 4, 42, 56), (16, 24, 14, 21), (5, 7, 5, 7), (2, 2, 7, 5)])
def test_bilinear_matches_library_half_pixel(h, w, H, W):
    x = RNG.normal(size=(3, h, w))
    ref = F.interpolate(T64(x)[None], size=(H, W), mode="bilinear", align_corners=False)[0].numpy()
    close(ops.bilinear(x, H, W), ref, 1e-13)


def test_bilinear_properties():
    x = RNG.normal(size=(2, 5, 6))
    close(ops.bilinear(np.full((1, 4, 4), 3.25), 9, 11), np.full((1, 9, 11), 3.25), 1e-15)
    close(ops.bilinear(x, 5, 6), x, 0.0)
    up = ops.bilinear(x, 10, 12)
    assert up.max() <= x.max() + 1e-15 and up.min() >= x.min() - 1e-15
    # an affine ramp is reproduced exactly wherever no clamping happens (interior)
    yy, xx = np.meshgrid(np.arange(5.0), np.arange(6.0), indexing="ij")
    ramp = (2.0 * yy - 3.0 * xx + 1.0)[None]
    up = ops.bilinear(ramp, 10, 12)[0]
    sy = (np.arange(10) + 0.5) / 2 - 0.5
    sx = (np.arange(12) + 0.5) / 2 - 0.5
    exp = 2.0 * sy[:, None] - 3.0 * sx[None, :] + 1.0
    close(up[1:-1, 1:-1], exp[1:-1, 1:-1], 1e-14)
    # x2 upsampling weights are the 1/4-3/4 pattern
    line = ops.bilinear(np.array([[[0.0, 4.0]]]), 1, 4)[0, 0]
    close(line, np.array([0.0, 1.0, 3.0, 4.0]), 1e-15)


# ---------------------------------------------------------------- operators of the full DPT head
@pytest.mark.parametrize("H,W", [(7, 9), (8, 6), (1, 5), (34, 45)])
def test_conv3x3_stride2_matches_library(H, W):
    x, w, b = RNG.normal(size=(5, H, W)), RNG.normal(size=(4, 5, 3, 3)), RNG.normal(size=4)
    ref = F.conv2d(T64(x)[None], T64(w), T64(b), stride=2, padding=1)[0].numpy()
    close(ops.conv3x3_s2(x, w, b), ref, 1e-13)
    assert ops.conv3x3_s2(x, w, b).shape == (4, (H + 1) // 2, (W + 1) // 2)


def test_conv3x3_stride2_hand_cases():
    x = np.arange(30.0).reshape(1, 5, 6)
    delta = np.zeros((1, 1, 3, 3)); delta[0, 0, 1, 1] = 1.0
    close(ops.conv3x3_s2(x, delta, None), x[:, ::2, ::2], 0.0)                 # centre tap: every second pixel
    right = np.zeros((1, 1, 3, 3)); right[0, 0, 1, 2] = 1.0                     # tap (0, +1): in[2y][2x + 1]
    close(ops.conv3x3_s2(x, right, None), x[:, ::2, 1::2], 0.0)
    up = np.zeros((1, 1, 3, 3)); up[0, 0, 0, 1] = 1.0                           # tap (-1, 0): zero above the image
    exp = np.zeros((1, 3, 3)); exp[0, 1:] = x[0, 1:4:2, ::2]
    close(ops.conv3x3_s2(x, up, None), exp, 0.0)
    ones = ops.conv3x3_s2(np.ones((2, 4, 4)), np.ones((1, 2, 3, 3)), np.array([0.5]))
    close(ones, np.array([[[8.5, 12.5], [12.5, 18.5]]]), 0.0)                   # neighbours inside the image, x 2 channels


@pytest.mark.parametrize("s", [2, 4])
def test_conv_transpose_matches_library(s):
    x, w, b = RNG.normal(size=(5, 3, 4)), RNG.normal(size=(5, 6, s, s)), RNG.normal(size=6)
    ref = F.conv_transpose2d(T64(x)[None], T64(w), T64(b), stride=s)[0].numpy()
    close(ops.conv_transpose(x, w, b, s), ref, 1e-13)


def test_conv_transpose_paints_one_block_per_pixel():
    x = np.zeros((2, 3, 3)); x[1, 2, 0] = 2.0
    w = RNG.normal(size=(2, 3, 4, 4))
    out = ops.conv_transpose(x, w, None, 4)
    exp = np.zeros((3, 12, 12)); exp[:, 8:12, 0:4] = 2.0 * w[1]                 # input channel 1 -> all outputs
    close(out, exp, 0.0)
    close(ops.conv_transpose(np.zeros((2, 2, 2)), w, np.array([1.0, 2.0, 3.0]), 4)[:, 3, 5], np.array([1.0, 2.0, 3.0]), 0.0)


@pytest.mark.parametrize("h,w,H,W", [(3, 4, 6, 8), (17, 23, 34, 45), (16, 24, 14, 21), (5, 7, 5, 7), (2, 2, 7, 5), (4, 4, 1, 1), (1, 1, 3, 3)])
def test_bilinear_aligned_corners_matches_library(h, w, H, W):
    x = RNG.normal(size=(3, h, w))
    ref = F.interpolate(T64(x)[None], size=(H, W), mode="bilinear", align_corners=True)[0].numpy()
    close(ops.bilinear_ac(x, H, W), ref, 1e-13)


def test_bilinear_aligned_corners_properties():
    x = RNG.normal(size=(2, 5, 6))
    up = ops.bilinear_ac(x, 13, 16)
    close(up[:, [0, 0, -1, -1], [0, -1, 0, -1]], x[:, [0, 0, -1, -1], [0, -1, 0, -1]], 0.0)     # corners are copied
    close(ops.bilinear_ac(x, 5, 6), x, 1e-15)
    close(ops.bilinear_ac(x, 9, 11)[:, ::2, ::2], x, 1e-15)                     # 2 n - 1 samples contain the source
    # an affine ramp is reproduced exactly everywhere (no clamping region with aligned corners)
    yy, xx = np.meshgrid(np.arange(5.0), np.arange(6.0), indexing="ij")
    ramp = (2.0 * yy - 3.0 * xx + 1.0)[None]
    sy, sx = np.arange(13) * 4.0 / 12.0, np.arange(16) * 5.0 / 15.0
    close(ops.bilinear_ac(ramp, 13, 16)[0], 2.0 * sy[:, None] - 3.0 * sx[None, :] + 1.0, 1e-14)
    close(ops.bilinear_ac(np.array([[[0.0, 3.0]]]), 1, 4)[0, 0], np.array([0.0, 1.0, 2.0, 3.0]), 1e-15)
    # it differs from the half-pixel resize (which repeats the border)
    assert np.max(np.abs(ops.bilinear_ac(x, 10, 12) - ops.bilinear(x, 10, 12))) > 1e-2


def test_argmax_channels_ties_go_to_lowest_index():
    x = np.array([[[1.0, 5.0]], [[3.0, 5.0]], [[3.0, 2.0]]])        # [C=3][1][2]
    out = ops.argmax_channels(x)
    assert out.dtype == np.int32 and out.tolist() == [[1, 0]]
    z = RNG.normal(size=(9, 4, 5))
    assert np.array_equal(ops.argmax_channels(z), np.argmax(z, axis=0))
