"""Pins for the convolution-chain oracle (CPU only).

The paper gives the conv chains as a table of shapes only (Evaluation, "The configuration of
conv chain"), so the oracle's definition -- stride 1, zero padding k/2, cross-correlation,
channels-last -- is pinned to independent routines and closed forms:
  * torch's CPU conv2d in float64 (a library routine with its own layouts: NCHW / OIHW), for
    odd kernels 1, 3, 5 in both positions, non-square images and channel counts,
  * the 1x1 / 1x1 case against the (separately pinned) GEMM-chain oracle on the pixel rows,
  * delta kernels: a single tap with the identity over channels must shift the image and
    leave zeros at the border it shifted in from,
  * a pure-Python brute-force twin with a different loop nest,
  * zero weights, and the negative twin of the activation rule: summing taps AFTER the
    activation must not reproduce the result (Sec. 4.3 Rule 3 carries over to the taps).
"""
import numpy as np
import pytest
import torch

import oracle
from oracle import ACT_GELU_TANH, ACT_IDENTITY, ACT_RELU, ACT_SILU


def rnd(seed, shape, scale=1.0):
    return np.random.default_rng(seed).standard_normal(shape).astype(np.float32) * np.float32(scale)


def torch_act(kind, t):
    if kind == ACT_RELU:
        return torch.relu(t)
    if kind == ACT_GELU_TANH:
        return torch.nn.functional.gelu(t, approximate="tanh")
    if kind == ACT_SILU:
        return torch.nn.functional.silu(t)
    return t


def torch_chain(X, W1, W2, kind):
    x = torch.from_numpy(X.astype(np.float64)).permute(0, 3, 1, 2)          # NHWC -> NCHW
    w1 = torch.from_numpy(W1.astype(np.float64)).permute(3, 2, 0, 1)        # HWIO -> OIHW
    w2 = torch.from_numpy(W2.astype(np.float64)).permute(3, 2, 0, 1)
    a = torch_act(kind, torch.nn.functional.conv2d(x, w1, padding=W1.shape[0] // 2))
    y = torch.nn.functional.conv2d(a, w2, padding=W2.shape[0] // 2)
    return y.permute(0, 2, 3, 1).numpy(), a.permute(0, 2, 3, 1).numpy()


@pytest.mark.parametrize("k1,k2", [(1, 1), (3, 1), (1, 3), (3, 3), (5, 1), (3, 5)])
@pytest.mark.parametrize("kind", [ACT_RELU, ACT_GELU_TANH, ACT_SILU])
def test_against_torch_conv2d_float64(k1, k2, kind):
    B, H, W, IC, OC1, OC2 = 2, 5, 7, 6, 10, 4
    X = rnd(1, (B, H, W, IC))
    W1 = rnd(2, (k1, k1, IC, OC1), (k1 * k1 * IC) ** -0.5)
    W2 = rnd(3, (k2, k2, OC1, OC2), (k2 * k2 * OC1) ** -0.5)
    Y, A = oracle.conv_chain(X, W1, W2, kind, want_a=True)
    Yt, At = torch_chain(X, W1, W2, kind)
    assert np.max(np.abs(A - At)) <= 1e-12 * max(1.0, np.max(np.abs(At)))
    assert np.max(np.abs(Y - Yt)) <= 1e-12 * max(1.0, np.max(np.abs(Yt)))


def test_image_smaller_than_the_kernel():
    X = rnd(4, (1, 2, 1, 3))
    W1 = rnd(5, (5, 5, 3, 4))
    W2 = rnd(6, (3, 3, 4, 2))
    Y = oracle.conv_chain(X, W1, W2, ACT_SILU)
    Yt, _ = torch_chain(X, W1, W2, ACT_SILU)
    assert np.allclose(Y, Yt, rtol=0, atol=1e-12)


@pytest.mark.parametrize("kind", [ACT_RELU, ACT_GELU_TANH])
def test_pointwise_chain_is_the_gemm_chain_on_pixel_rows(kind):
    B, H, W, IC, OC1, OC2 = 2, 3, 5, 12, 20, 8
    X = rnd(7, (B, H, W, IC))
    W1 = rnd(8, (1, 1, IC, OC1), IC ** -0.5)
    W2 = rnd(9, (1, 1, OC1, OC2), OC1 ** -0.5)
    Y = oracle.conv_chain(X, W1, W2, kind)
    ref = oracle.ffn(X.reshape(B * H * W, IC), W1.reshape(IC, OC1), None, W2.reshape(OC1, OC2), kind)
    assert np.array_equal(Y.reshape(B * H * W, OC2), ref)


@pytest.mark.parametrize("tap", [(0, 0), (0, 2), (1, 1), (2, 0), (2, 1)])
def test_delta_kernel_shifts_the_image_and_pads_with_zeros(tap):
    """W1 = identity over channels at one tap (kh, kw): A[h][w] = X[h+kh-1][w+kw-1], zero outside."""
    B, H, W, C = 1, 4, 5, 3
    X = rnd(10, (B, H, W, C))
    W1 = np.zeros((3, 3, C, C), np.float32)
    W1[tap[0], tap[1]] = np.eye(C, dtype=np.float32)
    W2 = np.eye(C, dtype=np.float32).reshape(1, 1, C, C)
    Y = oracle.conv_chain(X, W1, W2, ACT_IDENTITY)
    want = np.zeros((B, H, W, C))
    dh, dw = tap[0] - 1, tap[1] - 1
    for h in range(H):
        for w in range(W):
            if 0 <= h + dh < H and 0 <= w + dw < W:
                want[0, h, w] = X[0, h + dh, w + dw]
    assert np.array_equal(Y, want)


def test_brute_force_twin():
    B, H, W, IC, OC1, OC2, k1, k2 = 1, 3, 4, 2, 3, 2, 3, 3
    X = rnd(11, (B, H, W, IC)).astype(np.float64)
    W1 = rnd(12, (k1, k1, IC, OC1)).astype(np.float64)
    W2 = rnd(13, (k2, k2, OC1, OC2)).astype(np.float64)
    A = np.zeros((B, H, W, OC1))
    for o in range(OC1):                      # output channel outermost: not the oracle's nest
        for h in range(H):
            for w in range(W):
                s = 0.0
                for ic in range(IC):
                    for kw in range(k1):
                        for kh in range(k1):
                            hh, ww = h + kh - 1, w + kw - 1
                            if 0 <= hh < H and 0 <= ww < W:
                                s += X[0, hh, ww, ic] * W1[kh, kw, ic, o]
                A[0, h, w, o] = max(s, 0.0)
    Y = np.zeros((B, H, W, OC2))
    for q in range(OC2):
        for h in range(H):
            for w in range(W):
                s = 0.0
                for o in range(OC1):
                    for kh in range(k2):
                        for kw in range(k2):
                            hh, ww = h + kh - 1, w + kw - 1
                            if 0 <= hh < H and 0 <= ww < W:
                                s += A[0, hh, ww, o] * W2[kh, kw, o, q]
                Y[0, h, w, q] = s
    got = oracle.conv_chain(X.astype(np.float32), W1.astype(np.float32), W2.astype(np.float32), ACT_RELU)
    assert np.max(np.abs(got - Y)) <= 1e-13 * max(1.0, np.max(np.abs(Y)))


def test_zero_weights_and_activation_sees_complete_tap_sums():
    B, H, W, IC, OC1, OC2 = 1, 4, 4, 5, 6, 3
    X = rnd(14, (B, H, W, IC))
    W1 = rnd(15, (3, 3, IC, OC1), 0.3)
    W2 = rnd(16, (1, 1, OC1, OC2), 0.4)
    assert np.all(oracle.conv_chain(X, np.zeros_like(W1), W2, ACT_GELU_TANH) == 0.0)
    assert np.all(oracle.conv_chain(X, W1, np.zeros_like(W2), ACT_GELU_TANH) == 0.0)
    full = oracle.conv_chain(X, W1, W2, ACT_RELU)
    # negative twin: activating each tap's partial sum separately is a different function
    per_tap = np.zeros_like(full)
    for kh in range(3):
        for kw in range(3):
            one = np.zeros_like(W1)
            one[kh, kw] = W1[kh, kw]
            per_tap += oracle.conv_chain(X, one, W2, ACT_RELU)
    assert np.max(np.abs(per_tap - full)) > 1e-3 * np.max(np.abs(full))
    # ... while with no activation the taps do add up
    lin = oracle.conv_chain(X, W1, W2, ACT_IDENTITY)
    lin_taps = np.zeros_like(lin)
    for kh in range(3):
        for kw in range(3):
            one = np.zeros_like(W1)
            one[kh, kw] = W1[kh, kw]
            lin_taps += oracle.conv_chain(X, one, W2, ACT_IDENTITY)
    assert np.max(np.abs(lin_taps - lin)) <= 1e-12 * np.max(np.abs(lin))


def test_16_bit_operands_and_bad_arguments():
    X = rnd(17, (1, 3, 3, 8)).astype(np.float16)
    W1 = rnd(18, (3, 3, 8, 8), 0.2).astype(np.float16)
    W2 = rnd(19, (1, 1, 8, 8), 0.3).astype(np.float16)
    Y = oracle.conv_chain(X, W1, W2, ACT_RELU)
    Yt, _ = torch_chain(X.astype(np.float32), W1.astype(np.float32), W2.astype(np.float32), ACT_RELU)
    assert np.allclose(Y, Yt, rtol=0, atol=1e-12)
    with pytest.raises(ValueError):
        oracle.conv_chain(X, rnd(20, (2, 2, 8, 8)).astype(np.float16), W2, ACT_RELU)   # even kernel
    with pytest.raises(ValueError):
        oracle.conv_chain(X, W1, rnd(21, (1, 1, 4, 8)).astype(np.float16), ACT_RELU)   # channel mismatch
