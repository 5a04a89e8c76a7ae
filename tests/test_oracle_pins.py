"""Pins for the fp64 CPU oracle (CPU only).

The paper prints no worked numeric example for the chain, so the oracle is pinned to what
mathematics and independent library routines fix:
  * format widening against torch / numpy conversions over ALL 65536 16-bit patterns,
  * activations against torch's CPU library kernels and known constants,
  * closed forms (identity first layer, zero weights, rank-1 ReLU case),
  * the odd-part identity act(x) - act(-x) = x, which collapses the whole chain to plain
    float64 matrix products (numpy ``@``),
  * a pure-Python brute-force twin with a different loop nest on tiny shapes,
  * invariants: row independence, linearity in W2, ReLU homogeneity, the hidden-split
    identity (paper Sec. 4.1 "reduce" strategy) and its negative twin -- splitting K before
    the activation must NOT reproduce the result (Sec. 4.3 Rule 3) -- and the equivalence of
    the two gated-FFN realisations (Sec. 4.1, last paragraphs).
Non-square shapes are used throughout so a transposed operand or swapped index fails.
"""
import math

import numpy as np
import pytest
import torch

import oracle
from oracle import ACT_GELU_TANH, ACT_IDENTITY, ACT_RELU, ACT_SILU
from paper_2512_12949_amd import inputs

ACTS = [ACT_RELU, ACT_GELU_TANH, ACT_SILU]


def rnd(seed, shape, scale=1.0):
    return np.random.default_rng(seed).standard_normal(shape).astype(np.float32) * np.float32(scale)


def relerr(a, b):
    d = np.max(np.abs(a - b))
    s = max(np.max(np.abs(b)), 1e-300)
    return d / s


# ---------------------------------------------------------------- number formats

def test_widen_bf16_all_patterns_match_torch():
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle.widen(bits, bf16=True)
    ref = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(got, ref, equal_nan=True)


def test_widen_f16_all_patterns_match_numpy():
    h = np.arange(65536, dtype=np.uint16).view(np.float16)
    got = oracle.widen(h)
    assert np.array_equal(got, h.astype(np.float64), equal_nan=True)


def test_widen_f32_exact():
    f = rnd(3, (1000,), 37.0)
    assert np.array_equal(oracle.widen(f), f.astype(np.float64))


# ---------------------------------------------------------------- activations

def test_activation_known_values():
    assert oracle.act(ACT_RELU, -2.5) == 0.0 and oracle.act(ACT_RELU, 2.5) == 2.5
    for a in (ACT_IDENTITY, ACT_RELU, ACT_GELU_TANH, ACT_SILU):
        assert oracle.act(a, 0.0) == 0.0
    assert oracle.act(ACT_SILU, 1.0) == pytest.approx(1.0 / (1.0 + math.exp(-1.0)), rel=1e-15)
    assert oracle.act(ACT_SILU, 1.0) == pytest.approx(0.7310585786300049, rel=1e-14)
    assert oracle.act(ACT_GELU_TANH, 1.0) == pytest.approx(0.8411919906082768, rel=1e-13)
    assert oracle.act(ACT_GELU_TANH, -1.0) == pytest.approx(-0.15880800939172324, rel=1e-12)
    assert oracle.act(ACT_GELU_TANH, 10.0) == pytest.approx(10.0, rel=1e-12)
    assert abs(oracle.act(ACT_GELU_TANH, -10.0)) < 1e-12
    assert oracle.act(ACT_SILU, -40.0) == pytest.approx(-40.0 * math.exp(-40.0), rel=1e-12)


def test_activations_match_torch_library():
    xs = np.linspace(-9.0, 9.0, 2001)
    t = torch.from_numpy(xs)
    refs = {
        ACT_RELU: torch.relu(t),
        ACT_GELU_TANH: torch.nn.functional.gelu(t, approximate="tanh"),
        ACT_SILU: torch.nn.functional.silu(t),
        ACT_IDENTITY: t,
    }
    for a, r in refs.items():
        got = np.array([oracle.act(a, float(x)) for x in xs])
        assert np.max(np.abs(got - r.numpy())) < 1e-14, a


@pytest.mark.parametrize("a", ACTS)
def test_odd_part_of_activation_is_identity(a):
    for x in np.linspace(-6, 6, 241):
        assert oracle.act(a, x) - oracle.act(a, -x) == pytest.approx(x, abs=1e-14)


# ---------------------------------------------------------------- closed forms

def test_identity_first_layer_reduces_to_one_product():
    M, K, N2 = 7, 12, 5
    X, W2 = rnd(1, (M, K)), rnd(2, (K, N2))
    Y = oracle.ffn(X, np.eye(K, dtype=np.float32), None, W2, ACT_IDENTITY)
    assert relerr(Y, X.astype(np.float64) @ W2.astype(np.float64)) < 1e-14


@pytest.mark.parametrize("a", ACTS)
@pytest.mark.parametrize("which", ["W1", "W2", "W3"])
def test_zero_weights_give_exact_zero(a, which):
    M, K, N1, N2 = 5, 6, 9, 4
    X, W1, W3, W2 = rnd(1, (M, K)), rnd(2, (K, N1)), rnd(3, (K, N1)), rnd(4, (N1, N2))
    if which == "W1":
        W1 = np.zeros_like(W1)
    elif which == "W2":
        W2 = np.zeros_like(W2)
    else:
        W3 = np.zeros_like(W3)
    gated = which == "W3"
    Y = oracle.ffn(X, W1, W3 if gated else None, W2, a)
    assert np.all(Y == 0.0)
    if which != "W3":  # gated chain with a zero gate or a zero W2 is zero too
        assert np.all(oracle.ffn(X, W1, W3, W2, a) == 0.0)


def test_rank_one_relu_closed_form():
    rng = np.random.default_rng(5)
    M, K, N1, N2 = 6, 10, 8, 3
    u = np.abs(rng.standard_normal(M)).astype(np.float32)
    v = rng.standard_normal(K).astype(np.float32)
    a = v * np.float32(0.5) + np.float32(0.1) * np.sign(v).astype(np.float32)  # v.a > 0
    b = rng.standard_normal(N1).astype(np.float32)
    c = rng.standard_normal(N1).astype(np.float32)
    d = rng.standard_normal(N2).astype(np.float32)
    X, W1, W2 = np.outer(u, v), np.outer(a, b), np.outer(c, d)
    assert float(v.astype(np.float64) @ a.astype(np.float64)) > 0
    Y = oracle.ffn(X.astype(np.float32), W1.astype(np.float32), None, W2.astype(np.float32), ACT_RELU)
    # build the closed form from the ROUNDED fp32 matrices' factors is not possible once the
    # outer products are rounded, so compare with a tolerance of a few fp32 ulps
    va = float(v.astype(np.float64) @ a.astype(np.float64))
    rbc = float(np.maximum(b.astype(np.float64), 0.0) @ c.astype(np.float64))
    ref = va * rbc * np.outer(u.astype(np.float64), d.astype(np.float64))
    assert relerr(Y, ref) < 5e-6


# ---------------------------------------------------------------- odd-part identity

@pytest.mark.parametrize("a", ACTS)
def test_standard_chain_odd_part_is_plain_matmul(a):
    M, K, N1, N2 = 9, 20, 33, 7
    X, W1, W2 = rnd(11, (M, K)), rnd(12, (K, N1), K ** -0.5), rnd(13, (N1, N2), N1 ** -0.5)
    d = oracle.ffn(X, W1, None, W2, a) - oracle.ffn(-X, W1, None, W2, a)
    ref = (X.astype(np.float64) @ W1.astype(np.float64)) @ W2.astype(np.float64)
    assert relerr(d, ref) < 1e-13


@pytest.mark.parametrize("a", ACTS)
def test_gated_chain_even_part_is_plain_matmul(a):
    M, K, N1, N2 = 8, 18, 29, 6
    X, W1, W3, W2 = (rnd(21, (M, K)), rnd(22, (K, N1), K ** -0.5), rnd(23, (K, N1), K ** -0.5),
                     rnd(24, (N1, N2), N1 ** -0.5))
    s = oracle.ffn(X, W1, W3, W2, a) + oracle.ffn(-X, W1, W3, W2, a)
    Xd, W1d, W3d, W2d = (t.astype(np.float64) for t in (X, W1, W3, W2))
    ref = ((Xd @ W1d) * (Xd @ W3d)) @ W2d
    assert relerr(s, ref) < 1e-13


# ---------------------------------------------------------------- brute force twin

def _py_act(a, x):
    if a == ACT_RELU:
        return max(x, 0.0)
    if a == ACT_GELU_TANH:
        return float(torch.nn.functional.gelu(torch.tensor(x, dtype=torch.float64), approximate="tanh"))
    if a == ACT_SILU:
        return float(torch.nn.functional.silu(torch.tensor(x, dtype=torch.float64)))
    return x


def _brute(X, W1, W3, W2, a):
    """j outermost, then i, then n, then k: a different nest from the oracle's, exact sums."""
    M, K = X.shape
    N1, N2 = W2.shape
    Y = np.zeros((M, N2))
    for j in range(N2):
        for i in range(M):
            terms = []
            for n in range(N1):
                g = math.fsum(float(X[i, k]) * float(W1[k, n]) for k in range(K))
                h = _py_act(a, g)
                if W3 is not None:
                    h *= math.fsum(float(X[i, k]) * float(W3[k, n]) for k in range(K))
                terms.append(h * float(W2[n, j]))
            Y[i, j] = math.fsum(terms)
    return Y


@pytest.mark.parametrize("shape", [(1, 1, 1, 1), (1, 5, 1, 3), (3, 4, 5, 2), (8, 8, 8, 8), (2, 7, 3, 6)])
@pytest.mark.parametrize("a", [ACT_IDENTITY] + ACTS)
@pytest.mark.parametrize("gated", [False, True])
def test_brute_force_tiny(shape, a, gated):
    M, K, N1, N2 = shape
    X, W1, W3, W2 = rnd(31, (M, K)), rnd(32, (K, N1)), rnd(33, (K, N1)), rnd(34, (N1, N2))
    Y = oracle.ffn(X, W1, W3 if gated else None, W2, a)
    ref = _brute(X, W1, W3 if gated else None, W2, a)
    assert np.max(np.abs(Y - ref)) <= 1e-13 * max(1.0, np.max(np.abs(ref)))


# ---------------------------------------------------------------- library cross-check

def _np_chain(X, W1, W3, W2, a):
    Xd, W1d, W2d = (np.asarray(t, dtype=np.float64) for t in (X, W1, W2))
    g = torch.from_numpy(Xd @ W1d)
    h = {ACT_RELU: torch.relu, ACT_SILU: torch.nn.functional.silu, ACT_IDENTITY: lambda t: t,
         ACT_GELU_TANH: lambda t: torch.nn.functional.gelu(t, approximate="tanh")}[a](g).numpy()
    if W3 is not None:
        h = h * (Xd @ np.asarray(W3, dtype=np.float64))
    return h @ W2d


@pytest.mark.parametrize("a", ACTS)
@pytest.mark.parametrize("gated", [False, True])
def test_medium_shape_against_float64_library(a, gated):
    M, K, N1, N2 = 96, 200, 328, 136
    X, W1, W3, W2 = (rnd(41, (M, K)), rnd(42, (K, N1), K ** -0.5), rnd(43, (K, N1), K ** -0.5),
                     rnd(44, (N1, N2), N1 ** -0.5))
    Y = oracle.ffn(X, W1, W3 if gated else None, W2, a)
    assert relerr(Y, _np_chain(X, W1, W3 if gated else None, W2, a)) < 1e-12


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_sixteen_bit_operands_against_float64_library(dtype):
    w = inputs.custom("t", 40, 64, 96, 48, dtype=dtype, act=ACT_SILU, gated=True)
    t = inputs.make(w)
    if dtype == "bf16":
        wide = {k: inputs.bf16_bits_to_f32(v).astype(np.float64) for k, v in t.items()}
    else:
        wide = {k: v.astype(np.float64) for k, v in t.items()}
    Y = oracle.ffn(t["X"], t["W1"], t["W3"], t["W2"], ACT_SILU, bf16=(dtype == "bf16"))
    assert relerr(Y, _np_chain(wide["X"], wide["W1"], wide["W3"], wide["W2"], ACT_SILU)) < 1e-12


# ---------------------------------------------------------------- invariants

def test_row_independence_and_row_subsets():
    M, K, N1, N2 = 11, 16, 24, 5
    X, W1, W2 = rnd(51, (M, K)), rnd(52, (K, N1)), rnd(53, (N1, N2))
    Y = oracle.ffn(X, W1, None, W2, ACT_GELU_TANH)
    perm = np.random.default_rng(0).permutation(M)
    assert np.array_equal(oracle.ffn(X[perm], W1, None, W2, ACT_GELU_TANH), Y[perm])
    rows = [10, 0, 3, 3]
    Ys, Hs = oracle.ffn_rows(X, W1, None, W2, ACT_GELU_TANH, rows=rows, want_h=True)
    assert np.array_equal(Ys, Y[rows])
    g = X.astype(np.float64) @ W1.astype(np.float64)
    ref_h = torch.nn.functional.gelu(torch.from_numpy(g), approximate="tanh").numpy()[rows]
    assert relerr(Hs, ref_h) < 1e-13


def test_linearity_in_second_weight_and_relu_homogeneity():
    M, K, N1, N2 = 6, 10, 14, 9
    X, W1, W2a, W2b = rnd(61, (M, K)), rnd(62, (K, N1)), rnd(63, (N1, N2)), rnd(64, (N1, N2))
    Ya = oracle.ffn(X, W1, None, W2a, ACT_SILU)
    Yb = oracle.ffn(X, W1, None, W2b, ACT_SILU)
    # W2a + 2*W2b is formed in fp64 and fed as fp32 only if exactly representable: use powers of two
    W2c = (W2a.astype(np.float64) * 0.5).astype(np.float32)
    assert relerr(oracle.ffn(X, W1, None, W2c, ACT_SILU), 0.5 * Ya) < 1e-15
    assert relerr(Ya + Yb, Yb + Ya) == 0
    Y4 = oracle.ffn((X * np.float32(4.0)), W1, None, W2a, ACT_RELU)
    assert relerr(Y4, 4.0 * oracle.ffn(X, W1, None, W2a, ACT_RELU)) < 1e-15


@pytest.mark.parametrize("a", ACTS)
@pytest.mark.parametrize("gated", [False, True])
def test_hidden_split_identity(a, gated):
    """Sum over hidden slices of act(X W1[:,s]) W2[s,:] equals the whole chain."""
    M, K, N1, N2 = 7, 12, 30, 8
    X, W1, W3, W2 = rnd(71, (M, K)), rnd(72, (K, N1)), rnd(73, (K, N1)), rnd(74, (N1, N2))
    Y = oracle.ffn(X, W1, W3 if gated else None, W2, a)
    acc = np.zeros_like(Y)
    for lo, hi in [(0, 7), (7, 8), (8, 30)]:
        acc += oracle.ffn(X, W1[:, lo:hi], W3[:, lo:hi] if gated else None, W2[lo:hi], a)
    assert relerr(acc, Y) < 1e-13


@pytest.mark.parametrize("a", ACTS)
def test_splitting_k_before_activation_is_wrong(a):
    """Negative twin: activating partial K-sums must give a different answer."""
    M, K, N1, N2 = 7, 12, 30, 8
    X, W1, W2 = rnd(81, (M, K)), rnd(82, (K, N1)), rnd(83, (N1, N2))
    Y = oracle.ffn(X, W1, None, W2, a)
    bad = oracle.ffn(X[:, :5], W1[:5], None, W2, a) + oracle.ffn(X[:, 5:], W1[5:], None, W2, a)
    assert relerr(bad, Y) > 1e-3
    ok = oracle.ffn(X[:, :5], W1[:5], None, W2, ACT_IDENTITY) + oracle.ffn(X[:, 5:], W1[5:], None, W2, ACT_IDENTITY)
    assert relerr(ok, oracle.ffn(X, W1, None, W2, ACT_IDENTITY)) < 1e-13


def test_two_gated_realisations_agree():
    """Branches computed apart and joined by a multiply == both branches in one pass."""
    M, K, N1, N2 = 6, 9, 13, 5
    X, W1, W3, W2 = rnd(91, (M, K)), rnd(92, (K, N1)), rnd(93, (K, N1)), rnd(94, (N1, N2))
    Y = oracle.ffn(X, W1, W3, W2, ACT_SILU)
    _, gate = oracle.ffn_rows(X, W1, None, W2, ACT_SILU, want_h=True)
    _, up = oracle.ffn_rows(X, W3, None, W2, ACT_IDENTITY, want_h=True)
    joined = (gate * up) @ W2.astype(np.float64)
    assert relerr(joined, Y) < 1e-13
    # the activated branch is W1, not W3
    assert relerr(oracle.ffn(X, W3, W1, W2, ACT_SILU), Y) > 1e-3


def test_argument_errors():
    X, W1, W2 = rnd(1, (4, 6)), rnd(2, (6, 8)), rnd(3, (8, 3))
    with pytest.raises(ValueError):
        oracle.ffn(X, W1.T.copy(), None, W2, ACT_RELU)
    with pytest.raises(ValueError):
        oracle.ffn_rows(X, W1, None, W2, ACT_RELU, rows=[4])
    with pytest.raises(TypeError):
        oracle.ffn(X.astype(np.float64), W1, None, W2, ACT_RELU)
    assert oracle.ffn_rows(X, W1, None, W2, ACT_RELU, rows=[]).shape == (0, 3)
