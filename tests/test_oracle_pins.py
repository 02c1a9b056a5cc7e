"""Pins for the CPU oracle (no GPU needed).

The paper prints no convolution formula or worked example, so the oracle is
pinned to mathematics and to independent routines instead: a hand-computed
example, an explicit patch-matrix product, numpy matmul for 1x1 filters, a
delta filter, closed-form border counts, the adjoint identities, backward-data
rebuilt from a forward pass on the zero-dilated gradient, PyTorch's CPU float64
convolution and its autograd derivatives, and scatter-vs-gather agreement of the
oracle's two families of routines.
"""
import itertools
import os

import numpy as np
import pytest

from paper_1512_01274_amd import inputs as gen

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")

SHAPES = [
    # N, C, H, W, K, R, S, stride, pad
    (1, 1, 3, 3, 1, 2, 2, 1, 0),
    (2, 3, 5, 6, 3, 3, 3, 1, 1),
    (1, 2, 6, 5, 2, 3, 2, 2, 1),
    (2, 1, 6, 6, 3, 2, 3, 3, 2),
    (1, 3, 5, 4, 2, 1, 1, 2, 0),
    (2, 2, 4, 6, 2, 3, 3, 2, 0),   # (H+2pad-R) % stride != 0: floor rule
    (1, 2, 7, 7, 2, 5, 5, 1, 2),
    (1, 1, 6, 6, 1, 3, 3, 1, 2),
    (2, 2, 9, 8, 3, 4, 3, 4, 2),
    (1, 2, 3, 3, 2, 1, 1, 1, 1),   # pad larger than R-1
]


def _rand(shape, seed):
    g = np.random.Generator(np.random.Philox(key=seed))
    # small dyadic values: exact in float32, sums exact in float64
    return (g.integers(-8, 9, size=shape).astype(np.float32)) / np.float32(4.0)


def _case(dims, seed=1):
    N, C, H, W, K, R, S, st, pad = dims
    P = (H + 2 * pad - R) // st + 1
    Q = (W + 2 * pad - S) // st + 1
    return (_rand((N, C, H, W), seed), _rand((K, C, R, S), seed + 1), _rand((N, K, P, Q), seed + 2), P, Q)


# ---- P6: hand example (fixture) ------------------------------------------------

def _read_fixture(path):
    out, cur, rows, shape = {}, None, [], None
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        tok = line.split()
        if tok[0].isalpha():
            if cur:
                out[cur] = np.array(rows, dtype=np.float64).reshape(shape)
            cur, shape, rows = tok[0], (int(tok[1]), int(tok[2])), []
        else:
            rows.append([float(t) for t in tok])
    out[cur] = np.array(rows, dtype=np.float64).reshape(shape)
    return out


def test_hand_example(oracle):
    f = _read_fixture(os.path.join(GOLDEN, "hand_example_3x3_2x2.txt"))
    x = f["x"][None, None].astype(np.float32)
    w = f["w"][None, None].astype(np.float32)
    dy = f["dy"][None, None].astype(np.float32)
    np.testing.assert_array_equal(oracle.conv2d_fwd(x, w, 1, 0)[0, 0], f["y"])
    np.testing.assert_array_equal(oracle.conv2d_bwd_weight(x, dy, w.shape, 1, 0)[0, 0], f["dw"])
    np.testing.assert_array_equal(oracle.conv2d_bwd_data(dy, w, x.shape, 1, 0)[0, 0], f["dx"])
    assert (f["y"] * f["dy"]).sum() == (f["x"] * f["dx"]).sum() == (f["w"] * f["dw"]).sum() == -16


# ---- P1: explicit patch matrix x weight matrix ---------------------------------

def _patch_matrix(x, R, S, st, pad):
    """[N*P*Q, C*R*S] matrix of zero-padded patches, built by slicing a padded copy."""
    N, C, H, W = x.shape
    xp = np.zeros((N, C, H + 2 * pad, W + 2 * pad), dtype=np.float64)
    xp[:, :, pad:pad + H, pad:pad + W] = x
    P = (H + 2 * pad - R) // st + 1
    Q = (W + 2 * pad - S) // st + 1
    rows = []
    for n, p, q in itertools.product(range(N), range(P), range(Q)):
        rows.append(xp[n, :, p * st:p * st + R, q * st:q * st + S].reshape(-1))
    return np.array(rows), P, Q


@pytest.mark.parametrize("dims", SHAPES)
def test_fwd_equals_patch_matrix_product(oracle, dims):
    N, C, H, W, K, R, S, st, pad = dims
    x, w, _, P, Q = _case(dims)
    A, P2, Q2 = _patch_matrix(x, R, S, st, pad)
    assert (P, Q) == (P2, Q2) == (oracle.out_dim(H, R, st, pad), oracle.out_dim(W, S, st, pad))
    Y = A @ w.reshape(K, -1).astype(np.float64).T            # [N*P*Q, K]
    ref = Y.reshape(N, P, Q, K).transpose(0, 3, 1, 2)
    np.testing.assert_array_equal(oracle.conv2d_fwd(x, w, st, pad), ref)


@pytest.mark.parametrize("dims", SHAPES)
def test_bwd_from_patch_matrix(oracle, dims):
    """dw = dY^T A (patch matrix), an independent route to backward-weight."""
    N, C, H, W, K, R, S, st, pad = dims
    x, w, dy, P, Q = _case(dims, seed=7)
    A, _, _ = _patch_matrix(x, R, S, st, pad)
    dY = dy.astype(np.float64).transpose(0, 2, 3, 1).reshape(-1, K)
    np.testing.assert_array_equal(oracle.conv2d_bwd_weight(x, dy, w.shape, st, pad),
                                  (dY.T @ A).reshape(K, C, R, S))


# ---- library routine: torch CPU float64 conv + autograd ------------------------

@pytest.mark.parametrize("dims", SHAPES)
def test_against_torch_cpu_float64(oracle, dims):
    torch = pytest.importorskip("torch")
    N, C, H, W, K, R, S, st, pad = dims
    g = np.random.Generator(np.random.Philox(key=99))
    x = g.standard_normal((N, C, H, W)).astype(np.float32)
    w = g.standard_normal((K, C, R, S)).astype(np.float32)
    P = (H + 2 * pad - R) // st + 1
    Q = (W + 2 * pad - S) // st + 1
    dy = g.standard_normal((N, K, P, Q)).astype(np.float32)
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    tw = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    ty = torch.nn.functional.conv2d(tx, tw, stride=st, padding=pad)
    gx, gw = torch.autograd.grad(ty, (tx, tw), torch.tensor(dy, dtype=torch.float64))
    np.testing.assert_allclose(oracle.conv2d_fwd(x, w, st, pad), ty.detach().numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.conv2d_bwd_data(dy, w, x.shape, st, pad), gx.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.conv2d_bwd_weight(x, dy, w.shape, st, pad), gw.numpy(), rtol=0, atol=1e-12)


# ---- P2: 1x1 stride-1 pad-0 convolution is a matmul ----------------------------

def test_1x1_is_matmul(oracle):
    N, C, H, W, K = 2, 5, 4, 3, 7
    x, w = _rand((N, C, H, W), 3), _rand((K, C, 1, 1), 4)
    ref = np.einsum("kc,nchw->nkhw", w[:, :, 0, 0].astype(np.float64), x.astype(np.float64))
    np.testing.assert_array_equal(oracle.conv2d_fwd(x, w, 1, 0), ref)
    Wm = w[:, :, 0, 0].astype(np.float64)
    for n in range(N):
        np.testing.assert_array_equal(oracle.conv2d_fwd(x, w, 1, 0)[n].reshape(K, -1),
                                      np.matmul(Wm, x[n].reshape(C, -1).astype(np.float64)))
    dy = _rand((N, K, H, W), 5)
    np.testing.assert_array_equal(oracle.conv2d_bwd_data(dy, w, x.shape, 1, 0),
                                  np.einsum("kc,nkhw->nchw", Wm, dy.astype(np.float64)))
    np.testing.assert_array_equal(oracle.conv2d_bwd_weight(x, dy, w.shape, 1, 0)[:, :, 0, 0],
                                  np.einsum("nkhw,nchw->kc", dy.astype(np.float64), x.astype(np.float64)))


# ---- P3: delta filter reproduces (a shift of) the input ------------------------

@pytest.mark.parametrize("R,S,r0,s0,st,pad", [(3, 3, 1, 1, 1, 1), (3, 3, 0, 2, 1, 1), (5, 3, 4, 0, 2, 2),
                                              (2, 2, 1, 0, 1, 0), (3, 3, 2, 2, 3, 0)])
def test_delta_filter(oracle, R, S, r0, s0, st, pad):
    N, C, H, W = 2, 3, 7, 6
    x = _rand((N, C, H, W), 11)
    w = np.zeros((C, C, R, S), dtype=np.float32)
    for c in range(C):
        w[c, c, r0, s0] = 1.0
    y = oracle.conv2d_fwd(x, w, st, pad)
    P, Q = y.shape[2:]
    ref = np.zeros_like(y)
    for p in range(P):
        for q in range(Q):
            h, v = p * st - pad + r0, q * st - pad + s0
            if 0 <= h < H and 0 <= v < W:
                ref[:, :, p, q] = x[:, :, h, v]
    np.testing.assert_array_equal(y, ref)
    if st == 1 and r0 == pad and s0 == pad and R == 2 * pad + 1 and S == 2 * pad + 1:
        np.testing.assert_array_equal(y, x.astype(np.float64))


# ---- P5: all-ones closed form with border counts -------------------------------

@pytest.mark.parametrize("dims", SHAPES)
def test_all_ones_closed_form(oracle, dims):
    N, C, H, W, K, R, S, st, pad = dims
    x = np.ones((N, C, H, W), np.float32)
    w = np.ones((K, C, R, S), np.float32)
    y = oracle.conv2d_fwd(x, w, st, pad)
    P, Q = y.shape[2:]
    cnt_h = [sum(1 for r in range(R) if 0 <= p * st - pad + r < H) for p in range(P)]
    cnt_w = [sum(1 for s in range(S) if 0 <= q * st - pad + s < W) for q in range(Q)]
    ref = C * np.outer(cnt_h, cnt_w).astype(np.float64)
    for n in range(N):
        for k in range(K):
            np.testing.assert_array_equal(y[n, k], ref)
    # interior value is C*R*S wherever the whole window is inside the image
    for p in range(P):
        for q in range(Q):
            if p * st - pad >= 0 and p * st - pad + R <= H and q * st - pad >= 0 and q * st - pad + S <= W:
                assert y[0, 0, p, q] == C * R * S
    # with dy == 1 the weight gradient counts the same windows: sum of y over (n,p,q) per (k): equal
    dy = np.ones((N, K, P, Q), np.float32)
    dw = oracle.conv2d_bwd_weight(x, dy, w.shape, st, pad)
    assert dw.sum() == y.sum()


# ---- P4: adjoint identities ----------------------------------------------------

@pytest.mark.parametrize("dims", SHAPES + [(2, 4, 11, 9, 5, 3, 3, 2, 1), (1, 3, 12, 12, 4, 11, 11, 4, 2)])
def test_adjoint_identities(oracle, dims):
    N, C, H, W, K, R, S, st, pad = dims
    g = np.random.Generator(np.random.Philox(key=1234))
    x = g.standard_normal((N, C, H, W)).astype(np.float32)
    w = g.standard_normal((K, C, R, S)).astype(np.float32)
    P = (H + 2 * pad - R) // st + 1
    Q = (W + 2 * pad - S) // st + 1
    dy = g.standard_normal((N, K, P, Q)).astype(np.float32)
    a = (oracle.conv2d_fwd(x, w, st, pad) * dy).sum()
    b = (oracle.conv2d_bwd_data(dy, w, x.shape, st, pad) * x).sum()
    c = (oracle.conv2d_bwd_weight(x, dy, w.shape, st, pad) * w).sum()
    scale = (np.abs(x).sum() * np.abs(w).max() * np.abs(dy).max()) + 1.0
    assert abs(a - b) <= 1e-12 * scale and abs(a - c) <= 1e-12 * scale


# ---- P7: backward-data as a forward pass on the zero-dilated gradient ----------

@pytest.mark.parametrize("dims", [d for d in SHAPES if d[8] <= d[5] - 1 and d[8] <= d[6] - 1 and d[5] == d[6]])
def test_bwd_data_as_forward(oracle, dims):
    N, C, H, W, K, R, S, st, pad = dims
    x, w, dy, P, Q = _case(dims, seed=21)
    # dilate dy by the stride, then extend so that a stride-1 "full" correlation covers all of dx
    Hd, Wd = H + 2 * pad - R + 1, W + 2 * pad - S + 1       # size a stride-1 conv would give
    dil = np.zeros((N, K, Hd, Wd), np.float32)
    dil[:, :, 0:(P - 1) * st + 1:st, 0:(Q - 1) * st + 1:st] = dy
    wt = np.ascontiguousarray(w[:, :, ::-1, ::-1].transpose(1, 0, 2, 3))   # [C,K,R,S], flipped
    ref = oracle.conv2d_fwd(dil, wt, 1, R - 1 - pad)
    assert ref.shape == (N, C, H, W)
    np.testing.assert_array_equal(oracle.conv2d_bwd_data(dy, w, x.shape, st, pad), ref)


# ---- P8: linearity, zeros, untouched gradient positions ------------------------

def test_linearity_and_zero(oracle):
    dims = (2, 3, 6, 5, 4, 3, 3, 2, 1)
    x1, w, dy, P, Q = _case(dims, seed=31)
    x2 = _rand(x1.shape, 32)
    lhs = oracle.conv2d_fwd((2.0 * x1 + x2).astype(np.float32), w, 2, 1)
    np.testing.assert_array_equal(lhs, 2.0 * oracle.conv2d_fwd(x1, w, 2, 1) + oracle.conv2d_fwd(x2, w, 2, 1))
    assert not oracle.conv2d_fwd(np.zeros_like(x1), w, 2, 1).any()
    assert not oracle.conv2d_bwd_data(np.zeros_like(dy), w, x1.shape, 2, 1).any()
    assert not oracle.conv2d_bwd_weight(x1, np.zeros_like(dy), w.shape, 2, 1).any()


def test_untouched_dx_is_exact_zero(oracle):
    # 1x1 stride 2: only even (h,v) receive gradient.  And the floor rule: the last rows/cols of a
    # 3x3 stride-2 pad-0 layer on an 8x8 image are never read, so their gradient is 0.
    dy = np.ones((1, 2, 3, 3), np.float32)
    w = np.ones((2, 2, 1, 1), np.float32)
    dx = oracle.conv2d_bwd_data(dy, w, (1, 2, 6, 6), 2, 0)
    mask = np.zeros((6, 6), bool); mask[::2, ::2] = True
    assert (dx[0, 0][mask] == 2).all() and (dx[0, 0][~mask] == 0).all()
    dy = np.ones((1, 1, 3, 3), np.float32)
    w = np.ones((1, 1, 3, 3), np.float32)
    dx = oracle.conv2d_bwd_data(dy, w, (1, 1, 8, 8), 2, 0)
    assert (dx[0, 0, 7, :] == 0).all() and (dx[0, 0, :, 7] == 0).all() and dx[0, 0, 6, 6] == 1


# ---- scatter (full) vs gather (_at) families, and P9: |value| <= D -------------

@pytest.mark.parametrize("dims", SHAPES)
def test_full_vs_at(oracle, dims):
    N, C, H, W, K, R, S, st, pad = dims
    g = np.random.Generator(np.random.Philox(key=77))
    x = g.standard_normal((N, C, H, W)).astype(np.float32)
    w = g.standard_normal((K, C, R, S)).astype(np.float32)
    P = (H + 2 * pad - R) // st + 1
    Q = (W + 2 * pad - S) // st + 1
    dy = g.standard_normal((N, K, P, Q)).astype(np.float32)
    y = oracle.conv2d_fwd(x, w, st, pad)
    dx = oracle.conv2d_bwd_data(dy, w, x.shape, st, pad)
    dw = oracle.conv2d_bwd_weight(x, dy, w.shape, st, pad)
    v, d = oracle.conv2d_fwd_at(x, w, st, pad, np.arange(y.size))
    np.testing.assert_array_equal(v, y.ravel()); assert (np.abs(v) <= d * (1 + 1e-15)).all()
    np.testing.assert_array_equal(d, oracle.conv2d_fwd(np.abs(x), np.abs(w), st, pad).ravel())
    v, d = oracle.conv2d_bwd_data_at(dy, w, x.shape, st, pad, np.arange(dx.size))
    np.testing.assert_allclose(v, dx.ravel(), rtol=0, atol=1e-13); assert (np.abs(v) <= d * (1 + 1e-15)).all()
    np.testing.assert_allclose(d, oracle.conv2d_bwd_data(np.abs(dy), np.abs(w), x.shape, st, pad).ravel(),
                               rtol=1e-14, atol=0)
    v, d = oracle.conv2d_bwd_weight_at(x, dy, w.shape, st, pad, np.arange(dw.size))
    np.testing.assert_allclose(v, dw.ravel(), rtol=0, atol=1e-13); assert (np.abs(v) <= d * (1 + 1e-15)).all()
    np.testing.assert_allclose(d, oracle.conv2d_bwd_weight(np.abs(x), np.abs(dy), w.shape, st, pad).ravel(),
                               rtol=1e-14, atol=0)


def test_at_accepts_subset_and_order(oracle):
    dims = (2, 3, 5, 6, 3, 3, 3, 1, 1)
    x, w, dy, P, Q = _case(dims)
    y = oracle.conv2d_fwd(x, w, 1, 1).ravel()
    idx = np.array([y.size - 1, 0, 17, 17, 5])
    v, _ = oracle.conv2d_fwd_at(x, w, 1, 1, idx)
    np.testing.assert_array_equal(v, y[idx])


# ---- input generators: determinism and bf16 rounding ---------------------------

def test_generators_are_deterministic_and_bf16_exact():
    cfg = gen.CONFIGS[0]
    L, a = gen.layer_inputs(cfg, 0)
    _, b = gen.layer_inputs(cfg, 0)
    for t in ("x", "w", "dy"):
        np.testing.assert_array_equal(a[t], b[t])
        assert np.abs(a[t]).max() <= 1.0 and a[t].std() > 0.4
    assert a["x"].shape == (2, 16, 16, 16) and a["w"].shape == (32, 16, 3, 3) and a["dy"].shape == (2, 32, 16, 16)
    v = np.array([1.0, 1.00390625, 1.001953125, 1.005859375, -3.1415927, 1e-3], np.float32)
    r = gen.round_to_bf16(v)
    assert (r.view(np.uint32) & 0xFFFF == 0).all()
    # ties go to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7 -> 1 ; 1 + 3*2^-8 -> 1 + 2^-6
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == 1.0 and r[3] == 1.0078125
    assert (np.abs(r - v) <= np.abs(v) * 2.0 ** -8).all()
    np.testing.assert_array_equal(gen.bf16_bits_to_f32(gen.f32_to_bf16_bits(r)), r)


def test_config_shapes_match_benchmark_definition():
    c = {cfg.name: cfg for cfg in gen.CONFIGS}
    assert [len(cfg.layers) for cfg in gen.CONFIGS] == [1, 5, 6, 8, 7]
    a = c["alexnet_b128"].layers
    assert (a[0].P, a[1].P, a[2].P) == (55, 27, 13)
    assert sum(l.flops_per_pass for l in a) == pytest.approx(167.8e9, rel=2e-3)
    assert sum(l.flops_per_pass for l in c["vgg_a_b64"].layers) == pytest.approx(958.1e9, rel=2e-3)
    assert sum(l.flops_per_pass for l in c["inception3a_b128"].layers) == pytest.approx(32.8e9, rel=2e-3)
    assert sum(l.flops_per_pass for l in c["resnet_bottleneck_b256"].layers) == pytest.approx(276.2e9, rel=2e-3)
    assert c["resnet_bottleneck_b256"].layers[3].P == 28


# ---- convolution grouped with bias and ReLU ---------------------------------------------------

FUSED_DIMS = [(2, 3, 7, 6, 4, 3, 3, 1, 1), (1, 5, 9, 9, 6, 3, 3, 2, 1), (2, 8, 5, 5, 8, 1, 1, 1, 0)]


@pytest.mark.parametrize("dims", FUSED_DIMS)
def test_fused_forms_against_torch_cpu_float64(oracle, dims):
    """torch's conv2d with a bias argument, relu, and autograd through relu(conv(...)) are an
    independent implementation of all three grouped forms."""
    torch = pytest.importorskip("torch")
    N, C, H, W, K, R, S, st, pad = dims
    x, w, dy, _, _ = _case(dims, seed=21)
    bias = _rand((K,), 22)
    # the layer below produced x through a ReLU: make it non-negative with exact zeros
    xin = np.maximum(x, 0.0).astype(np.float32)
    tz = torch.tensor(xin, dtype=torch.float64, requires_grad=True)
    tw = torch.tensor(w, dtype=torch.float64)
    tb = torch.tensor(bias, dtype=torch.float64, requires_grad=True)
    lin = torch.nn.functional.conv2d(tz, tw, tb, stride=st, padding=pad)
    a, _ = oracle.conv2d_fwd_bias_act(xin, w, bias, True, st, pad)
    z, _ = oracle.conv2d_fwd_bias_act(xin, w, bias, False, st, pad)
    np.testing.assert_allclose(z, lin.detach().numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(a, torch.relu(lin).detach().numpy(), rtol=1e-12, atol=1e-12)
    # backward: x = relu(pre) with pre = x where positive (any negative value where x == 0)
    pre = torch.tensor(np.where(xin > 0, xin, -1.0), dtype=torch.float64, requires_grad=True)
    out = torch.nn.functional.conv2d(torch.relu(pre), tw, tb, stride=st, padding=pad)
    out.backward(torch.tensor(dy, dtype=torch.float64))
    dz, _ = oracle.conv2d_bwd_data_relu(dy, w, xin, st, pad)
    np.testing.assert_allclose(dz, pre.grad.numpy(), rtol=1e-12, atol=1e-12)
    db, _ = oracle.bias_grad(dy)
    np.testing.assert_allclose(db, tb.grad.numpy(), rtol=1e-12, atol=1e-12)


def test_fused_forward_closed_forms(oracle):
    """Zero filter: the output is act(bias) everywhere.  Delta filter, zero bias: act(x)."""
    x = _rand((2, 3, 6, 6), 31)
    bias = np.array([-1.5, 0.0, 2.25, 0.5], dtype=np.float32)
    a, den = oracle.conv2d_fwd_bias_act(x, np.zeros((4, 3, 3, 3), np.float32), bias, True, 1, 1)
    assert np.array_equal(a, np.broadcast_to(np.maximum(bias, 0)[None, :, None, None].astype(np.float64), a.shape))
    assert np.array_equal(den, np.broadcast_to(np.abs(bias)[None, :, None, None].astype(np.float64), den.shape))
    w = np.zeros((3, 3, 1, 1), np.float32)
    for c in range(3):
        w[c, c, 0, 0] = 1.0
    a, _ = oracle.conv2d_fwd_bias_act(x, w, np.zeros(3, np.float32), True, 1, 0)
    assert np.array_equal(a, np.maximum(x, 0).astype(np.float64))
    z, _ = oracle.conv2d_fwd_bias_act(x, w, np.zeros(3, np.float32), False, 1, 0)
    assert np.array_equal(z, x.astype(np.float64))


def test_relu_mask_special_cases(oracle):
    """All-positive x: the masked gradient is the plain one.  All-zero x: it is zero.  A single
    positive element keeps exactly that element."""
    dims = (1, 4, 6, 6, 5, 3, 3, 1, 1)
    x, w, dy, _, _ = _case(dims, seed=41)
    plain = oracle.conv2d_bwd_data(dy, w, x.shape, 1, 1)
    g, den = oracle.conv2d_bwd_data_relu(dy, w, np.abs(x) + 1.0, 1, 1)
    assert np.array_equal(g, plain)
    g, den = oracle.conv2d_bwd_data_relu(dy, w, np.zeros_like(x), 1, 1)
    assert not g.any() and not den.any()
    one = np.zeros_like(x)
    one[0, 2, 3, 4] = 0.5
    g, _ = oracle.conv2d_bwd_data_relu(dy, w, one, 1, 1)
    assert g[0, 2, 3, 4] == plain[0, 2, 3, 4] and np.count_nonzero(g) <= 1
    neg = -np.abs(x)
    g, _ = oracle.conv2d_bwd_data_relu(dy, w, neg, 1, 1)
    assert not g.any()


def test_bias_grad_is_bwd_weight_of_a_ones_image(oracle):
    """db equals the weight gradient of a 1x1 filter on an all-ones single-channel input: the
    bias is such a filter's weight."""
    dy = _rand((3, 5, 4, 6), 51)
    db, den = oracle.bias_grad(dy)
    ones = np.ones((3, 1, 4, 6), np.float32)
    dw = oracle.conv2d_bwd_weight(ones, dy, (5, 1, 1, 1), 1, 0)
    np.testing.assert_allclose(db, dw[:, 0, 0, 0], rtol=1e-13)
    assert np.all(den >= np.abs(db))
    # closed form: constant gradient
    db, _ = oracle.bias_grad(np.full((2, 3, 4, 5), 0.25, np.float32))
    assert np.array_equal(db, np.full(3, 0.25 * 2 * 4 * 5))


# ---- weight update ------------------------------------------------------------------------------

def test_sgd_update_closed_forms(oracle):
    """mu = lambda = 0: the paper's w - eta*g.  Constant gradient with momentum: the velocity is a
    geometric series.  Weight decay alone: geometric shrinkage."""
    w0 = _rand((3, 4), 61).astype(np.float64)
    g = _rand((3, 4), 62).astype(np.float64)
    w1, v1 = oracle.sgd_update(w0, g, None, 0.125, 0.0, 0.0)
    assert np.array_equal(w1, w0 - 0.125 * g) and np.array_equal(v1, -0.125 * g)
    w, v = w0, None
    mu, lr, T = 0.5, 0.25, 12
    for _ in range(T):
        w, v = oracle.sgd_update(w, g, v, lr, mu, 0.0)
    np.testing.assert_allclose(v, -lr * g * (1 - mu ** T) / (1 - mu), rtol=1e-13)
    # sum of the velocities: -lr*g/(1-mu) * (T - mu*(1-mu^T)/(1-mu))
    np.testing.assert_allclose(w - w0, -lr * g / (1 - mu) * (T - mu * (1 - mu ** T) / (1 - mu)), rtol=1e-12)
    w = w0
    for _ in range(7):
        w, _ = oracle.sgd_update(w, np.zeros_like(w0), None, 0.5, 0.0, 0.25)
    np.testing.assert_allclose(w, w0 * (1 - 0.5 * 0.25) ** 7, rtol=1e-13)


# ---- FullyConnected --------------------------------------------------------------------------------

def test_fc_is_a_1x1_convolution_on_a_1x1_image(oracle):
    """The matrix-product forms against the seven-loop convolution nests on H = W = R = S = 1, which
    share nothing with numpy's matmul; plus torch's linear layer and its autograd."""
    torch = pytest.importorskip("torch")
    N, C, K = 5, 7, 4
    x, w, dy = _rand((N, C), 71), _rand((K, C), 72), _rand((N, K), 73)
    bias = _rand((K,), 74)
    y, den = oracle.fc_fwd(x, w)
    assert np.array_equal(y, oracle.conv2d_fwd(x.reshape(N, C, 1, 1), w.reshape(K, C, 1, 1), 1, 0).reshape(N, K))
    assert np.array_equal(den, oracle.conv2d_fwd(np.abs(x).reshape(N, C, 1, 1), np.abs(w).reshape(K, C, 1, 1), 1, 0).reshape(N, K))
    dx, _ = oracle.fc_bwd_data(dy, w)
    assert np.array_equal(dx, oracle.conv2d_bwd_data(dy.reshape(N, K, 1, 1), w.reshape(K, C, 1, 1), (N, C, 1, 1), 1, 0).reshape(N, C))
    dw, _ = oracle.fc_bwd_weight(x, dy)
    assert np.array_equal(dw, oracle.conv2d_bwd_weight(x.reshape(N, C, 1, 1), dy.reshape(N, K, 1, 1), (K, C, 1, 1), 1, 0).reshape(K, C))
    tx = torch.tensor(np.maximum(x, 0), dtype=torch.float64)
    pre = torch.tensor(np.where(x > 0, x, -1.0), dtype=torch.float64, requires_grad=True)
    tw = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    tb = torch.tensor(bias, dtype=torch.float64)
    out = torch.relu(torch.nn.functional.linear(torch.relu(pre), tw, tb))
    a, _ = oracle.fc_fwd(np.maximum(x, 0), w, bias, True)
    np.testing.assert_allclose(a, out.detach().numpy(), rtol=1e-13, atol=1e-13)
    lin = torch.nn.functional.linear(torch.relu(pre), tw, tb)
    lin.backward(torch.tensor(dy, dtype=torch.float64))
    g, _ = oracle.fc_bwd_data(dy, w, np.maximum(x, 0))
    np.testing.assert_allclose(g, pre.grad.numpy(), rtol=1e-13, atol=1e-13)
    gw, _ = oracle.fc_bwd_weight(np.maximum(x, 0), dy)
    np.testing.assert_allclose(gw, tw.grad.numpy(), rtol=1e-13, atol=1e-13)
    assert tx.shape == (N, C)


# ---- Softmax output layer ----------------------------------------------------------------------------

def test_softmax_closed_forms_and_torch(oracle):
    torch = pytest.importorskip("torch")
    z = _rand((6, 9), 81).astype(np.float64) * 3
    p = oracle.softmax_fwd(z)
    np.testing.assert_allclose(p.sum(axis=1), 1.0, rtol=1e-15)
    np.testing.assert_allclose(oracle.softmax_fwd(z + 1000.0), p, rtol=1e-12)              # shift invariance, no overflow
    np.testing.assert_allclose(oracle.softmax_fwd(np.zeros((2, 8))), 1.0 / 8)              # uniform
    two = oracle.softmax_fwd(np.array([[0.75, -0.5]]))
    np.testing.assert_allclose(two[0, 0], 1.0 / (1.0 + np.exp(-1.25)), rtol=1e-15)         # two classes: the logistic function
    np.testing.assert_allclose(p, torch.softmax(torch.tensor(z), dim=1).numpy(), rtol=1e-13)
    labels = np.array([0, 8, 3, 3, 5, 1])
    tz = torch.tensor(z, requires_grad=True)
    torch.nn.functional.cross_entropy(tz, torch.tensor(labels), reduction="sum").backward()
    np.testing.assert_allclose(oracle.softmax_xent_bwd(p, labels), tz.grad.numpy(), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(oracle.softmax_xent_bwd(p, labels, 0.25).sum(axis=1), 0.0, atol=1e-15)   # rows of the gradient sum to 0


def test_transform_domain_identity_and_budget(oracle):
    """The matrices the transform-domain forward (and the tests' error budget for it) are built on reproduce the
    plain definition exactly: At[(G g Gt) .* (Bt d B)]A summed over channels equals the oracle's forward, and the
    budget (the same expression on absolute values) bounds it."""
    from tests import util
    rng = np.random.Generator(np.random.Philox(key=99))
    x = rng.standard_normal((2, 3, 7, 8)).astype(np.float32)
    w = rng.standard_normal((4, 3, 3, 3)).astype(np.float32)
    G = np.array([[1, 0, 0], [.5, .5, .5], [.5, -.5, .5], [0, 0, 1]])
    Bt = np.array([[1, 0, -1, 0], [0, 1, 1, 0], [0, -1, 1, 0], [0, 1, 0, -1]], dtype=np.float64)
    At = np.array([[1, 1, 1, 0], [0, 1, -1, -1]], dtype=np.float64)
    for pad in (0, 1, 2):
        ref = oracle.conv2d_fwd(x, w, 1, pad)
        P, Q = ref.shape[2], ref.shape[3]
        TP, TQ = (P + 1) // 2, (Q + 1) // 2
        xp = np.zeros((2, 3, 2 * TP + 2, 2 * TQ + 2))
        xp[:, :, pad:pad + 7, pad:pad + 8] = x
        U = np.einsum("ir,kcrs,js->kcij", G, w.astype(np.float64), G)
        out = np.zeros((2, 4, 2 * TP, 2 * TQ))
        for tp in range(TP):
            for tq in range(TQ):
                V = np.einsum("ia,ncab,jb->ncij", Bt, xp[:, :, 2 * tp:2 * tp + 4, 2 * tq:2 * tq + 4], Bt)
                out[:, :, 2 * tp:2 * tp + 2, 2 * tq:2 * tq + 2] = np.einsum("ai,nkij,bj->nkab", At, np.einsum("kcij,ncij->nkij", U, V), At)
        assert np.max(np.abs(out[:, :, :P, :Q] - ref)) < 1e-12
        budget = util.transform_domain_budget(x, w, pad)
        assert budget.shape == ref.shape and np.all(budget + 1e-12 >= np.abs(ref))
