"""Pins for the oracle's sparse optimizer step: torch.optim.SGD and torch.optim.Adagrad in float64
on the same rows (the library routine), the row-wise rule by hand and through its relation to the
element-wise rule, and the rounding to 16-bit types against numpy's correctly rounded casts."""
import numpy as np
import pytest
import torch

import oracle
from helpers import bf16_bits_from_f32, f32_from_bf16_bits

SGD, ROWWISE, ADAGRAD = oracle.OPT_SGD, oracle.OPT_ADAGRAD_ROWWISE, oracle.OPT_ADAGRAD


def torch_steps(W0, steps, opt_name, lr, eps):
    """Dense float64 parameter, gradient zero outside the touched rows: rows with zero gradient do not
    move under either rule (Adagrad: 0 / (sqrt(s) + eps) = 0), so this is the sparse step."""
    p = torch.nn.Parameter(torch.tensor(W0, dtype=torch.float64))
    opt = torch.optim.SGD([p], lr=lr) if opt_name == "sgd" else torch.optim.Adagrad([p], lr=lr, eps=eps)
    for rows, g in steps:
        p.grad = torch.zeros_like(p)
        p.grad[torch.as_tensor(rows)] = torch.tensor(g, dtype=torch.float64)
        opt.step()
    return p.detach().numpy()


@pytest.mark.parametrize("opt_name,opt", [("sgd", SGD), ("adagrad", ADAGRAD)])
def test_float32_table_follows_torch_optim(opt_name, opt):
    rng = np.random.default_rng(3)
    R, D = 50, 8
    W0 = rng.standard_normal((R, D)).astype(np.float32)
    W = W0.copy()
    state = np.zeros((R, D), np.float32) if opt == ADAGRAD else None
    lr, eps = 0.1, 1e-6
    steps = []
    for _ in range(3):
        rows = np.sort(rng.choice(R, 17, replace=False))
        g = rng.standard_normal((17, D)).astype(np.float32)
        steps.append((rows, g))
        assert oracle.sparse_update(W, rows, g, opt, lr, eps, state) == (0, 0)
    ref = torch_steps(W0, steps, opt_name, float(np.float32(lr)), float(np.float32(eps)))
    # the table is float32: each step rounds once, so after three steps the two differ by a few units in the last place
    assert np.allclose(W, ref, rtol=4e-7, atol=1e-7)
    untouched = np.setdiff1d(np.arange(R), np.concatenate([r for r, _ in steps]))
    assert np.array_equal(W[untouched], W0[untouched])
    if opt == ADAGRAD:
        s_ref = np.zeros((R, D))
        for rows, g in steps:
            s_ref[rows] += g.astype(np.float64) ** 2
        assert np.allclose(state, s_ref, rtol=3e-7)


def test_rowwise_by_hand_and_against_elementwise():
    # one row, D = 4, two steps by hand: s = mean(g^2), w -= lr g / (sqrt(s) + eps)
    W = np.array([[1.0, 2.0, 3.0, 4.0]], np.float32)
    s = np.zeros(1, np.float32)
    g1 = np.array([[2.0, 0.0, -2.0, 0.0]], np.float32)          # mean square 2
    assert oracle.sparse_update(W, [0], g1, ROWWISE, 0.5, 0.0, s) == (0, 0)
    assert s[0] == 2.0
    assert np.allclose(W[0], [1 - 1 / np.sqrt(2), 2, 3 + 1 / np.sqrt(2), 4], rtol=1e-7)
    g2 = np.array([[1.0, 1.0, 1.0, 1.0]], np.float32)           # mean square 1 -> s = 3
    w_before = W[0].astype(np.float64)
    assert oracle.sparse_update(W, [0], g2, ROWWISE, 0.5, 0.25, s) == (0, 0)
    assert s[0] == 3.0
    assert np.allclose(W[0], w_before - 0.5 / (np.sqrt(3) + 0.25), rtol=1e-7)
    # a gradient that is constant along the row: the mean square is every element's square, so the
    # row-wise rule moves the row exactly as the element-wise rule does
    rng = np.random.default_rng(0)
    Wa = rng.standard_normal((9, 8)).astype(np.float32)
    Wb = Wa.copy()
    g = np.repeat(rng.standard_normal((5, 1)).astype(np.float32), 8, axis=1)
    rows = [7, 1, 3, 8, 0]
    sa, sb = np.zeros(9, np.float32), np.zeros((9, 8), np.float32)
    for _ in range(2):
        oracle.sparse_update(Wa, rows, g, ROWWISE, 0.3, 1e-3, sa)
        oracle.sparse_update(Wb, rows, g, ADAGRAD, 0.3, 1e-3, sb)
    assert np.array_equal(Wa, Wb) and np.array_equal(sb[:, 0], sa)


def test_rounding_to_16_bit_types_is_numpy_s():
    # SGD with lr = 1 and w = 0 writes -g rounded to the table's type: compare with numpy's casts
    rng = np.random.default_rng(1)
    g = np.concatenate([rng.standard_normal(4000) * 10.0 ** rng.integers(-9, 6, 4000),
                        [0.0, -0.0, 65504.0, 65520.0, 65519.9, 1e-8, 6e-8, 2.98e-8, 2.99e-8, 3e38, -3e38,
                         2 ** -14, 2 ** -14 * (1 - 2 ** -11), 1 + 2 ** -11, 1 + 3 * 2 ** -11, 1 + 2 ** -8, 1 + 3 * 2 ** -8]])
    g = np.concatenate([g, np.zeros((-len(g)) % 8)]).astype(np.float32).reshape(-1, 8)
    m = g.shape[0]
    Wh = np.zeros((m, 8), np.float16)
    assert oracle.sparse_update(Wh, np.arange(m), g, SGD, 1.0, 0.0, dtype=oracle.F16) == (0, 0)
    with np.errstate(over="ignore"):
        want = (0.0 - g.astype(np.float64)).astype(np.float16)
    assert np.array_equal(Wh.view(np.uint16), want.view(np.uint16))
    Wb = np.zeros((m, 8), np.uint16)
    assert oracle.sparse_update(Wb, np.arange(m), g, SGD, 1.0, 0.0, dtype=oracle.BF16) == (0, 0)
    finite = np.isfinite(g)
    assert np.array_equal(Wb[finite], bf16_bits_from_f32(np.float32(0.0) - g)[finite])
    # a sum that is not a float32: 1 + 2^-6 + 2^-8 + 2^-31 lies just above a bfloat16 tie and must round
    # up; going through float32 first would land on the tie and round to even (down)
    Wt = bf16_bits_from_f32(np.full((1, 8), 1.0 + 2.0 ** -6, np.float32))
    gt = np.full((1, 8), -(2.0 ** -8 + 2.0 ** -31), np.float32)
    assert f32_from_bf16_bits(Wt)[0, 0] == 1.0 + 2.0 ** -6 and float(gt[0, 0]) == -(2.0 ** -8 + 2.0 ** -31)
    oracle.sparse_update(Wt, [0], gt, SGD, 1.0, 0.0, dtype=oracle.BF16)
    assert f32_from_bf16_bits(Wt)[0, 0] == 1.0 + 2.0 ** -6 + 2.0 ** -7


def test_store_mirror_faults_and_edges():
    W = np.arange(6 * 4, dtype=np.float32).reshape(6, 4)
    W0 = W.copy()
    store = np.full((2, 4), -1, np.float32)
    slots = np.array([-1, 1, -1, -1, 0, -1], np.int32)
    g = np.ones((3, 4), np.float32)
    rc, st = oracle.sparse_update(W, [4, 9, 2], g, SGD, 0.5, 0.0, store=store, slot_of_row=slots)
    assert (rc, st) == (0, oracle.BAD_ID)
    assert np.array_equal(W[4], W0[4] - 0.5) and np.array_equal(W[2], W0[2] - 0.5)
    assert np.array_equal(store[0], W[4]) and np.all(store[1] == -1)       # row 2 has no slot, row 1 was not touched
    assert np.array_equal(W[[0, 1, 3, 5]], W0[[0, 1, 3, 5]])
    assert oracle.sparse_update(W, [], np.zeros((0, 4), np.float32), SGD, 1.0, 0.0) == (0, 0)
    assert oracle.sparse_update(W, [0], g[:1], 7, 1.0, 0.0)[0] == 6
    assert oracle.sparse_update(W, [0], g[:1], ADAGRAD, 1.0, 0.0, None)[0] == 1
    assert oracle.sparse_update(W, [0], g[:1], SGD, 1.0, 0.0, store=store)[0] == 1
    assert oracle.sparse_update(W[:, :3].copy(), [0], g[:1, :3].copy(), SGD, 1.0, 0.0)[0] == 4
