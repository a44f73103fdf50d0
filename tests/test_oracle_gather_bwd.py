"""Pins for the oracle's sequence gather and its backward.

Gather (Section 2, "Embedding Pooling": every looked-up row is materialised)
reduces to numpy.take.  The backward sums the gradients of a row's duplicates
(Section 3.2, metrics 4-6); its pins are fp64 numpy.add.at (exact for
half-precision inputs), numpy.unique, exact special cases, and hand-computed
fp32 rounding cases that tell the stated summation order from any other.
"""
import numpy as np
import pytest
import torch

import oracle
from helpers import bf16_bits_from_f32, f32_from_bf16_bits

TWO24 = float(2 ** 24)


# ----------------------------------------------------------------- gather
@pytest.mark.parametrize("dt", ["f32", "f16", "bf16"])
def test_gather_is_take(dt):
    rng = np.random.default_rng(3)
    R, D, n = 200, {"f32": 12, "f16": 24, "bf16": 8}[dt], 333
    if dt == "f32":
        W, code = rng.standard_normal((R, D)).astype(np.float32), oracle.F32
    elif dt == "f16":
        W, code = rng.standard_normal((R, D)).astype(np.float16), oracle.F16
    else:
        W, code = bf16_bits_from_f32(rng.standard_normal((R, D))), oracle.BF16
    g = rng.integers(0, R, n)
    perm = rng.permutation(n).astype(np.int32)          # any bucketised order
    rows = g[perm]
    out = np.zeros((n, D), W.dtype)
    rc, st = oracle.seq_gather_fwd(W, rows, perm, 0, n, out, dtype=code)
    assert rc == 0 and st == 0
    assert np.array_equal(out.view(np.uint8), np.take(W, g, axis=0).view(np.uint8))
    # a partial range leaves the other rows untouched
    sentinel = np.full((n, D), 7, W.dtype)
    rc, st = oracle.seq_gather_fwd(W, rows, perm, 100, 180, sentinel, dtype=code)
    touched = np.zeros(n, bool)
    touched[perm[100:180]] = True
    assert np.array_equal(sentinel[touched], np.take(W, g, axis=0)[touched])
    assert np.all(sentinel[~touched] == 7)


def test_gather_faults():
    W = np.arange(8 * 4, dtype=np.float32).reshape(8, 4)
    out = np.full((3, 4), -1, np.float32)
    rc, st = oracle.seq_gather_fwd(W, [1, 9, 2, -1, 3], np.array([0, 1, 5, 2, 2], np.int32), 0, 5, out)
    assert rc == 0 and st == oracle.BAD_ID
    assert np.array_equal(out[0], W[1]) and np.all(out[1] == -1) and np.array_equal(out[2], W[3])
    assert oracle.seq_gather_fwd(W[:, :3].copy(), [0], np.array([0], np.int32), 0, 1, out[:, :3].copy())[0] == 4
    assert oracle.seq_gather_fwd(W, [0], np.array([0], np.int32), 1, 0, out)[0] == 2
    assert oracle.seq_gather_fwd(W, [0], np.array([0], np.int32), 0, 0, out) == (0, 0)


# --------------------------------------------------------------- backward
def _bwd(grad, rows, pos=None, tile=oracle.BWD_TILE, R=None, **kw):
    rows = np.asarray(rows, np.int64)
    pos = np.arange(len(rows), dtype=np.int32) if pos is None else np.asarray(pos, np.int32)
    R = int(rows.max()) + 1 if R is None else R
    return oracle.seq_grad_bwd(grad, rows, pos, 0, len(rows), R, tile=tile, **kw)


def col(values):
    """[m] values -> [m, 4] fp32 grad_out whose columns are v, -v, 0, 2v."""
    v = np.asarray(values, np.float32)[:, None]
    return np.concatenate([v, -v, 0 * v, 2 * v], 1).astype(np.float32)


def test_rounding_cases_fix_the_order():
    # one run starting at k = 0, tile 4: partials (2^24+1+1+1) = 2^24 and (1+1) = 2
    rc, st, u, g, g64, nu = _bwd(col([TWO24, 1, 1, 1, 1, 1]), [5] * 6, tile=4)
    assert nu == 1 and u.tolist() == [5]
    assert g[0].tolist() == [TWO24 + 2, -(TWO24 + 2), 0.0, 2 * (TWO24 + 2)]
    assert g64[0, 0] == TWO24 + 5
    # plain left-to-right (one partial) would give 2^24: tile 8 shows it
    assert _bwd(col([TWO24, 1, 1, 1, 1, 1]), [5] * 6, tile=8)[3][0, 0] == TWO24
    # a run starting at k = 3 behind another row: partials [2^24] and (1+1+1): 2^24 + 3 -> ties to even 2^24 + 4
    rc, st, u, g, g64, nu = _bwd(col([9, 9, 9, TWO24, 1, 1, 1]), [2, 2, 2, 7, 7, 7, 7], tile=4)
    assert u.tolist() == [2, 7] and g[0, 0] == 27.0 and g[1, 0] == TWO24 + 4
    # partials are folded left to right: tile 1, (2^24 + 1) + 1 = 2^24 (right to left would be 2^24 + 2)
    assert _bwd(col([TWO24, 1, 1]), [0, 0, 0], tile=1)[3][0, 0] == TWO24
    assert _bwd(col([1, 1, TWO24]), [0, 0, 0], tile=1)[3][0, 0] == TWO24 + 2
    # the order inside a run is ascending pos, whatever the order in j
    rc, st, u, g, _, _ = _bwd(col([1, 1, TWO24, 3]), [4, 4, 4, 1], pos=[2, 1, 0, 3], tile=8)
    #   pos 0 holds 1, pos 1 holds 1, pos 2 holds 2^24: j order is pos 2,1,0 -> sorted by pos: 1, 1, 2^24
    assert u.tolist() == [1, 4] and g[0, 0] == 3.0 and g[1, 0] == TWO24 + 2 and st == oracle.POS_ORDER
    # the first term initialises the sum: a lone -0.0 stays -0.0
    z = _bwd(np.full((1, 4), -0.0, np.float32), [0])[3]
    assert np.all(np.signbit(z))


def test_tile_boundaries():
    """Runs of exactly TILE, TILE + 1, and one straddling a boundary, integer-valued so every
    order agrees."""
    T = oracle.BWD_TILE
    rows = np.concatenate([np.full(T, 0), np.full(T + 1, 1), np.full(T // 2, 2), np.full(T, 3)])
    rng = np.random.default_rng(0)
    grad = rng.integers(-8, 9, size=(len(rows), 4)).astype(np.float32)
    rc, st, u, g, g64, nu = _bwd(grad, rows)
    ref = np.zeros((4, 4))
    np.add.at(ref, rows, grad.astype(np.float64))
    assert nu == 4 and np.array_equal(g.astype(np.float64), ref) and np.array_equal(g64, ref)


def test_tile_boundary_probe_exact():
    """A run that starts inside one tile and ends inside the third; the 2^24 head term makes
    every other grouping of the ones give a different fp32 result."""
    T = oracle.BWD_TILE
    rows = np.concatenate([np.full(3, 0), np.full(2 * T, 1)])          # run of row 1 covers k = 3 .. 2T+2
    v = np.ones(len(rows), np.float32)
    v[3] = TWO24                                                       # first element of the run
    # partial A: k = 3 .. T-1     -> 2^24 then (T-4) ones, each lost to a tie           = 2^24
    # partial B: k = T .. 2T-1    -> T ones                                             = T
    # partial C: k = 2T .. 2T+2   -> 3 ones                                             = 3
    # fold: (2^24 + T) + 3 ; T = 256 exact, then + 3 -> 2^24 + 259 -> tie to even mantissa: 2^24 + 260
    g = _bwd(col(v), rows)[3]
    assert g[0, 0] == 3.0
    assert g[1, 0] == TWO24 + T + 4


@pytest.mark.parametrize("dt", ["f16", "bf16", "f32"])
def test_matches_fp64_add_at_and_unique(dt):
    rng = np.random.default_rng(5)
    R, D, n = 5000, 8, 60_000
    ranks = np.minimum((rng.pareto(0.9, n)).astype(np.int64), R - 1)     # heavy duplicates
    rows = rng.permutation(R)[ranks]
    x = rng.standard_normal((n, D)).astype(np.float32)
    if dt == "f16":
        grad, code, xf = x.astype(np.float16), oracle.F16, x.astype(np.float16).astype(np.float64)
    elif dt == "bf16":
        bits = bf16_bits_from_f32(x)
        grad, code, xf = bits, oracle.BF16, f32_from_bf16_bits(bits).astype(np.float64)
    else:
        grad, code, xf = x, oracle.F32, x.astype(np.float64)
    pos = rng.permutation(n).astype(np.int32)
    rc, st, u, g, g64, nu = oracle.seq_grad_bwd(grad, rows, pos, 0, n, R, dtype=code)
    assert rc == 0 and (st & ~oracle.POS_ORDER) == 0
    uniq, inv = np.unique(rows, return_inverse=True)
    assert nu == len(uniq) and np.array_equal(u, uniq)
    ref = np.zeros((len(uniq), D))
    np.add.at(ref, inv, xf[pos])
    sq = np.zeros((len(uniq), D))
    np.add.at(sq, inv, xf[pos] ** 2)
    if dt != "f32":
        assert np.array_equal(g64, ref)                      # fp64 sums of 8/11-bit values are exact
    else:
        assert np.allclose(g64, ref, rtol=1e-12, atol=1e-11)
    # the fp32 result in the stated order meets the bound the atomic variant is held to
    tol = 1e-5 * np.maximum(np.abs(ref), np.sqrt(sq))
    assert np.all(np.abs(g.astype(np.float64) - ref) <= tol)
    # invariant: the sum of the row gradients is the sum of the output gradients
    assert np.allclose(g.astype(np.float64).sum(0), xf[pos].sum(0), rtol=0, atol=1e-5 * np.sqrt((xf ** 2).sum(0)))


def test_distinct_rows_is_a_conversion_exhaustive_fp16():
    """All rows distinct: row_grads == f32(grad_out) bit for bit; run over every finite and
    infinite binary16 pattern this pins the oracle's half -> float conversion to numpy's."""
    bits = np.arange(65536, dtype=np.uint16)
    h = bits.view(np.float16)
    keep = ~np.isnan(h)
    h = h[keep]
    pad = (-len(h)) % 8
    h = np.concatenate([h, np.zeros(pad, np.float16)]).reshape(-1, 8)
    n = h.shape[0]
    rng = np.random.default_rng(1)
    rows = rng.permutation(n)
    rc, st, u, g, _, nu = oracle.seq_grad_bwd(h, rows, np.arange(n, dtype=np.int32), 0, n, n, dtype=oracle.F16)
    assert nu == n and np.array_equal(u, np.arange(n))
    expect = h.astype(np.float32)[np.argsort(rows)]
    assert np.array_equal(g.view(np.uint32), expect.view(np.uint32))


def test_bf16_conversion_matches_torch():
    bits = np.arange(65536, dtype=np.uint16)
    t = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).to(torch.float32).numpy()
    keep = ~np.isnan(t)
    b = bits[keep]
    pad = (-len(b)) % 8
    b = np.concatenate([b, np.zeros(pad, np.uint16)]).reshape(-1, 8)
    n = b.shape[0]
    rc, st, u, g, _, nu = oracle.seq_grad_bwd(b, np.arange(n), np.arange(n, dtype=np.int32), 0, n, n, dtype=oracle.BF16)
    expect = np.concatenate([t[keep], np.zeros(pad, np.float32)]).reshape(-1, 8)
    assert np.array_equal(g.view(np.uint32), expect.view(np.uint32))


def test_range_capacity_and_faults():
    grad = np.arange(40, dtype=np.float32).reshape(10, 4)
    rows = np.array([3, 3, 1, 1, 1, 9, 2, 2, 0, 0])
    pos = np.arange(10, dtype=np.int32)
    # sub-range [2, 7): rows 1,1,1,9,2
    rc, st, u, g, _, nu = oracle.seq_grad_bwd(grad, rows, pos, 2, 7, 10)
    assert u.tolist() == [1, 2, 9] and np.array_equal(g[0], grad[2] + grad[3] + grad[4]) and np.array_equal(g[2], grad[5])
    # capacity smaller than the number of distinct rows
    rc, st, u, g, _, nu = oracle.seq_grad_bwd(grad, rows, pos, 0, 10, 10, cap_unique=2)
    assert nu == 5 and st == oracle.UNIQUE_OVERFLOW and u.tolist() == [0, 1]
    # empty range
    rc, st, u, g, _, nu = oracle.seq_grad_bwd(grad, rows, pos, 4, 4, 10)
    assert rc == 0 and nu == 0
    # bad row / pos are replaced by 0
    rc, st, u, g, _, nu = oracle.seq_grad_bwd(grad, np.array([12, 1]), np.array([0, 50], np.int32), 0, 2, 10)
    assert st & oracle.BAD_ID and u.tolist() == [0, 1] and np.array_equal(g[1], grad[0])
    assert oracle.seq_grad_bwd(grad[:, :3].copy(), rows, pos, 0, 10, 10)[0] == 4
    assert oracle.seq_grad_bwd(grad, rows, pos, 3, 2, 10)[0] == 2


def test_sort_lookups_is_lexsort_by_row_then_pos():
    """The backward's order written out: numpy's lexsort of the range, faults replaced and flagged."""
    rng = np.random.default_rng(12)
    n, R = 5000, 300
    rows = np.minimum(rng.pareto(0.8, n).astype(np.int64), R - 1)
    pos = rng.permutation(n).astype(np.int32)
    for j0, j1 in ((0, n), (17, 4000), (n, n)):
        rc, st, srows, spos = oracle.sort_lookups(rows, pos, j0, j1, R, n)
        order = np.lexsort((pos[j0:j1], rows[j0:j1]))
        assert (rc, st) == (0, 0) and srows.dtype == np.uint32 and spos.dtype == np.uint32
        assert np.array_equal(srows, rows[j0:j1][order]) and np.array_equal(spos, pos[j0:j1][order])
    # it is the order the backward sums in: the run of each row, and the row list, follow from it
    rc, st, srows, spos = oracle.sort_lookups(rows, pos, 0, n, R, n)
    assert np.array_equal(np.unique(srows), oracle.seq_grad_bwd(np.zeros((n, 4), np.float32), rows, pos, 0, n, R)[2])
    # faults: a row or position out of range becomes 0 and is flagged
    rc, st, srows, spos = oracle.sort_lookups([5, -1, 2, 300], np.array([3, 2, 9, 0], np.int32), 0, 4, 300, 4)
    assert rc == 0 and st == oracle.BAD_ID and srows.tolist() == [0, 0, 2, 5] and spos.tolist() == [0, 2, 0, 3]
    assert oracle.sort_lookups([1], np.zeros(1, np.int32), 1, 0, 5, 1)[0] == 2
