"""GPU parity: fs_seq_grad_bwd against the CPU oracle.
variant 0 (sort + fixed summation order): bit-exact.
variant 1 (atomic partial sums): |x - ref64| <= 1e-5 * max(|ref64|, 2-norm of the terms)."""
import numpy as np
import pytest
import torch

import fs_inputs
import oracle
from helpers import bf16_bits_from_f32

pytestmark = pytest.mark.gpu

TWO24 = float(2 ** 24)


@pytest.fixture(scope="module")
def G():
    import gpu_common
    assert torch.cuda.is_available()
    return gpu_common


def _np_grad(x32: np.ndarray, dt: str):
    """float32 values -> (numpy array in the oracle's representation, torch tensor)."""
    if dt == "f32":
        return x32, torch.from_numpy(x32)
    if dt == "f16":
        h = x32.astype(np.float16)
        return h, torch.from_numpy(h)
    b = bf16_bits_from_f32(x32)
    return b, torch.from_numpy(b.view(np.int16)).view(torch.bfloat16)


def _check(G, grad_np, grad_t, rows, pos, j0, j1, R, dt, cap=None, atomic_too=True):
    code = G.oracle_dtype(dt)
    orc, ost, ou, og, og64, onu = oracle.seq_grad_bwd(grad_np, rows, pos, j0, j1, R, cap_unique=cap, dtype=code)
    gd, rd, pd = grad_t.to(G.DEV), G.to_dev(rows, torch.int64), G.to_dev(pos, torch.int32)
    rc, st, u, g, nu = G.hip_bwd(gd, rd, pd, j0, j1, R, 0, cap)
    assert rc == orc == 0 and st == ost and nu == onu
    assert np.array_equal(u.cpu().numpy(), ou)
    assert np.array_equal(G.bits(g), og.view(np.uint8).reshape(-1)), "variant 0 must match bit for bit"
    if atomic_too:
        rc, st, u1, g1, nu1 = G.hip_bwd(gd, rd, pd, j0, j1, R, 1, cap)
        assert rc == 0 and st == ost and nu1 == onu and np.array_equal(u1.cpu().numpy(), ou)
        # 2-norm of the terms per (row, column), from the fp64 side
        xf = (grad_t.double().numpy())[np.asarray(pos[j0:j1], np.int64)]
        uniq, inv = np.unique(np.asarray(rows[j0:j1]), return_inverse=True)
        sq = np.zeros((len(uniq), xf.shape[1]))
        np.add.at(sq, inv, xf ** 2)
        k = len(ou)
        tol = 1e-5 * np.maximum(np.abs(og64), np.sqrt(sq[:k]))
        assert np.all(np.abs(g1.double().cpu().numpy() - og64) <= tol)
    return ou, og


@pytest.mark.parametrize("dt,D", [("f32", 64), ("f16", 128), ("bf16", 256), ("f32", 4), ("f16", 8), ("bf16", 24),
                                  ("f32", 300), ("f16", 1024)])
def test_bwd_random_duplicates(G, dt, D):
    rng = np.random.default_rng(D + len(dt))
    R, n = 20_000, 9_001                               # 36 chunks, ragged tail, several sort tiles
    ranks = np.minimum(rng.pareto(0.8, n).astype(np.int64), R - 1)
    rows_i = rng.permutation(R)[ranks]                 # row of lookup i
    owner = rows_i % 5
    order = np.argsort(owner, kind="stable")           # a bucketised order: equal rows keep ascending pos
    rows, pos = rows_i[order], order.astype(np.int32)
    x = rng.standard_normal((n, D)).astype(np.float32)
    gnp, gt = _np_grad(x, dt)
    _check(G, gnp, gt, rows, pos, 0, n, R, dt)
    _check(G, gnp, gt, rows, pos, 1500, 7777, R, dt, atomic_too=False)      # a sub-range (one owner's share)


@pytest.mark.parametrize("R", [2 ** 32 - 2, 2 ** 31 + 5, 2 ** 24 + 1, 257])
def test_bwd_row_ids_up_to_the_largest_table(G, R):
    """Rows spread over the whole admitted id range (keys that use all 32 bits: four 8-bit sort passes for the
    largest table), the last row included; only the ids matter here, no table of that size exists."""
    rng = np.random.default_rng(R % 1000)
    n, D = 12_345, 8
    distinct = np.unique(np.concatenate([rng.integers(0, R, 3000), [0, R - 1, R // 2, min(R - 1, 2 ** 31 - 1), min(R - 1, 2 ** 31)]]))
    rows_i = distinct[np.minimum(rng.pareto(0.7, n).astype(np.int64), len(distinct) - 1)]
    order = np.argsort(rows_i % 3, kind="stable")
    rows, pos = rows_i[order].astype(np.int64), order.astype(np.int32)
    x = rng.standard_normal((n, D)).astype(np.float32)
    gnp, gt = _np_grad(x, "f32")
    ou, og = _check(G, gnp, gt, rows, pos, 0, n, R, "f32")
    assert ou[-1] == R - 1 and ou[0] == 0


def test_bwd_c1_end_to_end(G):
    cfg = fs_inputs.CONFIGS["c1"]
    b, pl = G.batch_on(cfg, "cpu")
    rc, st, bo, rows, pos, tc = G.hip_route(b["ids"].to(G.DEV), b["offsets"].to(G.DEV), cfg.T, cfg.B,
                                            b["row_base"].to(G.DEV), pl.to(G.DEV), cfg.U, cfg.W, 0)
    grad = fs_inputs.make_grad(cfg, b["n"])
    ou, og = _check(G, grad.numpy(), grad, rows.cpu().numpy(), pos.cpu().numpy(), 0, b["n"], cfg.R, "f32")
    # invariant: sum of row gradients = sum of output gradients
    assert np.allclose(og.astype(np.float64).sum(0), grad.double().sum(0).numpy(), rtol=0, atol=1e-3)
    # per bucket = what each owner would compute
    for bkt in range(cfg.U):
        _check(G, grad.numpy(), grad, rows.cpu().numpy(), pos.cpu().numpy(), int(bo[bkt]), int(bo[bkt + 1]), cfg.R,
               "f32", atomic_too=False)


def test_bwd_skewed_head_rows_span_many_chunks(G):
    """c5's skew on a small table: the head row owns thousands of lookups (dozens of partials)."""
    cfg = fs_inputs.CONFIGS["c5"].scaled(E=100_000, B=64, T=2)
    b, pl = G.batch_on(cfg, "cpu")
    n = b["n"]
    rc, st, bo, rows, pos, tc = G.hip_route(b["ids"].to(G.DEV), b["offsets"].to(G.DEV), cfg.T, cfg.B,
                                            b["row_base"].to(G.DEV), pl.to(G.DEV), cfg.U, cfg.W, 0)
    grad = fs_inputs.make_grad(cfg, n)
    rows_n, pos_n = rows.cpu().numpy(), pos.cpu().numpy()
    assert np.bincount(rows_n).max() > 8 * oracle.BWD_TILE
    _check(G, grad.numpy(), grad, rows_n, pos_n, 0, n, cfg.R, "f16")


def test_bwd_rounding_probes_follow_the_stated_order(G):
    """Same hand-computed cases that pin the oracle, run through the kernels."""
    T = oracle.BWD_TILE
    rows = np.concatenate([np.full(3, 0), np.full(2 * T, 1)])
    v = np.ones(len(rows), np.float32)
    v[3] = TWO24
    x = np.stack([v, -v, 0 * v, 2 * v], 1).astype(np.float32)
    pos = np.arange(len(rows), dtype=np.int32)
    rc, st, u, g, nu = G.hip_bwd(torch.from_numpy(x).to(G.DEV), G.to_dev(rows, torch.int64), G.to_dev(pos), 0, len(rows), 2, 0)
    g = g.cpu().numpy()
    assert nu == 2 and g[0, 0] == 3.0 and g[1, 0] == TWO24 + T + 4 and g[1, 1] == -(TWO24 + T + 4)
    # -0.0 survives (the first term initialises the sum)
    z = torch.full((1, 4), -0.0)
    rc, st, u, g, nu = G.hip_bwd(z.to(G.DEV), G.to_dev([0], torch.int64), G.to_dev([0], torch.int32), 0, 1, 1, 0)
    assert torch.all(torch.signbit(g.cpu()))


def test_bwd_integer_grads_every_order_agrees(G):
    rng = np.random.default_rng(77)
    R, n, D = 300, 20_000, 16
    rows = np.sort(rng.integers(0, R, n) ** 2 % R)
    pos = rng.permutation(n).astype(np.int32)
    order = np.lexsort((pos, rows))
    rows, pos = rows[order], pos[order]
    x = rng.integers(-16, 17, (n, D)).astype(np.float32)
    ref = np.zeros((R, D))
    np.add.at(ref, rows, x[pos].astype(np.float64))
    for variant in (0, 1):
        rc, st, u, g, nu = G.hip_bwd(torch.from_numpy(x).to(G.DEV), G.to_dev(rows, torch.int64), G.to_dev(pos), 0, n, R, variant)
        assert rc == 0 and st == 0
        assert np.array_equal(g.cpu().numpy().astype(np.float64), ref[u.cpu().numpy()])


def test_bwd_subnormals_and_half_conversion(G):
    """All rows distinct: row_grads is the converted gradient; every finite fp16 bit pattern."""
    bitsv = np.arange(65536, dtype=np.uint16)
    h = bitsv.view(np.float16)
    h = h[~np.isnan(h)]
    h = np.concatenate([h, np.zeros((-len(h)) % 8, np.float16)]).reshape(-1, 8)
    n = h.shape[0]
    rows = np.random.default_rng(1).permutation(n)
    _check(G, h, torch.from_numpy(h), rows, np.arange(n, dtype=np.int32), 0, n, n, "f16", atomic_too=False)
    # fp32 subnormal sums stay subnormal (no flush to zero)
    tiny = np.full((4, 4), 1e-41, np.float32)
    rc, st, u, g, nu = G.hip_bwd(torch.from_numpy(tiny).to(G.DEV), G.to_dev([2, 2, 2, 2], torch.int64),
                                 G.to_dev([0, 1, 2, 3], torch.int32), 0, 4, 3, 0)
    expect = np.float32(1e-41) + np.float32(1e-41) + np.float32(1e-41) + np.float32(1e-41)
    assert g.cpu().numpy()[0, 0] == expect and expect != 0


def test_bwd_capacity_faults_and_edges(G):
    import paper_2301_02959_amd as fs
    grad = torch.arange(40, dtype=torch.float32).reshape(10, 4)
    rows = np.array([3, 3, 1, 1, 1, 9, 2, 2, 0, 0])
    pos = np.arange(10, dtype=np.int32)
    gd, rd, pd = grad.to(G.DEV), G.to_dev(rows, torch.int64), G.to_dev(pos)
    rc, st, u, g, nu = G.hip_bwd(gd, rd, pd, 0, 10, 10, 0, cap=2)
    assert rc == 0 and nu == 5 and st == oracle.UNIQUE_OVERFLOW and u.tolist() == [0, 1]
    assert torch.equal(g.cpu()[1], grad[2] + grad[3] + grad[4])
    rc, st, u, g, nu = G.hip_bwd(gd, rd, pd, 4, 4, 10, 0)
    assert rc == 0 and nu == 0 and st == 0
    # descending pos inside a row: flagged
    rc, st, u, g, nu = G.hip_bwd(gd, G.to_dev([4, 4, 4, 1], torch.int64), G.to_dev([2, 1, 0, 3], torch.int32), 0, 4, 10, 0)
    assert st == oracle.POS_ORDER and u.tolist() == [1, 4] and nu == 2
    #   same flag, rows and count as the oracle; the values are the same terms summed (here small integers: exact)
    orc, ost, ou, og, og64, onu = oracle.seq_grad_bwd(grad.numpy(), np.array([4, 4, 4, 1]), np.array([2, 1, 0, 3], np.int32),
                                                      0, 4, 10)
    assert ost == oracle.POS_ORDER and ou.tolist() == [1, 4] and onu == 2
    assert np.array_equal(g.cpu().numpy().astype(np.float64), og64)
    # bad row / pos: flagged, in bounds
    rc, st, u, g, nu = G.hip_bwd(gd, G.to_dev([12, 1], torch.int64), G.to_dev([0, 50], torch.int32), 0, 2, 10, 0)
    assert st & oracle.BAD_ID and u.tolist() == [0, 1] and torch.equal(g.cpu()[1], grad[0])
    # host faults
    nu_t = torch.zeros(1, dtype=torch.int64, device=G.DEV)
    uq = torch.zeros(10, dtype=torch.int64, device=G.DEV)
    rg = torch.zeros(10, 4, device=G.DEV)
    call = lambda **kw: fs.fs_seq_grad_bwd(gd, rd, pd, kw.get("j0", 0), kw.get("j1", 10), kw.get("R", 10), kw.get("v", 0),
                                           uq, rg, kw.get("cap", 10), nu_t, None, raise_on_error=False,
                                           D=kw.get("D"), dtype=kw.get("dt"))
    assert call() == 0
    assert call(j0=3, j1=2) == 2 and call(R=0) == 2 and call(R=2 ** 32 - 1) == 2 and call(cap=-1) == 2
    assert call(v=2) == 6 and call(D=3) == 4 and call(dt=7) == 3
    torch.cuda.synchronize()


def test_bwd_is_deterministic(G):
    rng = np.random.default_rng(9)
    n, D, R = 30_000, 32, 500
    rows = np.sort(rng.integers(0, R, n))
    pos = np.arange(n, dtype=np.int32)
    x = torch.randn(n, D, generator=torch.Generator().manual_seed(3))
    outs = [G.hip_bwd(x.to(G.DEV), G.to_dev(rows, torch.int64), G.to_dev(pos), 0, n, R, 0)[3].clone() for _ in range(3)]
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])
