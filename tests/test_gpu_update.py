"""GPU parity: fs_sparse_update against the CPU oracle (the same rules in double precision).

Tolerance (derived from the arithmetic): the kernel computes in float32, one rounding per operation,
at most six operations between the inputs and the new weight, so the float32 value is within about
1e-6 (relative to |w| + |step|) of the exact one; rounding it to the table's type can then land one
unit in the last place away from the oracle's single rounding when the exact value lies next to a
rounding boundary, which is rare: float32 tables are compared within 1e-6, 16-bit tables within one
unit in the last place with at least 99.5 % of the elements bit-identical.  State: 1e-6 relative.
"""
import numpy as np
import pytest
import torch

import fs_inputs
import oracle

pytestmark = pytest.mark.gpu

TDT = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
OPTS = {"sgd": oracle.OPT_SGD, "rowwise": oracle.OPT_ADAGRAD_ROWWISE, "adagrad": oracle.OPT_ADAGRAD}


@pytest.fixture(scope="module")
def G():
    import gpu_common
    assert torch.cuda.is_available()
    return gpu_common


def as_f64(bits, dt):
    if dt == "bf16":
        return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return bits.astype(np.float64)


def ulp(x, dt):
    """One unit in the last place of the table's type at |x| (normal range)."""
    mant = {"f32": 23, "f16": 10, "bf16": 7}[dt]
    emin = {"f32": -126, "f16": -14, "bf16": -126}[dt]
    e = np.floor(np.log2(np.maximum(np.abs(x), 2.0 ** emin)))
    return 2.0 ** (e - mant)


def check_tables(got_bits, want_bits, dt, before_bits):
    """before_bits: the table before the step; |w| + |step| <= 3 max(|w_before|, |w_after|)."""
    got, want, before = as_f64(got_bits, dt), as_f64(want_bits, dt), as_f64(before_bits, dt)
    slack = 1e-6 * np.maximum(np.abs(want), np.abs(before))         # float32 arithmetic against exact
    if dt == "f32":
        assert np.all(np.abs(got - want) <= slack + ulp(want, dt))
    else:
        assert np.all(np.abs(got - want) <= ulp(want, dt) * 1.001 + slack)
        same = np.mean(got_bits.view(np.uint16) == want_bits.view(np.uint16))
        assert same >= 0.995, same


@pytest.mark.parametrize("opt", ["sgd", "rowwise", "adagrad"])
@pytest.mark.parametrize("dt,D", [("f32", 4), ("f32", 64), ("f16", 8), ("bf16", 128), ("bf16", 256), ("f16", 24),
                                  ("f32", 72), ("bf16", 1024), ("f32", 520)])
def test_update_matches_oracle(G, opt, dt, D):
    import paper_2301_02959_amd as fs
    rng = np.random.default_rng(D + len(opt))
    tdt = TDT[dt]
    R, n_u = 3000, 1357                                  # several waves and a ragged tail
    Wt = torch.randn(R, D, generator=torch.Generator().manual_seed(D)).to(tdt)
    rows = np.sort(rng.choice(R, n_u, replace=False)).astype(np.int64)
    code = G.oracle_dtype(dt)
    lr, eps = 0.05, 1e-4
    state_shape = {"sgd": None, "rowwise": (R,), "adagrad": (R, D)}[opt]
    W_d = Wt.to(G.DEV)
    W_h = fs_inputs.as_numpy_bits(Wt).copy()
    s_d = torch.zeros(state_shape, device=G.DEV) if state_shape else None
    s_h = np.zeros(state_shape, np.float32) if state_shape else None
    k = 200
    sel = rng.permutation(R)[:k].astype(np.int64)
    store_h = np.zeros((k, D), W_h.dtype)
    _, _, slots_h = oracle.replica_build(W_h, sel, store_h, dtype=code)
    store_d = torch.from_numpy(store_h.copy()).view(tdt if dt != "bf16" else torch.bfloat16).to(G.DEV) if dt != "bf16" \
        else torch.from_numpy(store_h.copy().view(np.int16)).view(torch.bfloat16).to(G.DEV)
    slots_d = torch.from_numpy(slots_h).to(G.DEV)
    rows_d = G.to_dev(rows, torch.int64)
    nu_d = torch.tensor([n_u], dtype=torch.int64, device=G.DEV)
    st = torch.zeros(1, dtype=torch.int32, device=G.DEV)
    for step in range(2):                               # the second step starts from a non-zero state
        W_before, store_before = W_h.copy(), store_h.copy()
        g = (rng.standard_normal((n_u, D)) * 10.0 ** rng.integers(-3, 2, (n_u, 1))).astype(np.float32)
        g_d = torch.from_numpy(g).to(G.DEV)
        assert fs.fs_sparse_update(W_d, rows_d, g_d, n_u + 50 if step else n_u, nu_d if step else None, OPTS[opt], lr, eps,
                                   s_d, store_d, slots_d, k, st) == 0
        assert oracle.sparse_update(W_h, rows, g, OPTS[opt], lr, eps, s_h, store_h, slots_h, dtype=code) == (0, 0)
        torch.cuda.synchronize()
        assert int(st.item()) == 0
        got = fs_inputs.as_numpy_bits(W_d.cpu())
        check_tables(got, W_h, dt, W_before)
        check_tables(fs_inputs.as_numpy_bits(store_d.cpu()), store_h, dt, store_before)
        # rows without a gradient are bit-identical to before
        untouched = np.setdiff1d(np.arange(R), rows)
        assert np.array_equal(got[untouched].view(np.uint8), W_before[untouched].view(np.uint8))
        if s_h is not None:
            assert np.allclose(s_d.cpu().numpy(), s_h, rtol=1e-6, atol=1e-30)
        # carry on from the oracle's table so that the two do not drift apart between steps
        W_d.copy_(torch.from_numpy(W_h.view(np.int16) if dt == "bf16" else W_h).view(tdt) if dt == "bf16"
                  else torch.from_numpy(W_h))
        store_d.copy_(torch.from_numpy(store_h.view(np.int16)).view(tdt) if dt == "bf16" else torch.from_numpy(store_h))
        if s_h is not None:
            s_d.copy_(torch.from_numpy(s_h))


def test_update_faults(G):
    import paper_2301_02959_amd as fs
    W = torch.arange(6 * 4, dtype=torch.float32).reshape(6, 4).to(G.DEV)
    W0 = W.clone()
    st = torch.zeros(1, dtype=torch.int32, device=G.DEV)
    store = torch.full((2, 4), -1.0, device=G.DEV)
    slots = torch.tensor([-1, 1, -1, -1, 0, -1], dtype=torch.int32, device=G.DEV)
    g = torch.ones(3, 4, device=G.DEV)
    rows = G.to_dev([4, 9, 2], torch.int64)
    assert fs.fs_sparse_update(W, rows, g, 3, None, fs.FS_OPT_SGD, 0.5, 0.0, None, store, slots, 2, st) == 0
    torch.cuda.synchronize()
    assert int(st.item()) == oracle.BAD_ID
    assert torch.equal(W[4], W0[4] - 0.5) and torch.equal(W[2], W0[2] - 0.5)
    assert torch.equal(store[0], W[4]) and torch.all(store[1] == -1)
    assert torch.equal(W[[0, 1, 3, 5]], W0[[0, 1, 3, 5]])
    # only the first *num_unique entries are applied
    W.copy_(W0)
    nu = torch.tensor([1], dtype=torch.int64, device=G.DEV)
    assert fs.fs_sparse_update(W, rows, g, 3, nu, fs.FS_OPT_SGD, 0.5, 0.0) == 0
    torch.cuda.synchronize()
    assert torch.equal(W[4], W0[4] - 0.5) and torch.equal(W[2], W0[2])
    # host faults
    kw = dict(raise_on_error=False)
    assert fs.fs_sparse_update(W, rows, g, 0, None, fs.FS_OPT_SGD, 0.5, 0.0) == 0
    assert fs.fs_sparse_update(W, rows, g, 3, None, 7, 0.5, 0.0, **kw) == 6
    assert fs.fs_sparse_update(W, rows, g, 3, None, fs.FS_OPT_ADAGRAD, 0.5, 0.0, None, **kw) == 1
    assert fs.fs_sparse_update(W, None, g, 3, None, fs.FS_OPT_SGD, 0.5, 0.0, **kw) == 1
    assert fs.fs_sparse_update(W, rows, g, 3, None, fs.FS_OPT_SGD, 0.5, 0.0, None, store, None, 2, **kw) == 1
    assert fs.fs_sparse_update(W, rows, g, -1, None, fs.FS_OPT_SGD, 0.5, 0.0, **kw) == 2
    assert fs.fs_sparse_update(W, rows, g, 3, None, fs.FS_OPT_SGD, 0.5, 0.0, D=3, **kw) == 4
    assert fs.fs_sparse_update(W, rows, g, 3, None, fs.FS_OPT_SGD, 0.5, 0.0, dtype=9, **kw) == 3
    torch.cuda.synchronize()


def test_backward_then_update_c1(G):
    """c1 end to end: route -> backward -> row-wise Adagrad step, against the oracle's own chain."""
    import paper_2301_02959_amd as fs
    cfg = fs_inputs.CONFIGS["c1"]
    b, pl = G.batch_on(cfg, G.DEV)
    n, R, D = b["n"], cfg.R, cfg.D
    Wt = fs_inputs.make_table(cfg)
    grad = fs_inputs.make_grad(cfg, n, G.DEV)
    rc, st, bo, rows, pos, tc = G.hip_route(b["ids"], b["offsets"], cfg.T, cfg.B, b["row_base"], pl, cfg.U, cfg.W, 0)
    rc, st, u, rg, nu = G.hip_bwd(grad, rows, pos, 0, n, R, 0)
    W_d = Wt.to(G.DEV)
    s_d = torch.zeros(R, device=G.DEV)
    status = torch.zeros(1, dtype=torch.int32, device=G.DEV)
    fs.fs_sparse_update(W_d, u, rg, nu, None, fs.FS_OPT_ADAGRAD_ROWWISE, 0.1, 1e-8, s_d, dev_status=status)
    torch.cuda.synchronize()
    W_h = Wt.numpy().copy()
    s_h = np.zeros(R, np.float32)
    orc, ost, ou, og, _, onu = oracle.seq_grad_bwd(grad.cpu().numpy(), rows.cpu().numpy(), pos.cpu().numpy(), 0, n, R)
    assert oracle.sparse_update(W_h, ou, og, oracle.OPT_ADAGRAD_ROWWISE, 0.1, 1e-8, s_h) == (0, 0)
    assert int(status.item()) == 0 and onu == nu
    check_tables(W_d.cpu().numpy(), W_h, "f32", Wt.numpy())
    assert np.allclose(s_d.cpu().numpy(), s_h, rtol=1e-6, atol=1e-30)
