"""GPU parity of fs_seq_grad_bwd_update (the backward that applies the optimizer step itself):
bit for bit the table, state, replica store, row list and multi-lookup gradients that
fs_seq_grad_bwd_sorted followed by fs_sparse_update write, and within the optimizer step's
tolerance of the oracle's composition (backward in the stated order, then the rules in double
precision)."""
import numpy as np
import pytest
import torch

import fs_inputs
import oracle
from test_gpu_update import OPTS, TDT, as_f64, ulp

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import gpu_common
    assert torch.cuda.is_available()
    return gpu_common


def _bits_t(t):
    return t.detach().contiguous().view(torch.uint8)


def check_rows(got_bits, want_bits, dt, before_bits, touched):
    """The optimizer step's tolerance against the double-precision rules (see test_gpu_update.py): every
    element within one unit in the last place of the table's type (plus the float32 slack), untouched rows
    bit-identical, and of the touched rows' elements at least 97 % bit-identical (float32 arithmetic rounded
    again to a 16-bit type lands on the neighbouring value for about 2 % of them)."""
    got, want, before = as_f64(got_bits, dt), as_f64(want_bits, dt), as_f64(before_bits, dt)
    slack = 1e-6 * np.maximum(np.abs(want), np.abs(before))
    assert np.all(np.abs(got - want) <= ulp(want, dt) * (1.001 if dt != "f32" else 1.0) + slack)
    mask = np.zeros(len(got_bits), bool)
    mask[touched] = True
    g8, w8 = got_bits.view(np.uint8).reshape(len(got_bits), -1), want_bits.view(np.uint8).reshape(len(got_bits), -1)
    assert np.array_equal(g8[~mask], w8[~mask])
    if dt != "f32" and mask.any():
        same = np.mean(got_bits[mask].view(np.uint16) == want_bits[mask].view(np.uint16))
        assert same >= 0.97, same


def _case(G, dt, D, opt, n=40_000, R=30_000, cap_frac=1.0, with_store=True, seed=0):
    import paper_2301_02959_amd as fs
    dev = G.DEV
    rng = np.random.default_rng(seed + D)
    tdt = TDT[dt]
    code = G.oracle_dtype(dt)
    # a hot head (runs over several summation tiles), a warm middle, a cold tail of rows looked up once
    hot = rng.choice(R, 30, replace=False)
    rows = np.where(rng.random(n) < 0.5, hot[np.minimum(rng.pareto(0.8, n).astype(np.int64), 29)], rng.integers(0, R, n))
    order = np.argsort(rows % 4, kind="stable")
    rows, pos = rows[order].astype(np.int64), order.astype(np.int32)
    Wt = torch.randn(R, D, generator=torch.Generator().manual_seed(D + 1)).to(tdt)
    grad = torch.randn(n, D, generator=torch.Generator().manual_seed(D + 2)).to(tdt)
    lr, eps = 0.05, 1e-4
    state_shape = {"sgd": None, "rowwise": (R,), "adagrad": (R, D)}[opt]
    k = 500
    sel = np.concatenate([hot[:10], rng.permutation(R)[:k - 10]]).astype(np.int64)
    W_h = fs_inputs.as_numpy_bits(Wt).copy()
    store_h = np.zeros((k, D), W_h.dtype)
    _, _, slots_h = oracle.replica_build(W_h, sel, store_h, dtype=code)

    rows_d, pos_d, grad_d = G.to_dev(rows, torch.int64), G.to_dev(pos, torch.int32), grad.to(dev)
    srows = torch.zeros(n, dtype=torch.int32, device=dev)
    spos = torch.zeros(n, dtype=torch.int32, device=dev)
    st = torch.zeros(1, dtype=torch.int32, device=dev)
    fs.fs_sort_lookups(rows_d, pos_d, 0, n, R, n, srows, spos, st)
    nu_true = len(np.unique(rows))
    cap = max(1, int(nu_true * cap_frac))

    def fresh():
        W = Wt.to(dev).clone()
        s = torch.full(state_shape, 0.25, device=dev) if state_shape else None
        store = (torch.from_numpy(store_h.copy().view(np.int16)).view(torch.bfloat16) if dt == "bf16"
                 else torch.from_numpy(store_h.copy())).to(dev) if with_store else None
        slots = torch.from_numpy(slots_h).to(dev) if with_store else None
        uniq = torch.full((cap,), -7, dtype=torch.int64, device=dev)
        rg = torch.full((cap, D), float("nan"), dtype=torch.float32, device=dev)
        nu = torch.full((1,), -7, dtype=torch.int64, device=dev)
        return W, s, store, slots, uniq, rg, nu

    # the two calls one after the other
    Wa, sa, store_a, slots_a, uniq_a, rg_a, nu_a = fresh()
    fs.fs_seq_grad_bwd_sorted(grad_d, srows, spos, n, R, 0, uniq_a, rg_a, cap, nu_a, st)
    fs.fs_sparse_update(Wa, uniq_a, rg_a, cap, nu_a, OPTS[opt], lr, eps, sa, store_a, slots_a, k if with_store else 0, st)
    # the one call
    Wb, sb, store_b, slots_b, uniq_b, rg_b, nu_b = fresh()
    fs.fs_seq_grad_bwd_update(grad_d, srows, spos, n, R, Wb, OPTS[opt], lr, eps, sb, store_b, slots_b,
                              k if with_store else 0, uniq_b, rg_b, cap, nu_b, st)
    torch.cuda.synchronize()
    want_status = oracle.UNIQUE_OVERFLOW if cap < nu_true else 0
    assert int(st.item()) == want_status
    assert int(nu_a.item()) == int(nu_b.item()) == nu_true and torch.equal(uniq_a, uniq_b)
    assert torch.equal(_bits_t(Wa), _bits_t(Wb)), "the fused call writes the rows the two calls write"
    if sa is not None:
        assert torch.equal(_bits_t(sa), _bits_t(sb))
    if with_store:
        assert torch.equal(_bits_t(store_a), _bits_t(store_b))
    # gradients of rows looked up more than once are written as before, those of rows looked up once are not
    uq, cnt = np.unique(rows, return_counts=True)
    multi = torch.as_tensor(np.nonzero(cnt[:cap] > 1)[0], device=dev)
    single = torch.as_tensor(np.nonzero(cnt[:cap] == 1)[0], device=dev)
    assert len(multi) > 0 and len(single) > 0
    assert torch.equal(rg_a[multi].view(torch.int32), rg_b[multi].view(torch.int32))
    if D * {"f32": 4, "f16": 2, "bf16": 2}[dt] <= 1024:               # longer rows take the two steps one after the other
        assert bool(torch.isnan(rg_b[single]).all())

    # the oracle's composition on the host
    g_h = fs_inputs.as_numpy_bits(grad)
    orc, ost, ou, og, _, onu = oracle.seq_grad_bwd(g_h, rows, pos, 0, n, R, cap_unique=cap, dtype=code, want64=False)
    assert orc == 0 and onu == nu_true and np.array_equal(uniq_b[:len(ou)].cpu().numpy(), ou)
    s_h = np.full(state_shape, 0.25, np.float32) if state_shape else None
    before = W_h.copy()
    store_o = store_h.copy()
    assert oracle.sparse_update(W_h, ou, og, OPTS[opt], lr, eps, s_h, store_o if with_store else None,
                                slots_h if with_store else None, dtype=code) == (0, 0)
    check_rows(fs_inputs.as_numpy_bits(Wb), W_h, dt, before, ou)
    if s_h is not None:
        assert np.allclose(sb.cpu().numpy(), s_h, rtol=1e-6, atol=1e-30)
    if with_store:
        touched_slots = slots_h[ou][slots_h[ou] >= 0]
        check_rows(fs_inputs.as_numpy_bits(store_b), store_o, dt, store_h, touched_slots)


@pytest.mark.parametrize("opt", ["sgd", "rowwise", "adagrad"])
@pytest.mark.parametrize("dt,D", [("f32", 64), ("f16", 128), ("bf16", 256), ("f32", 4), ("f16", 24), ("bf16", 512),
                                  ("f32", 72), ("bf16", 1024)])
def test_bwd_update_equals_bwd_then_update(G, opt, dt, D):
    _case(G, dt, D, opt, n=40_000 if D <= 256 else 12_000)


def test_bwd_update_capacity_and_no_store(G):
    _case(G, "bf16", 256, "rowwise", cap_frac=0.5, seed=3)
    _case(G, "f16", 128, "adagrad", with_store=False, seed=4)
    _case(G, "f32", 64, "sgd", cap_frac=0.01, with_store=False, seed=5)


def test_bwd_update_host_faults_and_empty(G):
    import paper_2301_02959_amd as fs
    dev = G.DEV
    W = torch.zeros(10, 8, device=dev)
    grad = torch.zeros(4, 8, device=dev)
    z32 = torch.zeros(4, dtype=torch.int32, device=dev)
    uniq = torch.zeros(4, dtype=torch.int64, device=dev)
    rg = torch.zeros(4, 8, device=dev)
    nu = torch.full((1,), -7, dtype=torch.int64, device=dev)
    state = torch.zeros(10, device=dev)
    call = lambda **kw: fs.fs_seq_grad_bwd_update(grad, z32, z32, kw.get("m", 4), kw.get("R", 10), kw.get("W", W), kw.get("opt", 1),
                                                  0.1, 1e-8, kw.get("state", state), None, kw.get("slots"), 0, uniq, rg,
                                                  kw.get("cap", 4), nu, None, raise_on_error=False)
    assert call() == 0
    assert call(m=-1) == 2 and call(R=0) == 2 and call(cap=-1) == 2 and call(opt=5) == 6
    assert call(W=None) == 1 and call(state=None) == 1 and call(slots=z32) == 1
    assert call(m=0) == 0
    torch.cuda.synchronize()
    assert int(nu.item()) == 0
