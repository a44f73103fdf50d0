"""fs_route_bucketize_noalloc (workspace in the library's static device array) writes what
fs_route_bucketize writes, bit for bit, on two calls in a row, the second on a smaller batch; sizes
beyond the array are refused."""
import numpy as np
import pytest
import torch

import paper_2301_02959_amd as fs
from helpers import random_jagged, random_placement

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _route_both(rng, T, B, E, max_len, U, W, self_):
    ids, offsets, row_base, n = random_jagged(rng, T, B, E, max_len)
    pl = random_placement(rng, T * E, U, W)
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    ids_d, off_d, rb_d = d(ids), d(offsets), d(row_base)
    pl_d = torch.from_numpy(pl.view(np.int32)).to(DEV)
    outs = []
    for entry in (fs.fs_route_bucketize, fs.fs_route_bucketize_noalloc):
        bo = torch.full((U + 1,), -7, dtype=torch.int64, device=DEV)
        rows = torch.full((max(n, 1),), -7, dtype=torch.int64, device=DEV)
        pos = torch.full((max(n, 1),), -7, dtype=torch.int32, device=DEV)
        tc = torch.full((3,), -7, dtype=torch.int64, device=DEV)
        st = torch.zeros(1, dtype=torch.int32, device=DEV)
        entry(ids_d, off_d, T, B, rb_d, pl_d, n, U, W, self_, bo, rows, pos, tc, st)
        torch.cuda.synchronize()
        outs.append((bo.cpu(), rows.cpu(), pos.cpu(), tc.cpu(), int(st.item())))
    return n, outs


def test_noalloc_matches_route_bucketize_twice_second_smaller():
    rng = np.random.default_rng(2959)
    # several 2048-lookup tiles and a ragged tail, then a smaller batch over the array's stale contents
    for (T, B, E, max_len, U, W, self_) in ((3, 700, 5000, 90, 64, 8, 9), (2, 97, 300, 30, 8, 4, 5)):
        print(f"noalloc case T={T} B={B} E={E} U={U}", flush=True)
        n, (a, b) = _route_both(rng, T, B, E, max_len, U, W, self_)
        assert n > 0 and a[4] == 0 and b[4] == 0
        for x, y in zip(a[:4], b[:4]):
            assert torch.equal(x, y)
        assert int(a[0][-1]) == n and sorted(b[2][:n].tolist()) == list(range(n))


def test_noalloc_empty_batch_and_size_limit():
    z = lambda k, dt: torch.zeros(k, dtype=dt, device=DEV)
    bo = torch.full((9,), -7, dtype=torch.int64, device=DEV)
    st = z(1, torch.int32)
    fs.fs_route_bucketize_noalloc(z(1, torch.int64), z(5, torch.int64), 1, 4, torch.tensor([0, 10], device=DEV),
                                  z(10, torch.int32), 0, 8, 8, 0, bo, z(1, torch.int64), z(1, torch.int32), None, st)
    torch.cuda.synchronize()
    assert bo.tolist() == [0] * 9 and int(st.item()) == 0
    # a batch whose workspace would not fit the array: refused on the host, nothing launched (the
    # pointers are never read, the sizes alone decide)
    n_big = fs.FS_ROUTE_NOALLOC_SCRATCH_BYTES // 6 + 4096
    assert fs.route_workspace_bytes(1, 4, n_big, 8, 8, 0) > fs.FS_ROUTE_NOALLOC_SCRATCH_BYTES
    rc = fs.fs_route_bucketize_noalloc(z(1, torch.int64), z(5, torch.int64), 1, 4, z(2, torch.int64), z(10, torch.int32),
                                       n_big, 8, 8, 0, bo, z(1, torch.int64), z(1, torch.int32), None, st,
                                       raise_on_error=False)
    assert rc == 5      # FS_ERR_WORKSPACE
