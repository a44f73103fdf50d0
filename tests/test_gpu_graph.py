"""The whole step captured in a HIP graph (no entry point allocates, synchronises or clears memory
with a memset node): every replay must write exactly what the eager calls write, also with eager
work and synchronisations between the replays and with the inputs changed in place."""
import numpy as np
import pytest
import torch

import fs_inputs

pytestmark = pytest.mark.gpu


def test_step_replays_bit_exact():
    import paper_2301_02959_amd as fs
    dev = "cuda:0"
    cfg = fs_inputs.CONFIGS["c1"].scaled(B=64)
    b = fs_inputs.make_batch(cfg, dev)
    pl = fs_inputs.make_placement(cfg, b["perms"], dev)
    n, R, D, U, W, T, B = b["n"], cfg.R, cfg.D, cfg.U, cfg.W, cfg.T, cfg.B
    Wt = fs_inputs.make_table(cfg, dev)
    grad = fs_inputs.make_grad(cfg, n, dev)
    ids, offsets, row_base = b["ids"], b["offsets"], b["row_base"]

    def buffers():
        return dict(bo=torch.zeros(U + 1, dtype=torch.int64, device=dev), rows=torch.zeros(n, dtype=torch.int64, device=dev),
                    pos=torch.zeros(n, dtype=torch.int32, device=dev), tc=torch.zeros(3, dtype=torch.int64, device=dev),
                    out=torch.zeros(n, D, device=dev), uniq=torch.zeros(n, dtype=torch.int64, device=dev),
                    rg=torch.zeros(n, D, device=dev), nu=torch.zeros(1, dtype=torch.int64, device=dev),
                    counts=torch.zeros(R, dtype=torch.int32, device=dev), sel=torch.zeros(64, dtype=torch.int64, device=dev),
                    nsel=torch.zeros(1, dtype=torch.int64, device=dev), st=torch.zeros(1, dtype=torch.int32, device=dev))

    import ctypes
    z = ctypes.c_void_p(0)
    L = fs.lib()

    def size_of(call):
        size = ctypes.c_size_t(0)
        assert call(ctypes.byref(size)) == 0
        return max(int(size.value), 256)

    ws_route = torch.empty(fs.route_workspace_bytes(T, B, n, U, W, 0) + 256, dtype=torch.uint8, device=dev)
    ws_bwd = torch.empty(size_of(lambda s: L.fs_seq_grad_bwd(
        z, ctypes.c_int64(n), ctypes.c_int32(D), ctypes.c_int(fs.FS_F32), z, z, ctypes.c_int64(0), ctypes.c_int64(n),
        ctypes.c_int64(R), ctypes.c_int32(0), z, z, ctypes.c_int64(n), z, z, s, z, z)), dtype=torch.uint8, device=dev)
    flags = fs.FS_PLAN_ACCUMULATE | fs.FS_PLAN_SELECT
    ws_plan = torch.empty(size_of(lambda s: L.fs_plan_replication(
        z, z, ctypes.c_int32(T), ctypes.c_int32(B), z, ctypes.c_int64(n), ctypes.c_int64(R), z, ctypes.c_int32(flags),
        ctypes.c_int64(64 * cfg.row_bytes), ctypes.c_int64(cfg.row_bytes), z, z, z, z, s, z, z)),
        dtype=torch.uint8, device=dev)

    def step(o):
        fs.fs_plan_replication(ids, offsets, T, B, row_base, n, R, o["counts"], flags, 64 * cfg.row_bytes, cfg.row_bytes,
                               o["sel"], o["nsel"], None, o["st"], workspace=ws_plan)
        fs.fs_route_bucketize(ids, offsets, T, B, row_base, pl, n, U, W, 0, o["bo"], o["rows"], o["pos"], o["tc"], o["st"],
                              workspace=ws_route)
        fs.fs_seq_gather_fwd(Wt, o["rows"], o["pos"], 0, n, o["out"], o["st"])
        fs.fs_seq_grad_bwd(grad, o["rows"], o["pos"], 0, n, R, 0, o["uniq"], o["rg"], n, o["nu"], o["st"], workspace=ws_bwd)

    eager, replay = buffers(), buffers()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                        # warm-up on the capture stream, as torch asks
        step(replay)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for v in replay.values():
        v.zero_()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(replay)

    def same():
        torch.cuda.synchronize()
        k = int(eager["nu"].item())
        assert k == int(replay["nu"].item()) and int(eager["st"].item()) == int(replay["st"].item()) == 0
        for name in ("bo", "rows", "pos", "tc", "out", "counts", "nsel"):
            assert torch.equal(eager[name], replay[name]), name
        assert torch.equal(eager["uniq"][:k], replay["uniq"][:k])
        assert torch.equal(eager["rg"][:k].view(torch.int32), replay["rg"][:k].view(torch.int32))
        ks = int(eager["nsel"].item())
        assert torch.equal(eager["sel"][:ks], replay["sel"][:ks])

    for round_ in range(4):
        step(eager)
        graph.replay()
        same()
        # eager work and a change of the inputs in place between the replays
        torch.cuda.synchronize()
        ids.copy_(torch.roll(ids, 1))
        grad.mul_(-0.5)
        _ = (Wt * 2).sum().item()
