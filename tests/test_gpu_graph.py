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


def test_sorted_step_with_the_optimizer_replays_bit_exact():
    """The step built on the shared sort -- plan, route, sort, row-order gather, the backward that applies the
    optimizer step -- captured once: every replay leaves the table, the optimizer state, the replica store and
    every output exactly as the eager calls leave theirs (the sort's fused scan counts its blocks with a ticket
    that a kernel, not a memset node, clears)."""
    import ctypes
    import paper_2301_02959_amd as fs
    dev = "cuda:0"
    cfg = fs_inputs.CONFIGS["c3"].scaled(E=30_000, B=256, T=3)
    b = fs_inputs.make_batch(cfg, dev)
    pl = fs_inputs.make_placement(cfg, b["perms"], dev)
    n, R, D, U, W, T, B = b["n"], cfg.R, cfg.D, cfg.U, cfg.W, cfg.T, cfg.B
    grad = fs_inputs.make_grad(cfg, n, dev)
    ids, offsets, row_base = b["ids"], b["offsets"], b["row_base"]
    dt = fs_inputs.DTYPE_CODE[cfg.dtype]
    table0 = fs_inputs.make_table(cfg, dev)
    k = 256
    flags = fs.FS_PLAN_ACCUMULATE | fs.FS_PLAN_SELECT
    z = ctypes.c_void_p(0)
    L = fs.lib()

    def size_of(call):
        size = ctypes.c_size_t(0)
        assert call(ctypes.byref(size)) == 0
        return max(int(size.value), 256)

    sizes = dict(
        route=fs.route_workspace_bytes(T, B, n, U, W, cfg.self_bucket) + 256,
        plan=size_of(lambda s: L.fs_plan_replication(
            z, z, ctypes.c_int32(T), ctypes.c_int32(B), z, ctypes.c_int64(n), ctypes.c_int64(R), z, ctypes.c_int32(flags),
            ctypes.c_int64(k * cfg.row_bytes), ctypes.c_int64(cfg.row_bytes), z, z, z, z, s, z, z)),
        sort=size_of(lambda s: L.fs_sort_lookups(z, z, ctypes.c_int64(0), ctypes.c_int64(n), ctypes.c_int64(R),
                                                 ctypes.c_int64(n), z, z, z, s, z, z)),
        fused=size_of(lambda s: L.fs_seq_grad_bwd_update(
            z, ctypes.c_int64(n), ctypes.c_int32(D), ctypes.c_int(dt), z, z, ctypes.c_int64(n), ctypes.c_int64(R), z,
            ctypes.c_int32(fs.FS_OPT_ADAGRAD_ROWWISE), ctypes.c_float(0.05), ctypes.c_float(1e-8), z, z, z,
            ctypes.c_int64(k), z, z, ctypes.c_int64(n), z, z, s, z, z)))

    # the replica store: the k rows the plan picks on the first batch (the same for both sides)
    sel0 = torch.arange(0, R, R // k, dtype=torch.int64, device=dev)[:k].contiguous()

    def buffers():
        o = dict(bo=torch.zeros(U + 1, dtype=torch.int64, device=dev), rows=torch.zeros(n, dtype=torch.int64, device=dev),
                 pos=torch.zeros(n, dtype=torch.int32, device=dev), tc=torch.zeros(3, dtype=torch.int64, device=dev),
                 srows=torch.zeros(n, dtype=torch.int32, device=dev), spos=torch.zeros(n, dtype=torch.int32, device=dev),
                 out=torch.zeros(n, D, dtype=cfg.torch_dtype, device=dev), uniq=torch.zeros(n, dtype=torch.int64, device=dev),
                 rg=torch.zeros(n, D, device=dev), nu=torch.zeros(1, dtype=torch.int64, device=dev),
                 counts=torch.zeros(R, dtype=torch.int32, device=dev), sel=torch.zeros(k, dtype=torch.int64, device=dev),
                 nsel=torch.zeros(1, dtype=torch.int64, device=dev), st=torch.zeros(1, dtype=torch.int32, device=dev),
                 table=table0.clone(), state=torch.full((R,), 0.1, device=dev),
                 store=torch.zeros(k, D, dtype=cfg.torch_dtype, device=dev),
                 slots=torch.full((R,), -1, dtype=torch.int32, device=dev))
        for name, size in sizes.items():
            o["ws_" + name] = torch.empty(size, dtype=torch.uint8, device=dev)
        fs.fs_replica_build(o["table"], sel0, k, None, o["store"], o["slots"], o["st"])
        return o

    def step(o):
        fs.fs_plan_replication(ids, offsets, T, B, row_base, n, R, o["counts"], flags, k * cfg.row_bytes, cfg.row_bytes,
                               o["sel"], o["nsel"], None, o["st"], workspace=o["ws_plan"])
        fs.fs_route_bucketize(ids, offsets, T, B, row_base, pl, n, U, W, cfg.self_bucket, o["bo"], o["rows"], o["pos"],
                              o["tc"], o["st"], workspace=o["ws_route"])
        fs.fs_sort_lookups(o["rows"], o["pos"], 0, n, R, n, o["srows"], o["spos"], o["st"], workspace=o["ws_sort"])
        fs.fs_seq_gather_fwd_sorted(o["table"], o["srows"], o["spos"], n, o["out"], o["st"])
        fs.fs_seq_grad_bwd_update(grad, o["srows"], o["spos"], n, R, o["table"], fs.FS_OPT_ADAGRAD_ROWWISE, 0.05, 1e-8,
                                  o["state"], o["store"], o["slots"], k, o["uniq"], o["rg"], n, o["nu"], o["st"],
                                  workspace=o["ws_fused"])

    eager, replay = buffers(), buffers()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(replay)
    torch.cuda.current_stream().wait_stream(side)
    step(eager)                                           # both sides have taken one step before the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(replay)                                      # captured, not run

    def same():
        torch.cuda.synchronize()
        nu = int(eager["nu"].item())
        assert nu == int(replay["nu"].item()) and int(eager["st"].item()) == int(replay["st"].item()) == 0
        for name in ("bo", "rows", "pos", "tc", "srows", "spos", "counts", "nsel", "state"):
            assert torch.equal(eager[name], replay[name]), name
        for name in ("out", "table", "store"):
            assert torch.equal(eager[name].view(torch.int16), replay[name].view(torch.int16)), name
        assert torch.equal(eager["uniq"][:nu], replay["uniq"][:nu])

    same()
    for round_ in range(4):
        step(eager)
        graph.replay()
        same()
        torch.cuda.synchronize()
        ids.copy_(torch.roll(ids, 3))
        grad.mul_(-0.5)
        _ = (table0.float() * 2).sum().item()
