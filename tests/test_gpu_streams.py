"""Entry points keep no state between calls: two pipelines that run side by side on two streams, each with its
own outputs and workspaces, write exactly what the same calls write one after the other on one stream."""
import ctypes

import pytest
import torch

import fs_inputs

pytestmark = pytest.mark.gpu


def test_two_streams_match_serial():
    import paper_2301_02959_amd as fs
    dev = "cuda:0"
    cfg = fs_inputs.CONFIGS["c3"].scaled(E=40_000, B=512, T=4)         # ~1 M lookups: long enough to overlap
    b = fs_inputs.make_batch(cfg, dev)
    pl = fs_inputs.make_placement(cfg, b["perms"], dev)
    n, R, D, U, W, T, B = b["n"], cfg.R, cfg.D, cfg.U, cfg.W, cfg.T, cfg.B
    Wt = fs_inputs.make_table(cfg, dev)
    grad = fs_inputs.make_grad(cfg, n, dev)
    ids, offsets, row_base = b["ids"], b["offsets"], b["row_base"]
    ids2 = torch.roll(ids, 7)                                           # the second pipeline's batch
    z = ctypes.c_void_p(0)
    L = fs.lib()
    dt = fs_inputs.DTYPE_CODE[cfg.dtype]

    def size_of(call):
        size = ctypes.c_size_t(0)
        assert call(ctypes.byref(size)) == 0
        return max(int(size.value), 256)

    flags = fs.FS_PLAN_ACCUMULATE | fs.FS_PLAN_SELECT
    k_sel = 4096

    def buffers():
        return dict(
            bo=torch.zeros(U + 1, dtype=torch.int64, device=dev), rows=torch.zeros(n, dtype=torch.int64, device=dev),
            pos=torch.zeros(n, dtype=torch.int32, device=dev), tc=torch.zeros(3, dtype=torch.int64, device=dev),
            out=torch.zeros(n, D, dtype=cfg.torch_dtype, device=dev), uniq=torch.zeros(n, dtype=torch.int64, device=dev),
            rg=torch.zeros(n, D, device=dev), nu=torch.zeros(1, dtype=torch.int64, device=dev),
            counts=torch.zeros(R, dtype=torch.int32, device=dev), sel=torch.zeros(k_sel, dtype=torch.int64, device=dev),
            nsel=torch.zeros(1, dtype=torch.int64, device=dev), st=torch.zeros(1, dtype=torch.int32, device=dev),
            ws_route=torch.empty(fs.route_workspace_bytes(T, B, n, U, W, cfg.self_bucket) + 256, dtype=torch.uint8, device=dev),
            ws_bwd=torch.empty(size_of(lambda s: L.fs_seq_grad_bwd(
                z, ctypes.c_int64(n), ctypes.c_int32(D), ctypes.c_int(dt), z, z, ctypes.c_int64(0), ctypes.c_int64(n),
                ctypes.c_int64(R), ctypes.c_int32(0), z, z, ctypes.c_int64(n), z, z, s, z, z)), dtype=torch.uint8, device=dev),
            ws_plan=torch.empty(size_of(lambda s: L.fs_plan_replication(
                z, z, ctypes.c_int32(T), ctypes.c_int32(B), z, ctypes.c_int64(n), ctypes.c_int64(R), z, ctypes.c_int32(flags),
                ctypes.c_int64(k_sel * cfg.row_bytes), ctypes.c_int64(cfg.row_bytes), z, z, z, z, s, z, z)),
                dtype=torch.uint8, device=dev))

    def step(o, ids_):
        fs.fs_plan_replication(ids_, offsets, T, B, row_base, n, R, o["counts"], flags, k_sel * cfg.row_bytes, cfg.row_bytes,
                               o["sel"], o["nsel"], None, o["st"], workspace=o["ws_plan"])
        fs.fs_route_bucketize(ids_, offsets, T, B, row_base, pl, n, U, W, cfg.self_bucket, o["bo"], o["rows"], o["pos"],
                              o["tc"], o["st"], workspace=o["ws_route"])
        fs.fs_seq_gather_fwd(Wt, o["rows"], o["pos"], 0, n, o["out"], o["st"])
        fs.fs_seq_grad_bwd(grad, o["rows"], o["pos"], 0, n, R, 0, o["uniq"], o["rg"], n, o["nu"], o["st"],
                           workspace=o["ws_bwd"])

    serial = [buffers(), buffers()]
    step(serial[0], ids)
    step(serial[1], ids2)
    torch.cuda.synchronize()

    side_by_side = [buffers(), buffers()]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    for _ in range(3):                                                  # three rounds: counts accumulate in both
        for o, s, ids_ in zip(side_by_side, streams, (ids, ids2)):
            with torch.cuda.stream(s):
                step(o, ids_)
    torch.cuda.synchronize()
    for o, ids_ in zip(serial, (ids, ids2)):                            # bring the serial pair to three rounds too
        step(o, ids_)
        step(o, ids_)
    torch.cuda.synchronize()

    for a, c in zip(serial, side_by_side):
        k = int(a["nu"].item())
        assert k == int(c["nu"].item()) and int(a["st"].item()) == int(c["st"].item()) == 0
        for name in ("bo", "rows", "pos", "tc", "counts", "nsel"):
            assert torch.equal(a[name], c[name]), name
        assert torch.equal(a["out"].view(torch.int16), c["out"].view(torch.int16))
        assert torch.equal(a["uniq"][:k], c["uniq"][:k])
        assert torch.equal(a["rg"][:k].view(torch.int32), c["rg"][:k].view(torch.int32))
        ks = int(a["nsel"].item())
        assert ks == int(c["nsel"].item()) and torch.equal(a["sel"][:ks], c["sel"][:ks])
