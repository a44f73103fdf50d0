"""fs_util_copy (the benchmark's plain-copy reference) and the timing hooks."""
import pytest
import torch

pytestmark = pytest.mark.gpu


def test_util_copy_and_faults():
    import paper_2301_02959_amd as fs
    dev = "cuda:0"
    for nbytes in (16, 4096, 4096 + 16, 1 << 20, (1 << 24) + 48):
        src = torch.randint(0, 255, (nbytes,), dtype=torch.uint8, device=dev)
        dst = torch.zeros(nbytes + 16, dtype=torch.uint8, device=dev)
        assert fs.fs_util_copy(dst, src, nbytes) == 0
        torch.cuda.synchronize()
        assert torch.equal(dst[:nbytes], src) and int(dst[nbytes:].sum()) == 0
    src = torch.zeros(64, dtype=torch.uint8, device=dev)
    dst = torch.zeros(64, dtype=torch.uint8, device=dev)
    assert fs.fs_util_copy(dst, src, 0) == 0
    assert fs.fs_util_copy(dst, src, 24, raise_on_error=False) == 4
    assert fs.fs_util_copy(dst[1:], src, 16, raise_on_error=False) == 4
    assert fs.fs_util_copy(dst, src, -16, raise_on_error=False) == 2
    assert fs.fs_util_copy(None, src, 16, raise_on_error=False) == 1


def test_timing_hooks_select_kernels():
    import paper_2301_02959_amd as fs
    dev = "cuda:0"
    src = torch.zeros(1 << 20, dtype=torch.uint8, device=dev)
    dst = torch.zeros(1 << 20, dtype=torch.uint8, device=dev)
    W = torch.randn(100, 8, device=dev)
    rows = torch.arange(50, device=dev)
    pos = torch.arange(50, dtype=torch.int32, device=dev)
    out = torch.zeros(50, 8, device=dev)

    def work():
        fs.fs_util_copy(dst, src)
        fs.fs_seq_gather_fwd(W, rows, pos, 0, 50, out)

    fs.fs_prof_begin(16)
    work()
    work()
    rec = fs.fs_prof_end(16)
    assert [n for n, _ in rec] == ["util_copy", "gather_rows"] * 2 and all(ms > 0 for _, ms in rec)
    fs.fs_prof_begin(16, only="gather_rows")
    work()
    rec = fs.fs_prof_end(16)
    assert [n for n, _ in rec] == ["gather_rows"] and rec[0][1] > 0
    work()                                              # timing off again
    assert fs.fs_prof_end(16) == []
    torch.cuda.synchronize()
    assert torch.equal(out, W[:50])


def test_read_write_mix_reference_stream():
    """The reference stream writes each group's running sum after every w pieces, in bounds and in order."""
    import paper_2301_02959_amd as fs
    dev = "cuda:0"
    pieces, w = 700, 64                                  # groups of 256, 256 and 188 pieces
    src = torch.ones(pieces * 128, dtype=torch.int32, device=dev)
    dst = torch.full((12 * 256,), -1, dtype=torch.int32, device=dev)
    fs.fs_util_read_write_mix(src, w, dst)
    fs.fs_util_read_write_mix(src, 0, None)              # reads only
    torch.cuda.synchronize()
    rows = dst.view(12, 256).cpu()
    want = [64, 128, 192, 256, 64, 128, 192, 256, 64, 128, -1, -1]
    assert all(bool((rows[r] == want[r]).all()) for r in range(12))
    assert fs.fs_util_read_write_mix(src[:100], w, dst, raise_on_error=False) == 4       # not whole pieces
    assert fs.fs_util_read_write_mix(src, w, None, raise_on_error=False) == 1
