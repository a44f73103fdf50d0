"""The C-ABI library loads and exports every symbol the header declares (no compute calls)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2301_02959_amd", "libflexshard_hip.so")


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "flexshard.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fs_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_four_entry_points():
    names = declared_symbols()
    for must in ("fs_plan_replication", "fs_route_bucketize", "fs_seq_gather_fwd", "fs_seq_grad_bwd"):
        assert must in names


@pytest.mark.skipif(not os.path.exists(LIB), reason="library not built (run __graft_entry__.build())")
def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(LIB)
    for name in declared_symbols():
        assert hasattr(lib, name), name
    lib.fs_version.restype = ctypes.c_int32
    lib.fs_bwd_tile.restype = ctypes.c_int32
    assert lib.fs_version() >= 1000 and lib.fs_bwd_tile() == 256


def test_binding_lists_the_same_names():
    import paper_2301_02959_amd as fs
    assert sorted(fs.EXPORTS) == declared_symbols()
    for name in fs.EXPORTS:
        assert callable(getattr(fs, name))


def test_oracle_and_library_constants_agree_by_value():
    """The two sides share no header; their constants must still mean the same."""
    import oracle
    import paper_2301_02959_amd as fs
    assert (oracle.BAD_ID, oracle.BAD_OFFSETS, oracle.BAD_PLACEMENT, oracle.COUNT_OVERFLOW, oracle.UNIQUE_OVERFLOW,
            oracle.POS_ORDER) == (fs.FS_DEV_BAD_ID, fs.FS_DEV_BAD_OFFSETS, fs.FS_DEV_BAD_PLACEMENT,
                                  fs.FS_DEV_COUNT_OVERFLOW, fs.FS_DEV_UNIQUE_OVERFLOW, fs.FS_DEV_POS_ORDER)
    assert oracle.NOT_SORTED == fs.FS_DEV_NOT_SORTED
    assert oracle.BWD_TILE == fs.FS_BWD_TILE
    assert (oracle.F32, oracle.F16, oracle.BF16) == (fs.FS_F32, fs.FS_F16, fs.FS_BF16)


@pytest.mark.skipif(not os.path.exists(LIB), reason="library not built (run __graft_entry__.build())")
def test_binding_refuses_host_tensors_and_wrong_element_types():
    """The binding passes device pointers through: a host tensor or a wrong element type never reaches the library."""
    import torch
    import paper_2301_02959_amd as fs
    host = torch.zeros(64, dtype=torch.uint8)
    with pytest.raises(TypeError):
        fs.fs_util_copy(host, host)
    w = torch.zeros(4, 8)
    with pytest.raises(TypeError):
        fs.fs_seq_gather_fwd(w, torch.zeros(1, dtype=torch.int64), torch.zeros(1, dtype=torch.int32), 0, 1, w.clone())
