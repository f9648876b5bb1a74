"""Host-only checks of the C ABI library: it loads without a GPU, exports every
symbol include/gnnd.h declares, sizes workspaces and refuses bad arguments
before anything is launched.  No compute calls."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def amd():
    import paper_2103_15386_amd as amd
    from paper_2103_15386_amd import build
    if not os.path.exists(amd.library_path()):
        build.build_library()
    return amd


def test_library_exports_every_declared_symbol(amd):
    header = open(os.path.join(ROOT, "include", "gnnd.h")).read()
    declared = set(re.findall(r"\b(gnnd_[a-z_]+)\s*\(", header))
    declared -= {"gnnd_workspace_bytes()"}
    assert {"gnnd_init_random", "gnnd_iterate", "gnnd_build", "gnnd_merge"} <= declared
    lib = C.CDLL(amd.library_path())
    for name in sorted(declared):
        assert hasattr(lib, name), f"{name} is declared but not exported"
    from paper_2103_15386_amd import binding
    assert set(binding.EXPORTS) == declared


def test_workspace_size_and_parameter_validation(amd):
    from paper_2103_15386_amd import binding
    lib = amd.load_library()
    small = amd.workspace_bytes(4096, 16, 10, 8, amd.L2SQ_F32)
    big = amd.workspace_bytes(1_000_000, 128, 32, 32, amd.L2SQ_F32)
    assert 0 < small < big < 8 << 30
    assert amd.workspace_bytes(10, 16, 10, 8, amd.L2SQ_F32) == 0      # k >= n
    assert amd.workspace_bytes(4096, 16, 129, 8, amd.L2SQ_F32) == 0   # k > 128
    assert amd.workspace_bytes(4096, 16, 128, 8, amd.L2SQ_F32) > 0
    assert amd.workspace_bytes((1 << 27) + 1, 16, 10, 8, amd.L2SQ_F32) == 0  # n <= 2^27
    assert amd.workspace_bytes(1 << 27, 16, 10, 8, amd.L2SQ_F32) > 0
    assert amd.workspace_bytes(4096, 16, 10, 11, amd.L2SQ_F32) == 0   # p > k
    assert amd.workspace_bytes(4096, 16, 40, 33, amd.L2SQ_F32) > 0    # sample lists of 66
    assert amd.workspace_bytes(4096, 16, 128, 65, amd.L2SQ_F32) == 0  # p > 64
    assert amd.workspace_bytes(4096, 0, 10, 8, amd.L2SQ_F32) == 0     # d < 1
    assert amd.workspace_bytes(4096, 16, 10, 8, 7) == 0               # metric
    # the float32 matrix-core join: float vectors, inner-product metrics, p <= 32; it keeps the
    # squared norms of all vectors in the workspace
    gram = amd.workspace_bytes(4096, 16, 10, 8, amd.L2SQ_F32, join_path=amd.JOIN_GRAM)
    assert gram >= amd.workspace_bytes(4096, 16, 10, 8, amd.L2SQ_F32, join_path=amd.JOIN_VALU) + 4096 * 4
    assert amd.workspace_bytes(4096, 16, 10, 8, amd.L2SQ_U8, join_path=amd.JOIN_GRAM) == 0
    assert amd.workspace_bytes(4096, 16, 10, 8, amd.CHI2_F32, join_path=amd.JOIN_GRAM) == 0
    assert amd.workspace_bytes(4096, 16, 40, 33, amd.COSINE_F32, join_path=amd.JOIN_GRAM) == 0
    assert amd.workspace_bytes(4096, 16, 10, 8, amd.ANGULAR_F32, amd.UPDATE_ALL_PAIRS,
                               join_path=amd.JOIN_GRAM) == 0
    assert amd.workspace_bytes(4096, 16, 10, 8, amd.L2SQ_F32, join_path=5) == 0
    # gnnd_create validates before touching the GPU: errors come back as codes
    ctx = C.c_void_p()
    prm = binding.make_params(50, 8, 50, 8, amd.L2SQ_F32)
    assert lib.gnnd_create(C.byref(ctx), C.byref(prm), 0x1000) == binding.EINVAL
    assert b"n must exceed k" in lib.gnnd_last_error(None)
    prm = binding.make_params(100, 8, 10, 8, amd.L2SQ_F32)
    assert lib.gnnd_create(C.byref(ctx), C.byref(prm), None) == binding.EINVAL
    prm.workspace_dev, prm.workspace_bytes = 0x100000, 16
    assert lib.gnnd_create(C.byref(ctx), C.byref(prm), 0x1000) == binding.ENOSPC
    assert b"workspace too small" in lib.gnnd_last_error(None)
    prm.workspace_dev = 0x100001
    assert lib.gnnd_create(C.byref(ctx), C.byref(prm), 0x1000) == binding.EINVAL
    assert lib.gnnd_iterate(None, None) == binding.EINVAL
    assert lib.gnnd_exact_knn(None, 10, 4, 0, None, 1, 3, None, None, None) == binding.EINVAL


def test_product_path_refuses_cpu_tensors(amd):
    import torch
    with pytest.raises(amd.GnndError):
        amd.Gnnd(torch.zeros(100, 8), 10, 8)
    with pytest.raises(amd.GnndError):
        amd.exact_knn(torch.zeros(100, 8), torch.zeros(4, dtype=torch.int32), 3)


def test_file_backed_shard_driver_checks_its_files_before_any_gpu_work(amd, tmp_path):
    """Arguments and files are validated on the host; the pointers below are never
    dereferenced because every call fails first."""
    import numpy as np
    from paper_2103_15386_amd import binding
    lib = amd.load_library()
    prm = binding.make_params(2000, 8, 8, 8, amd.L2SQ_F32)
    prm.workspace_dev, prm.workspace_bytes = 0x100000, 1 << 40
    prm.stream = 0x10
    args = (2, 4, 2, str(tmp_path / "i.bin").encode(), str(tmp_path / "d.bin").encode())
    call = lambda vec, stg, stg_bytes, copy: lib.gnnd_build_sharded_files(
        C.byref(prm), vec, args[0], args[1], args[2], args[3], args[4], stg, stg_bytes, copy, None)
    missing = str(tmp_path / "missing.bin").encode()
    assert call(missing, 0x2000, 1 << 20, 0x20) == binding.EIO
    assert b"cannot open" in lib.gnnd_last_error(None)
    assert call(missing, 0x2000, 1 << 10, 0x20) == binding.EINVAL   # staging too small
    assert call(missing, None, 1 << 20, 0x20) == binding.EINVAL     # no staging buffer
    assert call(missing, 0x2000, 1 << 20, 0x10) == binding.EINVAL   # copy stream = compute stream
    short = tmp_path / "short.bin"
    np.zeros(1000 * 8, dtype=np.float32).tofile(short)
    assert call(str(short).encode(), 0x2000, 1 << 20, 0x20) == binding.EIO
    assert b"shorter" in lib.gnnd_last_error(None)
    assert not (tmp_path / "i.bin").exists()  # nothing is created before the input is accepted
