"""The entry point that allocates nothing: gnnd_build_static takes its scratch
from a static device array inside the library.  Its output must equal what
the workspace-based entry points (gnnd_create + gnnd_build + gnnd_get_graph)
give for the same parameters - bit for bit, ids and distances - on two calls in
a row that share the array, the second with a smaller input, and again when
the first shape comes back."""
import ctypes as C
import os

import numpy as np
import pytest
import torch

import workloads as W

SEED = W.ALGO_SEED


def _reference(amd, xd, k, p, metric, iters, join_path):
    ctx = amd.Gnnd(xd, k, p, metric, SEED, join_path)
    ctx.build(iters, want_stats=False)
    ids, dist = ctx.graph()
    path = ctx.join_path()
    torch.cuda.synchronize()
    ctx.close()
    return ids, dist, path


@pytest.mark.gpu
def test_static_scratch_build_equals_the_workspace_build_on_calls_in_a_row():
    import paper_2103_15386_amd as amd
    cases = [
        # uint8 rows: matrix-core join, several tiles and a ragged tail (n not a multiple of 4)
        (W.sift_like_u8(6001, 64, seed=71, n_comp=8), 16, 16, amd.L2SQ_U8, 4, amd.JOIN_AUTO),
        # smaller input next, float rows, float32 matrix-core join, k < 64 lanes, p < k
        (W.uniform_f32(2500, 24, seed=72), 10, 8, amd.L2SQ_F32, 5, amd.JOIN_AUTO),
        # the first shape again: nothing may be left over from the smaller call
        (W.sift_like_u8(6001, 64, seed=71, n_comp=8), 16, 16, amd.L2SQ_U8, 4, amd.JOIN_AUTO),
        # long lists (two entries per lane), angular metric
        (W.deep_like_f32(1500, 32, seed=73, n_comp=8), 80, 20, amd.ANGULAR_F32, 3, amd.JOIN_VALU),
    ]
    for call, (x, k, p, metric, iters, jp) in enumerate(cases):
        xd = torch.from_numpy(x).cuda()
        want_ids, want_dist, path = _reference(amd, xd, k, p, metric, iters, jp)
        ids = torch.full((len(x), k), -7, dtype=torch.int32, device="cuda")
        dist = torch.zeros((len(x), k), dtype=want_dist.dtype, device="cuda")
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]
        got_ids, got_dist = amd.gnnd_build_static(xd, k, p, metric, SEED, iters, jp, ids, dist)
        torch.cuda.synchronize()
        # the call took no device memory (the outputs existed before it); the first call
        # on a device is the set-up that looks the array up, which is when the runtime
        # puts the array on the device
        if call > 0:
            assert torch.cuda.mem_get_info()[0] == free_before
        assert got_ids.data_ptr() == ids.data_ptr()
        assert torch.equal(got_ids, want_ids), f"ids differ (n={len(x)}, k={k})"
        assert torch.equal(got_dist, want_dist), f"distances differ (n={len(x)}, k={k})"
        if metric == amd.L2SQ_U8:
            assert path == amd.JOIN_MFMA  # the reference resolved to the same join
        elif jp == amd.JOIN_AUTO:
            assert path == amd.JOIN_GRAM


@pytest.mark.gpu
def test_static_scratch_build_refuses_what_does_not_fit():
    import paper_2103_15386_amd as amd
    from paper_2103_15386_amd import binding
    cap = binding.STATIC_SCRATCH_BYTES
    x = torch.zeros((200_000, 16), dtype=torch.float32, device="cuda")
    assert amd.workspace_bytes(200_000, 16, 32, 32, amd.L2SQ_F32) > cap
    with pytest.raises(amd.GnndError) as err:
        amd.gnnd_build_static(x, 32, 32, amd.L2SQ_F32, SEED, 1)
    assert err.value.code == binding.ENOSPC and "static array holds" in str(err.value)
    # float data cannot be promised to the matrix-core join without a look at them
    y = torch.zeros((1000, 16), dtype=torch.float32, device="cuda")
    with pytest.raises(amd.GnndError) as err:
        amd.gnnd_build_static(y, 8, 8, amd.L2SQ_F32, SEED, 1, amd.JOIN_MFMA)
    assert err.value.code == binding.EINVAL


def test_static_scratch_arguments_are_checked_on_the_host():
    # no GPU needed: every call below fails before anything is launched
    import paper_2103_15386_amd as amd
    from paper_2103_15386_amd import binding
    lib = amd.load_library()
    header = open(os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))),
                               "include", "gnnd.h")).read()
    assert "#define GNND_STATIC_SCRATCH_BYTES ((size_t)64 << 20)" in header
    assert binding.STATIC_SCRATCH_BYTES == 64 << 20
    prm = binding.make_params(10 ** 6, 128, 32, 32, amd.L2SQ_F32)
    assert lib.gnnd_build_static(C.byref(prm), 0x1000, 3, 0x2000, 0x3000) == binding.ENOSPC
    assert b"static array holds" in lib.gnnd_last_error(None)
    prm = binding.make_params(1000, 16, 8, 8, amd.L2SQ_F32)
    assert lib.gnnd_build_static(C.byref(prm), 0x1000, -1, 0x2000, 0x3000) == binding.EINVAL
    assert lib.gnnd_build_static(C.byref(prm), 0x1000, 3, None, 0x3000) == binding.EINVAL
    prm = binding.make_params(1000, 16, 8, 9, amd.L2SQ_F32)
    assert lib.gnnd_build_static(C.byref(prm), 0x1000, 3, 0x2000, 0x3000) == binding.EINVAL
