"""The entry point that allocates nothing (gqsa_gemv_static) against gqsa_gemv, through the C ABI.

Collected last (the file name sorts after the other test files): it shares one static device
array between all its calls, so it also checks that what one call leaves there does not
disturb the next, smaller one.
"""
from __future__ import annotations

import ctypes as C

import numpy as np
import pytest

import gqsa_inputs as gi
import oracle
import paper_2412_17560_amd as gq
from paper_2412_17560_amd import binding

pytestmark = pytest.mark.gpu

TOL = 2e-3


def _packed(N, K, seed, part):
    W = gi.dense_weight(N, K, seed=seed)
    keep = gi.imbalanced_keep_counts(N, K // 16, seed=seed)
    h = gq.gqsa_pack_rows(W, keep, 16, 4)
    if part:
        gq.gqsa_set_partition(h, *part)          # rows shared by wavefronts of several workgroups
        assert gq.gqsa_info(h)["needs_fixup"] == 1
    else:
        assert gq.gqsa_info(h)["needs_fixup"] == 0      # (the default here: whole rows per worker, tiles of a chosen shape)
    return h, oracle.pack(W, 16, 4, keep_per_row=keep)


def test_static_workspace_entry_point_matches_gqsa_gemv_two_calls_in_a_row():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a HIP device")
    lib = binding._lib()
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    # first a larger matrix (chains over three and more workgroups, meeting points, LDS fix-ups),
    # then a smaller one with another partition: it uses the front of the same static array
    cases = [(_packed(1000, 5120, 21, (600, 1)), 5), (_packed(257, 2048, 22, (37, 3)), 1), (_packed(96, 1024, 23, None), 2)]
    for (h, c), batch in cases:
        info = gq.gqsa_info(h)
        x_np = gi.activations(batch, info["K"], seed=31 + batch)
        x = torch.from_numpy(x_np).cuda()
        want = torch.full((batch, info["N"]), float("nan"), dtype=torch.float16, device="cuda")
        got = torch.full((batch, info["N"]), float("nan"), dtype=torch.float16, device="cuda")
        # not uploaded yet: the entry point must refuse rather than allocate
        assert lib.gqsa_gemv_static(h.ptr, C.c_void_p(x.data_ptr()), C.c_void_p(got.data_ptr()), batch, stream) == 3
        gq.gqsa_upload(h)
        assert lib.gqsa_gemv(h.ptr, C.c_void_p(x.data_ptr()), C.c_void_p(want.data_ptr()), batch, stream) == 0
        torch.cuda.synchronize()
        for call in range(2):
            got.fill_(float("nan"))
            assert lib.gqsa_gemv_static(h.ptr, C.c_void_p(x.data_ptr()), C.c_void_p(got.data_ptr()), batch, stream) == 0
            torch.cuda.synchronize()
            assert np.array_equal(got.cpu().numpy().view(np.uint16), want.cpu().numpy().view(np.uint16)), (info["N"], call)
        ref = oracle.gemv(c, x_np)
        y = got.cpu().numpy()
        for b in range(batch):
            assert oracle.rel_error(y[b], ref[b]) <= TOL
        gq.gqsa_free(h)


def test_static_workspace_entry_point_refuses_partitions_beyond_its_array():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a HIP device")
    lib = binding._lib()
    W = gi.dense_weight(64, 256, seed=3)
    h = gq.gqsa_pack(W, 16, 4, 0.5)
    gq.gqsa_set_partition(h, 4096, 5)               # 20480 wavefront workers: more than the array holds
    gq.gqsa_upload(h)
    x = torch.zeros((1, 256), dtype=torch.float16, device="cuda")
    y = torch.zeros((1, 64), dtype=torch.float16, device="cuda")
    assert lib.gqsa_gemv_static(h.ptr, C.c_void_p(x.data_ptr()), C.c_void_p(y.data_ptr()), 1, None) == 7
    assert lib.gqsa_gemv(h.ptr, C.c_void_p(x.data_ptr()), C.c_void_p(y.data_ptr()), 1, None) == 0
    torch.cuda.synchronize()
