"""bpdq_channel_order_noalloc (the entry point for callers that cannot allocate: its scratch is a
device array built into the library) against bpdq_channel_order, bit for bit, on two calls in a
row, the second smaller than the first, through the C ABI."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2602_04163_amd import binding as bq

pytestmark = pytest.mark.gpu


def _diag_matrix(diag, dev):
    d = diag.numel()
    H = torch.zeros(d * d, device=dev)
    H[:: d + 1] = diag.to(dev)
    return H.view(d, d)


def test_no_alloc_channel_order_matches_workspace_version():
    assert torch.cuda.is_available(), "this test needs the MI355X"
    lib = bq.load()
    dev = torch.device("cuda:0")
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    g = torch.Generator().manual_seed(29)
    for d_in, gs in [(8192, 1), (3584, 128), (640, 1)]:          # big, then smaller ones
        print(f"no-alloc channel order d_in={d_in} group_size={gs}", flush=True)
        diag = (torch.rand(d_in, generator=g) * 10).round(decimals=1)       # plenty of ties
        H = _diag_matrix(diag, dev)
        want = bq.bpdq_channel_order(H, gs)
        perm = torch.full((d_in,), -1, dtype=torch.int32, device=dev)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        rc = lib.bpdq_channel_order_noalloc(ctypes.c_void_p(H.data_ptr()), d_in, gs,
                                            ctypes.c_void_p(perm.data_ptr()), stream)
        assert rc == 0
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(perm, want)
        assert np.array_equal(np.sort(perm.cpu().numpy()), np.arange(d_in))
    # beyond the built-in scratch: rejected, nothing launched
    rc = lib.bpdq_channel_order_noalloc(ctypes.c_void_p(H.data_ptr()), 32768 * 2 + 64, 1,
                                        ctypes.c_void_p(perm.data_ptr()), stream)
    assert rc == -2
    rc = lib.bpdq_channel_order_noalloc(ctypes.c_void_p(H.data_ptr()), 640, 3,
                                        ctypes.c_void_p(perm.data_ptr()), stream)
    assert rc == -3
