"""ckpt_solve_batched_noalloc: the entry point for callers that cannot allocate (its workspace is
a static per-GPU array inside the library).  Through the C ABI, two calls in a row on the same
GPU, the second with a smaller input, each compared with ckpt_solve_batched bit for bit."""
import ctypes

import numpy as np
import pytest

from workloads import make_config, random_chain_batch




@pytest.mark.gpu
def test_noalloc_equals_the_workspace_entry_point_twice_in_a_row():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2302_02599_amd as amd
    lib = amd.load_library()
    from paper_2302_02599_amd.binding import _Chains
    first = make_config(2)                                                     # L = 48, M = 1024, B = 16
    second = random_chain_batch(21, 300, 3, 77, size_hi=9, overheads=True, own_wdelta=True)   # smaller, all arrays
    for batch in (first, second):
        print(f"case {batch.name}", flush=True)
        L, M, B = batch.L, batch.M, batch.B
        up = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()
        keep = [up(a) for a in (batch.uf, batch.ub, batch.wa, batch.wabar, batch.wdelta, batch.of, batch.ob)]
        ch = _Chains(*[None if t is None else t.data_ptr() for t in keep])
        n = amd.ckpt_table_elems(L, M, B)
        cost = torch.full((n,), -3, dtype=torch.int32, device="cuda")
        arg = torch.full((n,), 99, dtype=torch.uint8, device="cuda")
        ws = torch.empty(amd.ckpt_workspace_bytes(L, M, B), dtype=torch.uint8, device="cuda")
        want_cost, want_arg = torch.empty_like(cost), torch.empty_like(arg)
        stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        assert lib.ckpt_solve_batched(ctypes.byref(ch), L, M, B, stream, want_cost.data_ptr(), want_arg.data_ptr(),
                                      ws.data_ptr()) == 0
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        assert lib.ckpt_solve_batched_noalloc(ctypes.byref(ch), L, M, B, stream, cost.data_ptr(), arg.data_ptr()) == 0
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        pitch = amd.ckpt_row_pitch(M)
        view = lambda t: t.view(B, -1, pitch)[:, :, :M + 1]
        assert (view(cost) == view(want_cost)).all() and (view(arg) == view(want_arg)).all(), batch.name
        assert amd.ckpt_check_inputs(None, L, M, B).tolist() == [0] * B
        assert amd.ckpt_check_inputs(ws, L, M, B).tolist() == [0] * B


def test_noalloc_rejects_sizes_beyond_its_workspace():
    import paper_2302_02599_amd as amd
    lib = amd.load_library()
    from paper_2302_02599_amd.binding import _Chains
    ch = _Chains(256, 256, 256, 256, None, None, None)
    L, M, B = 200, 64, 40                                          # 3 L^2 B ints of thresholds: 19 MB
    assert amd.ckpt_workspace_bytes(L, M, B) > 16 << 20
    assert lib.ckpt_solve_batched_noalloc(ctypes.byref(ch), L, M, B, None, 256, 256) == -2
    assert lib.ckpt_solve_batched_noalloc(ctypes.byref(ch), 0, M, B, None, 256, 256) == -1
