"""The entry point that allocates nothing (rinr_decode_batch_noalloc) against rinr_decode_batch_ex with a caller's
workspace, through the C ABI: two calls in a row on the same GPU, the second with a smaller input, bit for bit."""
import ctypes as C

import numpy as np
import pytest

from paper_2306_16699_amd import rinr, synth

pytestmark = pytest.mark.gpu


def test_noalloc_matches_workspace_decode_twice():
    import torch
    assert torch.cuda.is_available()
    L = rinr.lib()
    w = synth.workload(5, n_images=300, pool=500, H=24, W=37)               # mixed widths and depths: the slot order is used
    st = rinr.Store(rinr.pack(w.models, w.w0, w.coord_lo, w.coord_hi))
    ids_h = w.image_ids.copy()
    ids_h[[5, 250]] = [-3, 10 ** 9]                                          # out-of-range ids are ordered too
    stream = torch.cuda.current_stream().cuda_stream or None
    for n, H, W in ((300, 24, 37), (41, 17, 9)):                             # the second call is smaller: stale entries beyond n stay unread
        ids = torch.from_numpy(ids_h[:n].copy()).cuda()
        ws = torch.empty(rinr.workspace_bytes(n), dtype=torch.uint8, device="cuda")
        for flags in (0, rinr.FLAG_FP32_MFMA):
            want = torch.full((n, 3, H, W), -1.0, device="cuda")
            want8 = torch.full((n, 3, H, W), 9, dtype=torch.uint8, device="cuda")
            o = rinr.DecodeOpts(rinr.OUT_F32_AND_U8, flags, want8.data_ptr())
            o.workspace, o.workspace_bytes = ws.data_ptr(), ws.numel()
            assert L.rinr_decode_batch_ex(st._h, ids.data_ptr(), n, H, W, want.data_ptr(), C.byref(o), stream) == rinr.OK
            launches = st.last_launch_info()["launches"]                     # ordering kernel + one decode per width class (small images)
            assert launches >= 2
            got = torch.full((n, 3, H, W), -2.0, device="cuda")
            got8 = torch.full((n, 3, H, W), 7, dtype=torch.uint8, device="cuda")
            o = rinr.DecodeOpts(rinr.OUT_F32_AND_U8, flags, got8.data_ptr())    # no workspace
            before = torch.cuda.memory_allocated()
            assert L.rinr_decode_batch_noalloc(st._h, ids.data_ptr(), n, H, W, got.data_ptr(), C.byref(o), stream) == rinr.OK
            assert torch.cuda.memory_allocated() == before
            assert st.last_launch_info()["launches"] == launches
            torch.cuda.synchronize()
            assert torch.equal(got, want) and torch.equal(got8, want8), (n, flags)
    assert st.status() == 4 * 2 + 4 * 1                                      # four decodes per batch; two bad ids in the first batch, one in the second
    # limits and argument errors
    o = rinr.DecodeOpts(rinr.OUT_F32, 0, None)
    out = torch.empty((1, 3, 4, 4), device="cuda")
    ids = torch.zeros(1, dtype=torch.int64, device="cuda")
    assert L.rinr_decode_batch_noalloc(st._h, ids.data_ptr(), 65537, 1, 1, out.data_ptr(), C.byref(o), stream) == rinr.E_SIZE
    assert L.rinr_decode_batch_noalloc(None, ids.data_ptr(), 1, 4, 4, out.data_ptr(), C.byref(o), stream) == rinr.E_NULL
    assert L.rinr_decode_batch_noalloc(st._h, ids.data_ptr(), 1, 4, 4, out.data_ptr(), None, stream) == rinr.E_NULL
    assert L.rinr_decode_batch_noalloc(st._h, ids.data_ptr(), 0, 4, 4, out.data_ptr(), C.byref(o), stream) == rinr.OK
    st.close()
