"""The decode entry points under HIP graph capture: a launch-bound training loop can record one decode per batch and
replay it.  Captured here through torch's graph wrapper on a side stream; every replay is compared, bit for bit, with
the same call issued eagerly, with eager work and synchronisations between the replays and new ids in the captured
tensor each time.  Only calls that allocate nothing are captured (a caller's workspace, or the no-allocation entry)."""
import numpy as np
import pytest

from paper_2306_16699_amd import rinr, synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("case", ["uniform", "ragged-workspace", "ragged-noalloc"])
def test_decode_replays_from_a_graph(case):
    import torch
    assert torch.cuda.is_available()
    if case == "uniform":
        w = synth.workload(2, n_images=96, H=32, W=32)
    else:
        w = synth.workload(5, n_images=96, pool=200, H=20, W=33)
    n, H, W = len(w.image_ids), w.H, w.W
    st = rinr.Store(rinr.pack(w.models, w.w0, w.coord_lo, w.coord_hi))
    rng = np.random.default_rng(5)
    n_models = len(w.models)
    ids = torch.from_numpy(w.image_ids.copy()).cuda()
    out = torch.empty((n, 3, H, W), device="cuda")
    out8 = torch.empty((n, 3, H, W), dtype=torch.uint8, device="cuda")
    ws = torch.empty(rinr.workspace_bytes(n), dtype=torch.uint8, device="cuda") if case != "ragged-noalloc" else None
    kw = dict(out_dtype=rinr.OUT_F32_AND_U8, out=out, out_u8=out8, workspace=ws, noalloc=case == "ragged-noalloc")

    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        st.decode_batch_ex(ids, H, W, stream=side, **kw)          # first use outside the capture (one-time set-up of the library)
    side.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        st.decode_batch_ex(ids, H, W, stream=torch.cuda.current_stream(), **kw)
    for rep in range(4):
        new_ids = rng.integers(0, n_models, size=n).astype(np.int64)
        if rep == 2:
            new_ids[3] = -1                                        # an id out of range: zero-filled slot, counted
        ids.copy_(torch.from_numpy(new_ids).cuda())
        out.fill_(-5.0)
        out8.fill_(77)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got, got8 = out.clone(), out8.clone()
        want, want8 = st.decode_batch_ex(ids, H, W, out_dtype=rinr.OUT_F32_AND_U8, workspace=ws)
        torch.cuda.synchronize()
        assert torch.equal(got, want) and torch.equal(got8, want8), (case, rep)
        assert float(got.abs().max()) <= 1.0
    assert st.status() == 2                                        # the bad id: once replayed, once eager
    st.close()
