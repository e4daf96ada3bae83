"""The single-launch MLP (one token tile): its in-kernel hand-over of H under graph replay, on a garbage
workspace, at the full size of the 1B-shaped layer with changing activations, and its failure handling
forced from the host (producers withhold the publication, consumers poll a few times and give up - every
kernel exits normally)."""
import ctypes as C

import numpy as np
import pytest

from oracle import oracle as orc
from paper_2507_03117_amd import synth
from tests.helpers import check_close, mask_dev, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def api():
    import torch

    assert torch.cuda.is_available()
    from paper_2507_03117_amd import api as _api

    _api.lib()
    return _api


def _layer(api, seed, E, I, b, sparsity):
    rng = np.random.default_rng(seed)
    ws_ = [synth.gauss_bf16(rng, s, 0.05) for s in ((I, E), (I, E), (E, I))]
    ms_ = [synth.uniform_mask(rng, r // b, c // b, sparsity) for r, c in ((I, E), (I, E), (E, I))]
    ms_[2][1, :] = 0  # an empty block row of the down projection: nothing to wait for, zeros
    dev = [api.bsr_pack(to_dev(w), b, mask=mask_dev(m)) for w, m in zip(ws_, ms_)]
    ref = [orc.pack(w, b, m) for w, m in zip(ws_, ms_)]
    return rng, dev, ref, ms_


@pytest.mark.parametrize("b,T", [(64, 1), (64, 16), (64, 32), (64, 50), (128, 5), (128, 16), (128, 30)])
def test_single_launch_form_replays_from_a_graph(api, b, T):
    """One token tile: the call is recorded as ONE kernel and every replay - with new activations, with eager
    calls on the same workspace between the replays - hands over its own H."""
    import torch

    E, I = 4 * b, 6 * b
    rng, dev, ref, _ = _layer(api, 8100 + b + T, E, I, b, 0.5)
    ws = torch.full((max(api.mlp_workspace_bytes(*dev, T), 256),), 0x5A, dtype=torch.uint8, device="cuda:0")  # garbage
    xs = to_dev(synth.gauss_bf16(rng, (T, E), 1.0))
    y = torch.empty((T, E), dtype=torch.float32, device="cuda:0")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        api.sparse_mlp(*dev, xs, out=y, ws=ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        api.sparse_mlp(*dev, xs, out=y, ws=ws)
        api.sparse_mlp(*dev, xs, out=y, ws=ws)  # two launches per replay: consecutive epochs inside one graph
    for rep in range(4):
        x = synth.gauss_bf16(rng, (T, E), 1.0)
        xs.copy_(to_dev(x))
        y.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        check_close(y.cpu().numpy().T, orc.mlp(*ref, x), f"replay {rep} b={b} T={T}")
        if rep % 2 == 0:  # an eager call in between, on the same workspace
            x2 = synth.gauss_bf16(rng, (T, E), 1.0)
            y2 = api.sparse_mlp(*dev, to_dev(x2), ws=ws)
            torch.cuda.synchronize()
            check_close(y2.cpu().numpy().T, orc.mlp(*ref, x2), f"eager between replays {rep}")
    assert api.sparse_mlp_status(dev[0], T, ws) == 0


def test_single_launch_form_at_the_1b_shape_with_changing_activations(api):
    """Full-size reuse: the 1B-shaped layer, one workspace, activations changing from call to call and the token
    count moving inside the tile: no call may see H lines or slots of an earlier one."""
    import torch

    wl = synth.WORKLOADS["llama1b_b64_s90"]
    inp = synth.make_mlp(wl)
    dev = [api.bsr_pack(to_dev(l.W), wl.b, mask=mask_dev(l.mask)) for l in (inp.gate, inp.up, inp.down)]
    ref = [orc.pack(l.W, wl.b, l.mask) for l in (inp.gate, inp.up, inp.down)]
    rng = np.random.default_rng(8200)
    Tmax = 64
    ws = torch.full((api.mlp_workspace_bytes(*dev, Tmax),), 0xC3, dtype=torch.uint8, device="cuda:0")
    for rep, T in enumerate((32, 1, 17, 64, 4, 32, 47, 16, 2)):
        x = synth.gauss_bf16(rng, (T, wl.hidden), 1.0)
        # the workspace layout depends on T: give each T the prefix it asks for, as a caller with one big buffer would
        y = api.sparse_mlp(*dev, to_dev(x), ws=ws[: api.mlp_workspace_bytes(*dev, T)],
                           out=torch.full((T, wl.hidden), float("nan"), device="cuda:0"))
        torch.cuda.synchronize()
        check_close(y.cpu().numpy().T, orc.mlp(*ref, x), f"1B single launch call {rep} T={T}")
        assert api.sparse_mlp_status(dev[0], T, ws[: api.mlp_workspace_bytes(*dev, T)]) == 0


@pytest.mark.parametrize("b,T", [(64, 3), (64, 40), (128, 16), (128, 24)])
def test_a_wait_that_expires_gives_nan_rows_and_a_status(api, b, T):
    """Forced from the host: the producers never publish, the consumers poll 20 times and give up.  Every
    workgroup exits normally; the rows of Y that depended on H are NaN, rows of empty block rows are zeros,
    the status word says 1 and is cleared by reading it; the next ordinary call on the same workspace is right."""
    import torch

    E, I = 4 * b, 6 * b
    rng, dev, ref, masks = _layer(api, 8300 + b, E, I, b, 0.5)
    L = api.lib()
    ws = torch.empty(max(api.mlp_workspace_bytes(*dev, T), 256), dtype=torch.uint8, device="cuda:0")
    x = synth.gauss_bf16(rng, (T, E), 1.0)
    xd = to_dev(x)
    y = torch.full((T, E), 7.0, device="cuda:0")
    vg, vu, vd = (p.view() for p in dev)
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    rc = L.blast_sparse_mlp_handover_test(C.byref(vg), C.byref(vu), C.byref(vd), C.c_void_p(xd.data_ptr()), E,
                                          api.TOKEN_MAJOR, T, api.ACT["silu"], C.c_void_p(y.data_ptr()), E, api.F32,
                                          C.c_void_p(ws.data_ptr()), ws.numel(), stream, 20, 1)
    assert rc == 0
    torch.cuda.synchronize()
    yh = y.cpu().numpy()
    has_blocks = masks[2].sum(axis=1) > 0  # per block row of the down projection
    for br in range(E // b):
        rows = yh[:, br * b:(br + 1) * b]
        if has_blocks[br]:
            assert np.isnan(rows).all(), f"block row {br}: waited-for rows must be NaN"
        else:
            assert not rows.any(), f"block row {br}: nothing to wait for, zeros"
    assert api.sparse_mlp_status(dev[0], T, ws) == 1
    assert api.sparse_mlp_status(dev[0], T, ws) == 0  # cleared by the read
    # argument check of the diagnostic call
    assert L.blast_sparse_mlp_handover_test(C.byref(vg), C.byref(vu), C.byref(vd), C.c_void_p(xd.data_ptr()), E,
                                            api.TOKEN_MAJOR, T, api.ACT["silu"], C.c_void_p(y.data_ptr()), E, api.F32,
                                            C.c_void_p(ws.data_ptr()), ws.numel(), stream, 0, 1) == -1
    # the workspace is fine afterwards
    y2 = api.sparse_mlp(*dev, xd, ws=ws)
    torch.cuda.synchronize()
    check_close(y2.cpu().numpy().T, orc.mlp(*ref, x), "after a timed-out launch")
    assert api.sparse_mlp_status(dev[0], T, ws) == 0
