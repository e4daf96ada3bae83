"""blast_sparse_mlp_static (scratch in the library's own device array, nothing allocated) against
blast_sparse_mlp (scratch in a caller's workspace), through the raw C ABI."""
import ctypes as C

import numpy as np
import pytest

from oracle import oracle as orc
from paper_2507_03117_amd import api, synth
from tests.helpers import check_close, mask_dev, to_dev

pytestmark = pytest.mark.gpu


def _layer(seed, E, I, b, sparsity):
    rng = np.random.default_rng(seed)
    ws_ = [synth.gauss_bf16(rng, s, 0.05) for s in ((I, E), (I, E), (E, I))]
    ms_ = [synth.uniform_mask(rng, r // b, c // b, sparsity) for r, c in ((I, E), (I, E), (E, I))]
    dev = [api.bsr_pack(to_dev(w), b, mask=mask_dev(m)) for w, m in zip(ws_, ms_)]
    ref = [orc.pack(w, b, m) for w, m in zip(ws_, ms_)]
    return rng, dev, ref


def _both(L, dev, x_bits, T, E):
    """Y of the static entry point and of blast_sparse_mlp for the same inputs (fp32, token-major)."""
    import torch

    x = to_dev(x_bits)
    vg, vu, vd = (p.view() for p in dev)
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    y_static = torch.full((T, E), float("nan"), device="cuda:0")
    y_ws = torch.full((T, E), float("nan"), device="cuda:0")
    ws = torch.empty(max(api.mlp_workspace_bytes(*dev, T), 256), dtype=torch.uint8, device="cuda:0")
    rc = L.blast_sparse_mlp_static(C.byref(vg), C.byref(vu), C.byref(vd), C.c_void_p(x.data_ptr()), E, api.TOKEN_MAJOR,
                                   T, api.ACT["silu"], C.c_void_p(y_static.data_ptr()), E, api.F32, stream)
    assert rc == 0, L.blast_strerror(rc)
    rc = L.blast_sparse_mlp(C.byref(vg), C.byref(vu), C.byref(vd), C.c_void_p(x.data_ptr()), E, api.TOKEN_MAJOR, T,
                            api.ACT["silu"], C.c_void_p(y_ws.data_ptr()), E, api.F32, C.c_void_p(ws.data_ptr()),
                            ws.numel(), stream)
    assert rc == 0, L.blast_strerror(rc)
    torch.cuda.synchronize()
    return y_static.cpu().numpy(), y_ws.cpu().numpy()


@pytest.mark.parametrize("b,E,I,tokens", [(64, 256, 512, (300, 24)), (128, 512, 768, (16, 3)), (64, 256, 384, (29, 1))])
def test_static_scratch_matches_workspace_form_on_two_calls_in_a_row(b, E, I, tokens):
    """Two calls in a row, the second with fewer tokens (it finds the first call's H and slots in the array);
    each must equal blast_sparse_mlp on the same inputs and meet the oracle's bar."""
    L = api.lib()
    rng, dev, ref = _layer(9100 + b + E, E, I, b, 0.5)
    for T in tokens:
        x = synth.gauss_bf16(rng, (T, E), 1.0)
        y_static, y_ws = _both(L, dev, x, T, E)
        # the same kernels on the same inputs in a fixed summation order: identical bits
        assert np.array_equal(y_static.view(np.uint32), y_ws.view(np.uint32)), (b, T)
        check_close(y_static.T, orc.mlp(*ref, x), f"static scratch b={b} T={T}")


def test_static_scratch_rejects_sizes_beyond_its_limit():
    """No launch and a clear error when T * I * 2 bytes of H do not fit the array."""
    L = api.lib()
    limit = int(L.blast_sparse_mlp_static_limit())
    assert limit == 36 << 20
    _, dev, _ = _layer(9200, 256, 512, 64, 0.5)
    import torch

    I, E = 512, 256
    T = limit // (2 * I) + 1
    x = torch.zeros((T, E), dtype=torch.bfloat16, device="cuda:0")
    y = torch.full((T, E), 7.0, device="cuda:0")
    vg, vu, vd = (p.view() for p in dev)
    rc = L.blast_sparse_mlp_static(C.byref(vg), C.byref(vu), C.byref(vd), C.c_void_p(x.data_ptr()), E, api.TOKEN_MAJOR,
                                   T, api.ACT["silu"], C.c_void_p(y.data_ptr()), E, api.F32,
                                   C.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == -5 and b"workspace" in L.blast_strerror(rc).lower()
    torch.cuda.synchronize()
    assert bool((y == 7.0).all())  # nothing was enqueued
    # the largest T that fits still runs
    T_ok = 600
    x = torch.zeros((T_ok, E), dtype=torch.bfloat16, device="cuda:0")
    y = torch.full((T_ok, E), 7.0, device="cuda:0")
    rc = L.blast_sparse_mlp_static(C.byref(vg), C.byref(vu), C.byref(vd), C.c_void_p(x.data_ptr()), E, api.TOKEN_MAJOR,
                                   T_ok, api.ACT["silu"], C.c_void_p(y.data_ptr()), E, api.F32,
                                   C.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == 0
    torch.cuda.synchronize()
    assert not bool(y.any())  # X = 0 gives Y = 0
