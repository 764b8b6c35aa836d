"""mote_layer_forward_static (the entry point for callers that cannot allocate) against
mote_layer_forward, through the C ABI: same inputs, bit-identical outputs and taps, on two
calls in a row of which the second is smaller, so that whatever the first call left in the
library's static scratch array cannot leak into the second."""
import ctypes
import dataclasses

import numpy as np
import pytest
import torch

import workloads as W
from tests.mote_testlib import GpuProblem

pytestmark = pytest.mark.gpu

CASES = [
    (W.C1.with_tokens(300, name="c1_T300"), 33),                        # large-batch kernels, then decode kernels
    (W.decode_config(64, 16), 5),                                       # the serving shape: 3B width, 64 then 5 tokens
    (W.MoteConfig("ragged_mid", 384, 640, 8, 2, 211, seed=11, outlier_channels=2), 210),
    (dataclasses.replace(W.C1, name="c1_T1_first", n_tokens=40), 1),
]
TAPS = ("topk_idx", "topk_p", "counts", "row_of", "acc_gate", "h", "q_h", "beta_h", "acc_down", "h_s", "y_s", "out_f32")


def _raw_forward_static(M, layer, x, out, taps):
    """The C ABI itself, no binding helper in between."""
    lib = M.load_library()
    ts = M.binding.MoteTapsStruct(*[taps[n].data_ptr() if n in taps else None for n in M.TAP_FIELDS])
    return lib.mote_layer_forward_static(ctypes.byref(layer.struct), ctypes.c_void_p(x.data_ptr()), x.shape[0],
                                         ctypes.c_void_p(out.data_ptr()), ctypes.byref(ts),
                                         ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))


@pytest.mark.parametrize("cfg,t_second", CASES, ids=lambda c: getattr(c, "name", str(c)))
def test_static_entry_point_matches_forward_on_two_calls_in_a_row(cfg, t_second):
    import paper_2506_14435_amd as M
    print(f"no-alloc entry point: {cfg.name} T={cfg.n_tokens} then T={t_second}", flush=True)
    gp = GpuProblem(cfg)
    assert gp.layer.workspace_bytes(cfg.n_tokens) <= M.binding.STATIC_WORKSPACE_BYTES
    for T in (cfg.n_tokens, t_second):
        x = gp.x[:T].contiguous()
        want_taps = M.alloc_taps(gp.layer, T, TAPS)
        got_taps = M.alloc_taps(gp.layer, T, TAPS)
        for t in (*want_taps.values(), *got_taps.values()):
            t.zero_()
        want = M.mote_layer_forward(gp.layer, x, taps=want_taps)
        got = torch.zeros_like(x)
        assert _raw_forward_static(M, gp.layer, x, got, got_taps) == 0
        torch.cuda.synchronize()
        assert torch.equal(got, want), f"T={T}: outputs differ"
        for n in TAPS:
            assert torch.equal(got_taps[n], want_taps[n]), f"T={T}: tap {n} differs"
        # once more on the shared array: same answer, and the device's free memory does not move
        # (the HIP runtime materialises the library's static array when the library's device code is
        # first used on a GPU, which the call above has done; from then on a call allocates nothing)
        again = torch.zeros_like(x)
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]
        M.mote_layer_forward_static(gp.layer, x, again)
        torch.cuda.synchronize()
        assert free_before - torch.cuda.mem_get_info()[0] <= (2 << 20)
        assert torch.equal(again, want)


def test_static_entry_point_refuses_batches_beyond_its_array():
    import paper_2506_14435_amd as M
    lib = M.load_library()
    L = M.binding.MoteLayerStruct(896, 4864, 4864, 8, 2, *([ctypes.c_void_p(256)] * 1), None, *([ctypes.c_void_p(256)] * 7))
    assert lib.mote_layer_workspace_bytes(ctypes.byref(L), 2048) > M.binding.STATIC_WORKSPACE_BYTES
    # refused on the host, before any launch: the dummy pointers are never dereferenced
    assert lib.mote_layer_forward_static(ctypes.byref(L), ctypes.c_void_p(256), 2048, ctypes.c_void_p(256), None, None) == 3
    assert lib.mote_status_string(3) == b"workspace too small"
    assert lib.mote_layer_forward_static(None, None, 4, None, None, None) == 1
    assert lib.mote_layer_forward_static(ctypes.byref(L), None, 0, None, None, None) == 0      # T == 0: no-op
    L.d_model = 900
    assert lib.mote_layer_forward_static(ctypes.byref(L), ctypes.c_void_p(256), 4, ctypes.c_void_p(256), None, None) == 2
