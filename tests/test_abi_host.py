"""Host-side checks that need no GPU: the C-ABI library loads, exports every symbol the
header declares, and validates arguments before touching the device."""
import ctypes
import os
import re

import pytest

import paper_2506_14435_amd as M

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(M.LIB_PATH):
        from paper_2506_14435_amd import build
        build.build()
    return M.load_library()


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "mote.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mote_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert set(names) == set(M.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_host_only_entry_points(lib):
    assert M.mote_version() >= 100
    assert M.mote_packed_bytes(11008, 2048) == 11008 * 2048 // 4
    assert M.mote_packed_bytes(0, 128) == 0
    assert lib.mote_status_string(0) == b"ok"
    assert lib.mote_status_string(3) == b"workspace too small"
    assert lib.mote_status_string(99) == b"unknown status"


def test_shape_validation_happens_on_the_host(lib):
    L = M.binding.MoteLayerStruct(2048, 11008, 11008, 16, 2, *([None] * 9))
    small = lib.mote_layer_workspace_bytes(ctypes.byref(L), 64)
    big = lib.mote_layer_workspace_bytes(ctypes.byref(L), 8192)
    assert 0 < small < big
    # R*F bf16 + R*F int8 + 4 planes of R*d int32 (tiles of a nearly empty last round are cut
    # into up to 4 K planes) + T*F bf16 + T*d fp32 + T*d int8 dominate
    T, k, d, F = 8192, 2, 2048, 11008
    floor = T * k * F * 3 + T * k * d * 4 * 4 + T * F * 2 + T * d * 7       # incl. LN(x^a) bf16 for the block entry point
    assert floor <= big <= floor * 1.01 + (1 << 20)
    L.d_model = 2000
    assert lib.mote_layer_workspace_bytes(ctypes.byref(L), 64) == 0
    L.d_model, L.top_k = 2048, 17
    assert lib.mote_layer_workspace_bytes(ctypes.byref(L), 64) == 0
    L.top_k, L.n_experts = 2, 65
    assert lib.mote_layer_workspace_bytes(ctypes.byref(L), 64) == 0
    # argument errors are reported before any launch (so these are safe without a GPU)
    assert lib.mote_pack_ternary(None, 0, 32, 128, None, None, None) == 1
    assert lib.mote_pack_ternary(ctypes.c_void_p(16), 0, 33, 128, ctypes.c_void_p(16), ctypes.c_void_p(16), None) == 2
    assert lib.mote_router_topk(None, None, None, 0, 256, 4, 2, None, None, None, None) == 0   # T == 0: no-op
    assert lib.mote_router_topk(None, None, None, 4, 200, 4, 2, None, None, None, None) == 2
    assert lib.mote_layer_forward(None, None, 4, None, None, 0, None, None) == 1
    assert lib.mote_stage_times(None) == 1


def test_workloads_are_seeded_and_shaped():
    import torch
    import workloads as W
    assert [c.name for c in (W.C1, W.C2, W.C3, W.C4, W.C5, W.P05, W.P15, W.P3)] == list(W.CONFIGS)
    assert all((c.n_experts, c.top_k, c.n_tokens) == (4, 1, 2048) for c in (W.P05, W.P15, W.P3))   # Section 4.1
    a, b = W.make_x(W.C1), W.make_x(W.C1)
    assert torch.equal(a, b) and a.dtype == torch.bfloat16 and a.shape == (64, 256)
    assert W.make_router(W.C2).shape == (896, 8)
    assert W.make_latent(W.C1, 1, 2).shape == (256, 512)
    assert not torch.equal(W.make_latent(W.C1, 0, 0), W.make_latent(W.C1, 0, 1))
    bias = W.make_router_bias(W.decode_config(16, 8))
    assert (bias == 30).sum() == 8 and bias.shape == (16,)
    z = W.make_router_bias(W.C5)
    assert z.max() == 0 and z.min() < -1.0
    x2 = W.make_x(W.C2).float()
    assert (x2.abs().amax(0) > 40).sum() == 4                       # the four outlier channels


def test_bench_refuses_more_than_one_gpu_and_names_every_workload():
    """`bench.py --gpus N` with N > 1 exits with a message before anything touches a GPU; the
    workload names of the benchmark definition and of the paper's own layer resolve to configs."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout == ""
    sys.path.insert(0, root)
    import bench
    import workloads as W
    assert bench.pick_config("c2") is W.C2 and bench.pick_config("p15") is W.P15
    dec = bench.pick_config("c4_T16_n8")
    assert (dec.n_tokens, dec.bias_subset, dec.d_model) == (16, 8, W.C4.d_model)
    work = bench.stage_work(W.C2, __import__("numpy").full(8, 512))
    # algorithmic work of the dominant kernel: 2 * R * 2 * d * F integer operations against the int8 MFMA peak
    bound, amount, unit, peak = work["routed_gate_up"]
    assert bound == "mfma" and peak == 5000.0 and amount == 2 * 4096 * 2 * 896 * 4864


@pytest.mark.parametrize("d,F,E,k,T_max", [(896, 4864, 8, 2, 300), (2048, 11008, 16, 2, 520),
                                            (1536, 8960, 4, 1, 2100), (256, 512, 4, 3, 700)])
def test_workspace_for_T_max_serves_every_smaller_batch(lib, d, F, E, k, T_max):
    """mote_layer_workspace_bytes(T) is what a forward of exactly T tokens needs at least, and the
    value for T_max must serve every T <= T_max although the number of K-split partial planes
    goes up when the batch gets smaller (the 0.5B shape needs more at T = 255 than at T = 256)."""
    L = M.binding.MoteLayerStruct(d, F, F, E, k, *([None] * 9))
    sizes = [lib.mote_layer_workspace_bytes(ctypes.byref(L), t) for t in range(1, T_max + 1)]
    assert all(s > 0 for s in sizes)
    assert all(a <= b for a, b in zip(sizes, sizes[1:]))      # a maximum over all smaller batches
    assert sizes[-1] == max(sizes)


def test_tuning_knobs_are_validated(lib):
    assert lib.mote_tuning_set(-1, 0) == 1
    assert lib.mote_tuning_set(len(M.KNOBS), 0) == 1
    assert lib.mote_tuning_set(M.KNOBS.index("group_m"), 2) == 0
    with pytest.raises(ValueError):
        M.mote_tuning_set("no_such_knob", 1)
    # the library's behaviour does not depend on the environment
    srcs = os.path.join(ROOT, "paper_2506_14435_amd", "csrc")
    for f in os.listdir(srcs):
        assert "getenv" not in open(os.path.join(srcs, f)).read(), f
