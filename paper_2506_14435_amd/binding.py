"""Thin ctypes binding of libmote.so: argument marshalling only.

Every function mirrors one entry point of include/mote.h.  torch supplies device memory
and the current stream; all arithmetic runs in the HIP kernels of the library.  There is
no fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, c_char_p, c_float, c_int, c_int32, c_int64, c_size_t, c_void_p

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmote.so")

MOTE_DTYPE_F32, MOTE_DTYPE_BF16 = 0, 1
STAGE_NAMES = ("router_quant", "dispatch", "routed_gate_up", "quant_h", "routed_down",
               "shared_gate_up", "shared_down", "combine")
# every symbol include/mote.h declares
EXPORTS = ("mote_status_string", "mote_version", "mote_packed_bytes", "mote_pack_ternary",
           "mote_router_topk", "mote_layer_workspace_bytes", "mote_layer_forward", "mote_layer_forward_static",
           "mote_block_forward", "mote_router_balance", "mote_pack_binary", "mote_rtn_packed_bytes", "mote_pack_rtn",
           "mote_ste_backward_workspace_bytes", "mote_ste_linear_backward",
           "mote_stage_timing", "mote_stage_times", "mote_event_pair_overhead", "mote_tuning_set", "mote_calib_copy")
KNOBS = ("no_fork", "fork_min_log2", "event_fence", "quant_wide", "routed_variant", "routed_down_variant",
         "shared_variant", "group_m", "dynamic_rounds", "decode_variant", "router_token_blocks", "down_split_tiles",
         "mid_rows_lo", "mid_rows_hi", "ste_batch_mib")


class MoteError(RuntimeError):
    pass


class MoteLayerStruct(ctypes.Structure):
    _fields_ = [("d_model", c_int), ("d_ff_shared", c_int), ("d_ff_routed", c_int),
                ("n_experts", c_int), ("top_k", c_int),
                ("w_router", c_void_p), ("router_bias", c_void_p),
                ("ws_gate", c_void_p), ("ws_up", c_void_p), ("ws_down", c_void_p),
                ("wt_gate", c_void_p), ("wt_up", c_void_p), ("wt_down", c_void_p),
                ("alpha", c_void_p),
                ("shared_bits", c_int), ("ss_gate", c_void_p), ("ss_up", c_void_p), ("ss_down", c_void_p)]


class MoteNormStruct(ctypes.Structure):
    _fields_ = [("kind", c_int), ("gamma", c_void_p), ("beta", c_void_p), ("eps", ctypes.c_double)]


NORM_RMS, NORM_LAYER = 1, 2


TAP_FIELDS = ("topk_idx", "topk_p", "counts", "row_of", "tok_of", "q_x", "beta_x", "acc_gate",
              "acc_up", "h", "q_h", "beta_h", "acc_down", "h_s", "y_s", "out_f32", "xn")


class MoteTapsStruct(ctypes.Structure):
    _fields_ = [(name, c_void_p) for name in TAP_FIELDS]


_lib = None


def load_library() -> ctypes.CDLL:
    """Loads the in-tree libmote.so (build it first with paper_2506_14435_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise MoteError(f"{LIB_PATH} is missing: run `python -m paper_2506_14435_amd.build` "
                        "(there is no CPU fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    lib.mote_status_string.restype = c_char_p
    lib.mote_status_string.argtypes = [c_int]
    lib.mote_version.restype = c_int
    lib.mote_packed_bytes.restype = c_size_t
    lib.mote_packed_bytes.argtypes = [c_int64, c_int64]
    lib.mote_pack_ternary.restype = c_int
    lib.mote_pack_ternary.argtypes = [c_void_p, c_int, c_int64, c_int64, c_void_p, c_void_p, c_void_p]
    lib.mote_router_topk.restype = c_int
    lib.mote_router_topk.argtypes = [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int,
                                     c_void_p, c_void_p, c_void_p, c_void_p]
    lib.mote_layer_workspace_bytes.restype = c_size_t
    lib.mote_layer_workspace_bytes.argtypes = [POINTER(MoteLayerStruct), c_int]
    lib.mote_layer_forward.restype = c_int
    lib.mote_layer_forward.argtypes = [POINTER(MoteLayerStruct), c_void_p, c_int, c_void_p, c_void_p,
                                       c_size_t, POINTER(MoteTapsStruct), c_void_p]
    lib.mote_block_forward.restype = c_int
    lib.mote_block_forward.argtypes = [POINTER(MoteLayerStruct), POINTER(MoteNormStruct), c_void_p, c_int, c_void_p,
                                       c_void_p, c_size_t, POINTER(MoteTapsStruct), c_void_p]
    lib.mote_router_balance.restype = c_int
    lib.mote_router_balance.argtypes = [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int,
                                        c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.mote_pack_binary.restype = c_int
    lib.mote_pack_binary.argtypes = [c_void_p, c_int, c_int64, c_int64, c_void_p, c_void_p, c_void_p]
    lib.mote_rtn_packed_bytes.restype = c_size_t
    lib.mote_rtn_packed_bytes.argtypes = [c_int64, c_int64, c_int]
    lib.mote_pack_rtn.restype = c_int
    lib.mote_pack_rtn.argtypes = [c_void_p, c_int64, c_int64, c_int, c_void_p, c_void_p, c_void_p]
    lib.mote_layer_forward_static.restype = c_int
    lib.mote_layer_forward_static.argtypes = [POINTER(MoteLayerStruct), c_void_p, c_int, c_void_p,
                                              POINTER(MoteTapsStruct), c_void_p]
    lib.mote_ste_backward_workspace_bytes.restype = c_size_t
    lib.mote_ste_backward_workspace_bytes.argtypes = [c_int, c_int, c_int, c_int]
    lib.mote_ste_linear_backward.restype = c_int
    lib.mote_ste_linear_backward.argtypes = [c_void_p, POINTER(ctypes.c_int32), c_void_p, c_void_p, c_int, c_void_p,
                                             c_void_p, c_int, c_int, c_int, c_int, c_void_p, c_void_p, c_void_p,
                                             c_size_t, c_void_p]
    lib.mote_stage_timing.restype = c_int
    lib.mote_stage_timing.argtypes = [c_int]
    lib.mote_stage_times.restype = c_int
    lib.mote_stage_times.argtypes = [POINTER(c_float)]
    lib.mote_event_pair_overhead.restype = c_int
    lib.mote_event_pair_overhead.argtypes = [POINTER(c_float), c_void_p]
    lib.mote_tuning_set.restype = c_int
    lib.mote_tuning_set.argtypes = [c_int, c_int]
    lib.mote_calib_copy.restype = c_int
    lib.mote_calib_copy.argtypes = [c_void_p, c_void_p, c_size_t, c_void_p]
    _lib = lib
    return lib


def _check(status: int, what: str) -> None:
    if status != 0:
        msg = load_library().mote_status_string(status).decode()
        raise MoteError(f"{what}: {msg} (status {status})")


def _ptr(t):
    return None if t is None else c_void_p(t.data_ptr())


def _stream() -> c_void_p:
    return c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t: torch.Tensor, dtype, name: str) -> torch.Tensor:
    if not t.is_cuda:
        raise MoteError(f"{name} must be a device tensor")
    if t.dtype != dtype:
        raise MoteError(f"{name} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise MoteError(f"{name} must be contiguous")
    return t


def mote_version() -> int:
    return load_library().mote_version()


def mote_packed_bytes(n_out: int, n_in: int) -> int:
    return load_library().mote_packed_bytes(n_out, n_in)


def mote_pack_ternary(w: torch.Tensor, packed: torch.Tensor = None, alpha: torch.Tensor = None, binary: bool = False):
    """w [n_out, n_in] fp32 or bf16 device tensor -> (packed int32 [n_out*n_in/16], alpha fp32 [1]).
    binary=True calls mote_pack_binary (the 1-bit quantiser in the same 2-bit container)."""
    lib = load_library()
    if w.dtype == torch.float32:
        dt = MOTE_DTYPE_F32
    elif w.dtype == torch.bfloat16:
        dt = MOTE_DTYPE_BF16
    else:
        raise MoteError(f"latent weights must be fp32 or bf16, got {w.dtype}")
    _dev(w, w.dtype, "w")
    n_out, n_in = w.shape
    if packed is None:
        packed = torch.empty(max(n_out * n_in // 16, 1), dtype=torch.int32, device=w.device)
    if alpha is None:
        alpha = torch.empty(1, dtype=torch.float32, device=w.device)
    fn = lib.mote_pack_binary if binary else lib.mote_pack_ternary
    _check(fn(_ptr(w), dt, n_out, n_in, _ptr(packed), _ptr(alpha), _stream()),
           "mote_pack_binary" if binary else "mote_pack_ternary")
    return packed, alpha


def mote_rtn_packed_bytes(n_out: int, n_in: int, bits: int) -> int:
    return load_library().mote_rtn_packed_bytes(n_out, n_in, bits)


def mote_pack_rtn(w: torch.Tensor, bits: int):
    """w [n_out, n_in] bf16 device tensor -> (packed uint8 [n_out*n_in*bits/8], scales fp32 [n_out])."""
    lib = load_library()
    _dev(w, torch.bfloat16, "w")
    n_out, n_in = w.shape
    nbytes = lib.mote_rtn_packed_bytes(n_out, n_in, bits)
    if nbytes == 0:
        raise MoteError("mote_pack_rtn: bits must be 8 or 4")
    packed = torch.empty(nbytes, dtype=torch.uint8, device=w.device)
    scales = torch.empty(n_out, dtype=torch.float32, device=w.device)
    _check(lib.mote_pack_rtn(_ptr(w), n_out, n_in, bits, _ptr(packed), _ptr(scales), _stream()), "mote_pack_rtn")
    return packed, scales


def mote_router_balance(x: torch.Tensor, w_router: torch.Tensor, k: int, router_bias: torch.Tensor = None):
    """Router plus Eq.12: returns (topk_idx, topk_p, counts, gate_p [T,E], gate_p_sum [E], loss [1])."""
    lib = load_library()
    _dev(x, torch.bfloat16, "x")
    _dev(w_router, torch.bfloat16, "w_router")
    if router_bias is not None:
        _dev(router_bias, torch.float32, "router_bias")
    n_tok, d = x.shape
    n_exp = w_router.shape[1]
    dev = x.device
    idx = torch.empty(n_tok, k, dtype=torch.int32, device=dev)
    p = torch.empty(n_tok, k, dtype=torch.float32, device=dev)
    counts = torch.zeros(n_exp, dtype=torch.int32, device=dev)
    gate_p = torch.empty(n_tok, n_exp, dtype=torch.float32, device=dev)
    gate_sum = torch.empty(n_exp, dtype=torch.float32, device=dev)
    loss = torch.empty(1, dtype=torch.float32, device=dev)
    _check(lib.mote_router_balance(_ptr(x), _ptr(w_router), _ptr(router_bias), n_tok, d, n_exp, k, _ptr(idx), _ptr(p),
                                   _ptr(counts), _ptr(gate_p), _ptr(gate_sum), _ptr(loss), _stream()),
           "mote_router_balance")
    return idx, p, counts, gate_p, gate_sum, loss


def mote_ste_linear_backward(dy: torch.Tensor, offsets, packed: torch.Tensor, alpha: torch.Tensor, alpha_stride: int,
                             q: torch.Tensor, beta: torch.Tensor, n_out: int, n_in: int, workspace: torch.Tensor = None):
    """Straight-through gradients of a grouped ternary linear layer (Section 3.2).  dy bf16 [R, N] grouped
    by expert, offsets: host sequence of E + 1 row offsets, packed: E packed matrices [N, K], alpha fp32
    (expert e at alpha[e * alpha_stride]), q int8 [R, K], beta fp32 [R] -> (dx fp32 [R, K], dw fp32 [E, N, K])."""
    lib = load_library()
    _dev(dy, torch.bfloat16, "dy")
    _dev(q, torch.int8, "q")
    _dev(beta, torch.float32, "beta")
    _dev(alpha, torch.float32, "alpha")
    offs = (ctypes.c_int32 * len(offsets))(*[int(v) for v in offsets])
    n_exp = len(offsets) - 1
    n_rows = dy.shape[0]
    need = lib.mote_ste_backward_workspace_bytes(n_rows, n_out, n_in, n_exp)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dy.device)
    dx = torch.empty(n_rows, n_in, dtype=torch.float32, device=dy.device)
    dw = torch.empty(n_exp, n_out, n_in, dtype=torch.float32, device=dy.device)
    _check(lib.mote_ste_linear_backward(_ptr(dy), offs, _ptr(packed), _ptr(alpha), alpha_stride, _ptr(q), _ptr(beta),
                                        n_rows, n_out, n_in, n_exp, _ptr(dx), _ptr(dw), _ptr(workspace),
                                        ctypes.c_size_t(workspace.numel()), _stream()), "mote_ste_linear_backward")
    return dx, dw


def mote_router_topk(x: torch.Tensor, w_router: torch.Tensor, k: int, router_bias: torch.Tensor = None,
                     want_counts: bool = True):
    """x bf16 [T,d], w_router bf16 [d,E] -> (topk_idx int32 [T,k], topk_p fp32 [T,k], counts int32 [E])."""
    lib = load_library()
    _dev(x, torch.bfloat16, "x")
    _dev(w_router, torch.bfloat16, "w_router")
    if router_bias is not None:
        _dev(router_bias, torch.float32, "router_bias")
    n_tok, d = x.shape
    n_exp = w_router.shape[1]
    idx = torch.empty(n_tok, k, dtype=torch.int32, device=x.device)
    p = torch.empty(n_tok, k, dtype=torch.float32, device=x.device)
    counts = torch.zeros(n_exp, dtype=torch.int32, device=x.device) if want_counts else None
    _check(lib.mote_router_topk(_ptr(x), _ptr(w_router), _ptr(router_bias), n_tok, d, n_exp, k, _ptr(idx),
                                _ptr(p), _ptr(counts), _stream()), "mote_router_topk")
    return idx, p, counts


class MoteLayer:
    """Holds the device tensors of one layer and the C struct that points at them."""

    def __init__(self, w_router, ws_gate, ws_up, ws_down, wt_gate, wt_up, wt_down, alpha, top_k,
                 router_bias=None, shared_bits=0, shared_scales=None):
        """shared_bits 0: ws_* are bf16 matrices.  8 / 4: ws_* are the packed uint8 codes of
        mote_pack_rtn and shared_scales = (s_gate [F_s], s_up [F_s], s_down [d]) fp32."""
        sdt = torch.bfloat16 if shared_bits == 0 else torch.uint8
        self.tensors = dict(w_router=_dev(w_router, torch.bfloat16, "w_router"),
                            ws_gate=_dev(ws_gate, sdt, "ws_gate"),
                            ws_up=_dev(ws_up, sdt, "ws_up"),
                            ws_down=_dev(ws_down, sdt, "ws_down"),
                            wt_gate=_dev(wt_gate, torch.int32, "wt_gate"),
                            wt_up=_dev(wt_up, torch.int32, "wt_up"),
                            wt_down=_dev(wt_down, torch.int32, "wt_down"),
                            alpha=_dev(alpha, torch.float32, "alpha"))
        if router_bias is not None:
            self.tensors["router_bias"] = _dev(router_bias, torch.float32, "router_bias")
        d, n_exp = w_router.shape
        if shared_bits == 0:
            f_s = ws_gate.shape[0]
            ss = (None, None, None)
        else:
            ss = tuple(_dev(t, torch.float32, "shared_scales") for t in shared_scales)
            f_s = ss[0].numel()
            if ws_gate.numel() != f_s * d * shared_bits // 8 or ss[2].numel() != d:
                raise MoteError("packed shared expert and its scales disagree in size")
            self.tensors.update(ss_gate=ss[0], ss_up=ss[1], ss_down=ss[2])
        f_r = wt_gate.numel() * 16 // (n_exp * d)
        self.d_model, self.d_ff_shared, self.d_ff_routed, self.n_experts, self.top_k = d, f_s, f_r, n_exp, top_k
        if tuple(alpha.shape) != (n_exp, 3):
            raise MoteError("alpha must be [E, 3]")
        if wt_gate.numel() != wt_up.numel() or wt_gate.numel() != wt_down.numel():
            raise MoteError("packed expert tensors disagree in size")
        self.struct = MoteLayerStruct(d, f_s, f_r, n_exp, top_k,
                                      w_router.data_ptr(),
                                      router_bias.data_ptr() if router_bias is not None else None,
                                      ws_gate.data_ptr(), ws_up.data_ptr(), ws_down.data_ptr(),
                                      wt_gate.data_ptr(), wt_up.data_ptr(), wt_down.data_ptr(),
                                      alpha.data_ptr(), shared_bits,
                                      *[t.data_ptr() if t is not None else None for t in ss])
        self._workspace = None

    def workspace_bytes(self, n_tokens: int) -> int:
        n = load_library().mote_layer_workspace_bytes(ctypes.byref(self.struct), n_tokens)
        if n == 0:
            raise MoteError("mote_layer_workspace_bytes: unsupported shape")
        return n

    def workspace(self, n_tokens: int) -> torch.Tensor:
        need = self.workspace_bytes(n_tokens)
        if self._workspace is None or self._workspace.numel() < need:
            self._workspace = torch.empty(need, dtype=torch.uint8, device=self.tensors["w_router"].device)
        return self._workspace


def alloc_taps(layer: MoteLayer, n_tokens: int, names=TAP_FIELDS):
    """Device tensors for the requested debug taps of mote_layer_forward."""
    dev = layer.tensors["w_router"].device
    k, d, fr, fs, e = layer.top_k, layer.d_model, layer.d_ff_routed, layer.d_ff_shared, layer.n_experts
    r = n_tokens * k
    spec = dict(topk_idx=((n_tokens, k), torch.int32), topk_p=((n_tokens, k), torch.float32),
                counts=((e,), torch.int32), row_of=((n_tokens, k), torch.int32), tok_of=((r,), torch.int32),
                q_x=((n_tokens, d), torch.int8), beta_x=((n_tokens,), torch.float32),
                acc_gate=((r, fr), torch.int32), acc_up=((r, fr), torch.int32), h=((r, fr), torch.bfloat16),
                q_h=((r, fr), torch.int8), beta_h=((r,), torch.float32), acc_down=((r, d), torch.int32),
                h_s=((n_tokens, fs), torch.bfloat16), y_s=((n_tokens, d), torch.float32),
                out_f32=((n_tokens, d), torch.float32), xn=((n_tokens, d), torch.bfloat16))
    return {n: torch.empty(spec[n][0], dtype=spec[n][1], device=dev) for n in names}


def mote_layer_forward(layer: MoteLayer, x: torch.Tensor, out: torch.Tensor = None, taps: dict = None,
                       workspace: torch.Tensor = None) -> torch.Tensor:
    """out = FFN(x) + MoE(x) for x bf16 [T, d]; returns out bf16 [T, d]."""
    lib = load_library()
    _dev(x, torch.bfloat16, "x")
    n_tok = x.shape[0]
    if x.shape[1] != layer.d_model:
        raise MoteError("x has the wrong width")
    if out is None:
        out = torch.empty_like(x)
    _dev(out, torch.bfloat16, "out")
    if workspace is None:
        workspace = layer.workspace(max(n_tok, 1))
    ts = None
    if taps is not None:
        ts = MoteTapsStruct(*[taps[n].data_ptr() if n in taps else None for n in TAP_FIELDS])
    _check(lib.mote_layer_forward(ctypes.byref(layer.struct), _ptr(x), n_tok, _ptr(out), _ptr(workspace),
                                  workspace.numel(), ctypes.byref(ts) if ts is not None else None, _stream()),
           "mote_layer_forward")
    return out


def mote_block_forward(layer: MoteLayer, x_a: torch.Tensor, gamma: torch.Tensor, beta: torch.Tensor = None,
                       eps: float = 1e-6, out: torch.Tensor = None, taps: dict = None,
                       workspace: torch.Tensor = None) -> torch.Tensor:
    """out = x_a + MoE(LN(x_a)) + FFN(LN(x_a)) (Eq.2); RMSNorm when beta is None, else layer normalisation."""
    lib = load_library()
    _dev(x_a, torch.bfloat16, "x_a")
    _dev(gamma, torch.bfloat16, "gamma")
    if beta is not None:
        _dev(beta, torch.bfloat16, "beta")
    n_tok = x_a.shape[0]
    if x_a.shape[1] != layer.d_model or gamma.numel() != layer.d_model:
        raise MoteError("x_a / gamma have the wrong width")
    if out is None:
        out = torch.empty_like(x_a)
    if workspace is None:
        workspace = layer.workspace(max(n_tok, 1))
    norm = MoteNormStruct(NORM_RMS if beta is None else NORM_LAYER, gamma.data_ptr(),
                          beta.data_ptr() if beta is not None else None, float(eps))
    ts = None
    if taps is not None:
        ts = MoteTapsStruct(*[taps[n].data_ptr() if n in taps else None for n in TAP_FIELDS])
    _check(lib.mote_block_forward(ctypes.byref(layer.struct), ctypes.byref(norm), _ptr(x_a), n_tok, _ptr(out),
                                  _ptr(workspace), workspace.numel(), ctypes.byref(ts) if ts is not None else None,
                                  _stream()), "mote_block_forward")
    return out


STATIC_WORKSPACE_BYTES = 64 << 20


def mote_layer_forward_static(layer: MoteLayer, x: torch.Tensor, out: torch.Tensor, taps: dict = None) -> torch.Tensor:
    """mote_layer_forward on the library's static scratch array: allocates nothing, so `out` is
    required; batches whose layout exceeds STATIC_WORKSPACE_BYTES raise."""
    lib = load_library()
    _dev(x, torch.bfloat16, "x")
    _dev(out, torch.bfloat16, "out")
    if x.shape[1] != layer.d_model or out.shape != x.shape:
        raise MoteError("x / out have the wrong shape")
    ts = None
    if taps is not None:
        ts = MoteTapsStruct(*[taps[n].data_ptr() if n in taps else None for n in TAP_FIELDS])
    _check(lib.mote_layer_forward_static(ctypes.byref(layer.struct), _ptr(x), x.shape[0], _ptr(out),
                                         ctypes.byref(ts) if ts is not None else None, _stream()),
           "mote_layer_forward_static")
    return out


class ForwardGraph:
    """One mote_layer_forward call (fixed layer, x, out and workspace buffers) captured into a HIP
    graph: replay() re-runs the same kernels with one launch instead of eight plus the fork/join
    events.  The buffers must stay alive and keep their addresses; x may be refilled in place."""

    def __init__(self, layer: MoteLayer, x: torch.Tensor, out: torch.Tensor, workspace: torch.Tensor):
        self.layer, self.x, self.out, self.workspace = layer, x, out, workspace
        # one eager call first: everything the library sets up lazily (helper stream, kernel
        # attributes) must exist before the capture starts
        mote_layer_forward(layer, x, out=out, workspace=workspace)
        torch.cuda.synchronize()
        self.graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self.graph):
            mote_layer_forward(layer, x, out=out, workspace=workspace)

    def replay(self) -> torch.Tensor:
        self.graph.replay()
        return self.out


def mote_stage_timing(enable: bool) -> None:
    _check(load_library().mote_stage_timing(1 if enable else 0), "mote_stage_timing")


def mote_stage_times() -> dict:
    buf = (c_float * len(STAGE_NAMES))()
    _check(load_library().mote_stage_times(buf), "mote_stage_times")
    return {n: float(buf[i]) for i, n in enumerate(STAGE_NAMES)}


def mote_event_pair_overhead() -> float:
    """Milliseconds two back-to-back event records on the current stream read with no kernel between them."""
    v = c_float()
    _check(load_library().mote_event_pair_overhead(ctypes.byref(v), _stream()), "mote_event_pair_overhead")
    return float(v.value)


def mote_tuning_set(knob, value: int) -> None:
    """knob: a name from KNOBS or its number."""
    kid = KNOBS.index(knob) if isinstance(knob, str) else int(knob)
    _check(load_library().mote_tuning_set(kid, int(value)), "mote_tuning_set")


def mote_calib_copy(dst: torch.Tensor, src: torch.Tensor) -> None:
    n = src.numel() * src.element_size()
    _check(load_library().mote_calib_copy(_ptr(dst), _ptr(src), n, _stream()), "mote_calib_copy")
