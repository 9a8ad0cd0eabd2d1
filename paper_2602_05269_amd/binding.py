"""ctypes binding of libhgf.so: the same entry points as include/hgf.h, taking torch
tensors.  Argument marshalling only -- every step of the layer runs in the HIP kernels;
torch provides device memory and the stream.  There is no fallback: a missing library
is an error."""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhgf.so")

HGF_OK = 0
STATUS_NAMES = {0: "HGF_OK", 1: "HGF_ERR_NULL", 2: "HGF_ERR_SHAPE", 3: "HGF_ERR_ALIGN",
                4: "HGF_ERR_UNSUPPORTED", 5: "HGF_ERR_WORKSPACE", 6: "HGF_ERR_DEVICE"}


class HgfError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {lib().hgf_status_string(status).decode()} (status {status})")


class hgf_layer(ctypes.Structure):
    _fields_ = [("d_in", ctypes.c_int), ("d_out", ctypes.c_int), ("rank", ctypes.c_int),
                ("W_packed", ctypes.c_void_p), ("s_w", ctypes.c_void_p),
                ("A_f16", ctypes.c_void_p), ("B_f16", ctypes.c_void_p), ("alpha_f16", ctypes.c_void_p),
                ("src_slot", ctypes.c_int), ("dst_slot", ctypes.c_int),
                ("ln_gamma", ctypes.c_void_p), ("ln_beta", ctypes.c_void_p), ("ln_eps", ctypes.c_float)]


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library.  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2602_05269_amd.build` "
                           "(there is no CPU or PyTorch fallback)")
    L = ctypes.CDLL(LIB_PATH)
    vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    L.hgf_status_string.restype = ctypes.c_char_p
    L.hgf_status_string.argtypes = [ci]
    L.hgf_version.restype = ci
    L.hgf_padded_k.restype = ci
    L.hgf_padded_k.argtypes = [ci]
    L.hgf_packed_weight_bytes.restype = sz
    L.hgf_packed_weight_bytes.argtypes = [ci, ci]
    L.hgf_workspace_bytes.restype = sz
    L.hgf_workspace_bytes.argtypes = [ci, ci, ci, ci]
    L.hgf_workspace_init.restype = ci
    L.hgf_workspace_init.argtypes = [vp, sz, vp]
    L.hgf_quantize_pack_weights.restype = ci
    L.hgf_quantize_pack_weights.argtypes = [vp, ci, ci, vp, vp, vp, sz, vp]
    L.hgf_unpack_weights.restype = ci
    L.hgf_unpack_weights.argtypes = [vp, ci, ci, vp, vp]
    L.hgf_quantize_activations.restype = ci
    L.hgf_quantize_activations.argtypes = [vp, ci, ci, vp, vp, vp, vp]
    L.hgf_layernorm_quantize_activations.restype = ci
    L.hgf_layernorm_quantize_activations.argtypes = [vp, ci, ci, vp, vp, ctypes.c_float, vp, vp, vp, vp]
    L.hgf_linear_forward.restype = ci
    L.hgf_linear_forward.argtypes = [vp, ci, ctypes.POINTER(hgf_layer), vp, vp, vp, sz, vp]
    L.hgf_static_scratch_bytes.restype = sz
    L.hgf_static_scratch_bytes.argtypes = []
    L.hgf_static_scratch_needed.restype = sz
    L.hgf_static_scratch_needed.argtypes = [ci, ci, ci, ci]
    L.hgf_linear_forward_static.restype = ci
    L.hgf_linear_forward_static.argtypes = [vp, ci, ctypes.POINTER(hgf_layer), vp, vp, vp]
    L.hgf_diff_attention_workspace_bytes.restype = sz
    L.hgf_diff_attention_workspace_bytes.argtypes = [ci, ci, ci, ci]
    L.hgf_diff_attention_decode.restype = ci
    L.hgf_diff_attention_decode.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ctypes.c_float, vp, vp, sz, vp]
    L.hgf_packed_weight_bytes_b3.restype = sz
    L.hgf_packed_weight_bytes_b3.argtypes = [ci, ci]
    L.hgf_quantize_pack_weights_b3.restype = ci
    L.hgf_quantize_pack_weights_b3.argtypes = [vp, ci, ci, vp, vp, vp, sz, vp]
    L.hgf_unpack_weights_b3.restype = ci
    L.hgf_unpack_weights_b3.argtypes = [vp, ci, ci, vp, vp]
    L.hgf_linear_forward_b3.restype = ci
    L.hgf_linear_forward_b3.argtypes = [vp, ci, ctypes.POINTER(hgf_layer), vp, vp, vp, sz, vp]
    L.hgf_swiglu_forward.restype = ci
    L.hgf_swiglu_forward.argtypes = [vp, ci, ctypes.POINTER(hgf_layer), ctypes.POINTER(hgf_layer), vp, vp, vp, vp, vp, sz, vp]
    L.hgf_stack_forward.restype = ci
    L.hgf_stack_forward.argtypes = [ctypes.POINTER(hgf_layer), ci, ctypes.POINTER(vp), ci, ci, vp, sz, vp]
    L.hgf_set_single_launch.restype = None
    L.hgf_set_single_launch.argtypes = [ci]
    L.hgf_set_wait_limit.restype = None
    L.hgf_set_wait_limit.argtypes = [ci]
    L.hgf_set_stack_trace.restype = None
    L.hgf_set_stack_trace.argtypes = [vp, sz, ci]
    L.hgf_profile_enable.restype = None
    L.hgf_profile_enable.argtypes = [ci]
    L.hgf_profile_collect.restype = ci
    L.hgf_profile_collect.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_longlong)]
    L.hgf_probe_mfma_rate.restype = ci
    L.hgf_probe_mfma_rate.argtypes = [ci, ci, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double), vp]
    _lib = L
    return L


def _check(status: int, where: str) -> None:
    if status != HGF_OK:
        raise HgfError(status, where)


def _stream(stream: Optional[torch.cuda.Stream] = None) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _dev(t: torch.Tensor, dtype: torch.dtype, name: str) -> torch.Tensor:
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous {dtype} tensor in device memory")
    return t


# --------------------------------------------------------------------------- sizes

def hgf_version() -> int:
    return lib().hgf_version()


def hgf_padded_k(d_in: int) -> int:
    return lib().hgf_padded_k(d_in)


def hgf_packed_weight_bytes(d_out: int, d_in: int) -> int:
    return lib().hgf_packed_weight_bytes(d_out, d_in)


def hgf_workspace_bytes(M_max: int, d_in_max: int, d_out_max: int, rank_max: int) -> int:
    return lib().hgf_workspace_bytes(M_max, d_in_max, d_out_max, rank_max)


class Workspace:
    """A device buffer of hgf_workspace_bytes, cleared by hgf_workspace_init."""

    def __init__(self, M_max: int, d_in_max: int, d_out_max: int, rank_max: int, device="cuda"):
        n = hgf_workspace_bytes(M_max, d_in_max, d_out_max, rank_max)
        if n == 0:
            raise ValueError("invalid workspace dimensions")
        self.buf = torch.empty(n, dtype=torch.uint8, device=device)
        self.bytes = n
        hgf_workspace_init(self)


def hgf_workspace_init(ws: Workspace, stream=None) -> None:
    _check(lib().hgf_workspace_init(ws.buf.data_ptr(), ws.bytes, _stream(stream)), "hgf_workspace_init")


def hgf_set_single_launch(level) -> None:
    """0: two launches per group; 1 (or True): one persistent launch per group; 2: per stack."""
    lib().hgf_set_single_launch(int(level))


def hgf_set_wait_limit(tries: int) -> None:
    """Test hook: every wait between workgroups of the whole-stack launch gives up after `tries`
    tries (0: the default bound of about a second)."""
    lib().hgf_set_wait_limit(int(tries))


TRACE_ROLES, TRACE_PHASES, TRACE_IDS = 11, 4, 8


def hgf_set_stack_trace(buf: Optional[torch.Tensor], first_phase: int = 0) -> None:
    """Time stamps of the whole-stack launch into `buf` (int64 [256, 11, 4, 8] on the device); None: off."""
    if buf is None:
        lib().hgf_set_stack_trace(None, 0, 0)
    else:
        lib().hgf_set_stack_trace(buf.data_ptr(), buf.numel() * buf.element_size(), int(first_phase))


def hgf_profile_enable(on: bool) -> None:
    lib().hgf_profile_enable(1 if on else 0)


def hgf_profile_collect():
    """((decode_ms, decode_launches), (prefill_ms, prefill_launches)) since the last collect."""
    ms = (ctypes.c_double * 2)()
    n = (ctypes.c_longlong * 2)()
    _check(lib().hgf_profile_collect(ms, n), "hgf_profile_collect")
    return (ms[0], n[0]), (ms[1], n[1])


def hgf_probe_mfma_rate(operand_kind: int, iters: int = 800, stream=None) -> Tuple[float, float]:
    """(int8 TOPS, shader clock in GHz) of a loop of nothing but the prefill kernel's MFMA, for
    operand values of kind 0 = constant, 1 = codes 0..2 against random int8, 2 = random int8."""
    tops, ghz = ctypes.c_double(0.0), ctypes.c_double(0.0)
    _check(lib().hgf_probe_mfma_rate(int(operand_kind), int(iters), ctypes.byref(tops), ctypes.byref(ghz),
                                     _stream(stream)), "hgf_probe_mfma_rate")
    return tops.value, ghz.value


# --------------------------------------------------------------------------- steps

def hgf_quantize_pack_weights(W: torch.Tensor, ws: Workspace, stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    """fp32 [d_out, d_in] -> (packed uint8 buffer, s_w fp32 scalar tensor)."""
    _dev(W, torch.float32, "W")
    d_out, d_in = W.shape
    packed = torch.empty(hgf_packed_weight_bytes(d_out, d_in), dtype=torch.uint8, device=W.device)
    s_w = torch.empty(1, dtype=torch.float32, device=W.device)
    _check(lib().hgf_quantize_pack_weights(W.data_ptr(), d_out, d_in, packed.data_ptr(), s_w.data_ptr(),
                                           ws.buf.data_ptr(), ws.bytes, _stream(stream)),
           "hgf_quantize_pack_weights")
    return packed, s_w


def hgf_unpack_weights(packed: torch.Tensor, d_out: int, d_in: int, stream=None) -> torch.Tensor:
    T = torch.empty((d_out, d_in), dtype=torch.int8, device=packed.device)
    _check(lib().hgf_unpack_weights(packed.data_ptr(), d_out, d_in, T.data_ptr(), _stream(stream)),
           "hgf_unpack_weights")
    return T


def hgf_quantize_activations(x: torch.Tensor, stream=None) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """fp16 [M, d_in] -> (x_q int8 [M, padded_k], s_x fp32 [M], rowsum int32 [M])."""
    _dev(x, torch.float16, "x")
    M, d_in = x.shape
    xq = torch.empty((M, hgf_padded_k(d_in)), dtype=torch.int8, device=x.device)
    s_x = torch.empty(M, dtype=torch.float32, device=x.device)
    rowsum = torch.empty(M, dtype=torch.int32, device=x.device)
    _check(lib().hgf_quantize_activations(x.data_ptr(), M, d_in, xq.data_ptr(), s_x.data_ptr(),
                                          rowsum.data_ptr(), _stream(stream)), "hgf_quantize_activations")
    return xq, s_x, rowsum


def hgf_layernorm_quantize_activations(x: torch.Tensor, gamma: torch.Tensor, beta: Optional[torch.Tensor],
                                       eps: float = 1e-5, stream=None):
    """fp16 [M, d_in] -> (x_q, s_x, rowsum) of layernorm(x) (fp32 gamma, beta [d_in]), fused."""
    _dev(x, torch.float16, "x")
    _dev(gamma, torch.float32, "gamma")
    M, d_in = x.shape
    xq = torch.empty((M, hgf_padded_k(d_in)), dtype=torch.int8, device=x.device)
    s_x = torch.empty(M, dtype=torch.float32, device=x.device)
    rowsum = torch.empty(M, dtype=torch.int32, device=x.device)
    _check(lib().hgf_layernorm_quantize_activations(x.data_ptr(), M, d_in, gamma.data_ptr(), _ptr(beta), float(eps),
                                                    xq.data_ptr(), s_x.data_ptr(), rowsum.data_ptr(), _stream(stream)),
           "hgf_layernorm_quantize_activations")
    return xq, s_x, rowsum


class Layer:
    """Device tensors of one HGF linear plus the hgf_layer record that points at them."""

    def __init__(self, packed: torch.Tensor, s_w: torch.Tensor, d_out: int, d_in: int,
                 A: Optional[torch.Tensor] = None, B: Optional[torch.Tensor] = None,
                 alpha: Optional[torch.Tensor] = None, src_slot: int = 0, dst_slot: int = 1,
                 ln_gamma: Optional[torch.Tensor] = None, ln_beta: Optional[torch.Tensor] = None,
                 ln_eps: float = 1e-5):
        self.packed, self.s_w, self.A, self.B, self.alpha = packed, s_w, A, B, alpha
        self.ln_gamma, self.ln_beta = ln_gamma, ln_beta
        for t, name in ((ln_gamma, "ln_gamma"), (ln_beta, "ln_beta")):
            if t is not None:
                _dev(t, torch.float32, name)
                if tuple(t.shape) != (d_in,):
                    raise ValueError(f"{name} must be [d_in]")
        rank = 0 if A is None else A.shape[0]
        if rank:
            _dev(A, torch.float16, "A"), _dev(B, torch.float16, "B"), _dev(alpha, torch.float16, "alpha")
            if tuple(A.shape) != (rank, d_in) or tuple(B.shape) != (d_out, rank) or tuple(alpha.shape) != (d_out,):
                raise ValueError("A must be [rank, d_in], B [d_out, rank], alpha [d_out]")
        if packed.numel() not in (hgf_packed_weight_bytes(d_out, d_in), hgf_packed_weight_bytes_b3(d_out, d_in)):
            raise ValueError("packed buffer has the wrong size for these dimensions")
        self.d_in, self.d_out, self.rank = d_in, d_out, rank
        self.c = hgf_layer(d_in, d_out, rank, packed.data_ptr(), s_w.data_ptr(), _ptr(A), _ptr(B), _ptr(alpha),
                           src_slot, dst_slot, _ptr(ln_gamma), _ptr(ln_beta), float(ln_eps))

    @classmethod
    def from_latent(cls, W: torch.Tensor, A, B, alpha, ws: Workspace, **kw) -> "Layer":
        packed, s_w = hgf_quantize_pack_weights(W, ws)
        return cls(packed, s_w, W.shape[0], W.shape[1], A, B, alpha, **kw)


def hgf_linear_forward(x: torch.Tensor, layer: Layer, ws: Workspace, y: Optional[torch.Tensor] = None,
                       acc_debug: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """One HGF linear: fp16 [M, d_in] -> fp16 [M, d_out] (written into `y` when given)."""
    _dev(x, torch.float16, "x")
    M, d_in = x.shape
    if d_in != layer.d_in:
        raise ValueError("x has the wrong d_in")
    if y is None:
        y = torch.empty((M, layer.d_out), dtype=torch.float16, device=x.device)
    _check(lib().hgf_linear_forward(x.data_ptr(), M, ctypes.byref(layer.c), y.data_ptr(), _ptr(acc_debug),
                                    ws.buf.data_ptr(), ws.bytes, _stream(stream)), "hgf_linear_forward")
    return y


def hgf_swiglu_forward(x: torch.Tensor, gate: Layer, up: Layer, ws: Workspace, z: Optional[torch.Tensor] = None,
                       amax: Optional[torch.Tensor] = None, acc_debug_gate: Optional[torch.Tensor] = None,
                       acc_debug_up: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """z = SiLU(gate(x)) * up(x) for two HGF linears of one shape, fp16 [M, d_out]."""
    _dev(x, torch.float16, "x")
    M, d_in = x.shape
    if d_in != gate.d_in or d_in != up.d_in or gate.d_out != up.d_out:
        raise ValueError("gate and up must share d_in and d_out with x")
    if z is None:
        z = torch.empty((M, up.d_out), dtype=torch.float16, device=x.device)
    if amax is not None:
        _dev(amax, torch.float32, "amax")
    _check(lib().hgf_swiglu_forward(x.data_ptr(), M, ctypes.byref(gate.c), ctypes.byref(up.c), z.data_ptr(),
                                    _ptr(amax), _ptr(acc_debug_gate), _ptr(acc_debug_up), ws.buf.data_ptr(),
                                    ws.bytes, _stream(stream)), "hgf_swiglu_forward")
    return z


def hgf_diff_attention_decode(q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor, lens: torch.Tensor,
                              lam: float, out: Optional[torch.Tensor] = None,
                              workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """One decode step of differential attention: q fp16 [B, 2H, d_h], k_cache [B, L, 2H, d_h],
    v_cache [B, L, H, d_h], lens int32 [B] -> fp16 [B, H, d_h]."""
    for t, n in ((q, "q"), (k_cache, "k_cache"), (v_cache, "v_cache")):
        _dev(t, torch.float16, n)
    _dev(lens, torch.int32, "lens")
    B, L, H2, d_h = k_cache.shape
    H = H2 // 2
    if tuple(q.shape) != (B, H2, d_h) or tuple(v_cache.shape) != (B, L, H, d_h) or tuple(lens.shape) != (B,):
        raise ValueError("shapes: q [B, 2H, d_h], k_cache [B, L, 2H, d_h], v_cache [B, L, H, d_h], lens [B]")
    need = lib().hgf_diff_attention_workspace_bytes(B, L, H, d_h)
    if need == 0:
        raise ValueError("unsupported attention dimensions")
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    if out is None:
        out = torch.empty((B, H, d_h), dtype=torch.float16, device=q.device)
    _check(lib().hgf_diff_attention_decode(q.data_ptr(), k_cache.data_ptr(), v_cache.data_ptr(), lens.data_ptr(), B, L,
                                           H, d_h, float(lam), out.data_ptr(), workspace.data_ptr(),
                                           workspace.numel(), _stream(stream)), "hgf_diff_attention_decode")
    return out


def hgf_packed_weight_bytes_b3(d_out: int, d_in: int) -> int:
    return lib().hgf_packed_weight_bytes_b3(d_out, d_in)


def hgf_quantize_pack_weights_b3(W: torch.Tensor, ws: Workspace, stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    """fp32 [d_out, d_in] -> (base-3 packed uint8 buffer, five weights per byte; s_w fp32 scalar tensor)."""
    _dev(W, torch.float32, "W")
    d_out, d_in = W.shape
    packed = torch.empty(hgf_packed_weight_bytes_b3(d_out, d_in), dtype=torch.uint8, device=W.device)
    s_w = torch.empty(1, dtype=torch.float32, device=W.device)
    _check(lib().hgf_quantize_pack_weights_b3(W.data_ptr(), d_out, d_in, packed.data_ptr(), s_w.data_ptr(),
                                              ws.buf.data_ptr(), ws.bytes, _stream(stream)),
           "hgf_quantize_pack_weights_b3")
    return packed, s_w


def hgf_unpack_weights_b3(packed: torch.Tensor, d_out: int, d_in: int, stream=None) -> torch.Tensor:
    T = torch.empty((d_out, d_in), dtype=torch.int8, device=packed.device)
    _check(lib().hgf_unpack_weights_b3(packed.data_ptr(), d_out, d_in, T.data_ptr(), _stream(stream)),
           "hgf_unpack_weights_b3")
    return T


def hgf_linear_forward_b3(x: torch.Tensor, layer: "Layer", ws: Workspace, y: Optional[torch.Tensor] = None,
                          acc_debug: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """One HGF linear whose `layer.packed` is a base-3 buffer (M <= 4)."""
    _dev(x, torch.float16, "x")
    M, d_in = x.shape
    if d_in != layer.d_in:
        raise ValueError("x has the wrong d_in")
    if y is None:
        y = torch.empty((M, layer.d_out), dtype=torch.float16, device=x.device)
    _check(lib().hgf_linear_forward_b3(x.data_ptr(), M, ctypes.byref(layer.c), y.data_ptr(), _ptr(acc_debug),
                                       ws.buf.data_ptr(), ws.bytes, _stream(stream)), "hgf_linear_forward_b3")
    return y


def hgf_static_scratch_bytes() -> int:
    return lib().hgf_static_scratch_bytes()


def hgf_static_scratch_needed(M: int, d_in: int, d_out: int, rank: int) -> int:
    return lib().hgf_static_scratch_needed(M, d_in, d_out, rank)


def hgf_linear_forward_static(x: torch.Tensor, layer: Layer, y: torch.Tensor,
                              acc_debug: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """hgf_linear_forward without a workspace (the library's own fixed scratch): `y` is the
    caller's output tensor, nothing is allocated here or in the library."""
    _dev(x, torch.float16, "x")
    _dev(y, torch.float16, "y")
    M, d_in = x.shape
    if d_in != layer.d_in or tuple(y.shape) != (M, layer.d_out):
        raise ValueError("x or y has the wrong shape")
    _check(lib().hgf_linear_forward_static(x.data_ptr(), M, ctypes.byref(layer.c), y.data_ptr(), _ptr(acc_debug),
                                           _stream(stream)), "hgf_linear_forward_static")
    return y


class Stack:
    """A layer list and its slot table, marshalled once so a forward is one C call."""

    def __init__(self, layers: Sequence[Layer], slots: Sequence[torch.Tensor], M: int):
        self.layers, self.slots, self.M = list(layers), list(slots), M
        self.c_layers = (hgf_layer * len(layers))(*[l.c for l in layers])
        self.c_slots = (ctypes.c_void_p * len(slots))(*[s.data_ptr() for s in slots])


def hgf_stack_forward(stack: Stack, ws: Workspace, stream=None) -> None:
    _check(lib().hgf_stack_forward(stack.c_layers, len(stack.layers), stack.c_slots, len(stack.slots), stack.M,
                                   ws.buf.data_ptr(), ws.bytes, _stream(stream)), "hgf_stack_forward")
