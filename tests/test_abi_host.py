"""CPU-only checks of the C ABI: the library loads, exports every symbol the header
declares, sizes are right, and every argument error is caught on the host (no GPU call)."""
import ctypes
import os
import re

import pytest

from paper_2602_05269_amd import binding as hb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "hgf.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hgf_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert {"hgf_quantize_pack_weights", "hgf_quantize_activations", "hgf_linear_forward",
            "hgf_stack_forward", "hgf_unpack_weights", "hgf_workspace_bytes"} <= set(names)
    lib = hb.lib()
    for n in names:
        assert hasattr(lib, n), f"libhgf.so does not export {n}"


def test_sizes():
    assert hb.hgf_version() >= 100
    assert hb.hgf_padded_k(1) == 128 and hb.hgf_padded_k(256) == 256 and hb.hgf_padded_k(1365) == 1408
    assert hb.hgf_padded_k(0) == 0 and hb.hgf_padded_k(1 << 20) == 0
    assert hb.hgf_packed_weight_bytes(32, 128) == 1024
    assert hb.hgf_packed_weight_bytes(33, 129) == 4096
    assert hb.hgf_packed_weight_bytes(11008, 4096) == 11008 * 4096 // 4      # 2 bits per weight
    assert hb.hgf_packed_weight_bytes(0, 5) == 0
    a = hb.hgf_workspace_bytes(1, 512, 512, 32)
    b = hb.hgf_workspace_bytes(64, 11008, 11008, 128)
    c = hb.hgf_workspace_bytes(2048, 8192, 8192, 64)
    assert 0 < a < b < c
    assert hb.hgf_workspace_bytes(1, 512, 512, 129) == 0
    assert hb.hgf_workspace_bytes(0, 512, 512, 8) == 0


def test_status_strings():
    lib = hb.lib()
    for code, name in hb.STATUS_NAMES.items():
        assert lib.hgf_status_string(code).decode().startswith(name)
    assert b"unknown" in lib.hgf_status_string(99)


def _layer(**kw):
    base = dict(d_in=256, d_out=256, rank=16, W_packed=0x1000, s_w=0x2000, A_f16=0x3000, B_f16=0x4000,
                alpha_f16=0x5000, src_slot=0, dst_slot=1)
    base.update(kw)
    return hb.hgf_layer(**base)


def test_linear_forward_rejects_bad_arguments_on_the_host():
    """Fake (never dereferenced) device addresses: every path below must return before any launch."""
    lib = hb.lib()
    X, Y, WS = 0x10000, 0x20000, 0x30000
    big = 1 << 30

    def call(x=X, M=8, L=None, y=Y, ws=WS, ws_bytes=big):
        L = L if L is not None else _layer()
        return lib.hgf_linear_forward(x, M, ctypes.byref(L), y, None, ws, ws_bytes, None)

    assert call(x=None) == 1 and call(y=None) == 1
    assert lib.hgf_linear_forward(X, 8, None, Y, None, WS, big, None) == 1
    assert call(L=_layer(W_packed=None)) == 1 and call(L=_layer(s_w=None)) == 1
    assert call(L=_layer(A_f16=None)) == 1 and call(L=_layer(alpha_f16=None)) == 1
    assert call(M=0) == 2 and call(M=-3) == 2
    assert call(L=_layer(d_in=0)) == 2 and call(L=_layer(d_out=70000)) == 2
    assert call(L=_layer(rank=129)) == 2 and call(L=_layer(rank=-1)) == 2
    assert call(M=1 << 20, L=_layer(d_in=4096)) == 2          # M * d_in overflows 2^31
    assert call(x=X + 2) == 3 and call(y=Y + 8) == 3 and call(L=_layer(W_packed=0x1004)) == 3
    assert call(ws=None) == 5 and call(ws_bytes=1024) == 5
    assert call(ws=WS + 4) == 3


def test_other_entry_points_reject_bad_arguments_on_the_host():
    lib = hb.lib()
    assert lib.hgf_quantize_activations(None, 1, 64, 0x100, 0x200, None, None) == 1
    assert lib.hgf_quantize_activations(0x100, 0, 64, 0x200, 0x300, None, None) == 2
    assert lib.hgf_quantize_activations(0x104, 1, 64, 0x200, 0x300, None, None) == 3
    assert lib.hgf_quantize_pack_weights(None, 4, 4, 0x100, 0x200, 0x300, 1 << 30, None) == 1
    assert lib.hgf_quantize_pack_weights(0x100, 4, 0, 0x100, 0x200, 0x300, 1 << 30, None) == 2
    assert lib.hgf_quantize_pack_weights(0x100, 4, 4, 0x100, 0x200, None, 0, None) == 5
    assert lib.hgf_quantize_pack_weights(0x100, 4, 4, 0x100, 0x200, 0x300, 16, None) == 5
    assert lib.hgf_unpack_weights(None, 4, 4, 0x100, None) == 1
    assert lib.hgf_unpack_weights(0x100, 4, -1, 0x100, None) == 2
    assert lib.hgf_workspace_init(None, 1 << 30, None) == 1
    assert lib.hgf_workspace_init(0x100, 64, None) == 5


def test_stack_forward_rejects_bad_wiring_on_the_host():
    lib = hb.lib()
    layers = (hb.hgf_layer * 2)(_layer(src_slot=0, dst_slot=1), _layer(src_slot=1, dst_slot=2))
    slots = (ctypes.c_void_p * 3)(0x1000, 0x2000, 0x3000)
    big = 1 << 30
    assert lib.hgf_stack_forward(None, 2, slots, 3, 1, 0x100, big, None) == 1
    assert lib.hgf_stack_forward(layers, 0, slots, 3, 1, 0x100, big, None) == 2
    assert lib.hgf_stack_forward(layers, 2, slots, 2, 1, 0x100, big, None) == 2     # dst_slot out of range
    bad = (hb.hgf_layer * 1)(_layer(src_slot=1, dst_slot=1))
    assert lib.hgf_stack_forward(bad, 1, slots, 3, 1, 0x100, big, None) == 2        # in-place layer
    holes = (ctypes.c_void_p * 3)(0x1000, None, 0x3000)
    assert lib.hgf_stack_forward(layers, 2, holes, 3, 1, 0x100, big, None) == 1
    assert lib.hgf_stack_forward(layers, 2, slots, 3, 1, None, 0, None) == 5
    assert lib.hgf_stack_forward(layers, 2, slots, 3, 1, 0x100, 4096, None) == 5


def test_refused_launch_is_reported_not_hidden():
    """Where the HIP runtime refuses a launch (here: a host without a GPU, so every launch is
    refused) the forward calls return HGF_ERR_DEVICE.  In particular a layer list that
    qualifies for the whole-stack launch must not report success after quietly trying other
    paths.  Arguments are valid but fake, so this runs only where nothing can be launched."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("needs a host where launches are refused (no GPU)")
    lib = hb.lib()
    layers = (hb.hgf_layer * 2)(_layer(src_slot=0, dst_slot=1), _layer(src_slot=1, dst_slot=2))
    slots = (ctypes.c_void_p * 3)(0x1000, 0x2000, 0x3000)
    for M in (1, 8, 100):
        assert lib.hgf_stack_forward(layers, 2, slots, 3, M, 0x100, 1 << 30, None) == 6
    L = _layer()
    for M in (1, 8, 100):
        assert lib.hgf_linear_forward(0x10000, M, ctypes.byref(L), 0x20000, None, 0x30000, 1 << 30, None) == 6
    assert lib.hgf_workspace_init(0x100, 1 << 30, None) == 6


def test_binding_refuses_cpu_tensors():
    import torch
    with pytest.raises(ValueError):
        hb.hgf_quantize_activations(torch.zeros(2, 64, dtype=torch.float16))
