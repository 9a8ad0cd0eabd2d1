"""GPU test of hgf_linear_forward_static, the entry point that allocates nothing: its scratch is a
fixed array inside the library instead of a caller's workspace.  Each case makes two calls in a
row through the C ABI, the second with a smaller input (fewer tokens and a smaller layer), and
compares both with hgf_linear_forward on an ordinary workspace: the same kernels run, so the
int32 accumulators and the fp16 outputs must agree bit for bit (and therefore meet the oracle's
bar, which the parity tests hold hgf_linear_forward to)."""
import numpy as np
import pytest
import torch

from paper_2602_05269_amd import binding as hb
from paper_2602_05269_amd import synth
from parity import GpuLayer, dev

pytestmark = pytest.mark.gpu


def _both(g: GpuLayer, x: np.ndarray, ws: hb.Workspace):
    xd = dev(x)
    M = x.shape[0]
    acc_ref = torch.full((M, g.N), -1, dtype=torch.int32, device="cuda")
    y_ref = hb.hgf_linear_forward(xd, g.layer, ws, acc_debug=acc_ref)
    acc = torch.full((M, g.N), -2, dtype=torch.int32, device="cuda")
    y = torch.full((M, g.N), float("nan"), dtype=torch.float16, device="cuda")
    before = torch.cuda.memory_allocated()
    hb.hgf_linear_forward_static(xd, g.layer, y, acc_debug=acc)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    assert np.array_equal(acc.cpu().numpy(), acc_ref.cpu().numpy()), "accumulators differ"
    assert np.array_equal(y.cpu().numpy().view(np.uint16), y_ref.cpu().numpy().view(np.uint16)), "outputs differ"
    return y.cpu().numpy(), acc.cpu().numpy()


# (tokens, d_in, d_out, rank) of the first call and of the smaller second call, one pair per path:
# the single persistent launch (M <= 4), the two-launch decode path, the prefill path
@pytest.mark.parametrize("first,second", [
    ((4, 4096, 1024, 64), (1, 1024, 320, 32)),
    ((32, 2048, 512, 64), (7, 1000, 130, 24)),
    ((300, 1536, 512, 64), (70, 512, 200, 16)),
])
def test_static_scratch_entry_matches_the_workspace_entry(first, second):
    ws = hb.Workspace(512, 4096, 4096, 128)
    for i, (M, K, N, r) in enumerate((first, second, first)):
        assert hb.hgf_static_scratch_needed(M, K, N, r) <= hb.hgf_static_scratch_bytes()
        c = synth.make_custom(9100 + 10 * i + M, M, K, N, r, act="student_t3")
        g = GpuLayer(c, ws)
        y, acc = _both(g, c["x"], ws)
        ref = g.oracle(c["x"])
        assert np.array_equal(acc, ref["acc"])
        err = np.abs(y.astype(np.float64) - ref["y"])
        assert (err <= 2e-3 + 1e-2 * np.abs(ref["y"])).all()


def test_static_scratch_entry_rejects_what_does_not_fit():
    """Sizes beyond the fixed array are refused on the host: nothing is enqueued (the pointers
    are fake and would fault if they were used)."""
    import ctypes
    lib = hb.lib()
    L = hb.hgf_layer(d_in=8192, d_out=256, rank=16, W_packed=0x1000, s_w=0x2000, A_f16=0x3000, B_f16=0x4000,
                     alpha_f16=0x5000, src_slot=0, dst_slot=1)
    assert hb.hgf_static_scratch_needed(2048, 8192, 256, 16) > hb.hgf_static_scratch_bytes()
    assert lib.hgf_linear_forward_static(0x10000, 2048, ctypes.byref(L), 0x20000, None, None) == 5
    assert lib.hgf_linear_forward_static(None, 1, ctypes.byref(L), 0x20000, None, None) == 1
    assert lib.hgf_linear_forward_static(0x10000, 0, ctypes.byref(L), 0x20000, None, None) == 2
