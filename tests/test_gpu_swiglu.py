"""GPU parity of hgf_swiglu_forward (the gated pair of the paper's MLP: z = SiLU(y_gate) * y_up on
two HGF linears of one input) against the CPU oracle: both layers' int32 accumulators bit-exact,
the fp16 product within 2e-3 + 1e-2 |z|, and the per-token max |z| equal, bit for bit, to the
maximum of the stored outputs."""
import numpy as np
import pytest
import torch

from oracle import hgf_oracle as orc
from paper_2602_05269_amd import binding as hb
from paper_2602_05269_amd import synth
from parity import GpuLayer, assert_close_fp16, dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ws():
    return hb.Workspace(2048, 11008, 11008, 128)


def _oracle_layer(g: GpuLayer):
    c = g.case
    d = {"T": g.T_ref, "s_w": g.s_w_ref}
    if g.rank:
        d.update(A=c["A"], B=c["B"], alpha=c["alpha"])
    return d


def _check_pair(gate: GpuLayer, up: GpuLayer, x: np.ndarray, ws, dense=False):
    M = x.shape[0]
    acc_g = torch.full((M, gate.N), -7, dtype=torch.int32, device="cuda")
    acc_u = torch.full((M, gate.N), -7, dtype=torch.int32, device="cuda")
    amax = torch.full((M,), -1.0, dtype=torch.float32, device="cuda")
    z = hb.hgf_swiglu_forward(dev(x), gate.layer, up.layer, ws, amax=amax, acc_debug_gate=acc_g, acc_debug_up=acc_u)
    torch.cuda.synchronize()
    z = z.cpu().numpy()
    ref = orc.swiglu_pair_forward(x, _oracle_layer(gate), _oracle_layer(up), dense_gemm=dense)
    assert np.array_equal(acc_g.cpu().numpy(), ref["gate"]["acc"]), "gate accumulators differ from the oracle"
    assert np.array_equal(acc_u.cpu().numpy(), ref["up"]["acc"]), "up accumulators differ from the oracle"
    assert_close_fp16(z, ref["z"], "z")
    got_amax = amax.cpu().numpy()
    assert np.array_equal(got_amax.view(np.uint32), np.abs(z).max(axis=1).astype(np.float32).view(np.uint32)), \
        "amax is not the maximum of the stored outputs"
    assert np.allclose(got_amax, ref["amax"], rtol=1e-2, atol=2e-3)
    # without the debug outputs and the maximum: the same product
    z2 = hb.hgf_swiglu_forward(dev(x), gate.layer, up.layer, ws)
    torch.cuda.synchronize()
    assert np.array_equal(z2.cpu().numpy(), z)
    return z, ref


@pytest.mark.parametrize("M,K,N,rg,ru", [
    (1, 64, 64, 16, 16), (1, 4096, 1000, 64, 64), (3, 200, 130, 8, 24), (4, 1365, 96, 32, 0), (8, 256, 192, 0, 16),
    (17, 2048, 257, 64, 64), (33, 704, 320, 128, 128), (40, 1024, 64, 16, 32),
    (41, 768, 200, 64, 64), (64, 512, 300, 8, 24), (130, 1365, 256, 32, 0), (300, 384, 129, 0, 0), (70, 4104, 96, 128, 128),
])
def test_swiglu_pair_shapes(M, K, N, rg, ru, ws):
    cg = synth.make_custom(8100 + M + K + N + rg, M, K, N, max(rg, 1), act="student_t3", lora_std=0.05)
    cu = synth.make_custom(8200 + M + K + N + ru, M, K, N, max(ru, 1), act="student_t3", lora_std=0.05)
    gate, up = GpuLayer(cg, ws, rank0=(rg == 0)), GpuLayer(cu, ws, rank0=(ru == 0))
    _check_pair(gate, up, cg["x"], ws)


def test_swiglu_pair_equals_two_layers_and_the_product(ws):
    """The pair against the library's own single layers: z must be SiLU(y_gate) * y_up of the
    two fp16 outputs up to their rounding (the pair keeps fp32 between the layers and the product)."""
    cg = synth.make_custom(8301, 8, 512, 256, 32, lora_std=0.05)
    cu = synth.make_custom(8302, 8, 512, 256, 32, lora_std=0.05)
    gate, up = GpuLayer(cg, ws), GpuLayer(cu, ws)
    z, _ = _check_pair(gate, up, cg["x"], ws)
    yg, _ = gate.forward(cg["x"])
    yu, _ = up.forward(cg["x"])
    two = orc.swiglu(yg.astype(np.float64), yu.astype(np.float64))
    assert_close_fp16(z, two, "z against the two single layers")


@pytest.mark.parametrize("cfg,M", [(4, 1), (4, 8), (4, 64), (2, 16), (3, 2048)])
def test_swiglu_pair_full_size(cfg, M, ws):
    """The up / gate projections of the benchmark configurations at full size, every element."""
    names = [p.name for p in synth.CONFIGS[cfg].projections]
    gate = GpuLayer(synth.make_weights(cfg, 0, names.index("gate")), ws)
    up = GpuLayer(synth.make_weights(cfg, 0, names.index("up")), ws)
    x = synth.make_activations(cfg, 0, names.index("up"), M)
    _check_pair(gate, up, x, ws, dense=True)
