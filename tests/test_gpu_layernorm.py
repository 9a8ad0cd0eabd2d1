"""GPU parity of the fused LayerNorm -> quantise prologue (the appendix implementation's BitLinear
normalises the backbone's input; the correction path reads x itself) against the CPU oracle:
x_q, the fp32 bits of s_x and the row sums bit-exact for the stand-alone entry; the int32
accumulators bit-exact and the fp16 outputs within 2e-3 + 1e-2 |y| for whole layers, alone and
in a layer list."""
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


def _ln_params(seed, K, with_beta=True):
    rng = np.random.default_rng([seed, 99])
    gamma = (1.0 + 0.25 * rng.standard_normal(K)).astype(np.float32)
    beta = (0.2 * rng.standard_normal(K)).astype(np.float32) if with_beta else None
    return gamma, beta


@pytest.mark.parametrize("M,K,kind", [(1, 1, "normal"), (3, 63, "normal"), (8, 512, "normal"), (5, 1365, "student_t3"),
                                      (16, 2048, "outlier"), (7, 11008, "student_t3"), (300, 3072, "student_t4")])
def test_layernorm_quantize_bit_exact(M, K, kind):
    x = synth.draw_activations(kind, np.random.default_rng([M, K, 5]), M, K)
    if M >= 3:
        x[1] = np.float16(0.75)                        # a constant token: normalises to beta
        x[2, K // 2] = np.float16(60000.0)             # a huge outlier
    gamma, beta = _ln_params(M + K, K, with_beta=(K % 2 == 1 or K > 100))
    xq, s_x, rowsum = hb.hgf_layernorm_quantize_activations(dev(x), dev(gamma), None if beta is None else dev(beta))
    torch.cuda.synchronize()
    v = orc.layernorm(x, gamma, np.zeros(K, np.float32) if beta is None else beta, 1e-5)
    xq_ref, s_ref, rs_ref = orc.quantize_act(v, allow_f32=True)
    xq = xq.cpu().numpy()
    assert np.array_equal(xq[:, :K], xq_ref)
    assert not xq[:, K:].any()
    assert np.array_equal(s_x.cpu().numpy().view(np.uint32), s_ref.view(np.uint32))
    assert np.array_equal(rowsum.cpu().numpy(), rs_ref)


class LnLayer(GpuLayer):
    """A GpuLayer whose hgf_layer carries LayerNorm parameters; its oracle normalises too."""

    def __init__(self, case, ws, seed, rank0=False, with_beta=True):
        super().__init__(case, ws, rank0=rank0)
        self.gamma, self.beta = _ln_params(seed, self.K, with_beta)
        self.d_gamma = dev(self.gamma)
        self.d_beta = None if self.beta is None else dev(self.beta)
        L = self.layer
        self.layer = hb.Layer(L.packed, L.s_w, self.N, self.K, L.A, L.B, L.alpha,
                              ln_gamma=self.d_gamma, ln_beta=self.d_beta, ln_eps=1e-5)

    def oracle(self, x, rows=None, dense=False):
        c = self.case
        A, B, alpha = (c["A"], c["B"], c["alpha"]) if self.rank else (None, None, None)
        beta = np.zeros(self.K, np.float32) if self.beta is None else self.beta
        return orc.linear_forward(x, self.T_ref, self.s_w_ref, A, B, alpha, dense_gemm=dense,
                                  ln=(self.gamma, beta, 1e-5))


@pytest.mark.parametrize("M,K,N,r", [
    (1, 64, 64, 16), (1, 4096, 1000, 64), (2, 100, 37, 8), (4, 1365, 130, 32), (8, 256, 192, 0),
    (17, 2048, 257, 64), (40, 1024, 64, 16), (41, 768, 200, 64), (130, 1365, 256, 32), (300, 384, 129, 0),
])
def test_layer_with_layernorm_parity(M, K, N, r, ws):
    c = synth.make_custom(8500 + M + K + N + r, M, K, N, max(r, 1), act="student_t3", lora_std=0.05)
    g = LnLayer(c, ws, seed=M + K, rank0=(r == 0), with_beta=(M % 2 == 1))
    y, ref = g.check_forward(c["x"])
    # the LayerNorm matters: the plain layer's accumulators are different
    plain = GpuLayer(c, ws, rank0=(r == 0))
    _, acc_plain = plain.forward(c["x"])
    assert not np.array_equal(acc_plain, ref["acc"])


@pytest.mark.parametrize("M", [1, 16, 100])
def test_layernorm_layers_in_a_layer_list(M, ws):
    """q, k, v with a LayerNorm each read one slot (so they cannot share a quantisation), a
    plain layer follows: every output against the oracle on the input the GPU gave that layer."""
    K = 512
    shapes = [(K, 512, 16, 0, 1, True), (K, 512, 16, 0, 2, True), (K, 256, 8, 0, 3, True), (256, 384, 16, 3, 4, False),
              (384, 128, 8, 4, 5, True)]
    cases, layers = [], []
    slots = [None] * 6
    for i, (k, n, r, src, dst, ln) in enumerate(shapes):
        c = synth.make_custom(8600 + 10 * M + i, M, k, n, r, act="student_t4", lora_std=0.05, w_std=0.05)
        if i == 0:
            slots[0] = dev(c["x"])
        g = LnLayer(c, ws, seed=i) if ln else GpuLayer(c, ws)
        g.layer.c.src_slot, g.layer.c.dst_slot = src, dst
        cases.append(g)
        layers.append(g.layer)
        slots[dst] = torch.zeros((M, n), dtype=torch.float16, device="cuda")
    hb.hgf_stack_forward(hb.Stack(layers, slots, M), ws)
    torch.cuda.synchronize()
    host = [s.cpu().numpy() for s in slots]
    for g, (k, n, r, src, dst, ln) in zip(cases, shapes):
        assert_close_fp16(host[dst], g.oracle(host[src])["y"], f"slot {dst}")


@pytest.mark.parametrize("cfg,proj,M", [(4, 2, 1), (4, 0, 32), (3, 6, 2048)])
def test_layer_with_layernorm_full_size(cfg, proj, M, ws):
    w = synth.make_weights(cfg, 0, proj)
    g = LnLayer(w, ws, seed=cfg * 10 + proj)
    x = synth.make_activations(cfg, 0, proj, M)
    y, acc = g.forward(x)
    ref = g.oracle(x, dense=True)
    assert np.array_equal(acc, ref["acc"])
    assert_close_fp16(y, ref["y"])
