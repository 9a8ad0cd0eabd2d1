"""One decode step of a whole block of the paper's model shape (d = 512, 8 heads, MLP width 1365),
put together from the library's calls the way the appendix implementation wires them: q, k, v
(BitLinears with their LayerNorm prologue; V maps d -> d/2) -> the new key and value rows appended
to the caches -> differential attention with the per-head gate -> the uncorrected output projection
-> residual -> the gated MLP pair -> down projection -> residual.  Every stage is checked against the
CPU oracle on the input the GPU gave that stage (the single-stage bar), and the block's output
against the oracle's own chain of the same stages.  The residual additions and the cache writes are
the caller's (plain tensor operations here); everything else runs in the library's kernels."""
import numpy as np
import pytest
import torch

from oracle import hgf_oracle as orc
from paper_2602_05269_amd import binding as hb
from paper_2602_05269_amd import synth
from parity import GpuLayer, assert_close_fp16, dev
from test_gpu_layernorm import LnLayer

pytestmark = pytest.mark.gpu


def _olayer(g):
    d = {"T": g.T_ref, "s_w": g.s_w_ref}
    if g.rank:
        d.update(A=g.case["A"], B=g.case["B"], alpha=g.case["alpha"])
    return d


@pytest.mark.parametrize("lens", [[511, 300, 17, 0], [5]])
def test_block_decode_step(lens):
    d, H, dh, hid, r = 512, 8, 32, 1365, 16
    B, L = len(lens), 512
    ws = hb.Workspace(64, 1408, 1408, 128)
    mk = lambda seed, k, n, rank: synth.make_custom(seed, B, k, n, max(rank, 1), act="student_t4", lora_std=0.05, w_std=0.05)
    q_l, k_l = LnLayer(mk(9301, d, d, r), ws, seed=1), LnLayer(mk(9302, d, d, r), ws, seed=2)
    v_l = LnLayer(mk(9303, d, d // 2, r), ws, seed=3)
    o_l = GpuLayer(mk(9304, d // 2, d, 0), ws, rank0=True)
    gate_l, up_l = GpuLayer(mk(9305, d, hid, r), ws), GpuLayer(mk(9306, d, hid, r), ws)
    down_l = GpuLayer(mk(9307, hid, d, r), ws)
    rng = np.random.default_rng(9300 + B)
    x = synth.draw_activations("student_t4", rng, B, d)
    k_cache = (rng.standard_normal((B, L, 2 * H, dh))).astype(np.float16)
    v_cache = (rng.standard_normal((B, L, H, dh))).astype(np.float16)
    lam = orc.diff_attention_lambda_init(2 * dh)

    # ---- the step on the GPU
    xd = dev(x)
    q = hb.hgf_linear_forward(xd, q_l.layer, ws)
    k = hb.hgf_linear_forward(xd, k_l.layer, ws)
    v = hb.hgf_linear_forward(xd, v_l.layer, ws)
    kc, vc = dev(k_cache), dev(v_cache)
    at = torch.tensor(lens, device="cuda", dtype=torch.long)
    rows = torch.arange(B, device="cuda")
    kc[rows, at] = k.view(B, 2 * H, dh)
    vc[rows, at] = v.view(B, H, dh)
    new_lens = torch.tensor([n + 1 for n in lens], dtype=torch.int32, device="cuda")
    a = hb.hgf_diff_attention_decode(q.view(B, 2 * H, dh), kc, vc, new_lens, lam)
    o = hb.hgf_linear_forward(a.view(B, d // 2), o_l.layer, ws)
    x1 = xd + o
    z = hb.hgf_swiglu_forward(x1, gate_l.layer, up_l.layer, ws)
    y = hb.hgf_linear_forward(z, down_l.layer, ws)
    x2 = x1 + y
    torch.cuda.synchronize()
    host = lambda t: t.cpu().numpy()

    # ---- every stage against the oracle on the input the GPU gave it
    for g, out in ((q_l, q), (k_l, k), (v_l, v)):
        assert_close_fp16(host(out), g.oracle(x)["y"], "q, k or v")
    kc_ref, vc_ref = k_cache.copy(), v_cache.copy()
    for b, n in enumerate(lens):
        kc_ref[b, n] = host(k)[b].reshape(2 * H, dh)
        vc_ref[b, n] = host(v)[b].reshape(H, dh)
    a_ref = orc.diff_attention_decode(host(q).reshape(B, 2 * H, dh), kc_ref, vc_ref, [n + 1 for n in lens], lam)
    assert_close_fp16(host(a), a_ref, "attention")
    assert_close_fp16(host(o), o_l.oracle(host(a).reshape(B, d // 2))["y"], "output projection")
    zr = orc.swiglu_pair_forward(host(x1), _olayer(gate_l), _olayer(up_l))
    assert_close_fp16(host(z), zr["z"], "gated pair")
    assert_close_fp16(host(y), down_l.oracle(host(z))["y"], "down projection")

    # ---- the block's output against the oracle's own chain (fp16 hand-over between the stages)
    f16 = lambda t: np.asarray(t, dtype=np.float64).astype(np.float16)
    qo, ko, vo = (f16(g.oracle(x)["y"]) for g in (q_l, k_l, v_l))
    kc2, vc2 = k_cache.copy(), v_cache.copy()
    for b, n in enumerate(lens):
        kc2[b, n] = ko[b].reshape(2 * H, dh)
        vc2[b, n] = vo[b].reshape(H, dh)
    ao = f16(orc.diff_attention_decode(qo.reshape(B, 2 * H, dh), kc2, vc2, [n + 1 for n in lens], lam))
    x1o = (x.astype(np.float32) + f16(o_l.oracle(ao.reshape(B, d // 2))["y"]).astype(np.float32)).astype(np.float16)
    zo = f16(orc.swiglu_pair_forward(x1o, _olayer(gate_l), _olayer(up_l))["z"])
    x2o = (x1o.astype(np.float32) + f16(down_l.oracle(zo)["y"]).astype(np.float32)).astype(np.float16)
    got, want = host(x2).astype(np.float64), x2o.astype(np.float64)
    rel = np.linalg.norm(got - want) / np.linalg.norm(want)
    assert rel < 2e-2, rel
    assert np.abs(want - x.astype(np.float64)).max() > 1e-2      # the block did something
