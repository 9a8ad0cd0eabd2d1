"""GPU parity of the base-3 packing (five ternary weights per byte, 1.6 bits per weight) and its
few-token decode kernel against the CPU oracle: unpacked codes and the fp32 bits of s_w equal to
the oracle's ternariser, every one of the 3^5 digit groups round-trips, int32 accumulators
bit-exact, fp16 outputs within 2e-3 + 1e-2 |y|."""
import itertools

import numpy as np
import pytest
import torch

from oracle import hgf_oracle as orc
from paper_2602_05269_amd import binding as hb
from paper_2602_05269_amd import synth
from parity import assert_close_fp16, dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ws():
    return hb.Workspace(64, 11008, 11008, 128)


class B3Layer:
    def __init__(self, case, ws, rank0=False):
        self.case, self.K, self.N = case, case["d_in"], case["d_out"]
        self.rank = 0 if rank0 else case["rank"]
        self.packed, self.s_w = hb.hgf_quantize_pack_weights_b3(dev(case["W"]), ws)
        A = B = alpha = None
        if self.rank:
            A, B, alpha = dev(case["A"]), dev(case["B"]), dev(case["alpha"])
        self.layer = hb.Layer(self.packed, self.s_w, self.N, self.K, A, B, alpha)
        self.T_ref, self.s_w_ref = orc.ternarize(case["W"])

    def check_weights(self):
        assert self.packed.numel() == self.N * ((-(-self.K // 5) + 15) // 16 * 16)
        T = hb.hgf_unpack_weights_b3(self.packed, self.N, self.K).cpu().numpy()
        assert self.s_w.cpu().numpy()[0].view(np.uint32) == np.float32(self.s_w_ref).view(np.uint32)
        assert np.array_equal(T, self.T_ref)

    def check_forward(self, x, ws, dense=False):
        M = x.shape[0]
        acc = torch.full((M, self.N), -5, dtype=torch.int32, device="cuda")
        y = hb.hgf_linear_forward_b3(dev(x), self.layer, ws, acc_debug=acc)
        torch.cuda.synchronize()
        c = self.case
        A, B, alpha = (c["A"], c["B"], c["alpha"]) if self.rank else (None, None, None)
        ref = orc.linear_forward(x, self.T_ref, self.s_w_ref, A, B, alpha, dense_gemm=dense)
        assert np.array_equal(acc.cpu().numpy(), ref["acc"]), "int32 accumulators differ from the oracle"
        assert_close_fp16(y.cpu().numpy(), ref["y"])


@pytest.mark.parametrize("N,K", [(1, 1), (3, 63), (64, 64), (65, 65), (100, 1365), (33, 4096), (7, 11008)])
def test_b3_pack_unpack_matches_oracle_ternariser(N, K, ws):
    B3Layer(synth.make_custom(N * 7 + K, 1, K, N, 8), ws).check_weights()


def test_b3_every_digit_group_round_trips(ws):
    """All 243 groups of five ternary weights, one group per row, through pack and unpack; the
    byte of a group is its base-3 value with the first column as the lowest digit; padding is 121."""
    groups = np.array(list(itertools.product((-1, 0, 1), repeat=5)), dtype=np.float32)    # [243, 5]
    W = groups * np.float32(0.5)       # mean |W| = 1/3, so W / s_w = +-1.5 -> +-2 -> clipped to +-1; zeros stay
    packed, s_w = hb.hgf_quantize_pack_weights_b3(dev(W), ws)
    T = hb.hgf_unpack_weights_b3(packed, 243, 5).cpu().numpy()
    T_ref, g_ref = orc.ternarize(W)
    assert np.array_equal(T, T_ref) and np.array_equal(T_ref, groups.astype(np.int8))
    raw = packed.cpu().numpy().reshape(243, 16)
    want = ((groups.astype(np.int64) + 1) * (3 ** np.arange(5))).sum(axis=1)
    assert np.array_equal(raw[:, 0].astype(np.int64), want)
    assert (raw[:, 1:] == 121).all()


@pytest.mark.parametrize("M,K,N,r", [
    (1, 1, 1, 1), (1, 64, 64, 16), (1, 4096, 1000, 64), (2, 63, 37, 8), (3, 1365, 130, 32), (4, 11008, 96, 128),
    (4, 700, 257, 0), (1, 12288, 31, 128), (2, 4101, 64, 24),
])
def test_b3_decode_parity(M, K, N, r, ws):
    c = synth.make_custom(9500 + M + K + N + r, M, K, N, max(r, 1), act="student_t3", lora_std=0.05)
    g = B3Layer(c, ws, rank0=(r == 0))
    g.check_forward(c["x"], ws)


@pytest.mark.parametrize("proj,M", [(0, 1), (2, 1), (2, 4)])
def test_b3_config4_full_size(proj, M, ws):
    g = B3Layer(synth.make_weights(4, 0, proj), ws)
    g.check_weights()
    g.check_forward(synth.make_activations(4, 0, proj, M), ws, dense=True)


def test_b3_refuses_what_it_does_not_serve(ws):
    c = synth.make_custom(1, 5, 64, 64, 8)
    g = B3Layer(c, ws)
    with pytest.raises(hb.HgfError) as e:
        hb.hgf_linear_forward_b3(dev(c["x"]), g.layer, ws)
    assert e.value.status == 4
    assert hb.hgf_packed_weight_bytes_b3(11008, 4096) == 11008 * 832      # 820 bytes of digits per row, padded to 832
    assert hb.hgf_packed_weight_bytes_b3(11008, 4096) < 0.82 * hb.hgf_packed_weight_bytes(11008, 4096)
