"""Pins for the CPU oracle: each oracle function is checked against something other
than itself -- values the paper prints (tests/golden/paper_values.txt), closed forms on
constructed inputs, brute-force dense products in numpy, and the invariants the paper
states (gate off / rank 0 reduce to a pure ternary layer; a ternary product is add /
subtract / skip).  CPU only."""
import math
import os

import numpy as np
import pytest
from scipy.special import expit

from oracle import hgf_oracle as orc
from paper_2602_05269_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_values.txt")


def _golden():
    out = {}
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, val, tol, _cite = [s.strip() for s in line.split("|")]
            out[name] = (float(val), float(tol))
    return out


PAPER = _golden()


def _near(name, got):
    val, tol = PAPER[name]
    assert abs(got - val) <= tol, f"{name}: oracle {got} vs paper {val} +- {tol}"


# ------------------------------------------------------------------ printed values

def test_paper_gate_values():
    _near("gate_init_tanh_0p1", orc.gate(0.1))
    _near("frozen_gate", orc.gate(math.atanh(0.1023)))


def test_paper_effective_bit_width():
    b = orc.effective_bit_width(0.1, 32, 512)
    _near("effective_bit_width", b)
    _near("effective_bit_increase", (b - math.log2(3)) / math.log2(3))


def test_paper_lora_ratio_and_speedup():
    ratio = orc.lora_param_ratio(512, 512, 32)
    assert ratio == 0.125                       # exact for the paper's square d=512, r=32 layer
    _near("lora_param_ratio", ratio)
    _near("theoretical_speedup", orc.theoretical_speedup(4.0, 0.12))


def test_paper_memory_wall():
    _near("memory_wall_tokens_s", orc.memory_wall_tokens_per_s(500e9, 7e9, 16))
    _near("fp16_7b_gigabytes", 7e9 * 16 / 8 / 1e9)


def test_correction_memory_overhead_band():
    """Correction-path bytes relative to the dense fp16 layer, for the paper's d=512 block
    mix (4 square + up/gate/down with FFN 2048, r=32): the paper quotes 10% -> ~15% of
    FP16 for BitNet -> HGF, i.e. roughly five points; the parameter count gives 9%."""
    tot = {"fp16_dense": 0.0, "ternary_2bit": 0.0, "correction": 0.0}
    for p in synth.CONFIGS[1].projections:
        b = orc.layer_bytes(p.d_in, p.d_out, 32)
        for k in tot:
            tot[k] += b[k]
    frac = tot["correction"] / tot["fp16_dense"]
    assert 0.05 < frac < 0.15, frac
    assert abs(tot["ternary_2bit"] / tot["fp16_dense"] - 0.125) < 1e-12


# ------------------------------------------------------------------ ternariser

def test_ternarize_equal_magnitudes():
    rng = np.random.default_rng(1)
    sign = rng.choice([-1.0, 1.0], size=(7, 13)).astype(np.float32)
    T, g = orc.ternarize(0.03125 * sign)
    assert g == np.float32(0.03125)
    assert np.array_equal(T, sign.astype(np.int8))


def test_ternarize_constructed_codes_and_ties():
    # mean |w| is exactly 1, so w/gamma = w: ties 0.5 -> 0 and 2.5 -> 2 (half to even), clip at +-1
    w = np.array([[0.5, -0.5, 1.5, -1.5], [0.25, -0.25, 1.75, -1.75]], dtype=np.float32)
    T, g = orc.ternarize(w)
    assert g == np.float32(1.0)
    assert T.tolist() == [[0, 0, 1, -1], [0, 0, 1, -1]]
    w2 = np.array([[0.49, 0.51, -0.51, -0.49, 3.0, -3.0, 0.0, 0.0]], dtype=np.float32)
    T2, g2 = orc.ternarize(w2)
    q = np.clip(np.rint(w2.astype(np.float64) / float(g2)), -1, 1)
    assert np.array_equal(T2, q.astype(np.int8))
    assert g2 == np.float32(1.0)                         # |w| sums to 8 over 8 entries
    assert T2.tolist() == [[0, 1, -1, 0, 1, -1, 0, 0]]   # 0.49 -> 0, 0.51 -> 1, 3 -> clip 1


def test_ternarize_layout_not_transposed():
    w = np.zeros((3, 5), dtype=np.float32)
    w[0, 4] = 1.0
    w[2, 1] = -1.0
    w[1, :] = 0.01
    T, _ = orc.ternarize(w)
    assert T[0, 4] == 1 and T[2, 1] == -1 and T.sum() == 0 and np.abs(T).sum() == 2


def test_ternarize_all_zero():
    T, g = orc.ternarize(np.zeros((4, 8), dtype=np.float32))
    assert g == np.float32(1e-5)
    assert not T.any()


def test_ternarize_gaussian_statistics():
    # W ~ N(0, s^2): gamma -> s*sqrt(2/pi); P(T=0) = P(|z| < 0.5*sqrt(2/pi)) = 0.3101
    rng = np.random.default_rng(7)
    W = (0.02 * rng.standard_normal((1024, 1024))).astype(np.float32)
    T, g = orc.ternarize(W)
    assert abs(float(g) / 0.02 - math.sqrt(2 / math.pi)) < 2e-3
    p0 = float((T == 0).mean())
    assert abs(p0 - math.erf(0.5 * math.sqrt(2 / math.pi) / math.sqrt(2))) < 2e-3
    assert abs(float((T == 1).mean()) - float((T == -1).mean())) < 3e-3
    # the scale is the mean of |W| (fp64 sum rounded once), not the max
    assert g == np.float32(np.abs(W.astype(np.float64)).mean())


# ------------------------------------------------------------------ activation quantiser

def test_quantize_exact_grid_and_ties():
    j = np.arange(-127, 128)
    x = (j / 8.0).astype(np.float16)[None, :]          # amax = 127/8  ->  127/amax = 8 exactly
    xq, s_x, rowsum = orc.quantize_act(x)
    assert np.array_equal(xq[0], j.astype(np.int8))
    assert s_x[0] == np.float32(1.0 / 8.0)
    assert rowsum[0] == 0
    ties = np.array([[127 / 8.0, 0.5 / 8, 1.5 / 8, 2.5 / 8, -0.5 / 8, -1.5 / 8, -2.5 / 8]], dtype=np.float16)
    xq2, _, rs2 = orc.quantize_act(ties)
    assert xq2[0].tolist() == [127, 0, 2, 2, 0, -2, -2]
    assert rs2[0] == 127


def test_quantize_properties():
    x = synth.draw_activations("student_t3", np.random.default_rng(3), 9, 333)
    xq, s_x, rowsum = orc.quantize_act(x)
    xf = x.astype(np.float64)
    amax = np.abs(xf).max(axis=1)
    assert np.array_equal(np.abs(xq.astype(np.int32)).max(axis=1), np.full(9, 127))
    assert np.allclose(s_x, amax / 127.0, rtol=1e-6)
    # the method's own error bound: half a quantisation step per element
    err = np.abs(xf - xq.astype(np.float64) * s_x[:, None].astype(np.float64))
    assert (err <= 0.5 * s_x[:, None] * (1 + 1e-5)).all()
    # odd symmetry and per-token independence
    xq_neg, s_neg, rs_neg = orc.quantize_act((-x).astype(np.float16))
    assert np.array_equal(xq_neg, -xq) and np.array_equal(s_neg, s_x) and np.array_equal(rs_neg, -rowsum)
    x2 = x.copy()
    x2[4] *= np.float16(3.0)
    xq2, _, _ = orc.quantize_act(x2)
    keep = [i for i in range(9) if i != 4]
    assert np.array_equal(xq2[keep], xq[keep])
    assert np.array_equal(rowsum, xq.astype(np.int64).sum(axis=1))


def test_quantize_zero_row_and_outlier():
    x = np.zeros((2, 64), dtype=np.float16)
    x[1, :] = 0.25
    x[1, 17] = -5.0                                   # one channel 20x the rest
    xq, s_x, rowsum = orc.quantize_act(x)
    assert not xq[0].any() and s_x[0] == np.float32(np.float32(1e-5) / np.float32(127.0))
    assert xq[1, 17] == -127 and set(np.delete(xq[1], 17).tolist()) == {6}   # 0.25*25.4 = 6.35
    assert rowsum[0] == 0 and rowsum[1] == 63 * 6 - 127


# ------------------------------------------------------------------ integer contraction

@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (3, 5, 7), (8, 33, 65), (2, 64, 1365)])
def test_int_gemm_equals_dense_product(M, N, K):
    rng = np.random.default_rng(M * 100 + N * 10 + K)
    T = rng.integers(-1, 2, size=(N, K)).astype(np.int8)
    xq = rng.integers(-127, 128, size=(M, K)).astype(np.int8)
    acc = orc.int_gemm(T, xq)
    ref = xq.astype(np.int64) @ T.astype(np.int64).T           # multiply formulation, numpy
    assert np.array_equal(acc.astype(np.int64), ref)
    assert np.array_equal(orc.int_gemm(-T, xq), -acc)          # sign flip
    assert not orc.int_gemm(np.zeros_like(T), xq).any()        # all-zero weights


def test_int_gemm_exhaustive_tiny():
    # every ternary row of length 3 against a fixed activation: brute force in Python
    x = np.array([[5, -7, 11]], dtype=np.int8)
    rows = [(a, b, c) for a in (-1, 0, 1) for b in (-1, 0, 1) for c in (-1, 0, 1)]
    T = np.array(rows, dtype=np.int8)
    acc = orc.int_gemm(T, x)
    assert acc[0].tolist() == [5 * a - 7 * b + 11 * c for a, b, c in rows]


def test_int_gemm_one_hot_rows_select_activations():
    K = 40
    T = np.zeros((K, K), dtype=np.int8)
    T[np.arange(K), (np.arange(K) * 7) % K] = 1
    xq = np.random.default_rng(0).integers(-127, 128, size=(3, K)).astype(np.int8)
    acc = orc.int_gemm(T, xq)
    assert np.array_equal(acc, xq[:, (np.arange(K) * 7) % K].astype(np.int32))


def test_int_gemm_extreme_accumulator():
    K = 11008
    T = np.ones((2, K), dtype=np.int8)
    T[1] = -1
    xq = np.full((1, K), 127, dtype=np.int8)
    assert orc.int_gemm(T, xq).tolist() == [[127 * K, -127 * K]]


@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (3, 5, 7), (8, 33, 65), (2, 64, 1365), (17, 130, 4096), (5, 40, 11008)])
def test_dense_shortcut_equals_the_triple_loop(M, N, K):
    """The BLAS product used for the full-size parity cases gives the loop's integers exactly:
    on random operands, on rows of all +1 / all -1 against all +-127 (the largest partial sums
    there are: 127 K = 1 398 016 < 2^24 at K = 11008), and through linear_forward."""
    rng = np.random.default_rng(M * 1000 + N * 10 + K)
    T = rng.integers(-1, 2, size=(N, K)).astype(np.int8)
    xq = rng.integers(-127, 128, size=(M, K)).astype(np.int8)
    T[0] = 1
    T[N - 1] = -1
    xq[0] = 127
    xq[M - 1] = -127
    loop = orc.int_gemm(T, xq)
    assert np.array_equal(orc.int_gemm_dense(T, xq), loop)
    assert abs(int(loop[0, 0])) == 127 * K
    if K <= 4096:
        c = synth.make_custom(K + N, M, K, N, 8, act="student_t3")
        Tc, s_w = orc.ternarize(c["W"])
        a = orc.linear_forward(c["x"], Tc, s_w, c["A"], c["B"], c["alpha"])
        b = orc.linear_forward(c["x"], Tc, s_w, c["A"], c["B"], c["alpha"], dense_gemm=True)
        assert np.array_equal(a["acc"], b["acc"]) and np.array_equal(a["y"], b["y"])


# ------------------------------------------------------------------ full layer

def _case(seed, M, K, N, r, **kw):
    c = synth.make_custom(seed, M, K, N, r, **kw)
    c["T"], c["s_w"] = orc.ternarize(c["W"])
    return c


def test_backbone_equals_dense_product_of_dequantised_operands():
    """Y_tern is the dense product of the de-quantised activations and weights (Sec. 2.2.1,
    quantised linear forward) -- checked against numpy's fp64 matmul."""
    c = _case(11, 5, 96, 40, 8)
    out = orc.linear_forward(c["x"], c["T"], c["s_w"], c["A"], c["B"], c["alpha"])
    x_hat = out["xq"].astype(np.float64) * out["s_x"].astype(np.float64)[:, None]
    w_hat = c["T"].astype(np.float64) * float(c["s_w"])
    assert np.allclose(out["y_tern"], x_hat @ w_hat.T, rtol=1e-12, atol=1e-14)
    # and it approximates the un-quantised product X W^T up to the quantisation error
    y_true = c["x"].astype(np.float64) @ c["W"].astype(np.float64).T
    rel = np.linalg.norm(out["y_tern"] - y_true) / np.linalg.norm(y_true)
    assert rel < 0.6


def test_gate_off_rank0_and_zero_B_reduce_to_pure_ternary_layer():
    c = _case(12, 4, 128, 72, 16)
    full = orc.linear_forward(c["x"], c["T"], c["s_w"], c["A"], c["B"], c["alpha"])
    off = orc.linear_forward(c["x"], c["T"], c["s_w"], c["A"], c["B"], np.zeros_like(c["alpha"]))
    r0 = orc.linear_forward(c["x"], c["T"], c["s_w"], None, None, None)
    b0 = orc.linear_forward(c["x"], c["T"], c["s_w"], c["A"], np.zeros_like(c["B"]), c["alpha"])
    for o in (off, r0, b0):
        assert np.array_equal(o["y"], full["y_tern"])
        assert np.array_equal(o["acc"], full["acc"])
    assert not np.array_equal(full["y"], full["y_tern"])


def test_correction_path_equals_textbook_dense_evaluation():
    """T = 0 leaves Y = tanh(alpha) * SiLU(X A) B  (Sec. 2.3): numpy + scipy.expit in fp64."""
    c = _case(13, 6, 80, 48, 12, lora_std=0.3)
    T0 = np.zeros_like(c["T"])
    out = orc.linear_forward(c["x"], T0, c["s_w"], c["A"], c["B"], c["alpha"])
    x = c["x"].astype(np.float64)
    h = x @ c["A"].astype(np.float64).T
    h = h * expit(h)
    ref = np.tanh(c["alpha"].astype(np.float64))[None, :] * (h @ c["B"].astype(np.float64).T)
    assert np.allclose(out["y"], ref, rtol=1e-11, atol=1e-13)
    assert not out["acc"].any()
    assert np.abs(ref).max() > 1e-2                      # the check is not vacuous


def test_silu_limits_and_gate_sign():
    # one-hot token picks A[:, 0]; B = identity-like so y_corr[n] = SiLU(A[n, 0] * x0)
    r = 4
    x = np.zeros((1, 8), dtype=np.float16)
    x[0, 0] = 2.0
    A = np.zeros((r, 8), dtype=np.float16)
    A[:, 0] = [0.0, 10.0, -10.0, 0.5]                    # h = 0, 20, -20, 1
    B = np.eye(r, dtype=np.float16)
    alpha = np.array([5.0, 5.0, -5.0, 0.1], dtype=np.float16)
    T0 = np.zeros((r, 8), dtype=np.int8)
    y = orc.linear_forward(x, T0, 1.0, A, B, alpha)["y"][0]
    g = np.tanh(alpha.astype(np.float64))
    assert y[0] == 0.0                                   # SiLU(0) = 0
    assert abs(y[1] - g[1] * 20.0) < 1e-6                # SiLU(h) -> h
    assert abs(y[2]) < 1e-6                              # SiLU(-20) -> 0
    assert abs(y[3] - g[3] * 1.0 / (1.0 + math.exp(-1.0))) < 1e-12
    assert g[2] < 0 and abs(g[3] - 0.0997) < 2e-4        # fp16(0.1) is 0.09998


def test_swiglu_against_library_silu_and_limits():
    """z = SiLU(y_gate) * y_up against torch's silu (a library routine) in fp64, and the limits:
    y_gate = 0 gives 0; a large y_gate passes y_up through scaled by y_gate; a very negative one
    closes the gate.  The pair forward is the two single layers and this product."""
    import torch
    rng = np.random.default_rng(5)
    yg = rng.standard_normal((7, 33)) * 3.0
    yu = rng.standard_normal((7, 33)) * 2.0
    z = orc.swiglu(yg, yu)
    ref = (torch.nn.functional.silu(torch.from_numpy(yg)) * torch.from_numpy(yu)).numpy()
    assert np.allclose(z, ref, rtol=1e-13, atol=1e-15)
    edge = orc.swiglu(np.array([[0.0, 40.0, -40.0, 1.0]]), np.array([[5.0, 3.0, 3.0, 2.0]]))[0]
    assert edge[0] == 0.0 and abs(edge[1] - 120.0) < 1e-12 and abs(edge[2]) < 1e-14
    assert abs(edge[3] - 2.0 / (1.0 + math.exp(-1.0))) < 1e-15
    a = _case(31, 5, 96, 40, 8, lora_std=0.3)
    b = _case(32, 5, 96, 40, 16, lora_std=0.3)
    out = orc.swiglu_pair_forward(a["x"], a, b)
    ya = orc.linear_forward(a["x"], a["T"], a["s_w"], a["A"], a["B"], a["alpha"])["y"]
    yb = orc.linear_forward(a["x"], b["T"], b["s_w"], b["A"], b["B"], b["alpha"])["y"]
    assert np.allclose(out["z"], ya * expit(ya) * yb, rtol=1e-13, atol=1e-15)
    assert out["z16"].dtype == np.float16
    assert np.array_equal(out["amax"], np.abs(out["z"].astype(np.float16)).max(axis=1).astype(np.float32))
    # both layers were quantised from the same activations
    assert np.array_equal(out["gate"]["xq"], out["up"]["xq"])


def test_layernorm_against_library_and_special_cases():
    """The LayerNorm in front of the quantiser against torch's layer_norm in fp64 (a library
    routine), and what the definition fixes: zero mean and unit variance of the un-scaled
    output, a constant row mapping to beta exactly, rows normalised independently."""
    import torch
    rng = np.random.default_rng(9)
    M, K = 6, 333
    x = (rng.standard_normal((M, K)) * 3.0 + 1.5).astype(np.float16)
    gamma = (1.0 + 0.2 * rng.standard_normal(K)).astype(np.float32)
    beta = (0.3 * rng.standard_normal(K)).astype(np.float32)
    out = orc.layernorm(x, gamma, beta, 1e-5)
    assert out.dtype == np.float32
    ref = torch.nn.functional.layer_norm(torch.from_numpy(x.astype(np.float64)), (K,),
                                         torch.from_numpy(gamma.astype(np.float64)),
                                         torch.from_numpy(beta.astype(np.float64)), 1e-5).numpy()
    assert np.allclose(out, ref, rtol=2e-6, atol=2e-6)
    plain = orc.layernorm(x, np.ones(K, np.float32), np.zeros(K, np.float32), 1e-5).astype(np.float64)
    assert np.abs(plain.mean(axis=1)).max() < 1e-6 and np.abs(plain.var(axis=1) - 1.0).max() < 1e-4
    const = np.full((1, K), 2.5, dtype=np.float16)
    assert np.array_equal(orc.layernorm(const, gamma, beta, 1e-5)[0], beta)
    x2 = x.copy()
    x2[3] = x2[3] * np.float16(2.0) + np.float16(1.0)
    out2 = orc.layernorm(x2, gamma, beta, 1e-5)
    keep = [i for i in range(M) if i != 3]
    assert np.array_equal(out2[keep], out[keep])
    # a shifted and scaled row normalises to (nearly) the same values: eps is all that differs
    assert np.allclose(out2[3], out[3], rtol=0, atol=5e-3)


def test_layer_with_layernorm_quantises_the_normalised_input_only():
    """With ln set, the backbone contracts Q(layernorm(x)) (checked against numpy's own LayerNorm
    inside the quantiser's error bound of half a step) while the correction path still reads x:
    y_corr is unchanged, y_tern is the dense product of the de-quantised normalised input."""
    c = _case(41, 5, 200, 48, 8, act="student_t3", lora_std=0.3)
    rng = np.random.default_rng(41)
    gamma = (1.0 + 0.3 * rng.standard_normal(200)).astype(np.float32)
    beta = (0.2 * rng.standard_normal(200)).astype(np.float32)
    base = orc.linear_forward(c["x"], c["T"], c["s_w"], c["A"], c["B"], c["alpha"])
    out = orc.linear_forward(c["x"], c["T"], c["s_w"], c["A"], c["B"], c["alpha"], ln=(gamma, beta, 1e-5))
    assert np.array_equal(out["y_corr"], base["y_corr"])
    assert not np.array_equal(out["xq"], base["xq"])
    xf = c["x"].astype(np.float64)
    mu, var = xf.mean(axis=1, keepdims=True), xf.var(axis=1, keepdims=True)
    v = (xf - mu) / np.sqrt(var + 1e-5) * gamma.astype(np.float64) + beta.astype(np.float64)
    s_x = out["s_x"].astype(np.float64)[:, None]
    assert np.allclose(s_x[:, 0] * 127.0, np.abs(v).max(axis=1), rtol=1e-5)
    assert (np.abs(v - out["xq"].astype(np.float64) * s_x) <= 0.5 * s_x * (1 + 1e-3) + 1e-5).all()
    w_hat = c["T"].astype(np.float64) * float(c["s_w"])
    assert np.allclose(out["y_tern"], (out["xq"].astype(np.float64) * s_x) @ w_hat.T, rtol=1e-12, atol=1e-14)
    assert np.allclose(out["y"], out["y_tern"] + np.tanh(c["alpha"].astype(np.float64))[None, :] * out["y_corr"],
                       rtol=1e-13, atol=1e-15)


def test_diff_attention_against_library_attention_and_special_cases():
    """The differential-attention decode step against torch's scaled_dot_product_attention (a
    library routine; the last row of a causal attention is the decode step), and the cases the
    definition fixes: identical branches give (1 - lambda)/2 times ordinary attention, a single
    cached position returns (1 - lambda)/2 times its value row, equal keys average the values."""
    import torch
    rng = np.random.default_rng(17)
    B, L, H, d = 2, 37, 3, 16
    q = rng.standard_normal((B, 2 * H, d)).astype(np.float16)
    k = rng.standard_normal((B, L, 2 * H, d)).astype(np.float16)
    v = rng.standard_normal((B, L, H, d)).astype(np.float16)
    lens = [L, 11]
    lam = 0.37
    out = orc.diff_attention_decode(q, k, v, lens, lam)
    for b in range(B):
        n = lens[b]
        tq = torch.from_numpy(q[b].astype(np.float64))[:, None, :]                     # [2H, 1, d]
        tk = torch.from_numpy(k[b, :n].astype(np.float64)).permute(1, 0, 2)            # [2H, n, d]
        tv = torch.from_numpy(v[b, :n].astype(np.float64)).permute(1, 0, 2)            # [H, n, d]
        a1 = torch.nn.functional.scaled_dot_product_attention(tq[:H], tk[:H], tv)[:, 0].numpy()
        a2 = torch.nn.functional.scaled_dot_product_attention(tq[H:], tk[H:], tv)[:, 0].numpy()
        assert np.allclose(out[b], (a1 - lam * a2) * 0.5, rtol=1e-12, atol=1e-14)
    q2, k2 = q.copy(), k.copy()
    q2[:, H:], k2[:, :, H:] = q2[:, :H], k2[:, :, :H]                                   # both branches alike
    same = orc.diff_attention_decode(q2, k2, v, [L, L], lam)
    one = orc.diff_attention_decode(q2, k2, v, [L, L], 0.0)                             # lambda 0: half of branch 1
    assert np.allclose(same, (1 - lam) * one, rtol=1e-12, atol=1e-14)
    single = orc.diff_attention_decode(q, k, v, [1, 1], lam)
    assert np.allclose(single, (1 - lam) * 0.5 * v[:, 0].astype(np.float64), rtol=1e-12)
    k3 = np.broadcast_to(k[:, :1], k.shape).copy()                                      # every key alike
    avg = orc.diff_attention_decode(q, k3, v, [L, L], lam)
    assert np.allclose(avg, (1 - lam) * 0.5 * v.astype(np.float64).mean(axis=1), rtol=1e-10, atol=1e-12)
    assert orc.diff_attention_lambda_init(0) == pytest.approx(0.2) and orc.diff_attention_lambda_init(64) == pytest.approx(0.8, abs=1e-8)
    assert orc.diff_attention_lambda_init(2) == pytest.approx(0.8 - 0.6 * math.exp(-0.6))


def test_stack_is_the_chain_of_fp16_rounded_layers():
    a = _case(21, 3, 64, 48, 8)
    b = _case(22, 3, 48, 32, 8)
    slots = orc.stack_forward([a, b], [(0, 1), (1, 2)], a["x"])
    y1 = orc.linear_forward(a["x"], a["T"], a["s_w"], a["A"], a["B"], a["alpha"])["y16"]
    y2 = orc.linear_forward(y1, b["T"], b["s_w"], b["A"], b["B"], b["alpha"])["y16"]
    assert np.array_equal(slots[1], y1) and np.array_equal(slots[2], y2)
    assert slots[1].dtype == np.float16


def test_synth_configs_match_the_benchmark_shapes():
    c4 = synth.CONFIGS[4]
    assert [(p.name, p.d_in, p.d_out) for p in c4.projections] == [
        ("up", 4096, 11008), ("gate", 4096, 11008), ("down", 11008, 4096)]
    w, inputs = synth.stack_wiring(1)
    assert len(w) == 56 and inputs == {0: 0}
    assert w[0][2:] == (0, 1) and w[3][2] == w[2][3] and w[6][2] == w[4][3] and w[7][2] == w[6][3]
    w2, inputs2 = synth.stack_wiring(1, chained=False)
    assert len(w2) == 56 and len(inputs2) == 8 and w2[7][2] in inputs2 and w2[7][2] != w2[6][3]
