"""Python face of the CPU oracle (TEST INFRASTRUCTURE, not the product).

Thin ctypes marshalling around ``hgf_oracle.c`` plus the closed-form helpers the
paper states (parameter ratio of the correction path, effective bit-width,
memory-wall throughput bound, theoretical speed-up).  Only the tests, the smoke
check and the benchmark's CPU-baseline leg import this module; the HIP library
and its binding never do.

Layouts are the mathematical ones: T is an int8 matrix [d_out, d_in] holding
-1/0/+1, A is [r, d_in], B is [d_out, r], alpha is [d_out]; nothing is packed.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hgf_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
MAX_RANK = 1024


def build(force: bool = False) -> str:
    """Compile hgf_oracle.c with gcc (plain -O2, OpenMP over output rows)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    """Threads the OpenMP loops of the oracle use (OMP_NUM_THREADS or the core count)."""
    v = os.environ.get("OMP_NUM_THREADS")
    if v:
        try:
            return max(1, int(v.split(",")[0]))
        except ValueError:
            pass
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:
        return os.cpu_count() or 1


# --------------------------------------------------------------------------- steps

def ternarize(W: np.ndarray) -> Tuple[np.ndarray, np.float32]:
    """Absmean ternarisation (Sec. 2.2, weight-quantisation definition) -> (T int8, gamma_W)."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    N, K = W.shape
    T = np.empty((N, K), dtype=np.int8)
    g = ctypes.c_float(0.0)
    _load().hgf_oracle_ternarize(_p(W), ctypes.c_long(N), ctypes.c_long(K), _p(T), ctypes.byref(g))
    return T, np.float32(g.value)


def layernorm(x: np.ndarray, gamma: np.ndarray, beta: np.ndarray, eps: float = 1e-5) -> np.ndarray:
    """LayerNorm of fp16 activations in fp32 (appendix implementation, BitLinear forward) -> fp32 [M, K]."""
    assert x.dtype == np.float16
    M, K = x.shape
    xf = np.ascontiguousarray(x.astype(np.float32))
    g = np.ascontiguousarray(gamma, dtype=np.float32)
    b = np.ascontiguousarray(beta, dtype=np.float32)
    assert g.shape == (K,) and b.shape == (K,)
    out = np.empty((M, K), dtype=np.float32)
    _load().hgf_oracle_layernorm(_p(xf), ctypes.c_long(M), ctypes.c_long(K), _p(g), _p(b),
                                 ctypes.c_float(float(eps)), _p(out))
    return out


def quantize_act(x: np.ndarray, allow_f32: bool = False) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Per-token absmax int8 quantisation (Algorithm 1 steps 1-2) -> (x_q, s_x, rowsum).
    allow_f32: the input is the fp32 output of layernorm() rather than fp16 activations."""
    assert x.dtype == np.float16 or (allow_f32 and x.dtype == np.float32), \
        "activations are fp16 (Sec. 2.1, input tensor definition)"
    M, K = x.shape
    xf = np.ascontiguousarray(x.astype(np.float32))
    xq = np.empty((M, K), dtype=np.int8)
    s_x = np.empty(M, dtype=np.float32)
    rowsum = np.empty(M, dtype=np.int32)
    _load().hgf_oracle_quantize_act(_p(xf), ctypes.c_long(M), ctypes.c_long(K), _p(xq), _p(s_x),
                                    _p(rowsum))
    return xq, s_x, rowsum


def int_gemm(T: np.ndarray, xq: np.ndarray) -> np.ndarray:
    """Exact int32 accumulators acc[m, n] = sum_k T[n, k] * x_q[m, k] (Algorithm 1 step 3)."""
    T = np.ascontiguousarray(T, dtype=np.int8)
    xq = np.ascontiguousarray(xq, dtype=np.int8)
    N, K = T.shape
    M, K2 = xq.shape
    assert K == K2
    acc = np.empty((M, N), dtype=np.int32)
    _load().hgf_oracle_int_gemm(_p(T), _p(xq), ctypes.c_long(M), ctypes.c_long(N),
                                ctypes.c_long(K), _p(acc))
    return acc


def int_gemm_dense(T: np.ndarray, xq: np.ndarray) -> np.ndarray:
    """The same accumulators as int_gemm for the full-size configurations, where the triple
    loop takes minutes: the product of the two integer-valued matrices by the BLAS matmul
    in fp32.  Exact, whatever order the library sums in: every partial sum is an integer
    of magnitude <= 127 K, and integers below 2^24 are fp32 numbers.  Pinned against the
    triple loop on small shapes and on the extreme accumulator by the CPU tests."""
    N, K = T.shape
    M, K2 = xq.shape
    assert K == K2 and 127 * K < (1 << 24)
    acc = xq.astype(np.float32) @ np.ascontiguousarray(T.astype(np.float32).T)
    return acc.astype(np.int32)


def linear_forward(x: np.ndarray, T: np.ndarray, s_w, A: Optional[np.ndarray],
                   B: Optional[np.ndarray], alpha: Optional[np.ndarray],
                   dense_gemm: bool = False, ln: Optional[Tuple] = None) -> Dict[str, np.ndarray]:
    """Algorithm 1 for one layer.  Returns y (fp64), y16 (its fp16 rounding), the
    integer intermediates (x_q, s_x, rowsum, acc) and both paths (y_tern, y_corr).
    dense_gemm: take step 3 from int_gemm_dense (full-size cases) instead of the loop.
    ln = (gamma, beta, eps): the backbone quantises layernorm(x) (the appendix
    implementation's BitLinear); the correction path still reads x itself."""
    M, K = x.shape
    N = T.shape[0]
    r = 0 if A is None else A.shape[0]
    assert r <= MAX_RANK
    if ln is None:
        xq, s_x, rowsum = quantize_act(x)
    else:
        xq, s_x, rowsum = quantize_act(layernorm(x, ln[0], ln[1], ln[2]), allow_f32=True)
    acc = int_gemm_dense(T, xq) if dense_gemm else int_gemm(T, xq)
    xf = np.ascontiguousarray(x.astype(np.float32))
    Af = None if r == 0 else np.ascontiguousarray(A.astype(np.float32))
    Bf = None if r == 0 else np.ascontiguousarray(B.astype(np.float32))
    al = None if r == 0 else np.ascontiguousarray(alpha.astype(np.float32))
    if r:
        assert Af.shape == (r, K) and Bf.shape == (N, r) and al.shape == (N,)
    y = np.empty((M, N), dtype=np.float64)
    yt = np.empty((M, N), dtype=np.float64)
    yc = np.empty((M, N), dtype=np.float64)
    _load().hgf_oracle_epilogue(_p(xf), _p(acc), _p(s_x), ctypes.c_float(float(s_w)), _p(Af), _p(Bf),
                                _p(al), ctypes.c_long(M), ctypes.c_long(N), ctypes.c_long(K),
                                ctypes.c_long(r), _p(y), _p(yt), _p(yc))
    return {"y": y, "y16": y.astype(np.float16), "xq": xq, "s_x": s_x, "rowsum": rowsum,
            "acc": acc, "y_tern": yt, "y_corr": yc}


def swiglu(y_gate: np.ndarray, y_up: np.ndarray) -> np.ndarray:
    """z = SiLU(y_gate) * y_up elementwise in fp64 (appendix implementation, block forward)."""
    yg = np.ascontiguousarray(y_gate, dtype=np.float64)
    yu = np.ascontiguousarray(y_up, dtype=np.float64)
    assert yg.shape == yu.shape and yg.ndim == 2
    z = np.empty_like(yg)
    _load().hgf_oracle_swiglu(_p(yg), _p(yu), ctypes.c_long(yg.shape[0]), ctypes.c_long(yg.shape[1]), _p(z))
    return z


def swiglu_pair_forward(x: np.ndarray, gate: Dict, up: Dict, dense_gemm: bool = False) -> Dict[str, np.ndarray]:
    """The gated pair of the paper's MLP: both HGF linears (Algorithm 1) on the same x, then
    z = SiLU(y_gate) * y_up on their UN-rounded outputs; z16 is z rounded to fp16 once, amax the
    per-token max |z16| (step 1 of Algorithm 1 for the layer that reads z16), as fp32.
    `gate` and `up` hold T, s_w, A, B, alpha."""
    g = linear_forward(x, gate["T"], gate["s_w"], gate.get("A"), gate.get("B"), gate.get("alpha"), dense_gemm)
    u = linear_forward(x, up["T"], up["s_w"], up.get("A"), up.get("B"), up.get("alpha"), dense_gemm)
    z = swiglu(g["y"], u["y"])
    z16 = z.astype(np.float16)
    return {"z": z, "z16": z16, "amax": np.abs(z16).max(axis=1).astype(np.float32),
            "gate": g, "up": u}


def diff_attention_lambda_init(d: int) -> float:
    """Sec. 2.4, Def. "Differential Attention": lambda_0 = 0.8 - 0.6 exp(-0.3 d)."""
    return 0.8 - 0.6 * math.exp(-0.3 * d)


def diff_attention_decode(q: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray, lens: Sequence[int],
                          lam: float) -> np.ndarray:
    """One decode step of differential attention in fp64, written out head by head.
    Sec. 2.4, Def. "Differential Attention":
        O = (softmax(Q1 K1^T / sqrt(d_h)) - lambda softmax(Q2 K2^T / sqrt(d_h))) V,
    with what the appendix implementation fixes: q, k hold 2H heads (0..H-1 branch 1, H..2H-1
    branch 2) of d_h columns, v holds H heads of d_h columns, head h of both branches reads head
    h of v, and the difference is multiplied by 0.5.  The newest token of sequence b attends
    to the cached positions 0 .. lens[b]-1.
    q [B, 2H, d_h], k_cache [B, L, 2H, d_h], v_cache [B, L, H, d_h] -> [B, H, d_h] fp64."""
    B, L, H2, d_h = k_cache.shape
    H = H2 // 2
    out = np.zeros((B, H, d_h), dtype=np.float64)
    for b in range(B):
        n = int(lens[b])
        if n == 0:
            continue
        for h in range(H):
            a = []
            for head in (h, H + h):
                s = k_cache[b, :n, head, :].astype(np.float64) @ q[b, head, :].astype(np.float64) / math.sqrt(d_h)
                e = np.exp(s - s.max())
                pr = e / e.sum()
                a.append(pr @ v_cache[b, :n, h, :].astype(np.float64))
            out[b, h] = (a[0] - lam * a[1]) * 0.5
    return out


def stack_forward(layers: Sequence[Dict], wiring: Sequence[Tuple[int, int]],
                  x0: np.ndarray) -> List[np.ndarray]:
    """A chain of HGF linears: layer i reads slot wiring[i][0] and writes slot
    wiring[i][1]; each layer's fp16-rounded output is what the next one reads.
    `layers[i]` holds T, s_w, A, B, alpha.  Returns the list of slots (fp16)."""
    n_slots = 1 + max(max(s, d) for s, d in wiring)
    slots: List[Optional[np.ndarray]] = [None] * n_slots
    slots[0] = x0
    for L, (src, dst) in zip(layers, wiring):
        out = linear_forward(slots[src], L["T"], L["s_w"], L.get("A"), L.get("B"), L.get("alpha"))
        slots[dst] = out["y16"]
    return slots


# ---------------------------------------------------- closed forms stated by the paper

def lora_param_ratio(d_in: int, d_out: int, r: int) -> float:
    """N_LoRA / N of Sec. 5.2: correction-path parameters over backbone parameters."""
    return r * (d_in + d_out) / float(d_in * d_out)


def effective_bit_width(g: float, r: int, d: int, b_corr: float = 16.0) -> float:
    """Sec. 4.1, Def. "Effective Bit-Width": log2(3) + g * b_corr * r / d."""
    return math.log2(3.0) + g * b_corr * r / d


def memory_wall_tokens_per_s(bandwidth_bytes_per_s: float, params: float, bits: float) -> float:
    """Sec. 1, memory-bandwidth bound: T_max = B_mem / (P * b / 8)."""
    return bandwidth_bytes_per_s / (params * bits / 8.0)


def theoretical_speedup(cmul_over_cadd: float, lora_ratio: float) -> float:
    """Sec. 5.2: N c_mul / (N c_add + N_LoRA c_mul)."""
    return cmul_over_cadd / (1.0 + lora_ratio * cmul_over_cadd)


def gate(alpha: float) -> float:
    """Sec. 2.3.1: g(alpha) = tanh(alpha)."""
    return math.tanh(alpha)


def layer_bytes(d_in: int, d_out: int, r: int) -> Dict[str, float]:
    """Bytes of one layer's parameters: dense fp16, 2-bit backbone, and the
    correction path (A, B in fp16 plus one fp16 gate per output channel)."""
    return {"fp16_dense": 2.0 * d_in * d_out,
            "ternary_2bit": d_in * d_out / 4.0,
            "correction": 2.0 * r * (d_in + d_out) + 2.0 * d_out}
