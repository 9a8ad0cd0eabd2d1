"""GPU parity of the differential-attention decode step against the CPU oracle (fp64): fp16 outputs
within 2e-3 + 1e-2 |o| over head sizes 8 .. 128, ragged cache lengths (one position, chunk
boundaries, an empty sequence), several sequences, and the shapes of the paper's own model
(d = 512, 8 heads: q, k 16 heads of 32 columns, v 8 heads of 32) and of a 7B-shape one."""
import numpy as np
import pytest
import torch

from oracle import hgf_oracle as orc
from paper_2602_05269_amd import binding as hb
from parity import assert_close_fp16, dev

pytestmark = pytest.mark.gpu


def _case(seed, B, L, H, d, scale=1.0):
    rng = np.random.default_rng(seed)
    q = (scale * rng.standard_normal((B, 2 * H, d))).astype(np.float16)
    k = (scale * rng.standard_normal((B, L, 2 * H, d))).astype(np.float16)
    v = rng.standard_normal((B, L, H, d)).astype(np.float16)
    return q, k, v


@pytest.mark.parametrize("B,L,H,d,lens", [
    (1, 1, 1, 8, [1]), (2, 37, 3, 16, [37, 11]), (3, 300, 2, 32, [256, 257, 1]), (2, 512, 8, 32, [512, 100]),
    (2, 700, 4, 64, [700, 0]), (1, 1024, 2, 128, [1000]), (4, 130, 5, 64, [130, 129, 128, 2]),
])
def test_diff_attention_decode_parity(B, L, H, d, lens):
    q, k, v = _case(B * 1000 + L + H + d, B, L, H, d)
    lam = orc.diff_attention_lambda_init(2 * d)
    out = hb.hgf_diff_attention_decode(dev(q), dev(k), dev(v), dev(np.array(lens, dtype=np.int32)), lam)
    torch.cuda.synchronize()
    ref = orc.diff_attention_decode(q, k, v, lens, lam)
    assert_close_fp16(out.cpu().numpy(), ref, "attention output")
    assert np.abs(ref).max() > 1e-2


def test_diff_attention_peaked_scores_and_cache_beyond_len_ignored():
    """Large scores (a softmax close to one-hot, where the chunk maxima differ widely) and
    garbage behind lens in the caches: rows past the length must not matter, NaNs included."""
    B, L, H, d = 2, 600, 2, 32
    q, k, v = _case(5, B, L, H, d, scale=3.0)
    lens = [300, 513]
    for b, n in enumerate(lens):
        k[b, n:] = np.float16(np.nan)
        v[b, n:] = np.float16(np.inf)
    out = hb.hgf_diff_attention_decode(dev(q), dev(k), dev(v), dev(np.array(lens, dtype=np.int32)), 0.5)
    torch.cuda.synchronize()
    ref = orc.diff_attention_decode(q, k, v, lens, 0.5)
    assert_close_fp16(out.cpu().numpy(), ref, "attention output")


def test_diff_attention_model_shapes():
    # the paper's model: d = 512, 8 heads -> q, k: 16 heads of 32; v: 8 heads of 32; context 512
    q, k, v = _case(11, 4, 512, 8, 32)
    lens = [512, 400, 17, 256]
    lam = orc.diff_attention_lambda_init(64)
    out = hb.hgf_diff_attention_decode(dev(q), dev(k), dev(v), dev(np.array(lens, dtype=np.int32)), lam)
    assert_close_fp16(out.cpu().numpy(), orc.diff_attention_decode(q, k, v, lens, lam))
    # a 7B-shape block: d = 4096, 32 heads -> q, k: 64 heads of 64; v: 32 heads of 64; 4096 cached positions
    q, k, v = _case(12, 1, 4096, 32, 64)
    out = hb.hgf_diff_attention_decode(dev(q), dev(k), dev(v), dev(np.array([4096], dtype=np.int32)), 0.8)
    assert_close_fp16(out.cpu().numpy(), orc.diff_attention_decode(q, k, v, [4096], 0.8))


def test_diff_attention_rejects_bad_arguments():
    lib = hb.lib()
    assert lib.hgf_diff_attention_workspace_bytes(1, 128, 4, 24) == 0          # d_h not a power of two
    assert lib.hgf_diff_attention_workspace_bytes(1, 128, 4, 256) == 0
    assert lib.hgf_diff_attention_workspace_bytes(1, 1 << 20, 64, 128) == 0    # a sequence's cache beyond 2 GiB
    assert lib.hgf_diff_attention_decode(None, 0x100, 0x100, 0x100, 1, 8, 1, 8, 0.5, 0x100, 0x100, 1 << 20, None) == 1
    assert lib.hgf_diff_attention_decode(0x100, 0x100, 0x100, 0x100, 1, 8, 1, 12, 0.5, 0x100, 0x100, 1 << 20, None) == 2
    assert lib.hgf_diff_attention_decode(0x100, 0x104, 0x100, 0x100, 1, 8, 1, 8, 0.5, 0x100, 0x100, 1 << 20, None) == 3
    assert lib.hgf_diff_attention_decode(0x100, 0x100, 0x100, 0x100, 1, 8, 1, 8, 0.5, 0x100, 0x100, 16, None) == 5
