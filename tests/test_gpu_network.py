"""GPU parity of the network kernels (MFMA GEMM, attention, whole forward) against the oracle."""
import math
import numpy as np
import pytest
import torch

from oracle import dit
from paper_2512_15347_amd import workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print(msg, flush=True)


def bf16_dev(a):
    """fp32 host array of bf16-representable values -> int16 device tensor of bit patterns."""
    return torch.from_numpy(workloads.bf16_bits(a).view(np.int16)).to(DEV)


# the later shapes are sized so that the launcher's tile heuristic takes each of its tile heights (160, 192, 224,
# 256 rows, and the 128x128 tile) with a ragged last tile in both directions
@pytest.mark.parametrize("M,N,K", [(300, 200, 128), (2356, 384, 512), (256, 256, 64), (1, 16, 64), (777, 4608, 1536),
                                   (12251, 768, 128), (12251, 2304, 64), (12283, 3072, 128), (24571, 1532, 64),
                                   (18848, 1536, 64), (9001, 520, 192)])
def test_gemm_matches_oracle_linear(lib, M, N, K):
    say(f"gemm M={M} N={N} K={K}")
    rng = np.random.default_rng(M + N + K)
    A = workloads.bf16_round(rng.standard_normal((M, K), dtype=np.float32))
    W = workloads.bf16_round(rng.standard_normal((N, K), dtype=np.float32) * 0.05)
    b = workloads.bf16_round(rng.standard_normal(N, dtype=np.float32))
    out = torch.full((M, N), float("nan"), device=DEV)
    lib.pg_gemm_bf16(bf16_dev(A), K, bf16_dev(W), K, bf16_dev(b), out, N, M, N, K)
    torch.cuda.synchronize()
    want = dit.linear(A.astype(np.float64), W, b)
    got = out.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    # fp32 accumulation of exact bf16 products: error ~ sqrt(K) * 2^-24 * |a||w|
    assert np.max(np.abs(got - want)) < 2e-5 * math.sqrt(K) * np.max(np.abs(want)) + 1e-6


def test_gemm_rejects_bad_shapes(lib):
    A = torch.zeros(64, 96, dtype=torch.int16, device=DEV)
    out = torch.zeros(64, 64, device=DEV)
    with pytest.raises(lib.PgError):
        lib.pg_gemm_bf16(A, 96, A, 96, None, out, 64, 64, 64, 96)       # K not a multiple of 64
    lib.pg_gemm_bf16(A, 96, A, 96, None, out, 64, 0, 64, 64)           # empty: no-op


@pytest.mark.parametrize("B,Lq,Lk,heads,hd", [(2, 90, 90, 2, 64), (1, 64, 13, 2, 64), (3, 64, 64, 4, 32),
                                              (1, 300, 1178, 3, 64), (2, 130, 77, 2, 32)])
def test_attention_matches_oracle(lib, B, Lq, Lk, heads, hd):
    say(f"attention B={B} Lq={Lq} Lk={Lk} heads={heads} hd={hd}")
    rng = np.random.default_rng(Lq * 7 + Lk)
    D = heads * hd
    q = workloads.bf16_round(rng.standard_normal((B, Lq, D), dtype=np.float32) * 1.5)
    k = workloads.bf16_round(rng.standard_normal((B, Lk, D), dtype=np.float32))
    v = workloads.bf16_round(rng.standard_normal((B, Lk, D), dtype=np.float32))
    Lkpad = (Lk + 63) // 64 * 64
    vt = np.full((B, D, Lkpad), np.nan, dtype=np.float32)          # padding must be ignored, whatever it holds
    vt[:, :, :Lk] = v.transpose(0, 2, 1)
    out = torch.zeros(B, Lq, D, dtype=torch.int16, device=DEV)
    lib.pg_attention_bf16(bf16_dev(q), bf16_dev(k), bf16_dev(vt), out, B, Lq, Lk, heads, hd)
    torch.cuda.synchronize()
    got = out.view(torch.bfloat16).float().cpu().numpy().astype(np.float64)
    want = dit.attention(q.astype(np.float64), k.astype(np.float64), v.astype(np.float64), heads)
    assert np.isfinite(got).all()
    # probabilities and outputs are rounded to bf16 (2^-9 relative)
    assert np.max(np.abs(got - want)) < 1.5e-2 * np.max(np.abs(want))
    assert np.sqrt(np.mean((got - want) ** 2)) < 4e-3 * np.sqrt(np.mean(want ** 2))
