"""tman_build_lut against the oracle's tables."""
import numpy as np
import pytest
import torch

import oracle
import synth
from gpu_helpers import build_lut

pytestmark = pytest.mark.gpu


def _ulp_diff(a16, b16):
    """distance in fp16 representable steps (same-sign finite values)"""
    def key(v):
        u = v.view(np.uint16).astype(np.int32)
        return np.where(u & 0x8000, -(u & 0x7FFF), u & 0x7FFF)
    return np.abs(key(a16) - key(b16))


@pytest.mark.parametrize("N,K,group", [(1, 512, 64), (3, 4096, 128), (8, 1024, 32), (1, 96, 32), (5, 11008, 64), (2, 2816, 64)])
def test_tables_and_group_sums(oracle_lib, N, K, group):
    x = synth.normal_fp16(900 + N + K, N * K).reshape(N, K)
    x[0, : min(K, 8)] = np.array([0, -0.0, 1, -1, 65504, 6e-8, -6e-5, 100], dtype=np.float16)[: min(K, 8)]
    buf = build_lut(x, group)
    torch.cuda.synchronize()
    raw = buf.cpu().numpy()
    T, S = oracle.lut_layout_decode(raw, N, K, group)
    Tref = oracle.build_tables(x, 4)  # exact sums in double
    with np.errstate(over="ignore"):
        Tref16 = Tref.astype(np.float16)
    finite = np.isfinite(Tref16.astype(np.float32))
    d = _ulp_diff(T[finite], Tref16[finite])
    assert d.max() <= 1, "table entry differs by more than one fp16 step from the correctly rounded sum"
    assert (d == 0).mean() > 0.999
    assert np.array_equal(np.isinf(T.astype(np.float32)), ~finite)
    # pattern 0 is exactly zero, single-bit patterns are the activations themselves
    assert np.all(T[:, :, 0] == 0)
    for t in range(4):
        assert np.array_equal(T[:, :, 1 << t], x.reshape(N, K // 4, 4)[:, :, t])  # by value: 0 + (-0) is +0
    Sref = x.astype(np.float64).reshape(N, K // group, group).sum(axis=2)
    scale = np.abs(x.astype(np.float64)).reshape(N, K // group, group).sum(axis=2)
    assert np.all(np.abs(S - Sref) <= 1e-5 * scale + 1e-30)
    # padding (tokens beyond N, columns beyond K) is zero
    NP = 1 if N == 1 else 2 if N == 2 else 4 if N <= 4 else 8
    nkt = -(-K // 128)
    allT, _ = oracle.lut_layout_decode(raw, NP, nkt * 128, group)  # every padded token and column
    assert np.all(allT[N:, :, :] == 0)
    assert np.all(allT[:, K // 4:, :] == 0)


def test_batched_build_matches_single_calls(oracle_lib):
    """One launch for several activations writes the same bytes as separate calls."""
    import paper_2511_11248_amd as tman
    from gpu_helpers import dev, to_dev

    N, group = 3, 64
    Ks = [512, 4096, 11008, 64, 128, 2816, 192, 1024, 64, 320, 8192]  # more than one launch's worth of jobs
    xs = [to_dev(synth.normal_fp16(990 + i, N * K).reshape(N, K)) for i, K in enumerate(Ks)]
    single = [build_lut(x, group) for x in xs]
    luts = [torch.full((tman.tman_lut_bytes(N, K, group),), 0x77, dtype=torch.uint8, device=dev()) for K in Ks]
    tman.tman_build_lut_batch(xs, N, Ks, group, luts)
    torch.cuda.synchronize()
    for a, b in zip(single, luts):
        assert torch.equal(a, b)
