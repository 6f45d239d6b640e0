"""Frequency-ablation tools (Sec. 3.2): the library's greedy mask (host integer work, runs without a GPU)
is bit-exact against the oracle; the device ablation routine is compared element by element."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import iwdft_oracle as orc
from paper_2507_20030_amd import binding as B


def _delta(seed, layers, C):
    r = np.random.default_rng(seed)
    d = r.normal(size=(layers, C)).astype(np.float32)
    d[1 % layers, :] = 0.5                       # every chunk equal
    d[2 % layers, [1, C // 2, C - 1]] = 9.0      # three-way tie at the top
    d[3 % layers, 0] = -np.inf
    d[4 % layers, C - 1] = np.inf
    return d


@pytest.mark.parametrize("M,C", [(8192, 22), (8252 - 60, 22), (1024, 22), (131072, 22), (1000, 7), (64, 64), (40, 3)])
@pytest.mark.parametrize("r", [0.094, 0.125, 0.25, 0.1, 0.5, 1.0, 0.0, 0.999, 3.0])
def test_select_bins_is_bit_exact_against_the_oracle(M, C, r):
    delta = _delta(M + C, 6, C)
    got = B.iwdft_select_bins(delta, M, r)
    ref = orc.select_bins(delta, M, r)
    assert len(got) == len(ref)
    for g, e in zip(got, ref):
        assert g.dtype == np.int32 and np.array_equal(g, e)


def test_select_bins_lists_are_valid_descriptor_input():
    delta = _delta(7, 4, 22)
    bins = B.iwdft_select_bins(delta, 8192, 0.25)
    d = B.Descriptor(4, 1, 2, 4, 128, B.IWDFT_BF16, 8192, bins)
    state, ws = B.iwdft_query_bytes(d)
    assert state > 0 and ws > 0
    assert all(len(b) > 0 and np.all(np.diff(b) > 0) for b in bins)


def test_select_bins_errors():
    lib = B.load_library()
    delta = np.zeros((2, 4), np.float32)
    dp = delta.ctypes.data_as(ctypes.POINTER(ctypes.c_float))
    off = (ctypes.c_int64 * 3)()
    bins = (ctypes.c_int32 * 64)()
    assert lib.iwdft_select_bins(None, 2, 4, 64, 0.5, off, bins, 64) == B.IWDFT_ERR_ARG
    assert lib.iwdft_select_bins(dp, 2, 4, 64, 0.5, None, bins, 64) == B.IWDFT_ERR_ARG
    assert lib.iwdft_select_bins(dp, 0, 4, 64, 0.5, off, bins, 64) == B.IWDFT_ERR_ARG
    assert lib.iwdft_select_bins(dp, 2, 0, 64, 0.5, off, bins, 64) == B.IWDFT_ERR_ARG
    assert lib.iwdft_select_bins(dp, 2, 4, 0, 0.5, off, bins, 64) == B.IWDFT_ERR_ARG
    assert lib.iwdft_select_bins(dp, 2, 4, 64, -0.1, off, bins, 64) == B.IWDFT_ERR_ARG
    assert lib.iwdft_select_bins(dp, 2, 4, 64, float("nan"), off, bins, 64) == B.IWDFT_ERR_ARG
    assert lib.iwdft_select_bins(dp, 2, 4, 64, 0.5, off, None, 64) == B.IWDFT_ERR_ARG
    assert lib.iwdft_select_bins(dp, 2, 4, 64, 0.5, off, bins, 63) == B.IWDFT_ERR_SIZE   # 2 layers x 32 bins
    assert list(off) == [0, 32, 64]                                                   # sizes are reported anyway
    assert lib.iwdft_select_bins(dp, 2, 4, 64, 0.5, off, bins, 64) == B.IWDFT_OK
    assert list(bins[:32]) == list(range(32))                                          # equal deltas: chunks 0, 1
    delta[1, 2] = np.nan
    assert lib.iwdft_select_bins(dp, 2, 4, 64, 0.5, off, bins, 64) == B.IWDFT_ERR_ARG
    delta[1, 2] = 0.0
    assert lib.iwdft_select_bins(dp, 2, 4, 2, 0.25, off, bins, 64) == B.IWDFT_ERR_BINS   # chunk 0 of M=2, C=4 is empty


def test_ablate_chunk_argument_errors_need_no_gpu():
    lib = B.load_library()
    p = ctypes.c_void_p(4096)
    q = ctypes.c_void_p(1 << 40)
    f = lib.iwdft_ablate_chunk
    assert f(None, q, 1, 1024, 128, 0, 22, 0, None) == B.IWDFT_ERR_ARG
    assert f(p, q, -1, 1024, 128, 0, 22, 0, None) == B.IWDFT_ERR_ARG
    assert f(p, q, 1, 1024, 128, 5, 22, 0, None) == B.IWDFT_ERR_ARG
    assert f(p, q, 1, 1024, 128, 0, 22, 22, None) == B.IWDFT_ERR_ARG
    assert f(p, q, 1, 1024, 128, 0, 0, 0, None) == B.IWDFT_ERR_ARG
    assert f(p, q, 1, 1024, 64, 0, 22, 0, None) == B.IWDFT_ERR_UNSUPPORTED
    assert f(p, q, 1, 1000, 128, 0, 22, 0, None) == B.IWDFT_ERR_UNSUPPORTED
    assert f(p, q, 1, 128, 128, 0, 22, 0, None) == B.IWDFT_ERR_UNSUPPORTED
    assert f(p, q, 1, 1 << 25, 128, 0, 22, 0, None) == B.IWDFT_ERR_UNSUPPORTED
    assert f(p, ctypes.c_void_p(4096 + 64), 1, 1024, 128, 0, 22, 0, None) == B.IWDFT_ERR_ARG   # overlap
    assert f(p, q, 0, 1024, 128, 0, 22, 0, None) == B.IWDFT_OK                                 # nothing to do


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("M,C,chunks", [(256, 22, (0, 7, 21)), (512, 5, (2,)), (1024, 22, (0, 11)), (2048, 1, (0,)),
                                        (4096, 22, (3,)), (8192, 22, (0, 10, 21)),
                                        # longer than one in-LDS transform: the subtractive form, in pieces
                                        (16384, 1, (0,)), (16384, 3, (0, 2)), (32768, 22, (0, 10, 21)),
                                        (131072, 22, (7,))])   # the study's chunking at the longest baseline context
def test_ablate_chunk_matches_the_oracle(dtype, M, C, chunks):
    dev = "cuda:0"
    g = torch.Generator(device=dev).manual_seed(M + C)
    shape = (3, 2, M, 128)   # e.g. (layers, heads): 6 slices
    scale = 10.0 ** (2 * torch.rand((3, 2, 1, 128), generator=g, device=dev) - 1)
    x = (torch.randn(shape, generator=g, device=dev) * scale).to(dtype)
    out = torch.empty_like(x)
    xh = x.detach().cpu().to(torch.float64).numpy()
    for c in chunks:
        out.fill_(float("nan"))
        B.iwdft_ablate_chunk(x, out, C, c)
        torch.cuda.synchronize()
        got = out.detach().cpu().to(torch.float64).numpy()
        for s in [(0, 0), (1, 1), (2, 0)]:
            ref = orc.ablate_chunk(xh[s], C, c)
            # one chunk holding every bin leaves nothing: the error is then measured against the input
            den = np.linalg.norm(ref) if C > 1 else np.linalg.norm(xh[s])
            err = np.linalg.norm(got[s] - ref) / max(den, 1e-30)
            # fp32 transforms: ~1e-6; bf16 output rounding alone is 2^-9 per element
            assert err < (1e-4 if dtype == torch.float32 else 4e-3), f"M={M} C={C} chunk={c} slice={s}: {err:.3e}"
        if C == 1:
            # a chunk of more than 4096 bins is taken off in pieces, and bf16 rounds what is left between them
            pieces = -(-(M // 2 + 1) // 4096) if M > 8192 else 1
            bar = 1e-3 if (dtype == torch.float32 or pieces == 1) else pieces * 2.0 ** -8
            assert float(out.float().abs().max()) < bar * float(x.float().abs().max())
