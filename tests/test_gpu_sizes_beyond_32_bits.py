"""Tensors whose element or byte offsets do not fit 32 bits, on the GPU against the oracle.

The tuned kernels index with 32-bit offsets where that is enough and the dispatcher routes larger
tensors to kernels that index with 64 bits (Sec. 2.1.1 and 2.1.2 state the operations for any
size).  These cases are the only ones that run those routes at sizes where a 32-bit offset
would wrap: a bit-pack of more than 2^31 elements (both kernels), a convolution whose packed
activations and whose output are larger than 4 GiB each, and a BGEMM with such an A and C.
"""
import numpy as np
import pytest
import torch

from paper_1908_05858_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dabnn():
    from paper_1908_05858_amd import binding
    binding.load()
    return binding


def tiled_activations(n_pixels, C, seed):
    """[n_pixels, C] fp32: a seeded block of 8191 pixels (a prime: no power-of-two offset error maps
    a pixel onto an equal one) with +-0.0 sprinkled in, repeated."""
    block = wl.inject_zeros(wl.activations((8191, C), seed), seed + 1)
    reps = (n_pixels + 8190) // 8191
    return np.tile(block, (reps, 1))[:n_pixels]


@pytest.mark.parametrize("C", [128, 129])
def test_bitpack_more_than_2_to_31_elements(dabnn, oracle, C):
    n_pixels = (1 << 31) // C + 4099          # C = 129: three words per pixel, the last one bit long
    assert n_pixels * C > (1 << 31)
    print("bitpack", n_pixels, "x", C, "=", n_pixels * C, "elements", flush=True)
    x = tiled_activations(n_pixels, C, 7100 + C)
    want = oracle.bitpack(x)
    xg = torch.from_numpy(x).cuda()
    del x
    got = dabnn.bitpack(xg)
    del xg
    assert got.shape == want.shape
    assert np.array_equal(got.cpu().numpy().view(np.uint64), want)


def window_signs(a_words, hs, ws, H, W):
    """+-1 float windows [S, 3, 3, 64*Cw] under the outputs (hs, ws) of a 3x3, stride 1, pad 1
    convolution over packed words [H, W, Cw]: bit 1 is -1, a tap outside the image is +1."""
    S, Cw = len(hs), a_words.shape[-1]
    out = np.ones((S, 3, 3, 64 * Cw), dtype=np.float32)
    for i in range(3):
        for j in range(3):
            hi, wi = hs - 1 + i, ws - 1 + j
            inside = (hi >= 0) & (hi < H) & (wi >= 0) & (wi < W)
            w = a_words[hi[inside], wi[inside]]                       # [S', Cw] uint64
            bits = np.unpackbits(w.view(np.uint8), axis=-1, bitorder="little")  # [S', 64*Cw], LSB first
            out[inside, i, j] = 1.0 - 2.0 * bits.astype(np.float32)
    return out


def test_conv_with_tensors_above_4_gib(dabnn, oracle):
    """1 x 8200 x 8200 x 512 -> 16: 4.30 GB of packed activations, 4.30 GB of int32 output.  The
    default route (not the activation-stationary family, whose offsets are 32-bit), the
    reference kernel and the fused threshold epilogue, on sampled outputs: corners, edges, the
    rows whose byte offsets lie above 2^32, and random positions."""
    H = W = 8200
    Cin, Cout, Cw = 512, 16, 8
    assert dabnn.pick_algo(1, H, W, Cin, Cout, 3, 3, 1, 1) != dabnn.ALGO_AREG
    rng = np.random.default_rng(7200)
    a_words = rng.integers(0, 1 << 64, size=(H, W, Cw), dtype=np.uint64)
    wf = wl.weights((Cout, 3, 3, Cin), 7201, 0.3)

    hs = [0, 0, H - 1, H - 1, 0, H - 1, 4100, 4100]
    ws = [0, W - 1, 0, W - 1, 4100, 4100, 0, W - 1]
    for h in range(8180, H):                      # pixel offsets * 64 bytes >= 2^32 from row 8184 on
        hs += [h] * 4
        ws += [0, 1, 4099, W - 1]
    hs = np.concatenate([np.array(hs), rng.integers(0, H, size=3000)])
    ws = np.concatenate([np.array(ws), rng.integers(0, W, size=3000)])
    windows = window_signs(a_words, hs, ws, H, W)
    want = oracle.bconv2d_signed(windows, oracle.sign(wf), 1, 0)[:, 0, 0, :]
    gamma = rng.uniform(-1.5, 1.5, Cout).astype(np.float32)
    beta = rng.normal(0, 0.5, Cout).astype(np.float32)
    mean = rng.normal(0, 30.0, Cout).astype(np.float32)
    var = rng.uniform(0.5, 40.0, Cout).astype(np.float32)
    want_bits = oracle.bconv2d_bnsign(windows, wf, gamma, beta, mean, var, 1e-5, 1, 0)[:, 0, 0, :]

    a = torch.from_numpy(a_words.view(np.int64)).cuda().view(1, H, W, Cw)
    del a_words
    wp = dabnn.pack_weights(torch.from_numpy(wf).cuda())
    hs_t, ws_t = torch.from_numpy(hs).cuda(), torch.from_numpy(ws).cuda()
    for algo in (dabnn.ALGO_AUTO, dabnn.ALGO_REFERENCE):
        print("conv above 4 GiB, algo", algo, flush=True)
        y = dabnn.bconv2d(a, wp, Cin, 1, 1, algo=algo)
        assert y.shape == (1, H, W, Cout)
        got = y[0, hs_t, ws_t, :].cpu().numpy()
        del y
        assert np.array_equal(got, want), algo
    # the fused threshold epilogue over the same activations (next-layer bits, Sec. 2.1.1)
    print("fused threshold above 4 GiB", flush=True)
    thr, flip = dabnn.bn_thresholds(gamma, beta, mean, var, 1e-5, 9 * Cin)
    bits = dabnn.bconv2d_bnsign(a, wp, thr, flip, Cin, 1, 1)
    assert bits.shape == (1, H, W, 1)
    assert np.array_equal(bits[0, hs_t, ws_t, :].cpu().numpy().view(np.uint64), want_bits)


def row_signs(words):
    """+-1 floats [S, 64*Kw] of packed rows [S, Kw]: bit 1 is -1, LSB first."""
    bits = np.unpackbits(np.ascontiguousarray(words).view(np.uint8), axis=-1, bitorder="little")
    return 1.0 - 2.0 * bits.astype(np.float32)


@pytest.mark.parametrize("mode", [0, 1], ids=["signed", "matches"])
def test_bgemm_with_matrices_above_4_gib(dabnn, oracle, mode):
    """Eq. 1 with A = 70,000,001 rows of 8 words (4.48 GB: past the fast kernel's 32-bit byte
    offsets, so the kernel that indexes with 64 bits runs) and 16 columns (4.48 GB of output):
    sampled rows, among them the first, the last and those around byte offset 2^32."""
    M, Kw, N = 70_000_001, 8, 16
    rng = np.random.default_rng(7300)
    A = rng.integers(0, 1 << 64, size=(M, Kw), dtype=np.uint64)
    B = rng.integers(0, 1 << 64, size=(N, Kw), dtype=np.uint64)
    wrap = (1 << 32) // (8 * Kw)                       # the row whose byte offset in A (and C) is 2^32
    rows = np.concatenate([np.array([0, 1, M - 2, M - 1, wrap - 1, wrap, wrap + 1]),
                           rng.integers(0, M, size=3000)])
    want = oracle.bgemm_signed(row_signs(A[rows]), row_signs(B), mode)
    Ag = torch.from_numpy(A.view(np.int64)).cuda()
    del A
    C = dabnn.bgemm(Ag, torch.from_numpy(B.view(np.int64)).cuda(), 64 * Kw, mode=mode)
    assert C.shape == (M, N)
    assert np.array_equal(C[torch.from_numpy(rows).cuda()].cpu().numpy(), want)
