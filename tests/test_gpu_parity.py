"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle, bit-exactly.

Integer outputs and packed words are unique, so every comparison is `==` with zero tolerance.
Inputs are the seeded synthetic tensors of `workloads`; expected values always come from
`oracle/`, never from the GPU.
"""
import numpy as np
import pytest
import torch

from paper_1908_05858_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dabnn():
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: the gpu-marked tests need a real MI355X")
    from paper_1908_05858_amd import binding
    binding.load()
    return binding


@pytest.fixture
def option(dabnn):
    """Sets tuning/test options of the library for one test and restores the defaults after."""
    touched = []

    def set_(opt, value):
        touched.append(opt)
        dabnn.set_option(opt, value)
    yield set_
    for opt in touched:
        dabnn.set_option(opt, 0)


def gpu(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def words(t):
    return t.cpu().numpy().view(np.uint64)


# ------------------------------------------------------------------------------- bit-pack

@pytest.mark.parametrize("shape", wl.CFG3_SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("mode", [0, 1])
def test_bitpack_cfg3(dabnn, oracle, shape, mode):
    print("bitpack", shape, "mode", mode, flush=True)
    x = wl.inject_zeros(wl.activations(shape, wl.seed_for(3, shape[-1] + shape[0])), wl.seed_for(3, 1))
    got = words(dabnn.bitpack(gpu(x), sign_mode=mode))
    want = oracle.bitpack(x, mode)
    assert got.shape == want.shape
    assert np.array_equal(got, want)


@pytest.mark.parametrize("C", [1, 3, 63, 64, 65, 80, 127, 128, 200, 256, 1000])
@pytest.mark.parametrize("n_pixels", [1, 5, 63, 64, 1025])
def test_bitpack_ragged(dabnn, oracle, C, n_pixels):
    print("bitpack ragged", C, n_pixels, flush=True)
    x = wl.inject_zeros(wl.activations((n_pixels, C), 1000 + C + n_pixels), 17, frac=0.05)
    for mode in (0, 1):
        # guard words on both sides of the output catch out-of-bounds writes
        Cw = (C + 63) // 64
        buf = torch.full((n_pixels * Cw + 16,), 0x5A5A5A5A5A5A5A5A, dtype=torch.int64, device="cuda")
        out = buf[8:8 + n_pixels * Cw].view(n_pixels, Cw)
        dabnn.bitpack(gpu(x), out=out, sign_mode=mode)
        assert np.array_equal(words(out), oracle.bitpack(x, mode))
        assert torch.all(buf[:8] == 0x5A5A5A5A5A5A5A5A) and torch.all(buf[-8:] == 0x5A5A5A5A5A5A5A5A)


@pytest.mark.parametrize("kernel", [1, 2])
def test_bitpack_other_tail_kernels_forced(dabnn, oracle, option, kernel):
    """Channel counts that are not multiples of 64 default to the flat-stream kernel with 32-bit
    indices; the row-wise kernel (1) and the flat-stream kernel with 64-bit indices (2, otherwise
    used from 2^31 elements) on the same shapes through the library's option."""
    option(dabnn.OPT_BITPACK_ROWWISE, kernel)
    for n_pixels, C in [(1, 1), (5, 3), (63, 65), (1025, 80), (64, 200), (77, 1000), (4099, 129)]:
        x = wl.inject_zeros(wl.activations((n_pixels, C), 4300 + C), 4301 + C)
        for mode in (0, 1):
            assert np.array_equal(words(dabnn.bitpack(gpu(x), sign_mode=mode)), oracle.bitpack(x, mode))


@pytest.mark.parametrize("C", [1, 2, 31, 33, 63, 65, 96, 127, 129, 191, 320, 1000, 4097])
def test_bitpack_flat_stream_tail_kernel(dabnn, oracle, C):
    """Small word counts: one wavefront, the tensor ending inside its chunks."""
    Cw = (C + 63) // 64
    for n_words in (1, 31, 32, 33, 127, 128, 129, 4 * 32 * 7 + 5):
        n_pixels = max(1, n_words // Cw)
        x = wl.inject_zeros(wl.activations((n_pixels, C), 4400 + C + n_pixels), 4401 + C)
        assert np.array_equal(words(dabnn.bitpack(gpu(x))), oracle.bitpack(x)), (n_pixels, C)


@pytest.mark.parametrize("kernel", [0, 2])
@pytest.mark.parametrize("C", [1, 3, 31, 33, 65, 80, 127, 200, 4097])
def test_bitpack_flat_stream_chunk_boundaries(dabnn, oracle, option, C, kernel):
    """Element counts around the 2048 floats a wavefront owns and the 8192 of a workgroup (a
    wavefront writes the words that start in its chunks: several passes of 64 for short rows),
    with guard words around the output; 32-bit and 64-bit index variants."""
    option(dabnn.OPT_BITPACK_ROWWISE, kernel)
    Cw = (C + 63) // 64
    for n_floats in (2047, 2048, 2049, 2048 + 64, 4096 + 63, 8191, 8192, 8193, 3 * 8192 + 2111, 70001):
        n_pixels = max(1, n_floats // C)
        x = wl.inject_zeros(wl.activations((n_pixels, C), 4500 + C + n_pixels), 4501 + C, frac=0.05)
        for mode in (0, 1):
            buf = torch.full((n_pixels * Cw + 16,), 0x5A5A5A5A5A5A5A5A, dtype=torch.int64, device="cuda")
            out = buf[8:8 + n_pixels * Cw].view(n_pixels, Cw)
            dabnn.bitpack(gpu(x), out=out, sign_mode=mode)
            assert np.array_equal(words(out), oracle.bitpack(x, mode)), (n_pixels, C, mode)
            assert torch.all(buf[:8] == 0x5A5A5A5A5A5A5A5A) and torch.all(buf[-8:] == 0x5A5A5A5A5A5A5A5A)


@pytest.mark.parametrize("kernel", [0, 1, 2])
def test_bitpack_very_long_rows(dabnn, oracle, option, kernel):
    """Rows much longer than what a wavefront covers (a million channels, not a multiple of 64)."""
    option(dabnn.OPT_BITPACK_ROWWISE, kernel)
    x = wl.inject_zeros(wl.activations((3, 1_000_003), 4600), 4601)
    for mode in (0, 1):
        assert np.array_equal(words(dabnn.bitpack(gpu(x), sign_mode=mode)), oracle.bitpack(x, mode))


def test_bitpack_special_values(dabnn, oracle):
    row = wl.special_values()
    x = np.tile(row, (3, 13))[:, :200].copy()       # C = 200: specials in every word, with a tail
    for mode in (0, 1):
        assert np.array_equal(words(dabnn.bitpack(gpu(x), sign_mode=mode)), oracle.bitpack(x, mode))


def test_bitpack_empty(dabnn):
    x = torch.empty((0, 64), dtype=torch.float32, device="cuda")
    assert dabnn.bitpack(x).shape == (0, 1)


@pytest.mark.parametrize("C", [1, 64, 65, 200, 512])
def test_bitpack_i32(dabnn, oracle, C):
    rng = np.random.default_rng(300 + C)
    x = rng.integers(-1000, 1000, size=(3, 37, C)).astype(np.int32)
    x[0, 0, :] = np.iinfo(np.int32).min
    x[0, 1, :] = 0
    assert np.array_equal(words(dabnn.bitpack_i32(gpu(x))), oracle.bitpack_i32(x))


def test_bitpack_i32_binarizes_a_conv_output(dabnn, oracle):
    x = wl.activations((2, 14, 14, 64), 311)
    wf = wl.weights((128, 3, 3, 64), 312)
    y = dabnn.bconv2d(dabnn.bitpack(gpu(x)), dabnn.pack_weights(gpu(wf)), 64, 1, 1)
    assert np.array_equal(words(dabnn.bitpack_i32(y)), oracle.bitpack_i32(oracle.bconv2d(x, wf, 1, 1)))


@pytest.mark.parametrize("shape", [(1, 1, 1, 1), (2, 5, 7, 2), (3, 9, 4, 3), (2, 14, 14, 8), (1, 3, 3, 5)],
                         ids=lambda s: "x".join(map(str, s)))
def test_nc1hwc2_round_trip(dabnn, oracle, shape):
    rng = np.random.default_rng(sum(shape))
    a = rng.integers(0, 2**63, size=shape, dtype=np.uint64)
    a_gpu = gpu(a.view(np.int64))
    g = dabnn.nhwc_to_nc1hwc2(a_gpu)
    assert np.array_equal(words(g), oracle.nhwc_to_nc1hwc2(a))
    back = dabnn.nc1hwc2_to_nhwc(g, shape[3])
    assert torch.equal(back, a_gpu)


@pytest.mark.parametrize("C", [1, 64, 80, 128, 200, 512])
@pytest.mark.parametrize("with_r,with_x", [(False, False), (True, True), (True, False), (False, True)])
def test_bn_sign_pack(dabnn, oracle, C, with_r, with_x):
    rng = np.random.default_rng(600 + C)
    y = rng.integers(-1152, 1153, size=(5, 41, C)).astype(np.int32)
    scale = rng.uniform(-0.1, 0.1, C).astype(np.float32)
    scale[::6] = 0.0
    shift = rng.normal(0, 1, C).astype(np.float32)
    r = rng.normal(0, 2, y.shape).astype(np.float32) if with_r else None
    x, bits = dabnn.bn_sign_pack(gpu(y), gpu(scale), gpu(shift), gpu(r) if with_r else None, want_x=with_x)
    want_x, want_bits = oracle.bn_sign_pack(y, scale, shift, r)
    assert np.array_equal(words(bits), want_bits)
    if with_x:
        assert np.array_equal(x.cpu().numpy().view(np.uint32), want_x.view(np.uint32))  # bit for bit
    else:
        assert x is None


RESIDUAL_SHAPES = [  # N, H, W, Cin, Cout, k, stride, pad
    (1, 14, 14, 64, 64, 3, 1, 1), (3, 28, 28, 128, 128, 3, 1, 1), (2, 28, 28, 128, 256, 3, 2, 1),
    (2, 9, 13, 256, 192, 3, 1, 1), (2, 7, 7, 512, 512, 3, 1, 1), (5, 57, 30, 64, 64, 3, 1, 1),
    (1, 3, 3, 64, 64, 3, 1, 1), (3, 11, 10, 64, 128, 3, 2, 1),
    # the two-kernel route: other kernel sizes, channel counts, strides
    (2, 6, 6, 128, 64, 1, 1, 0), (1, 10, 17, 200, 33, 3, 2, 1), (1, 12, 12, 64, 16, 5, 1, 2),
    (2, 13, 11, 80, 130, 3, 1, 1),
]


@pytest.mark.parametrize("route", [0, 1, 2], ids=["by-size", "one-kernel", "two-kernels"])
@pytest.mark.parametrize("with_r", [True, False])
@pytest.mark.parametrize("shape", RESIDUAL_SHAPES, ids=lambda s: "-".join(map(str, s)))
def test_bconv2d_bn_residual(dabnn, oracle, option, shape, with_r, route):
    """One call against the oracle's convolution followed by the oracle's BN + shortcut + sign +
    pack layer; z compared bit for bit.  Small launches default to the two-kernel route, so the
    one-kernel route is also forced (where the shape has one) and so is the other."""
    option(dabnn.OPT_RES_FUSED, route)
    check_bn_residual(dabnn, oracle, shape, with_r)


def check_bn_residual(dabnn, oracle, shape, with_r):
    N, H, W, Cin, Cout, k, stride, pad = shape
    print("residual", shape, with_r, flush=True)
    seed = 7000 + sum(shape)
    x = wl.activations((N, H, W, Cin), seed)
    wf = wl.weights((Cout, k, k, Cin), seed + 1)
    rng = np.random.default_rng(seed + 2)
    scale = rng.uniform(-0.1, 0.1, Cout).astype(np.float32)
    scale[::7] = 0.0
    shift = rng.normal(0, 1, Cout).astype(np.float32)
    oy = oracle.bconv2d(x, wf, stride, pad)
    r = rng.normal(0, 2, oy.shape).astype(np.float32) if with_r else None
    want_z, want_bits = oracle.bn_sign_pack(oy, scale, shift, r)
    z, bits = dabnn.bconv2d_bn_residual(dabnn.bitpack(gpu(x)), dabnn.pack_weights(gpu(wf)), gpu(scale),
                                        gpu(shift), gpu(r) if with_r else None, Cin, stride, pad)
    assert np.array_equal(z.cpu().numpy().view(np.uint32), want_z.view(np.uint32))
    assert np.array_equal(words(bits), want_bits)


@pytest.mark.parametrize("slots", [1, 5, 64])
def test_bconv2d_bn_residual_work_split(dabnn, oracle, slots, option):
    option(dabnn.OPT_AREG_SLOTS, slots)
    option(dabnn.OPT_RES_FUSED, 1)
    check_bn_residual(dabnn, oracle, (2, 14, 14, 128, 128, 3, 1, 1), True)
    check_bn_residual(dabnn, oracle, (3, 9, 7, 64, 192, 3, 2, 1), False)


def test_bconv2d_bn_residual_sixteen_channel_groups_forced(dabnn, oracle, option):
    """One-word-per-pixel layers default to 32-channel groups in the fused block kernel; the
    16-channel variant of the same shapes through the library's option."""
    option(dabnn.OPT_RES_CHANNELS, 16)
    option(dabnn.OPT_RES_FUSED, 1)
    for shape in [(1, 14, 14, 64, 64, 3, 1, 1), (5, 57, 30, 64, 64, 3, 1, 1), (3, 11, 10, 64, 128, 3, 2, 1)]:
        check_bn_residual(dabnn, oracle, shape, True)


def test_bconv2d_bn_residual_full_batch_layer(dabnn, oracle):
    """Batch 256 at a benchmark shape: every z (bit for bit) and every packed word against the
    oracle chain, and the whole result against the library's own two-call sequence."""
    L = wl.BIREAL18_BODY[5]
    N = wl.CFG5_BATCH
    x = wl.activations((N, L.H, L.W, L.Cin), wl.seed_for(5, 105))
    wf = wl.weights((L.Cout, 3, 3, L.Cin), wl.seed_for(5, 5))
    rng = np.random.default_rng(55)
    scale = rng.uniform(0.01, 0.05, L.Cout).astype(np.float32)
    shift = rng.normal(0, 1, L.Cout).astype(np.float32)
    r = rng.normal(0, 1, (N, L.Ho, L.Wo, L.Cout)).astype(np.float32)
    a, wp = dabnn.bitpack(gpu(x)), dabnn.pack_weights(gpu(wf))
    rg, sg, hg = gpu(r), gpu(scale), gpu(shift)
    z, bits = dabnn.bconv2d_bn_residual(a, wp, sg, hg, rg, L.Cin, L.stride, 1)
    z2, bits2 = dabnn.bn_sign_pack(dabnn.bconv2d(a, wp, L.Cin, L.stride, 1), sg, hg, rg)
    assert torch.equal(z.view(torch.int32), z2.view(torch.int32)) and torch.equal(bits, bits2)
    oz, ob = oracle.bn_sign_pack(oracle.bconv2d(x, wf, L.stride, 1), scale, shift, r)
    assert np.array_equal(z.cpu().numpy().view(np.uint32), oz.view(np.uint32))
    assert np.array_equal(words(bits), ob)


def test_bireal_block_chain(dabnn, oracle):
    """Two Bi-Real-style blocks: bits -> conv -> BN + shortcut + sign + pack -> conv, against the
    oracle chain; the second conv consumes the fused layer's words directly."""
    N, H, W, C = 2, 14, 14, 128
    x0 = wl.activations((N, H, W, C), 6100)
    w1, w2 = wl.weights((C, 3, 3, C), 6101), wl.weights((C, 3, 3, C), 6102)
    gamma, beta = wl.affine(C, 6103)
    scale = (gamma / np.sqrt(np.float32(9 * C))).astype(np.float32)
    y1 = dabnn.bconv2d(dabnn.bitpack(gpu(x0)), dabnn.pack_weights(gpu(w1)), C, 1, 1)
    x1, a1 = dabnn.bn_sign_pack(y1, gpu(scale), gpu(beta), gpu(x0))
    y2 = dabnn.bconv2d(a1, dabnn.pack_weights(gpu(w2)), C, 1, 1)
    oy1 = oracle.bconv2d(x0, w1, 1, 1)
    ox1, oa1 = oracle.bn_sign_pack(oy1, scale, beta, x0)
    assert np.array_equal(x1.cpu().numpy().view(np.uint32), ox1.view(np.uint32))
    assert np.array_equal(words(a1), oa1)
    assert np.array_equal(y2.cpu().numpy(), oracle.bconv2d(ox1, w2, 1, 1))


def test_pack_weights(dabnn, oracle):
    for shape in [(64, 3, 3, 64), (128, 3, 3, 80), (5, 1, 1, 200), (7, 5, 5, 3), (512, 3, 3, 512)]:
        w = wl.weights(shape, 77 + shape[0], p_plus=0.3)
        assert np.array_equal(words(dabnn.pack_weights(gpu(w))), oracle.bitpack(w))


# ------------------------------------------------------------------------------- convolution

def run_conv(dabnn, oracle, N, H, W, Cin, Cout, k, stride, pad, seed, algo, p_plus=0.5):
    x = wl.activations((N, H, W, Cin), seed)
    wf = wl.weights((Cout, k, k, Cin), seed + 1, p_plus)
    a = dabnn.bitpack(gpu(x))
    wp = dabnn.pack_weights(gpu(wf))
    Ho, Wo = oracle.conv_out_dim(H, k, stride, pad), oracle.conv_out_dim(W, k, stride, pad)
    # guard values around the output catch out-of-bounds writes
    n_out = N * Ho * Wo * Cout
    buf = torch.full((n_out + 512,), -123456789, dtype=torch.int32, device="cuda")
    out = buf[256:256 + n_out].view(N, Ho, Wo, Cout)
    try:
        dabnn.bconv2d(a, wp, Cin, stride, pad, out=out, algo=algo)
    except dabnn.DabnnError as e:
        # a forced family may refuse a shape it does not cover: then it must leave the output
        # alone, and the automatic choice must be another family
        if e.status == 4 and algo in (2, 3):
            assert torch.all(buf == -123456789)
            assert dabnn.pick_algo(N, H, W, Cin, Cout, k, k, stride, pad) != algo
            return
        raise
    want = oracle.bconv2d(x, wf, stride, pad)
    got = out.cpu().numpy()
    assert torch.all(buf[:256] == -123456789) and torch.all(buf[-256:] == -123456789)
    if not np.array_equal(got, want):
        bad = np.argwhere(got != want)
        raise AssertionError(f"{len(bad)} of {got.size} outputs differ, first at {bad[0]}: "
                             f"got {got[tuple(bad[0])]} want {want[tuple(bad[0])]}")


ALGOS = [1, 2, 3, 0]  # reference, filter-stationary, activation-stationary, auto


@pytest.mark.parametrize("algo", ALGOS)
def test_cfg1_single_conv(dabnn, oracle, algo):
    L = wl.CFG1_LAYER
    run_conv(dabnn, oracle, 1, L.H, L.W, L.Cin, L.Cout, 3, 1, 1, wl.seed_for(1), algo)


@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("N", wl.CFG2_BATCHES)
@pytest.mark.parametrize("li", range(4))
def test_cfg2_stride1_sweep(dabnn, oracle, li, N, algo):
    L = wl.CFG2_LAYERS[li]
    print("cfg2", L, N, algo, flush=True)
    run_conv(dabnn, oracle, N, L.H, L.W, L.Cin, L.Cout, 3, 1, 1, wl.seed_for(2, li), algo)


@pytest.mark.parametrize("algo", [2, 3, 0])
@pytest.mark.parametrize("li", range(3))
def test_cfg4_stride2(dabnn, oracle, li, algo):
    L = wl.CFG4_LAYERS[li]
    print("cfg4", L, algo, flush=True)
    run_conv(dabnn, oracle, wl.CFG4_BATCH, L.H, L.W, L.Cin, L.Cout, 3, 2, 1, wl.seed_for(4, li), algo,
             p_plus=wl.CFG4_P_PLUS)


ODD_SHAPES = [  # N, H, W, Cin, Cout, k, stride, pad
    (1, 1, 1, 1, 1, 1, 1, 0),
    (2, 5, 7, 3, 5, 3, 1, 1),
    (1, 9, 9, 63, 70, 3, 2, 1),
    (3, 8, 6, 65, 64, 3, 1, 0),
    (2, 13, 11, 80, 130, 3, 1, 1),
    (1, 10, 17, 200, 33, 3, 2, 1),
    (2, 6, 6, 128, 64, 1, 1, 0),
    (1, 12, 12, 64, 16, 5, 1, 2),
    (1, 7, 9, 100, 10, 3, 3, 1),
    (2, 4, 30, 64, 64, 3, 1, 2),
    (1, 3, 3, 512, 64, 3, 1, 1),
    (5, 2, 2, 256, 192, 3, 2, 1),
    (1, 33, 9, 64, 65, 3, 1, 1),
    (1, 15, 15, 320, 8, 3, 1, 1),
    (3, 9, 13, 64, 72, 3, 1, 1),
    (2, 11, 7, 128, 20, 3, 2, 1),
    (1, 20, 20, 256, 12, 3, 1, 0),
    (70, 3, 3, 64, 8, 3, 1, 1),
    # images smaller than the kernel: most taps (or all but one) lie in the padding
    (4, 1, 1, 64, 64, 3, 1, 1), (1, 1, 5, 128, 16, 3, 2, 1), (3, 2, 1, 64, 4, 3, 1, 2), (2, 1, 1, 512, 32, 3, 1, 1),
]


@pytest.mark.parametrize("algo", [1, 0])
@pytest.mark.parametrize("shape", ODD_SHAPES, ids=lambda s: "-".join(map(str, s)))
def test_odd_shapes(dabnn, oracle, shape, algo):
    print("odd", shape, algo, flush=True)
    run_conv(dabnn, oracle, *shape, seed=4242 + sum(shape), algo=algo)


@pytest.mark.parametrize("algo", [2, 3])
@pytest.mark.parametrize("shape", [s for s in ODD_SHAPES if s[5] == 3 and s[6] in (1, 2)],
                         ids=lambda s: "-".join(map(str, s)))
def test_odd_shapes_tuned(dabnn, oracle, shape, algo):
    print("odd tuned", shape, algo, flush=True)
    run_conv(dabnn, oracle, *shape, seed=999 + sum(shape), algo=algo)


@pytest.mark.parametrize("env", [("OPT_AREG_STORE", 1, 3), ("OPT_AREG_STORE", 16, 3), ("OPT_AREG_SPLIT", 4, 3),
                                 ("OPT_AREG_SPLIT", 8, 3), ("OPT_WREG_PIXELS", 7, 2), ("OPT_WREG_PIXELS", 8, 2)],
                         ids=lambda e: f"{e[0]}={e[1]}")
def test_kernel_variants(dabnn, oracle, env, option):
    """Both store variants of the activation-stationary family, its four-wavefront kernels at 4
    and 8 words per pixel, and both chunk widths of the filter-stationary family, forced through
    the library's options (launches as small as these take the direct store and the one-wavefront
    kernel by default)."""
    name, value, algo = env
    option(getattr(dabnn, name), value)
    for shape in [(2, 14, 14, 64, 64, 3, 1, 1), (3, 28, 28, 128, 128, 3, 2, 1), (2, 9, 13, 256, 96, 3, 1, 1),
                  (2, 7, 7, 512, 64, 3, 1, 1), (1, 57, 30, 64, 32, 3, 1, 1)]:
        print("variant", env, shape, flush=True)
        run_conv(dabnn, oracle, *shape, seed=31337 + sum(shape), algo=algo)


@pytest.mark.parametrize("slots", [1, 3, 7, 40, 1000])
@pytest.mark.parametrize("tail", [1, 2])
def test_work_split_and_remainder_pieces(dabnn, oracle, slots, tail, option):
    """The split of (tile, channel group) pairs over wavefronts, with the wavefront count forced
    small so that ranges span several tiles, and the uneven remainder handed out either as whole
    groups or as direct-store pieces; the four-wavefront kernels split over workgroups alike."""
    option(dabnn.OPT_AREG_SLOTS, slots)
    option(dabnn.OPT_AREG_TAIL, tail)
    option(dabnn.OPT_AREG_STORE, 16)   # the transposed store and the four-wavefront kernel at 8
    option(dabnn.OPT_AREG_SPLIT, 8)    # words, which launches this small would not take by default
    for shape in [(2, 14, 14, 64, 64, 3, 1, 1), (3, 28, 28, 128, 128, 3, 2, 1), (2, 9, 13, 256, 96, 3, 1, 1),
                  (1, 23, 17, 64, 48, 3, 1, 1), (2, 7, 7, 512, 64, 3, 1, 1), (2, 9, 7, 320, 48, 3, 1, 1),
                  (2, 6, 5, 1024, 32, 3, 1, 1), (1, 9, 9, 704, 32, 3, 2, 1)]:
        print("split", slots, tail, shape, flush=True)
        run_conv(dabnn, oracle, *shape, seed=1717 + slots + sum(shape), algo=3)
    shape = (2, 14, 14, 128, 128, 3, 1, 1)
    x = wl.activations(shape[:4], 1718 + slots)
    wf = wl.weights((128, 3, 3, 128), 1719 + slots)
    gamma, beta, mean, var = _bn_params(128, 1720 + slots)
    thr, flip = dabnn.bn_thresholds(gamma, beta, mean, var, 1e-5, 9 * 128)
    got = dabnn.bconv2d_bnsign(dabnn.bitpack(gpu(x)), dabnn.pack_weights(gpu(wf)), thr, flip, 128, 1, 1)
    assert np.array_equal(words(got), oracle.bconv2d_bnsign(x, wf, gamma, beta, mean, var, 1e-5, 1, 1))


WORD_COUNT_SHAPES = [  # N, H, W, Cin, Cout, k, stride, pad: every kernel of the family and every split of K
    (3, 14, 14, 160, 64, 3, 1, 1), (2, 9, 11, 192, 48, 3, 2, 1), (2, 14, 14, 320, 64, 3, 1, 1),
    (3, 7, 9, 384, 32, 3, 1, 1), (2, 8, 8, 448, 64, 3, 2, 1), (2, 7, 7, 576, 64, 3, 1, 1),
    (2, 6, 7, 640, 16, 3, 1, 1), (1, 9, 9, 704, 32, 3, 2, 1), (2, 7, 7, 768, 64, 3, 1, 1),
    (2, 5, 6, 832, 32, 3, 1, 1), (2, 7, 7, 1024, 128, 3, 1, 1), (1, 6, 6, 1088, 32, 3, 1, 1),
    (1, 5, 5, 2048, 32, 3, 1, 1), (1, 4, 6, 2240, 16, 3, 2, 1),
    # Cout % 16 != 0: direct stores, up to 8 words per pixel
    (2, 9, 9, 192, 24, 3, 1, 1), (2, 7, 7, 320, 40, 3, 1, 1), (2, 6, 6, 448, 8, 3, 2, 1),
    (2, 7, 7, 500, 8, 3, 1, 1), (2, 6, 6, 384, 20, 3, 1, 1),
]


@pytest.mark.parametrize("shape", WORD_COUNT_SHAPES, ids=lambda s: "-".join(map(str, s)))
def test_every_word_count(dabnn, oracle, shape):
    """Channel counts from 3 to 35 words per pixel run in the activation-stationary family: as one
    launch, or as several launches over parts of the channels that add into y."""
    print("words", shape, flush=True)
    assert dabnn.pick_algo(*shape[:5], 3, 3, shape[6], shape[7]) == dabnn.ALGO_AREG
    run_conv(dabnn, oracle, *shape, seed=6100 + sum(shape), algo=3)
    run_conv(dabnn, oracle, *shape, seed=6200 + sum(shape), algo=0)


@pytest.mark.parametrize("Cin", [160, 320, 384, 448, 1024])
def test_word_counts_at_batch_64(dabnn, oracle, Cin):
    """3, 5, 6, 7 and 16 words per pixel at batch 64 (several ranges per SIMD, many tiles), every
    output compared; the automatic choice must be the activation-stationary family."""
    shape = (64, 14, 14, Cin, 256, 3, 1, 1)
    print("words at batch 64", shape, flush=True)
    assert dabnn.pick_algo(*shape[:5], 3, 3, 1, 1) == dabnn.ALGO_AREG
    run_conv(dabnn, oracle, *shape, seed=6300 + Cin, algo=0)


def test_launches_that_add_into_y_follow_one_another(dabnn, oracle):
    """Word counts above 8 run as launches that add into y: repeated calls into the same output
    buffer (which then holds an old result, not zeros) must give the same values every time."""
    shape = (3, 9, 9, 1216, 64, 3, 1, 1)          # 19 words: 16 + 3
    N, H, W, Cin, Cout = shape[:5]
    x = wl.activations((N, H, W, Cin), 8400)
    wf = wl.weights((Cout, 3, 3, Cin), 8401)
    a, wp = dabnn.bitpack(gpu(x)), dabnn.pack_weights(gpu(wf))
    want = oracle.bconv2d(x, wf, 1, 1)
    out = torch.full(want.shape, 12345, dtype=torch.int32, device="cuda")
    for rep in range(3):
        dabnn.bconv2d(a, wp, Cin, 1, 1, out=out)
        assert np.array_equal(out.cpu().numpy(), want), rep


# ------------------------------------------------------------------- zero padding (ONNX Convolution)

ZEROPAD_SHAPES = ODD_SHAPES + [
    (2, 14, 14, 64, 64, 3, 1, 1),
    (3, 28, 28, 128, 128, 3, 2, 1),
    (2, 7, 7, 512, 512, 3, 1, 1),
    (4, 56, 56, 64, 64, 3, 1, 1),
    (1, 1, 1, 64, 8, 3, 1, 1),       # every tap but the centre is outside
    (2, 2, 9, 64, 8, 5, 1, 2),       # rows that are outside at the top and at the bottom at once
    (1, 5, 5, 70, 6, 3, 4, 2),       # stride larger than the pad
]


@pytest.mark.parametrize("shape", ZEROPAD_SHAPES, ids=lambda s: "-".join(map(str, s)))
def test_bconv2d_zeropad(dabnn, oracle, shape):
    N, H, W, Cin, Cout, k, stride, pad = shape
    print("zeropad", shape, flush=True)
    x = wl.activations((N, H, W, Cin), 777 + sum(shape))
    wf = wl.weights((Cout, k, k, Cin), 778 + sum(shape), p_plus=0.3)
    a = dabnn.bitpack(gpu(x))
    wp = dabnn.pack_weights(gpu(wf))
    y = dabnn.bconv2d_zeropad(a, wp, Cin, stride, pad)
    want = oracle.bconv2d_zeropad(x, wf, stride, pad)
    assert y.dtype == torch.int32 and tuple(y.shape) == want.shape
    assert np.array_equal(y.cpu().numpy(), want)


def test_bconv2d_zeropad_full_batch_layer(dabnn, oracle):
    """Batch 256 at a benchmark shape: every output against the oracle, and, at any size, the
    interior equals the +1-padded result while the border differs by an image-independent
    amount."""
    L = wl.BIREAL18_BODY[0]
    N = wl.CFG5_BATCH
    x = wl.activations((N, L.H, L.W, L.Cin), wl.seed_for(5, 100))
    wf = wl.weights((L.Cout, 3, 3, L.Cin), wl.seed_for(5, 0))
    a = dabnn.bitpack(gpu(x))
    wp = dabnn.pack_weights(gpu(wf))
    y0 = dabnn.bconv2d_zeropad(a, wp, L.Cin, L.stride, 1).cpu().numpy()
    y1 = dabnn.bconv2d(a, wp, L.Cin, L.stride, 1).cpu().numpy()
    assert np.array_equal(y0, oracle.bconv2d_zeropad(x, wf, L.stride, 1))
    d = y1 - y0
    assert not d[:, 1:-1, 1:-1, :].any()
    assert np.array_equal(d, np.broadcast_to(d[:1], d.shape))


# ------------------------------------------------------------------------------ BGEMM (Eq. 1)

BGEMM_SHAPES = [  # M, N, K  (Kw = ceil(K/64)); fast kernel: N % 16 == 0 and 2*Kw in its list
    (200, 64, 64), (1000, 32, 128), (130, 16, 190), (64, 48, 256), (65, 16, 384), (300, 128, 512),
    (77, 16, 576), (100, 32, 768), (50, 16, 1024), (90, 16, 1152), (40, 16, 1536), (33, 16, 2048),
    (70, 32, 2304), (20, 16, 3072), (10, 16, 4096), (129, 16, 4608), (4100, 256, 64),
    # reference kernel: other row lengths, N not a multiple of 16, tiny shapes
    (10, 10, 64), (33, 16, 320), (7, 16, 5000), (1, 1, 1), (64, 17, 128),
]


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("shape", BGEMM_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_bgemm(dabnn, oracle, shape, mode):
    M, N, K = shape
    print("bgemm", shape, mode, flush=True)
    xa = wl.activations((M, K), 881 + M + N)
    xb = wl.weights((N, K), 882 + K, p_plus=0.4)
    A = dabnn.bitpack(gpu(xa))   # rows are "pixels" of K channels: tails come out as 0
    B = dabnn.bitpack(gpu(xb))
    C = dabnn.bgemm(A, B, K, mode)
    want = oracle.bgemm_signed(oracle.sign(xa), oracle.sign(xb), mode)
    assert C.dtype == torch.int32 and tuple(C.shape) == (M, N)
    assert np.array_equal(C.cpu().numpy(), want)


def test_bgemm_sixteen_column_groups_forced(dabnn, oracle, option):
    """Short rows default to 32-column groups (whole 128-byte stores); the 16-column kernel of the
    same shapes through the library's option."""
    option(dabnn.OPT_BGEMM_COLUMNS, 16)
    for M, N, K in [(200, 64, 64), (1000, 32, 128), (300, 128, 512), (4100, 256, 64)]:
        xa = wl.activations((M, K), 883 + M)
        xb = wl.weights((N, K), 884 + K)
        C = dabnn.bgemm(dabnn.bitpack(gpu(xa)), dabnn.bitpack(gpu(xb)), K)
        assert np.array_equal(C.cpu().numpy(), oracle.bgemm_signed(oracle.sign(xa), oracle.sign(xb)))


IM2COL_SHAPES = [  # N, H, W, Cin, Cout, k, stride, pad
    (2, 14, 14, 64, 64, 3, 1, 1), (3, 28, 28, 128, 32, 3, 2, 1), (2, 9, 13, 256, 96, 3, 1, 1),
    (2, 7, 7, 512, 64, 3, 1, 1), (1, 10, 17, 200, 33, 3, 2, 1), (1, 12, 12, 64, 16, 5, 1, 2),
    (2, 6, 6, 100, 48, 1, 1, 0),
]


@pytest.mark.parametrize("shape", IM2COL_SHAPES, ids=lambda s: "-".join(map(str, s)))
def test_im2col_and_conv_as_bgemm(dabnn, oracle, shape):
    """The patch matrix word for word, and the BGEMM route (Fig. 4's comparison method) against the
    convolution oracle and against the direct kernel."""
    N, H, W, Cin, Cout, k, stride, pad = shape
    print("im2col", shape, flush=True)
    x = wl.activations((N, H, W, Cin), 991 + sum(shape))
    wf = wl.weights((Cout, k, k, Cin), 992 + sum(shape), p_plus=0.3)
    a = dabnn.bitpack(gpu(x))
    wp = dabnn.pack_weights(gpu(wf))
    cols = dabnn.im2col(a, Cin, k, k, stride, pad)
    Cw = (Cin + 63) // 64
    patch = oracle.im2col_signed(oracle.sign(x), k, k, stride, pad)      # [M, k*k, Cin]
    want_cols = oracle.bitpack(patch).reshape(patch.shape[0], k * k * Cw)
    assert np.array_equal(words(cols), want_cols)
    y = dabnn.bgemm(cols, wp.reshape(Cout, k * k * Cw), k * k * Cin)
    want = oracle.bconv2d(x, wf, stride, pad)
    assert np.array_equal(y.cpu().numpy().reshape(want.shape), want)
    assert torch.equal(y.reshape(want.shape), dabnn.bconv2d(a, wp, Cin, stride, pad))


@pytest.mark.parametrize("shape", [(2, 14, 14, 64, 64), (3, 9, 7, 128, 32), (1, 28, 28, 256, 512),
                                   (2, 7, 7, 512, 128), (1, 5, 5, 100, 16)],
                         ids=lambda s: "-".join(map(str, s)))
def test_pointwise_conv_runs_as_bgemm(dabnn, oracle, shape):
    N, H, W, Cin, Cout = shape
    assert dabnn.pick_algo(N, H, W, Cin, Cout, 1, 1, 1, 0) == dabnn.ALGO_BGEMM
    run_conv(dabnn, oracle, N, H, W, Cin, Cout, 1, 1, 0, seed=555 + sum(shape), algo=dabnn.ALGO_BGEMM)
    run_conv(dabnn, oracle, N, H, W, Cin, Cout, 1, 1, 0, seed=556 + sum(shape), algo=0)
    # strided or padded 1x1 convolutions are not a plain matrix product
    assert dabnn.pick_algo(N, H, W, Cin, Cout, 1, 1, 2, 0) == dabnn.ALGO_REFERENCE


# ------------------------------------------------- expanded-operand (int8 matrix core) comparison

INT8_SHAPES = [  # N, H, W, Cin, Cout, k, stride, pad
    (1, 14, 14, 64, 64, 3, 1, 1), (3, 28, 28, 128, 128, 3, 2, 1), (2, 9, 13, 256, 192, 3, 1, 1),
    (2, 7, 7, 512, 512, 3, 1, 1), (5, 11, 6, 64, 256, 3, 1, 1), (1, 12, 12, 64, 64, 5, 1, 2),
    (2, 6, 6, 128, 64, 1, 1, 0), (4, 56, 56, 64, 64, 3, 1, 1), (1, 7, 9, 192, 128, 3, 3, 1),
]


@pytest.mark.parametrize("shape", INT8_SHAPES, ids=lambda s: "-".join(map(str, s)))
def test_int8_matrix_core_route(dabnn, oracle, shape):
    """Bits -> +-1 bytes (against the sign oracle), then the int8 implicit GEMM against the
    convolution oracle and the XOR/popcount kernel."""
    N, H, W, Cin, Cout, k, stride, pad = shape
    print("int8", shape, flush=True)
    x = wl.activations((N, H, W, Cin), 661 + sum(shape))
    wf = wl.weights((Cout, k, k, Cin), 662 + sum(shape), p_plus=0.3)
    a = dabnn.bitpack(gpu(x))
    wp = dabnn.pack_weights(gpu(wf))
    a8 = dabnn.expand_int8(a, Cin)
    w8 = dabnn.expand_int8(wp, Cin)
    assert np.array_equal(a8.cpu().numpy(), oracle.sign(x).astype(np.int8))
    assert np.array_equal(w8.cpu().numpy(), oracle.sign(wf).astype(np.int8))
    n_out = N * oracle.conv_out_dim(H, k, stride, pad) * oracle.conv_out_dim(W, k, stride, pad) * Cout
    buf = torch.full((n_out + 512,), -123456789, dtype=torch.int32, device="cuda")
    want = oracle.bconv2d(x, wf, stride, pad)
    out = buf[256:256 + n_out].view(want.shape)
    dabnn.bconv2d_int8(a8, w8, stride, pad, out=out)
    assert torch.all(buf[:256] == -123456789) and torch.all(buf[-256:] == -123456789)
    assert np.array_equal(out.cpu().numpy(), want)
    assert torch.equal(out, dabnn.bconv2d(a, wp, Cin, stride, pad))


# ------------------------------------------------- matrix cores fed from the packed bits
MFMA_BITS_SHAPES = [  # N, H, W, Cin, Cout, stride, pad: every word count and stride, ragged pixel counts
    (3, 13, 11, 64, 64, 1, 1), (2, 9, 9, 64, 128, 2, 1), (2, 10, 7, 128, 128, 1, 1), (2, 9, 9, 128, 256, 2, 1),
    (3, 7, 7, 256, 256, 1, 1), (2, 8, 8, 256, 512, 2, 1), (2, 7, 7, 512, 512, 1, 1), (1, 12, 12, 512, 64, 2, 1),
    (5, 14, 14, 64, 192, 1, 0), (2, 11, 13, 128, 64, 1, 2), (4, 9, 9, 256, 128, 2, 0), (2, 8, 9, 512, 128, 1, 2),
    # fewer pixels than one wavefront tile: the masked kernel
    (1, 3, 3, 64, 64, 1, 1), (1, 7, 7, 128, 128, 1, 1), (1, 5, 5, 256, 64, 2, 1), (1, 4, 4, 512, 64, 1, 1),
    (1, 10, 10, 64, 64, 1, 1),   # 100 pixels: whole tiles of 64, masked tiles of 128
]


@pytest.mark.parametrize("fmt", [0, 1], ids=["int8", "fp4"])
@pytest.mark.parametrize("blocks", [2, 4])
@pytest.mark.parametrize("shape", MFMA_BITS_SHAPES, ids=lambda s: "-".join(map(str, s)))
def test_mfma_route_from_packed_bits(dabnn, oracle, option, shape, blocks, fmt):
    """dabnn_bconv2d_mfma (int8 or FP4 matrix instructions, activation operand expanded from the
    packed words in the kernel, filters prepared by dabnn_prepare_weights_mfma) against the float
    oracle, every output, with guard words around the output."""
    N, H, W, Cin, Cout, stride, pad = shape
    print("mfma from bits", shape, "pixel blocks", blocks, "format", fmt, flush=True)
    option(dabnn.OPT_MFMA_PIXEL_BLOCKS, blocks)
    x = wl.activations((N, H, W, Cin), 9100 + sum(shape))
    wf = wl.weights((Cout, 3, 3, Cin), 9101 + sum(shape), 0.4)
    a, wp = dabnn.bitpack(gpu(x)), dabnn.pack_weights(gpu(wf))
    n_bytes = dabnn.mfma_weights_bytes(Cin, Cout, fmt=fmt)
    assert n_bytes == Cout * 9 * Cin // (2 if fmt else 1) + 4 * Cout
    wq = dabnn.prepare_weights_mfma(wp, Cin, fmt=fmt)
    want = oracle.bconv2d(x, wf, stride, pad)
    buf = torch.full((want.size + 512,), -123456789, dtype=torch.int32, device="cuda")
    out = buf[256:256 + want.size].view(want.shape)
    dabnn.bconv2d_mfma(a, wq, Cin, Cout, stride, pad, out=out, fmt=fmt)
    got = out.cpu().numpy()
    assert torch.all(buf[:256] == -123456789) and torch.all(buf[-256:] == -123456789)
    if not np.array_equal(got, want):
        bad = np.argwhere(got != want)
        raise AssertionError(f"{len(bad)} of {got.size} outputs differ, first at {bad[0]}: "
                             f"got {got[tuple(bad[0])]} want {want[tuple(bad[0])]}")


@pytest.mark.parametrize("fmt", [0, 1], ids=["int8", "fp4"])
def test_mfma_route_full_batch_layers(dabnn, oracle, fmt):
    """The seven layer kinds of the benchmark body at batch 256 through dabnn_bconv2d_mfma, in the
    launch configuration bench.py times, every output against the oracle."""
    seen = set()
    for li, L in enumerate(wl.BIREAL18_BODY):
        key = (L.H, L.Cin, L.Cout, L.stride)
        if key in seen:
            continue
        seen.add(key)
        print("mfma from bits, batch 256", key, "format", fmt, flush=True)
        x = wl.activations((256, L.H, L.W, L.Cin), wl.seed_for(5, 100 + li))
        wf = wl.weights((L.Cout, 3, 3, L.Cin), wl.seed_for(5, li))
        a, wp = dabnn.bitpack(gpu(x)), dabnn.pack_weights(gpu(wf))
        got = dabnn.bconv2d_mfma(a, dabnn.prepare_weights_mfma(wp, L.Cin, fmt=fmt), L.Cin, L.Cout, L.stride, 1,
                                 fmt=fmt).cpu().numpy()
        want = oracle.bconv2d(x, wf, L.stride, 1)
        assert np.array_equal(got, want), key
        del a, wp, got, want


@pytest.mark.parametrize("fmt", [0, 1], ids=["int8", "fp4"])
@pytest.mark.parametrize("blocks", [2, 4])
@pytest.mark.parametrize("shape", MFMA_BITS_SHAPES[::2] + [(256, 14, 14, 256, 256, 1, 1)],
                         ids=lambda s: "-".join(map(str, s)))
def test_mfma_route_fused_threshold(dabnn, oracle, option, shape, blocks, fmt):
    """dabnn_bconv2d_bnsign_mfma: the packed next-layer activations against the oracle's
    sign(BN(conv)) in fp64, every word, with guard words; thresholds from dabnn_bn_thresholds."""
    N, H, W, Cin, Cout, stride, pad = shape
    print("mfma fused threshold", shape, "pixel blocks", blocks, "format", fmt, flush=True)
    option(dabnn.OPT_MFMA_PIXEL_BLOCKS, blocks)
    x = wl.activations((N, H, W, Cin), 9300 + sum(shape))
    wf = wl.weights((Cout, 3, 3, Cin), 9301 + sum(shape))
    gamma, beta, mean, var = _bn_params(Cout, 9302 + sum(shape))
    thr, flip = dabnn.bn_thresholds(gamma, beta, mean, var, 1e-5, 9 * Cin)
    a, wp = dabnn.bitpack(gpu(x)), dabnn.pack_weights(gpu(wf))
    wq = dabnn.prepare_weights_mfma(wp, Cin, fmt=fmt)
    want = oracle.bconv2d_bnsign(x, wf, gamma, beta, mean, var, 1e-5, stride, pad)
    buf = torch.full((want.size + 64,), 0x5a5a5a5a5a5a5a5a, dtype=torch.int64, device="cuda")
    out = buf[32:32 + want.size].view(want.shape)
    dabnn.bconv2d_bnsign_mfma(a, wq, thr, flip, Cin, Cout, stride, pad, out=out, fmt=fmt)
    assert torch.all(buf[:32] == 0x5a5a5a5a5a5a5a5a) and torch.all(buf[-32:] == 0x5a5a5a5a5a5a5a5a)
    assert np.array_equal(words(out), want)


def test_mfma_route_refuses_what_it_does_not_cover(dabnn):
    assert dabnn.mfma_weights_bytes(80, 64) == 0 and dabnn.mfma_weights_bytes(64, 48) == 0
    assert dabnn.mfma_weights_bytes(192, 64) == 0 and dabnn.mfma_weights_bytes(64, 64, 5, 5) == 0
    a = torch.zeros((1, 6, 6, 1), dtype=torch.int64, device="cuda")
    wq = torch.zeros((64 * 9 * 64 + 256,), dtype=torch.uint8, device="cuda")
    with pytest.raises(dabnn.DabnnError) as e:
        dabnn.bconv2d_mfma(a, wq, 64, 64, 3, 1)     # stride 3
    assert e.value.status == 4


def test_int8_route_refuses_other_channel_counts(dabnn):
    a8 = torch.ones((1, 4, 4, 80), dtype=torch.int8, device="cuda")
    w8 = torch.ones((64, 3, 3, 80), dtype=torch.int8, device="cuda")
    with pytest.raises(dabnn.DabnnError) as e:
        dabnn.bconv2d_int8(a8, w8, 1, 1)
    assert e.value.status == 4


# ------------------------------------------------------------------------------- fused BN + sign

def _bn_params(C, seed):
    rng = np.random.default_rng(seed)
    gamma = rng.uniform(-1.5, 1.5, C).astype(np.float32)
    gamma[::7] = 0.0
    beta = rng.normal(0, 0.5, C).astype(np.float32)
    mean = rng.normal(0, 8.0, C).astype(np.float32)
    var = rng.uniform(0.5, 40.0, C).astype(np.float32)
    return gamma, beta, mean, var


BNSIGN_SHAPES = [  # N, H, W, Cin, Cout, k, stride, pad
    (1, 14, 14, 64, 64, 3, 1, 1),
    (3, 28, 28, 128, 128, 3, 1, 1),
    (2, 56, 56, 64, 128, 3, 2, 1),
    (5, 14, 14, 256, 256, 3, 1, 1),
    (4, 14, 14, 256, 512, 3, 2, 1),
    (9, 7, 7, 512, 512, 3, 1, 1),
    (2, 9, 13, 80, 192, 3, 1, 1),       # tail in Cin, three output words
    (70, 3, 3, 64, 64, 3, 1, 1),        # ragged last tile
    (2, 9, 9, 64, 70, 3, 1, 1),         # Cout % 64 != 0: reference kernel, tail in the output word
    (1, 12, 12, 64, 16, 5, 1, 2),       # 5x5: reference kernel
    (2, 6, 6, 200, 33, 1, 1, 0),
]


@pytest.mark.parametrize("shape", BNSIGN_SHAPES, ids=lambda s: "-".join(map(str, s)))
def test_bconv2d_bnsign(dabnn, oracle, shape):
    """Fused conv + batch-norm threshold + bit-pack against sign(BN(conv)) of the oracle (fp64
    batch-norm), word for word."""
    N, H, W, Cin, Cout, k, stride, pad = shape
    print("bnsign", shape, flush=True)
    x = wl.activations((N, H, W, Cin), 7000 + sum(shape))
    wf = wl.weights((Cout, k, k, Cin), 7001 + sum(shape))
    gamma, beta, mean, var = _bn_params(Cout, 7002 + sum(shape))
    eps = 1e-5
    thr, flip = dabnn.bn_thresholds(gamma, beta, mean, var, eps, k * k * Cin)
    a = dabnn.bitpack(gpu(x))
    wp = dabnn.pack_weights(gpu(wf))
    Ho, Wo = oracle.conv_out_dim(H, k, stride, pad), oracle.conv_out_dim(W, k, stride, pad)
    words_out = (Cout + 63) // 64
    buf = torch.full((N * Ho * Wo * words_out + 32,), 0x5A5A5A5A5A5A5A5A, dtype=torch.int64, device="cuda")
    out = buf[16:16 + N * Ho * Wo * words_out].view(N, Ho, Wo, words_out)
    dabnn.bconv2d_bnsign(a, wp, thr, flip, Cin, stride, pad, out=out)
    want = oracle.bconv2d_bnsign(x, wf, gamma, beta, mean, var, eps, stride, pad)
    assert torch.all(buf[:16] == 0x5A5A5A5A5A5A5A5A) and torch.all(buf[-16:] == 0x5A5A5A5A5A5A5A5A)
    got = words(out)
    if not np.array_equal(got, want):
        bad = np.argwhere(got != want)
        raise AssertionError(f"{len(bad)} of {got.size} words differ, first at {bad[0]}: "
                             f"got {got[tuple(bad[0])]:#x} want {want[tuple(bad[0])]:#x}")


@pytest.mark.parametrize("shape", [(9, 7, 7, 512, 512, 3, 1, 1), (3, 14, 14, 512, 192, 3, 2, 1),
                                   (1, 5, 13, 512, 64, 3, 1, 1), (64, 7, 7, 512, 512, 3, 1, 1)],
                         ids=lambda s: "-".join(map(str, s)))
def test_bconv2d_bnsign_four_wavefront_kernel(dabnn, oracle, option, shape):
    """8 words per pixel: the fused threshold epilogue of the kernel whose four wavefronts share a
    channel group (the default from three groups per CU on; forced here for the small shapes)."""
    option(dabnn.OPT_AREG_SPLIT, 8)
    test_bconv2d_bnsign(dabnn, oracle, shape)


def test_bnsign_chain_feeds_next_layer(dabnn, oracle):
    """Two fused layers back to back: the packed output of the first is the packed input of the
    second, with no int32 tensor and no bit-pack pass in between."""
    N = 3
    x = wl.activations((N, 28, 28, 128), 7100)
    w1 = wl.weights((128, 3, 3, 128), 7101)
    w2 = wl.weights((256, 3, 3, 128), 7102)
    bn1, bn2 = _bn_params(128, 7103), _bn_params(256, 7104)
    eps = 1e-5
    t1 = dabnn.bn_thresholds(*bn1, eps, 9 * 128)
    t2 = dabnn.bn_thresholds(*bn2, eps, 9 * 128)
    a0 = dabnn.bitpack(gpu(x))
    a1 = dabnn.bconv2d_bnsign(a0, dabnn.pack_weights(gpu(w1)), *t1, 128, 1, 1)
    a2 = dabnn.bconv2d_bnsign(a1, dabnn.pack_weights(gpu(w2)), *t2, 128, 2, 1)
    o1 = oracle.bconv2d_bnsign(x, w1, *bn1, eps, 1, 1)
    assert np.array_equal(words(a1), o1)
    # unpack the oracle's first-layer bits to +-1 floats for its second layer
    bits = np.unpackbits(o1.view(np.uint8), axis=-1, bitorder="little")[..., :128]
    x1 = np.where(bits == 1, -1.0, 1.0).astype(np.float32)
    assert np.array_equal(words(a2), oracle.bconv2d_bnsign(x1, w2, *bn2, eps, 2, 1))


def test_closed_forms_on_gpu(dabnn):
    """All-equal gives +K, all-opposite gives -K, with the border taps counted as +1."""
    for (N, H, W, Cin, Cout, k, s, p) in [(2, 14, 14, 64, 64, 3, 1, 1), (1, 9, 9, 80, 70, 3, 2, 1)]:
        K = k * k * Cin
        ones_a = torch.ones((N, H, W, Cin), device="cuda")
        ones_w = torch.ones((Cout, k, k, Cin), device="cuda")
        a = dabnn.bitpack(ones_a)
        for algo in (1, 2, 0):
            y = dabnn.bconv2d(a, dabnn.pack_weights(ones_w), Cin, s, p, algo=algo)
            assert torch.all(y == K)
            y = dabnn.bconv2d(a, dabnn.pack_weights(-ones_w), Cin, s, p, algo=algo)
            assert torch.all(y == -K)


def test_unsupported_algo_is_refused(dabnn):
    a = torch.zeros((1, 4, 4, 1), dtype=torch.int64, device="cuda")
    w = torch.zeros((4, 5, 5, 1), dtype=torch.int64, device="cuda")
    with pytest.raises(dabnn.DabnnError) as e:
        dabnn.bconv2d(a, w, 64, 1, 2, algo=dabnn.ALGO_WREG)   # 5x5 is not a wreg shape
    assert e.value.status == 4


# ------------------------------------------------------------------------------- full network

def test_cfg5_chain_small_batch(dabnn, oracle):
    """The sixteen-layer Bi-Real-18 body at its real shapes, batch 2, every layer compared in
    full; the fp32 input of layer i+1 is generated by the oracle from the oracle's own y_i."""
    N = 2
    x = wl.activations((N, 56, 56, 64), wl.seed_for(5))
    for li, L in enumerate(wl.BIREAL18_BODY):
        print("cfg5 layer", li, L, flush=True)
        wf = wl.weights((L.Cout, 3, 3, L.Cin), wl.seed_for(5, li))
        a_gpu = dabnn.bitpack(gpu(x))
        assert np.array_equal(words(a_gpu), oracle.bitpack(x))
        y_gpu = dabnn.bconv2d(a_gpu, dabnn.pack_weights(gpu(wf)), L.Cin, L.stride, 1)
        y = oracle.bconv2d(x, wf, L.stride, 1)
        assert np.array_equal(y_gpu.cpu().numpy(), y)
        gamma, beta = wl.affine(L.Cout, wl.seed_for(5, li))
        x = oracle.glue(x, y, gamma, beta, L.K, L.stride)


@pytest.mark.parametrize("li", range(16))
def test_cfg5_full_batch_layers(dabnn, oracle, li):
    """Batch 256, the launch configuration the benchmark times: every packed word and every
    convolution output of all 256 images against the oracle."""
    L = wl.BIREAL18_BODY[li]
    N = wl.CFG5_BATCH
    print("cfg5 full", li, L, flush=True)
    x = wl.activations((N, L.H, L.W, L.Cin), wl.seed_for(5, 100 + li))
    wf = wl.weights((L.Cout, 3, 3, L.Cin), wl.seed_for(5, li))
    a_gpu = dabnn.bitpack(gpu(x))
    assert np.array_equal(words(a_gpu), oracle.bitpack(x))
    y_gpu = dabnn.bconv2d(a_gpu, dabnn.pack_weights(gpu(wf)), L.Cin, L.stride, 1).cpu().numpy()
    want = oracle.bconv2d(x, wf, L.stride, 1)
    assert y_gpu.shape == want.shape
    if not np.array_equal(y_gpu, want):
        bad = np.argwhere(y_gpu != want)
        raise AssertionError(f"{len(bad)} of {want.size} outputs differ, first at {bad[0]}")


# ------------------------------------------------------------------------ streams and HIP graphs

def test_calls_follow_the_current_stream(dabnn, oracle):
    """The binding passes torch's current stream; work enqueued on a side stream must be ordered
    after that stream's earlier work and produce the same result."""
    x = wl.activations((4, 28, 28, 128), 4101)
    wf = wl.weights((128, 3, 3, 128), 4102)
    xg, wg = gpu(x), gpu(wf)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        a = dabnn.bitpack(xg)
        y = dabnn.bconv2d(a, dabnn.pack_weights(wg), 128, 1, 1)
    side.synchronize()
    assert np.array_equal(y.cpu().numpy(), oracle.bconv2d(x, wf, 1, 1))


def test_hip_graph_replay_of_the_hot_path(dabnn, oracle):
    """The entry points neither allocate nor synchronise, so bit-pack + conv (+ the fused and the
    zero-padded variants) can be captured into a HIP graph; every replay, with the input changed
    by eager work in between, must equal the oracle."""
    N, H, W, Cin, Cout = 3, 14, 14, 128, 128
    wf = wl.weights((Cout, 3, 3, Cin), 4202)
    wp = dabnn.pack_weights(gpu(wf))
    gamma, beta, mean, var = _bn_params(Cout, 4203)
    thr, flip = dabnn.bn_thresholds(gamma, beta, mean, var, 1e-5, 9 * Cin)
    xg = torch.empty((N, H, W, Cin), dtype=torch.float32, device="cuda")
    a = torch.empty((N, H, W, Cin // 64), dtype=torch.int64, device="cuda")
    y = torch.empty((N, H, W, Cout), dtype=torch.int32, device="cuda")
    y0 = torch.empty_like(y)
    ym = torch.empty_like(y)
    bits = torch.empty((N, H, W, Cout // 64), dtype=torch.int64, device="cuda")
    wq = dabnn.prepare_weights_mfma(wp, Cin)

    def enqueue():
        dabnn.bitpack(xg, out=a)
        dabnn.bconv2d(a, wp, Cin, 1, 1, out=y)
        dabnn.bconv2d_zeropad(a, wp, Cin, 1, 1, out=y0)
        dabnn.bconv2d_bnsign(a, wp, thr, flip, Cin, 1, 1, out=bits)
        dabnn.bconv2d_mfma(a, wq, Cin, Cout, 1, 1, out=ym)

    xg.copy_(gpu(wl.activations((N, H, W, Cin), 4200)))
    enqueue()  # eager once: one-time occupancy queries happen outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        enqueue()
    for rep in range(4):
        x = wl.activations((N, H, W, Cin), 4210 + rep)
        xg.copy_(gpu(x))          # eager work between the replays
        y.zero_(); y0.zero_(); bits.zero_(); ym.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(words(a), oracle.bitpack(x)), rep
        assert np.array_equal(y.cpu().numpy(), oracle.bconv2d(x, wf, 1, 1)), rep
        assert np.array_equal(ym.cpu().numpy(), oracle.bconv2d(x, wf, 1, 1)), rep
        assert np.array_equal(y0.cpu().numpy(), oracle.bconv2d_zeropad(x, wf, 1, 1)), rep
        assert np.array_equal(words(bits), oracle.bconv2d_bnsign(x, wf, gamma, beta, mean, var, 1e-5, 1, 1)), rep


# -------------------------------------------------------------------- seeded random shapes

def _random_shapes(n, seed):
    rng = np.random.default_rng(seed)
    shapes = []
    while len(shapes) < n:
        k = int(rng.choice([1, 3, 3, 3, 5]))
        stride = int(rng.choice([1, 1, 2, 3]))
        pad = int(rng.integers(0, k))
        H, W = int(rng.integers(1, 21)), int(rng.integers(1, 21))
        if H + 2 * pad < k or W + 2 * pad < k:
            continue
        Cin = int(rng.choice([int(rng.integers(1, 600)), 64, 128, 256, 512]))
        Cout = int(rng.choice([int(rng.integers(1, 200)), 16, 64, 128, 192]))
        shapes.append((int(rng.integers(1, 5)), H, W, Cin, Cout, k, stride, pad))
    return shapes


@pytest.mark.parametrize("shape", _random_shapes(48, 20191908), ids=lambda s: "-".join(map(str, s)))
def test_random_shapes_every_entry_point(dabnn, oracle, shape):
    """Seeded random shapes through every convolution entry point the shape is valid for."""
    N, H, W, Cin, Cout, k, stride, pad = shape
    print("random", shape, flush=True)
    seed = 9000 + sum(shape)
    x = wl.activations((N, H, W, Cin), seed)
    wf = wl.weights((Cout, k, k, Cin), seed + 1, p_plus=0.4)
    a, wp = dabnn.bitpack(gpu(x)), dabnn.pack_weights(gpu(wf))
    want = oracle.bconv2d(x, wf, stride, pad)
    for algo in (0, 1, 2, 3, 4):
        try:
            got = dabnn.bconv2d(a, wp, Cin, stride, pad, algo=algo)
        except dabnn.DabnnError as e:
            assert e.status == 4 and algo in (2, 3, 4)   # that family does not cover the shape
            continue
        assert np.array_equal(got.cpu().numpy(), want), algo
    assert np.array_equal(dabnn.bconv2d_zeropad(a, wp, Cin, stride, pad).cpu().numpy(),
                          oracle.bconv2d_zeropad(x, wf, stride, pad))
    gamma, beta, mean, var = _bn_params(Cout, seed + 2)
    thr, flip = dabnn.bn_thresholds(gamma, beta, mean, var, 1e-5, k * k * Cin)
    assert np.array_equal(words(dabnn.bconv2d_bnsign(a, wp, thr, flip, Cin, stride, pad)),
                          oracle.bconv2d_bnsign(x, wf, gamma, beta, mean, var, 1e-5, stride, pad))
    Cw = (Cin + 63) // 64
    g = dabnn.bgemm(dabnn.im2col(a, Cin, k, k, stride, pad), wp.reshape(Cout, k * k * Cw), k * k * Cin)
    assert np.array_equal(g.cpu().numpy().reshape(want.shape), want)
    if Cin % 64 == 0 and Cout % 64 == 0:
        y8 = dabnn.bconv2d_int8(dabnn.expand_int8(a, Cin), dabnn.expand_int8(wp, Cin), stride, pad)
        assert np.array_equal(y8.cpu().numpy(), want)


def test_results_are_identical_run_to_run(dabnn, option):
    """Integer outputs and packed words must not depend on scheduling: five runs of every tuned
    kernel family on a shape that spans many wavefronts, compared byte for byte."""
    option(dabnn.OPT_RES_FUSED, 1)   # the one-kernel block route, whatever the launch's size
    x = gpu(wl.activations((16, 28, 28, 128), 8800))
    wf = gpu(wl.weights((128, 3, 3, 128), 8801))
    gamma, beta, mean, var = _bn_params(128, 8802)
    thr, flip = dabnn.bn_thresholds(gamma, beta, mean, var, 1e-5, 9 * 128)
    r = gpu(wl.activations((16, 28, 28, 128), 8803))
    sc = torch.full((128,), 0.03, device="cuda")
    sh = torch.zeros(128, device="cuda")
    first = None
    for rep in range(5):
        a = dabnn.bitpack(x)
        wp = dabnn.pack_weights(wf)
        outs = [a, dabnn.bconv2d(a, wp, 128, 1, 1, algo=3), dabnn.bconv2d(a, wp, 128, 1, 1, algo=2),
                dabnn.bconv2d_bnsign(a, wp, thr, flip, 128, 1, 1)]
        z, bits = dabnn.bconv2d_bn_residual(a, wp, sc, sh, r, 128, 1, 1)
        outs += [z.view(torch.int32), bits]
        if first is None:
            first = [o.clone() for o in outs]
        else:
            assert all(torch.equal(o, f) for o, f in zip(outs, first)), rep
