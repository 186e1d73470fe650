"""Pins for the CPU oracle: everything here checks oracle/ against something that is NOT the
oracle -- closed forms, invariants, brute force over Python ints, numpy.packbits, torch's CPU
conv2d.  The paper prints no worked numeric example for this path (its only packing example is a
figure), so these pins are what fixes the oracle.  No GPU is used.

Each pin is aimed at one plausible mistake: a dropped tap, a wrong padding value, a flipped
kernel, a transposed weight layout, a wrong bit order, a wrong sign convention at +-0.
"""
import itertools

import numpy as np
import pytest
import torch

from paper_1908_05858_amd import workloads as wl


def popcount(v):
    return bin(int(v)).count("1")


# ----------------------------------------------------------------------------- sign / packer

def test_sign_rules_on_special_values(oracle):
    x = wl.special_values()
    bits = x.view(np.uint32)
    s0 = oracle.sign(x, oracle.SIGN_BIT)
    # Sec. 2.1.1: the binary value is the IEEE sign bit, nothing else.
    assert np.array_equal(s0, np.where(bits >> 31 == 1, -1.0, 1.0).astype(np.float32))
    s1 = oracle.sign(x, oracle.SIGN_GE0)
    expect = []
    for v in x.tolist():
        expect.append(1.0 if v >= 0 else -1.0)  # Python float compare: -0.0 >= 0, NaN fails
    assert np.array_equal(s1, np.array(expect, dtype=np.float32))
    # the two rules differ exactly at -0.0 and at positive NaN
    differ = s0 != s1
    for i in np.nonzero(differ)[0]:
        assert bits[i] == 0x80000000 or (np.isnan(x[i]) and bits[i] >> 31 == 0)


def test_bitpack_matches_numpy_packbits(oracle):
    rng = np.random.default_rng(7)
    for C in (1, 3, 63, 64, 65, 80, 128, 200, 256):
        x = rng.standard_normal((5, 3, C)).astype(np.float32)
        x = wl.inject_zeros(x, 11 + C, frac=0.05)
        got = oracle.bitpack(x)
        words = (C + 63) // 64
        assert got.shape == (5, 3, words) and got.dtype == np.uint64
        sb = np.signbit(x)
        padded = np.zeros((5, 3, words * 64), dtype=bool)
        padded[..., :C] = sb
        ref = np.packbits(padded, axis=-1, bitorder="little").view("<u8")
        assert np.array_equal(got, ref)
        # popcount of all words == number of negative-signed elements
        assert sum(popcount(v) for v in got.ravel()) == int(sb.sum())


def test_bitpack_one_hot_and_tail(oracle):
    for C in (64, 80, 200):
        words = (C + 63) // 64
        x = np.ones((C, C), dtype=np.float32)
        x[np.arange(C), np.arange(C)] = -1.0  # pixel p has only channel p negative
        got = oracle.bitpack(x)
        for p in range(C):
            for j in range(words):
                want = (1 << (p % 64)) if j == p // 64 else 0
                assert int(got[p, j]) == want
        # all-negative row: exactly C low bits set, tail bits zero
        allneg = oracle.bitpack(-np.ones((1, C), dtype=np.float32))
        val = sum(int(allneg[0, j]) << (64 * j) for j in range(words))
        assert val == (1 << C) - 1


def test_bitpack_negation_complements(oracle):
    rng = np.random.default_rng(3)
    C = 200
    x = rng.standard_normal((4, C)).astype(np.float32)
    a, b = oracle.bitpack(x), oracle.bitpack(-x)
    for p in range(4):
        va = sum(int(a[p, j]) << (64 * j) for j in range(4))
        vb = sum(int(b[p, j]) << (64 * j) for j in range(4))
        assert va ^ vb == (1 << C) - 1


def test_bitpack_sign_rule_ge0(oracle):
    x = np.array([[0.0, -0.0, 1.0, -1.0, np.nan, -np.nan, np.inf, -np.inf]], dtype=np.float32)
    assert int(oracle.bitpack(x, oracle.SIGN_BIT)[0, 0]) == 0b10101010
    # x >= 0 rule: -0.0 becomes +1 (bit 0), both NaNs become -1 (bit 1)
    assert int(oracle.bitpack(x, oracle.SIGN_GE0)[0, 0]) == 0b10111000


def test_packed_size_is_one_32nd(oracle):
    # Sec. 3: packing compresses binary weights 32x
    w = wl.weights((64, 3, 3, 128), 5)
    assert oracle.bitpack(w).nbytes * 32 == w.nbytes


# ----------------------------------------------------------------------------- convolution

SHAPES = [  # N, H, W, Cin, Cout, k, stride, pad
    (1, 5, 6, 3, 4, 3, 1, 1),
    (2, 7, 7, 64, 8, 3, 2, 1),
    (1, 6, 5, 80, 5, 3, 1, 0),
    (1, 4, 4, 7, 3, 1, 1, 0),
    (1, 9, 8, 5, 2, 3, 2, 0),
    (1, 5, 5, 2, 3, 5, 1, 2),
]


@pytest.mark.parametrize("shape", SHAPES)
def test_closed_forms_plus_minus_K(oracle, shape):
    N, H, W, Cin, Cout, k, s, p = shape
    K = k * k * Cin
    ones_a = np.ones((N, H, W, Cin), np.float32)
    ones_w = np.ones((Cout, k, k, Cin), np.float32)
    # all-equal -> +K everywhere, borders included because padding taps are +1
    assert np.all(oracle.bconv2d_signed(ones_a, ones_w, s, p) == K)
    # activations +1, weights -1 -> -K everywhere
    assert np.all(oracle.bconv2d_signed(ones_a, -ones_w, s, p) == -K)
    # activations -1, weights +1: -K + 2*t*Cin with t = number of taps outside the image
    y = oracle.bconv2d_signed(-ones_a, ones_w, s, p)
    Ho, Wo = y.shape[1:3]
    for ho in range(Ho):
        for wo in range(Wo):
            t = 0
            for i in range(k):
                for j in range(k):
                    hi, wi = ho * s - p + i, wo * s - p + j
                    t += not (0 <= hi < H and 0 <= wi < W)
            assert np.all(y[:, ho, wo, :] == -K + 2 * t * Cin)


@pytest.mark.parametrize("shape", SHAPES)
def test_parity_bound_and_negation(oracle, shape):
    N, H, W, Cin, Cout, k, s, p = shape
    K = k * k * Cin
    A = oracle.sign(wl.activations((N, H, W, Cin), 21))
    Wt = wl.weights((Cout, k, k, Cin), 22)
    y = oracle.bconv2d_signed(A, Wt, s, p)
    assert y.dtype == np.int32
    assert np.all((y - K) % 2 == 0)          # outputs keep the parity of K
    assert np.all(np.abs(y) <= K)
    assert np.array_equal(oracle.bconv2d_signed(A, -Wt, s, p), -y)  # linear in the weights


@pytest.mark.parametrize("shape", SHAPES)
def test_all_plus_weights_count_negatives(oracle, shape):
    """W == +1 -> y = K - 2 * (#negative activations in the window), counted with an integral
    image of numpy.signbit, independently of any multiply-add."""
    N, H, W, Cin, Cout, k, s, p = shape
    x = wl.activations((N, H, W, Cin), 31)
    K = k * k * Cin
    neg = np.signbit(x).sum(axis=-1).astype(np.int64)            # [N,H,W]
    padded = np.zeros((N, H + 2 * p, W + 2 * p), np.int64)
    padded[:, p:p + H, p:p + W] = neg
    ii = np.zeros((N, H + 2 * p + 1, W + 2 * p + 1), np.int64)
    ii[:, 1:, 1:] = padded.cumsum(1).cumsum(2)
    y = oracle.bconv2d(x, np.ones((Cout, k, k, Cin), np.float32), s, p)
    Ho, Wo = y.shape[1:3]
    for ho in range(Ho):
        for wo in range(Wo):
            r0, c0 = ho * s, wo * s
            cnt = ii[:, r0 + k, c0 + k] - ii[:, r0, c0 + k] - ii[:, r0 + k, c0] + ii[:, r0, c0]
            assert np.array_equal(y[:, ho, wo, 0], K - 2 * cnt)
            assert np.all(y[:, ho, wo, :] == y[:, ho, wo, :1])


@pytest.mark.parametrize("shape", SHAPES + [(2, 14, 14, 64, 64, 3, 1, 1), (1, 14, 14, 128, 32, 3, 2, 1)])
def test_against_torch_cpu_conv2d(oracle, shape):
    """Library routine: fp32 conv2d on +-1 tensors is exact (integers below 2^24)."""
    N, H, W, Cin, Cout, k, s, p = shape
    A = oracle.sign(wl.activations((N, H, W, Cin), 41))
    Wt = wl.weights((Cout, k, k, Cin), 42, p_plus=0.3)
    y = oracle.bconv2d_signed(A, Wt, s, p)
    a_t = torch.from_numpy(A).permute(0, 3, 1, 2).contiguous()
    a_t = torch.nn.functional.pad(a_t, (p, p, p, p), value=1.0)
    w_t = torch.from_numpy(Wt).permute(0, 3, 1, 2).contiguous()
    ref = torch.nn.functional.conv2d(a_t, w_t, stride=s).permute(0, 2, 3, 1).contiguous()
    assert np.array_equal(y, ref.numpy().astype(np.int32))


def _brute_conv(a, w, H, W, Cin, Cout, k, s, p):
    """Ten-line definition over Python ints; a[h][w][c], w[co][i][j][c] in {+1,-1}."""
    Ho, Wo = (H + 2 * p - k) // s + 1, (W + 2 * p - k) // s + 1
    out = [[[0] * Cout for _ in range(Wo)] for _ in range(Ho)]
    for ho, wo, co in itertools.product(range(Ho), range(Wo), range(Cout)):
        acc = 0
        for i, j, c in itertools.product(range(k), range(k), range(Cin)):
            hi, wi = ho * s - p + i, wo * s - p + j
            av = a[hi][wi][c] if (0 <= hi < H and 0 <= wi < W) else 1
            acc += av * w[co][i][j][c]
        out[ho][wo][co] = acc
    return out


@pytest.mark.parametrize("H,W,Cin,k,s,p", [(2, 2, 2, 3, 1, 1), (3, 3, 1, 3, 2, 1), (2, 3, 2, 1, 1, 0),
                                          (3, 2, 1, 3, 1, 1)])
def test_brute_force_all_activation_patterns(oracle, H, W, Cin, k, s, p):
    """Every one of the 2^(H*W*Cin) activation sign patterns, against the Python-int definition."""
    Cout = 2
    nbits = H * W * Cin
    assert nbits <= 12
    wt = wl.weights((Cout, k, k, Cin), 51 + nbits)
    wl_list = wt.astype(int).tolist()
    pats = np.array(list(itertools.product([1.0, -1.0], repeat=nbits)), np.float32)
    A = pats.reshape(len(pats), H, W, Cin)
    y = oracle.bconv2d_signed(A, wt, s, p)
    for n in range(len(pats)):
        ref = _brute_conv(A[n].astype(int).tolist(), wl_list, H, W, Cin, Cout, k, s, p)
        assert y[n].tolist() == ref


def test_brute_force_all_weight_patterns(oracle):
    """Every 2^9 weight pattern of a 3x3x1 filter on a fixed non-symmetric image: catches a
    flipped kernel or swapped kh/kw axes."""
    H, W, Cin, k, s, p = 4, 3, 1, 3, 1, 1
    x = wl.activations((1, H, W, Cin), 61)
    A = oracle.sign(x)
    pats = np.array(list(itertools.product([1.0, -1.0], repeat=9)), np.float32)
    Wt = pats.reshape(len(pats), k, k, Cin)
    y = oracle.bconv2d_signed(A, Wt, s, p)          # Cout = 512
    ref = _brute_conv(A[0].astype(int).tolist(), Wt.astype(int).tolist(), H, W, Cin, len(pats), k, s, p)
    assert y[0].tolist() == ref


@pytest.mark.parametrize("Cin", [3, 64, 80, 200])
def test_xor_popcount_identity(oracle, Cin):
    """Eq. 1 / Eq. 6 with Python big ints: y = K - 2*popcount(a XOR w) over the packed window,
    where a and w come from the oracle's packer and out-of-image taps are zero words.  Ties the
    float oracle to the bit formula the GPU implements."""
    N, H, W, Cout, k, s, p = 1, 5, 4, 3, 3, 1, 1
    x = wl.inject_zeros(wl.activations((N, H, W, Cin), 71), 72, frac=0.05)
    wf = wl.weights((Cout, k, k, Cin), 73)
    y = oracle.bconv2d(x, wf, s, p)
    ap, wp = oracle.bitpack(x), oracle.bitpack(wf)
    words = ap.shape[-1]
    K = k * k * Cin
    for ho, wo, co in itertools.product(range(y.shape[1]), range(y.shape[2]), range(Cout)):
        diff = 0
        for i, j in itertools.product(range(k), range(k)):
            hi, wi = ho * s - p + i, wo * s - p + j
            for q in range(words):
                av = int(ap[0, hi, wi, q]) if (0 <= hi < H and 0 <= wi < W) else 0
                diff += popcount(av ^ int(wp[co, i, j, q]))
        assert int(y[0, ho, wo, co]) == K - 2 * diff


@pytest.mark.parametrize("Cin,Cout", [(64, 64), (80, 5), (512, 32)])
def test_one_pixel_image_closed_form(oracle, Cin, Cout):
    """A 1x1 image under a 3x3 kernel with pad 1: eight taps lie in the +1 padding, so
    y = (sum of all weights' signs) - (sum of the centre tap's) + <a, w_centre> (Sec. 2.1.2's
    convolution with the padding value of the benchmark definition)."""
    x = wl.activations((4, 1, 1, Cin), 610 + Cin)
    w = wl.weights((Cout, 3, 3, Cin), 611 + Cin)
    sx = np.where(np.signbit(x), -1, 1).astype(np.int64)[:, 0, 0, :]
    sw = np.where(np.signbit(w), -1, 1).astype(np.int64)
    want = sx @ sw[:, 1, 1, :].T + (sw.sum(axis=(1, 2, 3)) - sw[:, 1, 1, :].sum(axis=1))[None, :]
    assert np.array_equal(oracle.bconv2d(x, w, 1, 1)[:, 0, 0, :], want.astype(np.int32))


def test_bconv2d_at_matches_full(oracle):
    N, H, W, Cin, Cout, k, s, p = 2, 9, 7, 80, 6, 3, 2, 1
    A = oracle.sign(wl.activations((N, H, W, Cin), 81))
    Wt = wl.weights((Cout, k, k, Cin), 82)
    y = oracle.bconv2d_signed(A, Wt, s, p)
    idx = np.array(list(itertools.product(range(N), range(y.shape[1]), range(y.shape[2]), range(Cout))),
                   np.int32)
    assert np.array_equal(oracle.bconv2d_at(A, Wt, idx, s, p), y.ravel())


def test_out_dim_and_bad_args(oracle):
    assert oracle.conv_out_dim(56, 3, 1, 1) == 56
    assert oracle.conv_out_dim(56, 3, 2, 1) == 28
    assert oracle.conv_out_dim(7, 3, 2, 1) == 4
    assert oracle.conv_out_dim(2, 3, 1, 0) < 0
    with pytest.raises(ValueError):
        oracle.bconv2d_signed(np.ones((1, 2, 2, 3), np.float32), np.ones((1, 3, 3, 4), np.float32), 1, 1)


def test_glue_closed_form(oracle):
    """The input generator: stride 1 adds x itself; stride 2 adds the 2x2 mean, channels repeated."""
    N, H, W, C = 1, 4, 4, 2
    x = np.arange(N * H * W * C, dtype=np.float32).reshape(N, H, W, C)
    y = np.zeros((N, H, W, C), np.int32)
    g, b = np.ones(C, np.float32), np.zeros(C, np.float32)
    assert np.array_equal(oracle.glue(x, y, g, b, 4, 1), x)
    y[...] = 2
    out = oracle.glue(x, y, 3 * g, b + 1, 4, 1)
    assert np.allclose(out, 3 * 2 / 2 + 1 + x)
    y2 = np.zeros((N, 2, 2, 2 * C), np.int32)
    out2 = oracle.glue(x, y2, np.ones(2 * C, np.float32), np.zeros(2 * C, np.float32), 4, 2)
    pooled = x.reshape(N, 2, 2, 2, 2, C).mean(axis=(2, 4))
    assert np.allclose(out2, np.concatenate([pooled, pooled], axis=-1))


# ----------------------------------------------------------------------------- fused BN + sign

def _bn_params(C, seed):
    rng = np.random.default_rng(seed)
    gamma = rng.uniform(-1.5, 1.5, C).astype(np.float32)
    gamma[::7] = 0.0                                   # degenerate channels: constant output
    beta = rng.normal(0, 0.5, C).astype(np.float32)
    mean = rng.normal(0, 8.0, C).astype(np.float32)
    var = rng.uniform(0.5, 40.0, C).astype(np.float32)
    return gamma, beta, mean, var


@pytest.mark.parametrize("shape", [(1, 5, 6, 64, 70, 3, 1, 1), (2, 7, 7, 80, 64, 3, 2, 1), (1, 4, 4, 7, 3, 1, 1, 0)])
def test_bnsign_against_torch_batch_norm(oracle, shape):
    """sign(BN(conv)) with torch's CPU batch_norm in float64 on the (already pinned) integer conv
    output, packed with numpy.packbits."""
    N, H, W, Cin, Cout, k, s, p = shape
    x = wl.activations((N, H, W, Cin), 91)
    wf = wl.weights((Cout, k, k, Cin), 92)
    gamma, beta, mean, var = _bn_params(Cout, 93)
    eps = 1e-5
    got = oracle.bconv2d_bnsign(x, wf, gamma, beta, mean, var, eps, s, p)
    y = torch.from_numpy(oracle.bconv2d(x, wf, s, p)).double().permute(0, 3, 1, 2)
    z = torch.nn.functional.batch_norm(y, torch.from_numpy(mean).double(), torch.from_numpy(var).double(),
                                       torch.from_numpy(gamma).double(), torch.from_numpy(beta).double(),
                                       training=False, eps=eps).permute(0, 2, 3, 1).numpy()
    # torch evaluates (y - mean) / sqrt(var + eps) * gamma + beta; the oracle multiplies first.
    # Away from |z| ~ 1e-12 the sign is the same; such ties do not occur with these parameters.
    assert np.abs(z[z != 0]).min() > 1e-9
    words = (Cout + 63) // 64
    bits = np.zeros(z.shape[:-1] + (words * 64,), dtype=bool)
    bits[..., :Cout] = z < 0
    ref = np.packbits(bits, axis=-1, bitorder="little").view("<u8")
    assert np.array_equal(got, ref)


def test_bnsign_closed_forms(oracle):
    N, H, W, Cin, Cout, k, s, p = 1, 6, 5, 64, 66, 3, 1, 1
    x = wl.activations((N, H, W, Cin), 94)
    wf = wl.weights((Cout, k, k, Cin), 95)
    y = oracle.bconv2d(x, wf, s, p)
    one, zero = np.ones(Cout, np.float32), np.zeros(Cout, np.float32)

    def pack(b):
        full = np.zeros(b.shape[:-1] + (128,), dtype=bool)
        full[..., :Cout] = b
        return np.packbits(full, axis=-1, bitorder="little").view("<u8")

    # identity batch-norm: the bit is y < 0 (y == 0 counts as +1)
    assert np.array_equal(oracle.bconv2d_bnsign(x, wf, one, zero, zero, one, 0.0, s, p), pack(y < 0))
    # a pure threshold: gamma = 2, mean = m  ->  bit = y < m
    m = np.arange(Cout, dtype=np.float32) - 30.5
    assert np.array_equal(oracle.bconv2d_bnsign(x, wf, 2 * one, zero, m, one, 0.0, s, p), pack(y < m))
    # negative gamma reverses the comparison
    assert np.array_equal(oracle.bconv2d_bnsign(x, wf, -one, zero, m, one, 0.0, s, p), pack(y > m))
    # a huge shift decides everything: all +1 (no bit) or all -1 (every real channel, tail still 0)
    big = 1e6 * one
    assert not oracle.bconv2d_bnsign(x, wf, one, big, zero, one, 0.0, s, p).any()
    allneg = oracle.bconv2d_bnsign(x, wf, one, -big, zero, one, 0.0, s, p)
    assert np.all(allneg[..., 0] == np.uint64(0xFFFFFFFFFFFFFFFF)) and np.all(allneg[..., 1] == np.uint64(3))


# ---- zero-padded variant (ONNX Convolution semantics; Table 1 caption, Sec. 3) -----------------

def _valid_taps(H, W, k, s, p, ho, wo):
    return [(i, j) for i in range(k) for j in range(k)
            if 0 <= ho * s - p + i < H and 0 <= wo * s - p + j < W]


@pytest.mark.parametrize("shape", SHAPES + [(2, 14, 14, 64, 16, 3, 1, 1), (1, 14, 14, 128, 8, 3, 2, 1)])
def test_zeropad_against_torch_cpu_conv2d(oracle, shape):
    """Library routine: torch's conv2d pads with zeros by definition."""
    N, H, W, Cin, Cout, k, s, p = shape
    A = oracle.sign(wl.activations((N, H, W, Cin), 61))
    Wt = wl.weights((Cout, k, k, Cin), 62, p_plus=0.3)
    y = oracle.bconv2d_zeropad_signed(A, Wt, s, p)
    ref = torch.nn.functional.conv2d(torch.from_numpy(A).permute(0, 3, 1, 2).double(),
                                     torch.from_numpy(Wt).permute(0, 3, 1, 2).double(),
                                     stride=s, padding=p).permute(0, 2, 3, 1)
    assert y.dtype == np.int32
    assert np.array_equal(y, ref.numpy().astype(np.int32))


@pytest.mark.parametrize("shape", SHAPES)
def test_zeropad_closed_forms_and_relation_to_plus_one_padding(oracle, shape):
    N, H, W, Cin, Cout, k, s, p = shape
    ones_a = np.ones((N, H, W, Cin), np.float32)
    ones_w = np.ones((Cout, k, k, Cin), np.float32)
    A = oracle.sign(wl.activations((N, H, W, Cin), 63))
    Wt = wl.weights((Cout, k, k, Cin), 64, p_plus=0.3)
    y1 = oracle.bconv2d_zeropad_signed(ones_a, ones_w, s, p)
    y0 = oracle.bconv2d_zeropad_signed(A, Wt, s, p)
    yp = oracle.bconv2d_signed(A, Wt, s, p)
    Ho, Wo = y0.shape[1:3]
    for ho in range(Ho):
        for wo in range(Wo):
            taps = _valid_taps(H, W, k, s, p, ho, wo)
            # all +1: the output counts the taps inside the image
            assert np.all(y1[:, ho, wo, :] == len(taps) * Cin)
            # bounded by, and of the parity of, the number of products actually summed
            assert np.all(np.abs(y0[:, ho, wo, :]) <= len(taps) * Cin)
            assert np.all((y0[:, ho, wo, :] - len(taps) * Cin) % 2 == 0)
            # +1 padding adds the plain sum of the weights under every outside tap
            outside = [(i, j) for i in range(k) for j in range(k) if (i, j) not in taps]
            extra = sum(Wt[:, i, j, :].sum(axis=-1) for i, j in outside) if outside else 0
            assert np.array_equal(yp[:, ho, wo, :] - y0[:, ho, wo, :],
                                  np.broadcast_to(np.asarray(extra, np.int64), (N, Cout)))
    if p == 0:
        assert np.array_equal(y0, yp)
    assert np.array_equal(oracle.bconv2d_zeropad_signed(A, -Wt, s, p), -y0)


@pytest.mark.parametrize("H,W,Cin,k,s,p", [(2, 2, 2, 3, 1, 1), (3, 3, 1, 3, 2, 1), (3, 2, 1, 3, 1, 2)])
def test_zeropad_brute_force_all_activation_patterns(oracle, H, W, Cin, k, s, p):
    """Every activation sign pattern against a definition over Python ints."""
    Cout = 2
    Wt = wl.weights((Cout, k, k, Cin), 65)
    Ho, Wo = (H + 2 * p - k) // s + 1, (W + 2 * p - k) // s + 1
    for bits in range(1 << (H * W * Cin)):
        a = np.array([1.0 if (bits >> t) & 1 else -1.0 for t in range(H * W * Cin)],
                     np.float32).reshape(1, H, W, Cin)
        y = oracle.bconv2d_zeropad_signed(a, Wt, s, p)
        for ho, wo, co in itertools.product(range(Ho), range(Wo), range(Cout)):
            acc = 0
            for i, j in _valid_taps(H, W, k, s, p, ho, wo):
                for c in range(Cin):
                    acc += int(a[0, ho * s - p + i, wo * s - p + j, c]) * int(Wt[co, i, j, c])
            assert y[0, ho, wo, co] == acc


# ---- BGEMM (Sec. 2.1.2, Eq. 1) and the patch matrix ---------------------------------------------

BGEMM_SHAPES = [(1, 1, 1), (3, 5, 7), (17, 9, 64), (8, 33, 100), (70, 16, 576), (5, 4, 1300)]


@pytest.mark.parametrize("M,N,K", BGEMM_SHAPES)
def test_bgemm_against_numpy_matmul_and_popcount(oracle, M, N, K):
    A = oracle.sign(wl.activations((M, K), 71 + M))
    B = wl.weights((N, K), 72 + N, p_plus=0.4)
    dot = oracle.bgemm_signed(A, B, oracle.BGEMM_SIGNED)
    cnt = oracle.bgemm_signed(A, B, oracle.BGEMM_MATCHES)
    # library routine, fp64
    assert np.array_equal(dot, (A.astype(np.float64) @ B.astype(np.float64).T).astype(np.int32))
    # Eq. 1 on packed words with Python integers: bitcount(xnor) over the K real bits
    mask = (1 << K) - 1
    abits = [int("".join("1" if v < 0 else "0" for v in row[::-1]), 2) for row in A]
    bbits = [int("".join("1" if v < 0 else "0" for v in row[::-1]), 2) for row in B]
    for i in range(M):
        for j in range(N):
            assert cnt[i, j] == bin(~(abits[i] ^ bbits[j]) & mask).count("1")
    assert np.array_equal(dot, 2 * cnt - K)
    assert cnt.min() >= 0 and cnt.max() <= K


def test_bgemm_closed_forms(oracle):
    M, N, K = 6, 5, 130
    A = oracle.sign(wl.activations((M, K), 73))
    assert np.all(np.diag(oracle.bgemm_signed(A, A)) == K)
    assert np.all(np.diag(oracle.bgemm_signed(A, A, oracle.BGEMM_MATCHES)) == K)
    assert np.all(np.diag(oracle.bgemm_signed(A, -A)) == -K)
    assert np.all(np.diag(oracle.bgemm_signed(A, -A, oracle.BGEMM_MATCHES)) == 0)
    B = wl.weights((N, K), 74)
    assert np.array_equal(oracle.bgemm_signed(A, B).T, oracle.bgemm_signed(B, A))
    # a single flipped position changes exactly one row of the dot products by 2 * b_jk
    A2 = A.copy()
    A2[2, 17] = -A2[2, 17]
    d = oracle.bgemm_signed(A2, B) - oracle.bgemm_signed(A, B)
    assert not d[[0, 1, 3, 4, 5]].any() and np.array_equal(d[2], (2 * A2[2, 17] * B[:, 17]).astype(np.int32))


@pytest.mark.parametrize("shape", SHAPES)
def test_im2col_bgemm_equals_direct_convolution(oracle, shape):
    """The patch matrix times the filter matrix is the (separately pinned) direct convolution;
    its rows are checked element by element against the tensor as well."""
    N, H, W, Cin, Cout, k, s, p = shape
    A = oracle.sign(wl.activations((N, H, W, Cin), 75))
    Wt = wl.weights((Cout, k, k, Cin), 76, p_plus=0.3)
    cols = oracle.im2col_signed(A, k, k, s, p)
    y = oracle.bconv2d_signed(A, Wt, s, p)
    Ho, Wo = y.shape[1:3]
    assert cols.shape == (N * Ho * Wo, k * k, Cin)
    for n, ho, wo in itertools.product(range(N), range(Ho), range(Wo)):
        row = cols[(n * Ho + ho) * Wo + wo]
        for i, j in itertools.product(range(k), range(k)):
            hi, wi = ho * s - p + i, wo * s - p + j
            want = A[n, hi, wi] if (0 <= hi < H and 0 <= wi < W) else np.ones(Cin, np.float32)
            assert np.array_equal(row[i * k + j], want)
    g = oracle.bgemm_signed(cols.reshape(cols.shape[0], -1), Wt.reshape(Cout, -1))
    assert np.array_equal(g.reshape(y.shape), y)


# ---- int32 bit-packing (Sec. 2.1.1) and the NC1HWC2 layout (Sec. 2.1.2) --------------------------

@pytest.mark.parametrize("C", [1, 63, 64, 65, 130, 256])
def test_bitpack_i32_matches_numpy_packbits(oracle, C):
    rng = np.random.default_rng(81 + C)
    x = rng.integers(-5, 6, size=(7, 3, C)).astype(np.int32)
    x[0, 0, :] = np.iinfo(np.int32).min
    x[0, 1, :] = np.iinfo(np.int32).max
    x[0, 2, :] = 0
    got = oracle.bitpack_i32(x)
    pad = (-C) % 64
    bits = np.pad(x < 0, ((0, 0), (0, 0), (0, pad)))
    want = np.packbits(bits, axis=-1, bitorder="little").view(np.uint64)
    assert np.array_equal(got, want.reshape(got.shape))
    # an int32 and the float of the same sign pack alike, zero included (its sign bit is clear)
    assert np.array_equal(got, oracle.bitpack(x.astype(np.float32)))


@pytest.mark.parametrize("Cw", [1, 2, 3, 8])
def test_nc1hwc2_is_a_grouped_transpose(oracle, Cw):
    rng = np.random.default_rng(90 + Cw)
    a = rng.integers(0, 2**63, size=(2, 3, 5, Cw), dtype=np.uint64)
    got = oracle.nhwc_to_nc1hwc2(a)
    C1 = (Cw + 1) // 2
    padded = np.zeros((2, 3, 5, 2 * C1), np.uint64)
    padded[..., :Cw] = a
    want = padded.reshape(2, 3, 5, C1, 2).transpose(0, 3, 1, 2, 4)
    assert got.shape == (2, C1, 3, 5, 2) and np.array_equal(got, want)
    # bit c of a pixel sits in group c // 128, at bit c % 128 of that group's two words
    for c in (0, 63, 64 * Cw - 1):
        g, b = divmod(c, 128)
        assert ((got[1, g, 2, 4, b // 64] >> np.uint64(b % 64)) & np.uint64(1)) == \
               ((a[1, 2, 4, c // 64] >> np.uint64(c % 64)) & np.uint64(1))


# ---- fused BN + shortcut + sign + pack layer (Sec. 2.1.1 last sentence; Sec. 2.3 Bi-Real) --------

@pytest.mark.parametrize("C", [1, 64, 80, 200])
@pytest.mark.parametrize("with_r", [False, True])
def test_bn_sign_pack_against_numpy_float32(oracle, C, with_r):
    """numpy evaluates float32 expressions one rounded operation at a time, without fused
    multiply-add: the same arithmetic, written independently."""
    rng = np.random.default_rng(500 + C + with_r)
    y = rng.integers(-576, 577, size=(3, 11, C)).astype(np.int32)
    scale = rng.uniform(-0.2, 0.2, C).astype(np.float32)
    scale[::5] = 0.0
    shift = rng.normal(0, 1, C).astype(np.float32)
    r = rng.normal(0, 2, y.shape).astype(np.float32) if with_r else None
    x, bits = oracle.bn_sign_pack(y, scale, shift, r)
    z = scale * y.astype(np.float32)
    assert z.dtype == np.float32
    z = z + shift
    if with_r:
        z = z + r
    assert np.array_equal(x.view(np.uint32), z.view(np.uint32))          # bit for bit, -0.0 included
    assert np.array_equal(bits, oracle.bitpack(z))                        # sign rule of Sec. 2.1.1
    # the fp64 value agrees to float32 rounding, so no term was dropped or mis-signed
    z64 = scale.astype(np.float64) * y + shift + (r if with_r else 0.0)
    assert np.allclose(x, z64, rtol=0, atol=1e-4)
    assert oracle.bn_sign_pack(y, scale, shift, r, want_x=False)[0] is None


def test_bn_sign_pack_closed_forms(oracle):
    C = 70
    y = np.tile(np.arange(-35, 35, dtype=np.int32), (2, 1))
    one, zero = np.ones(C, np.float32), np.zeros(C, np.float32)
    x, bits = oracle.bn_sign_pack(y, one, zero)
    assert np.array_equal(x, y.astype(np.float32))
    assert np.array_equal(bits, oracle.bitpack_i32(y))                   # sign(y) itself
    x, bits = oracle.bn_sign_pack(y, -one, zero)
    # -1 * 0 = -0.0, but -0.0 + (+0.0 shift) = +0.0 under round-to-nearest: y = 0 packs as +1
    assert np.array_equal(bits, oracle.bitpack_i32(-y))
    assert not np.signbit(x[y == 0]).any()
    x, bits = oracle.bn_sign_pack(y, zero, one * 3, r=-4 * np.ones(y.shape, np.float32))
    assert np.all(x == -1.0) and np.array_equal(bits, oracle.bitpack(x))
