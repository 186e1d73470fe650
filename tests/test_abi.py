"""CPU-side checks of the C ABI: the library loads, exports every symbol include/dabnn.h
declares, and rejects bad arguments on the host without launching anything (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_1908_05858_amd", "libdabnn.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_1908_05858_amd import build
        build.build_library()
    from paper_1908_05858_amd import binding
    return binding.load()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "dabnn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dabnn_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert "dabnn_bitpack" in names and "dabnn_bconv2d" in names and "dabnn_pack_weights" in names
    for name in names:
        assert hasattr(lib, name), name
    from paper_1908_05858_amd import binding
    assert sorted(binding.EXPORTS) == names


def test_host_helpers(lib):
    assert lib.dabnn_packed_words(1) == 1 and lib.dabnn_packed_words(64) == 1
    assert lib.dabnn_packed_words(65) == 2 and lib.dabnn_packed_words(200) == 4
    assert lib.dabnn_packed_words(0) == -1
    assert lib.dabnn_conv_out_dim(56, 3, 1, 1) == 56
    assert lib.dabnn_conv_out_dim(56, 3, 2, 1) == 28
    assert lib.dabnn_conv_out_dim(7, 3, 2, 1) == 4
    assert lib.dabnn_conv_out_dim(2, 3, 1, 0) == -1
    assert lib.dabnn_conv_out_dim(5, 3, 1, 3) == -1
    assert lib.dabnn_status_string(0) == b"ok"
    assert lib.dabnn_status_string(99) == b"unknown status"


def test_bad_arguments_are_refused_before_any_launch(lib):
    P = ctypes.c_void_p
    good, good8, odd = P(0x10000), P(0x20000), P(0x10002)
    # bitpack
    assert lib.dabnn_bitpack(P(0), good8, 4, 64, 0, None) == 1
    assert lib.dabnn_bitpack(good, P(0), 4, 64, 0, None) == 1
    assert lib.dabnn_bitpack(good, good8, -1, 64, 0, None) == 2
    assert lib.dabnn_bitpack(good, good8, 4, 0, 0, None) == 2
    assert lib.dabnn_bitpack(odd, good8, 4, 64, 0, None) == 3
    assert lib.dabnn_bitpack(good, P(0x20004), 4, 64, 0, None) == 3
    assert lib.dabnn_bitpack(good, good8, 4, 64, 7, None) == 4
    assert lib.dabnn_bitpack(P(0), P(0), 0, 64, 0, None) == 0      # empty: nothing to do
    # pack_weights
    assert lib.dabnn_pack_weights(P(0), good8, 4, 3, 3, 64, 0, None) == 1
    assert lib.dabnn_pack_weights(good, good8, 0, 3, 3, 64, 0, None) == 2
    assert lib.dabnn_pack_weights(good, P(0x20004), 4, 3, 3, 64, 0, None) == 3
    assert lib.dabnn_pack_weights(good, good8, 4, 3, 3, 64, 2, None) == 4
    # bconv2d: (a, w, y, N, H, W, Cin, Cout, kh, kw, stride, pad, stream)
    a, w, y = P(0x10000), P(0x20000), P(0x30000)
    assert lib.dabnn_bconv2d(P(0), w, y, 1, 4, 4, 64, 8, 3, 3, 1, 1, None) == 1
    assert lib.dabnn_bconv2d(a, w, P(0), 1, 4, 4, 64, 8, 3, 3, 1, 1, None) == 1
    assert lib.dabnn_bconv2d(a, w, y, 0, 4, 4, 64, 8, 3, 3, 1, 1, None) == 2
    assert lib.dabnn_bconv2d(a, w, y, 1, 4, 4, 64, 8, 3, 3, 0, 1, None) == 2   # stride 0
    assert lib.dabnn_bconv2d(a, w, y, 1, 4, 4, 64, 8, 3, 3, 1, 3, None) == 2   # pad >= k
    assert lib.dabnn_bconv2d(a, w, y, 1, 2, 2, 64, 8, 5, 5, 1, 0, None) == 2   # empty output
    assert lib.dabnn_bconv2d(a, w, y, 1 << 20, 1 << 10, 1 << 10, 64, 8, 3, 3, 1, 1, None) == 2
    assert lib.dabnn_bconv2d(P(0x10004), w, y, 1, 4, 4, 64, 8, 3, 3, 1, 1, None) == 3
    assert lib.dabnn_bconv2d(a, w, P(0x30002), 1, 4, 4, 64, 8, 3, 3, 1, 1, None) == 3
    assert lib.dabnn_bconv2d_algo(a, w, y, 1, 4, 4, 64, 8, 3, 3, 1, 1, 9, None) == 4
    assert lib.dabnn_bconv2d_algo(a, w, y, 1, 4, 4, 64, 8, 5, 5, 1, 2, 2, None) == 4  # wreg is 3x3 only


def test_pick_algo(lib):
    assert lib.dabnn_bconv2d_pick_algo(256, 56, 56, 64, 64, 3, 3, 1, 1) in (2, 3)
    assert lib.dabnn_bconv2d_pick_algo(1, 56, 56, 64, 64, 5, 5, 1, 2) == 1
    assert lib.dabnn_bconv2d_pick_algo(1, 56, 56, 64, 64, 3, 3, 0, 1) == -1


def test_tensors_past_the_32bit_byte_offsets_leave_the_activation_stationary_family(lib):
    """The activation-stationary kernels address window taps with 32-bit byte offsets: a packed
    activation tensor of 4 GiB or more must be routed to a family that indexes with size_t."""
    AREG = 3
    # 8200 x 8200 pixels x 8 words = 4.30 GB of packed activations (below 2^31 words: a valid shape)
    assert lib.dabnn_bconv2d_pick_algo(1, 8200, 8200, 512, 16, 3, 3, 1, 1) not in (AREG, -1)
    # the same tensor with a channel count the fused modes would take (Cout % 64 == 0), stride 2
    assert lib.dabnn_bconv2d_pick_algo(1, 8200, 8200, 512, 64, 3, 3, 2, 1) not in (AREG, -1)
    # just below the limit the family is still used: 8192 x 8191 x 8 words x 8 B < 2^32
    assert lib.dabnn_bconv2d_pick_algo(1, 8192, 8191, 512, 16, 3, 3, 1, 1) == AREG
    assert lib.dabnn_bconv2d_pick_algo(1, 8192, 8192, 512, 16, 3, 3, 1, 1) != AREG
    # the 64 pixels of an output tile are addressed with a 32-bit byte offset too: 64 * Cout * 4 < 2^32
    assert lib.dabnn_bconv2d_pick_algo(1, 8, 8, 64, (1 << 24) - 16, 3, 3, 1, 1) == AREG
    assert lib.dabnn_bconv2d_pick_algo(1, 8, 8, 64, 1 << 24, 3, 3, 1, 1) not in (AREG, -1)


def test_bgemm_route_stops_where_an_output_tile_passes_32bit_byte_offsets(lib):
    """The BGEMM kernel (here through a 1x1 convolution) addresses the 64 rows of an output tile
    with 32-bit byte offsets: 64 rows of N int32 must stay below 4 GiB."""
    BGEMM = 4
    assert lib.dabnn_bconv2d_pick_algo(1, 1, 64, 64, (1 << 24) - 16, 1, 1, 1, 0) == BGEMM
    assert lib.dabnn_bconv2d_pick_algo(1, 1, 64, 64, 1 << 24, 1, 1, 1, 0) not in (BGEMM, -1)


def test_every_word_count_has_a_tuned_kernel(lib):
    """3x3 convolutions of any channel count resolve to the activation-stationary family: one
    launch up to 8 words per pixel, several that add up above."""
    AREG = 3
    for Cin in (1, 64, 100, 160, 192, 320, 384, 448, 512, 576, 704, 768, 1024, 1088, 2048, 4100):
        for Cout, stride in ((64, 1), (16, 2), (48, 1)):
            assert lib.dabnn_bconv2d_pick_algo(4, 14, 14, Cin, Cout, 3, 3, stride, 1) == AREG, (Cin, Cout)
    # direct stores (Cout % 16 != 0) exist for up to 8 words per pixel: 4-channel groups, 8 where
    # the word count is odd; everything else is left to the other families
    assert lib.dabnn_bconv2d_pick_algo(4, 14, 14, 64, 12, 3, 3, 1, 1) != AREG
    assert lib.dabnn_bconv2d_pick_algo(4, 14, 14, 128, 12, 3, 3, 1, 1) == AREG
    assert lib.dabnn_bconv2d_pick_algo(4, 14, 14, 320, 24, 3, 3, 1, 1) == AREG
    assert lib.dabnn_bconv2d_pick_algo(4, 14, 14, 576, 24, 3, 3, 1, 1) != AREG


def test_options(lib):
    """Options default to 0, are set and read back through the C ABI, and unknown ones are refused;
    the library ignores the environment."""
    import os
    n_options = 11
    text = open(os.path.join(ROOT, "include", "dabnn.h")).read()
    assert f"DABNN_OPT_COUNT = {n_options}" in text
    for opt in range(n_options):
        assert lib.dabnn_get_option(opt) == 0
    assert lib.dabnn_set_option(2, 16) == 0 and lib.dabnn_get_option(2) == 16
    assert lib.dabnn_set_option(2, 0) == 0 and lib.dabnn_get_option(2) == 0
    assert lib.dabnn_set_option(n_options, 1) == 4 and lib.dabnn_set_option(-1, 1) == 4
    assert lib.dabnn_set_option(0, -5) == 4
    assert lib.dabnn_get_option(n_options) == -1
    src = os.path.join(ROOT, "paper_1908_05858_amd", "csrc")
    for name in os.listdir(src):
        assert "getenv" not in open(os.path.join(src, name)).read(), name


def test_bn_thresholds_match_fp64_batch_norm_for_every_integer(lib):
    """The host helper, exhaustively: for every integer y in [-K, K] the threshold rule equals
    the sign of the fp64 batch-norm (numpy, evaluated in the same order)."""
    import numpy as np
    rng = np.random.default_rng(5)
    C, K = 200, 576
    gamma = rng.uniform(-2, 2, C).astype(np.float32)
    gamma[::9] = 0.0
    gamma[1] = 1e-30
    beta = rng.normal(0, 1.0, C).astype(np.float32)
    beta[3] = 0.0
    mean = rng.normal(0, 60.0, C).astype(np.float32)
    mean[3] = 17.0          # z is exactly 0 at y = 17: counts as +1
    mean[5] = 1e9           # never crosses zero inside [-K, K]
    var = rng.uniform(0.1, 90.0, C).astype(np.float32)
    eps = np.float32(1e-5)
    thr = np.empty(C, np.int32)
    flip = np.empty((C + 63) // 64, np.uint64)
    P = ctypes.c_void_p
    rc = lib.dabnn_bn_thresholds(P(gamma.ctypes.data), P(beta.ctypes.data), P(mean.ctypes.data),
                                 P(var.ctypes.data), ctypes.c_float(eps), C, K, P(thr.ctypes.data),
                                 P(flip.ctypes.data))
    assert rc == 0
    y = np.arange(-K, K + 1, dtype=np.float64)[:, None]
    z = gamma.astype(np.float64) * (y - mean.astype(np.float64)) / np.sqrt(var.astype(np.float64) + np.float64(eps)) \
        + beta.astype(np.float64)
    want = z < 0
    fl = np.array([(int(flip[c // 64]) >> (c % 64)) & 1 for c in range(C)], dtype=bool)
    got = (np.arange(-K, K + 1)[:, None] < thr[None, :]) ^ fl[None, :]
    assert np.array_equal(got, want)
    assert np.all(np.abs(thr) <= K + 1)
    # bad arguments
    assert lib.dabnn_bn_thresholds(P(0), P(beta.ctypes.data), P(mean.ctypes.data), P(var.ctypes.data),
                                   ctypes.c_float(eps), C, K, P(thr.ctypes.data), P(flip.ctypes.data)) == 1
    assert lib.dabnn_bn_thresholds(P(gamma.ctypes.data), P(beta.ctypes.data), P(mean.ctypes.data),
                                   P(var.ctypes.data), ctypes.c_float(eps), 0, K, P(thr.ctypes.data),
                                   P(flip.ctypes.data)) == 2


def test_bnsign_bad_arguments(lib):
    P = ctypes.c_void_p
    a, w, t, f, o = P(0x10000), P(0x20000), P(0x30000), P(0x40000), P(0x50000)
    assert lib.dabnn_bconv2d_bnsign(a, w, P(0), f, o, 1, 4, 4, 64, 64, 3, 3, 1, 1, None) == 1
    assert lib.dabnn_bconv2d_bnsign(a, w, t, f, P(0), 1, 4, 4, 64, 64, 3, 3, 1, 1, None) == 1
    assert lib.dabnn_bconv2d_bnsign(a, w, t, f, o, 1, 4, 4, 64, 0, 3, 3, 1, 1, None) == 2
    assert lib.dabnn_bconv2d_bnsign(a, w, t, P(0x40004), o, 1, 4, 4, 64, 64, 3, 3, 1, 1, None) == 3


def test_zeropad_bad_arguments(lib):
    P = ctypes.c_void_p
    a, w, y = P(0x10000), P(0x20000), P(0x30000)
    assert lib.dabnn_bconv2d_zeropad(a, w, P(0), 1, 4, 4, 64, 64, 3, 3, 1, 1, None) == 1
    assert lib.dabnn_bconv2d_zeropad(a, w, y, 1, 4, 4, 64, 64, 3, 3, 1, 3, None) == 2   # pad >= k
    assert lib.dabnn_bconv2d_zeropad(a, w, y, 1, 4, 4, 64, 64, 3, 3, 0, 1, None) == 2   # stride 0
    assert lib.dabnn_bconv2d_zeropad(a, w, P(0x30002), 1, 4, 4, 64, 64, 3, 3, 1, 1, None) == 3


def test_bgemm_and_im2col_bad_arguments(lib):
    P = ctypes.c_void_p
    A, B, C = P(0x10000), P(0x20000), P(0x30000)
    assert lib.dabnn_bgemm(A, B, P(0), 4, 4, 1, 64, 0, None) == 1
    assert lib.dabnn_bgemm(A, B, C, 0, 4, 1, 64, 0, None) == 2
    assert lib.dabnn_bgemm(A, B, C, 4, 4, 1, 65, 0, None) == 2       # K exceeds the row's bits
    assert lib.dabnn_bgemm(A, B, C, 4, 4, 1, 0, 0, None) == 2
    assert lib.dabnn_bgemm(A, B, C, 1 << 20, 1 << 12, 1, 64, 0, None) == 2  # C too large
    assert lib.dabnn_bgemm(P(0x10004), B, C, 4, 4, 1, 64, 0, None) == 3
    assert lib.dabnn_bgemm(A, B, C, 4, 4, 1, 64, 2, None) == 4       # unknown mode
    assert lib.dabnn_im2col(A, P(0), 1, 4, 4, 64, 3, 3, 1, 1, None) == 1
    assert lib.dabnn_im2col(A, B, 1, 4, 4, 64, 3, 3, 1, 3, None) == 2
    assert lib.dabnn_im2col(A, P(0x20001), 1, 4, 4, 64, 3, 3, 1, 1, None) == 3


def test_int8_route_bad_arguments(lib):
    P = ctypes.c_void_p
    a, w, y = P(0x10000), P(0x20000), P(0x30000)
    assert lib.dabnn_expand_int8(a, P(0), 4, 64, None) == 1
    assert lib.dabnn_expand_int8(a, w, -1, 64, None) == 2
    assert lib.dabnn_expand_int8(a, P(0x20008), 4, 64, None) == 3
    assert lib.dabnn_expand_int8(a, w, 4, 80, None) == 4
    assert lib.dabnn_expand_int8(P(0), P(0), 0, 64, None) == 0
    assert lib.dabnn_bconv2d_int8(a, w, P(0), 1, 4, 4, 64, 64, 3, 3, 1, 1, None) == 1
    assert lib.dabnn_bconv2d_int8(a, w, y, 1, 4, 4, 64, 64, 3, 3, 1, 3, None) == 2
    assert lib.dabnn_bconv2d_int8(P(0x10008), w, y, 1, 4, 4, 64, 64, 3, 3, 1, 1, None) == 3
    assert lib.dabnn_bconv2d_int8(a, w, y, 1, 4, 4, 80, 64, 3, 3, 1, 1, None) == 4
    assert lib.dabnn_bconv2d_int8(a, w, y, 1, 4, 4, 64, 48, 3, 3, 1, 1, None) == 4


def test_mfma_route_bad_arguments_and_buffer_size(lib):
    """The matrix-core route fed from packed bits: buffer size on the host, and every refusal
    before any launch."""
    P = ctypes.c_void_p
    a, w, y = P(0x10000), P(0x20000), P(0x30000)
    for Cin, Cout in ((64, 64), (128, 256), (256, 512), (512, 512)):
        assert lib.dabnn_mfma_weights_bytes(Cin, Cout, 3, 3, 0) == Cout * 9 * Cin + 4 * Cout
        assert lib.dabnn_mfma_weights_bytes(Cin, Cout, 3, 3, 1) == Cout * 9 * Cin // 2 + 4 * Cout
    for Cin, Cout, k in ((80, 64, 3), (192, 64, 3), (64, 32, 3), (64, 64, 1), (0, 64, 3), (64, 16384, 3)):
        assert lib.dabnn_mfma_weights_bytes(Cin, Cout, k, k, 0) == 0
    assert lib.dabnn_mfma_weights_bytes(64, 64, 3, 3, 2) == 0
    for fmt in (0, 1):
        assert lib.dabnn_prepare_weights_mfma(P(0), w, 64, 64, 3, 3, fmt, None) == 1
        assert lib.dabnn_prepare_weights_mfma(a, w, 64, 0, 3, 3, fmt, None) == 2
        assert lib.dabnn_prepare_weights_mfma(a, P(0x20008), 64, 64, 3, 3, fmt, None) == 3
        assert lib.dabnn_prepare_weights_mfma(a, w, 80, 64, 3, 3, fmt, None) == 4
        assert lib.dabnn_bconv2d_mfma(a, w, P(0), 1, 4, 4, 64, 64, 3, 3, 1, 1, fmt, None) == 1
        assert lib.dabnn_bconv2d_mfma(a, w, y, 1, 4, 4, 64, 64, 3, 3, 1, 3, fmt, None) == 2
        assert lib.dabnn_bconv2d_mfma(P(0x10008), w, y, 1, 4, 4, 64, 64, 3, 3, 1, 1, fmt, None) == 3
        assert lib.dabnn_bconv2d_mfma(a, w, y, 1, 4, 4, 64, 64, 3, 3, 3, 1, fmt, None) == 4
        assert lib.dabnn_bconv2d_mfma(a, w, y, 1, 4, 4, 320, 64, 3, 3, 1, 1, fmt, None) == 4
        assert lib.dabnn_bconv2d_mfma(a, w, y, 1, 4, 4, 64, 96, 3, 3, 1, 1, fmt, None) == 4
        assert lib.dabnn_bconv2d_bnsign_mfma(a, w, P(0), y, y, 1, 4, 4, 64, 64, 3, 3, 1, 1, fmt, None) == 1
        assert lib.dabnn_bconv2d_bnsign_mfma(a, w, y, y, y, 1, 4, 4, 64, 64, 3, 3, 1, 3, fmt, None) == 2
        assert lib.dabnn_bconv2d_bnsign_mfma(a, w, P(0x30002), y, y, 1, 4, 4, 64, 64, 3, 3, 1, 1, fmt, None) == 3
        assert lib.dabnn_bconv2d_bnsign_mfma(a, w, y, y, y, 1, 4, 4, 64, 96, 3, 3, 1, 1, fmt, None) == 4
    assert lib.dabnn_prepare_weights_mfma(a, w, 64, 64, 3, 3, 7, None) == 4
    assert lib.dabnn_bconv2d_mfma(a, w, y, 1, 4, 4, 64, 64, 3, 3, 1, 1, -1, None) == 4


def test_layout_and_int32_pack_bad_arguments(lib):
    P = ctypes.c_void_p
    a, o = P(0x10000), P(0x20000)
    assert lib.dabnn_bitpack_i32(a, P(0), 4, 64, None) == 1
    assert lib.dabnn_bitpack_i32(a, o, 4, 0, None) == 2
    assert lib.dabnn_bitpack_i32(P(0x10002), o, 4, 64, None) == 3
    assert lib.dabnn_bitpack_i32(P(0), P(0), 0, 64, None) == 0
    for f in (lib.dabnn_nhwc_to_nc1hwc2, lib.dabnn_nc1hwc2_to_nhwc):
        assert f(a, P(0), 1, 2, 2, 3, None) == 1
        assert f(a, o, 1, 0, 2, 3, None) == 2
        assert f(a, P(0x20004), 1, 2, 2, 3, None) == 3


def test_bn_sign_pack_bad_arguments(lib):
    P = ctypes.c_void_p
    y, sc, sh, r, x, b = P(0x10000), P(0x20000), P(0x30000), P(0x40000), P(0x50000), P(0x60000)
    assert lib.dabnn_bn_sign_pack(y, sc, P(0), r, x, b, 4, 64, None) == 1
    assert lib.dabnn_bn_sign_pack(y, sc, sh, P(0), P(0), P(0), 4, 64, None) == 1   # bits is required
    assert lib.dabnn_bn_sign_pack(y, sc, sh, r, x, b, -1, 64, None) == 2
    assert lib.dabnn_bn_sign_pack(y, sc, sh, P(0x40002), x, b, 4, 64, None) == 3
    assert lib.dabnn_bn_sign_pack(P(0), P(0), P(0), P(0), P(0), P(0), 0, 64, None) == 0


def test_bn_residual_bad_arguments(lib):
    P = ctypes.c_void_p
    a, w, sc, sh, r, x, b = (P(v) for v in (0x10000, 0x20000, 0x30000, 0x40000, 0x50000, 0x60000, 0x70000))
    args = (1, 4, 4, 64, 64, 3, 3, 1, 1, None)
    assert lib.dabnn_bconv2d_bn_residual(a, w, sc, sh, r, P(0), b, *args) == 1    # x_out is required
    assert lib.dabnn_bconv2d_bn_residual(a, w, P(0), sh, r, x, b, *args) == 1
    assert lib.dabnn_bconv2d_bn_residual(a, w, sc, sh, r, x, b, 1, 4, 4, 64, 64, 3, 3, 1, 3, None) == 2
    assert lib.dabnn_bconv2d_bn_residual(a, w, sc, sh, P(0x50002), x, b, *args) == 3
