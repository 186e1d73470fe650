"""ctypes binding of libdabnn.so: argument marshalling only.

Every function takes torch CUDA tensors (device memory) and enqueues the library's kernels on
torch's current stream.  There is no CPU path: if the HIP library is missing or the tensors are
not on the GPU, the call raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdabnn.so")

SIGN_BIT, SIGN_GE0 = 0, 1
ALGO_AUTO, ALGO_REFERENCE, ALGO_WREG, ALGO_AREG, ALGO_BGEMM = 0, 1, 2, 3, 4

_lib = None


class DabnnError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__(f"{what}: {status_string(status)} (status {status})")


def load():
    """Load libdabnn.so (built beforehand by ``__graft_entry__.build()`` / ``build.py``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = ctypes.CDLL(LIB_PATH)
    i32, i64, vp = ctypes.c_int, ctypes.c_int64, ctypes.c_void_p
    lib.dabnn_packed_words.argtypes, lib.dabnn_packed_words.restype = [i64], i64
    lib.dabnn_conv_out_dim.argtypes, lib.dabnn_conv_out_dim.restype = [i32] * 4, i32
    lib.dabnn_bitpack.argtypes, lib.dabnn_bitpack.restype = [vp, vp, i64, i32, i32, vp], i32
    lib.dabnn_pack_weights.argtypes, lib.dabnn_pack_weights.restype = [vp, vp] + [i32] * 5 + [vp], i32
    lib.dabnn_bconv2d.argtypes, lib.dabnn_bconv2d.restype = [vp] * 3 + [i32] * 9 + [vp], i32
    lib.dabnn_bconv2d_algo.argtypes, lib.dabnn_bconv2d_algo.restype = [vp] * 3 + [i32] * 10 + [vp], i32
    lib.dabnn_bgemm.argtypes, lib.dabnn_bgemm.restype = [vp] * 3 + [i64, i32, i32, i32, i32, vp], i32
    lib.dabnn_im2col.argtypes, lib.dabnn_im2col.restype = [vp] * 2 + [i32] * 8 + [vp], i32
    lib.dabnn_bitpack_i32.argtypes, lib.dabnn_bitpack_i32.restype = [vp, vp, i64, i32, vp], i32
    for f in (lib.dabnn_nhwc_to_nc1hwc2, lib.dabnn_nc1hwc2_to_nhwc):
        f.argtypes, f.restype = [vp, vp] + [i32] * 4 + [vp], i32
    lib.dabnn_bn_sign_pack.argtypes, lib.dabnn_bn_sign_pack.restype = [vp] * 6 + [i64, i32, vp], i32
    lib.dabnn_bconv2d_bn_residual.argtypes = [vp] * 7 + [i32] * 9 + [vp]
    lib.dabnn_bconv2d_bn_residual.restype = i32
    lib.dabnn_expand_int8.argtypes, lib.dabnn_expand_int8.restype = [vp, vp, i64, i32, vp], i32
    lib.dabnn_bconv2d_int8.argtypes, lib.dabnn_bconv2d_int8.restype = [vp] * 3 + [i32] * 9 + [vp], i32
    lib.dabnn_mfma_weights_bytes.argtypes, lib.dabnn_mfma_weights_bytes.restype = [i32] * 5, ctypes.c_size_t
    lib.dabnn_prepare_weights_mfma.argtypes, lib.dabnn_prepare_weights_mfma.restype = [vp, vp] + [i32] * 5 + [vp], i32
    lib.dabnn_bconv2d_mfma.argtypes, lib.dabnn_bconv2d_mfma.restype = [vp] * 3 + [i32] * 10 + [vp], i32
    lib.dabnn_bconv2d_bnsign_mfma.argtypes = [vp] * 5 + [i32] * 10 + [vp]
    lib.dabnn_bconv2d_bnsign_mfma.restype = i32
    lib.dabnn_bconv2d_zeropad.argtypes, lib.dabnn_bconv2d_zeropad.restype = [vp] * 3 + [i32] * 9 + [vp], i32
    lib.dabnn_bconv2d_pick_algo.argtypes, lib.dabnn_bconv2d_pick_algo.restype = [i32] * 9, i32
    lib.dabnn_status_string.argtypes, lib.dabnn_status_string.restype = [i32], ctypes.c_char_p
    lib.dabnn_bconv2d_bnsign.argtypes, lib.dabnn_bconv2d_bnsign.restype = [vp] * 5 + [i32] * 9 + [vp], i32
    lib.dabnn_bn_thresholds.argtypes = [vp] * 4 + [ctypes.c_float, i32, i32, vp, vp]
    lib.dabnn_bn_thresholds.restype = i32
    lib.dabnn_set_option.argtypes, lib.dabnn_set_option.restype = [i32, i32], i32
    lib.dabnn_get_option.argtypes, lib.dabnn_get_option.restype = [i32], i32
    _lib = lib
    return lib


EXPORTS = ["dabnn_packed_words", "dabnn_conv_out_dim", "dabnn_bitpack", "dabnn_pack_weights",
           "dabnn_bconv2d", "dabnn_bconv2d_algo", "dabnn_bconv2d_pick_algo", "dabnn_status_string",
           "dabnn_bconv2d_bnsign", "dabnn_bn_thresholds", "dabnn_bconv2d_zeropad", "dabnn_bgemm", "dabnn_im2col",
           "dabnn_expand_int8", "dabnn_bconv2d_int8", "dabnn_bitpack_i32", "dabnn_nhwc_to_nc1hwc2",
           "dabnn_nc1hwc2_to_nhwc", "dabnn_bn_sign_pack", "dabnn_bconv2d_bn_residual",
           "dabnn_set_option", "dabnn_get_option", "dabnn_mfma_weights_bytes",
           "dabnn_prepare_weights_mfma", "dabnn_bconv2d_mfma", "dabnn_bconv2d_bnsign_mfma"]

(OPT_AREG_SLOTS, OPT_AREG_TAIL, OPT_AREG_STORE, OPT_RES_CHANNELS, OPT_WREG_PIXELS, OPT_BGEMM_COLUMNS,
 OPT_BITPACK_ROWWISE, OPT_AREG_SPLIT, OPT_AREG_RANGES_PER_SIMD, OPT_MFMA_PIXEL_BLOCKS,
 OPT_RES_FUSED) = range(11)


def set_option(option, value):
    """Tuning / test switch of the library (a dabnn_option); 0 restores the default."""
    _check(load().dabnn_set_option(option, value), "dabnn_set_option")


def get_option(option):
    return load().dabnn_get_option(option)


def status_string(status):
    return load().dabnn_status_string(int(status)).decode()


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, dtype, name):
    if not (isinstance(t, torch.Tensor) and t.is_cuda):
        raise TypeError(f"{name} must be a CUDA tensor")
    if t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{name} must be a contiguous {dtype} tensor")
    return ctypes.c_void_p(t.data_ptr())


def _check(rc, what):
    if rc != 0:
        raise DabnnError(rc, what)


def packed_words(C):
    return load().dabnn_packed_words(C)


def conv_out_dim(size, k, stride, pad):
    return load().dabnn_conv_out_dim(size, k, stride, pad)


def bitpack(x, out=None, sign_mode=SIGN_BIT):
    """x: fp32 [..., C] on the GPU -> int64 tensor [..., ceil(C/64)] holding the u64 words."""
    C = x.shape[-1]
    n_pixels = x.numel() // C if C else 0
    words = (C + 63) // 64
    if out is None:
        out = torch.empty(x.shape[:-1] + (words,), dtype=torch.int64, device=x.device)
    _check(load().dabnn_bitpack(_dev(x, torch.float32, "x"), _dev(out, torch.int64, "out"),
                                n_pixels, C, sign_mode, _stream()), "dabnn_bitpack")
    return out


def pack_weights(w, out=None, sign_mode=SIGN_BIT):
    """w: fp32 [Cout, kh, kw, Cin] -> int64 [Cout, kh, kw, ceil(Cin/64)] (canonical layout)."""
    Cout, kh, kw, Cin = w.shape
    if out is None:
        out = torch.empty((Cout, kh, kw, (Cin + 63) // 64), dtype=torch.int64, device=w.device)
    _check(load().dabnn_pack_weights(_dev(w, torch.float32, "w"), _dev(out, torch.int64, "out"),
                                     Cout, kh, kw, Cin, sign_mode, _stream()), "dabnn_pack_weights")
    return out


def bconv2d(a, w, Cin, stride=1, pad=0, out=None, algo=ALGO_AUTO):
    """a: int64 [N,H,W,Cw], w: int64 [Cout,kh,kw,Cw] (packed) -> int32 [N,Ho,Wo,Cout]."""
    N, H, W, Cw = a.shape
    Cout, kh, kw, Cw2 = w.shape
    if Cw != Cw2 or Cw != (Cin + 63) // 64:
        raise ValueError("packed word counts do not match Cin")
    Ho, Wo = conv_out_dim(H, kh, stride, pad), conv_out_dim(W, kw, stride, pad)
    if Ho <= 0 or Wo <= 0:
        raise DabnnError(2, "dabnn_bconv2d")
    if out is None:
        out = torch.empty((N, Ho, Wo, Cout), dtype=torch.int32, device=a.device)
    args = (_dev(a, torch.int64, "a"), _dev(w, torch.int64, "w"), _dev(out, torch.int32, "out"),
            N, H, W, Cin, Cout, kh, kw, stride, pad)
    if algo == ALGO_AUTO:
        rc = load().dabnn_bconv2d(*args, _stream())
    else:
        rc = load().dabnn_bconv2d_algo(*args, algo, _stream())
    _check(rc, "dabnn_bconv2d")
    return out


def bconv2d_zeropad(a, w, Cin, stride=1, pad=0, out=None):
    """As bconv2d, with the zero padding of ONNX Convolution (outside taps contribute nothing)."""
    N, H, W, Cw = a.shape
    Cout, kh, kw, Cw2 = w.shape
    if Cw != Cw2 or Cw != (Cin + 63) // 64:
        raise ValueError("packed word counts do not match Cin")
    Ho, Wo = conv_out_dim(H, kh, stride, pad), conv_out_dim(W, kw, stride, pad)
    if Ho <= 0 or Wo <= 0:
        raise DabnnError(2, "dabnn_bconv2d_zeropad")
    if out is None:
        out = torch.empty((N, Ho, Wo, Cout), dtype=torch.int32, device=a.device)
    _check(load().dabnn_bconv2d_zeropad(_dev(a, torch.int64, "a"), _dev(w, torch.int64, "w"),
                                        _dev(out, torch.int32, "out"), N, H, W, Cin, Cout, kh, kw,
                                        stride, pad, _stream()), "dabnn_bconv2d_zeropad")
    return out


BGEMM_SIGNED, BGEMM_MATCHES = 0, 1


def bgemm(A, B, K, mode=BGEMM_SIGNED, out=None):
    """A: int64 [M,Kw], B: int64 [N,Kw] (packed rows, K real bits) -> int32 [M,N] (Eq. 1)."""
    M, Kw = A.shape
    N, Kw2 = B.shape
    if Kw != Kw2:
        raise ValueError("row lengths differ")
    if out is None:
        out = torch.empty((M, N), dtype=torch.int32, device=A.device)
    _check(load().dabnn_bgemm(_dev(A, torch.int64, "A"), _dev(B, torch.int64, "B"),
                              _dev(out, torch.int32, "out"), M, N, Kw, K, mode, _stream()), "dabnn_bgemm")
    return out


def im2col(a, Cin, kh, kw, stride=1, pad=0, out=None):
    """a: int64 [N,H,W,Cw] -> patch matrix int64 [N*Ho*Wo, kh*kw*Cw] (outside taps zero words)."""
    N, H, W, Cw = a.shape
    if Cw != (Cin + 63) // 64:
        raise ValueError("packed word count does not match Cin")
    Ho, Wo = conv_out_dim(H, kh, stride, pad), conv_out_dim(W, kw, stride, pad)
    if Ho <= 0 or Wo <= 0:
        raise DabnnError(2, "dabnn_im2col")
    if out is None:
        out = torch.empty((N * Ho * Wo, kh * kw * Cw), dtype=torch.int64, device=a.device)
    _check(load().dabnn_im2col(_dev(a, torch.int64, "a"), _dev(out, torch.int64, "out"), N, H, W, Cin,
                               kh, kw, stride, pad, _stream()), "dabnn_im2col")
    return out


def bitpack_i32(x, out=None):
    """x: int32 [..., C] -> int64 [..., ceil(C/64)], bit = 1 iff x < 0."""
    C = x.shape[-1]
    n_pixels = x.numel() // C if C else 0
    if out is None:
        out = torch.empty(tuple(x.shape[:-1]) + ((C + 63) // 64,), dtype=torch.int64, device=x.device)
    _check(load().dabnn_bitpack_i32(_dev(x, torch.int32, "x"), _dev(out, torch.int64, "out"), n_pixels, C,
                                    _stream()), "dabnn_bitpack_i32")
    return out


def nhwc_to_nc1hwc2(a):
    """Packed int64 [N,H,W,Cw] -> [N,ceil(Cw/2),H,W,2] (C2 = 128 bits)."""
    N, H, W, Cw = a.shape
    out = torch.empty((N, (Cw + 1) // 2, H, W, 2), dtype=torch.int64, device=a.device)
    _check(load().dabnn_nhwc_to_nc1hwc2(_dev(a, torch.int64, "a"), _dev(out, torch.int64, "out"), N, H, W,
                                        Cw, _stream()), "dabnn_nhwc_to_nc1hwc2")
    return out


def nc1hwc2_to_nhwc(g, Cw):
    """Inverse of nhwc_to_nc1hwc2 for a tensor of Cw words per pixel."""
    N, C1, H, W, two = g.shape
    if two != 2 or C1 != (Cw + 1) // 2:
        raise ValueError("not an NC1HWC2 tensor of that channel count")
    out = torch.empty((N, H, W, Cw), dtype=torch.int64, device=g.device)
    _check(load().dabnn_nc1hwc2_to_nhwc(_dev(g, torch.int64, "g"), _dev(out, torch.int64, "out"), N, H, W,
                                        Cw, _stream()), "dabnn_nc1hwc2_to_nhwc")
    return out


def bn_sign_pack(y, scale, shift, r=None, x_out=None, want_x=True, out=None):
    """Fused BN + shortcut + sign + pack: y int32 [..., C], scale/shift float32 [C], r float32 like y
    or None -> (z float32 like y or None, bits int64 [..., ceil(C/64)])."""
    C = y.shape[-1]
    n_pixels = y.numel() // C if C else 0
    if x_out is None and want_x:
        x_out = torch.empty(y.shape, dtype=torch.float32, device=y.device)
    if out is None:
        out = torch.empty(tuple(y.shape[:-1]) + ((C + 63) // 64,), dtype=torch.int64, device=y.device)
    null = ctypes.c_void_p(0)
    _check(load().dabnn_bn_sign_pack(_dev(y, torch.int32, "y"), _dev(scale, torch.float32, "scale"),
                                     _dev(shift, torch.float32, "shift"),
                                     _dev(r, torch.float32, "r") if r is not None else null,
                                     _dev(x_out, torch.float32, "x_out") if x_out is not None else null,
                                     _dev(out, torch.int64, "out"), n_pixels, C, _stream()),
           "dabnn_bn_sign_pack")
    return x_out, out


def bconv2d_bn_residual(a, w, scale, shift, r, Cin, stride=1, pad=0, x_out=None, out=None):
    """Conv + BN + shortcut + sign + pack in one call: packed a, w -> (z float32 [N,Ho,Wo,Cout],
    bits int64 [N,Ho,Wo,ceil(Cout/64)]).  r may be None."""
    N, H, W, Cw = a.shape
    Cout, kh, kw, Cw2 = w.shape
    if Cw != Cw2 or Cw != (Cin + 63) // 64:
        raise ValueError("packed word counts do not match Cin")
    Ho, Wo = conv_out_dim(H, kh, stride, pad), conv_out_dim(W, kw, stride, pad)
    if Ho <= 0 or Wo <= 0:
        raise DabnnError(2, "dabnn_bconv2d_bn_residual")
    if x_out is None:
        x_out = torch.empty((N, Ho, Wo, Cout), dtype=torch.float32, device=a.device)
    if out is None:
        out = torch.empty((N, Ho, Wo, (Cout + 63) // 64), dtype=torch.int64, device=a.device)
    _check(load().dabnn_bconv2d_bn_residual(
        _dev(a, torch.int64, "a"), _dev(w, torch.int64, "w"), _dev(scale, torch.float32, "scale"),
        _dev(shift, torch.float32, "shift"),
        _dev(r, torch.float32, "r") if r is not None else ctypes.c_void_p(0),
        _dev(x_out, torch.float32, "x_out"), _dev(out, torch.int64, "out"), N, H, W, Cin, Cout, kh, kw,
        stride, pad, _stream()), "dabnn_bconv2d_bn_residual")
    return x_out, out


def expand_int8(bits, C, out=None):
    """Packed int64 [..., C/64] -> int8 [..., C], +1 for bit 0 and -1 for bit 1 (C % 64 == 0)."""
    if bits.shape[-1] * 64 != C:
        raise ValueError("packed word count does not match C")
    rows = bits.numel() // bits.shape[-1]
    if out is None:
        out = torch.empty(tuple(bits.shape[:-1]) + (C,), dtype=torch.int8, device=bits.device)
    _check(load().dabnn_expand_int8(_dev(bits, torch.int64, "bits"), _dev(out, torch.int8, "out"), rows, C,
                                    _stream()), "dabnn_expand_int8")
    return out


def bconv2d_int8(a8, w8, stride=1, pad=0, out=None):
    """Comparison route: a8 int8 [N,H,W,Cin], w8 int8 [Cout,kh,kw,Cin] (+-1) -> int32 [N,Ho,Wo,Cout]
    on the int8 matrix cores."""
    N, H, W, Cin = a8.shape
    Cout, kh, kw, Cin2 = w8.shape
    if Cin != Cin2:
        raise ValueError("channel counts differ")
    Ho, Wo = conv_out_dim(H, kh, stride, pad), conv_out_dim(W, kw, stride, pad)
    if Ho <= 0 or Wo <= 0:
        raise DabnnError(2, "dabnn_bconv2d_int8")
    if out is None:
        out = torch.empty((N, Ho, Wo, Cout), dtype=torch.int32, device=a8.device)
    _check(load().dabnn_bconv2d_int8(_dev(a8, torch.int8, "a8"), _dev(w8, torch.int8, "w8"),
                                     _dev(out, torch.int32, "out"), N, H, W, Cin, Cout, kh, kw, stride,
                                     pad, _stream()), "dabnn_bconv2d_int8")
    return out


MFMA_INT8, MFMA_FP4 = 0, 1


def mfma_weights_bytes(Cin, Cout, kh=3, kw=3, fmt=MFMA_INT8):
    """Bytes of the prepared filter buffer of dabnn_bconv2d_mfma; 0 for an unsupported layer."""
    return load().dabnn_mfma_weights_bytes(Cin, Cout, kh, kw, fmt)


def prepare_weights_mfma(w, Cin, out=None, fmt=MFMA_INT8):
    """Packed filters int64 [Cout, 3, 3, Cin/64] -> the uint8 buffer dabnn_bconv2d_mfma consumes
    (operands in kernel order, int8 or FP4, followed by one int32 constant per output channel)."""
    Cout, kh, kw, words = w.shape
    if words * 64 != Cin:
        raise ValueError("packed word count does not match Cin")
    n = mfma_weights_bytes(Cin, Cout, kh, kw, fmt)
    if n == 0:
        raise DabnnError(4, "dabnn_mfma_weights_bytes")
    if out is None:
        out = torch.empty((n,), dtype=torch.uint8, device=w.device)
    _check(load().dabnn_prepare_weights_mfma(_dev(w, torch.int64, "w"), _dev(out, torch.uint8, "out"),
                                             Cin, Cout, kh, kw, fmt, _stream()), "dabnn_prepare_weights_mfma")
    return out


def bconv2d_mfma(a, wq, Cin, Cout, stride=1, pad=1, out=None, fmt=MFMA_INT8):
    """a: packed int64 [N,H,W,Cin/64]; wq: prepare_weights_mfma of the layer's 3x3 filters in the
    same format -> int32 [N,Ho,Wo,Cout], the values of bconv2d, computed on the matrix cores."""
    N, H, W, words = a.shape
    if words * 64 != Cin:
        raise ValueError("packed word count does not match Cin")
    if wq.numel() != mfma_weights_bytes(Cin, Cout, 3, 3, fmt):
        raise ValueError("wq is not the prepared filter buffer of this layer shape and format")
    Ho, Wo = conv_out_dim(H, 3, stride, pad), conv_out_dim(W, 3, stride, pad)
    if Ho <= 0 or Wo <= 0:
        raise DabnnError(2, "dabnn_bconv2d_mfma")
    if out is None:
        out = torch.empty((N, Ho, Wo, Cout), dtype=torch.int32, device=a.device)
    _check(load().dabnn_bconv2d_mfma(_dev(a, torch.int64, "a"), _dev(wq, torch.uint8, "wq"),
                                     _dev(out, torch.int32, "out"), N, H, W, Cin, Cout, 3, 3, stride, pad,
                                     fmt, _stream()), "dabnn_bconv2d_mfma")
    return out


def bconv2d_bnsign_mfma(a, wq, thr, flip, Cin, Cout, stride=1, pad=1, out=None, fmt=MFMA_INT8):
    """bconv2d_bnsign on the matrix-core route: packed a, prepared filters wq -> int64
    [N,Ho,Wo,Cout/64], the next layer's packed activations."""
    N, H, W, words = a.shape
    if words * 64 != Cin:
        raise ValueError("packed word count does not match Cin")
    if wq.numel() != mfma_weights_bytes(Cin, Cout, 3, 3, fmt):
        raise ValueError("wq is not the prepared filter buffer of this layer shape and format")
    if thr.shape != (Cout,) or flip.shape != ((Cout + 63) // 64,):
        raise ValueError("thr / flip do not match Cout")
    Ho, Wo = conv_out_dim(H, 3, stride, pad), conv_out_dim(W, 3, stride, pad)
    if Ho <= 0 or Wo <= 0:
        raise DabnnError(2, "dabnn_bconv2d_bnsign_mfma")
    if out is None:
        out = torch.empty((N, Ho, Wo, Cout // 64), dtype=torch.int64, device=a.device)
    _check(load().dabnn_bconv2d_bnsign_mfma(_dev(a, torch.int64, "a"), _dev(wq, torch.uint8, "wq"),
                                            _dev(thr, torch.int32, "thr"), _dev(flip, torch.int64, "flip"),
                                            _dev(out, torch.int64, "out"), N, H, W, Cin, Cout, 3, 3, stride, pad,
                                            fmt, _stream()), "dabnn_bconv2d_bnsign_mfma")
    return out


def pick_algo(N, H, W, Cin, Cout, kh, kw, stride, pad):
    return load().dabnn_bconv2d_pick_algo(N, H, W, Cin, Cout, kh, kw, stride, pad)


def bn_thresholds(gamma, beta, mean, var, eps, K, device="cuda"):
    """Batch-norm parameters (host float32 arrays of length Cout) -> (thr int32 [Cout], flip
    int64 [ceil(Cout/64)]) on `device`, computed by the library's host helper."""
    import numpy as np
    arrs = [np.ascontiguousarray(v, dtype=np.float32) for v in (gamma, beta, mean, var)]
    Cout = arrs[0].shape[0]
    if any(v.shape != (Cout,) for v in arrs):
        raise ValueError("batch-norm parameters must all have shape (Cout,)")
    thr = np.empty(Cout, dtype=np.int32)
    flip = np.empty((Cout + 63) // 64, dtype=np.int64)
    _check(load().dabnn_bn_thresholds(*[ctypes.c_void_p(v.ctypes.data) for v in arrs], ctypes.c_float(eps),
                                      Cout, K, ctypes.c_void_p(thr.ctypes.data),
                                      ctypes.c_void_p(flip.ctypes.data)), "dabnn_bn_thresholds")
    return torch.from_numpy(thr).to(device), torch.from_numpy(flip).to(device)


def bconv2d_bnsign(a, w, thr, flip, Cin, stride=1, pad=0, out=None):
    """Fused conv + threshold + bit-pack: packed a, w -> int64 [N,Ho,Wo,ceil(Cout/64)] (the next
    layer's packed activations)."""
    N, H, W, Cw = a.shape
    Cout, kh, kw, Cw2 = w.shape
    if Cw != Cw2 or Cw != (Cin + 63) // 64:
        raise ValueError("packed word counts do not match Cin")
    if thr.shape != (Cout,) or flip.shape != ((Cout + 63) // 64,):
        raise ValueError("thr / flip do not match Cout")
    Ho, Wo = conv_out_dim(H, kh, stride, pad), conv_out_dim(W, kw, stride, pad)
    if Ho <= 0 or Wo <= 0:
        raise DabnnError(2, "dabnn_bconv2d_bnsign")
    if out is None:
        out = torch.empty((N, Ho, Wo, (Cout + 63) // 64), dtype=torch.int64, device=a.device)
    _check(load().dabnn_bconv2d_bnsign(_dev(a, torch.int64, "a"), _dev(w, torch.int64, "w"),
                                       _dev(thr, torch.int32, "thr"), _dev(flip, torch.int64, "flip"),
                                       _dev(out, torch.int64, "out"), N, H, W, Cin, Cout, kh, kw, stride,
                                       pad, _stream()), "dabnn_bconv2d_bnsign")
    return out
