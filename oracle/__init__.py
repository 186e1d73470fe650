"""CPU oracle for the daBNN hot path (arXiv 1908.05858) -- TEST INFRASTRUCTURE ONLY.

A thin ctypes loader around ``dabnn_oracle.c`` (plain C + OpenMP).  Only ``tests/``,
``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may import this
package.  It imports nothing from the GPU package and the GPU package imports nothing from here.

What each function computes, with the passage it follows, is stated in ``dabnn_oracle.c``:
``sign`` / ``bitpack`` / ``bitpack_i32`` follow Sec. 2.1.1; ``nhwc_to_nc1hwc2`` is the layout of
Sec. 2.1.2; ``bconv2d`` is the +-1 float cross-correlation that
Eq. 1 and Eq. 6-7 (Sec. 2.1.2) must equal (``bconv2d_zeropad``: the same with the zero padding
of the ONNX Convolution operator the paper builds on); ``bgemm_signed`` is Eq. 1 and the dot
product it stands for, ``im2col_signed`` the patch matrix that turns a convolution into that
BGEMM (Fig. 4's comparison route); ``bconv2d_bnsign`` is that convolution followed by
fp64 batch-norm and the sign (fused BN-binarization, Sec. 2.1.1); ``glue`` only generates inputs.

Every function here is pinned by ``tests/test_oracle_pins.py`` (closed forms, invariants, brute
force, torch's CPU conv2d, numpy.packbits); none is "parity unpinned".
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dabnn_oracle.c")
_LIB_PATH = os.path.join(_HERE, "libdabnn_oracle.so")
_lib = None

SIGN_BIT = 0  # -1 iff the IEEE sign bit is set (Sec. 2.1.1)
SIGN_GE0 = 1  # +1 iff x >= 0


def build(force=False):
    """Compile the oracle with gcc.  AVX2 baseline so one build runs on any host of this pool."""
    if not force and os.path.exists(_LIB_PATH) and os.path.getmtime(_LIB_PATH) >= os.path.getmtime(_SRC):
        return _LIB_PATH
    cmd = ["gcc", "-O3", "-march=x86-64-v3", "-fopenmp", "-fno-fast-math", "-ffp-contract=off", "-std=c11", "-Wall",
           "-Wextra", "-shared", "-fPIC", _SRC, "-o", _LIB_PATH, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB_PATH


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    lib = ctypes.CDLL(_LIB_PATH)
    i32, i64, vp = ctypes.c_int, ctypes.c_int64, ctypes.c_void_p
    lib.oracle_sign.argtypes = [vp, vp, i64, i32]
    lib.oracle_bitpack.argtypes = [vp, vp, i64, i32, i32]
    lib.oracle_conv_out_dim.argtypes = [i32] * 4
    lib.oracle_bconv2d.argtypes = [vp, vp, vp] + [i32] * 9
    lib.oracle_bconv2d_zeropad.argtypes = [vp, vp, vp] + [i32] * 9
    lib.oracle_bitpack_i32.argtypes = [vp, vp, i64, i32]
    lib.oracle_nhwc_to_nc1hwc2.argtypes = [vp, vp] + [i32] * 4
    lib.oracle_bn_sign_pack.argtypes = [vp] * 6 + [i64, i32]
    lib.oracle_bgemm.argtypes = [vp, vp, vp, i64, i32, i32, i32]
    lib.oracle_bconv2d_at.argtypes = [vp, vp, vp, i64, vp] + [i32] * 9
    lib.oracle_glue.argtypes = [vp] * 5 + [i32] * 9
    lib.oracle_bconv2d_bnsign.argtypes = [vp] * 6 + [ctypes.c_float, vp] + [i32] * 9
    for f in (lib.oracle_sign, lib.oracle_bitpack, lib.oracle_conv_out_dim, lib.oracle_bconv2d,
              lib.oracle_bconv2d_at, lib.oracle_glue, lib.oracle_bconv2d_bnsign,
              lib.oracle_bconv2d_zeropad, lib.oracle_bgemm, lib.oracle_bitpack_i32,
              lib.oracle_nhwc_to_nc1hwc2, lib.oracle_bn_sign_pack):
        f.restype = i32
    _lib = lib
    return lib


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle.{what}: bad argument (code {rc})")


def sign(x, sign_rule=SIGN_BIT):
    """+-1.0f tensor of the same shape as x (Sec. 2.1.1)."""
    x = _f32(x)
    s = np.empty_like(x)
    _check(_load().oracle_sign(x.ctypes.data, s.ctypes.data, x.size, sign_rule), "sign")
    return s


def bitpack(x, sign_rule=SIGN_BIT):
    """x: fp32 [..., C] -> uint64 [..., ceil(C/64)], LSB-first, tail bits 0 (Sec. 2.1.1)."""
    x = _f32(x)
    C = x.shape[-1]
    words = (C + 63) // 64
    n_pixels = x.size // C if C else 0
    out = np.empty(x.shape[:-1] + (words,), dtype=np.uint64)
    _check(_load().oracle_bitpack(x.ctypes.data, out.ctypes.data, n_pixels, C, sign_rule), "bitpack")
    return out


def bitpack_i32(x):
    """x: int32 [..., C] -> uint64 [..., ceil(C/64)], bit = 1 iff x < 0 (Sec. 2.1.1)."""
    x = np.ascontiguousarray(x, dtype=np.int32)
    C = x.shape[-1]
    out = np.empty(x.shape[:-1] + ((C + 63) // 64,), dtype=np.uint64)
    _check(_load().oracle_bitpack_i32(x.ctypes.data, out.ctypes.data, x.size // C, C), "bitpack_i32")
    return out


def nhwc_to_nc1hwc2(a):
    """Packed uint64 [N,H,W,Cw] -> [N,ceil(Cw/2),H,W,2] (NC1HWC2 with C2 = 128 bits, Sec. 2.1.2)."""
    a = np.ascontiguousarray(a, dtype=np.uint64)
    N, H, W, Cw = a.shape
    out = np.empty((N, (Cw + 1) // 2, H, W, 2), dtype=np.uint64)
    _check(_load().oracle_nhwc_to_nc1hwc2(a.ctypes.data, out.ctypes.data, N, H, W, Cw), "nhwc_to_nc1hwc2")
    return out


def bn_sign_pack(y, scale, shift, r=None, want_x=True):
    """Fused BN + (shortcut) + sign + pack in fp32, every operation rounded separately:
    z = (scale*y + shift) + r.  y: int32 [..., C] -> (z float32 [..., C] or None, bits uint64
    [..., ceil(C/64)])  (Sec. 2.1.1 fused BN-binarization; Sec. 2.3 Bi-Real shortcut)."""
    y = np.ascontiguousarray(y, dtype=np.int32)
    scale, shift = _f32(scale), _f32(shift)
    C = y.shape[-1]
    if scale.shape != (C,) or shift.shape != (C,):
        raise ValueError("scale/shift must have shape (C,)")
    if r is not None:
        r = _f32(r)
        if r.shape != y.shape:
            raise ValueError("shortcut shape differs")
    x = np.empty(y.shape, np.float32) if want_x else None
    bits = np.empty(y.shape[:-1] + ((C + 63) // 64,), dtype=np.uint64)
    _check(_load().oracle_bn_sign_pack(y.ctypes.data, scale.ctypes.data, shift.ctypes.data,
                                       r.ctypes.data if r is not None else None,
                                       x.ctypes.data if x is not None else None, bits.ctypes.data,
                                       y.size // C, C), "bn_sign_pack")
    return x, bits


def conv_out_dim(size, k, stride, pad):
    return _load().oracle_conv_out_dim(size, k, stride, pad)


def bconv2d_signed(A, Wt, stride=1, pad=0):
    """+-1 float cross-correlation, out-of-image taps = +1.  A: [N,H,W,Cin], Wt: [Cout,kh,kw,Cin]
    (values +-1.0f) -> int32 [N,Ho,Wo,Cout]  (Sec. 2.1.2, Eq. 6-7)."""
    A, Wt = _f32(A), _f32(Wt)
    N, H, W, Cin = A.shape
    Cout, kh, kw, Cin2 = Wt.shape
    if Cin != Cin2:
        raise ValueError("channel mismatch")
    Ho, Wo = conv_out_dim(H, kh, stride, pad), conv_out_dim(W, kw, stride, pad)
    if Ho <= 0 or Wo <= 0:
        raise ValueError("empty output")
    Y = np.empty((N, Ho, Wo, Cout), dtype=np.int32)
    _check(_load().oracle_bconv2d(A.ctypes.data, Wt.ctypes.data, Y.ctypes.data, N, H, W, Cin, Cout,
                                  kh, kw, stride, pad), "bconv2d")
    return Y


def bconv2d_zeropad_signed(A, Wt, stride=1, pad=0):
    """+-1 float cross-correlation with ZERO padding (ONNX Convolution; Table 1 caption, Sec. 3):
    same shapes as bconv2d_signed, out-of-image taps contribute nothing."""
    A, Wt = _f32(A), _f32(Wt)
    N, H, W, Cin = A.shape
    Cout, kh, kw, Cin2 = Wt.shape
    if Cin != Cin2:
        raise ValueError("channel mismatch")
    Ho, Wo = conv_out_dim(H, kh, stride, pad), conv_out_dim(W, kw, stride, pad)
    if Ho <= 0 or Wo <= 0:
        raise ValueError("empty output")
    Y = np.empty((N, Ho, Wo, Cout), dtype=np.int32)
    _check(_load().oracle_bconv2d_zeropad(A.ctypes.data, Wt.ctypes.data, Y.ctypes.data, N, H, W, Cin,
                                          Cout, kh, kw, stride, pad), "bconv2d_zeropad")
    return Y


def bconv2d_zeropad(x, w, stride=1, pad=0, sign_rule=SIGN_BIT):
    """Sign of both raw fp32 tensors, then the zero-padded convolution."""
    return bconv2d_zeropad_signed(sign(x, sign_rule), sign(w, sign_rule), stride, pad)


def bconv2d(x, w, stride=1, pad=0, sign_rule=SIGN_BIT):
    """The whole operator on raw fp32 tensors: binarize both, then convolve."""
    return bconv2d_signed(sign(x, sign_rule), sign(w, sign_rule), stride, pad)


def bconv2d_at(A, Wt, idx, stride=1, pad=0):
    """Selected outputs of bconv2d_signed: idx int32 [S,4] rows (n,ho,wo,co) -> int32 [S]."""
    A, Wt = _f32(A), _f32(Wt)
    idx = np.ascontiguousarray(idx, dtype=np.int32).reshape(-1, 4)
    N, H, W, Cin = A.shape
    Cout, kh, kw, Cin2 = Wt.shape
    if Cin != Cin2:
        raise ValueError("channel mismatch")
    out = np.empty(idx.shape[0], dtype=np.int32)
    _check(_load().oracle_bconv2d_at(A.ctypes.data, Wt.ctypes.data, idx.ctypes.data, idx.shape[0],
                                     out.ctypes.data, N, H, W, Cin, Cout, kh, kw, stride, pad),
           "bconv2d_at")
    return out


def bconv2d_bnsign(x, w, gamma, beta, mean, var, eps, stride=1, pad=0, sign_rule=SIGN_BIT):
    """sign(BN(bconv2d(x, w))) packed into words: uint64 [N,Ho,Wo,ceil(Cout/64)] (Sec. 2.1.1,
    fused BN-binarization; BN in fp64, bit = 1 iff z < 0)."""
    A, Wt = sign(x, sign_rule), sign(w, sign_rule)
    gamma, beta, mean, var = _f32(gamma), _f32(beta), _f32(mean), _f32(var)
    N, H, W, Cin = A.shape
    Cout, kh, kw, Cin2 = Wt.shape
    if Cin != Cin2 or any(v.shape != (Cout,) for v in (gamma, beta, mean, var)):
        raise ValueError("shape mismatch")
    Ho, Wo = conv_out_dim(H, kh, stride, pad), conv_out_dim(W, kw, stride, pad)
    if Ho <= 0 or Wo <= 0:
        raise ValueError("empty output")
    out = np.empty((N, Ho, Wo, (Cout + 63) // 64), dtype=np.uint64)
    _check(_load().oracle_bconv2d_bnsign(A.ctypes.data, Wt.ctypes.data, gamma.ctypes.data,
                                         beta.ctypes.data, mean.ctypes.data, var.ctypes.data,
                                         ctypes.c_float(eps), out.ctypes.data, N, H, W, Cin, Cout, kh,
                                         kw, stride, pad), "bconv2d_bnsign")
    return out


BGEMM_SIGNED = 0   # sum_k A_ik * B_jk = 2*C_ij - K
BGEMM_MATCHES = 1  # C_ij of Eq. 1: bitcount(xnor)


def bgemm_signed(A, B, mode=BGEMM_SIGNED):
    """BGEMM (Sec. 2.1.2, Eq. 1) on +-1.0f operands A [M,K], B [N,K] -> int32 [M,N]."""
    A, B = _f32(A), _f32(B)
    M, K = A.shape
    N, K2 = B.shape
    if K != K2:
        raise ValueError("inner dimensions differ")
    C = np.empty((M, N), dtype=np.int32)
    _check(_load().oracle_bgemm(A.ctypes.data, B.ctypes.data, C.ctypes.data, M, N, K, mode), "bgemm")
    return C


def im2col_signed(A, kh, kw, stride=1, pad=0):
    """Patch matrix of a +-1.0f NHWC tensor: [N*Ho*Wo, kh*kw, Cin], taps in (i, j) order,
    out-of-image taps +1.0 -- the matrix whose BGEMM with the [Cout, kh*kw*Cin] filter matrix is
    the convolution (the BGEMM route the paper compares its direct convolution with, Fig. 4)."""
    A = _f32(A)
    N, H, W, Cin = A.shape
    Ho, Wo = conv_out_dim(H, kh, stride, pad), conv_out_dim(W, kw, stride, pad)
    if Ho <= 0 or Wo <= 0:
        raise ValueError("empty output")
    padded = np.ones((N, H + 2 * pad, W + 2 * pad, Cin), np.float32)
    padded[:, pad:pad + H, pad:pad + W, :] = A
    cols = np.empty((N, Ho, Wo, kh * kw, Cin), np.float32)
    for i in range(kh):
        for j in range(kw):
            cols[:, :, :, i * kw + j, :] = padded[:, i:i + (Ho - 1) * stride + 1:stride,
                                                  j:j + (Wo - 1) * stride + 1:stride, :]
    return cols.reshape(N * Ho * Wo, kh * kw, Cin)


def glue(x, y, gamma, beta, K, stride):
    """Input generator for the next layer of the full-network workload (not the method)."""
    x, gamma, beta = _f32(x), _f32(gamma), _f32(beta)
    y = np.ascontiguousarray(y, dtype=np.int32)
    N, H, W, Cin = x.shape
    _, Ho, Wo, Cout = y.shape
    out = np.empty(y.shape, dtype=np.float32)
    _check(_load().oracle_glue(x.ctypes.data, y.ctypes.data, gamma.ctypes.data, beta.ctypes.data,
                               out.ctypes.data, N, H, W, Cin, Ho, Wo, Cout, K, stride), "glue")
    return out
