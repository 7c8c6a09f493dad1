"""ctypes front end of the NestQuant CPU oracle (oracle/nq_oracle.c).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's
cpu_baseline leg may import this; the product path never does.  It imports
nothing from the HIP package.  Array marshalling only -- every arithmetic
step lives in the C file, each next to the passage of the paper it follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nq_oracle.c")
_LIB = os.path.join(_HERE, "libnq_oracle.so")

ROUNDING = {"bitshift": 0, "rtn": 1, "up": 2, "down": 3}
LOW_UNSIGNED_L = 0      # true bit split, l bits, [0, 2^l-1]
LOW_SIGNED_L1 = 1       # extra-1-bit compensation, signed (l+1) bits
LOW_CLIP_SIGNED_L = 2   # Eq. 9 as printed (lossy)
KIND_CARRIER = 0        # dense-tile stream kind of the higher-bit page
KIND_BITSTRING = 1      # dense-tile stream kind of the lower-bit page


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-shared",
               "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oq_paper_words_per_row.restype = ctypes.c_int64
        _lib.oq_paper_words_per_row.argtypes = [ctypes.c_int64, ctypes.c_int]
        _lib.oq_dense_bytes.restype = ctypes.c_int64
        _lib.oq_dense_bytes.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int]
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None else None


def _i64(v):
    return ctypes.c_int64(int(v))


def _chk(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what}: error {rc} ({'bad argument' if rc == 1 else 'value out of range'})")


def threads() -> int:
    """Number of OpenMP threads the GEMM/conv loops use."""
    n = os.environ.get("OMP_NUM_THREADS")
    return int(n) if n else (os.cpu_count() or 1)


def quantize(w: np.ndarray, n_bits: int = 8):
    """Eq. 1, per output channel (rows of w [N,K])."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    N, K = w.shape
    wi = np.empty((N, K), np.int8)
    s = np.empty((N,), np.float32)
    _chk(lib().oq_quantize_rtn(_p(w), _i64(N), _i64(K), int(n_bits), _p(wi), _p(s)), "quantize")
    return wi, s


def decompose(w_int: np.ndarray, n_bits: int, l_bits: int, rounding: str = "bitshift"):
    """Eq. 5 + Alg. 1 step 2: returns (w_high int8, residual int16), same shape."""
    w_int = np.ascontiguousarray(w_int, dtype=np.int8)
    hi = np.empty(w_int.shape, np.int8)
    res = np.empty(w_int.shape, np.int16)
    _chk(lib().oq_decompose(_p(w_int), _i64(w_int.size), int(n_bits), int(l_bits),
                            ROUNDING[rounding], _p(hi), _p(res)), "decompose")
    return hi, res


def low_encode(residual: np.ndarray, l_bits: int, fmt: int = LOW_UNSIGNED_L):
    residual = np.ascontiguousarray(residual, dtype=np.int16)
    lo = np.empty(residual.shape, np.int8)
    _chk(lib().oq_low_encode(_p(residual), _i64(residual.size), int(l_bits), int(fmt), _p(lo)),
         "low_encode")
    return lo


def compose(w_high: np.ndarray, w_low: np.ndarray, l_bits: int):
    """Eq. 4: w_high * 2^l + w_low, int16."""
    w_high = np.ascontiguousarray(w_high, dtype=np.int8)
    w_low = np.ascontiguousarray(w_low, dtype=np.int8)
    out = np.empty(w_high.shape, np.int16)
    _chk(lib().oq_compose(_p(w_high), _p(w_low), _i64(w_high.size), int(l_bits), _p(out)), "compose")
    return out


def paper_words_per_row(K: int, k: int) -> int:
    return int(lib().oq_paper_words_per_row(int(K), int(k)))


def pack_paper(v: np.ndarray, k: int) -> np.ndarray:
    v = np.ascontiguousarray(v, dtype=np.int8)
    N, K = v.shape
    out = np.empty((N, paper_words_per_row(K, k)), np.uint64)
    _chk(lib().oq_pack_paper(_p(v), _i64(N), _i64(K), int(k), _p(out)), "pack_paper")
    return out


def unpack_paper(words: np.ndarray, N: int, K: int, k: int, signed: bool) -> np.ndarray:
    words = np.ascontiguousarray(words, dtype=np.uint64)
    v = np.empty((N, K), np.int8)
    _chk(lib().oq_unpack_paper(_p(words), _i64(N), _i64(K), int(k), int(bool(signed)), _p(v)),
         "unpack_paper")
    return v


def dense_bytes(N: int, K: int, k: int) -> int:
    return int(lib().oq_dense_bytes(int(N), int(K), int(k)))


def pack_dense(v: np.ndarray, k: int, kind: int) -> np.ndarray:
    v = np.ascontiguousarray(v, dtype=np.int8)
    N, K = v.shape
    out = np.empty((dense_bytes(N, K, k),), np.uint8)
    _chk(lib().oq_pack_dense(_p(v), _i64(N), _i64(K), int(k), int(kind), _p(out)), "pack_dense")
    return out


def unpack_dense(buf: np.ndarray, N: int, K: int, k: int, kind: int, signed: bool) -> np.ndarray:
    buf = np.ascontiguousarray(buf, dtype=np.uint8)
    assert buf.size == dense_bytes(N, K, k), "dense buffer size"
    v = np.empty((N, K), np.int8)
    _chk(lib().oq_unpack_dense(_p(buf), _i64(N), _i64(K), int(k), int(kind), int(bool(signed)), _p(v)),
         "unpack_dense")
    return v


def gemm_acc(x: np.ndarray, w: np.ndarray) -> np.ndarray:
    """acc[m,n] = sum_k x[m,k] * w[n,k] in int32; w is int16 (or int8)."""
    x = np.ascontiguousarray(x, dtype=np.int8)
    w = np.ascontiguousarray(w, dtype=np.int16)
    M, K = x.shape
    N, K2 = w.shape
    assert K == K2
    acc = np.empty((M, N), np.int32)
    _chk(lib().oq_gemm_i32(_p(x), _i64(M), _p(w), _i64(N), _i64(K), _p(acc)), "gemm")
    return acc


def conv_out_hw(H, W, KH, KW, stride, pad):
    return (H + 2 * pad - KH) // stride + 1, (W + 2 * pad - KW) // stride + 1


def conv_acc(x: np.ndarray, w: np.ndarray, stride: int, pad: int) -> np.ndarray:
    """Direct NHWC convolution; x [B,H,W,Cin] int8, w [Cout,KH,KW,Cin]; int32 [B,Ho,Wo,Cout]."""
    x = np.ascontiguousarray(x, dtype=np.int8)
    w = np.ascontiguousarray(w, dtype=np.int16)
    B, H, W, Cin = x.shape
    Cout, KH, KW, Cin2 = w.shape
    assert Cin == Cin2
    Ho, Wo = conv_out_hw(H, W, KH, KW, stride, pad)
    acc = np.empty((B, Ho, Wo, Cout), np.int32)
    _chk(lib().oq_conv_i32(_p(x), _i64(B), _i64(H), _i64(W), _i64(Cin), _p(w), _i64(Cout),
                           int(KH), int(KW), int(stride), int(pad), _p(acc)), "conv")
    return acc


def conv_grouped_acc(x: np.ndarray, w: np.ndarray, groups: int, stride: int, pad: int) -> np.ndarray:
    """Grouped NHWC convolution (depthwise for groups == Cin); x [B,H,W,Cin] int8, w [Cout,KH,KW,Cin/groups];
    int32 [B,Ho,Wo,Cout]."""
    x = np.ascontiguousarray(x, dtype=np.int8)
    w = np.ascontiguousarray(w, dtype=np.int16)
    B, H, W, Cin = x.shape
    Cout, KH, KW, cig = w.shape
    assert Cin == cig * groups
    Ho, Wo = conv_out_hw(H, W, KH, KW, stride, pad)
    acc = np.empty((B, Ho, Wo, Cout), np.int32)
    _chk(lib().oq_conv_grouped_i32(_p(x), _i64(B), _i64(H), _i64(W), _i64(Cin), _p(w), _i64(Cout), _i64(groups),
                                   int(KH), int(KW), int(stride), int(pad), _p(acc)), "grouped conv")
    return acc


def epilogue(acc: np.ndarray, s_a: float, s_w: np.ndarray, part_l_bits: int = 0, bias=None,
             residual=None, s_r: float = 0.0, relu: bool = False, out_int8: bool = False,
             inv_s_out: float = 1.0) -> np.ndarray:
    """Fixed-order fp32 dequantisation (Eq. 2 / Eq. 8) over the last axis = output channel."""
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    N = acc.shape[-1]
    M = acc.size // N if N else 0
    s_w = np.ascontiguousarray(s_w, dtype=np.float32)
    assert s_w.shape == (N,)
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
    if residual is not None:
        residual = np.ascontiguousarray(residual, dtype=np.int8)
        assert residual.size == acc.size
    yf = None if out_int8 else np.empty(acc.shape, np.float32)
    yi = np.empty(acc.shape, np.int8) if out_int8 else None
    _chk(lib().oq_epilogue(_p(acc), _i64(M), _i64(N), ctypes.c_float(s_a), _p(s_w), int(part_l_bits),
                           _p(bias), _p(residual), ctypes.c_float(s_r), int(bool(relu)),
                           int(bool(out_int8)), ctypes.c_float(inv_s_out), _p(yf), _p(yi)), "epilogue")
    return yi if out_int8 else yf


def maxpool(x: np.ndarray, ksize: int, stride: int, pad: int) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.int8)
    B, H, W, C = x.shape
    Ho, Wo = conv_out_hw(H, W, ksize, ksize, stride, pad)
    y = np.empty((B, Ho, Wo, C), np.int8)
    _chk(lib().oq_maxpool_i8(_p(x), _i64(B), _i64(H), _i64(W), _i64(C), int(ksize), int(stride),
                             int(pad), _p(y)), "maxpool")
    return y


def avgpool(x: np.ndarray, s_in: float, inv_s_out: float) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.int8)
    B, H, W, C = x.shape
    y = np.empty((B, C), np.int8)
    _chk(lib().oq_avgpool_i8(_p(x), _i64(B), _i64(H * W), _i64(C), ctypes.c_float(s_in),
                             ctypes.c_float(inv_s_out), _p(y)), "avgpool")
    return y


# ---------------------------------------------------------------------------
# The path end to end, from packed pages, in the paper's order: load the pages
# (Sec. 3.3.4 "Storing & Scheduling"), recompose (Eq. 4) or keep the higher-bit
# page alone, integer GEMM / convolution, dequantise (Eq. 2 / Eq. 8).
# ---------------------------------------------------------------------------
def decompose_pack(w_int: np.ndarray, n_bits: int, l_bits: int, layout: str = "dense"):
    """BitShift split then pack; returns (packed_high, packed_low) byte arrays."""
    h_bits = n_bits - l_bits
    hi, res = decompose(w_int, n_bits, l_bits, "bitshift")
    lo = low_encode(res, l_bits, LOW_UNSIGNED_L)
    if layout == "dense":
        return pack_dense(hi, h_bits, KIND_CARRIER), pack_dense(lo, l_bits, KIND_BITSTRING)
    return pack_paper(hi, h_bits).view(np.uint8).ravel(), pack_paper(lo, l_bits).view(np.uint8).ravel()


def weights_from_pages(packed_high, packed_low, N, K, n_bits, l_bits, layout="dense"):
    """Unpack; full-bit weights if the lower-bit page is given, else the higher-bit part."""
    h_bits = n_bits - l_bits
    if layout == "dense":
        hi = unpack_dense(packed_high, N, K, h_bits, KIND_CARRIER, True)
        lo = None if packed_low is None else unpack_dense(packed_low, N, K, l_bits, KIND_BITSTRING, False)
    else:
        hi = unpack_paper(np.frombuffer(packed_high, np.uint64).reshape(N, -1), N, K, h_bits, True)
        lo = None if packed_low is None else unpack_paper(
            np.frombuffer(packed_low, np.uint64).reshape(N, -1), N, K, l_bits, False)
    if lo is None:
        return hi.astype(np.int16)
    return compose(hi, lo, l_bits)
