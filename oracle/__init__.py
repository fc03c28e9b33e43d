"""CPU oracle for the QUOTA hot path -- TEST INFRASTRUCTURE ONLY.

Thin numpy/ctypes front end over ``quota_oracle.c`` (plain C, written from the
paper's Method section) plus the layer composite in ``layer.py``.  Nothing in
the product package may import this module; only ``tests/``, the smoke check
and the benchmark's CPU-baseline leg do.  The oracle shares no code with the
HIP library.

fp16 tensors are ``np.float16`` arrays, int4 codes are unpacked ``np.int8``
arrays in [-8, 7].
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "quota_oracle.c")
_LIB = os.path.join(_HERE, "libquota_oracle.so")

GROUP_W = 128   # weight group along the reduction dim (workload definition)
GROUP_KV = 64   # KV group along head_dim (workload definition)


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no contraction: every fp32 step rounds)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
               "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dt):
    a = np.ascontiguousarray(a, dtype=dt)
    return a


def f16_to_f32(h):
    h = _c(h, np.float16)
    out = np.empty(h.shape, np.float32)
    lib().orc_f16_to_f32(_p(h), ctypes.c_long(h.size), _p(out))
    return out


def f64_to_f16(x):
    x = _c(x, np.float64)
    out = np.empty(x.shape, np.float16)
    lib().orc_f64_to_f16(_p(x), ctypes.c_long(x.size), _p(out))
    return out


def quantize_weights(w, g: int = GROUP_W):
    """fp32 [N, K] -> (int8 codes [N, K], fp16 scales [N, ceil(K/g)])."""
    w = _c(w, np.float32)
    N, K = w.shape
    G = (K + g - 1) // g
    codes = np.empty((N, K), np.int8)
    scales = np.empty((N, G), np.float16)
    lib().orc_quantize_weights(_p(w), N, K, g, _p(codes), _p(scales))
    return codes, scales


def rmsnorm(x, gamma, eps: float):
    x = _c(x, np.float16)
    M, d = x.shape
    gamma = _c(gamma, np.float32)
    h = np.empty((M, d), np.float16)
    lib().orc_rmsnorm(_p(x), M, d, _p(gamma), ctypes.c_float(eps), _p(h))
    return h


def quantize_act(x):
    """fp16 [M, d] -> (codes int8 [M, d], scale f32 [M], sumsq f32 [M], ressq f32 [M])."""
    x = _c(x, np.float16)
    M, d = x.shape
    q = np.empty((M, d), np.int8)
    s = np.empty(M, np.float32)
    ss = np.empty(M, np.float32)
    rs = np.empty(M, np.float32)
    lib().orc_quantize_act(_p(x), M, d, _p(q), _p(s), _p(ss), _p(rs))
    return q, s, ss, rs


def w4a4_gemm(qa, sa, qw, sw, residual=None, g: int = GROUP_W, want_acc: bool = False):
    """codes [M,K] x codes [N,K]^T with scales -> fp16 [M,N] (and int32 acc)."""
    qa = _c(qa, np.int8)
    qw = _c(qw, np.int8)
    sa = _c(sa, np.float32)
    sw = _c(sw, np.float16)
    M, K = qa.shape
    N = qw.shape[0]
    assert qw.shape[1] == K and sw.shape == (N, (K + g - 1) // g)
    if residual is not None:
        residual = _c(residual, np.float16)
        assert residual.shape == (M, N)
    y = np.empty((M, N), np.float16)
    acc = np.empty((M, N), np.int32) if want_acc else None
    lib().orc_w4a4_gemm(_p(qa), _p(sa), M, K, _p(qw), _p(sw), N, g, _p(residual), _p(y), _p(acc))
    return (y, acc) if want_acc else y


def rope(x, H: int, dh: int, pos, cos, sin):
    """x fp16 [M, H*dh]; pos int32 [M]; cos/sin f32 [P, dh/2]."""
    x = _c(x, np.float16)
    M = x.shape[0]
    pos = _c(pos, np.int32)
    cos = _c(cos, np.float32)
    sin = _c(sin, np.float32)
    assert pos.max(initial=0) < cos.shape[0] and cos.shape[1] == dh // 2
    out = np.empty_like(x)
    lib().orc_rope(_p(x), M, H, dh, ctypes.c_long(H * dh), _p(pos), _p(cos), _p(sin),
                   _p(out), ctypes.c_long(H * dh))
    return out


def kv_quant(x, g: int = GROUP_KV):
    """fp16 [M, H*dh] -> (codes int8 [M,Hdh], scales f16 [M,Hdh/g], xhat f16 [M,Hdh])."""
    x = _c(x, np.float16)
    M, Hdh = x.shape
    assert Hdh % g == 0
    codes = np.empty((M, Hdh), np.int8)
    scales = np.empty((M, Hdh // g), np.float16)
    xhat = np.empty((M, Hdh), np.float16)
    lib().orc_kv_quant(_p(x), M, Hdh, ctypes.c_long(Hdh), g, _p(codes), _p(scales), _p(xhat))
    return codes, scales, xhat


def attention(q, khat, vhat, B: int, N: int, H: int, dh: int, vis_begin: int, Nv: int,
              want_P: bool = False, Hkv: int = None):
    """q fp16 [B*N, H*dh], khat/vhat fp16 [B*N, Hkv*dh] (Hkv = H unless given: grouped-query
    attention, query head h reads K/V head h // (H // Hkv)) ->
    (o fp16, cm_inter f32 [B,Nv], cm_intra f32 [B,Nv]); the cues average over the H query heads."""
    Hkv = H if Hkv is None else Hkv
    q = _c(q, np.float16)
    khat = _c(khat, np.float16)
    vhat = _c(vhat, np.float16)
    assert q.shape == (B * N, H * dh) and khat.shape == (B * N, Hkv * dh) == vhat.shape and H % Hkv == 0
    o = np.empty_like(q)
    ci = np.zeros((B, Nv), np.float32)
    cv = np.zeros((B, Nv), np.float32)
    P = np.empty((B, H, N, N), np.float64) if want_P else None
    lib().orc_attention(_p(q), _p(khat), _p(vhat), B, N, H, Hkv, dh, vis_begin, Nv,
                        _p(o), _p(ci), _p(cv), _p(P))
    return (o, ci, cv, P) if want_P else (o, ci, cv)


DEFAULT_WEIGHTS = dict(w_m=0.25, w_c=0.45, w_s=0.10, w_r=0.20)  # Table 5, default row


def score(sumsq, ressq, cm_inter, cm_intra, w_m=0.25, w_c=0.45, w_s=0.10, w_r=0.20,
          p_lo: int = 10, p_hi: int = 90, want_normed: bool = False):
    sumsq = _c(sumsq, np.float32)
    B, Nv = sumsq.shape
    ressq = _c(ressq, np.float32)
    cm_inter = _c(cm_inter, np.float32)
    cm_intra = _c(cm_intra, np.float32)
    out = np.zeros((B, Nv), np.float32)
    normed = np.zeros((4, B, Nv), np.float32) if want_normed else None
    cf = ctypes.c_float
    lib().orc_score(_p(sumsq), _p(ressq), _p(cm_inter), _p(cm_intra), B, Nv,
                    cf(w_m), cf(w_c), cf(w_s), cf(w_r), p_lo, p_hi, _p(out), _p(normed))
    return (out, normed) if want_normed else out


def topk(score_, K: int):
    score_ = _c(score_, np.float32)
    B, Nv = score_.shape
    k = max(0, min(K, Nv))
    idx = np.empty((B, k), np.int32)
    if k > 0:
        lib().orc_topk(_p(score_), B, Nv, K, _p(idx))
    return idx


def silu_mul(gu, F: int):
    gu = _c(gu, np.float16)
    M = gu.shape[0]
    assert gu.shape[1] == 2 * F
    z = np.empty((M, F), np.float16)
    lib().orc_silu_mul(_p(gu), M, F, _p(z))
    return z


def budget(r: float, V0: int) -> int:
    """K = ceil(r * V0) (Eq. 5), on exact rationals so 0.3*576 does not wobble."""
    from fractions import Fraction
    import math
    return int(math.ceil(Fraction(str(r)) * V0))


from .layer import (prefill_layer, decode_layer, decode_attention, dequant_kv, cache_from_prefill,  # noqa: E402,F401
                    LayerWeights)
from . import recipe  # noqa: E402,F401
