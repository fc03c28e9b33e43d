"""ctypes binding of libquota's C ABI (argument marshalling only).

Every function has the name and argument order of its C counterpart in
``include/quota.h``; tensors are torch CUDA tensors whose ``data_ptr()`` is
passed through, the stream is torch's current stream.  There is no fallback:
if the HIP library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libquota.so")

OK = 0
KEEP_ALL = -1          # K_l of a layer outside the candidate set (QUOTA_KEEP_ALL)
ERR_NULL, ERR_INVALID_ARG, ERR_SHAPE, ERR_CAPACITY, ERR_HIP = -1, -2, -3, -4, -5


class QuotaError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {strerror(code)} ({code})")
        self.code = code


class Weights(C.Structure):
    _fields_ = [("N", C.c_int), ("K", C.c_int), ("packed", C.c_void_p), ("scales", C.c_void_p)]


class KVCache(C.Structure):
    _fields_ = [("B", C.c_int), ("capacity", C.c_int), ("H", C.c_int), ("dh", C.c_int),
                ("len", C.c_int), ("k_codes", C.c_void_p), ("k_scales", C.c_void_p),
                ("v_codes", C.c_void_p), ("v_scales", C.c_void_p), ("step_dev", C.c_void_p), ("max_steps", C.c_int)]


class ScoreParams(C.Structure):
    _fields_ = [("w_m", C.c_float), ("w_c", C.c_float), ("w_s", C.c_float), ("w_r", C.c_float),
                ("pct_lo", C.c_int), ("pct_hi", C.c_int)]


class Layer(C.Structure):
    _fields_ = [("H", C.c_int), ("dh", C.c_int), ("F", C.c_int), ("eps", C.c_float),
                ("gamma1", C.c_void_p), ("gamma2", C.c_void_p),
                ("qkv", Weights), ("o", Weights), ("gu", Weights), ("down", Weights),
                ("cosT", C.c_void_p), ("sinT", C.c_void_p), ("n_pos", C.c_int), ("Hkv", C.c_int)]


class FpLayer(C.Structure):
    _fields_ = [("H", C.c_int), ("dh", C.c_int), ("F", C.c_int), ("Hkv", C.c_int), ("eps", C.c_float),
                ("gamma1", C.c_void_p), ("gamma2", C.c_void_p), ("wqkv", C.c_void_p), ("wo", C.c_void_p),
                ("wgu", C.c_void_p), ("wdown", C.c_void_p), ("cosT", C.c_void_p), ("sinT", C.c_void_p),
                ("n_pos", C.c_int)]


class State(C.Structure):
    _fields_ = [("B", C.c_int), ("N", C.c_int), ("vis_begin", C.c_int), ("Nv", C.c_int),
                ("x", C.c_void_p), ("pos", C.c_void_p), ("x_out", C.c_void_p), ("pos_out", C.c_void_p)]


class Taps(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ["qkv", "q_rot", "o", "sumsq", "ressq", "cm_inter", "cm_intra", "score", "keep_idx",
                 "rows", "x1", "gu", "z", "inject_o", "inject_cm_inter", "inject_cm_intra", "inject_z"]]


class KernelStat(C.Structure):
    _fields_ = [("launches", C.c_long), ("total_ms", C.c_double), ("ops", C.c_double), ("bytes", C.c_double)]


KERNEL_COUNT = 21

_lib = None


def lib() -> C.CDLL:
    """Loads libquota.so (built in-tree by ``build.py``); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2604_17320_amd.build` "
                               "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        L.quota_strerror.restype = C.c_char_p
        L.quota_kernel_name.restype = C.c_char_p
        for name in ["quota_weights_packed_bytes", "quota_weights_scale_bytes",
                     "quota_attention_workspace_bytes", "quota_prefill_workspace_bytes",
                     "quota_decode_workspace_bytes", "quota_fp_block_workspace_bytes",
                     "quota_profile_block_workspace_bytes"]:
            getattr(L, name).restype = C.c_size_t
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().quota_strerror(int(code)).decode()


def _ptr(t, dtype=None):
    if t is None:
        return C.c_void_p(0)
    assert t.is_cuda and t.is_contiguous(), "device, contiguous tensors only"
    if dtype is not None:
        assert t.dtype == dtype, f"expected {dtype}, got {t.dtype}"
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc, what):
    if rc != OK:
        raise QuotaError(rc, what)


def quota_version() -> int:
    return lib().quota_version()


def quota_weights_packed_bytes(N, K):
    return lib().quota_weights_packed_bytes(int(N), int(K))


def quota_weights_scale_bytes(N, K):
    return lib().quota_weights_scale_bytes(int(N), int(K))


def quota_quantize_weights(w, codes, scales):
    N, K = w.shape
    _check(lib().quota_quantize_weights(_ptr(w, torch.float32), N, K, _ptr(codes, torch.int8),
                                        _ptr(scales, torch.float16), _stream()), "quota_quantize_weights")


def quota_pack_weights(codes, scales, W: Weights):
    _check(lib().quota_pack_weights(_ptr(codes, torch.int8), _ptr(scales, torch.float16),
                                    C.byref(W), _stream()), "quota_pack_weights")


def quota_quantize_act(x, M, d, ldx, q_packed, scale, sumsq=None, ressq=None):
    _check(lib().quota_quantize_act(_ptr(x, torch.float16), M, d, ldx, _ptr(q_packed, torch.uint8),
                                    _ptr(scale, torch.float32), _ptr(sumsq), _ptr(ressq), _stream()),
           "quota_quantize_act")


def quota_rmsnorm_quantize_act(x, M, d, ldx, gamma, eps, q_packed, scale, sumsq=None, ressq=None, h=None):
    _check(lib().quota_rmsnorm_quantize_act(_ptr(x, torch.float16), M, d, ldx, _ptr(gamma, torch.float32),
                                            C.c_float(eps), _ptr(q_packed, torch.uint8),
                                            _ptr(scale, torch.float32), _ptr(sumsq), _ptr(ressq),
                                            _ptr(h), _stream()), "quota_rmsnorm_quantize_act")


def quota_silu_mul_quantize_act(gu, M, F, q_packed, scale, z=None, z_inject=None):
    _check(lib().quota_silu_mul_quantize_act(_ptr(gu, torch.float16), M, F, _ptr(q_packed, torch.uint8),
                                             _ptr(scale, torch.float32), _ptr(z), _ptr(z_inject),
                                             _stream()), "quota_silu_mul_quantize_act")


def quota_w4a4_gemm(qa, sa, M, W: Weights, y, ldy, residual=None, ldr=0, acc_i32=None):
    _check(lib().quota_w4a4_gemm(_ptr(qa, torch.uint8), _ptr(sa, torch.float32), M, C.byref(W),
                                 _ptr(y), ldy, _ptr(residual), ldr, _ptr(acc_i32), _stream()),
           "quota_w4a4_gemm")


def quota_set_gemm_variant(variant: int):
    _check(lib().quota_set_gemm_variant(int(variant)), "quota_set_gemm_variant")


def quota_rope_kv_quant(qkv, M, H, dh, pos, cosT, sinT, n_pos, q_rot, khat, vhat, k_codes, k_scales,
                        v_codes, v_scales):
    _check(lib().quota_rope_kv_quant(_ptr(qkv, torch.float16), M, H, dh, _ptr(pos, torch.int32),
                                     _ptr(cosT, torch.float32), _ptr(sinT, torch.float32), n_pos,
                                     _ptr(q_rot), _ptr(khat), _ptr(vhat), _ptr(k_codes), _ptr(k_scales),
                                     _ptr(v_codes), _ptr(v_scales), _stream()), "quota_rope_kv_quant")


def quota_kv_quant_append(k, v, B, N, H, dh, keep_rows, n_keep, cache: KVCache):
    _check(lib().quota_kv_quant_append(_ptr(k, torch.float16), _ptr(v, torch.float16), B, N, H, dh,
                                       _ptr(keep_rows), n_keep, C.byref(cache), _stream()),
           "quota_kv_quant_append")


def quota_attention_prefill_gqa(q, khat, vhat, B, N, H, Hkv, dh, vis_begin, Nv, o, cm_inter, cm_intra, ws):
    _check(lib().quota_attention_prefill_gqa(_ptr(q, torch.float16), _ptr(khat, torch.float16),
                                             _ptr(vhat, torch.float16), B, N, H, Hkv, dh, vis_begin, Nv,
                                             _ptr(o), _ptr(cm_inter), _ptr(cm_intra), _ptr(ws), _stream()),
           "quota_attention_prefill_gqa")


def quota_attention_prefill_static(q, khat, vhat, B, N, H, Hkv, dh, vis_begin, Nv, o, cm_inter, cm_intra):
    _check(lib().quota_attention_prefill_static(_ptr(q, torch.float16), _ptr(khat, torch.float16),
                                                _ptr(vhat, torch.float16), B, N, H, Hkv, dh, vis_begin, Nv,
                                                _ptr(o), _ptr(cm_inter), _ptr(cm_intra), _stream()),
           "quota_attention_prefill_static")


def quota_attention_workspace_bytes(B, N, H, dh):
    return lib().quota_attention_workspace_bytes(B, N, H, dh)


def quota_attention_prefill(q, khat, vhat, B, N, H, dh, vis_begin, Nv, o, cm_inter, cm_intra, ws):
    _check(lib().quota_attention_prefill(_ptr(q, torch.float16), _ptr(khat, torch.float16),
                                         _ptr(vhat, torch.float16), B, N, H, dh, vis_begin, Nv,
                                         _ptr(o), _ptr(cm_inter), _ptr(cm_intra), _ptr(ws), _stream()),
           "quota_attention_prefill")


def quota_score_params_default() -> ScoreParams:
    p = ScoreParams()
    lib().quota_score_params_default(C.byref(p))
    return p


def quota_score_tokens(sumsq, ressq, cm_inter, cm_intra, B, Nv, p: ScoreParams, score, normed=None):
    _check(lib().quota_score_tokens(_ptr(sumsq, torch.float32), _ptr(ressq, torch.float32),
                                    _ptr(cm_inter, torch.float32), _ptr(cm_intra, torch.float32), B, Nv,
                                    C.byref(p), _ptr(score, torch.float32), _ptr(normed), _stream()),
           "quota_score_tokens")


def quota_score_tokens_from_hidden(v, B, Nv, d, ldv, stride_b, cm_inter, cm_intra, p: ScoreParams,
                                   score, normed, ws):
    _check(lib().quota_score_tokens_from_hidden(_ptr(v, torch.float16), B, Nv, d, ldv, C.c_long(stride_b),
                                                _ptr(cm_inter, torch.float32), _ptr(cm_intra, torch.float32),
                                                C.byref(p), _ptr(score, torch.float32), _ptr(normed),
                                                _ptr(ws), _stream()), "quota_score_tokens_from_hidden")


def quota_topk_prune(score, B, Nv, K, keep_idx):
    _check(lib().quota_topk_prune(_ptr(score, torch.float32), B, Nv, K, _ptr(keep_idx, torch.int32),
                                  _stream()), "quota_topk_prune")


def quota_prefill_workspace_bytes(L: Layer, B, N):
    return lib().quota_prefill_workspace_bytes(C.byref(L), B, N)


def quota_prefill_layer(L: Layer, st: State, K_l, p: ScoreParams, cache: KVCache, taps, ws):
    _check(lib().quota_prefill_layer(C.byref(L), C.byref(st), int(K_l), C.byref(p), C.byref(cache),
                                     C.byref(taps) if taps is not None else None, _ptr(ws), _stream()),
           "quota_prefill_layer")


def quota_sensitivity(diff_norm, ref_norm, eta: float) -> float:
    """Eq. 1 for one layer from per-sample norms (host sequences of floats)."""
    n = len(diff_norm)
    a, b = (C.c_double * n)(*diff_norm), (C.c_double * n)(*ref_norm)
    out = C.c_double(0.0)
    _check(lib().quota_sensitivity(a, b, n, C.c_double(eta), C.byref(out)), "quota_sensitivity")
    return out.value


def quota_make_recipe(S, tau: float, p_min: float, V0: int):
    """Eq. 2-5 on the host: returns dict(s_norm, pi, r, K) as Python lists."""
    m = len(S)
    s = (C.c_double * m)(*S)
    sn, pi, r = (C.c_double * m)(), (C.c_double * m)(), (C.c_double * m)()
    K = (C.c_int32 * m)()
    _check(lib().quota_make_recipe(s, m, C.c_double(tau), C.c_double(p_min), int(V0), sn, pi, r, K),
           "quota_make_recipe")
    return dict(s_norm=list(sn), pi=list(pi), r=list(r), K=list(K))


def quota_gflops_ratio(V_hat, V0: int, T: int, d: int, F: int, F_vt: float = 0.0, F_pj: float = 0.0) -> float:
    L = len(V_hat)
    v = (C.c_int32 * L)(*[int(x) for x in V_hat])
    out = C.c_double(0.0)
    _check(lib().quota_gflops_ratio(v, L, int(V0), int(T), int(d), int(F), C.c_double(F_vt), C.c_double(F_pj),
                                    C.byref(out)), "quota_gflops_ratio")
    return out.value


def quota_fp_block_workspace_bytes(L: FpLayer, B, N):
    return lib().quota_fp_block_workspace_bytes(C.byref(L), int(B), int(N))


def quota_fp_block(L: FpLayer, x, pos, B, N, x_out, ws):
    _check(lib().quota_fp_block(C.byref(L), _ptr(x, torch.float16), _ptr(pos, torch.int32), int(B), int(N),
                                _ptr(x_out, torch.float16), _ptr(ws), _stream()), "quota_fp_block")


def quota_activation_deviation(xq, x, B, n_per_sample, diff_norm, ref_norm):
    _check(lib().quota_activation_deviation(_ptr(xq, torch.float16), _ptr(x, torch.float16), int(B),
                                            C.c_long(n_per_sample), _ptr(diff_norm, torch.float64),
                                            _ptr(ref_norm, torch.float64), _stream()),
           "quota_activation_deviation")


def quota_profile_block_workspace_bytes(Lq: Layer, Lf: FpLayer, B, N):
    return lib().quota_profile_block_workspace_bytes(C.byref(Lq), C.byref(Lf), int(B), int(N))


def quota_profile_block(Lq: Layer, Lf: FpLayer, x, pos, B, N, scratch_cache: KVCache, diff_norm, ref_norm, ws):
    _check(lib().quota_profile_block(C.byref(Lq), C.byref(Lf), _ptr(x, torch.float16), _ptr(pos, torch.int32),
                                     int(B), int(N), C.byref(scratch_cache), _ptr(diff_norm, torch.float64),
                                     _ptr(ref_norm, torch.float64), _ptr(ws), _stream()), "quota_profile_block")


def quota_attention_decode(q, cache: KVCache, o):
    _check(lib().quota_attention_decode(_ptr(q, torch.float16), C.byref(cache), _ptr(o, torch.float16), _stream()),
           "quota_attention_decode")


def quota_attention_decode_gqa(q, Hq, cache: KVCache, o):
    _check(lib().quota_attention_decode_gqa(_ptr(q, torch.float16), int(Hq), C.byref(cache),
                                            _ptr(o, torch.float16), _stream()), "quota_attention_decode_gqa")


def quota_advance_step(step_dev):
    _check(lib().quota_advance_step(_ptr(step_dev, torch.int32), _stream()), "quota_advance_step")


def quota_decode_workspace_bytes(L: Layer, B):
    return lib().quota_decode_workspace_bytes(C.byref(L), B)


def quota_decode_layer(L: Layer, x, pos, B, cache: KVCache, x_out, taps, ws):
    _check(lib().quota_decode_layer(C.byref(L), _ptr(x, torch.float16), _ptr(pos, torch.int32), int(B),
                                    C.byref(cache), _ptr(x_out, torch.float16),
                                    C.byref(taps) if taps is not None else None, _ptr(ws), _stream()),
           "quota_decode_layer")


def quota_profile_begin(max_launches: int):
    _check(lib().quota_profile_begin(int(max_launches)), "quota_profile_begin")


def quota_profile_bracket_ms(reps: int = 64):
    """(cost of an event pair with no kernel in it, what one empty kernel adds), both in ms."""
    bracket, empty = C.c_float(0.0), C.c_float(0.0)
    _check(lib().quota_profile_bracket_ms(int(reps), _stream(), C.byref(bracket), C.byref(empty)),
           "quota_profile_bracket_ms")
    return bracket.value, empty.value


def quota_profile_collect():
    """Returns {kernel name: dict(launches, total_ms, ops, bytes)} for the kernels that ran."""
    arr = (KernelStat * KERNEL_COUNT)()
    _check(lib().quota_profile_collect(arr), "quota_profile_collect")
    out = {}
    for i in range(KERNEL_COUNT):
        if arr[i].launches:
            out[lib().quota_kernel_name(i).decode()] = dict(launches=arr[i].launches, total_ms=arr[i].total_ms,
                                                            ops=arr[i].ops, bytes=arr[i].bytes)
    return out


def quota_kernel_name(kernel_id: int) -> str:
    return lib().quota_kernel_name(int(kernel_id)).decode()


def quota_strerror(code: int) -> str:
    return lib().quota_strerror(int(code)).decode()
