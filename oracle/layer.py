"""Oracle composite: one W4A4 decoder layer with in-layer visual-token pruning.

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).  Follows the paper's
deployment description step by step (Method overview; Eq. 5-9; the compaction
paragraph after Eq. 9): run the quantized layer on all tokens that entered it,
compute the four cues from that quantized forward pass, normalise, fuse, take
the budgeted top-k, and propagate only the kept visual tokens (plus every text
token) -- hidden state, positions and 4-bit K/V alike -- to the next block.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass
class LayerWeights:
    """int4 codes (unpacked int8) + fp16 group scales of one decoder layer.

    qkv: [3d, d] rows ordered q | k | v;  o: [d, d];  gu: [2F, d] rows ordered
    gate | up;  down: [d, F].  gamma1/gamma2: fp32 [d] RMSNorm gains.
    """
    qkv: tuple
    o: tuple
    gu: tuple
    down: tuple
    gamma1: np.ndarray
    gamma2: np.ndarray
    eps: float
    H: int
    dh: int
    F: int
    Hkv: int = None     # K/V heads (grouped-query attention); None = H.  qkv then has (H + 2 Hkv) dh rows

    @property
    def kv_heads(self) -> int:
        return self.H if self.Hkv is None else self.Hkv


def kept_rows(keep_idx, B, N, vis_begin, Nv):
    """Rows (per sequence, ascending) that survive: kept visual + all text."""
    rows = []
    for b in range(B):
        vis = vis_begin + keep_idx[b].astype(np.int64)
        txt = np.concatenate([np.arange(0, vis_begin), np.arange(vis_begin + Nv, N)])
        rows.append(np.sort(np.concatenate([vis, txt])))
    return np.stack(rows).astype(np.int32)          # [B, n_keep]


def prefill_layer(W: LayerWeights, x, pos, B, N, vis_begin, Nv, K, cos, sin,
                  score_params=None, prune_mid=False, inject=None):
    """One layer.  x fp16 [B*N, d]; pos int32 [B*N] (original position ids).

    Returns a dict of every tensor that crosses a step boundary.  With
    ``prune_mid`` the rows are compacted right after selection and the output
    projection / FFN run on kept rows only; the result for kept rows must be
    identical (every remaining step is token-wise) -- a test checks that.
    ``inject`` may override 'o', 'cm_inter', 'cm_intra' (tests only).
    """
    from . import (quantize_act, rmsnorm, w4a4_gemm, rope, kv_quant, attention,
                   score, topk, silu_mul)
    sp = dict(w_m=0.25, w_c=0.45, w_s=0.10, w_r=0.20, p_lo=10, p_hi=90)
    if score_params:
        sp.update(score_params)
    d = W.H * W.dh
    x = np.ascontiguousarray(x, np.float16).reshape(B * N, d)
    pos = np.ascontiguousarray(pos, np.int32).reshape(B * N)
    out = {}

    # Eq. 6 vector cues of the hidden state entering the layer
    _, _, sumsq, ressq = quantize_act(x)
    vis_rows = (np.arange(B)[:, None] * N + vis_begin + np.arange(Nv)[None, :]).reshape(-1)
    out["sumsq"] = sumsq[vis_rows].reshape(B, Nv)
    out["ressq"] = ressq[vis_rows].reshape(B, Nv)

    # attention half, on all tokens that entered the layer
    h1 = rmsnorm(x, W.gamma1, W.eps)
    qa1, sa1, _, _ = quantize_act(h1)
    qkv = w4a4_gemm(qa1, sa1, *W.qkv)
    dkv = W.kv_heads * W.dh
    q = rope(qkv[:, :d], W.H, W.dh, pos, cos, sin)
    k = rope(qkv[:, d:d + dkv], W.kv_heads, W.dh, pos, cos, sin)
    v = np.ascontiguousarray(qkv[:, d + dkv:])
    kc, ks, khat = kv_quant(k)
    vc, vs, vhat = kv_quant(v)
    o, cm_inter, cm_intra = attention(q, khat, vhat, B, N, W.H, W.dh, vis_begin, Nv, Hkv=W.kv_heads)
    if inject:
        o = inject.get("o", o)
        cm_inter = inject.get("cm_inter", cm_inter)
        cm_intra = inject.get("cm_intra", cm_intra)
    out.update(h1=h1, qa1=qa1, sa1=sa1, qkv=qkv, q=q, k=k, kc=kc, ks=ks, vc=vc, vs=vs,
               khat=khat, vhat=vhat, o=o, cm_inter=cm_inter, cm_intra=cm_intra)

    # Eq. 7-9
    sc, normed = score(out["sumsq"], out["ressq"], cm_inter, cm_intra, want_normed=True, **sp)
    keep_idx = topk(sc, K)
    rows = kept_rows(keep_idx, B, N, vis_begin, Nv)
    n_keep = rows.shape[1]
    flat = (np.arange(B)[:, None] * N + rows).reshape(-1)
    out.update(score=sc, normed=normed, keep_idx=keep_idx, rows=rows, n_keep=n_keep)

    def rest(xr, orow):
        qa2, sa2, _, _ = quantize_act(orow)
        x1 = w4a4_gemm(qa2, sa2, *W.o, residual=xr)
        h2 = rmsnorm(x1, W.gamma2, W.eps)
        qa3, sa3, _, _ = quantize_act(h2)
        gu = w4a4_gemm(qa3, sa3, *W.gu)
        z = silu_mul(gu, W.F)
        if inject and "z" in inject and z.shape == inject["z"].shape:
            z = inject["z"]
        qa4, sa4, _, _ = quantize_act(z)
        xn = w4a4_gemm(qa4, sa4, *W.down, residual=x1)
        return dict(qa2=qa2, sa2=sa2, x1=x1, h2=h2, qa3=qa3, sa3=sa3, gu=gu, z=z,
                    qa4=qa4, sa4=sa4, x_next=xn)

    if prune_mid:
        r = rest(x[flat], o[flat])
        out.update(r)
    else:
        r = rest(x, o)
        out.update({k_: (v_[flat] if isinstance(v_, np.ndarray) else v_) for k_, v_ in r.items()})
    out["pos_next"] = pos[flat]
    # this layer's 4-bit KV cache holds kept rows only
    out.update(cache_kc=kc[flat], cache_ks=ks[flat], cache_vc=vc[flat], cache_vs=vs[flat])
    out["Nv_next"] = keep_idx.shape[1]
    return out


def dequant_kv(codes, scales, g: int = 64):
    """x_hat = fp16(code * scale): what attention sees of a 4-bit K or V row.

    codes int8 [..., D] in [-8, 7]; scales fp16 [..., D/g].  The product of a
    4-bit integer and an fp16 value is exact in fp32, so the only rounding is
    the one back to fp16 -- the same value the quantizer reports as x_hat.
    """
    s = np.repeat(np.asarray(scales, np.float16).astype(np.float32), g, axis=-1)
    return (np.asarray(codes, np.int8).astype(np.float32) * s).astype(np.float16)


def decode_attention(q, kc, ks, vc, vs, H: int, dh: int, Hkv: int = None):
    """Single-query attention of one new token per sequence over its 4-bit cache.

    q fp16 [B, H*dh] (rotated); kc/vc int8 [B, L, H*dh]; ks/vs fp16 [B, L, H*dh/64];
    the L cached rows include the new token's own K/V (appended before the read).
    Per head: s_t = q . k_hat_t / sqrt(dh), p = softmax_t(s), o = sum_t p_t v_hat_t,
    all in fp64, o rounded once to fp16.  (Decode stage of the deployment pipeline:
    attention over the pruned quantized KV cache.)
    """
    from . import f64_to_f16
    B, L, D = kc.shape
    Hkv = H if Hkv is None else Hkv
    rep = H // Hkv                      # query head h reads K/V head h // rep
    khat = dequant_kv(kc, ks).astype(np.float64).reshape(B, L, Hkv, dh)
    vhat = dequant_kv(vc, vs).astype(np.float64).reshape(B, L, Hkv, dh)
    qf = np.asarray(q, np.float16).astype(np.float64).reshape(B, H, dh)
    o = np.zeros((B, H, dh), np.float64)
    for b in range(B):
        for h in range(H):
            s = khat[b, :, h // rep, :] @ qf[b, h] / np.sqrt(float(dh))
            p = np.exp(s - s.max())
            p /= p.sum()
            o[b, h] = p @ vhat[b, :, h // rep, :]
    return f64_to_f16(o.reshape(B, H * dh))


def decode_layer(W: LayerWeights, x, pos, cache, cos, sin, inject=None):
    """One decode step of one layer: a single new token per sequence.

    x fp16 [B, d]; pos int32 [B] (the new token's original position id); cache: dict
    with kc/vc int8 [B, L, d] and ks/vs fp16 [B, L, d/64] -- the layer's pruned
    4-bit KV cache (kept prefill rows, then earlier decode tokens).  The new
    token's K (post-RoPE) and V are quantized exactly like prefill rows, appended,
    and attention reads the L+1 rows back from their 4-bit form.  Nothing is
    pruned at decode time.  ``inject`` may override 'o' and 'z' (tests only).
    Returns the step's tensors and the grown cache under 'cache'.
    """
    from . import quantize_act, rmsnorm, w4a4_gemm, rope, kv_quant, silu_mul
    d = W.H * W.dh
    x = np.ascontiguousarray(x, np.float16).reshape(-1, d)
    B = x.shape[0]
    pos = np.ascontiguousarray(pos, np.int32).reshape(B)
    h1 = rmsnorm(x, W.gamma1, W.eps)
    qa1, sa1, _, _ = quantize_act(h1)
    qkv = w4a4_gemm(qa1, sa1, *W.qkv)
    dkv = W.kv_heads * W.dh
    q = rope(qkv[:, :d], W.H, W.dh, pos, cos, sin)
    k = rope(qkv[:, d:d + dkv], W.kv_heads, W.dh, pos, cos, sin)
    v = np.ascontiguousarray(qkv[:, d + dkv:])
    kc, ks, _ = kv_quant(k)
    vc, vs, _ = kv_quant(v)
    grown = dict(kc=np.concatenate([cache["kc"], kc[:, None, :]], axis=1),
                 ks=np.concatenate([cache["ks"], ks[:, None, :]], axis=1),
                 vc=np.concatenate([cache["vc"], vc[:, None, :]], axis=1),
                 vs=np.concatenate([cache["vs"], vs[:, None, :]], axis=1))
    o = decode_attention(q, grown["kc"], grown["ks"], grown["vc"], grown["vs"], W.H, W.dh, W.kv_heads)
    if inject and "o" in inject:
        o = inject["o"]
    qa2, sa2, _, _ = quantize_act(o)
    x1 = w4a4_gemm(qa2, sa2, *W.o, residual=x)
    h2 = rmsnorm(x1, W.gamma2, W.eps)
    qa3, sa3, _, _ = quantize_act(h2)
    gu = w4a4_gemm(qa3, sa3, *W.gu)
    z = silu_mul(gu, W.F)
    if inject and "z" in inject:
        z = inject["z"]
    qa4, sa4, _, _ = quantize_act(z)
    x_next = w4a4_gemm(qa4, sa4, *W.down, residual=x1)
    return dict(qkv=qkv, q=q, kc=kc, ks=ks, vc=vc, vs=vs, o=o, x1=x1, gu=gu, z=z, x_next=x_next,
                cache=grown)


def cache_from_prefill(out, B):
    """The [B, L, .] cache arrays that a prefill_layer result appended."""
    return {k: out["cache_" + k].reshape(B, -1, out["cache_" + k].shape[-1]) for k in ("kc", "ks", "vc", "vs")}
