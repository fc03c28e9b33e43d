"""Oracle for the sensitivity profiling that feeds the offline allocator (Eq. 1).

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).  Eq. 1 compares, per candidate layer and
per calibration sample, a full-precision activation x with its low-bit counterpart x^q computed
by the deployed low-bit operators.  Readings where the paper is silent:

* the activation of layer l is the hidden state that LEAVES block l;
* both runs of a block start from the same block input (a per-block deviation; errors of earlier
  blocks do not accumulate into it);
* the low-bit run prunes nothing (calibration precedes the recipe);
* a sample is one sequence, and the norms run over all of its tokens and channels;
* "full precision" is plain fp64 arithmetic on the stored (fp16) weights and input.

``block_full_precision`` is the ordinary decoder block (RMSNorm, q|k|v projection, rotate-half
RoPE at the tokens' position ids, causal softmax attention with grouped K/V heads, output
projection + residual, RMSNorm, SwiGLU, + residual) with no quantizer anywhere.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

from . import recipe
from .layer import LayerWeights, prefill_layer


@dataclass
class FullPrecisionWeights:
    """Float weights of one decoder layer, same shapes and row orders as ``LayerWeights``:
    qkv [(H + 2 Hkv) dh, d] rows q | k | v, o [d, d], gu [2F, d] rows gate | up, down [d, F]."""
    qkv: np.ndarray
    o: np.ndarray
    gu: np.ndarray
    down: np.ndarray
    gamma1: np.ndarray
    gamma2: np.ndarray
    eps: float
    H: int
    dh: int
    F: int
    Hkv: int = None

    @property
    def kv_heads(self) -> int:
        return self.H if self.Hkv is None else self.Hkv


def _rms_norm(t, gamma, eps):
    ms = np.mean(t * t, axis=-1, keepdims=True)
    return t / np.sqrt(ms + eps) * gamma


def _rotate(t, heads, dh, c, s):
    """t [N, heads*dh]; c, s [N, dh/2] at each token's position id.  Pairs (i, i + dh/2)."""
    N = t.shape[0]
    t = t.reshape(N, heads, dh)
    lo, hi = t[:, :, :dh // 2], t[:, :, dh // 2:]
    c, s = c[:, None, :], s[:, None, :]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=2).reshape(N, heads * dh)


def block_full_precision(W: FullPrecisionWeights, x, pos, B, N, cos, sin):
    """x [B*N, d] (fp16 values), pos int32 [B*N] original position ids, cos/sin [P, dh/2].
    Returns the block output, fp64 [B*N, d]."""
    H, dh, Hkv, F = W.H, W.dh, W.kv_heads, W.F
    d, dkv, rep = H * dh, Hkv * dh, H // Hkv
    x = np.asarray(x, np.float64).reshape(B, N, d)
    pos = np.asarray(pos, np.int64).reshape(B, N)
    g1, g2 = np.asarray(W.gamma1, np.float64), np.asarray(W.gamma2, np.float64)
    Wqkv, Wo, Wgu, Wd = (np.asarray(w, np.float64) for w in (W.qkv, W.o, W.gu, W.down))
    cos, sin = np.asarray(cos, np.float64), np.asarray(sin, np.float64)
    causal = np.tril(np.ones((N, N), bool))
    out = np.empty((B, N, d))
    for b in range(B):
        xb = x[b]
        qkv = _rms_norm(xb, g1, W.eps) @ Wqkv.T
        c, s = cos[pos[b]], sin[pos[b]]
        q = _rotate(qkv[:, :d], H, dh, c, s)
        k = _rotate(qkv[:, d:d + dkv], Hkv, dh, c, s)
        v = qkv[:, d + dkv:]
        o = np.empty((N, d))
        for h in range(H):
            kv = h // rep
            logits = q[:, h * dh:(h + 1) * dh] @ k[:, kv * dh:(kv + 1) * dh].T / np.sqrt(dh)
            logits = np.where(causal, logits, -np.inf)
            e = np.exp(logits - logits.max(axis=1, keepdims=True))
            o[:, h * dh:(h + 1) * dh] = (e / e.sum(axis=1, keepdims=True)) @ v[:, kv * dh:(kv + 1) * dh]
        x1 = xb + o @ Wo.T
        gu = _rms_norm(x1, g2, W.eps) @ Wgu.T
        gate, up = gu[:, :F], gu[:, F:]
        out[b] = x1 + (gate / (1.0 + np.exp(-gate)) * up) @ Wd.T
    return out.reshape(B * N, d)


def activation_deviation(xq, x, B):
    """Numerator and denominator of Eq. 1 per sample: ||x^q - x||_2 and ||x||_2 over all of a
    sample's tokens and channels.  xq, x [B*N, d] -> (diff_norm [B], ref_norm [B])."""
    xq = np.asarray(xq, np.float64).reshape(B, -1)
    x = np.asarray(x, np.float64).reshape(B, -1)
    return np.sqrt(((xq - x) ** 2).sum(axis=1)), np.sqrt((x ** 2).sum(axis=1))


def profile_block(Wq: LayerWeights, Wf: FullPrecisionWeights, x, pos, B, N, vis_begin, Nv, cos, sin):
    """One block, both ways, on the same input: (diff_norm [B], ref_norm [B])."""
    low = prefill_layer(Wq, x, pos, B, N, vis_begin, Nv, Nv, cos, sin)       # K = Nv: nothing pruned
    full = block_full_precision(Wf, x, pos, B, N, cos, sin)
    return activation_deviation(low["x_next"].astype(np.float64), full, B)


def profile_sensitivity(Wq, Wf, x, pos, B, N, vis_begin, Nv, cos, sin, eta: float = 1e-6) -> float:
    """S of Eq. 1 for one layer over the B samples of x."""
    diff_norm, ref_norm = profile_block(Wq, Wf, x, pos, B, N, vis_begin, Nv, cos, sin)
    return recipe.sensitivity(diff_norm, ref_norm, eta)
