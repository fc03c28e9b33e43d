"""Device-memory plumbing around the C ABI: packed weights, KV caches, the
layer descriptor and a layer-stack runner.  No arithmetic happens here -- every
step of the path runs in libquota's kernels; torch only owns the buffers and
the stream.
"""
from __future__ import annotations

import ctypes as C
from typing import List, Optional

import torch

from . import binding as qb


def _dev():
    return torch.device("cuda", torch.cuda.current_device())


class PackedLinear:
    """One W4 matrix in the library's GEMM layout (buffers owned here)."""

    def __init__(self, N: int, K: int):
        self.N, self.K = N, K
        self.packed = torch.empty(qb.quota_weights_packed_bytes(N, K), dtype=torch.uint8, device=_dev())
        self.scales = torch.empty(qb.quota_weights_scale_bytes(N, K) // 2, dtype=torch.float16, device=_dev())
        self.desc = qb.Weights(N, K, self.packed.data_ptr(), self.scales.data_ptr())

    @classmethod
    def from_codes(cls, codes: torch.Tensor, scales: torch.Tensor) -> "PackedLinear":
        """codes int8 [N,K] in [-8,7], scales fp16 [N, ceil(K/128)] (device tensors)."""
        N, K = codes.shape
        self = cls(N, K)
        qb.quota_pack_weights(codes.contiguous(), scales.contiguous(), self.desc)
        return self

    @classmethod
    def from_fp32(cls, w: torch.Tensor, keep_plain: bool = False) -> "PackedLinear":
        """Quantize an fp32 [N,K] device matrix on the GPU, then pack it."""
        N, K = w.shape
        G = (K + 127) // 128
        codes = torch.empty((N, K), dtype=torch.int8, device=w.device)
        scales = torch.empty((N, G), dtype=torch.float16, device=w.device)
        qb.quota_quantize_weights(w.contiguous(), codes, scales)
        self = cls.from_codes(codes, scales)
        if keep_plain:
            self.codes, self.plain_scales = codes, scales
        return self

    def nbytes(self) -> int:
        return self.packed.numel() + self.scales.numel() * 2


class KVCache4:
    """4-bit KV cache of one layer."""

    def __init__(self, B: int, capacity: int, H: int, dh: int):
        d = H * dh
        dev = _dev()
        self.k_codes = torch.empty((B, capacity, d // 2), dtype=torch.uint8, device=dev)
        self.v_codes = torch.empty((B, capacity, d // 2), dtype=torch.uint8, device=dev)
        self.k_scales = torch.empty((B, capacity, d // 64), dtype=torch.float16, device=dev)
        self.v_scales = torch.empty((B, capacity, d // 64), dtype=torch.float16, device=dev)
        self.desc = qb.KVCache(B, capacity, H, dh, 0, self.k_codes.data_ptr(), self.k_scales.data_ptr(),
                               self.v_codes.data_ptr(), self.v_scales.data_ptr())

    @property
    def len(self) -> int:
        return self.desc.len

    def reset(self):
        self.desc.len = 0


class PrefillLayer:
    """Descriptor + buffers of one decoder layer."""

    def __init__(self, H: int, dh: int, F: int, qkv: PackedLinear, o: PackedLinear, gu: PackedLinear,
                 down: PackedLinear, gamma1: torch.Tensor, gamma2: torch.Tensor, eps: float,
                 cosT: torch.Tensor, sinT: torch.Tensor, Hkv: Optional[int] = None):
        self.H, self.dh, self.F, self.d = H, dh, F, H * dh
        self.Hkv = H if Hkv is None else Hkv          # K/V heads (grouped-query attention)
        self.qkv, self.o, self.gu, self.down = qkv, o, gu, down
        self.gamma1, self.gamma2, self.cosT, self.sinT = gamma1, gamma2, cosT, sinT
        self.desc = qb.Layer(H, dh, F, eps, gamma1.data_ptr(), gamma2.data_ptr(), qkv.desc, o.desc,
                             gu.desc, down.desc, cosT.data_ptr(), sinT.data_ptr(), cosT.shape[0], self.Hkv)

    def workspace_bytes(self, B: int, N: int) -> int:
        return qb.quota_prefill_workspace_bytes(self.desc, B, N)

    def decode_workspace_bytes(self, B: int) -> int:
        return qb.quota_decode_workspace_bytes(self.desc, B)

    def decode(self, x: torch.Tensor, pos: torch.Tensor, cache: "KVCache4", x_out: torch.Tensor,
               ws: torch.Tensor, taps=None):
        """One decode step of this layer: x fp16 [B, d], pos int32 [B]; appends to ``cache``."""
        qb.quota_decode_layer(self.desc, x, pos, x.shape[0], cache.desc, x_out, taps, ws)

    def weight_bytes(self) -> int:
        return sum(w.nbytes() for w in (self.qkv, self.o, self.gu, self.down))


class FullPrecisionLayer:
    """fp16 weights of one decoder layer for the calibration-time full-precision block (Eq. 1)."""

    def __init__(self, H: int, dh: int, F: int, wqkv: torch.Tensor, wo: torch.Tensor, wgu: torch.Tensor,
                 wdown: torch.Tensor, gamma1: torch.Tensor, gamma2: torch.Tensor, eps: float,
                 cosT: torch.Tensor, sinT: torch.Tensor, Hkv: Optional[int] = None):
        self.H, self.dh, self.F, self.d = H, dh, F, H * dh
        self.Hkv = H if Hkv is None else Hkv
        self.w = [t.to(torch.float16).contiguous() for t in (wqkv, wo, wgu, wdown)]
        self.gamma1, self.gamma2, self.cosT, self.sinT = gamma1, gamma2, cosT, sinT
        self.desc = qb.FpLayer(H, dh, F, self.Hkv, eps, gamma1.data_ptr(), gamma2.data_ptr(),
                               *[t.data_ptr() for t in self.w], cosT.data_ptr(), sinT.data_ptr(), cosT.shape[0])

    def forward(self, x: torch.Tensor, pos: torch.Tensor, B: int, N: int) -> torch.Tensor:
        ws = torch.empty(qb.quota_fp_block_workspace_bytes(self.desc, B, N), dtype=torch.uint8, device=x.device)
        out = torch.empty_like(x)
        qb.quota_fp_block(self.desc, x, pos, B, N, out, ws)
        return out


def profile_sensitivity(layer: PrefillLayer, full: FullPrecisionLayer, x: torch.Tensor, pos: torch.Tensor,
                        B: int, N: int, eta: float = 1e-6):
    """S of Eq. 1 for one block over the B calibration samples in x (fp16 [B*N, d]): the low-bit and
    the full-precision block run on the same input; returns (S, diff_norm, ref_norm)."""
    dev = x.device
    scratch = KVCache4(B, N, layer.Hkv, layer.dh)
    ws = torch.empty(qb.quota_profile_block_workspace_bytes(layer.desc, full.desc, B, N), dtype=torch.uint8, device=dev)
    dn = torch.empty(B, dtype=torch.float64, device=dev)
    rn = torch.empty(B, dtype=torch.float64, device=dev)
    qb.quota_profile_block(layer.desc, full.desc, x, pos, B, N, scratch.desc, dn, rn, ws)
    dn, rn = dn.cpu().tolist(), rn.cpu().tolist()
    return qb.quota_sensitivity(dn, rn, eta), dn, rn


def make_taps(**tensors) -> qb.Taps:
    t = qb.Taps()
    for k, v in tensors.items():
        setattr(t, k, v.data_ptr() if v is not None else None)
    return t


class PrefillStack:
    """Runs a stack of layers over one batch: ping-pong hidden-state buffers,
    one KV cache per layer, one shared workspace.  ``run`` only enqueues."""

    def __init__(self, layers: List[PrefillLayer], B: int, N: int, vis_begin: int, Nv: int,
                 budgets: List[int], params: Optional[qb.ScoreParams] = None, decode_capacity: int = 0):
        assert len(budgets) == len(layers)
        self.layers, self.B, self.N0, self.vis_begin, self.Nv0 = layers, B, N, vis_begin, Nv
        self.budgets = list(budgets)
        self.params = params or qb.quota_score_params_default()
        L0 = layers[0]
        dev = _dev()
        self.ws = torch.empty(max(l.workspace_bytes(B, N) for l in layers), dtype=torch.uint8, device=dev)
        self.xbuf = [torch.empty((B * N, L0.d), dtype=torch.float16, device=dev) for _ in range(2)]
        self.posbuf = [torch.empty((B * N,), dtype=torch.int32, device=dev) for _ in range(2)]
        # cache capacity per layer = rows that layer keeps
        self.caches = []
        n, nv = N, Nv
        self.n_keep = []
        for K in budgets:
            k = nv if K < 0 else min(K, nv)      # K < 0 (qb.KEEP_ALL): not a candidate layer, nothing pruned
            n = n - nv + k
            nv = k
            self.n_keep.append(n)
            self.caches.append(KVCache4(B, n + decode_capacity, L0.Hkv, L0.dh))
        self.dec_ws = None
        if decode_capacity:
            self.dec_ws = torch.empty(max(l.decode_workspace_bytes(B) for l in layers), dtype=torch.uint8,
                                      device=dev)
            self.dec_x = [torch.empty((B, L0.d), dtype=torch.float16, device=dev) for _ in range(2)]

    def run(self, x0: torch.Tensor, pos0: torch.Tensor, taps: Optional[List] = None):
        """x0 fp16 [B*N, d], pos0 int32 [B*N].  Returns (x_out view, pos_out view, N, Nv)."""
        B = self.B
        x_in, pos_in = x0, pos0
        N, Nv = self.N0, self.Nv0
        for i, (L, K) in enumerate(zip(self.layers, self.budgets)):
            x_out, pos_out = self.xbuf[i & 1], self.posbuf[i & 1]
            self.caches[i].reset()
            st = qb.State(B, N, self.vis_begin, Nv, x_in.data_ptr(), pos_in.data_ptr(),
                          x_out.data_ptr(), pos_out.data_ptr())
            qb.quota_prefill_layer(L.desc, st, K, self.params, self.caches[i].desc,
                                   taps[i] if taps else None, self.ws)
            N, Nv = st.N, st.Nv
            x_in, pos_in = x_out, pos_out
        d = self.layers[0].d
        return x_in[: B * N].view(B * N, d), pos_in[: B * N], N, Nv

    def begin_stepped_decode(self, max_steps: int) -> torch.Tensor:
        """Switches every layer's cache to a device-side step count (for decode loops captured in a HIP
        graph): decode() then appends at row len + step and leaves the host lengths alone.  Returns
        the int32 [1] device counter (zeroed); advance it with qb.quota_advance_step between steps."""
        self.step_dev = torch.zeros(1, dtype=torch.int32, device=_dev())
        for c in self.caches:
            c.desc.step_dev, c.desc.max_steps = self.step_dev.data_ptr(), int(max_steps)
        return self.step_dev

    def end_stepped_decode(self, steps_done: int):
        """Folds the steps of a stepped decode loop into the host lengths and returns to host-side lengths."""
        for c in self.caches:
            c.desc.len += int(steps_done)
            c.desc.step_dev, c.desc.max_steps = None, 0
        self.step_dev = None

    def decode(self, x: torch.Tensor, pos: torch.Tensor, taps: Optional[List] = None):
        """One decode step through every layer for one new token per sequence: x fp16 [B, d],
        pos int32 [B] (original position ids).  Each layer appends the token's 4-bit K/V to its own
        pruned cache and attends over it.  Returns the last layer's output (a view of an internal
        buffer, valid until the next call)."""
        assert self.dec_ws is not None, "construct the stack with decode_capacity > 0"
        x_in = x
        for i, L in enumerate(self.layers):
            x_out = self.dec_x[i & 1]
            L.decode(x_in, pos, self.caches[i], x_out, self.dec_ws, taps[i] if taps else None)
            x_in = x_out
        return x_in
