"""Memory plumbing around the C-ABI library: allocates the CPU expert cache (pinned), the GPU
expert cache (slots), router / shared weights and the workspace with torch, fills them from the
seeded generators and binds them to a MoeContext.  No arithmetic of the method lives here.
"""
from __future__ import annotations

import numpy as np
import torch

from . import synth as S
from .binding import MoeContext


def np_to_dev(a: np.ndarray, device="cuda:0") -> torch.Tensor:
    """uint16 (bf16 bits) / float32 / int32 numpy array -> device tensor with the same bits."""
    t = torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).to(device)
    # the copy is ordered on torch's current stream only; the library's streams are independent of it,
    # so the tensor must have landed before it is handed to a call
    torch.cuda.current_stream(t.device).synchronize()
    return t


def dev_to_np_u16(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().view(torch.int16).numpy().view(np.uint16)


class HostPool:
    """All experts of one layer in pinned host memory: the CPU expert cache (Section V-A).
    fmt 0: bf16 blobs; 1 (or q8=True): e4m3 codes with per-row scales; 2: 4-bit codes in groups of 128 with
    scale and zero point; 3: MXFP4 -- all quantised from the seeded bf16 blobs."""

    def __init__(self, w: S.Workload, layer: int, fill: bool = True, share_from: "HostPool | None" = None,
                 q8: bool = False, fmt: "int | None" = None):
        self.fmt = (1 if q8 else 0) if fmt is None else fmt
        self.w, self.layer, self.q8 = w, layer, self.fmt != 0     # q8: "holds a quantised form"
        self.bytes_per_expert = {0: lambda: w.blob_bytes, 1: lambda: S.q8_blob_bytes(w.d, w.I),
                                 2: lambda: S.q4_blob_bytes(w.d, w.I), 3: lambda: S.mx4_blob_bytes(w.d, w.I)}[self.fmt]()
        if share_from is not None:
            assert share_from.fmt == self.fmt
            self.buf = share_from.buf
        else:
            self.buf = torch.empty((w.E, self.bytes_per_expert), dtype=torch.uint8, pin_memory=True)
            if fill:
                for e in range(w.E):
                    if self.fmt == 1:
                        S.quantize_blob_into(self.ptr(e), S.expert_blob(w, layer, e), w.d, w.I)
                    elif self.fmt == 2:
                        S.quantize4_blob_into(self.ptr(e), S.expert_blob(w, layer, e), w.d, w.I)
                    elif self.fmt == 3:
                        S.quantize_mx4_blob_into(self.ptr(e), S.expert_blob(w, layer, e), w.d, w.I)
                    else:
                        S.expert_blob_into(self.ptr(e), w, layer, e)

    def ptr(self, e: int) -> int:
        return self.buf.data_ptr() + e * self.bytes_per_expert

    def ptrs(self):
        return [self.ptr(e) for e in range(self.w.E)]

    def blob_np(self, e: int) -> np.ndarray:
        """The stored bytes of expert e: bf16 bit patterns, or (q8) the raw 8-bit blob."""
        raw = self.buf[e].numpy()
        return raw if self.q8 else raw.view(np.uint16)


class DeviceLayer:
    """Device-side memory of one layer, bound to `ctx` as layer `layer`."""

    def __init__(self, ctx: MoeContext, w: S.Workload, layer: int, pool: HostPool, initial=None,
                 device="cuda:0", poison: bool = False, slots=None):
        """slots: an existing slot tensor to bind (contexts with shared_slots: one for all layers)."""
        self.ctx, self.w, self.layer, self.pool = ctx, w, layer, pool
        Sslots = ctx.cfg.cache_slots
        self.router_np = S.router_weight(w, layer)
        self.router = np_to_dev(self.router_np, device)
        self.shared_np = S.shared_blob(w, layer)
        self.shared = np_to_dev(self.shared_np, device) if self.shared_np is not None else None
        own = slots is None
        # the cache: Sslots slots of one bf16 blob each and then (4-bit integer host format) one staging area
        # per slot; for an e4m3 or MXFP4 pool the slots hold the quantised blobs themselves (each rounded up
        # to 256 bytes)
        self.cache = torch.empty(ctx.moe_cache_bytes() // 2, dtype=torch.int16, device=device) if own else slots
        direct = pool.fmt in (1, 3)
        self.slot_bytes = (pool.bytes_per_expert + 255) // 256 * 256 if direct else w.blob_bytes
        self.slots = self.cache.view(-1)[:Sslots * self.slot_bytes // 2].view(Sslots, self.slot_bytes // 2)
        if poison and own:
            self.cache.fill_(0x7FC0)  # bf16 NaN pattern (0xC0 0x7F as e4m3 codes: -2 and NaN): an unfilled slot shows up
        if initial is not None:
            assert pool.fmt in (0, 1, 3), "initial residents are blobs in the form the slots hold"
            for s, e in enumerate(initial):
                if e >= 0:
                    self.slots[s].view(torch.uint8)[:pool.bytes_per_expert].copy_(pool.buf[e], non_blocking=False)
        # fills and uploads above ran on torch's current stream; the library's streams are independent
        # of it, so everything must have landed before the layer is used
        torch.cuda.current_stream(self.cache.device).synchronize()
        ctx.moe_bind_layer(layer, pool.ptrs(), self.router, self.shared, self.cache, initial)


class Buffers:
    """x / y / workspace / routing-table tensors for calls on T tokens."""

    def __init__(self, ctx: MoeContext, T: int, device="cuda:0"):
        c = ctx.cfg
        self.T = T
        self.ws = torch.empty(ctx.moe_workspace_bytes(T), dtype=torch.uint8, device=device)
        assert self.ws.data_ptr() % 256 == 0
        self.y = torch.empty((T, c.d), dtype=torch.int16, device=device)
        n = T * c.k
        self.ids = torch.empty((T, c.k), dtype=torch.int32, device=device)
        self.wts = torch.empty((T, c.k), dtype=torch.float32, device=device)
        self.counts = torch.empty(c.E, dtype=torch.int32, device=device)
        self.offsets = torch.empty(c.E + 1, dtype=torch.int32, device=device)
        self.perm = torch.empty(n, dtype=torch.int32, device=device)
        self.inv_perm = torch.empty(n, dtype=torch.int32, device=device)

    def routing(self, ctx: MoeContext, stream) -> dict:
        ctx.moe_debug_routing(self.ws, self.T, self.ids, self.wts, self.counts, self.offsets, self.perm,
                              self.inv_perm, stream)
        stream.synchronize()
        return dict(ids=self.ids.cpu().numpy(), w=self.wts.cpu().numpy(), counts=self.counts.cpu().numpy(),
                    offsets=self.offsets.cpu().numpy(), perm=self.perm.cpu().numpy(),
                    inv_perm=self.inv_perm.cpu().numpy())
