"""The four entry points of the method on the oracle's side, with host arrays.

TEST INFRASTRUCTURE ONLY.  `RefMoe` has the call names and argument order of the library's
interface (expert_cache_prefetch, predictor_score, moe_prefill_layer, moe_decode_layer, plus bind,
counters and cache state), so a test can drive the library and the oracle through one table of
calls and compare after every call.  Nothing is computed here: each call is a composition of the
oracle's pinned pieces, in the order the paper gives them:

  moe_prefill_layer / moe_decode_layer   gate -> Top-k -> grouping -> experts -> weighted sum
                                         (Sections II-A, V-B), then the cache serves the experts
                                         that received tokens (hits first, misses re-fetched:
                                         Sections V-B, V-C)
  expert_cache_prefetch                  the cache simulator's prefetch (Sections V-B, V-C)
  predictor_score                        the linear stand-in scorer summed over the batch, top-m
                                         (Sections IV-B, V-C)

The numbers of a layer never depend on the cache state (Section V-C), so the two halves do not
interact: the layer's output comes from the numerical oracle, the counters from the simulator.
Quantised CPU expert caches are expanded with the oracle's own expansion first.
"""
from __future__ import annotations

import numpy as np

from . import (dequant4_blob, dequant_blob, dequant_mx4_blob, moe_layer, predictor_score as _predictor_score)
from .cache_sim import CacheSim, SharedCacheSim

_EXPAND = {1: dequant_blob, 2: dequant4_blob, 3: dequant_mx4_blob}


class RefMoe:
    def __init__(self, d, I, E, k, n_layers, cache_slots, I_shared=0, renormalize=True, shared_slots=False,
                 host_format=0, blob_bytes=None):
        self.d, self.I, self.E, self.k, self.L, self.S = d, I, E, k, n_layers, cache_slots
        self.I_shared, self.renormalize, self.shared_slots, self.fmt = I_shared, renormalize, shared_slots, host_format
        self.blob_bytes = blob_bytes if blob_bytes is not None else 6 * d * I
        self.layers = [None] * n_layers
        self.shared_cache = SharedCacheSim(n_layers, E, cache_slots, self.blob_bytes) if shared_slots else None
        self.caches = [None] * n_layers
        self.calls = [0] * n_layers

    # ---- moe_bind_layer: host_expert_blob[E], router_w [E, d], shared blob or None, initial_resident [S] or None
    def moe_bind_layer(self, layer, host_expert_blob, router_w, shared_blob=None, initial_resident=None):
        blobs = list(host_expert_blob)
        if self.fmt:
            blobs = [_EXPAND[self.fmt](b, self.d, self.I) for b in blobs]
        self.layers[layer] = dict(blobs=blobs, router=router_w, shared=shared_blob)
        if not self.shared_slots:
            self.caches[layer] = CacheSim(self.E, self.S, self.blob_bytes, initial_resident)

    def expert_cache_prefetch(self, layer, host_ids):
        if self.shared_slots:
            self.shared_cache.prefetch(layer, host_ids)
        else:
            self.caches[layer].prefetch(host_ids)

    def predictor_score(self, layer, x, T, wp, m):
        assert wp.shape[0] == self.E and x.shape[0] == T
        return _predictor_score(x, wp, m)

    def _layer(self, layer, x, T, route_bias, bias_stride):
        L = self.layers[layer]
        bias = route_bias
        if bias is not None:
            bias = np.asarray(bias, dtype=np.float32)
            bias = bias.reshape(T, self.E) if bias_stride else bias.reshape(self.E)
        r = moe_layer(x, L["router"], L["blobs"], self.k, bias=bias, renormalize=self.renormalize,
                      shared_blob=L["shared"], I=self.I, I_shared=self.I_shared)
        before = self.moe_get_stats(layer)
        active = np.nonzero(r["counts"])[0].tolist()
        if self.shared_slots:
            self.shared_cache.serve(layer, active)
        else:
            self.caches[layer].serve(active)
        self.calls[layer] += 1
        after = self.moe_get_stats(layer)
        r["call_stats"] = {key: after[key] - before[key] for key in after}
        return r

    def moe_prefill_layer(self, layer, x, T, route_bias=None, bias_stride=0):
        return self._layer(layer, x, T, route_bias, bias_stride)

    def moe_decode_layer(self, layer, x, T, route_bias=None, bias_stride=0):
        return self._layer(layer, x, T, route_bias, bias_stride)

    def moe_get_stats(self, layer):
        c = self.shared_cache.counters(layer) if self.shared_slots else self.caches[layer].counters()
        c["layer_calls"] = self.calls[layer]
        return c

    def moe_cache_state(self, layer):
        if self.shared_slots:
            return list(self.shared_cache.state(layer))
        return list(self.caches[layer].slot_expert)
