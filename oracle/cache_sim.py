"""Reference simulator of the GPU expert cache's bookkeeping (integers only).

TEST INFRASTRUCTURE ONLY.  The paper keeps every expert in a CPU expert cache and a
few in a GPU expert cache that is filled just before use (Section V-A); experts are
prefetched ahead of the layer (Sections V-B, V-C) and, when the gate's choice is
not in the cache, the right ones are fetched again (Section V-C).  The paper gives
no replacement rule; the rule simulated here is the reading this build takes:

  K1  An expert is resident iff one of the layer's S slots holds it (a copy still in
      flight counts: the compute stream waits for it).
  K2  Victim for a new expert: the lowest-numbered empty slot; else, among slots whose
      expert is not protected, the one used least recently (ties: lowest slot).
      No candidate: the request for that expert is dropped.
  K3  Use order is a per-layer counter; a slot is stamped when its expert is served,
      placed, or named again by a prefetch request.
  K4  Counters: hits / misses per served active expert, copies issued by prefetch,
      prefetched copies that were later served before eviction, bytes copied.

prefetch(ids): protected = the ids of the request.  For each id in order (repeats
skipped): resident -> stamp; else pick a victim, copy, stamp, mark "prefetched".

serve(active): active experts ascending.  Resident ones are hits (stamped in ascending
id, computed first); the others are misses and stream through victims chosen with an
empty protected set, in ascending id, each stamped when placed.
"""
from __future__ import annotations


class CacheSim:
    def __init__(self, E: int, S: int, blob_bytes: int, initial=None):
        assert S >= 1 and E >= 1
        self.E, self.S, self.blob_bytes = E, S, blob_bytes
        self.slot_expert = [-1] * S
        self.stamp = [0] * S
        self.prefetched = [False] * S
        self.clock = 0
        self.hits = self.misses = 0
        self.prefetch_issued = self.prefetch_useful = self.prefetch_dropped = 0
        self.bytes_h2d = 0
        self.copies = []  # (expert, slot) in issue order
        if initial is not None:
            for s, e in enumerate(initial):
                if e >= 0:
                    self.slot_expert[s] = int(e)

    def slot_of(self, e: int) -> int:
        return self.slot_expert.index(e) if e in self.slot_expert else -1

    def _touch(self, s: int) -> None:
        self.clock += 1
        self.stamp[s] = self.clock

    def _victim(self, protected) -> int:
        for s in range(self.S):
            if self.slot_expert[s] < 0:
                return s
        best = -1
        for s in range(self.S):
            if self.slot_expert[s] in protected:
                continue
            if best < 0 or self.stamp[s] < self.stamp[best]:
                best = s
        return best

    def _place(self, e: int, s: int, prefetched: bool) -> None:
        self.slot_expert[s] = e
        self.prefetched[s] = prefetched
        self._touch(s)
        self.bytes_h2d += self.blob_bytes
        self.copies.append((e, s))

    def prefetch(self, ids):
        protected = set(int(i) for i in ids)
        seen = set()
        issued = []
        for e in ids:
            e = int(e)
            assert 0 <= e < self.E
            if e in seen:
                continue
            seen.add(e)
            s = self.slot_of(e)
            if s >= 0:
                self._touch(s)
                continue
            s = self._victim(protected)
            if s < 0:
                self.prefetch_dropped += 1
                continue
            self._place(e, s, True)
            self.prefetch_issued += 1
            issued.append((e, s))
        return issued

    def serve(self, active):
        active = sorted(set(int(e) for e in active))
        hits = [e for e in active if self.slot_of(e) >= 0]
        misses = [e for e in active if self.slot_of(e) < 0]
        for e in hits:
            s = self.slot_of(e)
            self._touch(s)
            if self.prefetched[s]:
                self.prefetch_useful += 1
                self.prefetched[s] = False
        self.hits += len(hits)
        self.misses += len(misses)
        fetched = []
        for e in misses:
            s = self._victim(())
            self._place(e, s, False)
            fetched.append((e, s))
        return hits, misses, fetched

    def counters(self):
        return dict(hits=self.hits, misses=self.misses, prefetch_issued=self.prefetch_issued,
                    prefetch_useful=self.prefetch_useful, prefetch_dropped=self.prefetch_dropped,
                    bytes_h2d=self.bytes_h2d)


class SharedCacheSim:
    """The same rules for ONE cache of S slots that serves all layers in turn (Section V-A: the GPU
    expert cache holds as many experts as a token activates and is refilled layer after layer).

    A slot holds (layer, expert).  Residency, hits and misses are per layer; the use counter and
    the victim rule K2 are the cache's: an empty slot first, else the least recently used slot whose
    content is not protected, where only experts of the layer that is asking can be protected.
    Counters are kept per layer, as the per-layer caches keep them.
    """

    def __init__(self, n_layers: int, E: int, S: int, blob_bytes: int):
        assert S >= 1 and E >= 1 and n_layers >= 1
        self.L, self.E, self.S, self.blob_bytes = n_layers, E, S, blob_bytes
        self.slot = [None] * S          # (layer, expert) or None
        self.stamp = [0] * S
        self.prefetched = [False] * S
        self.clock = 0
        self.ctr = [dict(hits=0, misses=0, prefetch_issued=0, prefetch_useful=0, prefetch_dropped=0,
                         bytes_h2d=0) for _ in range(n_layers)]
        self.copies = []                # (layer, expert, slot) in issue order

    def slot_of(self, layer: int, e: int) -> int:
        return self.slot.index((layer, e)) if (layer, e) in self.slot else -1

    def state(self, layer: int):
        return [c[1] if c is not None and c[0] == layer else -1 for c in self.slot]

    def _touch(self, s: int) -> None:
        self.clock += 1
        self.stamp[s] = self.clock

    def _victim(self, layer: int, protected) -> int:
        for s in range(self.S):
            if self.slot[s] is None:
                return s
        best = -1
        for s in range(self.S):
            if self.slot[s][0] == layer and self.slot[s][1] in protected:
                continue
            if best < 0 or self.stamp[s] < self.stamp[best]:
                best = s
        return best

    def _place(self, layer: int, e: int, s: int, prefetched: bool) -> None:
        self.slot[s] = (layer, e)
        self.prefetched[s] = prefetched
        self._touch(s)
        self.ctr[layer]["bytes_h2d"] += self.blob_bytes
        self.copies.append((layer, e, s))

    def prefetch(self, layer: int, ids):
        protected = set(int(i) for i in ids)
        seen = set()
        for e in ids:
            e = int(e)
            assert 0 <= e < self.E
            if e in seen:
                continue
            seen.add(e)
            s = self.slot_of(layer, e)
            if s >= 0:
                self._touch(s)
                continue
            s = self._victim(layer, protected)
            if s < 0:
                self.ctr[layer]["prefetch_dropped"] += 1
                continue
            self._place(layer, e, s, True)
            self.ctr[layer]["prefetch_issued"] += 1

    def serve(self, layer: int, active):
        active = sorted(set(int(e) for e in active))
        hits = [e for e in active if self.slot_of(layer, e) >= 0]
        misses = [e for e in active if self.slot_of(layer, e) < 0]
        for e in hits:
            s = self.slot_of(layer, e)
            self._touch(s)
            if self.prefetched[s]:
                self.ctr[layer]["prefetch_useful"] += 1
                self.prefetched[s] = False
        self.ctr[layer]["hits"] += len(hits)
        self.ctr[layer]["misses"] += len(misses)
        for e in misses:
            s = self._victim(layer, ())
            self._place(layer, e, s, False)
        return hits, misses

    def counters(self, layer: int):
        return dict(self.ctr[layer])
