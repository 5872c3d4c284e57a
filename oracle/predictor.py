"""Preprocessing statistics and the predictor's input (Sections IV-A, IV-B).

TEST INFRASTRUCTURE ONLY.  Plain definitions:

  popularity (Eq. 2)   P[l, i] = (# episodes whose selection at layer l contains expert i)
                                 / (total # of selections at layer l)
  affinity (Eq. 3)     A[l, i, j] = (# episodes with i selected at layer l and j at layer l + 1)
                                 / (the same count summed over j); a row of an expert that is never
                                 selected at layer l is all zero
  state vector (Eq. 4-5)  s_l = [h_l, p_l, a_{l-1,l}] as one fp32 vector of fixed length:
      h_l        the expert indices selected at layers 0 .. l-1 in the order the gate emitted them,
                 flattened, each index i stored as (i + 1) / M, zero-padded to L * k entries
      p_l        the popularity row P[l, :]
      a_{l-1,l}  for each of the k experts selected at layer l - 1, its affinity row A[l-1, i, :]
                 (k * M entries); zeros for l = 0

The paper fixes none of the encodings (Eq. 4-5 only say that the index history is flattened and
padded with zeros to a fixed length); the choices above are this build's reading.  An episode is one token's pass through all layers.
"""
from __future__ import annotations

import numpy as np


def popularity(trace: np.ndarray, M: int) -> np.ndarray:
    """trace [N, L, k] expert ids -> P [L, M] float64, rows sum to 1."""
    N, L, k = trace.shape
    P = np.zeros((L, M), dtype=np.float64)
    for n in range(N):
        for l in range(L):
            for i in set(int(e) for e in trace[n, l]):
                P[l, i] += 1.0
    tot = P.sum(axis=1, keepdims=True)
    return np.divide(P, tot, out=np.zeros_like(P), where=tot > 0)


def affinity(trace: np.ndarray, M: int) -> np.ndarray:
    """trace [N, L, k] -> A [L-1, M, M] float64; row i of A[l] sums to 1 if i was ever selected at l."""
    N, L, k = trace.shape
    A = np.zeros((max(L - 1, 0), M, M), dtype=np.float64)
    for n in range(N):
        for l in range(L - 1):
            here = set(int(e) for e in trace[n, l])
            nxt = set(int(e) for e in trace[n, l + 1])
            for i in here:
                for j in nxt:
                    A[l, i, j] += 1.0
    tot = A.sum(axis=2, keepdims=True)
    return np.divide(A, tot, out=np.zeros_like(A), where=tot > 0)


def state_dim(L: int, M: int, k: int) -> int:
    return L * k + M + k * M


def state_vector(history, layer: int, P: np.ndarray, A: np.ndarray, k: int) -> np.ndarray:
    """history[j] = the k ids selected at layer j (j < layer), gate order.  Returns s_layer fp32."""
    L, M = P.shape
    s = np.zeros(state_dim(L, M, k), dtype=np.float32)
    for j in range(layer):
        for q in range(k):
            s[j * k + q] = np.float32((int(history[j][q]) + 1) / M)
    s[L * k:L * k + M] = P[layer].astype(np.float32)
    if layer > 0:
        for q in range(k):
            i = int(history[layer - 1][q])
            s[L * k + M + q * M:L * k + M + (q + 1) * M] = A[layer - 1, i].astype(np.float32)
    return s
