"""Second, independent oracle: the fused kernel's blockwise procedure (Alg. 1).

Test infrastructure only.  Where ``longflow_oracle.c`` writes out the plain
definitions (eq. 1, eq. 6, argmin), this module follows the *procedure* the
paper gives for its fused operator (Sec. 3.4 "Fused Attention and Eviction
Kernel", Alg. 1), in the paper's notation, for a single query head:

  * one loop over the cache in blocks of B_k rows (no loop over queries);
  * logits S_j = q K_j^T / sqrt(d), masked rows set to -inf;
  * softmax numerators P_j = exp(S_j) with NO running maximum, in wide
    floating point (float64 here), denominator l_acc += sum(P_j);
  * un-normalised contribution vectors C_j = P_j (.) V_j (row i of V_j scaled
    by P_j[i]); o_acc += column sums of C_j; s_loss rows = L1 norms of C_j;
  * after the loop: o = o_acc / l_acc, S_final_loss = S_loss / l_acc,
    i_evict = argmin(S_final_loss).

The loop bounds printed in Alg. 1 are garbled (1-based start, stride B_k, end
t-1); the reading taken is "every row of the cache, in consecutive blocks,
the last one ragged".  Results must not depend on B_k.
"""
from __future__ import annotations

import numpy as np


def fused_blockwise(q, K, V, M, B_k):
    """q [d]; K, V [T, d]; M [T] in {0,1}; returns (o [d], S_final_loss [T], i_evict)."""
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    M = np.asarray(M).astype(bool)
    T, d = K.shape
    o_acc = np.zeros(d)
    l_acc = 0.0
    S_loss = np.zeros(T)
    for j in range(0, T, B_k):
        K_j, V_j, M_j = K[j:j + B_k], V[j:j + B_k], M[j:j + B_k]
        S_j = (K_j @ q) / np.sqrt(d)
        S_j = np.where(M_j, S_j, -np.inf)
        P_j = np.exp(S_j)
        l_acc = l_acc + P_j.sum()
        # masked rows may hold anything (even NaN): their P is exactly 0 and
        # they contribute nothing, so scale only the live rows
        C_j = np.where(M_j[:, None], P_j[:, None] * np.where(M_j[:, None], V_j, 0.0), 0.0)
        o_acc = o_acc + C_j.sum(axis=0)
        S_loss[j:j + B_k] = np.abs(C_j).sum(axis=1)
    o = o_acc / l_acc
    S_final_loss = S_loss / l_acc
    i_evict = int(np.argmin(S_final_loss))
    return o, S_final_loss, i_evict


def fused_blockwise_group(q, K, V, M, B_k):
    """Group form used by this build: q [G, d]; scores summed over the G heads
    that share the KV head (the paper leaves heads out, Sec. 2.1)."""
    q = np.asarray(q, dtype=np.float64)
    outs, total = [], 0.0
    for h in range(q.shape[0]):
        o, s, _ = fused_blockwise(q[h], K, V, M, B_k)
        outs.append(o)
        total = total + s
    return np.stack(outs), total
