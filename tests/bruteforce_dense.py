"""Dense-graph restatement of the method in numpy, used only to pin the oracle.

Independent of oracle/: it builds the full P x P cosine matrix (every node pair,
not only source rows), takes neighbourhoods and sources with a stable argsort
and applies Eq. 5 literally, set by set.  Only usable for tiny P.
"""
import numpy as np
from scipy.special import softmax


def stable_topk(x, k):
    """First k of the order (value descending, index ascending)."""
    order = np.argsort(-np.asarray(x, dtype=np.float64), kind="stable")
    return [int(i) for i in order[:k]]


def dense_cosine(K, other=None):
    """Eq. 1 for every pair: E[i, j] = cos(K[i], other[j]); other = K if not given."""
    K = np.asarray(K, dtype=np.float64)
    other = K if other is None else np.asarray(other, dtype=np.float64)
    na = np.sqrt((K * K).sum(axis=1))
    nb = np.sqrt((other * other).sum(axis=1))
    E = np.zeros((K.shape[0], other.shape[0]))
    for i in range(K.shape[0]):
        for j in range(other.shape[0]):
            if na[i] > 0 and nb[j] > 0:
                E[i, j] = float(K[i] @ other[j]) / (na[i] * nb[j])
    return E


def propagate_dense(K, s, S, m, T, alpha=1.0, reselect=1, signal=0, other=None):
    """K [P,d] float64 (prefix keys of one head), s [P].  Returns s^(T).  With `other`
    [P,d] the edge from source i to node j is cos(K[i], other[j])."""
    s = np.array(s, dtype=np.float64)
    P = s.size
    E = dense_cosine(K, other)
    nbrs = None
    for t in range(T):
        if t == 0 or reselect:
            sources = sorted(stable_topk(s, S))                       # Eq. 2
            nbrs = {}
            for i in sources:
                others = [j for j in range(P) if j != i]              # Eq. 3: j != i
                order = stable_topk([E[i, j] for j in others], m)
                nbrs[i] = {others[o] for o in order}
        new = s.copy()
        for j in range(P):
            hit = [i for i in sorted(nbrs) if j in nbrs[i]]
            if not hit:
                continue
            if signal == 2:
                new[j] = -np.inf
                continue
            # Eq. 4, one source after the other: the change is alpha * e_ij times the size of the
            # score, taken away by the decay signal and added by the enhanced one.  For a score
            # that is not negative this is Eq. 5's product of (1 - alpha e_ij).
            v = s[j]
            for i in hit:
                step = alpha * E[i, j] * abs(v)
                v = v + step if signal == 1 else v - step
            new[j] = v
        s = new
    return s


def score_dense(K, Q, window, pool_kernel, pool_mode=0, scale=None):
    """K [N,d], Q [G,w,d] float64 for one KV head.  Library softmax, explicit mask."""
    N, d = K.shape
    G, w, _ = Q.shape
    P = N - window
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    total = np.zeros(P)
    half = (pool_kernel - 1) // 2
    for g in range(G):
        logits = (Q[g] @ K.T) * scale                                  # [w, N]
        mask = np.arange(N)[None, :] > (P + np.arange(w))[:, None]
        logits = np.where(mask, -np.inf, logits)
        p = softmax(logits, axis=1)
        vote = p[:, :P].sum(axis=0)
        pad = np.full(half, 0.0 if pool_mode == 0 else -np.inf)
        ext = np.concatenate([pad, vote, pad])
        win = np.lib.stride_tricks.sliding_window_view(ext, pool_kernel)
        pooled = win.sum(axis=1) / pool_kernel if pool_mode == 0 else win.max(axis=1)
        total += pooled
    return total / G
