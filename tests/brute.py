"""Independent numpy fp64 brute force of the decode-step path, for tiny shapes.

Written separately from the C oracle (different language, library routines
instead of loops: einsum, argsort, a dense softmax) so that a mistake in either
shows up as a disagreement.  Inputs are fp64 value arrays.
"""
import numpy as np


def scores(q, K_lr, A):
    """Token importance s[b,k,n]: Eq. (1) low-rank logits summed over the query
    heads that share KV head k."""
    B, Hq, d = q.shape
    Hk = A.shape[0]
    qpk = Hq // Hk
    qg = q.reshape(B, Hk, qpk, d)
    q_lr = np.einsum("bkhd,kdr->bkhr", qg, A)
    return np.einsum("bkhr,bknr->bkn", q_lr, K_lr)


def group_scores(s, G, mean=False):
    B, Hk, N = s.shape
    g = s.reshape(B, Hk, N // G, G)
    return g.mean(-1) if mean else g.max(-1)


def topk_groups(gs, M):
    """M largest per row, ties to the lower index, returned ascending."""
    order = np.argsort(-gs, axis=-1, kind="stable")[..., :M]
    return np.sort(order, axis=-1).astype(np.int32)


def attention_over_tokens(q, K, V, tokens_per_kv, scale=None):
    """tokens_per_kv[b][k] is a 1-D integer array of token positions."""
    B, Hq, d = q.shape
    Hk = K.shape[1]
    qpk = Hq // Hk
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    out = np.zeros((B, Hq, d))
    for b in range(B):
        for h in range(Hq):
            k = h // qpk
            t = np.asarray(tokens_per_kv[b][k])
            z = scale * (K[b, k, t] @ q[b, h])
            w = np.exp(z - z.max())
            w /= w.sum()
            out[b, h] = w @ V[b, k, t]
    return out


def sparse_attention(q, K, V, idx, G, scale=None):
    B, Hk, _ = idx.shape
    toks = [[(idx[b, k][:, None] * G + np.arange(G)[None, :]).ravel() for k in range(Hk)]
            for b in range(B)]
    return attention_over_tokens(q, K, V, toks, scale)


def dense_attention(q, K, V, scale=None):
    B, Hk, N, _ = K.shape
    toks = [[np.arange(N) for _ in range(Hk)] for _ in range(B)]
    return attention_over_tokens(q, K, V, toks, scale)


# ---- joint-head design: one adapter over the flattened keys, one selection per sequence ----
def flatten_keys(K):
    """[B,H_kv,N,d] -> [B,N,H_kv*d], head-major inside a row (Flatten(K) of Sec. 3.2)."""
    B, Hk, N, d = K.shape
    return np.transpose(K, (0, 2, 1, 3)).reshape(B, N, Hk * d)


def joint_metadata(K, A):
    """K_lr = Flatten(K) . A with A given as [H_kv,d,r] (= [(H_kv d), r] row-major)."""
    Hk, d, r = A.shape
    return flatten_keys(K) @ A.reshape(Hk * d, r)


def joint_scores(q, K_lr, A):
    """s[b,n] = sum over ALL query heads of (q_h . A_{g(h)}) . K_lr[b,n]  (Eq. 1)."""
    B, Hq, d = q.shape
    Hk = A.shape[0]
    qpk = Hq // Hk
    A_of_head = np.repeat(A, qpk, axis=0)                  # [Hq,d,r]: block of each head's KV head
    q_lr = np.einsum("bhd,hdr->bhr", q, A_of_head)
    return np.einsum("bhr,bnr->bn", q_lr, K_lr)
