"""Dense brute-force attention (test infrastructure only).

A second CPU implementation, independent of ppd_oracle.c: it never sees pages.  It takes the un-paged,
token-major K/V of ONE sequence, forms the whole (L+n) x (L+n) causal score matrix as a full recompute
prefill would (paper section 4.1: full prefill over the same total sequence length), applies a dense
softmax in float64 and returns the last n rows -- which is what append-prefill must reproduce.
"""
import numpy as np


def bf16_bits_to_f64(a):
    a = np.asarray(a, dtype=np.uint16)
    return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def dense_attention(q_bits, k_bits, v_bits, L, n, scale):
    """q_bits: [n, Hq, D]; k_bits, v_bits: [L+n, Hkv, D] (uint16 bf16 bits).  Returns [n, Hq, D] float64."""
    q = bf16_bits_to_f64(q_bits)
    k = bf16_bits_to_f64(k_bits)
    v = bf16_bits_to_f64(v_bits)
    n_, Hq, D = q.shape
    S, Hkv, _ = k.shape
    assert n_ == n and S == L + n
    G = Hq // Hkv
    out = np.empty((n, Hq, D), dtype=np.float64)
    # Full-sequence queries do not exist for the cached part; their rows would be discarded anyway, so the
    # square score matrix is built with the new queries placed in its last n rows and zeros above.
    causal = np.tril(np.ones((S, S), dtype=bool))
    for h in range(Hq):
        kh = k[:, h // G, :]
        vh = v[:, h // G, :]
        qfull = np.zeros((S, D))
        qfull[L:, :] = q[:, h, :]
        scores = float(np.float32(scale)) * (qfull @ kh.T)
        scores = np.where(causal, scores, -np.inf)
        scores -= scores.max(axis=1, keepdims=True)
        w = np.exp(scores)
        w /= w.sum(axis=1, keepdims=True)
        out[:, h, :] = (w @ vh)[L:, :]
    return out
