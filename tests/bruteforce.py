"""Dense brute-force statement of the MoE layer in numpy float64, used to pin the oracle.

Written independently of oracle/moe_oracle.c: every expert is evaluated on every token with
library matmuls, experts are chosen by one full lexicographic sort, and the result is masked.
There is no grouping, no permutation and no per-row loop here.
"""
import numpy as np


def select(logits, K):
    """Top-K by a full sort on (-logit, expert id): descending logit, ties to the lower id."""
    T, E = logits.shape
    eid = np.broadcast_to(np.arange(E), (T, E))
    order = np.lexsort((eid, -logits.astype(np.float64)), axis=1)
    return order[:, :K].astype(np.int32)


def gate_weights(logits, ids, renorm):
    l = logits.astype(np.float64)
    z = np.exp(l - l.max(axis=1, keepdims=True))
    p = z / z.sum(axis=1, keepdims=True)
    w = np.take_along_axis(p, ids.astype(np.int64), axis=1)
    if renorm:
        w = w / w.sum(axis=1, keepdims=True)
    return w


def swiglu_ffn(v, Wg, Wu, Wd):
    """v [T,H]; Wg,Wu [I,H]; Wd [H,I] -> [T,H] in float64."""
    v, Wg, Wu, Wd = (a.astype(np.float64) for a in (v, Wg, Wu, Wd))
    g = v @ Wg.T
    u = v @ Wu.T
    return ((g / (1.0 + np.exp(-g))) * u) @ Wd.T


def dense_layer(x, Wr, bias, Wg, Wu, Wd, shared, K, renorm, logits=None):
    """Returns (out [T,H] f64, ids [T,K], w [T,K] f64).  `logits` overrides the float64 router
    product (pass the fp32 logits whose selection is to be reproduced)."""
    x64 = x.astype(np.float64)
    T, H = x.shape
    E = Wr.shape[0]
    if logits is None:
        logits = x64 @ Wr.astype(np.float64).T
        if bias is not None:
            logits = logits + bias.astype(np.float64)
    ids = select(logits, K)
    w = gate_weights(logits, ids, renorm)
    full = np.zeros((T, E))
    np.put_along_axis(full, ids.astype(np.int64), w, axis=1)
    out = np.zeros((T, H))
    for e in range(E):                      # every expert on every token, then masked
        out += full[:, e:e + 1] * swiglu_ffn(x, Wg[e], Wu[e], Wd[e])
    if shared is not None:
        Wsg, Wsu, Wsd, wgate = shared
        gate = 1.0 / (1.0 + np.exp(-(x64 @ wgate.astype(np.float64))))
        out += gate[:, None] * swiglu_ffn(x, Wsg, Wsu, Wsd)
    return out, ids, w
