"""Independent restatements used to pin the CPU oracle.

Nothing here calls the oracle: these helpers compute, by brute force and with
exact or NumPy arithmetic, what the paper's definitions fix, so that the oracle
can be compared against something other than itself.
"""
import itertools
import math

import numpy as np


def markov_model(P0, Pcond):
    """Wrap an explicit first-order Markov chain as (E, U, prompt, scale).

    P0[v] = P(X_1 = v); Pcond[a][v] = P(X_{t+1} = v | X_t = a).  Adds one
    begin-of-sequence symbol (index V) that is never emitted (logit -inf) and
    whose row is P0.  With E the identity and scale = sqrt(d) the bigram logits
    are exactly log P.
    """
    P0 = np.asarray(P0, dtype=np.float64)
    Pcond = np.asarray(Pcond, dtype=np.float64)
    V = P0.shape[0]
    d = V + 1
    table = np.vstack([Pcond, P0[None, :]])             # row V = BOS
    with np.errstate(divide="ignore"):
        U = np.log(table)
    U = np.hstack([U, np.full((d, 1), -np.inf)])        # BOS column
    E = np.eye(d, dtype=np.float64)
    return E, U, V, math.sqrt(d)


def enumerate_codebook(P0, Pcond, L, eos_id=-1):
    """All padded length-L sequences in dictionary order with their intervals.

    Brute force from the definition: a sequence's probability is the product of
    its conditionals (up to and including its first EOS; afterwards it is
    padding, written as repeated EOS); sequences are sorted as tuples; the
    interval of the k-th one starts at the total probability of those before
    it.  Returns (list of tuples, starts, probs).
    """
    P0 = np.asarray(P0, dtype=np.float64)
    Pcond = np.asarray(Pcond, dtype=np.float64)
    V = P0.shape[0]
    seqs = {}
    for tup in itertools.product(range(V), repeat=L):
        prob = 1.0
        prev = None
        out = []
        done = False
        for t, v in enumerate(tup):
            if done:
                out.append(eos_id)
                continue
            prob *= P0[v] if prev is None else Pcond[prev][v]
            out.append(v)
            prev = v
            if eos_id >= 0 and v == eos_id:
                done = True
        key = tuple(out)
        if key in seqs:
            continue            # same padded sequence reached through padding positions
        seqs[key] = prob
    keys = sorted(seqs)
    probs = np.array([seqs[k] for k in keys])
    starts = np.concatenate([[0.0], np.cumsum(probs)[:-1]])
    return keys, starts, probs


def softmax64(x, temp=1.0):
    x = np.asarray(x, dtype=np.float64) / temp
    x = x - np.max(x)
    e = np.exp(x)
    return e / e.sum()


def topk_keep(x, k):
    """Boolean keep mask: the k highest logits, ties at the k-th value all kept."""
    x = np.asarray(x, dtype=np.float64)
    if k <= 0 or k >= x.shape[0]:
        return np.ones_like(x, dtype=bool)
    kth = np.sort(x)[::-1][k - 1]
    return x >= kth


def nucleus_keep(x, temp, top_p, keep=None):
    """Smallest set of highest-probability value groups whose mass reaches top_p."""
    x = np.asarray(x, dtype=np.float64)
    keep = np.ones_like(x, dtype=bool) if keep is None else keep
    if top_p <= 0 or top_p >= 1:
        return keep
    p = np.zeros_like(x)
    p[keep] = softmax64(x[keep], temp)
    vals = np.unique(x[keep])[::-1]
    cum = 0.0
    thr = vals[-1]
    for v in vals:
        cum += p[keep & (x == v)].sum()
        if cum >= top_p:
            thr = v
            break
    return keep & (x >= thr)
