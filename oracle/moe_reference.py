"""fp64 numpy oracle for one MoE layer: expert outputs, subset enumeration, skipping.

TEST INFRASTRUCTURE ONLY -- see the package docstring.  Every function states the
passage of the paper it follows.  All arithmetic is fp64 and follows the
definition directly: no Gram shortcut, no fusion, no reordering.  The only
decision taken in a lower precision is the skip predicate (`skip_decision`),
which both this oracle and the GPU kernel take in fp32 on purpose (see there).

Conventions (the paper is silent on them; they are this build's readings):
  * weights are stored "out-features x in-features", i.e. y = x @ W.T;
  * W1 is the SiLU-gated branch, W3 the linear branch, W2 the down projection;
  * the j-th selected expert e_j (footnote to Eq. 1) is found by comparing
    routing LOGITS, ties going to the lower expert index;
  * subsets of kept experts are indexed in lexicographic order of their sorted
    index tuples; bit e of a subset's mask is set iff expert e is kept;
  * the reconstruction loss returned is the SQUARED Frobenius norm of Eq. 3.
"""
from __future__ import annotations

import itertools
import math

import numpy as np


# --------------------------------------------------------------------------- #
# Sec. 3.1: the MoE layer
# --------------------------------------------------------------------------- #
def silu(a: np.ndarray) -> np.ndarray:
    """a * sigmoid(a), the gate non-linearity of the SwiGLU expert (Sec. 3.1)."""
    a = np.asarray(a, dtype=np.float64)
    return a / (1.0 + np.exp(-a))


def expert_ffn(x: np.ndarray, W1e: np.ndarray, W3e: np.ndarray, W2e: np.ndarray) -> np.ndarray:
    """One SwiGLU expert E_i(x) (Sec. 3.1): (silu(x W1^T) * (x W3^T)) W2^T.

    x [T,H]; W1e, W3e [F,H]; W2e [H,F]  ->  [T,H].
    """
    x = np.asarray(x, dtype=np.float64)
    gate = x @ np.asarray(W1e, dtype=np.float64).T
    up = x @ np.asarray(W3e, dtype=np.float64).T
    return (silu(gate) * up) @ np.asarray(W2e, dtype=np.float64).T


def expert_outputs(x, Wgate, W1, W3, W2):
    """Router logits l = x Wgate^T and the outputs of ALL experts on ALL tokens (Sec. 3.1).

    x [T,H]; Wgate [E,H]; W1, W3 [E,F,H]; W2 [E,H,F]  ->  logits [T,E], Y [E,T,H].
    """
    x = np.asarray(x, dtype=np.float64)
    logits = x @ np.asarray(Wgate, dtype=np.float64).T
    E = len(W1)
    Y = np.empty((E, x.shape[0], x.shape[1]), dtype=np.float64)
    for e in range(E):
        Y[e] = expert_ffn(x, W1[e], W3[e], W2[e])
    return logits, Y


def routing_order(logits: np.ndarray) -> np.ndarray:
    """order[t, j] = index of the j-th largest routing weight of token t (footnote to Eq. 1).

    Softmax is monotone, so the order of the weights is the order of the logits;
    equal logits are ordered by ascending expert index (stable sort).
    """
    logits = np.asarray(logits, dtype=np.float64)
    return np.argsort(-logits, axis=1, kind="stable")


def renormalised_weights(logits: np.ndarray, selected: np.ndarray) -> np.ndarray:
    """Eq. 1 for every token: w~_e = w_e / sum_{m in S} w_m for e in S, else 0.

    `selected` is a boolean [T,E] matrix marking each token's set S.  With
    w = Softmax(l) over any superset of S this equals exp(l_e - m) / sum_{j in S}
    exp(l_j - m), m = max_{j in S} l_j, which is what is evaluated here.
    """
    logits = np.asarray(logits, dtype=np.float64)
    masked = np.where(selected, logits, -np.inf)
    m = masked.max(axis=1, keepdims=True)
    ex = np.exp(masked - m)                     # exp(-inf) = 0 outside S
    return ex / ex.sum(axis=1, keepdims=True)


def _first_in_order(order: np.ndarray, allowed: np.ndarray, count: int) -> np.ndarray:
    """Boolean [T,E]: for each token the first `count` experts of its order with allowed[e]."""
    T, E = order.shape
    flags = allowed[order]                                  # [T,E], rank order
    taken = flags & (np.cumsum(flags, axis=1) <= count)     # first `count` allowed ranks
    selected = np.zeros((T, E), dtype=bool)
    np.put_along_axis(selected, order, taken, axis=1)       # back to expert positions
    return selected


def layer_output(logits: np.ndarray, Y: np.ndarray, k: int) -> np.ndarray:
    """Eq. 2: z_t = sum_{j<k} w~_{e_j} E_{e_j}(x_t), from the logits and the expert outputs."""
    Y = np.asarray(Y, dtype=np.float64)
    E = Y.shape[0]
    order = routing_order(logits)
    sel = _first_in_order(order, np.ones(E, dtype=bool), min(k, E))
    a = renormalised_weights(logits, sel)
    return np.einsum("te,eth->th", a, Y)


# --------------------------------------------------------------------------- #
# Sec. 3.2: enumeration of kept-expert subsets, Eq. 3
# --------------------------------------------------------------------------- #
def kept_subsets(E: int, r: int):
    """All C(E,r) kept sets C as sorted tuples, in lexicographic order; each exactly once."""
    return list(itertools.combinations(range(E), r))


def subset_mask(kept) -> int:
    m = 0
    for e in kept:
        m |= 1 << int(e)
    return m


def pruned_layer_output(logits: np.ndarray, Y: np.ndarray, kept, k: int) -> np.ndarray:
    """F'(x, C) of Sec. 3.2: the layer with only the experts in `kept`.

    The removed experts and their routing weights are gone, so each token is
    routed to its top-min(k,|C|) experts AMONG `kept` and Eq. 1 renormalises over
    those.
    """
    Y = np.asarray(Y, dtype=np.float64)
    E = Y.shape[0]
    allowed = np.zeros(E, dtype=bool)
    allowed[list(kept)] = True
    order = routing_order(logits)
    sel = _first_in_order(order, allowed, min(k, len(kept)))
    b = renormalised_weights(logits, sel)
    return np.einsum("te,eth->th", b, Y)


def prune_enumerate(logits: np.ndarray, Y: np.ndarray, k: int, r: int):
    """Eq. 3 for every kept set of size r.

    logits [T,E], Y [E,T,H]  ->  loss [C(E,r)] (squared Frobenius norm of
    F'(x,C) - F(x) over all tokens), argmin (lowest index attaining the minimum),
    masks [C(E,r)] (bit e set iff expert e kept).  F(x) is recomputed from the
    same logits and Y by Eq. 2, so keeping every expert gives exactly 0.
    """
    logits = np.asarray(logits, dtype=np.float64)
    Y = np.asarray(Y, dtype=np.float64)
    E = Y.shape[0]
    if not (1 <= r <= E and 1 <= k <= E):
        raise ValueError("need 1 <= r <= E and 1 <= k <= E")
    full = layer_output(logits, Y, k)
    subsets = kept_subsets(E, r)
    loss = np.empty(len(subsets), dtype=np.float64)
    for i, kept in enumerate(subsets):
        diff = pruned_layer_output(logits, Y, kept, k) - full      # [T,H], materialised
        loss[i] = np.sum(diff * diff)
    masks = np.array([subset_mask(c) for c in subsets], dtype=np.uint32)
    return loss, int(np.argmin(loss)), masks


def prune_enumerate_gram_form(logits: np.ndarray, Y: np.ndarray, k: int, r: int):
    """Eq. 3 for every kept set of size r, evaluated in fp64 through the per-token Gram matrix.

    A SECOND oracle, for sizes the direct definition above cannot reach in seconds (thousands of
    subsets over thousands of tokens): with a = Eq. 1 weights of the full layer, b = those of the
    layer pruned to C and d = b - a, F'(x_t, C) - F(x_t) = sum_e d_e E_e(x_t), hence its squared
    norm is d^T G_t d with G_t = Y_t Y_t^T.  The same real number as `prune_enumerate`, never the
    primary reference: a test pins it to `prune_enumerate` on small inputs, and results checked
    against it are labelled as such.  d is formed explicitly (expanding the quadratic form in a
    and b separately would cancel), and a token whose selection is unchanged contributes 0 exactly.

    Returns loss [C(E,r)], argmin, masks like `prune_enumerate`.
    """
    logits = np.asarray(logits, dtype=np.float64)
    Y = np.asarray(Y, dtype=np.float64)
    E, T, _ = Y.shape
    if not (1 <= r <= E and 1 <= k <= E):
        raise ValueError("need 1 <= r <= E and 1 <= k <= E")
    G = np.einsum("eth,fth->tef", Y, Y)                          # [T,E,E]
    order = routing_order(logits)
    sel_full = _first_in_order(order, np.ones(E, dtype=bool), min(k, E))
    a = renormalised_weights(logits, sel_full)
    subsets = kept_subsets(E, r)
    loss = np.empty(len(subsets), dtype=np.float64)
    for i, kept in enumerate(subsets):
        allowed = np.zeros(E, dtype=bool)
        allowed[list(kept)] = True
        sel = _first_in_order(order, allowed, min(k, r))
        d = renormalised_weights(logits, sel) - a
        d[np.all(sel == sel_full, axis=1)] = 0.0                  # unchanged routing: exactly nothing
        loss[i] = np.einsum("te,tef,tf->", d, G, d)
    masks = np.array([subset_mask(c) for c in subsets], dtype=np.uint32)
    return loss, int(np.argmin(loss)), masks


def prune_enumerate_streamed(logits, Y, k: int, r: int, chunk: int = 8192, to_f64=None):
    """`prune_enumerate` over token chunks, summed: Eq. 3 is a sum over tokens.

    For inputs whose fp64 copy does not fit in host memory.  `Y` may be any
    object sliceable as Y[:, t0:t1, :]; `to_f64` turns such a slice (and a slice
    of `logits`) into an fp64 numpy array.
    """
    if to_f64 is None:
        to_f64 = lambda a: np.asarray(a, dtype=np.float64)  # noqa: E731
    T = logits.shape[0]
    total = None
    masks = None
    for t0 in range(0, T, chunk):
        t1 = min(T, t0 + chunk)
        part, _, masks = prune_enumerate(to_f64(logits[t0:t1]), to_f64(Y[:, t0:t1, :]), k, r)
        total = part if total is None else total + part
    return total, int(np.argmin(total)), masks


# --------------------------------------------------------------------------- #
# Sec. 3.3 / App. A.2: dynamic skipping, top-2
# --------------------------------------------------------------------------- #
def skip_decision(logits: np.ndarray, beta: float, kept=None):
    """Top-2 experts and the rule of Sec. 3.3: skip e1 iff w_e1 < beta * w_e0.

    With `kept` (an iterable of expert indices, at least two) the layer is the pruned
    one of Sec. 3.2 -- the other experts and their routing weights are gone -- and
    the top-2 are taken among the kept experts; Sec. 3.3 notes that skipping and
    pruning can be used together.

    w_e1 / w_e0 = exp(l_e1 - l_e0) whichever softmax the weights came from, so the
    rule is l_e1 - l_e0 < ln(beta).  This is the one place where floating point
    decides an integer, and the paper fixes no precision for it; both this oracle
    and the GPU kernel therefore take it in the kernel's precision: the fp32
    difference of the fp32 logits against the fp32 rounding of ln(beta), beta
    itself being an fp32 value.  beta = 0 never skips.

    Returns e0 [T], e1 [T], skip [T] (bool), delta [T] (fp32 l_e1 - l_e0).
    """
    l32 = np.asarray(logits, dtype=np.float32)
    order = routing_order(l32)
    t = np.arange(l32.shape[0])
    if kept is None:
        e0, e1 = order[:, 0], order[:, 1]
    else:
        allowed = np.zeros(l32.shape[1], dtype=bool)
        allowed[list(kept)] = True
        if allowed.sum() < 2:
            raise ValueError("top-2 routing needs at least two kept experts")
        flags = allowed[order]                            # rank order
        nth = np.cumsum(flags, axis=1)
        e0 = order[t, np.argmax(flags & (nth == 1), axis=1)]
        e1 = order[t, np.argmax(flags & (nth == 2), axis=1)]
    delta = (l32[t, e1] - l32[t, e0]).astype(np.float32)
    b = float(np.float32(beta))
    theta = np.float32(-np.inf) if b <= 0.0 else np.float32(math.log(b))
    return e0, e1, delta < theta, delta


def forward_skip(x, Wgate, W1, W3, W2, beta: float, logits=None, kept=None):
    """The MoE forward with dynamic skipping, k = 2 (Sec. 3.3; output per App. A.2).

    Tokens that skip keep only e0 and renormalise over the survivors, i.e.
    out = E_{e0}(x); the others get Eq. 2.  Only the routed (token, expert) pairs
    are pushed through an expert.  If `logits` is given it replaces x Wgate^T
    (so that the decision can be checked on the very logits another
    implementation produced).  `kept` restricts the layer to a kept set of experts
    (the pruned layer F'(x, C) of Sec. 3.2, here with k = 2).

    Returns out [T,H], skip [T] bool, e0 [T], e1 [T].
    """
    x = np.asarray(x, dtype=np.float64)
    if logits is None:
        logits = x @ np.asarray(Wgate, dtype=np.float64).T
    e0, e1, skip, _ = skip_decision(logits, beta, kept)
    l64 = np.asarray(logits, dtype=np.float64)
    t = np.arange(x.shape[0])
    rho = np.exp(l64[t, e1] - l64[t, e0])                 # w_e1 / w_e0
    a0 = np.where(skip, 1.0, 1.0 / (1.0 + rho))
    a1 = np.where(skip, 0.0, rho / (1.0 + rho))
    out = np.zeros_like(x)
    for e in range(len(W1)):
        first = np.nonzero(e0 == e)[0]
        second = np.nonzero((e1 == e) & ~skip)[0]
        if len(first):
            out[first] += a0[first, None] * expert_ffn(x[first], W1[e], W3[e], W2[e])
        if len(second):
            out[second] += a1[second, None] * expert_ffn(x[second], W1[e], W3[e], W2[e])
    return out, skip, e0, e1


def median_skip_ratio(logits, kept=None) -> float:
    """beta of Sec. 3.3 / App. A.7: the median over tokens of w_e1 / w_e0.

    For an even token count the mean of the two middle order statistics.  With
    `kept`, e0 and e1 are the top-2 among the kept experts (the pruned layer).
    """
    l64 = np.asarray(logits, dtype=np.float64)
    if kept is not None:
        allowed = np.zeros(l64.shape[1], dtype=bool)
        allowed[list(kept)] = True
        l64 = np.where(allowed[None, :], l64, -np.inf)
    order = routing_order(l64)
    t = np.arange(l64.shape[0])
    rho = np.exp(l64[t, order[:, 1]] - l64[t, order[:, 0]])
    return float(np.median(rho))


def skip_topk_decision(logits: np.ndarray, k: int, beta: float, kept=None):
    """Generalised dynamic skipping for top-k routing (appendix on the theory of skipping).

    Per token, with w_1 >= ... >= w_k the weights of its top-k experts (among `kept`
    if given; ties to the lower index), keep the top-i* experts where
        i* = min { i in 1..k : sum_{m>i} w_m <= beta * sum_{m<=k} w_m }.
    Any common factor of the weights cancels, so w_m = exp(l_m - l_1) is used.  The
    paper fixes no precision for this decision; it is taken in fp64 on the fp32
    logits, the tail sums accumulated from the smallest weight upwards, and the GPU
    kernel does the same.

    Returns experts [T,k] (descending weight), i_star [T], w [T,k] fp64 (un-normalised).
    """
    l32 = np.asarray(logits, dtype=np.float32)
    T, E = l32.shape
    l64 = l32.astype(np.float64)
    if kept is not None:
        allowed = np.zeros(E, dtype=bool)
        allowed[list(kept)] = True
        if allowed.sum() < k:
            raise ValueError("top-k routing needs at least k kept experts")
        l64 = np.where(allowed[None, :], l64, -np.inf)
    experts = routing_order(l64)[:, :k]
    b = float(np.float32(beta))
    i_star = np.zeros(T, dtype=np.int64)
    w = np.zeros((T, k), dtype=np.float64)
    for t in range(T):
        lt = l64[t, experts[t]]
        wt = np.exp(lt - lt[0])
        tail = np.zeros(k + 1)                       # tail[i] = sum_{m>i} w_m, 1-based m
        for i in range(k - 1, -1, -1):
            tail[i] = tail[i + 1] + wt[i]
        total = tail[0]
        i = 1
        while tail[i] > b * total:                   # tail[k] = 0 always passes
            i += 1
        i_star[t] = i
        w[t] = wt
    return experts, i_star, w


def forward_skip_topk(x, Wgate, W1, W3, W2, k: int, beta: float, logits=None, kept=None):
    """MoE forward with the generalised skipping rule: each token's output is Eq. 2 over
    its top-i* experts, weights renormalised over those i* (the reduced output of the
    theory appendix).  Only routed (token, expert) pairs go through an expert.

    Returns out [T,H], i_star [T], experts [T,k].
    """
    x = np.asarray(x, dtype=np.float64)
    if logits is None:
        logits = x @ np.asarray(Wgate, dtype=np.float64).T
    experts, i_star, _ = skip_topk_decision(logits, k, beta, kept)
    out = np.zeros_like(x)
    T = x.shape[0]
    lsel = np.take_along_axis(np.asarray(logits, dtype=np.float64), experts, axis=1)
    w = np.exp(lsel - lsel[:, :1])                 # the decision is in fp32 logits, the weights are not
    used = np.arange(k)[None, :] < i_star[:, None]                 # [T,k]
    coef = np.where(used, w, 0.0)
    coef = coef / coef.sum(axis=1, keepdims=True)
    for e in range(len(W1)):
        for m in range(k):
            rows = np.nonzero((experts[:, m] == e) & used[:, m])[0]
            if len(rows):
                out[rows] += coef[rows, m][:, None] * expert_ffn(x[rows], W1[e], W3[e], W2[e])
    return out, i_star, experts


def expert_selection_stats(logits: np.ndarray, k: int):
    """Selection statistics over a calibration set (baselines of Sec. 4.1; appendix on expert
    selection tendency): count[e] = number of tokens whose top-k contains expert e, and
    co[i, j] = number of tokens whose top-k contains both i and j (so co[e, e] = count[e]).
    Top-k as everywhere else: larger logit first, ties to the lower index.
    """
    order = routing_order(np.asarray(logits))
    T, E = order.shape
    count = np.zeros(E, dtype=np.int64)
    co = np.zeros((E, E), dtype=np.int64)
    for t in range(T):
        chosen = order[t, :k]
        for i in chosen:
            count[i] += 1
            for j in chosen:
                co[i, j] += 1
    return count, co


def frequency_kept(count: np.ndarray, r: int):
    """The activation-frequency baseline of Sec. 4.1: discard the experts selected least often,
    i.e. keep the r most frequently selected.  The paper does not say what happens on equal
    counts; the lower index is kept.  Returns the kept experts as a sorted tuple.
    """
    E = len(count)
    ranked = sorted(range(E), key=lambda e: (-int(count[e]), e))
    return tuple(sorted(ranked[:r]))
