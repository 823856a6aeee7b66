"""Independent checkers the oracle is pinned against.  None of them imports oracle code.

* all_paths_best: exhaustive enumeration of every path of a micro graph (fp64).
* trellis_viterbi: dense fp64 dynamic programme over the (T+1) x S trellis with
  Bellman-Ford relaxation of epsilon arcs.
* greedy_ctc: argmax per frame, collapse repeats, drop blanks.
* resum_path: cost of a given arc sequence, fp32 in the decoder's association and fp64.
* all_paths: every path of a micro graph as its arc sequence (for the lattice pins).
* trellis_alphas: the fp64 trellis of every frame (for the lattice-beam rule).
"""
from __future__ import annotations

import numpy as np


def all_paths_best(g, ll, use_final=True):
    """Returns (best_cost, set of word tuples achieving it within 1e-9, reached_final).
    Enumerates every path that consumes exactly len(ll) frames from the start state,
    including epsilon arcs anywhere (the epsilon sub-graph is acyclic)."""
    T = ll.shape[0]
    fin = g.final_cost.astype(np.float64)
    ends = []      # (cost_without_final, state, words)

    def rec(s, t, cost, words):
        if t == T:
            ends.append((cost, s, words))
        for a in g.arcs_of(s):
            il, ol = int(g.ilabel[a]), int(g.olabel[a])
            w = float(g.weight[a])
            nw = words + ((ol,) if ol != 0 else ())
            if il == 0:
                rec(int(g.next_state[a]), t, cost + w, nw)
            elif t < T:
                rec(int(g.next_state[a]), t + 1, cost + w - float(ll[t, il - 1]), nw)

    rec(g.start_state, 0, 0.0, ())
    with_final = [(c + fin[s], wd) for (c, s, wd) in ends if np.isfinite(fin[s])] if use_final else []
    if with_final:
        best = min(c for c, _ in with_final)
        return best, {wd for c, wd in with_final if c <= best + 1e-9}, True
    if not ends:
        return np.inf, set(), False
    best = min(c for c, _, _ in ends)
    return best, {wd for c, _, wd in ends if c <= best + 1e-9}, False


def _split(g):
    src = g.src_of_arcs()
    e = np.nonzero(g.ilabel != 0)[0]
    x = np.nonzero(g.ilabel == 0)[0]
    return src, e, x


def trellis_viterbi(g, ll):
    """alpha[t][s] = least cost (fp64) of reaching s having consumed t frames.
    Returns (alpha_T, best_cost_with_final_or_raw, reached_final)."""
    src, e, x = _split(g)
    S, T = g.num_states, ll.shape[0]
    w = g.weight.astype(np.float64)

    def relax_eps(alpha):
        for _ in range(S + 1):
            cand = alpha[src[x]] + w[x]
            new = alpha.copy()
            np.minimum.at(new, g.next_state[x], cand)
            if np.array_equal(new, alpha):
                return alpha
            alpha = new
        raise RuntimeError("epsilon relaxation did not converge")

    alpha = np.full(S, np.inf)
    alpha[g.start_state] = 0.0
    alpha = relax_eps(alpha)
    for t in range(T):
        cand = alpha[src[e]] + w[e] - ll[t].astype(np.float64)[g.ilabel[e] - 1]
        new = np.full(S, np.inf)
        np.minimum.at(new, g.next_state[e], cand)
        alpha = relax_eps(new)
    f = alpha + g.final_cost.astype(np.float64)
    if np.isfinite(f).any():
        return alpha, float(f.min()), True
    return alpha, float(alpha.min()), False


def greedy_ctc(ll):
    """(words, cost) of greedy decoding: classes are 0=blank, k>=1 tokens; the cost is the
    fp32 running sum, frame by frame, of -max log-likelihood."""
    best = ll.argmax(axis=1)
    words, prev = [], 0
    for k in best:
        if k != 0 and k != prev:
            words.append(int(k))
        prev = int(k)
    c = np.float32(0.0)
    for t in range(ll.shape[0]):
        c = np.float32(np.float32(c + np.float32(0.0)) + np.float32(-ll[t, best[t]]))
    return np.array(words, dtype=np.int32), float(c)


def resum_path(g, ll, orig_arcs):
    """Follow arcs (indices into g's arrays) from the start state.  Returns
    (fp32 cost in the ((c + w) + -L) association, fp64 cost, end state, frames used, words);
    raises if the arcs do not chain."""
    s, t = g.start_state, 0
    c32, c64 = np.float32(0.0), 0.0
    words = []
    for a in orig_arcs:
        a = int(a)
        lo, hi = int(g.row_offsets[s]), int(g.row_offsets[s + 1])
        if not (lo <= a < hi):
            raise AssertionError(f"arc {a} does not leave state {s}")
        w, il = np.float32(g.weight[a]), int(g.ilabel[a])
        if il == 0:
            c32 = np.float32(c32 + w)
            c64 += float(w)
        else:
            c32 = np.float32(np.float32(c32 + w) + np.float32(-ll[t, il - 1]))
            c64 += float(w) - float(ll[t, il - 1])
            t += 1
        if g.olabel[a] != 0:
            words.append(int(g.olabel[a]))
        s = int(g.next_state[a])
    return float(c32), c64, s, t, words


def all_paths(g, ll):
    """Every path from the start state that consumes exactly len(ll) frames (epsilon arcs
    anywhere), as {tuple of arc indices: (fp64 cost without final cost, end state)}."""
    T = ll.shape[0]
    out = {}

    def rec(s, t, cost, arcs):
        if t == T:
            out[arcs] = (cost, s)
        for a in g.arcs_of(s):
            il, w = int(g.ilabel[a]), float(g.weight[a])
            if il == 0:
                rec(int(g.next_state[a]), t, cost + w, arcs + (a,))
            elif t < T:
                rec(int(g.next_state[a]), t + 1, cost + w - float(ll[t, il - 1]), arcs + (a,))

    rec(g.start_state, 0, 0.0, ())
    return out


def trellis_alphas(g, ll):
    """[T+1][S] fp64: least cost of reaching each state having consumed t frames (dense
    dynamic programme, epsilon arcs relaxed to the fixpoint)."""
    src, e, x = _split(g)
    S, T = g.num_states, ll.shape[0]
    w = g.weight.astype(np.float64)

    def relax_eps(alpha):
        for _ in range(S + 1):
            new = alpha.copy()
            np.minimum.at(new, g.next_state[x], alpha[src[x]] + w[x])
            if np.array_equal(new, alpha):
                return alpha
            alpha = new
        raise RuntimeError("epsilon relaxation did not converge")

    alphas = np.full((T + 1, S), np.inf)
    alphas[0, g.start_state] = 0.0
    alphas[0] = relax_eps(alphas[0])
    for t in range(T):
        new = np.full(S, np.inf)
        np.minimum.at(new, g.next_state[e], alphas[t][src[e]] + w[e] - ll[t].astype(np.float64)[g.ilabel[e] - 1])
        alphas[t + 1] = relax_eps(new)
    return alphas
