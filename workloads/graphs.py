"""Seeded decoding-graph generators.

A graph is a CSR weighted transducer.  Label conventions (shared by every consumer):
ilabel 0 is epsilon (non-emitting); ilabel k >= 1 consumes log-likelihood column k-1, so
the CTC blank (column 0) is ilabel 1.  olabel 0 means "no output".  final_cost[s] = +inf
marks a non-final state.  The epsilon sub-graph of every generated graph is acyclic.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass
class Graph:
    num_states: int
    start_state: int
    num_classes: int           # V = number of log-likelihood columns
    row_offsets: np.ndarray    # int64 [S+1]
    next_state: np.ndarray     # int32 [A]
    ilabel: np.ndarray         # int32 [A]
    olabel: np.ndarray         # int32 [A]
    weight: np.ndarray         # float32 [A]
    final_cost: np.ndarray     # float32 [S]
    meta: dict | None = None

    @property
    def num_arcs(self) -> int:
        return int(self.row_offsets[-1])

    def arcs_of(self, s: int):
        lo, hi = int(self.row_offsets[s]), int(self.row_offsets[s + 1])
        return range(lo, hi)

    def src_of_arcs(self) -> np.ndarray:
        deg = np.diff(self.row_offsets)
        return np.repeat(np.arange(self.num_states, dtype=np.int32), deg)


def _from_arc_list(num_states, start, V, arcs, final_cost, meta=None) -> Graph:
    """arcs: list of (src, dst, ilabel, olabel, weight); kept in the given order per state."""
    src = np.array([a[0] for a in arcs], dtype=np.int64)
    order = np.argsort(src, kind="stable")
    deg = np.bincount(src, minlength=num_states).astype(np.int64)
    off = np.zeros(num_states + 1, dtype=np.int64)
    np.cumsum(deg, out=off[1:])
    take = lambda k, dt: np.array([arcs[i][k] for i in order], dtype=dt)
    return Graph(num_states, start, V, off, take(1, np.int32), take(2, np.int32),
                 take(3, np.int32), take(4, np.float32),
                 np.asarray(final_cost, dtype=np.float32), meta or {})


# --------------------------------------------------------------------------------------
# Config-1 style: CTC topology x lexicon x unigram(+a few bigram arcs), built directly.
# --------------------------------------------------------------------------------------
def tiny_lexicon_graph(seed: int = 1, num_words: int = 200, num_chars: int = 28,
                       min_len: int = 2, max_len: int = 8, bigram_per_end: int = 8) -> Graph:
    """Root state (start, final) with a blank self-loop; each word is a chain of char states
    C_i (self-loop on the char) and blank states B_i (blank self-loop).  The word id is
    emitted on the first arc of the word (output labels pushed to the front).  Word ends
    go back to the root over an epsilon "backoff" arc, and directly into a few seeded
    next words ("bigram" arcs).  V = num_chars + 1 classes, class 0 = blank."""
    rng = np.random.default_rng(seed)
    V = num_chars + 1
    BLANK = 1                                     # ilabel of the blank class
    rw = lambda: float(-np.log(rng.uniform(0.01, 1.0)))
    arcs = [(0, 0, BLANK, 0, 0.0)]
    words = []
    nstates = 1
    first_state, first_char, end_states = [], [], []
    for w in range(num_words):
        n = int(rng.integers(min_len, max_len + 1))
        chars = rng.integers(1, num_chars + 1, size=n)
        words.append(chars)
        C = [nstates + 2 * i for i in range(n)]
        B = [nstates + 2 * i + 1 for i in range(n)]
        nstates += 2 * n
        first_state.append(C[0])
        first_char.append(int(chars[0]))
        arcs.append((0, C[0], int(chars[0]) + 1, w + 1, rw()))
        for i in range(n):
            il = int(chars[i]) + 1
            arcs.append((C[i], C[i], il, 0, 0.0))           # repeat the char
            arcs.append((C[i], B[i], BLANK, 0, rw()))       # char -> blank
            arcs.append((B[i], B[i], BLANK, 0, 0.0))        # repeat blank
            if i + 1 < n:
                nl = int(chars[i + 1]) + 1
                if chars[i + 1] != chars[i]:
                    arcs.append((C[i], C[i + 1], nl, 0, rw()))
                arcs.append((B[i], C[i + 1], nl, 0, rw()))
        end_states.append((C[-1], B[-1], int(chars[-1])))
    for (ce, be, lastc) in end_states:
        arcs.append((ce, 0, 0, 0, rw()))                    # epsilon backoff to the root
        arcs.append((be, 0, 0, 0, rw()))
        nxt = rng.choice(num_words, size=bigram_per_end, replace=False)
        for w2 in nxt:
            il = first_char[w2] + 1
            if first_char[w2] != lastc:                     # CTC: same char needs a blank
                arcs.append((ce, first_state[w2], il, int(w2) + 1, rw()))
            arcs.append((be, first_state[w2], il, int(w2) + 1, rw()))
    final = np.full(nstates, np.inf, dtype=np.float32)
    final[0] = 0.0
    return _from_arc_list(nstates, 0, V, arcs, final,
                          {"kind": "tiny_lexicon", "seed": seed, "num_words": num_words})


# --------------------------------------------------------------------------------------
# Config-2/3 style: TLG-shaped random graph (vectorised; 10 M states in a few seconds).
# --------------------------------------------------------------------------------------
def tlg_shaped_graph(seed: int, num_states: int, target_arcs: int, num_classes: int = 129,
                     alpha: float = 1.8, k_max: int = 5000, p_eps: float = 0.15,
                     p_olabel: float = 0.2, num_words: int = 20000,
                     w_lo: float = 0.001, extra_lo: int = 0, extra_hi: int = 0) -> Graph:
    """Out-degree 1 + min(k_max, floor(x_min * u^(-1/(alpha-1)))) with x_min bisected so the
    total is ~target_arcs.  Arc 0 of every state is a blank self-loop (weight 0).  Every
    other arc is, with probability p_eps, an epsilon backoff arc to a state of strictly
    lower level (levels 0..3 seeded per state; level-0 states have none, so the epsilon
    sub-graph is a DAG), else an emitting arc with a uniform non-blank ilabel, a uniform
    destination, and an output word with probability p_olabel.  Weights -log U(w_lo, 1).
    Every state is final with cost 0; start state 0, which is given the largest degree.
    With extra_hi > 0 every state gets U{extra_lo..extra_hi} more arcs on top (a "branchy" graph
    in which no state has the self-loop alone); the power-law part then fills what is left of
    target_arcs."""
    rng = np.random.default_rng(seed)
    S, V = int(num_states), int(num_classes)
    u = rng.random(S)
    tail = u ** (-1.0 / (alpha - 1.0))
    flat = rng.integers(extra_lo, extra_hi + 1, size=S).astype(np.int64) if extra_hi > 0 else np.zeros(S, np.int64)
    want = max(0, int(target_arcs) - S - int(flat.sum()))

    def total(xm):
        return int(np.minimum(k_max, np.floor(xm * tail)).sum())
    if S * int(k_max) < want:
        raise ValueError(f"target_arcs {target_arcs} cannot be reached with {S} states of at most 1 + {k_max} arcs")
    lo, hi = 0.0, 1.0
    while total(hi) < want:
        hi *= 2.0
    for _ in range(60):
        mid = 0.5 * (lo + hi)
        if total(mid) < want:
            lo = mid
        else:
            hi = mid
    x_min = hi
    extra = np.minimum(k_max, np.floor(x_min * tail)).astype(np.int64) + flat
    hub = int(np.argmax(extra))                   # the start state is a hub, like a TLG root
    extra[0], extra[hub] = extra[hub], extra[0]
    deg = 1 + extra
    off = np.zeros(S + 1, dtype=np.int64)
    np.cumsum(deg, out=off[1:])
    A = int(off[-1])
    del u, tail

    level = rng.integers(0, 4, size=S).astype(np.int8)
    by_level = np.argsort(level, kind="stable").astype(np.int32)
    cnt_lt = np.zeros(5, dtype=np.int64)
    cnt_lt[1:] = np.cumsum(np.bincount(level, minlength=4))   # cnt_lt[L] = #states with level < L

    src = np.repeat(np.arange(S, dtype=np.int32), deg)
    is_first = np.zeros(A, dtype=bool)
    is_first[off[:-1]] = True
    src_level = level[src]
    # p_eps is the fraction of ALL arcs; only non-self-loop arcs of level>0 states qualify
    eligible = (~is_first) & (src_level > 0)
    p_arc = min(1.0, p_eps * A / max(1, int(eligible.sum())))
    is_eps = (rng.random(A) < p_arc) & eligible
    del eligible

    nxt = rng.integers(0, S, size=A, dtype=np.int64).astype(np.int32)
    # epsilon destinations: uniform among states of strictly lower level
    r = rng.random(A)
    eps_idx = np.nonzero(is_eps)[0]
    pick = np.minimum((r[eps_idx] * cnt_lt[src_level[eps_idx]]).astype(np.int64),
                      cnt_lt[src_level[eps_idx]] - 1)
    nxt[eps_idx] = by_level[pick]
    del r, pick
    nxt[is_first] = src[is_first]

    il = rng.integers(2, V + 1, size=A, dtype=np.int64).astype(np.int32)
    il[is_eps] = 0
    il[is_first] = 1
    ol = rng.integers(1, num_words + 1, size=A, dtype=np.int64).astype(np.int32)
    ol[rng.random(A) >= p_olabel] = 0
    ol[is_eps | is_first] = 0
    w = (-np.log(rng.uniform(w_lo, 1.0, size=A))).astype(np.float32)
    w[is_first] = 0.0
    final = np.zeros(S, dtype=np.float32)
    return Graph(S, 0, V, off, nxt, il, ol, w, final,
                 {"kind": "tlg_shaped", "seed": seed, "x_min": x_min, "alpha": alpha,
                  "k_max": k_max, "p_eps": p_eps, "p_olabel": p_olabel,
                  "num_words": num_words, "num_eps": int(is_eps.sum())})


# --------------------------------------------------------------------------------------
# "Normal" CTC topology T alone (Algorithm description, figure of the normal T transducer):
# blank is never output, and repeating a token on the output needs a blank in between.
# --------------------------------------------------------------------------------------
def ctc_topology_graph(num_classes: int) -> Graph:
    """States 0..V-1: 0 = start / after blank, k = after token k (class k).  Every label
    sequence is accepted; all weights 0; all states final."""
    V = num_classes
    arcs = []
    for s in range(V):
        arcs.append((s, 0, 1, 0, 0.0))                      # blank -> state 0, no output
        for k in range(1, V):
            if k == s:
                arcs.append((s, s, k + 1, 0, 0.0))          # repeat of the same token
            else:
                arcs.append((s, k, k + 1, k, 0.0))          # new token: output it
    return _from_arc_list(V, 0, V, arcs, np.zeros(V, dtype=np.float32), {"kind": "ctc_T"})


# --------------------------------------------------------------------------------------
# Micro graphs for brute-force checks: epsilon arcs, negative weights, exact ties.
# --------------------------------------------------------------------------------------
def micro_graph(seed: int, num_states: int = 6, num_classes: int = 3, max_deg: int = 4,
                p_eps: float = 0.3, p_final: float = 0.6, dyadic: bool = True,
                neg_eps: bool = True, num_words: int = 5) -> Graph:
    """Small random graph.  With dyadic=True weights are multiples of 1/4 so equal-cost
    paths (exact ties) are frequent.  Epsilon arcs only go to lower-numbered states."""
    rng = np.random.default_rng(seed)
    S, V = num_states, num_classes
    arcs = []
    for s in range(S):
        d = int(rng.integers(1, max_deg + 1))
        for _ in range(d):
            if dyadic:
                w = float(rng.integers(0, 9)) / 4.0
            else:
                w = float(-np.log(rng.uniform(0.01, 1.0)))
            ol = int(rng.integers(0, num_words + 1)) if rng.random() < 0.5 else 0
            if s > 0 and rng.random() < p_eps:
                if neg_eps and rng.random() < 0.3:
                    w = -w
                arcs.append((s, int(rng.integers(0, s)), 0, ol, w))
            else:
                arcs.append((s, int(rng.integers(0, S)), int(rng.integers(1, V + 1)), ol, w))
    final = np.where(rng.random(S) < p_final,
                     rng.integers(0, 5, size=S).astype(np.float32) / 2.0, np.inf)
    if not np.isfinite(final).any():
        final[int(rng.integers(0, S))] = 0.0
    return _from_arc_list(S, 0, V, arcs, final.astype(np.float32), {"kind": "micro", "seed": seed})


def permute_arcs_within_states(g: Graph, seed: int) -> Graph:
    """Same transducer with the arcs of each state shuffled (changes arc ids only)."""
    rng = np.random.default_rng(seed)
    A = g.num_arcs
    key = g.src_of_arcs().astype(np.float64) + rng.random(A) * 0.5
    perm = np.argsort(key, kind="stable")
    return Graph(g.num_states, g.start_state, g.num_classes, g.row_offsets.copy(),
                 g.next_state[perm], g.ilabel[perm], g.olabel[perm], g.weight[perm],
                 g.final_cost.copy(), dict(g.meta or {}, permuted=seed))


# --------------------------------------------------------------------------------------
# Stress shapes for the decoder's less common paths (not paper workloads).
# --------------------------------------------------------------------------------------
def _csr(num_states, start, V, src, dst, il, ol, w, final_cost=None, meta=None) -> Graph:
    """Arrays of arcs (any order) -> Graph; arcs of a state keep their given relative order."""
    src = np.asarray(src, dtype=np.int64)
    order = np.argsort(src, kind="stable")
    off = np.zeros(num_states + 1, dtype=np.int64)
    np.cumsum(np.bincount(src, minlength=num_states), out=off[1:])
    fc = np.zeros(num_states, dtype=np.float32) if final_cost is None else np.asarray(final_cost, np.float32)
    return Graph(num_states, start, V, off, np.asarray(dst, np.int32)[order], np.asarray(il, np.int32)[order],
                 np.asarray(ol, np.int32)[order], np.asarray(w, np.float32)[order], fc, meta or {})


def dense_graph(seed: int, num_states: int, degree: int, num_classes: int, num_words: int = 50) -> Graph:
    """Every state has `degree` emitting arcs to uniform destinations (no epsilon arcs)."""
    rng = np.random.default_rng([seed, 0xDE45E])
    A = num_states * degree
    src = np.repeat(np.arange(num_states), degree)
    dst = rng.integers(0, num_states, A)
    il = rng.integers(1, num_classes + 1, A)
    ol = np.where(rng.random(A) < 0.05, rng.integers(1, num_words + 1, A), 0)
    w = -np.log(rng.uniform(0.001, 1.0, A))
    return _csr(num_states, 0, num_classes, src, dst, il, ol, w)


def giant_state_graph(seed: int, fan: int, num_states: int, num_classes: int, num_words: int = 50) -> Graph:
    """The start state has `fan` emitting arcs; every other state has 3 (one back to the start)."""
    rng = np.random.default_rng([seed, 0x61A47])
    rest = num_states - 1
    src = np.concatenate([np.zeros(fan, np.int64), np.repeat(np.arange(1, num_states), 3)])
    dst = np.concatenate([rng.integers(1, num_states, fan),
                          np.stack([np.zeros(rest, np.int64), rng.integers(1, num_states, rest),
                                    rng.integers(1, num_states, rest)], axis=1).ravel()])
    A = len(src)
    il = rng.integers(1, num_classes + 1, A)
    ol = np.where(rng.random(A) < 0.05, rng.integers(1, num_words + 1, A), 0)
    w = -np.log(rng.uniform(0.001, 1.0, A))
    return _csr(num_states, 0, num_classes, src, dst, il, ol, w)


def eps_layers_graph(seed: int, width: int, num_classes: int, fan: int = 3, num_words: int = 50) -> Graph:
    """Start state -> `width` states over epsilon arcs -> `fan` states each of a second layer of
    `width` states over epsilon arcs (so a closure round has `width` items and `fan * width`
    arcs); every second-layer state has two emitting arcs, one of them back to the start."""
    rng = np.random.default_rng([seed, 0xE9517])
    S = 1 + 2 * width
    l1 = np.arange(1, 1 + width); l2 = np.arange(1 + width, S)
    src = [np.zeros(width, np.int64), np.repeat(l1, fan), np.repeat(l2, 2)]
    dst = [l1, rng.integers(1 + width, S, width * fan),
           np.stack([np.zeros(width, np.int64), rng.integers(1 + width, S, width)], axis=1).ravel()]
    il = [np.zeros(width, np.int64), np.zeros(width * fan, np.int64), rng.integers(1, num_classes + 1, 2 * width)]
    src, dst, il = np.concatenate(src), np.concatenate(dst), np.concatenate(il)
    A = len(src)
    ol = np.where(rng.random(A) < 0.1, rng.integers(1, num_words + 1, A), 0)
    w = -np.log(rng.uniform(0.01, 1.0, A))
    return _csr(S, 0, num_classes, src, dst, il, ol, w)


def loop_tie_graph(seed: int, num_states: int, num_classes: int, p_loop: float = 0.85, max_extra: int = 3,
                   p_eps: float = 0.1, num_words: int = 30) -> Graph:
    """Exact cost ties around self-loops.  A share p_loop of the states starts with a blank
    self-loop (ilabel 1, weight 0, no output label); the others start with some other arc or a
    self-loop of another kind (another label, a weight, an output label).  Every state has
    0..max_extra more arcs to uniform destinations, many of them with the blank label as well, with
    weights from {0, 0.5, 1} and output labels on half of them; a share p_eps of the extra arcs are
    epsilon arcs (weight 0 or 0.5) to a higher-numbered state.  With log-likelihoods that are
    multiples of 0.5 every cost is a small dyadic number, so the candidate of a self-loop and the
    candidates of arcs entering the same state tie exactly all the time."""
    rng = np.random.default_rng([seed, 0x7E100])
    S, V = int(num_states), int(num_classes)
    src, dst, il, ol, w = [], [], [], [], []
    for s in range(S):
        u = rng.random()
        if u < p_loop:
            src.append(s); dst.append(s); il.append(1); ol.append(0); w.append(0.0)
        elif u < p_loop + 0.05:                                  # a self-loop with an output label
            src.append(s); dst.append(s); il.append(1); ol.append(int(rng.integers(1, num_words + 1))); w.append(0.0)
        elif u < p_loop + 0.10:                                  # a self-loop with another label or weight
            src.append(s); dst.append(s); il.append(int(rng.integers(1, V + 1))); ol.append(0); w.append(float(rng.choice([0.0, 0.5])))
        for _ in range(8 if s == 0 else int(rng.integers(0, max_extra + 1))):    # the start state leads somewhere
            if rng.random() < p_eps and s + 1 < S:
                src.append(s); dst.append(int(rng.integers(s + 1, S))); il.append(0)
                w.append(float(rng.choice([0.0, 0.5])))
            else:
                src.append(s); dst.append(int(rng.integers(0, S)))
                il.append(1 if rng.random() < 0.5 else int(rng.integers(1, V + 1)))
                w.append(float(rng.choice([0.0, 0.5, 1.0])))
            ol.append(int(rng.integers(1, num_words + 1)) if rng.random() < 0.5 else 0)
    return _csr(S, 0, V, src, dst, il, ol, w)
