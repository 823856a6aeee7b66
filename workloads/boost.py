"""Seeded boosting acceptors (inputs of word / phrase boosting).

A boosting acceptor B is a deterministic automaton over the graph's OUTPUT labels, state 0 its
root, every arc carrying a score (negative = preferred).  Targets are label sequences; B is their
trie with every node that has no continuation merged into the root (after a complete target the
next label starts afresh), so targets of one label give the one-state acceptor with self-loops.
What a decoder does when no arc matches (the failure arc back to the root) is the decoder's
business and is not encoded here.  Pure data generation: none of the decoder's arithmetic.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass
class BoostFst:
    num_states: int
    arc_from: np.ndarray     # int32 [n]
    arc_label: np.ndarray    # int32 [n], output labels (> 0)
    arc_to: np.ndarray       # int32 [n]
    arc_score: np.ndarray    # float32 [n]

    @property
    def num_arcs(self) -> int:
        return len(self.arc_from)


def boost_trie(targets, score=-2.0) -> BoostFst:
    """Trie of the label sequences `targets`; every arc scores `score` (a number, or a function
    of (depth, label)).  Nodes without children are the root."""
    children = [{}]                                   # node -> {label: node}
    for seq in targets:
        node = 0
        for lab in seq:
            lab = int(lab)
            if lab not in children[node]:
                children[node][lab] = len(children)
                children.append({})
            node = children[node][lab]
    # number the nodes that have continuations; the others are the root
    number, depth = {0: 0}, {0: 0}
    order = [0]
    for node in order:
        for lab, ch in sorted(children[node].items()):
            depth[ch] = depth[node] + 1
            if children[ch]:
                number[ch] = len(number)
                order.append(ch)
    arcs = []
    for node in order:
        for lab, ch in sorted(children[node].items()):
            sc = score(depth[node], lab) if callable(score) else score
            arcs.append((number[node], lab, number.get(ch, 0), float(sc)))
    a = np.array(arcs, dtype=np.float64).reshape(-1, 4)
    return BoostFst(len(number), a[:, 0].astype(np.int32), a[:, 1].astype(np.int32), a[:, 2].astype(np.int32),
                    a[:, 3].astype(np.float32))


def random_targets(rng, n_targets, vocab, min_len=1, max_len=4):
    """n_targets label sequences, lengths uniform on {min_len..max_len}, labels uniform over `vocab`
    (an array of output labels)."""
    vocab = np.asarray(vocab)
    return [vocab[rng.integers(0, len(vocab), size=int(rng.integers(min_len, max_len + 1)))].tolist()
            for _ in range(n_targets)]


def boost_fsts(seed: int, batch: int, num_words: int, per_utt: int = 100, max_len: int = 4,
               score: float = -2.0, hot_words: int | None = None):
    """One acceptor per utterance: per_utt targets of 1..max_len labels, uniform over the word ids
    1..num_words (or, with hot_words, over a seeded subset of that many words, which makes longer
    matches frequent), every matched label scoring `score`."""
    out = []
    for b in range(batch):
        rng = np.random.default_rng([seed, 0xB0F5, b])
        vocab = np.arange(1, num_words + 1)
        if hot_words:
            vocab = rng.choice(vocab, size=hot_words, replace=False)
        out.append(boost_trie(random_targets(rng, per_utt, vocab, 1, max_len), score))
    return out
