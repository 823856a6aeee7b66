"""The benchmark configurations as seeded recipes (shapes follow the paper's workloads:
~128 BPE tokens + blank at 40 ms frames, 2-35 s utterances, a 3-gram-scale graph,
beam 17 / max-active 10,000, batch 256)."""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

from .boost import boost_fsts
from .graphs import Graph, tiny_lexicon_graph, tlg_shaped_graph
from .loglikes import ctc_loglikes, random_lengths

FRAME_SECONDS = 0.040

CONFIGS = {
    # name: graph recipe, batch, frame range, log-likelihood recipe, pruning
    "c1_tiny": dict(graph=("tiny", dict(seed=1)), batch=1, len_lo=100, len_hi=100, seed=1,
                    ll=dict(sigma=1.0, p_blank=0.70, blank_boost=5.0, token_boost=0.0),
                    beam=10.0, max_active=1000),
    "c2_medium": dict(graph=("tlg", dict(seed=2, num_states=200_000, target_arcs=1_000_000,
                                         num_classes=129, alpha=1.8, k_max=5000, p_eps=0.15,
                                         num_words=20_000)),
                      batch=32, len_lo=50, len_hi=875, seed=2,
                      ll=dict(sigma=2.0, p_blank=0.65, blank_boost=6.0, token_boost=4.0),
                      beam=17.0, max_active=7000),
    "c3_large": dict(graph=("tlg", dict(seed=3, num_states=10_000_000, target_arcs=30_000_000,
                                        num_classes=129, alpha=1.8, k_max=5000, p_eps=0.20,
                                        num_words=200_000)),
                     batch=256, len_lo=50, len_hi=875, seed=3,
                     ll=dict(sigma=2.0, p_blank=0.65, blank_boost=6.0, token_boost=4.0),
                     beam=17.0, max_active=10000),
    # config 2 with a word-boost table per utterance (100 words of the vocabulary at -2.0)
    "c5_boost": dict(graph=("tlg", dict(seed=2, num_states=200_000, target_arcs=1_000_000,
                                        num_classes=129, alpha=1.8, k_max=5000, p_eps=0.15,
                                        num_words=20_000)),
                     batch=32, len_lo=50, len_hi=875, seed=2,
                     ll=dict(sigma=2.0, p_blank=0.65, blank_boost=6.0, token_boost=4.0),
                     beam=17.0, max_active=7000, boost=dict(seed=5, per_utt=100, score=-2.0)),
    # config 5: config 2, every utterance composed on the fly with its own boosting acceptor of 100
    # targets of 1-4 output labels (trie; a decoder takes the failure arc to the root on a mismatch)
    "c5_boost_fst": dict(graph=("tlg", dict(seed=2, num_states=200_000, target_arcs=1_000_000,
                                            num_classes=129, alpha=1.8, k_max=5000, p_eps=0.15,
                                            num_words=20_000)),
                         batch=32, len_lo=50, len_hi=875, seed=2,
                         ll=dict(sigma=2.0, p_blank=0.65, blank_boost=6.0, token_boost=4.0),
                         beam=17.0, max_active=7000, boost_fst=dict(seed=5, per_utt=100, max_len=4, score=-2.0)),
    # config 3 on a graph in which no state has the blank self-loop alone: every state has 1-3 more
    # arcs (not a configuration of the paper's workloads; it shows what the decoder does when the
    # shortcut for self-loop-only states never applies)
    "c3_branchy": dict(graph=("tlg", dict(seed=3, num_states=10_000_000, target_arcs=40_000_000,
                                          num_classes=129, alpha=1.8, k_max=5000, p_eps=0.20,
                                          num_words=200_000, extra_lo=1, extra_hi=3)),
                       batch=256, len_lo=50, len_hi=875, seed=3,
                       ll=dict(sigma=2.0, p_blank=0.65, blank_boost=6.0, token_boost=4.0),
                       beam=17.0, max_active=10000),
    # a scaled-down graph of the c3 family for quick runs (not a reported configuration)
    "c3_mini": dict(graph=("tlg", dict(seed=3, num_states=1_000_000, target_arcs=3_000_000,
                                       num_classes=129, alpha=1.8, k_max=5000, p_eps=0.20,
                                       num_words=200_000)),
                    batch=64, len_lo=50, len_hi=875, seed=3,
                    ll=dict(sigma=2.0, p_blank=0.65, blank_boost=6.0, token_boost=4.0),
                    beam=17.0, max_active=10000),
}


def boost_tables(seed: int, batch: int, num_words: int, per_utt: int = 100, score: float = -2.0):
    """Per-utterance word-boost tables: per_utt distinct word ids uniform over the graph's
    vocabulary, every one boosted by `score` (negative = preferred).  List of (ids, scores)."""
    out = []
    for b in range(batch):
        rng = np.random.default_rng([seed, 0xB005, b])
        ids = rng.choice(num_words, size=per_utt, replace=False).astype(np.int32) + 1
        out.append((ids, np.full(per_utt, score, dtype=np.float32)))
    return out


@dataclass
class Workload:
    name: str
    graph: Graph
    lengths: np.ndarray      # int32 [B]
    loglikes: np.ndarray     # float32 [B, T, V]
    beam: float
    max_active: int
    boosts: list | None = None   # per-utterance (word ids, scores) or None
    boost_fsts: list | None = None   # per-utterance boosting acceptors (workloads.boost.BoostFst) or None

    @property
    def audio_seconds(self) -> float:
        return float(self.lengths.sum()) * FRAME_SECONDS


def make_graph(name: str) -> Graph:
    kind, kw = CONFIGS[name]["graph"]
    return tiny_lexicon_graph(**kw) if kind == "tiny" else tlg_shaped_graph(**kw)


def make_config(name: str, batch: int | None = None, graph: Graph | None = None) -> Workload:
    c = CONFIGS[name]
    g = graph if graph is not None else make_graph(name)
    B = c["batch"] if batch is None else int(batch)
    lengths = random_lengths(c["seed"], B, c["len_lo"], c["len_hi"])
    T = int(lengths.max())
    ll = ctc_loglikes(c["seed"], lengths, T, g.num_classes, **c["ll"])
    boosts = None
    if "boost" in c:
        boosts = boost_tables(c["boost"]["seed"], B, int(g.meta["num_words"]), c["boost"]["per_utt"], c["boost"]["score"])
    fsts = None
    if "boost_fst" in c:
        fsts = boost_fsts(c["boost_fst"]["seed"], B, int(g.meta["num_words"]), c["boost_fst"]["per_utt"],
                          c["boost_fst"]["max_len"], c["boost_fst"]["score"])
    return Workload(name, g, lengths, ll, float(c["beam"]), int(c["max_active"]), boosts, fsts)
