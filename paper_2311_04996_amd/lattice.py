"""Host-side view of a lattice returned by wfst_get_lattice, and n-best paths through it.

The links are found on the GPU; what is here is bookkeeping over the returned arrays (numpy,
plain Python), for callers that want paths rather than links.
"""
from __future__ import annotations

import heapq
from dataclasses import dataclass

import numpy as np


@dataclass
class Lattice:
    """Tokens of the closed sets A_0..A_T numbered consecutively (A_t = [frame_off[t],
    frame_off[t+1])), their graph state and stored cost, and the links between them (structured
    array: src, dst, ilabel, olabel, graph_cost, acoustic_cost, cost, frame)."""
    frame_off: np.ndarray
    state: np.ndarray
    cost: np.ndarray
    links: np.ndarray

    @property
    def num_frames(self) -> int:
        return len(self.frame_off) - 2

    def start_token(self, start_state: int) -> int:
        lo, hi = int(self.frame_off[0]), int(self.frame_off[1])
        hit = np.nonzero(self.state[lo:hi] == start_state)[0]
        if len(hit) != 1:
            raise ValueError("the first token set does not hold exactly one start token")
        return lo + int(hit[0])

    def nbest(self, n: int, start_state: int, final_cost=None):
        """The n least-cost paths from the start token to a token of the last set, by the sum of
        (cost - stored cost of the source token) over their links, i.e. graph + acoustic (+ boost)
        costs, plus final_cost[state] of the last token when given (non-final tokens are then
        skipped if any token is final).  Exact: best-first search with the exact cost-to-go of
        every token as the heuristic.  Returns a list of (cost, [link indices], [words])."""
        L = self.links
        T = self.num_frames
        lo, hi = int(self.frame_off[T]), int(self.frame_off[T + 1])
        ntok = len(self.state)
        inc = (L["cost"].astype(np.float64) - self.cost[L["src"]].astype(np.float64))
        # exact cost-to-go: tokens in reverse topological order of the link graph
        end = np.full(ntok, np.inf)
        if final_cost is not None:
            fc = np.asarray(final_cost, dtype=np.float64)[self.state[lo:hi]]
            end[lo:hi] = fc if np.isfinite(fc).any() else 0.0
        else:
            end[lo:hi] = 0.0
        out_of = [[] for _ in range(ntok)]
        indeg = np.zeros(ntok, np.int64)
        for k in range(len(L)):
            out_of[int(L["src"][k])].append(k)
            indeg[int(L["dst"][k])] += 1
        order, ready = [], [i for i in range(ntok) if indeg[i] == 0]
        while ready:
            i = ready.pop()
            order.append(i)
            for k in out_of[i]:
                d = int(L["dst"][k])
                indeg[d] -= 1
                if indeg[d] == 0:
                    ready.append(d)
        if len(order) != ntok:
            raise ValueError("the links contain a cycle")
        togo = end.copy()
        for i in reversed(order):
            for k in out_of[i]:
                togo[i] = min(togo[i], inc[k] + togo[int(L["dst"][k])])
        start = self.start_token(start_state)
        heap = [(togo[start], 0.0, start, ())]
        out = []
        while heap and len(out) < n:
            est, g, i, path = heapq.heappop(heap)
            if not np.isfinite(est):
                break
            if path and path[-1] == -1:          # a finished path
                links = list(path[:-1])
                out.append((g, links, [int(L["olabel"][k]) for k in links if L["olabel"][k] != 0]))
                continue
            if lo <= i < hi and np.isfinite(end[i]):
                heapq.heappush(heap, (g + end[i], g + end[i], i, path + (-1,)))
            for k in out_of[i]:
                d = int(L["dst"][k])
                if np.isfinite(togo[d]):
                    heapq.heappush(heap, (g + inc[k] + togo[d], g + inc[k], d, path + (k,)))
        return out
