"""Brute-force definition of the boosting tree on token strings -- no trie, no failure links.

Used only to pin the oracle on tiny inputs.  Everything is expressed on tuples of
tokens and one Python set of phrase prefixes:

  * the state after a blank-free token history h is the longest suffix of h that
    is a prefix of some phrase (Sec. II-A: Aho-Corasick prefix tree + failure links);
  * acc(x) of a prefix x is the sum of the arc scores on the way to it, each arc
    scored by the first phrase in list order that contains it (Alg. 1, Stage 1:
    a score is assigned only when the arc is created);
  * a query steps down the suffixes of the state that are tree prefixes, longest
    first, paying acc(shorter) - acc(longer) for every abandoned one -- nothing if
    the abandoned one is a complete phrase (Sec. II-B, backoff paragraph) -- until
    the token extends one of them or the empty string is reached, where an unknown
    token costs c_unk and stays at the root.
"""
from __future__ import annotations

import math
from typing import Dict, List, Sequence, Tuple

import numpy as np

f32 = np.float32


class BruteTree:
    def __init__(self, phrases: Sequence[Tuple[int, ...]], weights: Sequence[float], mode: str = "uniform",
                 beta: float = 2.0, c_unk: float = 0.0, final_zero_backoff: bool = True, blank: int = -1):
        self.phrases = [tuple(p) for p in phrases]
        self.c_unk = f32(c_unk)
        self.fzb = final_zero_backoff
        self.blank = blank
        self.finals = set(self.phrases)
        self.arc: Dict[Tuple[int, ...], float] = {}
        self.acc: Dict[Tuple[int, ...], float] = {(): 0.0}
        beta64 = float(f32(beta))
        plain: Dict[Tuple[int, ...], float] = {(): 0.0}
        for p, w in zip(self.phrases, weights):
            c0 = float(f32(w))
            for d in range(1, len(p) + 1):
                x = p[:d]
                if x in self.acc:
                    continue
                if mode == "uniform":
                    a = c0
                elif mode == "uniform_final":
                    # uniform arcs; the arc that completes a phrase also pays the uniform scores of all
                    # transitions of that phrase (Sec. II-B: reward = accumulated score, final node only)
                    plain[x] = plain[x[:-1]] + c0
                    a = c0 + (plain[x] if x in self.finals else 0.0)
                elif mode == "logdepth":
                    a = c0 if d == 1 else c0 * beta64 + math.log(float(d))
                else:
                    raise ValueError(mode)
                self.arc[x] = a
                self.acc[x] = self.acc[x[:-1]] + a
        self.prefixes = set(self.acc.keys())

    # longest suffix of `h` that is a tree prefix
    def state_of(self, h: Tuple[int, ...]) -> Tuple[int, ...]:
        for start in range(len(h) + 1):
            if h[start:] in self.prefixes:
                return h[start:]
        raise AssertionError("the empty string is always a prefix")

    def suffix_chain(self, y: Tuple[int, ...]) -> List[Tuple[int, ...]]:
        """Suffixes of y that are tree prefixes, longest first, ending with ()."""
        return [y[i:] for i in range(len(y) + 1) if y[i:] in self.prefixes]

    def bw(self, y: Tuple[int, ...], y_next: Tuple[int, ...]) -> np.float32:
        if self.fzb and y in self.finals:
            return f32(0.0)
        return f32(self.acc[y_next] - self.acc[y])

    def query(self, y0: Tuple[int, ...], v: int):
        """(score fp32, next state string) for state string y0 and token v."""
        if v == self.blank:
            return f32(0.0), y0
        chain = self.suffix_chain(y0)
        p = f32(0.0)
        i = 0
        while chain[i] != () and chain[i] + (v,) not in self.prefixes:
            p = f32(p + self.bw(chain[i], chain[i + 1]))
            i += 1
        ext = chain[i] + (v,)
        if ext in self.prefixes:
            return f32(p + f32(self.arc[ext])), ext
        return f32(p + self.c_unk), ()

    def abandoned(self, y0: Tuple[int, ...], v: int) -> List[Tuple[int, ...]]:
        """Tree prefixes left behind by the query (the failure chain it walked)."""
        chain = self.suffix_chain(y0)
        out = []
        i = 0
        while chain[i] != () and chain[i] + (v,) not in self.prefixes:
            out.append(chain[i])
            i += 1
        return out


def kmp_automaton(pattern: Sequence[int], vocab: int) -> List[List[int]]:
    """Textbook Knuth-Morris-Pratt automaton: delta[j][v] = matched length after reading v."""
    L = len(pattern)
    pi = [0] * L
    k = 0
    for i in range(1, L):
        while k > 0 and pattern[i] != pattern[k]:
            k = pi[k - 1]
        if pattern[i] == pattern[k]:
            k += 1
        pi[i] = k
    delta = [[0] * vocab for _ in range(L + 1)]
    for j in range(L + 1):
        for v in range(vocab):
            k = j
            while k > 0 and (k == L or pattern[k] != v):
                k = pi[k - 1]
            if k < L and pattern[k] == v:
                k += 1
            delta[j][v] = k
    return delta


def topk_reference(totals: np.ndarray, K: int):
    """K best of a flat fp32 array by (value descending, flat index ascending), via numpy."""
    idx = np.arange(totals.size)
    order = np.lexsort((idx, -totals.astype(np.float64)))
    return order[:K]
