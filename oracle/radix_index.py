"""Oracle for the prefix-trie index maps (I_gather, I_scatter).

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).  Plain Python, slow on purpose.

Two independent implementations:

* ``build_index_trie``  - sequential trie insertion, the computation of the paper's
  Algorithm 2 ("Radix Tree Creation") in a structure of its own (one edge dictionary):
  sequences are inserted one after the other from the root, a node is identified by its
  parent and the next (token id, position id) pair, a node that is created gets the next
  compact index and records the original position that created it.
* ``build_index_bruteforce`` - the plain definition (Section "The RadixMLP Layout",
  paragraph "Trie Construction", and the "Index semantics" paragraph of the appendix):
  two original positions are the same node iff they have the same offset in their
  sequences and the (token, position) pairs of their whole causal histories agree;
  I_gather lists, in increasing order, the first original position of every class, and
  I_scatter maps every original position to the rank of its class in that list.

Pins (tests/test_oracle_index.py): the paper's printed toy example, the closed form
N' = P + B*S with the (N, N') pairs of the paper's Qwen3-4B sweep table, structural
invariants, trivial cases, the path-specificity rule, and agreement of the two
implementations on random small batches.
"""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple

import numpy as np


def _positions(cu_seqlens: Sequence[int], pos: Optional[Sequence[int]]) -> np.ndarray:
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    n = int(cu[-1]) if len(cu) else 0
    if pos is not None:
        p = np.asarray(pos, dtype=np.int64)
        assert p.shape == (n,)
        return p
    p = np.zeros(n, dtype=np.int64)
    for s in range(len(cu) - 1):
        p[cu[s]:cu[s + 1]] = np.arange(cu[s + 1] - cu[s])
    return p


def node_key(position: int, token: int) -> int:
    """64-bit node key of Algorithm 2: (position << 32) XOR token.

    For 0 <= token < 2**31 and 0 <= position < 2**31 this is a one-to-one encoding of the
    pair, so it is an exact key, not a lossy hash.
    """
    return (int(position) << 32) ^ int(token)


def build_index_trie(tok: Sequence[int], cu_seqlens: Sequence[int],
                     pos: Optional[Sequence[int]] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Sequential trie insertion (what Algorithm 2 computes).  Returns (I_scatter[N], I_gather[N']) as int32 arrays.

    A trie node is named by its compact index, which is its creation rank; the root ("sequence start") is -1.
    The trie itself is one dictionary of edges, (parent node, node_key of the next token) -> child node.  Walking a
    sequence from the root, an edge that is missing creates the child: it gets the next compact index and the
    original position that created it becomes its I_gather entry; every original position records the node it
    reached as its I_scatter entry.
    """
    tok = np.asarray(tok, dtype=np.int64)
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    position_ids = _positions(cu, pos)
    n = int(cu[-1]) if len(cu) else 0
    edges = {}
    first_position: List[int] = []              # compact index -> original position that created the node
    scatter = np.zeros(n, dtype=np.int32)
    for s in range(len(cu) - 1):
        node = -1
        for i in range(int(cu[s]), int(cu[s + 1])):
            edge = (node, node_key(position_ids[i], tok[i]))
            child = edges.get(edge)
            if child is None:
                child = len(first_position)
                edges[edge] = child
                first_position.append(i)
            scatter[i] = child
            node = child
    return scatter, np.asarray(first_position, dtype=np.int32)


def build_index_bruteforce(tok: Sequence[int], cu_seqlens: Sequence[int],
                           pos: Optional[Sequence[int]] = None) -> Tuple[np.ndarray, np.ndarray]:
    """The definition, O(N * B * L).  For tiny inputs only."""
    tok = np.asarray(tok, dtype=np.int64)
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    position_ids = _positions(cu, pos)
    n = int(cu[-1]) if len(cu) else 0
    B = len(cu) - 1
    rep = np.arange(n, dtype=np.int64)
    for s in range(B):
        for p in range(int(cu[s + 1] - cu[s])):
            j = int(cu[s]) + p
            # smallest earlier original position with the same offset and the same history
            for s2 in range(s):
                if cu[s2 + 1] - cu[s2] <= p:
                    continue
                a0, b0 = int(cu[s]), int(cu[s2])
                same = all(tok[a0 + q] == tok[b0 + q] and position_ids[a0 + q] == position_ids[b0 + q]
                           for q in range(p + 1))
                if same:
                    rep[j] = b0 + p
                    break
    firsts = [j for j in range(n) if rep[j] == j]
    rank = {j: r for r, j in enumerate(firsts)}
    scatter = np.asarray([rank[int(rep[j])] for j in range(n)], dtype=np.int32)
    return scatter, np.asarray(firsts, dtype=np.int32)


def compression(n: int, n_compact: int) -> Tuple[float, float]:
    """(r, gamma) = (N / N', N' / N) as defined in "The RadixMLP Layout"."""
    return n / n_compact, n_compact / n
