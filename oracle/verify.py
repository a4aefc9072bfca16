"""Oracle: the glue between the draft tree and the target model's verification pass
(Sec. 2.1: the target verifies the drafted tokens in parallel and accepts a contiguous
prefix; Fig. 3 "Tree Attention").

Two plain routines over a drafted tree (tokens, parents as `tree_prune` emits them):

`tree_positions` -- depth of every node below the root.  Node i of the tree is the
candidate for sequence position ctx_len + depth(i), so these are the position ids a
tree-attention verification pass needs (the ancestor mask is already an output of
pruning).

`accept_greedy` -- the temperature-0 case of the acceptance rule: the target model
emits its own next token at every tree node; starting at the root, a child is accepted
iff its token equals the target's token at its parent, and the walk ends at the first
node none of whose children matches.  The target's token at the last accepted node is
the next root ("bonus" token).  With sibling tokens distinct the path is unique.
"""
from __future__ import annotations

import numpy as np


def tree_positions(parents: np.ndarray, n_nodes: int) -> np.ndarray:
    """depth[i] = number of edges from the root to node i; -1 beyond n_nodes."""
    depth = np.full(len(parents), -1, dtype=np.int32)
    for i in range(n_nodes):
        d, j = 0, i
        while parents[j] >= 0:
            j = int(parents[j])
            d += 1
        depth[i] = d
    return depth


def accept_greedy(tokens: np.ndarray, parents: np.ndarray, n_nodes: int, target_next: np.ndarray):
    """Walk from the root.  Returns (path, next_token): path = node indices accepted, root
    first (its length - 1 is the number of accepted draft tokens); next_token = the target's
    token at the last node of the path."""
    path = [0]
    while True:
        cur = path[-1]
        want = int(target_next[cur])
        nxt = -1
        for c in range(n_nodes):                      # children in node order
            if int(parents[c]) == cur and int(tokens[c]) == want:
                nxt = c
                break
        if nxt < 0:
            return path, want
        path.append(nxt)
