"""Draft tree construction, tree position ids / ancestor mask, greedy acceptance
(oracle; test infrastructure only).

The paper names the strategy (tree drafting with a width, a depth and a total
number of draft tokens; section 4.1 "Implementations") and leaves the procedure to
its citations.  The reading taken here, in the paper's three knobs:

  width k      every expanded node proposes its k most probable next tokens, and at
               most k nodes are expanded per depth;
  depth L      number of drafter passes = length of the longest draft path;
  total N      draft nodes kept for verification, the N highest-scoring candidates.

A candidate's score is the sum of the drafter's log-probabilities along its path
(kept in float32: decisions are taken in the precision the kernels use).  Ties
go to the lower token id (children of one node) and to the earlier candidate
(anywhere else).  Since log-probabilities are <= 0 a parent never scores below
its child and comes earlier, so the kept set is closed under "parent of".
"""
import numpy as np


class TreeBuilder:
    """Level-by-level expansion.  Usage:

        tb = TreeBuilder(k, L, N)
        for d in 1..L:   rows = tb.frontier()           # nodes to expand at this depth
                         tb.push(ids[rows, k], logp[rows, k])
        tree = tb.finalize(t)

    frontier() returns candidate-pool indices (or [-1] = the root at depth 1), in
    expansion order.  push() takes, per frontier row, the k best tokens in rank order
    and their float32 log-probabilities.
    """

    def __init__(self, top_k, depth, total_tokens):
        self.k, self.L, self.N = top_k, depth, total_tokens
        self.token, self.parent, self.depth, self.score = [], [], [], []
        self._frontier = [-1]
        self.expanded = {}         # expanded node (candidate index, -1 = the root) -> candidate indices of its k children, in the order given
        self.d = 0
        self.margins = []          # score gaps at every keep/drop boundary (diagnostics)

    def frontier(self):
        return list(self._frontier)

    def _score_of(self, v):
        return np.float32(0.0) if v < 0 else self.score[v]

    def push(self, ids, logp):
        self.d += 1
        first = len(self.token)
        for r, v in enumerate(self._frontier):
            self.expanded[v] = list(range(first + r * self.k, first + (r + 1) * self.k))
            for c in range(self.k):
                self.token.append(int(ids[r][c]))
                self.parent.append(v)
                self.depth.append(self.d)
                self.score.append(np.float32(self._score_of(v) + np.float32(logp[r][c])))
        if self.d < self.L:
            level = list(range(first, len(self.token)))
            order = sorted(level, key=lambda i: (-float(self.score[i]), i))
            self._frontier = order[:self.k]
            if len(order) > self.k:
                self.margins.append(float(self.score[order[self.k - 1]] - self.score[order[self.k]]))
        else:
            self._frontier = []

    def finalize(self, t):
        """Keep the N best candidates and emit the verification tree (node 0 = root at
        sequence position t)."""
        pool = list(range(len(self.token)))
        order = sorted(pool, key=lambda i: (-float(self.score[i]), i))
        n_keep = min(self.N, len(pool))
        if len(order) > n_keep:
            self.margins.append(float(self.score[order[n_keep - 1]] - self.score[order[n_keep]]))
        kept = sorted(order[:n_keep])                 # candidate order => parents first
        new_index = {p: i + 1 for i, p in enumerate(kept)}
        new_index[-1] = 0
        tree = Tree(
            token=[None] + [self.token[p] for p in kept],
            parent=[-1] + [new_index[self.parent[p]] for p in kept],
            depth=[0] + [self.depth[p] for p in kept],
            score=[np.float32(0.0)] + [self.score[p] for p in kept],
            pool_index=[-1] + kept)
        tree.finish(t)
        return tree


class Tree:
    """Verification tree: parallel lists over nodes; node 0 is the root (the last
    committed token)."""

    def __init__(self, token, parent, depth=None, score=None, pool_index=None):
        self.token, self.parent = list(token), list(parent)
        n = len(self.token)
        if depth is None:
            depth = [0] * n
            for i in range(1, n):
                depth[i] = depth[self.parent[i]] + 1
        self.depth = list(depth)
        self.score = list(score) if score is not None else [np.float32(0)] * n
        self.pool_index = list(pool_index) if pool_index is not None else [-1] * n
        self.pos, self.mask = None, None

    @property
    def n(self):
        return len(self.token)

    def finish(self, t):
        self.pos, self.mask = tree_positions(self.depth, t), ancestor_masks(self.parent)
        return self

    def allowed(self, n_ctx):
        """[n, n_ctx + n] visibility: all context keys, plus tree rows on the node's root path."""
        a = np.ones((self.n, n_ctx + self.n), dtype=bool)
        for i in range(self.n):
            for j in range(self.n):
                a[i, n_ctx + j] = bool((self.mask[i] >> j) & 1)
        return a

    def mask_words(self, words):
        out = np.zeros((self.n, words), dtype=np.uint64)
        for i, m in enumerate(self.mask):
            for w in range(words):
                out[i, w] = (m >> (64 * w)) & 0xFFFFFFFFFFFFFFFF
        return out


def tree_positions(depth, t):
    """Sequence position of a node = t + its depth (the root is committed token x_t)."""
    return [t + d for d in depth]


def ancestor_masks(parent):
    """mask[i] has bit j set iff node j is i itself or one of its ancestors."""
    mask = [0] * len(parent)
    for i, p in enumerate(parent):
        if p >= i:
            raise ValueError("parent index must precede the node")
        mask[i] = (1 << i) | (mask[p] if p >= 0 else 0)
    return mask


def validate_tree(token, parent):
    """Structural checks shared by callers that take a tree from outside."""
    if len(token) < 1 or len(token) != len(parent) or parent[0] != -1:
        return False
    seen = set()
    for i in range(1, len(parent)):
        if not (0 <= parent[i] < i):
            return False
        key = (parent[i], token[i])
        if key in seen:                 # siblings must carry distinct tokens
            return False
        seen.add(key)
    return True


def accept_walk(token, parent, g):
    """Greedy acceptance (section 2.1; A_i subset of A_{i-1}, section 3.1).

    g[i] is the target's greedy token after node i.  Starting at the root, step to
    the child whose token equals g[current]; stop when there is none.
    Returns (path of node indices starting with 0, bonus token g[last])."""
    children = {}
    for i in range(1, len(parent)):
        children.setdefault(parent[i], []).append(i)
    cur, path = 0, [0]
    while True:
        nxt = [c for c in children.get(cur, []) if token[c] == g[cur]]
        if not nxt:
            break
        cur = nxt[0]
        path.append(cur)
    return path, int(g[cur])


def accept_bruteforce(token, parent, g):
    """Enumerate every root-to-node path; return the longest one all of whose draft
    tokens equal the target's greedy token at their parent."""
    best = [0]
    for v in range(len(parent)):
        path, u = [], v
        while u != -1:
            path.append(u)
            u = parent[u]
        path.reverse()
        ok = all(token[path[j]] == g[path[j - 1]] for j in range(1, len(path)))
        if ok and len(path) > len(best):
            best = path
    return best, int(g[best[-1]])


class AcceptStats:
    """c[i] = number of rounds that accepted at least i draft tokens (i = 1..L).

    P(A_i) = c[i]/R; pos-acc_i = c[i]/c[i-1] for i > 1 (Eq. 3); the chain rule of Eq. 4
    gives P(A_1 .. A_k) = c[k]/R; the mean number of accepted draft tokens per round is
    sum_i c[i] / R.  tau_gen adds the bonus token every round produces."""

    def __init__(self, depth):
        self.L, self.rounds, self.c = depth, 0, [0] * (depth + 1)
        self.committed = 0

    def add(self, m):
        self.rounds += 1
        self.committed += m + 1
        for i in range(1, m + 1):
            self.c[i] += 1

    def p_accept(self, i):
        return self.c[i] / self.rounds

    def pos_acc(self, i):
        if i <= 1:
            raise ValueError("pos-acc is defined for i > 1")
        return self.c[i] / self.c[i - 1] if self.c[i - 1] else float("nan")

    @property
    def tau_acc(self):
        return sum(self.c[1:]) / self.rounds

    @property
    def tau_gen(self):
        return self.tau_acc + 1.0
