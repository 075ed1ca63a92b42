"""Tree construction, masks, acceptance walk and statistics of the oracle, against brute
force, hand-derived values and the identities of Eq. 3 and Eq. 4."""
import numpy as np
import pytest

from oracle.tree import (TreeBuilder, Tree, ancestor_masks, tree_positions, accept_walk,
                         accept_bruteforce, AcceptStats, validate_tree)


def test_masks_and_positions_by_hand():
    #        0
    #      /   \
    #     1     2
    #    / \     \
    #   3   4     5
    parent = [-1, 0, 0, 1, 1, 2]
    assert ancestor_masks(parent) == [0b1, 0b11, 0b101, 0b1011, 0b10011, 0b100101]
    assert tree_positions([0, 1, 1, 2, 2, 2], 100) == [100, 101, 101, 102, 102, 102]
    tr = Tree(token=[9, 1, 2, 3, 4, 5], parent=parent).finish(7)
    assert tr.depth == [0, 1, 1, 2, 2, 2] and tr.pos == [7, 8, 8, 9, 9, 9]
    a = tr.allowed(3)
    assert a.shape == (6, 9) and a[:, :3].all()
    assert a[4, 3:].tolist() == [True, True, False, False, True, False]
    w = tr.mask_words(2)
    assert w[5].tolist() == [0b100101, 0]
    with pytest.raises(ValueError):
        ancestor_masks([-1, 2, 1])


def _random_tree(rng, n, vocab):
    parent, token = [-1], [int(rng.integers(vocab))]
    for i in range(1, n):
        while True:
            p, tk = int(rng.integers(0, i)), int(rng.integers(vocab))
            if all(not (parent[j] == p and token[j] == tk) for j in range(1, i)):
                break
        parent.append(p)
        token.append(tk)
    return token, parent


def test_accept_walk_equals_bruteforce_and_is_a_root_path():
    rng = np.random.default_rng(0)
    lengths = set()
    for trial in range(300):
        n = int(rng.integers(1, 40))
        token, parent = _random_tree(rng, n, vocab=6)
        assert validate_tree(token, parent)
        g = [int(rng.integers(6)) for _ in range(n)]
        path, bonus = accept_walk(token, parent, g)
        bpath, bbonus = accept_bruteforce(token, parent, g)
        assert path == bpath and bonus == bbonus == g[path[-1]]
        assert path[0] == 0 and all(parent[path[j]] == path[j - 1] for j in range(1, len(path)))
        assert all(token[path[j]] == g[path[j - 1]] for j in range(1, len(path)))
        lengths.add(len(path))
    assert len(lengths) >= 4          # the sample really contains accepted paths of several lengths


def _bruteforce_keep(pool_parent, pool_score, n_keep):
    """Rank every candidate by counting who beats it: (score desc, index asc)."""
    n = len(pool_score)
    keep = []
    for i in range(n):
        beaten_by = sum(1 for j in range(n) if (pool_score[j] > pool_score[i]) or
                        (pool_score[j] == pool_score[i] and j < i))
        if beaten_by < n_keep:
            keep.append(i)
    return keep


@pytest.mark.parametrize("k,L,N,ties", [(4, 6, 24, False), (3, 4, 10, True), (10, 6, 60, False),
                                          (2, 3, 50, True), (10, 7, 80, True)])
def test_tree_builder_against_bruteforce(k, L, N, ties):
    rng = np.random.default_rng(k * 100 + L)
    tb = TreeBuilder(k, L, N)
    vocab = 1000
    for d in range(1, L + 1):
        front = tb.frontier()
        assert len(front) == (1 if d == 1 else k)
        if d > 1:     # the frontier is the k best of the previous level, best first
            lvl = [i for i in range(len(tb.token)) if tb.depth[i] == d - 1]
            ref = sorted(lvl, key=lambda i: (-float(tb.score[i]), i))[:k]
            assert front == ref
        ids = np.stack([rng.choice(vocab, size=k, replace=False) for _ in front])
        if ties:      # exactly representable values drawn from a small set: many equal scores
            lp = -np.sort(rng.integers(1, 4, size=(len(front), k)), axis=1).astype(np.float32) * 0.5
        else:
            lp = -np.sort(rng.exponential(2.0, size=(len(front), k)), axis=1).astype(np.float32)
        tb.push(ids, lp)
    assert len(tb.token) == k + (L - 1) * k * k
    # scores are float32 running sums along the path
    for i in range(len(tb.token)):
        assert tb.score[i].dtype == np.float32
    tree = tb.finalize(t=50)
    keep = _bruteforce_keep(tb.parent, [float(s) for s in tb.score], min(N, len(tb.token)))
    assert tree.pool_index[1:] == keep
    assert tree.n == min(N, len(tb.token)) + 1
    # closed under "parent of", parents first, tokens/depths/positions/masks consistent
    for i in range(1, tree.n):
        p = tree.parent[i]
        assert 0 <= p < i
        assert tree.pool_index[p] == tb.parent[tree.pool_index[i]]
        assert tree.depth[i] == tree.depth[p] + 1 == tb.depth[tree.pool_index[i]]
        assert tree.pos[i] == 50 + tree.depth[i]
        assert tree.mask[i] == (1 << i) | tree.mask[p]
        assert tree.token[i] == tb.token[tree.pool_index[i]]
    assert validate_tree([0] + tree.token[1:], tree.parent)


def test_stats_identities_eq3_eq4():
    rng = np.random.default_rng(5)
    L = 6
    st = AcceptStats(L)
    ms = rng.integers(0, L + 1, size=500)
    for m in ms:
        st.add(int(m))
    R = len(ms)
    for i in range(1, L + 1):
        assert st.c[i] == int((ms >= i).sum())                 # A_i: at least i draft tokens accepted
        assert st.c[i] <= st.c[i - 1] or i == 1                # A_i subset of A_{i-1}
    for k in range(1, L + 1):                                  # Eq. 4: chain rule
        prod = st.p_accept(1)
        for i in range(2, k + 1):
            prod *= st.pos_acc(i)                              # Eq. 3
        assert np.isclose(prod, (ms >= k).mean())
    assert np.isclose(st.tau_acc, ms.mean()) and np.isclose(st.tau_gen, ms.mean() + 1)
    assert st.committed == int(ms.sum()) + R
    with pytest.raises(ValueError):
        st.pos_acc(1)
