"""The PosS round: draft a tree with position specialists, verify it with the target,
accept greedily, commit (oracle; test infrastructure only).

State after prefill / after every round: committed tokens x_0..x_t, target features
f_0..f_{t-1} and target keys/values of positions 0..t-1.  x_t (the root of the next
tree) has no feature yet: it is the token the target chose last.

Draft position i (0-based; depth d = i+1) is served by specialist ceil((i+1)/n)
(Eq. 7).  The specialist at depth d sees the pair sequence of Eq. 9:
[x_1; f_0] .. [x_t; f_{t-1}] with target features, then the drafted pairs
[token(v); f^(S)(parent(v))] along the path to the node it expands.  Pair [x_j; .]
has drafter sequence index j-1.  This file applies each specialist to that whole
sequence afresh (no cache): the HIP library's per-specialist key/value caches and
catch-up passes (section 3.3, overhead (1)) must reproduce it.
"""
import numpy as np

from .model import (target_rows, head, causal_allowed, empty_kv, specialist_pass,
                    specialist_index)
from .numerics import log_softmax
from .tree import TreeBuilder, Tree, accept_walk, AcceptStats
from .sampling import sample_token, softmax_t, sample_children, reject_or_accept, draw_from


def topk_lowest_id(row, k):
    """Indices of the k largest entries, ordered by (value descending, index ascending)."""
    row = np.asarray(row)
    order = np.lexsort((np.arange(row.size), -row))
    return order[:k]


class PossOracle:
    def __init__(self, W, cfg, act=None):
        self.W, self.cfg, self.act = W, cfg, act
        self.tokens, self.feats, self.kv = [], [], empty_kv(cfg)
        self.stats = AcceptStats(cfg.depth)
        self.margins = []                 # decision gaps seen so far (screening / near-tie accounting)
        self.last = {}

    # ------------------------------------------------------------------ prefill
    @property
    def t(self):
        return len(self.tokens) - 1

    def prefill(self, prompt, temperature=0.0, U=None):
        """Causal target pass over the prompt; x_P = greedy token after the prompt (temperature
        > 0: drawn with U[P], see oracle/sampling.py)."""
        cfg, P = self.cfg, len(prompt)
        f, kv = target_rows(self.W, cfg, prompt, np.arange(P), empty_kv(cfg),
                            causal_allowed(0, P), self.act)
        logits = head(self.W, cfg, f[-1:], self.act)[0]
        self._note_margin(logits)
        first = sample_token(logits, temperature, U[P]) if temperature > 0 else int(np.argmax(logits))
        self.tokens = [int(x) for x in prompt] + [first]
        self.feats = [f[i] for i in range(P)]
        self.kv = kv
        return self.tokens[-1]

    def _note_margin(self, logits):
        top2 = np.partition(np.asarray(logits), -2)[-2:]
        self.margins.append(float(top2[1] - top2[0]))

    # ------------------------------------------------------------------ draft
    def draft_tree(self, sampling=None):
        """sampling = (temperature, UD): the k children of an expanded node are drawn without replacement from the
        drafter's softmax(logits / temperature), child i of the node of frontier rank r at depth d with
        UD[d - 1][r][i], and scored with their log-probability under it (oracle/sampling.py, second reading);
        None: its k most probable tokens."""
        cfg, W, t = self.cfg, self.W, self.t
        k, L = cfg.top_k, cfg.depth
        n, S = cfg.positions_per_specialist, cfg.n_specialists
        # committed pairs [x_j ; f_{j-1}], j = 1..t, drafter index j-1
        seq_tok = list(self.tokens[1:t + 1])
        seq_feat = [self.feats[j - 1] for j in range(1, t + 1)]
        seq_pos = list(range(t))
        row_of = {}                      # pool index of an expanded node -> its row in seq_*
        fhat = {}                        # pool index (-1 = root) -> drafted feature
        tb = TreeBuilder(k, L, cfg.total_tokens)
        dbg_logp = []
        draft_q, self.draw_margins = {}, []      # sampled children: the distribution each expanded node's children came from
        for d in range(1, L + 1):
            s = specialist_index(d - 1, n, S)
            front = tb.frontier()
            if d == 1:
                q_rows = [t - 1]                                   # the root pair [x_t ; f_{t-1}]
                allowed = np.ones((1, t), dtype=bool)
            else:
                for v in front:
                    row_of[v] = len(seq_tok)
                    seq_tok.append(tb.token[v])
                    seq_feat.append(fhat[tb.parent[v]])
                    seq_pos.append(t - 1 + tb.depth[v])
                q_rows = [row_of[v] for v in front]
                allowed = np.zeros((len(front), len(seq_tok)), dtype=bool)
                allowed[:, :t] = True
                for r, v in enumerate(front):
                    u = v
                    while u != -1:                                 # v itself and its drafted ancestors
                        allowed[r, row_of[u]] = True
                        u = tb.parent[u]
            out = specialist_pass(W, cfg, s, seq_tok, np.stack(seq_feat), seq_pos, allowed,
                                  q_rows, self.act)
            for r, v in enumerate(front):
                fhat[v] = out[r]
            logits = head(W, cfg, out, self.act).astype(np.float32)
            logp = log_softmax(logits.astype(np.float64)).astype(np.float32)
            ids = np.zeros((len(front), k), dtype=np.int64)
            lp = np.zeros((len(front), k), dtype=np.float32)
            for r in range(len(front)):
                if sampling is not None:
                    temperature, UD = sampling
                    cids, q = sample_children(logits[r], temperature, UD[d - 1][r][:k], self.draw_margins)
                    ids[r], lp[r] = cids, np.log(q[cids]).astype(np.float32)
                    draft_q[front[r]] = q
                    continue
                order = topk_lowest_id(logits[r], k + 1)
                ids[r], lp[r] = order[:k], logp[r, order[:k]]
                gaps = -np.diff(logits[r, order].astype(np.float64))
                self.margins.append(float(gaps.min()))
            n_before = len(tb.token)
            tb.push(ids, lp)
            if d < L:                    # order inside the kept frontier fixes the next candidate order
                lvl = sorted(range(n_before, len(tb.token)), key=lambda i: (-float(tb.score[i]), i))
                sc = np.array([float(tb.score[i]) for i in lvl[:k + 1]])
                if len(sc) > 1:
                    self.margins.append(float((-np.diff(sc)).min()))
            dbg_logp.append((ids, lp))
        tree = tb.finalize(t)
        tree.token[0] = self.tokens[t]
        self.margins += tb.margins
        self.last["builder"], self.last["topk"], self.last["draft_q"] = tb, dbg_logp, draft_q
        return tree

    def score_tree(self, tree):
        """Cumulative drafter log-probability (float64) of every node of a tree built elsewhere:
        node v at depth d scores score(parent) + log P_d(token_v | path), P_d from the specialist
        serving draft position d-1.  Used to judge a tree that differs from draft_tree()'s only
        through near-ties.  Also returns, per expanded node, its full log-probability row."""
        cfg, W, t = self.cfg, self.W, self.t
        n, S = cfg.positions_per_specialist, cfg.n_specialists
        seq_tok = list(self.tokens[1:t + 1])
        seq_feat = [self.feats[j - 1] for j in range(1, t + 1)]
        seq_pos = list(range(t))
        children = {}
        for i in range(1, tree.n):
            children.setdefault(tree.parent[i], []).append(i)
        depth = tree.depth
        score = [0.0] * tree.n
        row_of, fhat, logp_rows = {}, {}, {}
        for d in range(1, max(depth) + 1):
            s = specialist_index(d - 1, n, S)
            expand = [v for v in range(tree.n) if depth[v] == d - 1 and v in children]
            if d == 1:
                q_rows, allowed = [t - 1], np.ones((1, t), dtype=bool)
            else:
                for v in expand:
                    row_of[v] = len(seq_tok)
                    seq_tok.append(tree.token[v])
                    seq_feat.append(fhat[tree.parent[v]])
                    seq_pos.append(t - 1 + depth[v])
                q_rows = [row_of[v] for v in expand]
                allowed = np.zeros((len(expand), len(seq_tok)), dtype=bool)
                allowed[:, :t] = True
                for r, v in enumerate(expand):
                    u = v
                    while u != 0:
                        allowed[r, row_of[u]] = True
                        u = tree.parent[u]
            if not expand:
                continue
            out = specialist_pass(W, cfg, s, seq_tok, np.stack(seq_feat), seq_pos, allowed, q_rows, self.act)
            lp = log_softmax(head(W, cfg, out, self.act))
            for r, v in enumerate(expand):
                fhat[v] = out[r]
                logp_rows[v] = lp[r]
                for c in children[v]:
                    score[c] = score[v] + lp[r, tree.token[c]]
        return np.array(score), logp_rows

    # ------------------------------------------------------------------ verify
    def verify_tree(self, tree, temperature=0.0, U=None):
        """One target pass over all tree rows (section 2.1, second phase).
        Returns (the target's token after each node, logits, features): the argmax, or at
        temperature > 0 a draw with U[position of that token] = U[t + depth + 1]."""
        cfg, t = self.cfg, self.t
        if tree.pos is None:
            tree.finish(t)
        F, new_kv = target_rows(self.W, cfg, tree.token, tree.pos, self.kv, tree.allowed(t), self.act)
        logits = head(self.W, cfg, F, self.act)
        if temperature > 0:
            g = [sample_token(logits[i], temperature, U[t + tree.depth[i] + 1]) for i in range(tree.n)]
        else:
            g = [int(np.argmax(logits[i])) for i in range(tree.n)]
        self.last.update(tree=tree, F=F, new_kv=new_kv, logits=logits, g=g)
        return g, logits, F

    def verify_tree_sampled(self, tree, temperature, UA):
        """Verification of a tree whose children were drawn (draft_tree(sampling=...)) by the rejection rule.  One
        target pass as in verify_tree; then from the root: the k drawn children of the current node are tested in
        the order drawn with UA[depth][0 .. k-1]; an accepted child that the tree kept becomes the current node; an
        accepted child that the rerank dropped, the token drawn from the last residual (with UA[depth][k]) when all
        are rejected, or - at a node that was not expanded - the token drawn from the target's own distribution,
        ends the walk and is committed in the bonus token's place.  Returns (path, that last token)."""
        cfg, t, k = self.cfg, self.t, self.cfg.top_k
        if tree.pos is None:
            tree.finish(t)
        F, new_kv = target_rows(self.W, cfg, tree.token, tree.pos, self.kv, tree.allowed(t), self.act)
        logits = head(self.W, cfg, F, self.act)
        tb, dq = self.last["builder"], self.last["draft_q"]
        node_of = {pool: i for i, pool in enumerate(tree.pool_index)}
        self.accept_margins = []
        cur, path = 0, [0]
        while True:
            d = tree.depth[cur]
            p = softmax_t(logits[cur].astype(np.float32), temperature)
            pv = tree.pool_index[cur]
            if pv not in tb.expanded:
                last = draw_from(p, UA[d][k], self.accept_margins)
                break
            cand = tb.expanded[pv]
            i, resid = reject_or_accept(p, dq[pv], [tb.token[c] for c in cand], UA[d][:k], self.accept_margins)
            if i < 0:
                last = draw_from(resid, UA[d][k], self.accept_margins)
                break
            if cand[i] not in node_of:
                last = tb.token[cand[i]]
                break
            cur = node_of[cand[i]]
            path.append(cur)
        self.last.update(tree=tree, F=F, new_kv=new_kv, logits=logits, g=None)
        return path, int(last)

    # ------------------------------------------------------------------ accept + commit
    def accept_and_commit(self, path=None, bonus=None):
        """Walk, then append the accepted rows' features and keys/values and the new tokens.
        A caller in lock-step may impose (path, bonus)."""
        tree, F, new_kv, g = (self.last[x] for x in ("tree", "F", "new_kv", "g"))
        if path is None:
            path, bonus = accept_walk(tree.token, tree.parent, g)
        for node in path:
            self._note_margin(self.last["logits"][node])
        m = len(path) - 1
        for node in path:
            self.feats.append(F[node])
        self.kv = [(np.concatenate([kc, kn[path]], axis=0), np.concatenate([vc, vn[path]], axis=0))
                   for (kc, vc), (kn, vn) in zip(self.kv, new_kv)]
        self.tokens += [tree.token[p] for p in path[1:]] + [int(bonus)]
        self.stats.add(m)
        return list(path), m, int(bonus)

    # ------------------------------------------------------------------ whole run
    def generate(self, prompt, n_new, record=None, temperature=0.0, U=None):
        """prefill + rounds until n_new new tokens exist; the stream is cut to exactly n_new
        (a last round that overshoots still counts fully in the statistics)."""
        P = len(prompt)
        self.prefill(prompt, temperature, U)
        while len(self.tokens) - P < n_new:
            tree = self.draft_tree()
            g, _, _ = self.verify_tree(tree, temperature, U)
            path, m, bonus = self.accept_and_commit()
            if record is not None:
                record.append(dict(tree=tree, g=g, path=path, m=m, bonus=bonus))
        return self.tokens[:P + n_new]
