"""CPU oracle, part 3: the draft-verify cycle with a draft TREE instead of a chain (float64, numpy).

TEST INFRASTRUCTURE ONLY (see oracle/model.py).

Section 4 ("Training and Inference Setting") states the inference setting of the paper's
experiments: the drafter expands a top-k tree to a fixed depth lambda and the candidates
with the highest cumulative probability are kept for verification (k = 10, lambda = 6, 60
candidates; the supplementary comparison uses 30 candidates, depth 4, k = 8).  Section 2.1
names the structure as the draft tree of EAGLE-2 (Li et al. 2024).  The paper gives no more
detail; the reading taken here, step by step:

  pool       level 1: the k most probable tokens after the drafter's pending hidden state f'_1,
             each scored with its log-probability.  Level j+1 (j = 1..lambda-1): the k best-scored
             nodes of level j are EXPANDED: each goes through the drafter as one row (input
             f'_parent w1 + Embed(token) w2 + r^j w: Algorithm 1's drafting step with the residual of
             its depth), attending to the text-only cache plus its own ancestors, and its k most
             probable continuations join the pool scored parent score + log-probability.
             Pool size k + (lambda-1) k^2, indexed level by level, parent by parent, rank by rank.
  candidates the n_nodes best-scored pool nodes (ties: lower pool index).  A child never scores
             above its parent and sits after it in the pool, so the set is closed under ancestors.
  verify     one target pass over [x_{l+1}, candidates in pool order]; a row sits at position
             v + l + depth and sees the whole visual+text cache, its ancestors and itself.
  accept     greedy: from the root, follow the child whose token equals the target's greedy token
             at the current node until there is none; emit the followed tokens plus the target's
             token at the last node (section 2.1's rule, on a tree).
  roll       the target keeps the rows of the followed path only; the drafter drops every tree row and
             is re-fed the true features of the path (as after a chain round).

With k = 1 every step above is Algorithm 1's chain (tests/test_oracle_tree.py pins that).
"""
import numpy as np

from .model import F64, argmax_lowest
from .hivis import HivisOracle, fuse


def log_softmax(logits):
    """log of softmax(logits) along the last axis."""
    z = np.asarray(logits, F64)
    z = z - np.max(z, axis=-1, keepdims=True)
    return z - np.log(np.sum(np.exp(z), axis=-1, keepdims=True))


def top_k_lowest(values, k):
    """Indices of the k largest values, best first; equal values in index order."""
    v = np.asarray(values, F64)
    return [int(i) for i in np.argsort(-v, kind="stable")[:k]]


def pool_size(top_k, depth):
    return top_k + (depth - 1) * top_k * top_k


def ancestors_visible(parents):
    """parents[i] = index of row i's parent among the rows (-1: none).  Returns boolean [m][m]:
    row i sees row j iff j == i or j is an ancestor of i."""
    m = len(parents)
    vis = np.zeros((m, m), bool)
    for i in range(m):
        j = i
        while j >= 0:
            vis[i, j] = True
            j = int(parents[j])
    return vis


def accept_path(parents, tokens, target_tokens):
    """Rows 0..N of a verified tree (row 0 = root, parents[0] = -1, tokens[i] = token of row i,
    target_tokens[i] = the target's greedy token after row i).  Returns the list of followed rows
    (without the root)."""
    path, cur = [], 0
    while True:
        nxt = [c for c in range(1, len(parents)) if int(parents[c]) == cur and int(tokens[c]) == int(target_tokens[cur])]
        if not nxt:
            return path
        cur = nxt[0]
        path.append(cur)


def sample_tree_tokens(logits, depths, T, u):
    """Acceptance at T > 0 with a tree of DETERMINISTIC candidates (the tree is built from top-k choices, nothing in it
    is drawn).  Section 2.1 describes the T > 0 rule for a chain of drawn drafts; for a tree the paper only reports
    results (Table 2, T = 1), so this is a reading: after every visited row the target DRAWS its next token from
    softmax(logits / T) by inversion, and a candidate child is followed exactly when it is the drawn token.  The
    emitted tokens are then draws from the target's own distribution whatever the tree holds, and with the same
    uniform numbers they are the very tokens token-by-token sampling emits (pinned in the tests).
    One walk visits one row per depth, so row i (depth d_i, the root has depth 0) uses u[d_i].
    Returns the drawn token after every row; accept_path() with these in place of the greedy tokens is the walk."""
    from .hivis import softmax_temperature, sample_inverse_cdf
    return [sample_inverse_cdf(softmax_temperature(np.asarray(logits[i], F64), T), float(u[int(depths[i])])) for i in range(len(depths))]


class HivisTreeOracle(HivisOracle):
    """HivisOracle whose draft round builds a tree.  prefill() is inherited."""

    def tree_draft(self, top_k, depth, n_nodes, follow=None):
        """Builds the pool and picks the candidates.  follow (optional): dict with the choices of
        another implementation, which are then used instead of this oracle's own wherever a choice
        feeds forward: 'pool_tokens' [P], 'expand' [depth-1][k] (pool indices), 'selected' [n_nodes].
        Returns a dict:
          pool_tokens, pool_parents (pool index, -1 = root), pool_scores [P]  (scores: this oracle's)
          expand: list of depth-1 lists of pool indices (the rows expanded at each level, in row order)
          logp:   [1 + (depth-1) k][V] log-probabilities of the row that produced each group of children
          own_top: [1 + (depth-1) k][k] this oracle's own top-k tokens per such row
          selected: sorted pool indices of the candidates
          tokens, parents, depths: the tree rows 1..n_nodes (parents as ROW indices, 0 = root)"""
        k, l = int(top_k), self.l
        P = pool_size(k, depth)
        assert 1 <= n_nodes <= P
        assert self.drafter.kv_len == l
        pool_tok = np.zeros(P, np.int64)
        pool_par = np.full(P, -1, np.int64)
        pool_score = np.zeros(P, F64)
        pool_depth = np.zeros(P, np.int64)
        hid_of = np.zeros(P, np.int64)        # which hidden row's distribution the node was taken from
        H = [np.asarray(self.f_next, F64)]    # hidden rows: f'_1, then the expanded rows level by level
        logp_rows, own_top = [], []

        def children(row, parent, parent_score, dep, first):
            lp = log_softmax(self.target.logits(H[row]))
            top = top_k_lowest(lp, k)
            logp_rows.append(lp)
            own_top.append(top)
            for r in range(k):
                i = first + r
                tok = top[r] if follow is None else int(follow["pool_tokens"][i])
                pool_tok[i], pool_par[i], pool_depth[i], hid_of[i] = tok, parent, dep, row
                pool_score[i] = parent_score + lp[tok]

        children(0, -1, 0.0, 1, 0)
        expand = []
        slot_of = {}                          # pool index -> row among the drafter's tree rows
        level_first, level_n = 0, k
        for j in range(1, depth):
            if follow is None:
                E = [level_first + i for i in top_k_lowest(pool_score[level_first:level_first + level_n], k)]
            else:
                E = [int(e) for e in follow["expand"][j - 1]]
                assert all(level_first <= e < level_first + level_n for e in E) and len(set(E)) == k
            expand.append(E)
            # one drafter pass over the k rows of this level
            u = np.stack([fuse(H[hid_of[e]], self.target.embed([pool_tok[e]])[0], self.w["fuse_w"], self.rho(j)) for e in E])
            n_prev = (j - 1) * k
            vis = np.zeros((k, l + n_prev + k), bool)
            vis[:, :l] = True
            for r, e in enumerate(E):
                slot_of[e] = n_prev + r
                a = e
                while a >= 0:
                    vis[r, l + slot_of[a]] = True
                    a = int(pool_par[a])
            out = self.drafter.forward(u, 0, pos=np.full(k, l + j - 1), visible=vis)
            next_first = level_first + level_n
            for r, e in enumerate(E):
                H.append(out[r])
                children(len(H) - 1, e, pool_score[e], j + 1, next_first + r * k)
            level_first, level_n = next_first, k * k
        if follow is None:
            selected = sorted(top_k_lowest(pool_score, n_nodes))
        else:
            selected = [int(s) for s in follow["selected"]]
            assert selected == sorted(set(selected)) and len(selected) == n_nodes
        row_of = {p: i + 1 for i, p in enumerate(selected)}
        row_of[-1] = 0
        self.tree = {
            "pool_tokens": pool_tok, "pool_parents": pool_par, "pool_scores": pool_score, "pool_depths": pool_depth,
            "expand": expand, "logp": np.stack(logp_rows), "own_top": np.asarray(own_top), "hidden": np.stack(H),
            "selected": selected,
            "tokens": [int(pool_tok[p]) for p in selected],
            "parents": [row_of[int(pool_par[p])] for p in selected],
            "depths": [int(pool_depth[p]) for p in selected],
        }
        return self.tree

    def tree_verify(self):
        """Target pass over [root, candidates].  Returns (g [N+1][d], logits [N+1][V], t [N+1])."""
        t = self.tree
        rows = [self.text[-1]] + t["tokens"]
        parents = [-1] + t["parents"]
        depths = [0] + t["depths"]
        base = self.v + self.l
        m = len(rows)
        vis = np.ones((m, base + m), bool)
        vis[:, base:] = ancestors_visible(parents)
        g = self.target.forward(self.target.embed(rows), 0, pos=base + np.asarray(depths), visible=vis)
        logits = self.target.logits(g)
        return g, logits, [int(x) for x in argmax_lowest(logits)]

    def tree_accept(self, g, t, force=None):
        """Follows the matching path, emits, rolls the state forward.  Returns (n, emitted, path rows).
        force=(path, emitted) replaces this oracle's own decision (follow mode)."""
        tr = self.tree
        path = accept_path([-1] + tr["parents"], [self.text[-1]] + tr["tokens"], t)
        last = path[-1] if path else 0
        emitted = [tr["tokens"][r - 1] for r in path] + [int(t[last])]
        if force is not None:
            path, emitted = [int(r) for r in force[0]], [int(x) for x in force[1]]
        n = len(path)
        base = self.v + self.l
        self.target.keep(list(range(base)) + [base] + [base + r for r in path])
        self.drafter.truncate(self.l)
        self.text = self.text + emitted
        nxt = self.text[self.l + 1: self.l + n + 2]
        self.f_next = self._refeed(np.asarray(g)[[0] + path], nxt, self.l)
        self.l += n + 1
        return n, emitted, path

    def tree_accept_sample(self, g, logits, T, u, force=None):
        """tree_accept with the target's tokens drawn at temperature T (see sample_tree_tokens); u: [depth + 1]."""
        t = sample_tree_tokens(logits, [0] + self.tree["depths"], T, u)
        n, emitted, path = self.tree_accept(g, t, force)
        return n, emitted, path, t

    def tree_cycle(self, top_k, depth, n_nodes):
        tree = self.tree_draft(top_k, depth, n_nodes)
        g, logits, t = self.tree_verify()
        n, emitted, path = self.tree_accept(g, t)
        return {"tree": tree, "g": g, "verify_logits": logits, "target_tokens": t, "n": n, "emitted": emitted, "path": path}
