"""Draft-then-verify decoding loop of SpecASR (Sec. IV) on top of the C ABI.

Host-side orchestration only: every model evaluation is a call into libspecasr.so through two
``runtime.Verifier`` objects -- the draft model (``specasr_tree_forward_top2``: per node the two
most probable ids and the probability of the first) and the target model
(``specasr_verify_tree``: greedy acceptance of the longest matching path, in-place commit).

One round (Sec. IV-A, IV-C, IV-B):

1. *Trunk* (adaptive single-sequence prediction).  The draft model extends a chain below the
   root (the last committed token, whose K/V is not cached yet) by its greedy token, up to
   ``max_draft`` tokens.  A token whose probability is below ``threshold`` is uncertain: in mode
   ``"asp"`` drafting stops there and the draft is verified early; in mode ``"tsp"`` the position
   is marked together with the token of second highest probability and drafting goes on.
2. *Branches* (two-pass sparse tree, mode ``"tsp"``).  Every marked position gets a sibling
   holding the second token; all open branches are extended together, one draft forward per
   level (the draft model sees the tree through the same ancestor mask as the target).  A
   branch whose next token equals the trunk's token at the same or an adjacent position is not
   extended any further: the rest of the trunk is appended to it instead (no draft steps).
3. *Verification.*  The target verifies the whole tree in one pass; the accepted path is
   committed in both caches; the target's own token after the last accepted node becomes the
   next root.  The output therefore equals the target's greedy decoding, whatever the draft.
4. *Recycling.*  The part of the trunk behind the failed position is kept.  While the next trunk
   is drafted, each new token is compared with the kept tokens at the corresponding and the two
   adjacent positions; on a match the kept tokens behind the match are appended to the new
   trunk without running the draft model for them.

The draft model runs on the whole current tree at every step (its cost is the weight stream,
which does not depend on the number of rows), so no draft-side cache state has to be rolled
back: tree rows live in scratch slots until ``commit``.

Tokens that are appended to the tree behind the last draft forward of a round (the last trunk
token, recycled tokens, the last level of the branches) have no draft-side K/V row when the
target accepts them.  No extra forward is spent on them: they stay *pending* and ride in front
of the next round's tree as a chain (pending tokens -> root -> ...), so that the next round's
first draft forward computes their rows, and the draft cache is committed one step behind the
target's: ``draft.kv_len + len(pending) == target.kv_len``.
"""
import numpy as np


class RoundStats:
    def __init__(self):
        self.rounds = 0
        self.draft_forwards = 0
        self.accepted = []        # accepted draft tokens per round (root excluded)
        self.tree_nodes = []
        self.branch_hits = 0      # rounds whose accepted path leaves the trunk
        self.recycled = 0         # draft tokens taken from the previous round's rejected suffix


class SpecDecoder:
    """target, draft: ``Verifier`` objects for one sequence each (batch 1, max_nodes 64, same
    vocabulary) whose caches already hold the same prefix; ``root`` is the last committed token
    (not yet cached on either side)."""

    def __init__(self, target, draft, root, max_draft=24, threshold=0.4, mode="tsp",
                 max_branches=8, branch_depth=5, recycle=True):
        assert mode in ("asp", "tsp")
        assert target.batch == 1 and draft.batch == 1
        assert target.kv_len[0] == draft.kv_len[0], "both caches must hold the same prefix"
        self.t, self.d = target, draft
        self.root = int(root)
        self.max_draft, self.threshold, self.mode = max_draft, threshold, mode
        self.max_branches, self.branch_depth, self.recycle = max_branches, branch_depth, recycle
        self.max_nodes = min(target.max_nodes, draft.max_nodes)
        self.max_pending = 8      # more accepted tokens than this without a draft-side row: catch up at once
        self.pending = []         # accepted tokens whose draft-side K/V row is still to be computed
        self._fresh = 0           # nodes of the current tree that the last draft forward covered
        self._cap = self.max_nodes
        self.kept = {}            # absolute position -> token of the previous round's rejected suffix
        self.stats = RoundStats()
        # Optional recording for tests: set to a list and every round appends a dict with its
        # inputs (root, pos0, kept), its tree and the draft read-out of every node it consulted,
        # keyed by the node's root path (a causal model's read-out depends on nothing else).
        self.trace = None
        self._read = {}

    # -- draft side ---------------------------------------------------------------------------
    def _draft_forward(self, tokens, parents):
        """Draft forward over [pending chain -> tree]; returns the read-out of the tree's nodes."""
        P = len(self.pending)
        dt = list(self.pending) + list(tokens)
        dp = list(range(-1, P - 1)) + [P - 1] + [P + q for q in parents[1:]]
        out = self.d.tree_forward_top2([np.asarray(dt, np.int32)], [np.asarray(dp, np.int32)])
        if out["status"] != 0:
            raise RuntimeError("draft forward failed: status %d" % out["status"])
        self.stats.draft_forwards += 1
        self._fresh = len(tokens)                     # these nodes (and the pending ones) now have a draft-side K/V row
        top2, prob = out["top2"][0, P:].cpu().numpy(), out["prob"][0, P:].cpu().numpy()
        if self.trace is not None:
            for i in range(len(tokens)):
                path, j = [], i
                while j >= 0:
                    path.append(int(tokens[j]))
                    j = parents[j]
                self._read[tuple(reversed(path))] = (int(top2[i, 0]), int(top2[i, 1]), float(prob[i]))
        return top2, prob

    def _build_tree(self):
        """Returns (tokens, parents, trunk node ids)."""
        pos0 = int(self.t.kv_len[0])                  # absolute position of the root
        tokens, parents, trunk = [self.root], [-1], [0]
        marks = []                                    # (index into trunk, second token, probability)
        self._fresh = 0
        # the pending chain shares the draft model's tree with this round's nodes
        self._cap = min(self.t.max_nodes, self.d.max_nodes - len(self.pending))
        while len(trunk) - 1 < self.max_draft and len(tokens) < self._cap:
            top2, prob = self._draft_forward(tokens, parents)
            leaf = trunk[-1]
            t1, t2, p = int(top2[leaf, 0]), int(top2[leaf, 1]), float(prob[leaf])
            tokens.append(t1)
            parents.append(leaf)
            trunk.append(len(tokens) - 1)
            uncertain = p < self.threshold
            if uncertain and self.mode == "tsp" and t2 >= 0:
                marks.append((len(trunk) - 1, t2, p))
            # recycling: the kept tokens at the corresponding or an adjacent position
            pos = pos0 + len(trunk) - 1
            hit = next((q for q in (pos, pos - 1, pos + 1) if self.kept.get(q) == t1), None)
            if self.recycle and hit is not None:
                q = hit + 1
                while q in self.kept and len(trunk) - 1 < self.max_draft and len(tokens) < self._cap:
                    tokens.append(self.kept[q])
                    parents.append(trunk[-1])
                    trunk.append(len(tokens) - 1)
                    self.stats.recycled += 1
                    q += 1
                self.kept = {}
            if uncertain and self.mode == "asp":
                break
        self.kept = {}
        if self.mode == "tsp" and marks:
            self._grow_branches(tokens, parents, trunk, marks)
        return tokens, parents, trunk

    def _grow_branches(self, tokens, parents, trunk, marks):
        marks = sorted(marks, key=lambda m: m[2])[:self.max_branches]      # least confident first
        open_ = []                                    # [leaf node, depth in branch, trunk index of its first node]
        for k, alt, _ in sorted(marks):
            if len(tokens) >= self._cap or alt == tokens[trunk[k]]:
                continue
            tokens.append(alt)
            parents.append(trunk[k - 1])
            open_.append([len(tokens) - 1, 1, k])
        while open_ and len(tokens) < self._cap:
            open_ = [b for b in open_ if b[1] < self.branch_depth]
            if not open_:
                break
            top2, _ = self._draft_forward(tokens, parents)
            still = []
            for leaf, depth, k in open_:
                if len(tokens) >= self._cap:
                    break
                t1 = int(top2[leaf, 0])
                pos = k + depth                        # trunk index the next token corresponds to
                join = next((q for q in (pos, pos + 1, pos - 1)
                             if 0 < q < len(trunk) and tokens[trunk[q]] == t1), None)
                if join is not None:                   # concatenate the rest of the trunk, then close
                    node = leaf
                    for q in range(join, len(trunk)):
                        if depth >= self.branch_depth or len(tokens) >= self._cap:
                            break
                        tokens.append(tokens[trunk[q]])
                        parents.append(node)
                        node = len(tokens) - 1
                        depth += 1
                    continue
                tokens.append(t1)
                parents.append(leaf)
                still.append([len(tokens) - 1, depth + 1, k])
            open_ = still

    # -- one round ----------------------------------------------------------------------------
    def round(self):
        """Drafts a tree, verifies it, commits the accepted path on both sides.  Returns the tokens
        this round adds to the output: the accepted draft tokens, then the target's own token."""
        pos0 = int(self.t.kv_len[0])
        kept_in, self._read = dict(self.kept), {}
        recycled_before = self.stats.recycled
        tokens, parents, trunk = self._build_tree()
        n = len(tokens)
        out = self.t.verify_tree([np.asarray(tokens, np.int32)], [np.asarray(parents, np.int32)])
        if out["status"] != 0:
            raise RuntimeError("verify failed: status %d" % out["status"])
        alen = int(out["accept_len"][0])
        path = [int(v) for v in out["path"][0, :alen]]
        nxt = int(out["next_token"][0])
        # draft side: commit the pending chain and the accepted nodes the last draft forward covered
        # (a node appended behind it has no row, nor has anything below it: they form the path's
        # tail); the tail waits in front of the next round's tree
        P = len(self.pending)
        fresh = [v for v in path if v < self._fresh]
        assert path[:len(fresh)] == fresh
        if self.d.commit([P + self._fresh], [list(range(P)) + [P + v for v in fresh]]) != 0:
            raise RuntimeError("draft commit failed")
        self.pending = [tokens[v] for v in path[len(fresh):]]
        if len(self.pending) > self.max_pending:
            self._catch_up()
        assert self.d.kv_len[0] + len(self.pending) == self.t.kv_len[0] == pos0 + alen
        st = self.stats
        st.rounds += 1
        st.accepted.append(alen - 1)
        st.tree_nodes.append(n)
        st.branch_hits += int(any(v not in trunk for v in path))
        # keep the trunk behind the failure: trunk node i sits at absolute position pos0 + i; the
        # path covers positions pos0 .. pos0+alen-1, the target's token takes pos0+alen
        if self.recycle:
            self.kept = {pos0 + i: tokens[trunk[i]] for i in range(alen + 1, len(trunk))}
        if self.trace is not None:
            self.trace.append(dict(root=tokens[0], pos0=pos0, kept=kept_in, max_nodes=self._cap, tokens=list(tokens),
                                   parents=list(parents), trunk=list(trunk), read=self._read,
                                   accept_len=alen, path=path, kept_out=dict(self.kept),
                                   recycled=self.stats.recycled - recycled_before))
        self.root = nxt
        return [tokens[v] for v in path[1:]] + [nxt]

    def _catch_up(self):
        """One draft forward over the pending tokens alone (a chain), committed at once."""
        n = len(self.pending)
        out = self.d.tree_forward_top2([np.asarray(self.pending, np.int32)], [np.arange(-1, n - 1, dtype=np.int32)])
        if out["status"] != 0 or self.d.commit([n], [list(range(n))]) != 0:
            raise RuntimeError("draft catch-up failed")
        self.stats.draft_forwards += 1
        self.pending = []

    def decode(self, n_new):
        """Runs rounds until at least n_new tokens are produced (or the cache is full)."""
        out = []
        cap = min(self.t.capacity, self.d.capacity)
        while len(out) < n_new and int(self.t.kv_len[0]) + self.max_nodes <= cap:
            out.extend(self.round())
        return out
