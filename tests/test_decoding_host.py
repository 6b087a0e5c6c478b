"""Host logic of the draft-then-verify loop (paper_2507_18181_amd.decoding) without a GPU: the two
models are replaced by toy stand-ins with the Verifier's interface whose "networks" are
deterministic functions of the token context, so that every property of the orchestration can be
checked exactly: the output is the target's greedy decoding (Sec. II-B: lossless), every round's
tree is the one the oracle's constructor builds from the same read-outs (Sec. IV-A/B/C), and the
draft-side cache bookkeeping -- commit one step behind the target, accepted tokens without a
draft-side row riding in front of the next tree -- never loses or duplicates a token."""
import hashlib

import numpy as np
import pytest
import torch

import oracle
from oracle import sparse_tree as ost
from paper_2507_18181_amd.decoding import SpecDecoder

VOCAB = 11


def _h(*parts):
    return int.from_bytes(hashlib.sha256(repr(parts).encode()).digest()[:8], "little")


def target_next(ctx):
    """The toy target's greedy token after a context (depends on the last three tokens)."""
    return _h("t", tuple(ctx[-3:])) % VOCAB


def draft_readout(ctx, agree):
    """The toy draft's (top1, top2, prob): agrees with the target in `agree` of 8 contexts; when it
    does not, the target's token is its second candidate half of the time."""
    t = target_next(ctx)
    r = _h("d", tuple(ctx[-4:]))
    right = r % 8 < agree
    t1 = t if right else (t + 1 + r // 8 % (VOCAB - 1)) % VOCAB
    t2 = ((t1 + 1 + r // 97 % (VOCAB - 1)) % VOCAB) if right or r // 11 % 2 else t
    return t1, t2, (r // 1000 % 1000) / 1000.0


class Toy:
    """Verifier look-alike.  `ctx` plays the KV cache: the committed tokens, one per position."""

    def __init__(self, prefix, agree=8, capacity=4000, max_nodes=64):
        self.ctx = list(prefix)
        self.kv_len = np.array([len(prefix)], np.int32)
        self.max_nodes, self.batch, self.capacity, self.agree = max_nodes, 1, capacity, agree
        self.rows = None                      # token of every node that has a row after the last forward
        self.forwards = 0

    def _paths(self, tokens, parents):
        out = []
        for i in range(len(tokens)):
            p, j = [], i
            while j >= 0:
                p.append(int(tokens[j]))
                j = int(parents[j])
            out.append(self.ctx + p[::-1])
        return out

    def _check_tree(self, tokens, parents):
        n = len(tokens)
        assert 1 <= n <= self.max_nodes and parents[0] == -1 and all(0 <= parents[i] < i for i in range(1, n))
        assert self.kv_len[0] == len(self.ctx) and len(self.ctx) + n <= self.capacity

    def tree_forward_top2(self, tokens, parents, **kw):
        tok, par = np.asarray(tokens[0]), np.asarray(parents[0])
        self._check_tree(tok, par)
        self.forwards += 1
        self.rows = [int(t) for t in tok]
        top2 = torch.full((1, self.max_nodes, 2), -7, dtype=torch.int32)
        prob = torch.full((1, self.max_nodes), -1.0)
        for i, ctx in enumerate(self._paths(tok, par)):
            t1, t2, p = draft_readout(ctx, self.agree)
            top2[0, i, 0], top2[0, i, 1], prob[0, i] = t1, t2, p
        return dict(status=0, top2=top2, prob=prob)

    def verify_tree(self, tokens, parents, **kw):
        tok, par = np.asarray(tokens[0], np.int32), np.asarray(parents[0], np.int32)
        self._check_tree(tok, par)
        amax = np.array([target_next(c) for c in self._paths(tok, par)], np.int32)
        path, alen, nxt = oracle.accept(tok, par, amax)
        self.ctx += [int(tok[v]) for v in path]
        self.kv_len[0] += alen
        full = np.full((1, self.max_nodes), -1, np.int32)
        full[0, :alen] = path
        return dict(status=0, accept_len=np.array([alen]), path=full, next_token=np.array([nxt]))

    def commit(self, n_nodes, paths, **kw):
        path = list(paths[0])
        assert self.rows is not None and n_nodes[0] == len(self.rows), "commit must name the tree of the last forward"
        assert path[0] == 0 and all(a < b for a, b in zip(path, path[1:])) and path[-1] < n_nodes[0]
        self.ctx += [self.rows[v] for v in path]      # only nodes that HAVE a row can be committed
        self.kv_len[0] += len(path)
        self.rows = None
        return 0


def greedy(prefix, root, n):
    ctx, out = list(prefix) + [root], []
    for _ in range(n):
        out.append(target_next(ctx))
        ctx.append(out[-1])
    return out


@pytest.mark.parametrize("mode", ["asp", "tsp"])
@pytest.mark.parametrize("agree", [8, 6, 3, 0])
@pytest.mark.parametrize("threshold", [0.0, 0.3, 0.9])
def test_loop_is_lossless_follows_the_constructor_and_keeps_both_caches_in_step(mode, agree, threshold):
    prefix, root, n_new = [1, 2, 3, 4, 5], 6, 300
    target, draft = Toy(prefix), Toy(prefix, agree=agree)
    sd = SpecDecoder(target, draft, root=root, threshold=threshold, mode=mode, max_draft=24)
    sd.trace = []
    out = []
    while len(out) < n_new:
        got = sd.round()
        out += got
        # both caches hold the same tokens, the draft's short by the pending ones -- and the next
        # root is the token the target produced last
        assert draft.ctx + sd.pending == target.ctx
        assert target.ctx == prefix + [root] + out[:-1] and sd.root == out[-1]
        assert len(sd.pending) <= sd.max_pending
    assert out[:n_new] == greedy(prefix, root, n_new)
    for t in sd.trace:
        prm = ost.Params(max_draft=24, threshold=threshold, mode=mode, max_branches=sd.max_branches,
                         branch_depth=sd.branch_depth, max_nodes=t["max_nodes"], recycle=True)
        r = ost.build_round(lambda path: t["read"][path], t["root"], t["pos0"], t["kept"], prm)
        assert (r.tokens, r.parents, r.trunk) == (t["tokens"], t["parents"], t["trunk"])
        assert ost.kept_after([t["tokens"][v] for v in t["trunk"]], t["pos0"], t["accept_len"]) == t["kept_out"]
    st = sd.stats
    if agree == 8 and threshold == 0.0:
        # a perfect, always-confident draft: 24 drafts accepted per round, one draft forward per drafted token
        assert all(a == 24 for a in st.accepted) and st.draft_forwards <= 24 * st.rounds + st.rounds
    if agree == 0:
        assert max(st.accepted) <= 1 or mode == "tsp"


def test_catch_up_when_many_accepted_tokens_have_no_draft_side_row():
    """A kept suffix that is reused wholesale puts up to 23 tokens into the tree without a draft
    forward; when the target accepts them all, the draft side catches up with one forward over the
    pending chain instead of carrying them into the next tree."""
    prefix, root = [1, 2, 3], 4
    target, draft = Toy(prefix), Toy(prefix, agree=8)
    sd = SpecDecoder(target, draft, root=root, threshold=0.0, mode="asp", max_draft=20)   # the reuse fills the draft
    want = greedy(prefix, root, 60)
    # pretend the previous round left the target's own continuation as the kept suffix
    pos0 = len(prefix)
    sd.kept = {pos0 + 1 + i: want[i] for i in range(0, 20)}
    f0 = draft.forwards
    got = sd.round()
    assert got == want[:len(got)] and len(got) == 21                     # 20 drafts accepted + the target's own token
    assert sd.stats.recycled == 19 and draft.forwards - f0 == 1 + 1     # one drafted token, then the catch-up
    assert sd.pending == [] and draft.ctx == target.ctx
