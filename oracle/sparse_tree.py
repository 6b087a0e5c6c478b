"""Draft-side control of one SpecASR round, written out plainly -- TEST INFRASTRUCTURE, not the product.

What is defined here (paper Sec. IV; the places where the paper gives no number or order are the
readings listed in the design notes, repeated next to the step that takes them):

* adaptive single-sequence prediction (Sec. IV-A): greedy drafting of a trunk of at most
  ``max_draft`` tokens, cut short at the first token whose normalised logit is below a threshold;
* draft sequence recycling, merging stage (Sec. IV-B): every newly drafted trunk token is compared
  with the tokens kept from the previous round at the corresponding or an adjacent position; on a
  match the kept tokens behind the match are reused without running the draft model;
* two-pass sparse-tree prediction (Sec. IV-C): uncertain trunk positions are marked together with
  the token of second highest probability; a second pass grows one branch per mark and stops a
  branch as soon as it can be concatenated to the trunk.

The draft model enters only as a function ``read_out(path) -> (top1, top2, prob)``: the two most
probable next tokens after the token sequence ``path`` (root first) and the probability of the
first.  A causal model's read-out of a node depends on its root path only, so a table keyed by
paths is a complete recording of a model.  Nothing here computes logits.

Output format: ``tokens[i]``, ``parents[i]`` with node 0 the root (the last committed token),
trunk nodes first and in order, then the first node of every branch in trunk order, then the
branches level by level.
"""
from dataclasses import dataclass, field


@dataclass
class Params:
    max_draft: int = 24        # Sec. IV-A: maximum prediction length
    threshold: float = 0.4     # Sec. IV-A / Sec. V-C: truncation threshold on the normalised logit
    mode: str = "tsp"          # "asp": truncate at the uncertain token; "tsp": mark it and go on
    max_branches: int = 8      # branches of the sparse tree (the workloads use up to 8)
    branch_depth: int = 5      # nodes per branch at most
    max_nodes: int = 64        # one verification pass takes at most 64 tree nodes
    recycle: bool = True


@dataclass
class Round:
    tokens: list
    parents: list
    trunk: list                                   # node index of trunk position 0, 1, ...
    marks: list = field(default_factory=list)     # (trunk position, second token, probability)
    recycled: int = 0                             # trunk tokens taken from the kept suffix
    read_outs: int = 0                            # nodes whose read-out was consulted


def root_path(tokens, parents, node):
    """Token sequence from the root to ``node``."""
    out = []
    while node >= 0:
        out.append(tokens[node])
        node = parents[node]
    return tuple(reversed(out))


def build_round(read_out, root, pos0, kept, prm):
    """One round of drafting.  ``root``: last committed token, at absolute position ``pos0``;
    ``kept``: {absolute position: token} of the previous round's rejected trunk suffix."""
    tokens, parents, trunk = [int(root)], [-1], [0]
    rnd = Round(tokens, parents, trunk)
    kept = dict(kept) if prm.recycle else {}

    def full():
        return len(tokens) >= prm.max_nodes

    def consult(node):
        rnd.read_outs += 1
        t1, t2, p = read_out(root_path(tokens, parents, node))
        return int(t1), int(t2), float(p)

    # ---- first pass: the trunk (Sec. IV-A) ---------------------------------------------------
    while len(trunk) - 1 < prm.max_draft and not full():
        t1, t2, p = consult(trunk[-1])
        tokens.append(t1)
        parents.append(trunk[-1])
        trunk.append(len(tokens) - 1)
        k = len(trunk) - 1                        # trunk position of the new token
        uncertain = p < prm.threshold             # strictly below: a token AT the threshold is kept as certain
        # Sec. IV-C: instead of truncating, remember the position and the second candidate
        if uncertain and prm.mode == "tsp" and t2 >= 0:
            rnd.marks.append((k, t2, p))
        # Sec. IV-B, merging: compare with the kept tokens at the corresponding position first,
        # then one position earlier, then one later (the paper's "adjacent" read as +-1).  On a
        # match the kept tokens that FOLLOW the matching one continue the trunk, position by
        # position while they are contiguous; the kept suffix is used at most once.
        pos = pos0 + k
        for q in (pos, pos - 1, pos + 1):
            if kept.get(q) == t1:
                q += 1
                while q in kept and len(trunk) - 1 < prm.max_draft and not full():
                    tokens.append(kept[q])
                    parents.append(trunk[-1])
                    trunk.append(len(tokens) - 1)
                    rnd.recycled += 1
                    q += 1
                kept = {}
                break
        # Sec. IV-A: the uncertain token itself is part of the draft (it may still be right);
        # drafting stops behind it and the draft goes to verification early
        if uncertain and prm.mode == "asp":
            break

    # ---- second pass: branches at the marked positions (Sec. IV-C) ---------------------------
    if prm.mode == "tsp" and rnd.marks:
        least = sorted(rnd.marks, key=lambda m: m[2])[:prm.max_branches]   # the least confident positions
        branches = []                             # [leaf node, nodes in the branch, trunk position of its first node]
        for k, alt, _ in sorted(least):           # in trunk order
            if full() or alt == tokens[trunk[k]]:
                continue
            tokens.append(alt)                    # the alternative to trunk token k hangs off trunk token k-1
            parents.append(trunk[k - 1])
            branches.append([len(tokens) - 1, 1, k])
        while branches and not full():
            branches = [b for b in branches if b[1] < prm.branch_depth]
            grown = []
            for leaf, size, k in branches:
                if full():
                    break
                t1, _, _ = consult(leaf)
                at = k + size                     # trunk position the branch's next token corresponds to
                # can the branch be concatenated to the trunk?  Same token at the corresponding
                # trunk position, else one later, else one earlier (never the root)
                join = next((q for q in (at, at + 1, at - 1)
                             if 0 < q < len(trunk) and tokens[trunk[q]] == t1), None)
                if join is None:
                    tokens.append(t1)
                    parents.append(leaf)
                    grown.append([len(tokens) - 1, size + 1, k])
                    continue
                # yes: it is not extended by the draft model any further; the trunk's tokens from
                # the joining position on are appended below it, up to the branch size
                node = leaf
                for q in range(join, len(trunk)):
                    if size >= prm.branch_depth or full():
                        break
                    tokens.append(tokens[trunk[q]])
                    parents.append(node)
                    node = len(tokens) - 1
                    size += 1
            branches = grown
    return rnd


def kept_after(trunk_tokens, pos0, accept_len):
    """What a round keeps for the next one (Sec. IV-B, first stage: the complete draft is retained
    next to the verified part).  Trunk position i sits at absolute position pos0 + i; the accepted
    path fills positions pos0 .. pos0 + accept_len - 1 and the target's own token takes position
    pos0 + accept_len, so the trunk tokens behind that position are the ones worth comparing with."""
    return {pos0 + i: int(trunk_tokens[i]) for i in range(accept_len + 1, len(trunk_tokens))}


def path_set(tokens, parents):
    """The tree as the set of its root-to-node token sequences (independent of node numbering)."""
    return {root_path(tokens, parents, i) for i in range(len(tokens))}
