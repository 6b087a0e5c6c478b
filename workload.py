"""Seeded synthetic inputs shared by the oracle-side tests and the HIP-side tests/bench.

Holds NO arithmetic of the method: only random draws, the storage rounding of
those draws, and the shapes of the workloads.  The inputs stand in for the
paper's LibriSpeech / Whisper / Llama trajectories (Sec. V-A), which are not
available: decoder shapes follow the decoder families the paper names
(TinyLlama-, Llama-7B-class), tree shapes follow its settings (trunk of up to 24
tokens, Sec. IV-A; top-2 alternatives at low-confidence positions, Sec. IV-C
and Sec. V-C).
"""
from concurrent.futures import ThreadPoolExecutor

import numpy as np

MODELS = {
    # tiny fp32 correctness model
    "tiny": dict(n_layers=2, d_model=256, n_heads=4, n_kv_heads=4, head_dim=64, d_ffn=688,
                 vocab=1000, rms_eps=1e-5, rope_theta=10000.0),
    # TinyLlama-class (1.1B)
    "1b": dict(n_layers=22, d_model=2048, n_heads=32, n_kv_heads=4, head_dim=64, d_ffn=5632,
               vocab=32000, rms_eps=1e-5, rope_theta=10000.0),
    # Llama-7B-class
    "7b": dict(n_layers=32, d_model=4096, n_heads=32, n_kv_heads=32, head_dim=128, d_ffn=11008,
               vocab=32000, rms_eps=1e-5, rope_theta=10000.0),
    # Llama/Vicuna-13B-class (the largest target of Sec. V-A)
    "13b": dict(n_layers=40, d_model=5120, n_heads=40, n_kv_heads=40, head_dim=128, d_ffn=13824,
                vocab=32000, rms_eps=1e-5, rope_theta=10000.0),
}

# name -> (model, dtype, n_audio, n_text, tree recipe, base seed)
WORKLOADS = {
    "cfg1_tiny": dict(model="tiny", dtype="f32", n_audio=48, n_text=16, tree="cfg1", seed=1001),
    "cfg2_1b_n16": dict(model="1b", dtype="bf16", n_audio=300, n_text=30,
                        tree=dict(trunk=12, n_branches=2, branch_depth=2, rule="below0.6"),
                        seed=1002),
    "cfg3_7b_n32": dict(model="7b", dtype="bf16", n_audio=750, n_text=60,
                        tree=dict(trunk=16, n_branches=4, branch_depth=4, rule="lowest"),
                        seed=1003),
    "cfg4_1b_b16": dict(model="1b", dtype="bf16", batch=16, prefix_range=(200, 1500),
                        tree=dict(trunk=16, n_branches=2, branch_depth=4, rule="lowest"),
                        seed=1004),
    "cfg5_7b_n64": dict(model="7b", dtype="bf16", n_audio=3000, n_text=200, rounds=20,
                        tree=dict(trunk=24, n_branches=8, branch_depth=5, rule="lowest"),
                        seed=1005),
    # the 13B-class target on config 3's prefix and tree shape
    "cfg6_13b_n32": dict(model="13b", dtype="bf16", n_audio=750, n_text=60,
                         tree=dict(trunk=16, n_branches=4, branch_depth=4, rule="lowest"),
                         seed=1006),
    # draft side (Sec. IV-B): the 1.1B-class draft model on the recycling tree, previous 24-token
    # draft + 12-token regenerated part; same weights as cfg2 (one draft model per system)
    "draft_1b_recycle": dict(model="1b", dtype="bf16", n_audio=300, n_text=30,
                             tree=dict(two_branch=(24, 12)), seed=1002),
}

_LAYER_MATS = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")


def bf16_bits(a):
    """float32 array -> uint16 bf16 bit patterns, round-to-nearest-even (storage rounding)."""
    u = np.ascontiguousarray(a, np.float32).view(np.uint32)
    return ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)).astype(np.uint16)


def bf16_to_f32(b):
    return (np.asarray(b, np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _store(a, dtype):
    return bf16_bits(a) if dtype == "bf16" else np.ascontiguousarray(a, np.float32)


def weight_shapes(cfg):
    d, dq, dkv, F = cfg["d_model"], cfg["n_heads"] * cfg["head_dim"], \
        cfg["n_kv_heads"] * cfg["head_dim"], cfg["d_ffn"]
    return dict(wq=(dq, d), wk=(dkv, d), wv=(dkv, d), wo=(d, dq), w_gate=(F, d), w_up=(F, d),
                w_down=(d, F))


def make_weights(cfg, seed, dtype="f32", n_layers=None, threads=8):
    """Random-init decoder: matrices and embeddings ~ N(0, 0.02); norm gains ~ 1 + N(0, 0.02)
    (gains of N(0, 0.02) would zero the network, all-ones would hide a dropped gain).
    One independent stream per tensor: seed sequence (seed, tensor id)."""
    nl = cfg["n_layers"] if n_layers is None else n_layers
    shapes = weight_shapes(cfg)
    jobs = []  # (key path, shape, kind)
    jobs.append((("tok_embed",), (cfg["vocab"], cfg["d_model"]), "mat"))
    jobs.append((("final_norm",), (cfg["d_model"],), "gain"))
    jobs.append((("lm_head",), (cfg["vocab"], cfg["d_model"]), "mat"))
    for l in range(nl):
        jobs.append((("layers", l, "attn_norm"), (cfg["d_model"],), "gain"))
        jobs.append((("layers", l, "ffn_norm"), (cfg["d_model"],), "gain"))
        for m in _LAYER_MATS:
            jobs.append((("layers", l, m), shapes[m], "mat"))

    def draw(job_id):
        _, shape, kind = jobs[job_id]
        rng = np.random.default_rng([seed, job_id])
        a = rng.standard_normal(shape, dtype=np.float32)
        a *= np.float32(0.02)
        if kind == "gain":
            a += np.float32(1.0)
        return _store(a, dtype)

    with ThreadPoolExecutor(max_workers=threads) as ex:
        arrays = list(ex.map(draw, range(len(jobs))))
    w = {"layers": [dict() for _ in range(nl)]}
    for (path, _, _), a in zip(jobs, arrays):
        if path[0] == "layers":
            w["layers"][path[1]][path[2]] = a
        else:
            w[path[0]] = a
    return w


def make_prefix_inputs(cfg, seed, n_audio, n_text):
    """Audio-embedding vectors ~ N(0,1) in R^d (stand-ins for the projected encoder
    output, Sec. II-A) and uniformly drawn prompt/accepted token ids."""
    rng = np.random.default_rng([seed, 900001])
    audio = rng.standard_normal((n_audio, cfg["d_model"]), dtype=np.float32)
    text = rng.integers(0, cfg["vocab"], size=n_text, dtype=np.int64).astype(np.int32)
    return audio, text


def seeded_cache(cfg, seed, kv_len, capacity, dtype="bf16", batch=1):
    """A directly seeded KV cache, K and V ~ N(0,1) in slots [0, kv_len), zeros beyond.
    Layout [batch][n_layers][n_kv_heads][capacity][head_dim].  The cache is an INPUT of
    the verify step, so both sides are handed the same bits."""
    shape = (batch, cfg["n_layers"], cfg["n_kv_heads"], capacity, cfg["head_dim"])
    out = []
    for t in range(2):
        rng = np.random.default_rng([seed, 900010 + t])
        a = np.zeros(shape, np.float32)
        lens = np.broadcast_to(np.asarray(kv_len), (batch,))
        for b in range(batch):
            a[b, :, :, :lens[b], :] = rng.standard_normal(
                (cfg["n_layers"], cfg["n_kv_heads"], int(lens[b]), cfg["head_dim"]), dtype=np.float32)
        out.append(_store(a, dtype))
    return out[0], out[1]


def tree_cfg1():
    """8 nodes: a 6-token chain plus a 2-token branch forking from the chain node of depth 2."""
    return np.array([-1, 0, 1, 2, 3, 4, 2, 6], np.int32)


def sparse_tree(rng, trunk, n_branches, branch_depth, rule="lowest"):
    """Parent array of a two-pass sparse tree: nodes 0..trunk-1 are the main trunk (node t at
    depth t, node 0 the root = last committed token); each branch is the alternative to a
    low-confidence trunk position p (1 <= p < trunk): its first node hangs off trunk node p-1
    and the rest chain below it.  Confidences are seeded draws: rule "lowest" takes the
    n_branches smallest of U(0,1) draws; rule "below0.6" plants exactly n_branches positions
    with U(0,0.6) among U(0.6,1) others.  Returns (parents, branch_positions, confidences)."""
    pos = np.arange(1, trunk)
    if rule == "below0.6":
        low = np.sort(rng.choice(pos, size=n_branches, replace=False))
        conf = rng.uniform(0.6, 1.0, size=trunk)
        conf[low] = rng.uniform(0.0, 0.6, size=n_branches)
    else:
        conf = rng.uniform(0.0, 1.0, size=trunk)
        low = np.sort(pos[np.argsort(conf[1:], kind="stable")[:n_branches]])
    conf[0] = 1.0
    parents = list(range(-1, trunk - 1))
    for p in low:
        parents.append(int(p) - 1)
        for _ in range(branch_depth - 1):
            parents.append(len(parents) - 1)
    return np.array(parents, np.int32), low.astype(np.int32), conf


def tree_tokens(rng, parents, vocab):
    """Uniform draft tokens; siblings are made distinct (top-1 vs top-2 alternatives differ)."""
    n = len(parents)
    tok = rng.integers(0, vocab, size=n, dtype=np.int64).astype(np.int32)
    for i in range(1, n):
        sib = {int(tok[j]) for j in range(i) if parents[j] == parents[i]}
        while int(tok[i]) in sib:
            tok[i] = (tok[i] + 1) % vocab
    return tok


def random_tree(rng, n, max_children=2):
    """Random parent array in topological order (for property tests)."""
    parents = [-1]
    kids = [0]
    for i in range(1, n):
        cand = [j for j in range(i) if kids[j] < max_children]
        p = int(rng.choice(cand))
        parents.append(p)
        kids[p] += 1
        kids.append(0)
    return np.array(parents, np.int32)


def two_branch_tree(len_old, len_new):
    """Parent array of the draft model's recycling tree (Sec. IV-B): node 0 is the last verified
    token; nodes 1..len_old chain below it (the previous draft, kept as sequence 1); nodes
    len_old+1..len_old+len_new chain below node 0 as well (the part being regenerated, sequence
    2).  The two branches never see each other."""
    parents = [-1]
    for i in range(len_old):
        parents.append(i)                       # node i+1 hangs off node i
    for i in range(len_new):
        parents.append(0 if i == 0 else len_old + i)
    return np.array(parents, np.int32)


def make_tree(name, rng=None):
    """(parents, tokens) of a named workload's tree."""
    wl = WORKLOADS[name]
    cfg = MODELS[wl["model"]]
    rng = rng if rng is not None else np.random.default_rng([wl["seed"], 900020])
    if wl["tree"] == "cfg1":
        parents = tree_cfg1()
    elif "two_branch" in wl["tree"]:
        parents = two_branch_tree(*wl["tree"]["two_branch"])
    else:
        t = wl["tree"]
        parents, _, _ = sparse_tree(rng, t["trunk"], t["n_branches"], t["branch_depth"], t["rule"])
    return parents, tree_tokens(rng, parents, cfg["vocab"])


def planted_logits(rng, parents, tokens, vocab, p_trunk=0.9, p_branch=2.0 / 3.0, trunk=None):
    """Seeded [n, vocab] float32 logits ~ N(0,1) with +10 at one planted target token per node,
    for driving acceptance without a trained model: the planted target of a trunk node equals
    its trunk child's token with probability p_trunk (the paper reports a 94.4 % per-round
    decoding-acceptance ratio, Sec. V-B); when it does not and the node also has a branch
    child, the branch child's token is planted with probability p_branch (more than 2/3 of
    top-1 failures are the rank-2 token, Sec. V-C).  Otherwise a random token."""
    n = len(parents)
    lg = rng.standard_normal((n, vocab), dtype=np.float32)
    kids = [[] for _ in range(n)]
    for i in range(1, n):
        kids[parents[i]].append(i)
    for i in range(n):
        target = int(rng.integers(0, vocab))
        if kids[i]:
            first = kids[i][0]
            u = rng.uniform()
            if u < p_trunk:
                target = int(tokens[first])
            elif len(kids[i]) > 1 and rng.uniform() < p_branch:
                target = int(tokens[kids[i][1]])
        lg[i, target] += np.float32(10.0)
    return lg
