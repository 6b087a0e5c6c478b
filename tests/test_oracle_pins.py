"""Pins for the CPU oracle: closed forms, textbook special cases, brute force, invariants.

The paper prints no worked numeric example, so the oracle is pinned by what the
method and the mathematics fix (each test names what it would catch).
"""
import itertools
import math

import numpy as np
import pytest

import oracle
from oracle import form_s
import workload as wl

TINY = dict(n_layers=2, d_model=32, n_heads=4, n_kv_heads=2, head_dim=8, d_ffn=40, vocab=17,
            rms_eps=1e-5, rope_theta=10000.0)


def _boost(w, s):
    """Scale the matrices of an f32 model (tests only) so attention is peaked and SiLU nonlinear."""
    for lw in w["layers"]:
        for m in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down"):
            lw[m] = (lw[m] * np.float32(s)).astype(np.float32)
    w["lm_head"] = (w["lm_head"] * np.float32(s)).astype(np.float32)
    w["tok_embed"] = (w["tok_embed"] * np.float32(s)).astype(np.float32)
    return w


def _prefill(om, cfg, audio, text, cap):
    kc, vc = om.empty_cache(cap)
    L, last = om.prefill(kc, vc, 0, audio.astype(np.float64), text)
    return kc, vc, L, last


def _prefix_rows(cfg, w, audio, text):
    E = form_s.widen(w["tok_embed"])
    return np.concatenate([audio.astype(np.float64), E[text]], axis=0)


# --------------------------------------------------------------------------- primitives

def test_rmsnorm_closed_forms():
    # constant vector: every element becomes g * c / sqrt(c^2 + eps)
    g = np.linspace(0.5, 1.5, 7)
    y = oracle.rmsnorm(np.full(7, -3.0), g, 1e-5)
    assert np.allclose(y, g * (-3.0) / math.sqrt(9.0 + 1e-5), rtol=0, atol=1e-15)
    # 3-4-5: mean square 12.5
    y = oracle.rmsnorm(np.array([3.0, 4.0]), np.ones(2), 0.0)
    assert np.allclose(y, np.array([3.0, 4.0]) / math.sqrt(12.5), atol=1e-15)
    # eps sits inside the root, next to the MEAN (not the sum) of squares
    y = oracle.rmsnorm(np.array([1.0, 1.0, 1.0, 1.0]), np.ones(4), 3.0)
    assert np.allclose(y, 0.5, atol=1e-15)


def test_rope_closed_forms():
    rng = np.random.default_rng(1)
    x = rng.standard_normal(16)
    assert np.array_equal(oracle.rope(x, 0, 10000.0), x)            # position 0 is the identity
    # hd = 2: a plain rotation by pos radians (theta^0 = 1)
    y = oracle.rope(np.array([1.0, 0.0]), 3, 10000.0)
    assert np.allclose(y, [math.cos(3.0), math.sin(3.0)], atol=1e-15)
    # hd = 4: second pair (1, 3) turns by pos * theta^(-1/2) = pos / 100
    y = oracle.rope(np.array([0.0, 1.0, 0.0, 0.0]), 7, 10000.0)
    assert np.allclose(y, [0.0, math.cos(0.07), 0.0, math.sin(0.07)], atol=1e-15)
    # norm is preserved; <R_m q, R_n k> depends on m - n only
    q, k = rng.standard_normal(16), rng.standard_normal(16)
    assert np.isclose(np.linalg.norm(oracle.rope(q, 911, 10000.0)), np.linalg.norm(q))
    a = oracle.rope(q, 40, 1e4) @ oracle.rope(k, 33, 1e4)
    b = oracle.rope(q, 840, 1e4) @ oracle.rope(k, 833, 1e4)
    assert np.isclose(a, b, atol=1e-12)
    c = oracle.rope(q, 40, 1e4) @ oracle.rope(k, 34, 1e4)
    assert not np.isclose(a, c, atol=1e-6)
    # complex-multiplication form of the same rotation
    half = 8
    z = (x[:half] + 1j * x[half:]) * np.exp(1j * 5 * 10000.0 ** (-np.arange(half) * 2.0 / 16))
    assert np.allclose(oracle.rope(x, 5, 1e4), np.concatenate([z.real, z.imag]), atol=1e-14)


def test_softmax_and_silu_closed_forms():
    assert np.allclose(oracle.softmax(np.zeros(5)), 0.2, atol=1e-16)
    assert np.allclose(oracle.softmax(np.array([0.0, math.log(3.0)])), [0.25, 0.75], atol=1e-15)
    s = np.array([1.0, -2.0, 0.5, 700.0])
    p = oracle.softmax(s)
    assert np.isfinite(p).all() and np.isclose(p.sum(), 1.0)
    assert np.allclose(oracle.softmax(s[:3] + 123.0), oracle.softmax(s[:3]), atol=1e-13)
    assert oracle.silu(0.0) == 0.0
    assert np.isclose(oracle.silu(math.log(3.0)), math.log(3.0) * 0.75, atol=1e-15)
    for z in (0.3, 2.0, 9.0):
        assert np.isclose(oracle.silu(z) - oracle.silu(-z), z, atol=1e-14)


def test_tree_meta_against_parent_walk():
    rng = np.random.default_rng(2)
    for n in (1, 2, 7, 33, 64):
        par = wl.random_tree(rng, n, max_children=3)
        depth, anc = oracle.tree_meta(par)
        for i in range(n):
            path = form_s.root_path(par, i)
            assert depth[i] == len(path) - 1
            assert sorted(np.nonzero(anc[i])[0].tolist()) == sorted(path)
    for bad in ([0], [-1, 1], [-1, 0, 5], [-1, -1]):
        with pytest.raises(ValueError):
            oracle.tree_meta(np.array(bad, np.int32))


# --------------------------------------------------------------------------- form S itself

def test_form_s_against_torch_library_ops():
    """The numpy causal decoder equals one assembled from torch's library routines
    (rms_norm, linear, scaled_dot_product_attention(is_causal), silu) in float64."""
    import torch
    import torch.nn.functional as F
    cfg = dict(TINY)
    w = _boost(wl.make_weights(cfg, 11, "f32"), 6.0)
    rng = np.random.default_rng(3)
    T = 13
    x_in = rng.standard_normal((T, cfg["d_model"]))
    ref = form_s.causal_decoder(cfg, w, x_in)

    H, Hkv, hd = cfg["n_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    t = lambda a: torch.from_numpy(form_s.widen(a))
    pos = torch.arange(T, dtype=torch.float64)
    inv = 1.0 / (cfg["rope_theta"] ** (torch.arange(0, hd, 2, dtype=torch.float64) / hd))
    ang = torch.outer(pos, inv)
    cos, sin = torch.cat([ang.cos(), ang.cos()], -1), torch.cat([ang.sin(), ang.sin()], -1)

    def rot(v):  # v: [heads, T, hd]; the "rotate half" formulation
        v1, v2 = v[..., :hd // 2], v[..., hd // 2:]
        return v * cos + torch.cat([-v2, v1], -1) * sin

    x = torch.from_numpy(x_in)
    for lw in w["layers"]:
        h = F.rms_norm(x, (cfg["d_model"],), t(lw["attn_norm"]), cfg["rms_eps"])
        q = F.linear(h, t(lw["wq"])).view(T, H, hd).transpose(0, 1)
        k = F.linear(h, t(lw["wk"])).view(T, Hkv, hd).transpose(0, 1)
        v = F.linear(h, t(lw["wv"])).view(T, Hkv, hd).transpose(0, 1)
        q, k = rot(q), rot(k)
        k = k.repeat_interleave(H // Hkv, dim=0)
        v = v.repeat_interleave(H // Hkv, dim=0)
        o = F.scaled_dot_product_attention(q[None], k[None], v[None], is_causal=True)[0]
        x = x + F.linear(o.transpose(0, 1).reshape(T, H * hd), t(lw["wo"]))
        h = F.rms_norm(x, (cfg["d_model"],), t(lw["ffn_norm"]), cfg["rms_eps"])
        x = x + F.linear(F.silu(F.linear(h, t(lw["w_gate"]))) * F.linear(h, t(lw["w_up"])),
                         t(lw["w_down"]))
    out = F.linear(F.rms_norm(x, (cfg["d_model"],), t(w["final_norm"]), cfg["rms_eps"]),
                   t(w["lm_head"])).numpy()
    assert np.abs(out).max() > 0.5
    assert np.allclose(out, ref, rtol=1e-10, atol=1e-11)


# --------------------------------------------------------------------------- tree == brute force

def _all_parent_arrays(n):
    for tail in itertools.product(*[range(i) for i in range(1, n)]):
        yield np.array((-1,) + tail, np.int32)


def _check_tree_equals_form_s(cfg, w, audio, text, parents, tokens, atol=1e-9):
    om = oracle.OracleModel(cfg, w)
    kc, vc, L, _ = _prefill(om, cfg, audio, text, len(text) + audio.shape[0] + len(parents))
    r = om.tree_forward(kc, vc, L, tokens, parents)
    rows = _prefix_rows(cfg, w, audio, text)
    for i in range(len(parents)):
        ref = form_s.node_logits(cfg, w, rows, tokens, parents, i)
        assert np.allclose(r["logits"][i], ref, rtol=1e-9, atol=atol), (parents, i)
        assert r["amax"][i] == int(np.argmax(ref))
    return r


def test_tree_equals_sequential_decode_exhaustive_small_trees():
    """Every parent array with up to 5 nodes, GQA model: each node's logits equal a cache-free
    causal decode of its root path (mask, depth positions, slot handling, GQA mapping)."""
    cfg = dict(TINY)
    w = _boost(wl.make_weights(cfg, 21, "f32"), 6.0)
    rng = np.random.default_rng(4)
    audio = rng.standard_normal((5, cfg["d_model"])).astype(np.float32)
    text = rng.integers(0, cfg["vocab"], 3).astype(np.int32)
    for n in range(1, 6):
        for parents in _all_parent_arrays(n):
            tokens = rng.integers(0, cfg["vocab"], n).astype(np.int32)
            _check_tree_equals_form_s(cfg, w, audio, text, parents, tokens)


def test_tree_equals_sequential_decode_random_trees_n10():
    cfg = dict(TINY, n_layers=1, n_heads=2, n_kv_heads=1, head_dim=16)
    w = _boost(wl.make_weights(cfg, 22, "f32"), 6.0)
    rng = np.random.default_rng(5)
    audio = rng.standard_normal((4, cfg["d_model"])).astype(np.float32)
    text = rng.integers(0, cfg["vocab"], 4).astype(np.int32)
    for _ in range(6):
        parents = wl.random_tree(rng, 10, max_children=3)
        tokens = rng.integers(0, cfg["vocab"], 10).astype(np.int32)
        _check_tree_equals_form_s(cfg, w, audio, text, parents, tokens)


def test_config1_tree_equals_sequential_decode():
    """The tiny fp32 workload (2 layers, d 256, 4 heads, FFN 688, vocab 1000; prefix 48 audio + 16
    text; 8-node tree with a branch) node by node against form S."""
    cfg = wl.MODELS["tiny"]
    spec = wl.WORKLOADS["cfg1_tiny"]
    w = wl.make_weights(cfg, spec["seed"], "f32")
    audio, text = wl.make_prefix_inputs(cfg, spec["seed"], spec["n_audio"], spec["n_text"])
    parents, tokens = wl.make_tree("cfg1_tiny")
    assert parents.tolist() == [-1, 0, 1, 2, 3, 4, 2, 6]
    _check_tree_equals_form_s(cfg, w, audio, text, parents, tokens, atol=1e-10)


def test_chain_tree_is_causal_attention():
    """A chain-shaped tree equals ONE causal pass over [prefix ; chain] (all rows at once), and
    equals N single-node trees applied one after another with commits."""
    cfg = dict(TINY)
    w = _boost(wl.make_weights(cfg, 23, "f32"), 6.0)
    rng = np.random.default_rng(6)
    audio = rng.standard_normal((6, cfg["d_model"])).astype(np.float32)
    text = rng.integers(0, cfg["vocab"], 2).astype(np.int32)
    n = 9
    tokens = rng.integers(0, cfg["vocab"], n).astype(np.int32)
    parents = np.arange(-1, n - 1, dtype=np.int32)
    om = oracle.OracleModel(cfg, w)
    kc, vc, L, _ = _prefill(om, cfg, audio, text, 8 + n)
    r = om.tree_forward(kc, vc, L, tokens, parents)
    E = form_s.widen(w["tok_embed"])
    full = form_s.causal_decoder(cfg, w, np.concatenate([_prefix_rows(cfg, w, audio, text), E[tokens]]))
    assert np.allclose(r["logits"], full[L:], rtol=1e-9, atol=1e-10)
    # sequential single-node rounds
    kc2, vc2, L2 = kc.copy(), vc.copy(), L
    for i in range(n):
        s = om.tree_forward(kc2, vc2, L2, tokens[i:i + 1], np.array([-1], np.int32))
        assert np.allclose(s["logits"][0], r["logits"][i], rtol=1e-9, atol=1e-10)
        L2 = om.commit(kc2, vc2, L2, s["ktree"], s["vtree"], [0])


def test_node_relabelling_permutes_outputs():
    """Any topological relabelling of the nodes permutes logits and K/V rows and nothing else
    (slot and position are different things)."""
    cfg = dict(TINY)
    w = _boost(wl.make_weights(cfg, 24, "f32"), 6.0)
    rng = np.random.default_rng(7)
    om = oracle.OracleModel(cfg, w)
    audio = rng.standard_normal((3, cfg["d_model"])).astype(np.float32)
    kc, vc, L, _ = _prefill(om, cfg, audio, np.array([1, 2], np.int32), 16)
    parents = np.array([-1, 0, 1, 2, 0, 4, 1], np.int32)
    tokens = rng.integers(0, cfg["vocab"], 7).astype(np.int32)
    order = [0, 4, 1, 5, 6, 2, 3]          # new index -> old index, parents still precede children
    inv = {o: nw for nw, o in enumerate(order)}
    par2 = np.array([-1 if parents[o] < 0 else inv[int(parents[o])] for o in order], np.int32)
    tok2 = tokens[order]
    a = om.tree_forward(kc, vc, L, tokens, parents)
    b = om.tree_forward(kc, vc, L, tok2, par2)
    assert np.allclose(b["logits"], a["logits"][order], rtol=1e-12, atol=1e-13)
    assert np.allclose(b["ktree"], a["ktree"][:, :, order], rtol=1e-12, atol=1e-13)


def test_sibling_independence_bit_identical():
    """Changing the tokens of one branch leaves every logit outside it bit-identical."""
    cfg = dict(TINY)
    w = _boost(wl.make_weights(cfg, 25, "f32"), 6.0)
    rng = np.random.default_rng(8)
    om = oracle.OracleModel(cfg, w)
    audio = rng.standard_normal((3, cfg["d_model"])).astype(np.float32)
    kc, vc, L, _ = _prefill(om, cfg, audio, np.array([5], np.int32), 16)
    parents = wl.tree_cfg1()
    tokens = rng.integers(0, cfg["vocab"], 8).astype(np.int32)
    a = om.tree_forward(kc, vc, L, tokens, parents)
    t2 = tokens.copy()
    t2[6] = (t2[6] + 1) % cfg["vocab"]
    t2[7] = (t2[7] + 3) % cfg["vocab"]
    b = om.tree_forward(kc, vc, L, t2, parents)
    assert np.array_equal(a["logits"][:6], b["logits"][:6])
    assert not np.allclose(a["logits"][6:], b["logits"][6:])


def test_gqa_equals_mha_with_replicated_kv_heads():
    cfg = dict(TINY)                      # 4 query heads, 2 KV heads
    w = _boost(wl.make_weights(cfg, 26, "f32"), 6.0)
    hd, Hkv, g = cfg["head_dim"], cfg["n_kv_heads"], cfg["n_heads"] // cfg["n_kv_heads"]
    cfg2 = dict(cfg, n_kv_heads=cfg["n_heads"])
    w2 = {k: v for k, v in w.items() if k != "layers"}
    w2["layers"] = []
    for lw in w["layers"]:
        l2 = dict(lw)
        for m in ("wk", "wv"):
            blocks = lw[m].reshape(Hkv, hd, -1)
            l2[m] = np.ascontiguousarray(np.repeat(blocks, g, axis=0).reshape(Hkv * g * hd, -1))
        w2["layers"].append(l2)
    rng = np.random.default_rng(9)
    parents = wl.random_tree(rng, 6)
    tokens = rng.integers(0, cfg["vocab"], 6).astype(np.int32)
    out = []
    for c, ww in ((cfg, w), (cfg2, w2)):
        om = oracle.OracleModel(c, ww)
        kc, vc = om.empty_cache(12)
        L, _ = om.prefill(kc, vc, 0, None, np.array([3, 1, 4, 1, 5], np.int32))
        out.append(om.tree_forward(kc, vc, L, tokens, parents)["logits"])
    assert np.allclose(out[0], out[1], rtol=1e-12, atol=1e-13)


def test_storage_dtypes_are_widened_exactly():
    """bf16-bit weights give exactly the results of the same values held as float32."""
    cfg = dict(TINY)
    wb = wl.make_weights(cfg, 27, "bf16")
    wf = {k: (wl.bf16_to_f32(v) if k != "layers" else None) for k, v in wb.items()}
    wf["layers"] = [{k: wl.bf16_to_f32(v) for k, v in lw.items()} for lw in wb["layers"]]
    rng = np.random.default_rng(10)
    parents = wl.tree_cfg1()
    tokens = rng.integers(0, cfg["vocab"], 8).astype(np.int32)
    res = []
    for ww in (wb, wf):
        om = oracle.OracleModel(cfg, ww)
        kc, vc = om.empty_cache(16)
        L, _ = om.prefill(kc, vc, 0, None, np.array([3, 1, 4], np.int32))
        res.append(om.tree_forward(kc, vc, L, tokens, parents)["logits"])
    assert np.array_equal(res[0], res[1])


def test_tree_rows_take_the_cache_storage_type():
    """The K/V rows of the tree nodes are cache entries (slot L + node): over an f32 or bf16 cache
    they are rounded to that type before attention reads them.  (a) The first layer's rows equal
    an independent rounding of the fp64 rows (inputs of layer 0 do not depend on the cache
    type).  (b) Consequence: a chain evaluated in one pass over a bf16 cache equals node-by-node
    decoding that writes each row into the bf16 cache and reads it back -- the property that
    makes tree verification equal to sequential decoding through a real cache."""
    cfg = dict(TINY)
    w = _boost(wl.make_weights(cfg, 28, "f32"), 4.0)
    om = oracle.OracleModel(cfg, w)
    rng = np.random.default_rng(11)
    L, cap, n = 5, 16, 6
    kc, vc = om.empty_cache(cap)
    om.prefill(kc, vc, 0, None, rng.integers(0, cfg["vocab"], L).astype(np.int32))
    kb, vb = wl.bf16_bits(kc.astype(np.float32)), wl.bf16_bits(vc.astype(np.float32))
    k64, v64 = wl.bf16_to_f32(kb).astype(np.float64), wl.bf16_to_f32(vb).astype(np.float64)
    tokens = rng.integers(0, cfg["vocab"], n).astype(np.int32)
    chain = np.arange(-1, n - 1, dtype=np.int32)
    r64 = om.tree_forward(k64, v64, L, tokens, chain)
    rb = om.tree_forward(kb, vb, L, tokens, chain)
    r32 = om.tree_forward(k64.astype(np.float32), v64.astype(np.float32), L, tokens, chain)
    for name in ("ktree", "vtree"):
        want = wl.bf16_to_f32(wl.bf16_bits(r64[name][0].astype(np.float32))).astype(np.float64)
        assert np.array_equal(rb[name][0], want)
        assert np.array_equal(r32[name][0], r64[name][0].astype(np.float32).astype(np.float64))
        assert not np.array_equal(rb[name][0], r64[name][0])
    # (b) node by node through the bf16 cache
    kk, vv = kb.copy(), vb.copy()
    for i in range(n):
        r = om.tree_forward(kk, vv, L + i, tokens[i:i + 1], np.array([-1], np.int32))
        kk[:, :, L + i] = wl.bf16_bits(r["ktree"][:, :, 0].astype(np.float32))
        vv[:, :, L + i] = wl.bf16_bits(r["vtree"][:, :, 0].astype(np.float32))
        assert np.allclose(r["logits"][0], rb["logits"][i], rtol=1e-9, atol=1e-11)
    assert not np.allclose(r64["logits"][n - 1], rb["logits"][n - 1], rtol=1e-9, atol=1e-11)


# --------------------------------------------------------------------------- acceptance

def _accept_by_enumeration(tokens, parents, amax):
    """Walk every root-to-node path token by token; keep the deepest fully matching one,
    lowest node index among equals."""
    best, best_len = 0, 1
    for i in range(len(parents)):
        path = form_s.root_path(parents, i)
        ok = all(tokens[path[k]] == amax[path[k - 1]] for k in range(1, len(path)))
        if ok and len(path) > best_len:
            best, best_len = i, len(path)
    return form_s.root_path(parents, best), best_len, int(amax[best])


def test_accept_against_path_enumeration():
    rng = np.random.default_rng(12)
    for trial in range(400):
        n = int(rng.integers(1, 25))
        parents = wl.random_tree(rng, n, max_children=3)
        vocab = int(rng.integers(2, 5))    # tiny vocab: many matches and duplicate sibling tokens
        tokens = rng.integers(0, vocab, n).astype(np.int32)
        amax = rng.integers(0, vocab, n).astype(np.int32)
        path, alen, nxt = oracle.accept(tokens, parents, amax)
        rp, rl, rn = _accept_by_enumeration(tokens, parents, amax)
        assert (path.tolist(), alen, nxt) == (rp, rl, rn), (parents, tokens, amax)


def test_accept_stops_at_first_failure_on_a_chain():
    parents = np.arange(-1, 7, dtype=np.int32)
    tokens = np.array([9, 1, 2, 3, 4, 5, 6, 7], np.int32)
    for k in range(1, 9):                 # first mismatch at draft k (k = 8: all accepted)
        amax = np.array([1, 2, 3, 4, 5, 6, 7, 8], np.int32)
        if k < 8:
            amax[k - 1] = 0
            amax[min(k + 1, 7)] = tokens[min(k + 1, 7)]  # later matches must not resurrect it
        path, alen, nxt = oracle.accept(tokens, parents, amax)
        assert alen == k and path.tolist() == list(range(k)) and nxt == amax[k - 1]


def test_accept_takes_the_branch():
    parents = wl.tree_cfg1()
    tokens = np.array([10, 11, 12, 13, 14, 15, 23, 24], np.int32)
    amax = np.array([11, 12, 23, 0, 0, 0, 24, 99], np.int32)   # trunk fails at depth 3, branch matches
    path, alen, nxt = oracle.accept(tokens, parents, amax)
    assert path.tolist() == [0, 1, 2, 6, 7] and alen == 5 and nxt == 99


# --------------------------------------------------------------------------- end to end

def test_lossless_rounds_equal_greedy_autoregressive_decode():
    """Whatever trees are drafted, the tokens emitted over verify/accept/commit rounds are the
    greedy autoregressive output of the same model."""
    cfg = dict(TINY)
    w = _boost(wl.make_weights(cfg, 31, "f32"), 6.0)
    rng = np.random.default_rng(13)
    audio = rng.standard_normal((4, cfg["d_model"])).astype(np.float32)
    text = np.array([2, 7, 1], np.int32)
    n_new = 14
    ref = form_s.greedy_decode(cfg, w, _prefix_rows(cfg, w, audio, text[:-1]), text[-1], n_new)
    assert len(set(ref)) > 2

    om = oracle.OracleModel(cfg, w)
    kc, vc = om.empty_cache(64)
    L, _ = om.prefill(kc, vc, 0, audio.astype(np.float64), text[:-1])   # last token is the first root
    root, emitted, rounds = int(text[-1]), [], 0
    while len(emitted) < n_new:
        n = int(rng.integers(1, 9))
        parents = wl.random_tree(rng, n)
        tokens = rng.integers(0, cfg["vocab"], n).astype(np.int32)
        tokens[0] = root
        # a drafter that is right most of the time: children of a node copy the true continuation
        depth, _ = oracle.tree_meta(parents)
        for i in range(1, n):
            k = len(emitted) + depth[i] - 1
            if k < len(ref) and rng.uniform() < 0.7:
                tokens[i] = ref[k]
        r = om.tree_forward(kc, vc, L, tokens, parents)
        path, alen, nxt = oracle.accept(tokens, parents, r["amax"])
        emitted += [int(tokens[j]) for j in path[1:]] + [nxt]
        L = om.commit(kc, vc, L, r["ktree"], r["vtree"], path)
        root = nxt
        rounds += 1
    assert emitted[:n_new] == ref
    assert rounds < n_new                     # some drafts were accepted


def test_commit_equals_prefill_of_accepted_tokens():
    cfg = dict(TINY)
    w = _boost(wl.make_weights(cfg, 32, "f32"), 6.0)
    rng = np.random.default_rng(14)
    om = oracle.OracleModel(cfg, w)
    text = np.array([2, 7, 1, 8], np.int32)
    kc, vc = om.empty_cache(32)
    L, _ = om.prefill(kc, vc, 0, None, text)
    parents = wl.tree_cfg1()
    tokens = rng.integers(0, cfg["vocab"], 8).astype(np.int32)
    r = om.tree_forward(kc, vc, L, tokens, parents)
    path = [0, 1, 2, 6, 7]
    L2 = om.commit(kc, vc, L, r["ktree"], r["vtree"], path)
    kr, vr = om.empty_cache(32)
    Lr, _ = om.prefill(kr, vr, 0, None, np.concatenate([text, tokens[path]]))
    assert L2 == Lr == 9
    assert np.allclose(kc[:, :, :L2], kr[:, :, :Lr], rtol=1e-10, atol=1e-12)
    assert np.allclose(vc[:, :, :L2], vr[:, :, :Lr], rtol=1e-10, atol=1e-12)


def test_workload_tree_shapes():
    """Node counts of the named workloads: 6+2, 12+2*2, 16+4*4, 16+2*4, 24+8*5."""
    want = dict(cfg1_tiny=8, cfg2_1b_n16=16, cfg3_7b_n32=32, cfg4_1b_b16=24, cfg5_7b_n64=64,
                cfg6_13b_n32=32)
    for name, n in want.items():
        parents, tokens = wl.make_tree(name)
        assert len(parents) == n == len(tokens)
        depth, _ = oracle.tree_meta(parents)
        assert depth.max() < 24 + 5
        kids = np.bincount(parents[1:], minlength=n)
        assert kids.max() <= 2                     # trunk token plus one top-2 alternative
        for i in range(1, n):
            sib = [int(tokens[j]) for j in range(n) if j != i and parents[j] == parents[i]]
            assert int(tokens[i]) not in sib


def test_argmax_takes_lowest_index_on_exact_ties():
    """Two identical LM-head rows give bit-equal logits: the lower token id wins."""
    cfg = dict(TINY)
    w = _boost(wl.make_weights(cfg, 33, "f32"), 6.0)
    om = oracle.OracleModel(cfg, w)
    kc, vc = om.empty_cache(8)
    tok, par = np.array([4], np.int32), np.array([-1], np.int32)
    t = int(om.tree_forward(kc, vc, 0, tok, par)["amax"][0])
    for u in (t + 1 if t + 1 < cfg["vocab"] else t - 1, (t + 5) % cfg["vocab"]):
        w2 = dict(w)
        w2["lm_head"] = w["lm_head"].copy()
        w2["lm_head"][u] = w2["lm_head"][t]
        r = oracle.OracleModel(cfg, w2).tree_forward(kc, vc, 0, tok, par)
        assert r["logits"][0, u] == r["logits"][0, t]
        assert r["amax"][0] == min(t, u)


def test_oracle_regression_against_stored_results():
    """The oracle still produces what tests/golden/make_golden.py (oracle-only script) stored."""
    import json
    import os
    import importlib.util
    here = os.path.dirname(os.path.abspath(__file__))
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(here, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    got = mod.compute()
    want = json.load(open(os.path.join(here, "golden", "cfg1_oracle.json")))
    for k in ("kv_len", "tokens", "parents", "amax", "path", "accept_len", "next_token"):
        assert got[k] == want[k], k
    for k in ("logits_node0_first8", "logits_node7_first8"):
        assert np.allclose(got[k], want[k], rtol=1e-9, atol=1e-12)


# --------------------------------------------------------------------------- draft-side read-out
def test_top2_closed_forms_and_ties():
    """Values that follow from the definition alone (Sec. IV-A normalised logit; Sec. IV-C tokens
    of highest probability): equal logits, a two-token row with a known ratio, shift
    invariance, no overflow, a single-token vocabulary, ties resolved towards the lower id."""
    top, p = oracle.top2(np.zeros((1, 7)))
    assert top.tolist() == [[0, 1]] and abs(p[0] - 1 / 7) < 1e-15
    top, p = oracle.top2(np.array([[0.0, np.log(3.0)]]))
    assert top.tolist() == [[1, 0]] and abs(p[0] - 0.75) < 1e-15
    x = np.array([[0.3, -1.2, 2.5, 2.4, 0.0]])
    t0, p0 = oracle.top2(x)
    t1, p1 = oracle.top2(x + 1000.0)                      # would overflow without the max shift
    assert t0.tolist() == t1.tolist() == [[2, 3]] and abs(p0[0] - p1[0]) < 1e-12
    assert abs(p0[0] - np.exp(2.5) / np.exp(x).sum()) < 1e-15
    top, p = oracle.top2(np.array([[4.2]]))
    assert top.tolist() == [[0, -1]] and p[0] == 1.0
    top, p = oracle.top2(np.array([[5.0, 1.0, 5.0, 5.0], [1.0, 7.0, 7.0, 0.0], [2.0, 9.0, 2.0, 1.0]]))
    assert top.tolist() == [[0, 2], [1, 2], [1, 0]]
    assert abs(p[0] - 1 / (3 + np.exp(-4.0))) < 1e-15
    # a dominant logit: probability -> 1, the runner-up is still reported
    top, p = oracle.top2(np.array([[0.0, 50.0, 1.0]]))
    assert top.tolist() == [[1, 2]] and 1 - p[0] < 1e-20 + 2e-21 + np.exp(-49.0) * 1.1


def test_top2_against_sort_and_library_softmax():
    """Random rows (with planted duplicates of the two largest values): the two ids equal the head
    of a (value descending, id ascending) sort, p1 equals scipy's softmax at the first id."""
    from scipy.special import softmax as sp_softmax
    rng = np.random.default_rng(404)
    for V in (2, 3, 17, 1000):
        x = rng.standard_normal((40, V)) * 3.0
        for r in range(0, 40, 4):                          # exact ties among the leaders
            j, k = rng.integers(0, V, 2)
            x[r, j] = x[r].max()
            x[r, k] = np.sort(x[r])[-2] if r % 8 else x[r].max()
        top, p = oracle.top2(x)
        ids = np.arange(V)
        for r in range(40):
            order = np.lexsort((ids, -x[r]))
            assert top[r].tolist() == order[:2].tolist()
            assert abs(p[r] - sp_softmax(x[r])[order[0]]) < 1e-14
            assert x[r, top[r, 0]] >= x[r, top[r, 1]]


def test_top2_first_id_is_the_forward_pass_argmax():
    """On the logits of a tree forward, the first id of the read-out is the argmax the verify
    path uses (same tie rule), for every node."""
    cfg = dict(TINY)
    w = _boost(wl.make_weights(cfg, 35, "f32"), 4.0)
    om = oracle.OracleModel(cfg, w)
    kc, vc = om.empty_cache(16)
    parents = wl.tree_cfg1()
    tokens = np.random.default_rng(36).integers(0, cfg["vocab"], 8).astype(np.int32)
    r = om.tree_forward(kc, vc, 0, tokens, parents)
    top, p = oracle.top2(r["logits"])
    assert top[:, 0].tolist() == r["amax"].tolist()
    assert np.all((p > 0) & (p <= 1))
