"""GPU parity on the tiny model: HIP path (through the C ABI) vs the CPU oracle, element by element."""
import numpy as np
import pytest

import oracle
from oracle import form_s
import workload as wl
from parity_util import (TOL_F32, TOL_BF16, check_forward, check_tree_kv, oracle_prefilled,
                         row_rel_err, widen_cache, walk_is_decisive, check_top2,
                         check_top2_against_oracle_forward)

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _verifier(*a, **k):
    from paper_2507_18181_amd.runtime import Verifier
    return Verifier(*a, **k)


def _cfg1(dtype="f32"):
    spec = wl.WORKLOADS["cfg1_tiny"]
    cfg = wl.MODELS["tiny"]
    w = wl.make_weights(cfg, spec["seed"], dtype)
    audio, text = wl.make_prefix_inputs(cfg, spec["seed"], spec["n_audio"], spec["n_text"])
    parents, tokens = wl.make_tree("cfg1_tiny")
    return cfg, w, audio, text, parents, tokens


def _store_cache(kc, dtype):
    a = kc[None].astype(np.float32)
    return wl.bf16_bits(a) if dtype == "bf16" else a


@pytest.mark.parametrize("dtype,flags,tol", [("f32", 0, TOL_F32), ("bf16", 1, TOL_BF16),
                                             ("bf16", 0, TOL_BF16)])
def test_cfg1_forward_and_round(dtype, flags, tol):
    """Tiny workload: 2 layers, d 256, 4 heads, FFN 688, vocab 1000; prefix 48 audio + 16 text;
    8-node tree with a branch.  fp32 model at 1e-4; bf16-rounded model at 2e-2."""
    cfg, w, audio, text, parents, tokens = _cfg1(dtype)
    om, kc, vc, L, _ = oracle_prefilled(cfg, w, audio, text, 96)
    ver = _verifier(cfg, w, dtype, max_nodes=8, capacity=96, flags=flags)
    from paper_2507_18181_amd import binding as B
    assert B.specasr_uses_mfma(ver.ctx, 8) == (1 if (dtype == "bf16" and flags == 0) else 0)
    ver.set_cache(_store_cache(kc, dtype), _store_cache(vc, dtype), [L])
    k0, v0 = ver.get_cache()
    ref = om.tree_forward(k0[0], v0[0], L, tokens, parents)       # oracle reads the GPU's cache bits

    fw = ver.tree_forward([tokens], [parents])
    assert fw["status"] == 0
    check_forward(ref, fw["logits"][0].cpu().numpy(), fw["argmax"][0].cpu().numpy(), tol)
    k1, v1 = ver.get_cache()
    check_tree_kv(k1[0], v1[0], L, ref, tol)
    assert np.array_equal(k1[:, :, :, :L], k0[:, :, :, :L]) and np.array_equal(v1[:, :, :, :L], v0[:, :, :, :L])
    assert ver.kv_len[0] == L

    out = ver.verify_tree([tokens], [parents], want_logits=True)
    assert out["status"] == 0
    n = len(parents)
    path, alen, nxt = oracle.accept(tokens, parents, out["argmax"][0, :n])   # integer stage, same argmax
    assert out["accept_len"][0] == alen and out["next_token"][0] == nxt
    assert out["path"][0, :alen].tolist() == path.tolist() and np.all(out["path"][0, alen:] == -1)
    assert ver.kv_len[0] == L + alen
    k2, v2 = ver.get_cache()
    for k in range(alen):     # compaction is a byte move of the rows computed by the forward
        assert np.array_equal(k2[0, :, :, L + k], k1[0, :, :, L + path[k]])
        assert np.array_equal(v2[0, :, :, L + k], v1[0, :, :, L + path[k]])
    assert np.array_equal(k2[:, :, :, :L], k0[:, :, :, :L])
    ver.close()


@pytest.mark.parametrize("dtype,tol", [("f32", TOL_F32), ("bf16", TOL_BF16)])
def test_planted_drafts_sweep_accept_len_and_take_the_branch(dtype, tol):
    """Draft tokens follow the oracle's own greedy continuation for k steps, so accept_len sweeps
    1..6 on the trunk; then the branch carries the right continuation and is taken."""
    cfg, w, audio, text, parents, tokens = _cfg1(dtype)
    om, kc, vc, L, _ = oracle_prefilled(cfg, w, audio, text, 96)
    rows = np.concatenate([audio.astype(np.float64), form_s.widen(w["tok_embed"])[text]])
    greedy = form_s.greedy_decode(cfg, w, rows, tokens[0], 7)
    ver = _verifier(cfg, w, dtype, max_nodes=8, capacity=96)
    cases = []
    for k in range(6):                   # trunk matches k drafts
        t = tokens.copy()
        t[1:1 + k] = greedy[:k]
        for i in range(1 + k, 6):
            t[i] = (greedy[i - 1] + 1 + i) % cfg["vocab"]
        t[6] = (greedy[2] + 1) % cfg["vocab"]
        cases.append((t, k + 1))
    t = tokens.copy()                    # trunk right for 2 drafts, branch right for 2 more
    t[1:3] = greedy[:2]
    t[3] = (greedy[2] + 1) % cfg["vocab"]
    t[6], t[7] = greedy[2], greedy[3]
    cases.append((t, 5))
    for t, want_len in cases:
        ver.set_cache(_store_cache(kc, dtype), _store_cache(vc, dtype), [L])
        k0, v0 = ver.get_cache()
        ref = om.tree_forward(k0[0], v0[0], L, t, parents)
        rpath, rlen, rnext = oracle.accept(t, parents, ref["amax"])
        out = ver.verify_tree([t], [parents], want_logits=True)
        assert out["status"] == 0
        check_forward(ref, out["logits"][0].cpu().numpy(), out["argmax"][0], tol)
        if walk_is_decisive(ref["logits"], t, parents, rpath, rlen):
            assert out["accept_len"][0] == rlen and out["next_token"][0] == rnext
            assert out["path"][0, :rlen].tolist() == rpath.tolist()
            if dtype == "f32":
                assert rlen == want_len
        k2, v2 = ver.get_cache()
        alen = int(out["accept_len"][0])
        got_k = widen_cache(k2[0, :, :, L:L + alen])
        want_k = ref["ktree"][:, :, out["path"][0, :alen]]
        assert np.abs(got_k - want_k).max() <= tol * np.abs(want_k).max()
    ver.close()


@pytest.mark.parametrize("dtype,tol,flags", [("f32", TOL_F32, 0), ("bf16", TOL_BF16, 0),
                                             ("bf16", TOL_BF16, 1)])
def test_random_trees_all_sizes(dtype, tol, flags):
    """Ragged tree sizes 1..64 (several 16-row tiles and tails), random shapes, varying kv_len."""
    cfg = wl.MODELS["tiny"]
    w = wl.make_weights(cfg, 77, dtype)
    rng = np.random.default_rng(78)
    audio = rng.standard_normal((40, cfg["d_model"])).astype(np.float32)
    text = rng.integers(0, cfg["vocab"], 300).astype(np.int32)
    om, kc, vc, Lfull, _ = oracle_prefilled(cfg, w, audio, text, 420)
    ver = _verifier(cfg, w, dtype, max_nodes=64, capacity=420, flags=flags)
    for n, L in ((1, 0), (1, 5), (2, 64), (7, 63), (15, 255), (16, 256), (17, 257), (33, 100),
                 (48, 340), (63, 129), (64, 340), (64, 356)):   # the last: kv_len + n == capacity exactly
        parents = wl.random_tree(rng, n, max_children=3)
        tokens = rng.integers(0, cfg["vocab"], n).astype(np.int32)
        ver.set_cache(_store_cache(kc, dtype), _store_cache(vc, dtype), [L])
        k0, v0 = ver.get_cache()
        ref = om.tree_forward(k0[0], v0[0], L, tokens, parents)
        fw = ver.tree_forward([tokens], [parents])
        assert fw["status"] == 0
        check_forward(ref, fw["logits"][0].cpu().numpy(), fw["argmax"][0].cpu().numpy(), tol)
        k1, v1 = ver.get_cache()
        check_tree_kv(k1[0], v1[0], L, ref, tol)
    ver.close()


def test_batch_of_ragged_sequences():
    """Three sequences with different prefix lengths and trees in one call: each equals the
    oracle run on it alone."""
    cfg = wl.MODELS["tiny"]
    w = wl.make_weights(cfg, 79, "f32")
    rng = np.random.default_rng(80)
    ver = _verifier(cfg, w, "f32", max_nodes=16, capacity=128, max_batch=3)
    om = oracle.OracleModel(cfg, w)
    caches, Ls = [], [37, 90, 5]
    K = np.zeros((3, cfg["n_layers"], cfg["n_kv_heads"], 128, cfg["head_dim"]), np.float32)
    V = np.zeros_like(K)
    for b, L in enumerate(Ls):
        kc, vc = om.empty_cache(128)
        om.prefill(kc, vc, 0, None, rng.integers(0, cfg["vocab"], L).astype(np.int32))
        K[b], V[b] = kc, vc
    ver.set_cache(K, V, Ls)
    k0, v0 = ver.get_cache()
    trees = [wl.random_tree(rng, n) for n in (16, 3, 9)]
    toks = [rng.integers(0, cfg["vocab"], len(p)).astype(np.int32) for p in trees]
    out = ver.verify_tree(toks, trees, want_logits=True)
    assert out["status"] == 0
    k2, v2 = ver.get_cache()
    for b in range(3):
        ref = om.tree_forward(k0[b], v0[b], Ls[b], toks[b], trees[b])
        n = len(trees[b])
        check_forward(ref, out["logits"][b].cpu().numpy(), out["argmax"][b], TOL_F32)
        path, alen, nxt = oracle.accept(toks[b], trees[b], out["argmax"][b, :n])
        assert out["accept_len"][b] == alen and out["next_token"][b] == nxt
        assert out["path"][b, :alen].tolist() == path.tolist()
        assert ver.kv_len[b] == Ls[b] + alen
        want = ref["ktree"][:, :, path]
        got = widen_cache(k2[b, :, :, Ls[b]:Ls[b] + alen])
        assert np.abs(got - want).max() <= TOL_F32 * np.abs(want).max()
        assert np.all(out["argmax"][b, n:] == -1)
    ver.close()


@pytest.mark.parametrize("sizes,no_wide", [
    ((20, 30, 14, 40, 1, 5, 16), True),    # 126 rows, wide passes off: groups of whole sequences, <= 64 rows each
    ((20, 30, 14, 64, 1, 5, 16), True),    # 150 rows in groups, one of them a full 64-node tree
    ((20, 30, 14, 1, 1, 5, 16), False),    # 87 rows: one pass on the wide (tiled GEMM) kernels, one row tile
    ((20, 30, 14, 64, 1, 5, 16), False),   # 150 rows: wide, 2 row tiles
    ((64, 64, 64, 64, 3, 64, 64), False),  # 387 rows: wide, 4 row tiles, the last almost empty
])
def test_batch_above_64_rows_runs_on_the_mfma_path(sizes, no_wide):
    """Seven bf16 sequences with more than 64 tree nodes in total: one pass whose projections run
    on the tiled GEMM -- or, where wide passes are not available (here: a context created with
    SPECASR_FLAG_NO_WIDE), consecutive groups of whole sequences with at most 64 rows each on the skinny
    kernels, spread over several streams.  Either way every sequence equals the oracle run on it
    alone, tree_forward agrees with verify_tree, and the draft-side read-out equals the oracle's
    read-out of the same logits."""
    from paper_2507_18181_amd import binding as B
    cfg = wl.MODELS["tiny"]
    w = wl.make_weights(cfg, 91, "bf16")
    rng = np.random.default_rng(92)
    Ls = [37, 90, 5, 60, 0, 33, 64]
    nb, cap = len(sizes), 160
    ver = _verifier(cfg, w, "bf16", max_nodes=64, capacity=cap, max_batch=nb,
                    flags=B.SPECASR_FLAG_NO_WIDE if no_wide else 0)
    assert B.specasr_uses_mfma(ver.ctx, sum(sizes)) == 1
    om = oracle.OracleModel(cfg, w)
    K, V = wl.seeded_cache(cfg, 93, np.asarray(Ls, np.int32), cap, "bf16", batch=nb)
    ver.set_cache(K, V, Ls)
    trees = [wl.random_tree(rng, n) for n in sizes]
    toks = [wl.tree_tokens(rng, p, cfg["vocab"]) for p in trees]
    fwd = ver.tree_forward(toks, trees, want_logits=True)
    assert fwd["status"] == 0
    ver.set_cache(K, V, Ls)                      # tree_forward wrote the tree rows; start again
    out = ver.verify_tree(toks, trees, want_logits=True)
    assert out["status"] == 0
    k2, v2 = ver.get_cache()
    for b in range(nb):
        n = sizes[b]
        ref = om.tree_forward(np.ascontiguousarray(K[b]), np.ascontiguousarray(V[b]), Ls[b], toks[b], trees[b])
        check_forward(ref, out["logits"][b].cpu().numpy(), out["argmax"][b], TOL_BF16)
        assert np.array_equal(fwd["argmax"][b, :n].cpu().numpy(), out["argmax"][b, :n])
        assert torch.equal(fwd["logits"][b, :n], out["logits"][b, :n])
        path, alen, nxt = oracle.accept(toks[b], trees[b], out["argmax"][b, :n])
        assert out["accept_len"][b] == alen and out["next_token"][b] == nxt
        assert out["path"][b, :alen].tolist() == path.tolist()
        assert ver.kv_len[b] == Ls[b] + alen
        want = ref["ktree"][:, :, path]
        got = widen_cache(k2[b, :, :, Ls[b]:Ls[b] + alen])
        assert np.abs(got - want).max() <= TOL_BF16 * np.abs(want).max()
        assert np.all(out["argmax"][b, n:] == -1)
    ver.set_cache(K, V, Ls)
    dr = ver.tree_forward_top2(toks, trees, want_logits=True)
    assert dr["status"] == 0
    for b in range(nb):
        n = sizes[b]
        assert torch.equal(dr["logits"][b, :n], fwd["logits"][b, :n])
        check_top2(dr["logits"][b].cpu().numpy(), dr["top2"][b].cpu().numpy(), dr["prob"][b].cpu().numpy(), n)
    ver.close()


@pytest.mark.parametrize("dtype,flags,tol", [("f32", 0, TOL_F32), ("bf16", 1, TOL_BF16),
                                             ("bf16", 0, TOL_BF16)])
def test_draft_readout_two_branch_tree(dtype, flags, tol):
    """Draft-side forward on the recycling tree (old draft and regenerated part as two branches
    below the last verified token): per node the two most probable ids and the probability of
    the first.  (a) read-out against the oracle's read-out of the SAME fp32 logits: ids exact,
    probability 1e-5; (b) against the oracle's own forward within the bound the logit tolerance
    implies; (c) logits and first id identical to specasr_tree_forward; (d) exact ties (two equal
    LM-head rows) resolved towards the lower id in both positions; (e) the K/V rows of the nodes
    are in the cache, kv_len is unchanged."""
    cfg = wl.MODELS["tiny"]
    w = wl.make_weights(cfg, 57, dtype)
    lm = w["lm_head"]
    for a, b in ((17, 901), (640, 5)):   # equal rows tie exactly; x4 (exact in both storage types)
        row = wl.bf16_to_f32(lm[a]) * 4.0 if dtype == "bf16" else lm[a] * 4.0   # makes them frequent leaders
        lm[a] = wl.bf16_bits(row) if dtype == "bf16" else row
        lm[b] = lm[a]
    tie_rows = 0
    rng = np.random.default_rng(58)
    L, cap = 41, 128
    ver = _verifier(cfg, w, dtype, max_nodes=64, capacity=cap, flags=flags)
    om = oracle.OracleModel(cfg, w)
    K, V = wl.seeded_cache(cfg, 59, L, cap, dtype)
    for parents in (wl.two_branch_tree(24, 9), wl.two_branch_tree(1, 1), np.array([-1], np.int32),
                    wl.two_branch_tree(40, 23)):
        n = len(parents)
        tokens = wl.tree_tokens(rng, parents, cfg["vocab"])
        ver.set_cache(K, V, [L])
        out = ver.tree_forward_top2([tokens], [parents], want_logits=True)
        assert out["status"] == 0 and ver.kv_len[0] == L
        lg = out["logits"][0].cpu().numpy()
        top2 = out["top2"][0].cpu().numpy()
        prob = out["prob"][0].cpu().numpy()
        check_top2(lg, top2, prob, n)
        ref = om.tree_forward(np.ascontiguousarray(K[0]), np.ascontiguousarray(V[0]), L, tokens, parents)
        check_top2_against_oracle_forward(ref["logits"], top2, prob, tol)
        kc, vc = ver.get_cache()
        check_tree_kv(kc[0], vc[0], L, ref, tol)
        ver.set_cache(K, V, [L])
        fwd = ver.tree_forward([tokens], [parents], want_logits=True)
        assert torch.equal(fwd["logits"][0, :n], out["logits"][0, :n])
        assert np.array_equal(fwd["argmax"][0, :n].cpu().numpy(), top2[:n, 0])
        for a, b in ((17, 901), (640, 5)):
            lo, hi = min(a, b), max(a, b)
            assert np.all(lg[:n, a] == lg[:n, b])
            assert not np.any(top2[:n, 0] == hi)             # the lower id always comes first
            rows = np.nonzero(top2[:n, 0] == lo)[0]
            assert np.all(top2[rows, 1] == hi)
            tie_rows += len(rows)
    assert tie_rows > 0
    ver.close()


def test_calls_on_a_caller_stream_give_the_same_results():
    """Every entry point takes a raw hipStream_t: a round enqueued on a non-default stream (with
    the cache upload ordered before it) equals the same round on the default stream."""
    cfg = wl.MODELS["tiny"]
    w = wl.make_weights(cfg, 61, "bf16")
    rng = np.random.default_rng(62)
    L, cap = 50, 128
    K, V = wl.seeded_cache(cfg, 63, L, cap, "bf16")
    parents = wl.random_tree(rng, 40)
    tokens = wl.tree_tokens(rng, parents, cfg["vocab"])
    ver = _verifier(cfg, w, "bf16", max_nodes=64, capacity=cap)
    ver.set_cache(K, V, [L])
    ref = ver.verify_tree([tokens], [parents], want_logits=True)
    k_ref, v_ref = ver.get_cache()
    stream = torch.cuda.Stream()
    ver.set_cache(K, V, [L])
    torch.cuda.synchronize()
    out = ver.verify_tree([tokens], [parents], want_logits=True, stream=stream.cuda_stream)
    stream.synchronize()
    assert out["status"] == 0
    for key in ("argmax", "path", "accept_len", "next_token"):
        assert np.array_equal(out[key], ref[key]), key
    assert torch.equal(out["logits"], ref["logits"])
    k2, v2 = ver.get_cache()
    assert np.array_equal(k2, k_ref) and np.array_equal(v2, v_ref)
    ver.set_cache(K, V, [L])
    torch.cuda.synchronize()
    top = ver.tree_forward_top2([tokens], [parents], stream=stream.cuda_stream)
    stream.synchronize()
    assert np.array_equal(top["top2"][0, :40, 0].cpu().numpy(), ref["argmax"][0, :40])
    ver.close()


def test_accept_stage_bit_exact_against_oracle():
    """Acceptance from device argmax arrays and from logits, random trees with tiny vocabularies
    (many matches, duplicate sibling tokens), batch of 5, sizes 1..64."""
    cfg = wl.MODELS["tiny"]
    w = wl.make_weights(cfg, 81, "f32")
    ver = _verifier(cfg, w, "f32", max_nodes=64, capacity=64, max_batch=5)
    rng = np.random.default_rng(82)
    for trial in range(40):
        sizes = [int(rng.integers(1, 65)) for _ in range(5)]
        if trial == 0:
            sizes = [1, 64, 63, 2, 33]
        trees = [wl.random_tree(rng, n, max_children=3) for n in sizes]
        voc = int(rng.integers(2, 6))
        toks = [rng.integers(0, voc, n).astype(np.int32) for n in sizes]
        am = np.full((5, 64), -1, np.int32)
        for b, n in enumerate(sizes):
            am[b, :n] = rng.integers(0, voc, n)
        r = ver.accept(toks, trees, argmax_dev=torch.from_numpy(am).to(ver.device))
        assert r["status"] == 0
        for b, n in enumerate(sizes):
            path, alen, nxt = oracle.accept(toks[b], trees[b], am[b, :n])
            assert r["accept_len"][b] == alen and r["next_token"][b] == nxt
            assert r["path"][b, :alen].tolist() == path.tolist()
            assert np.all(r["path"][b, alen:] == -1)
    # from logits: planted targets; ties resolved to the lowest token id
    parents, _ = wl.make_tree("cfg5_7b_n64")
    tokens = wl.tree_tokens(rng, parents, cfg["vocab"])
    lg = wl.planted_logits(rng, parents, tokens, cfg["vocab"])
    lg[3, 10] = lg[3, 500] = lg[3].max() + 1.0          # exact tie
    full = np.zeros((5, 64, cfg["vocab"]), np.float32)
    full[2] = lg
    r = ver.accept([tokens[:1]] * 2 + [tokens] + [tokens[:1]] * 2,
                   [parents[:1]] * 2 + [parents] + [parents[:1]] * 2,
                   logits_dev=torch.from_numpy(full).to(ver.device))
    am = lg.argmax(axis=1).astype(np.int32)
    assert am[3] == 10
    assert np.array_equal(r["argmax"][2].cpu().numpy(), am)
    path, alen, nxt = oracle.accept(tokens, parents, am)
    assert r["accept_len"][2] == alen and r["next_token"][2] == nxt
    assert r["path"][2, :alen].tolist() == path.tolist()
    ver.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_commit_moves_rows_in_place_without_races(dtype):
    """Adversarial paths whose destinations are other moves' sources (0,1,3,5: slot 3 is written
    by k=2 and read by k=3's predecessor), against a plain gather of the pre-commit cache."""
    cfg = wl.MODELS["tiny"]
    w = wl.make_weights(cfg, 83, dtype)
    rng = np.random.default_rng(84)
    ver = _verifier(cfg, w, dtype, max_nodes=64, capacity=200, max_batch=2)
    paths = [([0, 1, 3, 5], [0]), ([0, 2, 3, 4, 5, 6, 7, 8], [0, 1, 2]), (list(range(0, 64, 2)), [0, 63]),
             ([0] + list(range(33, 64)), list(range(64))), ([0, 1, 2, 3], [0, 5, 6])]
    for pa, pb in paths:
        K, V = wl.seeded_cache(cfg, int(rng.integers(1 << 30)), 200, 200, dtype, batch=2)
        ver.set_cache(K, V, [100, 7])
        rc = ver.commit([64, 64], [pa, pb])
        assert rc == 0
        assert ver.kv_len.tolist() == [100 + len(pa), 7 + len(pb)]
        k2, v2 = ver.get_cache()
        for b, (L, p) in enumerate(((100, pa), (7, pb))):
            for src, got in ((K, k2), (V, v2)):
                want = src[b].copy()
                want[:, :, L:L + len(p)] = src[b][:, :, [L + j for j in p]]
                # rows behind the accepted ones are scratch; everything else must be exact
                keep = np.ones(200, bool)
                keep[L + len(p):L + 64] = False
                assert np.array_equal(got[b][:, :, keep], want[:, :, keep])
    ver.close()


def test_lossless_rounds_on_gpu_equal_greedy_decode():
    """Verify/accept/commit rounds through the library emit exactly the oracle's greedy
    autoregressive tokens (fp32 model, all decisions checked to be decisive)."""
    cfg = wl.MODELS["tiny"]
    w = wl.make_weights(cfg, 85, "f32")
    for lw in w["layers"]:                     # sharpen the logits so that greedy choices are decisive
        for m in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down"):
            lw[m] = (lw[m] * np.float32(4.0)).astype(np.float32)
    w["lm_head"] = (w["lm_head"] * np.float32(8.0)).astype(np.float32)
    rng = np.random.default_rng(86)
    audio = rng.standard_normal((20, cfg["d_model"])).astype(np.float32)
    text = rng.integers(0, cfg["vocab"], 6).astype(np.int32)
    rows = np.concatenate([audio.astype(np.float64), form_s.widen(w["tok_embed"])[text[:-1]]])
    n_new = 24
    ref = form_s.greedy_decode(cfg, w, rows, text[-1], n_new)
    om, kc, vc, L, _ = oracle_prefilled(cfg, w, audio, text[:-1], 128)
    ver = _verifier(cfg, w, "f32", max_nodes=16, capacity=128)
    ver.set_cache(kc[None].astype(np.float32), vc[None].astype(np.float32), [L])
    root, emitted, rounds = int(text[-1]), [], 0
    while len(emitted) < n_new:
        n = int(rng.integers(1, 17))
        parents = wl.random_tree(rng, n)
        depth, _ = oracle.tree_meta(parents)
        tokens = rng.integers(0, cfg["vocab"], n).astype(np.int32)
        tokens[0] = root
        for i in range(1, n):
            k = len(emitted) + depth[i] - 1
            if k < len(ref) and rng.uniform() < 0.75:
                tokens[i] = ref[k]
        out = ver.verify_tree([tokens], [parents])
        assert out["status"] == 0
        alen = int(out["accept_len"][0])
        emitted += [int(tokens[j]) for j in out["path"][0, 1:alen]] + [int(out["next_token"][0])]
        root = int(out["next_token"][0])
        rounds += 1
    assert emitted[:n_new] == ref
    assert rounds < n_new
    assert ver.kv_len[0] == L + len(emitted)
    ver.close()


@pytest.mark.parametrize("dtype,tol", [("f32", TOL_F32), ("bf16", TOL_BF16)])
def test_chain_prefill_with_audio_embeddings(dtype, tol):
    """Audio-embedding rows enter as input embeddings of a chain tree; committing the whole chain
    is prefill.  The resulting cache equals the oracle's prefill."""
    cfg = wl.MODELS["tiny"]
    w = wl.make_weights(cfg, 87, dtype)
    rng = np.random.default_rng(88)
    n_a, n_t = 21, 11
    audio = rng.standard_normal((n_a, cfg["d_model"])).astype(np.float32)
    if dtype == "bf16":
        audio = wl.bf16_to_f32(wl.bf16_bits(audio))
    text = rng.integers(0, cfg["vocab"], n_t).astype(np.int32)
    om, kc, vc, L, last = oracle_prefilled(cfg, w, audio, text, 64)
    ver = _verifier(cfg, w, dtype, max_nodes=32, capacity=64)
    n = n_a + n_t
    emb = torch.zeros((1, 32, cfg["d_model"]), dtype=ver.tdtype, device=ver.device)
    emb[0, :n_a] = torch.from_numpy(audio).to(ver.device).to(ver.tdtype)
    tok = np.zeros(n, np.int32)
    tok[n_a:] = text
    fw = ver.tree_forward([tok], [np.arange(-1, n - 1)], embeds=emb,
                          use_embed=[[1] * n_a + [0] * n_t])
    assert fw["status"] == 0
    assert ver.commit([n], [list(range(n))]) == 0
    assert ver.kv_len[0] == n == L
    k1, v1 = ver.get_cache()
    for got, want in ((k1, kc), (v1, vc)):
        g = widen_cache(got[0, :, :, :n])
        assert np.abs(g - want[:, :, :n]).max() <= tol * np.abs(want[:, :, :n]).max()
    err = row_rel_err(fw["logits"][0, n - 1].cpu().numpy()[None], last[None])
    assert err.max() <= tol
    ver.close()


@pytest.mark.parametrize("dtype,tol,max_nodes", [("f32", TOL_F32, 16), ("bf16", TOL_BF16, 64),
                                                 ("bf16", TOL_BF16, 24)])
def test_prefill_entry_point_equals_oracle_prefill(dtype, tol, max_nodes):
    """specasr_prefill on a batch of three sequences (audio embeddings then prompt tokens; lengths
    that are not multiples of the chunk size; one sequence that already holds a prefix; one with
    nothing to add): cache rows, kv_len and the greedy token after the last position equal the
    oracle's prefill of each sequence alone."""
    _check_prefill(dtype, tol, max_nodes, n_audio=[70, 0, 33], n_text=[41, 0, 9], L0=[0, 12, 20],
                   cap=192, max_pos=120)


@pytest.mark.parametrize("max_nodes,n_audio,n_text", [
    (16, [250, 100, 64], [63, 15, 16]),     # 313 positions: passes of 256 and 57 rows; 115 rows (8 pieces, last of 3); 80 rows
    (64, [150, 0, 140], [52, 0, 10]),       # 202 rows (4 pieces, last of 10; half a row tile empty); nothing; 150 rows
    (24, [300, 20, 0], [0, 0, 49]),         # 300 rows (13 pieces), embeddings only; one chunk on the skinny kernels; 49 rows in 3 pieces, tokens only
    (16, [200, 17, 0], [57, 0, 0]),         # 257 positions: a full pass of 256 rows and a pass of ONE row; 17 positions: pieces of 16 + 1; nothing
])
def test_prefill_wide_passes_equal_oracle_prefill(max_nodes, n_audio, n_text):
    """Long prefixes: the library takes a sequence that adds more than one chunk in passes of up
    to 16 chunks at once, whose projections run on the tiled (matrix-core-bound) GEMM
    -- row counts that fill, half fill and overflow its 128-row tiles, feature counts that leave a
    partial 256-feature tile (gate|up has 44 bands) and an odd number of k-steps (down: 43).  The
    result is the same as the oracle's position-by-chunk prefill."""
    _check_prefill("bf16", TOL_BF16, max_nodes, n_audio=n_audio, n_text=n_text, L0=[7, 0, 20],
                   cap=400, max_pos=320)


def test_prefill_without_wide_passes_runs_chunks_on_two_lanes():
    """A context created with SPECASR_FLAG_NO_WIDE has no wide buffers: the same long prefixes go through
    chunks of max_nodes positions, consecutive chunks alternating between two streams that are
    ordered layer by layer with events.  Same result."""
    from paper_2507_18181_amd import binding as B
    _check_prefill("bf16", TOL_BF16, 16, n_audio=[250, 100, 64], n_text=[63, 15, 16], L0=[7, 0, 20],
                   cap=400, max_pos=320, flags=B.SPECASR_FLAG_NO_WIDE)


def _check_prefill(dtype, tol, max_nodes, n_audio, n_text, L0, cap, max_pos, flags=0):
    cfg = wl.MODELS["tiny"]
    w = wl.make_weights(cfg, 97, dtype)
    rng = np.random.default_rng(98)
    d = cfg["d_model"]
    om = oracle.OracleModel(cfg, w)
    nb = 3
    ver = _verifier(cfg, w, dtype, max_nodes=max_nodes, capacity=cap, max_batch=nb, flags=flags)
    K, V = wl.seeded_cache(cfg, 99, np.asarray(L0, np.int32), cap, dtype, batch=nb)
    ver.set_cache(K, V, L0)
    emb = torch.zeros((nb, max_pos, d), dtype=ver.tdtype, device=ver.device)
    toks, flags, audio = [], [], []
    for b in range(nb):
        a = rng.standard_normal((n_audio[b], d)).astype(np.float32)
        if dtype == "bf16":
            a = wl.bf16_to_f32(wl.bf16_bits(a))
        audio.append(a)
        emb[b, :n_audio[b]] = torch.from_numpy(a).to(ver.device).to(ver.tdtype)
        text = rng.integers(0, cfg["vocab"], n_text[b]).astype(np.int32)
        toks.append(np.concatenate([np.zeros(n_audio[b], np.int32), text]))
        flags.append([1] * n_audio[b] + [0] * n_text[b])
    out = ver.prefill(toks, embeds=emb, use_embed=flags)
    assert out["status"] == 0
    k1, v1 = ver.get_cache()
    for b in range(nb):
        n = n_audio[b] + n_text[b]
        assert ver.kv_len[b] == L0[b] + n
        kc, vc = K[b].copy(), V[b].copy()         # the oracle prefills a cache of the same storage type
        L, last = om.prefill(kc, vc, L0[b], audio[b].astype(np.float64), toks[b][n_audio[b]:], chunk=max_nodes)
        assert L == L0[b] + n
        if n == 0:
            assert out["next_token"][b] == -1
            assert np.array_equal(k1[b], K[b]) and np.array_equal(v1[b], V[b])
            continue
        # bf16: both sides store rounded rows, so elements may differ by one bf16 step (2^-8 of
        # the element) on top of the arithmetic difference
        row_tol = tol if dtype == "f32" else 5e-3
        for got, want, before in ((k1[b], kc, K[b]), (v1[b], vc, V[b])):
            g, wv = widen_cache(got[:, :, L0[b]:L]), widen_cache(want[:, :, L0[b]:L])
            assert np.abs(g - wv).max() <= row_tol * np.abs(wv).max()
            assert np.array_equal(got[:, :, :L0[b]], before[:, :, :L0[b]])   # the old prefix is untouched
        srt = np.sort(last)
        if srt[-1] - srt[-2] > 0.05:
            assert out["next_token"][b] == int(np.argmax(last))
    # error paths enqueue nothing: overflow and a bad token id leave kv_len alone
    before = ver.kv_len.copy()
    assert ver.prefill([[1] * (cap + 8), [], []])["status"] == -4
    assert ver.prefill([[cfg["vocab"]], [], []])["status"] == -3
    assert np.array_equal(ver.kv_len, before)
    ver.close()


@pytest.mark.parametrize("shape", [
    dict(n_heads=4, n_kv_heads=2, head_dim=64),     # grouped-query, 2 query heads per KV head
    dict(n_heads=8, n_kv_heads=1, head_dim=64, d_model=512),   # 8 query heads on one KV head
    dict(n_heads=2, n_kv_heads=2, head_dim=128),    # head_dim 128, multi-head
    dict(n_heads=4, n_kv_heads=1, head_dim=128, d_model=512),  # head_dim 128, grouped
    dict(n_heads=8, n_kv_heads=8, head_dim=32),     # head_dim the MFMA attention does not cover
])
def test_attention_shapes_bf16(shape):
    """GQA groupings and head sizes through the bf16 path, trees up to 64 nodes (several 32-query
    groups per KV head), ragged prefix lengths around the 32-key tile size."""
    cfg = dict(wl.MODELS["tiny"], **shape)
    w = wl.make_weights(cfg, 91, "bf16")
    rng = np.random.default_rng(92)
    text = rng.integers(0, cfg["vocab"], 200).astype(np.int32)
    om, kc, vc, Lfull, _ = oracle_prefilled(cfg, w, None, text, 280)
    ver = _verifier(cfg, w, "bf16", max_nodes=64, capacity=280)
    for n, L in ((1, 1), (5, 31), (32, 32), (33, 95), (64, 200), (17, 0)):
        parents = wl.random_tree(rng, n, max_children=3)
        tokens = rng.integers(0, cfg["vocab"], n).astype(np.int32)
        ver.set_cache(_store_cache(kc, "bf16"), _store_cache(vc, "bf16"), [L])
        k0, v0 = ver.get_cache()
        ref = om.tree_forward(k0[0], v0[0], L, tokens, parents)
        fw = ver.tree_forward([tokens], [parents])
        assert fw["status"] == 0
        check_forward(ref, fw["logits"][0].cpu().numpy(), fw["argmax"][0].cpu().numpy(), TOL_BF16)
        k1, v1 = ver.get_cache()
        check_tree_kv(k1[0], v1[0], L, ref, TOL_BF16)
    ver.close()


@pytest.mark.parametrize("shape", [
    dict(n_heads=2, n_kv_heads=2, head_dim=128),                      # head_dim 128: two bands per rotary half
    dict(n_heads=8, n_kv_heads=1, head_dim=64, d_model=512),          # 8 query heads on one KV head
    dict(n_heads=4, n_kv_heads=2, head_dim=128, d_model=272, d_ffn=1008, vocab=1003),  # 17 / 63 k-steps, partial tiles everywhere
    dict(n_heads=1, n_kv_heads=1, head_dim=64, d_model=48, d_ffn=80, vocab=97),        # 3 / 5 k-steps: shorter than a k-split
])
def test_wide_pass_shapes_bf16(shape):
    """A batch of 5 sequences with 190 tree nodes in all, i.e. one wide pass (tiled GEMM, band-block
    finishing kernels, direct or merged attention output), over head sizes, GQA groupings and widths
    that leave partial feature tiles, partial row tiles and odd k-step counts: every sequence equals
    the oracle run on it alone; then the same model prefills 150 positions in a wide pass."""
    from paper_2507_18181_amd import binding as B
    cfg = dict(wl.MODELS["tiny"], **shape)
    w = wl.make_weights(cfg, 141, "bf16")
    rng = np.random.default_rng(142)
    sizes, Ls = (64, 7, 33, 64, 22), [150, 0, 31, 64, 97]
    nb, cap = len(sizes), 224
    K, V = wl.seeded_cache(cfg, 143, np.asarray(Ls, np.int32), cap, "bf16", batch=nb)
    om = oracle.OracleModel(cfg, w)
    ver = _verifier(cfg, w, "bf16", max_nodes=64, capacity=cap, max_batch=nb)
    assert B.specasr_uses_mfma(ver.ctx, sum(sizes)) == 1
    ver.set_cache(K, V, Ls)
    trees = [wl.random_tree(rng, n, max_children=3) for n in sizes]
    toks = [rng.integers(0, cfg["vocab"], n).astype(np.int32) for n in sizes]
    fw = ver.tree_forward(toks, trees, want_logits=True)
    assert fw["status"] == 0
    k1, v1 = ver.get_cache()
    for b in range(nb):
        ref = om.tree_forward(np.ascontiguousarray(K[b]), np.ascontiguousarray(V[b]), Ls[b], toks[b], trees[b])
        check_forward(ref, fw["logits"][b].cpu().numpy(), fw["argmax"][b].cpu().numpy(), TOL_BF16)
        check_tree_kv(k1[b], v1[b], Ls[b], ref, TOL_BF16)
    # prefill of sequence 1 (empty so far): 150 positions = one wide pass of 128 + 22 rows
    text = rng.integers(0, cfg["vocab"], 150).astype(np.int32)
    ver.set_cache(K, V, Ls)
    out = ver.prefill([[], text, [], [], []])
    assert out["status"] == 0 and ver.kv_len[1] == 150
    kc, vc = K[1].copy(), V[1].copy()
    Lp, last = om.prefill(kc, vc, 0, None, text, chunk=64)
    k2, v2 = ver.get_cache()
    for got, want in ((k2[1], kc), (v2[1], vc)):
        g, wv = widen_cache(got[:, :, :Lp]), widen_cache(want[:, :, :Lp])
        assert np.abs(g - wv).max() <= 5e-3 * np.abs(wv).max()
    srt = np.sort(last)
    if srt[-1] - srt[-2] > 0.05:
        assert out["next_token"][1] == int(np.argmax(last))
    ver.close()


@pytest.mark.parametrize("shape", [
    dict(d_model=48, d_ffn=80, n_heads=1, n_kv_heads=1, head_dim=64, vocab=97),      # 3 k-steps: fewer than wavefronts
    dict(d_model=272, d_ffn=1008, n_heads=4, n_kv_heads=2, head_dim=64, vocab=1003),  # 17 / 63 k-steps, 31.5 FFN bands
    dict(d_model=1040, d_ffn=2064, n_heads=8, n_kv_heads=2, head_dim=128, vocab=515, n_layers=1),  # 65 / 129 k-steps
    dict(d_model=2064, d_ffn=272, n_heads=2, n_kv_heads=1, head_dim=128, vocab=33, n_layers=1),    # wide model, narrow FFN
])
def test_gemm_tiling_edge_shapes_bf16(shape):
    """Model widths that do not divide into the GEMM's tiles evenly (k-steps that are not multiples
    of the 8 wavefronts or of the split count, output widths that end inside a 32-row band,
    vocabularies that are not multiples of anything), at 1, 31, 33 and 64 rows."""
    from paper_2507_18181_amd import binding as B
    cfg = dict(wl.MODELS["tiny"], **shape)
    w = wl.make_weights(cfg, 131, "bf16")
    rng = np.random.default_rng(132)
    L, cap = 45, 128
    K, V = wl.seeded_cache(cfg, 133, L, cap, "bf16")
    om = oracle.OracleModel(cfg, w)
    ver = _verifier(cfg, w, "bf16", max_nodes=64, capacity=cap)
    assert B.specasr_uses_mfma(ver.ctx, 8) == 1
    for n in (1, 31, 33, 64):
        parents = wl.random_tree(rng, n, max_children=3)
        tokens = rng.integers(0, cfg["vocab"], n).astype(np.int32)
        ver.set_cache(K, V, [L])
        ref = om.tree_forward(np.ascontiguousarray(K[0]), np.ascontiguousarray(V[0]), L, tokens, parents)
        fw = ver.tree_forward([tokens], [parents])
        assert fw["status"] == 0
        check_forward(ref, fw["logits"][0].cpu().numpy(), fw["argmax"][0].cpu().numpy(), TOL_BF16)
        k1, v1 = ver.get_cache()
        check_tree_kv(k1[0], v1[0], L, ref, TOL_BF16)
    ver.close()


@pytest.mark.parametrize("seed", range(8))
def test_seeded_random_models_and_batches_bf16(seed):
    """Seeded random draws of everything the kernels' shapes depend on -- width, FFN width, head
    count and grouping, head size, depth, vocabulary, prefix lengths, batch and tree sizes (so
    that a call lands on the skinny kernels with one or two row groups or on a wide pass, with
    single-chunk or chunked attention) -- each a whole verify round per sequence against the oracle
    run on that sequence alone, integer stages bit-exact."""
    from paper_2507_18181_amd import binding as B
    rng = np.random.default_rng([4242, seed])
    hd = int(rng.choice([64, 128]))
    Hkv = int(rng.choice([1, 2, 4]))
    H = Hkv * int(rng.choice([1, 2, 4]))
    cfg = dict(wl.MODELS["tiny"], n_layers=int(rng.integers(1, 4)), d_model=16 * int(rng.integers(3, 40)),
               d_ffn=16 * int(rng.integers(3, 70)), n_heads=H, n_kv_heads=Hkv, head_dim=hd,
               vocab=int(rng.integers(40, 1500)))
    nb = int(rng.choice([1, 1, 2, 3, 5]))
    sizes = [int(rng.integers(1, 65)) for _ in range(nb)]
    Ls = [int(rng.integers(0, 700)) for _ in range(nb)]
    cap = max(Ls) + 64
    print("cfg", {k: cfg[k] for k in ("n_layers", "d_model", "d_ffn", "n_heads", "n_kv_heads", "head_dim", "vocab")},
          "sizes", sizes, "prefixes", Ls, flush=True)
    w = wl.make_weights(cfg, 4300 + seed, "bf16")
    om = oracle.OracleModel(cfg, w)
    ver = _verifier(cfg, w, "bf16", max_nodes=64, capacity=cap, max_batch=nb)
    assert B.specasr_uses_mfma(ver.ctx, sum(sizes)) == 1
    K, V = wl.seeded_cache(cfg, 4400 + seed, np.asarray(Ls, np.int32), cap, "bf16", batch=nb)
    ver.set_cache(K, V, Ls)
    trees = [wl.random_tree(rng, n, max_children=3) for n in sizes]
    toks = [wl.tree_tokens(rng, p, cfg["vocab"]) for p in trees]
    out = ver.verify_tree(toks, trees, want_logits=True)
    assert out["status"] == 0
    k2, v2 = ver.get_cache()
    for b, n in enumerate(sizes):
        ref = om.tree_forward(np.ascontiguousarray(K[b]), np.ascontiguousarray(V[b]), Ls[b], toks[b], trees[b])
        check_forward(ref, out["logits"][b].cpu().numpy(), out["argmax"][b], TOL_BF16)
        path, alen, nxt = oracle.accept(toks[b], trees[b], out["argmax"][b, :n])
        assert out["accept_len"][b] == alen and out["next_token"][b] == nxt
        assert out["path"][b, :alen].tolist() == path.tolist()
        assert ver.kv_len[b] == Ls[b] + alen
        sub = {"ktree": ref["ktree"][:, :, path], "vtree": ref["vtree"][:, :, path]}
        check_tree_kv(k2[b], v2[b], Ls[b], sub, TOL_BF16)
        assert np.array_equal(k2[b][:, :, :Ls[b]], K[b][:, :, :Ls[b]])      # the prefix is untouched
    ver.close()
