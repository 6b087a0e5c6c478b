"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and every validation error is raised on the host before anything is enqueued."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import workload as wl
from paper_2507_18181_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000  # 256-aligned non-NULL "device address"; never dereferenced by a failing call


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2507_18181_amd import build
        build.build(verbose=False)
    return B.load_library()


def _fake_weights(cfg):
    w = {k: FAKE for k in ("tok_embed", "final_norm", "lm_head")}
    w["layers"] = [{f: FAKE for f in B.LAYER_FIELDS} for _ in range(cfg["n_layers"])]
    return B.make_weights(w)


@pytest.fixture()
def ctx(lib):
    cfg = wl.MODELS["tiny"]
    sw, keep = _fake_weights(cfg)
    rc, c = B.specasr_create(B.make_config(cfg, B.SPECASR_F32, 8, 2), sw)
    assert rc == B.SPECASR_OK
    yield c
    B.specasr_destroy(c)


def test_exports_match_header(lib):
    hdr = "".join(open(os.path.join(ROOT, "include", h)).read() for h in ("specasr.h", "specasr_profile.h"))
    declared = set(re.findall(r"\b(specasr_[a-z0-9_]+)\s*\(", hdr))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert B.specasr_abi_version() == 1
    for s in range(-8, 1):
        assert B.specasr_strerror(s) not in ("", "unknown status")


def test_struct_sizes_match_header_layout():
    assert C.sizeof(B.specasr_config) == 13 * 4
    assert C.sizeof(B.specasr_layer_weights) == 9 * 8
    assert C.sizeof(B.specasr_kv) == 8 + 8 + 8 + 4 + 4 + 8
    assert C.sizeof(B.specasr_tree) == 5 * 8
    assert C.sizeof(B.specasr_out) == 5 * 8


def test_create_rejects_bad_configs(lib):
    cfg = wl.MODELS["tiny"]
    sw, keep = _fake_weights(cfg)
    bad = [dict(n_heads=3, n_kv_heads=2), dict(head_dim=12), dict(d_model=250), dict(d_ffn=5),
           dict(vocab=0), dict(n_layers=0), dict(rope_theta=0.0), dict(head_dim=96)]
    for delta in bad:
        c2 = dict(cfg, **delta)
        rc, c = B.specasr_create(B.make_config(c2, B.SPECASR_F32, 8, 1), sw)
        assert rc == B.SPECASR_E_CONFIG, delta
    for mn, mb, dt in ((0, 1, 0), (65, 1, 0), (8, 0, 0), (8, 1, 7)):
        rc, c = B.specasr_create(B.make_config(cfg, dt, mn, mb), sw)
        assert rc == B.SPECASR_E_CONFIG
    rc, c = B.specasr_create(None, sw)
    assert rc == B.SPECASR_E_NULL
    w = {k: FAKE for k in ("tok_embed", "final_norm", "lm_head")}
    w["layers"] = [{f: (None if f == "wo" else FAKE) for f in B.LAYER_FIELDS} for _ in range(2)]
    sw2, keep2 = B.make_weights(w)
    rc, c = B.specasr_create(B.make_config(cfg, B.SPECASR_F32, 8, 1), sw2)
    assert rc == B.SPECASR_E_NULL


def _call(ctx, tokens, parents, n_nodes, kv_len, capacity=100, ws=FAKE, ws_bytes=None, batch=None):
    nb = len(n_nodes)
    tok = np.zeros((nb, 8), np.int32)
    par = np.full((nb, 8), -1, np.int32)
    for b in range(nb):
        tok[b, :len(tokens[b])] = tokens[b]
        par[b, :len(parents[b])] = parents[b]
    nn = np.asarray(n_nodes, np.int32)
    kvl = np.asarray(kv_len, np.int32)
    before = kvl.copy()
    kv = B.make_kv(FAKE, FAKE, capacity, kvl)
    tree = B.make_tree(tok, par, nn)
    out = B.make_out(np.zeros((nb, 8), np.int32), np.zeros((nb, 8), np.int32),
                     np.zeros(nb, np.int32), np.zeros(nb, np.int32))
    if ws_bytes is None:
        ws_bytes = B.specasr_workspace_bytes(ctx, nb)
    rc = B.specasr_verify_tree(ctx, kv, tree, out, ws, ws_bytes)
    assert np.array_equal(kvl, before)      # a failing call leaves kv_len alone
    return rc


def test_tree_and_kv_validation_happens_on_the_host(ctx):
    good_t, good_p = [1, 2, 3], [-1, 0, 1]
    assert B.specasr_workspace_bytes(ctx, 1) > 0
    assert B.specasr_workspace_bytes(ctx, 3) == 0                       # beyond max_batch
    assert _call(ctx, [good_t], [[0, 0, 1]], [3], [10]) == B.SPECASR_E_TREE      # root parent != -1
    assert _call(ctx, [good_t], [[-1, 1, 1]], [3], [10]) == B.SPECASR_E_TREE     # parent >= child
    assert _call(ctx, [good_t], [[-1, 0, 5]], [3], [10]) == B.SPECASR_E_TREE
    assert _call(ctx, [good_t], [[-1, -1, 0]], [3], [10]) == B.SPECASR_E_TREE    # second root
    assert _call(ctx, [good_t], [good_p], [0], [10]) == B.SPECASR_E_TREE
    assert _call(ctx, [good_t], [good_p], [9], [10]) == B.SPECASR_E_TREE         # > max_nodes
    assert _call(ctx, [[1, 1000, 3]], [good_p], [3], [10]) == B.SPECASR_E_TREE   # token == vocab
    assert _call(ctx, [[1, -1, 3]], [good_p], [3], [10]) == B.SPECASR_E_TREE
    assert _call(ctx, [good_t], [good_p], [3], [98]) == B.SPECASR_E_KV_OVERFLOW  # 98 + 3 > 100
    assert _call(ctx, [good_t], [good_p], [3], [-1]) == B.SPECASR_E_KV_OVERFLOW
    assert _call(ctx, [good_t] * 2, [good_p] * 2, [3, 3], [10, 99]) == B.SPECASR_E_KV_OVERFLOW
    assert _call(ctx, [good_t] * 3, [good_p] * 3, [3, 3, 3], [1, 1, 1]) == B.SPECASR_E_TREE  # batch > max
    assert _call(ctx, [good_t], [good_p], [3], [10], ws=None) == B.SPECASR_E_WORKSPACE
    assert _call(ctx, [good_t], [good_p], [3], [10], ws=FAKE + 8) == B.SPECASR_E_WORKSPACE
    assert _call(ctx, [good_t], [good_p], [3], [10], ws_bytes=1024) == B.SPECASR_E_WORKSPACE


def test_null_arguments(ctx):
    kvl = np.array([5], np.int32)
    kv = B.make_kv(FAKE, FAKE, 100, kvl)
    tok, par, nn = np.zeros((1, 8), np.int32), np.full((1, 8), -1, np.int32), np.array([1], np.int32)
    tree = B.make_tree(tok, par, nn)
    out = B.make_out(None, np.zeros((1, 8), np.int32), np.zeros(1, np.int32), np.zeros(1, np.int32))
    wsb = B.specasr_workspace_bytes(ctx, 1)
    assert B.specasr_verify_tree(ctx, kv, tree, out, FAKE, wsb) == B.SPECASR_E_NULL
    kv0 = B.make_kv(None, FAKE, 100, kvl)
    out = B.make_out(*[np.zeros((1, 8), np.int32)] * 2, np.zeros(1, np.int32), np.zeros(1, np.int32))
    assert B.specasr_verify_tree(ctx, kv0, tree, out, FAKE, wsb) == B.SPECASR_E_NULL
    assert B.specasr_tree_forward(ctx, kv, tree, None, None, FAKE, wsb) == B.SPECASR_E_NULL
    assert B.specasr_accept(ctx, tree, 1, None, FAKE, FAKE, FAKE, FAKE, wsb) == B.SPECASR_E_NULL
    # embeddings and their flags must come together
    t2 = B.make_tree(tok, par, nn, input_embeds=FAKE, use_embed=None)
    assert B.specasr_tree_forward(ctx, kv, t2, FAKE, None, FAKE, wsb) == B.SPECASR_E_NULL


def test_commit_path_validation(ctx):
    wsb = B.specasr_workspace_bytes(ctx, 1)

    def commit(path, n, kv_len=10, cap=100):
        kvl = np.array([kv_len], np.int32)
        kv = B.make_kv(FAKE, FAKE, cap, kvl)
        p = np.full((1, 8), -1, np.int32)
        p[0, :len(path)] = path
        rc = B.specasr_commit(ctx, kv, np.array([n], np.int32), p, np.array([len(path)], np.int32),
                              FAKE, wsb)
        assert kvl[0] == kv_len
        return rc

    assert commit([1, 2], 4) == B.SPECASR_E_PATH        # must start at the root
    assert commit([0, 2, 2], 4) == B.SPECASR_E_PATH     # strictly increasing
    assert commit([0, 3, 2], 4) == B.SPECASR_E_PATH
    assert commit([0, 4], 4) == B.SPECASR_E_PATH        # node index beyond the tree
    assert commit([], 4) == B.SPECASR_E_PATH
    assert commit([0, 1], 0) == B.SPECASR_E_TREE
    assert commit([0, 1], 4, kv_len=98) == B.SPECASR_E_KV_OVERFLOW


def test_prefill_and_draft_forward_validate_on_the_host(ctx):
    """specasr_prefill / specasr_tree_forward_top2: argument errors are found before anything is
    enqueued (no GPU here), and kv_len is left alone."""
    wsb = B.specasr_workspace_bytes(ctx, 1)
    kvl = np.array([90], np.int32)
    kv = B.make_kv(FAKE, FAKE, 100, kvl)
    tok = np.zeros((1, 16), np.int32)
    one = np.array([5], np.int32)
    flags = np.zeros((1, 16), np.uint8)
    nxt = np.zeros(1, np.int32)
    assert B.specasr_prefill(ctx, kv, tok, None, None, None, 16, nxt, FAKE, wsb) == B.SPECASR_E_NULL
    assert B.specasr_prefill(ctx, kv, None, None, None, one, 16, nxt, FAKE, wsb) == B.SPECASR_E_NULL
    assert B.specasr_prefill(ctx, kv, tok, FAKE, None, one, 16, nxt, FAKE, wsb) == B.SPECASR_E_NULL
    assert B.specasr_prefill(ctx, kv, tok, None, None, np.array([17], np.int32), 16, nxt, FAKE, wsb) == B.SPECASR_E_TREE
    assert B.specasr_prefill(ctx, kv, tok, None, None, np.array([-1], np.int32), 16, nxt, FAKE, wsb) == B.SPECASR_E_TREE
    assert B.specasr_prefill(ctx, kv, tok, None, None, np.array([11], np.int32), 16, nxt, FAKE, wsb) == B.SPECASR_E_KV_OVERFLOW
    bad = tok.copy()
    bad[0, 3] = 1000                                         # == vocab
    assert B.specasr_prefill(ctx, kv, bad, None, None, one, 16, nxt, FAKE, wsb) == B.SPECASR_E_TREE
    flags[0, 3] = 1                                          # ... but ignored where an embedding is used
    assert B.specasr_prefill(ctx, kv, bad, FAKE, flags, one, 16, nxt, FAKE, 1024) == B.SPECASR_E_WORKSPACE
    assert B.specasr_prefill(ctx, kv, tok, None, None, one, 16, nxt, None, wsb) == B.SPECASR_E_WORKSPACE
    assert kvl[0] == 90
    par, nn = np.full((1, 8), -1, np.int32), np.array([1], np.int32)
    tree = B.make_tree(np.zeros((1, 8), np.int32), par, nn)
    assert B.specasr_tree_forward_top2(ctx, kv, tree, None, FAKE, None, FAKE, wsb) == B.SPECASR_E_NULL
    assert B.specasr_tree_forward_top2(ctx, kv, tree, FAKE, None, None, FAKE, wsb) == B.SPECASR_E_NULL
    assert B.specasr_tree_forward_top2(ctx, kv, tree, FAKE, FAKE, None, FAKE, 1024) == B.SPECASR_E_WORKSPACE
    kv2 = B.make_kv(FAKE, FAKE, 100, np.array([100], np.int32))
    assert B.specasr_tree_forward_top2(ctx, kv2, tree, FAKE, FAKE, None, FAKE, wsb) == B.SPECASR_E_KV_OVERFLOW


def test_measurement_aids_need_the_mfma_path(ctx):
    """specasr_profile_stage / specasr_stage_time / specasr_stage_rows: a context without repacked
    weights (fp32, or no GPU) reports UNSUPPORTED, bad stages and NULL handles are rejected."""
    assert B.specasr_profile_stage(ctx, 2, 1) == B.SPECASR_E_UNSUPPORTED
    assert B.specasr_profile_stage(ctx, 7, 1) == B.SPECASR_E_UNSUPPORTED
    assert B.specasr_profile_stage(None, 2, 1) == B.SPECASR_E_NULL
    assert B.specasr_stage_time(ctx)[0] == B.SPECASR_E_UNSUPPORTED
    assert B.specasr_stage_rows(ctx)[0] == B.SPECASR_E_UNSUPPORTED
    assert B.specasr_stage_rows(None)[0] == B.SPECASR_E_NULL
    assert B.specasr_uses_mfma(ctx, 200) == 0
    # the read-ceiling probe validates its arguments before it touches a GPU
    assert B.specasr_read_ceiling(None, 0x1000, 1 << 22)[0] == B.SPECASR_E_NULL
    assert B.specasr_read_ceiling(ctx, None, 1 << 22)[0] == B.SPECASR_E_NULL
    assert B.specasr_read_ceiling(ctx, 0x1000, 1 << 10)[0] == B.SPECASR_E_UNSUPPORTED      # under 1 MiB
    assert B.specasr_read_ceiling(ctx, 0x1008, 1 << 22)[0] == B.SPECASR_E_UNSUPPORTED      # not 16-byte aligned
    assert B.specasr_read_ceiling(ctx, 0x1000, 1 << 22, reps=0)[0] == B.SPECASR_E_UNSUPPORTED


def test_static_entry_point_rejects_sizes_beyond_its_device_array(lib):
    """specasr_accept_from_logits_static holds at most SPECASR_STATIC_MAX_BATCH trees: a larger
    batch is refused on the host, before anything touches a GPU."""
    cfg = wl.MODELS["tiny"]
    sw, keep = _fake_weights(cfg)
    nb = B.SPECASR_STATIC_MAX_BATCH + 1
    rc, c = B.specasr_create(B.make_config(cfg, B.SPECASR_F32, 8, nb), sw)
    assert rc == B.SPECASR_OK
    tok = np.zeros((nb, 8), np.int32)
    par = np.full((nb, 8), -1, np.int32)
    nn = np.ones(nb, np.int32)
    tree = B.make_tree(tok, par, nn)
    fake = 0x1000
    assert B.specasr_accept_from_logits_static(c, tree, nb, fake, fake, fake, fake, fake) == B.SPECASR_E_UNSUPPORTED
    assert B.specasr_accept_from_logits_static(c, tree, nb, None, fake, fake, fake, fake) == B.SPECASR_E_NULL
    par[0, 0] = 0                                   # invalid tree: reported as such, as by the workspace variant
    assert B.specasr_accept_from_logits_static(c, tree, 2, fake, fake, fake, fake, fake) == B.SPECASR_E_TREE
    B.specasr_destroy(c)
