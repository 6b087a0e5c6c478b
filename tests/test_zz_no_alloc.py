"""specasr_accept_from_logits_static -- the entry point that allocates nothing -- against
specasr_accept_from_logits (the same stage with a caller workspace), bit for bit, through the C
ABI: two calls in a row on the shared device array, the second with a smaller input, so that
whatever the first call left in the array must not leak into the second."""
import numpy as np
import pytest
import torch

import oracle
import workload as wl
from paper_2507_18181_amd import binding as B
from paper_2507_18181_amd.runtime import Verifier

pytestmark = pytest.mark.gpu


def _case(rng, sizes, vocab, max_nodes):
    trees = [wl.random_tree(rng, n, max_children=3) for n in sizes]
    # few distinct ids: many matches, duplicate siblings, exact ties in the logits
    toks = [rng.integers(0, 5, n).astype(np.int32) for n in sizes]
    lg = np.zeros((len(sizes), max_nodes, vocab), np.float32)
    for b, n in enumerate(sizes):
        lg[b, :n] = rng.standard_normal((n, vocab)).astype(np.float32)
        hot = rng.integers(0, 5, n)
        lg[b, np.arange(n), hot] += 10.0
        if n > 2:
            lg[b, 2, 4] = lg[b, 2, 1] = lg[b, 2].max() + 1.0      # tie: lowest id wins
    return trees, toks, lg


def _run(ver, trees, toks, lg, static):
    nb = len(trees)
    dev = ver.device
    tree, keep = ver._tree(toks, trees)
    am = torch.full((nb, ver.max_nodes), -9, dtype=torch.int32, device=dev)
    path = torch.full((nb, ver.max_nodes), -9, dtype=torch.int32, device=dev)
    alen = torch.full((nb,), -9, dtype=torch.int32, device=dev)
    nxt = torch.full((nb,), -9, dtype=torch.int32, device=dev)
    lgd = torch.from_numpy(lg).to(dev)
    if static:
        rc = B.specasr_accept_from_logits_static(ver.ctx, tree, nb, lgd, am, path, alen, nxt, None)
    else:
        rc = B.specasr_accept_from_logits(ver.ctx, tree, nb, lgd, am, path, alen, nxt, ver.ws_ptr,
                                          ver.ws_bytes, None)
    torch.cuda.synchronize()
    assert rc == 0, B.specasr_strerror(rc)
    return [t.cpu().numpy() for t in (am, path, alen, nxt)]


def test_static_entry_point_equals_the_workspace_one_on_two_calls_in_a_row():
    cfg = wl.MODELS["tiny"]
    w = wl.make_weights(cfg, 91, "f32")
    ver = Verifier(cfg, w, "f32", max_nodes=64, capacity=64, max_batch=B.SPECASR_STATIC_MAX_BATCH + 1)
    rng = np.random.default_rng(92)
    # first call: a full batch of large trees; second call: fewer and smaller trees
    for sizes in ([64, 1, 33, 64, 17, 2, 64, 48, 5, 64, 31, 64, 9, 64, 3, 64], [7, 1, 12]):
        trees, toks, lg = _case(rng, sizes, cfg["vocab"], 64)
        got = _run(ver, trees, toks, lg, static=True)
        want = _run(ver, trees, toks, lg, static=False)
        for b, n in enumerate(sizes):
            assert np.array_equal(got[0][b, :n], want[0][b, :n])          # argmax
            assert got[2][b] == want[2][b] and got[3][b] == want[3][b]    # accept_len, next_token
            assert np.array_equal(got[1][b], want[1][b])                  # path incl. the -1 tail
            # and both equal the oracle's acceptance on that argmax
            p, alen, nx = oracle.accept(toks[b], trees[b], got[0][b, :n])
            assert alen == got[2][b] and nx == got[3][b] and got[1][b, :alen].tolist() == p.tolist()
    # beyond the limit: refused before anything is enqueued, outputs untouched
    sizes = [3] * (B.SPECASR_STATIC_MAX_BATCH + 1)
    trees, toks, lg = _case(rng, sizes, cfg["vocab"], 64)
    tree, keep = ver._tree(toks, trees)
    am = torch.full((len(sizes), 64), -9, dtype=torch.int32, device=ver.device)
    rc = B.specasr_accept_from_logits_static(ver.ctx, tree, len(sizes), torch.from_numpy(lg).to(ver.device),
                                             am, am, am, am, None)
    torch.cuda.synchronize()
    assert rc == B.SPECASR_E_UNSUPPORTED
    assert int(am.min()) == -9 and int(am.max()) == -9
    ver.close()
