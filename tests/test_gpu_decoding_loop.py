"""The draft-then-verify loop (paper_2507_18181_amd.decoding) on the GPU against the definition:
speculative decoding is lossless (Sec. II-B), so whatever the draft model proposes, the produced
tokens are the target model's own greedy decoding -- here computed by the fp64 oracle, one
single-node round per token."""
import numpy as np
import pytest

import oracle
import workload as wl
from parity_util import TOL_F32

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

CAP = 256


def _peaky(w, k):
    """LM head scaled by k: sharper output distributions, so that probabilities cross thresholds."""
    w = dict(w)
    w["lm_head"] = (w["lm_head"] * np.float32(k)).astype(np.float32)
    return w


def _oracle_greedy(cfg, w, audio, text, n_new):
    """(tokens, decisive flags): the target's greedy continuation after the prompt."""
    om = oracle.OracleModel(cfg, w)
    kc, vc = om.empty_cache(CAP)
    L, _ = om.prefill(kc, vc, 0, audio.astype(np.float64), text[:-1])
    t, toks, dec = int(text[-1]), [], []
    for _ in range(n_new):
        r = om.tree_forward(kc, vc, L, np.array([t], np.int32), np.array([-1], np.int32))
        L = om.commit(kc, vc, L, r["ktree"], r["vtree"], [0])
        # fp32 model: the GPU's logits are within TOL_F32 * max|logit| of these, so a gap of ten
        # times that cannot flip
        srt = np.sort(r["logits"][0])
        dec.append(srt[-1] - srt[-2] > 10 * TOL_F32 * np.abs(srt).max())
        t = int(r["amax"][0])
        toks.append(t)
    return toks, dec


def _pair(cfg, w_target, w_draft, audio, text):
    from paper_2507_18181_amd.runtime import Verifier
    vers = []
    for w in (w_target, w_draft):
        v = Verifier(cfg, w, "f32", max_nodes=64, capacity=CAP)
        emb = torch.zeros((1, len(audio) + len(text) - 1, cfg["d_model"]), dtype=torch.float32, device=v.device)
        emb[0, :len(audio)] = torch.from_numpy(audio).to(v.device)
        tok = np.concatenate([np.zeros(len(audio), np.int32), text[:-1]])
        out = v.prefill([tok], embeds=emb, use_embed=[[1] * len(audio) + [0] * (len(text) - 1)], want_next=False)
        assert out["status"] == 0
        vers.append(v)
    return vers


def _check_lossless(got, want, dec):
    """Equal up to (and including) the first step at which the oracle itself is not decisive."""
    n = min(len(got), len(want))
    stop = next((i for i in range(n) if not dec[i]), n)
    assert got[:stop] == want[:stop]
    return stop


@pytest.mark.parametrize("mode", ["asp", "tsp"])
@pytest.mark.parametrize("kind", ["self", "foreign", "noisy"])
def test_loop_reproduces_the_targets_greedy_decoding(mode, kind):
    """Three draft models for one target: the target itself (every draft accepted), an unrelated
    model (nothing but the root accepted), the target with 3 % weight noise (partial acceptance,
    branches and recycling in play).  In every case the output is the oracle's greedy decoding."""
    from paper_2507_18181_amd.decoding import SpecDecoder
    cfg = wl.MODELS["tiny"]
    w_t = _peaky(wl.make_weights(cfg, 321, "f32"), 6.0)   # a seed whose 90 greedy steps are all decisive
    if kind == "self":
        w_d = w_t
    elif kind == "foreign":
        w_d = _peaky(wl.make_weights(cfg, 999, "f32"), 6.0)
    else:
        rng = np.random.default_rng(312)
        w_d = {k: (v if k == "layers" else (v * (1 + 0.03 * rng.standard_normal(v.shape))).astype(np.float32))
               for k, v in w_t.items()}
        w_d["layers"] = [{k: (v * (1 + 0.03 * rng.standard_normal(v.shape))).astype(np.float32)
                          for k, v in lw.items()} for lw in w_t["layers"]]
    audio, text = wl.make_prefix_inputs(cfg, 313, 20, 6)
    n_new = 90
    want, dec = _oracle_greedy(cfg, w_t, audio, text, n_new)
    target, draft = _pair(cfg, w_t, w_d, audio, text)
    sd = SpecDecoder(target, draft, root=int(text[-1]), threshold=0.05, mode=mode, max_draft=24)   # about a third of the tokens fall below it
    got = sd.decode(n_new)
    st = sd.stats
    print("%s/%s: %d tokens in %d rounds, %d draft forwards, accepted/round %.2f, nodes/round %.1f, "
          "branch hits %d, recycled %d" % (kind, mode, len(got), st.rounds, st.draft_forwards,
                                           np.mean(st.accepted), np.mean(st.tree_nodes), st.branch_hits, st.recycled))
    stop = _check_lossless(got, want, dec)
    assert stop == n_new
    assert len(got) >= n_new and max(st.tree_nodes) <= 64
    assert target.kv_len[0] == draft.kv_len[0] == len(audio) + len(text) - 1 + len(got)
    if kind == "self" and stop == n_new:
        # the draft equals the target: only the length limit or (asp) an uncertain token ends a trunk,
        # and every drafted trunk token is accepted
        assert all(a >= 1 for a in st.accepted)
        if mode == "tsp":
            assert st.rounds <= n_new // 24 + 2
    if kind == "foreign":
        assert np.mean(st.accepted) < 1.0
    target.close()
    draft.close()
