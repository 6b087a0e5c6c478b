"""Device-memory plumbing around the C ABI: PyTorch tensors hold weights, KV cache, workspace
and logits; every computation is a call into libspecasr.so through ``binding``.
"""
import numpy as np
import torch

from . import binding as B


def _to_device(a, device):
    """numpy storage array (float32, or uint16 bf16 bit patterns) -> device tensor, bits unchanged."""
    if a.dtype == np.uint16:
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(device)


def _to_host(t):
    """device tensor -> numpy in storage form (bf16 as uint16 bit patterns)."""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def upload_weights(w, device="cuda:0"):
    out = {k: _to_device(v, device) for k, v in w.items() if k != "layers"}
    out["layers"] = [{k: _to_device(v, device) for k, v in lw.items()} for lw in w["layers"]]
    return out


class Verifier:
    """One model + one KV cache + one workspace on one GPU."""

    def __init__(self, cfg, weights, dtype, max_nodes, capacity, max_batch=1, flags=0,
                 device="cuda:0", weights_on_device=False):
        self.cfg, self.max_nodes, self.batch, self.capacity = dict(cfg), max_nodes, max_batch, capacity
        self.device = torch.device(device)
        self.dtype = B.SPECASR_BF16 if dtype in ("bf16", B.SPECASR_BF16) else B.SPECASR_F32
        self.tdtype = torch.bfloat16 if self.dtype == B.SPECASR_BF16 else torch.float32
        torch.cuda.set_device(self.device)
        self.w = weights if weights_on_device else upload_weights(weights, self.device)
        self._wstruct, self._keep = B.make_weights(self.w)
        self._config = B.make_config(cfg, self.dtype, max_nodes, max_batch, flags)
        rc, self.ctx = B.specasr_create(self._config, self._wstruct)
        if rc != B.SPECASR_OK:
            raise B.SpecasrError(rc)
        self.ws_bytes = B.specasr_workspace_bytes(self.ctx, max_batch)
        self.ws = torch.empty(self.ws_bytes + 256, dtype=torch.uint8, device=self.device)
        self.ws_ptr = (self.ws.data_ptr() + 255) // 256 * 256
        shape = (max_batch, cfg["n_layers"], cfg["n_kv_heads"], capacity, cfg["head_dim"])
        self.k = torch.zeros(shape, dtype=self.tdtype, device=self.device)
        self.v = torch.zeros(shape, dtype=self.tdtype, device=self.device)
        self.kv_len = np.zeros(max_batch, np.int32)
        self._kv = B.make_kv(self.k, self.v, capacity, self.kv_len)

    def close(self):
        if self.ctx is not None:
            B.specasr_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- cache I/O ------------------------------------------------------------
    def set_cache(self, k_np, v_np, kv_len):
        """k_np/v_np: storage arrays [batch][layers][kv heads][<=capacity][head_dim]."""
        n = k_np.shape[3]
        self.k[:, :, :, :n].copy_(_to_device(k_np, self.device))
        self.v[:, :, :, :n].copy_(_to_device(v_np, self.device))
        self.kv_len[:] = np.asarray(kv_len, np.int32)

    def get_cache(self):
        torch.cuda.synchronize()
        return _to_host(self.k), _to_host(self.v)

    def get_rows(self, lo, hi):
        """Cache slots [lo, hi) of every sequence/layer/head as host arrays (K, V)."""
        torch.cuda.synchronize()
        return (_to_host(self.k[:, :, :, lo:hi].contiguous()), _to_host(self.v[:, :, :, lo:hi].contiguous()))

    # -- marshalling helpers ----------------------------------------------------
    def _tree(self, tokens, parents, embeds=None, use_embed=None):
        """tokens/parents: list (one per sequence) of int sequences."""
        nb = len(tokens)
        tok = np.zeros((nb, self.max_nodes), np.int32)
        par = np.full((nb, self.max_nodes), -1, np.int32)
        nn = np.zeros(nb, np.int32)
        for b in range(nb):
            n = len(tokens[b])
            nn[b] = n
            tok[b, :min(n, self.max_nodes)] = np.asarray(tokens[b], np.int32)[:self.max_nodes]
            par[b, :min(n, self.max_nodes)] = np.asarray(parents[b], np.int32)[:self.max_nodes]
        ue = None
        if use_embed is not None:
            ue = np.zeros((nb, self.max_nodes), np.uint8)
            for b in range(nb):
                ue[b, :len(use_embed[b])] = use_embed[b]
        keep = (tok, par, nn, ue, embeds)
        return B.make_tree(tok, par, nn, embeds, ue), keep

    def verify_tree(self, tokens, parents, want_logits=False, stream=None):
        """One full round.  Returns dict(status, argmax, path, accept_len, next_token, logits)."""
        nb = self.batch
        tree, keep = self._tree(tokens, parents)
        argmax = np.full((nb, self.max_nodes), -1, np.int32)
        path = np.full((nb, self.max_nodes), -1, np.int32)
        alen = np.zeros(nb, np.int32)
        nxt = np.zeros(nb, np.int32)
        logits = None
        if want_logits:
            logits = torch.zeros((nb, self.max_nodes, self.cfg["vocab"]), dtype=torch.float32,
                                 device=self.device)
        out = B.make_out(argmax, path, alen, nxt, logits)
        rc = B.specasr_verify_tree(self.ctx, self._kv, tree, out, self.ws_ptr, self.ws_bytes, stream)
        return dict(status=rc, argmax=argmax, path=path, accept_len=alen, next_token=nxt,
                    logits=logits)

    def tree_forward(self, tokens, parents, want_logits=True, embeds=None, use_embed=None,
                     stream=None):
        nb = self.batch
        tree, keep = self._tree(tokens, parents, embeds, use_embed)
        argmax = torch.full((nb, self.max_nodes), -1, dtype=torch.int32, device=self.device)
        logits = None
        if want_logits:
            logits = torch.zeros((nb, self.max_nodes, self.cfg["vocab"]), dtype=torch.float32,
                                 device=self.device)
        rc = B.specasr_tree_forward(self.ctx, self._kv, tree, argmax, logits, self.ws_ptr,
                                    self.ws_bytes, stream)
        torch.cuda.synchronize()
        return dict(status=rc, argmax=argmax, logits=logits)

    def tree_forward_top2(self, tokens, parents, want_logits=False, embeds=None, use_embed=None,
                          stream=None):
        """Draft-side forward: per node the two most probable token ids and the probability of
        the first.  Returns dict(status, top2 [batch][max_nodes][2], prob, logits)."""
        nb = self.batch
        tree, keep = self._tree(tokens, parents, embeds, use_embed)
        top2 = torch.full((nb, self.max_nodes, 2), -7, dtype=torch.int32, device=self.device)
        prob = torch.full((nb, self.max_nodes), -1.0, dtype=torch.float32, device=self.device)
        logits = None
        if want_logits:
            logits = torch.zeros((nb, self.max_nodes, self.cfg["vocab"]), dtype=torch.float32,
                                 device=self.device)
        rc = B.specasr_tree_forward_top2(self.ctx, self._kv, tree, top2, prob, logits, self.ws_ptr,
                                         self.ws_bytes, stream)
        torch.cuda.synchronize()
        return dict(status=rc, top2=top2, prob=prob, logits=logits)

    def prefill(self, tokens, embeds=None, use_embed=None, want_next=True, stream=None):
        """Append positions to every sequence: tokens = list (one per sequence) of int sequences,
        embeds = optional device tensor [batch][max_pos][d_model], use_embed = list of flag lists.
        Returns dict(status, next_token)."""
        nb = self.batch
        n_pos = np.asarray([len(t) for t in tokens], np.int32)
        max_pos = int(embeds.shape[1]) if embeds is not None else max(1, int(n_pos.max()))
        tok = np.zeros((nb, max_pos), np.int32)
        ue = None
        if use_embed is not None:
            ue = np.zeros((nb, max_pos), np.uint8)
        for b in range(nb):
            tok[b, :n_pos[b]] = np.asarray(tokens[b], np.int32)
            if ue is not None:
                ue[b, :len(use_embed[b])] = use_embed[b]
        nxt = np.full(nb, -7, np.int32) if want_next else None
        rc = B.specasr_prefill(self.ctx, self._kv, tok, embeds, ue, n_pos, max_pos, nxt, self.ws_ptr,
                               self.ws_bytes, stream)
        torch.cuda.synchronize()
        return dict(status=rc, next_token=nxt)

    def accept(self, tokens, parents, argmax_dev=None, logits_dev=None, stream=None):
        nb = len(tokens)
        tree, keep = self._tree(tokens, parents)
        path = torch.full((nb, self.max_nodes), -7, dtype=torch.int32, device=self.device)
        alen = torch.zeros(nb, dtype=torch.int32, device=self.device)
        nxt = torch.zeros(nb, dtype=torch.int32, device=self.device)
        if logits_dev is not None:
            argmax_dev = torch.full((nb, self.max_nodes), -1, dtype=torch.int32, device=self.device)
            rc = B.specasr_accept_from_logits(self.ctx, tree, nb, logits_dev, argmax_dev, path,
                                              alen, nxt, self.ws_ptr, self.ws_bytes, stream)
        else:
            rc = B.specasr_accept(self.ctx, tree, nb, argmax_dev, path, alen, nxt, self.ws_ptr,
                                  self.ws_bytes, stream)
        torch.cuda.synchronize()
        return dict(status=rc, argmax=argmax_dev, path=path.cpu().numpy(),
                    accept_len=alen.cpu().numpy(), next_token=nxt.cpu().numpy())

    def commit(self, n_nodes, paths, stream=None):
        nb = self.batch
        p = np.full((nb, self.max_nodes), -1, np.int32)
        alen = np.zeros(nb, np.int32)
        for b in range(nb):
            alen[b] = len(paths[b])
            p[b, :len(paths[b])] = paths[b]
        nn = np.asarray(n_nodes, np.int32)
        rc = B.specasr_commit(self.ctx, self._kv, nn, p, alen, self.ws_ptr, self.ws_bytes, stream)
        torch.cuda.synchronize()
        return rc
