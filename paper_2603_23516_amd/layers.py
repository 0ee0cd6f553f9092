"""The routed layers of a Memory Sparse Attention model as one per-token loop over the C-ABI entry points.

Section 3.2.1 applies routing in the latter half of the model's layers; Section 3.4.2 keeps, for every routed layer,
the routing keys in device memory and the pooled content bank (K-bar, V-bar) either in device memory or, tiered, in
host DRAM from which the selected documents are fetched.  A LayerStack holds those per-layer banks and runs, for one
batch of query tokens, score + top-k -> (fetch) -> attention in every layer.  Scoring runs on one stream and fetch +
attention on another: layer l + 1 is routed while layer l's winners are still being fetched and attended (the
layers' queries are inputs here; in a model they come out of the layer below, which orders the streams the same
way through events).

Orchestration only: every step of the path runs in the library's kernels.
"""
import torch

from . import (MsaConfig, msa_build_routing_keys, msa_fetch_selected, msa_pool_kv, msa_score_topk,
               msa_sparse_attend, score_topk_workspace_bytes, sparse_attend_workspace_bytes, alloc_routing_index,
               fetch_slots)


class LayerStack:
    def __init__(self, cfg, n_layers, B, M, k, Lloc, tier="hbm", device="cuda"):
        """cfg: the config of the un-pooled bank (N documents of G tokens, chunk P).  tier: "hbm" keeps every
        layer's pooled bank in device memory, "host" in pinned host memory (fetched per step)."""
        assert tier in ("hbm", "host")
        self.cfg, self.L, self.B, self.M, self.k, self.Lloc, self.tier, self.dev = cfg, n_layers, B, M, k, Lloc, tier, device
        C = cfg.chunks_per_doc
        # the pooled bank is a bank of N documents of C rows whose keys carry their positions
        self.pcfg = MsaConfig(cfg.n_docs, C, C, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.rope_base,
                              sim=cfg.sim, select_scope=cfg.select_scope, token_pool=cfg.token_pool,
                              bank_keys_rotated=1)
        self.KR, self.inv, self.Kbar, self.Vbar = [], [], [], []
        shape = (cfg.n_docs, cfg.n_kv_heads, C, cfg.head_dim)
        for _ in range(n_layers):
            kr, inv = alloc_routing_index(cfg, device)
            self.KR.append(kr)
            self.inv.append(inv)
            if tier == "hbm":
                self.Kbar.append(torch.empty(shape, dtype=torch.bfloat16, device=device))
                self.Vbar.append(torch.empty(shape, dtype=torch.bfloat16, device=device))
        if tier == "host":
            # As many distinct pooled banks as the machine lets this process pin (at least one); when that is
            # fewer than n_layers, layer l reads bank l % n_banks -- the same bytes travel per layer, which is what
            # a timing needs; a model needs every layer's own bank.
            for l in range(n_layers):
                try:
                    kb = torch.empty(shape, dtype=torch.bfloat16, pin_memory=True)
                    vb = torch.empty(shape, dtype=torch.bfloat16, pin_memory=True)
                except RuntimeError:
                    if l == 0:
                        raise
                    break
                self.Kbar.append(kb)
                self.Vbar.append(vb)
        self.n_banks = len(self.Kbar)
        m_sel = 1 if cfg.token_pool else M
        n_sel = 1 if cfg.select_scope == 1 else cfg.n_kv_heads
        self.idx = [torch.empty((B, m_sel, n_sel, k), dtype=torch.int32, device=device) for _ in range(n_layers)]
        self.val = [torch.empty((B, m_sel, n_sel, k), dtype=torch.float32, device=device) for _ in range(n_layers)]
        self.ws_s = torch.empty(score_topk_workspace_bytes(cfg, B, M, k), dtype=torch.uint8, device=device)
        self.acfg = self.pcfg
        if tier == "host":
            n_slots = fetch_slots(self.pcfg, B, M, k)
            self.K_stage = torch.empty((n_slots, cfg.n_kv_heads, C, cfg.head_dim), dtype=torch.bfloat16, device=device)
            self.V_stage = torch.empty_like(self.K_stage)
            self.idx_stage = torch.empty_like(self.idx[0])
            self.acfg = self.pcfg.replace(n_docs=n_slots)
        self.ws_a = torch.empty(sparse_attend_workspace_bytes(self.acfg, B, M, k, Lloc), dtype=torch.uint8, device=device)
        self.s_route, self.s_attend = torch.cuda.Stream(device), torch.cuda.Stream(device)
        self.ev_scored = [torch.cuda.Event() for _ in range(n_layers)]

    # ---- offline stage (Section 3.4.1, Stage 1), one layer at a time; K and V may be the same buffer refilled ----
    def set_layer_keys(self, layer, K):
        """Routing index and pooled, position-encoded key bank of one layer from its keys K [N][Hkv][G][d]."""
        msa_build_routing_keys(self.cfg, K, KR=self.KR[layer], inv_norm=self.inv[layer])
        if layer >= self.n_banks:
            return
        if self.tier == "hbm":
            msa_pool_kv(self.cfg, K, None, Kbar=self.Kbar[layer])
        else:
            tmp, _ = msa_pool_kv(self.cfg, K, None)
            self.Kbar[layer].copy_(tmp)

    def set_layer_values(self, layer, V):
        if layer >= self.n_banks:
            return
        if self.tier == "hbm":
            msa_pool_kv(self.cfg, None, V, Vbar=self.Vbar[layer])
        else:
            _, tmp = msa_pool_kv(self.cfg, None, V)
            self.Vbar[layer].copy_(tmp)

    def bytes(self):
        index = sum(t.numel() * 2 for t in self.KR) + sum(t.numel() * 4 for t in self.inv)
        bank = sum(t.numel() * 2 for t in self.Kbar) + sum(t.numel() * 2 for t in self.Vbar)
        return index, bank

    # ---- online: one batch of query tokens through every routed layer --------------------------------------
    def step(self, qs, Klocs, Vlocs, pos0, q_pos, outs, lses, overlap=True):
        """qs[l] bf16 [B][M][Hq][d]: the routing/attention query of layer l; Klocs[l], Vlocs[l] its local cache;
        outs[l], lses[l] receive its attention output.  overlap=False runs everything on one stream."""
        s_r = self.s_route
        s_a = self.s_attend if overlap else self.s_route
        cur = torch.cuda.current_stream(self.dev)
        s_r.wait_stream(cur)
        if overlap:
            s_a.wait_stream(cur)
        for l in range(self.L):
            msa_score_topk(self.cfg, qs[l], self.KR[l], self.inv[l], self.k, self.idx[l], self.val[l], self.ws_s,
                           stream=s_r)
            if overlap:
                self.ev_scored[l].record(s_r)
                s_a.wait_event(self.ev_scored[l])
            if self.tier == "host":
                msa_fetch_selected(self.pcfg, self.Kbar[l % self.n_banks], self.Vbar[l % self.n_banks], self.idx[l], self.B, self.M, self.K_stage,
                                   self.V_stage, self.idx_stage, stream=s_a)
                msa_sparse_attend(self.acfg, qs[l], self.K_stage, self.V_stage, self.idx_stage, Klocs[l], Vlocs[l],
                                  pos0, q_pos, outs[l], lses[l], self.ws_a, stream=s_a)
            else:
                msa_sparse_attend(self.acfg, qs[l], self.Kbar[l], self.Vbar[l], self.idx[l], Klocs[l], Vlocs[l],
                                  pos0, q_pos, outs[l], lses[l], self.ws_a, stream=s_a)
        cur.wait_stream(s_r)
        if overlap:
            cur.wait_stream(s_a)
