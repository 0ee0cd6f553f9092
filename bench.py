#!/usr/bin/env python3
"""Benchmark of the MSA routed-decode hot path on one MI355X.

A "step" is one pass of the online path over one batch of synthetic queries: msa_score_topk
(relevance scores, document max, top-k) followed by msa_sparse_attend (gather with document-wise
RoPE + attention) with every input already resident in HBM.  The routing index is built once before
the timed region by msa_build_routing_keys -- the paper's Stage 1 is offline, once per bank version
(Section 3.4.1) -- and its own time and bandwidth are reported in the "build" object.

Prints ONE JSON line: metric value = routed decode queries/s from the wall clock around the K timed
steps; "roofline" = achieved HBM GB/s (or MFMA TFLOP/s) of the dominant kernel (the routing scan / the
scoring GEMM), its duration taken from HIP events that the library records on the launch stream
immediately around that kernel (the per-call profile events of msa_config_t) in a second run of the same K steps, next
to "entry_point_ms", the whole msa_score_topk call from events inside the timed steps; "attend" the same
for msa_sparse_attend; "cpu_baseline" = the float64 oracle timed on this machine's host cores on a bounded
sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0

# HBM traffic per entry-point call (bytes, read + write, all kernels of the call) from rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE runs of this file, each counter scaled by its reading for a plain copy of known size; the summaries, with
# the kernel signatures and the commit they were measured at, are profiles/pmc_traffic_<workload>.txt.  Only with the
# default flags (un-pooled bank, per-group selection); None where no such run exists.
MEASURED_TRAFFIC = {     # measured at commit f514938
    "cfg5_decode_50m": {"score": 1642.2e6, "attend": 621.7e6},     # algorithmic 1625.0 / 604.0 MB: x1.011 / x1.029
    "cfg3_batch32_4m": {"score": 156.0e6, "attend": 1359.3e6},     # 136.3 / 1342.2 MB: x1.144 (score matrix round trip) / x1.013
    "cfg2_decode_1m": {"score": 34.8e6, "attend": 52.5e6},         # 34.1 / 41.9 MB: x1.021 / x1.252 (split partials)
    # score: fold 25.7 + one-pass GEMM 570.9 (index 536.9 MB read once) + exact scores of the candidates 363.1 MB;
    # attend: gather 34368.1 MB: x1.021
    "cfg4_prefill_16m": {"score": 959.7e6, "attend": 35073.3e6},
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg5_decode_50m",
                    help="cfg5_decode_50m (default), cfg3_batch32_4m, cfg2_decode_1m, cfg1_tiny_32k")
    ap.add_argument("--bank", default="full", choices=("full", "pooled"),
                    help="what msa_sparse_attend reads: the un-pooled K/V bank (default) or the pooled, "
                         "position-encoded bank written by msa_pool_kv (Section 3.4.1, Stage 1)")
    ap.add_argument("--scope", default="group", choices=("group", "all"),
                    help="head mean of Eq. 2 over the r heads of a KV group (default, one selection per KV head) "
                         "or over every head (as printed, one selection for all heads)")
    ap.add_argument("--token-pool", action="store_true",
                    help="max over the query tokens of a batch row (Eq. 2 as printed): one selection per batch row, "
                         "and for many tokens the tiled shared-selection attention kernel")
    ap.add_argument("--tier", default="hbm", choices=("hbm", "host"),
                    help="host: additionally time the tiered bank of Section 3.4.2 (K/V in pinned host memory, the "
                         "selected documents fetched over the host link); reported in \"host_tier\", never in value")
    ap.add_argument("--ragged", action="store_true",
                    help="documents of different lengths: seeded lengths in [G/8, G] passed as cfg.doc_lens (the "
                         "bank keeps its G-row slots); byte counts then follow the lengths")
    ap.add_argument("--local-tokens", type=int, default=None,
                    help="decode workloads: local-context length instead of the workload's (the benchmark definition does not state "
                         "it for configs 3 and 5; 2048 is used, 0 is the other case asked for)")
    ap.add_argument("--cold", action="store_true",
                    help="additionally time the step with nothing left in the 256 MB Infinity Cache from the step "
                         "before: round-robin over copies of the routing index (> 512 MB in all) and over 16 "
                         "different query batches (so other documents are gathered); reported in \"cold\"")
    ap.add_argument("--in-flight", type=int, default=1,
                    help="independent batches in flight, each on its own stream with its own outputs and workspaces "
                         "(a serving loop with several requests); reported in \"in_flight\", never in value")
    ap.add_argument("--graph", action="store_true",
                    help="capture the step once into a HIP graph and time replays (the per-stage times still come "
                         "from an eager pass with HIP events); pays off where the step is launch-bound (config 2)")
    ap.add_argument("--layers", type=int, default=0,
                    help="additionally time the per-token loop over this many routed layers (the paper's model routes in "
                         "18, Section 3.2.1 / 3.4.2): per layer its own routing index and pooled content bank (needs "
                         "--bank pooled; with --tier host the pooled banks live in pinned host memory), score -> (fetch) "
                         "-> attention in every layer, routing of layer l + 1 overlapped with fetch + attention of layer "
                         "l on a second stream; reported in \"layers\", never in value (it runs after the one-layer "
                         "step, whose bank is freed first: one layer's K or V at a time is staged to build the banks)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-docs", type=int, default=1024)
    return ap.parse_args()


def cpu_baseline(wl, cfg, KR, sample_docs):
    """Time the oracle, as it stands, on a bounded sample of the workload (10-30 s of CPU work):
      routing  : Eq. 2, document max and top-k over ALL N documents of the routing index, one KV head at a time, for
                 every query of a decode batch (prefill: 64 evenly spaced query tokens).  The index values are the
                 GPU-built index copied back -- input data for the timing, nothing is compared here;
      attention: one query, all its KV groups, over its k selected documents (regenerated on the host) + the
                 local context;
      pooling  : `sample_docs` documents through the oracle's chunk pooling (offline stage, not in value).
    value = 1 / (routing seconds per query + attention seconds per query)."""
    import numpy as np
    import msa_synth as S
    import paper_2603_23516_amd as msa
    from msa_synth import device as SD
    from msa_synth import workloads as W
    from oracle import msa_oracle as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count()
    bits = SD.torch_to_bits(msa.untile_routing_keys(cfg, KR))          # [Hkv, N*C, d]
    nq = wl.B * wl.M
    q_all = wl.q_host.reshape(nq, 1, wl.Hq, wl.d)
    sel_q = np.arange(nq) if wl.M == 1 else np.linspace(0, nq - 1, 64).astype(np.int64)
    q = q_all[sel_q]
    t_route = 0.0
    idx = None
    for g in range(wl.Hkv):
        KRb = S.bf16_bits_to_f64(bits[g])[None]
        t0 = time.perf_counter()
        oi, _, _ = O.score_topk(q[:, :, g * wl.r:(g + 1) * wl.r], KRb, wl.C, wl.k)
        t_route += time.perf_counter() - t0
        idx = oi if idx is None else np.concatenate([idx, oi], axis=2)
        del KRb
    n_s = min(sample_docs, wl.N)
    Ks = np.stack([W.host_doc(wl, "K", i)[1] for i in range(n_s)])
    t0 = time.perf_counter()
    O.routing_keys(Ks, wl.P)
    t_build = time.perf_counter() - t0
    del Ks
    n_att = min(len(sel_q), 8)                                          # queries whose attention the oracle computes
    t_att = 0.0
    for j in range(n_att):
        sel = idx[j, 0]                                                 # [Hkv, k]: this query's documents
        docs = sorted(set(sel.reshape(-1).tolist()))
        pos = {dd: i for i, dd in enumerate(docs)}
        K_sel = np.stack([W.host_doc(wl, "K", int(i))[1] for i in docs])    # [n, Hkv, G, d]
        V_sel = np.stack([W.host_doc(wl, "V", int(i))[1] for i in docs])
        local = np.array([[[pos[int(dd)] for dd in sel[g]] for g in range(wl.Hkv)]])[None]      # [1, 1, Hkv, k]
        b0, m0 = divmod(int(sel_q[j]), wl.M)
        per_b = wl.Hkv * wl.Lloc * wl.d
        Kl = S.normal_bf16(wl.seeds["Kloc"], (1, wl.Hkv, wl.Lloc, wl.d), start=b0 * per_b)[1] if wl.Lloc else None
        Vl = S.normal_bf16(wl.seeds["Vloc"], (1, wl.Hkv, wl.Lloc, wl.d), start=b0 * per_b)[1] if wl.Lloc else None
        t0 = time.perf_counter()
        O.sparse_attend(q[j:j + 1], K_sel, V_sel, local, Kl, Vl, wl.pos0, wl.q_pos_host[b0:b0 + 1, m0:m0 + 1], wl.base)
        t_att += time.perf_counter() - t0
    t_att /= n_att
    per_query = t_route / len(sel_q) + t_att
    return {
        "value": 1.0 / per_query, "unit": "queries/s", "cores": int(threads), "kind": "oracle",
        "sample": (f"float64 NumPy oracle, {os.cpu_count()} host cpus visible: routing (Eq. 2, document max, top-k) of "
                   f"{len(sel_q)} of {nq} queries over all {wl.N} documents of the routing index {t_route:.2f}s; "
                   f"attention of {n_att} queries (all {wl.Hkv} KV groups, {wl.k} documents each + {wl.Lloc} local tokens) "
                   f"{t_att:.2f}s per query; pooling {n_s} documents {t_build:.2f}s (offline, not in value)"),
    }


def host_tier(msa, wl, cfg, acfg, bank_K, bank_V, pos0, q_pos, KR, inv, idx, val, ws_s, out, lse, stream, steps):
    """The same step with the content bank (the K/V bank, or with --bank pooled the pooled K-bar / V-bar, which is
    what Section 3.4.2 keeps in host DRAM) in pinned host memory: score+top-k, fetch of the selected documents into
    a staging bank (one kernel reading host memory over the host link), attention over the staging bank.  Timed
    serially on one stream, and with two independent batches in flight on two streams (one batch's fetch then
    overlaps the other's scoring)."""
    import torch
    Kh = torch.empty(bank_K.shape, dtype=torch.bfloat16, pin_memory=True)
    Vh = torch.empty(bank_V.shape, dtype=torch.bfloat16, pin_memory=True)
    Kh.copy_(bank_K)
    Vh.copy_(bank_V)
    torch.cuda.synchronize()
    B, M, k = wl.B, wl.M, wl.k

    class Batch:
        pass

    def make_batch(st, idx_b, val_b, ws_b, out_b, lse_b):
        bt = Batch()
        bt.stream, bt.idx, bt.val, bt.ws_s, bt.out, bt.lse = st, idx_b, val_b, ws_b, out_b, lse_b
        bt.Ks, bt.Vs, bt.idx_s, bt.scfg = msa.msa_fetch_selected(acfg, Kh, Vh, idx_b, B, M)
        bt.ws_a = torch.empty(msa.sparse_attend_workspace_bytes(bt.scfg, B, M, k, wl.Lloc), dtype=torch.uint8,
                              device="cuda")
        return bt

    def run(bt, ev=None):
        if ev:
            ev[0].record(bt.stream)
        msa.msa_score_topk(cfg, wl.q, KR, inv, k, bt.idx, bt.val, bt.ws_s, stream=bt.stream)
        if ev:
            ev[1].record(bt.stream)
        msa.msa_fetch_selected(acfg, Kh, Vh, bt.idx, B, M, bt.Ks, bt.Vs, bt.idx_s, stream=bt.stream)
        if ev:
            ev[2].record(bt.stream)
        msa.msa_sparse_attend(bt.scfg, wl.q, bt.Ks, bt.Vs, bt.idx_s, wl.Kloc, wl.Vloc, pos0, q_pos, bt.out, bt.lse,
                              bt.ws_a, stream=bt.stream)
        if ev:
            ev[3].record(bt.stream)

    b0 = make_batch(stream, idx, val, ws_s, out, lse)
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
    for i in range(steps):
        run(b0, ev[i])
    torch.cuda.synchronize()
    fetch_ms = sum(e[1].elapsed_time(e[2]) for e in ev[1:]) / (steps - 1)
    step_ms = sum(e[0].elapsed_time(e[3]) for e in ev[1:]) / (steps - 1)
    # two batches in flight (same queries, their own selections, staging banks and workspaces)
    s1 = torch.cuda.Stream()
    b1 = make_batch(s1, torch.empty_like(idx), torch.empty_like(val), torch.empty_like(ws_s),
                    torch.empty_like(out), torch.empty_like(lse))
    run(b1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        run(b0)
        run(b1)
    torch.cuda.synchronize()
    two_ms = (time.perf_counter() - t0) * 1e3 / (2 * steps)
    n_sel = idx.shape[2]
    heads_per_entry = wl.Hkv if n_sel == 1 else 1
    fetched = idx.numel() * heads_per_entry * acfg.doc_len * wl.d * 2 * 2
    return {"bank": "pooled K-bar / V-bar" if acfg is not cfg else "un-pooled K / V",
            "fetch_ms": fetch_ms, "fetched_bytes": fetched, "fetch_GBps": fetched / (fetch_ms * 1e-3) / 1e9,
            "ms_per_step": step_ms, "queries_per_s": B * M / (step_ms * 1e-3),
            "two_in_flight_ms_per_step": two_ms, "two_in_flight_queries_per_s": B * M / (two_ms * 1e-3),
            "host_bank_bytes": 2 * Kh.numel() * 2,
            "note": "host-link inclusive; ms_per_step is serial on one stream, two_in_flight overlaps one batch's "
                    "fetch with the other's scoring on a second stream"}


def layer_loop(args, msa, wl, cfg):
    """The routed layers of the tiered engine (Section 3.4.2; routing in the latter half of the layers, Section
    3.2.1): n_layers routing indices in HBM, n_layers pooled banks K-bar / V-bar in HBM or pinned host memory, and per
    token batch score -> (fetch) -> attention in every layer."""
    import torch
    import msa_synth as S
    from msa_synth import device as SD
    from paper_2603_23516_amd.layers import LayerStack
    L, B, M, k = args.layers, wl.B, wl.M, wl.k
    t0 = time.perf_counter()
    stack = LayerStack(cfg, L, B, M, k, wl.Lloc, tier=args.tier)
    buf = torch.empty(wl.shape_bank, dtype=torch.bfloat16, device="cuda")      # one layer's K, then its V
    qs, Klocs, Vlocs = [], [], []
    for l in range(L):
        sd = {t: S.seed_for(wl.cfg_id, 100 + 5 * l + i) for i, t in enumerate(("K", "V", "q", "Kloc", "Vloc"))}
        SD.fill_normal_(buf, sd["K"])
        stack.set_layer_keys(l, buf)
        SD.fill_normal_(buf, sd["V"])
        stack.set_layer_values(l, buf)
        qs.append(SD.bits_to_torch(S.normal_bf16(sd["q"], (B, M, wl.Hq, wl.d))[0], "cuda"))
        kl = torch.empty((B, wl.Hkv, wl.Lloc, wl.d), dtype=torch.bfloat16, device="cuda")
        vl = torch.empty_like(kl)
        SD.fill_normal_(kl, sd["Kloc"])
        SD.fill_normal_(vl, sd["Vloc"])
        Klocs.append(kl)
        Vlocs.append(vl)
    torch.cuda.synchronize()
    del buf
    torch.cuda.empty_cache()
    setup_s = time.perf_counter() - t0
    pos0 = k                                                        # Section 3.2.2: local positions start at k
    q_pos = (wl.q_pos - wl.pos0 + pos0).contiguous()
    outs = [torch.empty_like(qs[0]) for _ in range(L)]
    lses = [torch.empty((B, M, wl.Hq), dtype=torch.float32, device="cuda") for _ in range(L)]

    def timed(overlap):
        for _ in range(max(2, args.warmup // 4)):
            stack.step(qs, Klocs, Vlocs, pos0, q_pos, outs, lses, overlap=overlap)
        torch.cuda.synchronize()
        n = max(5, args.steps // 4)
        t0 = time.perf_counter()
        for _ in range(n):
            stack.step(qs, Klocs, Vlocs, pos0, q_pos, outs, lses, overlap=overlap)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / n, n
    serial_ms, n = timed(False)
    ref = [o.clone() for o in outs]
    overlap_ms, _ = timed(True)
    same = all(torch.equal(a.view(torch.int16), b.view(torch.int16)) for a, b in zip(ref, outs))
    index_bytes, bank_bytes = stack.bytes()
    nq = B * M
    return {"n_layers": L, "tier": args.tier, "routing_index_bytes": index_bytes, "pooled_bank_bytes": bank_bytes,
            "pooled_bank_in": "pinned host memory" if args.tier == "host" else "HBM",
            "distinct_pooled_banks": stack.n_banks,
            "memory_tokens_per_layer": wl.N * wl.G, "batch": nq, "timed_steps": n,
            "ms_per_token_batch_one_stream": serial_ms, "ms_per_token_batch_overlapped": overlap_ms,
            "ms_per_layer_overlapped": overlap_ms / L,
            "token_batches_per_s": 1e3 / overlap_ms, "tokens_per_s": nq * 1e3 / overlap_ms,
            "overlap_gain": 1.0 - overlap_ms / serial_ms, "overlapped_equals_serial_bitwise": bool(same),
            "setup_s": setup_s,
            "note": "score+top-k -> (fetch) -> attention over the pooled bank + local context in every routed layer; "
                    "routing of layer l+1 runs on a second stream while layer l is fetched and attended; the other "
                    "layers of the model (local attention only) and its projections are outside this path"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2603_23516_amd as msa
    from msa_synth import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    msa.load_library()
    torch.cuda.set_device(0)
    if args.layers > 0:
        assert args.bank == "pooled" and not args.ragged, "--layers runs over the pooled bank (add --bank pooled)"
    wl = W.make(args.workload, Lloc=args.local_tokens)
    scope = msa.MSA_SCOPE_ALL if args.scope == "all" else msa.MSA_SCOPE_GROUP
    n_sel = 1 if args.scope == "all" else wl.Hkv
    lens = torch.from_numpy(W.doc_lens(wl)).cuda() if args.ragged else None
    cfg = msa.MsaConfig(wl.N, wl.G, wl.P, wl.Hq, wl.Hkv, wl.d, wl.base, select_scope=scope,
                        token_pool=int(args.token_pool), doc_lens=lens)
    ab = W.algorithmic_bytes(wl)
    if args.ragged:
        assert args.bank == "full" and args.tier == "hbm", "--ragged is measured on the full bank in HBM"
        ab["build"] = int(lens.sum().item()) * wl.Hkv * wl.d * 2 + ab["score"]
    stream = torch.cuda.current_stream()

    # ---- offline stage: routing index (timed on its own, outside the metric) -------------------
    KR, inv = msa.alloc_routing_index(cfg)
    msa.msa_build_routing_keys(cfg, wl.K, KR=KR, inv_norm=inv)          # warm-up
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    msa.msa_build_routing_keys(cfg, wl.K, KR=KR, inv_norm=inv)
    e1.record(stream)
    torch.cuda.synchronize()
    build_ms = e0.elapsed_time(e1)

    # ---- offline stage, pooled reading: K-bar / V-bar of Stage 1, attended in place of the full bank
    bank_K, bank_V, acfg, pos0, q_pos = wl.K, wl.V, cfg, wl.pos0, wl.q_pos
    pool_ms = None
    if args.bank == "pooled":
        bank_K, bank_V = msa.msa_pool_kv(cfg, wl.K, wl.V)                # warm-up
        torch.cuda.synchronize()
        e0.record(stream)
        msa.msa_pool_kv(cfg, wl.K, wl.V, Kbar=bank_K, Vbar=bank_V)
        e1.record(stream)
        torch.cuda.synchronize()
        pool_ms = e0.elapsed_time(e1)
        acfg = msa.MsaConfig(wl.N, wl.C, wl.C, wl.Hq, wl.Hkv, wl.d, wl.base, select_scope=scope,
                             token_pool=int(args.token_pool), bank_keys_rotated=1)
        pos0 = wl.k                                                      # Section 3.2.2: local positions start at k
        q_pos = (wl.q_pos - wl.pos0 + pos0).contiguous()
        ab["attend"] = wl.B * wl.Hkv * (wl.M * wl.k * wl.C + wl.Lloc) * wl.d * 2 * 2   # local context read once
        ab["pool"] = 2 * wl.N * wl.Hkv * (wl.G + wl.C) * wl.d * 2

    # ---- online path: everything preallocated, nothing allocated inside the timed region --------
    B, M, k = wl.B, wl.M, wl.k
    m_sel = 1 if args.token_pool else M
    idx = torch.empty((B, m_sel, n_sel, k), dtype=torch.int32, device="cuda")
    val = torch.empty((B, m_sel, n_sel, k), dtype=torch.float32, device="cuda")
    out = torch.empty_like(wl.q)
    lse = torch.empty((B, M, wl.Hq), dtype=torch.float32, device="cuda")
    ws_s = torch.empty(msa.score_topk_workspace_bytes(cfg, B, M, k), dtype=torch.uint8, device="cuda")
    ws_a = torch.empty(msa.sparse_attend_workspace_bytes(acfg, B, M, k, wl.Lloc), dtype=torch.uint8, device="cuda")

    cfg_prof, acfg_prof = cfg.replace(), acfg.replace()    # copies that carry the per-call profile events

    def step(ev=None, kev=None):
        # ev: [before score, between, after attend] around the entry points; kev: (start, stop) pairs that the
        # library records immediately around the dominant kernel of each entry point
        if ev:
            ev[0].record(stream)
        c_s, c_a = cfg, acfg
        if kev:
            c_s, c_a = cfg_prof.set_profile_events(kev[0], kev[1]), acfg_prof.set_profile_events(kev[2], kev[3])
        msa.msa_score_topk(c_s, wl.q, KR, inv, k, idx, val, ws_s, stream=stream)
        if ev:
            ev[1].record(stream)
        msa.msa_sparse_attend(c_a, wl.q, bank_K, bank_V, idx, wl.Kloc, wl.Vloc, pos0, q_pos, out, lse,
                              ws_a, stream=stream)
        if ev:
            ev[2].record(stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.ragged:     # rows the attention really reads: the lengths of the documents selected (same every step)
        sel_rows = int(lens[idx.long().reshape(-1)].sum().item()) * (wl.Hkv if n_sel == 1 else 1)
        if args.token_pool:
            sel_rows *= M
        local = ab["attend"] - B * M * wl.Hkv * k * wl.G * wl.d * 2 * 2
        ab["attend"] = sel_rows * wl.d * 2 * 2 + local
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(events[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    # The same K steps once more with events recorded by the library around the dominant kernel of each entry
    # point (four more event records per step cost ~10 us of stream time, so they stay out of the steps that
    # `value` is taken from).
    kevents = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    for e in kevents:                     # torch creates the underlying event at its first record
        for x in e:
            x.record(stream)
    torch.cuda.synchronize()
    for i in range(args.steps):
        step(None, kevents[i])
    torch.cuda.synchronize()
    eager_ms = wall * 1e3 / args.steps
    if args.graph:      # same work, launched as one graph: the library only enqueues kernels on the given stream
        cap = torch.cuda.Stream()
        cap.wait_stream(stream)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=cap):
            msa.msa_score_topk(cfg, wl.q, KR, inv, k, idx, val, ws_s, stream=cap)
            msa.msa_sparse_attend(acfg, wl.q, bank_K, bank_V, idx, wl.Kloc, wl.Vloc, pos0, q_pos, out, lse,
                                  ws_a, stream=cap)
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0

    score_all = sorted(e[0].elapsed_time(e[1]) for e in events)
    attend_all = sorted(e[1].elapsed_time(e[2]) for e in events)
    score_call_ms = sum(score_all) / args.steps      # whole entry points (small kernels around the dominant one)
    attend_call_ms = sum(attend_all) / args.steps
    score_all = sorted(e[0].elapsed_time(e[1]) for e in kevents)    # the dominant kernels alone
    attend_all = sorted(e[2].elapsed_time(e[3]) for e in kevents)
    score_ms = sum(score_all) / args.steps
    attend_ms = sum(attend_all) / args.steps

    cold = None
    if args.cold:
        import msa_synth as S
        from msa_synth import device as SD
        index_bytes = KR.numel() * 2 + inv.numel() * 4
        n_idx = max(1, -(-(512 << 20) // index_bytes))
        idx_copies = [(KR, inv)] + [(KR.clone(), inv.clone()) for _ in range(n_idx - 1)]
        qs = [wl.q] + [SD.bits_to_torch(S.normal_bf16(wl.seeds["q"] + 7919 * (j + 1), tuple(wl.q.shape))[0], "cuda")
                       for j in range(15)]
        torch.cuda.synchronize()
        n_cold = min(args.steps, 64)
        evc = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(n_cold)]
        for i in range(n_cold + 4):
            KRi, invi = idx_copies[i % n_idx]
            qi = qs[i % 16]
            ev = evc[i - 4] if i >= 4 else None
            if ev:
                ev[0].record(stream)
            msa.msa_score_topk(cfg, qi, KRi, invi, k, idx, val, ws_s, stream=stream)
            if ev:
                ev[1].record(stream)
            msa.msa_sparse_attend(acfg, qi, bank_K, bank_V, idx, wl.Kloc, wl.Vloc, pos0, q_pos, out, lse,
                                  ws_a, stream=stream)
            if ev:
                ev[2].record(stream)
        torch.cuda.synchronize()
        cs = sorted(e[0].elapsed_time(e[1]) for e in evc)
        ca = sorted(e[1].elapsed_time(e[2]) for e in evc)
        cold = {"index_copies": n_idx, "query_batches": 16, "steps": n_cold,
                "score_ms": {"avg": sum(cs) / n_cold, "median": cs[n_cold // 2], "min": cs[0]},
                "attend_ms": {"avg": sum(ca) / n_cold, "median": ca[n_cold // 2], "min": ca[0]},
                "score_GBps": ab["score"] / (sum(cs) / n_cold * 1e-3) / 1e9,
                "attend_GBps": ab["attend"] / (sum(ca) / n_cold * 1e-3) / 1e9}
        del idx_copies, qs
    ms_per_step = wall * 1e3 / args.steps
    nq = B * M
    qps = nq / (ms_per_step * 1e-3)
    score_gbs = ab["score"] / (score_ms * 1e-3) / 1e9
    attend_gbs = ab["attend"] / (attend_ms * 1e-3) / 1e9
    build_gbs = ab["build"] / (build_ms * 1e-3) / 1e9

    # the MFMA GEMM path (many query tokens).  Algorithmic flops: the folded form of Eq. 2, one routing query per (token,
    # KV group): 2 * tokens * Hkv * keys * d.  Issued: twice that where the query travels as a bf16 (hi, lo) pair (head
    # mean over every head; d = 64; 4 or 16 chunks per document), once where the product runs on the hi parts alone and
    # the few candidates inside the error band are scored again exactly (per-group selections, cosine, d = 128, C = 8)
    flops = flops_issued = None
    one_pass = False
    if nq >= 64 and k <= 16 and wl.C in (4, 8, 16):          # both selection scopes do the same matrix work
        tiles = (wl.N * wl.C + 15) // 16
        one_pass = args.scope == "group" and wl.d == 128 and wl.C == 8
        flops = 2.0 * nq * wl.Hkv * wl.N * wl.C * wl.d
        flops_issued = 2.0 * nq * wl.Hkv * tiles * 16 * (1 if one_pass else 2) * wl.d
    # shared selection and many tokens: attention is a dense contraction on the matrix cores.  Algorithmic flops: two
    # products (QK, PV) of 2 flops per multiply-add over the keys each token sees; issued: twice that (bf16 (hi, lo) pairs
    # of Q and P)
    att_flops = att_flops_issued = None
    if args.token_pool and M >= 8 and args.bank == "full":
        keys = M * k * wl.G + M * (M + 1) // 2           # memory rows + causal local rows, summed over the tokens
        att_flops = 4.0 * B * wl.Hq * keys * wl.d
        att_flops_issued = 2 * att_flops
    default_flags = (args.bank == "full" and args.scope == "group" and not args.token_pool and not args.ragged and
                     args.local_tokens is None)
    TRAFFIC = MEASURED_TRAFFIC.get(wl.name, {}) if default_flags else {}
    res = {
        "metric": "routed decode queries/sec (score+top-k then sparse attend, one MSA layer)",
        "value": qps, "unit": "queries/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "launch": "hip_graph" if args.graph else "eager", "ragged": bool(args.ragged), "bank": args.bank, "select_scope": args.scope, "token_pool": int(args.token_pool),
                   "memory_tokens": wl.N * wl.G, "docs": wl.N, "doc_len": wl.G,
                   "chunk": wl.P, "q_heads": wl.Hq, "kv_heads": wl.Hkv, "head_dim": wl.d, "batch": B,
                   "query_tokens": M, "top_k": k, "local_tokens": wl.Lloc, "rope_base": wl.base},
        "roofline": ({"bound": "hbm", "kernel": "score_scan_kernel (inside msa_score_topk = prep + scan + merge)",
                      "achieved": score_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                      "frac": score_gbs / HBM_PEAK_GBS, "traffic": TRAFFIC.get("score"),
                      "algorithmic_bytes_per_launch": ab["score"], "avg_ms": score_ms,
                      "median_ms": score_all[args.steps // 2], "min_ms": score_all[0],
                      "entry_point_ms": score_call_ms,
                      "entry_point_frac": ab["score"] / (score_call_ms * 1e-3) / 1e9 / HBM_PEAK_GBS} if flops is None else
                     {"bound": "mfma", "kernel": ("score_gemm_all_kernel" if args.scope == "all" else "score_gemm_kernel") +
                      (" on the hi parts of the queries (inside msa_score_topk = fold + one-pass GEMM + candidates and exact "
                       "scores + gated two-pass GEMM and merge)" if one_pass else " (inside msa_score_topk = fold + GEMM + merge)"),
                      "achieved": flops / (score_ms * 1e-3) / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS,
                      "unit": "TFLOP/s", "frac": flops / (score_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                      "traffic": TRAFFIC.get("score"),
                      "algorithmic_flops_per_launch": flops, "flops_issued_per_launch": flops_issued,
                      "frac_issued": flops_issued / (score_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                      "avg_ms": score_ms, "median_ms": score_all[args.steps // 2], "min_ms": score_all[0],
                      "entry_point_ms": score_call_ms,
                      "entry_point_frac": flops / (score_call_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS}),
        "attend": ({"bound": "hbm", "kernel": "attend_partial_kernel (inside msa_sparse_attend)",
                    "achieved": attend_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": attend_gbs / HBM_PEAK_GBS, "traffic": TRAFFIC.get("attend"),
                    "algorithmic_bytes_per_launch": ab["attend"],
                    "avg_ms": attend_ms, "median_ms": attend_all[args.steps // 2], "min_ms": attend_all[0],
                    "entry_point_ms": attend_call_ms,
                    "entry_point_frac": ab["attend"] / (attend_call_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
                   if att_flops is None else
                   {"bound": "mfma", "kernel": "attend_prefill_kernel (shared selection)",
                    "achieved": att_flops / (attend_ms * 1e-3) / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": att_flops / (attend_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                    "algorithmic_flops_per_launch": att_flops, "flops_issued_per_launch": att_flops_issued,
                    "frac_issued": att_flops_issued / (attend_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                    "avg_ms": attend_ms, "median_ms": attend_all[args.steps // 2], "min_ms": attend_all[0],
                    "entry_point_ms": attend_call_ms,
                    "entry_point_frac": att_flops / (attend_call_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS}),
        "build": {"bound": "hbm", "achieved": build_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                  "frac": build_gbs / HBM_PEAK_GBS, "algorithmic_bytes_per_launch": ab["build"],
                  "ms": build_ms, "note": "offline Stage 1, once per bank version; outside the timed steps"},
    }
    if args.in_flight > 1:
        nf = args.in_flight
        sts = [torch.cuda.Stream() for _ in range(nf)]
        bufs = []
        for j in range(nf):
            bufs.append((torch.empty_like(idx), torch.empty_like(val), torch.empty_like(out), torch.empty_like(lse),
                         torch.empty_like(ws_s), torch.empty_like(ws_a)))
        torch.cuda.synchronize()

        def run_all(n):
            for i in range(n):
                j = i % nf
                bi, bv, bo, bl, bws, bwa = bufs[j]
                msa.msa_score_topk(cfg, wl.q, KR, inv, k, bi, bv, bws, stream=sts[j])
                msa.msa_sparse_attend(acfg, wl.q, bank_K, bank_V, bi, wl.Kloc, wl.Vloc, pos0, q_pos, bo, bl, bwa,
                                      stream=sts[j])
        run_all(args.warmup)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run_all(args.steps)
        torch.cuda.synchronize()
        w2 = time.perf_counter() - t0
        res["in_flight"] = {"batches": nf, "ms_per_step": w2 * 1e3 / args.steps,
                            "queries_per_s": nq / (w2 / args.steps),
                            "note": "steps of different batches overlap on separate streams; a single batch still "
                                    "takes ms_per_step above"}
    if cold is not None:
        res["cold"] = cold
    if args.graph:
        res["eager_ms_per_step"] = eager_ms
    if args.tier == "host":
        res["host_tier"] = host_tier(msa, wl, cfg, acfg, bank_K, bank_V, pos0, q_pos, KR, inv, idx, val, ws_s, out,
                                     lse, stream, min(args.steps, 20))
    if pool_ms is not None:
        res["pool"] = {"bound": "hbm", "achieved": ab["pool"] / (pool_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                       "unit": "GB/s", "frac": ab["pool"] / (pool_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                       "algorithmic_bytes_per_launch": ab["pool"], "ms": pool_ms,
                       "note": "msa_pool_kv, offline Stage 1; outside the timed steps"}
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(wl, cfg, KR, args.cpu_sample_docs)
    if args.layers > 0:
        # free the one-layer bank (2 x 95 GiB at config 5) before the per-layer banks are built
        bank_K = bank_V = KR = inv = ws_s = ws_a = idx = val = out = lse = None
        wl.K = wl.V = None
        torch.cuda.empty_cache()
        res["layers"] = layer_loop(args, msa, wl, cfg)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
