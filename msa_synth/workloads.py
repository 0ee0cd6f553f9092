"""Synthetic workloads shaped like the paper's memory banks (inputs only, no method arithmetic).

The paper evaluates on banks of 16K to 100M tokens built from public QA corpora (Section 4.1,
Section 5.2); those corpora are not used here.  These seeded banks stand in for them: Qwen3-4B
attention geometry (32 query heads / 8 KV heads / head_dim 128), pooling size P = 64, documents of
G = 512 tokens, standard-normal bf16 keys / values / queries.

Each bank is generated in place on the GPU by the counter-based generator (msa_synth.device), so
the 50M-token bank (2 x 95 GiB) never exists on the host; any document can be regenerated on the
host bit-for-bit with msa_synth.doc_slice.  "Planted" documents (host-made, copied over the noise)
give a query a known winner set: one chunk of the document is a * u + noise, u the direction of the
group's mean unit query scaled to unit per-dimension variance.
"""
import numpy as np
import torch

import msa_synth as S
from msa_synth import device as SD

# name: N docs, G, P, Hq, Hkv, d, B, M, k, Lloc, rope base, config number (seed family)
WORKLOADS = {
    "cfg1_tiny_32k": dict(N=64, G=512, P=64, Hq=8, Hkv=2, d=64, B=1, M=1, k=4, Lloc=256, base=1e4, cfg_id=1),
    "cfg2_decode_1m": dict(N=2048, G=512, P=64, Hq=32, Hkv=8, d=128, B=1, M=1, k=16, Lloc=2048, base=1e6, cfg_id=2),
    "cfg3_batch32_4m": dict(N=8192, G=512, P=64, Hq=32, Hkv=8, d=128, B=32, M=1, k=16, Lloc=2048, base=1e6, cfg_id=3),
    "cfg4_prefill_16m": dict(N=32768, G=512, P=64, Hq=32, Hkv=8, d=128, B=1, M=2048, k=8, Lloc=2048, base=1e6, cfg_id=4),
    "cfg5_decode_50m": dict(N=97656, G=512, P=64, Hq=32, Hkv=8, d=128, B=8, M=1, k=32, Lloc=2048, base=1e6, cfg_id=5),
}


class Workload:
    pass


def planted_chunk(q_b, r, g, noise, a):
    """Tokens of one planted chunk for KV group g of one query token.
    q_b [Hq, d] float64 query; noise [P, d] float64 (the chunk's original contents).
    Returns bf16 bits [P, d] of a * u + noise, where u points along the plain sum of the group's query heads (an
    input recipe: a direction that correlates with every head of the group) and has unit per-dim variance."""
    u = q_b[g * r:(g + 1) * r].sum(axis=0)
    u = u / np.linalg.norm(u) * np.sqrt(u.shape[0])
    return S.f64_to_bf16_bits(a * u[None, :] + noise)


def make(name, device="cuda", plant_per_query=0, plant_a=0.12, plant_chunk=3, Lloc=None, alloc_bank=True):
    """Allocate and fill the workload `name` on the device.  Returns a Workload with the shapes,
    device tensors (K, V, q, Kloc, Vloc, q_pos) and, if plant_per_query > 0, the planted documents
    (wl.planted[(b, j)] = doc id; their K slices are in wl.planted_K[doc] as bits [Hkv, G, d]).
    alloc_bank=False leaves out the K / V bank (wl.K = wl.V = None) for callers that fill their own buffers."""
    p = WORKLOADS[name]
    wl = Workload()
    wl.name = name
    for key, v in p.items():
        setattr(wl, key, v)
    if Lloc is not None:                              # decode workloads only: another local-context length
        assert wl.M == 1 and Lloc >= 0
        wl.Lloc = Lloc
    wl.r = wl.Hq // wl.Hkv
    wl.C = wl.G // wl.P
    wl.pos0 = wl.G                                   # local context follows a document's last token
    seeds = {t: S.seed_for(wl.cfg_id, i) for i, t in enumerate(("K", "V", "q", "Kloc", "Vloc"))}
    wl.seeds = seeds
    shape_bank = (wl.N, wl.Hkv, wl.G, wl.d)
    wl.shape_bank = shape_bank
    wl.K = wl.V = None
    if alloc_bank:
        wl.K = torch.empty(shape_bank, dtype=torch.bfloat16, device=device)
        wl.V = torch.empty(shape_bank, dtype=torch.bfloat16, device=device)
        SD.fill_normal_(wl.K, seeds["K"])
        SD.fill_normal_(wl.V, seeds["V"])
    else:
        assert plant_per_query == 0
    wl.q_bits, wl.q_host = S.normal_bf16(seeds["q"], (wl.B, wl.M, wl.Hq, wl.d))
    wl.q = SD.bits_to_torch(wl.q_bits, device)
    if wl.Lloc > 0:
        wl.Kloc = torch.empty((wl.B, wl.Hkv, wl.Lloc, wl.d), dtype=torch.bfloat16, device=device)
        wl.Vloc = torch.empty_like(wl.Kloc)
        SD.fill_normal_(wl.Kloc, seeds["Kloc"])
        SD.fill_normal_(wl.Vloc, seeds["Vloc"])
    else:
        wl.Kloc = wl.Vloc = None
    if wl.M == 1:     # decode: the query is the last local token (position pos0 when there is no local context)
        wl.q_pos_host = np.full((wl.B, wl.M), wl.pos0 + max(wl.Lloc, 1) - 1, dtype=np.int32)
    else:             # prefill: the local context IS the M query tokens, causal (token m sees 0..m)
        assert wl.Lloc == wl.M
        wl.q_pos_host = np.tile(wl.pos0 + np.arange(wl.M, dtype=np.int32), (wl.B, 1))
    wl.q_pos = torch.from_numpy(wl.q_pos_host).to(device)
    wl.planted, wl.planted_K = {}, {}
    if plant_per_query > 0:
        rng = np.random.default_rng(S.seed_for(wl.cfg_id, 99))
        docs = rng.choice(wl.N, size=wl.B * wl.M * plant_per_query, replace=False)
        for qi in range(wl.B * wl.M):
            b, m = divmod(qi, wl.M)
            for j in range(plant_per_query):
                doc = int(docs[qi * plant_per_query + j])
                bits, val = S.doc_slice(seeds["K"], wl.Hkv, wl.G, wl.d, doc)
                bits = bits.copy()
                lo, hi = plant_chunk * wl.P, (plant_chunk + 1) * wl.P
                for g in range(wl.Hkv):
                    bits[g, lo:hi] = planted_chunk(wl.q_host[b, m], wl.r, g, val[g, lo:hi], plant_a)
                wl.planted[(qi, j)] = doc
                wl.planted_K[doc] = bits
                wl.K[doc].copy_(SD.bits_to_torch(bits, device))
    torch.cuda.synchronize()
    return wl


def host_doc(wl, which, doc):
    """(bits, float64) [Hkv, G, d] of document `doc` of bank 'K' or 'V' as it is on the device."""
    if which == "K" and doc in wl.planted_K:
        bits = wl.planted_K[doc]
        return bits, S.bf16_bits_to_f64(bits)
    return S.doc_slice(wl.seeds[which], wl.Hkv, wl.G, wl.d, doc)


def doc_lens(wl, lo_frac=0.125):
    """Seeded document lengths for banks whose documents differ in length (the paper's G is an average,
    Section 5.1): uniform integers in [lo_frac * G, G], int32 [N] on the host."""
    rng = np.random.default_rng(S.seed_for(wl.cfg_id, 55))
    return rng.integers(max(1, int(lo_frac * wl.G)), wl.G + 1, size=wl.N).astype(np.int32)


def algorithmic_bytes(wl):
    """Bytes each stage must move once (the roofline's numerator)."""
    NC = wl.N * wl.C
    tiles = (NC + 15) // 16
    elem = 2
    build = wl.N * wl.Hkv * wl.G * wl.d * elem + wl.Hkv * tiles * 16 * (wl.d * elem + 4)
    n_pass = 1 if wl.B * wl.M <= 32 else (wl.B * wl.M + 31) // 32
    score_once = wl.Hkv * tiles * 16 * (wl.d * elem + 4)
    if wl.M == 1:
        attend = wl.B * wl.M * wl.Hkv * (wl.k * wl.G + wl.Lloc) * wl.d * elem * 2
    else:   # prefill: every token gathers its own k documents; the local context is shared by the tokens (once)
        attend = wl.B * wl.Hkv * (wl.M * wl.k * wl.G + wl.Lloc) * wl.d * elem * 2
    return dict(build=build, score=score_once, score_passes=n_pass, attend=attend)
