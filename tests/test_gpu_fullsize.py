"""Parity at the full sizes of the benchmark configurations, in the launch configuration bench.py times (same workload
builder, same B / M / k, same entry points), COMPLETE for the routing stage:

  index   : the oracle builds its own routing index of the WHOLE bank on the host (every document regenerated from
            the seed in worker processes, pooled by the oracle); the GPU-built index is copied back and compared
            element by element (a difference is allowed only one bf16 step away, next to a rounding tie)
  score   : msa_score_topk on the ORACLE's index (re-tiled, uploaded) and on the GPU's own index, against the
            oracle's chunk_scores -> doc_scores -> topk_docs over ALL documents for ALL queries (configs 2, 3, 5),
            one KV head at a time; config 4: all documents for a stated sample of 64 of the 2048 query tokens per
            token, and all 2048 tokens with token pooling.  Indices must be bit-exact wherever the oracle's order
            is clear (tie band 1e-3 relative, see fullsize_oracle.compare_selection).
  attend  : the oracle's attention for EVERY (query, KV group) of configs 2, 3, 5 (config 4: the sampled tokens)
            over the selected documents regenerated on the host and the local context.
  pooled  : the pooled, position-encoded bank on sampled documents, and attention over it (decode configs).
"""
import time

import numpy as np
import pytest
import torch

import msa_synth as S
import paper_2603_23516_amd as msa
from fullsize_oracle import OraclePool, compare_selection
from msa_synth import device as SD
from msa_synth import workloads as W
from oracle import msa_oracle as O

pytestmark = pytest.mark.gpu

SCORE_ATOL = 2e-5          # fp32 accumulation + bf16 (hi, lo) query split, scores of magnitude <= 1
CHAINED_ATOL = 2e-4        # the GPU's own index may hold a key one bf16 step off next to a rounding tie


def say(*a):
    print(*a, flush=True)


@pytest.fixture(scope="module")
def pool():
    p = OraclePool()
    yield p
    p.close()


def gpu_index_bits(cfg, KR, inv):
    bits = SD.torch_to_bits(msa.untile_routing_keys(cfg, KR))                  # [Hkv, NC, d]
    NC = cfg.n_docs * cfg.chunks_per_doc
    return bits, inv[:, :NC].cpu().numpy().astype(np.float64)


def check_full_index(wl, gbits, ginv, obits, oinv, lens=None):
    """Every key of the GPU-built index against the oracle's."""
    C = wl.C
    valid = np.ones(wl.N * C, dtype=bool) if lens is None else O.chunk_valid(lens, wl.G, wl.P)
    if lens is not None:
        # slots of chunks a document does not have repeat its chunk 0 (key and norm), bit for bit
        first = np.repeat(np.arange(wl.N) * C, C)
        assert np.array_equal(gbits[:, ~valid], gbits[:, first[~valid]])
        assert np.array_equal(ginv[:, ~valid], ginv[:, first[~valid]])
        assert np.all(oinv[:, ~valid] == -1.0)
    diff = (gbits != obits) & valid[None, :, None]
    n_diff = int(diff.sum())
    frac = n_diff / diff.size
    assert frac < 2e-4, frac
    if n_diff:
        g, c, e = np.nonzero(diff)
        got = S.bf16_bits_to_f64(gbits[g, c, e])
        want = S.bf16_bits_to_f64(obits[g, c, e])
        assert np.all(np.abs(got - want) <= np.abs(want) * 2.0 ** -7 + 1e-30), "more than one bf16 step off"
        # ... and only next to a rounding tie: the exact mean lies within the error bound of an fp32 sum of the
        # chunk's n terms, n * 2^-24 * mean|x_t|, of the midpoint between the two candidates (first 48 checked)
        for j in range(min(n_diff, 48)):
            doc, ch = divmod(int(c[j]), C)
            Kd = W.host_doc(wl, "K", doc)[1][None]
            exact = O.pool_chunks(Kd, wl.P, None if lens is None else lens[doc:doc + 1])[g[j], ch, e[j]]
            hi = (ch + 1) * wl.P if lens is None else min((ch + 1) * wl.P, int(lens[doc]))
            terms = np.abs(Kd[0, g[j], ch * wl.P:hi, e[j]])
            mid = (got[j] + want[j]) / 2
            assert abs(exact - mid) <= terms.size * 2.0 ** -24 * terms.mean() + 1e-12, (doc, ch, exact, got[j], want[j])
    same_key = ~diff.any(axis=-1) & valid[None, :]
    assert np.allclose(ginv[same_key], oinv[same_key], rtol=1e-6, atol=0)
    gnorm = 1.0 / np.maximum(np.linalg.norm(S.bf16_bits_to_f64(gbits[~same_key & valid[None, :]]), axis=-1),
                             O.EPS_NORM)
    assert np.allclose(ginv[~same_key & valid[None, :]], gnorm, rtol=1e-6, atol=0)
    return n_diff


def upload_index(cfg, bits, inv, lens_valid=None, C=1):
    """Oracle index (bits [Hkv, NC, d], inv [Hkv, NC]) -> the library's tiled layout on the device (re-indexing
    only).  With document lengths, the slots of chunks that do not exist take the library's encoding: they repeat
    the document's chunk 0."""
    Hkv, NC, d = bits.shape
    tiles = cfg.n_tiles
    if lens_valid is not None:
        first = np.repeat(np.arange(NC // C) * C, C)
        bits = bits.copy()
        inv = inv.copy()
        bits[:, ~lens_valid] = bits[:, first[~lens_valid]]
        inv[:, ~lens_valid] = inv[:, first[~lens_valid]]
    pad = np.zeros((Hkv, tiles * 16, d), dtype=np.uint16)
    pad[:, :NC] = bits
    tiled = np.ascontiguousarray(pad.reshape(Hkv, tiles, 16, d // 8, 8).transpose(0, 1, 3, 2, 4))
    invp = np.zeros((Hkv, tiles * 16), dtype=np.float32)
    invp[:, :NC] = inv.astype(np.float32)
    return SD.bits_to_torch(tiled), torch.from_numpy(invp).cuda()


def check_all_selections(wl, obits, q_host, runs, k, valid=None, tokens=None):
    """The oracle's top-k over ALL documents, one KV head at a time, against every GPU run in `runs`
    ([(label, idx, val, atol)], idx / val [B, M, Hkv, k] on the host).  q_host [B, M, Hq, d]; tokens: the query
    tokens (second axis) that q_host holds when it is a sample.  Returns the oracle's indices [B, M, Hkv, k]."""
    B, Mq = q_host.shape[0], q_host.shape[1]
    oi_all = np.empty((B, Mq, wl.Hkv, k), dtype=np.int64)
    n_band = {label: 0 for label, _, _, _ in runs}
    for g in range(wl.Hkv):
        KRb = S.bf16_bits_to_f64(obits[g])[None]                               # [1, NC, d]
        oi, ov, s = O.score_topk(q_host[:, :, g * wl.r:(g + 1) * wl.r], KRb, wl.C, k, valid=valid)
        oi_all[:, :, g] = oi[:, :, 0]
        for b in range(B):
            for mi in range(Mq):
                m = mi if tokens is None else int(tokens[mi])
                for label, gi, gv, atol in runs:
                    n_band[label] += compare_selection(s[b, mi, 0], oi[b, mi, 0], ov[b, mi, 0], gi[b, m, g],
                                                       gv[b, m, g], k, wl.N, atol)
        del KRb, s
    return oi_all, n_band


def check_attention(pool, wl, triples, gi, go, gl, lens=None, what="attend"):
    res = pool.attend(wl, triples, gi, lens)
    worst, worst_rel = 0.0, 0.0
    num = den = 0.0
    for (b, m, g), (oo, ol) in res.items():
        got = go[b, m, g * wl.r:(g + 1) * wl.r]
        err = np.abs(got - oo)
        rel = np.linalg.norm(err) / np.linalg.norm(oo)
        worst, worst_rel = max(worst, err.max()), max(worst_rel, rel)
        num += (err ** 2).sum()
        den += (oo ** 2).sum()
        assert err.max() <= 2e-2 and rel <= 5e-3, (b, m, g, err.max(), rel)
        assert np.allclose(gl[b, m, g * wl.r:(g + 1) * wl.r], ol, rtol=0, atol=5e-3), (b, m, g)
    say(f"   {what}: {len(res)} (query, KV group) outputs, worst max-abs {worst:.3e}, worst rel-L2 {worst_rel:.3e}, "
        f"overall rel-L2 {np.sqrt(num / den):.3e}")


@pytest.mark.parametrize("name,plant,a", [("cfg2_decode_1m", 8, 0.2), ("cfg3_batch32_4m", 25, 0.08),
                                          ("cfg5_decode_50m", 16, 0.2)])
def test_fullsize_decode_complete_parity(pool, name, plant, a):
    t_start = time.time()
    say(f"workload {name}: generating the bank on the device (planted {plant} documents per query, a={a})")
    wl = W.make(name, plant_per_query=plant, plant_a=a)
    cfg = msa.MsaConfig(wl.N, wl.G, wl.P, wl.Hq, wl.Hkv, wl.d, wl.base)
    B, M, k = wl.B, wl.M, wl.k
    assert M == 1
    handle = pool.start_index(wl)                       # the oracle's index, in the background

    say("   build_routing_keys")
    KR, inv = msa.msa_build_routing_keys(cfg, wl.K)
    torch.cuda.synchronize()
    gbits, ginv = gpu_index_bits(cfg, KR, inv)
    obits, oinv = OraclePool.finish_index(handle)
    say(f"   oracle index of {wl.N} documents ready ({time.time() - t_start:.0f} s)")
    n_diff = check_full_index(wl, gbits, ginv, obits, oinv)
    say(f"   all {gbits.size} index elements compared: {n_diff} tie-adjacent roundings, the rest bit-identical")
    del gbits, ginv

    say("   score_topk on the oracle's index and on the GPU's own, against the oracle over all documents")
    dKRo, dinvo = upload_index(cfg, obits, oinv)
    idx_o, val_o = msa.msa_score_topk(cfg, wl.q, dKRo, dinvo, k)
    idx, val = msa.msa_score_topk(cfg, wl.q, KR, inv, k)
    torch.cuda.synchronize()
    runs = [("oracle index", idx_o.cpu().numpy().astype(np.int64), val_o.cpu().numpy().astype(np.float64), SCORE_ATOL),
            ("own index", idx.cpu().numpy().astype(np.int64), val.cpu().numpy().astype(np.float64),
             CHAINED_ATOL if n_diff else SCORE_ATOL)]
    oi, n_band = check_all_selections(wl, obits, wl.q_host, runs, k)
    say(f"   {B * wl.Hkv} selections of {k} among {wl.N} documents equal the oracle's "
        f"(inside the tie band: {n_band}) ({time.time() - t_start:.0f} s)")
    gi = runs[1][1]
    n_own = sum(len({wl.planted[(b, j)] for j in range(plant)} & set(gi[b, 0, g].tolist()))
                for b in range(B) for g in range(wl.Hkv))
    assert n_own >= B * wl.Hkv * min(plant, k) // 2, "planted documents should dominate their own query"

    say("   the same with the head mean over every head (select_scope = ALL)")
    cfg_all = cfg.replace(select_scope=msa.MSA_SCOPE_ALL)
    idx_a, val_a = msa.msa_score_topk(cfg_all, wl.q, dKRo, dinvo, k)
    torch.cuda.synchronize()
    ga, gva = idx_a.cpu().numpy().astype(np.int64), val_a.cpu().numpy().astype(np.float64)
    KRb_all = S.bf16_bits_to_f64(obits)
    oia, ova, s_all = O.score_topk(wl.q_host, KRb_all, wl.C, k, select_scope="all")
    del KRb_all
    nb = sum(compare_selection(s_all[b, 0, 0], oia[b, 0, 0], ova[b, 0, 0], ga[b, 0, 0], gva[b, 0, 0], k, wl.N,
                               SCORE_ATOL) for b in range(B))
    say(f"   {B} all-head selections equal the oracle's (inside the tie band: {nb})")
    del dKRo, dinvo, s_all

    say("   sparse_attend, every (query, KV group)")
    out, lse = msa.msa_sparse_attend(cfg, wl.q, wl.K, wl.V, idx, wl.Kloc, wl.Vloc, wl.pos0, wl.q_pos)
    torch.cuda.synchronize()
    go = out.float().cpu().numpy().astype(np.float64)
    gl = lse.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(go)) and np.all(np.isfinite(gl))
    triples = [(b, 0, g) for b in range(B) for g in range(wl.Hkv)]
    check_attention(pool, wl, triples, gi, go, gl)

    # ---- the pooled, position-encoded bank (Section 3.4.1, Stage 1) and Eq. 3 over it -----------------
    say("   pool_kv + sparse_attend over the pooled bank")
    rng = np.random.default_rng(S.seed_for(wl.cfg_id, 77))
    planted_docs = sorted(set(wl.planted.values()))
    sample = [0, wl.N - 1] + planted_docs[:2] + rng.choice(wl.N, size=6, replace=False).tolist()
    Kbar, Vbar = msa.msa_pool_kv(cfg, wl.K, wl.V)
    torch.cuda.synchronize()
    bad = 0
    for doc in sample:
        for which, bank, pooled in (("K", Kbar, lambda x: O.pool_rotated_keys(x, wl.P, wl.base)),
                                    ("V", Vbar, lambda x: O.pool_values(x, wl.P))):
            exact = pooled(W.host_doc(wl, which, doc)[1][None])[0]
            want = O.bf16_round(exact)
            got = S.bf16_bits_to_f64(SD.torch_to_bits(bank[doc]))
            diff = got != want
            if diff.any():                   # one bf16 step, next to a rounding tie
                # (or, for a mean that cancels to ~0, within the fp32 error of the rotated terms)
                assert np.all(np.abs(got[diff] - want[diff]) <= np.maximum(np.abs(want[diff]) * 2.0 ** -7, 1e-6))
                assert np.all(np.abs(exact[diff] - (got[diff] + want[diff]) / 2) <= 2e-5)
                bad += int(diff.sum())
    assert bad <= 40, bad
    say(f"   pooled K/V of {len(sample)} sampled documents ok ({bad} tie-adjacent roundings)")
    acfg = msa.MsaConfig(wl.N, wl.C, wl.C, wl.Hq, wl.Hkv, wl.d, wl.base, bank_keys_rotated=1)
    pos0 = k                                                   # Section 3.2.2: local positions start at k
    qpos_p = (wl.q_pos - wl.pos0 + pos0).contiguous()
    out, lse = msa.msa_sparse_attend(acfg, wl.q, Kbar, Vbar, idx, wl.Kloc, wl.Vloc, pos0, qpos_p)
    torch.cuda.synchronize()
    go = out.float().cpu().numpy().astype(np.float64)
    gl = lse.cpu().numpy().astype(np.float64)
    per_bg = wl.Lloc * wl.d
    for b, g in ((0, 0), (B - 1, wl.Hkv - 1)):
        docs = gi[b, 0, g]
        Kb_sel = np.stack([O.bf16_round(O.pool_rotated_keys(W.host_doc(wl, "K", int(i))[1][None, g:g + 1],
                                                             wl.P, wl.base))[0] for i in docs])
        Vb_sel = np.stack([O.bf16_round(O.pool_values(W.host_doc(wl, "V", int(i))[1][None, g:g + 1],
                                                       wl.P))[0] for i in docs])
        start = (b * wl.Hkv + g) * per_bg
        Kl = S.normal_bf16(wl.seeds["Kloc"], (1, 1, wl.Lloc, wl.d), start=start)[1]
        Vl = S.normal_bf16(wl.seeds["Vloc"], (1, 1, wl.Lloc, wl.d), start=start)[1]
        qh = wl.q_host[b:b + 1, :, g * wl.r:(g + 1) * wl.r]
        oo, ol = O.sparse_attend(qh, Kb_sel, Vb_sel, np.arange(k)[None, None, None], Kl, Vl, pos0,
                                 wl.q_pos_host[b:b + 1] - wl.pos0 + pos0, wl.base, mem_rotated=True)
        got = go[b, 0, g * wl.r:(g + 1) * wl.r]
        err = np.abs(got - oo[0, 0])
        rel = np.linalg.norm(err) / np.linalg.norm(oo)
        say(f"   pooled attend (b={b}, g={g}): max-abs {err.max():.3e} rel-L2 {rel:.3e}")
        assert err.max() <= 2e-2 and rel <= 5e-3
        assert np.allclose(gl[b, 0, g * wl.r:(g + 1) * wl.r], ol[0, 0], rtol=0, atol=5e-3)
    say(f"   done in {time.time() - t_start:.0f} s")
    del Kbar, Vbar, wl, KR, inv
    torch.cuda.empty_cache()


N_TOKEN_SAMPLE = 64


def test_fullsize_cfg4_prefill_complete_index_sampled_tokens(pool):
    """Benchmark config 4 (2048 question tokens, 16M-token bank): the whole index against the oracle's; per-token
    routing (the scoring GEMM) for 64 sampled tokens against the oracle over ALL 32768 documents; question-level
    routing (token_pool = 1) for all 2048 tokens against the oracle over all documents; attention for the
    sampled tokens, per-token and shared selections."""
    t_start = time.time()
    name = "cfg4_prefill_16m"
    say(f"workload {name}")
    wl = W.make(name, plant_per_query=0)
    cfg = msa.MsaConfig(wl.N, wl.G, wl.P, wl.Hq, wl.Hkv, wl.d, wl.base)
    B, M, k = wl.B, wl.M, wl.k
    handle = pool.start_index(wl)
    KR, inv = msa.msa_build_routing_keys(cfg, wl.K)
    torch.cuda.synchronize()
    gbits, ginv = gpu_index_bits(cfg, KR, inv)
    obits, oinv = OraclePool.finish_index(handle)
    n_diff = check_full_index(wl, gbits, ginv, obits, oinv)
    say(f"   all {gbits.size} index elements compared: {n_diff} tie-adjacent roundings ({time.time() - t_start:.0f} s)")
    del gbits, ginv
    rng = np.random.default_rng(S.seed_for(wl.cfg_id, 78))
    tokens = np.sort(rng.choice(M, size=N_TOKEN_SAMPLE, replace=False))
    tokens[0], tokens[-1] = 0, M - 1
    say(f"   per-token routing of all {M} tokens; oracle over all documents for tokens {tokens.tolist()}")
    dKRo, dinvo = upload_index(cfg, obits, oinv)
    idx_o, val_o = msa.msa_score_topk(cfg, wl.q, dKRo, dinvo, k)
    idx, val = msa.msa_score_topk(cfg, wl.q, KR, inv, k)
    torch.cuda.synchronize()
    runs = [("oracle index", idx_o.cpu().numpy().astype(np.int64), val_o.cpu().numpy().astype(np.float64), SCORE_ATOL),
            ("own index", idx.cpu().numpy().astype(np.int64), val.cpu().numpy().astype(np.float64),
             CHAINED_ATOL if n_diff else SCORE_ATOL)]
    _, n_band = check_all_selections(wl, obits, wl.q_host[:, tokens], runs, k, tokens=tokens)
    say(f"   {N_TOKEN_SAMPLE * wl.Hkv} per-token selections equal the oracle's (inside the tie band: {n_band}) "
        f"({time.time() - t_start:.0f} s)")
    gi = runs[1][1]
    assert gi.min() >= 0 and gi.max() < wl.N                       # every token's list, not only the sampled ones
    gv_all = runs[1][2]
    assert np.all(np.diff(gv_all, axis=-1) <= 0)

    say("   question-level routing (token_pool = 1), all tokens, oracle over all documents")
    cfg_p = cfg.replace(token_pool=1)
    idx_p, val_p = msa.msa_score_topk(cfg_p, wl.q, dKRo, dinvo, k)
    torch.cuda.synchronize()
    gp, gvp = idx_p.cpu().numpy().astype(np.int64), val_p.cpu().numpy().astype(np.float64)
    assert gp.shape == (B, 1, wl.Hkv, k)
    nb = 0
    blk = 256
    for g in range(wl.Hkv):
        KRb = S.bf16_bits_to_f64(obits[g])[None]
        Sc = None
        for m0 in range(0, M, blk):          # max over the tokens = max over blocks of tokens of the blocks' maxima
            part = O.chunk_scores(wl.q_host[:, m0:m0 + blk, g * wl.r:(g + 1) * wl.r], KRb, token_pool=True)
            Sc = part if Sc is None else np.maximum(Sc, part)
        s = O.doc_scores(Sc, wl.C)[:, 0, 0]                             # [B, N]
        oi, ov = O.topk_docs(s, k)
        for b in range(B):
            nb += compare_selection(s[b], oi[b], ov[b], gp[b, 0, g], gvp[b, 0, g], k, wl.N, SCORE_ATOL)
    say(f"   {B * wl.Hkv} pooled selections equal the oracle's (inside the tie band: {nb}) ({time.time() - t_start:.0f} s)")
    del dKRo, dinvo

    say("   sparse_attend with per-token selections, sampled tokens x every KV group")
    out, lse = msa.msa_sparse_attend(cfg, wl.q, wl.K, wl.V, idx, wl.Kloc, wl.Vloc, wl.pos0, wl.q_pos)
    torch.cuda.synchronize()
    go = out.float().cpu().numpy().astype(np.float64)
    gl = lse.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(go)) and np.all(np.isfinite(gl))
    triples = [(0, int(m), g) for m in tokens for g in range(wl.Hkv)]
    check_attention(pool, wl, triples, gi, go, gl, what="attend (per-token selections)")
    say("   sparse_attend with the shared selection (tiled kernel), sampled tokens x every KV group")
    out, lse = msa.msa_sparse_attend(cfg_p, wl.q, wl.K, wl.V, idx_p, wl.Kloc, wl.Vloc, wl.pos0, wl.q_pos)
    torch.cuda.synchronize()
    go = out.float().cpu().numpy().astype(np.float64)
    gl = lse.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(go)) and np.all(np.isfinite(gl))
    check_attention(pool, wl, triples, gp, go, gl, what="attend (shared selection)")
    say(f"   done in {time.time() - t_start:.0f} s")
    del wl, KR, inv
    torch.cuda.empty_cache()


def test_fullsize_cfg3_documents_of_different_lengths(pool):
    """Benchmark config 3 with seeded document lengths in [G/8, G] (cfg.doc_lens): the whole index, every
    selection and every output against the oracle's lens / valid reading."""
    t_start = time.time()
    name = "cfg3_batch32_4m"
    say(f"workload {name} with document lengths")
    wl = W.make(name, plant_per_query=0)
    lens = W.doc_lens(wl).astype(np.int64)
    dlens = torch.from_numpy(lens.astype(np.int32)).cuda()
    cfg = msa.MsaConfig(wl.N, wl.G, wl.P, wl.Hq, wl.Hkv, wl.d, wl.base, doc_lens=dlens)
    B, k = wl.B, wl.k
    handle = pool.start_index(wl, lens)
    KR, inv = msa.msa_build_routing_keys(cfg, wl.K)
    torch.cuda.synchronize()
    gbits, ginv = gpu_index_bits(cfg, KR, inv)
    obits, oinv = OraclePool.finish_index(handle)
    n_diff = check_full_index(wl, gbits, ginv, obits, oinv, lens)
    say(f"   all existing chunks compared: {n_diff} tie-adjacent roundings; missing chunks repeat chunk 0")
    valid = O.chunk_valid(lens, wl.G, wl.P)
    dKRo, dinvo = upload_index(cfg, obits, oinv, valid, wl.C)
    idx_o, val_o = msa.msa_score_topk(cfg, wl.q, dKRo, dinvo, k)
    idx, val = msa.msa_score_topk(cfg, wl.q, KR, inv, k)
    torch.cuda.synchronize()
    runs = [("oracle index", idx_o.cpu().numpy().astype(np.int64), val_o.cpu().numpy().astype(np.float64), SCORE_ATOL),
            ("own index", idx.cpu().numpy().astype(np.int64), val.cpu().numpy().astype(np.float64),
             CHAINED_ATOL if n_diff else SCORE_ATOL)]
    _, n_band = check_all_selections(wl, obits, wl.q_host, runs, k, valid=valid)
    say(f"   {B * wl.Hkv} selections equal the oracle's (inside the tie band: {n_band})")
    gi = runs[1][1]
    out, lse = msa.msa_sparse_attend(cfg, wl.q, wl.K, wl.V, idx, wl.Kloc, wl.Vloc, wl.pos0, wl.q_pos)
    torch.cuda.synchronize()
    go = out.float().cpu().numpy().astype(np.float64)
    gl = lse.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(go)) and np.all(np.isfinite(gl))
    triples = [(b, 0, g) for b in range(B) for g in range(wl.Hkv)]
    check_attention(pool, wl, triples, gi, go, gl, lens=lens, what="attend (document lengths)")
    say(f"   done in {time.time() - t_start:.0f} s")
    del wl, KR, inv
    torch.cuda.empty_cache()
