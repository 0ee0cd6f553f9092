"""Parity at the full sizes of the benchmark configurations, in the launch configuration bench.py times (same workload
builder, same B / M / k, same entry points).  The banks (2 GiB .. 191 GiB of K/V) are generated on the
device; the oracle works on documents regenerated on the host bit-for-bit, so it can check SAMPLED
outputs one by one:

  build   : routing keys + inv_norm of sampled documents (first, last, planted, random)
  score   : the oracle's own score of every document the GPU selected (for sampled queries) must match
            the reported score, the list must be ordered, every planted document that beats the k-th
            score by more than the tie band must be in the list, and no sampled or planted
            non-selected document may beat the k-th score by more than the band
  attend  : oracle attention for sampled (query, KV group) pairs over the selected documents'
            regenerated K/V and the local context, same tolerances as the small cases
"""
import numpy as np
import pytest
import torch

import msa_synth as S
import paper_2603_23516_amd as msa
from msa_synth import device as SD
from msa_synth import workloads as W
from oracle import msa_oracle as O

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


def kr_rows(cfg, KR, inv, doc):
    """Routing keys of one document from the tiled index: (bits [Hkv, C, d] host, inv [Hkv, C])."""
    C = cfg.chunks_per_doc
    c = torch.arange(doc * C, (doc + 1) * C, device=KR.device)
    # two index tensors separated by a slice: the indexed axis comes first -> [C, Hkv, d/8, 8]
    rows = KR[:, c // 16, :, c % 16, :].permute(1, 0, 2, 3)
    bits = SD.torch_to_bits(rows.reshape(cfg.n_kv_heads, C, cfg.head_dim))
    return bits, inv[:, c].cpu().numpy().astype(np.float64)


def oracle_doc_scores(wl, q_sel, docs):
    """Oracle score of each listed document for the queries q_sel [nq, Hq, d]: [nq, Hkv, len(docs)]."""
    Ks = np.stack([W.host_doc(wl, "K", int(i))[1] for i in docs])
    KRb, _ = O.routing_keys(Ks, wl.P)
    s = O.doc_scores(O.chunk_scores(q_sel[:, None], KRb), wl.C)   # [nq, 1, Hkv, n]
    return s[:, 0]


@pytest.mark.parametrize("name,plant,a", [("cfg2_decode_1m", 8, 0.2), ("cfg3_batch32_4m", 25, 0.08),
                                          ("cfg5_decode_50m", 16, 0.2), ("cfg4_prefill_16m", 0, 0.0)])
def test_fullsize_sampled_parity(name, plant, a):
    say(f"workload {name}: generating the bank on the device (planted {plant} documents per query, a={a})")
    wl = W.make(name, plant_per_query=plant, plant_a=a)
    cfg = msa.MsaConfig(wl.N, wl.G, wl.P, wl.Hq, wl.Hkv, wl.d, wl.base)
    rng = np.random.default_rng(S.seed_for(wl.cfg_id, 77))
    B, M, k = wl.B, wl.M, wl.k

    # ---- build ------------------------------------------------------------------------------
    say("   build_routing_keys")
    KR, inv = msa.msa_build_routing_keys(cfg, wl.K)
    torch.cuda.synchronize()
    planted_docs = sorted(set(wl.planted.values()))
    sample = [0, wl.N - 1] + planted_docs[:6] + rng.choice(wl.N, size=16, replace=False).tolist()
    bad = 0
    for doc in sample:
        bits, ginv = kr_rows(cfg, KR, inv, doc)
        got = S.bf16_bits_to_f64(bits)
        Kd = W.host_doc(wl, "K", doc)[1][None]
        want, winv = O.routing_keys(Kd, wl.P)
        diff = got != want
        if diff.any():                       # only next to a rounding tie, one bf16 ulp
            assert np.all(np.abs(got[diff] - want[diff]) <= np.abs(want[diff]) * 2.0 ** -7 + 1e-30)
            bad += int(diff.sum())
        assert np.allclose(ginv, 1.0 / np.maximum(np.linalg.norm(got, axis=-1), O.EPS_NORM), rtol=1e-6)
    assert bad <= 4, bad
    say(f"   routing keys of {len(sample)} sampled documents ok ({bad} tie-adjacent roundings)")

    # ---- score + top-k ------------------------------------------------------------------------
    say("   score_topk")
    idx, val = msa.msa_score_topk(cfg, wl.q, KR, inv, k)
    torch.cuda.synchronize()
    gi = idx.cpu().numpy().astype(np.int64).reshape(B * M, 1, wl.Hkv, k)      # one row per query token
    gv = val.cpu().numpy().astype(np.float64).reshape(B * M, 1, wl.Hkv, k)
    q_flat = wl.q_host.reshape(B * M, 1, wl.Hq, wl.d)
    B = B * M
    assert gi.min() >= 0 and gi.max() < wl.N
    for b in range(B):
        for g in range(wl.Hkv):
            assert len(set(gi[b, 0, g].tolist())) == k
            d = np.diff(gv[b, 0, g])
            assert np.all(d <= 0)
            tie = d == 0
            assert np.all(np.diff(gi[b, 0, g])[tie] > 0)          # equal scores: ascending index
    q_sample = sorted({0, B - 1})
    for b in q_sample:
        docs = sorted(set(gi[b, 0].reshape(-1).tolist()))
        s = oracle_doc_scores(wl, q_flat[b], docs)                # [1, Hkv, n]
        pos = {dd: i for i, dd in enumerate(docs)}
        for g in range(wl.Hkv):
            want = np.array([s[0, g, pos[int(dd)]] for dd in gi[b, 0, g]])
            assert np.allclose(gv[b, 0, g], want, rtol=0, atol=1e-4), np.abs(gv[b, 0, g] - want).max()
    # non-selected documents: planted ones and a random sample must not beat the k-th score
    others = sorted(set(planted_docs[:160]) | set(rng.choice(wl.N, size=96, replace=False).tolist()))
    q_chk = sorted(set(range(0, B, max(1, B // 32))) | {B - 1})    # all queries, or 33 sampled tokens in prefill
    s_all = oracle_doc_scores(wl, q_flat[q_chk, 0], others)         # [len(q_chk), Hkv, n]
    n_planted_in = 0
    for bi, b in enumerate(q_chk):
        for g in range(wl.Hkv):
            kth = gv[b, 0, g, k - 1]
            band = 1e-3 * abs(kth) + 1e-4
            chosen = set(gi[b, 0, g].tolist())
            for j, dd in enumerate(others):
                if dd in chosen:
                    n_planted_in += dd in wl.planted_K
                    continue
                assert s_all[bi, g, j] <= kth + band, (b, g, dd, s_all[bi, g, j], kth)
    n_own = 0
    for b in range(B if plant else 0):
        own = {wl.planted[(b, j)] for j in range(plant)}
        for g in range(wl.Hkv):
            n_own += len(own & set(gi[b, 0, g].tolist()))
    say(f"   top-k ok; {n_own} of {B * wl.Hkv * k} selections are the query's own planted documents "
        f"({n_planted_in} hits among the sampled non-random documents)")
    assert n_own >= B * wl.Hkv * min(plant, k) // 2, "planted documents should dominate their own query"

    # ---- attention -----------------------------------------------------------------------------
    say("   sparse_attend")
    out, lse = msa.msa_sparse_attend(cfg, wl.q, wl.K, wl.V, idx, wl.Kloc, wl.Vloc, wl.pos0, wl.q_pos)
    torch.cuda.synchronize()
    go = out.float().cpu().numpy().astype(np.float64).reshape(B, 1, wl.Hq, wl.d)
    gl = lse.cpu().numpy().astype(np.float64).reshape(B, 1, wl.Hq)
    assert np.all(np.isfinite(go)) and np.all(np.isfinite(gl))
    pairs = [(0, 0), (B - 1, wl.Hkv - 1)] if B > 1 else [(0, 0), (0, wl.Hkv - 1)]
    if M > 1:
        pairs.append((M // 3, 3))             # a token in the middle of the causal window
    per_bg = wl.Lloc * wl.d
    qpos_flat = wl.q_pos_host.reshape(B, 1)
    for b, g in pairs:
        docs = gi[b, 0, g]
        K_sel = np.stack([W.host_doc(wl, "K", int(i))[1][g:g + 1] for i in docs])   # [k, 1, G, d]
        V_sel = np.stack([W.host_doc(wl, "V", int(i))[1][g:g + 1] for i in docs])
        start = ((b // M) * wl.Hkv + g) * per_bg
        Kl = S.normal_bf16(wl.seeds["Kloc"], (1, 1, wl.Lloc, wl.d), start=start)[1]
        Vl = S.normal_bf16(wl.seeds["Vloc"], (1, 1, wl.Lloc, wl.d), start=start)[1]
        qh = q_flat[b:b + 1, :, g * wl.r:(g + 1) * wl.r]
        oo, ol = O.sparse_attend(qh, K_sel, V_sel, np.arange(k)[None, None, None], Kl, Vl, wl.pos0,
                                 qpos_flat[b:b + 1], wl.base)
        got = go[b, 0, g * wl.r:(g + 1) * wl.r]
        err = np.abs(got - oo[0, 0])
        rel = np.linalg.norm(err) / np.linalg.norm(oo)
        say(f"   attend (b={b}, g={g}): max-abs {err.max():.3e} rel-L2 {rel:.3e}")
        assert err.max() <= 2e-2 and rel <= 5e-3
        assert np.allclose(gl[b, 0, g * wl.r:(g + 1) * wl.r], ol[0, 0], rtol=0, atol=5e-3)
    # ---- the pooled, position-encoded bank (Section 3.4.1, Stage 1) and Eq. 3 over it -----------------
    if M == 1:
        say("   pool_kv + sparse_attend over the pooled bank")
        Kbar, Vbar = msa.msa_pool_kv(cfg, wl.K, wl.V)
        torch.cuda.synchronize()
        bad = 0
        for doc in sample[:10]:
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
        say(f"   pooled K/V of 10 sampled documents ok ({bad} tie-adjacent roundings)")
        acfg = msa.MsaConfig(wl.N, wl.C, wl.C, wl.Hq, wl.Hkv, wl.d, wl.base, bank_keys_rotated=1)
        pos0 = k                                                   # Section 3.2.2: local positions start at k
        qpos_p = (wl.q_pos - wl.pos0 + pos0).contiguous()
        out, lse = msa.msa_sparse_attend(acfg, wl.q, Kbar, Vbar, idx, wl.Kloc, wl.Vloc, pos0, qpos_p)
        torch.cuda.synchronize()
        go = out.float().cpu().numpy().astype(np.float64).reshape(B, 1, wl.Hq, wl.d)
        gl = lse.cpu().numpy().astype(np.float64).reshape(B, 1, wl.Hq)
        for b, g in pairs:
            docs = gi[b, 0, g]
            Kb_sel = np.stack([O.bf16_round(O.pool_rotated_keys(W.host_doc(wl, "K", int(i))[1][None, g:g + 1],
                                                                 wl.P, wl.base))[0] for i in docs])
            Vb_sel = np.stack([O.bf16_round(O.pool_values(W.host_doc(wl, "V", int(i))[1][None, g:g + 1],
                                                           wl.P))[0] for i in docs])
            start = (b * wl.Hkv + g) * per_bg
            Kl = S.normal_bf16(wl.seeds["Kloc"], (1, 1, wl.Lloc, wl.d), start=start)[1]
            Vl = S.normal_bf16(wl.seeds["Vloc"], (1, 1, wl.Lloc, wl.d), start=start)[1]
            qh = q_flat[b:b + 1, :, g * wl.r:(g + 1) * wl.r]
            oo, ol = O.sparse_attend(qh, Kb_sel, Vb_sel, np.arange(k)[None, None, None], Kl, Vl, pos0,
                                     qpos_flat[b:b + 1] - wl.pos0 + pos0, wl.base, mem_rotated=True)
            got = go[b, 0, g * wl.r:(g + 1) * wl.r]
            err = np.abs(got - oo[0, 0])
            rel = np.linalg.norm(err) / np.linalg.norm(oo)
            say(f"   pooled attend (b={b}, g={g}): max-abs {err.max():.3e} rel-L2 {rel:.3e}")
            assert err.max() <= 2e-2 and rel <= 5e-3
            assert np.allclose(gl[b, 0, g * wl.r:(g + 1) * wl.r], ol[0, 0], rtol=0, atol=5e-3)
        del Kbar, Vbar
    del wl, KR, inv
    torch.cuda.empty_cache()


def test_fullsize_cfg4_question_level_routing():
    """benchmark config 4 with Eq. 2 as printed over the tokens (token_pool = 1): one selection per KV head
    for the whole 2048-token question (GEMM scoring + token pooling), then the tiled shared-selection
    attention kernel.  Sampled checks against the oracle as above."""
    name = "cfg4_prefill_16m"
    say(f"workload {name}, token_pool = 1")
    wl = W.make(name, plant_per_query=0)
    cfg = msa.MsaConfig(wl.N, wl.G, wl.P, wl.Hq, wl.Hkv, wl.d, wl.base, token_pool=1)
    rng = np.random.default_rng(S.seed_for(wl.cfg_id, 78))
    B, M, k = wl.B, wl.M, wl.k
    KR, inv = msa.msa_build_routing_keys(cfg, wl.K)
    idx, val = msa.msa_score_topk(cfg, wl.q, KR, inv, k)
    torch.cuda.synchronize()
    assert tuple(idx.shape) == (B, 1, wl.Hkv, k)
    gi = idx.cpu().numpy().astype(np.int64)
    gv = val.cpu().numpy().astype(np.float64)
    assert gi.min() >= 0 and gi.max() < wl.N
    others = rng.choice(wl.N, size=64, replace=False).tolist()
    for b in range(B):
        docs = sorted(set(gi[b, 0].reshape(-1).tolist()) | set(others))
        Ks = np.stack([W.host_doc(wl, "K", int(i))[1] for i in docs])
        KRb, _ = O.routing_keys(Ks, wl.P)
        s = O.doc_scores(O.chunk_scores(wl.q_host[b:b + 1], KRb, token_pool=True), wl.C)[0, 0]   # [Hkv, n]
        pos = {dd: i for i, dd in enumerate(docs)}
        for g in range(wl.Hkv):
            assert len(set(gi[b, 0, g].tolist())) == k and np.all(np.diff(gv[b, 0, g]) <= 0)
            want = np.array([s[g, pos[int(dd)]] for dd in gi[b, 0, g]])
            assert np.allclose(gv[b, 0, g], want, rtol=0, atol=1e-4), np.abs(gv[b, 0, g] - want).max()
            kth = gv[b, 0, g, k - 1]
            chosen = set(gi[b, 0, g].tolist())
            for dd in others:
                if dd not in chosen:
                    assert s[g, pos[dd]] <= kth + 1e-3 * abs(kth) + 1e-4
    say("   pooled top-k ok")
    out, lse = msa.msa_sparse_attend(cfg, wl.q, wl.K, wl.V, idx, wl.Kloc, wl.Vloc, wl.pos0, wl.q_pos)
    torch.cuda.synchronize()
    go = out.float().cpu().numpy().astype(np.float64)
    gl = lse.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(go)) and np.all(np.isfinite(gl))
    per_bg = wl.Lloc * wl.d
    for b, m, g in ((0, 0, 0), (B - 1, M // 3, 3), (B - 1, M - 1, wl.Hkv - 1)):
        docs = gi[b, 0, g]
        K_sel = np.stack([W.host_doc(wl, "K", int(i))[1][g:g + 1] for i in docs])
        V_sel = np.stack([W.host_doc(wl, "V", int(i))[1][g:g + 1] for i in docs])
        start = (b * wl.Hkv + g) * per_bg
        Kl = S.normal_bf16(wl.seeds["Kloc"], (1, 1, wl.Lloc, wl.d), start=start)[1]
        Vl = S.normal_bf16(wl.seeds["Vloc"], (1, 1, wl.Lloc, wl.d), start=start)[1]
        qh = wl.q_host[b:b + 1, m:m + 1, g * wl.r:(g + 1) * wl.r]
        oo, ol = O.sparse_attend(qh, K_sel, V_sel, np.arange(k)[None, None, None], Kl, Vl, wl.pos0,
                                 wl.q_pos_host[b:b + 1, m:m + 1], wl.base)
        got = go[b, m, g * wl.r:(g + 1) * wl.r]
        err = np.abs(got - oo[0, 0])
        rel = np.linalg.norm(err) / np.linalg.norm(oo)
        say(f"   shared-selection attend (b={b}, m={m}, g={g}): max-abs {err.max():.3e} rel-L2 {rel:.3e}")
        assert err.max() <= 2e-2 and rel <= 5e-3
        assert np.allclose(gl[b, m, g * wl.r:(g + 1) * wl.r], ol[0, 0], rtol=0, atol=5e-3)
    del wl, KR, inv
    torch.cuda.empty_cache()


def test_fullsize_cfg3_documents_of_different_lengths():
    """benchmark config 3 with seeded document lengths in [G/8, G] (cfg.doc_lens): sampled checks of the index,
    the selection and the attention against the oracle's lens / valid arguments."""
    name = "cfg3_batch32_4m"
    say(f"workload {name} with document lengths")
    wl = W.make(name, plant_per_query=0)
    lens = W.doc_lens(wl).astype(np.int64)
    dlens = torch.from_numpy(lens.astype(np.int32)).cuda()
    cfg = msa.MsaConfig(wl.N, wl.G, wl.P, wl.Hq, wl.Hkv, wl.d, wl.base, doc_lens=dlens)
    rng = np.random.default_rng(S.seed_for(wl.cfg_id, 79))
    B, k, C = wl.B, wl.k, wl.C
    KR, inv = msa.msa_build_routing_keys(cfg, wl.K)
    torch.cuda.synchronize()
    sample = [0, wl.N - 1, int(np.argmin(lens)), int(np.argmax(lens))] + rng.choice(wl.N, size=12, replace=False).tolist()
    bad = 0
    for doc in sample:
        bits, ginv = kr_rows(cfg, KR, inv, doc)
        got = S.bf16_bits_to_f64(bits)
        want, winv = O.routing_keys(W.host_doc(wl, "K", doc)[1][None], wl.P, lens[doc:doc + 1])
        ok = winv[0] > 0                                           # chunks the document has
        diff = (got != want) & ok[None, :, None]
        if diff.any():
            assert np.all(np.abs(got[diff] - want[diff]) <= np.abs(want[diff]) * 2.0 ** -7 + 1e-30)
            bad += int(diff.sum())
        assert np.array_equal(got[:, ~ok], np.repeat(got[:, :1], int((~ok).sum()), axis=1))   # repeat chunk 0
        assert np.allclose(ginv, 1.0 / np.maximum(np.linalg.norm(got, axis=-1), O.EPS_NORM), rtol=1e-6)
    assert bad <= 4, bad
    say(f"   routing keys of {len(sample)} sampled documents ok ({bad} tie-adjacent roundings)")

    idx, val = msa.msa_score_topk(cfg, wl.q, KR, inv, k)
    torch.cuda.synchronize()
    gi = idx.cpu().numpy().astype(np.int64)
    gv = val.cpu().numpy().astype(np.float64)
    assert gi.min() >= 0 and gi.max() < wl.N
    others = rng.choice(wl.N, size=96, replace=False).tolist()

    def scores(q_sel, docs):                                       # oracle document scores [nq, Hkv, n]
        Ks = np.stack([W.host_doc(wl, "K", int(i))[1] for i in docs])
        dl = lens[np.asarray(docs)]
        KRb, _ = O.routing_keys(Ks, wl.P, dl)
        return O.doc_scores(O.chunk_scores(q_sel[:, None], KRb, valid=O.chunk_valid(dl, wl.G, wl.P)), C)[:, 0]

    for b in (0, B // 2, B - 1):
        docs = sorted(set(gi[b, 0].reshape(-1).tolist()) | set(others))
        s = scores(wl.q_host[b], docs)[0]
        pos = {dd: i for i, dd in enumerate(docs)}
        for g in range(wl.Hkv):
            assert len(set(gi[b, 0, g].tolist())) == k and np.all(np.diff(gv[b, 0, g]) <= 0)
            want = np.array([s[g, pos[int(dd)]] for dd in gi[b, 0, g]])
            assert np.allclose(gv[b, 0, g], want, rtol=0, atol=1e-4), np.abs(gv[b, 0, g] - want).max()
            kth = gv[b, 0, g, k - 1]
            chosen = set(gi[b, 0, g].tolist())
            for dd in others:
                if dd not in chosen:
                    assert s[g, pos[dd]] <= kth + 1e-3 * abs(kth) + 1e-4
    say("   top-k ok")

    out, lse = msa.msa_sparse_attend(cfg, wl.q, wl.K, wl.V, idx, wl.Kloc, wl.Vloc, wl.pos0, wl.q_pos)
    torch.cuda.synchronize()
    go = out.float().cpu().numpy().astype(np.float64)
    gl = lse.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(go)) and np.all(np.isfinite(gl))
    per_bg = wl.Lloc * wl.d
    for b, g in ((0, 0), (B - 1, wl.Hkv - 1), (B // 2, 3)):
        docs = gi[b, 0, g]
        K_sel = np.stack([W.host_doc(wl, "K", int(i))[1][g:g + 1] for i in docs])
        V_sel = np.stack([W.host_doc(wl, "V", int(i))[1][g:g + 1] for i in docs])
        start = (b * wl.Hkv + g) * per_bg
        Kl = S.normal_bf16(wl.seeds["Kloc"], (1, 1, wl.Lloc, wl.d), start=start)[1]
        Vl = S.normal_bf16(wl.seeds["Vloc"], (1, 1, wl.Lloc, wl.d), start=start)[1]
        qh = wl.q_host[b:b + 1, :, g * wl.r:(g + 1) * wl.r]
        oo, ol = O.sparse_attend(qh, K_sel, V_sel, np.arange(k)[None, None, None], Kl, Vl, wl.pos0,
                                 wl.q_pos_host[b:b + 1], wl.base, lens=lens[docs])
        got = go[b, 0, g * wl.r:(g + 1) * wl.r]
        err = np.abs(got - oo[0, 0])
        rel = np.linalg.norm(err) / np.linalg.norm(oo)
        say(f"   attend (b={b}, g={g}, lengths {lens[docs].min()}..{lens[docs].max()}): max-abs {err.max():.3e} "
            f"rel-L2 {rel:.3e}")
        assert err.max() <= 2e-2 and rel <= 5e-3
        assert np.allclose(gl[b, 0, g * wl.r:(g + 1) * wl.r], ol[0, 0], rtol=0, atol=5e-3)
    del wl, KR, inv
    torch.cuda.empty_cache()
