"""GPU parity for documents of different lengths (the paper's G is an average document length, Section
5.1): every stage with cfg.doc_lens against the float64 oracle's `lens` / `valid` arguments.

Reading under test: document i holds lens[i] <= G tokens in the first rows of its slot; it has
ceil(lens[i] / P) chunks, the last one the mean over the tokens it holds (phi of Section 3.2.1 averages the
tokens of a chunk); chunks past the end do not score; attention (Eq. 3-4) sees only the rows that exist.
Tolerances are those of test_gpu_parity.py.
"""
import numpy as np
import pytest
import torch

import msa_synth as S
import paper_2603_23516_amd as msa
from oracle import msa_oracle as O
from test_gpu_parity import (Case, bf16_to_f64, check_pooled, check_topk_generic, dev, say)

pytestmark = pytest.mark.gpu


def make_lens(seed, N, G, P):
    """Seeded lengths in [1, G] with the edge values planted: one token, a full slot, whole chunks, one
    token into a chunk, one short of a 32-row step."""
    rng = np.random.default_rng(seed)
    lens = rng.integers(1, G + 1, size=N)
    plant = [1, G, P, min(G, P + 1), min(G, 31), min(G, 33), G - 1 if G > 1 else 1]
    for i, v in enumerate(plant[:N]):
        lens[i] = max(1, v)
    return lens.astype(np.int64)


def ragged_index_for_upload(KRo, invo, lens, C):
    """The oracle's index in the library's encoding of "no such chunk": the slot repeats the document's
    chunk 0 (pure re-indexing of oracle values)."""
    KR, inv = KRo.copy(), invo.copy()
    N = lens.size
    for i in range(N):
        for j in range(C):
            if inv[0, i * C + j] < 0:
                KR[:, i * C + j] = KRo[:, i * C]
                inv[:, i * C + j] = invo[:, i * C]
    return KR, inv


def upload_index(cfg, KRb, inv):
    from test_gpu_parity import upload_oracle_index
    return upload_oracle_index(cfg, KRb, inv)


def attend_err(out, lse, oo, ol):
    go = out.float().cpu().numpy().astype(np.float64)
    gl = lse.cpu().numpy().astype(np.float64)
    err = np.abs(go - oo)
    rel = np.linalg.norm(err) / max(np.linalg.norm(oo), 1e-30)
    say(f"   attend: max-abs {err.max():.3e}  rel-L2 {rel:.3e}")
    assert err.max() <= 2e-2 and rel <= 5e-3, (err.max(), rel)
    fin = np.isfinite(ol)
    assert np.array_equal(np.isfinite(gl), fin)
    assert np.allclose(gl[fin], ol[fin], rtol=0, atol=5e-3), np.abs(gl[fin] - ol[fin]).max()


RAGGED_CASES = {
    # name: (seed, N, Hkv, r, G, d, P, B, M, Lloc, base, k, scope, pool)
    "decode_c8_d128": (61000, 60, 2, 4, 512, 128, 64, 2, 1, 50, 1e6, 6, "group", False),
    "decode_c4_d64_batch": (62000, 203, 2, 2, 128, 64, 32, 9, 2, 33, 1e4, 5, "group", False),
    "scope_all_hkv4": (63000, 150, 4, 2, 64, 64, 16, 3, 1, 20, 1e4, 7, "all", False),
    "c1_whole_doc_chunk": (64000, 90, 3, 1, 64, 64, 64, 1, 3, 64, 1e6, 7, "group", False),
    "c16_r8_no_local": (65000, 21, 1, 8, 256, 128, 16, 1, 2, 0, 1e4, 9, "group", False),
    "prefill_gemm_token_pool": (66000, 120, 2, 4, 64, 128, 8, 2, 80, 80, 1e6, 8, "group", True),
    "prefill_gemm_per_token": (67000, 77, 2, 2, 128, 64, 32, 1, 100, 40, 1e4, 5, "group", False),
    "eq2_as_printed": (68000, 64, 2, 4, 128, 128, 32, 2, 12, 30, 1e6, 4, "all", True),
}


@pytest.mark.parametrize("name", list(RAGGED_CASES))
def test_ragged_stage_parity(name):
    seed, N, Hkv, r, G, d, P, B, M, Lloc, base, k, scope, pool = RAGGED_CASES[name]
    say(f"ragged case {name}: N={N} Hkv={Hkv} r={r} G={G} d={d} P={P} B={B} M={M} Lloc={Lloc} k={k} "
        f"scope={scope} token_pool={pool}")
    case = Case(seed, N, Hkv, r, G, d, P, B, M, Lloc, base).to_device()
    C = G // P
    lens = make_lens(seed + 9, N, G, P)
    dlens = torch.from_numpy(lens.astype(np.int32)).cuda()
    cfg = case.cfg(select_scope=msa.MSA_SCOPE_ALL if scope == "all" else msa.MSA_SCOPE_GROUP, token_pool=int(pool),
                   doc_lens=dlens)
    valid = O.chunk_valid(lens, G, P)

    say("   build_routing_keys")
    KR, inv = msa.msa_build_routing_keys(cfg, case.dK)
    torch.cuda.synchronize()
    KRo, invo = O.routing_keys(case.K, P, lens)
    exact = O.pool_chunks(case.K, P, lens)
    got = bf16_to_f64(msa.untile_routing_keys(cfg, KR))
    gi = inv.cpu().numpy().astype(np.float64)[:, :N * C]
    diff = (got != KRo) & valid[None, :, None]
    if diff.any():
        mid = (got[diff] + KRo[diff]) / 2
        assert np.all(np.abs(got[diff] - KRo[diff]) <= np.abs(KRo[diff]) * 2.0 ** -7 + 1e-30), "more than one bf16 ulp"
        assert np.all(np.abs(exact[diff] - mid) <= 64 * 2.0 ** -24 * np.abs(exact[diff]) + 1e-12), "not a tie"
    assert diff.mean() < 1e-3
    gnorm = 1.0 / np.maximum(np.linalg.norm(got, axis=-1), O.EPS_NORM)
    assert np.allclose(gi, gnorm, rtol=1e-6)
    # slots of chunks that do not exist repeat chunk 0 of their document, bit for bit
    first = (np.arange(N * C) // C) * C
    assert np.array_equal(got[:, ~valid], got[:, first[~valid]])
    assert np.array_equal(gi[:, ~valid], gi[:, first[~valid]])
    say(f"   routing keys ok ({int(diff.sum())} tie-adjacent roundings, {int((~valid).sum())} slots without a chunk)")

    say("   score_topk on the oracle's index")
    KRu, invu = ragged_index_for_upload(KRo, invo, lens, C)
    dKRo, dinvo = upload_index(cfg, KRu, invu)
    idx_s, val_s = msa.msa_score_topk(cfg, case.dq, dKRo, dinvo, k)
    torch.cuda.synchronize()
    oi, n_band = check_topk_generic(case.q, KRo, C, N, idx_s, val_s, k, "cos", scope, pool, valid=valid)
    say(f"   top-k ok, shape {tuple(idx_s.shape)} ({n_band} inside the tie band)")
    say("   score_topk on the GPU's own index")
    idx, val = msa.msa_score_topk(cfg, case.dq, KR, inv, k)
    torch.cuda.synchronize()
    _, n_band = check_topk_generic(case.q, KRo, C, N, idx, val, k, "cos", scope, pool,
                                   atol=2e-4 if diff.any() else 2e-5, valid=valid)
    say(f"   chained top-k ok ({n_band} inside the tie band)")
    # the lengths matter: the same bank read as full-length documents selects differently somewhere
    oi_full, _, _ = O.score_topk(case.q, O.routing_keys(case.K, P)[0], C, k, "cos", scope, pool)
    say(f"   selections that differ from the full-length reading: {int((oi_full != oi).any(axis=-1).sum())}")

    say("   sparse_attend (oracle's indices)")
    pos0 = G
    q_pos = np.array([[pos0 + (min(Lloc - 1, (3 * m + b) % Lloc) if Lloc else 0) for m in range(M)]
                      for b in range(B)])
    if M == 1 and Lloc:
        q_pos[:] = pos0 + Lloc - 1
    dpos = torch.from_numpy(q_pos.astype(np.int32)).cuda()
    sel = oi.copy()
    sel[0, 0, 0, k // 2] = -1                                       # a pad among ragged documents
    # make sure the planted edge lengths (one token, whole chunks, 31 / 33 rows ...) are attended
    flat = sel.reshape(-1, k)
    for row in range(min(flat.shape[0], 3)):
        flat[row, :min(k - 1, 3)] = [(3 * row + t) % min(N, 7) for t in range(min(k - 1, 3))]
    didx = torch.from_numpy(sel.astype(np.int32)).cuda()
    out, lse = msa.msa_sparse_attend(cfg, case.dq, case.dK, case.dV, didx, case.dKl, case.dVl, pos0, dpos)
    torch.cuda.synchronize()
    oo, ol = O.sparse_attend(case.q, case.K, case.V, sel, case.Kl, case.Vl, pos0, q_pos, base, lens=lens)
    attend_err(out, lse, oo, ol)
    say("   rows past a document's end are never read into the result")
    K2, V2 = case.dK.clone(), case.dV.clone()
    rows = torch.arange(G, device="cuda")[None, :] >= dlens[:, None]          # [N][G]
    K2.masked_fill_(rows[:, None, :, None], 300.0)
    V2.masked_fill_(rows[:, None, :, None], -7e4)
    out2, lse2 = msa.msa_sparse_attend(cfg, case.dq, K2, V2, didx, case.dKl, case.dVl, pos0, dpos)
    torch.cuda.synchronize()
    assert torch.equal(out2.view(torch.int16), out.view(torch.int16)) and torch.equal(lse2, lse)


POOLED_RAGGED = {
    # name: (seed, N, Hkv, r, G, d, P, B, M, Lloc, base, k)
    "c8_short_docs": (71000, 40, 2, 4, 512, 128, 64, 2, 1, 50, 1e6, 16),
    "c16_d64": (72000, 23, 2, 2, 256, 64, 16, 1, 3, 37, 1e4, 5),
    "c32_whole_steps": (73000, 12, 2, 4, 256, 128, 8, 1, 2, 33, 1e6, 3),
    "c64_two_steps_d64": (74000, 9, 1, 2, 512, 64, 8, 2, 1, 0, 1e4, 4),
    "c2_r8": (75000, 19, 1, 8, 128, 128, 64, 1, 2, 64, 1e6, 19),
}


@pytest.mark.parametrize("name", list(POOLED_RAGGED))
def test_ragged_pooled_bank(name):
    seed, N, Hkv, r, G, d, P, B, M, Lloc, base, k = POOLED_RAGGED[name]
    say(f"ragged pooled case {name}: N={N} Hkv={Hkv} r={r} G={G} d={d} P={P} B={B} M={M} Lloc={Lloc} k={k}")
    case = Case(seed, N, Hkv, r, G, d, P, B, M, Lloc, base).to_device()
    Gp = G // P
    lens = make_lens(seed + 9, N, G, P)
    dlens = torch.from_numpy(lens.astype(np.int32)).cuda()
    cfg = case.cfg(doc_lens=dlens)
    Kbar, Vbar, plens = msa.msa_pool_kv(cfg, case.dK, case.dV)
    torch.cuda.synchronize()
    want_lens = (lens + P - 1) // P
    assert np.array_equal(plens.cpu().numpy().astype(np.int64), want_lens)
    nk, Kbar_o = check_pooled(Kbar, O.pool_rotated_keys(case.K, P, base, lens), "Kbar", 2e-5)
    nv, Vbar_o = check_pooled(Vbar, O.pool_values(case.V, P, lens), "Vbar", 2e-5)
    say(f"   pooled bank ok ({nk} + {nv} tie-adjacent roundings); entries per document {want_lens.min()}..{want_lens.max()}")

    rng = np.random.default_rng(seed)
    sel = np.stack([rng.permutation(N)[:k] for _ in range(B * M * Hkv)]).reshape(B, M, Hkv, k)
    sel[0, 0, 0, k // 2] = -1
    sel[0, 0, 0, 0] = 0                                             # the one-token document
    pos0 = k
    q_pos = np.array([[pos0 + (Lloc - 1 - (5 * m + b) % Lloc if Lloc else 0) for m in range(M)]
                      for b in range(B)])
    acfg = msa.MsaConfig(N, Gp, Gp, case.Hq, Hkv, d, base, bank_keys_rotated=1, doc_lens=plens)
    didx = torch.from_numpy(sel.astype(np.int32)).cuda()
    dpos = torch.from_numpy(q_pos.astype(np.int32)).cuda()
    oo, ol = O.sparse_attend(case.q, Kbar_o, Vbar_o, sel, case.Kl, case.Vl, pos0, q_pos, base, mem_rotated=True,
                             lens=want_lens)
    say("   sparse_attend over the oracle's pooled bank")
    dKo, dVo = dev(S.f64_to_bf16_bits(Kbar_o)), dev(S.f64_to_bf16_bits(Vbar_o))
    out, lse = msa.msa_sparse_attend(acfg, case.dq, dKo, dVo, didx, case.dKl, case.dVl, pos0, dpos)
    torch.cuda.synchronize()
    attend_err(out, lse, oo, ol)
    say("   chained: the GPU's own pooled bank and lengths")
    out2, lse2 = msa.msa_sparse_attend(acfg, case.dq, Kbar, Vbar, didx, case.dKl, case.dVl, pos0, dpos)
    torch.cuda.synchronize()
    attend_err(out2, lse2, oo, ol)


def test_ragged_full_lengths_are_the_uniform_bank():
    """doc_lens = G everywhere gives bit-identical results to no doc_lens at all, stage by stage; values
    outside [1, G] are clamped."""
    say("ragged case: all lengths G == no lengths; clamping")
    case = Case(76000, 50, 2, 4, 128, 128, 32, 2, 2, 40, 1e6).to_device()
    N, G, k = 50, 128, 5
    full = torch.full((N,), G, dtype=torch.int32, device="cuda")
    over = full.clone()
    over[::3] = G + 1000
    pos0 = G
    dpos = torch.full((2, 2), pos0 + 39, dtype=torch.int32, device="cuda")
    ref = None
    for lens_t in (None, full, over):
        cfg = case.cfg(doc_lens=lens_t)
        KR, inv = msa.msa_build_routing_keys(cfg, case.dK)
        idx, val = msa.msa_score_topk(cfg, case.dq, KR, inv, k)
        out, lse = msa.msa_sparse_attend(cfg, case.dq, case.dK, case.dV, idx, case.dKl, case.dVl, pos0, dpos)
        torch.cuda.synchronize()
        res = (KR.view(torch.int16), inv, idx, val, out.view(torch.int16), lse)
        if ref is None:
            ref = res
        else:
            for a, b in zip(ref, res):
                assert torch.equal(a, b)
    say("   lengths below 1 are read as 1")
    zero = torch.zeros((N,), dtype=torch.int32, device="cuda")
    one = torch.ones((N,), dtype=torch.int32, device="cuda")
    outs = []
    for lens_t in (zero, one):
        cfg = case.cfg(doc_lens=lens_t)
        KR, inv = msa.msa_build_routing_keys(cfg, case.dK)
        idx, val = msa.msa_score_topk(cfg, case.dq, KR, inv, k)
        out, lse = msa.msa_sparse_attend(cfg, case.dq, case.dK, case.dV, idx, case.dKl, case.dVl, pos0, dpos)
        torch.cuda.synchronize()
        outs.append((KR.view(torch.int16), inv, idx, val, out.view(torch.int16), lse))
    for a, b in zip(*outs):
        assert torch.equal(a, b)


def test_ragged_fetch_from_host_bank():
    """Tiered bank with lengths: only the rows a document holds travel, the staging bank carries the
    lengths, and attention over it equals attention over the device bank bit for bit."""
    say("ragged case: fetch from a pinned host bank (scope ALL)")
    seed, N, Hkv, r, G, d, P, B, M, Lloc, base, k = 77000, 40, 2, 4, 128, 128, 32, 2, 3, 20, 1e6, 4
    case = Case(seed, N, Hkv, r, G, d, P, B, M, Lloc, base).to_device()
    lens = make_lens(seed + 9, N, G, P)
    dlens = torch.from_numpy(lens.astype(np.int32)).cuda()
    cfg = case.cfg(select_scope=msa.MSA_SCOPE_ALL, doc_lens=dlens)
    rng = np.random.default_rng(seed)
    sel = np.stack([rng.permutation(N)[:k] for _ in range(B * M)]).reshape(B, M, 1, k)
    sel[0, 0, 0, 1] = -1
    sel[1, 2, 0, 0] = 0
    didx = torch.from_numpy(sel.astype(np.int32)).cuda()
    Kh = torch.empty(case.dK.shape, dtype=torch.bfloat16, pin_memory=True)
    Vh = torch.empty(case.dV.shape, dtype=torch.bfloat16, pin_memory=True)
    Kh.copy_(case.dK)
    Vh.copy_(case.dV)
    n_slots = msa.fetch_slots(cfg, B, M, k)
    Ks = torch.full((n_slots, Hkv, G, d), 9.0, dtype=torch.bfloat16, device="cuda")
    Vs = torch.full((n_slots, Hkv, G, d), 9.0, dtype=torch.bfloat16, device="cuda")
    Ks, Vs, idx_s, scfg = msa.msa_fetch_selected(cfg, Kh, Vh, didx, B, M, Ks, Vs)
    torch.cuda.synchronize()
    ls = scfg.doc_lens_tensor.cpu().numpy()
    slots = idx_s.cpu().numpy()
    for (b, m, _, j), doc in np.ndenumerate(sel):
        slot = (b * M + m) * k + j
        if doc < 0:
            assert slots[b, m, 0, j] == -1
            continue
        assert slots[b, m, 0, j] == slot and ls[slot] == lens[doc]
        n = int(lens[doc])
        assert torch.equal(Ks[slot, :, :n].view(torch.int16), case.dK[doc, :, :n].view(torch.int16))
        assert torch.equal(Vs[slot, :, :n].view(torch.int16), case.dV[doc, :, :n].view(torch.int16))
        assert torch.all(Ks[slot, :, n:] == 9.0) and torch.all(Vs[slot, :, n:] == 9.0)   # nothing else travelled
    pos0 = G
    q_pos = np.full((B, M), pos0 + Lloc - 1)
    dpos = torch.from_numpy(q_pos.astype(np.int32)).cuda()
    out_t, lse_t = msa.msa_sparse_attend(scfg, case.dq, Ks, Vs, idx_s, case.dKl, case.dVl, pos0, dpos)
    out_d, lse_d = msa.msa_sparse_attend(cfg, case.dq, case.dK, case.dV, didx, case.dKl, case.dVl, pos0, dpos)
    torch.cuda.synchronize()
    assert torch.equal(out_t.view(torch.int16), out_d.view(torch.int16)) and torch.equal(lse_t, lse_d)
    oo, ol = O.sparse_attend(case.q, case.K, case.V, sel, case.Kl, case.Vl, pos0, q_pos, base, lens=lens)
    attend_err(out_t, lse_t, oo, ol)


def test_length_zero_is_clamped_to_one_token():
    """The library has no empty documents: doc_lens values are clamped to [1, G] (a document holds at least one
    token), so an entry of 0 (or below, or above G) behaves exactly like 1 (or G) in every stage.  The oracle's
    lens = 0 (a document that never scores and contributes no rows) has no library counterpart; this pins the
    documented behaviour instead."""
    say("case doc_lens with 0, negative and too large entries: clamped to [1, G]")
    seed, N, Hkv, r, G, d, P, B, M, Lloc, base, k = 69000, 40, 2, 4, 128, 64, 32, 2, 1, 20, 1e4, 6
    case = Case(seed, N, Hkv, r, G, d, P, B, M, Lloc, base).to_device()
    lens = make_lens(seed + 9, N, G, P)
    raw = lens.copy()
    raw[[3, 11]] = 0
    raw[17] = -5
    raw[23] = G + 1000
    clamped = np.clip(raw, 1, G)
    res = []
    for l in (raw, clamped):
        dl = torch.from_numpy(l.astype(np.int32)).cuda()
        cfg = case.cfg(doc_lens=dl)
        KR, inv = msa.msa_build_routing_keys(cfg, case.dK)
        idx, val = msa.msa_score_topk(cfg, case.dq, KR, inv, k)
        sel = idx.clone()
        sel[0, 0, 0, :4] = torch.tensor([3, 11, 17, 23], dtype=torch.int32)     # attend the clamped documents
        dpos = torch.full((B, M), G + Lloc - 1, dtype=torch.int32, device="cuda")
        out, lse = msa.msa_sparse_attend(cfg, case.dq, case.dK, case.dV, sel, case.dKl, case.dVl, G, dpos)
        Kbar, Vbar, plens = msa.msa_pool_kv(cfg, case.dK, case.dV)
        torch.cuda.synchronize()
        res.append((KR, inv, idx, val, out.view(torch.int16), lse, Kbar.view(torch.int16), Vbar.view(torch.int16), plens))
    for a, b in zip(*res):
        assert torch.equal(a, b)
    # and the clamped reading is the oracle's reading of those lengths
    oo, ol = O.sparse_attend(case.q, case.K, case.V, sel.cpu().numpy().astype(np.int64), case.Kl, case.Vl, G,
                             np.full((B, M), G + Lloc - 1), base, lens=clamped)
    attend_err(out, lse, oo, ol)
