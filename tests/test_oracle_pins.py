"""Pins of the CPU oracle against things other than itself: brute force, library routines, closed
forms, invariants, and the one number the paper prints for this path.  CPU only."""
import os

import numpy as np
import pytest
from scipy.special import softmax as sp_softmax

import msa_synth as S
from oracle import msa_oracle as O

HERE = os.path.dirname(os.path.abspath(__file__))


def _bank(seed, N, Hkv, G, d):
    return S.normal_bf16(seed, (N, Hkv, G, d))[1]


def _tiny(seed=11, N=6, Hkv=2, r=2, G=16, d=8, B=2, M=2, Lloc=5):
    K = _bank(seed, N, Hkv, G, d)
    V = _bank(seed + 1, N, Hkv, G, d)
    q = S.normal_bf16(seed + 2, (B, M, Hkv * r, d))[1]
    Kl = S.normal_bf16(seed + 3, (B, Hkv, Lloc, d))[1]
    Vl = S.normal_bf16(seed + 4, (B, Hkv, Lloc, d))[1]
    return K, V, q, Kl, Vl


# ------------------------------------------------------------------------------------------
# bf16 rounding against PyTorch's CPU cast (an independent implementation of RNE)
# ------------------------------------------------------------------------------------------
def test_bf16_round_matches_torch_cast():
    import torch
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(20000), rng.standard_normal(2000) * 1e-3,
                        np.array([0.0, 1.0, 1.00390625, 1.01171875, -1.00390625, 255.5, 3e-40])])
    want = torch.tensor(x, dtype=torch.float64).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(O.bf16_round(x), want)


def test_bf16_round_ties_to_even():
    # 1 + 2^-8 is exactly halfway between 1 and 1 + 2^-7 -> even mantissa (1.0);
    # 1 + 3*2^-8 is halfway between 1+2^-7 and 1+2^-6 -> 1 + 2^-6
    assert O.bf16_round(1 + 2.0 ** -8) == 1.0
    assert O.bf16_round(1 + 3 * 2.0 ** -8) == 1 + 2.0 ** -6


# ------------------------------------------------------------------------------------------
# pooling closed forms
# ------------------------------------------------------------------------------------------
def test_pool_closed_forms():
    N, Hkv, G, d, P = 3, 2, 8, 4, 4
    K = np.zeros((N, Hkv, G, d))
    row = np.array([1.0, -2.0, 0.5, 4.0])
    K[1, 0, 0:4] = row                      # constant chunk -> that row
    K[2, 1, 5, 2] = 1.0                     # one-hot token -> 1/P
    K[0, 1, 0:2] = 2.0                      # halves a,b -> (a+b)/2
    K[0, 1, 2:4] = 6.0
    R = O.pool_chunks(K, P)
    assert R.shape == (Hkv, N * 2, d)
    assert np.array_equal(R[0, 1 * 2 + 0], row)
    assert R[1, 2 * 2 + 1, 2] == 0.25 and R[1, 2 * 2 + 1].sum() == 0.25
    assert np.array_equal(R[1, 0], np.full(d, 4.0))
    assert np.count_nonzero(R) == d + 1 + d


def test_pool_matches_reshape_mean_and_layout():
    K = _bank(3, 5, 2, 32, 8)
    R = O.pool_chunks(K, 8)
    want = K.reshape(5, 2, 4, 8, 8).mean(axis=3).transpose(1, 0, 2, 3).reshape(2, 20, 8)
    assert np.allclose(R, want, rtol=0, atol=1e-15)


def test_routing_keys_rounding_and_inv_norm():
    import torch
    K = _bank(4, 4, 2, 16, 8)
    KRb, inv = O.routing_keys(K, 4)
    exact = O.pool_chunks(K, 4)
    assert np.all(np.abs(KRb - exact) <= np.abs(exact) * 2.0 ** -8 + 1e-300)   # within half an ulp
    assert np.array_equal(torch.from_numpy(KRb).to(torch.bfloat16).to(torch.float64).numpy(), KRb)   # representable (PyTorch's cast)
    assert np.allclose(inv * np.linalg.norm(KRb, axis=-1), 1.0, rtol=1e-14)
    Kz = np.zeros((1, 1, 4, 4))
    assert O.routing_keys(Kz, 4)[1][0, 0] == 1.0 / O.EPS_NORM                  # zero key: guarded


# ------------------------------------------------------------------------------------------
# scoring (Eq. 2) closed forms
# ------------------------------------------------------------------------------------------
def test_cosine_range_scale_invariance_and_zero():
    rng = np.random.default_rng(1)
    x = rng.standard_normal(16)
    Y = rng.standard_normal((50, 16))
    c = O.similarity(x, Y)
    assert np.all(np.abs(c) <= 1 + 1e-15)
    scale = rng.uniform(0.1, 10, size=50)[:, None]
    assert np.allclose(O.similarity(x, Y * scale), c, rtol=1e-13, atol=1e-15)
    assert np.allclose(O.similarity(x, Y, "dot"), Y @ x)
    assert np.all(O.similarity(np.zeros(16), Y) == 0.0)
    assert O.similarity(x, np.zeros((1, 16)))[0] == 0.0
    assert np.isclose(O.similarity(x, x[None] * 3.0)[0], 1.0, rtol=1e-15)
    assert np.isclose(O.similarity(x, -x[None])[0], -1.0, rtol=1e-15)


def test_planted_chunk_scores_norm_of_mean_unit_query_and_ranks_first():
    rng = np.random.default_rng(2)
    Hkv, r, d, NC = 2, 3, 16, 40
    q = rng.standard_normal((1, 1, Hkv * r, d))
    KR = rng.standard_normal((Hkv, NC, d))
    qhat = q[0, 0] / np.linalg.norm(q[0, 0], axis=-1, keepdims=True)
    for g in range(Hkv):
        u = qhat[g * r:(g + 1) * r].mean(axis=0)
        KR[g, 7 + g] = 5.0 * u                  # any positive multiple of the mean unit query
    Sc = O.chunk_scores(q, KR)
    for g in range(Hkv):
        u = qhat[g * r:(g + 1) * r].mean(axis=0)
        assert np.isclose(Sc[0, 0, g, 7 + g], np.linalg.norm(u), rtol=1e-13)
        assert Sc[0, 0, g].argmax() == 7 + g    # Cauchy-Schwarz: nothing can beat it


def test_head_mean_then_max_order_and_scopes():
    rng = np.random.default_rng(3)
    B, M, Hkv, r, d, N, C = 2, 3, 2, 2, 8, 5, 4
    q = rng.standard_normal((B, M, Hkv * r, d))
    KR = rng.standard_normal((Hkv, N * C, d))
    Sg = O.chunk_scores(q, KR)                                    # per group
    Sa = O.chunk_scores(q, KR, select_scope="all")                # literal Eq. 2 head mean
    assert Sg.shape == (B, M, Hkv, N * C) and Sa.shape == (B, M, 1, N * C)
    assert np.allclose(Sa[:, :, 0], Sg.mean(axis=2), rtol=1e-13)  # all-head mean = mean of groups
    # explicit per-head loop (different code path: scalar cosine per pair)
    b, m, g, c = 1, 2, 1, 13
    want = np.mean([q[b, m, h] @ KR[g, c] / (np.linalg.norm(q[b, m, h]) * np.linalg.norm(KR[g, c]))
                    for h in (2, 3)])
    assert np.isclose(Sg[b, m, g, c], want, rtol=1e-13)
    St = O.chunk_scores(q, KR, select_scope="all", token_pool=True)
    assert St.shape == (B, 1, 1, N * C)
    assert np.array_equal(St[:, 0], Sa.max(axis=1))
    # document score is the max over the document's own C chunks
    s = O.doc_scores(Sg, C)
    assert s.shape == (B, M, Hkv, N)
    assert s[0, 1, 1, 3] == Sg[0, 1, 1, 12:16].max()
    # the mean does not commute with the max: head mean must be taken at chunk level first
    per_head_docmax = np.stack([O.doc_scores(O.chunk_scores(q[:, :, h:h + 1], KR[h // r:h // r + 1]), C)
                                for h in range(Hkv * r)], axis=2)[:, :, :, 0]
    wrong = per_head_docmax.reshape(B, M, Hkv, r, N).mean(axis=3)
    assert np.all(s <= wrong + 1e-15) and np.any(s < wrong - 1e-6)


# ------------------------------------------------------------------------------------------
# top-k: ordering, ties, shard merge
# ------------------------------------------------------------------------------------------
def test_topk_order_and_ties():
    s = np.array([0.5, 0.9, 0.9, 0.1, 0.5, 0.9])
    idx, val = O.topk_docs(s, 4)
    assert idx.tolist() == [1, 2, 5, 0] and val.tolist() == [0.9, 0.9, 0.9, 0.5]
    idx, _ = O.topk_docs(np.zeros(7), 3)
    assert idx.tolist() == [0, 1, 2]
    rng = np.random.default_rng(4)
    s = rng.standard_normal((3, 2, 50))
    idx, val = O.topk_docs(s, 5)
    # brute force: k-th largest by repeated argmax
    for a in range(3):
        for b in range(2):
            row = s[a, b].copy()
            for j in range(5):
                t = int(row.argmax())
                assert idx[a, b, j] == t and val[a, b, j] == s[a, b, t]
                row[t] = -np.inf


def test_duplicate_documents_lowest_slot_first():
    K = _bank(5, 8, 2, 8, 8)
    K[6] = K[2]                                  # duplicate document at slots 2 < 6
    q = S.normal_bf16(6, (1, 1, 4, 8))[1]
    KRb, _ = O.routing_keys(K, 4)
    idx, val, s = O.score_topk(q, KRb, 2, 8)
    assert np.array_equal(s[..., 2], s[..., 6])
    for g in range(2):
        order = idx[0, 0, g].tolist()
        assert order.index(2) + 1 == order.index(6)


def test_shard_merge_equals_global_topk():
    rng = np.random.default_rng(5)
    s = rng.standard_normal(1000)
    s[[10, 500, 900]] = s.max() + 1.0            # a three-way tie across shards at the top
    k = 16
    gi, gv = O.topk_docs(s, k)
    for bounds in ([0, 333, 700, 1000], [0, 20, 21, 999, 1000]):
        cands = []
        for a, b in zip(bounds[:-1], bounds[1:]):
            li, lv = O.topk_docs(s[a:b], min(k, b - a))
            cands.append((li + a, lv))
        mi, mv = O.merge_shard_topk(cands, k)
        assert np.array_equal(mi, gi) and np.array_equal(mv, gv)


# ------------------------------------------------------------------------------------------
# RoPE identities
# ------------------------------------------------------------------------------------------
def test_rope_identities():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((5, 16))
    y = rng.standard_normal((5, 16))
    assert np.array_equal(O.rope(x, np.zeros(5), 1e4), x)
    for base in (1e4, 1e6):
        p = np.array([1, 7, 100, 511, 4000])
        assert np.allclose(np.linalg.norm(O.rope(x, p, base), axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-13)
        a = (O.rope(x, p + 37, base) * O.rope(y, p, base)).sum(-1)
        b = (O.rope(x, np.full(5, 37), base) * y).sum(-1)
        assert np.allclose(a, b, rtol=1e-10, atol=1e-10)
    # d = 2: a plain rotation of the plane by p radians (theta_0 = 1 for any base)
    v = O.rope(np.array([1.0, 0.0]), 0.5, 123.0)
    assert np.allclose(v, [np.cos(0.5), np.sin(0.5)], rtol=1e-15)
    v = O.rope(np.array([0.0, 1.0]), 0.5, 123.0)
    assert np.allclose(v, [-np.sin(0.5), np.cos(0.5)], rtol=1e-15)
    # frequencies and pairing: d = 4, base 100 -> theta = [1, 0.1]; pairs (0,2) and (1,3)
    v = O.rope(np.array([1.0, 1.0, 0.0, 0.0]), 3.0, 100.0)
    assert np.allclose(v, [np.cos(3.0), np.cos(0.3), np.sin(3.0), np.sin(0.3)], rtol=1e-15)


def test_rope_matches_complex_multiplication():
    rng = np.random.default_rng(7)
    d, base = 32, 1e6
    x = rng.standard_normal((9, d))
    p = rng.integers(0, 3000, size=9)
    z = (x[:, :d // 2] + 1j * x[:, d // 2:]) * np.exp(1j * p[:, None] * base ** (-np.arange(d // 2) / (d / 2)))
    assert np.allclose(O.rope(x, p, base), np.concatenate([z.real, z.imag], -1), rtol=1e-12, atol=1e-12)


# ------------------------------------------------------------------------------------------
# attention (Eq. 3-4): brute force, library reduction, invariants
# ------------------------------------------------------------------------------------------
def _dense_bruteforce(q, K, V, Kl, Vl, pos0, q_pos, base):
    """Separate, loop-only dense attention over EVERY document (positions restart per document)
    followed by the visible local tokens.  Scalar arithmetic; shares nothing with the oracle."""
    import math
    B, M, Hq, d = q.shape
    N, Hkv, G, _ = K.shape
    r = Hq // Hkv
    half = d // 2

    def rot(vec, p):
        out = [0.0] * d
        for u in range(half):
            ang = p * base ** (-2.0 * u / d)
            out[u] = vec[u] * math.cos(ang) - vec[u + half] * math.sin(ang)
            out[u + half] = vec[u + half] * math.cos(ang) + vec[u] * math.sin(ang)
        return out

    res = np.zeros((B, M, Hq, d))
    for b in range(B):
        for m in range(M):
            for h in range(Hq):
                g = h // r
                qt = rot(list(q[b, m, h]), q_pos[b, m])
                zs, vs = [], []
                for i in range(N):
                    for p in range(G):
                        kt = rot(list(K[i, g, p]), p)
                        zs.append(sum(a * c for a, c in zip(qt, kt)) / math.sqrt(d))
                        vs.append(V[i, g, p])
                for t in range(Kl.shape[2]):
                    if pos0 + t <= q_pos[b, m]:
                        kt = rot(list(Kl[b, g, t]), pos0 + t)
                        zs.append(sum(a * c for a, c in zip(qt, kt)) / math.sqrt(d))
                        vs.append(Vl[b, g, t])
                zmax = max(zs)
                ws = [math.exp(z - zmax) for z in zs]
                tot = sum(ws)
                res[b, m, h] = sum((w / tot) * v for w, v in zip(ws, vs))
    return res


def test_full_selection_equals_dense_bruteforce():
    K, V, q, Kl, Vl = _tiny()
    B, M = q.shape[:2]
    N, Hkv, G, d = K.shape
    pos0 = G
    q_pos = np.array([[pos0 + 2, pos0 + 4], [pos0 + 0, pos0 + 4]])          # causal masks differ
    KRb, _ = O.routing_keys(K, 4)
    idx, _, _ = O.score_topk(q, KRb, G // 4, N)                              # k = N: everything selected
    assert sorted(idx[0, 0, 0].tolist()) == list(range(N))
    out, lse = O.sparse_attend(q, K, V, idx, Kl, Vl, pos0, q_pos, 1e4)
    want = _dense_bruteforce(q, K, V, Kl, Vl, pos0, q_pos, 1e4)
    assert np.allclose(out, want, rtol=1e-11, atol=1e-12)


def test_reduction_to_library_softmax_attention():
    """G = 1, no local context, q_pos = 0: RoPE is the identity everywhere and the path is plain
    softmax(QK^T/sqrt(d))V over the selected one-token documents."""
    import torch
    N, Hkv, r, d, k = 12, 2, 2, 16, 5
    K = _bank(21, N, Hkv, 1, d)
    V = _bank(22, N, Hkv, 1, d)
    q = S.normal_bf16(23, (1, 1, Hkv * r, d))[1]
    rng = np.random.default_rng(8)
    idx = np.stack([rng.permutation(N)[:k] for _ in range(Hkv)])[None, None]
    out, lse = O.sparse_attend(q, K, V, idx, None, None, 0, np.zeros((1, 1), dtype=int), 1e6)
    for h in range(Hkv * r):
        g = h // r
        Ks, Vs = K[idx[0, 0, g], g, 0], V[idx[0, 0, g], g, 0]
        z = Ks @ q[0, 0, h] / np.sqrt(d)
        assert np.allclose(out[0, 0, h], sp_softmax(z) @ Vs, rtol=1e-13, atol=1e-14)
        assert np.isclose(lse[0, 0, h], np.log(np.exp(z).sum()), rtol=1e-13)
        t = torch.nn.functional.scaled_dot_product_attention(
            torch.tensor(q[0, 0, h])[None, None], torch.tensor(Ks)[None], torch.tensor(Vs)[None])
        assert np.allclose(out[0, 0, h], t[0, 0].numpy(), rtol=1e-12, atol=1e-13)


def test_softmax_invariants():
    K, V, q, Kl, Vl = _tiny(seed=31)
    N, Hkv, G, d = K.shape
    B, M = q.shape[:2]
    idx = np.tile(np.array([1, 4])[None, None, None], (B, M, Hkv, 1))
    pos0, q_pos = G, np.full((B, M), G + 4)
    # all value rows equal v -> out = v
    v = np.arange(d, dtype=float)
    out, _ = O.sparse_attend(q, K, np.broadcast_to(v, V.shape), idx, Kl, np.broadcast_to(v, Vl.shape),
                             pos0, q_pos, 1e4)
    assert np.allclose(out, v, rtol=1e-13, atol=1e-13)
    # q = 0 -> plain mean of the visible value rows; lse = log(count)
    out, lse = O.sparse_attend(np.zeros_like(q), K, V, idx, Kl, Vl, pos0, q_pos, 1e4)
    for g in range(Hkv):
        mean = (V[1, g].sum(0) + V[4, g].sum(0) + Vl[0, g].sum(0)) / (2 * G + Kl.shape[2])
        assert np.allclose(out[0, 0, 2 * g], mean, rtol=1e-13, atol=1e-14)
    assert np.allclose(lse, np.log(2 * G + Kl.shape[2]), rtol=1e-13)
    # a single visible key -> its value row, whatever the query
    one = np.full((B, M, Hkv, 1), -1)
    out, _ = O.sparse_attend(q, K, V, one, Kl, Vl, pos0, np.full((B, M), pos0), 1e4)
    assert np.allclose(out[1, 0, 3], Vl[1, 1, 0], rtol=1e-14)
    # nothing visible -> zeros and -inf
    out, lse = O.sparse_attend(q, K, V, one, None, None, pos0, q_pos, 1e4)
    assert np.all(out == 0) and np.all(np.isneginf(lse))
    # weights: non-negative, sum to one (recomputed from lse)
    keys, vals = O.assemble_context(K, V, [1, 4], 0, Kl[0, 0], Vl[0, 0], pos0, pos0 + 4, 1e4)
    qt = O.rope(q[0, 0, 0], np.float64(pos0 + 4), 1e4)
    o, l = O.softmax_attend(qt, keys, vals)
    w = np.exp(keys @ qt / np.sqrt(d) - l)
    assert np.all(w >= 0) and abs(w.sum() - 1) < 1e-12 and np.allclose(w @ vals, o, rtol=1e-12)


def test_causal_visibility_of_local_tokens():
    K, V, q, Kl, Vl = _tiny(seed=41, Lloc=6)
    N, Hkv, G, d = K.shape
    B, M = q.shape[:2]
    idx = np.full((B, M, Hkv, 1), 2)
    pos0 = 50
    q_pos = np.array([[pos0 + 1, pos0 + 5], [pos0 + 3, pos0 + 3]])
    out, _ = O.sparse_attend(q, K, V, idx, Kl, Vl, pos0, q_pos, 1e4)
    # truncating the local cache to the visible prefix must not change anything
    for b in range(B):
        for m in range(M):
            n_vis = q_pos[b, m] - pos0 + 1
            o2, _ = O.sparse_attend(q[b:b + 1, m:m + 1], K, V, idx[b:b + 1, m:m + 1],
                                    Kl[b:b + 1, :, :n_vis], Vl[b:b + 1, :, :n_vis], pos0,
                                    q_pos[b:b + 1, m:m + 1], 1e4)
            assert np.allclose(o2[0, 0], out[b, m], rtol=1e-13, atol=1e-14)
    # and making a hidden token's key/value huge changes nothing
    Kl2, Vl2 = Kl.copy(), Vl.copy()
    Kl2[0, :, 2:] = 1e3
    Vl2[0, :, 2:] = 1e3
    o3, _ = O.sparse_attend(q, K, V, idx, Kl2, Vl2, pos0, q_pos, 1e4)
    assert np.array_equal(o3[0, 0], out[0, 0])


def test_docwise_rope_permutation_invariant():
    """Section 3.2.2: a document's keys do not depend on where it sits in the bank."""
    K, V, q, Kl, Vl = _tiny(seed=51, N=7)
    N, Hkv, G, d = K.shape
    B, M = q.shape[:2]
    rng = np.random.default_rng(9)
    idx = np.stack([rng.permutation(N)[:3] for _ in range(B * M * Hkv)]).reshape(B, M, Hkv, 3)
    pos0, q_pos = G, np.full((B, M), G + 4)
    out, lse = O.sparse_attend(q, K, V, idx, Kl, Vl, pos0, q_pos, 1e6)
    perm = rng.permutation(N)                         # new slot s holds old document perm[s]
    inv = np.argsort(perm)
    out2, lse2 = O.sparse_attend(q, K[perm], V[perm], inv[idx], Kl, Vl, pos0, q_pos, 1e6)
    assert np.allclose(out2, out, rtol=1e-13, atol=1e-13) and np.allclose(lse2, lse, rtol=1e-13)
    out3, _ = O.sparse_attend(q, K, V, idx[..., ::-1], Kl, Vl, pos0, q_pos, 1e6)   # order of ids
    assert np.allclose(out3, out, rtol=1e-13, atol=1e-13)
    # the choice of local_pos0 shifts q and local keys together: only relative positions to the
    # local context matter, but distances to memory tokens change -> outputs differ in general;
    # with NO memory selected the output is exactly shift-invariant.
    none = np.full((B, M, Hkv, 1), -1)
    a, _ = O.sparse_attend(q, K, V, none, Kl, Vl, G, np.full((B, M), G + 4), 1e6)
    b, _ = O.sparse_attend(q, K, V, none, Kl, Vl, 3, np.full((B, M), 3 + 4), 1e6)
    assert np.allclose(a, b, rtol=1e-10, atol=1e-11)


def test_lse_merge_associativity():
    K, V, q, Kl, Vl = _tiny(seed=61)
    keys, vals = O.assemble_context(K, V, [0, 3, 5], 1, Kl[0, 1], Vl[0, 1], 16, 20, 1e4)
    qt = O.rope(q[0, 0, 2], np.float64(20), 1e4)
    full, lse = O.softmax_attend(qt, keys, vals)
    rng = np.random.default_rng(10)
    for cuts in ([0, 1, 2, 30, keys.shape[0]], [0, 17, keys.shape[0]], [0, keys.shape[0]]):
        parts = [O.softmax_attend(qt, keys[a:b], vals[a:b]) for a, b in zip(cuts[:-1], cuts[1:])]
        parts.insert(1, O.softmax_attend(qt, keys[:0], vals[:0]))           # an empty split
        rng.shuffle(parts)
        o, l = O.merge_partials(parts)
        assert np.allclose(o, full, rtol=1e-13, atol=1e-14) and np.isclose(l, lse, rtol=1e-14)


def test_selected_documents_dominate_when_planted():
    """End to end on a tiny case: a document whose keys align with the query is selected and its
    value dominates the output."""
    N, Hkv, r, G, d, P = 16, 1, 2, 8, 16, 4
    K = 0.1 * _bank(71, N, Hkv, G, d)
    V = _bank(72, N, Hkv, G, d)
    q = S.normal_bf16(73, (1, 1, r, d))[1]
    K[9, 0, :, :] = 8.0 * q[0, 0].mean(axis=0)       # un-rotated keys drive the routing index
    KRb, _ = O.routing_keys(K, P)
    idx, val, s = O.score_topk(q, KRb, G // P, 2)
    assert idx[0, 0, 0, 0] == 9 and val[0, 0, 0, 0] > 0.5


# ------------------------------------------------------------------------------------------
# pooled K-bar / V-bar (Eq. 3 as the paper writes it)
# ------------------------------------------------------------------------------------------
def test_pooled_bank_reduces_to_unpooled_path_when_P_is_1():
    """With P = 1 the pooled, position-encoded bank is just RoPE(K) and V: attention over it with
    mem_rotated=True must equal the default path (raw bank, rotation in the gather)."""
    K, V, q, Kl, Vl = _tiny(seed=81)
    N, Hkv, G, d = K.shape
    B, M = q.shape[:2]
    rng = np.random.default_rng(11)
    idx = np.stack([rng.permutation(N)[:3] for _ in range(B * M * Hkv)]).reshape(B, M, Hkv, 3)
    pos0, q_pos = G, np.full((B, M), G + 4)
    want, lw = O.sparse_attend(q, K, V, idx, Kl, Vl, pos0, q_pos, 1e4)
    Kbar, Vbar = O.pool_rotated_keys(K, 1, 1e4), O.pool_values(V, 1)
    got, lg = O.sparse_attend(q, Kbar, Vbar, idx, Kl, Vl, pos0, q_pos, 1e4, mem_rotated=True)
    assert np.allclose(got, want, rtol=1e-13, atol=1e-13) and np.allclose(lg, lw, rtol=1e-13)


def test_pooled_bank_closed_forms():
    N, Hkv, G, d, P = 2, 1, 8, 4, 4
    K = np.zeros((N, Hkv, G, d))
    V = np.zeros((N, Hkv, G, d))
    K[0, 0, 0] = [1.0, 0.0, 0.0, 0.0]            # position 0: identity rotation
    K[1, 0, 5] = [1.0, 0.0, 0.0, 0.0]            # position 5: pair (0, 2) rotated by 5 rad (theta_0 = 1)
    V[1, 0, 4:8] = [2.0, 4.0, 6.0, 8.0]
    Kb, Vb = O.pool_rotated_keys(K, P, 100.0), O.pool_values(V, P)
    assert Kb.shape == (N, Hkv, 2, d) and Vb.shape == (N, Hkv, 2, d)
    assert np.allclose(Kb[0, 0, 0], [0.25, 0, 0, 0], atol=1e-16)
    assert np.allclose(Kb[1, 0, 1], [np.cos(5.0) / 4, 0, np.sin(5.0) / 4, 0], rtol=1e-15)
    assert np.array_equal(Vb[1, 0, 1], [2.0, 4.0, 6.0, 8.0]) and np.count_nonzero(Vb) == 4
    # pooling commutes with nothing position-dependent: constant K over a chunk is NOT kept constant
    K2 = np.ones((1, 1, 8, 4))
    assert not np.allclose(O.pool_rotated_keys(K2, 4, 100.0)[0, 0, 0], 1.0)
    # context length of the pooled variant (paper, Section 5.1): M + k G / P keys
    K3, V3, q3, Kl3, Vl3 = _tiny(seed=91, G=16, Lloc=5)
    keys, vals = O.assemble_context(O.pool_rotated_keys(K3, 4, 1e4), O.pool_values(V3, 4), [0, 2, 5], 0,
                                    Kl3[0, 0], Vl3[0, 0], 3, 3 + 4, 1e4, mem_rotated=True)
    assert keys.shape[0] == 5 + 3 * 16 // 4


# ------------------------------------------------------------------------------------------
# the number the paper prints (Section 3.4.2)
# ------------------------------------------------------------------------------------------
def test_paper_memory_estimate():
    line = [l for l in open(os.path.join(HERE, "golden", "paper_memory_estimate.txt")) if not l.startswith("#")][0]
    tokens, P, heads, d, layers, bpe, total_gb, routing_gb = (int(x) for x in line.split())
    total = O.pooled_bank_bytes(tokens, P, heads, d, layers, bpe, tensors=3)
    routing = O.pooled_bank_bytes(tokens, P, heads, d, layers, bpe, tensors=1)
    assert total == 3 * routing
    assert round(total / 2 ** 30) == total_gb            # "approximately 169GB" (168.75 GiB)
    assert round(routing / 2 ** 30) == routing_gb        # "~56GB" (56.25 GiB)
    assert total / 2 ** 30 == 168.75 and routing / 2 ** 30 == 56.25


# ------------------------------------------------------------------------------------------
# the synthetic-input generator (host side): determinism, slicing, distribution
# ------------------------------------------------------------------------------------------
def test_synth_slices_and_distribution():
    bits, val = S.normal_bf16(1234, (3, 2, 8, 4))
    b2, v2 = S.doc_slice(1234, 2, 8, 4, 1)
    assert np.array_equal(bits[1], b2) and np.array_equal(val[1], v2)
    assert np.array_equal(S.normal_bf16_bits(1234, 37, 50), bits.reshape(-1)[37:87])
    _, big = S.normal_bf16(99, (200000,))
    assert abs(big.mean()) < 0.01 and abs(big.std() - 1.0) < 0.01
    assert not np.array_equal(S.normal_bf16_bits(1, 0, 64), S.normal_bf16_bits(2, 0, 64))
    t = S.bf16_bits_to_f64(S.quantile_table())
    assert np.all(np.diff(t) >= 0) and t[0] < -4 and t[-1] > 4 and np.allclose(t, -t[::-1])


# --------------------------------------------------------------------------------------------
# documents of different lengths (lens): tail chunks, chunks that do not exist, shorter contexts
# --------------------------------------------------------------------------------------------
def _ragged_case(seed=900):
    rng = np.random.default_rng(seed)
    N, Hkv, r, G, d, P = 7, 2, 2, 32, 8, 8
    K = rng.standard_normal((N, Hkv, G, d))
    V = rng.standard_normal((N, Hkv, G, d))
    q = rng.standard_normal((2, 3, Hkv * r, d))
    lens = np.array([32, 5, 0, 17, 8, 31, 24])
    return N, Hkv, r, G, d, P, K, V, q, lens


def test_ragged_full_lengths_reduce_to_uniform():
    N, Hkv, r, G, d, P, K, V, q, _ = _ragged_case()
    full = np.full(N, G)
    a, ai = O.routing_keys(K, P)
    b, bi = O.routing_keys(K, P, full)
    assert np.array_equal(a, b) and np.array_equal(ai, bi)
    assert np.all(O.chunk_valid(full, G, P))
    assert np.array_equal(O.pool_rotated_keys(K, P, 1e4), O.pool_rotated_keys(K, P, 1e4, full))
    assert np.array_equal(O.pool_values(V, P), O.pool_values(V, P, full))
    idx = np.tile(np.arange(3), (2, 3, Hkv, 1))
    qp = np.full((2, 3), G + 4)
    o1, l1 = O.sparse_attend(q, K, V, idx, None, None, G, qp, 1e4)
    o2, l2 = O.sparse_attend(q, K, V, idx, None, None, G, qp, 1e4, lens=full)
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)


def test_ragged_chunks_closed_forms():
    N, Hkv, r, G, d, P, K, V, q, lens = _ragged_case()
    C = G // P
    valid = O.chunk_valid(lens, G, P)
    assert valid.reshape(N, C).sum(axis=1).tolist() == [-(-int(n) // P) for n in lens]     # ceil(len / P) chunks
    # rows that are constant inside a document: every existing chunk, the short tail included, is that row
    Kc = np.broadcast_to(K[:, :, :1, :], K.shape)
    pooled = O.pool_chunks(Kc, P, lens)
    for i in range(N):
        for j in range(C):
            want = Kc[i, :, 0, :] if j * P < lens[i] else 0.0
            assert np.allclose(pooled[:, i * C + j, :], want, rtol=1e-15, atol=0)
    # the tail chunk is the mean over the tokens that exist, not over P
    i, j = 3, 2                                                                           # lens[3] = 17: one token in chunk 2
    assert np.allclose(O.pool_chunks(K, P, lens)[:, i * C + j, :], K[i, :, 16, :], rtol=1e-15)
    assert np.allclose(O.pool_values(V, P, lens)[i, :, j, :], V[i, :, 16, :], rtol=1e-15)
    assert np.allclose(O.pool_rotated_keys(K, P, 1e4, lens)[i, :, j, :], O.rope(K[i, :, 16, :], 16, 1e4), rtol=1e-13)
    KRb, inv = O.routing_keys(K, P, lens)
    assert np.all(inv[:, ~valid] == -1.0) and np.all(inv[:, valid] > 0)
    # chunks that do not exist score -inf; the empty document ranks last and a full ranking lists it last
    Sc = O.chunk_scores(q, KRb, valid=valid)
    assert np.all(np.isneginf(Sc[..., ~valid])) and np.all(np.isfinite(Sc[..., valid]))
    idx, val, s = O.score_topk(q, KRb, C, N, valid=valid)
    assert np.all(idx[..., -1] == 2) and np.all(np.isneginf(val[..., -1]))
    # scores of existing chunks do not depend on what lies past the end of a document
    K2 = K.copy()
    for i in range(N):
        K2[i, :, lens[i]:, :] = 99.0
    KRb2, inv2 = O.routing_keys(K2, P, lens)
    assert np.array_equal(KRb2[:, valid], KRb[:, valid]) and np.array_equal(inv2, inv)


def test_ragged_attention_is_attention_over_the_existing_tokens():
    """k = N and lens given: plain softmax attention (PyTorch SDPA, float64) over the concatenation of the
    rows every document really has, each rotated by its in-document position with the complex form of RoPE
    written out here, plus the visible local rows."""
    import torch
    N, Hkv, r, G, d, P, K, V, q, lens = _ragged_case(901)
    base, Lloc, pos0 = 1e4, 6, 11
    rng = np.random.default_rng(5)
    Kl = rng.standard_normal((2, Hkv, Lloc, d))
    Vl = rng.standard_normal((2, Hkv, Lloc, d))
    q_pos = np.array([[pos0 + 5, pos0 + 2, pos0 - 1], [pos0, pos0 + 3, pos0 + 5]])
    idx = np.tile(np.arange(N), (2, 3, Hkv, 1))
    out, lse = O.sparse_attend(q, K, V, idx, Kl, Vl, pos0, q_pos, base, lens=lens)

    def rot(x, p):                                                   # (x_u + i x_{u+d/2}) * exp(i p theta_u)
        th = base ** (-2.0 * np.arange(d // 2) / d)
        z = (x[..., :d // 2] + 1j * x[..., d // 2:]) * np.exp(1j * np.asarray(p)[..., None] * th)
        return np.concatenate([z.real, z.imag], axis=-1)
    for b in range(2):
        for m in range(3):
            for h in range(Hkv * r):
                g = h // r
                ks = [rot(K[i, g, :lens[i]], np.arange(lens[i])) for i in range(N)]
                vs = [V[i, g, :lens[i]] for i in range(N)]
                nv = int(np.clip(q_pos[b, m] - pos0 + 1, 0, Lloc))
                ks.append(rot(Kl[b, g, :nv], pos0 + np.arange(nv)))
                vs.append(Vl[b, g, :nv])
                kk, vv = np.concatenate(ks), np.concatenate(vs)
                assert kk.shape[0] == lens.sum() + nv
                qq = rot(q[b, m, h], q_pos[b, m])
                want = torch.nn.functional.scaled_dot_product_attention(
                    torch.from_numpy(qq)[None, None], torch.from_numpy(kk)[None], torch.from_numpy(vv)[None])[0, 0].numpy()
                assert np.allclose(out[b, m, h], want, rtol=1e-12, atol=1e-13)


def test_ragged_whole_chunk_lengths_equal_a_shorter_uniform_bank():
    """Documents that all have the same length n < G (a multiple of P): the existing chunks and the attention
    are those of the uniform bank cut to n tokens."""
    N, Hkv, r, G, d, P, K, V, q, _ = _ragged_case(902)
    n = 16
    lens = np.full(N, n)
    valid = O.chunk_valid(lens, G, P)
    KRb, inv = O.routing_keys(K, P, lens)
    KRs, invs = O.routing_keys(K[:, :, :n], P)
    assert np.array_equal(KRb[:, valid], KRs) and np.array_equal(inv[:, valid], invs)
    i1, v1, _ = O.score_topk(q, KRb, G // P, 3, valid=valid)
    i2, v2, _ = O.score_topk(q, KRs, n // P, 3)
    assert np.array_equal(i1, i2) and np.allclose(v1, v2, rtol=1e-13, atol=0)    # BLAS blocks the two shapes differently
    qp = np.full((2, 3), G)
    o1, l1 = O.sparse_attend(q, K, V, i1, None, None, G, qp, 1e4, lens=lens)
    o2, l2 = O.sparse_attend(q, K[:, :, :n], V[:, :, :n], i1, None, None, G, qp, 1e4)
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)
