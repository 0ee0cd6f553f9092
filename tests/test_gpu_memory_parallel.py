"""Memory Parallel (Section 3.4.2) rehearsed on ONE GPU: the bank is cut into two shards, every shard goes
through the same entry points at its own shape (index build, score + top-k, attention over the winners it owns),
and the two small exchanges of the sharded design -- candidates (score, global id), then attention partials
(out, lse) -- are done on the host with the oracle's merges.  The result must equal the unsharded run of the HIP
path and the oracle.  No second GPU and no collective is involved."""
import numpy as np
import pytest
import torch

import msa_synth as S
import paper_2603_23516_amd as msa
from oracle import msa_oracle as O
from test_gpu_parity import dev, say

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("scope", ["group", "all"])
def test_two_shards_equal_the_whole_bank(scope):
    seed, N, Hkv, r, G, d, P, B, M, Lloc, base, k = 81000, 240, 2, 4, 64, 128, 8, 3, 1, 40, 1e6, 8
    cut = 131                                                        # shards of different sizes
    say(f"memory parallel rehearsal: N={N} cut at {cut} Hkv={Hkv} r={r} G={G} d={d} B={B} k={k} scope={scope}")
    Hq = Hkv * r
    Kb, K = S.normal_bf16(seed, (N, Hkv, G, d))
    Vb, V = S.normal_bf16(seed + 1, (N, Hkv, G, d))
    qb, q = S.normal_bf16(seed + 2, (B, M, Hq, d))
    Klb, Kl = S.normal_bf16(seed + 3, (B, Hkv, Lloc, d))
    Vlb, Vl = S.normal_bf16(seed + 4, (B, Hkv, Lloc, d))
    dK, dV, dq, dKl, dVl = dev(Kb), dev(Vb), dev(qb), dev(Klb), dev(Vlb)
    sc = msa.MSA_SCOPE_ALL if scope == "all" else msa.MSA_SCOPE_GROUP
    pos0 = G
    q_pos = np.full((B, M), pos0 + Lloc - 1)
    dpos = torch.from_numpy(q_pos.astype(np.int32)).cuda()

    # the unsharded run
    cfg = msa.MsaConfig(N, G, P, Hq, Hkv, d, base, select_scope=sc)
    KR, inv = msa.msa_build_routing_keys(cfg, dK)
    idx_w, val_w = msa.msa_score_topk(cfg, dq, KR, inv, k)
    out_w, lse_w = msa.msa_sparse_attend(cfg, dq, dK, dV, idx_w, dKl, dVl, pos0, dpos)
    torch.cuda.synchronize()
    idx_w, val_w = idx_w.cpu().numpy(), val_w.cpu().numpy()

    # every shard: its own index and its own top-k, with local document numbers
    shards = [(0, cut), (cut, N)]
    cands = []
    for lo, hi in shards:
        cfg_s = msa.MsaConfig(hi - lo, G, P, Hq, Hkv, d, base, select_scope=sc)
        Ks = dK[lo:hi].contiguous()
        KR_s, inv_s = msa.msa_build_routing_keys(cfg_s, Ks)
        i_s, v_s = msa.msa_score_topk(cfg_s, dq, KR_s, inv_s, k)
        torch.cuda.synchronize()
        cands.append((i_s.cpu().numpy().astype(np.int64) + lo, v_s.cpu().numpy()))
    # exchange 1: candidates only, merged by (score descending, global id ascending)
    n_sel = idx_w.shape[2]
    merged = np.zeros_like(idx_w)
    for b in range(B):
        for m in range(M):
            for s_ in range(n_sel):
                mi, mv = O.merge_shard_topk([(c[0][b, m, s_], c[1][b, m, s_]) for c in cands], k)
                merged[b, m, s_] = mi
                assert np.array_equal(mv, val_w[b, m, s_]), (b, m, s_)   # a document's score does not depend on its shard
    assert np.array_equal(merged, idx_w)
    say("   merged shard candidates equal the top-k over the whole bank")

    # every shard attends the winners it owns; shard 0 also holds the local context
    parts = []
    for si, (lo, hi) in enumerate(shards):
        cfg_s = msa.MsaConfig(hi - lo, G, P, Hq, Hkv, d, base, select_scope=sc)
        own = np.where((merged >= lo) & (merged < hi), merged - lo, -1).astype(np.int32)
        o_s, l_s = msa.msa_sparse_attend(cfg_s, dq, dK[lo:hi].contiguous(), dV[lo:hi].contiguous(),
                                         torch.from_numpy(own).cuda(), dKl if si == 0 else None,
                                         dVl if si == 0 else None, pos0, dpos)
        torch.cuda.synchronize()
        parts.append((o_s.float().cpu().numpy().astype(np.float64), l_s.cpu().numpy().astype(np.float64)))
    # exchange 2: (out, lse) partials, merged with log-sum-exp weights
    out_m = np.zeros((B, M, Hq, d))
    lse_m = np.zeros((B, M, Hq))
    for b in range(B):
        for m in range(M):
            for h in range(Hq):
                out_m[b, m, h], lse_m[b, m, h] = O.merge_partials([(p[0][b, m, h], p[1][b, m, h]) for p in parts])
    gw = out_w.float().cpu().numpy().astype(np.float64)
    d_hip = np.abs(out_m - gw).max()
    oo, ol = O.sparse_attend(q, K, V, merged, Kl, Vl, pos0, q_pos, base)
    err = np.abs(out_m - oo)
    rel = np.linalg.norm(err) / np.linalg.norm(oo)
    say(f"   merged partials: max-abs {err.max():.3e} rel-L2 {rel:.3e} against the oracle; "
        f"{d_hip:.3e} from the unsharded HIP run")
    assert err.max() <= 2e-2 and rel <= 5e-3
    assert d_hip <= 2e-2
    assert np.allclose(lse_m, ol, rtol=0, atol=5e-3)
    assert np.allclose(lse_m, lse_w.cpu().numpy(), rtol=0, atol=5e-3)
