"""The per-token loop over several routed layers (Section 3.2.1: routing in the latter half of the layers; Section
3.4.2: per layer routing keys in device memory, pooled content bank in device or host memory): three layers with
their own banks and queries chained through paper_2603_23516_amd.layers.LayerStack, every layer's selection and
attention output against the oracle, with the pooled banks in HBM and in pinned host memory, on one stream and with
routing overlapped with fetch + attention on two streams."""
import numpy as np
import pytest
import torch

import msa_synth as S
import paper_2603_23516_amd as msa
from msa_synth import device as SD
from oracle import msa_oracle as O
from paper_2603_23516_amd.layers import LayerStack

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("tier", ["hbm", "host"])
def test_three_routed_layers_against_the_oracle(tier):
    L, N, Hkv, r, G, d, P, B, M, k, Lloc, base = 3, 90, 2, 4, 256, 128, 32, 3, 1, 5, 40, 1e6
    print(f"3 routed layers, pooled banks in {tier}: N={N} Hkv={Hkv} r={r} G={G} P={P} B={B} k={k} Lloc={Lloc}", flush=True)
    Hq, C = Hkv * r, G // P
    cfg = msa.MsaConfig(N, G, P, Hq, Hkv, d, base)
    stack = LayerStack(cfg, L, B, M, k, Lloc, tier=tier)
    host = []
    qs, Kls, Vls = [], [], []
    for l in range(L):
        sd = 95000 + 10 * l
        Kb, K = S.normal_bf16(sd, (N, Hkv, G, d))
        Vb, V = S.normal_bf16(sd + 1, (N, Hkv, G, d))
        qb, q = S.normal_bf16(sd + 2, (B, M, Hq, d))
        Klb, Kl = S.normal_bf16(sd + 3, (B, Hkv, Lloc, d))
        Vlb, Vl = S.normal_bf16(sd + 4, (B, Hkv, Lloc, d))
        host.append((K, V, q, Kl, Vl))
        buf = SD.bits_to_torch(Kb)                        # one staging buffer per layer: keys, then values
        stack.set_layer_keys(l, buf)
        buf.copy_(SD.bits_to_torch(Vb))
        stack.set_layer_values(l, buf)
        qs.append(SD.bits_to_torch(qb))
        Kls.append(SD.bits_to_torch(Klb))
        Vls.append(SD.bits_to_torch(Vlb))
    torch.cuda.synchronize()
    pos0 = k                                              # Section 3.2.2: local positions start at k
    q_pos = np.full((B, M), pos0 + Lloc - 1)
    dpos = torch.from_numpy(q_pos.astype(np.int32)).cuda()
    results = {}
    for overlap in (False, True, True):
        outs = [torch.zeros_like(qs[0]) for _ in range(L)]
        lses = [torch.zeros((B, M, Hq), dtype=torch.float32, device="cuda") for _ in range(L)]
        stack.step(qs, Kls, Vls, pos0, dpos, outs, lses, overlap=overlap)
        torch.cuda.synchronize()
        results[overlap] = ([o.clone() for o in outs], [x.clone() for x in lses], [i.clone() for i in stack.idx])
    for a, b in zip(results[False][0] + results[False][1] + results[False][2],
                    results[True][0] + results[True][1] + results[True][2]):
        assert torch.equal(a.view(torch.int32) if a.dtype == torch.float32 else a.view(torch.int16) if a.dtype == torch.bfloat16 else a,
                           b.view(torch.int32) if b.dtype == torch.float32 else b.view(torch.int16) if b.dtype == torch.bfloat16 else b)
    outs, lses, idxs = results[True]
    for l, (K, V, q, Kl, Vl) in enumerate(host):
        KRb, _ = O.routing_keys(K, P)
        oi, ov, _ = O.score_topk(q, KRb, C, k)
        assert np.array_equal(idxs[l].cpu().numpy(), oi), f"layer {l}: selection"
        Kbar = O.bf16_round(O.pool_rotated_keys(K, P, base))
        Vbar = O.bf16_round(O.pool_values(V, P))
        oo, ol = O.sparse_attend(q, Kbar, Vbar, oi, Kl, Vl, pos0, q_pos, base, mem_rotated=True)
        go = outs[l].float().cpu().numpy().astype(np.float64)
        gl = lses[l].cpu().numpy().astype(np.float64)
        err = np.abs(go - oo)
        rel = np.linalg.norm(err) / np.linalg.norm(oo)
        print(f"   layer {l}: max-abs {err.max():.3e} rel-L2 {rel:.3e}", flush=True)
        assert err.max() <= 2e-2 and rel <= 5e-3
        assert np.allclose(gl, ol, rtol=0, atol=5e-3)
    index_bytes, bank_bytes = stack.bytes()
    assert index_bytes == L * (msa.routing_keys_bytes(cfg) + msa.inv_norm_bytes(cfg))
    assert bank_bytes == L * 2 * N * Hkv * C * d * 2
