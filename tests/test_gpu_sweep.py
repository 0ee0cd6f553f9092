"""Seeded sweep over the configuration space the library accepts: geometry (d, Hkv, r, C, P), batch shape,
k, local context, similarity, selection scope, token pooling and document lengths are drawn at random within
the documented limits, and every draw runs the whole chain (index build, score + top-k, attention) against
the float64 oracle with the tolerances of test_gpu_parity.py.  The draws are fixed by the seed, so a failure
names its case."""

import numpy as np
import pytest
import torch

import paper_2603_23516_amd as msa
from oracle import msa_oracle as O
from test_gpu_parity import Case, check_topk_generic, say
from test_gpu_ragged import attend_err, make_lens

pytestmark = pytest.mark.gpu

FIRST_DRAW, N_DRAWS = 0, 96


def draw(i):
    rng = np.random.default_rng(90000 + i)
    d = int(rng.choice([64, 128]))
    while True:
        C = int(rng.choice([1, 2, 4, 8, 16]))
        P = int(rng.choice([8, 16, 32, 64]))
        if (C * P) % 32 == 0 and C * P <= 512:
            break
    scope = str(rng.choice(["group", "group", "all"]))
    Hkv = int(rng.choice([1, 2, 4, 8] if scope == "all" else [1, 2, 3, 4, 5, 8]))
    r = int(rng.choice([1, 2, 4, 8]))
    while Hkv * r > 32:
        r //= 2
    shape = str(rng.choice(["decode", "batch", "prefill", "prefill_big"]))
    if shape == "decode":
        B, M = int(rng.integers(1, 4)), 1
    elif shape == "batch":
        B, M = int(rng.integers(4, 41)), 1
    elif shape == "prefill":
        B, M = int(rng.integers(1, 3)), int(rng.integers(2, 24))
    else:
        B, M = 1, int(rng.integers(64, 130))
    G = C * P
    N = int(rng.integers(8, max(9, min(400, 120000 // (G * Hkv)))))
    k = int(rng.integers(1, min(N, 24) + 1))
    Lloc = int(rng.choice([0, int(rng.integers(1, 80))]))
    if M > 1 and Lloc == 0:
        Lloc = M
    return dict(d=d, C=C, P=P, G=G, Hkv=Hkv, r=r, B=B, M=M, N=N, k=k, Lloc=Lloc, scope=scope,
                pool=bool(rng.integers(0, 2)) and M > 1, sim=str(rng.choice(["cos", "cos", "dot"])),
                ragged=bool(rng.integers(0, 2)), base=float(rng.choice([1e4, 1e6])), seed=91000 + 17 * i)


@pytest.mark.parametrize("i", range(FIRST_DRAW, FIRST_DRAW + N_DRAWS))
def test_random_configuration(i):
    c = draw(i)
    say(f"draw {i}: {c}")
    N, G, P, C, k, B, M, Lloc = c["N"], c["G"], c["P"], c["C"], c["k"], c["B"], c["M"], c["Lloc"]
    case = Case(c["seed"], N, c["Hkv"], c["r"], G, c["d"], P, B, M, Lloc, c["base"]).to_device()
    lens = make_lens(c["seed"] + 5, N, G, P) if c["ragged"] else None
    dlens = None if lens is None else torch.from_numpy(lens.astype(np.int32)).cuda()
    cfg = case.cfg(sim=msa.MSA_SIM_COS if c["sim"] == "cos" else msa.MSA_SIM_DOT,
                   select_scope=msa.MSA_SCOPE_ALL if c["scope"] == "all" else msa.MSA_SCOPE_GROUP,
                   token_pool=int(c["pool"]), doc_lens=dlens)
    KR, inv = msa.msa_build_routing_keys(cfg, case.dK)
    idx, val = msa.msa_score_topk(cfg, case.dq, KR, inv if c["sim"] == "cos" else None, k)
    torch.cuda.synchronize()
    KRo, _ = O.routing_keys(case.K, P, lens)
    valid = None if lens is None else O.chunk_valid(lens, G, P)
    # chained on the GPU's own index: a tie-adjacent rounding of a key moves a score by up to ~1e-3 relative
    # chained on the GPU-built index: a key one bf16 step off (next to a rounding tie) moves a cosine by <= 1e-4 and an
    # un-normalised dot product (|q| ~ 11, |q_i k_i| up to ~1) by up to 2^-8 |q_i k_i| ~ 4e-3
    atol = 2e-4 if c["sim"] == "cos" else 5e-3
    oi, n_band = check_topk_generic(case.q, KRo, C, N, idx, val, k, c["sim"], c["scope"], c["pool"], atol=atol,
                                    valid=valid)
    say(f"   top-k ok, shape {tuple(idx.shape)} ({n_band} inside the tie band)")
    pos0 = G
    q_pos = np.array([[pos0 + (min(Lloc - 1, (3 * m + b) % Lloc) if Lloc else 0) for m in range(M)]
                      for b in range(B)])
    if M == 1 and Lloc:
        q_pos[:] = pos0 + Lloc - 1
    dpos = torch.from_numpy(q_pos.astype(np.int32)).cuda()
    out, lse = msa.msa_sparse_attend(cfg, case.dq, case.dK, case.dV, idx, case.dKl, case.dVl, pos0, dpos)
    torch.cuda.synchronize()
    gi = idx.cpu().numpy().astype(np.int64)
    oo, ol = O.sparse_attend(case.q, case.K, case.V, gi, case.Kl, case.Vl, pos0, q_pos, c["base"], lens=lens)
    attend_err(out, lse, oo, ol)
