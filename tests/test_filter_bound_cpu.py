"""The arithmetic claim behind the one-pass filter of the prefill scoring GEMM, checked on the CPU.

The GEMM multiplies only hi = bf16(q) of a folded fp32 routing query q and treats the result s~ as the exact
cosine score s within eps = 1.01 |q - hi| + 2e-5 |q| + 1e-7 (fold_queries_kernel writes exactly this bound).  Every
list entry with s~ >= t~ - 2 eps, t~ the k-th largest s~, is then scored again exactly.  Two facts are needed:
  (1) |s~ - s| <= eps for any stored key whose |key| * inv_norm <= 1 (up to bf16 rounding of the key), with the
      product accumulated in fp32 in any order;
  (2) the candidate set {s~ >= t~ - 2 eps} contains the exact top-k.
Neither needs a GPU: fp32 accumulation is emulated with numpy float32 in shuffled orders, the exact score is
float64.  (This checks the inequality, not the kernels; the kernels' selections are compared with the oracle
in the GPU parity tests.)"""
import numpy as np

import msa_synth as S


def bf16(x):
    return S.bf16_bits_to_f64(S.f64_to_bf16_bits(x))


def eps_bound(q):
    hi = bf16(q)
    lo = q - hi
    return 1.01 * np.linalg.norm(lo, axis=-1) + 2e-5 * np.linalg.norm(q, axis=-1) + 1e-7, hi


def fp32_dot_shuffled(a, b, rng):
    """sum_i a_i b_i in float32, products and partial sums rounded to float32, in a random order."""
    perm = rng.permutation(a.shape[-1])
    acc = np.float32(0.0)
    for i in perm:
        acc = np.float32(acc + np.float32(np.float32(a[i]) * np.float32(b[i])))
    return float(acc)


def make_queries(rng, n, d, r):
    """Folded queries as the fold computes them: mean over r heads of unit-normalised bf16 head queries (fp32)."""
    qh = bf16(rng.standard_normal((n, r, d)))
    qh = qh / np.maximum(np.linalg.norm(qh, axis=-1, keepdims=True), 1e-12)
    return qh.mean(axis=1).astype(np.float32).astype(np.float64)


def test_one_pass_score_is_within_eps_of_the_exact_score():
    rng = np.random.default_rng(20260323)
    d = 128
    worst = 0.0
    for r in (1, 2, 4):
        q = make_queries(rng, 40, d, r)
        eps, hi = eps_bound(q)
        lo = q - hi
        for i in range(q.shape[0]):
            keys = [bf16(rng.standard_normal(d)),                      # a random key
                    bf16(lo[i] / max(np.linalg.norm(lo[i]), 1e-30)),    # the key aligned with the dropped part
                    bf16(-lo[i] * 37.0),                                 # ... and against it, not unit length
                    bf16(q[i] * 0.01)]                                   # a short key along the query
            for key in keys:
                inv = np.float32(1.0 / max(np.linalg.norm(key), 1e-12))
                exact = float(np.dot(q[i], key)) * float(inv)
                one_pass = np.float32(fp32_dot_shuffled(hi[i], key, rng)) * inv
                err = abs(float(one_pass) - exact)
                assert err <= eps[i], (r, i, err, eps[i])
                worst = max(worst, err / eps[i])
    assert worst > 0.5, worst   # the aligned key comes close to the bound: the bound is not vacuous


def test_candidate_band_contains_the_exact_top_k():
    rng = np.random.default_rng(7)
    d, n_docs, k = 128, 600, 8
    for trial in range(6):
        q = make_queries(rng, 1, d, 2)[0]
        eps, hi = eps_bound(q[None])
        eps, hi = float(eps[0]), hi[0]
        keys = bf16(rng.standard_normal((n_docs, d)))
        # documents packed around the k-th score so that the one-pass order differs from the exact one
        base = q / np.linalg.norm(q)
        for j in range(60):
            v = rng.standard_normal(d)
            v -= base * np.dot(v, base)
            v /= np.linalg.norm(v)
            c = 0.5 + (j % 7) * 1e-4
            keys[j] = bf16(c * base + np.sqrt(1 - c * c) * v)
        inv = 1.0 / np.maximum(np.linalg.norm(keys, axis=-1), 1e-12)
        exact = (keys @ q) * inv
        one_pass = (keys.astype(np.float32) @ hi.astype(np.float32)).astype(np.float64) * inv.astype(np.float32)
        assert np.max(np.abs(one_pass - exact)) <= eps
        t = np.sort(one_pass)[-k]
        cand = set(np.nonzero(one_pass >= t - 2 * eps)[0].tolist())
        order = np.lexsort((np.arange(n_docs), -exact))      # score descending, index ascending
        assert set(order[:k].tolist()) <= cand
        assert len(cand) < n_docs // 4                        # and it is a filter: few survive
