"""Host-side helpers of the full-size parity tests: the ORACLE's routing index of a whole benchmark bank and the
oracle's attention outputs, computed from the seed in worker processes (NumPy only, nothing here touches the GPU).

A bank of the benchmark configurations never exists on the host as a whole (2 GiB .. 191 GiB of keys); every
document is regenerated from the counter-based generator, pooled by the oracle and dropped again, so the oracle's
index (34 MB .. 1.6 GB as bf16 bits) is built without any value that came from the HIP path.
"""
import multiprocessing as mp
import os

import numpy as np

DOCS_PER_TASK = 32


def n_workers():
    return max(1, min(16, os.cpu_count() or 1))


def _index_task(args):
    seed, Hkv, G, d, P, lo, hi, planted, lens = args
    import msa_synth as S
    from oracle import msa_oracle as O
    Ks = np.empty((hi - lo, Hkv, G, d), dtype=np.float64)
    for i in range(lo, hi):
        Ks[i - lo] = S.bf16_bits_to_f64(planted[i]) if i in planted else S.doc_slice(seed, Hkv, G, d, i)[1]
    KRb, inv = O.routing_keys(Ks, P, None if lens is None else lens)
    return lo, hi, S.f64_to_bf16_bits(KRb), inv


def _attend_task(args):
    """Oracle attention of one (batch row, query token, KV group): (out [r, d], lse [r])."""
    (seeds, Hkv, G, d, r, Lloc, pos0, base, b, m, g, docs, planted, q_heads, q_pos, lens) = args
    import msa_synth as S
    from oracle import msa_oracle as O

    def doc(which, i):
        if which == "K" and i in planted:
            return S.bf16_bits_to_f64(planted[i])[g:g + 1]
        per_doc = Hkv * G * d
        return S.normal_bf16(seeds[which], (1, G, d), start=i * per_doc + g * G * d)[1]
    K_sel = np.stack([doc("K", int(i)) for i in docs])            # [k, 1, G, d]
    V_sel = np.stack([doc("V", int(i)) for i in docs])
    Kl = Vl = None
    if Lloc > 0:
        start = (b * Hkv + g) * Lloc * d
        Kl = S.normal_bf16(seeds["Kloc"], (1, 1, Lloc, d), start=start)[1]
        Vl = S.normal_bf16(seeds["Vloc"], (1, 1, Lloc, d), start=start)[1]
    sel_lens = None if lens is None else np.asarray(lens)
    oo, ol = O.sparse_attend(q_heads[None, None], K_sel, V_sel, np.arange(len(docs))[None, None, None], Kl, Vl,
                             pos0, np.array([[q_pos]]), base, lens=sel_lens)
    return b, m, g, oo[0, 0], ol[0, 0]


class OraclePool:
    """A pool of worker processes (spawned: the parent has initialised the GPU, the workers never do)."""

    def __init__(self):
        self.pool = mp.get_context("spawn").Pool(n_workers())

    def close(self):
        self.pool.close()
        self.pool.join()

    def start_index(self, wl, lens=None):
        """Begin building the oracle's routing index of workload wl; returns a handle for finish_index."""
        tasks = []
        for lo in range(0, wl.N, DOCS_PER_TASK):
            hi = min(lo + DOCS_PER_TASK, wl.N)
            planted = {i: wl.planted_K[i] for i in range(lo, hi) if i in wl.planted_K}
            tasks.append((wl.seeds["K"], wl.Hkv, wl.G, wl.d, wl.P, lo, hi, planted,
                          None if lens is None else np.asarray(lens[lo:hi])))
        return wl, self.pool.imap_unordered(_index_task, tasks, chunksize=4)

    @staticmethod
    def finish_index(handle):
        """(bits uint16 [Hkv, N*C, d], inv float64 [Hkv, N*C]) of the oracle's index."""
        wl, it = handle
        NC = wl.N * wl.C
        bits = np.empty((wl.Hkv, NC, wl.d), dtype=np.uint16)
        inv = np.empty((wl.Hkv, NC), dtype=np.float64)
        for lo, hi, b, v in it:
            bits[:, lo * wl.C:hi * wl.C] = b
            inv[:, lo * wl.C:hi * wl.C] = v
        return bits, inv

    def attend(self, wl, triples, gi, lens=None):
        """Oracle outputs for (b, m, g) triples; gi [B, M', S, k] the selection attended (int64).
        Returns {(b, m, g): (out [r, d], lse [r])}."""
        tasks = []
        Mi, Si = gi.shape[1], gi.shape[2]
        for b, m, g in triples:
            docs = gi[b, m if Mi > 1 else 0, g if Si > 1 else 0]
            planted = {int(i): wl.planted_K[int(i)] for i in docs if int(i) in wl.planted_K}
            tasks.append((wl.seeds, wl.Hkv, wl.G, wl.d, wl.r, wl.Lloc, wl.pos0, wl.base, b, m, g,
                          [int(i) for i in docs], planted, wl.q_host[b, m, g * wl.r:(g + 1) * wl.r],
                          int(wl.q_pos_host[b, m]), None if lens is None else [int(lens[int(i)]) for i in docs]))
        res = {}
        for b, m, g, oo, ol in self.pool.imap_unordered(_attend_task, tasks, chunksize=1):
            res[(b, m, g)] = (oo, ol)
        return res


def compare_selection(srow, want_idx, want_val, got_idx, got_val, k, N, atol):
    """One selection against the oracle's.  srow [N]: the oracle's document scores; (want_idx, want_val): its top-k
    by (score desc, index asc); (got_idx, got_val): the GPU's.  Bit-exact indices wherever the oracle's order is
    clear; inside the tie band (1e-3 relative around the k-th score) any document whose oracle score lies within the
    band is accepted.  Returns 1 if the lists differ (inside the band), else 0."""
    assert len(set(got_idx.tolist())) == k and got_idx.min() >= 0 and got_idx.max() < N
    assert np.allclose(got_val, srow[got_idx], rtol=0, atol=atol), np.abs(got_val - srow[got_idx]).max()
    d = np.diff(got_val)
    assert np.all(d <= 0)
    assert np.all(np.diff(got_idx)[d == 0] > 0)                 # equal scores: ascending index
    if np.array_equal(got_idx, want_idx):
        return 0
    sk = want_val[k - 1]
    band = 1e-3 * abs(sk)
    sure = want_idx[srow[want_idx] > sk + band]
    assert set(sure.tolist()) <= set(got_idx.tolist()), "a clear winner is missing"
    assert np.all(srow[got_idx] >= sk - band), "selected a document outside the tie band"
    # the oracle's own list must be ambiguous somewhere: two neighbours, or the k-th and (k+1)-th, within the band
    nxt = np.partition(srow, N - k - 1)[N - k - 1] if k < N else -np.inf
    clear = np.all(np.abs(np.diff(srow[want_idx])) > band) and srow[want_idx[-1]] - nxt > band
    assert not clear, (got_idx, want_idx)
    return 1
