"""Float64 CPU oracle for the routed-attention hot path of Memory Sparse Attention (MSA).

THIS FILE IS TEST INFRASTRUCTURE.  It is the plain, slow, obviously-correct statement of what the
GPU library must compute.  Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may
import it; the product path (paper_2603_23516_amd/) never does, and the two share no code.

Every function follows one passage of the paper (Section 3.2.1 "Sparse Attention Mechanism",
Eq. 1-4; Section 3.2.2 "Parallel and Global RoPE"; Section 3.4.2 "Memory Parallel") and says which.
Arithmetic is float64 throughout.  The only rounding performed is the round-to-nearest-even of the
pooled routing keys to bfloat16, because bfloat16 is the storage format of the routing index.

Notation (paper, Section 5.1): N documents, G tokens per document, P chunk size, C = G/P chunks
per document, Hq query heads, Hkv key/value heads, r = Hq/Hkv, d head dimension, B sequences,
M query tokens per sequence, k selected documents, Lloc local-context tokens.
Query head h belongs to KV-head group g = h // r.

Readings of the paper where it is silent (all listed again in the design document):
  * routing keys are pooled from un-rotated keys;
  * cosine uses max(norm, 1e-12) guards, so a zero vector scores 0;
  * default selection scope is one selection per KV-head group (mean over the r heads of the
    group); select_scope="all" is the literal Eq. 2 mean over every head;
  * default is one selection per query token; token_pool=True is the literal Eq. 2 max over tokens;
  * ties are broken towards the lower document index, output sorted by (score desc, index asc);
  * RoPE pairs element u with u + d/2, angle p * base**(-2u/d); values are never rotated;
  * memory keys are always visible; local key t is visible iff pos0 + t <= q_pos.

The paper's own variant of Eq. 3 (pooled K-bar / V-bar of position-encoded keys, used as stored) is
pool_rotated_keys / pool_values + sparse_attend(..., mem_rotated=True).

Pins (tests/test_oracle_pins.py): brute-force dense attention when k = N, library softmax /
scaled-dot-product attention on the G = 1 reduction, softmax and RoPE closed forms, the
document-wise RoPE permutation invariant, log-sum-exp merge associativity, pooling and scoring
closed forms, tie-break cases, shard-merge of top-k, and the paper's printed memory estimate
(Section 3.4.2: about 169 GB total, about 56 GB of routing keys).  No function here is unpinned.
"""
import numpy as np

EPS_NORM = 1e-12


# --------------------------------------------------------------------------------------------
# bfloat16 rounding (storage format of the routing index)
# --------------------------------------------------------------------------------------------
def bf16_round(x):
    """Nearest bfloat16-representable value (ties to even), returned as float64.

    bfloat16 keeps 8 significant bits; below 2**-126 the spacing is fixed at 2**-133.
    Values are assumed far from the overflow threshold (inputs are O(1))."""
    x = np.asarray(x, dtype=np.float64)
    m, e = np.frexp(x)                      # x = m * 2**e with 0.5 <= |m| < 1
    e = np.maximum(e, -125)                 # subnormal range: fixed quantum 2**-133
    q = np.rint(np.ldexp(x, 8 - e))         # np.rint rounds half to even
    return np.ldexp(q, e - 8)


# --------------------------------------------------------------------------------------------
# Section 3.2.1, chunk-wise mean pooling phi(.)  ->  routing keys
# --------------------------------------------------------------------------------------------
def chunk_valid(lens, G, P):
    """Documents of different lengths (the paper's G is an average, Section 5.1) in slots of G tokens:
    document i holds lens[i] <= G tokens, i.e. ceil(lens[i] / P) chunks, the last one possibly short.
    Returns valid [N*C] bool: chunk j of document i exists iff j * P < lens[i]."""
    lens = np.asarray(lens, dtype=np.int64)
    C = G // P
    assert np.all((lens >= 0) & (lens <= G))
    return (np.arange(C)[None, :] * P < lens[:, None]).reshape(-1)


def pool_chunks(K, P, lens=None):
    """phi(K): mean over each fixed-length chunk of P tokens (Section 3.2.1, after Eq. 1).

    K  [N, Hkv, G, d]  ->  [Hkv, N*C, d], row i*C + j is chunk j of document i.  With lens (document
    lengths, see chunk_valid) a chunk is the mean over the tokens the document really has in it (the
    tail chunk is short); chunks past the end are zero."""
    K = np.asarray(K, dtype=np.float64)
    N, Hkv, G, d = K.shape
    assert G % P == 0
    C = G // P
    out = np.zeros((Hkv, N * C, d), dtype=np.float64)
    for i in range(N):
        n_i = G if lens is None else int(lens[i])
        for g in range(Hkv):
            for j in range(C):
                hi = min((j + 1) * P, n_i)
                if hi > j * P:
                    out[g, i * C + j, :] = K[i, g, j * P:hi, :].sum(axis=0) / (hi - j * P)
    return out


def routing_keys(K, P, lens=None):
    """The stored routing index: pooled keys rounded to bfloat16, and 1/max(norm, eps) of the
    ROUNDED key (what the scoring stage multiplies by).  Returns (KRb [Hkv,N*C,d], inv_norm [Hkv,N*C]).
    With lens, chunks past a document's end carry inv_norm = -1: the stored mark of "no such chunk"
    (a real reciprocal norm is positive)."""
    KRb = bf16_round(pool_chunks(K, P, lens))
    nrm = np.sqrt((KRb * KRb).sum(axis=-1))
    inv = 1.0 / np.maximum(nrm, EPS_NORM)
    if lens is not None:
        inv[:, ~chunk_valid(lens, K.shape[2], P)] = -1.0
    return KRb, inv


def pool_rotated_keys(K, P, base, lens=None):
    """K-bar of Stage 1 (Section 3.4.1): the document is encoded with its own positions 0..G-1
    (Section 3.2.2), then chunk-mean pooled (Section 3.2.1): mean over each chunk of RoPE(K[i,g,t], t).
    K [N,Hkv,G,d] -> [N,Hkv,C,d] (exact float64; the stored bank is bf16_round of this).  With lens a
    chunk is the mean over the tokens the document has in it; chunks past the end are zero."""
    K = np.asarray(K, dtype=np.float64)
    N, Hkv, G, d = K.shape
    assert G % P == 0
    C = G // P
    out = np.zeros((N, Hkv, C, d), dtype=np.float64)
    pos = np.arange(G)
    for i in range(N):
        n_i = G if lens is None else int(lens[i])
        for g in range(Hkv):
            rot = rope(K[i, g], pos, base)
            for j in range(C):
                hi = min((j + 1) * P, n_i)
                if hi > j * P:
                    out[i, g, j, :] = rot[j * P:hi, :].sum(axis=0) / (hi - j * P)
    return out


def pool_values(V, P, lens=None):
    """V-bar = phi(V): chunk-wise mean of the values (Section 3.2.1).  [N,Hkv,G,d] -> [N,Hkv,C,d];
    lens as in pool_rotated_keys."""
    V = np.asarray(V, dtype=np.float64)
    N, Hkv, G, d = V.shape
    assert G % P == 0
    C = G // P
    out = np.zeros((N, Hkv, C, d), dtype=np.float64)
    for i in range(N):
        n_i = G if lens is None else int(lens[i])
        for g in range(Hkv):
            for j in range(C):
                hi = min((j + 1) * P, n_i)
                if hi > j * P:
                    out[i, g, j, :] = V[i, g, j * P:hi, :].sum(axis=0) / (hi - j * P)
    return out


# --------------------------------------------------------------------------------------------
# Section 3.2.1, Eq. 2: relevance scores
# --------------------------------------------------------------------------------------------
def similarity(x, Y, sim="cos"):
    """sim(x, Y[c]) for every row c of Y.  cos(x,y) = x.y / (max(|x|,eps) * max(|y|,eps)).
    x [d] -> [NC]; a matrix of queries x [n, d] -> [n, NC] (one matrix product)."""
    x = np.asarray(x, dtype=np.float64)
    dots = Y @ x if x.ndim == 1 else x @ Y.T
    if sim == "dot":
        return dots
    nx = np.maximum(np.sqrt((x * x).sum(axis=-1)), EPS_NORM)
    ny = np.maximum(np.sqrt((Y * Y).sum(axis=-1)), EPS_NORM)
    return dots / (nx * ny) if x.ndim == 1 else dots / (nx[:, None] * ny[None, :])


def chunk_scores(qr, KRb, sim="cos", select_scope="group", token_pool=False, valid=None):
    """Eq. 2.  qr [B,M,Hq,d], KRb [Hkv,NC,d]  ->  Sc [B, M', S, NC].  valid [NC] bool (documents of
    different lengths, see chunk_valid): a chunk that does not exist scores -inf.

    Head h is compared with the routing keys of its own KV head g = h // r.  The head mean is
    taken first, at chunk level; select_scope="group" averages the r heads of each group
    (S = Hkv), "all" averages every head (S = 1, literal Eq. 2).  token_pool=True then takes the
    max over the M query tokens (M' = 1, literal Eq. 2), otherwise M' = M."""
    qr = np.asarray(qr, dtype=np.float64)
    KRb = np.asarray(KRb, dtype=np.float64)
    B, M, Hq, d = qr.shape
    Hkv, NC, _ = KRb.shape
    assert Hq % Hkv == 0
    r = Hq // Hkv
    per_head = np.empty((B, M, Hq, NC), dtype=np.float64)
    for g in range(Hkv):          # the r heads of group g, all query tokens at once, against that group's keys
        heads = qr[:, :, g * r:(g + 1) * r, :].reshape(B * M * r, d)
        per_head[:, :, g * r:(g + 1) * r, :] = similarity(heads, KRb[g], sim).reshape(B, M, r, NC)
    if select_scope == "group":
        Sc = per_head.reshape(B, M, Hkv, r, NC).sum(axis=3) / r
    elif select_scope == "all":
        Sc = per_head.sum(axis=2, keepdims=True) / Hq
    else:
        raise ValueError(select_scope)
    if valid is not None:
        Sc[..., ~np.asarray(valid, dtype=bool)] = -np.inf
    if token_pool:
        Sc = Sc.max(axis=1, keepdims=True)
    return Sc


def doc_scores(Sc, C):
    """s_i = max_j S_ij (Section 3.2.1, after Eq. 2).  [..., N*C] -> [..., N]."""
    NC = Sc.shape[-1]
    assert NC % C == 0
    return Sc.reshape(Sc.shape[:-1] + (NC // C, C)).max(axis=-1)


def topk_docs(s, k):
    """I = Top-k({s_i}) (Section 3.2.1).  s [..., N] -> (idx [..., k] int64, val [..., k]).

    Order: score descending, then document index ascending (lowest index wins a tie)."""
    s = np.asarray(s, dtype=np.float64)
    N = s.shape[-1]
    assert 1 <= k <= N
    flat = s.reshape(-1, N)
    idx = np.empty((flat.shape[0], k), dtype=np.int64)
    val = np.empty((flat.shape[0], k), dtype=np.float64)
    ids = np.arange(N)
    for row in range(flat.shape[0]):
        order = np.lexsort((ids, -flat[row]))      # primary key -score, secondary key index
        idx[row] = order[:k]
        val[row] = flat[row][order[:k]]
    return idx.reshape(s.shape[:-1] + (k,)), val.reshape(s.shape[:-1] + (k,))


def score_topk(qr, KRb, C, k, sim="cos", select_scope="group", token_pool=False, valid=None):
    """Eq. 2 -> document max -> top-k, chained.  Returns (idx, val, s) with s the document scores."""
    s = doc_scores(chunk_scores(qr, KRb, sim, select_scope, token_pool, valid), C)
    idx, val = topk_docs(s, k)
    return idx, val, s


# --------------------------------------------------------------------------------------------
# Section 3.2.2: rotary position embedding, restarted per document / global for the active context
# --------------------------------------------------------------------------------------------
def rope(x, pos, base):
    """Rotate x [..., d] to position pos (scalar or array broadcastable to x.shape[:-1]).

    theta_u = base**(-2u/d); pair (u, u + d/2):
      y[u]       = x[u] cos(p theta_u) - x[u+d/2] sin(p theta_u)
      y[u + d/2] = x[u+d/2] cos(p theta_u) + x[u] sin(p theta_u)"""
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[-1]
    half = d // 2
    theta = np.float64(base) ** (-2.0 * np.arange(half, dtype=np.float64) / d)
    ang = np.asarray(pos, dtype=np.float64)[..., None] * theta
    c, s = np.cos(ang), np.sin(ang)
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


# --------------------------------------------------------------------------------------------
# Section 3.2.1, Eq. 3-4: context assembly and attention
# --------------------------------------------------------------------------------------------
def softmax_attend(qt, keys, vals):
    """Attention of one already-rotated query qt [d] over keys [n,d] / vals [n,d] (Eq. 4).

    Returns (out [d], lse) with lse = log sum_j exp(z_j), z = keys.qt / sqrt(d).
    No visible key: out = 0, lse = -inf."""
    d = qt.shape[-1]
    if keys.shape[0] == 0:
        return np.zeros(d), -np.inf
    z = (keys @ qt) / np.sqrt(np.float64(d))
    zmax = z.max()
    w = np.exp(z - zmax)
    den = w.sum()
    return (w / den) @ vals, zmax + np.log(den)


def merge_partials(parts):
    """Combine attention results over disjoint key sets: parts = [(out_i, lse_i)], weights
    exp(lse_i) / sum exp(lse_j).  Equals attention over the union of the key sets."""
    lses = np.array([p[1] for p in parts], dtype=np.float64)
    if not np.isfinite(lses.max()):
        return np.zeros_like(parts[0][0]), -np.inf
    top = lses.max()
    w = np.exp(lses - top)
    out = sum(wi * p[0] for wi, p in zip(w, parts)) / w.sum()
    return out, top + np.log(w.sum())


def assemble_context(K, V, doc_ids, g, Kloc_bg, Vloc_bg, pos0, q_pos, base, mem_rotated=False, lens=None):
    """Eq. 3 with document-wise RoPE (Section 3.2.2).  K, V [N,Hkv,G,d]; doc_ids: the selected
    documents of this (query, scope), -1 entries skipped; Kloc_bg, Vloc_bg [Lloc,d] or None.

    Every selected document contributes all its G tokens, rotated with positions 0..G-1
    (positions restart in every document).  With mem_rotated=True the bank's keys already carry
    their positions (the pooled bank of Stage 1, see pool_rotated_keys) and are used as stored.
    Local token t sits at position pos0 + t and is visible iff pos0 + t <= q_pos.
    lens [N]: document i contributes only its first lens[i] rows (positions 0..lens[i]-1).
    Returns (keys [n,d], vals [n,d])."""
    G, d = K.shape[2], K.shape[3]
    keys, vals = [], []
    for i in doc_ids:
        if i < 0:
            continue
        n_i = G if lens is None else int(lens[i])
        if mem_rotated:
            keys.append(np.asarray(K[i, g, :n_i], dtype=np.float64))
        else:
            keys.append(rope(K[i, g, :n_i], np.arange(n_i), base))
        vals.append(np.asarray(V[i, g, :n_i], dtype=np.float64))
    if Kloc_bg is not None and Kloc_bg.shape[0] > 0:
        t = np.arange(Kloc_bg.shape[0])
        vis = (pos0 + t) <= q_pos
        if vis.any():
            keys.append(rope(np.asarray(Kloc_bg, dtype=np.float64)[vis], pos0 + t[vis], base))
            vals.append(np.asarray(Vloc_bg, dtype=np.float64)[vis])
    if not keys:
        return np.zeros((0, d)), np.zeros((0, d))
    return np.concatenate(keys, axis=0), np.concatenate(vals, axis=0)


def sparse_attend(q, K, V, idx, Kloc, Vloc, pos0, q_pos, base, mem_rotated=False, lens=None):
    """Eq. 3-4 for every query.  q [B,M,Hq,d]; K,V [N,Hkv,G,d]; idx [B,M',S,k] (M' in {1,M},
    S in {1,Hkv}); Kloc,Vloc [B,Hkv,Lloc,d] or None; q_pos [B,M] int.

    out[b,m,h] = softmax_j( RoPE(q[b,m,h], q_pos[b,m]) . key_j / sqrt(d) ) . val_j over the keys of
    assemble_context for the selection of head h's group.  Returns (out [B,M,Hq,d], lse [B,M,Hq])."""
    q = np.asarray(q, dtype=np.float64)
    B, M, Hq, d = q.shape
    Hkv = K.shape[1]
    r = Hq // Hkv
    Mi, S = idx.shape[1], idx.shape[2]
    out = np.zeros((B, M, Hq, d), dtype=np.float64)
    lse = np.full((B, M, Hq), -np.inf, dtype=np.float64)
    for b in range(B):
        for m in range(M):
            for g in range(Hkv):
                ids = idx[b, m if Mi > 1 else 0, g if S > 1 else 0]
                kl = None if Kloc is None else Kloc[b, g]
                vl = None if Vloc is None else Vloc[b, g]
                keys, vals = assemble_context(K, V, ids, g, kl, vl, pos0, int(q_pos[b, m]), base, mem_rotated,
                                              lens)
                for h in range(g * r, (g + 1) * r):
                    qt = rope(q[b, m, h], np.float64(q_pos[b, m]), base)
                    out[b, m, h], lse[b, m, h] = softmax_attend(qt, keys, vals)
    return out, lse


# --------------------------------------------------------------------------------------------
# Section 3.4.2 (Memory Parallel): storage estimate and shard merge
# --------------------------------------------------------------------------------------------
def pooled_bank_bytes(tokens, P, heads, d, layers, bytes_per_elem=2, tensors=3):
    """Bytes of the pooled bank (K-bar, V-bar, routing keys => tensors=3; routing keys alone => 1)."""
    assert tokens % P == 0
    return tensors * layers * (tokens // P) * heads * d * bytes_per_elem


def merge_shard_topk(cands, k):
    """Global top-k from per-shard candidate lists [(idx array, val array), ...] with global
    document indices: the 'scores reduced globally' step of Memory Parallel, candidates only."""
    idx = np.concatenate([c[0] for c in cands])
    val = np.concatenate([c[1] for c in cands])
    order = np.lexsort((idx, -val))[:k]
    return idx[order], val[order]
