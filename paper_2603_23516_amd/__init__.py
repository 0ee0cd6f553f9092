"""Thin Python binding of libmsa.so (include/msa.h): argument marshalling only.

Every step of the path runs in the HIP kernels behind the C ABI; PyTorch is used here for device
memory and streams.  There is no CPU fallback: if the library is not built the calls raise.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmsa.so")

MSA_SIM_DOT, MSA_SIM_COS = 0, 1
MSA_SCOPE_GROUP, MSA_SCOPE_ALL = 0, 1
MSA_MAX_TOPK = 64
MSA_OK, MSA_ERR_INVALID_ARG, MSA_ERR_UNSUPPORTED, MSA_ERR_WORKSPACE, MSA_ERR_MISALIGNED, MSA_ERR_HIP = \
    0, -1, -2, -3, -4, -5

EXPORTS = ("msa_version", "msa_status_string", "msa_routing_keys_bytes", "msa_inv_norm_bytes",
           "msa_pooled_bank_bytes", "msa_score_topk_workspace_bytes",
           "msa_sparse_attend_workspace_bytes", "msa_build_routing_keys", "msa_pool_kv", "msa_score_topk",
           "msa_sparse_attend", "msa_fetch_slots", "msa_fetch_selected",
           "msa_noalloc_scratch_bytes", "msa_score_topk_noalloc")


class MsaConfig(ctypes.Structure):
    """Mirror of msa_config_t."""
    _fields_ = [("n_docs", ctypes.c_int32), ("doc_len", ctypes.c_int32), ("chunk", ctypes.c_int32),
                ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("rope_base", ctypes.c_float), ("sim", ctypes.c_int32),
                ("select_scope", ctypes.c_int32), ("token_pool", ctypes.c_int32),
                ("bank_keys_rotated", ctypes.c_int32), ("doc_lens", ctypes.c_void_p),
                ("profile_start_event", ctypes.c_void_p), ("profile_stop_event", ctypes.c_void_p)]

    def __init__(self, n_docs, doc_len, chunk, n_q_heads, n_kv_heads, head_dim, rope_base=1e6,
                 sim=MSA_SIM_COS, select_scope=MSA_SCOPE_GROUP, token_pool=0, bank_keys_rotated=0,
                 doc_lens=None):
        """doc_lens: None, or a contiguous CUDA int32 tensor [n_docs] (kept alive by this object)."""
        if doc_lens is not None:
            if not (doc_lens.is_cuda and doc_lens.dtype == torch.int32 and doc_lens.is_contiguous() and
                    doc_lens.numel() == n_docs):
                raise ValueError("doc_lens: expected a contiguous CUDA int32 tensor of n_docs entries")
        self.doc_lens_tensor = doc_lens
        super().__init__(n_docs, doc_len, chunk, n_q_heads, n_kv_heads, head_dim, rope_base, sim,
                         select_scope, token_pool, bank_keys_rotated,
                         None if doc_lens is None else doc_lens.data_ptr(), None, None)
        self._profile_events = None

    def set_profile_events(self, start_event=None, stop_event=None):
        """Per-call timing aid: torch.cuda.Event objects with timing enabled that have been recorded once (torch
        creates the underlying event at the first record), recorded by msa_score_topk / msa_sparse_attend around
        their dominant kernel when called with this config; (None, None) switches it off."""
        self._profile_events = (start_event, stop_event)           # kept alive by this object
        self.profile_start_event = None if start_event is None else start_event.cuda_event
        self.profile_stop_event = None if stop_event is None else stop_event.cuda_event
        return self

    def replace(self, **kw):
        """A copy with some fields changed (doc_lens: a tensor or None)."""
        f = dict(n_docs=self.n_docs, doc_len=self.doc_len, chunk=self.chunk, n_q_heads=self.n_q_heads,
                 n_kv_heads=self.n_kv_heads, head_dim=self.head_dim, rope_base=self.rope_base, sim=self.sim,
                 select_scope=self.select_scope, token_pool=self.token_pool,
                 bank_keys_rotated=self.bank_keys_rotated, doc_lens=self.doc_lens_tensor)
        f.update(kw)
        return MsaConfig(**f)

    @property
    def chunks_per_doc(self):
        return self.doc_len // self.chunk

    @property
    def n_tiles(self):
        return (self.n_docs * self.chunks_per_doc + 15) // 16


class MsaError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


_lib = None


def load_library():
    """Load libmsa.so and declare its prototypes.  Raises if the library has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is not built; run: python -c 'import __graft_entry__ as g; g.build()'")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    cfgp = ctypes.POINTER(MsaConfig)
    lib.msa_version.restype = ctypes.c_int
    lib.msa_version.argtypes = []
    lib.msa_status_string.restype = ctypes.c_char_p
    lib.msa_status_string.argtypes = [ctypes.c_int]
    lib.msa_routing_keys_bytes.restype = sz
    lib.msa_routing_keys_bytes.argtypes = [cfgp]
    lib.msa_inv_norm_bytes.restype = sz
    lib.msa_inv_norm_bytes.argtypes = [cfgp]
    lib.msa_pooled_bank_bytes.restype = ctypes.c_uint64
    lib.msa_pooled_bank_bytes.argtypes = [ctypes.c_uint64] + [ctypes.c_uint32] * 6
    lib.msa_score_topk_workspace_bytes.restype = sz
    lib.msa_score_topk_workspace_bytes.argtypes = [cfgp, i32, i32, i32]
    lib.msa_sparse_attend_workspace_bytes.restype = sz
    lib.msa_sparse_attend_workspace_bytes.argtypes = [cfgp, i32, i32, i32, i32]
    lib.msa_build_routing_keys.restype = ctypes.c_int
    lib.msa_build_routing_keys.argtypes = [cfgp, vp, i32, i32, vp, vp, vp]
    lib.msa_pool_kv.restype = ctypes.c_int
    lib.msa_pool_kv.argtypes = [cfgp, vp, vp, i32, i32, vp, vp, vp, vp]
    lib.msa_fetch_slots.restype = ctypes.c_int64
    lib.msa_fetch_slots.argtypes = [cfgp, i32, i32, i32]
    lib.msa_fetch_selected.restype = ctypes.c_int
    lib.msa_fetch_selected.argtypes = [cfgp, vp, vp, vp, i32, i32, i32, vp, vp, vp, vp, vp]
    lib.msa_score_topk.restype = ctypes.c_int
    lib.msa_score_topk.argtypes = [cfgp, vp, i32, i32, vp, vp, i32, vp, vp, vp, sz, vp]
    lib.msa_noalloc_scratch_bytes.restype = sz
    lib.msa_noalloc_scratch_bytes.argtypes = []
    lib.msa_score_topk_noalloc.restype = ctypes.c_int
    lib.msa_score_topk_noalloc.argtypes = [cfgp, vp, i32, i32, vp, vp, i32, vp, vp, vp]
    lib.msa_sparse_attend.restype = ctypes.c_int
    lib.msa_sparse_attend.argtypes = [cfgp, vp, i32, i32, vp, vp, vp, i32, vp, vp, i32, i32, vp, vp,
                                      vp, vp, sz, vp]
    _lib = lib
    return lib


def status_string(status):
    return load_library().msa_status_string(int(status)).decode()


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream, device):
    s = stream if stream is not None else torch.cuda.current_stream(device)
    return ctypes.c_void_p(s.cuda_stream)


def _check(rc, where):
    if rc != MSA_OK:
        raise MsaError(rc, where)


def _need(t, dtype, name):
    if not (t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise ValueError(f"{name}: expected a contiguous CUDA tensor of {dtype}")


# ---- size helpers -------------------------------------------------------------------------------
def routing_keys_bytes(cfg):
    return load_library().msa_routing_keys_bytes(ctypes.byref(cfg))


def inv_norm_bytes(cfg):
    return load_library().msa_inv_norm_bytes(ctypes.byref(cfg))


def pooled_bank_bytes(tokens, chunk, heads, head_dim, n_layers, bytes_per_elem=2, n_tensors=3):
    return load_library().msa_pooled_bank_bytes(tokens, chunk, heads, head_dim, n_layers, bytes_per_elem,
                                                n_tensors)


def score_topk_workspace_bytes(cfg, B, M, k):
    return load_library().msa_score_topk_workspace_bytes(ctypes.byref(cfg), B, M, k)


def sparse_attend_workspace_bytes(cfg, B, M, k, Lloc):
    return load_library().msa_sparse_attend_workspace_bytes(ctypes.byref(cfg), B, M, k, Lloc)


def alloc_routing_index(cfg, device="cuda"):
    """(KR, inv_norm) buffers of the tiled routing index: bf16 [Hkv][tiles][d/8][16][8], fp32 [Hkv][tiles*16]."""
    KR = torch.empty((cfg.n_kv_heads, cfg.n_tiles, cfg.head_dim // 8, 16, 8), dtype=torch.bfloat16,
                     device=device)
    inv = torch.empty((cfg.n_kv_heads, cfg.n_tiles * 16), dtype=torch.float32, device=device)
    assert KR.numel() * 2 == routing_keys_bytes(cfg) and inv.numel() * 4 == inv_norm_bytes(cfg)
    return KR, inv


def untile_routing_keys(cfg, KR):
    """Re-index the tiled KR to plain order [Hkv][N*C][d] (a copy; used by tests and tools)."""
    Hkv, tiles, d = cfg.n_kv_heads, cfg.n_tiles, cfg.head_dim
    plain = KR.reshape(Hkv, tiles, d // 8, 16, 8).permute(0, 1, 3, 2, 4).reshape(Hkv, tiles * 16, d)
    return plain[:, :cfg.n_docs * cfg.chunks_per_doc].contiguous()


# ---- the three operations -----------------------------------------------------------------------
def msa_build_routing_keys(cfg, K, doc_begin=0, doc_count=None, KR=None, inv_norm=None, stream=None):
    """K bf16 [N][Hkv][G][d] -> (KR, inv_norm) for documents [doc_begin, doc_begin + doc_count)."""
    _need(K, torch.bfloat16, "K")
    if doc_count is None:
        doc_count = cfg.n_docs - doc_begin
    if KR is None or inv_norm is None:
        KR, inv_norm = alloc_routing_index(cfg, K.device)
    rc = load_library().msa_build_routing_keys(ctypes.byref(cfg), _ptr(K), doc_begin, doc_count, _ptr(KR),
                                               _ptr(inv_norm), _stream(stream, K.device))
    _check(rc, "msa_build_routing_keys")
    return KR, inv_norm


def msa_pool_kv(cfg, K, V, doc_begin=0, doc_count=None, Kbar=None, Vbar=None, pooled_lens=None, stream=None):
    """K, V bf16 [N][Hkv][G][d] -> pooled bank (Kbar, Vbar) bf16 [N][Hkv][C][d]; Kbar is the chunk mean of the
    position-encoded keys.  Read it with a config whose doc_len = C and bank_keys_rotated = 1.  K or V may be None:
    that half is skipped and comes back as None.  When cfg carries doc_lens the result is (Kbar, Vbar, pooled_lens
    int32 [N]), pooled_lens being the pooled bank's doc_lens."""
    if K is None and V is None:
        raise ValueError("msa_pool_kv: K and V are both None")
    src = K if K is not None else V
    if K is not None:
        _need(K, torch.bfloat16, "K")
    if V is not None:
        _need(V, torch.bfloat16, "V")
    if doc_count is None:
        doc_count = cfg.n_docs - doc_begin
    shape = (cfg.n_docs, cfg.n_kv_heads, cfg.chunks_per_doc, cfg.head_dim)
    if Kbar is None and K is not None:
        Kbar = torch.empty(shape, dtype=torch.bfloat16, device=src.device)
    if Vbar is None and V is not None:
        Vbar = torch.empty(shape, dtype=torch.bfloat16, device=src.device)
    if K is None:
        Kbar = None
    if V is None:
        Vbar = None
    ragged = cfg.doc_lens_tensor is not None
    if ragged and pooled_lens is None:
        pooled_lens = torch.empty(cfg.n_docs, dtype=torch.int32, device=src.device)
    rc = load_library().msa_pool_kv(ctypes.byref(cfg), _ptr(K), _ptr(V), doc_begin, doc_count, _ptr(Kbar),
                                    _ptr(Vbar), _ptr(pooled_lens), _stream(stream, src.device))
    _check(rc, "msa_pool_kv")
    return (Kbar, Vbar, pooled_lens) if ragged else (Kbar, Vbar)


def msa_score_topk(cfg, q_route, KR, inv_norm, k, out_idx=None, out_score=None, workspace=None,
                   stream=None):
    """q_route bf16 [B][M][Hq][d] -> (idx int32 [B][M'][S][k], score fp32 [B][M'][S][k]); S = Hkv, or 1 with
    select_scope = ALL; M' = M, or 1 with token_pool = 1."""
    _need(q_route, torch.bfloat16, "q_route")
    B, M = q_route.shape[0], q_route.shape[1]
    dev = q_route.device
    shape = (B, 1 if cfg.token_pool else M, 1 if cfg.select_scope == MSA_SCOPE_ALL else cfg.n_kv_heads, k)
    if out_idx is None:
        out_idx = torch.empty(shape, dtype=torch.int32, device=dev)
    if out_score is None:
        out_score = torch.empty(shape, dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = torch.empty(max(score_topk_workspace_bytes(cfg, B, M, k), 256), dtype=torch.uint8,
                                device=dev)
    rc = load_library().msa_score_topk(ctypes.byref(cfg), _ptr(q_route), B, M, _ptr(KR), _ptr(inv_norm), k,
                                       _ptr(out_idx), _ptr(out_score), _ptr(workspace), workspace.numel(),
                                       _stream(stream, dev))
    _check(rc, "msa_score_topk")
    return out_idx, out_score


def noalloc_scratch_bytes():
    return load_library().msa_noalloc_scratch_bytes()


def msa_score_topk_noalloc(cfg, q_route, KR, inv_norm, k, out_idx, out_score, stream=None):
    """msa_score_topk on the library's built-in scratch buffer: the caller passes every output, nothing is
    allocated here or in the library."""
    _need(q_route, torch.bfloat16, "q_route")
    _need(out_idx, torch.int32, "out_idx")
    B, M = q_route.shape[0], q_route.shape[1]
    rc = load_library().msa_score_topk_noalloc(ctypes.byref(cfg), _ptr(q_route), B, M, _ptr(KR), _ptr(inv_norm),
                                               k, _ptr(out_idx), _ptr(out_score), _stream(stream, q_route.device))
    _check(rc, "msa_score_topk_noalloc")
    return out_idx, out_score


def msa_sparse_attend(cfg, q, K, V, idx, Kloc, Vloc, local_pos0, q_pos, out=None, lse=None,
                      workspace=None, stream=None):
    """q bf16 [B][M][Hq][d], bank K/V, idx int32 [B][M'][S][k] as msa_score_topk writes it for cfg, local cache
    -> (out bf16, lse fp32)."""
    _need(q, torch.bfloat16, "q")
    _need(idx, torch.int32, "idx")
    _need(q_pos, torch.int32, "q_pos")
    B, M = q.shape[0], q.shape[1]
    k = idx.shape[-1]
    Lloc = 0 if Kloc is None else Kloc.shape[2]
    dev = q.device
    if out is None:
        out = torch.empty_like(q)
    if lse is None:
        lse = torch.empty((B, M, cfg.n_q_heads), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = torch.empty(max(sparse_attend_workspace_bytes(cfg, B, M, k, Lloc), 256),
                                dtype=torch.uint8, device=dev)
    rc = load_library().msa_sparse_attend(ctypes.byref(cfg), _ptr(q), B, M, _ptr(K), _ptr(V), _ptr(idx), k,
                                          _ptr(Kloc), _ptr(Vloc), Lloc, local_pos0, _ptr(q_pos), _ptr(out),
                                          _ptr(lse), _ptr(workspace), workspace.numel(), _stream(stream, dev))
    _check(rc, "msa_sparse_attend")
    return out, lse


def fetch_slots(cfg, B, M, k):
    return load_library().msa_fetch_slots(ctypes.byref(cfg), B, M, k)


def msa_fetch_selected(cfg, K_host, V_host, idx, B, M, K_stage=None, V_stage=None, idx_stage=None,
                       lens_stage=None, stream=None):
    """K_host, V_host: pinned host bf16 [N][Hkv][G][d]; idx: device int32 [B][M'][S][k] ->
    (K_stage, V_stage device bf16 [n_slots][Hkv][G][d], idx_stage device int32 like idx, staging config; the
    staging config carries lens_stage as its doc_lens when cfg has doc_lens)."""
    if not (K_host.is_pinned() and V_host.is_pinned() and K_host.dtype == torch.bfloat16 and
            V_host.dtype == torch.bfloat16 and K_host.is_contiguous() and V_host.is_contiguous()):
        raise ValueError("K_host, V_host: expected contiguous pinned host tensors of torch.bfloat16")
    _need(idx, torch.int32, "idx")
    k = idx.shape[-1]
    n_slots = fetch_slots(cfg, B, M, k)
    shape = (n_slots, cfg.n_kv_heads, cfg.doc_len, cfg.head_dim)
    dev = idx.device
    if K_stage is None:
        K_stage = torch.empty(shape, dtype=torch.bfloat16, device=dev)
    if V_stage is None:
        V_stage = torch.empty(shape, dtype=torch.bfloat16, device=dev)
    if idx_stage is None:
        idx_stage = torch.empty_like(idx)
    if cfg.doc_lens_tensor is not None and lens_stage is None:
        lens_stage = torch.empty(n_slots, dtype=torch.int32, device=dev)
    rc = load_library().msa_fetch_selected(ctypes.byref(cfg), _ptr(K_host), _ptr(V_host), _ptr(idx), B, M, k,
                                           _ptr(K_stage), _ptr(V_stage), _ptr(idx_stage), _ptr(lens_stage),
                                           _stream(stream, dev))
    _check(rc, "msa_fetch_selected")
    scfg = cfg.replace(n_docs=n_slots, doc_lens=lens_stage if cfg.doc_lens_tensor is not None else None)
    return K_stage, V_stage, idx_stage, scfg
