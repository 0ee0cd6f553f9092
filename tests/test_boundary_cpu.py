"""Host-side checks of the C-ABI boundary that need no GPU: the library loads and exports every
symbol the header declares, every argument-validation path returns its status before any launch,
and the size helpers reproduce the closed forms (including the paper's printed memory estimate)."""
import ctypes
import os
import re

import pytest

import paper_2603_23516_amd as msa

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(msa.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return msa.load_library()


def _cfg(**kw):
    base = dict(n_docs=64, doc_len=512, chunk=64, n_q_heads=8, n_kv_heads=2, head_dim=64, rope_base=1e4)
    base.update(kw)
    return msa.MsaConfig(**base)


def test_exports_match_header(lib):
    text = open(os.path.join(ROOT, "include", "msa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(msa_[a-z_0-9]+)\s*\(", text))
    assert declared == set(msa.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert lib.msa_version() == 105
    for st in (0, -1, -2, -3, -4, -5, -99):
        assert len(msa.status_string(st)) > 0


def test_profile_events_are_per_call_config_fields(lib):
    """The timing aid is a pair of fields of the per-call config (no library state): one event without the other is
    refused by every entry point that reads the config, before anything is enqueued."""
    p = ctypes.c_void_p(0x10000)
    c = _cfg()
    c.profile_start_event = 16
    assert lib.msa_score_topk(ctypes.byref(c), p, 1, 1, p, p, 4, p, p, p, 1 << 30, None) == msa.MSA_ERR_INVALID_ARG
    c.profile_start_event, c.profile_stop_event = None, 16
    assert lib.msa_score_topk(ctypes.byref(c), p, 1, 1, p, p, 4, p, p, p, 1 << 30, None) == msa.MSA_ERR_INVALID_ARG
    assert msa.score_topk_workspace_bytes(c, 1, 1, 4) == 0
    c.profile_start_event = 32
    assert msa.score_topk_workspace_bytes(c, 1, 1, 4) > 0          # a complete pair is a valid config
    assert not hasattr(lib, "msa_profile_dominant_kernel") or "msa_profile_dominant_kernel" not in msa.EXPORTS


def test_sizes_and_paper_estimate(lib):
    c = _cfg()
    assert msa.routing_keys_bytes(c) == 2 * (64 * 8) * 64 * 2             # Hkv * N*C * d * 2 B
    assert msa.inv_norm_bytes(c) == 2 * (64 * 8) * 4
    c5 = _cfg(n_docs=97656, n_q_heads=32, n_kv_heads=8, head_dim=128)
    assert msa.routing_keys_bytes(c5) == 8 * 781248 * 128 * 2              # ~1.6 GB
    odd = _cfg(n_docs=3, doc_len=64, chunk=32)                             # 6 keys -> one padded tile
    assert msa.routing_keys_bytes(odd) == 2 * 16 * 64 * 2
    # paper, Section 3.4.2: about 169 GB for K-bar, V-bar and routing keys, ~56 GB for routing keys
    line = [l for l in open(os.path.join(ROOT, "tests", "golden", "paper_memory_estimate.txt"))
            if not l.startswith("#")][0]
    tokens, P, heads, d, layers, bpe, total_gb, routing_gb = (int(x) for x in line.split())
    total = msa.pooled_bank_bytes(tokens, P, heads, d, layers, bpe, 3)
    routing = msa.pooled_bank_bytes(tokens, P, heads, d, layers, bpe, 1)
    assert total == int(168.75 * 2 ** 30) and routing == int(56.25 * 2 ** 30)
    assert round(total / 2 ** 30) == total_gb and round(routing / 2 ** 30) == routing_gb
    assert msa.pooled_bank_bytes(100, 64, 8, 128, 18, 2, 3) == 0           # tokens % P != 0


def test_workspace_sizes(lib):
    c = _cfg(n_docs=2048, n_q_heads=32, n_kv_heads=8, head_dim=128, rope_base=1e6)
    w = msa.score_topk_workspace_bytes(c, 1, 1, 16)
    assert w > 0 and w % 256 == 0
    assert msa.score_topk_workspace_bytes(c, 1, 1, 0) == 0
    assert msa.score_topk_workspace_bytes(c, 1, 1, 65) == 0
    assert msa.score_topk_workspace_bytes(c, 1, 1, 4096) == 0
    wa = msa.sparse_attend_workspace_bytes(c, 1, 1, 16, 2048)
    assert wa > 0 and wa % 256 == 0
    assert msa.sparse_attend_workspace_bytes(c, 1, 1, 16, -1) == 0
    assert msa.sparse_attend_workspace_bytes(_cfg(doc_len=48, chunk=16), 1, 1, 4, 0) == 0   # G % 32


def test_config_validation(lib):
    bad = [
        (dict(n_docs=0), msa.MSA_ERR_INVALID_ARG),
        (dict(doc_len=500), msa.MSA_ERR_INVALID_ARG),                 # G % P != 0
        (dict(n_q_heads=7), msa.MSA_ERR_INVALID_ARG),                 # Hq % Hkv != 0
        (dict(sim=5), msa.MSA_ERR_INVALID_ARG),
        (dict(rope_base=1.0), msa.MSA_ERR_INVALID_ARG),
        (dict(head_dim=96), msa.MSA_ERR_UNSUPPORTED),
        (dict(chunk=4, doc_len=32), msa.MSA_ERR_UNSUPPORTED),         # P % 8 != 0
        (dict(doc_len=64 * 12), msa.MSA_ERR_UNSUPPORTED),             # C = 12
        (dict(doc_len=64 * 32), msa.MSA_ERR_UNSUPPORTED),             # C = 32
        (dict(n_q_heads=32, n_kv_heads=2), msa.MSA_ERR_UNSUPPORTED),  # r = 16
        (dict(select_scope=msa.MSA_SCOPE_ALL, n_q_heads=6, n_kv_heads=3), msa.MSA_ERR_UNSUPPORTED),
        (dict(select_scope=7), msa.MSA_ERR_INVALID_ARG),
        (dict(token_pool=2), msa.MSA_ERR_INVALID_ARG),
    ]
    p = ctypes.c_void_p(0x10000)
    for kw, want in bad:
        c = _cfg(**kw)
        assert lib.msa_build_routing_keys(ctypes.byref(c), p, 0, 1, p, p, None) == want, kw
        assert msa.routing_keys_bytes(c) == 0
    assert lib.msa_build_routing_keys(None, p, 0, 1, p, p, None) == msa.MSA_ERR_INVALID_ARG


def test_argument_validation_before_launch(lib):
    c = _cfg()
    cb = ctypes.byref(c)
    p = ctypes.c_void_p(0x10000)
    odd = ctypes.c_void_p(0x10008)
    big = 1 << 30
    E = msa
    # build
    assert lib.msa_build_routing_keys(cb, None, 0, 1, p, p, None) == E.MSA_ERR_INVALID_ARG
    assert lib.msa_build_routing_keys(cb, p, 0, 1, None, p, None) == E.MSA_ERR_INVALID_ARG
    assert lib.msa_build_routing_keys(cb, p, 0, 1, p, None, None) == E.MSA_ERR_INVALID_ARG   # cosine needs inv_norm
    assert lib.msa_build_routing_keys(cb, p, -1, 1, p, p, None) == E.MSA_ERR_INVALID_ARG
    assert lib.msa_build_routing_keys(cb, p, 60, 5, p, p, None) == E.MSA_ERR_INVALID_ARG
    assert lib.msa_build_routing_keys(cb, odd, 0, 1, p, p, None) == E.MSA_ERR_MISALIGNED
    # score
    assert lib.msa_score_topk(cb, None, 1, 1, p, p, 4, p, p, p, big, None) == E.MSA_ERR_INVALID_ARG
    assert lib.msa_score_topk(cb, p, 1, 1, p, None, 4, p, p, p, big, None) == E.MSA_ERR_INVALID_ARG
    assert lib.msa_score_topk(cb, p, 0, 1, p, p, 4, p, p, p, big, None) == E.MSA_ERR_INVALID_ARG
    assert lib.msa_score_topk(cb, p, 1, 1, p, p, 0, p, p, p, big, None) == E.MSA_ERR_INVALID_ARG
    assert lib.msa_score_topk(cb, p, 1, 1, p, p, 65, p, p, p, big, None) == E.MSA_ERR_INVALID_ARG   # k > N = 64
    c2 = _cfg(n_docs=1000)
    assert lib.msa_score_topk(ctypes.byref(c2), p, 1, 1, p, p, 65, p, p, p, big, None) == E.MSA_ERR_UNSUPPORTED
    assert lib.msa_score_topk(cb, p, 1, 1, odd, p, 4, p, p, p, big, None) == E.MSA_ERR_MISALIGNED
    assert lib.msa_score_topk(cb, p, 1, 1, p, p, 4, p, p, p, 16, None) == E.MSA_ERR_WORKSPACE
    assert lib.msa_score_topk(cb, p, 1, 1, p, p, 4, p, p, None, big, None) == E.MSA_ERR_INVALID_ARG
    # attend
    args = [cb, p, 1, 1, p, p, p, 4, p, p, 256, 512, p, p, p, p, big, None]

    def call(**repl):
        a = list(args)
        for i, v in repl.items():
            a[int(i[1:])] = v
        return lib.msa_sparse_attend(*a)
    assert call(a1=None) == E.MSA_ERR_INVALID_ARG           # q
    assert call(a6=None) == E.MSA_ERR_INVALID_ARG           # idx
    assert call(a8=None) == E.MSA_ERR_INVALID_ARG           # Kloc null with Lloc > 0
    assert call(a12=None) == E.MSA_ERR_INVALID_ARG          # q_pos
    assert call(a7=0) == E.MSA_ERR_INVALID_ARG              # k
    assert call(a10=-1) == E.MSA_ERR_INVALID_ARG            # Lloc
    assert call(a7=65) == E.MSA_ERR_UNSUPPORTED
    assert call(a4=odd) == E.MSA_ERR_MISALIGNED
    assert call(a16=64) == E.MSA_ERR_WORKSPACE
    c3 = _cfg(doc_len=48, chunk=8 * 3)                      # C = 2, G % 32 != 0
    a = list(args)
    a[0] = ctypes.byref(c3)
    assert lib.msa_sparse_attend(*a) == E.MSA_ERR_UNSUPPORTED
    # pooled bank: short documents are read only when the bank's keys are stored rotated
    for G, rot, want in ((8, 1, E.MSA_ERR_WORKSPACE), (8, 0, E.MSA_ERR_UNSUPPORTED), (1, 1, E.MSA_ERR_WORKSPACE),
                         (24, 1, E.MSA_ERR_UNSUPPORTED), (64, 1, E.MSA_ERR_WORKSPACE), (8, 2, E.MSA_ERR_INVALID_ARG)):
        cp = _cfg(doc_len=G, chunk=G, bank_keys_rotated=rot)
        a = list(args)
        a[0] = ctypes.byref(cp)
        a[16] = 64                                          # valid requests get as far as the workspace check
        assert lib.msa_sparse_attend(*a) == want, (G, rot)
    assert msa.sparse_attend_workspace_bytes(_cfg(doc_len=8, chunk=8, bank_keys_rotated=1), 1, 1, 16, 100) > 0
    assert msa.sparse_attend_workspace_bytes(_cfg(doc_len=8, chunk=8), 1, 1, 16, 100) == 0
    # pool_kv
    assert lib.msa_pool_kv(cb, None, p, 0, 1, p, p, None, None) == E.MSA_ERR_INVALID_ARG      # Kbar wanted, no K
    assert lib.msa_pool_kv(cb, p, None, 0, 1, p, p, None, None) == E.MSA_ERR_INVALID_ARG
    assert lib.msa_pool_kv(cb, p, p, 60, 5, p, p, None, None) == E.MSA_ERR_INVALID_ARG
    assert lib.msa_pool_kv(cb, p, p, -1, 1, p, p, None, None) == E.MSA_ERR_INVALID_ARG
    assert lib.msa_pool_kv(cb, p, odd, 0, 1, p, p, None, None) == E.MSA_ERR_MISALIGNED
    assert lib.msa_pool_kv(cb, p, p, 0, 0, p, p, None, None) == E.MSA_OK                      # nothing to do, nothing launched
    assert lib.msa_pool_kv(ctypes.byref(_cfg(head_dim=96)), p, p, 0, 1, p, p, None, None) == E.MSA_ERR_UNSUPPORTED


def test_noalloc_entry_point_validation(lib):
    """The entry point on the built-in scratch buffer validates like msa_score_topk and refuses a request
    beyond its buffer before it touches a device."""
    E = msa
    c = _cfg()
    cb = ctypes.byref(c)
    p = ctypes.c_void_p(0x10000)
    odd = ctypes.c_void_p(0x10008)
    f = lib.msa_score_topk_noalloc
    assert msa.noalloc_scratch_bytes() == 32 << 20
    assert f(cb, None, 1, 1, p, p, 4, p, p, None) == E.MSA_ERR_INVALID_ARG
    assert f(cb, p, 1, 1, p, None, 4, p, p, None) == E.MSA_ERR_INVALID_ARG       # cosine needs inv_norm
    assert f(cb, p, 1, 1, p, p, 4, None, p, None) == E.MSA_ERR_INVALID_ARG
    assert f(cb, p, 0, 1, p, p, 4, p, p, None) == E.MSA_ERR_INVALID_ARG
    assert f(cb, p, 1, 1, p, p, 65, p, p, None) == E.MSA_ERR_INVALID_ARG         # k > N
    assert f(cb, p, 1, 1, odd, p, 4, p, p, None) == E.MSA_ERR_MISALIGNED
    assert f(None, p, 1, 1, p, p, 4, p, p, None) == E.MSA_ERR_INVALID_ARG
    # 8192 query tokens against 64K documents: folded queries plus candidate lists exceed 32 MiB
    big = _cfg(n_docs=65536, n_q_heads=32, n_kv_heads=8, head_dim=128)
    assert msa.score_topk_workspace_bytes(big, 1, 8192, 8) > msa.noalloc_scratch_bytes()
    assert f(ctypes.byref(big), p, 1, 8192, p, p, 8, p, p, None) == E.MSA_ERR_WORKSPACE
    # the five benchmark configurations fit
    for N, B, M, k in ((2048, 1, 1, 16), (8192, 32, 1, 16), (32768, 1, 2048, 8), (97656, 8, 1, 32)):
        cc = _cfg(n_docs=N, n_q_heads=32, n_kv_heads=8, head_dim=128)
        assert 0 < msa.score_topk_workspace_bytes(cc, B, M, k) <= msa.noalloc_scratch_bytes(), N


def test_fetch_validation(lib):
    c = _cfg()
    cb = ctypes.byref(c)
    p = ctypes.c_void_p(0x10000)
    odd = ctypes.c_void_p(0x10008)
    E = msa
    assert msa.fetch_slots(c, 2, 5, 4) == 2 * 5 * 4
    assert msa.fetch_slots(_cfg(token_pool=1), 2, 5, 4) == 2 * 4
    assert msa.fetch_slots(c, 2, 5, 65) == 0
    f = lib.msa_fetch_selected
    assert f(cb, None, p, p, 1, 1, 4, p, p, p, None, None) == E.MSA_ERR_INVALID_ARG
    assert f(cb, p, p, None, 1, 1, 4, p, p, p, None, None) == E.MSA_ERR_INVALID_ARG
    assert f(cb, p, p, p, 1, 1, 4, p, p, None, None, None) == E.MSA_ERR_INVALID_ARG
    assert f(cb, p, p, p, 0, 1, 4, p, p, p, None, None) == E.MSA_ERR_INVALID_ARG
    assert f(cb, p, p, p, 1, 1, 65, p, p, p, None, None) == E.MSA_ERR_UNSUPPORTED
    assert f(cb, odd, p, p, 1, 1, 4, p, p, p, None, None) == E.MSA_ERR_MISALIGNED
    # document lengths: a length per staging slot is an output, and needs one document per slot
    ca = _cfg(select_scope=msa.MSA_SCOPE_ALL)
    ca.doc_lens = 0x20000
    assert f(ctypes.byref(ca), p, p, p, 1, 1, 4, p, p, p, None, None) == E.MSA_ERR_INVALID_ARG
    cg = _cfg()
    cg.doc_lens = 0x20000
    assert f(ctypes.byref(cg), p, p, p, 1, 1, 4, p, p, p, p, None) == E.MSA_ERR_UNSUPPORTED
    ca.doc_lens = 0x20002
    assert f(ctypes.byref(ca), p, p, p, 1, 1, 4, p, p, p, p, None) == E.MSA_ERR_MISALIGNED
    # a bank that is not pinned, device-mapped host memory is refused before anything is launched
    assert f(cb, p, p, p, 1, 1, 4, p, p, p, None, None) == E.MSA_ERR_INVALID_ARG


def test_literal_eq2_variants_are_planned(lib):
    """select_scope = ALL and token_pool = 1 are valid requests with their own workspace sizes."""
    base = msa.score_topk_workspace_bytes(_cfg(), 2, 5, 4)
    pooled = msa.score_topk_workspace_bytes(_cfg(token_pool=1), 2, 5, 4)
    assert pooled >= base + 2 * 5 * 2 * 4 * 8                       # + per-token winner keys [B*M][Hkv][k]
    assert msa.score_topk_workspace_bytes(_cfg(select_scope=msa.MSA_SCOPE_ALL), 2, 5, 4) > 0
    assert msa.score_topk_workspace_bytes(_cfg(select_scope=msa.MSA_SCOPE_ALL, token_pool=1), 2, 5, 4) > 0


def test_binding_refuses_cpu_tensors(lib):
    import torch
    c = _cfg()
    with pytest.raises(ValueError):
        msa.msa_build_routing_keys(c, torch.zeros((64, 2, 512, 64), dtype=torch.bfloat16))


def test_host_sanitizers_on_extreme_sizes():
    """The C-ABI layer's host code (validation, work plans, workspace-size arithmetic) compiled with
    AddressSanitizer + UndefinedBehaviorSanitizer + the integer sanitizer (host side only) and driven by
    tests/csrc/boundary_sanitize.cpp with sizes at the limits: N*C just below 2^31 keys per head, B*M = 2^20,
    k = 64, local contexts of 2^24 tokens.  No device is visible to the driver, so nothing can launch; a valid
    request must come back as MSA_ERR_HIP from the launch stage with no sanitizer report on the way."""
    import glob
    import subprocess
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out_dir = os.path.join(ROOT, "tests", "_build")
    os.makedirs(out_dir, exist_ok=True)
    lib_san = os.path.join(out_dir, "libmsa_san.so")
    exe = os.path.join(out_dir, "boundary_sanitize")
    srcs = sorted(glob.glob(os.path.join(ROOT, "paper_2603_23516_amd", "csrc", "*.hip")))
    deps = srcs + glob.glob(os.path.join(ROOT, "paper_2603_23516_amd", "csrc", "*.h")) + \
        [os.path.join(ROOT, "include", "msa.h"), os.path.join(ROOT, "tests", "csrc", "boundary_sanitize.cpp")]
    san = []
    for f in ("-fsanitize=address", "-fsanitize=undefined", "-fsanitize=integer", "-fno-sanitize-recover=all"):
        san += ["-Xarch_host", f]
    newest = max(os.path.getmtime(f) for f in deps)
    if not (os.path.exists(exe) and os.path.exists(lib_san) and
            min(os.path.getmtime(exe), os.path.getmtime(lib_san)) >= newest):
        common = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
                  "-packed-fp32-ops", "-Wno-unused-command-line-argument"] + san + ["-I", os.path.join(ROOT, "include")]
        r = subprocess.run(common + ["-fPIC", "-shared"] + srcs + ["-o", lib_san], stdout=subprocess.PIPE,
                           stderr=subprocess.STDOUT, text=True, timeout=900)
        assert r.returncode == 0, r.stdout[-3000:]
        r = subprocess.run(common + [os.path.join(ROOT, "tests", "csrc", "boundary_sanitize.cpp"), "-L", out_dir,
                                     "-lmsa_san", "-Wl,-rpath," + out_dir, "-o", exe], stdout=subprocess.PIPE,
                           stderr=subprocess.STDOUT, text=True, timeout=300)
        assert r.returncode == 0, r.stdout[-3000:]
    env = dict(os.environ, HIP_VISIBLE_DEVICES="-1", ROCR_VISIBLE_DEVICES="", ASAN_OPTIONS="detect_leaks=0")
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300, env=env)
    assert r.returncode == 0 and "boundary_sanitize: ok" in r.stdout, r.stdout[-3000:]
