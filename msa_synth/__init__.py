"""Seeded synthetic inputs for the MSA hot path (host side).

This package holds NO arithmetic of the method: it only produces reproducible bfloat16 tensors
(standard-normal values) that both the GPU library's tests/bench and the CPU oracle's tests consume.
A tensor is defined element by element by a counter-based generator, so any slice of a bank that is
too large for host memory (tens of GiB) can be regenerated on the host on demand, and the device
fill kernel (msa_synth/csrc/synth_fill.hip) writes the same bits in place:

    word(e)  = splitmix64_finalize(seed * 0x9E3779B97F4A7C15 + (e >> 2))      (64-bit, wrapping)
    index(e) = (word(e) >> (16 * (e & 3))) & 0xFFFF
    value(e) = QUANTILE_TABLE[index(e)]                                       (bfloat16 bits)

QUANTILE_TABLE[i] is the standard-normal quantile at (i + 0.5) / 65536 rounded to bfloat16
(round to nearest even), built once in float64.
"""
import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)

_table_cache = None


def f64_to_bf16_bits(x):
    """float64 array -> uint16 bfloat16 bit patterns, round to nearest even (normal range)."""
    x = np.asarray(x, dtype=np.float64)
    m, e = np.frexp(x)
    q = np.rint(np.ldexp(x, 8 - e))
    y = np.ldexp(q, e - 8).astype(np.float32)          # exact: 8 significant bits
    return (y.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f64(bits):
    """uint16 bfloat16 bit patterns -> float64 values (exact)."""
    bits = np.asarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def quantile_table():
    """65536 bfloat16 bit patterns: normal quantiles at (i + 0.5) / 65536."""
    global _table_cache
    if _table_cache is None:
        from scipy.special import ndtri
        p = (np.arange(65536, dtype=np.float64) + 0.5) / 65536.0
        _table_cache = f64_to_bf16_bits(ndtri(p))
    return _table_cache


def _mix64(z):
    z = z.copy()
    z ^= z >> np.uint64(30)
    z *= _M1
    z ^= z >> np.uint64(27)
    z *= _M2
    z ^= z >> np.uint64(31)
    return z


def normal_bf16_bits(seed, start, count):
    """bfloat16 bit patterns of elements [start, start + count) of the tensor with this seed."""
    start = int(start)
    count = int(count)
    if count == 0:
        return np.zeros(0, dtype=np.uint16)
    w0, w1 = start >> 2, (start + count + 3) >> 2            # 64-bit words covering the range
    with np.errstate(over="ignore"):
        base = np.uint64(seed) * _GOLDEN
        word = _mix64(base + np.arange(w0, w1, dtype=np.uint64))
    idx = np.empty((w1 - w0, 4), dtype=np.uint16)
    for lane in range(4):
        idx[:, lane] = (word >> np.uint64(16 * lane)).astype(np.uint16)   # truncation keeps 16 bits
    idx = idx.reshape(-1)[start - 4 * w0: start - 4 * w0 + count]
    return quantile_table()[idx]


def normal_bf16(seed, shape, start=0):
    """(bits uint16, values float64) of a tensor of this shape whose flat element 0 is element
    `start` of the seeded stream."""
    n = int(np.prod(shape))
    bits = normal_bf16_bits(seed, start, n).reshape(shape)
    return bits, bf16_bits_to_f64(bits)


def doc_slice(seed, n_kv_heads, doc_len, head_dim, doc):
    """Document `doc` of a bank laid out [N][Hkv][G][d]: (bits, float64) of shape [Hkv, G, d]."""
    per_doc = n_kv_heads * doc_len * head_dim
    return normal_bf16(seed, (n_kv_heads, doc_len, head_dim), start=doc * per_doc)


def seed_for(cfg_id, tensor_id):
    """Seed convention: 1000 * config number + tensor id (K=0, V=1, q=2, Kloc=3, Vloc=4)."""
    return 1000 * int(cfg_id) + int(tensor_id)
