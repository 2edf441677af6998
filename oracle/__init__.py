"""CPU oracle for DistAttention decode attention: TEST INFRASTRUCTURE ONLY.

A thin ctypes loader over ``oracle/da_oracle.c`` (fp64, plain loops).  Only the
tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import this
package; the product path never does.  It shares nothing with the HIP library.

Arrays are numpy: fp32 data as ``float32``, bf16 data as ``uint16`` holding the
raw bit patterns.  Pools are addressed as
``pool[pb*stride_block + g*stride_head + slot*stride_token + c]`` in elements.

  attention()        Section 4, Eq. 1 (plain definition, two passes)
  micro_attention()  Section 4, m_j / e_j equation and Eq. 2
  aggregate()        Section 4, m_g / e_g equation and Eq. 3
  append()           Section 4: a new token's K/V rows join the block layout
  move_blocks()      Section 5.3, move_kvcache of Algorithm 1: whole KV blocks go from one pool to another
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "da_oracle.c")
_LIB = os.path.join(_HERE, "libda_oracle.so")

F32, BF16, F16 = 0, 1, 2


def build(force=False):
    """Compile the oracle with gcc (plain -O2, OpenMP only to spread (request, head) pairs)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Problem(ctypes.Structure):
    _fields_ = [
        ("q", ctypes.c_void_p), ("k_pool", ctypes.c_void_p), ("v_pool", ctypes.c_void_p),
        ("block_table", ctypes.c_void_p), ("seq_lens", ctypes.c_void_p),
        ("q_dtype", ctypes.c_int), ("kv_dtype", ctypes.c_int),
        ("B", ctypes.c_int), ("Hq", ctypes.c_int), ("Hkv", ctypes.c_int), ("d", ctypes.c_int),
        ("T", ctypes.c_int), ("max_blocks", ctypes.c_int),
        ("stride_block", ctypes.c_int64), ("stride_head", ctypes.c_int64),
        ("stride_token", ctypes.c_int64),
        ("scale", ctypes.c_double),
        ("q_len", ctypes.c_int),
    ]


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_attention.restype = ctypes.c_int
        _lib.oracle_attention.argtypes = [ctypes.POINTER(_Problem), ctypes.c_void_p, ctypes.c_int64,
                                          ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int]
        _lib.oracle_micro_attention.restype = ctypes.c_int
        _lib.oracle_micro_attention.argtypes = [ctypes.POINTER(_Problem), ctypes.c_void_p, ctypes.c_void_p,
                                                ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int]
        _lib.oracle_aggregate.restype = ctypes.c_int
        _lib.oracle_aggregate.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
                                          ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                          ctypes.c_void_p, ctypes.c_void_p]
        _lib.oracle_append.restype = ctypes.c_int
        _lib.oracle_append.argtypes = [ctypes.c_void_p] * 6 + [ctypes.c_int] * 7 + [ctypes.c_int64] * 3
        _lib.oracle_move_blocks.restype = ctypes.c_int
        _lib.oracle_move_blocks.argtypes = [ctypes.c_void_p] * 6 + [ctypes.c_int] * 7 + [ctypes.c_int64] * 6
    return _lib


def _dtype_code(a):
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    if a.dtype == np.float16:
        return F16
    raise TypeError("oracle takes float32, float16 or uint16 (bf16 bits), got %s" % a.dtype)


def _pool_strides(a):
    """Element strides (block, head, token) of a pool array if the oracle can address it in place, else None."""
    if a.strides[3] != a.itemsize or any(s <= 0 or s % a.itemsize for s in a.strides[:3]):
        return None
    return tuple(s // a.itemsize for s in a.strides[:3])


def _problem(q, k_pool, v_pool, block_table, seq_lens, block_tokens, scale, keep):
    q_len = 1
    if q.ndim == 4:  # multi-query form [B][q_len][Hq][d]
        q_len = q.shape[1]
        q = q.reshape(q.shape[0], q_len * q.shape[2], q.shape[3])
    B, Hq, d = q.shape
    Hq //= q_len
    if k_pool.ndim != 4 or v_pool.shape != k_pool.shape:
        raise ValueError("pools must be [num_phys_blocks][Hkv][T][d]")
    _, Hkv, T, dd = k_pool.shape
    if dd != d or T != block_tokens:
        raise ValueError("pool shape does not match q / block_tokens")
    # Pools may be views with any positive (block, head, token) strides and contiguous rows, e.g. the K and V
    # halves of one [P][2][Hkv][T][d] array or pools with padded rows: they are read in place through their
    # strides (both pools must then share them); anything else is copied to the packed layout first.
    strides = _pool_strides(k_pool)
    if strides is None or _pool_strides(v_pool) != strides:
        k_pool = np.ascontiguousarray(k_pool)
        v_pool = np.ascontiguousarray(v_pool)
        strides = (Hkv * T * d, T * d, d)
    q = np.ascontiguousarray(q)
    block_table = np.ascontiguousarray(block_table, dtype=np.int32)
    seq_lens = np.ascontiguousarray(seq_lens, dtype=np.int32)
    if _dtype_code(k_pool) != _dtype_code(v_pool):
        raise TypeError("K and V pools must share a dtype")
    keep.extend([q, k_pool, v_pool, block_table, seq_lens])
    p = _Problem()
    p.q, p.k_pool, p.v_pool = q.ctypes.data, k_pool.ctypes.data, v_pool.ctypes.data
    p.block_table, p.seq_lens = block_table.ctypes.data, seq_lens.ctypes.data
    p.q_dtype, p.kv_dtype = _dtype_code(q), _dtype_code(k_pool)
    p.B, p.Hq, p.Hkv, p.d, p.T = B, Hq, Hkv, d, T
    p.max_blocks = block_table.shape[1]
    p.stride_block, p.stride_head, p.stride_token = strides
    p.scale = float(scale)
    p.q_len = q_len
    return p


def attention(q, k_pool, v_pool, block_table, seq_lens, block_tokens, scale,
              pairs=None, n_threads=1):
    """Eq. 1.  Returns (out, lse) in fp64: [B][Hq][d], [B][Hq]; or [n][d], [n] for ``pairs`` (n x 2: r, h).

    q may also be [B][q_len][Hq][d] (several new tokens per request, causal among them): outputs are then
    [B][q_len][Hq][d], [B][q_len][Hq], and a pair's second entry is the virtual head t * Hq + h."""
    keep = []
    p = _problem(q, k_pool, v_pool, block_table, seq_lens, block_tokens, scale, keep)
    if pairs is None:
        n = p.B * p.Hq * p.q_len
        pairs_ptr = None
    else:
        pairs = np.ascontiguousarray(pairs, dtype=np.int32).reshape(-1, 2)
        n = pairs.shape[0]
        pairs_ptr = pairs.ctypes.data
    out = np.empty((n, p.d), dtype=np.float64)
    lse = np.empty((n,), dtype=np.float64)
    rc = _load().oracle_attention(ctypes.byref(p), pairs_ptr, n, out.ctypes.data, lse.ctypes.data, n_threads)
    if rc != 0:
        raise ValueError("oracle_attention rejected its arguments")
    if pairs is None:
        if p.q_len > 1 or q.ndim == 4:
            return out.reshape(p.B, p.q_len, p.Hq, p.d), lse.reshape(p.B, p.q_len, p.Hq)
        return out.reshape(p.B, p.Hq, p.d), lse.reshape(p.B, p.Hq)
    return out, lse


def micro_attention(q, k_pool, v_pool, block_table, seq_lens, block_tokens, scale, bounds,
                    n_threads=1):
    """Eq. 2 over caller-chosen partitions.

    ``bounds[r]`` is the increasing list of token boundaries of request r
    (len = nparts[r] + 1).  Returns (MA [rows][d], m [rows], e [rows], nparts [B]) with
    row(r, h, j) = Hq * sum_{r'<r} nparts[r'] + h * nparts[r] + j.
    """
    keep = []
    p = _problem(q, k_pool, v_pool, block_table, seq_lens, block_tokens, scale, keep)
    nparts = np.array([len(b) - 1 for b in bounds], dtype=np.int32)
    flat = np.ascontiguousarray(np.concatenate([np.asarray(b, dtype=np.int64) for b in bounds]))
    rows = int(nparts.sum()) * p.Hq * p.q_len
    MA = np.empty((rows, p.d), dtype=np.float64)
    m = np.empty((rows,), dtype=np.float64)
    e = np.empty((rows,), dtype=np.float64)
    rc = _load().oracle_micro_attention(ctypes.byref(p), nparts.ctypes.data, flat.ctypes.data,
                                        MA.ctypes.data, m.ctypes.data, e.ctypes.data, n_threads)
    if rc != 0:
        raise ValueError("oracle_micro_attention rejected its arguments")
    return MA, m, e, nparts


def aggregate(MA, m, e, nparts, num_q_heads):
    """Eq. 3.  Returns (out [B][Hq][d], lse [B][Hq]) in fp64."""
    MA = np.ascontiguousarray(MA, dtype=np.float64)
    m = np.ascontiguousarray(m, dtype=np.float64)
    e = np.ascontiguousarray(e, dtype=np.float64)
    nparts = np.ascontiguousarray(nparts, dtype=np.int32)
    B, d = nparts.shape[0], MA.shape[1]
    out = np.empty((B, num_q_heads, d), dtype=np.float64)
    lse = np.empty((B, num_q_heads), dtype=np.float64)
    rc = _load().oracle_aggregate(B, num_q_heads, d, nparts.ctypes.data, MA.ctypes.data, m.ctypes.data,
                                  e.ctypes.data, out.ctypes.data, lse.ctypes.data)
    if rc != 0:
        raise ValueError("oracle_aggregate rejected its arguments")
    return out, lse


def append(k_new, v_new, k_pool, v_pool, block_table, seq_lens):
    """KV append in place: writes the new rows into the (contiguous, writable) numpy pools and bumps seq_lens.

    k_new / v_new: [B][Hkv][d]; pools [P][Hkv][T][d]; block_table int32 [B][max_blocks]; seq_lens int32 [B]."""
    B, Hkv, d = k_new.shape
    P, Hkv2, T, d2 = k_pool.shape
    assert (Hkv2, d2) == (Hkv, d) and v_pool.shape == k_pool.shape and v_new.shape == k_new.shape
    assert k_pool.dtype == k_new.dtype == v_pool.dtype == v_new.dtype and _dtype_code(k_pool) in (F32, BF16, F16)
    for a in (k_pool, v_pool, seq_lens):
        assert a.flags["C_CONTIGUOUS"] and a.flags["WRITEABLE"]
    assert block_table.dtype == np.int32 and seq_lens.dtype == np.int32 and block_table.flags["C_CONTIGUOUS"]
    k_new = np.ascontiguousarray(k_new)
    v_new = np.ascontiguousarray(v_new)
    rc = _load().oracle_append(k_new.ctypes.data, v_new.ctypes.data, k_pool.ctypes.data, v_pool.ctypes.data,
                               block_table.ctypes.data, seq_lens.ctypes.data, B, Hkv, d, T, block_table.shape[1], P,
                               k_pool.itemsize, Hkv * T * d, T * d, d)
    if rc != 0:
        raise ValueError("oracle_append rejected its arguments")


def move_blocks(k_src, v_src, k_dst, v_dst, src_ids, dst_ids):
    """Copies blocks src_ids[i] of the source pools to blocks dst_ids[i] of the (writable) destination pools.

    Pools are contiguous numpy arrays [P][Hkv][T][d] of one dtype; ids are int32 arrays of equal length; a pair
    with an id outside its pool is skipped."""
    Ps, Hkv, T, d = k_src.shape
    Pd = k_dst.shape[0]
    assert k_dst.shape[1:] == (Hkv, T, d) and v_src.shape == k_src.shape and v_dst.shape == k_dst.shape
    assert k_src.dtype == v_src.dtype == k_dst.dtype == v_dst.dtype
    for a in (k_src, v_src, k_dst, v_dst):
        assert a.flags["C_CONTIGUOUS"]
    assert k_dst.flags["WRITEABLE"] and v_dst.flags["WRITEABLE"]
    src_ids = np.ascontiguousarray(src_ids, dtype=np.int32)
    dst_ids = np.ascontiguousarray(dst_ids, dtype=np.int32)
    assert src_ids.shape == dst_ids.shape and src_ids.ndim == 1
    rc = _load().oracle_move_blocks(k_src.ctypes.data, v_src.ctypes.data, k_dst.ctypes.data, v_dst.ctypes.data,
                                    src_ids.ctypes.data, dst_ids.ctypes.data, len(src_ids), Hkv, d, T, k_src.itemsize,
                                    Ps, Pd, Hkv * T * d, T * d, d, Hkv * T * d, T * d, d)
    if rc != 0:
        raise ValueError("oracle_move_blocks rejected its arguments")
