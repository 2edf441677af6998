"""ctypes binding over ``libdistattn.so`` (the C ABI declared in ``include/distattn.h``).

Argument marshalling only: torch tensors supply device pointers and the current
HIP stream; every step of the path runs in the library's kernels.  There is no
fallback: if the library is missing or a call fails, an exception is raised.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdistattn.so")

DA_OK, DA_ERR_INVALID_ARG, DA_ERR_UNSUPPORTED, DA_ERR_WORKSPACE, DA_ERR_HIP, DA_ERR_NO_SPACE = range(6)
DA_F32, DA_BF16, DA_F16 = 0, 1, 2
DA_KERNEL_AUTO, DA_KERNEL_VALU, DA_KERNEL_MFMA = 0, 1, 2

EXPORTS = [
    "da_status_string", "da_plan_schedule", "da_plan_create", "da_plan_update", "da_plan_destroy",
    "da_plan_num_partials", "da_plan_split", "da_plan_nsplits", "da_plan_describe", "da_workspace_bytes", "da_plan_error",
    "da_partial", "da_combine", "da_combine_multi", "da_attention", "da_attention_noalloc", "da_append",
    "da_block_pool_create", "da_block_pool_destroy", "da_block_pool_free_count", "da_block_pool_grow",
    "da_block_pool_release", "da_move_blocks",
]


class DaProblem(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("block_tokens", ctypes.c_int32), ("max_blocks_per_seq", ctypes.c_int32),
        ("num_phys_blocks", ctypes.c_int32), ("kv_dtype", ctypes.c_int32), ("q_dtype", ctypes.c_int32),
        ("scale", ctypes.c_float),
        ("kv_block_stride", ctypes.c_int64), ("kv_head_stride", ctypes.c_int64), ("kv_token_stride", ctypes.c_int64),
        ("q_len", ctypes.c_int32),
    ]


class DaTuning(ctypes.Structure):
    _fields_ = [("blocks_per_split", ctypes.c_int32), ("num_cus", ctypes.c_int32), ("kernel", ctypes.c_int32)]


class DaPartialSet(ctypes.Structure):
    _fields_ = [("plan", ctypes.c_void_p), ("part_o", ctypes.c_void_p), ("part_m", ctypes.c_void_p),
                ("part_e", ctypes.c_void_p)]


class DistAttnError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__("%s: %s" % (what, status_string(status)))


_lib = None


def lib():
    """The loaded C library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("%s is missing: run `python -c 'import __graft_entry__ as g; g.build()'`" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp, i32p, i64p = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64)
        L.da_status_string.restype = ctypes.c_char_p
        L.da_status_string.argtypes = [ctypes.c_int]
        L.da_plan_schedule.argtypes = [ctypes.POINTER(DaProblem), vp, ctypes.POINTER(DaTuning), vp, i64p, i64p, i32p, i32p, i64p]
        L.da_plan_create.argtypes = [ctypes.POINTER(DaProblem), vp, ctypes.POINTER(DaTuning), vp, ctypes.POINTER(vp)]
        L.da_plan_update.argtypes = [vp, vp, vp]
        L.da_plan_destroy.argtypes = [vp]
        L.da_plan_num_partials.argtypes = [vp, i64p]
        L.da_plan_split.argtypes = [vp, ctypes.c_int32, ctypes.c_int32, i64p, i64p]
        L.da_plan_nsplits.argtypes = [vp, ctypes.c_int32, i32p]
        L.da_plan_describe.argtypes = [vp, i32p, i32p, i32p]
        L.da_workspace_bytes.argtypes = [vp, ctypes.POINTER(ctypes.c_size_t)]
        L.da_plan_error.argtypes = [vp, vp, i32p]
        L.da_partial.argtypes = [vp] * 10
        L.da_combine.argtypes = [vp] * 7
        L.da_attention.argtypes = [vp] * 9 + [ctypes.c_size_t, vp]
        L.da_attention_noalloc.argtypes = [vp] * 9
        L.da_combine_multi.argtypes = [vp, ctypes.c_int32, vp, vp, vp]
        L.da_append.argtypes = [ctypes.POINTER(DaProblem)] + [vp] * 8
        L.da_move_blocks.argtypes = [ctypes.POINTER(DaProblem)] * 2 + [vp] * 6 + [ctypes.c_int32, vp, vp]
        L.da_block_pool_create.argtypes = [ctypes.c_int32, ctypes.POINTER(vp)]
        L.da_block_pool_destroy.argtypes = [vp]
        L.da_block_pool_free_count.argtypes = [vp, i32p]
        L.da_block_pool_grow.argtypes = [vp, ctypes.c_int32, ctypes.c_int32, vp, ctypes.c_int32, ctypes.c_int32]
        L.da_block_pool_release.argtypes = [vp, ctypes.c_int32, vp, ctypes.c_int32]
        for name in EXPORTS[1:]:
            getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def status_string(status):
    return lib().da_status_string(int(status)).decode()


def _check(status, what):
    if status != DA_OK:
        raise DistAttnError(status, what)


def _dtype_code(t):
    if t.dtype == torch.float32:
        return DA_F32
    if t.dtype == torch.bfloat16:
        return DA_BF16
    if t.dtype == torch.float16:
        return DA_F16
    raise TypeError("q / K / V must be float32, bfloat16 or float16, got %s" % t.dtype)


def make_problem(q, k_pool, block_table, scale):
    """da_problem for q [B][Hq][d] (or [B][q_len][Hq][d]) and a pool tensor [P][Hkv][T][d] (any strides with a
    contiguous last dim)."""
    q_len = 1
    if q.dim() == 4:
        q_len = q.shape[1]
        B, _, Hq, d = q.shape
    else:
        B, Hq, d = q.shape
    P, Hkv, T, dd = k_pool.shape
    assert dd == d and k_pool.stride(3) == 1 and q.is_contiguous()
    p = DaProblem()
    p.batch, p.num_q_heads, p.num_kv_heads, p.head_dim = B, Hq, Hkv, d
    p.block_tokens, p.max_blocks_per_seq, p.num_phys_blocks = T, block_table.shape[1], P
    p.kv_dtype, p.q_dtype = _dtype_code(k_pool), _dtype_code(q)
    p.scale = float(scale)
    p.kv_block_stride, p.kv_head_stride, p.kv_token_stride = k_pool.stride(0), k_pool.stride(1), k_pool.stride(2)
    p.q_len = q_len
    return p


def _host_i32(seq_lens_host):
    arr = (ctypes.c_int32 * len(seq_lens_host))(*[int(x) for x in seq_lens_host])
    return arr


def plan_schedule(problem, seq_lens_host, blocks_per_split=0, num_cus=0, kernel=DA_KERNEL_AUTO):
    """Host-only schedule (no GPU needed): dict(nsplits, num_items, num_partials, kernel, workgroups,
    max_workgroup_tokens)."""
    B = problem.batch
    lens = _host_i32(seq_lens_host)
    ns = (ctypes.c_int32 * B)()
    items, parts, kern, wgs = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int32(), ctypes.c_int32()
    worst = ctypes.c_int64()
    tuning = DaTuning(blocks_per_split, num_cus, kernel)
    st = lib().da_plan_schedule(ctypes.byref(problem), ctypes.cast(lens, ctypes.c_void_p), ctypes.byref(tuning),
                                ctypes.cast(ns, ctypes.c_void_p), ctypes.byref(items), ctypes.byref(parts),
                                ctypes.byref(kern), ctypes.byref(wgs), ctypes.byref(worst))
    _check(st, "da_plan_schedule")
    return dict(nsplits=list(ns), num_items=items.value, num_partials=parts.value, kernel=kern.value,
                workgroups=wgs.value, max_workgroup_tokens=worst.value)


def _stream_ptr(stream=None):
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


class Plan:
    """Owns a da_plan.  ``seq_lens_host`` is any sequence of ints (the lengths the device seq_lens hold)."""

    def __init__(self, problem, seq_lens_host, blocks_per_split=0, num_cus=0, kernel=DA_KERNEL_AUTO, stream=None):
        self.problem = problem
        self._h = ctypes.c_void_p()
        tuning = DaTuning(blocks_per_split, num_cus, kernel)
        lens = _host_i32(seq_lens_host)
        st = lib().da_plan_create(ctypes.byref(problem), ctypes.cast(lens, ctypes.c_void_p), ctypes.byref(tuning),
                                  _stream_ptr(stream), ctypes.byref(self._h))
        _check(st, "da_plan_create")

    def update(self, seq_lens_host, stream=None):
        lens = _host_i32(seq_lens_host)
        _check(lib().da_plan_update(self._h, ctypes.cast(lens, ctypes.c_void_p), _stream_ptr(stream)), "da_plan_update")

    def update_raw(self, lens_array, stream_ptr):
        """Same as update() with a prebuilt ctypes int32 array and stream pointer (no per-call marshalling)."""
        return lib().da_plan_update(self._h, ctypes.cast(lens_array, ctypes.c_void_p), stream_ptr)

    def close(self):
        if self._h:
            lib().da_plan_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def num_partials(self):
        n = ctypes.c_int64()
        _check(lib().da_plan_num_partials(self._h, ctypes.byref(n)), "da_plan_num_partials")
        return n.value

    @property
    def workspace_bytes(self):
        n = ctypes.c_size_t()
        _check(lib().da_workspace_bytes(self._h, ctypes.byref(n)), "da_workspace_bytes")
        return n.value

    def describe(self):
        """dict(kernel, head_tile, wavefront_splits) of the current schedule."""
        k, t, w = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
        _check(lib().da_plan_describe(self._h, ctypes.byref(k), ctypes.byref(t), ctypes.byref(w)), "da_plan_describe")
        return dict(kernel=k.value, head_tile=t.value, wavefront_splits=w.value)

    def nsplits(self, r):
        n = ctypes.c_int32()
        _check(lib().da_plan_nsplits(self._h, r, ctypes.byref(n)), "da_plan_nsplits")
        return n.value

    def split(self, r, j):
        a, b = ctypes.c_int64(), ctypes.c_int64()
        _check(lib().da_plan_split(self._h, r, j, ctypes.byref(a), ctypes.byref(b)), "da_plan_split")
        return a.value, b.value

    def error_flags(self, stream=None):
        f = ctypes.c_int32()
        _check(lib().da_plan_error(self._h, _stream_ptr(stream), ctypes.byref(f)), "da_plan_error")
        return f.value

    def _out_shape(self):
        p = self.problem
        return (p.batch, p.num_q_heads) if p.q_len <= 1 else (p.batch, p.q_len, p.num_q_heads)

    # ---- launches -------------------------------------------------------------------------
    def partial(self, q, k_pool, v_pool, block_table, seq_lens, part_o=None, part_m=None, part_e=None, stream=None):
        if part_o is None:
            n = self.num_partials
            dev = k_pool.device
            part_o = torch.empty((n, self.problem.head_dim), dtype=torch.float32, device=dev)
            part_m = torch.empty((n,), dtype=torch.float32, device=dev)
            part_e = torch.empty((n,), dtype=torch.float32, device=dev)
        st = lib().da_partial(self._h, _ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(block_table), _ptr(seq_lens),
                              _ptr(part_o), _ptr(part_m), _ptr(part_e), _stream_ptr(stream))
        _check(st, "da_partial")
        return part_o, part_m, part_e

    def combine(self, part_o, part_m, part_e, out=None, lse=None, stream=None):
        p = self.problem
        if out is None:
            out = torch.empty(self._out_shape() + (p.head_dim,), dtype=torch.float32, device=part_o.device)
            lse = torch.empty(self._out_shape(), dtype=torch.float32, device=part_o.device)
        st = lib().da_combine(self._h, _ptr(part_o), _ptr(part_m), _ptr(part_e), _ptr(out), _ptr(lse),
                              _stream_ptr(stream))
        _check(st, "da_combine")
        return out, lse

    def attention(self, q, k_pool, v_pool, block_table, seq_lens, out=None, lse=None, workspace=None, stream=None):
        p = self.problem
        if out is None:
            out = torch.empty(self._out_shape() + (p.head_dim,), dtype=torch.float32, device=q.device)
            lse = torch.empty(self._out_shape(), dtype=torch.float32, device=q.device)
        if workspace is None:
            workspace = torch.empty((max(self.workspace_bytes, 256),), dtype=torch.uint8, device=q.device)
        st = lib().da_attention(self._h, _ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(block_table), _ptr(seq_lens),
                                _ptr(out), _ptr(lse), _ptr(workspace), workspace.numel(), _stream_ptr(stream))
        _check(st, "da_attention")
        return out, lse

    def attention_noalloc(self, q, k_pool, v_pool, block_table, seq_lens, out, lse=None, stream=None):
        """da_attention_noalloc: the caller passes inputs and outputs only; partials go to the library's fixed array."""
        st = lib().da_attention_noalloc(self._h, _ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(block_table), _ptr(seq_lens),
                                        _ptr(out), _ptr(lse), _stream_ptr(stream))
        _check(st, "da_attention_noalloc")
        return out, lse


def append(problem, k_new, v_new, k_pool, v_pool, block_table, seq_lens, err_flags=None, stream=None):
    """Enqueue da_append: one new token per request joins the pools; seq_lens is incremented on the device."""
    st = lib().da_append(ctypes.byref(problem), _ptr(k_new), _ptr(v_new), _ptr(k_pool), _ptr(v_pool), _ptr(block_table),
                         _ptr(seq_lens), _ptr(err_flags), _stream_ptr(stream))
    _check(st, "da_append")


def move_blocks(src_layout, dst_layout, k_src, v_src, k_dst, v_dst, src_ids, dst_ids, err_flags=None, stream=None):
    """Enqueue da_move_blocks: blocks src_ids[i] of the source pools are copied to blocks dst_ids[i] of the
    destination pools (device int32 id tensors of equal length)."""
    assert src_ids.dtype == torch.int32 and dst_ids.dtype == torch.int32 and src_ids.numel() == dst_ids.numel()
    st = lib().da_move_blocks(ctypes.byref(src_layout), ctypes.byref(dst_layout), _ptr(k_src), _ptr(v_src), _ptr(k_dst),
                              _ptr(v_dst), _ptr(src_ids), _ptr(dst_ids), src_ids.numel(), _ptr(err_flags),
                              _stream_ptr(stream))
    _check(st, "da_move_blocks")


class BlockPool:
    """Host free list of physical KV blocks (da_block_pool).  Rows are numpy int32 views of the host block table."""

    def __init__(self, num_phys_blocks):
        self._h = ctypes.c_void_p()
        _check(lib().da_block_pool_create(num_phys_blocks, ctypes.byref(self._h)), "da_block_pool_create")

    def close(self):
        if self._h:
            lib().da_block_pool_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def free_count(self):
        n = ctypes.c_int32()
        _check(lib().da_block_pool_free_count(self._h, ctypes.byref(n)), "da_block_pool_free_count")
        return n.value

    def grow(self, row, block_tokens, cur_len, new_len):
        assert row.dtype.itemsize == 4 and row.flags["C_CONTIGUOUS"]
        st = lib().da_block_pool_grow(self._h, block_tokens, row.shape[0], ctypes.c_void_p(row.ctypes.data), cur_len, new_len)
        _check(st, "da_block_pool_grow")

    def release(self, row, block_tokens, length):
        assert row.dtype.itemsize == 4 and row.flags["C_CONTIGUOUS"]
        st = lib().da_block_pool_release(self._h, block_tokens, ctypes.c_void_p(row.ctypes.data), length)
        _check(st, "da_block_pool_release")


def combine_multi(sets, out=None, lse=None, stream=None):
    """da_combine_multi.  ``sets`` is a list of (plan, part_o, part_m, part_e), one per KV share."""
    arr = (DaPartialSet * len(sets))()
    for i, (plan, po, pm, pe) in enumerate(sets):
        arr[i].plan, arr[i].part_o, arr[i].part_m, arr[i].part_e = plan._h, po.data_ptr(), pm.data_ptr(), pe.data_ptr()
    plan0 = sets[0][0]
    if out is None:
        out = torch.empty(plan0._out_shape() + (plan0.problem.head_dim,), dtype=torch.float32, device=sets[0][1].device)
        lse = torch.empty(plan0._out_shape(), dtype=torch.float32, device=sets[0][1].device)
    st = lib().da_combine_multi(ctypes.cast(arr, ctypes.c_void_p), len(sets), _ptr(out), _ptr(lse), _stream_ptr(stream))
    _check(st, "da_combine_multi")
    return out, lse
