"""ctypes binding of oracle/sw_oracle.c (argument marshalling only).

TEST INFRASTRUCTURE: see the header of sw_oracle.c.  Nothing in the GPU
package imports this module.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sw_oracle.c")
_LIB = os.path.join(_HERE, "libsw_oracle.so")
_lib = None


def lib_path():
    return _LIB


def build(force=False):
    """Compile sw_oracle.c with gcc (OpenMP over (request, head) units)."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    tmp = _LIB + ".tmp.%d" % os.getpid()
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
           "-ffp-contract=off", "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.sw_oracle_decode_attn.restype = ctypes.c_int
        lib.sw_oracle_decode_attn.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int]
        lib.sw_oracle_decode_attn_paged.restype = ctypes.c_int
        lib.sw_oracle_decode_attn_paged.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_int,
            ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int]
        lib.sw_oracle_kv_append.restype = ctypes.c_int
        lib.sw_oracle_kv_append.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_int64, ctypes.c_int64, ctypes.c_int64]
        lib.sw_oracle_kv_append_paged.restype = ctypes.c_int
        lib.sw_oracle_kv_append_paged.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_int64, ctypes.c_int64, ctypes.c_int64]
        lib.sw_oracle_prefill_attn.restype = ctypes.c_int
        lib.sw_oracle_prefill_attn.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int64,
            ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int]
        lib.sw_oracle_kv_pack.restype = ctypes.c_int
        lib.sw_oracle_kv_pack.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_int,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_int,
            ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64]
        lib.sw_oracle_kv_span_plan.restype = ctypes.c_int
        lib.sw_oracle_kv_span_plan.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int]
        lib.sw_oracle_mixed_attn.restype = ctypes.c_int
        lib.sw_oracle_mixed_attn.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int]
        lib.sw_oracle_mixed_attn_paged.restype = ctypes.c_int
        lib.sw_oracle_mixed_attn_paged.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_int, ctypes.c_int,
            ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int]
        lib.sw_oracle_kv_store.restype = ctypes.c_int
        lib.sw_oracle_kv_store.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int64,
            ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_int64, ctypes.c_int64, ctypes.c_int64]
        lib.sw_oracle_half_to_double.restype = ctypes.c_double
        lib.sw_oracle_half_to_double.argtypes = [ctypes.c_uint16]
        lib.sw_oracle_max_threads.restype = ctypes.c_int
        lib.sw_oracle_max_threads.argtypes = []
        _lib = lib
    return _lib


def half_to_double(bits):
    return _load().sw_oracle_half_to_double(int(bits) & 0xFFFF)


def max_threads():
    return _load().sw_oracle_max_threads()


def _as_u16(a, name):
    a = np.asarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    if a.dtype != np.uint16:
        raise TypeError("%s must be float16 or uint16 bits, got %s" % (name, a.dtype))
    if not a.flags["C_CONTIGUOUS"]:
        raise ValueError("%s must be C-contiguous (strides are passed separately)" % name)
    return a


def decode_attn(q, k, v, seq_lens, n_req, n_qh, n_kvh, head_dim, max_len,
                stride_req, stride_kvh, stride_tok, n_threads=0, return_stats=False):
    """Run the oracle.

    q: float16/uint16, n_req*n_qh*head_dim elements, dense.
    k, v: flat float16/uint16 buffers addressed by the element strides given.
    Returns ref float64 [n_req, n_qh, head_dim] (and, if return_stats, the
    per-(request, head) score maximum m, the sum l of exp(s - m), and the
    thread count used).
    """
    lib = _load()
    q = _as_u16(q, "q")
    k = _as_u16(k, "k")
    v = _as_u16(v, "v")
    lens = np.ascontiguousarray(np.asarray(seq_lens, dtype=np.int32))
    if lens.size != n_req:
        raise ValueError("seq_lens has %d entries, n_req is %d" % (lens.size, n_req))
    if q.size != n_req * n_qh * head_dim:
        raise ValueError("q has %d elements, expected %d" % (q.size, n_req * n_qh * head_dim))
    need = 0
    if n_req > 0:
        need = ((n_req - 1) * stride_req + (n_kvh - 1) * stride_kvh
                + (max_len - 1) * stride_tok + head_dim)
    if k.size < need or v.size < need:
        raise ValueError("k/v buffers (%d, %d elements) are smaller than the strides address (%d)"
                         % (k.size, v.size, need))
    ref = np.zeros((n_req, n_qh, head_dim), dtype=np.float64)
    m = np.zeros((n_req, n_qh), dtype=np.float64)
    l = np.zeros((n_req, n_qh), dtype=np.float64)
    rc = lib.sw_oracle_decode_attn(
        q.ctypes.data, k.ctypes.data, v.ctypes.data, lens.ctypes.data,
        ref.ctypes.data, m.ctypes.data, l.ctypes.data,
        n_req, n_qh, n_kvh, head_dim, max_len,
        stride_req, stride_kvh, stride_tok, int(n_threads))
    if rc < 0:
        raise ValueError("sw_oracle_decode_attn rejected its arguments (code %d)" % rc)
    if return_stats:
        return ref, m, l, rc
    return ref


def decode_attn_paged(q, k_pool, v_pool, block_table, seq_lens, n_req, n_qh, n_kvh, head_dim,
                      block_size, max_blocks, n_blocks, stride_block, stride_kvh, stride_tok,
                      n_threads=0):
    """Run the oracle on a block-table cache.  Returns ref float64 [n_req, n_qh, head_dim]."""
    lib = _load()
    q = _as_u16(q, "q")
    k_pool = _as_u16(k_pool, "k_pool")
    v_pool = _as_u16(v_pool, "v_pool")
    lens = np.ascontiguousarray(np.asarray(seq_lens, dtype=np.int32))
    table = np.ascontiguousarray(np.asarray(block_table, dtype=np.int32))
    if lens.size != n_req or table.size != n_req * max_blocks:
        raise ValueError("seq_lens / block_table have the wrong number of entries")
    need = (n_blocks - 1) * stride_block + (n_kvh - 1) * stride_kvh + (block_size - 1) * stride_tok + head_dim
    if k_pool.size < need or v_pool.size < need:
        raise ValueError("pools are smaller than the strides address")
    ref = np.zeros((n_req, n_qh, head_dim), dtype=np.float64)
    rc = lib.sw_oracle_decode_attn_paged(
        q.ctypes.data, k_pool.ctypes.data, v_pool.ctypes.data, table.ctypes.data, lens.ctypes.data,
        ref.ctypes.data, n_req, n_qh, n_kvh, head_dim, block_size, max_blocks, n_blocks,
        stride_block, stride_kvh, stride_tok, int(n_threads))
    if rc < 0:
        raise ValueError("sw_oracle_decode_attn_paged rejected its arguments (code %d)" % rc)
    return ref


def mixed_attn_paged(q, k_pool, v_pool, block_table, seq_lens, q_starts, q_lens, n_req, n_qh, n_kvh,
                     head_dim, block_size, max_blocks, n_blocks, max_q_len, stride_block, stride_kvh,
                     stride_tok, n_threads=0):
    """Mixed-batch causal attention over a block-table cache (q_lens None: every cached token is a
    query, i.e. the prompt phase).  Returns ref float64 [n_tokens, n_qh, head_dim]."""
    lib = _load()
    q = _as_u16(q, "q")
    k_pool = _as_u16(k_pool, "k_pool")
    v_pool = _as_u16(v_pool, "v_pool")
    lens = np.ascontiguousarray(np.asarray(seq_lens, dtype=np.int32))
    starts = np.ascontiguousarray(np.asarray(q_starts, dtype=np.int32))
    table = np.ascontiguousarray(np.asarray(block_table, dtype=np.int32))
    qlens = None if q_lens is None else np.ascontiguousarray(np.asarray(q_lens, dtype=np.int32))
    if lens.size != n_req or starts.size != n_req or table.size != n_req * max_blocks or \
            (qlens is not None and qlens.size != n_req):
        raise ValueError("seq_lens / q_starts / q_lens / block_table have the wrong number of entries")
    if q.size % (n_qh * head_dim):
        raise ValueError("q is not a whole number of token rows")
    n_tokens = q.size // (n_qh * head_dim)
    need = (n_blocks - 1) * stride_block + (n_kvh - 1) * stride_kvh + (block_size - 1) * stride_tok + head_dim
    if k_pool.size < need or v_pool.size < need:
        raise ValueError("pools are smaller than the strides address")
    ref = np.zeros((n_tokens, n_qh, head_dim), dtype=np.float64)
    rc = lib.sw_oracle_mixed_attn_paged(
        q.ctypes.data, k_pool.ctypes.data, v_pool.ctypes.data, table.ctypes.data, lens.ctypes.data,
        starts.ctypes.data, None if qlens is None else qlens.ctypes.data, ref.ctypes.data,
        n_req, n_qh, n_kvh, head_dim, block_size, max_blocks, n_blocks, max_q_len, n_tokens,
        stride_block, stride_kvh, stride_tok, int(n_threads))
    if rc < 0:
        raise ValueError("sw_oracle_mixed_attn_paged rejected its arguments (code %d)" % rc)
    return ref


def kv_store(k_rows, v_rows, k, v, seq_lens, q_starts, q_lens, n_req, n_kvh, head_dim, max_len, max_q_len,
             stride_req, stride_kvh, stride_tok, block_table=None, block_size=0, max_blocks=0, n_blocks=0):
    """Store the K/V rows of every request's query tokens at their positions, IN PLACE in k and v.

    k_rows, v_rows: [n_tokens, n_kvh, head_dim] binary16 (bits or float16).  Dense caches by default;
    with block_table, k and v are block pools and stride_req is their block stride.  q_lens None:
    every cached token of a request is new (a whole prompt).
    """
    lib = _load()
    k_rows = _as_u16(k_rows, "k_rows")
    v_rows = _as_u16(v_rows, "v_rows")
    k = _writable_u16(k, "k")
    v = _writable_u16(v, "v")
    lens = np.ascontiguousarray(np.asarray(seq_lens, dtype=np.int32))
    starts = np.ascontiguousarray(np.asarray(q_starts, dtype=np.int32))
    qlens = None if q_lens is None else np.ascontiguousarray(np.asarray(q_lens, dtype=np.int32))
    table = None if block_table is None else np.ascontiguousarray(np.asarray(block_table, dtype=np.int32))
    if lens.size != n_req or starts.size != n_req or (qlens is not None and qlens.size != n_req):
        raise ValueError("seq_lens / q_starts / q_lens need n_req entries")
    if k_rows.size != v_rows.size or k_rows.size % (n_kvh * head_dim):
        raise ValueError("k_rows / v_rows are not whole token rows of the same count")
    n_tokens = k_rows.size // (n_kvh * head_dim)
    if table is None:
        need = ((n_req - 1) * stride_req + (n_kvh - 1) * stride_kvh + (max_len - 1) * stride_tok + head_dim) if n_req else 0
    else:
        if table.size != n_req * max_blocks:
            raise ValueError("block_table has the wrong number of entries")
        need = (n_blocks - 1) * stride_req + (n_kvh - 1) * stride_kvh + (block_size - 1) * stride_tok + head_dim
    if k.size < need or v.size < need:
        raise ValueError("k/v buffers are smaller than the strides address")
    rc = lib.sw_oracle_kv_store(k_rows.ctypes.data, v_rows.ctypes.data, k.ctypes.data, v.ctypes.data,
                                None if table is None else table.ctypes.data, lens.ctypes.data,
                                starts.ctypes.data, None if qlens is None else qlens.ctypes.data,
                                n_req, n_kvh, head_dim, max_len, max_q_len, n_tokens,
                                block_size, max_blocks, n_blocks, stride_req, stride_kvh, stride_tok)
    if rc < 0:
        raise ValueError("sw_oracle_kv_store rejected its arguments (code %d)" % rc)


def _writable_u16(a, name):
    if not isinstance(a, np.ndarray) or a.dtype != np.uint16 or not a.flags["C_CONTIGUOUS"] \
            or not a.flags["WRITEABLE"]:
        raise TypeError("%s must be a writable C-contiguous uint16 array (it is updated in place)" % name)
    return a


def kv_append(k_new, v_new, k, v, seq_lens, n_req, n_kvh, head_dim, max_len,
              stride_req, stride_kvh, stride_tok):
    """Store the newest token's rows at each request's next position, IN PLACE in k and v.

    Returns the lengths after the append (int32 [n_req]); full caches are left alone.
    """
    lib = _load()
    k_new = _as_u16(k_new, "k_new")
    v_new = _as_u16(v_new, "v_new")
    k = _writable_u16(k, "k")
    v = _writable_u16(v, "v")
    lens = np.ascontiguousarray(np.asarray(seq_lens, dtype=np.int32))
    if lens.size != n_req or k_new.size != n_req * n_kvh * head_dim or v_new.size != k_new.size:
        raise ValueError("seq_lens / k_new / v_new have the wrong number of entries")
    need = 0
    if n_req > 0:
        need = ((n_req - 1) * stride_req + (n_kvh - 1) * stride_kvh
                + (max_len - 1) * stride_tok + head_dim)
    if k.size < need or v.size < need:
        raise ValueError("k/v buffers are smaller than the strides address")
    out = np.zeros(n_req, dtype=np.int32)
    rc = lib.sw_oracle_kv_append(k_new.ctypes.data, v_new.ctypes.data, k.ctypes.data, v.ctypes.data,
                                 lens.ctypes.data, out.ctypes.data, n_req, n_kvh, head_dim, max_len,
                                 stride_req, stride_kvh, stride_tok)
    if rc < 0:
        raise ValueError("sw_oracle_kv_append rejected its arguments (code %d)" % rc)
    return out


def kv_append_paged(k_new, v_new, k_pool, v_pool, block_table, seq_lens, n_req, n_kvh, head_dim,
                    block_size, max_blocks, n_blocks, stride_block, stride_kvh, stride_tok):
    """kv_append over block pools (updated in place).  Returns the lengths after the append."""
    lib = _load()
    k_new = _as_u16(k_new, "k_new")
    v_new = _as_u16(v_new, "v_new")
    k_pool = _writable_u16(k_pool, "k_pool")
    v_pool = _writable_u16(v_pool, "v_pool")
    lens = np.ascontiguousarray(np.asarray(seq_lens, dtype=np.int32))
    table = np.ascontiguousarray(np.asarray(block_table, dtype=np.int32))
    if lens.size != n_req or table.size != n_req * max_blocks \
            or k_new.size != n_req * n_kvh * head_dim or v_new.size != k_new.size:
        raise ValueError("seq_lens / block_table / k_new / v_new have the wrong number of entries")
    need = (n_blocks - 1) * stride_block + (n_kvh - 1) * stride_kvh + (block_size - 1) * stride_tok + head_dim
    if k_pool.size < need or v_pool.size < need:
        raise ValueError("pools are smaller than the strides address")
    out = np.zeros(n_req, dtype=np.int32)
    rc = lib.sw_oracle_kv_append_paged(
        k_new.ctypes.data, v_new.ctypes.data, k_pool.ctypes.data, v_pool.ctypes.data,
        table.ctypes.data, lens.ctypes.data, out.ctypes.data, n_req, n_kvh, head_dim,
        block_size, max_blocks, n_blocks, stride_block, stride_kvh, stride_tok)
    if rc < 0:
        raise ValueError("sw_oracle_kv_append_paged rejected its arguments (code %d)" % rc)
    return out


def prefill_attn(q, k, v, seq_lens, q_starts, n_req, n_qh, n_kvh, head_dim, max_len,
                 stride_req, stride_kvh, stride_tok, n_threads=0, return_threads=False):
    """Causal (prompt-phase) attention.  q: [n_tokens, n_qh, head_dim]; request r's token i is row
    q_starts[r] + i.  Returns ref float64 [n_tokens, n_qh, head_dim] (rows of no request are 0)."""
    lib = _load()
    q = _as_u16(q, "q")
    k = _as_u16(k, "k")
    v = _as_u16(v, "v")
    lens = np.ascontiguousarray(np.asarray(seq_lens, dtype=np.int32))
    starts = np.ascontiguousarray(np.asarray(q_starts, dtype=np.int32))
    if lens.size != n_req or starts.size != n_req:
        raise ValueError("seq_lens / q_starts need n_req entries")
    if q.size % (n_qh * head_dim):
        raise ValueError("q is not a whole number of token rows")
    n_tokens = q.size // (n_qh * head_dim)
    need = 0
    if n_req > 0:
        need = ((n_req - 1) * stride_req + (n_kvh - 1) * stride_kvh
                + (max_len - 1) * stride_tok + head_dim)
    if k.size < need or v.size < need:
        raise ValueError("k/v buffers are smaller than the strides address")
    ref = np.zeros((n_tokens, n_qh, head_dim), dtype=np.float64)
    rc = lib.sw_oracle_prefill_attn(q.ctypes.data, k.ctypes.data, v.ctypes.data, lens.ctypes.data,
                                    starts.ctypes.data, ref.ctypes.data, n_req, n_qh, n_kvh,
                                    head_dim, max_len, n_tokens, stride_req, stride_kvh, stride_tok,
                                    int(n_threads))
    if rc < 0:
        raise ValueError("sw_oracle_prefill_attn rejected its arguments (code %d)" % rc)
    return (ref, rc) if return_threads else ref


def kv_pack(k_pool, v_pool, block_table, seq_lens, k_dense, v_dense, to_dense, n_req, n_kvh,
            head_dim, max_len, block_size, max_blocks, n_blocks, stride_block, p_stride_kvh,
            d_stride_req, d_stride_kvh, stride_tok):
    """Copy every request's valid rows pools -> dense (to_dense) or dense -> pools, IN PLACE in
    the destination arrays (writable uint16)."""
    lib = _load()
    dst = (k_dense, v_dense) if to_dense else (k_pool, v_pool)
    src = (k_pool, v_pool) if to_dense else (k_dense, v_dense)
    for a in dst:
        _writable_u16(a, "destination")
    src = [_as_u16(a, "source") for a in src]
    lens = np.ascontiguousarray(np.asarray(seq_lens, dtype=np.int32))
    table = np.ascontiguousarray(np.asarray(block_table, dtype=np.int32))
    if lens.size != n_req or table.size != n_req * max_blocks:
        raise ValueError("seq_lens / block_table have the wrong number of entries")
    need_p = (n_blocks - 1) * stride_block + (n_kvh - 1) * p_stride_kvh + (block_size - 1) * stride_tok + head_dim
    need_d = 0 if n_req == 0 else ((n_req - 1) * d_stride_req + (n_kvh - 1) * d_stride_kvh
                                   + (max_len - 1) * stride_tok + head_dim)
    kp, vp = (src if to_dense else dst)
    kd, vd = (dst if to_dense else src)
    if kp.size < need_p or vp.size < need_p or kd.size < need_d or vd.size < need_d:
        raise ValueError("a buffer is smaller than its strides address")
    rc = lib.sw_oracle_kv_pack(kp.ctypes.data, vp.ctypes.data, table.ctypes.data, lens.ctypes.data,
                               kd.ctypes.data, vd.ctypes.data, 0 if to_dense else 1,
                               n_req, n_kvh, head_dim, max_len, block_size, max_blocks, n_blocks,
                               stride_block, p_stride_kvh, d_stride_req, d_stride_kvh, stride_tok)
    if rc < 0:
        raise ValueError("sw_oracle_kv_pack rejected its arguments (code %d)" % rc)


def kv_span_plan(block_table, seq_lens, n_req, block_size, max_blocks, n_blocks, fill=-1):
    """Returns (span_first [n_req, max_blocks], span_blocks [n_req, max_blocks], n_spans [n_req]);
    entries past a request's span count hold `fill`."""
    lib = _load()
    lens = np.ascontiguousarray(np.asarray(seq_lens, dtype=np.int32))
    table = np.ascontiguousarray(np.asarray(block_table, dtype=np.int32))
    if lens.size != n_req or table.size != n_req * max_blocks:
        raise ValueError("seq_lens / block_table have the wrong number of entries")
    first = np.full((n_req, max_blocks), fill, dtype=np.int32)
    count = np.full((n_req, max_blocks), fill, dtype=np.int32)
    n = np.full(n_req, fill, dtype=np.int32)
    rc = lib.sw_oracle_kv_span_plan(table.ctypes.data, lens.ctypes.data, first.ctypes.data,
                                    count.ctypes.data, n.ctypes.data, n_req, block_size, max_blocks,
                                    n_blocks)
    if rc < 0:
        raise ValueError("sw_oracle_kv_span_plan rejected its arguments (code %d)" % rc)
    return first, count, n


def mixed_attn(q, k, v, seq_lens, q_starts, q_lens, n_req, n_qh, n_kvh, head_dim, max_len, max_q_len,
               stride_req, stride_kvh, stride_tok, n_threads=0, return_threads=False):
    """Mixed-batch causal attention: request r's last q_lens[r] tokens are its queries (rows
    q_starts[r] .. of q).  Returns ref float64 [n_tokens, n_qh, head_dim] (rows of no query are 0)."""
    lib = _load()
    q = _as_u16(q, "q")
    k = _as_u16(k, "k")
    v = _as_u16(v, "v")
    lens = np.ascontiguousarray(np.asarray(seq_lens, dtype=np.int32))
    starts = np.ascontiguousarray(np.asarray(q_starts, dtype=np.int32))
    qlens = np.ascontiguousarray(np.asarray(q_lens, dtype=np.int32))
    if lens.size != n_req or starts.size != n_req or qlens.size != n_req:
        raise ValueError("seq_lens / q_starts / q_lens need n_req entries")
    if q.size % (n_qh * head_dim):
        raise ValueError("q is not a whole number of token rows")
    n_tokens = q.size // (n_qh * head_dim)
    need = 0
    if n_req > 0:
        need = ((n_req - 1) * stride_req + (n_kvh - 1) * stride_kvh
                + (max_len - 1) * stride_tok + head_dim)
    if k.size < need or v.size < need:
        raise ValueError("k/v buffers are smaller than the strides address")
    ref = np.zeros((n_tokens, n_qh, head_dim), dtype=np.float64)
    rc = lib.sw_oracle_mixed_attn(q.ctypes.data, k.ctypes.data, v.ctypes.data, lens.ctypes.data,
                                  starts.ctypes.data, qlens.ctypes.data, ref.ctypes.data, n_req, n_qh,
                                  n_kvh, head_dim, max_len, max_q_len, n_tokens, stride_req,
                                  stride_kvh, stride_tok, int(n_threads))
    if rc < 0:
        raise ValueError("sw_oracle_mixed_attn rejected its arguments (code %d)" % rc)
    return (ref, rc) if return_threads else ref
