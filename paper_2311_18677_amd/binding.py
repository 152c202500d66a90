"""Thin ctypes binding of include/sw_decode.h (argument marshalling only).

Every step of the decode-attention path runs in the HIP kernels of
libsw_decode.so.  There is no fallback: if the library has not been built the
first call raises.  PyTorch appears only in the helpers that allocate device
memory; the ABI functions take any object with a data_ptr() method, or a raw
integer address.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsw_decode.so")

SW_OK = 0
SW_ERR_NULL = -1
SW_ERR_SHAPE = -2
SW_ERR_UNSUPPORTED = -3
SW_ERR_ALIGN = -4
SW_ERR_HIP = -5
SW_ERR_PARAM = -6
SW_ERR_STATE = -7
SW_F16 = 1
SW_PARAM_CHUNK = 1
SW_PARAM_KERNEL = 2
SW_PARAM_COMBINE = 3
SW_PARAM_WAVES = 4
SW_PARAM_PREFILL_HEADS = 5
SW_PARAM_PREFILL_WAVES = 6
SW_PARAM_PREFILL_KERNEL = 7
SW_PARAM_MIXED_MERGE = 8

EXPORTS = ("sw_kv_layout", "sw_decode_attn", "sw_decode_attn_static", "sw_kv_paged_layout", "sw_decode_attn_paged",
           "sw_decode_attn_append", "sw_decode_attn_paged_append", "sw_advance_lens",
           "sw_prefill_attn", "sw_mixed_attn", "sw_prefill_attn_paged", "sw_mixed_attn_paged", "sw_kv_store", "sw_kv_store_paged", "sw_kv_pack", "sw_kv_unpack", "sw_kv_span_plan",
           "sw_last_error", "sw_version", "sw_release", "sw_device_status",
           "sw_set_param", "sw_get_param", "sw_prof_start", "sw_prof_stop", "sw_prof_last_gap", "sw_stream_read")


class sw_kv_layout_t(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("elem_bytes", ctypes.c_int32),
                ("stride_req", ctypes.c_int64), ("stride_kvh", ctypes.c_int64),
                ("stride_tok", ctypes.c_int64), ("stride_dim", ctypes.c_int64),
                ("total_elems", ctypes.c_int64),
                ("base_align", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class sw_kv_paged_layout_t(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("elem_bytes", ctypes.c_int32),
                ("stride_block", ctypes.c_int64), ("stride_kvh", ctypes.c_int64),
                ("stride_tok", ctypes.c_int64), ("stride_dim", ctypes.c_int64),
                ("total_elems", ctypes.c_int64),
                ("base_align", ctypes.c_int32), ("block_size", ctypes.c_int32)]


class SwError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("sw_decode error %d: %s" % (code, text))
        self.code = code


_lib = None


def load():
    """Load libsw_decode.so; raise if it is not built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            "libsw_decode.so is not built (%s); run `python -m paper_2311_18677_amd.build`"
            % LIB_PATH)
    # PyTorch ships its own copy of the HIP runtime.  The streams and device
    # pointers handed to this library come from torch, so both must live in ONE
    # runtime instance: torch is imported first, and the library's dependency on
    # libamdhip64.so.7 then binds to the copy torch has already loaded.
    import torch  # noqa: F401
    lib = ctypes.CDLL(LIB_PATH)
    vp, ci = ctypes.c_void_p, ctypes.c_int
    lib.sw_kv_layout.restype = ci
    lib.sw_kv_layout.argtypes = [ci, ci, ci, ci, ctypes.POINTER(sw_kv_layout_t)]
    lib.sw_decode_attn.restype = ci
    lib.sw_decode_attn.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, vp]
    lib.sw_decode_attn_static.restype = ci
    lib.sw_decode_attn_static.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, vp]
    lib.sw_kv_paged_layout.restype = ci
    lib.sw_kv_paged_layout.argtypes = [ci, ci, ci, ci, ctypes.POINTER(sw_kv_paged_layout_t)]
    lib.sw_decode_attn_paged.restype = ci
    lib.sw_decode_attn_paged.argtypes = [vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, vp]
    lib.sw_decode_attn_append.restype = ci
    lib.sw_decode_attn_append.argtypes = [vp, vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, vp]
    lib.sw_decode_attn_paged_append.restype = ci
    lib.sw_decode_attn_paged_append.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp,
                                                ci, ci, ci, ci, ci, ci, ci, vp]
    lib.sw_advance_lens.restype = ci
    lib.sw_advance_lens.argtypes = [vp, ci, ci, vp]
    lib.sw_prefill_attn.restype = ci
    lib.sw_prefill_attn.argtypes = [vp, vp, vp, vp, vp, vp, ctypes.c_longlong, ci, ci, ci, ci, ci, vp]
    lib.sw_mixed_attn.restype = ci
    lib.sw_mixed_attn.argtypes = [vp, vp, vp, vp, vp, vp, vp, ctypes.c_longlong, ci, ci, ci, ci, ci, ci, vp]
    for fn in (lib.sw_kv_pack, lib.sw_kv_unpack):
        fn.restype = ci
        fn.argtypes = [vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, vp]
    lib.sw_kv_span_plan.restype = ci
    lib.sw_kv_span_plan.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, vp]
    lib.sw_last_error.restype = ctypes.c_char_p
    lib.sw_last_error.argtypes = []
    lib.sw_version.restype = ci
    lib.sw_version.argtypes = []
    lib.sw_release.restype = ci
    lib.sw_release.argtypes = []
    lib.sw_device_status.restype = ci
    lib.sw_device_status.argtypes = [ctypes.POINTER(ci)]
    lib.sw_set_param.restype = ci
    lib.sw_set_param.argtypes = [ci, ci]
    lib.sw_get_param.restype = ci
    lib.sw_get_param.argtypes = [ci, ctypes.POINTER(ci)]
    lib.sw_prefill_attn_paged.restype = ci
    lib.sw_prefill_attn_paged.argtypes = [vp, vp, vp, vp, vp, vp, vp, ctypes.c_longlong,
                                          ci, ci, ci, ci, ci, ci, ci, vp]
    lib.sw_mixed_attn_paged.restype = ci
    lib.sw_mixed_attn_paged.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_longlong,
                                        ci, ci, ci, ci, ci, ci, ci, ci, vp]
    lib.sw_kv_store.restype = ci
    lib.sw_kv_store.argtypes = [vp, vp, vp, vp, vp, vp, vp, ctypes.c_longlong, ci, ci, ci, ci, ci, vp]
    lib.sw_kv_store_paged.restype = ci
    lib.sw_kv_store_paged.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_longlong,
                                      ci, ci, ci, ci, ci, ci, ci, vp]
    lib.sw_stream_read.restype = ci
    lib.sw_stream_read.argtypes = [vp, ctypes.c_longlong, vp, ci, vp]
    lib.sw_prof_start.restype = ci
    lib.sw_prof_start.argtypes = [ci]
    lib.sw_prof_last_gap.restype = ci
    lib.sw_prof_last_gap.argtypes = [ctypes.POINTER(ctypes.c_double)]
    lib.sw_prof_stop.restype = ci
    lib.sw_prof_stop.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double),
                                 ctypes.POINTER(ci)]
    _lib = lib
    return lib


def _ptr(x):
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    return int(x)


def _stream(s):
    if s is None:
        return None
    if hasattr(s, "cuda_stream"):
        return s.cuda_stream
    return int(s)


def _check(rc):
    if rc != SW_OK:
        raise SwError(rc, sw_last_error())
    return rc


def sw_last_error():
    return load().sw_last_error().decode("utf-8", "replace")


def sw_version():
    return load().sw_version()


def sw_kv_layout(n_req, n_kvh, head_dim, max_len, check=True):
    """Returns the sw_kv_layout_t the library fills in (or the error code if check=False)."""
    lay = sw_kv_layout_t()
    rc = load().sw_kv_layout(n_req, n_kvh, head_dim, max_len, ctypes.byref(lay))
    if check:
        _check(rc)
        return lay
    return rc, lay


def sw_decode_attn(q, k_cache, v_cache, seq_lens, out, n_req, n_qh, n_kvh, head_dim, max_len,
                   stream=None, check=True):
    """One decode step's attention; enqueues on `stream` and returns without waiting."""
    rc = load().sw_decode_attn(_ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(seq_lens), _ptr(out),
                               n_req, n_qh, n_kvh, head_dim, max_len, _stream(stream))
    return _check(rc) if check else rc


def sw_decode_attn_static(q, k_cache, v_cache, seq_lens, out, n_req, n_qh, n_kvh, head_dim, max_len,
                          stream=None, check=True):
    """sw_decode_attn over the library's static scratch array: allocates nothing."""
    rc = load().sw_decode_attn_static(_ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(seq_lens), _ptr(out),
                                      n_req, n_qh, n_kvh, head_dim, max_len, _stream(stream))
    return _check(rc) if check else rc


def sw_kv_paged_layout(n_blocks, n_kvh, head_dim, block_size, check=True):
    """Returns the sw_kv_paged_layout_t the library fills in (or (code, layout) if check=False)."""
    lay = sw_kv_paged_layout_t()
    rc = load().sw_kv_paged_layout(n_blocks, n_kvh, head_dim, block_size, ctypes.byref(lay))
    if check:
        _check(rc)
        return lay
    return rc, lay


def sw_decode_attn_paged(q, k_pool, v_pool, block_table, seq_lens, out, n_req, n_qh, n_kvh,
                         head_dim, block_size, max_blocks, n_blocks, stream=None, check=True):
    """One decode step's attention over block pools; enqueues on `stream`."""
    rc = load().sw_decode_attn_paged(_ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(block_table),
                                     _ptr(seq_lens), _ptr(out), n_req, n_qh, n_kvh, head_dim,
                                     block_size, max_blocks, n_blocks, _stream(stream))
    return _check(rc) if check else rc


def sw_decode_attn_append(q, k_new, v_new, k_cache, v_cache, seq_lens, out, n_req, n_qh, n_kvh,
                          head_dim, max_len, stream=None, check=True):
    """Store the newest token's K/V rows in the cache and attend over it, in one pass."""
    rc = load().sw_decode_attn_append(_ptr(q), _ptr(k_new), _ptr(v_new), _ptr(k_cache),
                                      _ptr(v_cache), _ptr(seq_lens), _ptr(out),
                                      n_req, n_qh, n_kvh, head_dim, max_len, _stream(stream))
    return _check(rc) if check else rc


def sw_decode_attn_paged_append(q, k_new, v_new, k_pool, v_pool, block_table, seq_lens, out,
                                n_req, n_qh, n_kvh, head_dim, block_size, max_blocks, n_blocks,
                                stream=None, check=True):
    """sw_decode_attn_append over block pools."""
    rc = load().sw_decode_attn_paged_append(_ptr(q), _ptr(k_new), _ptr(v_new), _ptr(k_pool),
                                            _ptr(v_pool), _ptr(block_table), _ptr(seq_lens),
                                            _ptr(out), n_req, n_qh, n_kvh, head_dim,
                                            block_size, max_blocks, n_blocks, _stream(stream))
    return _check(rc) if check else rc


def sw_advance_lens(seq_lens, n_req, max_len, stream=None, check=True):
    """End of a model step: every length grows by one, saturating at max_len (on the device)."""
    rc = load().sw_advance_lens(_ptr(seq_lens), n_req, max_len, _stream(stream))
    return _check(rc) if check else rc


def sw_prefill_attn(q, k_cache, v_cache, seq_lens, q_starts, out, n_tokens, n_req, n_qh, n_kvh,
                    head_dim, max_len, stream=None, check=True):
    """Prompt-phase (causal) attention of every prompt token over its request's cache."""
    rc = load().sw_prefill_attn(_ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(seq_lens),
                                _ptr(q_starts), _ptr(out), int(n_tokens), n_req, n_qh, n_kvh,
                                head_dim, max_len, _stream(stream))
    return _check(rc) if check else rc


def sw_mixed_attn(q, k_cache, v_cache, seq_lens, q_starts, q_lens, out, n_tokens, n_req, n_qh, n_kvh,
                  head_dim, max_len, max_q_len, stream=None, check=True):
    """Mixed-batch causal attention: the last q_lens[r] cached tokens of request r are its queries."""
    rc = load().sw_mixed_attn(_ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(seq_lens), _ptr(q_starts),
                              _ptr(q_lens), _ptr(out), int(n_tokens), n_req, n_qh, n_kvh, head_dim,
                              max_len, max_q_len, _stream(stream))
    return _check(rc) if check else rc


def sw_kv_pack(k_pool, v_pool, block_table, seq_lens, k_dense, v_dense, n_req, n_kvh, head_dim,
               max_len, block_size, max_blocks, n_blocks, stream=None, check=True):
    """Block pools -> dense caches (every request's valid rows)."""
    rc = load().sw_kv_pack(_ptr(k_pool), _ptr(v_pool), _ptr(block_table), _ptr(seq_lens),
                           _ptr(k_dense), _ptr(v_dense), n_req, n_kvh, head_dim, max_len,
                           block_size, max_blocks, n_blocks, _stream(stream))
    return _check(rc) if check else rc


def sw_kv_unpack(k_dense, v_dense, block_table, seq_lens, k_pool, v_pool, n_req, n_kvh, head_dim,
                 max_len, block_size, max_blocks, n_blocks, stream=None, check=True):
    """Dense caches -> the pool blocks the table names."""
    rc = load().sw_kv_unpack(_ptr(k_dense), _ptr(v_dense), _ptr(block_table), _ptr(seq_lens),
                             _ptr(k_pool), _ptr(v_pool), n_req, n_kvh, head_dim, max_len,
                             block_size, max_blocks, n_blocks, _stream(stream))
    return _check(rc) if check else rc


def sw_kv_span_plan(block_table, seq_lens, span_first, span_blocks, n_spans, n_req, block_size,
                    max_blocks, n_blocks, stream=None, check=True):
    """Runs of consecutive pool block ids per request (the transfers a layer needs)."""
    rc = load().sw_kv_span_plan(_ptr(block_table), _ptr(seq_lens), _ptr(span_first),
                                _ptr(span_blocks), _ptr(n_spans), n_req, block_size, max_blocks,
                                n_blocks, _stream(stream))
    return _check(rc) if check else rc


def sw_release():
    return _check(load().sw_release())


def sw_device_status():
    """1 if a single-launch merge on the current device ever gave up waiting, else 0 (synchronises)."""
    flag = ctypes.c_int(0)
    _check(load().sw_device_status(ctypes.byref(flag)))
    return flag.value


def sw_set_param(key, value, check=True):
    rc = load().sw_set_param(key, value)
    return _check(rc) if check else rc


def sw_get_param(key):
    v = ctypes.c_int(0)
    _check(load().sw_get_param(key, ctypes.byref(v)))
    return v.value


def sw_prof_start(capacity):
    return _check(load().sw_prof_start(capacity))


def sw_prof_last_gap():
    """Microseconds between the partial kernel's end and the combine kernel's start, summed
    over the calls the last sw_prof_stop reported."""
    g = ctypes.c_double(0.0)
    _check(load().sw_prof_last_gap(ctypes.byref(g)))
    return g.value


def sw_prof_stop():
    """Returns (partial_us_sum, combine_us_sum, n_calls)."""
    p, c, n = ctypes.c_double(0), ctypes.c_double(0), ctypes.c_int(0)
    _check(load().sw_prof_stop(ctypes.byref(p), ctypes.byref(c), ctypes.byref(n)))
    return p.value, c.value, n.value


def sw_prefill_attn_paged(q, k_pool, v_pool, block_table, seq_lens, q_starts, out, n_tokens, n_req, n_qh,
                          n_kvh, head_dim, block_size, max_blocks, n_blocks, stream=None, check=True):
    """Prompt-phase (causal) attention over block pools + block table."""
    rc = load().sw_prefill_attn_paged(_ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(block_table),
                                      _ptr(seq_lens), _ptr(q_starts), _ptr(out), int(n_tokens), n_req,
                                      n_qh, n_kvh, head_dim, block_size, max_blocks, n_blocks,
                                      _stream(stream))
    return _check(rc) if check else rc


def sw_mixed_attn_paged(q, k_pool, v_pool, block_table, seq_lens, q_starts, q_lens, out, n_tokens, n_req,
                        n_qh, n_kvh, head_dim, block_size, max_blocks, n_blocks, max_q_len,
                        stream=None, check=True):
    """Mixed-batch attention over block pools + block table."""
    rc = load().sw_mixed_attn_paged(_ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(block_table),
                                    _ptr(seq_lens), _ptr(q_starts), _ptr(q_lens), _ptr(out),
                                    int(n_tokens), n_req, n_qh, n_kvh, head_dim, block_size, max_blocks,
                                    n_blocks, max_q_len, _stream(stream))
    return _check(rc) if check else rc


def sw_kv_store(k_rows, v_rows, k_cache, v_cache, seq_lens, q_starts, q_lens, n_tokens, n_req, n_kvh,
                head_dim, max_len, max_q_len, stream=None, check=True):
    """Store the new tokens' K/V rows at their positions in the dense caches (q_lens None: all)."""
    rc = load().sw_kv_store(_ptr(k_rows), _ptr(v_rows), _ptr(k_cache), _ptr(v_cache), _ptr(seq_lens),
                            _ptr(q_starts), _ptr(q_lens), int(n_tokens), n_req, n_kvh, head_dim, max_len,
                            max_q_len, _stream(stream))
    return _check(rc) if check else rc


def sw_kv_store_paged(k_rows, v_rows, k_pool, v_pool, block_table, seq_lens, q_starts, q_lens, n_tokens,
                      n_req, n_kvh, head_dim, block_size, max_blocks, n_blocks, max_q_len,
                      stream=None, check=True):
    """The same into block pools + block table."""
    rc = load().sw_kv_store_paged(_ptr(k_rows), _ptr(v_rows), _ptr(k_pool), _ptr(v_pool),
                                  _ptr(block_table), _ptr(seq_lens), _ptr(q_starts), _ptr(q_lens),
                                  int(n_tokens), n_req, n_kvh, head_dim, block_size, max_blocks,
                                  n_blocks, max_q_len, _stream(stream))
    return _check(rc) if check else rc


def sw_stream_read(src, n_bytes, sink, workgroups=0, stream=None, check=True):
    """Measurement support: read n_bytes once; sink[b] = XOR of the words workgroup b read."""
    rc = load().sw_stream_read(_ptr(src), int(n_bytes), _ptr(sink), int(workgroups), _stream(stream))
    return _check(rc) if check else rc


# ---- device-memory plumbing (PyTorch) ------------------------------------------------

def upload_batch(batch, device="cuda:0", pad_bits=0):
    """Allocate device buffers for a workloads.Batch in the library's layout and fill them.

    Returns a dict with q, k_cache, v_cache, seq_lens, out (torch tensors), the
    layout, and the host copies of the packed caches (for the CPU oracle in tests).
    """
    import numpy as np
    import torch
    from . import workloads as wl

    cfg = batch.cfg
    lay = sw_kv_layout(cfg.n_req, cfg.n_kvh, cfg.head_dim, cfg.max_len)
    k_host = wl.pack_cache(batch.k_rows, cfg, lay.stride_req, lay.stride_kvh, lay.stride_tok,
                           lay.total_elems, pad_bits)
    v_host = wl.pack_cache(batch.v_rows, cfg, lay.stride_req, lay.stride_kvh, lay.stride_tok,
                           lay.total_elems, pad_bits)
    dev = torch.device(device)
    as_dev = lambda a: torch.from_numpy(a.view(np.int16)).to(dev).view(torch.float16)
    res = {
        "layout": lay,
        "k_host": k_host,
        "v_host": v_host,
        "q": as_dev(np.ascontiguousarray(batch.q).view(np.uint16).reshape(-1)),
        "k_cache": as_dev(k_host),
        "v_cache": as_dev(v_host),
        "seq_lens": torch.from_numpy(np.ascontiguousarray(batch.seq_lens, dtype=np.int32)).to(dev),
        "out": torch.full((cfg.n_req, cfg.n_qh, cfg.head_dim), float("nan"),
                          dtype=torch.float16, device=dev),
    }
    for name in ("q", "k_cache", "v_cache", "out"):
        assert res[name].data_ptr() % lay.base_align == 0, name
    return res


def run_batch(bufs, cfg, stream=None):
    """sw_decode_attn on buffers made by upload_batch."""
    return sw_decode_attn(bufs["q"], bufs["k_cache"], bufs["v_cache"], bufs["seq_lens"],
                          bufs["out"], cfg.n_req, cfg.n_qh, cfg.n_kvh, cfg.head_dim, cfg.max_len,
                          stream)


def upload_paged_batch(batch, block_size, spare_blocks=3, seed=0, device="cuda:0", pad_bits=0,
                       table=None, room=0):
    """Like upload_batch, for the block-table layout: shuffled pool blocks plus spares.

    room > 0 also allots blocks for each request's next `room` positions (append variant).
    """
    import numpy as np
    import torch
    from . import workloads as wl

    cfg = batch.cfg
    max_blocks = -(-cfg.max_len // block_size)
    n_blocks = sum(-(-min(int(L) + room, cfg.max_len) // block_size)
                   for L in batch.valid_lens) + spare_blocks
    lay = sw_kv_paged_layout(n_blocks, cfg.n_kvh, cfg.head_dim, block_size)
    k_host, v_host, tab = wl.pack_paged(batch.k_rows, batch.v_rows, cfg, block_size, lay.stride_block,
                                        lay.stride_kvh, lay.stride_tok, n_blocks, seed=seed,
                                        pad_bits=pad_bits, room=room)
    if table is not None:
        tab = table(tab)
    dev = torch.device(device)
    as_dev = lambda a: torch.from_numpy(a.view(np.int16)).to(dev).view(torch.float16)
    return {
        "layout": lay, "k_host": k_host, "v_host": v_host, "table_host": tab,
        "block_size": block_size, "max_blocks": max_blocks, "n_blocks": n_blocks,
        "q": as_dev(np.ascontiguousarray(batch.q).view(np.uint16).reshape(-1)),
        "k_pool": as_dev(k_host), "v_pool": as_dev(v_host),
        "block_table": torch.from_numpy(np.ascontiguousarray(tab, dtype=np.int32)).to(dev),
        "seq_lens": torch.from_numpy(np.ascontiguousarray(batch.seq_lens, dtype=np.int32)).to(dev),
        "out": torch.full((cfg.n_req, cfg.n_qh, cfg.head_dim), float("nan"),
                          dtype=torch.float16, device=dev),
    }


def run_paged_batch(bufs, cfg, stream=None):
    """sw_decode_attn_paged on buffers made by upload_paged_batch."""
    return sw_decode_attn_paged(bufs["q"], bufs["k_pool"], bufs["v_pool"], bufs["block_table"],
                                bufs["seq_lens"], bufs["out"], cfg.n_req, cfg.n_qh, cfg.n_kvh,
                                cfg.head_dim, bufs["block_size"], bufs["max_blocks"],
                                bufs["n_blocks"], stream)
