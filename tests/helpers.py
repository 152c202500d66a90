"""Shared test helpers: the parity rule and the oracle call on packed caches."""
import numpy as np

import oracle

MAX_ABS = 2e-3      # spec tolerance: fp16 inputs, fp32 accumulation, fp16 output
MAX_REL_L2 = 1e-3   # per (request, head) row


def oracle_on_packed(batch, k_host, v_host, lay, n_threads=0):
    cfg = batch.cfg
    return oracle.decode_attn(batch.q, k_host, v_host, batch.seq_lens, cfg.n_req, cfg.n_qh,
                              cfg.n_kvh, cfg.head_dim, cfg.max_len,
                              lay.stride_req, lay.stride_kvh, lay.stride_tok, n_threads=n_threads)


def parity_errors(out_f16, ref):
    """out_f16: float16 array [R,Hq,d]; ref: float64.  Returns (max_abs, max_row_rel_l2, whole_rel_l2)."""
    out = np.asarray(out_f16).astype(np.float64)
    assert out.shape == ref.shape
    assert np.all(np.isfinite(out)), "NaN or Inf in the GPU output"
    diff = out - ref
    max_abs = float(np.max(np.abs(diff))) if diff.size else 0.0
    num = np.sqrt((diff ** 2).sum(axis=-1))
    den = np.sqrt((ref ** 2).sum(axis=-1))
    zero = den == 0
    # rows whose reference is exactly zero (length 0) must be exactly +0
    if zero.any():
        rows = out[zero]
        assert np.all(rows == 0) and not np.signbit(rows).any(), "length-0 row is not +0"
    rel = np.where(zero, 0.0, num / np.where(zero, 1.0, den))
    whole = float(np.sqrt((diff ** 2).sum()) / max(np.sqrt((ref ** 2).sum()), 1e-300))
    return max_abs, float(rel.max()) if rel.size else 0.0, whole


def assert_parity(out_f16, ref, what=""):
    max_abs, rel, whole = parity_errors(out_f16, ref)
    assert max_abs <= MAX_ABS, "%s: max abs error %.3e > %.1e" % (what, max_abs, MAX_ABS)
    assert rel <= MAX_REL_L2, "%s: max row rel-L2 %.3e > %.1e" % (what, rel, MAX_REL_L2)
    return max_abs, rel, whole
