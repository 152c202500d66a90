"""Seeded synthetic decode batches (inputs only -- none of the method's arithmetic).

The paper characterises the token phase on production traces that are not
public here; it gives the models (table "Models we evaluate": Llama2-70B,
BLOOM-176B), the tensor-parallel degree (section 2.5: 8 GPUs), the decode batch
range (section 3.4: up to 64) and the context-length medians (section 3.1:
prompt median 1500 tokens for coding, 1020 for conversation).  These
generators stand in for those traces: same shapes, lengths drawn around those
medians, values i.i.d. N(0, 1) rounded once to binary16.

Both the CPU oracle's tests and the GPU library's tests and bench draw their
inputs here, so that they see the same bytes.  numpy only.
"""
from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 231118677


@dataclass(frozen=True)
class Config:
    name: str
    n_req: int
    n_qh: int
    n_kvh: int
    head_dim: int
    max_len: int
    lens: tuple            # ("fixed", [..]) | ("uniform", lo, hi) | ("lognormal", median, sigma, lo, hi)
    k_row_scale: tuple = ()   # () or (probability, factor)
    n_layers: int = 1      # layers of the model the share belongs to (for steps/s)
    seed_index: int = 0


CONFIGS = {
    # 1. tiny multi-head case the CPU oracle finishes in milliseconds
    "tiny_mha": Config("tiny_mha", 4, 8, 8, 64, 128, ("fixed", (1, 17, 64, 128)),
                       n_layers=1, seed_index=1),
    # 2. Llama-2-70B, one GPU's share at 8-way tensor parallelism: 8 query heads on 1 KV head
    "llama70b_tp8": Config("llama70b_tp8", 64, 8, 1, 128, 4096, ("uniform", 1000, 2600),
                           n_layers=80, seed_index=2),
    # 3. BLOOM-176B, one GPU's share: 112 / 8 = 14 heads, multi-head attention
    "bloom176b_tp8": Config("bloom176b_tp8", 32, 14, 14, 128, 8192,
                            ("lognormal", 1000.0, 0.8, 16, 8192), n_layers=70, seed_index=3),
    # 4. large skewed batch, Llama share, 10 % of the key rows scaled by 8
    "skewed_256": Config("skewed_256", 256, 8, 1, 128, 8192,
                         ("lognormal", 1020.0, 1.0, 16, 8192), k_row_scale=(0.1, 8.0),
                         n_layers=80, seed_index=4),
    # 5. few requests, long context
    "longctx_8x32k": Config("longctx_8x32k", 8, 8, 1, 128, 32768,
                            ("fixed", (32768,) * 8), n_layers=80, seed_index=5),
}


def _streams(seed, n=5):
    """Independent Philox sub-streams: seq_lens, q, K, V, K-row-scale mask."""
    return [np.random.Generator(np.random.Philox(s))
            for s in np.random.SeedSequence(int(seed)).spawn(n)]


def draw_seq_lens(cfg, rng):
    kind = cfg.lens[0]
    if kind == "fixed":
        lens = np.asarray(cfg.lens[1], dtype=np.int64)
        if lens.size != cfg.n_req:
            raise ValueError("fixed lens need n_req entries")
    elif kind == "uniform":
        lens = rng.integers(cfg.lens[1], cfg.lens[2] + 1, size=cfg.n_req)
    elif kind == "lognormal":
        _, median, sigma, lo, hi = cfg.lens
        z = rng.standard_normal(cfg.n_req)
        lens = np.clip(np.rint(np.exp(np.log(median) + sigma * z)), lo, hi)
    else:
        raise ValueError(kind)
    return lens.astype(np.int32)


@dataclass
class Batch:
    """One decode batch: q dense, K/V as compact valid rows in (req, kv_head, token, dim) order."""
    cfg: Config
    seed: int
    seq_lens: np.ndarray              # int32 [n_req] (as handed to the library; may be out of range)
    q: np.ndarray                     # float16 [n_req, n_qh, head_dim]
    k_rows: list = field(default_factory=list)   # per request: float16 [n_kvh, L_r, head_dim]
    v_rows: list = field(default_factory=list)

    @property
    def valid_lens(self):
        return np.clip(self.seq_lens, 0, self.cfg.max_len)

    @property
    def total_tokens(self):
        return int(self.valid_lens.astype(np.int64).sum())

    @property
    def kv_bytes(self):
        """Bytes of K and V rows at valid positions: tokens * n_kvh * head_dim * 2 B * 2."""
        return self.total_tokens * self.cfg.n_kvh * self.cfg.head_dim * 4


def make_batch(cfg, seed=None, seq_lens=None):
    """Draw one batch for `cfg`.  seq_lens overrides the config's length recipe."""
    if isinstance(cfg, str):
        cfg = CONFIGS[cfg]
    if seed is None:
        seed = BASE_SEED + cfg.seed_index
    r_len, r_q, r_k, r_v, r_mask = _streams(seed)
    if seq_lens is None:
        lens = draw_seq_lens(cfg, r_len)
    else:
        lens = np.asarray(seq_lens, dtype=np.int32)
        if lens.size != cfg.n_req:
            raise ValueError("seq_lens override needs n_req entries")
    d = cfg.head_dim
    q = r_q.standard_normal((cfg.n_req, cfg.n_qh, d), dtype=np.float32).astype(np.float16)
    k_rows, v_rows = [], []
    valid = np.clip(lens, 0, cfg.max_len)
    for r in range(cfg.n_req):
        L = int(valid[r])
        k = r_k.standard_normal((cfg.n_kvh, L, d), dtype=np.float32)
        v = r_v.standard_normal((cfg.n_kvh, L, d), dtype=np.float32)
        if cfg.k_row_scale:
            prob, factor = cfg.k_row_scale
            hit = r_mask.random((cfg.n_kvh, L)) < prob
            k = np.where(hit[:, :, None], k * np.float32(factor), k)
        k_rows.append(k.astype(np.float16))
        v_rows.append(v.astype(np.float16))
    return Batch(cfg, int(seed), lens, q, k_rows, v_rows)


def make_new_rows(cfg, seed, step=0):
    """K and V rows of the token each request generates next: float16 [n_req, n_kvh, head_dim] each.

    Same value distribution as the cached rows; `step` selects an independent draw per
    decode iteration (and per layer, if the caller folds the layer into it).
    """
    ss = np.random.SeedSequence([int(seed), 0x6E6577, int(step)]).spawn(2)
    shape = (cfg.n_req, cfg.n_kvh, cfg.head_dim)
    k = np.random.Generator(np.random.Philox(ss[0])).standard_normal(shape, dtype=np.float32)
    v = np.random.Generator(np.random.Philox(ss[1])).standard_normal(shape, dtype=np.float32)
    return k.astype(np.float16), v.astype(np.float16)


# Prompt-phase batches (section 4.2: a prompt machine batches prompts up to 2048 tokens in
# total; section 3.1: prompt medians 1500 tokens for coding, 1020 for conversation).
PREFILL_CONFIGS = {
    "prefill_tiny": Config("prefill_tiny", 3, 4, 2, 128, 160, ("fixed", (1, 37, 160)),
                           n_layers=1, seed_index=11),
    # Llama-2-70B share: one coding-median prompt plus a short one, 2048 tokens in all
    "prefill_llama70b_tp8": Config("prefill_llama70b_tp8", 2, 8, 1, 128, 2048,
                                   ("fixed", (1500, 548)), n_layers=80, seed_index=12),
    # BLOOM-176B share: two conversation-median prompts
    "prefill_bloom176b_tp8": Config("prefill_bloom176b_tp8", 2, 14, 14, 128, 2048,
                                    ("fixed", (1020, 1020)), n_layers=70, seed_index=13),
    # one long prompt, where the quadratic term dominates
    "prefill_long_8k": Config("prefill_long_8k", 1, 8, 1, 128, 8192, ("fixed", (8192,)),
                              n_layers=80, seed_index=14),
    "prefill_long_32k": Config("prefill_long_32k", 1, 8, 1, 128, 32768, ("fixed", (32768,)),
                               n_layers=80, seed_index=15),
}

# Mixed batches (section 2.4: prompt and token phases of different requests in one forward
# pass).  name -> (shape and context-length recipe, prompts in the batch, tokens per prompt):
# the first `prompts` requests are prompts of that many tokens, all of them queries; the
# others are token-phase requests (one query each) with contexts from the recipe.
MIXED_CONFIGS = {
    # the Llama-2-70B decode batch with one coding-median prompt riding along
    "mixed_llama70b_tp8": (Config("mixed_llama70b_tp8", 64, 8, 1, 128, 4096, ("uniform", 1000, 2600),
                                  n_layers=80, seed_index=16), 1, 1500),
    "mixed_tiny": (Config("mixed_tiny", 6, 4, 2, 128, 160, ("uniform", 1, 160),
                          n_layers=1, seed_index=17), 2, 70),
}


def make_mixed_batch(name, seed=None):
    """(Batch, q_lens int32 [n_req]) of a MIXED_CONFIGS entry."""
    cfg, n_prompts, prompt_len = MIXED_CONFIGS[name]
    drawn = make_batch(cfg, seed=seed)
    lens = np.array(drawn.seq_lens, dtype=np.int64)
    lens[:n_prompts] = prompt_len
    batch = make_batch(cfg, seed=drawn.seed, seq_lens=lens.tolist())
    q_lens = np.ones(cfg.n_req, dtype=np.int32)
    q_lens[:n_prompts] = prompt_len
    return batch, q_lens


def make_prefill_queries(batch, seed=None):
    """Queries of every prompt token of a Batch, packed request after request.

    Returns (q_tokens float16 [n_tokens, n_qh, head_dim], q_starts int32 [n_req]): token i of
    request r is row q_starts[r] + i; n_tokens is the sum of the valid lengths.
    """
    cfg = batch.cfg
    lens = batch.valid_lens.astype(np.int64)
    starts = np.concatenate([[0], np.cumsum(lens)[:-1]]).astype(np.int32)
    n_tokens = int(lens.sum())
    ss = np.random.SeedSequence([int(batch.seed if seed is None else seed), 0x70726F6D])
    rng = np.random.Generator(np.random.Philox(ss))
    q = rng.standard_normal((n_tokens, cfg.n_qh, cfg.head_dim), dtype=np.float32).astype(np.float16)
    return q, starts


def make_mixed_queries(batch, q_lens, seed=None):
    """Queries of a mixed batch: request r contributes its last q_lens[r] tokens (clamped to its
    valid length), packed request after request.

    Returns (q_tokens float16 [n_tokens, n_qh, head_dim], q_starts int32 [n_req], q_lens int32 as
    clamped).
    """
    cfg = batch.cfg
    nq = np.minimum(np.clip(np.asarray(q_lens, dtype=np.int64), 0, None), batch.valid_lens.astype(np.int64))
    starts = np.concatenate([[0], np.cumsum(nq)[:-1]]).astype(np.int32)
    n_tokens = int(nq.sum())
    ss = np.random.SeedSequence([int(batch.seed if seed is None else seed), 0x6D697864])
    rng = np.random.Generator(np.random.Philox(ss))
    q = rng.standard_normal((n_tokens, cfg.n_qh, cfg.head_dim), dtype=np.float32).astype(np.float16)
    return q, starts, nq.astype(np.int32)


def token_rows(batch, q_lens=None):
    """K and V rows of every request's last q_lens[r] tokens (all of them when q_lens is None),
    packed request after request the way a forward pass produces them.

    Returns (k_tok, v_tok float16 [n_tokens, n_kvh, head_dim], q_starts int32, nq int32 as clamped).
    """
    cfg = batch.cfg
    lens = batch.valid_lens.astype(np.int64)
    nq = lens if q_lens is None else np.minimum(np.clip(np.asarray(q_lens, dtype=np.int64), 0, None), lens)
    starts = np.concatenate([[0], np.cumsum(nq)[:-1]]).astype(np.int32)
    n_tokens = int(nq.sum())
    k_tok = np.zeros((n_tokens, cfg.n_kvh, cfg.head_dim), dtype=np.float16)
    v_tok = np.zeros((n_tokens, cfg.n_kvh, cfg.head_dim), dtype=np.float16)
    for r in range(cfg.n_req):
        L, n = int(lens[r]), int(nq[r])
        if n:
            k_tok[starts[r]:starts[r] + n] = batch.k_rows[r][:, L - n:L, :].transpose(1, 0, 2)
            v_tok[starts[r]:starts[r] + n] = batch.v_rows[r][:, L - n:L, :].transpose(1, 0, 2)
    return k_tok, v_tok, starts, nq.astype(np.int32)


def mixed_flops(cfg, lens, q_lens):
    """Algorithmic flops of a mixed batch: 4*head_dim per (query, visible key) pair and head."""
    lens = np.clip(np.asarray(lens, dtype=np.int64), 0, cfg.max_len)
    nq = np.minimum(np.clip(np.asarray(q_lens, dtype=np.int64), 0, None), lens)
    pairs = int((nq * (lens - nq) + nq * (nq + 1) // 2).sum())
    return 4 * cfg.head_dim * pairs * cfg.n_qh


def prefill_flops(cfg, lens):
    """Algorithmic flops of causal attention: 4*head_dim per (query, visible key) pair and head."""
    lens = np.clip(np.asarray(lens, dtype=np.int64), 0, cfg.max_len)
    pairs = int((lens * (lens + 1) // 2).sum())
    return 4 * cfg.head_dim * pairs * cfg.n_qh


def custom_config(name, n_req, n_qh, n_kvh, head_dim, max_len, n_layers=1):
    """A free-form shape for edge-case tests; pass seq_lens to make_batch."""
    return Config(name, n_req, n_qh, n_kvh, head_dim, max_len, ("fixed", (0,) * n_req),
                  n_layers=n_layers, seed_index=0)


def pack_cache(rows, cfg, stride_req, stride_kvh, stride_tok, total_elems, pad_bits=0):
    """Scatter compact valid rows into one flat cache buffer addressed by element strides.

    Everything that is not a valid position (positions >= the request's length,
    stride padding) is filled with the bit pattern pad_bits, e.g. 0x7E00 (a NaN)
    to show that the library never lets padding reach a result.
    Returns a flat uint16 array of total_elems elements.
    """
    buf = np.full(int(total_elems), np.uint16(pad_bits), dtype=np.uint16)
    d = cfg.head_dim
    view = np.lib.stride_tricks.as_strided(
        buf, shape=(cfg.n_req, cfg.n_kvh, cfg.max_len, d),
        strides=(2 * stride_req, 2 * stride_kvh, 2 * stride_tok, 2), writeable=True)
    for r, blk in enumerate(rows):
        L = blk.shape[1]
        if L:
            view[r, :, :L, :] = blk.view(np.uint16)
    return buf


def dense_layout(cfg):
    """Plain dense strides (for CPU-only tests that have no library to ask)."""
    d = cfg.head_dim
    st = d
    sg = cfg.max_len * d
    sr = cfg.n_kvh * sg
    return sr, sg, st, cfg.n_req * sr


def pack_paged(k_rows, v_rows, cfg, block_size, stride_block, stride_kvh, stride_tok, n_blocks,
               seed=0, pad_bits=0, spare_bits=None, room=0):
    """Scatter compact valid rows into K and V block pools with a shuffled block table.

    Request r gets ceil(L_r / block_size) pool blocks drawn without replacement from
    a seeded permutation of all n_blocks, so neighbouring positions land in
    unrelated blocks; blocks that no request owns, the unused tail of a request's
    last block and stride padding hold pad_bits.  Table entries past a request's
    last block hold spare_bits (default: an id far out of range), which the
    library must never follow.
    room > 0 also allots the blocks of the next `room` positions of every request
    (up to max_len), for callers that go on to append tokens.
    Returns (k_pool, v_pool, block_table) as flat uint16 / uint16 / int32 [n_req, max_blocks].
    """
    d = cfg.head_dim
    max_blocks = -(-cfg.max_len // block_size)

    def owned(L):
        return -(-min(L + room, cfg.max_len) // block_size)

    need = sum(owned(blk.shape[1]) for blk in k_rows)
    if need > n_blocks:
        raise ValueError("pool of %d blocks cannot hold %d" % (n_blocks, need))
    total = int(n_blocks) * int(stride_block)
    k_pool = np.full(total, np.uint16(pad_bits), dtype=np.uint16)
    v_pool = np.full(total, np.uint16(pad_bits), dtype=np.uint16)
    shape = (n_blocks, cfg.n_kvh, block_size, d)
    strides = (2 * stride_block, 2 * stride_kvh, 2 * stride_tok, 2)
    kv = np.lib.stride_tricks.as_strided(k_pool, shape=shape, strides=strides, writeable=True)
    vv = np.lib.stride_tricks.as_strided(v_pool, shape=shape, strides=strides, writeable=True)
    order = np.random.Generator(np.random.Philox(int(seed) + 77)).permutation(n_blocks)
    table = np.full((cfg.n_req, max_blocks), 0x3FFFFFF0 if spare_bits is None else spare_bits,
                    dtype=np.int32)
    nxt = 0
    for r, (kb, vb) in enumerate(zip(k_rows, v_rows)):
        L = kb.shape[1]
        for i in range(owned(L)):
            b = int(order[nxt])
            nxt += 1
            table[r, i] = b
            n = min(block_size, L - i * block_size)
            if n <= 0:
                continue
            kv[b, :, :n, :] = kb[:, i * block_size:i * block_size + n, :].view(np.uint16)
            vv[b, :, :n, :] = vb[:, i * block_size:i * block_size + n, :].view(np.uint16)
    return k_pool, v_pool, table


def dense_paged_layout(cfg, block_size):
    """Plain dense pool strides (for CPU-only tests that have no library to ask)."""
    st = cfg.head_dim
    sg = block_size * st
    sb = cfg.n_kvh * sg
    return sb, sg, st
