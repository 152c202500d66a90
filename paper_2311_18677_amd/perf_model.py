"""Piece-wise linear performance model of the token-phase attention call.

The paper drives its cluster simulator with a piece-wise linear performance
model fitted to profiles at various batch and sequence sizes and validates it
on an 80:20 train:test split (section 5.2, "Performance model": mean absolute
percentage error below 3 %).  This module does the same for this library's own
measurements on one MI355X:

    python -m paper_2311_18677_amd.perf_model --sweep out.txt     (needs the GPU)
    python -m paper_2311_18677_amd.perf_model --fit out.txt       (CPU only)

The model is a continuous function of (batch size, context length) that is
linear inside every cell of a knot grid: a tensor product of one-dimensional
"hat" bases, fitted by least squares.  Both axes are used in log2 units, which
is how the profile points are spaced.
"""
import argparse
import math
import sys
import time

import numpy as np


def hat_basis(x, knots):
    """Values of the piece-wise linear hat functions on `knots` at points x: [len(x), len(knots)].

    Rows sum to one; points outside the knot range take the value of the nearest end
    (clamped), so the model never extrapolates a slope.
    """
    knots = np.asarray(knots, dtype=np.float64)
    if knots.ndim != 1 or knots.size < 2 or np.any(np.diff(knots) <= 0):
        raise ValueError("knots must be at least two strictly increasing values")
    x = np.clip(np.asarray(x, dtype=np.float64), knots[0], knots[-1])
    idx = np.clip(np.searchsorted(knots, x, side="right") - 1, 0, knots.size - 2)
    w = (x - knots[idx]) / (knots[idx + 1] - knots[idx])
    out = np.zeros((x.size, knots.size))
    rows = np.arange(x.size)
    out[rows, idx] = 1.0 - w
    out[rows, idx + 1] += w
    return out


class PiecewiseLinearModel:
    """time(batch, context): linear inside every cell of (batch knots) x (context knots)."""

    def __init__(self, batch_knots, context_knots, log_time=False):
        """log_time: fit log2(time) instead of time, i.e. a power law inside every cell; the
        choice for quantities that grow faster than linearly (prompt attention is quadratic
        in the prompt length)."""
        self.bk = np.log2(np.asarray(batch_knots, dtype=np.float64))
        self.ck = np.log2(np.asarray(context_knots, dtype=np.float64))
        self.log_time = bool(log_time)
        self.coef = None

    def _design(self, batch, context):
        hb = hat_basis(np.log2(np.asarray(batch, dtype=np.float64)), self.bk)
        hc = hat_basis(np.log2(np.asarray(context, dtype=np.float64)), self.ck)
        return (hb[:, :, None] * hc[:, None, :]).reshape(hb.shape[0], -1)

    def fit(self, batch, context, t):
        a = self._design(batch, context)
        # a small ridge keeps grid nodes that no training point touches finite
        lam = 1e-9
        ata = a.T @ a + lam * np.eye(a.shape[1])
        t = np.asarray(t, dtype=np.float64)
        self.coef = np.linalg.solve(ata, a.T @ (np.log2(t) if self.log_time else t))
        return self

    def predict(self, batch, context):
        if self.coef is None:
            raise RuntimeError("fit first")
        y = self._design(batch, context) @ self.coef
        return np.exp2(y) if self.log_time else y


class RegimeModel:
    """Separate piece-wise linear surfaces per context regime (discontinuous at the breaks).

    The library changes how it works at fixed context limits (one chunk per request up to
    256 positions, a single launch up to 1024, two kernels beyond, longer chunks beyond 4096),
    and the call time steps there; a continuous model would smear each step over a whole knot interval.
    regimes: list of (upper context bound inclusive, context knots inside the regime).
    """

    def __init__(self, batch_knots, regimes):
        self.regimes = [(float(hi), PiecewiseLinearModel(batch_knots, ck)) for hi, ck in regimes]

    def _which(self, context):
        context = np.asarray(context, dtype=np.float64)
        idx = np.zeros(context.shape, dtype=np.int64)
        for i, (hi, _) in enumerate(self.regimes[:-1]):
            idx[context > hi] = i + 1
        return idx

    def fit(self, batch, context, t):
        batch, context, t = (np.asarray(x, dtype=np.float64) for x in (batch, context, t))
        idx = self._which(context)
        for i, (_, m) in enumerate(self.regimes):
            sel = idx == i
            if sel.any():
                m.fit(batch[sel], context[sel], t[sel])
        return self

    def predict(self, batch, context):
        batch, context = (np.asarray(x, dtype=np.float64) for x in (batch, context))
        idx = self._which(context)
        out = np.zeros(batch.shape)
        for i, (_, m) in enumerate(self.regimes):
            sel = idx == i
            if sel.any():
                if m.coef is None:
                    raise RuntimeError("regime %d was never fitted" % i)
                out[sel] = m.predict(batch[sel], context[sel])
        return out


def mape(pred, true):
    pred, true = np.asarray(pred, dtype=np.float64), np.asarray(true, dtype=np.float64)
    return float(np.mean(np.abs(pred - true) / np.abs(true))) * 100.0


def split_80_20(n, seed=0):
    """Seeded 80:20 split of range(n): (train indices, test indices)."""
    order = np.random.Generator(np.random.Philox(int(seed))).permutation(n)
    n_test = max(1, int(round(0.2 * n)))
    return np.sort(order[n_test:]), np.sort(order[:n_test])


def evaluate(batch, context, t, batch_knots, context_knots, seed=0, regimes=None, log_time=False):
    """Fit on 80 %, report MAPE on the held-out 20 % and on the training points.

    With `regimes` (see RegimeModel) the context axis is cut there and context_knots is unused.
    """
    batch, context, t = (np.asarray(x, dtype=np.float64) for x in (batch, context, t))
    tr, te = split_80_20(batch.size, seed)
    if regimes is not None:
        m = RegimeModel(batch_knots, regimes)
    else:
        m = PiecewiseLinearModel(batch_knots, context_knots, log_time=log_time)
    m.fit(batch[tr], context[tr], t[tr])
    return {"train_mape": mape(m.predict(batch[tr], context[tr]), t[tr]),
            "test_mape": mape(m.predict(batch[te], context[te]), t[te]),
            "n_train": int(tr.size), "n_test": int(te.size), "model": m}


# ---- measurement on the GPU -------------------------------------------------------------

BATCHES = (1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64, 96, 128)
CONTEXTS = (128, 192, 256, 384, 512, 768, 1024, 1536, 2048, 3072, 4096, 6144, 8192)
# knots at the powers of two; the profile grid also has the points half-way between them
BATCH_KNOTS = (1, 2, 4, 8, 16, 32, 64, 128)
CONTEXT_KNOTS = (128, 256, 512, 1024, 2048, 4096, 8192)
# where sw_decode_attn's call time steps (context = max_len): one chunk per request up to 256
# positions, a single launch up to 1024 (four chunks), two kernels beyond; context knots inside
# each regime
REGIMES = ((256, (128, 256)), (1024, (384, 1024)), (8192, (1536, 4096, 8192)))
REGIME_BATCH_KNOTS = (1, 8, 16, 32, 64, 128)


def measure_point(sw, torch, n_req, ctx, n_qh=8, n_kvh=1, d=128, calls=1500, budget_bytes=1 << 30):
    """Microseconds per sw_decode_attn call, all requests at context ctx, rotating over
    enough cache sets to keep the rows out of the last-level cache (at most 48 sets)."""
    dev = torch.device("cuda:0")
    lay = sw.sw_kv_layout(n_req, n_kvh, d, ctx)
    kv_bytes = n_req * n_kvh * ctx * d * 4
    n_sets = int(min(48, max(2, budget_bytes // max(kv_bytes, 1))))
    g = torch.Generator(device=dev)
    g.manual_seed(1000 * n_req + ctx)
    sets = []
    for _ in range(n_sets):
        s = {}
        for name in ("k", "v"):
            s[name] = torch.empty(lay.total_elems, dtype=torch.float16, device=dev).normal_(0.0, 1.0, generator=g)
        s["q"] = torch.empty(n_req * n_qh * d, dtype=torch.float16, device=dev).normal_(0.0, 1.0, generator=g)
        s["lens"] = torch.full((n_req,), ctx, dtype=torch.int32, device=dev)
        s["out"] = torch.zeros(n_req * n_qh * d, dtype=torch.float16, device=dev)
        sets.append(s)
    stream = torch.cuda.Stream(device=dev)

    def call(s, st):
        sw.sw_decode_attn(s["q"], s["k"], s["v"], s["lens"], s["out"], n_req, n_qh, n_kvh, d, ctx, st)

    call(sets[0], stream)
    stream.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        for s in sets:
            call(s, torch.cuda.current_stream())
    torch.cuda.synchronize()
    reps = max(2, calls // n_sets)
    with torch.cuda.stream(stream):
        for _ in range(max(1, reps // 5)):
            graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    with torch.cuda.stream(stream):
        for _ in range(reps):
            graph.replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / (reps * n_sets) * 1e6


def sweep(path):
    import torch
    from . import binding as sw
    if not torch.cuda.is_available():
        print("perf_model: no GPU visible", file=sys.stderr)
        return 1
    sw.load()
    with open(path, "w") as f:
        f.write("# sw_decode_attn, 8 query heads on 1 KV head, head_dim 128, every request at the "
                "given context\n# batch context microseconds_per_call\n")
        for b in BATCHES:
            for c in CONTEXTS:
                us = measure_point(sw, torch, b, c)
                f.write("%d %d %.3f\n" % (b, c, us))
                f.flush()
            print("batch", b, "done", flush=True)
            sw.sw_release()
            torch.cuda.empty_cache()
    return 0


# ---- the prompt phase: time of one sw_prefill_attn call vs (prompts in the batch, prompt length)

PROMPT_COUNTS = (1, 2, 3, 4, 6, 8, 12, 16)
PROMPT_LENS = (64, 96, 128, 192, 256, 384, 512, 768, 1024, 1536, 2048, 3072, 4096, 6144, 8192)
PROMPT_MAX_TOKENS = 32768           # batches above this many tokens are left out of the grid
PROMPT_COUNT_KNOTS = (1, 2, 4, 8, 16)
PROMPT_LEN_KNOTS = (64, 128, 256, 512, 1024, 2048, 4096, 8192)


def measure_prompt_point(sw, torch, n_req, plen, n_qh=8, n_kvh=1, d=128, calls=960, n_sets=3):
    """Microseconds per sw_prefill_attn call on n_req prompts of plen tokens each."""
    dev = torch.device("cuda:0")
    lay = sw.sw_kv_layout(n_req, n_kvh, d, plen)
    n_tokens = n_req * plen
    g = torch.Generator(device=dev)
    g.manual_seed(7000 * n_req + plen)
    sets = []
    for _ in range(n_sets):
        s = {}
        for name in ("k", "v"):
            s[name] = torch.empty(lay.total_elems, dtype=torch.float16, device=dev).normal_(0.0, 1.0, generator=g)
        s["q"] = torch.empty(n_tokens * n_qh * d, dtype=torch.float16, device=dev).normal_(0.0, 1.0, generator=g)
        s["out"] = torch.zeros(n_tokens * n_qh * d, dtype=torch.float16, device=dev)
        sets.append(s)
    lens = torch.full((n_req,), plen, dtype=torch.int32, device=dev)
    starts = (torch.arange(n_req, dtype=torch.int32, device=dev) * plen).contiguous()
    stream = torch.cuda.Stream(device=dev)

    def call(s, st):
        sw.sw_prefill_attn(s["q"], s["k"], s["v"], lens, starts, s["out"], n_tokens, n_req, n_qh, n_kvh, d, plen, st)

    call(sets[0], stream)
    stream.synchronize()
    # many calls per graph, so that the cost of starting a replay disappears in them
    rounds = 16
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        for _ in range(rounds):
            for s in sets:
                call(s, torch.cuda.current_stream())
    torch.cuda.synchronize()
    per_replay = rounds * n_sets
    # long calls need few repetitions: aim at a few tens of milliseconds per point
    with torch.cuda.stream(stream):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    with torch.cuda.stream(stream):
        graph.replay()
    torch.cuda.synchronize()
    once = max(time.perf_counter() - t0, 1e-6)
    reps = int(max(1, min(max(1, calls // per_replay), 0.03 / once)))
    t0 = time.perf_counter()
    with torch.cuda.stream(stream):
        for _ in range(reps):
            graph.replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / (reps * per_replay) * 1e6


def sweep_prompt(path):
    import torch
    from . import binding as sw
    if not torch.cuda.is_available():
        print("perf_model: no GPU visible", file=sys.stderr)
        return 1
    sw.load()
    with open(path, "w") as f:
        f.write("# sw_prefill_attn, 8 query heads on 1 KV head, head_dim 128, every prompt of the "
                "given length\n# prompts prompt_tokens microseconds_per_call\n")
        for b in PROMPT_COUNTS:
            for c in PROMPT_LENS:
                if b * c > PROMPT_MAX_TOKENS:
                    continue
                us = measure_prompt_point(sw, torch, b, c)
                f.write("%d %d %.3f\n" % (b, c, us))
                f.flush()
            print("prompts", b, "done", flush=True)
            torch.cuda.empty_cache()
    return 0


def load_points(path):
    rows = [ln.split() for ln in open(path) if ln.strip() and not ln.startswith("#")]
    arr = np.array(rows, dtype=np.float64)
    return arr[:, 0], arr[:, 1], arr[:, 2]


MIXED_BATCHES = [8, 16, 32, 64]
MIXED_PROMPTS = [0, 64, 128, 256, 512, 1024, 1536, 2048]
MIXED_CONTEXT = 1536


MIXED_MAX_LEN = 4096


def measure_mixed_point(sw, torch, n_decode, ctx, prompt_tokens, n_qh=8, n_kvh=1, d=128, calls=960, n_sets=6,
                        max_len=MIXED_MAX_LEN):
    """Microseconds per sw_mixed_attn call: n_decode token-phase requests at context ctx and,
    if prompt_tokens > 0, one whole prompt of that many tokens in the same call (section 2.4).
    The caches are laid out for max_len positions, as a token machine's are."""
    dev = torch.device("cuda:0")
    n_req = n_decode + (1 if prompt_tokens > 0 else 0)
    max_len = max(max_len, ctx, prompt_tokens)
    lay = sw.sw_kv_layout(n_req, n_kvh, d, max_len)
    n_tokens = n_decode + prompt_tokens
    g = torch.Generator(device=dev)
    g.manual_seed(9000 * n_decode + prompt_tokens)
    sets = []
    for _ in range(n_sets):
        s = {}
        for name in ("k", "v"):
            s[name] = torch.empty(lay.total_elems, dtype=torch.float16, device=dev).normal_(0.0, 1.0, generator=g)
        s["q"] = torch.empty(n_tokens * n_qh * d, dtype=torch.float16, device=dev).normal_(0.0, 1.0, generator=g)
        s["out"] = torch.zeros(n_tokens * n_qh * d, dtype=torch.float16, device=dev)
        sets.append(s)
    lens = [ctx] * n_decode + ([prompt_tokens] if prompt_tokens > 0 else [])
    q_lens = [1] * n_decode + ([prompt_tokens] if prompt_tokens > 0 else [])
    starts = [0]
    for x in q_lens[:-1]:
        starts.append(starts[-1] + x)
    lens_d = torch.tensor(lens, dtype=torch.int32, device=dev)
    q_lens_d = torch.tensor(q_lens, dtype=torch.int32, device=dev)
    starts_d = torch.tensor(starts, dtype=torch.int32, device=dev)
    stream = torch.cuda.Stream(device=dev)

    def call(s, st):
        sw.sw_mixed_attn(s["q"], s["k"], s["v"], lens_d, starts_d, q_lens_d, s["out"], n_tokens, n_req,
                         n_qh, n_kvh, d, max_len, max(1, prompt_tokens), st)

    call(sets[0], stream)
    stream.synchronize()
    rounds = 8
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        for _ in range(rounds):
            for s in sets:
                call(s, torch.cuda.current_stream())
    torch.cuda.synchronize()
    per_replay = rounds * n_sets
    reps = max(2, calls // per_replay)
    with torch.cuda.stream(stream):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    with torch.cuda.stream(stream):
        for _ in range(reps):
            graph.replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / (reps * per_replay) * 1e6


def sweep_mixed(path):
    """What a prompt riding along costs the token phase (the paper's mixed batching, section 2.4):
    token-phase batch x prompt tokens in the same call, written as a table."""
    import torch
    from . import binding as sw
    if not torch.cuda.is_available():
        print("perf_model: no GPU visible", file=sys.stderr)
        return 1
    sw.load()
    with open(path, "w") as f:
        f.write("# sw_mixed_attn, 8 query heads on 1 KV head, head_dim 128: token-phase requests at context %d "
                "(caches laid out for %d positions) plus one whole prompt in the same call\n"
                "# token_requests prompt_tokens microseconds_per_call\n" % (MIXED_CONTEXT, MIXED_MAX_LEN))
        for b in MIXED_BATCHES:
            for p in MIXED_PROMPTS:
                us = measure_mixed_point(sw, torch, b, MIXED_CONTEXT, p)
                f.write("%d %d %.3f\n" % (b, p, us))
                f.flush()
            print("token-phase batch", b, "done", flush=True)
            sw.sw_release()
            torch.cuda.empty_cache()
    return 0


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--sweep", metavar="FILE", help="measure the grid on the GPU and write it to FILE")
    ap.add_argument("--fit", metavar="FILE", help="fit the model to FILE (80:20 split) and print the errors")
    ap.add_argument("--sweep-prompt", metavar="FILE", help="the prompt-phase grid: measure and write to FILE")
    ap.add_argument("--fit-prompt", metavar="FILE", help="fit the prompt-phase model to FILE (80:20 split)")
    ap.add_argument("--sweep-mixed", metavar="FILE", help="token-phase batch x prompt tokens in one call: measure, write")
    ap.add_argument("--seed", type=int, default=0)
    args = ap.parse_args(argv)
    if args.sweep_mixed:
        return sweep_mixed(args.sweep_mixed)
    if args.sweep_prompt or args.fit_prompt:
        if args.sweep_prompt:
            rc = sweep_prompt(args.sweep_prompt)
            if rc:
                return rc
        b, c, t = load_points(args.fit_prompt or args.sweep_prompt)
        res = evaluate(b, c, t, PROMPT_COUNT_KNOTS, PROMPT_LEN_KNOTS, seed=args.seed, log_time=True)
        print("prompt phase: points %d (train %d, test %d)  train MAPE %.2f %%  held-out MAPE %.2f %%"
              % (b.size, res["n_train"], res["n_test"], res["train_mape"], res["test_mape"]))
        lin = evaluate(b, c, t, PROMPT_COUNT_KNOTS, PROMPT_LEN_KNOTS, seed=args.seed)
        print("(linear in time inside a cell instead of a power law: held-out MAPE %.2f %%)" % lin["test_mape"])
        return 0
    if args.sweep:
        rc = sweep(args.sweep)
        if rc:
            return rc
    path = args.fit or args.sweep
    if not path:
        ap.error("give --sweep FILE or --fit FILE")
    b, c, t = load_points(path)
    res = evaluate(b, c, t, REGIME_BATCH_KNOTS, None, seed=args.seed, regimes=REGIMES)
    print("points %d (train %d, test %d)  train MAPE %.2f %%  held-out MAPE %.2f %%"
          % (b.size, res["n_train"], res["n_test"], res["train_mape"], res["test_mape"]))
    one = evaluate(b, c, t, BATCH_KNOTS, CONTEXT_KNOTS, seed=args.seed)
    print("(one continuous surface instead of one per regime: held-out MAPE %.2f %%)" % one["test_mape"])
    return 0


if __name__ == "__main__":
    sys.exit(main())
