"""CPU oracle for the partition hot path of model-distributed LLM inference.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library, its
Python binding, the pipeline driver) may import or call this module; it is used
by tests/, by __graft_entry__.smoke() and by the cpu_baseline leg of bench.py.
It shares no code with the HIP path and imports nothing from the package.

What it computes.  The paper fixes the *schedule* of model-distributed
inference (Sec. III-A..III-E, Alg. 1 and Alg. 2): a node owns a contiguous
slice of decoder layers, receives the activations of sample n, runs its slice
with the n-th KV cache, and passes the result on; the first visit of a sample
carries the whole prompt, later visits only the newest token (Sec. III-D).  It
gives no equations for the layers themselves and points to the Llama family
(RoPE, GQA, KV caching; Sec. IV-A).  Partitioning, pipelining and caching do
not approximate anything: they reach exactly the forward pass of the unsplit,
uncached decoder.  The oracle is therefore that plain definition written out
with numpy, in float64 (weights arrive as fp32 values, possibly bf16-rounded,
and are widened), with `matmul` as the only library step.  Passing
dtype=np.float32 gives the precision the paper's testbed ran in (Sec. IV-A).

Pins (tests/test_oracle_*.py): softmax rows sum to 1; attention against
explicit triple loops; causality; GQA == MHA with repeated kv heads; cached
decode == full-prefix recompute; composed partitions == unsplit model;
interleaved samples == each sample alone; norm/RoPE/activation closed forms;
identity layer when the output matrices vanish; the output layers (final norm,
then the vocabulary projection, tied and untied) against scalar loops;
Alg. 1/2 visit counts; the counter-based generator against its published known answers; the sampler
against the distribution it is defined to draw from.
Whole-model numeric values are "parity unpinned" by the paper: it prints no
logits or tokens and its trained weights are not available.
"""
from __future__ import annotations

import math

import numpy as np
from scipy.special import erf as _erf

# integer codes of the configuration fields (same meaning as in the C header)
NORM_LAYERNORM, NORM_RMSNORM = 0, 1
MLP_GELU_TANH, MLP_GELU_ERF, MLP_SWIGLU = 0, 1, 2
POS_LEARNED, POS_ROPE = 0, 1


# --------------------------------------------------------------------------
# elementwise pieces
def layernorm(x, g, b, eps):
    """(x - mean) / sqrt(var + eps) * g + b over the last axis, biased variance."""
    mu = x.mean(axis=-1, keepdims=True)
    xc = x - mu
    var = (xc * xc).mean(axis=-1, keepdims=True)
    return xc / np.sqrt(var + eps) * g + b


def rmsnorm(x, g, eps):
    """x / sqrt(mean(x^2) + eps) * g over the last axis."""
    ms = (x * x).mean(axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * g


def gelu_tanh(x):
    return 0.5 * x * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (x + 0.044715 * x ** 3)))


def gelu_erf(x):
    return 0.5 * x * (1.0 + _erf(x / math.sqrt(2.0)))


def silu(x):
    return x / (1.0 + np.exp(-x))


def softmax_rows(s):
    """exp(s - max) / sum over the last axis."""
    e = np.exp(s - s.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def rope_rotate(x, positions, base):
    """Rotary embedding, half-split pairing.

    x: [T, n_heads, h]; positions: [T].  For i in [0, h/2) the pair
    (x[..., i], x[..., i + h/2]) is rotated by the angle p * base**(-2i/h).
    """
    T, nh, h = x.shape
    half = h // 2
    inv_freq = np.asarray(base, dtype=np.float64) ** (-2.0 * np.arange(half, dtype=np.float64) / h)
    ang = np.asarray(positions, dtype=np.float64)[:, None] * inv_freq[None, :]      # [T, half]
    c = np.cos(ang).astype(x.dtype)[:, None, :]
    s = np.sin(ang).astype(x.dtype)[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, a * s + b * c], axis=-1)


def causal_attention(q, k, v, q_pos0):
    """Scaled dot-product attention with grouped kv heads.

    q: [T, H, h] are queries at absolute positions q_pos0 .. q_pos0+T-1;
    k, v: [c, K, h] hold keys/values of positions 0 .. c-1 (c = q_pos0 + T).
    Query head j reads kv head j // (H/K) and sees positions <= its own.
    """
    T, H, h = q.shape
    c, K, _ = k.shape
    group = H // K
    out = np.empty_like(q)
    scale = 1.0 / math.sqrt(h)
    for j in range(H):
        kj, vj = k[:, j // group, :], v[:, j // group, :]
        s = (q[:, j, :] @ kj.T) * scale                                  # [T, c]
        key_pos = np.arange(c)[None, :]
        qry_pos = (q_pos0 + np.arange(T))[:, None]
        s = np.where(key_pos <= qry_pos, s, -np.inf)
        out[:, j, :] = softmax_rows(s) @ vj
    return out


# --------------------------------------------------------------------------
# one decoder block and the two ends of the model
def _norm(cfg, x, g, b):
    if cfg["norm_kind"] == NORM_LAYERNORM:
        return layernorm(x, g, b, cfg["norm_eps"])
    return rmsnorm(x, g, cfg["norm_eps"])


def _lin(x, w, b=None):
    y = x @ w.T
    return y if b is None else y + b


def block_forward(cfg, lw, x, cache, pos0):
    """Pre-norm decoder block on rows x[T, d] sitting at positions pos0..pos0+T-1.

    `cache` is {"k": [c0, K, h], "v": [c0, K, h]} for positions < pos0 and is
    extended in place by the T new rows (pass empty arrays for no history).
    """
    T, d = x.shape
    H, K, h = cfg["n_head"], cfg["n_kv_head"], cfg["head_dim"]
    a = _norm(cfg, x, lw["ln1_g"], lw.get("ln1_b"))
    q = _lin(a, lw["wq"], lw.get("bq")).reshape(T, H, h)
    k = _lin(a, lw["wk"], lw.get("bk")).reshape(T, K, h)
    v = _lin(a, lw["wv"], lw.get("bv")).reshape(T, K, h)
    if cfg["pos_kind"] == POS_ROPE:
        pos = pos0 + np.arange(T)
        q = rope_rotate(q, pos, cfg["rope_base"])
        k = rope_rotate(k, pos, cfg["rope_base"])
    cache["k"] = np.concatenate([cache["k"], k], axis=0)
    cache["v"] = np.concatenate([cache["v"], v], axis=0)
    o = causal_attention(q, cache["k"], cache["v"], pos0).reshape(T, H * h)
    x = x + _lin(o, lw["wo"], lw.get("bo"))
    m = _norm(cfg, x, lw["ln2_g"], lw.get("ln2_b"))
    if cfg["mlp_kind"] == MLP_SWIGLU:
        u = silu(_lin(m, lw["wg"])) * _lin(m, lw["wu"])
        x = x + _lin(u, lw["wd"])
    else:
        act = gelu_tanh if cfg["mlp_kind"] == MLP_GELU_TANH else gelu_erf
        u = act(_lin(m, lw["w1"], lw.get("b1")))
        x = x + _lin(u, lw["w2"], lw.get("b2"))
    return x


def embed(cfg, w, ids, pos0):
    x = w["wte"][np.asarray(ids, dtype=np.int64)]
    if cfg["pos_kind"] == POS_LEARNED:
        x = x + w["wpe"][pos0:pos0 + len(ids)]
    return x


def head_logits(cfg, w, x):
    """Final norm followed by the vocabulary projection; x: [T, d] -> [T, V]."""
    return _lin(_norm(cfg, x, w["lnf_g"], w.get("lnf_b")), w["lm_head"])


def greedy(logits):
    """Index of the largest logit, the lowest index on exact ties."""
    return int(np.argmax(logits))


def pmf(logits):
    """The probability mass function the paper samples from (Alg. 1)."""
    return softmax_rows(np.asarray(logits))


# --------------------------------------------------------------------------
def _cast_tree(w, dtype):
    if isinstance(w, dict):
        return {k: _cast_tree(v, dtype) for k, v in w.items()}
    return None if w is None else np.asarray(w, dtype=dtype)


class Partition:
    """One node's model chunk (Sec. III-A/III-B): layers [lo, hi) with one KV
    cache per sample, optionally the embedding (starter's input portion) and
    the final norm + vocabulary projection (starter's output portion)."""

    def __init__(self, cfg, weights, lo, hi, has_embed=False, has_head=False, dtype=np.float64):
        self.cfg, self.lo, self.hi = dict(cfg), lo, hi
        self.has_embed, self.has_head = has_embed, has_head
        self.dtype = dtype
        self.w = {k: _cast_tree(v, dtype) for k, v in weights.items() if k != "layers"}
        self.layers = [_cast_tree(weights["layers"][L], dtype) for L in range(lo, hi)]
        self.caches = {}                       # sample id -> list over local layers of {"k","v"}

    def seq_len(self, n):
        return self.caches[n]["len"] if n in self.caches else 0

    def _empty_cache(self):
        K, h = self.cfg["n_kv_head"], self.cfg["head_dim"]
        z = lambda: np.zeros((0, K, h), dtype=self.dtype)
        return {"len": 0, "layers": [{"k": z(), "v": z()} for _ in self.layers]}

    def _forward(self, n, acts):
        st = self.caches[n]
        pos0 = st["len"]
        if self.has_embed:
            x = embed(self.cfg, self.w, acts, pos0).astype(self.dtype)
        else:
            x = np.asarray(acts, dtype=self.dtype)
            x = x.reshape(-1, self.cfg["d_model"])
        if pos0 + x.shape[0] > self.cfg["max_ctx"]:
            raise ValueError("context overflow")
        for lw, cache in zip(self.layers, st["layers"]):
            x = block_forward(self.cfg, lw, x, cache, pos0)
        st["len"] = pos0 + x.shape[0]
        return x

    def prefill(self, n, acts):
        """First visit of sample n: initialise its cache, run all T rows (Alg. 2)."""
        if n in self.caches:
            raise RuntimeError("sample already has a cache")
        self.caches[n] = self._empty_cache()
        return self._forward(n, acts)

    def prefill_chunk(self, n, acts):
        """The next piece of a first visit: the rows continue at the cache length (an empty cache is created for a
        fresh sample).  Pieces compute what one first visit of the whole prompt computes."""
        if n not in self.caches:
            self.caches[n] = self._empty_cache()
        return self._forward(n, acts)

    def decode_step(self, n, act):
        """Later visit: newest token only, extending cache n (Sec. III-D)."""
        if n not in self.caches:
            raise RuntimeError("decode before first visit")
        if self.has_embed:
            act = np.asarray(act).reshape(1)
        return self._forward(n, act)[0]

    def logits(self, x):
        return head_logits(self.cfg, self.w, np.asarray(x, dtype=self.dtype).reshape(1, -1))[0]

    def sample_greedy(self, x):
        lg = self.logits(x)
        return greedy(lg), lg

    def sample_topk(self, x, temperature, top_k, seed, sample, step):
        """Output layers, then a draw from the top-k tempered pmf with the counter-based uniform of
        (seed, sample, step).  Returns (token, logits)."""
        lg = self.logits(x)
        return sample_topk(lg, temperature, top_k, uniform01(seed, sample, step)), lg

    def reset(self, n):
        self.caches.pop(n, None)


# --------------------------------------------------------------------------
# stochastic sampling of the output pmf (Alg. 1, "sample the output distribution"; the paper names no knobs: the
# usual ones of the Llama-family generation loops it builds on, temperature and top-k, are taken)
_PHILOX_M0, _PHILOX_M1, _PHILOX_W0, _PHILOX_W1 = 0xD2511F53, 0xCD9E8D57, 0x9E3779B9, 0xBB67AE85


def philox4x32_10(counter, key):
    """Philox-4x32 with 10 rounds (Salmon et al., "Parallel random numbers: as easy as 1, 2, 3", SC'11): a
    counter-based generator, i.e. a keyed bijection of 128-bit counters; plain Python integers."""
    c0, c1, c2, c3 = (int(v) & 0xFFFFFFFF for v in counter)
    k0, k1 = (int(v) & 0xFFFFFFFF for v in key)
    for rnd in range(10):
        if rnd:
            k0 = (k0 + _PHILOX_W0) & 0xFFFFFFFF
            k1 = (k1 + _PHILOX_W1) & 0xFFFFFFFF
        p0, p1 = _PHILOX_M0 * c0, _PHILOX_M1 * c2
        c0, c1, c2, c3 = ((p1 >> 32) ^ c1 ^ k0) & 0xFFFFFFFF, p1 & 0xFFFFFFFF, ((p0 >> 32) ^ c3 ^ k1) & 0xFFFFFFFF, p0 & 0xFFFFFFFF
    return c0, c1, c2, c3


def uniform01(seed, sample, step):
    """The uniform number in [0, 1) that decides the token of `sample` at generation step `step`: the top 24 bits
    of the first Philox word for counter (sample, step, 0, 0) and key = the two halves of the 64-bit seed, so that
    it is exactly representable in binary32."""
    x0 = philox4x32_10((sample, step, 0, 0), (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF))[0]
    return (x0 >> 8) / float(1 << 24)


def sample_topk(logits, temperature, top_k, u):
    """Token drawn from softmax(logits / temperature) restricted to the top_k largest logits (ties: the lower
    index ranks first), by inverting the cumulative distribution at u: candidates in rank order, weights
    w_j = exp((l_j - l_max) / temperature), the token is the first j with u * sum(w) < w_0 + ... + w_j.
    The arithmetic that decides the token runs in binary32, in this order, because a floating-point comparison
    decides an integer here and the GPU kernel takes it in binary32 too."""
    lg = np.asarray(logits, dtype=np.float32)
    k = int(min(top_k, lg.shape[0]))
    order = sorted(range(lg.shape[0]), key=lambda i: (-float(lg[i]), i))[:k]
    inv_t = np.float32(1.0) / np.float32(temperature)
    lmax = lg[order[0]]
    w = [np.exp((lg[i] - lmax) * inv_t, dtype=np.float32) for i in order]
    total = np.float32(0.0)
    for x in w:
        total = np.float32(total + x)
    target = np.float32(np.float32(u) * total)
    acc = np.float32(0.0)
    for j, x in enumerate(w):
        acc = np.float32(acc + x)
        if target < acc:
            return order[j]
    return order[-1]


def topk_pmf(logits, temperature, top_k):
    """The distribution sample_topk draws from, in float64: {token: probability}."""
    lg = np.asarray(logits, dtype=np.float64)
    order = sorted(range(lg.shape[0]), key=lambda i: (-lg[i], i))[:int(min(top_k, lg.shape[0]))]
    w = np.exp((lg[order] - lg[order[0]]) / float(temperature))
    return dict(zip(order, w / w.sum()))


def forward_no_cache(cfg, weights, ids_or_acts, lo, hi, has_embed, dtype=np.float64):
    """The mode the paper argues against (Sec. III-D): every pass carries the
    whole context and recomputes all keys and values.  Returns all rows."""
    p = Partition(cfg, weights, lo, hi, has_embed=has_embed, dtype=dtype)
    return p.prefill(0, ids_or_acts)


# --------------------------------------------------------------------------
# the schedule (Alg. 1 and Alg. 2)
def starter_schedule(n_samples, n_rounds):
    """Iterations of the starter loop, Alg. 1, with k read as 0-based.

    Iteration k serves sample n = k mod n_samples in round r = k // n_samples.
    Round 0 initialises the cache and forwards the whole prompt; every later
    round first applies the output layers and appends a token; every round but
    the last forwards (the newest token) through the input layers and enqueues
    the result.  Returns a list of (k, n, r, runs_head, runs_forward, is_prefill).
    """
    out = []
    for k in range(n_samples * n_rounds):
        n, r = k % n_samples, k // n_samples
        first = k < n_samples
        fwd = k < n_samples * (n_rounds - 1)
        out.append((k, n, r, not first, fwd, first and fwd))
    return out


def generate(parts, prompts, n_new, trace=None, sampling=None, head=None):
    """Recurrent pipeline parallelism on a chain of partitions (Sec. III-C).

    parts[0] owns the embedding, parts[-1] (or a separate head-only partition
    at the end) owns the output layers.  Each sample gets exactly n_new new
    tokens, i.e. n_new + 1 rounds of Alg. 1; the token of the last round is not
    fed back.  Messages travel stage to stage in the order the starter emits
    them, which is what FIFO queues on a ring give.  Returns (tokens, logits,
    hidden): per sample the list of new token ids, the logits rows they came
    from, and the activations (last block's output) those were computed from.
    sampling: None for greedy tokens, else (temperature, top_k, seed) for draws from the top-k tempered pmf.
    """
    head = parts[-1] if head is None else head        # the paper's starter also owns the output layers: head=parts[0]
    blocks = [p for p in parts if p.hi > p.lo]
    toks = [[] for _ in prompts]
    logit_rows = [[] for _ in prompts]
    hidden_rows = [[] for _ in prompts]
    inbox = {}                                         # sample -> activation back at the starter
    for k, n, r, runs_head, runs_fwd, is_prefill in starter_schedule(len(prompts), n_new + 1):
        if runs_head:
            x = inbox.pop(n)
            if sampling is None:
                t, lg = head.sample_greedy(x)
            else:                                      # (temperature, top_k, seed): token j of sample n uses counter (n, j)
                t, lg = head.sample_topk(x, sampling[0], sampling[1], sampling[2], n, len(toks[n]))
            toks[n].append(t)
            logit_rows[n].append(lg)
            hidden_rows[n].append(x)
        if runs_fwd:
            msg = prompts[n] if is_prefill else np.array([toks[n][-1]], dtype=np.int32)
            for si, p in enumerate(blocks):           # Alg. 2 on every stage of the ring
                if trace is not None:
                    trace.append((k, n, si, "prefill" if is_prefill else "decode"))
                msg = p.prefill(n, msg) if is_prefill else p.decode_step(n, msg)
            inbox[n] = msg[-1] if is_prefill else msg
    return toks, logit_rows, hidden_rows


def pipeline_ticks(n_samples, n_nodes, n_rounds):
    """Tick-level picture of Fig. 2 for balanced stages.

    Every stage takes one tick per message and serves its FIFO in arrival
    order; a message processed in one tick is available to the next stage
    (the starter after the last one) in the following tick.  The starter's
    visit in round r >= 1 applies the output layers and, unless r is the last
    of the n_rounds rounds of Alg. 1, forwards the new token.  Returns
    busy[tick][stage] = sample id or None.
    """
    queues = [[] for _ in range(n_nodes)]
    queues[0] = [(n, 0) for n in range(n_samples)]    # (sample, round)
    busy = []
    done = 0
    while done < n_samples:
        row, moves = [None] * n_nodes, []
        for s in range(n_nodes):
            if queues[s]:
                n, r = queues[s].pop(0)
                row[s] = n
                moves.append((s, n, r))
        for s, n, r in moves:
            if s == 0 and r == n_rounds - 1:
                done += 1                              # last round: output layers only
            elif s + 1 < n_nodes:
                queues[s + 1].append((n, r))
            else:
                queues[0].append((n, r + 1))
        busy.append(row)
    return busy
