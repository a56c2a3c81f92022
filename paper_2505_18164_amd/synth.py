"""Seeded synthetic inputs shared by the CPU oracle tests and the HIP path.

This module holds data recipes only: model shape presets, random weights,
prompts and activations, and the fp32 <-> bf16 storage conversion.  It contains
none of the transformer arithmetic and imports neither the oracle nor the HIP
binding, so both sides can be fed the very same buffers.

The paper evaluates on a Tiny-Shakespeare-trained 304M "NanoLlama" and on
TinyLlama-1.1B-Chat (Sec. IV-A); neither checkpoint is available, and neither
throughput nor parity depends on trained values, so every tensor here is
random-init of the same shape.
"""
from __future__ import annotations

import copy
from concurrent.futures import ThreadPoolExecutor

import numpy as np

# enum values mirror include/mdi.h (plain integers; the header is the authority)
NORM_LAYERNORM, NORM_RMSNORM = 0, 1
MLP_GELU_TANH, MLP_GELU_ERF, MLP_SWIGLU = 0, 1, 2
POS_LEARNED, POS_ROPE = 0, 1
DT_F32, DT_BF16 = 0, 1

BASE_SEED = 20250518
WEIGHT_STD = 0.02


def _cfg(**kw):
    c = dict(n_layer=0, d_model=0, n_head=0, n_kv_head=0, head_dim=0, d_ff=0, vocab=0,
             max_ctx=0, norm_kind=NORM_RMSNORM, norm_eps=1e-5, mlp_kind=MLP_SWIGLU,
             pos_kind=POS_ROPE, rope_base=10000.0, has_bias=0, tie_embed=0, dtype=DT_BF16)
    c.update(kw)
    assert c["head_dim"] * c["n_head"] > 0
    return c


def gpt2_small(n_layer=12, dtype=DT_BF16, max_ctx=1024):
    return _cfg(n_layer=n_layer, d_model=768, n_head=12, n_kv_head=12, head_dim=64, d_ff=3072,
                vocab=50257, max_ctx=max_ctx, norm_kind=NORM_LAYERNORM, mlp_kind=MLP_GELU_TANH,
                pos_kind=POS_LEARNED, has_bias=1, tie_embed=1, dtype=dtype)


def tinyllama(dtype=DT_BF16, max_ctx=2048):
    return _cfg(n_layer=22, d_model=2048, n_head=32, n_kv_head=4, head_dim=64, d_ff=5632,
                vocab=32000, max_ctx=max_ctx, rope_base=10000.0, dtype=dtype)


def llama2_7b(dtype=DT_BF16, max_ctx=4096):
    return _cfg(n_layer=32, d_model=4096, n_head=32, n_kv_head=32, head_dim=128, d_ff=11008,
                vocab=32000, max_ctx=max_ctx, rope_base=10000.0, dtype=dtype)


def llama3_8b(dtype=DT_BF16, max_ctx=8192):
    return _cfg(n_layer=32, d_model=4096, n_head=32, n_kv_head=8, head_dim=128, d_ff=14336,
                vocab=128256, max_ctx=max_ctx, rope_base=500000.0, dtype=dtype)


def nanollama(dtype=DT_F32, max_ctx=2048):
    """Shape of the paper's 304M toy model (Sec. IV-A); the MLP width is not
    printed there, 5120 makes the parameter count come out at 304M untied."""
    return _cfg(n_layer=12, d_model=1024, n_head=16, n_kv_head=16, head_dim=64, d_ff=5120,
                vocab=32000, max_ctx=max_ctx, dtype=dtype)


def tiny(norm_kind=NORM_RMSNORM, mlp_kind=MLP_SWIGLU, pos_kind=POS_ROPE, has_bias=0, tie_embed=0,
         n_layer=2, d_model=32, n_head=4, n_kv_head=2, head_dim=8, d_ff=48, vocab=61, max_ctx=64,
         dtype=DT_F32, rope_base=10000.0):
    """A few-hundred-parameter shape for brute-force checks."""
    return _cfg(n_layer=n_layer, d_model=d_model, n_head=n_head, n_kv_head=n_kv_head,
                head_dim=head_dim, d_ff=d_ff, vocab=vocab, max_ctx=max_ctx, norm_kind=norm_kind,
                mlp_kind=mlp_kind, pos_kind=pos_kind, has_bias=has_bias, tie_embed=tie_embed,
                dtype=dtype, rope_base=rope_base)


# The five benchmark workloads (index = position in the configs list + 1).
WORKLOADS = {
    1: dict(name="C1 gpt2-small-shaped 4 layers fp32", cfg=lambda: gpt2_small(4, DT_F32, 64),
            parts=[(0, 4)], n_seqs=2, prompt=16, n_new=32),
    2: dict(name="C2 gpt2-small-shaped 12 layers as 3x4 bf16", cfg=lambda: gpt2_small(12, DT_BF16, 384),
            parts=[(0, 4), (4, 8), (8, 12)], n_seqs=3, prompt=128, n_new=256),
    3: dict(name="C3 tinyllama-shaped layers 0-10 bf16", cfg=lambda: tinyllama(DT_BF16, 2048),
            parts=[(0, 11)], n_seqs=4, prompt=512, n_new=1536),
    4: dict(name="C4 llama2-7b-shaped layers 8-15 bf16", cfg=lambda: llama2_7b(DT_BF16, 4096),
            parts=[(8, 16)], n_seqs=8, prompt=1024, n_new=3072),
    5: dict(name="C5 llama3-8b-shaped 32 layers as 4x8 bf16", cfg=lambda: llama3_8b(DT_BF16, 8192),
            parts=[(0, 8), (8, 16), (16, 24), (24, 32)], n_seqs=16, prompt=2048, n_new=6144),
}


def workload_seed(index):
    return BASE_SEED + index


# ----------------------------------------------------------------------------
# bf16 storage: round-to-nearest-even of fp32, kept as uint16 bit patterns.
def f32_to_bf16_bits(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b):
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(a):
    """fp32 array whose values are exactly representable in bf16."""
    return bf16_bits_to_f32(f32_to_bf16_bits(a))


def storage_round(a, dtype):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return round_to_bf16(a) if dtype == DT_BF16 else a


# ----------------------------------------------------------------------------
# One generator per tensor, keyed by (seed, layer, slot), so that a partition's
# weights do not depend on which other layers were drawn.
_SLOTS = dict(wte=0, wpe=1, lnf_g=2, lnf_b=3, lm_head=4,
              ln1_g=10, ln1_b=11, wq=12, wk=13, wv=14, bq=15, bk=16, bv=17, wo=18, bo=19,
              ln2_g=20, ln2_b=21, w1=22, b1=23, w2=24, b2=25, wg=26, wu=27, wd=28)
_GLOBAL_LAYER = 1_000_000


def _rng(seed, layer, slot):
    return np.random.Generator(np.random.PCG64([int(seed), int(layer), int(slot)]))


def _normal(seed, layer, name, shape, std):
    g = _rng(seed, layer, _SLOTS[name])
    out = g.standard_normal(size=shape, dtype=np.float32)
    out *= np.float32(std)
    return out


def layer_tensor_shapes(cfg):
    d, H, K, h, F = cfg["d_model"], cfg["n_head"], cfg["n_kv_head"], cfg["head_dim"], cfg["d_ff"]
    s = dict(wq=(H * h, d), wk=(K * h, d), wv=(K * h, d), wo=(d, H * h))
    if cfg["mlp_kind"] == MLP_SWIGLU:
        s.update(wg=(F, d), wu=(F, d), wd=(d, F))
    else:
        s.update(w1=(F, d), w2=(d, F))
    return s


def make_weights(cfg, seed, layer_lo=0, layer_hi=None, embed=True, head=True, exercise=False):
    """Random-init weights as fp32 arrays already rounded to the storage dtype.

    Matrices use the `[out_features, in_features]` row-major layout.  Benchmark
    recipe (exercise=False): matrices and embeddings i.i.d. N(0, 0.02^2), norm
    gains 1, every bias 0.  exercise=True draws non-trivial gains and biases so
    that those code paths change the result.  Returns
    {"layers": {global_layer_index: {...}}, "wte":..., "wpe":..., "lnf_g":..., "lnf_b":..., "lm_head":...}.
    """
    layer_hi = cfg["n_layer"] if layer_hi is None else layer_hi
    d, V = cfg["d_model"], cfg["vocab"]
    dt = cfg["dtype"]
    ln = cfg["norm_kind"] == NORM_LAYERNORM
    jobs = []

    def mat(dst, key, layer, name, shape):
        jobs.append((dst, key, layer, name, shape, WEIGHT_STD, 0.0))

    def vec(dst, key, layer, name, n, centre):
        if exercise:
            jobs.append((dst, key, layer, name, (n,), 0.1, centre))
        else:
            dst[key] = np.full((n,), centre, dtype=np.float32)

    w = {"layers": {}}
    for L in range(layer_lo, layer_hi):
        lw = {}
        w["layers"][L] = lw
        for name, shape in layer_tensor_shapes(cfg).items():
            mat(lw, name, L, name, shape)
        vec(lw, "ln1_g", L, "ln1_g", d, 1.0)
        vec(lw, "ln2_g", L, "ln2_g", d, 1.0)
        if ln:
            vec(lw, "ln1_b", L, "ln1_b", d, 0.0)
            vec(lw, "ln2_b", L, "ln2_b", d, 0.0)
        if cfg["has_bias"]:
            shapes = layer_tensor_shapes(cfg)
            for bname, wname in (("bq", "wq"), ("bk", "wk"), ("bv", "wv"), ("bo", "wo")):
                vec(lw, bname, L, bname, shapes[wname][0], 0.0)
            if cfg["mlp_kind"] == MLP_SWIGLU:
                pass  # Llama-family MLPs carry no bias
            else:
                vec(lw, "b1", L, "b1", shapes["w1"][0], 0.0)
                vec(lw, "b2", L, "b2", shapes["w2"][0], 0.0)
    if embed or (head and cfg["tie_embed"]):
        mat(w, "wte", _GLOBAL_LAYER, "wte", (V, d))
    if embed and cfg["pos_kind"] == POS_LEARNED:
        mat(w, "wpe", _GLOBAL_LAYER, "wpe", (cfg["max_ctx"], d))
    if head:
        vec(w, "lnf_g", _GLOBAL_LAYER, "lnf_g", d, 1.0)
        if ln:
            vec(w, "lnf_b", _GLOBAL_LAYER, "lnf_b", d, 0.0)
        if not cfg["tie_embed"]:
            mat(w, "lm_head", _GLOBAL_LAYER, "lm_head", (V, d))

    def run(job):
        dst, key, layer, name, shape, std, centre = job
        a = _normal(seed, layer, name, shape, std)
        if centre:
            a += np.float32(centre)
        # norm parameters and biases stay fp32 on both sides; matrices take the storage dtype
        dst[key] = storage_round(a, dt) if len(shape) == 2 else a

    with ThreadPoolExecutor(max_workers=8) as ex:
        list(ex.map(run, jobs))
    if head and cfg["tie_embed"]:
        w["lm_head"] = w["wte"]
    return w


def zero_like_weights(w):
    return copy.deepcopy(w)


def make_prompts(cfg, seed, n_seqs, prompt_len):
    """Token ids i.i.d. uniform on [0, vocab), one stream per sequence."""
    out = []
    for s in range(n_seqs):
        g = _rng(seed + 1, s, 0)
        out.append(g.integers(0, cfg["vocab"], size=prompt_len, dtype=np.int64).astype(np.int32))
    return out


def make_activations(cfg, seed, seq, T, step=0):
    """N(0,1) activations [T, d] for a partition that does not own the embedding,
    rounded to the storage dtype (what the previous stage would hand over)."""
    g = _rng(seed + 2, seq, step)
    a = g.standard_normal(size=(T, cfg["d_model"]), dtype=np.float32)
    return storage_round(a, cfg["dtype"])
