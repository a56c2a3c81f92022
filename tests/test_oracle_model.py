"""Pins for the oracle's block, partition and cache logic."""
import math
import os

import numpy as np
import pytest

from oracle import mdi_oracle as O
from paper_2505_18164_amd import synth as S

VARIANTS = {
    "llama_gqa": dict(),
    "llama_mha": dict(n_kv_head=4),
    "gpt2": dict(norm_kind=S.NORM_LAYERNORM, mlp_kind=S.MLP_GELU_TANH, pos_kind=S.POS_LEARNED, has_bias=1,
                 tie_embed=1, n_kv_head=4),
    "gelu_erf": dict(norm_kind=S.NORM_LAYERNORM, mlp_kind=S.MLP_GELU_ERF, pos_kind=S.POS_LEARNED, has_bias=1,
                     n_kv_head=4),
}


def model(name, n_layer=3, seed=11):
    cfg = S.tiny(n_layer=n_layer, **VARIANTS[name])
    w = S.make_weights(cfg, seed, exercise=True)
    # larger weights than the benchmark recipe so that every term matters
    for lw in w["layers"].values():
        for k in lw:
            if lw[k].ndim == 2:
                lw[k] = lw[k] * 8.0
    return cfg, w


# ------------------------------------------------------------ brute force block
def scalar_block(cfg, lw, x, pos0, past_k, past_v):
    """One decoder block with Python floats and explicit loops only.
    x: list of T rows; past_k/past_v: lists of [K][h] rows for positions < pos0."""
    d, H, K, h, F = cfg["d_model"], cfg["n_head"], cfg["n_kv_head"], cfg["head_dim"], cfg["d_ff"]
    f = lambda a: [[float(v) for v in row] for row in a] if getattr(a, "ndim", 1) == 2 else [float(v) for v in a]

    def norm(row, g, b):
        if cfg["norm_kind"] == S.NORM_LAYERNORM:
            mu = sum(row) / d
            var = sum((v - mu) ** 2 for v in row) / d
            return [(row[i] - mu) / math.sqrt(var + cfg["norm_eps"]) * g[i] + b[i] for i in range(d)]
        ms = sum(v * v for v in row) / d
        return [row[i] / math.sqrt(ms + cfg["norm_eps"]) * g[i] for i in range(d)]

    def lin(row, w, b):
        return [sum(w[o][i] * row[i] for i in range(len(row))) + (b[o] if b is not None else 0.0) for o in range(len(w))]

    def rope(vec, nh, p):
        out = list(vec)
        for j in range(nh):
            for i in range(h // 2):
                ang = p * cfg["rope_base"] ** (-2.0 * i / h)
                a, b = vec[j * h + i], vec[j * h + i + h // 2]
                out[j * h + i] = a * math.cos(ang) - b * math.sin(ang)
                out[j * h + i + h // 2] = a * math.sin(ang) + b * math.cos(ang)
        return out

    g = lambda k: f(lw[k]) if k in lw else None
    ks, vs = [list(r) for r in past_k], [list(r) for r in past_v]
    out = []
    for t, row in enumerate(x):
        p = pos0 + t
        a = norm(row, g("ln1_g"), g("ln1_b"))
        q, k, v = lin(a, g("wq"), g("bq")), lin(a, g("wk"), g("bk")), lin(a, g("wv"), g("bv"))
        if cfg["pos_kind"] == S.POS_ROPE:
            q, k = rope(q, H, p), rope(k, K, p)
        ks.append(k); vs.append(v)
        o = [0.0] * (H * h)
        for j in range(H):
            kv = j // (H // K)
            sc = [sum(q[j * h + e] * ks[u][kv * h + e] for e in range(h)) / math.sqrt(h) for u in range(p + 1)]
            m = max(sc); wts = [math.exp(s - m) for s in sc]; z = sum(wts)
            for e in range(h):
                o[j * h + e] = sum(wts[u] * vs[u][kv * h + e] for u in range(p + 1)) / z
        y = lin(o, g("wo"), g("bo"))
        row = [row[i] + y[i] for i in range(d)]
        m2 = norm(row, g("ln2_g"), g("ln2_b"))
        if cfg["mlp_kind"] == S.MLP_SWIGLU:
            gate, up = lin(m2, g("wg"), None), lin(m2, g("wu"), None)
            u = [gate[i] / (1 + math.exp(-gate[i])) * up[i] for i in range(F)]
            y = lin(u, g("wd"), None)
        else:
            pre = lin(m2, g("w1"), g("b1"))
            if cfg["mlp_kind"] == S.MLP_GELU_TANH:
                u = [0.5 * z_ * (1 + math.tanh(math.sqrt(2 / math.pi) * (z_ + 0.044715 * z_ ** 3))) for z_ in pre]
            else:
                u = [0.5 * z_ * (1 + math.erf(z_ / math.sqrt(2))) for z_ in pre]
            y = lin(u, g("w2"), g("b2"))
        out.append([row[i] + y[i] for i in range(d)])
    return out


@pytest.mark.parametrize("name", list(VARIANTS))
def test_block_vs_scalar_brute_force(name):
    cfg, w = model(name, n_layer=1)
    cfg = dict(cfg, d_model=32)
    rng = np.random.default_rng(3)
    x = rng.standard_normal((5, cfg["d_model"]))
    lw = {k: np.asarray(v, dtype=np.float64) for k, v in w["layers"][0].items()}
    cache = {"k": np.zeros((0, cfg["n_kv_head"], cfg["head_dim"])), "v": np.zeros((0, cfg["n_kv_head"], cfg["head_dim"]))}
    got = O.block_forward(cfg, lw, x, cache, 0)
    want = np.array(scalar_block(cfg, lw, x.tolist(), 0, [], []))
    np.testing.assert_allclose(got, want, rtol=1e-10, atol=1e-12)
    # and a second call at a later position with history (the decode form)
    x2 = rng.standard_normal((1, cfg["d_model"]))
    pk = cache["k"].reshape(5, -1).tolist(); pv = cache["v"].reshape(5, -1).tolist()
    got2 = O.block_forward(cfg, lw, x2, cache, 5)
    want2 = np.array(scalar_block(cfg, lw, x2.tolist(), 5, pk, pv))
    np.testing.assert_allclose(got2, want2, rtol=1e-10, atol=1e-12)
    assert cache["k"].shape[0] == 6


def test_linear_is_w_times_x():
    w = np.arange(6.0).reshape(2, 3)                     # [out, in]
    np.testing.assert_array_equal(O._lin(np.array([[1.0, 10.0, 100.0]]), w, np.array([0.5, -0.5])), [[210.5, 543.5 - 1.0]])


# ------------------------------------------------------------ structure pins
@pytest.mark.parametrize("name", ["llama_gqa", "gpt2"])
def test_identity_when_output_matrices_vanish(name):
    cfg, w = model(name, n_layer=2)
    for lw in w["layers"].values():
        for k in ("wo", "wd", "w2", "bo", "b2"):
            if k in lw:
                lw[k] = np.zeros_like(lw[k])
    x = np.random.default_rng(0).standard_normal((4, cfg["d_model"]))
    p = O.Partition(cfg, w, 0, 2)
    np.testing.assert_array_equal(p.prefill(0, x), x)


def test_swiglu_gate_zero_gives_attention_only():
    cfg, w = model("llama_gqa", n_layer=1)
    w2 = {"layers": {0: dict(w["layers"][0])}}
    w2["layers"][0]["wg"] = np.zeros_like(w["layers"][0]["wg"])
    w3 = {"layers": {0: dict(w["layers"][0])}}
    w3["layers"][0]["wd"] = np.zeros_like(w["layers"][0]["wd"])
    x = np.random.default_rng(1).standard_normal((4, cfg["d_model"]))
    a = O.Partition(cfg, w2, 0, 1).prefill(0, x)
    b = O.Partition(cfg, w3, 0, 1).prefill(0, x)
    np.testing.assert_allclose(a, b, rtol=1e-14)
    assert np.abs(a - x).max() > 1e-3


@pytest.mark.parametrize("name", list(VARIANTS))
def test_cached_decode_equals_full_prefix_recompute(name):
    """Sec. III-D: caching only avoids recomputing K and V; the result is that
    of forwarding the whole context."""
    cfg, w = model(name)
    ids = S.make_prompts(cfg, 5, 1, 12)[0]
    p = O.Partition(cfg, w, 0, cfg["n_layer"], has_embed=True, has_head=True)
    rows = [p.prefill(0, ids[:4])[-1]]
    for t in range(4, 12):
        rows.append(p.decode_step(0, ids[t]))
    full = O.forward_no_cache(cfg, w, ids, 0, cfg["n_layer"], True)
    np.testing.assert_allclose(np.array(rows), full[3:], rtol=1e-11, atol=1e-13)
    assert p.seq_len(0) == 12


@pytest.mark.parametrize("name", ["llama_gqa", "gpt2"])
def test_composed_partitions_equal_unsplit_bit_for_bit(name):
    cfg, w = model(name, n_layer=4)
    L = cfg["n_layer"]
    ids = S.make_prompts(cfg, 9, 1, 7)[0]
    whole = O.Partition(cfg, w, 0, L, has_embed=True, has_head=True)
    ref_rows = whole.prefill(0, ids)
    ref_dec = whole.decode_step(0, 5)
    ref_logits = whole.logits(ref_dec)
    for k in range(1, L):
        a = O.Partition(cfg, w, 0, k, has_embed=True)
        b = O.Partition(cfg, w, k, L, has_head=True)
        rows = b.prefill(0, a.prefill(0, ids))
        np.testing.assert_array_equal(rows, ref_rows)
        dec = b.decode_step(0, a.decode_step(0, 5))
        np.testing.assert_array_equal(dec, ref_dec)
        np.testing.assert_array_equal(b.logits(dec), ref_logits)
    # the paper's starter layout: output portion without transformer blocks (Sec. III-E)
    head_only = O.Partition(cfg, w, L, L, has_head=True)
    np.testing.assert_array_equal(head_only.logits(ref_dec), ref_logits)
    assert head_only.layers == []


def test_interleaved_samples_equal_each_sample_alone():
    """Sec. III-D/III-E: one cache per sample, selected by the sample id."""
    cfg, w = model("llama_gqa")
    prompts = S.make_prompts(cfg, 21, 3, 6)
    L = cfg["n_layer"]
    solo = []
    for s in range(3):
        p = O.Partition(cfg, w, 0, L, has_embed=True)
        r = [p.prefill(s, prompts[s])[-1]] + [p.decode_step(s, (7 * s + t) % cfg["vocab"]) for t in range(5)]
        solo.append(np.array(r))
    p = O.Partition(cfg, w, 0, L, has_embed=True)
    inter = [[p.prefill(s, prompts[s])[-1]] for s in range(3)]
    for t in range(5):
        for s in (2, 0, 1):
            inter[s].append(p.decode_step(s, (7 * s + t) % cfg["vocab"]))
    for s in range(3):
        np.testing.assert_array_equal(np.array(inter[s]), solo[s])


def test_state_errors():
    cfg, w = model("llama_gqa", n_layer=1)
    p = O.Partition(dict(cfg, max_ctx=4), w, 0, 1)
    x = np.zeros((3, cfg["d_model"]))
    with pytest.raises(RuntimeError):
        p.decode_step(0, x[0])
    p.prefill(0, x)
    with pytest.raises(RuntimeError):
        p.prefill(0, x)
    p.decode_step(0, x[0])
    with pytest.raises(ValueError):
        p.decode_step(0, x[0])


def test_float32_variant_is_close_to_float64():
    cfg, w = model("gpt2")
    ids = S.make_prompts(cfg, 2, 1, 10)[0]
    a = O.forward_no_cache(cfg, w, ids, 0, cfg["n_layer"], True, dtype=np.float64)
    b = O.forward_no_cache(cfg, w, ids, 0, cfg["n_layer"], True, dtype=np.float32)
    assert b.dtype == np.float32
    rel = np.linalg.norm(a - b) / np.linalg.norm(a)
    assert rel < 1e-5


def test_learned_positions_are_added_at_embed():
    cfg, w = model("gpt2", n_layer=1)
    x = O.embed(cfg, {k: np.asarray(v, dtype=np.float64) for k, v in w.items() if k != "layers"}, [3, 3], 5)
    np.testing.assert_array_equal(x[0], w["wte"][3].astype(np.float64) + w["wpe"][5])
    np.testing.assert_array_equal(x[1], w["wte"][3].astype(np.float64) + w["wpe"][6])
    assert w["lm_head"] is w["wte"]                    # tied output projection


def test_parameter_accounting_matches_paper_sizes():
    """Sec. IV-A/IV-C print model sizes; they pin the per-layer size formula
    used for the bandwidth roofline (loosely: the text rounds)."""
    rows = [l.split() for l in open(os.path.join(os.path.dirname(__file__), "golden", "paper_sizes.txt")) if not l.startswith("#")]
    for name, blocks, d, heads, vocab, stated, gb in [(r[0], int(r[1]), int(r[2]), int(r[3]), int(r[4]), float(r[5]), float(r[6])) for r in rows]:
        cfg = getattr(S, name)()
        assert (cfg["n_layer"], cfg["d_model"], cfg["n_head"], cfg["vocab"]) == (blocks, d, heads, vocab)
        per_layer = sum(a * b for a, b in S.layer_tensor_shapes(cfg).values()) + 2 * d
        total = blocks * per_layer + 2 * vocab * d + d
        assert abs(total - stated) / stated < 0.03
        assert abs(total * 4 / 1e9 - gb) / gb < 0.12


@pytest.mark.parametrize("variant", ["llama", "gpt2"])
def test_first_visit_in_pieces_equals_the_whole_first_visit(variant):
    """Causal attention over the cache plus the new rows: forwarding a prompt in pieces (of any sizes, one of them a
    single row, which is exactly a later visit) gives the rows of one first visit of the whole prompt, and the later
    visits that follow do not see a difference."""
    kw = dict(norm_kind=S.NORM_LAYERNORM, mlp_kind=S.MLP_GELU_TANH, pos_kind=S.POS_LEARNED, has_bias=1, tie_embed=1, n_kv_head=4) if variant == "gpt2" else {}
    cfg = S.tiny(n_layer=3, max_ctx=40, **kw)
    w = S.make_weights(cfg, 19, exercise=True)
    ids = S.make_prompts(cfg, 19, 1, 23)[0]
    whole, pieces = O.Partition(cfg, w, 0, 3, has_embed=True), O.Partition(cfg, w, 0, 3, has_embed=True)
    want = whole.prefill(0, ids)
    at, rows = 0, []
    for n in (7, 1, 11, 4):
        rows.append(pieces.prefill_chunk(0, ids[at:at + n]))
        at += n
    got = np.concatenate(rows)
    assert got.shape == want.shape and np.abs(got - want).max() <= 1e-11 * np.abs(want).max()
    assert pieces.seq_len(0) == whole.seq_len(0) == 23
    for t in (3, 9):
        a, b = whole.decode_step(0, t), pieces.decode_step(0, t)
        assert np.abs(a - b).max() <= 1e-11 * np.abs(a).max()
    # a piece of one row IS a later visit: same code path, same bits
    one, other = O.Partition(cfg, w, 0, 3, has_embed=True), O.Partition(cfg, w, 0, 3, has_embed=True)
    one.prefill(0, ids[:5]); other.prefill(0, ids[:5])
    assert np.array_equal(one.prefill_chunk(0, ids[5:6])[0], other.decode_step(0, int(ids[5])))


# ------------------------------------------------------------ output layers
@pytest.mark.parametrize("tie", [0, 1], ids=["untied", "tied"])
@pytest.mark.parametrize("norm_kind", [S.NORM_LAYERNORM, S.NORM_RMSNORM], ids=["layernorm", "rmsnorm"])
def test_output_layers_against_scalar_loops(norm_kind, tie):
    """The starter's output portion (Sec. III-B "final layers", Alg. 1 "process output layers"): final norm of the
    last block's output, THEN the vocabulary projection, with the matrix taken row per token ([V, d]; the
    embedding matrix itself when tied).  Written out with Python floats; gains and biases are non-trivial and the
    matrix is not square, so a missing norm, the block norm's gain in place of the final one, a dropped bias or a
    transposed matrix all change the numbers."""
    cfg = S.tiny(n_layer=1, norm_kind=norm_kind, tie_embed=tie, d_model=8, n_head=2, n_kv_head=1, head_dim=4, d_ff=16,
                 vocab=13, pos_kind=S.POS_LEARNED if norm_kind == S.NORM_LAYERNORM else S.POS_ROPE)
    w = S.make_weights(cfg, 41, exercise=True)
    w["wte"] = w["wte"] * 20.0
    if tie:
        w["lm_head"] = w["wte"]
    else:
        w["lm_head"] = w["lm_head"] * 20.0
    d, V, eps = cfg["d_model"], cfg["vocab"], cfg["norm_eps"]
    rng = np.random.default_rng(3)
    xs = rng.normal(size=(3, d)) * 2.0 + 0.7                 # non-zero mean: LayerNorm's centring matters
    g = [float(v) for v in w["lnf_g"]]
    b = [float(v) for v in w["lnf_b"]] if norm_kind == S.NORM_LAYERNORM else None
    M = [[float(v) for v in row] for row in (w["wte"] if tie else w["lm_head"])]
    want = []
    for x in xs:
        x = [float(v) for v in x]
        if norm_kind == S.NORM_LAYERNORM:
            mu = sum(x) / d
            var = sum((v - mu) ** 2 for v in x) / d
            xn = [(x[i] - mu) / math.sqrt(var + eps) * g[i] + b[i] for i in range(d)]
        else:
            ms = sum(v * v for v in x) / d
            xn = [x[i] / math.sqrt(ms + eps) * g[i] for i in range(d)]
        want.append([sum(M[t][i] * xn[i] for i in range(d)) for t in range(V)])
    want = np.array(want)
    got = O.head_logits(cfg, O._cast_tree({k: v for k, v in w.items() if k != "layers"}, np.float64), xs)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)
    # the same through a partition, row by row, and the token it yields
    p = O.Partition(cfg, w, 1, 1, has_head=True)
    for x, row in zip(xs, want):
        np.testing.assert_allclose(p.logits(x), row, rtol=1e-12, atol=1e-12)
        assert p.sample_greedy(x)[0] == max(range(V), key=lambda t: (row[t], -t))
    # what the plausible mistakes would give is far from it (the pin can tell them apart)
    no_norm = np.array([[sum(M[t][i] * float(x[i]) for i in range(d)) for t in range(V)] for x in xs])
    assert np.abs(no_norm - want).max() > 1e-2
    if norm_kind == S.NORM_LAYERNORM:
        no_bias = want - np.array([[sum(M[t][i] * b[i] for i in range(d)) for t in range(V)]] * 3)
        assert np.abs(no_bias - want).max() > 1e-3


def test_output_layers_use_the_final_norm_not_a_block_norm():
    """A wrong gain vector (a block's pre-MLP gain instead of the final one) must change the logits."""
    cfg = S.tiny(n_layer=1, d_model=8, n_head=2, n_kv_head=1, head_dim=4, d_ff=16, vocab=13)
    w = S.make_weights(cfg, 43, exercise=True)
    x = np.linspace(-1.0, 2.0, cfg["d_model"])
    p = O.Partition(cfg, w, 1, 1, has_head=True)
    ms = float((x * x).mean())
    xn = x / math.sqrt(ms + cfg["norm_eps"]) * w["lnf_g"].astype(np.float64)
    np.testing.assert_allclose(p.logits(x), w["lm_head"].astype(np.float64) @ xn, rtol=1e-12, atol=1e-14)
    assert not np.allclose(w["lnf_g"], w["layers"][0]["ln2_g"])
