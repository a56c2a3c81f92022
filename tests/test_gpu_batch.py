"""GPU parity of mdi_decode_batch: several queued messages taken through the local layers with ONE pass over the
weights (matrix-core products over all messages, attention per sample), against the float64 oracle's one-message-
at-a-time decode (Sec. III-D), message by message, at the bf16 bar (rel-L2 <= 2e-2 on hidden states)."""
import numpy as np
import pytest
import torch

from oracle import mdi_oracle as O
from paper_2505_18164_amd import mdi, synth as S
from gpu_util import check, dev_acts, dev_ids, host, pair, rel_l2, scale_matrices, tol

pytestmark = pytest.mark.gpu

# shapes whose widths are multiples of 32 (what one pass over the weights needs)
SHAPES = {
    "gqa_h16": dict(d_model=64, n_head=4, n_kv_head=2, head_dim=16, d_ff=96),
    "mha_h16": dict(d_model=64, n_head=4, n_kv_head=4, head_dim=16, d_ff=96),
    "gqa8_h8": dict(d_model=64, n_head=8, n_kv_head=1, head_dim=8, d_ff=160),
    "h64": dict(d_model=128, n_head=2, n_kv_head=1, head_dim=64, d_ff=288),
    "gelu_rms_bias": dict(d_model=64, n_head=4, n_kv_head=4, head_dim=16, d_ff=96, mlp_kind=S.MLP_GELU_TANH, has_bias=1),
    "gelu_erf_learned_pos": dict(d_model=96, n_head=6, n_kv_head=2, head_dim=16, d_ff=128, mlp_kind=S.MLP_GELU_ERF,
                                 pos_kind=S.POS_LEARNED),
    "swiglu_attn_bias": dict(d_model=64, n_head=4, n_kv_head=2, head_dim=16, d_ff=96, has_bias=1),
    "wide": dict(d_model=256, n_head=4, n_kv_head=2, head_dim=64, d_ff=704),
    # 9 column steps of 32 in the down projection: some wavefronts of a workgroup get none
    "idle_wavefronts": dict(d_model=256, n_head=4, n_kv_head=2, head_dim=64, d_ff=288),
    # the GPT-2 family: LayerNorm (its mean and bias enter the products through precomputed vectors), GELU, biases,
    # learned positions
    "gpt2_like": dict(d_model=96, n_head=6, n_kv_head=6, head_dim=16, d_ff=192, norm_kind=S.NORM_LAYERNORM,
                      mlp_kind=S.MLP_GELU_TANH, pos_kind=S.POS_LEARNED, has_bias=1),
    "layernorm_swiglu": dict(d_model=64, n_head=4, n_kv_head=2, head_dim=16, d_ff=96, norm_kind=S.NORM_LAYERNORM),
    "layernorm_rope_gelu_erf": dict(d_model=64, n_head=4, n_kv_head=2, head_dim=16, d_ff=96, norm_kind=S.NORM_LAYERNORM,
                                    mlp_kind=S.MLP_GELU_ERF),
}


@pytest.mark.parametrize("n_msg", [2, 5, 16])
@pytest.mark.parametrize("name", list(SHAPES))
def test_batched_pass_against_the_oracle(name, n_msg):
    cfg = S.tiny(n_layer=3, dtype=S.DT_BF16, max_ctx=64, vocab=211, **SHAPES[name])
    w = scale_matrices(S.make_weights(cfg, 17, exercise=True), 2.0)   # every sub-layer moves the residual stream, bf16 noise stays small
    o, g = pair(cfg, w, 0, 3, embed=True, head=False, max_seqs=n_msg, kv_page_tokens=8)
    assert g.info(4) == 16, "this shape should take the batched pass"
    prompts = S.make_prompts(cfg, 17, n_msg, 23)
    for s in range(n_msg):
        prompts[s] = prompts[s][:3 + (5 * s) % 20]                 # ragged contexts, some shorter than a page
        check(g.prefill(s, dev_ids(prompts[s])), o.prefill(s, prompts[s]), cfg, ("prefill", s))
    rng = np.random.default_rng(3)
    worst = 0.0
    for step in range(12):                                        # crosses page boundaries of 8 tokens
        order = [int(s) for s in rng.permutation(n_msg)]
        toks = [int(rng.integers(0, cfg["vocab"])) for _ in order]
        outs = g.decode_batch(order, [dev_ids([t]) for t in toks])
        for s, t, got in zip(order, toks, outs):
            worst = max(worst, check(got, o.decode_step(s, t), cfg, ("batched decode", step, s)))
    for s in range(n_msg):
        assert g.seq_len(s) == len(prompts[s]) + 12
    g.sync()
    print(f"{name} x{n_msg}: worst rel-L2 {worst:.2e}", flush=True)


@pytest.mark.parametrize("heads", [2, 4])
@pytest.mark.parametrize("name", ["gqa_h16", "gqa8_h8", "h64", "idle_wavefronts"])
def test_batched_pass_with_pairs_of_query_heads_and_context_splits(name, heads, monkeypatch):
    """Long contexts (or more attention work items than workgroups) let two query heads share a pass over their kv
    head's cache, and contexts of more than 128 positions are split among workgroups and folded; both are reached
    here on small shapes by lowering the switch-over length and by a context of a few hundred positions."""
    shape = dict(SHAPES[name])
    if heads == 4:                                                 # four heads per work item need groups of a multiple of four
        if name != "gqa8_h8":
            shape.update(n_head=4 * shape["n_kv_head"], d_model=4 * shape["n_kv_head"] * shape["head_dim"])
        monkeypatch.setenv("MDI_BATCH_GROUP", "4")
    monkeypatch.setenv("MDI_GROUP_CTX", "12")
    cfg = S.tiny(n_layer=2, dtype=S.DT_BF16, max_ctx=512, vocab=211, **shape)
    w = scale_matrices(S.make_weights(cfg, 29, exercise=True), 2.0)
    o, g = pair(cfg, w, 0, 2, embed=True, max_seqs=3, kv_page_tokens=16)
    lens = (300, 7, 140)
    for s, T in enumerate(lens):
        ids = S.make_prompts(cfg, 29 + s, 1, T)[0]
        check(g.prefill(s, dev_ids(ids)), o.prefill(s, ids), cfg, ("prefill", s))
    rng = np.random.default_rng(4)
    for step in range(8):
        toks = [int(rng.integers(0, cfg["vocab"])) for _ in range(3)]
        outs = g.decode_batch([2, 0, 1], [dev_ids([toks[s]]) for s in (2, 0, 1)])
        for s, got in zip((2, 0, 1), outs):
            check(got, o.decode_step(s, toks[s]), cfg, ("batched decode", step, s))
    g.sync()


def test_batched_pass_on_a_mid_partition_and_more_messages_than_one_pass():
    """Activations in and out (a secondary node, Alg. 2), 19 messages = a pass of 16 and one of 3, then a lone
    message (forwarded as by mdi_decode_step); a second partition fed the same calls reproduces the bits."""
    cfg = S.tiny(n_layer=4, dtype=S.DT_BF16, max_ctx=48, d_model=64, n_head=4, n_kv_head=2, head_dim=16, d_ff=96)
    w = scale_matrices(S.make_weights(cfg, 23, exercise=True), 3.0)
    n = 19
    o, g = pair(cfg, w, 1, 3, max_seqs=n, kv_page_tokens=16)
    g2 = mdi.Partition(cfg, w, 1, 3, max_seqs=n, kv_page_tokens=16)
    for s in range(n):
        a = S.make_activations(cfg, 23, s, 2 + s % 7)
        check(g.prefill(s, dev_acts(a, cfg)), o.prefill(s, a), cfg, ("prefill", s))
        g2.prefill(s, dev_acts(a, cfg))
    for step in range(5):
        order = list(range(n)) if step < 4 else [7]
        xs = [S.make_activations(cfg, 23, s, 1, step=step + 1)[0] for s in order]
        outs = g.decode_batch(order, [dev_acts(x, cfg) for x in xs])
        outs2 = g2.decode_batch(order, [dev_acts(x, cfg) for x in xs])
        for s, x, got, got2 in zip(order, xs, outs, outs2):
            check(got, o.decode_step(s, x), cfg, ("batched decode", step, s))
            assert torch.equal(got, got2), (step, s)
    g.sync()
    g2.sync()


def test_shapes_that_cannot_share_a_pass_fall_back_to_one_pass_per_message():
    for over in (dict(dtype=S.DT_F32), dict(d_ff=48), dict(d_model=48, n_head=3, n_kv_head=3)):
        cfg = S.tiny(n_layer=2, max_ctx=32, **dict(dict(dtype=S.DT_BF16, d_model=64, n_head=4, n_kv_head=2, head_dim=16, d_ff=96), **over))
        w = scale_matrices(S.make_weights(cfg, 5, exercise=True), 3.0)
        o, g = pair(cfg, w, 0, 2, embed=True, max_seqs=3, kv_page_tokens=8)
        assert g.info(4) == 0
        prompts = S.make_prompts(cfg, 5, 3, 6)
        for s in range(3):
            g.prefill(s, dev_ids(prompts[s]))
            o.prefill(s, prompts[s])
        outs = g.decode_batch([2, 0, 1], [dev_ids([4]), dev_ids([9]), dev_ids([1])])
        for s, t, got in zip((2, 0, 1), (4, 9, 1), outs):
            check(got, o.decode_step(s, t), cfg, ("fallback", s))
        g.sync()


def test_batched_pass_error_paths():
    cfg = S.tiny(n_layer=1, dtype=S.DT_BF16, max_ctx=16, d_model=64, n_head=4, n_kv_head=2, head_dim=16, d_ff=96)
    w = S.make_weights(cfg, 3)
    g = mdi.Partition(cfg, w, 0, 1, has_embed=True, max_seqs=3, kv_page_tokens=8, kv_pages=3)
    ids = dev_ids(np.arange(8))
    g.prefill(0, ids)
    g.prefill(1, ids)
    t = dev_ids([1])
    for seqs, status in (([0, 0], mdi.MDI_ERR_ARG), ([0, 2], mdi.MDI_ERR_STATE), ([0, 7], mdi.MDI_ERR_ARG)):
        with pytest.raises(mdi.MdiError) as e:
            g.decode_batch(seqs, [t, t])
        assert e.value.status == status
        assert g.seq_len(0) == 8 and g.seq_len(1) == 8          # a refused call advances no sample
    with pytest.raises(mdi.MdiError) as e:                       # both need a new page, one is left
        g.decode_batch([0, 1], [t, t])
    assert e.value.status == mdi.MDI_ERR_NOMEM and g.seq_len(0) == 8
    g.sync()


def test_token_id_out_of_range_in_a_batched_pass_is_reported():
    cfg = S.tiny(n_layer=2, dtype=S.DT_BF16, max_ctx=32, d_model=64, n_head=4, n_kv_head=2, head_dim=16, d_ff=96)
    w = S.make_weights(cfg, 5)
    g = mdi.Partition(cfg, w, 0, 2, has_embed=True, max_seqs=2)
    good = dev_ids(np.arange(4))
    g.prefill(0, good)
    g.prefill(1, good)
    g.sync()
    g.decode_batch([0, 1], [dev_ids([3]), dev_ids([cfg["vocab"]])])
    with pytest.raises(mdi.MdiError) as e:
        g.sync()
    assert e.value.status == mdi.MDI_ERR_ARG


def test_driver_with_shared_passes_on_a_three_node_ring():
    """Alg. 1 / Alg. 2 through the recurrent-pipeline driver with every stage taking the waiting messages of all
    samples through ONE pass over its weights and the starter drawing all their tokens with one pass over the
    vocabulary matrix.  The oracle follows the GPU's tokens sample by sample (its own one-message-at-a-time
    arithmetic, Sec. III-D), so every step is comparable at the bf16 bar whatever a near-tie decided."""
    from paper_2505_18164_amd.pipeline import RecurrentPipeline
    cfg = S.tiny(n_layer=6, dtype=S.DT_BF16, max_ctx=64, vocab=1003, **SHAPES["wide"])
    w = scale_matrices(S.make_weights(cfg, 41, exercise=True), 2.0)
    n_seqs, n_new = 5, 7
    prompts = [p[:2 + 3 * s] for s, p in enumerate(S.make_prompts(cfg, 41, n_seqs, 16))]
    bounds = [0, 2, 4, 6]
    parts = [mdi.Partition(cfg, w, bounds[i], bounds[i + 1], has_embed=i == 0, has_head=i == 0, max_seqs=n_seqs,
                           kv_page_tokens=8, stream=torch.cuda.Stream()) for i in range(3)]
    assert all(p.info(4) == 16 for p in parts) and parts[0].info(6) == 16
    pipe = RecurrentPipeline(parts, head=parts[0])
    toks, logits, hidden = pipe.generate([dev_ids(p) for p in prompts], n_new, keep_logits=True, keep_hidden=True, drain="shared")
    torch.cuda.synchronize()
    for p in parts:
        p.sync()
    toks, logits, hidden = host(toks).astype(np.int64), host(logits), host(hidden)
    ops = [O.Partition(cfg, w, bounds[i], bounds[i + 1], has_embed=i == 0, has_head=i == 0) for i in range(3)]
    worst = 0.0
    for s in range(n_seqs):
        x = prompts[s]
        for o in ops:
            x = o.prefill(s, x)
        x = x[-1]
        for j in range(n_new):
            worst = max(worst, check(hidden[s, j], x, cfg, ("hidden", s, j)))
            xr = S.storage_round(x.astype(np.float32), cfg["dtype"])
            want_tok, want = ops[0].sample_greedy(xr)
            check(logits[s, j], want, cfg, ("logits", s, j))
            assert toks[s, j] == int(np.flatnonzero(logits[s, j] == logits[s, j].max())[0])
            top2 = np.sort(want)[-2:]
            if top2[1] - top2[0] > 10 * np.abs(logits[s, j] - want).max():
                assert toks[s, j] == want_tok
            if j + 1 < n_new:
                x = np.array([toks[s, j]], dtype=np.int32)
                for o in ops:
                    x = o.decode_step(s, x)
    print(f"driver, shared passes: worst hidden rel-L2 {worst:.2e}", flush=True)
    # sampled tokens: the same driver with draws from the top-k pmf gives every sample the draw of (seed, sample, step)
    pipe.reset(n_seqs)
    t2, lg2, _ = pipe.generate([dev_ids(p) for p in prompts], 3, keep_logits=True, drain="shared", sampling=(0.9, 8, 77))
    torch.cuda.synchronize()
    t2, lg2 = host(t2).astype(np.int64), host(lg2)
    for s in range(n_seqs):
        for j in range(3):
            u = O.uniform01(77, s, j)
            pmf = O.topk_pmf(lg2[s, j].astype(np.float64), 0.9, 8)
            assert int(t2[s, j]) in pmf
            if np.abs(np.cumsum(list(pmf.values())) - u).min() > 1e-5:
                assert int(t2[s, j]) == O.sample_topk(lg2[s, j], 0.9, 8, u), (s, j)


def test_layernorm_vectors_far_from_zero_mean():
    """LayerNorm in the shared pass publishes (x - c) g in bf16 with c close to the vector's mean.  With a residual
    stream whose mean is far from zero (embeddings with a large common offset) the bf16 hand-off itself limits what
    any path can deliver, so the measure is the error relative to the centred vector - the part that carries
    information - next to that of the one-message path on the same inputs: the shared pass must not be worse by
    more than a half, which x g rounded to bf16 would be several times over."""
    cfg = S.tiny(n_layer=3, dtype=S.DT_BF16, max_ctx=64, vocab=211, **SHAPES["gpt2_like"])
    w = scale_matrices(S.make_weights(cfg, 53, exercise=True), 2.0)
    w["wte"] = S.storage_round(w["wte"] + np.float32(6.0), cfg["dtype"])      # mean / std of an embedding row: about 150
    n = 6
    o, g = pair(cfg, w, 0, 3, embed=True, max_seqs=n, kv_page_tokens=8)
    g1 = mdi.Partition(cfg, w, 0, 3, has_embed=True, max_seqs=n, kv_page_tokens=8)
    assert g.info(4) == 16
    prompts = S.make_prompts(cfg, 53, n, 9)
    for s in range(n):
        check(g.prefill(s, dev_ids(prompts[s])), o.prefill(s, prompts[s]), cfg, ("prefill", s))
        g1.prefill(s, dev_ids(prompts[s]))
    rng = np.random.default_rng(8)
    worst, worst1 = 0.0, 0.0
    for step in range(6):
        toks = [int(rng.integers(0, cfg["vocab"])) for _ in range(n)]
        outs = g.decode_batch(list(range(n)), [dev_ids([t]) for t in toks])
        for s, t, got in zip(range(n), toks, outs):
            want = o.decode_step(s, t)
            scale = np.linalg.norm(want - want.mean())
            worst = max(worst, float(np.linalg.norm(host(got).astype(np.float64) - want) / scale))
            worst1 = max(worst1, float(np.linalg.norm(host(g1.decode_step(s, dev_ids([t]))).astype(np.float64) - want) / scale))
    g.sync()
    g1.sync()
    print(f"far-from-zero mean: worst error relative to the centred vector {worst:.2e} (one message at a time: {worst1:.2e})", flush=True)
    assert worst < 1.5 * worst1 + 2e-3
