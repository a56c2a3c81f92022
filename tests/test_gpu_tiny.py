"""GPU parity on small shapes: every model variant, both storage types, ragged
prompt lengths, page-boundary crossings; error paths of the boundary."""
import numpy as np
import pytest
import torch

from oracle import mdi_oracle as O
from paper_2505_18164_amd import mdi, synth as S
from gpu_util import check, dev_acts, dev_ids, host, pair, rel_l2, scale_matrices, tol

pytestmark = pytest.mark.gpu

VARIANTS = {
    "llama_gqa": dict(),
    "llama_mha": dict(n_kv_head=4),
    "llama_gqa8": dict(n_head=8, n_kv_head=1, d_model=64),
    "llama_group3": dict(n_head=6, n_kv_head=2, d_model=48),
    "gpt2": dict(norm_kind=S.NORM_LAYERNORM, mlp_kind=S.MLP_GELU_TANH, pos_kind=S.POS_LEARNED, has_bias=1, tie_embed=1, n_kv_head=4),
    "gelu_erf": dict(norm_kind=S.NORM_LAYERNORM, mlp_kind=S.MLP_GELU_ERF, pos_kind=S.POS_LEARNED, has_bias=1, n_kv_head=4),
    "wide_head": dict(head_dim=64, n_head=2, n_kv_head=1, d_model=128, d_ff=264),
}


@pytest.mark.parametrize("path", [0, 1], ids=["persistent", "per_op"])
@pytest.mark.parametrize("dtype", [S.DT_F32, S.DT_BF16], ids=["f32", "bf16"])
@pytest.mark.parametrize("name", list(VARIANTS))
def test_full_model_teacher_forced(name, dtype, path):
    cfg = S.tiny(n_layer=3, dtype=dtype, max_ctx=48, **VARIANTS[name])
    # matrices scaled up so that every sub-layer moves the residual stream by O(1);
    # less so with bf16 storage, whose rounding noise three such layers amplify
    w = scale_matrices(S.make_weights(cfg, 31, exercise=True), 6.0 if dtype == S.DT_F32 else 3.0)
    o, g = pair(cfg, w, 0, 3, embed=True, head=True, max_seqs=2, kv_page_tokens=8, decode_path=path)
    prompts = S.make_prompts(cfg, 31, 2, 13)
    prompts[1] = prompts[1][:5]
    rng = np.random.default_rng(5)
    for s in (0, 1):
        want = o.prefill(s, prompts[s])
        got = g.prefill(s, dev_ids(prompts[s]))
        check(got, want, cfg, ("prefill", s))
    V = cfg["vocab"]
    for step in range(22):                      # crosses page boundaries at 8-token pages
        for s in (1, 0):
            t = int(rng.integers(0, V))
            want = o.decode_step(s, t)
            got = g.decode_step(s, dev_ids([t]))
            check(got, want, cfg, ("decode", step, s))
            # the oracle's own activation goes into both heads
            x = S.storage_round(want.astype(np.float32), dtype)
            wt, wl = o.sample_greedy(x)
            lg = torch.empty(V, dtype=torch.float32, device="cuda:0")
            gt = g.sample_greedy(s, dev_acts(x, cfg), logits_out=lg)
            check(lg, wl, cfg, ("logits", step, s))
            gap = np.sort(wl)[-1] - np.sort(wl)[-2]
            if gap > 10 * np.abs(host(lg) - wl).max():
                assert int(gt.item()) == wt
    assert g.seq_len(0) == 13 + 22 and g.seq_len(1) == 5 + 22
    g.sync()


@pytest.mark.parametrize("path", [0, 1], ids=["persistent", "per_op"])
@pytest.mark.parametrize("dtype", [S.DT_F32, S.DT_BF16], ids=["f32", "bf16"])
def test_mid_partition_activations_in_and_out(dtype, path):
    cfg = S.tiny(n_layer=4, dtype=dtype)
    w = scale_matrices(S.make_weights(cfg, 8, exercise=True), 6.0 if dtype == S.DT_F32 else 3.0)
    o, g = pair(cfg, w, 1, 3, max_seqs=1, decode_path=path)
    a = S.make_activations(cfg, 8, 0, 19)
    check(g.prefill(0, dev_acts(a, cfg)), o.prefill(0, a), cfg, "prefill")
    for step in range(5):
        x = S.make_activations(cfg, 8, 0, 1, step=step + 1)[0]
        check(g.decode_step(0, dev_acts(x, cfg)), o.decode_step(0, x), cfg, ("decode", step))


@pytest.mark.parametrize("path", [0, 1], ids=["persistent", "per_op"])
@pytest.mark.parametrize("page_tokens", [5, 12])
def test_page_sizes_that_are_not_powers_of_two(page_tokens, path):
    # the attention kernels locate a cached row by position / page size and position % page size: shifts for the
    # usual page sizes, a division otherwise
    cfg = S.tiny(n_layer=2, dtype=S.DT_F32, max_ctx=64)
    w = scale_matrices(S.make_weights(cfg, 44, exercise=True), 6.0)
    o, g = pair(cfg, w, 0, 2, embed=True, max_seqs=2, kv_page_tokens=page_tokens, decode_path=path)
    prompts = [S.make_prompts(cfg, 44, 1, 17)[0], S.make_prompts(cfg, 45, 1, 6)[0]]
    for s in (0, 1):
        check(g.prefill(s, dev_ids(prompts[s])), o.prefill(s, prompts[s]), cfg, ("prefill", s))
    rng = np.random.default_rng(9)
    for step in range(14):                      # every sample crosses several page boundaries
        toks = [int(rng.integers(0, cfg["vocab"])) for _ in range(2)]
        if step % 2:
            outs = g.decode_steps([1, 0], [dev_ids([toks[1]]), dev_ids([toks[0]])])
            check(outs[0], o.decode_step(1, toks[1]), cfg, ("queued", step, 1))
            check(outs[1], o.decode_step(0, toks[0]), cfg, ("queued", step, 0))
        else:
            for s in (0, 1):
                check(g.decode_step(s, dev_ids([toks[s]])), o.decode_step(s, toks[s]), cfg, ("decode", step, s))
    assert g.seq_len(0) == 17 + 14 and g.seq_len(1) == 6 + 14
    g.sync()


@pytest.mark.parametrize("dtype", [S.DT_F32, S.DT_BF16], ids=["f32", "bf16"])
@pytest.mark.parametrize("name", ["llama_gqa", "llama_gqa8"])
def test_pairs_of_query_heads_share_a_pass_over_the_cache(name, dtype, monkeypatch):
    # long contexts switch the decode kernel to two query heads per pass over their kv head's cache; the switch-over
    # length is lowered here so that small shapes take that path, alone and with queued messages
    monkeypatch.setenv("MDI_GROUP_CTX", "12")
    cfg = S.tiny(n_layer=2, dtype=dtype, max_ctx=48, **VARIANTS[name])
    w = scale_matrices(S.make_weights(cfg, 52, exercise=True), 6.0 if dtype == S.DT_F32 else 3.0)
    o, g = pair(cfg, w, 0, 2, embed=True, max_seqs=2, kv_page_tokens=8)
    prompts = [S.make_prompts(cfg, 52, 1, 9)[0], S.make_prompts(cfg, 53, 1, 4)[0]]
    for s in (0, 1):
        check(g.prefill(s, dev_ids(prompts[s])), o.prefill(s, prompts[s]), cfg, ("prefill", s))
    rng = np.random.default_rng(3)
    for step in range(16):                      # contexts 5..25: both sides of the switch-over
        toks = [int(rng.integers(0, cfg["vocab"])) for _ in range(2)]
        if step % 2:
            outs = g.decode_steps([0, 1], [dev_ids([toks[0]]), dev_ids([toks[1]])])
            for s in (0, 1):
                check(outs[s], o.decode_step(s, toks[s]), cfg, ("queued", step, s))
        else:
            for s in (0, 1):
                check(g.decode_step(s, dev_ids([toks[s]])), o.decode_step(s, toks[s]), cfg, ("decode", step, s))
    g.sync()


def test_prefill_of_one_token_and_argmax_ties():
    cfg = S.tiny(n_layer=1, dtype=S.DT_F32)
    w = S.make_weights(cfg, 2)
    o, g = pair(cfg, w, 0, 1, embed=True, head=True)
    ids = np.array([7], dtype=np.int32)
    assert rel_l2(host(g.prefill(0, dev_ids(ids))), o.prefill(0, ids)) < 1e-4
    # zero activation -> all logits equal (RMSNorm of 0 is 0) -> lowest index wins
    z = torch.zeros(cfg["d_model"], device="cuda:0")
    assert int(g.sample_greedy(0, z).item()) == 0


def test_error_paths_and_page_pool():
    cfg = S.tiny(n_layer=1, dtype=S.DT_F32, max_ctx=16)
    w = S.make_weights(cfg, 3)
    g = mdi.Partition(cfg, w, 0, 1, has_embed=True, max_seqs=3, kv_page_tokens=8, kv_pages=3)
    ids = dev_ids(np.arange(8))
    out = torch.empty(cfg["d_model"], device="cuda:0")

    def status(fn, *a):
        with pytest.raises(mdi.MdiError) as e:
            fn(*a)
        return e.value.status

    assert status(g.decode_step, 0, ids[:1], out) == mdi.MDI_ERR_STATE        # no first visit yet
    assert status(g.prefill, 5, ids) == mdi.MDI_ERR_ARG                      # sample id out of range
    assert status(g.sample_greedy, 0, out) == mdi.MDI_ERR_STATE              # no output layers here
    first = host(g.prefill(0, ids))
    assert status(g.prefill, 0, ids) == mdi.MDI_ERR_STATE                    # cache already live
    g.prefill(1, ids)                                                        # pool: 2 of 3 pages used
    g.decode_step(0, ids[:1], out)                                           # third page
    assert status(g.decode_step, 1, ids[:1], out) == mdi.MDI_ERR_NOMEM       # pool exhausted
    assert status(g.prefill, 2, ids) == mdi.MDI_ERR_NOMEM
    for _ in range(7):
        g.decode_step(0, ids[:1], out)
    assert g.seq_len(0) == 16
    assert status(g.decode_step, 0, ids[:1], out) == mdi.MDI_ERR_CTX         # cache full
    big = dev_ids(np.zeros(17))
    g.seq_reset(0)
    assert g.seq_len(0) == 0
    assert status(g.prefill, 0, big) == mdi.MDI_ERR_CTX
    again = host(g.prefill(0, ids))                                          # pages were returned and are reusable
    np.testing.assert_array_equal(again, first)
    g.sync()


@pytest.mark.parametrize("path", [0, 1], ids=["persistent", "per_op"])
@pytest.mark.parametrize("dtype", [S.DT_F32, S.DT_BF16], ids=["f32", "bf16"])
def test_streams_do_not_change_results(dtype, path):
    """Three chunks on three streams (the single-GPU stand-in for three nodes, Sec. III-C) give the
    bits of the same chunks on one stream, run after run: nothing read by one kernel may be a stale
    copy of what an earlier kernel, or another workgroup of the same kernel, wrote.  Small heads make
    several cache rows share a cache line, the worst case for that."""
    from paper_2505_18164_amd.pipeline import RecurrentPipeline
    cfg = S.tiny(n_layer=6, dtype=dtype, max_ctx=96, vocab=211)
    w = S.make_weights(cfg, 17, exercise=True)
    prompts = [dev_ids(p) for p in S.make_prompts(cfg, 17, 4, 9)]

    def run(streams):
        parts = [mdi.Partition(cfg, w, 0, 2, has_embed=True, max_seqs=4, stream=streams[0], kv_page_tokens=8, decode_path=path),
                 mdi.Partition(cfg, w, 2, 4, max_seqs=4, stream=streams[1], kv_page_tokens=8, decode_path=path),
                 mdi.Partition(cfg, w, 4, 6, has_head=True, max_seqs=4, stream=streams[2], kv_page_tokens=8, decode_path=path)]
        t, _, h = RecurrentPipeline(parts).generate(prompts, 60, keep_hidden=True)
        torch.cuda.synchronize()
        for p in parts:
            p.sync()
        return t.cpu(), h.float().cpu()

    ref = run([None, None, None])
    for rep in range(4):
        got = run([torch.cuda.Stream() for _ in range(3)])
        assert torch.equal(got[0], ref[0]), rep
        assert torch.equal(got[1], ref[1]), rep


@pytest.mark.parametrize("shape", [dict(head_dim=64, n_head=4, n_kv_head=2, d_model=256, d_ff=384),
                                   dict(head_dim=128, n_head=2, n_kv_head=2, d_model=256, d_ff=384),
                                   dict(head_dim=64, n_head=4, n_kv_head=4, d_model=128, d_ff=256, norm_kind=S.NORM_LAYERNORM,
                                        mlp_kind=S.MLP_GELU_TANH, pos_kind=S.POS_LEARNED, has_bias=1)],
                         ids=["gqa_h64", "mha_h128", "gpt2_h64"])
@pytest.mark.parametrize("T", [1, 63, 64, 129, 200, 333])
def test_first_visit_attention_on_matrix_cores(shape, T):
    """bf16 first visits with 64- and 128-wide heads run their causal attention on the matrix cores
    (transposed products, one query per lane).  Prompt lengths around the 64-key and 128-query block
    edges, then decode steps that read the cache the first visit wrote."""
    cfg = S.tiny(n_layer=2, dtype=S.DT_BF16, max_ctx=352, vocab=97, **shape)
    w = scale_matrices(S.make_weights(cfg, 77, exercise=True), 2.0)
    o, g = pair(cfg, w, 0, 2, embed=True, max_seqs=1, kv_page_tokens=16)
    ids = S.make_prompts(cfg, 77, 1, T)[0]
    check(g.prefill(0, dev_ids(ids)), o.prefill(0, ids), cfg, ("prefill", T))
    for step in range(3):
        t = (7 * step + 3) % cfg["vocab"]
        check(g.decode_step(0, dev_ids([t])), o.decode_step(0, t), cfg, ("decode", step))
    g.sync()


@pytest.mark.parametrize("path", [0, 1], ids=["persistent", "per_op"])
@pytest.mark.parametrize("dtype", [S.DT_F32, S.DT_BF16], ids=["f32", "bf16"])
@pytest.mark.parametrize("name", ["llama_gqa", "llama_group3", "gpt2", "wide_head"])
def test_queued_messages_taken_together(name, dtype, path):
    """Several samples' later visits handed over in one call (Sec. III-A: messages wait in the input queue;
    Sec. III-C: several samples in flight) match the oracle, agree with the same visits taken one call at a time
    far inside that bar (only the order of a row's partial sums may differ) and reproduce their own bits when
    the same calls are made again; samples have different lengths, cross page boundaries at different steps, and
    the number of messages is odd as well as even."""
    cfg = S.tiny(n_layer=3, dtype=dtype, max_ctx=48, **VARIANTS[name])
    w = scale_matrices(S.make_weights(cfg, 41, exercise=True), 6.0 if dtype == S.DT_F32 else 3.0)
    n_seq = 5
    o, g = pair(cfg, w, 0, 3, embed=True, max_seqs=n_seq, kv_page_tokens=8, decode_path=path)
    g1 = mdi.Partition(cfg, w, 0, 3, has_embed=True, max_seqs=n_seq, kv_page_tokens=8, decode_path=path)
    g2 = mdi.Partition(cfg, w, 0, 3, has_embed=True, max_seqs=n_seq, kv_page_tokens=8, decode_path=path)
    prompts = S.make_prompts(cfg, 41, n_seq, 11)
    for s in range(n_seq):
        prompts[s] = prompts[s][:3 + 2 * s]
        o.prefill(s, prompts[s])
        g.prefill(s, dev_ids(prompts[s]))
        g1.prefill(s, dev_ids(prompts[s]))
        g2.prefill(s, dev_ids(prompts[s]))
    rng = np.random.default_rng(9)
    V = cfg["vocab"]
    for step in range(12):
        order = [int(s) for s in rng.permutation(n_seq)][: (n_seq if step % 3 else n_seq - 1 - step % 2)]
        toks = [int(rng.integers(0, V)) for _ in order]
        ins = [dev_ids([t]) for t in toks]
        outs = g.decode_steps(order, ins)
        again = g2.decode_steps(order, ins)
        for s, t, x, got, rep in zip(order, toks, ins, outs, again):
            check(got, o.decode_step(s, t), cfg, ("decode", step, s))
            assert torch.equal(got, rep), (step, s)
            assert rel_l2(host(got), host(g1.decode_step(s, x)).astype(np.float64)) <= 0.25 * tol(cfg), (step, s)
    for s in range(n_seq):
        assert g.seq_len(s) == g1.seq_len(s) == g2.seq_len(s)
    g.sync()
    g1.sync()
    g2.sync()


@pytest.mark.parametrize("path", [0, 1], ids=["persistent", "per_op"])
def test_token_id_out_of_range_is_reported_not_followed(path):
    """Token ids live in device memory, so only the kernels can check them: an id outside [0, vocab) must not be
    used as an index; the next mdi_partition_sync reports it."""
    cfg = S.tiny(n_layer=2, dtype=S.DT_F32, max_ctx=32)
    w = S.make_weights(cfg, 5)
    V = cfg["vocab"]
    for where in ("first visit", "later visit", "queued"):
        if where == "queued" and path != 0:
            continue
        g = mdi.Partition(cfg, w, 0, 2, has_embed=True, max_seqs=2, decode_path=path)
        good = dev_ids(np.arange(4))
        if where == "first visit":
            g.prefill(0, dev_ids([1, V + 3, 2, -7]))
        else:
            g.prefill(0, good)
            g.prefill(1, good)
            g.sync()
            if where == "later visit":
                g.decode_step(0, dev_ids([2 ** 30]))
            else:
                g.decode_steps([0, 1], [dev_ids([3]), dev_ids([V])])
        with pytest.raises(mdi.MdiError) as e:
            g.sync()
        assert e.value.status == mdi.MDI_ERR_ARG, where


def test_queued_messages_error_paths():
    cfg = S.tiny(n_layer=1, dtype=S.DT_F32, max_ctx=16)
    w = S.make_weights(cfg, 3)
    g = mdi.Partition(cfg, w, 0, 1, has_embed=True, max_seqs=3, kv_page_tokens=8, kv_pages=3)
    ids = dev_ids(np.arange(8))

    def status(seqs):
        with pytest.raises(mdi.MdiError) as e:
            g.decode_steps(seqs, [ids[:1]] * len(seqs))
        return e.value.status

    g.prefill(0, ids)
    g.prefill(1, ids)
    assert status([0, 2]) == mdi.MDI_ERR_STATE            # sample 2 has no first visit yet
    assert status([0, 0]) == mdi.MDI_ERR_ARG              # one message per sample
    assert status([0, 7]) == mdi.MDI_ERR_ARG
    assert status([0, 1]) == mdi.MDI_ERR_NOMEM            # both need a new page, one is free
    assert g.seq_len(0) == 8 and g.seq_len(1) == 8        # a refused call advances nothing
    g.decode_steps([1], [ids[:1]])
    assert g.seq_len(1) == 9
    g.sync()


@pytest.mark.parametrize("dtype", [S.DT_F32, S.DT_BF16], ids=["f32", "bf16"])
def test_stochastic_sampling_matches_the_oracle_draw_for_draw(dtype):
    """Alg. 1 samples the output distribution.  Same counter-based uniform number on both sides, so the token must be
    the same whenever the number does not fall within the logits' error of a boundary of the cumulative
    distribution; top_k = 1 is greedy; a draw is a function of (seed, sample, step) only; and over many steps the
    GPU's tokens follow the oracle's pmf."""
    cfg = S.tiny(n_layer=1, dtype=dtype, vocab=211, d_model=64, n_head=4, n_kv_head=2, head_dim=16, d_ff=96)
    w = scale_matrices(S.make_weights(cfg, 77, exercise=True), 8.0)
    o, g = pair(cfg, w, 0, 1, embed=True, head=True, max_seqs=2)
    ids = S.make_prompts(cfg, 77, 1, 6)[0]
    x = S.storage_round(o.prefill(0, ids)[-1].astype(np.float32), dtype)
    g.prefill(0, dev_ids(ids))
    xd = dev_acts(x, cfg)
    lg_o = o.logits(x)
    lg_g = torch.empty(cfg["vocab"], dtype=torch.float32, device="cuda:0")
    seed, temperature, top_k = 0x1234567890ABCDEF, 0.8, 12
    err = None
    decided = agree = 0
    counts = {}
    n = 400
    for step in range(n):
        tok = int(g.sample_topk(1, xd, temperature, top_k, seed, step, logits_out=lg_g if step == 0 else None).item())
        if step == 0:
            check(lg_g, lg_o, cfg, "logits")
            err = float(np.abs(host(lg_g) - lg_o).max()) / temperature      # bound on the shift of a log-weight
        counts[tok] = counts.get(tok, 0) + 1
        want = O.sample_topk(lg_o, temperature, top_k, O.uniform01(seed, 1, step))
        pmf = O.topk_pmf(lg_o, temperature, top_k)
        assert tok in pmf
        edges = np.cumsum(list(pmf.values()))
        margin = np.abs(edges - O.uniform01(seed, 1, step)).min()
        if margin > 4 * err + 1e-5:                                         # a boundary moves by less than 2 err
            decided += 1
            agree += tok == want
    assert decided >= 0.8 * n and agree == decided, (decided, agree)
    chi2 = sum((counts.get(t, 0) - n * p) ** 2 / (n * p) for t, p in O.topk_pmf(lg_o, temperature, top_k).items() if n * p >= 5)
    assert chi2 < 40.0, chi2
    # top_k = 1 is the greedy token whatever the seed; a draw depends on (seed, sample, step) only
    assert int(g.sample_topk(0, xd, 1.3, 1, 5, 9).item()) == int(g.sample_greedy(0, xd).item())
    a = [int(g.sample_topk(0, xd, 1.5, 40, 7, s).item()) for s in range(30)]
    b = [int(g.sample_topk(0, xd, 1.5, 40, 7, s).item()) for s in range(30)]
    c = [int(g.sample_topk(0, xd, 1.5, 40, 8, s).item()) for s in range(30)]
    assert a == b and a != c and len(set(a)) > 5
    with pytest.raises(mdi.MdiError):
        g.sample_topk(0, xd, 0.0, 5, 1, 1)
    with pytest.raises(mdi.MdiError):
        g.sample_topk(0, xd, 1.0, 65, 1, 1)
    g.sync()


def test_generation_with_sampled_tokens_through_the_ring():
    """Alg. 1 with its own token rule (a draw from the pmf) on a three-node ring in fp32: the sampled sequences are
    those of the oracle, with every stage on its own stream and with stages draining their queues."""
    from paper_2505_18164_amd.pipeline import RecurrentPipeline
    cfg = S.tiny(n_layer=3, dtype=S.DT_F32, max_ctx=40, vocab=97)
    w = scale_matrices(S.make_weights(cfg, 23, exercise=True), 6.0)
    prompts = S.make_prompts(cfg, 23, 3, 4)
    sampling = (0.9, 8, 424242)
    ops = [O.Partition(cfg, w, 0, 1, has_embed=True, has_head=True), O.Partition(cfg, w, 1, 3)]
    toks_o, _, _ = O.generate(ops, prompts, 20, sampling=sampling, head=ops[0])
    assert len({tuple(t) for t in toks_o}) == 3                      # samples differ: each has its own counter
    for drain in (False, True):
        parts = [mdi.Partition(cfg, w, 0, 1, has_embed=True, has_head=True, max_seqs=3, stream=torch.cuda.Stream()),
                 mdi.Partition(cfg, w, 1, 3, max_seqs=3, stream=torch.cuda.Stream())]
        t, _, _ = RecurrentPipeline(parts, head=parts[0]).generate([dev_ids(p) for p in prompts], 20, drain=drain, sampling=sampling)
        torch.cuda.synchronize()
        for p in parts:
            p.sync()
        assert t.cpu().numpy().tolist() == [list(x) for x in toks_o], drain


@pytest.mark.parametrize("path", [0, 1], ids=["persistent", "per_op"])
@pytest.mark.parametrize("dtype", [S.DT_F32, S.DT_BF16], ids=["f32", "bf16"])
@pytest.mark.parametrize("name", ["llama_gqa", "gpt2", "wide_head"])
def test_first_visit_in_pieces(name, dtype, path):
    """A prompt forwarded in several pieces (each continuing at the cache length, crossing page boundaries, one of
    them a single position) gives the rows of the oracle's one first visit of the whole prompt, the later visits
    that follow agree as well, and another sample's visits fit in between the pieces."""
    cfg = S.tiny(n_layer=3, dtype=dtype, max_ctx=48, **VARIANTS[name])
    w = scale_matrices(S.make_weights(cfg, 61, exercise=True), 6.0 if dtype == S.DT_F32 else 3.0)
    o, g = pair(cfg, w, 0, 3, embed=True, max_seqs=2, kv_page_tokens=8)
    prompts = S.make_prompts(cfg, 61, 2, 21)
    want = o.prefill(0, prompts[0])
    o2 = O.Partition(cfg, w, 0, 3, has_embed=True)                  # the oracle taking the same pieces
    check(g.prefill(1, dev_ids(prompts[1][:6])), o.prefill(1, prompts[1][:6]), cfg, "other sample, first visit")
    at = 0
    for piece in (5, 1, 9, 6):
        got = g.prefill_chunk(0, dev_ids(prompts[0][at:at + piece]))
        check(got, want[at:at + piece], cfg, ("piece at", at))
        check(got, o2.prefill_chunk(0, prompts[0][at:at + piece]), cfg, ("piece at, oracle in pieces", at))
        at += piece
        check(g.decode_step(1, dev_ids([at])), o.decode_step(1, at), cfg, ("other sample between pieces", at))
    assert g.seq_len(0) == 21
    for step in range(4):
        check(g.decode_step(0, dev_ids([step + 3])), o.decode_step(0, step + 3), cfg, ("later visit", step))
    with pytest.raises(mdi.MdiError) as e:
        g.prefill_chunk(0, dev_ids(np.zeros(30)))
    assert e.value.status == mdi.MDI_ERR_CTX
    g.sync()


def test_more_queued_messages_than_one_launch_carries():
    """Eleven samples' messages in one call: launches of 8 and of 3 (sets of 2 and 1), every sample against the oracle."""
    cfg = S.tiny(n_layer=2, dtype=S.DT_F32, max_ctx=32)
    w = scale_matrices(S.make_weights(cfg, 13, exercise=True), 6.0)
    n = 11
    o, g = pair(cfg, w, 0, 2, embed=True, max_seqs=n, kv_page_tokens=8)
    prompts = S.make_prompts(cfg, 13, n, 9)
    for s in range(n):
        prompts[s] = prompts[s][:1 + s % 9]
        o.prefill(s, prompts[s])
        g.prefill(s, dev_ids(prompts[s]))
    for step in range(10):                       # every sample crosses a page boundary at some step
        outs = g.decode_steps(list(range(n)), [dev_ids([(7 * s + step) % cfg["vocab"]]) for s in range(n)])
        for s in range(n):
            check(outs[s], o.decode_step(s, (7 * s + step) % cfg["vocab"]), cfg, ("decode", step, s))
    g.sync()
