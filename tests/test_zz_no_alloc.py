"""The entry point that allocates nothing (mdi_sample_topk_static) against the entry point it is a variant of
(mdi_sample_topk), through the C ABI: token and logits bit-identical, on two calls in a row of which the second
has the smaller input, so that whatever the first call left in the library's fixed scratch array must not leak
into the second."""
import numpy as np
import pytest
import torch

from paper_2505_18164_amd import mdi, synth as S
from gpu_util import dev_acts

pytestmark = pytest.mark.gpu


def head_partition(vocab, d, dtype, decode_path=0, seed=5):
    cfg = S.tiny(n_layer=1, d_model=d, n_head=d // 16, n_kv_head=d // 16, head_dim=16, d_ff=2 * d, vocab=vocab, dtype=dtype)
    w = S.make_weights(cfg, seed, 1, 1, embed=False, head=True, exercise=True)
    w["lm_head"] = w["lm_head"] * np.float32(10.0)                 # logits of O(1): the draw is not a coin flip among equals
    return cfg, mdi.Partition(cfg, w, 1, 1, has_head=True, max_seqs=4, decode_path=decode_path)


@pytest.mark.parametrize("decode_path", [0, 1], ids=["streaming_head", "per_op_head"])
@pytest.mark.parametrize("dtype", [S.DT_F32, S.DT_BF16], ids=["f32", "bf16"])
def test_static_scratch_variant_equals_the_arena_variant(dtype, decode_path):
    big_cfg, big = head_partition(50257, 256, dtype, decode_path)
    small_cfg, small = head_partition(997, 64, dtype, decode_path, seed=6)
    token = torch.empty((1,), dtype=torch.int32, device="cuda:0")
    for rep in range(2):                                           # the pair of calls twice: state left behind is harmless
        for cfg, part, (temperature, top_k) in ((big_cfg, big, (0.8, 40)), (small_cfg, small, (1.3, 7))):
            V = cfg["vocab"]
            for step in range(3):
                x = dev_acts(S.make_activations(cfg, 11 + rep, step, 1)[0], cfg)
                want_logits = torch.empty(V, dtype=torch.float32, device="cuda:0")
                got_logits = torch.full((V,), float("nan"), dtype=torch.float32, device="cuda:0")
                want = part.sample_topk(2, x, temperature, top_k, 1234, step, logits_out=want_logits)
                got = part.sample_topk_static(2, x, temperature, top_k, 1234, step, token_out=token, logits_out=got_logits)
                torch.cuda.synchronize()
                assert int(got.item()) == int(want.item()), (V, step)
                assert torch.equal(got_logits, want_logits), (V, step)
                # top_k = 1 is the greedy token; no logits asked for
                g = part.sample_topk_static(1, x, 1.0, 1, 99, step, token_out=token)
                assert int(g.item()) == int(part.sample_greedy(1, x).item()) == int(torch.argmax(want_logits).item())
    big.sync()
    small.sync()


def test_static_scratch_limit_and_argument_errors():
    cfg, part = head_partition(262144 + 8, 32, S.DT_BF16)
    x = dev_acts(S.make_activations(cfg, 3, 0, 1)[0], cfg)
    token = torch.empty((1,), dtype=torch.int32, device="cuda:0")
    with pytest.raises(mdi.MdiError) as e:
        part.sample_topk_static(0, x, 1.0, 4, 1, 0, token_out=token)
    assert e.value.status == mdi.MDI_ERR_LIMIT
    assert "scratch" in str(e.value)
    part.sample_topk(0, x, 1.0, 4, 1, 0, token_out=token)           # the arena variant takes the same vocabulary
    cfg2, ok = head_partition(262144, 32, S.DT_BF16)
    x2 = dev_acts(S.make_activations(cfg2, 3, 0, 1)[0], cfg2)
    a = ok.sample_topk(0, x2, 1.0, 4, 1, 0)
    b = ok.sample_topk_static(0, x2, 1.0, 4, 1, 0, token_out=token)  # exactly at the limit
    torch.cuda.synchronize()
    assert int(a.item()) == int(b.item())
    for bad in (dict(temperature=0.0), dict(top_k=0), dict(top_k=65), dict(seq=99)):
        kw = dict(seq=0, temperature=1.0, top_k=4)
        kw.update(bad)
        with pytest.raises(mdi.MdiError) as e:
            ok.sample_topk_static(kw["seq"], x2, kw["temperature"], kw["top_k"], 1, 0, token_out=token)
        assert e.value.status == mdi.MDI_ERR_ARG
    # a partition without output layers
    cfgb = S.tiny(n_layer=1, dtype=S.DT_F32)
    blocks = mdi.Partition(cfgb, S.make_weights(cfgb, 1, 0, 1, embed=False, head=False), 0, 1, max_seqs=1)
    with pytest.raises(mdi.MdiError) as e:
        blocks.sample_topk_static(0, dev_acts(S.make_activations(cfgb, 1, 0, 1)[0], cfgb), 1.0, 2, 1, 0, token_out=token)
    assert e.value.status == mdi.MDI_ERR_STATE
    part.sync()
    ok.sync()
