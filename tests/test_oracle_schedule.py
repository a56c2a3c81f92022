"""Pins for the schedule: Alg. 1 (starter), Alg. 2 (secondary), Fig. 2."""
import os

import numpy as np
import pytest

from oracle import mdi_oracle as O
from paper_2505_18164_amd import synth as S

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_starter_loop_counts():
    """Alg. 1: n_iterations = n_samples * n_tokens; the first visit of each
    sample initialises its cache; every later visit applies the output layers;
    the last visit of each sample forwards nothing."""
    ns, nt = 3, 5
    sch = O.starter_schedule(ns, nt)
    assert len(sch) == ns * nt
    assert [n for _, n, *_ in sch] == [k % ns for k in range(ns * nt)]
    assert sum(1 for s in sch if s[5]) == ns                              # prefills
    assert all(s[5] == (s[2] == 0) for s in sch)
    assert sum(1 for s in sch if s[3]) == ns * (nt - 1)                   # tokens appended
    assert sum(1 for s in sch if s[4]) == ns * (nt - 1)                   # messages sent round the ring
    assert all(not s[4] for s in sch[-ns:]) and all(s[3] for s in sch[-ns:])


def test_fig2_walkthrough():
    want = [l.split() for l in open(os.path.join(GOLD, "fig2_schedule_3nodes_3samples.txt")) if not l.startswith("#")]
    busy = O.pipeline_ticks(3, 3, 4)
    got = [["-" if n is None else str(n + 1) for n in row] for row in busy[:len(want)]]
    assert got == want


@pytest.mark.parametrize("ns,nn", [(3, 3), (5, 3), (2, 3), (1, 4), (8, 4), (4, 1)])
def test_no_idle_nodes_when_samples_cover_nodes(ns, nn):
    """Sec. III-C: with balanced stages nobody idles once n_samples >= n_nodes;
    with fewer samples a node is busy n_samples out of n_nodes ticks."""
    rounds = 12
    busy = O.pipeline_ticks(ns, nn, rounds)
    period = max(ns, nn)
    steady = busy[2 * period:-2 * period]
    assert len(steady) >= period
    util = np.mean([[b is not None for b in row] for row in steady], axis=0)
    np.testing.assert_allclose(util, min(1.0, ns / nn), atol=1.0 / len(steady) * period)
    # total work at the starter = n_samples * rounds visits (Alg. 1's iteration count)
    assert sum(row[0] is not None for row in busy) == ns * rounds


def test_generate_visits_and_token_counts():
    cfg = S.tiny(n_layer=3)
    w = S.make_weights(cfg, 4)
    prompts = S.make_prompts(cfg, 4, 2, 5)
    parts = [O.Partition(cfg, w, 0, 1, has_embed=True), O.Partition(cfg, w, 1, 3), O.Partition(cfg, w, 3, 3, has_head=True)]
    trace = []
    toks, logits, hidden = O.generate(parts, prompts, 4, trace=trace)
    assert [len(t) for t in toks] == [4, 4]
    # every stage sees each sample once per round, prefill first, in sample order
    for stage in (0, 1):
        seen = [(n, kind) for _, n, s, kind in trace if s == stage]
        assert seen == [(0, "prefill"), (1, "prefill")] + [(0, "decode"), (1, "decode")] * 3
    # the last token is never fed back: caches hold prompt + n_new - 1 positions
    assert parts[0].seq_len(0) == 5 + 3 and parts[1].seq_len(1) == 5 + 3
    # same tokens as one unsplit partition generating each sample on its own
    for s in range(2):
        one = O.Partition(cfg, w, 0, 3, has_embed=True, has_head=True)
        t1, _, _ = O.generate([one], [prompts[s]], 4)
        assert t1[0] == toks[s]
    # tokens are the argmax of the returned logits, and the pmf is a distribution
    for s in range(2):
        for t, lg in zip(toks[s], logits[s]):
            assert t == int(np.argmax(lg))
            np.testing.assert_allclose(O.pmf(lg).sum(), 1.0, atol=1e-12)
        for x, lg in zip(hidden[s], logits[s]):
            np.testing.assert_array_equal(parts[-1].logits(x), lg)
