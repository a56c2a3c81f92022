"""Helpers for the GPU parity tests: build the same partition on both sides."""
import numpy as np
import torch

from oracle import mdi_oracle as O
from paper_2505_18164_amd import mdi, synth as S


def rel_l2(got, want):
    got = np.asarray(got, dtype=np.float64).ravel()
    want = np.asarray(want, dtype=np.float64).ravel()
    return float(np.linalg.norm(got - want) / np.linalg.norm(want))


def host(t):
    return t.detach().float().cpu().numpy()


def dev_acts(a, cfg):
    return mdi.to_device(a, cfg["dtype"], "cuda:0")


def dev_ids(ids):
    return torch.from_numpy(np.ascontiguousarray(ids, dtype=np.int32)).to("cuda:0")


def tol(cfg):
    """The parity bar: relative L2 error of hidden states and logits against the
    float64 oracle, 1e-4 with fp32 storage, 2e-2 with bf16 storage."""
    return 1e-4 if cfg["dtype"] == S.DT_F32 else 2e-2


def scale_matrices(w, k):
    for lw in w["layers"].values():
        for name in lw:
            if lw[name].ndim == 2:
                lw[name] = lw[name] * np.float32(k)
    return w


def pair(cfg, w, lo, hi, embed=False, head=False, max_seqs=1, **kw):
    o = O.Partition(cfg, w, lo, hi, has_embed=embed, has_head=head)
    g = mdi.Partition(cfg, w, lo, hi, has_embed=embed, has_head=head, max_seqs=max_seqs, **kw)
    return o, g


def rel_l2_rows(got, want):
    """Relative L2 error of every row (position) of a [T, d] result."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    return np.linalg.norm(got - want, axis=-1) / np.linalg.norm(want, axis=-1)


def check(got, want, cfg, what, bar=None):
    """Assert the parity bar with a short message (no array dumps).  A [T, d] result must meet the bar in EVERY
    row as well as over the whole tensor: one wrong row among thousands would vanish in the overall norm."""
    got = host(got) if isinstance(got, torch.Tensor) else np.asarray(got)
    want = np.asarray(want)
    err = rel_l2(got, want)
    bar = tol(cfg) if bar is None else bar
    if not err < bar:
        raise AssertionError(f"{what}: rel-L2 {err:.3e} exceeds {bar:.1e}")
    if want.ndim == 2 and want.shape[0] > 1:
        rows = rel_l2_rows(got.reshape(want.shape), want)
        worst = int(np.argmax(rows))
        if not rows[worst] < bar:
            raise AssertionError(f"{what}: row {worst} of {want.shape[0]} has rel-L2 {rows[worst]:.3e}, exceeds {bar:.1e}")
        err = max(err, float(rows[worst]))
    return err


def teacher_forced(parts, prompts, tokens, want_logits=True, head=None):
    """Run GPU partitions (a chain; the last one owns the output layers) over
    the given prompts, feeding `tokens[s][j]` (the oracle's) as the j-th new
    token instead of the GPU's own argmax.  Samples are visited round-robin as
    in Alg. 1.  Returns hidden[s][j] (input of the output layers when token j
    was produced), logits[s][j], gpu_tokens[s][j].

    All partitions must be on the current stream: nothing here orders one partition's stream after
    another's, and the tensors handed from call to call are released as soon as the next call returns."""
    assert all(p.stream == torch.cuda.current_stream() for p in parts), "teacher_forced needs partitions on the current stream"
    blocks = [p for p in parts if p.hi > p.lo]
    head = parts[-1] if head is None else head           # the paper's starter: head = parts[0]
    ns, n_new = len(prompts), len(tokens[0])
    hidden = [[] for _ in range(ns)]
    logits = [[] for _ in range(ns)]
    toks = [[] for _ in range(ns)]
    back = [None] * ns
    for r in range(n_new + 1):
        for s in range(ns):
            if r >= 1:
                x = back[s]
                lg = torch.empty(head.V, dtype=torch.float32, device="cuda:0") if want_logits else None
                t = head.sample_greedy(s, x, logits_out=lg)
                hidden[s].append(host(x))
                toks[s].append(int(t.item()))
                if want_logits:
                    logits[s].append(host(lg))
            if r < n_new:
                msg = dev_ids(prompts[s]) if r == 0 else dev_ids([tokens[s][r - 1]])
                for p in blocks:
                    msg = p.prefill(s, msg) if r == 0 else p.decode_step(s, msg)
                back[s] = msg[-1] if r == 0 else msg
    return hidden, logits, toks
