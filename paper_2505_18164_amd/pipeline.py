"""Single-GPU recurrent-pipeline driver (Sec. III-C, Alg. 1 and Alg. 2).

Several partitions live on one MI355X, each on its own HIP stream (the stand-in
for a node of the ring).  Samples circulate round-robin: the starter's visit
k serves sample k mod n_samples; a first visit forwards the whole prompt, later
visits forward the newest token; the output layers turn the returning
activation into the next token, which stays in device memory and is the next
input of the embedding stage.  Hand-offs between stages are stream events (the
analogue of the paper's FIFO queues); the host never waits inside the loop.
With `drain=True` a stage takes all the messages waiting in its queue in one
call (mdi_decode_steps) instead of one call per message: on one GPU every
sample's message is waiting when a stage gets its turn.  With `drain="shared"`
the waiting messages also share one pass over the stage's weights
(mdi_decode_batch) and over the vocabulary matrix (mdi_sample_batch).
No arithmetic happens here.
"""
from __future__ import annotations

import torch


class RecurrentPipeline:
    def __init__(self, parts, head=None):
        """parts: chain of mdi.Partition in ring order; parts[0] owns the embedding.  head: the partition
        that owns the output layers - by default parts[-1] (it may be a head-only partition); pass parts[0]
        for the paper's starter node, which holds the embedding, the first blocks AND the output layers
        (Sec. III-B) and so closes the ring."""
        head = parts[-1] if head is None else head
        if not (parts[0].flags & 1) or not (head.flags & 2):
            raise ValueError("first partition needs the embedding, the head partition the output layers")
        self.parts = parts if any(p is head for p in parts) else parts + [head]
        self.blocks = [p for p in parts if p.hi > p.lo]
        self.head = head
        self.sampling = None
        self.device = parts[0].device

    def _token(self, s, r, x, out, logits):
        """Output layers for sample s in round r: greedy, or a draw from the top-k tempered pmf (Alg. 1)."""
        if self.sampling is None:
            self.head.sample_greedy(s, x, out, logits)
        else:
            temperature, top_k, seed = self.sampling
            self.head.sample_topk(s, x, temperature, top_k, seed, r - 1, out, logits)

    def generate(self, prompts, n_new, keep_logits=False, keep_hidden=False, drain=False, sampling=None):
        """prompts: list of int32 device tensors.  Returns tokens [n_seqs, n_new] (int32, device)
        and optionally per-token logits [n_seqs, n_new, V] / final hidden states [n_seqs, n_new, d].
        sampling: None for greedy tokens, or (temperature, top_k, seed): token j of sample s is drawn with the
        counter-based uniform number of (seed, s, j)."""
        self.sampling = sampling
        if drain:
            return self._generate_draining(prompts, n_new, keep_logits, keep_hidden, shared=(drain == "shared"))
        ns, dev = len(prompts), self.device
        d, V = self.head.d, self.head.V
        toks = torch.zeros((ns, n_new), dtype=torch.int32, device=dev)
        logits = torch.zeros((ns, n_new, V), dtype=torch.float32, device=dev) if keep_logits else None
        hidden = torch.zeros((ns, n_new, d), dtype=self.head.tdtype, device=dev) if keep_hidden else None
        nb = len(self.blocks)
        pre = [[torch.empty((len(prompts[s]), d), dtype=self.head.tdtype, device=dev) for _ in range(nb)] for s in range(ns)]
        act = [[torch.empty((d,), dtype=self.head.tdtype, device=dev) for _ in range(nb)] for s in range(ns)]
        back = [None] * ns                       # activation waiting at the starter, per sample
        ev_back = [None] * ns
        main = torch.cuda.current_stream(dev)
        start = torch.cuda.Event()
        start.record(main)
        for p in self.parts:
            p.stream.wait_event(start)
        n_rounds = n_new + 1
        for k in range(ns * n_rounds):
            s, r = k % ns, k // ns
            if r >= 1:                            # output layers, then the new token joins the sample
                hs = self.head.stream
                hs.wait_event(ev_back[s])
                x = back[s]
                if keep_hidden:
                    with torch.cuda.stream(hs):
                        hidden[s, r - 1].copy_(x)
                self._token(s, r, x, toks[s, r - 1:r], logits[s, r - 1] if keep_logits else None)
                ev_tok = torch.cuda.Event()
                ev_tok.record(hs)
            if r < n_rounds - 1:                  # forward through the ring
                msg = prompts[s] if r == 0 else toks[s, r - 1:r]
                ev = ev_tok if r >= 1 else None
                for i, p in enumerate(self.blocks):
                    if ev is not None:
                        p.stream.wait_event(ev)
                    if r == 0:
                        out = p.prefill(s, msg, pre[s][i])
                    else:
                        out = p.decode_step(s, msg, act[s][i])
                    ev = torch.cuda.Event()
                    ev.record(p.stream)
                    msg = out
                back[s] = msg[-1] if r == 0 else msg
                ev_back[s] = ev
        for p in self.parts:
            done = torch.cuda.Event()
            done.record(p.stream)
            main.wait_event(done)
        return toks, logits, hidden

    def _generate_draining(self, prompts, n_new, keep_logits, keep_hidden, shared=False):
        """Same schedule, but in every round after the first a stage takes the messages of all samples in one
        call; a sample's values are those of the one-message-at-a-time schedule up to summation order (shared:
        within the storage type's parity bar, the vectors between the matrix products being rounded)."""
        ns, dev = len(prompts), self.device
        d, V = self.head.d, self.head.V
        tdt = self.head.tdtype
        # stored round-major: a round's tokens (and logits) of all samples are contiguous, as one call writes them
        toks = torch.zeros((n_new, ns), dtype=torch.int32, device=dev)
        logits = torch.zeros((n_new, ns, V), dtype=torch.float32, device=dev) if keep_logits else None
        hidden = torch.zeros((ns, n_new, d), dtype=tdt, device=dev) if keep_hidden else None
        nb = len(self.blocks)
        act = [[torch.empty((d,), dtype=tdt, device=dev) for _ in range(nb)] for s in range(ns)]
        # every buffer a stage writes lives until the end: the stages run on streams the allocator does not know
        pre = [[torch.empty((len(prompts[s]), d), dtype=tdt, device=dev) for _ in range(nb)] for s in range(ns)]
        main = torch.cuda.current_stream(dev)
        ev = torch.cuda.Event()
        ev.record(main)
        back = [None] * ns
        for s in range(ns):                       # first visits: one sample per message, as always
            msg, e = prompts[s], ev
            for i, p in enumerate(self.blocks):
                p.stream.wait_event(e)
                msg = p.prefill(s, msg, pre[s][i])
                e = torch.cuda.Event()
                e.record(p.stream)
            back[s] = msg[-1]
            last = e
        hs = self.head.stream
        for r in range(1, n_new + 1):
            hs.wait_event(last)
            for s in range(ns):
                if keep_hidden:
                    with torch.cuda.stream(hs):
                        hidden[s, r - 1].copy_(back[s])
                if not shared:
                    self._token(s, r, back[s], toks[r - 1, s:s + 1], logits[r - 1, s] if keep_logits else None)
            if shared:
                temperature, top_k, seed = self.sampling if self.sampling is not None else (1.0, 1, 0)
                self.head.sample_batch(list(range(ns)), back, temperature, top_k, seed, [r - 1] * ns, toks[r - 1],
                                       logits[r - 1] if keep_logits else None)
            last = torch.cuda.Event()
            last.record(hs)
            if r == n_new:
                break
            msgs = [toks[r - 1, s:s + 1] for s in range(ns)]
            for i, p in enumerate(self.blocks):
                p.stream.wait_event(last)
                step = p.decode_batch if shared else p.decode_steps
                msgs = step(list(range(ns)), msgs, [act[s][i] for s in range(ns)])
                last = torch.cuda.Event()
                last.record(p.stream)
            back = msgs
        for p in self.parts:
            done = torch.cuda.Event()
            done.record(p.stream)
            main.wait_event(done)
        return toks.t(), (logits.transpose(0, 1) if keep_logits else None), hidden

    def reset(self, n_seqs):
        for p in self.blocks:
            for s in range(n_seqs):
                p.seq_reset(s)
