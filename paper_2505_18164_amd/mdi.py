"""ctypes binding of libmdi (include/mdi.h).  Argument marshalling only: every
step of the path runs in the library's HIP kernels; PyTorch supplies device
memory and streams.  Loading fails loudly when the shared object is missing;
there is no CPU or PyTorch fallback."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmdi.so")

MDI_ABI_VERSION = 1
MDI_OK, MDI_ERR_ARG, MDI_ERR_STATE, MDI_ERR_CTX, MDI_ERR_NOMEM, MDI_ERR_HIP, MDI_ERR_LIMIT = 0, -1, -2, -3, -4, -5, -6
MDI_F32, MDI_BF16 = 0, 1
MDI_HAS_EMBED, MDI_HAS_HEAD = 1, 2

EXPORTS = ["mdi_partition_bytes", "mdi_partition_create", "mdi_prefill", "mdi_prefill_chunk", "mdi_decode_step", "mdi_decode_steps", "mdi_decode_batch",
           "mdi_sample_greedy", "mdi_sample_topk", "mdi_sample_topk_static", "mdi_sample_batch", "mdi_partition_sync", "mdi_seq_reset", "mdi_seq_len", "mdi_step_bytes", "mdi_time_kernel",
           "mdi_partition_info", "mdi_partition_trace", "mdi_partition_destroy", "mdi_strerror"]


class MdiConfig(C.Structure):
    _fields_ = [(n, C.c_uint32) for n in ("abi_version", "n_layer", "d_model", "n_head", "n_kv_head", "head_dim",
                                          "d_ff", "vocab", "max_ctx", "max_seqs", "kv_page_tokens", "kv_pages",
                                          "max_prefill", "norm_kind")] + \
               [("norm_eps", C.c_float), ("mlp_kind", C.c_uint32), ("pos_kind", C.c_uint32), ("rope_base", C.c_float),
                ("has_bias", C.c_uint32), ("tie_embed", C.c_uint32), ("dtype", C.c_uint32), ("decode_path", C.c_uint32)]


_LAYER_FIELDS = ("ln1_g", "ln1_b", "wq", "wk", "wv", "bq", "bk", "bv", "wo", "bo", "ln2_g", "ln2_b",
                 "w_gate", "w_up", "b_up", "w_down", "b_down")


class MdiLayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _LAYER_FIELDS]


class MdiWeights(C.Structure):
    _fields_ = [("wte", C.c_void_p), ("wpe", C.c_void_p), ("lnf_g", C.c_void_p), ("lnf_b", C.c_void_p),
                ("lm_head", C.c_void_p), ("layers", C.POINTER(MdiLayerWeights))]


class MdiError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__(f"{what}: {strerror(status)} ({status})")


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built; run `python -m paper_2505_18164_amd.build`")
        L = C.CDLL(LIB_PATH)
        vp, u32 = C.c_void_p, C.c_uint32
        L.mdi_partition_bytes.argtypes = [C.POINTER(MdiConfig), u32, u32, u32, C.POINTER(C.c_size_t)]
        L.mdi_partition_create.argtypes = [C.POINTER(MdiConfig), u32, u32, C.POINTER(MdiWeights), u32, vp, C.c_size_t,
                                           vp, C.POINTER(vp)]
        L.mdi_prefill.argtypes = [vp, u32, vp, u32, vp]
        L.mdi_prefill_chunk.argtypes = [vp, u32, vp, u32, vp]
        L.mdi_decode_step.argtypes = [vp, u32, vp, vp]
        L.mdi_decode_steps.argtypes = [vp, u32, C.POINTER(u32), C.POINTER(vp), C.POINTER(vp)]
        L.mdi_decode_batch.argtypes = [vp, u32, C.POINTER(u32), C.POINTER(vp), C.POINTER(vp)]
        L.mdi_sample_greedy.argtypes = [vp, u32, vp, vp, vp]
        L.mdi_sample_topk.argtypes = [vp, u32, vp, C.c_float, u32, C.c_uint64, u32, vp, vp]
        L.mdi_sample_topk_static.argtypes = [vp, u32, vp, C.c_float, u32, C.c_uint64, u32, vp, vp]
        L.mdi_sample_batch.argtypes = [vp, u32, C.POINTER(u32), C.POINTER(vp), C.c_float, u32, C.c_uint64, C.POINTER(u32), vp, vp]
        L.mdi_partition_sync.argtypes = [vp]
        L.mdi_seq_reset.argtypes = [vp, u32]
        L.mdi_seq_len.argtypes = [vp, u32, C.POINTER(u32)]
        L.mdi_step_bytes.argtypes = [vp, u32, C.c_int, C.POINTER(C.c_uint64)]
        L.mdi_time_kernel.argtypes = [vp, C.c_int, u32, C.POINTER(C.c_float), C.POINTER(C.c_uint64)]
        L.mdi_partition_info.argtypes = [vp, u32, C.POINTER(C.c_uint64)]
        L.mdi_partition_trace.argtypes = [vp, vp]
        L.mdi_partition_destroy.argtypes = [vp]
        L.mdi_partition_destroy.restype = None
        L.mdi_strerror.argtypes = [C.c_int]
        L.mdi_strerror.restype = C.c_char_p
        for name in EXPORTS[:18]:
            getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def strerror(status):
    return lib().mdi_strerror(int(status)).decode()


def make_config(cfg, max_seqs, kv_page_tokens=0, kv_pages=0, max_prefill=0, decode_path=0):
    """cfg: the dict produced by synth.* shape presets (plain integers and floats)."""
    c = MdiConfig()
    c.abi_version = MDI_ABI_VERSION
    for k in ("n_layer", "d_model", "n_head", "n_kv_head", "head_dim", "d_ff", "vocab", "max_ctx", "norm_kind",
              "mlp_kind", "pos_kind", "has_bias", "tie_embed", "dtype"):
        setattr(c, k, int(cfg[k]))
    c.norm_eps = float(cfg["norm_eps"])
    c.rope_base = float(cfg["rope_base"])
    c.max_seqs, c.kv_page_tokens, c.kv_pages, c.max_prefill = max_seqs, kv_page_tokens, kv_pages, max_prefill
    c.decode_path = decode_path
    return c


def partition_bytes(c, lo, hi, flags):
    n = C.c_size_t(0)
    st = lib().mdi_partition_bytes(C.byref(c), lo, hi, flags, C.byref(n))
    if st != MDI_OK:
        raise MdiError(st, "mdi_partition_bytes")
    return n.value


def torch_dtype(dtype):
    return torch.bfloat16 if dtype == MDI_BF16 else torch.float32


def to_device(a, dtype, device):
    """numpy fp32 array (values already representable in the storage dtype) -> device tensor."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)
    return t.to(torch_dtype(dtype)).contiguous() if dtype == MDI_BF16 else t.contiguous()


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(None)


class Partition:
    """One model chunk on the GPU (layers [lo, hi), optional embedding / output layers)."""

    def __init__(self, cfg, weights, lo, hi, has_embed=False, has_head=False, max_seqs=1, stream=None,
                 kv_page_tokens=0, kv_pages=0, max_prefill=0, decode_path=0, device="cuda:0"):
        """weights: {"layers": {L: {name: array}}, "wte": ...} with numpy arrays (see synth.make_weights)
        or tensors already on the device in storage dtype (vectors fp32)."""
        self.cfg = dict(cfg)
        self.lo, self.hi = lo, hi
        self.flags = (MDI_HAS_EMBED if has_embed else 0) | (MDI_HAS_HEAD if has_head else 0)
        self.device = torch.device(device)
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        self.c = make_config(cfg, max_seqs, kv_page_tokens, kv_pages, max_prefill, decode_path)
        self.dtype = int(cfg["dtype"])
        self.tdtype = torch_dtype(self.dtype)
        self.d, self.V = int(cfg["d_model"]), int(cfg["vocab"])
        self._h = C.c_void_p(None)
        nbytes = partition_bytes(self.c, lo, hi, self.flags)
        self.arena_bytes = nbytes
        self.arena = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        base = (self.arena.data_ptr() + 255) & ~255

        keep = []

        def dev(a, matrix):
            if a is None:
                return None
            if isinstance(a, torch.Tensor):
                t = a
            else:
                t = to_device(a, self.dtype if matrix else MDI_F32, self.device)
            keep.append(t)
            return t

        layers = (MdiLayerWeights * max(1, hi - lo))()
        mats = {"wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down"}
        for i, L in enumerate(range(lo, hi)):
            lw = weights["layers"][L]
            src = dict(lw)
            # names used by the input recipe -> header fields
            src["w_gate"] = lw.get("wg")
            src["w_up"] = lw.get("wu") if "wu" in lw else lw.get("w1")
            src["b_up"] = lw.get("b1")
            src["w_down"] = lw.get("wd") if "wd" in lw else lw.get("w2")
            src["b_down"] = lw.get("b2")
            for f in _LAYER_FIELDS:
                setattr(layers[i], f, _ptr(dev(src.get(f), f in mats)))
        w = MdiWeights()
        if has_embed or (has_head and cfg["tie_embed"]):
            w.wte = _ptr(dev(weights.get("wte"), True))
        if has_embed:
            w.wpe = _ptr(dev(weights.get("wpe"), True))
        if has_head:
            w.lnf_g = _ptr(dev(weights.get("lnf_g"), False))
            w.lnf_b = _ptr(dev(weights.get("lnf_b"), False))
            if not cfg["tie_embed"]:
                w.lm_head = _ptr(dev(weights.get("lm_head"), True))
        w.layers = C.cast(layers, C.POINTER(MdiLayerWeights))
        # the source tensors were produced on the current stream; the repacking runs on the partition's
        self.stream.wait_stream(torch.cuda.current_stream(self.device))
        with torch.cuda.stream(self.stream):
            st = lib().mdi_partition_create(C.byref(self.c), lo, hi, C.byref(w), self.flags, C.c_void_p(base), nbytes,
                                            C.c_void_p(self.stream.cuda_stream), C.byref(self._h))
        if st != MDI_OK:
            raise MdiError(st, "mdi_partition_create")
        self.stream.synchronize()     # the sources in `keep` may go now
        del keep

    # -- the four calls of the hot path ---------------------------------
    def prefill(self, seq, acts_in, acts_out=None):
        T = acts_in.shape[0]
        if acts_out is None:
            acts_out = torch.empty((T, self.d), dtype=self.tdtype, device=self.device)
        st = lib().mdi_prefill(self._h, seq, _ptr(acts_in), T, _ptr(acts_out))
        if st != MDI_OK:
            raise MdiError(st, "mdi_prefill")
        return acts_out

    def prefill_chunk(self, seq, acts_in, acts_out=None):
        """The next piece of a first visit: positions continue at the sample's current cache length."""
        T = acts_in.shape[0]
        if acts_out is None:
            acts_out = torch.empty((T, self.d), dtype=self.tdtype, device=self.device)
        st = lib().mdi_prefill_chunk(self._h, seq, _ptr(acts_in), T, _ptr(acts_out))
        if st != MDI_OK:
            raise MdiError(st, "mdi_prefill_chunk")
        return acts_out

    def decode_step(self, seq, act_in, act_out=None):
        if act_out is None:
            act_out = torch.empty((self.d,), dtype=self.tdtype, device=self.device)
        st = lib().mdi_decode_step(self._h, seq, _ptr(act_in), _ptr(act_out))
        if st != MDI_OK:
            raise MdiError(st, "mdi_decode_step")
        return act_out

    def decode_steps(self, seqs, acts_in, acts_out=None):
        """Later visits of several different samples, as mdi_decode_steps takes them (lists of equal length)."""
        n = len(seqs)
        if acts_out is None:
            acts_out = [torch.empty((self.d,), dtype=self.tdtype, device=self.device) for _ in range(n)]
        ids = (C.c_uint32 * n)(*seqs)
        ins = (C.c_void_p * n)(*[t.data_ptr() for t in acts_in])
        outs = (C.c_void_p * n)(*[t.data_ptr() for t in acts_out])
        st = lib().mdi_decode_steps(self._h, n, ids, ins, outs)
        if st != MDI_OK:
            raise MdiError(st, "mdi_decode_steps")
        return acts_out

    def decode_batch(self, seqs, acts_in, acts_out=None):
        """Later visits of several different samples with one pass over the weights (mdi_decode_batch)."""
        n = len(seqs)
        if acts_out is None:
            acts_out = [torch.empty((self.d,), dtype=self.tdtype, device=self.device) for _ in range(n)]
        ids = (C.c_uint32 * n)(*seqs)
        ins = (C.c_void_p * n)(*[t.data_ptr() for t in acts_in])
        outs = (C.c_void_p * n)(*[t.data_ptr() for t in acts_out])
        st = lib().mdi_decode_batch(self._h, n, ids, ins, outs)
        if st != MDI_OK:
            raise MdiError(st, "mdi_decode_batch")
        return acts_out

    def sample_greedy(self, seq, act_in, token_out=None, logits_out=None):
        if token_out is None:
            token_out = torch.empty((1,), dtype=torch.int32, device=self.device)
        st = lib().mdi_sample_greedy(self._h, seq, _ptr(act_in), _ptr(token_out), _ptr(logits_out))
        if st != MDI_OK:
            raise MdiError(st, "mdi_sample_greedy")
        return token_out

    def sample_topk(self, seq, act_in, temperature, top_k, seed, step, token_out=None, logits_out=None):
        if token_out is None:
            token_out = torch.empty((1,), dtype=torch.int32, device=self.device)
        st = lib().mdi_sample_topk(self._h, seq, _ptr(act_in), temperature, top_k, seed, step, _ptr(token_out), _ptr(logits_out))
        if st != MDI_OK:
            raise MdiError(st, "mdi_sample_topk")
        return token_out

    def sample_topk_static(self, seq, act_in, temperature, top_k, seed, step, token_out=None, logits_out=None):
        """mdi_sample_topk with the kernels' scratch in the library's fixed array; token_out must be passed by
        callers that may not allocate."""
        if token_out is None:
            token_out = torch.empty((1,), dtype=torch.int32, device=self.device)
        st = lib().mdi_sample_topk_static(self._h, seq, _ptr(act_in), temperature, top_k, seed, step, _ptr(token_out), _ptr(logits_out))
        if st != MDI_OK:
            raise MdiError(st, "mdi_sample_topk_static")
        return token_out

    def sample_batch(self, seqs, acts_in, temperature=1.0, top_k=1, seed=0, steps=None, tokens_out=None, logits_out=None):
        """Output layers of several samples with one pass over the vocabulary matrix (mdi_sample_batch)."""
        n = len(seqs)
        if tokens_out is None:
            tokens_out = torch.empty((n,), dtype=torch.int32, device=self.device)
        ids = (C.c_uint32 * n)(*seqs)
        ins = (C.c_void_p * n)(*[t.data_ptr() for t in acts_in])
        st_arr = (C.c_uint32 * n)(*steps) if steps is not None else None
        st = lib().mdi_sample_batch(self._h, n, ids, ins, temperature, top_k, seed, st_arr,
                                    _ptr(tokens_out), _ptr(logits_out))
        if st != MDI_OK:
            raise MdiError(st, "mdi_sample_batch")
        return tokens_out

    # -- bookkeeping --------------------------------------------------------
    def sync(self):
        st = lib().mdi_partition_sync(self._h)
        if st != MDI_OK:
            raise MdiError(st, "mdi_partition_sync")

    def seq_reset(self, seq):
        st = lib().mdi_seq_reset(self._h, seq)
        if st != MDI_OK:
            raise MdiError(st, "mdi_seq_reset")

    def seq_len(self, seq):
        n = C.c_uint32(0)
        st = lib().mdi_seq_len(self._h, seq, C.byref(n))
        if st != MDI_OK:
            raise MdiError(st, "mdi_seq_len")
        return n.value

    def step_bytes(self, ctx, head=False):
        n = C.c_uint64(0)
        st = lib().mdi_step_bytes(self._h, ctx, 1 if head else 0, C.byref(n))
        if st != MDI_OK:
            raise MdiError(st, "mdi_step_bytes")
        return n.value

    def time_kernel(self, which, reps):
        """(mean microseconds per launch, matrix bytes per launch) of one decode kernel kind."""
        us, nb = C.c_float(0), C.c_uint64(0)
        st = lib().mdi_time_kernel(self._h, which, reps, C.byref(us), C.byref(nb))
        if st != MDI_OK:
            raise MdiError(st, "mdi_time_kernel")
        return us.value, nb.value

    def trace(self, buf):
        """buf: int64 device tensor [2, workgroups, layers, 5, 8] (second half: second message of a launch) or None."""
        st = lib().mdi_partition_trace(self._h, _ptr(buf))
        if st != MDI_OK:
            raise MdiError(st, "mdi_partition_trace")
        self._trace = buf

    def info(self, what):
        v = C.c_uint64(0)
        st = lib().mdi_partition_info(self._h, what, C.byref(v))
        if st != MDI_OK:
            raise MdiError(st, "mdi_partition_info")
        return v.value

    def close(self):
        if self._h:
            lib().mdi_partition_destroy(self._h)
            self._h = C.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
