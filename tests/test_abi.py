"""The C-ABI library loads and exports every symbol include/mdi.h declares;
host-side argument checking works without a GPU (no compute calls here)."""
import ctypes as C
import os
import re

import pytest

from paper_2505_18164_amd import mdi as libmdi, synth as S

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(libmdi.LIB_PATH):
        from paper_2505_18164_amd.build import build
        build()
    return libmdi.lib()


def test_every_declared_symbol_is_exported(L):
    hdr = open(os.path.join(ROOT, "include", "mdi.h")).read()
    declared = re.findall(r"MDI_API\s+[\w\s\*]+?\b(mdi_\w+)\s*\(", hdr)
    assert sorted(declared) == sorted(libmdi.EXPORTS)
    for name in declared:
        assert getattr(L, name) is not None


def test_strerror(L):
    assert libmdi.strerror(0) == "ok"
    assert "context" in libmdi.strerror(libmdi.MDI_ERR_CTX)
    assert libmdi.strerror(-99) == "unknown status"


def test_config_struct_size_matches_header():
    # 22 four-byte fields
    assert C.sizeof(libmdi.MdiConfig) == 22 * 4
    assert C.sizeof(libmdi.MdiLayerWeights) == 17 * 8
    assert C.sizeof(libmdi.MdiWeights) == 6 * 8


def test_partition_bytes_accounts_for_weights_and_cache(L):
    cfg = S.llama2_7b()
    c = libmdi.make_config(cfg, max_seqs=8, kv_page_tokens=64)
    n = libmdi.partition_bytes(c, 8, 16, 0)
    weights = 8 * 202_375_168 * 2
    kv = 8 * 8 * 4096 * 2 * 4096 * 2
    assert weights + kv < n < (weights + kv) * 1.35
    # head-only partition: vocabulary projection + a little
    n_head = libmdi.partition_bytes(c, 32, 32, libmdi.MDI_HAS_HEAD)
    assert 32000 * 4096 * 2 < n_head < 32000 * 4096 * 2 * 1.01


def test_argument_validation(L):
    cfg = S.tiny()
    n = C.c_size_t(0)

    def status(lo, hi, flags, **over):
        c = libmdi.make_config(dict(cfg, **over), max_seqs=2)
        return L.mdi_partition_bytes(C.byref(c), lo, hi, flags, C.byref(n))

    assert status(0, 2, 1) == libmdi.MDI_OK
    assert status(1, 1, 0) == libmdi.MDI_ERR_ARG              # no blocks and no head
    assert status(2, 2, 2) == libmdi.MDI_OK                   # output portion without blocks (Sec. III-E)
    assert status(2, 2, 3) == libmdi.MDI_ERR_ARG
    assert status(1, 2, 1) == libmdi.MDI_ERR_ARG              # ids enter at layer 0
    assert status(0, 3, 0) == libmdi.MDI_ERR_ARG              # beyond n_layer
    assert status(0, 2, 0, head_dim=12) == libmdi.MDI_ERR_ARG
    assert status(0, 2, 0, d_model=30) == libmdi.MDI_ERR_ARG
    assert status(0, 2, 0, n_kv_head=3) == libmdi.MDI_ERR_ARG
    assert status(0, 2, 0, dtype=7) == libmdi.MDI_ERR_ARG
    c = libmdi.make_config(cfg, max_seqs=0)
    assert L.mdi_partition_bytes(C.byref(c), 0, 2, 0, C.byref(n)) == libmdi.MDI_ERR_ARG
    # position / page size is one multiplication in the decode kernel, exact while max_ctx * page size < 2^32
    c = libmdi.make_config(dict(cfg, max_ctx=1 << 20), max_seqs=1)
    c.kv_page_tokens = 1 << 11
    assert L.mdi_partition_bytes(C.byref(c), 0, 2, 0, C.byref(n)) == libmdi.MDI_OK
    c.kv_page_tokens = 1 << 12
    assert L.mdi_partition_bytes(C.byref(c), 0, 2, 0, C.byref(n)) == libmdi.MDI_ERR_ARG
    c = libmdi.make_config(cfg, max_seqs=1)
    c.abi_version = 99
    assert L.mdi_partition_bytes(C.byref(c), 0, 2, 0, C.byref(n)) == libmdi.MDI_ERR_ARG
    assert L.mdi_partition_bytes(None, 0, 2, 0, C.byref(n)) == libmdi.MDI_ERR_ARG
    # null handles are rejected, not dereferenced
    assert L.mdi_decode_step(None, 0, None, None) == libmdi.MDI_ERR_ARG
    assert L.mdi_prefill(None, 0, None, 1, None) == libmdi.MDI_ERR_ARG
    assert L.mdi_sample_greedy(None, 0, None, None, None) == libmdi.MDI_ERR_ARG
    assert L.mdi_seq_reset(None, 0) == libmdi.MDI_ERR_ARG
    L.mdi_partition_destroy(None)


def test_reciprocal_page_division_is_exact_below_the_checked_bound():
    # the decode kernel computes position // page_size as the high word of position * (0xFFFFFFFF // page_size + 1)
    # for page sizes that are not powers of two; exhaustive near the boundaries, random elsewhere
    import numpy as np
    rng = np.random.default_rng(0)
    for pt in [3, 5, 6, 7, 12, 24, 48, 100, 255, 1000, 4097]:
        magic = np.uint64(0xFFFFFFFF // pt + 1)
        top = (1 << 32) // pt                                   # positions with position * pt < 2^32
        pos = np.unique(np.concatenate([np.arange(0, min(top, 5000)), np.arange(max(0, top - 5000), top),
                                        rng.integers(0, top, 20000), (np.arange(1, 3000) * pt - 1) % top,
                                        (np.arange(1, 3000) * pt) % top])).astype(np.uint64)
        assert np.array_equal((pos * magic) >> np.uint64(32), pos // np.uint64(pt)), pt
