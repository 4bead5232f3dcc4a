"""The C-ABI library loads, exports every symbol the header declares, and rejects host-detectable
misuse without launching anything (no GPU needed: every call below fails validation on the host)."""
import ctypes
import os
import re

import pytest

from paper_2509_04377_amd import binding as pe

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = ctypes.c_void_p(0x1000)      # never dereferenced: validation fails first


def _declared():
    src = open(os.path.join(ROOT, "include", "pe.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(pe_[a-z_]+)\s*\(", src)))


def test_every_declared_symbol_is_exported():
    names = _declared()
    assert set(names) == set(pe.EXPORTS), (names, pe.EXPORTS)
    L = pe.lib()
    for n in names:
        assert getattr(L, n) is not None


def test_version_and_status_strings():
    assert pe.pe_version() >= 100
    seen = {pe.status_string(s) for s in (0, -1, -2, -3, -4)}
    assert len(seen) == 5 and pe.status_string(-99) == "unknown status"


def _desc(**kw):
    d = dict(dtype=pe.PE_BF16, num_seqs=4, num_kv_heads=8, num_q_heads=32, head_dim=128, block_size=16,
             max_blocks=128, num_phys_blocks=4096)
    d.update(kw)
    return pe.make_desc(**d)


@pytest.mark.parametrize("kw,want", [
    (dict(head_dim=96), pe.PE_ERR_UNSUPPORTED), (dict(block_size=8), pe.PE_ERR_UNSUPPORTED),
    (dict(dtype=7), pe.PE_ERR_UNSUPPORTED), (dict(num_q_heads=30), pe.PE_ERR_INVALID_ARG),
    (dict(num_q_heads=128), pe.PE_ERR_UNSUPPORTED), (dict(num_seqs=0), pe.PE_ERR_INVALID_ARG),
    (dict(max_blocks=0), pe.PE_ERR_INVALID_ARG), (dict(layout=5), pe.PE_ERR_UNSUPPORTED),
    (dict(decode_splits=-1), pe.PE_ERR_INVALID_ARG), (dict(decode_splits=257), pe.PE_ERR_INVALID_ARG),
    (dict(decode_flat_order=2), pe.PE_ERR_INVALID_ARG), (dict(decode_shape=823), pe.PE_ERR_UNSUPPORTED),
    (dict(decode_shape=424, head_dim=64), pe.PE_ERR_UNSUPPORTED),
    (dict(decode_shape=432, layout=1), pe.PE_ERR_UNSUPPORTED)])
def test_bad_descriptors(kw, want):
    d = _desc(**kw)
    L = pe.lib()
    assert L.pe_score_blocks(ctypes.byref(d), FAKE, FAKE, FAKE, FAKE, FAKE, None, 0, None) == want
    assert L.pe_evict_blocks(ctypes.byref(d), FAKE, FAKE, FAKE, 256, FAKE, FAKE, None) == want
    assert L.pe_paged_decode(ctypes.byref(d), FAKE, FAKE, FAKE, FAKE, FAKE, ctypes.c_float(0.1), FAKE, FAKE, 1 << 30,
                             None) == want
    assert pe.pe_workspace_bytes(pe.PE_OP_PAGED_DECODE, d) == 0 and pe.pe_decode_splits(d) == 0


def test_null_pointers_and_bad_budget():
    d = _desc()
    L = pe.lib()
    assert L.pe_score_blocks(ctypes.byref(d), None, FAKE, FAKE, FAKE, FAKE, None, 0, None) == pe.PE_ERR_INVALID_ARG
    assert L.pe_score_blocks(None, FAKE, FAKE, FAKE, FAKE, FAKE, None, 0, None) == pe.PE_ERR_INVALID_ARG
    assert L.pe_evict_blocks(ctypes.byref(d), FAKE, FAKE, None, 256, FAKE, FAKE, None) == pe.PE_ERR_INVALID_ARG
    assert L.pe_score_evict(ctypes.byref(d), FAKE, FAKE, FAKE, None, 256, None, FAKE, FAKE, None) == pe.PE_ERR_INVALID_ARG
    assert L.pe_score_evict(ctypes.byref(d), FAKE, FAKE, FAKE, FAKE, 256, None, None, FAKE, None) == pe.PE_ERR_INVALID_ARG
    for bad in (0, -16, 250):
        assert L.pe_evict_blocks(ctypes.byref(d), FAKE, FAKE, FAKE, bad, FAKE, FAKE, None) == pe.PE_ERR_INVALID_ARG
        assert L.pe_score_evict(ctypes.byref(d), FAKE, FAKE, FAKE, FAKE, bad, None, FAKE, FAKE, None) == pe.PE_ERR_INVALID_ARG
        assert L.pe_prefill_prune(ctypes.byref(d), FAKE, FAKE, FAKE, 1000, 1000, bad, FAKE, FAKE, FAKE, FAKE, None,
                                  FAKE, 1 << 30, None) == pe.PE_ERR_INVALID_ARG
    assert L.pe_paged_decode(ctypes.byref(d), FAKE, FAKE, FAKE, FAKE, FAKE, ctypes.c_float(float("nan")), FAKE, FAKE,
                             1 << 30, None) == pe.PE_ERR_INVALID_ARG
    assert L.pe_prefill_prune(ctypes.byref(d), FAKE, FAKE, FAKE, 1000, 2000, 256, FAKE, FAKE, FAKE, FAKE, None, FAKE,
                              1 << 30, None) == pe.PE_ERR_INVALID_ARG   # max_seqlen > total_tokens
    # the pruned row would not fit a table row: ceil(min(max_seqlen, C)/B) > max_blocks
    small = _desc(max_blocks=8)
    assert L.pe_prefill_prune(ctypes.byref(small), FAKE, FAKE, FAKE, 4000, 1000, 256, FAKE, FAKE, FAKE, FAKE, None,
                              FAKE, 1 << 30, None) == pe.PE_ERR_INVALID_ARG
    assert L.pe_prefill_prune(ctypes.byref(small), FAKE, FAKE, FAKE, 4000, 100, 256, FAKE, FAKE, FAKE, FAKE, None,
                              None, 0, None) == pe.PE_ERR_WORKSPACE      # 7 pages fit: the next check is reached
    misaligned = ctypes.c_void_p(0x1004)
    assert L.pe_score_blocks(ctypes.byref(d), misaligned, FAKE, FAKE, FAKE, FAKE, None, 0, None) == pe.PE_ERR_INVALID_ARG


def test_layers_call_host_checks():
    d = _desc()
    L = pe.lib()
    f = ctypes.c_float(0.1)
    args = lambda n, first=FAKE: (ctypes.byref(d), n, first, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 2, f,
                                  FAKE, FAKE, 1 << 30, None)
    assert L.pe_append_paged_decode_layers(*args(0)) == pe.PE_ERR_INVALID_ARG
    assert L.pe_append_paged_decode_layers(*args(3, None)) == pe.PE_ERR_INVALID_ARG
    # the per-layer checks apply too: seq_lens_out must not alias seq_lens (both FAKE here)
    assert L.pe_append_paged_decode_layers(*args(3)) == pe.PE_ERR_INVALID_ARG


def test_shared_layout_host_checks():
    d = _desc(layout=pe.PE_LAYOUT_SHARED)
    L = pe.lib()
    assert L.pe_score_evict(ctypes.byref(d), FAKE, FAKE, FAKE, FAKE, 256, None, FAKE, FAKE, None) == pe.PE_ERR_UNSUPPORTED
    # the shared prune keeps one more score row (the head mean) in its workspace
    per_head = pe.pe_workspace_bytes(pe.PE_OP_PREFILL_PRUNE, _desc(), 4000)
    assert pe.pe_workspace_bytes(pe.PE_OP_PREFILL_PRUNE, d, 4000) >= per_head + 4000 * 4


def test_workspace_checks():
    d = _desc()
    L = pe.lib()
    need = pe.pe_workspace_bytes(pe.PE_OP_PREFILL_PRUNE, d, 4 * 1000)
    assert need > 4 * 8 * 1000 * 4
    args = (ctypes.byref(d), FAKE, FAKE, FAKE, 4000, 1000, 256, FAKE, FAKE, FAKE, FAKE, None)
    assert L.pe_prefill_prune(*args, None, 0, None) == pe.PE_ERR_WORKSPACE
    assert L.pe_prefill_prune(*args, FAKE, need - 1, None) == pe.PE_ERR_WORKSPACE
    assert L.pe_prefill_prune(*args, ctypes.c_void_p(0x1010), need, None) == pe.PE_ERR_WORKSPACE   # misaligned
    # decode: the split count (and with it the workspace) follows the descriptor
    d1 = _desc(decode_splits=1)
    assert pe.pe_decode_splits(d1) == 1 and pe.pe_workspace_bytes(pe.PE_OP_PAGED_DECODE, d1) == 0
    d4 = _desc(decode_splits=4)
    w4 = pe.pe_workspace_bytes(pe.PE_OP_PAGED_DECODE, d4)
    assert pe.pe_decode_splits(d4) == 4 and w4 == 4 * 32 * 4 * (128 + 2) * 4
    assert L.pe_paged_decode(ctypes.byref(d4), FAKE, FAKE, FAKE, FAKE, FAKE, ctypes.c_float(0.1), FAKE, FAKE,
                             w4 - 1, None) == pe.PE_ERR_WORKSPACE
    # two descriptors in one process do not interfere, and the automatic choice covers the compute units
    assert pe.pe_decode_splits(d1) == 1 and pe.pe_decode_splits(d) >= 1
    assert pe.pe_workspace_bytes(pe.PE_OP_PAGED_DECODE, d) == pe.pe_decode_splits(d) * 4 * 32 * (128 + 2) * 4 * (
        pe.pe_decode_splits(d) > 1)
    assert pe.pe_workspace_bytes(pe.PE_OP_SCORE_BLOCKS, d) == 0 and pe.pe_workspace_bytes(pe.PE_OP_EVICT_BLOCKS, d) == 0


def test_static_scratch_rejects_oversized_partials():
    """pe_paged_decode_static refuses a shape whose split partials exceed its static array (host check)."""
    S, Hk, Hq, D = 64, 8, 64, 128
    desc = pe.make_desc(pe.PE_BF16, S, Hk, Hq, D, 16, 64, 4096, decode_splits=64)
    assert pe.pe_workspace_bytes(pe.PE_OP_PAGED_DECODE, desc) > pe.PE_STATIC_SCRATCH_BYTES
    fake = ctypes.c_void_p(0x1000)
    rc = pe.lib().pe_paged_decode_static(ctypes.byref(desc), fake, fake, fake, fake, fake, ctypes.c_float(0.1), fake, None)
    assert rc == pe.PE_ERR_WORKSPACE


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(pe, "_lib", None)
    monkeypatch.setattr(pe, "LIB_PATH", "/nonexistent/libpe.so")
    with pytest.raises(RuntimeError, match="not built"):
        pe.lib()
