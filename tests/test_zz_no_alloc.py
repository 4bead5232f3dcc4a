"""The allocation-free attention entry point (pe_paged_decode_static) against pe_paged_decode and the oracle.

Two calls in a row on the same GPU share the library's static partials array; the second call is smaller, so
anything the first left behind would show if the kernels did not rewrite every record they read.
"""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_2509_04377_amd import binding as pe

from _util import f32, i32, rel_err
from test_gpu_ops import make_paged

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _run_both(seed, lens, Hk, G, D, B, dtype, splits):
    k_pool, v_pool, table, sl = make_paged(seed, lens, Hk, D, B, dtype)
    g = torch.Generator().manual_seed(seed + 1)
    S, Hq = len(lens), Hk * G
    q = torch.randn((S, Hq, D), generator=g).to(dtype)
    want = oracle.paged_decode(f32(q), f32(k_pool), f32(v_pool), i32(table), i32(sl))
    desc = pe.make_desc(dtype, S, Hk, Hq, D, B, table.shape[2], k_pool.shape[0], decode_splits=splits)
    kd, vd, td, ld, qd = (x.to(DEV) for x in (k_pool, v_pool, table, sl, q))
    ws = pe.alloc_workspace(pe.PE_OP_PAGED_DECODE, desc)
    ref = torch.full((S, Hq, D), 7.0, dtype=dtype, device=DEV)
    pe.pe_paged_decode(desc, qd, kd, vd, td, ld, D ** -0.5, ref, ws)
    torch.cuda.synchronize()
    out = torch.full((S, Hq, D), -7.0, dtype=dtype, device=DEV)
    # through the C ABI directly: no workspace argument exists, nothing is allocated by the call
    L = pe.lib()
    rc = L.pe_paged_decode_static(ctypes.byref(desc), ctypes.c_void_p(qd.data_ptr()), ctypes.c_void_p(kd.data_ptr()),
                                  ctypes.c_void_p(vd.data_ptr()), ctypes.c_void_p(td.data_ptr()),
                                  ctypes.c_void_p(ld.data_ptr()), ctypes.c_float(D ** -0.5),
                                  ctypes.c_void_p(out.data_ptr()),
                                  ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == pe.PE_OK, pe.status_string(rc)
    torch.cuda.synchronize()
    return f32(out), f32(ref), want, sl


def test_static_scratch_matches_workspace_variant_twice():
    print("case no_alloc two calls", flush=True)
    tol = {torch.float32: 1e-5, torch.bfloat16: 2e-2}
    # first call: 7 splits over long ragged rows; second call: fewer, shorter rows and fewer splits
    for seed, lens, Hk, G, D, B, dtype, splits in (
            (901, [0, 1, 700, 1300, 2047, 33, 512, 4000], 4, 4, 128, 16, torch.bfloat16, 7),
            (902, [17, 300, 0], 2, 3, 64, 32, torch.float32, 3)):
        got, ref, want, sl = _run_both(seed, lens, Hk, G, D, B, dtype, splits)
        assert np.array_equal(got.view(np.int32), ref.view(np.int32)), "static and workspace variants differ"
        empty = [s for s, n in enumerate(lens) if n == 0]
        assert np.all(got[empty] == 0.0)
        keep = [s for s, n in enumerate(lens) if n > 0]
        e2, emax = rel_err(got[keep], want[keep])
        assert e2 <= tol[dtype] and emax <= tol[dtype], (seed, e2, emax)
