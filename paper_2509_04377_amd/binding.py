"""Python front end of libpe.so: argument marshalling only.

Every function below has the name and argument order of the C-ABI entry point it calls
(include/pe.h), takes torch tensors that already live on the GPU, and enqueues the library's HIP
kernels on torch's current stream.  No step of the path is computed here or on the CPU and no
control flow of the method lives here (the host-side sequencing of calls is engine.py); if libpe.so
has not been built, the first call raises.
"""
import ctypes
import os
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpe.so")

PE_OK = 0
PE_ERR_INVALID_ARG, PE_ERR_UNSUPPORTED, PE_ERR_WORKSPACE, PE_ERR_HIP = -1, -2, -3, -4
PE_F32, PE_BF16 = 0, 1
PE_OP_SCORE_BLOCKS, PE_OP_PREFILL_PRUNE, PE_OP_EVICT_BLOCKS, PE_OP_PAGED_DECODE = 0, 1, 2, 3
PE_OP_APPEND_PAGED_DECODE = 4
PE_STATIC_SCRATCH_BYTES = 8 * 1024 * 1024

EXPORTS = ["pe_workspace_bytes", "pe_status_string", "pe_version", "pe_decode_splits",
           "pe_score_blocks", "pe_prefill_prune", "pe_evict_blocks", "pe_paged_decode", "pe_append_kv",
           "pe_append_paged_decode", "pe_score_recent_blocks", "pe_evict_blocks_cached", "pe_evict_blocks_ex", "pe_score_evict",
           "pe_score_triggered_blocks", "pe_paged_decode_static", "pe_append_paged_decode_layers"]


class pe_cache_desc(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("num_seqs", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32),
                ("num_q_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("block_size", ctypes.c_int32),
                ("max_blocks", ctypes.c_int32), ("num_phys_blocks", ctypes.c_int64), ("layout", ctypes.c_int32),
                ("decode_splits", ctypes.c_int32), ("decode_shape", ctypes.c_int32),
                ("decode_flat_order", ctypes.c_int32)]


class pe_evict_opts(ctypes.Structure):
    _fields_ = [("policy", ctypes.c_int32), ("protect_first", ctypes.c_int32), ("protect_last", ctypes.c_int32),
                ("share_heads", ctypes.c_int32), ("cached_scores", ctypes.c_int32)]


PE_POLICY_LOWEST_SCORE, PE_POLICY_OLDEST = 0, 1
PE_LAYOUT_PER_HEAD, PE_LAYOUT_SHARED = 0, 1


class PeError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (where, status_string(status), status))


_lib = None


def lib():
    """The loaded libpe.so.  Raises if it is missing: there is no fallback path."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libpe.so is not built (%s): run `python -c 'import __graft_entry__ as g; g.build()'` "
                               "or `python paper_2509_04377_amd/build.py`" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
        dp = ctypes.POINTER(pe_cache_desc)
        L.pe_workspace_bytes.restype = sz
        L.pe_workspace_bytes.argtypes = [ctypes.c_int, dp, i64]
        L.pe_status_string.restype = ctypes.c_char_p
        L.pe_status_string.argtypes = [ctypes.c_int]
        L.pe_version.restype = ctypes.c_int
        L.pe_version.argtypes = []
        L.pe_decode_splits.restype = ctypes.c_int
        L.pe_decode_splits.argtypes = [dp]
        L.pe_score_blocks.restype = ctypes.c_int
        L.pe_score_blocks.argtypes = [dp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.pe_prefill_prune.restype = ctypes.c_int
        L.pe_prefill_prune.argtypes = [dp, vp, vp, vp, i64, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp]
        L.pe_evict_blocks.restype = ctypes.c_int
        L.pe_evict_blocks.argtypes = [dp, vp, vp, vp, i32, vp, vp, vp]
        L.pe_score_triggered_blocks.restype = ctypes.c_int
        L.pe_score_triggered_blocks.argtypes = [dp, vp, vp, vp, vp, i32, vp, vp]
        L.pe_score_evict.restype = ctypes.c_int
        L.pe_score_evict.argtypes = [dp, vp, vp, vp, vp, i32, vp, vp, vp, vp]
        L.pe_paged_decode.restype = ctypes.c_int
        L.pe_paged_decode.argtypes = [dp, vp, vp, vp, vp, vp, ctypes.c_float, vp, vp, sz, vp]
        L.pe_paged_decode_static.restype = ctypes.c_int
        L.pe_paged_decode_static.argtypes = [dp, vp, vp, vp, vp, vp, ctypes.c_float, vp, vp]
        L.pe_append_kv.restype = ctypes.c_int
        L.pe_append_kv.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp]
        L.pe_append_paged_decode.restype = ctypes.c_int
        L.pe_append_paged_decode.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, ctypes.c_float, vp, vp, sz,
                                             vp]
        L.pe_append_paged_decode_layers.restype = ctypes.c_int
        L.pe_append_paged_decode_layers.argtypes = [dp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, ctypes.c_float,
                                                    vp, vp, sz, vp]
        L.pe_evict_blocks_ex.restype = ctypes.c_int
        L.pe_evict_blocks_ex.argtypes = [dp, ctypes.POINTER(pe_evict_opts), vp, vp, vp, i32, vp, vp, vp]
        L.pe_score_recent_blocks.restype = ctypes.c_int
        L.pe_score_recent_blocks.argtypes = [dp, vp, vp, vp, vp, i32, vp, vp]
        L.pe_evict_blocks_cached.restype = ctypes.c_int
        L.pe_evict_blocks_cached.argtypes = [dp, vp, vp, vp, i32, vp, vp, vp]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().pe_status_string(int(status)).decode()


def pe_version() -> int:
    return int(lib().pe_version())


def pe_decode_splits(desc: pe_cache_desc) -> int:
    return int(lib().pe_decode_splits(ctypes.byref(desc)))


def make_desc(dtype, num_seqs, num_kv_heads, num_q_heads, head_dim, block_size, max_blocks, num_phys_blocks,
              layout=0, decode_splits=0, decode_shape=0, decode_flat_order=0):
    code = {torch.float32: PE_F32, torch.bfloat16: PE_BF16}.get(dtype, dtype if isinstance(dtype, int) else -1)
    return pe_cache_desc(int(code), int(num_seqs), int(num_kv_heads), int(num_q_heads), int(head_dim),
                         int(block_size), int(max_blocks), int(num_phys_blocks), int(layout), int(decode_splits),
                         int(decode_shape), int(decode_flat_order))


def check(status, where):
    if status != PE_OK:
        raise PeError(status, where)


def ptr(t, name, dtype=None, optional=False):
    if t is None:
        if optional:
            return None
        raise PeError(PE_ERR_INVALID_ARG, name + " is None")
    if not t.is_cuda:
        raise ValueError(name + " must be a GPU tensor")
    if not t.is_contiguous():
        raise ValueError(name + " must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise ValueError("%s must be %s, got %s" % (name, dtype, t.dtype))
    return ctypes.c_void_p(t.data_ptr())


def stream_arg():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def ws_args(workspace):
    if workspace is None:
        return None, 0
    return ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size()


def pe_workspace_bytes(op: int, desc: pe_cache_desc, total_tokens: int = 0) -> int:
    return int(lib().pe_workspace_bytes(int(op), ctypes.byref(desc), int(total_tokens)))


def alloc_workspace(op: int, desc: pe_cache_desc, total_tokens: int = 0, device="cuda"):
    """A torch buffer of the size pe_workspace_bytes() asks for (None if the op needs none)."""
    n = pe_workspace_bytes(op, desc, total_tokens)
    if n == 0:
        return None
    return torch.empty((n + 255) // 256 * 256, dtype=torch.uint8, device=device)


def pe_score_blocks(desc, k_pool, v_pool, block_table, seq_lens, scores_out, workspace=None):
    wp, wn = ws_args(workspace)
    check(lib().pe_score_blocks(ctypes.byref(desc), ptr(k_pool, "k_pool"), ptr(v_pool, "v_pool"),
                                 ptr(block_table, "block_table", torch.int32), ptr(seq_lens, "seq_lens", torch.int32),
                                 ptr(scores_out, "scores_out", torch.float32), wp, wn, stream_arg()), "pe_score_blocks")


def pe_prefill_prune(desc, k_in, v_in, cu_seqlens, total_tokens, max_seqlen, budget_tokens, k_pool, v_pool,
                     block_table, seq_lens_out, kept_idx_out, workspace):
    wp, wn = ws_args(workspace)
    check(lib().pe_prefill_prune(ctypes.byref(desc), ptr(k_in, "k_in"), ptr(v_in, "v_in"),
                                  ptr(cu_seqlens, "cu_seqlens", torch.int32), int(total_tokens), int(max_seqlen),
                                  int(budget_tokens), ptr(k_pool, "k_pool"), ptr(v_pool, "v_pool"),
                                  ptr(block_table, "block_table", torch.int32),
                                  ptr(seq_lens_out, "seq_lens_out", torch.int32),
                                  ptr(kept_idx_out, "kept_idx_out", torch.int32, optional=True), wp, wn, stream_arg()),
           "pe_prefill_prune")


def pe_evict_blocks(desc, scores, block_table, seq_lens, budget_tokens, evicted_logical_out, freed_phys_out):
    check(lib().pe_evict_blocks(ctypes.byref(desc), ptr(scores, "scores", torch.float32),
                                 ptr(block_table, "block_table", torch.int32), ptr(seq_lens, "seq_lens", torch.int32),
                                 int(budget_tokens), ptr(evicted_logical_out, "evicted_logical_out", torch.int32),
                                 ptr(freed_phys_out, "freed_phys_out", torch.int32), stream_arg()), "pe_evict_blocks")


def pe_score_triggered_blocks(desc, k_pool, v_pool, block_table, seq_lens, budget_tokens, scores_inout):
    check(lib().pe_score_triggered_blocks(ctypes.byref(desc), ptr(k_pool, "k_pool"), ptr(v_pool, "v_pool"),
                                           ptr(block_table, "block_table", torch.int32),
                                           ptr(seq_lens, "seq_lens", torch.int32), int(budget_tokens),
                                           ptr(scores_inout, "scores_inout", torch.float32), stream_arg()),
           "pe_score_triggered_blocks")


def pe_score_evict(desc, k_pool, v_pool, block_table, seq_lens, budget_tokens, scores_out, evicted_logical_out,
                   freed_phys_out):
    check(lib().pe_score_evict(ctypes.byref(desc), ptr(k_pool, "k_pool"), ptr(v_pool, "v_pool"),
                                ptr(block_table, "block_table", torch.int32), ptr(seq_lens, "seq_lens", torch.int32),
                                int(budget_tokens), ptr(scores_out, "scores_out", torch.float32, optional=True),
                                ptr(evicted_logical_out, "evicted_logical_out", torch.int32),
                                ptr(freed_phys_out, "freed_phys_out", torch.int32), stream_arg()), "pe_score_evict")


def pe_score_recent_blocks(desc, k_pool, v_pool, block_table, seq_lens, recent, scores_inout):
    check(lib().pe_score_recent_blocks(ctypes.byref(desc), ptr(k_pool, "k_pool"), ptr(v_pool, "v_pool"),
                                        ptr(block_table, "block_table", torch.int32),
                                        ptr(seq_lens, "seq_lens", torch.int32), int(recent),
                                        ptr(scores_inout, "scores_inout", torch.float32), stream_arg()),
           "pe_score_recent_blocks")


def pe_evict_blocks_cached(desc, scores_inout, block_table, seq_lens, budget_tokens, evicted_logical_out,
                           freed_phys_out):
    check(lib().pe_evict_blocks_cached(ctypes.byref(desc), ptr(scores_inout, "scores_inout", torch.float32),
                                        ptr(block_table, "block_table", torch.int32),
                                        ptr(seq_lens, "seq_lens", torch.int32), int(budget_tokens),
                                        ptr(evicted_logical_out, "evicted_logical_out", torch.int32),
                                        ptr(freed_phys_out, "freed_phys_out", torch.int32), stream_arg()),
           "pe_evict_blocks_cached")


def pe_evict_blocks_ex(desc, opts, scores, block_table, seq_lens, budget_tokens, evicted_logical_out, freed_phys_out):
    check(lib().pe_evict_blocks_ex(ctypes.byref(desc), ctypes.byref(opts),
                                    ptr(scores, "scores", torch.float32, optional=True),
                                    ptr(block_table, "block_table", torch.int32),
                                    ptr(seq_lens, "seq_lens", torch.int32), int(budget_tokens),
                                    ptr(evicted_logical_out, "evicted_logical_out", torch.int32),
                                    ptr(freed_phys_out, "freed_phys_out", torch.int32), stream_arg()),
           "pe_evict_blocks_ex")


def pe_paged_decode(desc, q, k_pool, v_pool, block_table, seq_lens, softmax_scale, out, workspace=None):
    wp, wn = ws_args(workspace)
    check(lib().pe_paged_decode(ctypes.byref(desc), ptr(q, "q"), ptr(k_pool, "k_pool"), ptr(v_pool, "v_pool"),
                                 ptr(block_table, "block_table", torch.int32), ptr(seq_lens, "seq_lens", torch.int32),
                                 ctypes.c_float(softmax_scale), ptr(out, "out"), wp, wn, stream_arg()), "pe_paged_decode")


def pe_paged_decode_static(desc, q, k_pool, v_pool, block_table, seq_lens, softmax_scale, out):
    check(lib().pe_paged_decode_static(ctypes.byref(desc), ptr(q, "q"), ptr(k_pool, "k_pool"), ptr(v_pool, "v_pool"),
                                       ptr(block_table, "block_table", torch.int32),
                                       ptr(seq_lens, "seq_lens", torch.int32), ctypes.c_float(softmax_scale),
                                       ptr(out, "out"), stream_arg()), "pe_paged_decode_static")


def pe_append_kv(desc, new_k, new_v, k_pool, v_pool, block_table, seq_lens, freed_phys, spare, spare_used):
    check(lib().pe_append_kv(ctypes.byref(desc), ptr(new_k, "new_k"), ptr(new_v, "new_v"), ptr(k_pool, "k_pool"),
                              ptr(v_pool, "v_pool"), ptr(block_table, "block_table", torch.int32),
                              ptr(seq_lens, "seq_lens", torch.int32), ptr(freed_phys, "freed_phys", torch.int32),
                              ptr(spare, "spare", torch.int32), ptr(spare_used, "spare_used", torch.int32),
                              int(spare.shape[-1]), stream_arg()), "pe_append_kv")


def pe_append_paged_decode(desc, new_k, new_v, q, k_pool, v_pool, block_table, seq_lens, seq_lens_out, freed_phys, spare,
                           spare_used, softmax_scale, out, workspace=None):
    wp, wn = ws_args(workspace)
    check(lib().pe_append_paged_decode(ctypes.byref(desc), ptr(new_k, "new_k"), ptr(new_v, "new_v"), ptr(q, "q"),
                                        ptr(k_pool, "k_pool"), ptr(v_pool, "v_pool"),
                                        ptr(block_table, "block_table", torch.int32),
                                        ptr(seq_lens, "seq_lens", torch.int32),
                                        ptr(seq_lens_out, "seq_lens_out", torch.int32),
                                        ptr(freed_phys, "freed_phys", torch.int32), ptr(spare, "spare", torch.int32),
                                        ptr(spare_used, "spare_used", torch.int32), int(spare.shape[-1]),
                                        ctypes.c_float(softmax_scale), ptr(out, "out"), wp, wn, stream_arg()),
           "pe_append_paged_decode")


def pe_append_paged_decode_layers(desc, num_layers, new_k, new_v, q, k_pool, v_pool, block_table, seq_lens, seq_lens_out,
                                  freed_phys, spare, spare_used, softmax_scale, out, workspace=None):
    wp, wn = ws_args(workspace)
    check(lib().pe_append_paged_decode_layers(ctypes.byref(desc), int(num_layers), ptr(new_k, "new_k"), ptr(new_v, "new_v"),
                                              ptr(q, "q"), ptr(k_pool, "k_pool"), ptr(v_pool, "v_pool"),
                                              ptr(block_table, "block_table", torch.int32),
                                              ptr(seq_lens, "seq_lens", torch.int32),
                                              ptr(seq_lens_out, "seq_lens_out", torch.int32),
                                              ptr(freed_phys, "freed_phys", torch.int32), ptr(spare, "spare", torch.int32),
                                              ptr(spare_used, "spare_used", torch.int32), int(spare.shape[-1]),
                                              ctypes.c_float(softmax_scale), ptr(out, "out"), wp, wn, stream_arg()),
          "pe_append_paged_decode_layers")
