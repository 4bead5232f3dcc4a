"""Python front end of libpe.so: argument marshalling only.

Every function below has the name and argument order of the C-ABI entry point it calls
(include/pe.h), takes torch tensors that already live on the GPU, and enqueues the library's HIP
kernels on torch's current stream.  No step of the path is computed here or on the CPU; if
libpe.so has not been built, the first call raises.
"""
import ctypes
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpe.so")

PE_OK = 0
PE_ERR_INVALID_ARG, PE_ERR_UNSUPPORTED, PE_ERR_WORKSPACE, PE_ERR_HIP = -1, -2, -3, -4
PE_F32, PE_BF16 = 0, 1
PE_OP_SCORE_BLOCKS, PE_OP_PREFILL_PRUNE, PE_OP_EVICT_BLOCKS, PE_OP_PAGED_DECODE = 0, 1, 2, 3
PE_OP_APPEND_PAGED_DECODE = 4
PE_OPT_DECODE_SPLITS, PE_OPT_DECODE_XCD_MAP, PE_OPT_DECODE_WAVES, PE_OPT_DECODE_DEPTH = 0, 1, 2, 3
PE_OPT_DECODE_LOADS = 4

EXPORTS = ["pe_workspace_bytes", "pe_status_string", "pe_version", "pe_set_option", "pe_get_option",
           "pe_score_blocks", "pe_prefill_prune", "pe_evict_blocks", "pe_paged_decode", "pe_append_kv",
           "pe_append_paged_decode", "pe_score_recent_blocks", "pe_evict_blocks_cached", "pe_evict_blocks_ex", "pe_score_evict",
           "pe_score_triggered_blocks"]


class pe_cache_desc(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("num_seqs", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32),
                ("num_q_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("block_size", ctypes.c_int32),
                ("max_blocks", ctypes.c_int32), ("num_phys_blocks", ctypes.c_int64), ("layout", ctypes.c_int32)]


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
        L.pe_set_option.restype = ctypes.c_int
        L.pe_set_option.argtypes = [ctypes.c_int, ctypes.c_int]
        L.pe_get_option.restype = ctypes.c_int
        L.pe_get_option.argtypes = [ctypes.c_int]
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
        L.pe_append_kv.restype = ctypes.c_int
        L.pe_append_kv.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp]
        L.pe_append_paged_decode.restype = ctypes.c_int
        L.pe_append_paged_decode.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, ctypes.c_float, vp, vp, sz,
                                             vp]
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


def pe_set_option(key: int, value: int) -> None:
    _check(lib().pe_set_option(int(key), int(value)), "pe_set_option")


def pe_get_option(key: int) -> int:
    return int(lib().pe_get_option(int(key)))


def make_desc(dtype, num_seqs, num_kv_heads, num_q_heads, head_dim, block_size, max_blocks, num_phys_blocks,
              layout=0):
    code = {torch.float32: PE_F32, torch.bfloat16: PE_BF16}.get(dtype, dtype if isinstance(dtype, int) else -1)
    return pe_cache_desc(int(code), int(num_seqs), int(num_kv_heads), int(num_q_heads), int(head_dim),
                         int(block_size), int(max_blocks), int(num_phys_blocks), int(layout))


def _check(status, where):
    if status != PE_OK:
        raise PeError(status, where)


class _HostOnly:
    """While active, the kernel-launching wrappers below return without calling the library, so a driver can
    advance its host-side bookkeeping for a step whose launches are replayed from a captured HIP graph."""
    active = False

    def __enter__(self):
        _HostOnly.active = True

    def __exit__(self, *exc):
        _HostOnly.active = False


def host_only():
    return _HostOnly()


def _ptr(t, name, dtype=None, optional=False):
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


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ws(workspace):
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
    if _HostOnly.active:
        return
    wp, wn = _ws(workspace)
    _check(lib().pe_score_blocks(ctypes.byref(desc), _ptr(k_pool, "k_pool"), _ptr(v_pool, "v_pool"),
                                 _ptr(block_table, "block_table", torch.int32), _ptr(seq_lens, "seq_lens", torch.int32),
                                 _ptr(scores_out, "scores_out", torch.float32), wp, wn, _stream()), "pe_score_blocks")


def pe_prefill_prune(desc, k_in, v_in, cu_seqlens, total_tokens, max_seqlen, budget_tokens, k_pool, v_pool,
                     block_table, seq_lens_out, kept_idx_out, workspace):
    if _HostOnly.active:
        return
    wp, wn = _ws(workspace)
    _check(lib().pe_prefill_prune(ctypes.byref(desc), _ptr(k_in, "k_in"), _ptr(v_in, "v_in"),
                                  _ptr(cu_seqlens, "cu_seqlens", torch.int32), int(total_tokens), int(max_seqlen),
                                  int(budget_tokens), _ptr(k_pool, "k_pool"), _ptr(v_pool, "v_pool"),
                                  _ptr(block_table, "block_table", torch.int32),
                                  _ptr(seq_lens_out, "seq_lens_out", torch.int32),
                                  _ptr(kept_idx_out, "kept_idx_out", torch.int32, optional=True), wp, wn, _stream()),
           "pe_prefill_prune")


def pe_evict_blocks(desc, scores, block_table, seq_lens, budget_tokens, evicted_logical_out, freed_phys_out):
    if _HostOnly.active:
        return
    _check(lib().pe_evict_blocks(ctypes.byref(desc), _ptr(scores, "scores", torch.float32),
                                 _ptr(block_table, "block_table", torch.int32), _ptr(seq_lens, "seq_lens", torch.int32),
                                 int(budget_tokens), _ptr(evicted_logical_out, "evicted_logical_out", torch.int32),
                                 _ptr(freed_phys_out, "freed_phys_out", torch.int32), _stream()), "pe_evict_blocks")


def pe_score_triggered_blocks(desc, k_pool, v_pool, block_table, seq_lens, budget_tokens, scores_inout):
    if _HostOnly.active:
        return
    _check(lib().pe_score_triggered_blocks(ctypes.byref(desc), _ptr(k_pool, "k_pool"), _ptr(v_pool, "v_pool"),
                                           _ptr(block_table, "block_table", torch.int32),
                                           _ptr(seq_lens, "seq_lens", torch.int32), int(budget_tokens),
                                           _ptr(scores_inout, "scores_inout", torch.float32), _stream()),
           "pe_score_triggered_blocks")


def pe_score_evict(desc, k_pool, v_pool, block_table, seq_lens, budget_tokens, scores_out, evicted_logical_out,
                   freed_phys_out):
    if _HostOnly.active:
        return
    _check(lib().pe_score_evict(ctypes.byref(desc), _ptr(k_pool, "k_pool"), _ptr(v_pool, "v_pool"),
                                _ptr(block_table, "block_table", torch.int32), _ptr(seq_lens, "seq_lens", torch.int32),
                                int(budget_tokens), _ptr(scores_out, "scores_out", torch.float32, optional=True),
                                _ptr(evicted_logical_out, "evicted_logical_out", torch.int32),
                                _ptr(freed_phys_out, "freed_phys_out", torch.int32), _stream()), "pe_score_evict")


def pe_score_recent_blocks(desc, k_pool, v_pool, block_table, seq_lens, recent, scores_inout):
    if _HostOnly.active:
        return
    _check(lib().pe_score_recent_blocks(ctypes.byref(desc), _ptr(k_pool, "k_pool"), _ptr(v_pool, "v_pool"),
                                        _ptr(block_table, "block_table", torch.int32),
                                        _ptr(seq_lens, "seq_lens", torch.int32), int(recent),
                                        _ptr(scores_inout, "scores_inout", torch.float32), _stream()),
           "pe_score_recent_blocks")


def pe_evict_blocks_cached(desc, scores_inout, block_table, seq_lens, budget_tokens, evicted_logical_out,
                           freed_phys_out):
    if _HostOnly.active:
        return
    _check(lib().pe_evict_blocks_cached(ctypes.byref(desc), _ptr(scores_inout, "scores_inout", torch.float32),
                                        _ptr(block_table, "block_table", torch.int32),
                                        _ptr(seq_lens, "seq_lens", torch.int32), int(budget_tokens),
                                        _ptr(evicted_logical_out, "evicted_logical_out", torch.int32),
                                        _ptr(freed_phys_out, "freed_phys_out", torch.int32), _stream()),
           "pe_evict_blocks_cached")


def pe_evict_blocks_ex(desc, opts, scores, block_table, seq_lens, budget_tokens, evicted_logical_out, freed_phys_out):
    if _HostOnly.active:
        return
    _check(lib().pe_evict_blocks_ex(ctypes.byref(desc), ctypes.byref(opts),
                                    _ptr(scores, "scores", torch.float32, optional=True),
                                    _ptr(block_table, "block_table", torch.int32),
                                    _ptr(seq_lens, "seq_lens", torch.int32), int(budget_tokens),
                                    _ptr(evicted_logical_out, "evicted_logical_out", torch.int32),
                                    _ptr(freed_phys_out, "freed_phys_out", torch.int32), _stream()),
           "pe_evict_blocks_ex")


def pe_paged_decode(desc, q, k_pool, v_pool, block_table, seq_lens, softmax_scale, out, workspace=None):
    if _HostOnly.active:
        return
    wp, wn = _ws(workspace)
    _check(lib().pe_paged_decode(ctypes.byref(desc), _ptr(q, "q"), _ptr(k_pool, "k_pool"), _ptr(v_pool, "v_pool"),
                                 _ptr(block_table, "block_table", torch.int32), _ptr(seq_lens, "seq_lens", torch.int32),
                                 ctypes.c_float(softmax_scale), _ptr(out, "out"), wp, wn, _stream()), "pe_paged_decode")


def pe_append_kv(desc, new_k, new_v, k_pool, v_pool, block_table, seq_lens, freed_phys, spare, spare_used):
    if _HostOnly.active:
        return
    _check(lib().pe_append_kv(ctypes.byref(desc), _ptr(new_k, "new_k"), _ptr(new_v, "new_v"), _ptr(k_pool, "k_pool"),
                              _ptr(v_pool, "v_pool"), _ptr(block_table, "block_table", torch.int32),
                              _ptr(seq_lens, "seq_lens", torch.int32), _ptr(freed_phys, "freed_phys", torch.int32),
                              _ptr(spare, "spare", torch.int32), _ptr(spare_used, "spare_used", torch.int32),
                              int(spare.shape[-1]), _stream()), "pe_append_kv")


def pe_append_paged_decode(desc, new_k, new_v, q, k_pool, v_pool, block_table, seq_lens, seq_lens_out, freed_phys, spare,
                           spare_used, softmax_scale, out, workspace=None):
    if _HostOnly.active:
        return
    wp, wn = _ws(workspace)
    _check(lib().pe_append_paged_decode(ctypes.byref(desc), _ptr(new_k, "new_k"), _ptr(new_v, "new_v"), _ptr(q, "q"),
                                        _ptr(k_pool, "k_pool"), _ptr(v_pool, "v_pool"),
                                        _ptr(block_table, "block_table", torch.int32),
                                        _ptr(seq_lens, "seq_lens", torch.int32),
                                        _ptr(seq_lens_out, "seq_lens_out", torch.int32),
                                        _ptr(freed_phys, "freed_phys", torch.int32), _ptr(spare, "spare", torch.int32),
                                        _ptr(spare_used, "spare_used", torch.int32), int(spare.shape[-1]),
                                        ctypes.c_float(softmax_scale), _ptr(out, "out"), wp, wn, _stream()),
           "pe_append_paged_decode")


@dataclass
class PagedCache:
    """Device-side state of one paged KV cache (one layer, or several layers folded into num_seqs).

    Owns nothing but tensors; every operation is a C-ABI call."""
    desc: pe_cache_desc
    k_pool: torch.Tensor       # [P, B, D]
    v_pool: torch.Tensor       # [P, B, D]
    block_table: torch.Tensor  # [S, Hk, max_blocks] int32
    seq_lens: torch.Tensor     # [S] int32
    spare: torch.Tensor        # [S, Hk, n_spare] int32
    spare_used: torch.Tensor   # [S, Hk] int32
    freed_phys: torch.Tensor   # [S, Hk] int32
    evicted_logical: torch.Tensor  # [S, Hk] int32
    scores: torch.Tensor       # [S, Hk, max_blocks] fp32
    budget: int
    decode_ws: torch.Tensor = None
    host_lens: list = None     # host mirror of seq_lens (pure integer bookkeeping, never read back)
    seq_lens_alt: torch.Tensor = None  # second lengths array for pe_append_paged_decode (swapped after each call)
    cached_scores: bool = False    # keep `scores` alive across steps and score only newly filled pages
    host_scored: list = None       # per sequence: full pages whose score is in `scores` (host bookkeeping)
    evict_opts: pe_evict_opts = None  # eviction variant (policy, protected pages, shared heads); None = Alg. 3
    fused_evict: bool = False  # score + evict of a trigger step in one launch (pe_score_evict)

    @staticmethod
    def create(dtype, num_seqs, num_kv_heads, num_q_heads, head_dim, block_size, layout, budget, device="cuda",
               k_pool=None, v_pool=None, shared=False):
        """`layout`: block table, spare lists and pool size (synth.page_layout).  shared=True builds the
        head-shared cache (PE_LAYOUT_SHARED): `layout` then describes ONE row per sequence (a layout made for a
        single KV head), pools are [P, B, Hk, D] and the per-row arrays lose their head dimension."""
        desc = make_desc(dtype, num_seqs, num_kv_heads, num_q_heads, head_dim, block_size, layout.max_blocks,
                         layout.num_phys_blocks, PE_LAYOUT_SHARED if shared else PE_LAYOUT_PER_HEAD)
        table, spare = layout.block_table, layout.spare
        if shared:
            assert table.shape[1] == 1, "a shared cache takes a layout with one row per sequence"
            table, spare = table[:, 0], spare[:, 0]
            shape = (layout.num_phys_blocks, block_size, num_kv_heads, head_dim)
            per_row = (num_seqs,)
        else:
            shape = (layout.num_phys_blocks, block_size, head_dim)
            per_row = (num_seqs, num_kv_heads)
        if k_pool is None:
            k_pool = torch.zeros(shape, dtype=dtype, device=device)
            v_pool = torch.zeros(shape, dtype=dtype, device=device)
        i32 = dict(dtype=torch.int32, device=device)
        cache = PagedCache(desc, k_pool, v_pool, table.to(device).contiguous(),
                           torch.zeros(num_seqs, **i32), spare.to(device).contiguous(),
                           torch.zeros(per_row, **i32), torch.full(per_row, -1, **i32),
                           torch.full(per_row, -1, **i32),
                           torch.empty((num_seqs, num_kv_heads, layout.max_blocks), dtype=torch.float32, device=device),
                           int(budget))
        cache.decode_ws = alloc_workspace(PE_OP_PAGED_DECODE, desc, device=device)
        cache.host_lens = [0] * num_seqs
        return cache

    @property
    def shared(self) -> bool:
        return self.desc.layout == PE_LAYOUT_SHARED

    def prefill_prune(self, k_in, v_in, cu_seqlens, max_seqlen, kept_idx_out=None, workspace=None):
        total = k_in.shape[0]
        if workspace is None:
            workspace = alloc_workspace(PE_OP_PREFILL_PRUNE, self.desc, total, device=k_in.device)
        pe_prefill_prune(self.desc, k_in, v_in, cu_seqlens, total, max_seqlen, self.budget, self.k_pool, self.v_pool,
                         self.block_table, self.seq_lens, kept_idx_out, workspace)

    def set_host_lens(self, prompt_lens):
        """Tell the host mirror what the prune was given: cached length = min(L, C)."""
        self.host_lens = [min(int(L), self.budget) for L in prompt_lens]

    def any_trigger(self) -> bool:
        B = self.desc.block_size
        return any(n > 0 and n % B == 0 and n >= self.budget for n in self.host_lens)

    def _sp(self, name, dtype=None):
        """Checked device pointer of one of the cache's own tensors, remembered per tensor object (the state
        tensors are passed on every call of a decode loop; their checks need not be repeated)."""
        t = getattr(self, name)
        memo = self.__dict__.setdefault("_ptr_memo", {})
        hit = memo.get(name)
        if hit is not None and hit[0] is t:
            return hit[1]
        alt = memo.get(name + "~")          # the two lengths arrays alternate
        if alt is not None and alt[0] is t:
            memo[name], memo[name + "~"] = alt, hit
            return alt[1]
        p = _ptr(t, name, dtype)
        if hit is not None:
            memo[name + "~"] = hit
        memo[name] = (t, p)
        return p

    def append_paged_decode(self, new_k, new_v, q, out, softmax_scale=None):
        if softmax_scale is None:
            softmax_scale = float(self.desc.head_dim) ** -0.5
        if self.seq_lens_alt is None:
            self.seq_lens_alt = torch.empty_like(self.seq_lens)
        if not _HostOnly.active:
            i32 = torch.int32
            wp, wn = _ws(self.decode_ws)
            _check(lib().pe_append_paged_decode(
                ctypes.byref(self.desc), _ptr(new_k, "new_k"), _ptr(new_v, "new_v"), _ptr(q, "q"),
                self._sp("k_pool"), self._sp("v_pool"), self._sp("block_table", i32), self._sp("seq_lens", i32),
                self._sp("seq_lens_alt", i32), self._sp("freed_phys", i32), self._sp("spare", i32),
                self._sp("spare_used", i32), int(self.spare.shape[-1]), ctypes.c_float(softmax_scale),
                _ptr(out, "out"), wp, wn, _stream()), "pe_append_paged_decode")
        self.seq_lens, self.seq_lens_alt = self.seq_lens_alt, self.seq_lens

    def decode_step(self, new_k, new_v, q, out, softmax_scale=None, fused=True):
        """One decode iteration of one layer (Alg. 3): score + evict when some sequence's newest page has
        filled at budget, append the new token, attend.  Which steps trigger follows from the lengths
        alone, so the host decides it without reading anything back."""
        B = self.desc.block_size
        if self.any_trigger():
            self.score_and_evict()
            self.host_lens = [n - B if (n > 0 and n % B == 0 and n >= self.budget) else n for n in self.host_lens]
        if fused:
            self.append_paged_decode(new_k, new_v, q, out, softmax_scale)
        else:
            self.append_kv(new_k, new_v)
            self.paged_decode(q, out, softmax_scale)
        self.host_lens = [n + 1 for n in self.host_lens]

    def score_blocks(self):
        pe_score_blocks(self.desc, self.k_pool, self.v_pool, self.block_table, self.seq_lens, self.scores)

    def score_triggered_blocks(self):
        pe_score_triggered_blocks(self.desc, self.k_pool, self.v_pool, self.block_table, self.seq_lens, self.budget,
                                  self.scores)

    def evict_blocks(self):
        pe_evict_blocks(self.desc, self.scores, self.block_table, self.seq_lens, self.budget, self.evicted_logical,
                        self.freed_phys)

    def score_and_evict(self):
        """Score + evict of a trigger step.  With cached scores only the pages filled since the last call are
        scored (all of them the first time) and the eviction keeps the score rows aligned with the table."""
        B = self.desc.block_size
        if self.evict_opts is not None:
            o = self.evict_opts
            opts = pe_evict_opts(o.policy, o.protect_first, o.protect_last, o.share_heads, 0)
            if o.policy != PE_POLICY_OLDEST:
                self.score_triggered_blocks()
            pe_evict_blocks_ex(self.desc, opts, self.scores if o.policy != PE_POLICY_OLDEST else None,
                               self.block_table, self.seq_lens, self.budget, self.evicted_logical, self.freed_phys)
            return
        if self.fused_evict and not self.cached_scores:
            pe_score_evict(self.desc, self.k_pool, self.v_pool, self.block_table, self.seq_lens, self.budget, None,
                           self.evicted_logical, self.freed_phys)
            return
        if not self.cached_scores:   # Alg. 3: score the pages of the sequences that evict now, then evict
            self.score_triggered_blocks()
            self.evict_blocks()
            return
        full = [n // B for n in self.host_lens]
        if self.host_scored is None:
            self.score_blocks()
        else:
            recent = max(f - sc for f, sc in zip(full, self.host_scored))
            if recent > 0:
                pe_score_recent_blocks(self.desc, self.k_pool, self.v_pool, self.block_table, self.seq_lens, recent,
                                       self.scores)
        pe_evict_blocks_cached(self.desc, self.scores, self.block_table, self.seq_lens, self.budget,
                               self.evicted_logical, self.freed_phys)
        self.host_scored = [f - 1 if (n > 0 and n % B == 0 and n >= self.budget) else f
                            for f, n in zip(full, self.host_lens)]

    def append_kv(self, new_k, new_v):
        if _HostOnly.active:
            return
        i32 = torch.int32
        _check(lib().pe_append_kv(ctypes.byref(self.desc), _ptr(new_k, "new_k"), _ptr(new_v, "new_v"),
                                  self._sp("k_pool"), self._sp("v_pool"), self._sp("block_table", i32),
                                  self._sp("seq_lens", i32), self._sp("freed_phys", i32), self._sp("spare", i32),
                                  self._sp("spare_used", i32), int(self.spare.shape[-1]), _stream()), "pe_append_kv")

    def paged_decode(self, q, out, softmax_scale=None):
        if softmax_scale is None:
            softmax_scale = float(self.desc.head_dim) ** -0.5
        if _HostOnly.active:
            return
        wp, wn = _ws(self.decode_ws)
        _check(lib().pe_paged_decode(ctypes.byref(self.desc), _ptr(q, "q"), self._sp("k_pool"), self._sp("v_pool"),
                                     self._sp("block_table", torch.int32), self._sp("seq_lens", torch.int32),
                                     ctypes.c_float(softmax_scale), _ptr(out, "out"), wp, wn, _stream()),
               "pe_paged_decode")
