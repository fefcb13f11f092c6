"""ctypes binding of libvegas.so: the three calls of include/vegas.h under the same names.

Argument marshalling only -- every step of the path runs in the HIP kernels.  Tensors may be
torch tensors on the GPU (their ``data_ptr()`` is passed) or raw integer device addresses.  The
library is loaded on first use and a missing build is an error, never a fallback.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libvegas.so")

VEGAS_OK = 0
VEGAS_ERR_NULL = -1
VEGAS_ERR_SHAPE = -2
VEGAS_ERR_UNSUPPORTED = -3
VEGAS_ERR_ALIGN = -4
VEGAS_ERR_WORKSPACE = -5
VEGAS_ERR_LAUNCH = -6

COLLECT_NONE = 0
COLLECT_ALL_ROWS = 1
COLLECT_FIRST_LAST = 2

METRIC_PAGE_WEIGHTS = 0
METRIC_TOKEN_LOGITS = 1

TABLE_BLOCKS = 0
TABLE_SELECTION = 1
CHECK_LENGTH_RANGE = 1
CHECK_LENGTH_EXCEEDS_TABLE = 2
CHECK_PAGE_ID = 4
CHECK_SHORTER_THAN_QUERIES = 8

STAGE_STREAM = 1
STAGE_MERGE = 2

EXPORTS = ("vegas_init", "vegas_workspace_bytes", "vegas_verify_attention", "vegas_select_blocks",
           "vegas_select_tokens", "vegas_append_kv", "vegas_append_kv_extend", "vegas_extend_selection", "vegas_draft_attention",
           "vegas_draft_attention_static", "vegas_static_scratch_bytes",
           "vegas_debug_verify_attention_stages", "vegas_debug_draft_attention_stages", "vegas_debug_stream_read",
           "vegas_debug_check_tables", "vegas_debug_set_timeline", "vegas_strerror")


class VegasDesc(ctypes.Structure):
    """Mirror of ``vegas_desc`` (include/vegas.h)."""
    _fields_ = [
        ("batch", ctypes.c_int32),
        ("num_q_heads", ctypes.c_int32),
        ("num_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("page_size", ctypes.c_int32),
        ("num_queries", ctypes.c_int32),
        ("max_blocks", ctypes.c_int32),
        ("max_sel_blocks", ctypes.c_int32),
        ("max_seq_len", ctypes.c_int32),
        ("collect_rows", ctypes.c_int32),
        ("kv_chunk_tokens", ctypes.c_int32),
        ("reserved", ctypes.c_int32),
        ("softmax_scale", ctypes.c_float),
        ("score_metric", ctypes.c_int32),
        ("window", ctypes.c_int32),
        ("budget_ratio", ctypes.c_float),
        ("num_pages", ctypes.c_int64),
        ("kv_page_stride", ctypes.c_int64),
        ("kv_token_stride", ctypes.c_int64),
        ("kv_head_stride", ctypes.c_int64),
    ]


class VegasError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} (status {status})")


_lib = None


def load_library(path: Optional[str] = None):
    """Load libvegas.so (once).  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    path = path or os.environ.get("VEGAS_LIB", LIB_PATH)
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it first (python -m paper_2602_07223_amd.build, "
                           "or __graft_entry__.build()); there is no fallback path")
    lib = ctypes.CDLL(path)
    P = ctypes.c_void_p
    D = ctypes.POINTER(VegasDesc)
    lib.vegas_init.restype = ctypes.c_int
    lib.vegas_init.argtypes = []
    lib.vegas_workspace_bytes.restype = ctypes.c_size_t
    lib.vegas_workspace_bytes.argtypes = [D]
    lib.vegas_verify_attention.restype = ctypes.c_int
    lib.vegas_verify_attention.argtypes = [D, P, P, P, P, P, P, P, P, ctypes.c_size_t, P]
    lib.vegas_select_blocks.restype = ctypes.c_int
    lib.vegas_select_blocks.argtypes = [D, P, P, P, ctypes.c_int32, P, P, P, P, ctypes.c_size_t, P]
    lib.vegas_select_tokens.restype = ctypes.c_int
    lib.vegas_select_tokens.argtypes = [D, P, P, P, ctypes.c_int32, P, P, P, P, ctypes.c_size_t, P]
    lib.vegas_append_kv.restype = ctypes.c_int
    lib.vegas_append_kv.argtypes = [D, P, P, ctypes.c_int32, P, P, P, P, P]
    lib.vegas_append_kv_extend.restype = ctypes.c_int
    lib.vegas_append_kv_extend.argtypes = [D, P, P, ctypes.c_int32, P, P, P, P, P, P, ctypes.c_int32, P]
    lib.vegas_extend_selection.restype = ctypes.c_int
    lib.vegas_extend_selection.argtypes = [D, P, P, ctypes.c_int32, P, P, P]
    lib.vegas_draft_attention.restype = ctypes.c_int
    lib.vegas_draft_attention.argtypes = [D, P, P, P, P, P, P, P, ctypes.c_size_t, P]
    lib.vegas_draft_attention_static.restype = ctypes.c_int
    lib.vegas_draft_attention_static.argtypes = [D, P, P, P, P, P, P, P]
    lib.vegas_static_scratch_bytes.restype = ctypes.c_size_t
    lib.vegas_static_scratch_bytes.argtypes = []
    lib.vegas_debug_verify_attention_stages.restype = ctypes.c_int
    lib.vegas_debug_verify_attention_stages.argtypes = [D, P, P, P, P, P, P, P, P, ctypes.c_size_t, P, ctypes.c_int32]
    lib.vegas_debug_draft_attention_stages.restype = ctypes.c_int
    lib.vegas_debug_draft_attention_stages.argtypes = [D, P, P, P, P, P, P, P, ctypes.c_size_t, P, ctypes.c_int32]
    lib.vegas_debug_stream_read.restype = ctypes.c_int
    lib.vegas_debug_stream_read.argtypes = [P, P, ctypes.c_size_t, ctypes.c_int32, ctypes.c_int32, P, P]
    lib.vegas_debug_check_tables.restype = ctypes.c_int
    lib.vegas_debug_check_tables.argtypes = [D, ctypes.c_int32, P, P, P, P]
    lib.vegas_debug_set_timeline.restype = ctypes.c_int
    lib.vegas_debug_set_timeline.argtypes = [P, ctypes.c_size_t]
    lib.vegas_strerror.restype = ctypes.c_char_p
    lib.vegas_strerror.argtypes = [ctypes.c_int]
    _lib = lib
    return lib


def _ptr(x) -> Optional[int]:
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return int(x.data_ptr())


def _nbytes(x) -> int:
    return int(x.numel() * x.element_size())


def _avail_bytes(x) -> int:
    """Bytes from a tensor's first element to the end of its storage (what a kernel may address through it)."""
    return int(x.untyped_storage().nbytes()) - int(x.storage_offset()) * int(x.element_size())


def cache_extent_bytes(desc: "VegasDesc") -> int:
    """Bytes a K or V cache must span under the descriptor's strides: the kernels clamp page ids to
    [0, num_pages) and address every token slot and KV head of such a page."""
    last = ((desc.num_pages - 1) * desc.kv_page_stride + (desc.page_size - 1) * desc.kv_token_stride +
            (desc.num_kv_heads - 1) * desc.kv_head_stride + desc.head_dim)
    return 2 * int(last)


def _check_extents(where: str, **need) -> None:
    """The C ABI takes bare pointers and cannot see allocation sizes; where tensors (not raw addresses) are
    passed, refuse any that is smaller than what the descriptor lets the kernels touch."""
    for name, (x, nbytes) in need.items():
        if x is None or isinstance(x, int):
            continue
        have = _avail_bytes(x)
        if have < nbytes:
            raise ValueError(f"{where}: {name} spans {have} bytes, the descriptor needs {nbytes}")


def _stream(stream) -> Optional[int]:
    if stream is None:
        return None
    if isinstance(stream, int):
        return stream
    return int(stream.cuda_stream)


def strerror(status: int) -> str:
    return load_library().vegas_strerror(int(status)).decode()


def make_desc(*, batch: int, num_q_heads: int, num_kv_heads: int, num_queries: int, max_blocks: int,
              max_sel_blocks: int, max_seq_len: int, num_pages: int, softmax_scale: float,
              collect_rows: int = COLLECT_ALL_ROWS, head_dim: int = 128, page_size: int = 16,
              kv_chunk_tokens: int = 0, kv_page_stride: int = 0, kv_token_stride: int = 0,
              kv_head_stride: int = 0, score_metric: int = METRIC_PAGE_WEIGHTS,
              budget_ratio: float = 0.0, window: int = 0) -> VegasDesc:
    """Descriptor for a contiguous NHD cache unless strides are given (elements)."""
    d = VegasDesc()
    d.batch, d.num_q_heads, d.num_kv_heads = batch, num_q_heads, num_kv_heads
    d.head_dim, d.page_size, d.num_queries = head_dim, page_size, num_queries
    d.max_blocks, d.max_sel_blocks, d.max_seq_len = max_blocks, max_sel_blocks, max_seq_len
    d.collect_rows, d.kv_chunk_tokens, d.softmax_scale = collect_rows, kv_chunk_tokens, softmax_scale
    d.reserved = 0
    d.score_metric = score_metric
    d.budget_ratio = budget_ratio
    d.window = window
    d.num_pages = num_pages
    d.kv_head_stride = kv_head_stride or head_dim
    d.kv_token_stride = kv_token_stride or num_kv_heads * head_dim
    d.kv_page_stride = kv_page_stride or page_size * num_kv_heads * head_dim
    return d


def vegas_workspace_bytes(desc: VegasDesc) -> int:
    return int(load_library().vegas_workspace_bytes(ctypes.byref(desc)))


def vegas_init() -> None:
    """One-time set-up for the current device (see include/vegas.h); optional, the calls do it lazily otherwise."""
    rc = load_library().vegas_init()
    if rc != VEGAS_OK:
        raise VegasError(rc, "vegas_init")


def vegas_verify_attention(desc: VegasDesc, q, k_cache, v_cache, block_table, seq_lens, out, block_scores,
                           workspace, stream=None, workspace_bytes: Optional[int] = None, stages: int = 0) -> None:
    """stages != 0: vegas_debug_verify_attention_stages (a profiling aid: only those kernels of the call)."""
    wb = workspace_bytes if workspace_bytes is not None else (_nbytes(workspace) if workspace is not None else 0)
    if not (isinstance(q, int) and isinstance(k_cache, int)):      # raw addresses: the caller has checked (harness)
        d = desc
        rows = d.batch * d.num_queries * d.num_q_heads * d.head_dim * 2
        per_page = 16 if d.score_metric == METRIC_TOKEN_LOGITS else 1
        _check_extents("vegas_verify_attention", q=(q, rows), out=(out, rows),
                       k_cache=(k_cache, cache_extent_bytes(d)), v_cache=(v_cache, cache_extent_bytes(d)),
                       block_table=(block_table, d.batch * d.max_blocks * 4), seq_lens=(seq_lens, d.batch * 4),
                       block_scores=(block_scores if d.collect_rows != COLLECT_NONE else None,
                                     d.batch * d.max_blocks * per_page * 4))
    args = (ctypes.byref(desc), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(block_table), _ptr(seq_lens), _ptr(out),
            _ptr(block_scores), _ptr(workspace), wb, _stream(stream))
    if stages:
        rc = load_library().vegas_debug_verify_attention_stages(*args, int(stages))
    else:
        rc = load_library().vegas_verify_attention(*args)
    if rc != VEGAS_OK:
        raise VegasError(rc, "vegas_verify_attention")


def vegas_select_blocks(desc: VegasDesc, block_scores, block_table, seq_lens, budget_tokens: int, sel_table,
                        sel_seq_lens, budgets=None, workspace=None, stream=None) -> None:
    wb = _nbytes(workspace) if workspace is not None and not isinstance(workspace, int) else 0
    if not (isinstance(block_scores, int) and isinstance(sel_table, int)):
        d = desc
        _check_extents("vegas_select_blocks", block_scores=(block_scores, d.batch * d.max_blocks * 4),
                       block_table=(block_table, d.batch * d.max_blocks * 4), seq_lens=(seq_lens, d.batch * 4),
                       budgets=(budgets, d.batch * 4), sel_table=(sel_table, d.batch * d.max_sel_blocks * 4),
                       sel_seq_lens=(sel_seq_lens, d.batch * 4))
    rc = load_library().vegas_select_blocks(ctypes.byref(desc), _ptr(block_scores), _ptr(block_table),
                                            _ptr(seq_lens), int(budget_tokens), _ptr(budgets), _ptr(sel_table),
                                            _ptr(sel_seq_lens), _ptr(workspace), wb, _stream(stream))
    if rc != VEGAS_OK:
        raise VegasError(rc, "vegas_select_blocks")


def vegas_select_tokens(desc: VegasDesc, token_scores, block_table, seq_lens, budget_tokens: int, sel_table,
                        sel_seq_lens, workspace, budgets=None, stream=None, workspace_bytes: Optional[int] = None) -> None:
    wb = workspace_bytes if workspace_bytes is not None else (_nbytes(workspace) if workspace is not None else 0)
    if not (isinstance(token_scores, int) and isinstance(sel_table, int)):
        d = desc
        _check_extents("vegas_select_tokens", token_scores=(token_scores, d.batch * d.max_blocks * 16 * 4),
                       block_table=(block_table, d.batch * d.max_blocks * 4), seq_lens=(seq_lens, d.batch * 4),
                       budgets=(budgets, d.batch * 4), sel_table=(sel_table, d.batch * d.max_sel_blocks * 4),
                       sel_seq_lens=(sel_seq_lens, d.batch * 4))
    rc = load_library().vegas_select_tokens(ctypes.byref(desc), _ptr(token_scores), _ptr(block_table),
                                            _ptr(seq_lens), int(budget_tokens), _ptr(budgets), _ptr(sel_table),
                                            _ptr(sel_seq_lens), _ptr(workspace), wb, _stream(stream))
    if rc != VEGAS_OK:
        raise VegasError(rc, "vegas_select_tokens")


def vegas_append_kv(desc: VegasDesc, k_new, v_new, num_new: int, block_table, seq_lens, k_cache, v_cache,
                    stream=None) -> None:
    if not (isinstance(k_new, int) and isinstance(k_cache, int)):
        d = desc
        rows = d.batch * int(num_new) * d.num_kv_heads * d.head_dim * 2
        _check_extents("vegas_append_kv", k_new=(k_new, rows), v_new=(v_new, rows),
                       k_cache=(k_cache, cache_extent_bytes(d)), v_cache=(v_cache, cache_extent_bytes(d)),
                       block_table=(block_table, d.batch * d.max_blocks * 4), seq_lens=(seq_lens, d.batch * 4))
    rc = load_library().vegas_append_kv(ctypes.byref(desc), _ptr(k_new), _ptr(v_new), int(num_new), _ptr(block_table),
                                        _ptr(seq_lens), _ptr(k_cache), _ptr(v_cache), _stream(stream))
    if rc != VEGAS_OK:
        raise VegasError(rc, "vegas_append_kv")


def vegas_append_kv_extend(desc: VegasDesc, k_new, v_new, num_new: int, block_table, seq_lens, k_cache, v_cache,
                           sel_table, sel_seq_lens, sel_page_size: int, stream=None) -> None:
    if not (isinstance(k_new, int) and isinstance(k_cache, int)):
        d = desc
        rows = d.batch * int(num_new) * d.num_kv_heads * d.head_dim * 2
        _check_extents("vegas_append_kv_extend", k_new=(k_new, rows), v_new=(v_new, rows),
                       k_cache=(k_cache, cache_extent_bytes(d)), v_cache=(v_cache, cache_extent_bytes(d)),
                       block_table=(block_table, d.batch * d.max_blocks * 4), seq_lens=(seq_lens, d.batch * 4),
                       sel_table=(sel_table, d.batch * d.max_sel_blocks * 4), sel_seq_lens=(sel_seq_lens, d.batch * 4))
    rc = load_library().vegas_append_kv_extend(ctypes.byref(desc), _ptr(k_new), _ptr(v_new), int(num_new),
                                               _ptr(block_table), _ptr(seq_lens), _ptr(k_cache), _ptr(v_cache),
                                               _ptr(sel_table), _ptr(sel_seq_lens), int(sel_page_size), _stream(stream))
    if rc != VEGAS_OK:
        raise VegasError(rc, "vegas_append_kv_extend")


def vegas_extend_selection(desc: VegasDesc, block_table, seq_lens, num_new: int, sel_table, sel_seq_lens,
                           stream=None) -> None:
    if not (isinstance(block_table, int) and isinstance(sel_table, int)):
        d = desc
        _check_extents("vegas_extend_selection", block_table=(block_table, d.batch * d.max_blocks * 4),
                       seq_lens=(seq_lens, d.batch * 4), sel_table=(sel_table, d.batch * d.max_sel_blocks * 4),
                       sel_seq_lens=(sel_seq_lens, d.batch * 4))
    rc = load_library().vegas_extend_selection(ctypes.byref(desc), _ptr(block_table), _ptr(seq_lens), int(num_new),
                                               _ptr(sel_table), _ptr(sel_seq_lens), _stream(stream))
    if rc != VEGAS_OK:
        raise VegasError(rc, "vegas_extend_selection")


def vegas_draft_attention(desc: VegasDesc, q, k_cache, v_cache, sel_table, sel_seq_lens, out, workspace,
                          stream=None, workspace_bytes: Optional[int] = None, stages: int = 0) -> None:
    """stages != 0: vegas_debug_draft_attention_stages (a profiling aid: only those kernels of the call)."""
    wb = workspace_bytes if workspace_bytes is not None else (_nbytes(workspace) if workspace is not None else 0)
    if not (isinstance(q, int) and isinstance(k_cache, int)):
        d = desc
        rows = d.batch * d.num_q_heads * d.head_dim * 2
        _check_extents("vegas_draft_attention", q=(q, rows), out=(out, rows),
                       k_cache=(k_cache, cache_extent_bytes(d)), v_cache=(v_cache, cache_extent_bytes(d)),
                       sel_table=(sel_table, d.batch * d.max_sel_blocks * 4), sel_seq_lens=(sel_seq_lens, d.batch * 4))
    args = (ctypes.byref(desc), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(sel_table), _ptr(sel_seq_lens), _ptr(out),
            _ptr(workspace), wb, _stream(stream))
    if stages:
        rc = load_library().vegas_debug_draft_attention_stages(*args, int(stages))
    else:
        rc = load_library().vegas_draft_attention(*args)
    if rc != VEGAS_OK:
        raise VegasError(rc, "vegas_draft_attention")


def vegas_static_scratch_bytes() -> int:
    return int(load_library().vegas_static_scratch_bytes())


def vegas_draft_attention_static(desc: VegasDesc, q, k_cache, v_cache, sel_table, sel_seq_lens, out, stream=None) -> None:
    """vegas_draft_attention without a workspace argument: the library's built-in scratch array is used."""
    if not (isinstance(q, int) and isinstance(k_cache, int)):
        d = desc
        rows = d.batch * d.num_q_heads * d.head_dim * 2
        _check_extents("vegas_draft_attention_static", q=(q, rows), out=(out, rows),
                       k_cache=(k_cache, cache_extent_bytes(d)), v_cache=(v_cache, cache_extent_bytes(d)),
                       sel_table=(sel_table, d.batch * d.max_sel_blocks * 4), sel_seq_lens=(sel_seq_lens, d.batch * 4))
    rc = load_library().vegas_draft_attention_static(ctypes.byref(desc), _ptr(q), _ptr(k_cache), _ptr(v_cache),
                                                     _ptr(sel_table), _ptr(sel_seq_lens), _ptr(out), _stream(stream))
    if rc != VEGAS_OK:
        raise VegasError(rc, "vegas_draft_attention_static")


def vegas_debug_check_tables(desc: VegasDesc, which: int, table, lens, error_word, stream=None) -> None:
    """ORs VEGAS_CHECK_* bits for out-of-range lengths and page ids into the device word (see include/vegas.h)."""
    if not isinstance(table, int):
        stride = desc.max_blocks if which == TABLE_BLOCKS else desc.max_sel_blocks
        _check_extents("vegas_debug_check_tables", table=(table, desc.batch * stride * 4), lens=(lens, desc.batch * 4),
                       error_word=(error_word, 4))
    rc = load_library().vegas_debug_check_tables(ctypes.byref(desc), int(which), _ptr(table), _ptr(lens),
                                                 _ptr(error_word), _stream(stream))
    if rc != VEGAS_OK:
        raise VegasError(rc, "vegas_debug_check_tables")


def vegas_debug_set_timeline(buffer, nbytes: Optional[int] = None) -> None:
    """Profiling builds only: register (or, with None, drop) the buffer for the streaming kernels' phase stamps."""
    nb = 0 if buffer is None else (nbytes if nbytes is not None else _nbytes(buffer))
    rc = load_library().vegas_debug_set_timeline(_ptr(buffer), nb)
    if rc != VEGAS_OK:
        raise VegasError(rc, "vegas_debug_set_timeline")


def vegas_debug_stream_read(a, b, bytes_each: int, workgroups: int, non_temporal: bool, sink, stream=None) -> None:
    """The plain streaming read the benchmark uses as its yardstick (see include/vegas.h)."""
    if not isinstance(a, int):
        _check_extents("vegas_debug_stream_read", a=(a, bytes_each), b=(b, bytes_each), sink=(sink, workgroups * 256 * 4))
    rc = load_library().vegas_debug_stream_read(_ptr(a), _ptr(b), int(bytes_each), int(workgroups), int(bool(non_temporal)),
                                                _ptr(sink), _stream(stream))
    if rc != VEGAS_OK:
        raise VegasError(rc, "vegas_debug_stream_read")


# ---------------------------------------------------------------------------------------------
# HIP events on a raw stream (timing plumbing for the benchmark)
# ---------------------------------------------------------------------------------------------

_hip = None


def _hip_runtime():
    global _hip
    if _hip is None:
        for name in ("libamdhip64.so", "libamdhip64.so.7", "libamdhip64.so.6", "/opt/rocm/lib/libamdhip64.so"):
            try:
                _hip = ctypes.CDLL(name)
                break
            except OSError:
                continue
        if _hip is None:
            raise RuntimeError("libamdhip64.so not found")
        _hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        _hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        _hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        _hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        _hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
    return _hip


class HipEvent:
    """A hipEvent_t recorded on a raw stream handle (the stream the library's kernels are launched on)."""

    def __init__(self):
        self.handle = ctypes.c_void_p()
        rc = _hip_runtime().hipEventCreate(ctypes.byref(self.handle))
        if rc != 0:
            raise RuntimeError(f"hipEventCreate failed ({rc})")

    def record(self, stream=None) -> None:
        rc = _hip_runtime().hipEventRecord(self.handle, _stream(stream))
        if rc != 0:
            raise RuntimeError(f"hipEventRecord failed ({rc})")

    def synchronize(self) -> None:
        rc = _hip_runtime().hipEventSynchronize(self.handle)
        if rc != 0:
            raise RuntimeError(f"hipEventSynchronize failed ({rc})")

    def elapsed_ms(self, end: "HipEvent") -> float:
        ms = ctypes.c_float()
        rc = _hip_runtime().hipEventElapsedTime(ctypes.byref(ms), self.handle, end.handle)
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed ({rc})")
        return float(ms.value)

    def __del__(self):
        try:
            if self.handle:
                _hip_runtime().hipEventDestroy(self.handle)
        except Exception:
            pass
