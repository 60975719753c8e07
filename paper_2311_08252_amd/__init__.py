"""Thin Python binding of the gfx950 REST library (include/rest.h).

Argument marshalling only: every step of the hot path runs in the HIP kernels
of librest_gfx950.so.  PyTorch tensors are used as device buffers and the
current torch stream as the HIP stream.  There is no CPU fallback: if the
shared library is missing or fails to load, importing this package raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# REST_LIBRARY=checked loads the bounds-checked build of the same sources (librest_gfx950_checked.so: indices that
# depend on data or on the launch plan are clamped into their arrays and reported, every call waits for its kernels);
# it exists to run the test suite under, not to serve from.
LIB_PATH = os.path.join(_HERE, "librest_gfx950_checked.so" if os.environ.get("REST_LIBRARY") == "checked" else "librest_gfx950.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it first (python -m paper_2311_08252_amd.build, "
        "or __graft_entry__.build()); this package has no fallback path")
_lib = ctypes.CDLL(LIB_PATH)

REST_OK = 0
REST_INVALID_ARG = -1
REST_UNSUPPORTED = -2
REST_WORKSPACE_TOO_SMALL = -3
REST_OUT_OF_MEMORY = -4
REST_HIP_ERROR = -5
REST_IO_ERROR = -6
REST_BAD_FILE = -7
REST_BOUNDS_VIOLATION = -8
REST_BF16 = 0
REST_FP32 = 1
REST_KV_AS_DTYPE = 0
REST_KV_FP8_E4M3 = 1
REST_MAX_SUFFIX_LEN = 16
REST_MAX_CONT_LEN = 32
REST_MAX_MATCHES = 8192
REST_MAX_NODES = 256
REST_MAX_QUERY_ROWS = 1024
REST_STATIC_SCRATCH_BYTES = 64 * 1024 * 1024

EXPORTS = [
    "rest_status_string", "rest_version", "rest_build_index", "rest_index_from_sa", "rest_index_view",
    "rest_index_destroy", "rest_retrieve_workspace_bytes", "rest_retrieve",
    "rest_tree_attention_workspace_bytes", "rest_tree_attention", "rest_accept",
    "rest_rope_append", "rest_kv_compact", "rest_sample_ids", "rest_index_save", "rest_index_load",
    "rest_build_index_prefix", "rest_index_sort_depth", "rest_tree_attention_noalloc", "rest_sample_ids_workspace_bytes",
]


class RestError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {rest_status_string(status)} ({status})")


class rest_retrieve_params(ctypes.Structure):
    _fields_ = [("n_max", ctypes.c_int32), ("n_min", ctypes.c_int32), ("max_matches", ctypes.c_int32),
                ("cont_len", ctypes.c_int32), ("max_nodes", ctypes.c_int32), ("random_seqs", ctypes.c_int32),
                ("seed", ctypes.c_uint64), ("strided", ctypes.c_int32), ("reserved_", ctypes.c_int32)]


class rest_tree(ctypes.Structure):
    _fields_ = [("draft_tokens", ctypes.c_void_p), ("parent_idx", ctypes.c_void_p), ("pos_ids", ctypes.c_void_p),
                ("node_weight", ctypes.c_void_p), ("tree_mask", ctypes.c_void_p), ("n_nodes", ctypes.c_void_p),
                ("matched_len", ctypes.c_void_p), ("match_count", ctypes.c_void_p)]


class rest_attn_desc(ctypes.Structure):
    _fields_ = [("Nb", ctypes.c_int32), ("H", ctypes.c_int32), ("Tq", ctypes.c_int32), ("Tk", ctypes.c_int32),
                ("P", ctypes.c_int32), ("D", ctypes.c_int32), ("dtype", ctypes.c_int32), ("scale", ctypes.c_float),
                ("q_stride", ctypes.c_int64 * 3), ("k_stride", ctypes.c_int64 * 3), ("v_stride", ctypes.c_int64 * 3),
                ("o_stride", ctypes.c_int64 * 3), ("mask_per_batch", ctypes.c_int32), ("num_splits", ctypes.c_int32),
                ("mask_rows", ctypes.c_int32), ("kv_dtype", ctypes.c_int32), ("d_k_scale", ctypes.c_void_p),
                ("d_v_scale", ctypes.c_void_p)]


class rest_kv_desc(ctypes.Structure):
    _fields_ = [("Nb", ctypes.c_int32), ("H", ctypes.c_int32), ("T", ctypes.c_int32), ("D", ctypes.c_int32),
                ("P", ctypes.c_int32), ("pos_offset", ctypes.c_int32), ("per_batch", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("theta", ctypes.c_double),
                ("q_stride", ctypes.c_int64 * 3), ("kn_stride", ctypes.c_int64 * 3), ("vn_stride", ctypes.c_int64 * 3),
                ("kc_stride", ctypes.c_int64 * 3), ("vc_stride", ctypes.c_int64 * 3),
                ("cache_dtype", ctypes.c_int32), ("reserved_", ctypes.c_int32), ("d_k_scale", ctypes.c_void_p),
                ("d_v_scale", ctypes.c_void_p)]


_lib.rest_status_string.restype = ctypes.c_char_p
_lib.rest_status_string.argtypes = [ctypes.c_int32]
_lib.rest_version.restype = ctypes.c_char_p
_lib.rest_build_index.restype = ctypes.c_int32
_lib.rest_build_index.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p,
                                  ctypes.POINTER(ctypes.c_void_p)]
_lib.rest_build_index_prefix.restype = ctypes.c_int32
_lib.rest_build_index_prefix.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                         ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p)]
_lib.rest_index_sort_depth.restype = ctypes.c_int32
_lib.rest_index_sort_depth.argtypes = [ctypes.c_void_p]
_lib.rest_index_from_sa.restype = ctypes.c_int32
_lib.rest_index_from_sa.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int32, ctypes.c_int32,
                                    ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p)]
_lib.rest_index_view.restype = ctypes.c_int32
_lib.rest_index_view.argtypes = [ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p), ctypes.POINTER(ctypes.c_void_p),
                                 ctypes.POINTER(ctypes.c_uint64), ctypes.POINTER(ctypes.c_int32),
                                 ctypes.POINTER(ctypes.c_int32)]
_lib.rest_index_save.restype = ctypes.c_int32
_lib.rest_index_save.argtypes = [ctypes.c_void_p, ctypes.c_char_p, ctypes.c_void_p]
_lib.rest_index_load.restype = ctypes.c_int32
_lib.rest_index_load.argtypes = [ctypes.c_char_p, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int32, ctypes.c_void_p,
                                 ctypes.POINTER(ctypes.c_void_p)]
_lib.rest_index_destroy.restype = None
_lib.rest_index_destroy.argtypes = [ctypes.c_void_p]
_lib.rest_retrieve_workspace_bytes.restype = ctypes.c_size_t
_lib.rest_retrieve_workspace_bytes.argtypes = [ctypes.c_int32, ctypes.POINTER(rest_retrieve_params)]
_lib.rest_retrieve.restype = ctypes.c_int32
_lib.rest_retrieve.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32,
                               ctypes.POINTER(rest_retrieve_params), ctypes.POINTER(rest_tree), ctypes.c_void_p,
                               ctypes.c_size_t, ctypes.c_void_p]
_lib.rest_tree_attention_workspace_bytes.restype = ctypes.c_size_t
_lib.rest_tree_attention_workspace_bytes.argtypes = [ctypes.POINTER(rest_attn_desc)]
_lib.rest_tree_attention.restype = ctypes.c_int32
_lib.rest_tree_attention.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                     ctypes.POINTER(rest_attn_desc), ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
_lib.rest_tree_attention_noalloc.restype = ctypes.c_int32
_lib.rest_tree_attention_noalloc.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                             ctypes.POINTER(rest_attn_desc), ctypes.c_void_p]
_lib.rest_accept.restype = ctypes.c_int32
_lib.rest_accept.argtypes = [ctypes.c_void_p, ctypes.POINTER(rest_tree), ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                             ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
_lib.rest_sample_ids.restype = ctypes.c_int32
_lib.rest_sample_ids.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32,
                                 ctypes.c_float, ctypes.c_float, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
_lib.rest_sample_ids_workspace_bytes.restype = ctypes.c_size_t
_lib.rest_sample_ids_workspace_bytes.argtypes = [ctypes.c_int32, ctypes.c_int32]
_lib.rest_rope_append.restype = ctypes.c_int32
_lib.rest_rope_append.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                  ctypes.c_void_p, ctypes.POINTER(rest_kv_desc), ctypes.c_void_p]
_lib.rest_kv_compact.restype = ctypes.c_int32
_lib.rest_kv_compact.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32,
                                 ctypes.POINTER(rest_kv_desc), ctypes.c_void_p]


def rest_status_string(status: int) -> str:
    return _lib.rest_status_string(int(status)).decode()


def rest_version() -> str:
    return _lib.rest_version().decode()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


class _hipPointerAttribute(ctypes.Structure):
    _fields_ = [("type", ctypes.c_int), ("device", ctypes.c_int), ("devicePointer", ctypes.c_void_p),
                ("hostPointer", ctypes.c_void_p), ("isManaged", ctypes.c_int), ("allocationFlags", ctypes.c_uint)]


def _pinned_is_mapped(t: torch.Tensor) -> bool:
    """True if the GPU reads this pinned host tensor at its host address (asked of the HIP runtime, so that a
    pointer the device cannot follow is never handed to a kernel)."""
    try:
        hip = ctypes.CDLL("libamdhip64.so")
    except OSError:
        return False
    a = _hipPointerAttribute()
    rc = hip.hipPointerGetAttributes(ctypes.byref(a), ctypes.c_void_p(t.data_ptr()))
    return rc == 0 and a.devicePointer == t.data_ptr()


def _require(cond: bool, what: str) -> None:
    """Shapes and dtypes are checked on the host before any pointer reaches a kernel: the kernels index the buffers
    from the sizes in the call, so a buffer smaller than those sizes imply would be read or written out of bounds."""
    if not cond:
        raise ValueError(what)


def _dev(t: torch.Tensor, dtype=None, pinned_ok: bool = False) -> int:
    if not t.is_cuda:
        if not (pinned_ok and t.is_pinned() and _pinned_is_mapped(t)):
            raise TypeError("expected a device tensor" + (" or a pinned host tensor the device can address" if pinned_ok else ""))
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {t.dtype}")
    return t.data_ptr()


class RestIndex:
    """Owns a rest_index handle; keeps the borrowed tensors alive."""

    def __init__(self, handle: int, corpus: torch.Tensor, sa: torch.Tensor | None):
        self.handle = handle
        self._corpus = corpus
        self._sa = sa

    @property
    def n_tokens(self) -> int:
        return self.view()[2]

    def view(self):
        c, s = ctypes.c_void_p(), ctypes.c_void_p()
        n, tb, sb = ctypes.c_uint64(), ctypes.c_int32(), ctypes.c_int32()
        st = _lib.rest_index_view(self.handle, ctypes.byref(c), ctypes.byref(s), ctypes.byref(n), ctypes.byref(tb),
                                  ctypes.byref(sb))
        if st != REST_OK:
            raise RestError(st, "rest_index_view")
        return c.value, s.value, n.value, tb.value, sb.value

    @property
    def sort_depth(self) -> int:
        return int(_lib.rest_index_sort_depth(self.handle))

    def suffix_array(self) -> torch.Tensor:
        """Device copy of the suffix array held by the handle (int32 or int64)."""
        _, s, n, _, sb = self.view()

        class _Raw:
            __cuda_array_interface__ = {"shape": (n,), "typestr": "<i4" if sb == 4 else "<i8",
                                        "data": (s, False), "version": 2}

        return torch.as_tensor(_Raw(), device=self._corpus.device).clone()

    def destroy(self):
        if self.handle:
            _lib.rest_index_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def _token_bytes(corpus: torch.Tensor) -> int:
    if corpus.dtype == torch.int32:
        return 4
    if corpus.dtype in (torch.uint16, torch.int16):
        return 2
    raise TypeError("corpus must be int32 or uint16")


def rest_build_index(corpus: torch.Tensor, sa_bytes: int = 4) -> RestIndex:
    """corpus: contiguous 1-D device tensor of int32 or uint16 tokens."""
    assert corpus.is_contiguous() and corpus.dim() == 1
    h = ctypes.c_void_p()
    st = _lib.rest_build_index(_dev(corpus), corpus.numel(), _token_bytes(corpus), sa_bytes, _stream(), ctypes.byref(h))
    if st != REST_OK:
        raise RestError(st, "rest_build_index")
    return RestIndex(h.value, corpus, None)


def rest_build_index_prefix(corpus: torch.Tensor, sa_bytes: int = 4, depth: int = 32) -> RestIndex:
    """Positions ordered by their first `depth` tokens only (enough for n_max + cont_len <= depth)."""
    assert corpus.is_contiguous() and corpus.dim() == 1
    h = ctypes.c_void_p()
    st = _lib.rest_build_index_prefix(_dev(corpus), corpus.numel(), _token_bytes(corpus), sa_bytes, depth, _stream(),
                                      ctypes.byref(h))
    if st != REST_OK:
        raise RestError(st, "rest_build_index_prefix")
    return RestIndex(h.value, corpus, None)


def rest_index_from_sa(corpus: torch.Tensor, sa: torch.Tensor) -> RestIndex:
    """Wraps a token stream and its suffix array.  Both may also live in pinned host memory (a datastore larger than
    the GPU's memory): the kernels then read them over the host link, a few hundred small reads per context."""
    assert corpus.is_contiguous() and sa.is_contiguous() and corpus.numel() == sa.numel()
    sa_bytes = {torch.int32: 4, torch.int64: 8}[sa.dtype]
    h = ctypes.c_void_p()
    st = _lib.rest_index_from_sa(_dev(corpus, pinned_ok=True), _dev(sa, pinned_ok=True), corpus.numel(), _token_bytes(corpus), sa_bytes, _stream(),
                                 ctypes.byref(h))
    if st != REST_OK:
        raise RestError(st, "rest_index_from_sa")
    return RestIndex(h.value, corpus, sa)


def rest_index_save(index: RestIndex, path: str) -> None:
    """Writes the index's suffix array (with a header naming the token stream it belongs to) to a host file."""
    st = _lib.rest_index_save(index.handle, os.fsencode(path), _stream())
    if st != REST_OK:
        raise RestError(st, "rest_index_save")


def rest_index_load(path: str, corpus: torch.Tensor) -> RestIndex:
    """Reads a file written by rest_index_save for this (device) token stream."""
    assert corpus.is_contiguous()
    h = ctypes.c_void_p()
    st = _lib.rest_index_load(os.fsencode(path), _dev(corpus), corpus.numel(), _token_bytes(corpus), _stream(),
                              ctypes.byref(h))
    if st != REST_OK:
        raise RestError(st, "rest_index_load")
    return RestIndex(h.value, corpus, None)


@dataclass
class Tree:
    """Device buffers of rest_tree for B contexts with node capacity c."""
    draft_tokens: torch.Tensor
    parent_idx: torch.Tensor
    pos_ids: torch.Tensor
    node_weight: torch.Tensor
    tree_mask: torch.Tensor
    n_nodes: torch.Tensor
    matched_len: torch.Tensor
    match_count: torch.Tensor

    @staticmethod
    def empty(B: int, c: int, device="cuda", fill: int | None = None) -> "Tree":
        words = (c + 63) // 64
        mk = (lambda shape, dt: torch.empty(shape, dtype=dt, device=device)) if fill is None else \
             (lambda shape, dt: torch.full(shape, fill, dtype=dt, device=device))
        return Tree(mk((B, c), torch.int32), mk((B, c), torch.int32), mk((B, c), torch.int32), mk((B, c), torch.int32),
                    mk((B, c, words), torch.int64), mk((B,), torch.int32), mk((B,), torch.int32), mk((B,), torch.int64))

    def check(self, B: int, c: int) -> None:
        """Raises ValueError unless every buffer is a contiguous tensor of the shape and dtype rest_tree gives it for B
        contexts with node capacity c."""
        words = (c + 63) // 64
        for name, shape, dts in (("draft_tokens", (B, c), (torch.int32,)), ("parent_idx", (B, c), (torch.int32,)),
                                 ("pos_ids", (B, c), (torch.int32,)), ("node_weight", (B, c), (torch.int32,)),
                                 ("tree_mask", (B, c, words), (torch.int64, torch.uint64)),
                                 ("n_nodes", (B,), (torch.int32,)), ("matched_len", (B,), (torch.int32,)),
                                 ("match_count", (B,), (torch.int64,))):
            t = getattr(self, name)
            _require(tuple(t.shape) == shape and t.dtype in dts and t.is_contiguous(),
                     f"tree.{name}: expected contiguous {dts[0]} of shape {shape}, got {t.dtype} {tuple(t.shape)}")

    def as_struct(self) -> rest_tree:
        return rest_tree(self.draft_tokens.data_ptr(), self.parent_idx.data_ptr(), self.pos_ids.data_ptr(),
                         self.node_weight.data_ptr(), self.tree_mask.data_ptr(), self.n_nodes.data_ptr(),
                         self.matched_len.data_ptr(), self.match_count.data_ptr())


def rest_retrieve_workspace_bytes(B: int, n_max=16, n_min=2, max_matches=5000, cont_len=10, max_nodes=64) -> int:
    prm = rest_retrieve_params(n_max, n_min, max_matches, cont_len, max_nodes)
    return _lib.rest_retrieve_workspace_bytes(B, ctypes.byref(prm))


def rest_retrieve(index: RestIndex, contexts: torch.Tensor, ctx_len: torch.Tensor, out: Tree | None = None,
                  n_max=16, n_min=2, max_matches=5000, cont_len=10, max_nodes=64,
                  workspace: torch.Tensor | None = None, random_seqs: int = 0, seed: int = 0,
                  strided: bool = False) -> Tree:
    """contexts [B, ctx_stride] int32, ctx_len [B] int32 (device).  Enqueues on the current stream.
    random_seqs > 0: the ablation's strategy (that many randomly drawn candidates instead of the whole Trie)."""
    _require(contexts.dim() == 2 and contexts.is_contiguous() and ctx_len.is_contiguous(), "contexts [B, stride], ctx_len [B], contiguous")
    B, stride = contexts.shape
    _require(ctx_len.numel() == B, f"ctx_len holds {ctx_len.numel()} entries for {B} contexts")
    in_range = 1 <= max_nodes <= REST_MAX_NODES        # the library refuses other values before it touches `out`
    if out is None:
        out = Tree.empty(B, max_nodes if in_range else 1, contexts.device)
    if in_range:
        out.check(B, max_nodes)
    if workspace is not None:
        _require(workspace.is_contiguous(), "workspace must be contiguous")
    prm = rest_retrieve_params(n_max, n_min, max_matches, cont_len, max_nodes, random_seqs, seed, int(strided), 0)
    tree = out.as_struct()
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    st = _lib.rest_retrieve(index.handle, _dev(contexts, torch.int32), _dev(ctx_len, torch.int32), B, stride,
                            ctypes.byref(prm), ctypes.byref(tree), ws_ptr, ws_bytes, _stream())
    if st != REST_OK:
        raise RestError(st, "rest_retrieve")
    return out


def make_attn_desc(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, out: torch.Tensor, prefix_len: int,
                   scale: float, mask_per_batch: bool, num_splits: int = 0, mask_rows: int = 0,
                   k_scale: torch.Tensor | None = None, v_scale: torch.Tensor | None = None) -> rest_attn_desc:
    _require(q.dim() == 4 and k.dim() == 4 and v.dim() == 4 and out.dim() == 4, "q, k, v, out must be [Nb, H, rows, D]")
    Nb, H, Tq, D = q.shape
    Lk = k.shape[2]
    _require(tuple(k.shape) == (Nb, H, Lk, D) and tuple(v.shape) == (Nb, H, Lk, D),
             f"k {tuple(k.shape)} and v {tuple(v.shape)} must be [Nb={Nb}, H={H}, P+Tk, D={D}]")
    _require(tuple(out.shape) == (Nb, H, Tq, D) and out.dtype == q.dtype,
             f"out must have q's shape {tuple(q.shape)} and dtype, got {out.dtype} {tuple(out.shape)}")
    _require(0 <= prefix_len <= Lk, f"prefix_len {prefix_len} outside [0, {Lk}]")
    _require(q.dtype in (torch.bfloat16, torch.float32), "q must be bfloat16 or float32")
    dt = {torch.bfloat16: REST_BF16, torch.float32: REST_FP32}[q.dtype]
    d = rest_attn_desc()
    d.Nb, d.H, d.Tq, d.Tk, d.P, d.D = Nb, H, Tq, Lk - prefix_len, prefix_len, D
    d.dtype = dt
    d.scale = scale
    for name, t in (("q_stride", q), ("k_stride", k), ("v_stride", v), ("o_stride", out)):
        _require(t.stride(3) == 1, f"{name}: the last axis must be contiguous")
        getattr(d, name)[:] = [t.stride(0), t.stride(1), t.stride(2)]
    d.mask_per_batch = 1 if mask_per_batch else 0
    d.num_splits = num_splits
    d.mask_rows = mask_rows
    if k.dtype == torch.uint8:          # one OCP E4M3 byte per cached element
        _require(v.dtype == torch.uint8 and q.dtype == torch.bfloat16, "an 8-bit cache needs uint8 k and v and bfloat16 q")
        d.kv_dtype = REST_KV_FP8_E4M3
        for name, t in (("d_k_scale", k_scale), ("d_v_scale", v_scale)):
            if t is not None:
                _require(t.dtype == torch.float32 and t.is_contiguous() and t.numel() == Nb * H,
                         f"{name}: expected {Nb * H} contiguous float32 scales")
                setattr(d, name, _dev(t))
    else:
        _require(k_scale is None and v_scale is None and k.dtype == q.dtype and v.dtype == q.dtype,
                 "k and v must have q's dtype (scales belong to an 8-bit cache)")
        d.kv_dtype = REST_KV_AS_DTYPE
    return d


def _check_mask(mask: torch.Tensor, desc: rest_attn_desc, per_batch: bool, mask_rows: int) -> None:
    """The kernels read mask row (i % rows) of batch entry nb at [nb, i % rows, 0 .. words): the tensor must hold that."""
    rows, words = (mask_rows if mask_rows > 0 else desc.Tq), (desc.Tk + 63) // 64
    _require(0 <= mask_rows <= desc.Tq, f"mask_rows {mask_rows} outside [0, Tq]")
    if desc.Tk > 0:
        _require(mask.dtype in (torch.int64, torch.uint64) and mask.is_contiguous(), "mask must be contiguous int64/uint64 bit rows")
        want = (desc.Nb, rows, words) if per_batch else (rows, words)
        _require(tuple(mask.shape) == want, f"mask: expected shape {want} (one mask per batch entry if 3-D), got {tuple(mask.shape)}")


def rest_tree_attention_workspace_bytes(desc: rest_attn_desc) -> int:
    return _lib.rest_tree_attention_workspace_bytes(ctypes.byref(desc))


def rest_tree_attention(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, mask: torch.Tensor, prefix_len: int,
                        scale: float, out: torch.Tensor | None = None, num_splits: int = 0,
                        workspace: torch.Tensor | None = None, mask_rows: int = 0,
                        k_scale: torch.Tensor | None = None, v_scale: torch.Tensor | None = None) -> torch.Tensor:
    """q [Nb,H,Tq,128]; k, v [Nb,H,P+Tk,128] (bf16 or fp32, device); mask [Tq,words] or [Nb,Tq,words] int64/uint64.
    k, v of dtype uint8: an 8-bit (OCP E4M3) cache with optional per-(Nb, H) float32 scales.
    Enqueues on the current stream."""
    _require(q.dim() == 4, "q must be [Nb, H, Tq, D]")
    if out is None:
        out = torch.empty_like(q)
    per_batch = mask.dim() == 3
    desc = make_attn_desc(q, k, v, out, prefix_len, scale, per_batch, num_splits, mask_rows, k_scale, v_scale)
    _check_mask(mask, desc, per_batch, mask_rows)
    if workspace is not None:
        _require(workspace.is_contiguous(), "workspace must be contiguous")
    need = rest_tree_attention_workspace_bytes(desc)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    st = _lib.rest_tree_attention(_dev(q), _dev(k), _dev(v), _dev(mask) if mask.numel() else None, _dev(out),
                                  ctypes.byref(desc), ws_ptr, ws_bytes, _stream())
    if st != REST_OK:
        raise RestError(st, "rest_tree_attention")
    return out


def rest_tree_attention_noalloc(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, mask: torch.Tensor, prefix_len: int,
                                scale: float, out: torch.Tensor, num_splits: int = 0, mask_rows: int = 0,
                                k_scale: torch.Tensor | None = None, v_scale: torch.Tensor | None = None) -> torch.Tensor:
    """rest_tree_attention without a workspace and without any allocation (`out` is the caller's): partial results
    go to the library's own fixed device array.  Raises RestError(REST_WORKSPACE_TOO_SMALL) when they would not fit."""
    _require(q.dim() == 4, "q must be [Nb, H, Tq, D]")
    per_batch = mask.dim() == 3
    desc = make_attn_desc(q, k, v, out, prefix_len, scale, per_batch, num_splits, mask_rows, k_scale, v_scale)
    _check_mask(mask, desc, per_batch, mask_rows)
    st = _lib.rest_tree_attention_noalloc(_dev(q), _dev(k), _dev(v), _dev(mask) if mask.numel() else None, _dev(out),
                                          ctypes.byref(desc), _stream())
    if st != REST_OK:
        raise RestError(st, "rest_tree_attention_noalloc")
    return out


def rest_accept(ids: torch.Tensor, tree: Tree, path_cap: int,
                accept_len: torch.Tensor | None = None, accept_path: torch.Tensor | None = None,
                next_token: torch.Tensor | None = None):
    """ids [B, 1+c] int32 (device).  Returns (accept_len [B], accept_path [B, path_cap], next_token [B])."""
    _require(ids.dim() == 2 and ids.is_contiguous() and ids.shape[1] >= 2, "ids must be contiguous [B, 1 + c]")
    B, c1 = ids.shape
    c = c1 - 1
    tree.check(B, c)
    _require(1 <= path_cap <= REST_MAX_CONT_LEN, "path_cap out of range")
    dev = ids.device
    accept_len = accept_len if accept_len is not None else torch.empty(B, dtype=torch.int32, device=dev)
    accept_path = accept_path if accept_path is not None else torch.empty((B, path_cap), dtype=torch.int32, device=dev)
    next_token = next_token if next_token is not None else torch.empty(B, dtype=torch.int32, device=dev)
    for name, t, shape in (("accept_len", accept_len, (B,)), ("accept_path", accept_path, (B, path_cap)),
                           ("next_token", next_token, (B,))):
        _require(tuple(t.shape) == shape and t.dtype == torch.int32 and t.is_contiguous(),
                 f"{name}: expected contiguous int32 of shape {shape}, got {t.dtype} {tuple(t.shape)}")
    ts = tree.as_struct()
    st = _lib.rest_accept(_dev(ids, torch.int32), ctypes.byref(ts), B, c, path_cap, _dev(accept_len), _dev(accept_path),
                          _dev(next_token), _stream())
    if st != REST_OK:
        raise RestError(st, "rest_accept")
    return accept_len, accept_path, next_token


def make_kv_desc(k_cache: torch.Tensor, v_cache: torch.Tensor, T: int, prefix_len: int, pos_offset: int | None = None,
                 theta: float = 10000.0, per_batch: bool = False, q: torch.Tensor | None = None,
                 k_new: torch.Tensor | None = None, v_new: torch.Tensor | None = None,
                 k_scale: torch.Tensor | None = None, v_scale: torch.Tensor | None = None) -> rest_kv_desc:
    Nb, H, _, D = k_cache.shape
    d = rest_kv_desc()
    d.Nb, d.H, d.T, d.D, d.P = Nb, H, T, D, prefix_len
    d.pos_offset = prefix_len - 1 if pos_offset is None else pos_offset
    d.per_batch = 1 if per_batch else 0
    if k_cache.dtype == torch.uint8:          # one OCP E4M3 byte per cached element; the new rows arrive as bf16
        assert v_cache.dtype == torch.uint8
        d.dtype, d.cache_dtype = REST_BF16, REST_KV_FP8_E4M3
        for name, t in (("d_k_scale", k_scale), ("d_v_scale", v_scale)):
            if t is not None:
                assert t.dtype == torch.float32 and t.is_contiguous() and t.numel() == Nb * H
                setattr(d, name, t.data_ptr())
    else:
        assert k_scale is None and v_scale is None
        d.dtype = {torch.bfloat16: REST_BF16, torch.float32: REST_FP32}[k_cache.dtype]
        d.cache_dtype = REST_KV_AS_DTYPE
    d.theta = theta
    for name, t in (("q_stride", q), ("kn_stride", k_new), ("vn_stride", v_new), ("kc_stride", k_cache),
                    ("vc_stride", v_cache)):
        if t is not None:
            assert t.stride(3) == 1
            getattr(d, name)[:] = [t.stride(0), t.stride(1), t.stride(2)]
    return d


def rest_rope_append(q: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor, k_cache: torch.Tensor,
                     v_cache: torch.Tensor, pos_ids: torch.Tensor, prefix_len: int, pos_offset: int | None = None,
                     theta: float = 10000.0, k_scale: torch.Tensor | None = None,
                     v_scale: torch.Tensor | None = None) -> None:
    """q, k_new, v_new [Nb,H,T,128]; caches [Nb,H,>=P+T,128] (bf16, device); pos_ids [T] or [Nb,T] int32.
    Rotates q in place and writes the rotated keys and the values to cache rows P .. P+T-1.  Enqueues on the
    current stream."""
    assert q.dim() == 4 and q.shape == k_new.shape == v_new.shape and k_cache.shape == v_cache.shape
    T = q.shape[2]
    assert k_cache.shape[2] >= prefix_len + T and pos_ids.shape[-1] == T and pos_ids.is_contiguous()
    desc = make_kv_desc(k_cache, v_cache, T, prefix_len, pos_offset, theta, pos_ids.dim() == 2, q, k_new, v_new,
                        k_scale, v_scale)
    st = _lib.rest_rope_append(_dev(q), _dev(k_new), _dev(v_new), _dev(k_cache), _dev(v_cache),
                               _dev(pos_ids, torch.int32), ctypes.byref(desc), _stream())
    if st != REST_OK:
        raise RestError(st, "rest_rope_append")


def rest_kv_compact(k_cache: torch.Tensor, v_cache: torch.Tensor, accept_path: torch.Tensor, accept_len: torch.Tensor,
                    T: int, prefix_len: int) -> None:
    """caches [Nb,H,>=P+T,128] (bf16, device); accept_path [path_cap] or [Nb,path_cap], accept_len [1] or [Nb] int32
    as written by rest_accept.  Moves the accepted rows up behind the prefix, in place.  Enqueues on the current
    stream."""
    assert k_cache.shape == v_cache.shape and accept_path.is_contiguous()
    per_batch = accept_path.dim() == 2 and accept_path.shape[0] > 1
    if per_batch:
        assert accept_path.shape[0] == k_cache.shape[0] and accept_len.numel() == k_cache.shape[0]
    desc = make_kv_desc(k_cache, v_cache, T, prefix_len, per_batch=per_batch)
    st = _lib.rest_kv_compact(_dev(k_cache), _dev(v_cache), _dev(accept_path, torch.int32), _dev(accept_len, torch.int32),
                              accept_path.shape[-1], ctypes.byref(desc), _stream())
    if st != REST_OK:
        raise RestError(st, "rest_kv_compact")


def rest_sample_ids_workspace_bytes(R: int, V: int) -> int:
    return _lib.rest_sample_ids_workspace_bytes(R, V)


def rest_sample_ids(logits: torch.Tensor, u: torch.Tensor, temperature: float, top_p: float,
                    out: torch.Tensor | None = None, workspace: torch.Tensor | None = None) -> torch.Tensor:
    """logits [R, V] fp32 (rows may be strided), u [R] fp32 in [0, 1) (device).  Returns ids [R] int32: the nucleus
    sample of every row.  workspace: rest_sample_ids_workspace_bytes(R, V) bytes of device memory (allocated here if
    not given).  Enqueues on the current stream."""
    _require(logits.dim() == 2 and logits.stride(1) == 1 and logits.dtype == torch.float32, "logits must be [R, V] float32, tokens contiguous")
    R, V = logits.shape
    _require(u.numel() == R and u.is_contiguous() and u.dtype == torch.float32, f"u must hold {R} contiguous float32 numbers")
    if out is None:
        out = torch.empty(R, dtype=torch.int32, device=logits.device)
    _require(out.numel() == R and out.dtype == torch.int32 and out.is_contiguous(), f"out must hold {R} contiguous int32 ids")
    need = rest_sample_ids_workspace_bytes(R, V)
    if workspace is None:
        workspace = torch.empty(max(need, 8), dtype=torch.uint8, device=logits.device)
    _require(workspace.is_contiguous() and workspace.numel() * workspace.element_size() >= need, f"workspace smaller than {need} bytes")
    st = _lib.rest_sample_ids(_dev(logits, torch.float32), logits.stride(0) if R > 1 else V, _dev(u, torch.float32), R, V,
                              temperature, top_p, _dev(out, torch.int32), _dev(workspace), workspace.numel() * workspace.element_size(),
                              _stream())
    if st != REST_OK:
        raise RestError(st, "rest_sample_ids")
    return out
