"""TEST INFRASTRUCTURE ONLY: the CPU oracle for REST's draft-and-verify step.

A plain, slow statement of what each stage of the hot path computes, written
from the paper (arXiv 2311.08252) and independent of the GPU library: it
imports nothing from the product package and the product imports nothing from
here.  Only tests, the smoke check and the benchmark's CPU-baseline leg may
use it.

Integer stages (suffix array, Algorithm 1 retrieval, Algorithm 2 Trie
selection, breadth-first pseudo sequence + tree mask, acceptance) live in
rest_oracle.c and are reached through ctypes; tree attention is written here
with numpy in float64.

The steps either side of verification inside one model layer (rotary position
embedding of the draft tokens, appending their keys and values behind the
cached context, keeping the accepted path's rows afterwards) are written here
with numpy in float64 as well; the paper only implies them ("Draft
acceptance": accepted tokens become context), so their exact definition is a
stated reading.

Parity pins: every function below is pinned by tests/test_oracle_*.py against
facts that do not come from this code (textbook suffix arrays, Python's own
substring search and sort, collections.Counter prefix counts, a library
scaled-dot-product attention, closed forms).  The paper prints no worked
numerical example, so no paper-printed values exist to compare with.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rest_oracle.c")
_LIB = os.path.join(_HERE, "librest_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile rest_oracle.c with gcc into librest_oracle.so next to it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", _LIB, _SRC])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_check_suffix_array.restype = ctypes.c_int64
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _token_bytes(corpus: np.ndarray) -> int:
    if corpus.dtype == np.int32:
        return 4
    if corpus.dtype == np.uint16:
        return 2
    raise TypeError("corpus must be int32 or uint16")


# ---------------------------------------------------------------------------
# Suffix array ("Retrieving from the datastore": exact match via a suffix array)
# ---------------------------------------------------------------------------
def suffix_array(corpus: np.ndarray) -> np.ndarray:
    """int64 suffix array by sorting all suffixes (end of stream smallest)."""
    corpus = np.ascontiguousarray(corpus)
    sa = np.empty(corpus.shape[0], dtype=np.int64)
    rc = _load().oracle_suffix_array(_ptr(corpus), ctypes.c_uint64(corpus.shape[0]),
                                     _token_bytes(corpus), _ptr(sa))
    assert rc == 0
    return sa


def prefix_sorted_array(corpus: np.ndarray, depth: int) -> np.ndarray:
    """The depth-limited index: all positions ordered by their first `depth` tokens only (the end of the
    stream smaller than every token), positions with equal such prefixes in ascending position order.
    Algorithm 1 looks at no more than n_max tokens of a suffix and Algorithm 2 at the cont_len after
    them, so for depth >= n_max + cont_len this array serves every retrieval exactly as the suffix array
    does ("Retrieving from the datastore")."""
    corpus = np.ascontiguousarray(corpus)
    n, depth = corpus.shape[0], int(depth)
    assert depth >= 1
    tok = np.concatenate([corpus.astype(np.int64) + 1, np.zeros(depth, dtype=np.int64)])
    columns = [tok[j:j + n] for j in range(depth)]
    return np.lexsort(columns[::-1]).astype(np.int64)      # stable: the last key given is the primary one


def check_suffix_array(corpus: np.ndarray, sa: np.ndarray) -> int:
    """-1 if `sa` is the suffix array of `corpus` by definition (a permutation
    whose adjacent suffixes strictly increase), else the first bad rank."""
    corpus = np.ascontiguousarray(corpus)
    sa = np.ascontiguousarray(sa)
    assert sa.dtype in (np.int32, np.int64) and sa.shape[0] == corpus.shape[0]
    return int(_load().oracle_check_suffix_array(_ptr(corpus), ctypes.c_uint64(corpus.shape[0]),
                                                 _token_bytes(corpus), _ptr(sa), sa.dtype.itemsize))


# ---------------------------------------------------------------------------
# Algorithm 1: Retrieve(D, s)
# ---------------------------------------------------------------------------
@dataclass
class Retrieved:
    matched_len: int          # n of the longest matching suffix (0: none)
    match_count: int          # number of occurrences of that suffix
    row_pos: np.ndarray       # [R] stream position of each kept occurrence, suffix order
    rows: np.ndarray          # [R, m] continuation tokens, -1 padded
    row_len: np.ndarray       # [R]


def retrieve(corpus: np.ndarray, context: np.ndarray, n_max: int = 16, n_min: int = 2,
             max_matches: int = 5000, cont_len: int = 10, one_pass: bool = False,
             strided: bool = False) -> Retrieved:
    """Algorithm 1.  The paper only says that the set S of matches can be large; which max_matches of
    them are kept is a choice of this implementation: the first max_matches in suffix order, or, with
    strided=True, an evenly spaced sample of the whole sorted range: of S occurrences in suffix order,
    number i of the K kept ones is occurrence floor(i * S / K) (all of them if S <= K)."""
    if strided:
        count = retrieve(corpus, context, n_max, n_min, 0, cont_len, one_pass).match_count
        full = retrieve(corpus, context, n_max, n_min, max(count, 1), cont_len, one_pass)
        S, K = full.rows.shape[0], int(max_matches)
        if S <= K:
            return full
        pick = np.array([(i * S) // K for i in range(K)], dtype=np.int64)
        return Retrieved(full.matched_len, full.match_count, full.row_pos[pick], full.rows[pick], full.row_len[pick])
    corpus = np.ascontiguousarray(corpus)
    s = np.ascontiguousarray(context, dtype=np.int32)
    K, m = int(max_matches), int(cont_len)
    ml = ctypes.c_int32(0)
    mc = ctypes.c_int64(0)
    nr = ctypes.c_int64(0)
    row_pos = np.zeros(K, dtype=np.int64)
    rows = np.full((K, max(m, 1)), -1, dtype=np.int32)
    row_len = np.zeros(K, dtype=np.int32)
    rc = _load().oracle_retrieve(_ptr(corpus), ctypes.c_uint64(corpus.shape[0]), _token_bytes(corpus),
                                 _ptr(s), ctypes.c_int32(s.shape[0]),
                                 ctypes.c_int32(n_max), ctypes.c_int32(n_min), ctypes.c_int64(K),
                                 ctypes.c_int32(m), ctypes.c_int32(1 if one_pass else 0),
                                 ctypes.byref(ml), ctypes.byref(mc), ctypes.byref(nr),
                                 _ptr(row_pos), _ptr(rows), _ptr(row_len))
    assert rc == 0, rc
    R = nr.value
    return Retrieved(ml.value, mc.value, row_pos[:R].copy(), rows[:R, :m].copy(), row_len[:R].copy())


# ---------------------------------------------------------------------------
# Algorithm 2 + breadth-first pseudo sequence + tree attention mask
# ---------------------------------------------------------------------------
@dataclass
class DraftTree:
    n_nodes: int
    draft_tokens: np.ndarray   # [c] int32, -1 padded
    parent_idx: np.ndarray     # [c] int32, -1 = child of the last context token (and padding)
    pos_ids: np.ndarray        # [c] int32 depth, 0 padded
    node_weight: np.ndarray    # [c] int32
    tree_mask: np.ndarray      # [c, ceil(c/64)] uint64
    matched_len: int = 0
    match_count: int = 0
    total_trie_nodes: int = 0


def select_drafts(rows: np.ndarray, row_len: np.ndarray, max_nodes: int,
                  order: np.ndarray | None = None) -> DraftTree:
    """Trie over all prefixes of all rows, the max_nodes heaviest nodes, laid
    out breadth first with the mask.  `order` is the insertion order of the
    rows (default: as given)."""
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    row_len = np.ascontiguousarray(row_len, dtype=np.int32)
    R = rows.shape[0]
    m = rows.shape[1] if rows.ndim == 2 else 0
    c = int(max_nodes)
    words = max(1, (c + 63) // 64)
    n = ctypes.c_int32(0)
    tot = ctypes.c_int64(0)
    tok = np.zeros(max(c, 1), dtype=np.int32)
    par = np.zeros(max(c, 1), dtype=np.int32)
    pos = np.zeros(max(c, 1), dtype=np.int32)
    wgt = np.zeros(max(c, 1), dtype=np.int32)
    mask = np.zeros((max(c, 1), words), dtype=np.uint64)
    if order is not None:
        order = np.ascontiguousarray(order, dtype=np.int64)
        assert order.shape[0] == R
    if m == 0:
        rows = np.zeros((max(R, 1), 1), dtype=np.int32)
    rc = _load().oracle_select_drafts(_ptr(rows), _ptr(row_len),
                                      _ptr(order) if order is not None else None,
                                      ctypes.c_int64(R), ctypes.c_int32(max(m, 1)),
                                      ctypes.c_int32(c), ctypes.c_int32(words),
                                      ctypes.byref(n), _ptr(tok), _ptr(par), _ptr(pos), _ptr(wgt),
                                      _ptr(mask), ctypes.byref(tot))
    assert rc == 0, rc
    return DraftTree(n.value, tok[:c], par[:c], pos[:c], wgt[:c], mask[:c], 0, 0, tot.value)


def _mix64(z: int) -> int:
    z &= (1 << 64) - 1
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & ((1 << 64) - 1)
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & ((1 << 64) - 1)
    return z ^ (z >> 31)


def random_rows(n_rows: int, n_seq: int, seed: int, ctx_index: int) -> np.ndarray:
    """The candidates drawn by the random-selection strategy the paper compares the Trie with
    ("Effect of draft token selecting strategies": at most eight sequences sampled from all
    retrieved candidates).  The draws are the method's random numbers, so their generator is
    part of the definition and counter based: with G = 0x9E3779B97F4A7C15 and mix = the
    splitmix64 finaliser, h = mix(seed + G*(1 + ctx_index)), U_j = mix(h + G*(1 + j)) for
    j < n_seq, and draw j is candidate floor(U_j * n_rows / 2^64).  Equal draws collapse.
    Returns the distinct candidate indices in ascending order."""
    G = 0x9E3779B97F4A7C15
    h = _mix64(seed + G * (1 + ctx_index))
    picks = {(_mix64(h + G * (1 + j)) * n_rows) >> 64 for j in range(n_seq)} if n_rows > 0 else set()
    return np.array(sorted(picks), dtype=np.int64)


def draft_tree(corpus: np.ndarray, context: np.ndarray, n_max: int = 16, n_min: int = 2,
               max_matches: int = 5000, cont_len: int = 10, max_nodes: int = 64,
               one_pass: bool = False, random_seqs: int = 0, seed: int = 0, ctx_index: int = 0,
               strided: bool = False) -> DraftTree:
    """One context -> draft tree: Algorithm 1, then Algorithm 2 with the
    candidates inserted in stream-position order, then the layout.
    random_seqs > 0: the ablation's strategy instead -- only random_seqs randomly drawn
    candidates (each already cut to cont_len tokens) go into the Trie."""
    got = retrieve(corpus, context, n_max, n_min, max_matches, cont_len, one_pass, strided)
    if random_seqs > 0:
        sel = random_rows(got.rows.shape[0], random_seqs, seed, ctx_index)
        got = Retrieved(got.matched_len, got.match_count, got.row_pos[sel], got.rows[sel], got.row_len[sel])
    order = np.argsort(got.row_pos, kind="stable").astype(np.int64)
    tree = select_drafts(got.rows, got.row_len, max_nodes, order)
    tree.matched_len = got.matched_len
    tree.match_count = got.match_count
    return tree


def mask_from_parents(parent_idx: np.ndarray, n_nodes: int, words: int | None = None) -> np.ndarray:
    """Tree attention mask from parent pointers: row i has bit j set iff j is i
    or an ancestor of i ("Draft verification")."""
    c = parent_idx.shape[0]
    words = words or max(1, (c + 63) // 64)
    mask = np.zeros((c, words), dtype=np.uint64)
    for i in range(n_nodes):
        v = i
        while v != -1:
            mask[i, v // 64] |= np.uint64(1) << np.uint64(v % 64)
            v = int(parent_idx[v])
    return mask


# ---------------------------------------------------------------------------
# The index file ("Datastore construction": built once, reused): a 64-byte
# little-endian header -- "RESTSA01", n_tokens u64, token_bytes i32, sa_bytes
# i32, fingerprint u64, sort depth i32 (0 = a full suffix array, else the number
# of tokens the positions are ordered by), zeros -- then the array.  The fingerprint ties
# the array to its token stream: the sum over i of
# splitmix64-finaliser(token_i + (i+1) * 0x9E3779B97F4A7C15) modulo 2^64.
# ---------------------------------------------------------------------------
def corpus_fingerprint(corpus: np.ndarray) -> int:
    M = np.uint64
    total = M(0)
    with np.errstate(over="ignore"):
        for c0 in range(0, corpus.size, 1 << 24):
            tok = corpus[c0:c0 + (1 << 24)].astype(np.uint64)
            z = tok + (np.arange(c0 + 1, c0 + 1 + tok.size, dtype=np.uint64)) * M(0x9E3779B97F4A7C15)
            z = (z ^ (z >> M(30))) * M(0xBF58476D1CE4E5B9)
            z = (z ^ (z >> M(27))) * M(0x94D049BB133111EB)
            z = z ^ (z >> M(31))
            total = total + np.add.reduce(z, dtype=np.uint64)
    return int(total)


def write_index_file(path: str, corpus: np.ndarray, sa: np.ndarray, sort_depth: int = 0) -> None:
    import struct
    assert sa.dtype in (np.int32, np.int64) and sa.size == corpus.size
    with open(path, "wb") as f:
        f.write(b"RESTSA01" + struct.pack("<QiiQi", corpus.size, _token_bytes(corpus), sa.dtype.itemsize,
                                          corpus_fingerprint(corpus), sort_depth) + bytes(28))
        f.write(np.ascontiguousarray(sa).tobytes())


def read_index_file(path: str):
    """Returns (n_tokens, token_bytes, sa_bytes, fingerprint, array, sort depth)."""
    import struct
    with open(path, "rb") as f:
        head = f.read(64)
        assert len(head) == 64 and head[:8] == b"RESTSA01" and head[36:] == bytes(28)
        n, tb, sb, fp, depth = struct.unpack("<QiiQi", head[8:36])
        sa = np.frombuffer(f.read(), dtype=np.int32 if sb == 4 else np.int64)
    assert sa.size == n and depth >= 0
    return n, tb, sb, fp, sa, depth


# ---------------------------------------------------------------------------
# Tree attention ("Draft verification"): every draft token attends to the whole
# cached context and, among the draft tokens, only to itself and its ancestors.
# ---------------------------------------------------------------------------
def tree_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, mask: np.ndarray,
                   prefix_len: int, scale: float) -> np.ndarray:
    """float64 softmax attention with the tree mask, by the definition.

    q [..., Tq, D]; k, v [..., P+Tk, D] (exact values of the inputs, any float
    dtype, promoted to float64); mask [Tq, ceil(Tk/64)] uint64 shared by all
    leading dims, or [..., Tq, words] matching them.  Query row i sees keys
    0..P-1 and key P+j iff bit j of mask row i is set.  Returns float64
    [..., Tq, D]."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    Tq = q.shape[-2]
    Lk = k.shape[-2]
    P = int(prefix_len)
    Tk = Lk - P
    bits = np.zeros(mask.shape[:-1] + (Lk,), dtype=bool)
    bits[..., :P] = True
    for j in range(Tk):
        bits[..., P + j] = (mask[..., j // 64] >> np.uint64(j % 64)) & np.uint64(1) != 0
    assert bits.shape[-2] == Tq
    s = scale * np.matmul(q, np.swapaxes(k, -1, -2))
    s = np.where(bits, s, -np.inf)
    s = s - np.max(s, axis=-1, keepdims=True)
    p = np.exp(s)
    p = p / np.sum(p, axis=-1, keepdims=True)
    return np.matmul(p, v)


# ---------------------------------------------------------------------------
# 8-bit KV cache.  Not in the paper: the cache may hold K and V in the OCP 8-bit
# floating point format E4M3 (1 sign bit, 4 exponent bits with bias 7, 3 mantissa
# bits; exponent field 0 = subnormals m * 2^-9; no infinities; S.1111.111 = NaN;
# largest finite value 448), each (batch, head) slab with one float scale:
# k = k_scale * decode(k8), v = v_scale * decode(v8).  Attention on such a cache
# is, by definition, the attention above on those decoded values.
# ---------------------------------------------------------------------------
def fp8_e4m3_decode(codes: np.ndarray) -> np.ndarray:
    codes = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    sign = np.where(codes & 0x80, -1.0, 1.0)
    e, m = (codes >> 3) & 15, codes & 7
    val = np.where(e == 0, m * 2.0 ** -9, (1.0 + m / 8.0) * 2.0 ** (e.astype(np.float64) - 7))
    val = np.where((e == 15) & (m == 7), np.nan, val)
    return sign * val


def fp8_e4m3_encode(x: np.ndarray) -> np.ndarray:
    """Nearest E4M3 value, ties to the even mantissa, magnitudes beyond 448 saturate to 448, NaN -> 0x7f."""
    x = np.asarray(x, dtype=np.float64)
    grid = fp8_e4m3_decode(np.arange(0x7f))                       # the 127 finite magnitudes, ascending with the code
    a = np.abs(np.nan_to_num(x, nan=0.0))
    hi = np.clip(np.searchsorted(grid, a, side="left"), 1, 0x7e)  # grid[hi-1] <= a <= grid[hi] (or a beyond the ends)
    lo = hi - 1
    d_lo, d_hi = a - grid[lo], grid[hi] - a
    code = np.where(d_lo < d_hi, lo, np.where(d_hi < d_lo, hi, np.where(lo % 2 == 0, lo, hi)))
    code = np.where(np.signbit(x), code | 0x80, code)
    return np.where(np.isnan(x), 0x7f, code).astype(np.uint8)


def tree_attention_fp8kv(q: np.ndarray, k8: np.ndarray, v8: np.ndarray, k_scale, v_scale, mask: np.ndarray,
                         prefix_len: int, scale: float) -> np.ndarray:
    """q [Nb, H, Tq, D] (any float dtype); k8, v8 [Nb, H, P+Tk, D] uint8 E4M3 codes; k_scale, v_scale [Nb, H]."""
    k = fp8_e4m3_decode(k8) * np.asarray(k_scale, dtype=np.float64)[..., None, None]
    v = fp8_e4m3_decode(v8) * np.asarray(v_scale, dtype=np.float64)[..., None, None]
    return tree_attention(q, k, v, mask, prefix_len, scale)


def tree_attention_loops(q, k, v, mask, prefix_len: int, scale: float) -> np.ndarray:
    """The same definition as explicit Python loops for one [Tq, D] / [Lk, D]
    slab (small cases only)."""
    import math
    Tq, D = q.shape
    Lk = k.shape[0]
    P = prefix_len
    out = np.zeros((Tq, D), dtype=np.float64)
    for i in range(Tq):
        vis = [j for j in range(Lk)
               if j < P or (int(mask[i, (j - P) // 64]) >> ((j - P) % 64)) & 1]
        logits = [scale * sum(float(q[i, d]) * float(k[j, d]) for d in range(D)) for j in vis]
        mx = max(logits)
        e = [math.exp(x - mx) for x in logits]
        z = sum(e)
        for w, j in zip(e, vis):
            for d in range(D):
                out[i, d] += (w / z) * float(v[j, d])
    return out


# ---------------------------------------------------------------------------
# Around verification, inside one layer.  "Draft verification" builds the
# pseudo sequence and its mask but leaves positions unsaid; "Draft acceptance"
# turns accepted draft tokens into context.  For a model with rotary position
# embedding and a key/value cache that means: a draft node at depth d behind a
# context whose last token has position p0 is embedded at position p0 + d; its
# key and value are appended behind the cached context so that verification
# can read them; and after acceptance the accepted path's rows are the ones
# that stay, moved up to directly follow the context.
# ---------------------------------------------------------------------------
def rope(x: np.ndarray, positions: np.ndarray, theta: float = 10000.0) -> np.ndarray:
    """Rotary position embedding (Su et al., RoFormer) in the half-split layout
    of the Llama-family models the paper evaluates: with h = D/2, components
    (i, i+h) of row t form a plane vector that is rotated by the angle
    positions[t] * theta**(-2i/D).  x [..., T, D]; positions [T] or matching
    the leading dims [..., T]; returns float64."""
    x = np.asarray(x, dtype=np.float64)
    D = x.shape[-1]
    h = D // 2
    assert 2 * h == D
    freq = theta ** (-2.0 * np.arange(h, dtype=np.float64) / D)
    ang = np.asarray(positions, dtype=np.float64)[..., None] * freq
    c, s = np.cos(ang), np.sin(ang)
    a, b = x[..., :h], x[..., h:]
    return np.concatenate([a * c - b * s, a * s + b * c], axis=-1)


def rope_append(q, k_new, v_new, k_cache, v_cache, pos_ids, pos_offset: int, prefix_len: int,
                theta: float = 10000.0):
    """One layer's step before verification.  q, k_new, v_new [..., T, D] belong to
    the T draft tokens, pos_ids [T] (or [..., T]) are their depths; caches
    [..., L, D] with L >= prefix_len + T.  Returns (q embedded, k_cache with the
    embedded keys in rows prefix_len .. prefix_len+T-1, v_cache with the values
    there), all float64; other cache rows are unchanged."""
    pos = np.asarray(pos_ids, dtype=np.int64) + int(pos_offset)
    T = np.asarray(q).shape[-2]
    P = int(prefix_len)
    qr = rope(q, pos, theta)
    kc = np.array(k_cache, dtype=np.float64, copy=True)
    vc = np.array(v_cache, dtype=np.float64, copy=True)
    kc[..., P:P + T, :] = rope(k_new, pos, theta)
    vc[..., P:P + T, :] = np.asarray(v_new, dtype=np.float64)
    return qr, kc, vc


def rope_append_fp8kv(q, k_new, v_new, k_cache8, v_cache8, k_scale, v_scale, pos_ids, pos_offset: int,
                      prefix_len: int, theta: float = 10000.0):
    """The same step on an 8-bit cache: the embedded key divided by its slab's k_scale, and the value
    divided by v_scale, are stored as the nearest E4M3 codes (saturating).  q, k_new, v_new [Nb, H, T, D];
    caches [Nb, H, L, D] uint8; scales [Nb, H].  Returns (q embedded float64, k cache, v cache, and the two
    exact quotients [Nb, H, T, D] the new codes were rounded from)."""
    pos = np.asarray(pos_ids, dtype=np.int64) + int(pos_offset)
    if pos.ndim == 2:
        pos = pos[:, None, :]                       # [Nb, T]: shared by the heads
    T = np.asarray(q).shape[-2]
    P = int(prefix_len)
    kx = rope(k_new, pos, theta) / np.asarray(k_scale, dtype=np.float64)[..., None, None]
    vx = np.asarray(v_new, dtype=np.float64) / np.asarray(v_scale, dtype=np.float64)[..., None, None]
    kc = np.array(k_cache8, dtype=np.uint8, copy=True)
    vc = np.array(v_cache8, dtype=np.uint8, copy=True)
    kc[..., P:P + T, :] = fp8_e4m3_encode(kx)
    vc[..., P:P + T, :] = fp8_e4m3_encode(vx)
    return rope(q, pos, theta), kc, vc, kx, vx


def kv_compact(cache: np.ndarray, prefix_len: int, accept_path: np.ndarray, accept_len: int) -> np.ndarray:
    """After acceptance: row prefix_len + i of the result is row prefix_len +
    accept_path[i] of the input for i < accept_len; every other row is
    unchanged (rows from prefix_len + accept_len on are dead).  cache [..., L, D]."""
    out = np.array(cache, copy=True)
    P = int(prefix_len)
    for i in range(int(accept_len)):
        out[..., P + i, :] = cache[..., P + int(accept_path[i]), :]
    return out


# ---------------------------------------------------------------------------
# Acceptance ("Draft acceptance of REST")
# ---------------------------------------------------------------------------
def accept(ids: np.ndarray, draft_tokens: np.ndarray, parent_idx: np.ndarray, n_nodes: int,
           path_cap: int):
    """ids[0] = model token after the context, ids[1+i] = after node i.
    Returns (accept_len, accept_path[path_cap] node indices -1 padded, next_token)."""
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    tok = np.ascontiguousarray(draft_tokens, dtype=np.int32)
    par = np.ascontiguousarray(parent_idx, dtype=np.int32)
    al = ctypes.c_int32(0)
    nt = ctypes.c_int32(0)
    path = np.full(max(path_cap, 1), -1, dtype=np.int32)
    rc = _load().oracle_accept(_ptr(ids), _ptr(tok), _ptr(par), ctypes.c_int32(n_nodes),
                               ctypes.c_int32(path_cap), ctypes.byref(al), _ptr(path), ctypes.byref(nt))
    assert rc == 0
    return al.value, path[:path_cap], nt.value


# ---------------------------------------------------------------------------
# Nucleus sampling ("Sampling strategies"): the model's token at a position is
# drawn from the most probable tokens whose cumulative probability reaches the
# threshold p; REST accepts a draft token only if it equals the token sampled
# at its position, so acceptance is the same walk as in the greedy case on
# sampled ids.  The paper fixes temperature and top-p (Table 1 caption) but not
# the mechanics.  The reading here fixes them down to the last bit, so that an
# integer result (a token id) has one right answer whatever the order in which
# an implementation adds things up:
#   * probability masses are integers.  Token i weighs
#       w_i = floor(2^36 * E((x_i - x_max) * c)),   c = log2(e) / temperature,
#     where E(y) = 2^y is evaluated by a fixed sequence of float64 operations
#     (below), every one of them a single correctly rounded IEEE operation; the
#     most probable token weighs exactly 2^36, a token below 2^-36 of it
#     nothing.  Sums of such weights are exact (below 2^53 for up to 2^17
#     tokens), hence independent of the order of summation;
#   * tokens are ordered by logit, highest first (+0 and -0 are one value),
#     equal logits by ascending token id;
#   * the nucleus is the shortest prefix of that order whose mass C_k satisfies
#     float64(C_k) >= float32(top_p) * float64(W), W the total mass (one
#     float64 product);
#   * the draw is the first token whose cumulative mass satisfies
#     float64(C_j) > float32(u) * float64(M), M the nucleus mass, u in [0, 1)
#     the caller's uniform number.
# E(y) for y <= 0: n = floor(y), f = y - n in [0, 1), t = f * ln 2,
# E = 2^n * P(t), P the Taylor polynomial of exp of degree 13 in Horner form,
# each step one multiplication and one addition (no fused multiply-add);
# E(0) = 1 exactly.  |E(y) / 2^y - 1| < 1e-12, far below the weights' own step.
# ---------------------------------------------------------------------------
SAMPLE_WEIGHT_BITS = 36
_LOG2E = float.fromhex("0x1.71547652b82fep+0")
_LN2 = float.fromhex("0x1.62e42fefa39efp-1")
_EXP_TAYLOR = [float.fromhex(h) for h in (
    "0x1.0000000000000p+0", "0x1.0000000000000p+0", "0x1.0000000000000p-1", "0x1.5555555555555p-3",
    "0x1.5555555555555p-5", "0x1.1111111111111p-7", "0x1.6c16c16c16c17p-10", "0x1.a01a01a01a01ap-13",
    "0x1.a01a01a01a01ap-16", "0x1.71de3a556c734p-19", "0x1.27e4fb7789f5cp-22", "0x1.ae64567f544e4p-26",
    "0x1.1eed8eff8d898p-29", "0x1.6124613a86d09p-33")]   # 1 / k!, k = 0 .. 13


def nucleus_weights(logits: np.ndarray, temperature: float) -> np.ndarray:
    """Integer probability masses of one row (uint64), in units of 2^-36 of the largest probability."""
    x = np.asarray(logits, dtype=np.float32)
    c = np.float64(_LOG2E) / np.float64(np.float32(temperature))
    y = (x.astype(np.float64) - np.float64(x.max())) * c
    live = y >= -64.0                                     # below: less than 2^-64 of the largest, weight 0 (also -inf)
    y = np.where(live, y, 0.0)
    n = np.floor(y)
    t = (y - n) * np.float64(_LN2)
    poly = np.full_like(t, _EXP_TAYLOR[13])
    for k in range(12, -1, -1):
        poly = poly * t                                   # two separately rounded operations per step
        poly = poly + np.float64(_EXP_TAYLOR[k])
    w = np.floor(np.ldexp(poly, (n + SAMPLE_WEIGHT_BITS).astype(np.int32)))
    return np.where(live, w, 0.0).astype(np.uint64)


def nucleus_sample(logits: np.ndarray, temperature: float, top_p: float, u: float):
    """Returns (token, margin).  margin is the distance, as a fraction of the total mass, between the decision
    thresholds (top_p for the nucleus boundary, u * nucleus mass for the draw) and the nearest cumulative sum (a
    diagnostic: the result itself is exact)."""
    x = np.asarray(logits, dtype=np.float32)
    w = nucleus_weights(x, temperature)
    order = np.lexsort((np.arange(x.size), -x))          # logit descending, token id ascending
    cum = np.cumsum(w[order])                             # exact integers
    total = cum[-1]
    thr = np.float64(np.float32(top_p)) * np.float64(total)
    k = int(np.nonzero(cum.astype(np.float64) >= thr)[0][0])
    mass = cum[k]
    target = np.float64(np.float32(u)) * np.float64(mass)
    j = int(np.nonzero(cum.astype(np.float64) > target)[0][0])
    c64 = cum[:k + 1].astype(np.float64)
    margin = min(np.abs(c64 - thr).min(), np.abs(c64 - target).min()) / float(total)
    return int(order[j]), float(margin)


def sample_ids(logits: np.ndarray, temperature: float, top_p: float, u: np.ndarray):
    """logits [R, V], u [R] -> (ids [R] int32, margins [R])."""
    out = [nucleus_sample(logits[r], temperature, top_p, u[r]) for r in range(logits.shape[0])]
    return np.array([t for t, _ in out], dtype=np.int32), np.array([m for _, m in out])


# ---------------------------------------------------------------------------
# The decoding loop the acceptance rule is claimed to preserve: with a
# deterministic next-token function, REST's draft/verify/accept loop must emit
# exactly the tokens of one-token-at-a-time greedy decoding.
# ---------------------------------------------------------------------------
def greedy_decode(next_token_fn, prompt, n_new: int):
    seq = list(int(x) for x in prompt)
    for _ in range(n_new):
        seq.append(int(next_token_fn(seq)))
    return seq[len(prompt):]


def rest_decode(next_token_fn, prompt, n_new: int, corpus: np.ndarray, n_max=16, n_min=2,
                max_matches=1000, cont_len=10, max_nodes=32):
    """Returns (generated tokens, number of verification steps)."""
    seq = list(int(x) for x in prompt)
    base = len(seq)
    steps = 0
    while len(seq) - base < n_new:
        tree = draft_tree(corpus, np.asarray(seq, dtype=np.int32), n_max, n_min,
                          max_matches, cont_len, max_nodes)
        # one "forward pass": the model's token at the root and after every draft node
        ids = np.zeros(1 + max_nodes, dtype=np.int32)
        ids[0] = next_token_fn(seq)
        for i in range(tree.n_nodes):
            path, v = [], i
            while v != -1:
                path.append(int(tree.draft_tokens[v]))
                v = int(tree.parent_idx[v])
            ids[1 + i] = next_token_fn(seq + path[::-1])
        n_acc, path, nxt = accept(ids, tree.draft_tokens, tree.parent_idx, tree.n_nodes, cont_len)
        for j in range(n_acc):
            seq.append(int(tree.draft_tokens[path[j]]))
        seq.append(int(nxt))
        steps += 1
    return seq[base:base + n_new], steps
