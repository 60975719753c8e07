"""Seeded synthetic inputs for the REST draft-and-verify hot path.

This module only manufactures inputs (corpora, query contexts, random tree
shapes, Q/K/V tensors, sampled token ids).  It holds none of the method's
arithmetic: no suffix search, no Trie counting, no attention, no acceptance.
Both the CPU oracle's tests and the GPU path's tests/benchmarks draw their
inputs from here so that the two sides see identical bytes.

All randomness is counter based: value = f(splitmix64(seed, index)), so any
slice of any stream can be regenerated independently and in any order.

The corpora stand in for the paper's datastores (code / chat corpora,
"Datastores" paragraph of the experimental setup), which are not available:
tokens follow a Zipf(1.1) law over a 32000-word vocabulary with a small
fraction of planted, repeated motifs so that long exact matches exist, which
is what makes the matched-suffix-length mix resemble the one the paper shows
in its "matched suffix length" appendix figure.
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np

_U64 = np.uint64
_GOLDEN = _U64(0x9E3779B97F4A7C15)
_M1 = _U64(0xBF58476D1CE4E5B9)
_M2 = _U64(0x94D049BB133111EB)


def splitmix64(seed: int, index) -> np.ndarray:
    """Counter-based 64-bit hash: the splitmix64 output function applied to
    seed * golden + (index + 1) * golden (wrapping)."""
    idx = np.asarray(index, dtype=_U64)
    with np.errstate(over="ignore"):
        z = (idx + _U64(1)) * _GOLDEN + _U64(seed & 0xFFFFFFFFFFFFFFFF) * _M2
        z = (z ^ (z >> _U64(30))) * _M1
        z = (z ^ (z >> _U64(27))) * _M2
        z = z ^ (z >> _U64(31))
    return z


def uniform01(seed: int, index) -> np.ndarray:
    """float64 uniform in [0, 1) from the top 53 bits of splitmix64."""
    return (splitmix64(seed, index) >> _U64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)


def randint(seed: int, index, lo: int, hi: int) -> np.ndarray:
    """Integers uniform in [lo, hi) (hi - lo << 2**53, bias negligible)."""
    u = uniform01(seed, index)
    return (lo + np.floor(u * (hi - lo))).astype(np.int64)


class TokenLaw:
    """Zipf token law: rank r in [1, vocab] with P(r) ~ r**-s, mapped to token
    id (r * 7919 + 13) mod vocab so id order is not frequency order."""

    def __init__(self, vocab: int = 32000, s: float = 1.1):
        assert math.gcd(7919, vocab) == 1
        self.vocab = vocab
        self.s = s
        w = np.arange(1, vocab + 1, dtype=np.float64) ** (-s)
        self.cdf = np.cumsum(w) / np.sum(w)
        self.cdf[-1] = 1.0

    def tokens(self, seed: int, start: int, count: int) -> np.ndarray:
        """Tokens number start .. start+count of stream `seed` (int64)."""
        idx = np.arange(start, start + count, dtype=_U64)
        u = uniform01(seed, idx)
        r = np.searchsorted(self.cdf, u, side="right") + 1
        np.minimum(r, self.vocab, out=r)
        return (r * 7919 + 13) % self.vocab


@dataclass
class Corpus:
    tokens: np.ndarray            # [N] int32 or uint16
    motif_offsets: np.ndarray     # [n_motifs, copies] int64 start offset of each planted copy
    motif_lengths: np.ndarray     # [n_motifs] int64
    vocab: int


def make_corpus(n_tokens: int, seed: int, n_motifs: int, copies: int = 50,
                vocab: int = 32000, dtype=np.int32, motif_len=(8, 64),
                workers: int = 8) -> Corpus:
    """i.i.d. Zipf tokens, then `n_motifs` motifs (length uniform in
    motif_len, inclusive) each overwritten at `copies` uniform offsets, in
    generation order (later plants overwrite earlier ones)."""
    law = TokenLaw(vocab)
    out = np.empty(n_tokens, dtype=dtype)
    chunk = 1 << 22

    def fill(c0):
        c1 = min(n_tokens, c0 + chunk)
        out[c0:c1] = law.tokens(seed, c0, c1 - c0).astype(dtype)

    starts = list(range(0, n_tokens, chunk))
    if len(starts) > 1 and workers > 1:
        with ThreadPoolExecutor(workers) as ex:
            list(ex.map(fill, starts))
    else:
        for c0 in starts:
            fill(c0)

    lo, hi = motif_len
    hi = min(hi, n_tokens)
    lo = min(lo, hi)
    lengths = randint(seed + 1000003, np.arange(n_motifs), lo, hi + 1) if n_motifs else np.zeros(0, np.int64)
    offsets = np.zeros((n_motifs, copies), dtype=np.int64)
    tok_cursor = 0
    for j in range(n_motifs):
        L = int(lengths[j])
        motif = law.tokens(seed + 2000003, tok_cursor, L).astype(dtype)
        tok_cursor += L
        u = uniform01(seed + 3000017, np.arange(j * copies, (j + 1) * copies))
        offs = np.floor(u * (n_tokens - L + 1)).astype(np.int64)
        offsets[j] = offs
        for o in offs:
            out[o:o + L] = motif
    return Corpus(out, offsets, lengths, vocab)


def make_contexts(corpus: Corpus, batch: int, ctx_len: int, seed: int):
    """[batch, ctx_len] int32 contexts and [batch] int32 lengths.

    Even rows are copied from the corpus (every other one of them ends inside
    a planted motif copy, at least 4 tokens before the copy's end, when the
    corpus has motifs; the rest end at a uniform position); odd rows are
    i.i.d. from the token law."""
    law = TokenLaw(corpus.vocab)
    N = corpus.tokens.shape[0]
    ctx = np.zeros((batch, ctx_len), dtype=np.int32)
    n_m = corpus.motif_lengths.shape[0]
    for b in range(batch):
        if b % 2 == 1:
            ctx[b] = law.tokens(seed + 7, b * ctx_len, ctx_len).astype(np.int32)
            continue
        u = uniform01(seed, np.arange(b * 4, b * 4 + 4))
        e = None
        if n_m > 0 and (b // 2) % 2 == 0:
            j = int(u[0] * n_m)
            k = int(u[1] * corpus.motif_offsets.shape[1])
            L = int(corpus.motif_lengths[j])
            o = int(corpus.motif_offsets[j, k])
            back = 4 + int(u[2] * max(1, L - 4 - 2))
            e = o + L - min(back, L - 1)
        if e is None:
            e = int(u[3] * N)
        e = max(1, min(N, e))
        take = min(ctx_len, e)
        row = corpus.tokens[e - take:e].astype(np.int32)
        if take < ctx_len:
            pad = law.tokens(seed + 11, b * ctx_len, ctx_len - take).astype(np.int32)
            row = np.concatenate([pad, row])
        ctx[b] = row
    lens = np.full(batch, ctx_len, dtype=np.int32)
    return ctx, lens


def random_tree(n_nodes: int, seed: int, max_children: int = 8, max_depth: int = 16):
    """Random draft-tree shape: nodes are attached one at a time to a uniformly
    chosen eligible node (the virtual root, index -1, or an existing node with
    depth < max_depth and fewer than max_children children), then relabelled
    breadth first (by depth, then by creation order within a parent chain).

    Returns (parent[n_nodes] int32 with -1 for children of the root,
    depth[n_nodes] int32 1-based, tokens[n_nodes] int32 distinct among siblings,
    mask[n_nodes, ceil(n/64)] uint64 with bit j of row i set iff j == i or j
    is an ancestor of i)."""
    parent = []
    depth = []
    nchild = {-1: 0}
    for i in range(n_nodes):
        elig = [v for v in range(-1, i)
                if nchild.get(v, 0) < max_children and (v == -1 or depth[v] < max_depth)]
        u = float(uniform01(seed, np.asarray([i]))[0])
        v = elig[int(u * len(elig))]
        parent.append(v)
        depth.append(1 if v == -1 else depth[v] + 1)
        nchild[v] = nchild.get(v, 0) + 1
        nchild[i] = 0
    # breadth-first relabel: order by (depth, path of creation indices)
    paths = []
    for i in range(n_nodes):
        p, v = [], i
        while v != -1:
            p.append(v)
            v = parent[v]
        paths.append(tuple(reversed(p)))
    order = sorted(range(n_nodes), key=lambda i: (depth[i], paths[i]))
    new_of = {old: new for new, old in enumerate(order)}
    new_of[-1] = -1
    par = np.array([new_of[parent[old]] for old in order], dtype=np.int32)
    dep = np.array([depth[old] for old in order], dtype=np.int32)
    # sibling tokens: distinct, increasing with sibling order
    tok = np.zeros(n_nodes, dtype=np.int32)
    seen = {}
    for i in range(n_nodes):
        k = seen.get(int(par[i]), 0)
        seen[int(par[i])] = k + 1
        base = int(randint(seed + 99, np.asarray([i]), 0, 3000)[0])
        tok[i] = k * 3500 + base
    words = (n_nodes + 63) // 64
    mask = np.zeros((n_nodes, max(words, 1)), dtype=np.uint64)
    for i in range(n_nodes):
        v = i
        while v != -1:
            mask[i, v // 64] |= np.uint64(1) << np.uint64(v % 64)
            v = int(par[v])
    return par, dep, tok, mask


def normal_bf16_bits(seed: int, shape, start: int = 0) -> np.ndarray:
    """i.i.d. N(0,1) values rounded to bfloat16 (round to nearest even),
    returned as uint16 bit patterns of the given shape (Box-Muller on two
    counter-based uniforms)."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    chunk = 1 << 22
    for c0 in range(0, n, chunk):
        c1 = min(n, c0 + chunk)
        idx = np.arange(start + c0, start + c1, dtype=_U64)
        u1 = 1.0 - uniform01(seed, idx * _U64(2))
        u2 = uniform01(seed, idx * _U64(2) + _U64(1))
        z = (np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)).astype(np.float32)
        b = z.view(np.uint32)
        rounded = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
        out[c0:c1] = rounded.astype(np.uint16)
    return out.reshape(shape)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_f32(seed: int, shape, start: int = 0) -> np.ndarray:
    n = int(np.prod(shape))
    idx = np.arange(start, start + n, dtype=_U64)
    u1 = 1.0 - uniform01(seed, idx * _U64(2))
    u2 = uniform01(seed, idx * _U64(2) + _U64(1))
    return (np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)).astype(np.float32).reshape(shape)


def sampled_ids(seed: int, draft_tokens: np.ndarray, parent_idx: np.ndarray, n_nodes: int,
                vocab: int = 32000, p_follow: float = 0.7) -> np.ndarray:
    """Token id 'predicted' at every position of one draft tree: slot 0 is the
    virtual root, slot 1+i is node i.  With probability p_follow the id is the
    token of a uniformly chosen child of that position (if it has any), else a
    uniform random token.  Returns int32 [1 + len(draft_tokens)]."""
    c = draft_tokens.shape[0]
    out = np.zeros(1 + c, dtype=np.int32)
    children = {}
    for i in range(n_nodes):
        children.setdefault(int(parent_idx[i]), []).append(i)
    for slot in range(1 + c):
        node = slot - 1
        u = uniform01(seed, np.arange(slot * 3, slot * 3 + 3))
        ch = children.get(node, []) if node < n_nodes else []
        if ch and u[0] < p_follow:
            out[slot] = draft_tokens[ch[int(u[1] * len(ch))]]
        else:
            out[slot] = int(u[2] * vocab)
    return out


# ---------------------------------------------------------------------------
# Named workloads (shapes follow the five benchmark configurations)
# ---------------------------------------------------------------------------
@dataclass
class Workload:
    name: str
    n_tokens: int
    n_motifs: int
    corpus_seed: int
    token_dtype: type
    sa_bytes: int
    batch: int
    ctx_len: int
    query_seed: int
    n_max: int
    n_min: int
    max_matches: int
    cont_len: int
    max_nodes: int
    layers: int        # Nb for attention (layers, or contexts for the batched config)
    heads: int
    head_dim: int
    kv_len: int        # P: cached prefix length
    qkv_seed: int


WORKLOADS = {
    "tiny": Workload("tiny", 1_000_000, 2000, 1, np.int32, 4, 8, 64, 11, 16, 2, 1000, 10, 32,
                     1, 32, 128, 256, 22),
    "llama7b": Workload("llama7b", 100_000_000, 556, 2, np.int32, 4, 1, 512, 12, 16, 2, 5000, 16, 64,
                        32, 32, 128, 2048, 23),
    "llama13b": Workload("llama13b", 500_000_000, 2778, 3, np.int32, 4, 1, 512, 12, 16, 2, 5000, 16, 64,
                         40, 40, 128, 4096, 24),
    "batched2b": Workload("batched2b", 2_000_000_000, 11111, 5, np.uint16, 8, 32, 1024, 15, 16, 2, 5000, 16, 64,
                          32, 32, 128, 2048, 26),
}
