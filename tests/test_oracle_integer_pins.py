"""Pins for the integer half of the CPU oracle (no GPU).

Each test compares oracle/ against something that is not the oracle's own
code: textbook suffix arrays (tests/golden), Python's sort and substring
search, collections.Counter prefix counts, hand-derived small cases and
invariants the paper states.
"""
import os
from collections import Counter

import numpy as np
import pytest

import oracle
import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def py_suffix_array(tokens):
    toks = [int(x) for x in tokens]
    # Python tuple order: a proper prefix is smaller -> end of stream smallest
    return sorted(range(len(toks)), key=lambda i: tuple(toks[i:]))


def small_corpus(n, vocab, seed, dtype=np.int32):
    return synth.randint(seed, np.arange(n), 0, vocab).astype(dtype)


# ------------------------------------------------------------------ suffix array
def test_suffix_array_textbook_golden():
    with open(os.path.join(GOLDEN, "textbook_suffix_arrays.txt")) as f:
        lines = [ln for ln in f if ln.strip() and not ln.startswith("#")]
    assert len(lines) == 3
    for ln in lines:
        word, sa_txt = [x.strip() for x in ln.split("|")]
        want = [int(x) for x in sa_txt.split()]
        corpus = np.array([ord(ch) for ch in word], dtype=np.int32)
        assert oracle.suffix_array(corpus).tolist() == want
        assert py_suffix_array(corpus) == want          # the fixture itself is sane
        assert oracle.check_suffix_array(corpus, np.array(want, dtype=np.int64)) == -1


@pytest.mark.parametrize("dtype", [np.int32, np.uint16])
@pytest.mark.parametrize("n,vocab,seed", [(1, 3, 1), (2, 2, 2), (257, 2, 3), (500, 3, 4), (1000, 50, 5)])
def test_suffix_array_equals_python_sort(n, vocab, seed, dtype):
    corpus = small_corpus(n, vocab, seed, dtype)
    assert oracle.suffix_array(corpus).tolist() == py_suffix_array(corpus)


def test_suffix_array_closed_forms():
    n = 300
    same = np.full(n, 7, dtype=np.int32)
    assert oracle.suffix_array(same).tolist() == list(range(n - 1, -1, -1))
    inc = np.arange(n, dtype=np.int32)
    assert oracle.suffix_array(inc).tolist() == list(range(n))
    dec = np.arange(n, 0, -1).astype(np.int32)
    assert oracle.suffix_array(dec).tolist() == list(range(n - 1, -1, -1))


def test_check_suffix_array_rejects_wrong_arrays():
    corpus = small_corpus(400, 3, 9)
    sa = np.array(py_suffix_array(corpus), dtype=np.int64)
    assert oracle.check_suffix_array(corpus, sa) == -1
    assert oracle.check_suffix_array(corpus, sa.astype(np.int32)) == -1
    swapped = sa.copy()
    swapped[[100, 101]] = swapped[[101, 100]]
    assert oracle.check_suffix_array(corpus, swapped) == 100
    dup = sa.copy()
    dup[5] = dup[4]
    assert oracle.check_suffix_array(corpus, dup) == 5
    oob = sa.copy()
    oob[7] = 400
    assert oracle.check_suffix_array(corpus, oob) == 7


# ------------------------------------------------------------------ Algorithm 1
def encode(tokens):
    return b"".join(int(x).to_bytes(4, "big") for x in tokens)


def py_occurrences(corpus, q):
    """All (overlapping) occurrences via bytes.find on a 4-byte encoding."""
    hay, needle = encode(corpus), encode(q)
    out, start = [], 0
    while True:
        i = hay.find(needle, start)
        if i < 0:
            return out
        if i % 4 == 0:
            out.append(i // 4)
        start = i + 1


def py_retrieve(corpus, ctx, n_max, n_min, K, m):
    toks = [int(x) for x in corpus]
    t = len(ctx)
    for n in range(min(n_max, t), n_min - 1, -1):
        occ = py_occurrences(corpus, ctx[t - n:])
        if occ:
            occ_sorted = sorted(occ, key=lambda p: tuple(toks[p:]))[:K]
            rows = [toks[p + n:p + n + m] for p in occ_sorted]
            return n, len(occ), occ_sorted, rows
    return 0, 0, [], []


@pytest.mark.parametrize("one_pass", [False, True])
@pytest.mark.parametrize("dtype", [np.int32, np.uint16])
@pytest.mark.parametrize("n,vocab,seed", [(300, 2, 1), (1000, 3, 2), (3000, 4, 3), (2000, 40, 4)])
def test_retrieve_equals_python_bruteforce(n, vocab, seed, dtype, one_pass):
    corpus = small_corpus(n, vocab, seed, dtype)
    for qi in range(12):
        t = [1, 2, 3, 5, 16, 17, 40][qi % 7]
        if qi % 3 == 0:     # copied from the corpus, ending anywhere (also at the very end)
            e = n if qi == 0 else int(synth.randint(seed + 50, [qi], t, n + 1)[0])
            ctx = corpus[e - t:e].astype(np.int32)
        else:
            ctx = small_corpus(t, vocab + (qi % 2), seed * 100 + qi).astype(np.int32)
        for K, m in [(5, 3), (1000, 10)]:
            n_star, cnt, occ, rows = py_retrieve(corpus, ctx, 16, 2, K, m)
            got = oracle.retrieve(corpus, ctx, 16, 2, K, m, one_pass=one_pass)
            assert got.matched_len == n_star
            assert got.match_count == cnt
            assert got.row_pos.tolist() == occ
            assert got.row_len.tolist() == [len(r) for r in rows]
            for r, row in enumerate(rows):
                assert got.rows[r, :len(row)].tolist() == row
                assert (got.rows[r, len(row):] == -1).all()


def test_retrieve_overlapping_and_end_of_stream():
    # "aaaa...": suffix "aa" (n capped at 16) occurs at every position, overlapping
    corpus = np.full(40, 3, dtype=np.int32)
    got = oracle.retrieve(corpus, np.full(30, 3, dtype=np.int32), 16, 2, 1000, 4)
    assert got.matched_len == 16 and got.match_count == 40 - 16 + 1
    # suffix order of equal-letter suffixes: shortest (latest) first
    assert got.row_pos.tolist() == list(range(24, -1, -1))
    # the occurrence touching the end has an empty continuation but still counts
    assert got.row_len.tolist()[:6] == [0, 1, 2, 3, 4, 4]
    # too-short context and no match at all
    assert oracle.retrieve(corpus, np.array([3], dtype=np.int32)).matched_len == 0
    miss = oracle.retrieve(corpus, np.array([5, 6, 7], dtype=np.int32))
    assert (miss.matched_len, miss.match_count, miss.rows.shape[0]) == (0, 0, 0)


def test_retrieve_finds_planted_suffix_length():
    c = synth.make_corpus(20000, seed=5, n_motifs=20, copies=10, vocab=32000)
    toks = c.tokens
    for j in range(10):
        ell = 2 + j % 15
        o = int(c.motif_offsets[j, 3])
        L = int(c.motif_lengths[j])
        if ell > L:
            continue
        junk = np.array([31999 - j, 31998, 31997], dtype=np.int32)  # unlikely to extend the match
        ctx = np.concatenate([junk, toks[o:o + ell].astype(np.int32)])
        got = oracle.retrieve(toks, ctx, 16, 2, 1000, 10)
        assert got.matched_len >= ell
        n_star, cnt, _, _ = py_retrieve(toks, ctx, 16, 2, 1000, 10)
        assert (got.matched_len, got.match_count) == (n_star, cnt)


# ------------------------------------------------------------------ Algorithm 2
def py_trie(rows, lens):
    cnt = Counter()
    for row, ln in zip(rows, lens):
        for d in range(1, ln + 1):
            cnt[tuple(int(x) for x in row[:d])] += 1
    return cnt


def py_select(rows, lens, c):
    cnt = py_trie(rows, lens)
    top = sorted(cnt, key=lambda p: (-cnt[p], len(p), p))[:c]
    bfs = sorted(top, key=lambda p: (len(p), p))
    index = {p: i for i, p in enumerate(bfs)}
    return cnt, bfs, index


def random_rows(R, m, vocab, seed, ragged=False):
    rows = synth.randint(seed, np.arange(R * m), 0, vocab).astype(np.int32).reshape(R, m)
    lens = np.full(R, m, dtype=np.int32)
    if ragged:
        lens = synth.randint(seed + 1, np.arange(R), 0, m + 1).astype(np.int32)
    return rows, lens


@pytest.mark.parametrize("R,m,vocab,seed,ragged", [
    (1, 1, 2, 1, False), (50, 4, 2, 2, False), (200, 10, 3, 3, False),
    (300, 16, 2, 4, True), (64, 6, 5, 5, True), (500, 10, 30, 6, False)])
def test_select_drafts_equals_counter_topc(R, m, vocab, seed, ragged):
    rows, lens = random_rows(R, m, vocab, seed, ragged)
    order = np.argsort(synth.uniform01(seed + 9, np.arange(R))).astype(np.int64)
    for c in [1, 2, 7, 32, 64, 100]:
        cnt, bfs, index = py_select(rows, lens, c)
        tree = oracle.select_drafts(rows, lens, c, order)
        assert tree.total_trie_nodes == len(cnt)
        assert tree.n_nodes == len(bfs)
        for i, p in enumerate(bfs):
            assert tree.draft_tokens[i] == p[-1]
            assert tree.pos_ids[i] == len(p)
            assert tree.node_weight[i] == cnt[p]
            assert tree.parent_idx[i] == (-1 if len(p) == 1 else index[p[:-1]])
        T = tree.n_nodes
        assert (tree.draft_tokens[T:] == -1).all() and (tree.parent_idx[T:] == -1).all()
        assert (tree.pos_ids[T:] == 0).all() and (tree.node_weight[T:] == 0).all()
        assert (tree.tree_mask[T:] == 0).all()


def test_select_drafts_hand_cases():
    # all rows identical -> a single chain, every weight = R
    rows = np.tile(np.array([[4, 9, 2]], dtype=np.int32), (7, 1))
    t = oracle.select_drafts(rows, np.full(7, 3, np.int32), 8)
    assert t.n_nodes == 3 and t.draft_tokens[:3].tolist() == [4, 9, 2]
    assert t.parent_idx[:3].tolist() == [-1, 0, 1] and t.node_weight[:3].tolist() == [7, 7, 7]
    assert t.tree_mask[:3, 0].tolist() == [0b1, 0b11, 0b111]
    # all rows differ at token 1 -> R depth-1 nodes first (weight 1 each, depth before prefix)
    rows = np.array([[5, 1], [3, 1], [9, 1]], dtype=np.int32)
    t = oracle.select_drafts(rows, np.full(3, 2, np.int32), 4)
    assert t.draft_tokens[:4].tolist() == [3, 5, 9, 1]
    assert t.parent_idx[:4].tolist() == [-1, -1, -1, 0]
    assert t.pos_ids[:4].tolist() == [1, 1, 1, 2]
    assert t.tree_mask[:4, 0].tolist() == [0b1, 0b10, 0b100, 0b1001]
    # a tie between a parent and its child never selects the child alone
    rows = np.array([[1, 2], [1, 2], [7, 8]], dtype=np.int32)
    t = oracle.select_drafts(rows, np.full(3, 2, np.int32), 1)
    assert t.n_nodes == 1 and t.draft_tokens[0] == 1 and t.node_weight[0] == 2
    # empty candidate set -> empty tree
    t = oracle.select_drafts(np.zeros((0, 3), np.int32), np.zeros(0, np.int32), 5)
    assert t.n_nodes == 0 and (t.draft_tokens == -1).all()


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_trie_invariants(seed):
    rows, lens = random_rows(400, 10, 3, seed, ragged=(seed == 12))
    big = oracle.select_drafts(rows, lens, 5000)
    T = big.n_nodes
    assert T == big.total_trie_nodes                 # c >= number of nodes keeps the whole Trie
    w, par, dep = big.node_weight[:T], big.parent_idx[:T], big.pos_ids[:T]
    ends_at = Counter(tuple(int(x) for x in rows[r, :lens[r]]) for r in range(rows.shape[0]))
    # children's weights sum to the parent's weight minus candidates ending at the parent
    child_sum = np.zeros(T, dtype=np.int64)
    for i in range(T):
        if par[i] >= 0:
            child_sum[par[i]] += w[i]
            assert w[par[i]] >= w[i] and dep[par[i]] + 1 == dep[i] and par[i] < i
    for i in range(T):
        path, v = [], i
        while v != -1:
            path.append(int(big.draft_tokens[v]))
            v = int(par[v])
        assert child_sum[i] == w[i] - ends_at.get(tuple(path[::-1]), 0)
    # a shared prefix appears once: no two nodes have the same (parent, token)
    assert len({(int(par[i]), int(big.draft_tokens[i])) for i in range(T)}) == T
    roots = w[par == -1].sum()
    assert roots == int((lens > 0).sum())            # depth-1 weights sum to the candidates
    # result for c is a prefix (in weight order) of the result for c+1, and closed under parents
    prev = None
    for c in range(1, 40):
        t = oracle.select_drafts(rows, lens, c)
        nodes = set()
        for i in range(t.n_nodes):
            path, v = [], i
            while v != -1:
                path.append(int(t.draft_tokens[v]))
                v = int(t.parent_idx[v])
            nodes.add(tuple(path[::-1]))
        for p in nodes:
            assert len(p) == 1 or p[:-1] in nodes
        if prev is not None:
            assert prev <= nodes and len(nodes) == min(c, big.total_trie_nodes)
        prev = nodes


def test_mask_is_ancestor_set():
    rows, lens = random_rows(300, 12, 3, 21)
    t = oracle.select_drafts(rows, lens, 130)
    T = t.n_nodes
    assert T == 130 and t.tree_mask.shape == (130, 3)
    assert (t.tree_mask == oracle.mask_from_parents(t.parent_idx, T, 3)).all()
    for i in range(T):
        bits = {j for j in range(192) if (int(t.tree_mask[i, j // 64]) >> (j % 64)) & 1}
        anc, v = set(), i
        while v != -1:
            anc.add(v)
            v = int(t.parent_idx[v])
        assert bits == anc
        assert len(bits) == t.pos_ids[i]              # popcount = depth
        assert max(bits) == i                          # lower triangular with the diagonal set
    # siblings carry distinct tokens, so no (parent, token) pair repeats
    pairs = [(int(t.parent_idx[i]), int(t.draft_tokens[i])) for i in range(T)]
    assert len(set(pairs)) == T
    # synthetic tree generator's mask agrees with the oracle's mask rule
    par, dep, tok, mask = synth.random_tree(100, 3)
    assert (mask == oracle.mask_from_parents(par, 100, 2)).all()
    assert (np.diff(dep) >= 0).all() and dep.max() <= 16


def test_draft_tree_end_to_end_equals_python():
    corpus = small_corpus(4000, 4, 31)
    for qi in range(6):
        e = int(synth.randint(77, [qi], 20, 4000)[0])
        ctx = corpus[e - 20:e].astype(np.int32)
        n_star, cnt, occ, rows = py_retrieve(corpus, ctx, 16, 2, 50, 6)
        lens = [len(r) for r in rows]
        _, bfs, index = py_select(rows, lens, 16)
        tree = oracle.draft_tree(corpus, ctx, 16, 2, 50, 6, 16)
        assert (tree.matched_len, tree.match_count, tree.n_nodes) == (n_star, cnt, len(bfs))
        assert tree.draft_tokens[:len(bfs)].tolist() == [p[-1] for p in bfs]


# ------------------------------------------------------------------ acceptance
def test_accept_hand_cases():
    par, dep, tok, _ = synth.random_tree(40, 8)
    T = 40
    ids = np.full(41, -5, dtype=np.int32)            # never equals a draft token
    n, path, nxt = oracle.accept(ids, tok, par, T, 16)
    assert n == 0 and nxt == -5 and (path == -1).all()
    # ids that follow one root-to-leaf path accept exactly that path
    leaf = T - 1
    chain, v = [], leaf
    while v != -1:
        chain.append(v)
        v = int(par[v])
    chain = chain[::-1]
    ids = np.full(41, -5, dtype=np.int32)
    ids[0] = tok[chain[0]]
    for a, b in zip(chain[:-1], chain[1:]):
        ids[1 + a] = tok[b]
    ids[1 + leaf] = 1234
    n, path, nxt = oracle.accept(ids, tok, par, T, 16)
    assert n == dep[leaf] and path[:n].tolist() == chain and nxt == 1234
    # a disagreement in the middle rejects everything after it
    if len(chain) >= 2:
        ids[1 + chain[0]] = -7
        n, path, nxt = oracle.accept(ids, tok, par, T, 16)
        assert n == 1 and path[0] == chain[0] and nxt == -7


def test_rest_loop_on_a_fully_predictable_stream_emits_the_whole_draft_and_one_more_token_per_step():
    """A periodic stream and a model that continues the period: every draft token is accepted, and each verification
    step also yields the model's own token after the last accepted one ("Draft acceptance"), so a step emits
    cont_len + 1 tokens."""
    period, m = 50, 8
    corpus = np.tile(np.arange(period, dtype=np.int32), 40)
    model = lambda seq: (seq[-1] + 1) % period          # noqa: E731
    prompt = list(range(20))
    got, steps = oracle.rest_decode(model, prompt, 60, corpus, max_matches=200, cont_len=m, max_nodes=24)
    assert got == [(20 + i) % period for i in range(60)]
    assert steps == -(-60 // (m + 1))                    # 7 steps of 9 tokens, not 8 of 8


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_rest_loop_reproduces_greedy_decoding(seed):
    corp = synth.make_corpus(30000, seed=seed, n_motifs=40, copies=20, vocab=500)
    corpus = corp.tokens
    # deterministic toy model: usually continues the stream's most recent bigram
    # successor, otherwise a hash of the last three tokens
    succ = {}
    for a, b, c3 in zip(corpus[:-2], corpus[1:-1], corpus[2:]):
        succ[(int(a), int(b))] = int(c3)

    def model(seq):
        key = (seq[-2], seq[-1])
        h = (seq[-1] * 1000003 + seq[-2] * 10007 + seq[-3] * 101 + seed) % 7
        if key in succ and h != 0:
            return succ[key]
        return (seq[-1] * 31 + seq[-2] * 17 + seq[-3]) % 500

    o = int(corp.motif_offsets[0, 0])
    prompt = corpus[o:o + 6].astype(np.int32).tolist()
    want = oracle.greedy_decode(model, prompt, 60)
    got, steps = oracle.rest_decode(model, prompt, 60, corpus, max_matches=200, cont_len=8, max_nodes=24)
    assert got == want
    assert steps <= 60
    assert steps < 60      # drafts are accepted at least sometimes on this corpus


def test_index_file_fingerprint_and_round_trip(tmp_path):
    # the splitmix64 generator seeded with 0 emits 0xE220A8397B1DCDAF, then 0x6E789E6AA1B965F4 (its published first
    # outputs): these are the finaliser applied to 1 and 2 times the golden-ratio constant, i.e. the fingerprint
    # terms of a stream of zero tokens
    assert oracle.corpus_fingerprint(np.zeros(1, np.int32)) == 0xE220A8397B1DCDAF
    assert oracle.corpus_fingerprint(np.zeros(2, np.int32)) == (0xE220A8397B1DCDAF + 0x6E789E6AA1B965F4) % 2 ** 64
    # token value and position both count; uint16 and int32 streams of equal values agree
    a = np.array([5, 7, 7, 1], np.int32)
    assert oracle.corpus_fingerprint(a) != oracle.corpus_fingerprint(a[::-1].copy())
    assert oracle.corpus_fingerprint(a) == oracle.corpus_fingerprint(a.astype(np.uint16))
    py = 0
    for i, t in enumerate(a):
        z = (int(t) + (i + 1) * 0x9E3779B97F4A7C15) % 2 ** 64
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) % 2 ** 64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) % 2 ** 64
        py = (py + (z ^ (z >> 31))) % 2 ** 64
    assert oracle.corpus_fingerprint(a) == py
    corpus = np.array([1, 0, 1, 1, 0, 2], np.int32)
    sa = oracle.suffix_array(corpus).astype(np.int32)
    p = str(tmp_path / "x.restsa")
    oracle.write_index_file(p, corpus, sa)
    raw = open(p, "rb").read()
    assert len(raw) == 64 + 6 * 4 and raw[:8] == b"RESTSA01" and raw[8:16] == (6).to_bytes(8, "little")
    assert raw[16:20] == (4).to_bytes(4, "little") and raw[20:24] == (4).to_bytes(4, "little")
    n, tb, sb, fp, back, depth = oracle.read_index_file(p)
    assert (n, tb, sb, fp, depth) == (6, 4, 4, oracle.corpus_fingerprint(corpus), 0) and raw[32:64] == bytes(32)
    np.testing.assert_array_equal(back, sa)
    oracle.write_index_file(p, corpus, oracle.prefix_sorted_array(corpus, 2), sort_depth=2)
    raw = open(p, "rb").read()
    assert raw[32:36] == (2).to_bytes(4, "little") and raw[36:64] == bytes(28)
    assert oracle.read_index_file(p)[5] == 2 and oracle.read_index_file(p)[4].tolist() == [1, 4, 0, 3, 2, 5]


def test_random_selection_strategy():
    """The ablation's draft strategy: a few randomly drawn candidates instead of the whole Trie."""
    # the generator: published first outputs of splitmix64 seeded with 0 are its finaliser at G and 2G
    G = 0x9E3779B97F4A7C15
    assert oracle._mix64(G) == 0xE220A8397B1DCDAF and oracle._mix64(2 * G) == 0x6E789E6AA1B965F4
    # with seed = -G (mod 2^64) and context 0 the inner state is mix(0) = 0, so draw j uses the published output
    # number 1 + j of that generator (0xE220..., 0x6E78..., 0x06C4...) and takes its leading bits: floor(U * n / 2^64)
    assert oracle._mix64(0) == 0 and oracle._mix64(3 * G) == 0x06C45D188009454F
    np.testing.assert_array_equal(oracle.random_rows(16, 2, (1 << 64) - G, 0), [0x6, 0xE])
    np.testing.assert_array_equal(oracle.random_rows(256, 3, (1 << 64) - G, 0), [0x06, 0x6E, 0xE2])
    # one candidate: every draw is that candidate; no candidates: nothing
    np.testing.assert_array_equal(oracle.random_rows(1, 8, 3, 0), [0])
    assert oracle.random_rows(0, 8, 3, 0).size == 0
    # draws are in range, at most n_seq, sorted and distinct; contexts and seeds get different draws
    seen = set()
    for b in range(200):
        r = oracle.random_rows(1000, 8, 7, b)
        assert 1 <= r.size <= 8 and (np.diff(r) > 0).all() and r[0] >= 0 and r[-1] < 1000
        seen.add(tuple(r))
    assert len(seen) == 200 and tuple(oracle.random_rows(1000, 8, 8, 0)) not in seen
    # roughly uniform: 8 * 4000 draws over 10 candidates, each expected 3200 times
    hist = np.zeros(10)
    for b in range(4000):
        G1 = oracle._mix64(11 + G * (1 + b))
        for j in range(8):
            hist[(oracle._mix64(G1 + G * (1 + j)) * 10) >> 64] += 1
    assert (np.abs(hist - 3200) < 5 * np.sqrt(3200)).all()
    # the tree is the Trie of exactly the drawn candidates: compare with prefix counts of those rows
    corp = synth.make_corpus(50_000, 2, 40)
    ctx, lens = synth.make_contexts(corp, 12, 64, 5)
    some = 0
    for b in range(12):
        got = oracle.retrieve(corp.tokens, ctx[b], max_matches=1000, cont_len=8)
        tree = oracle.draft_tree(corp.tokens, ctx[b], max_matches=1000, cont_len=8, max_nodes=64, random_seqs=8, seed=21,
                                 ctx_index=b)
        if got.rows.shape[0] == 0:
            assert tree.n_nodes == 0
            continue
        sel = oracle.random_rows(got.rows.shape[0], 8, 21, b)
        counts = Counter()
        for r in sel:
            for d in range(1, got.row_len[r] + 1):
                counts[tuple(got.rows[r, :d])] += 1
        assert tree.n_nodes == len(counts) <= 64
        for i in range(tree.n_nodes):
            path, v = [], i
            while v != -1:
                path.append(int(tree.draft_tokens[v]))
                v = int(tree.parent_idx[v])
            assert counts[tuple(path[::-1])] == tree.node_weight[i]
        some += tree.n_nodes > 8
    assert some >= 2


def test_strided_match_sampling():
    """Which occurrences are kept when there are more than max_matches: an evenly spaced sample of the sorted range
    instead of its head."""
    # brute force: every occurrence sorted by its whole suffix in Python, then ranks floor(i*S/K)
    for n, vocab, seed in [(2000, 2, 31), (3000, 3, 32), (1500, 5, 33)]:
        corpus = small_corpus(n, vocab, seed)
        toks = [int(x) for x in corpus]
        capped = 0
        for qi in range(10):
            ctx = small_corpus([2, 3, 4, 6, 17][qi % 5], vocab, seed * 10 + qi).astype(np.int32)
            for K, m in [(7, 4), (64, 10), (1000, 3)]:
                n_star, cnt, occ, _ = py_retrieve(corpus, ctx, 16, 2, 10 ** 9, m)
                pick = occ if cnt <= K else [occ[(i * cnt) // K] for i in range(K)]
                got = oracle.retrieve(corpus, ctx, 16, 2, K, m, strided=True)
                assert (got.matched_len, got.match_count) == (n_star, cnt)
                assert got.row_pos.tolist() == pick
                for r, p in enumerate(pick):
                    row = toks[p + n_star:p + n_star + m]
                    assert got.rows[r, :len(row)].tolist() == row and got.row_len[r] == len(row)
                    assert (got.rows[r, len(row):] == -1).all()
                if cnt <= K:      # nothing to drop: the same rows as the head rule
                    head = oracle.retrieve(corpus, ctx, 16, 2, K, m)
                    np.testing.assert_array_equal(head.row_pos, got.row_pos)
                capped += cnt > K
        assert capped >= 3
    # closed form: the pair (5, 6) is followed 700 times by 1 and 300 times by 2 (separators 9 keep longer matches
    # away).  Sorted, the 700 come first, so the head rule with K = 100 sees only token 1; the evenly spaced sample
    # takes ranks 0, 10, ..., 990: exactly 70 and 30.
    order = np.array([1] * 700 + [2] * 300)
    order = order[np.argsort(synth.randint(77, np.arange(1000), 0, 1 << 30), kind="stable")]
    corpus = np.concatenate([[5, 6, int(a), 9] for a in order]).astype(np.int32)
    ctx = np.array([3, 5, 6], dtype=np.int32)
    head = oracle.draft_tree(corpus, ctx, max_matches=100, cont_len=1, max_nodes=8)
    even = oracle.draft_tree(corpus, ctx, max_matches=100, cont_len=1, max_nodes=8, strided=True)
    assert head.match_count == even.match_count == 1000 and head.matched_len == 2
    assert head.draft_tokens[:head.n_nodes].tolist() == [1] and head.node_weight[0] == 100
    assert even.draft_tokens[:even.n_nodes].tolist() == [1, 2] and even.node_weight[:2].tolist() == [70, 30]
    # with random selection on top, the draws index the strided sample
    got = oracle.retrieve(corpus, ctx, max_matches=100, cont_len=1, strided=True)
    sel = oracle.random_rows(100, 8, 5, 3)
    tree = oracle.draft_tree(corpus, ctx, max_matches=100, cont_len=1, max_nodes=8, strided=True, random_seqs=8, seed=5,
                             ctx_index=3)
    want = Counter(int(got.rows[r, 0]) for r in sel)
    assert {int(t): int(w) for t, w in zip(tree.draft_tokens[:tree.n_nodes], tree.node_weight)} == dict(want)


def test_depth_limited_order():
    """Positions ordered by their first `depth` tokens only, equal prefixes by position."""
    # by hand: stream 1 0 1 1 0 2, depth 2: prefixes (1,0)@0 (0,1)@1 (1,1)@2 (1,0)@3 (0,2)@4 (2)@5
    corpus = np.array([1, 0, 1, 1, 0, 2], np.int32)
    assert oracle.prefix_sorted_array(corpus, 2).tolist() == [1, 4, 0, 3, 2, 5]
    assert oracle.prefix_sorted_array(corpus, 1).tolist() == [1, 4, 0, 2, 3, 5]
    for n, vocab, seed, dtype in [(500, 2, 41, np.int32), (2000, 3, 42, np.uint16), (1500, 30, 43, np.int32)]:
        corpus = small_corpus(n, vocab, seed, dtype)
        toks = [int(x) for x in corpus]
        # depth 1 is a stable sort of the tokens; a depth no repeat reaches gives the suffix array itself
        np.testing.assert_array_equal(oracle.prefix_sorted_array(corpus, 1), np.argsort(corpus, kind="stable"))
        np.testing.assert_array_equal(oracle.prefix_sorted_array(corpus, n), oracle.suffix_array(corpus))
        for depth in (2, 5, 26):
            arr = oracle.prefix_sorted_array(corpus, depth)
            assert arr.tolist() == sorted(range(n), key=lambda p: (tuple(toks[p:p + depth]), p))
            # against the suffix array: same multiset, and position i's rank can only move within the run of
            # suffixes sharing its first `depth` tokens
            sa = oracle.suffix_array(corpus)
            assert [tuple(toks[p:p + depth]) for p in arr] == [tuple(toks[p:p + depth]) for p in sa]


def test_depth_limited_order_serves_retrieval_like_the_suffix_array():
    """Algorithm 1 + 2 evaluated on an explicit ordering of the positions (a range of occurrences, its first K
    members, their continuations): with the depth-limited order of depth n_max + cont_len the drafts equal those of
    the definition, which orders occurrences by their whole suffixes; with a smaller depth they need not."""
    def drafts_on(order, corpus, ctx, n_max, n_min, K, m, c):
        toks = corpus.tolist()
        for n in range(min(n_max, len(ctx)), n_min - 1, -1):
            q = ctx[len(ctx) - n:].tolist()
            occ = [p for p in order.tolist() if toks[p:p + n] == q][:K]
            if occ:
                rows = np.full((len(occ), m), -1, np.int32)
                lens = np.zeros(len(occ), np.int32)
                for r, p in enumerate(occ):
                    cont = toks[p + n:p + n + m]
                    rows[r, :len(cont)] = cont
                    lens[r] = len(cont)
                return oracle.select_drafts(rows, lens, c, np.argsort(np.array(occ), kind="stable"))
        return None
    n_max, m, K, c = 6, 4, 5, 12
    differs_when_too_shallow = 0
    for n, vocab, seed in [(1500, 2, 51), (2500, 3, 52)]:
        corpus = small_corpus(n, vocab, seed)
        full = oracle.prefix_sorted_array(corpus, n_max + m)
        shallow = oracle.prefix_sorted_array(corpus, 3)
        for qi in range(16):
            ctx = small_corpus(3 + qi % 6, vocab, seed * 10 + qi).astype(np.int32)
            want = oracle.draft_tree(corpus, ctx, n_max, 2, K, m, c)
            got = drafts_on(full, corpus, ctx, n_max, 2, K, m, c)
            if got is None:
                assert want.n_nodes == 0
                continue
            assert got.n_nodes == want.n_nodes
            for name in ("draft_tokens", "parent_idx", "pos_ids", "node_weight", "tree_mask"):
                np.testing.assert_array_equal(getattr(got, name), getattr(want, name), err_msg=name)
            bad = drafts_on(shallow, corpus, ctx, n_max, 2, K, m, c)
            differs_when_too_shallow += not (np.array_equal(bad.draft_tokens, want.draft_tokens) and
                                             np.array_equal(bad.node_weight, want.node_weight))
    assert differs_when_too_shallow >= 3


def test_c_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """The C half of the oracle, driven over 400 small irregular inputs (tests/oracle_sanitize_driver.c) in a build with
    -fsanitize=address,undefined: no out-of-bounds access, overflow or leak."""
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = str(tmp_path / "oracle_san")
    cmd = ["gcc", "-std=c99", "-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-static-libasan", "-static-libubsan", os.path.join(root, "oracle", "rest_oracle.c"),
           os.path.join(root, "tests", "oracle_sanitize_driver.c"), "-o", exe]
    built = subprocess.run(cmd, capture_output=True, text=True)
    if built.returncode != 0:
        pytest.skip("no sanitizer runtime for gcc here: " + built.stderr[-200:])
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert run.returncode == 0 and "ok" in run.stdout, run.stderr[-2000:]
