"""GPU parity tests: the HIP path (through the C ABI binding) against the CPU oracle, element by element,
on the same seeded inputs.  Integer outputs must be bit-exact; attention within the stated tolerances."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import synth

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2311_08252_amd as rest


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def small_corpus(n, vocab, seed, dtype=np.int32):
    return synth.randint(seed, np.arange(n), 0, vocab).astype(dtype)


def tree_to_numpy(tree, b):
    return dict(
        n_nodes=int(tree.n_nodes[b].item()), matched_len=int(tree.matched_len[b].item()),
        match_count=int(tree.match_count[b].item()),
        draft_tokens=tree.draft_tokens[b].cpu().numpy(), parent_idx=tree.parent_idx[b].cpu().numpy(),
        pos_ids=tree.pos_ids[b].cpu().numpy(), node_weight=tree.node_weight[b].cpu().numpy(),
        tree_mask=tree.tree_mask[b].cpu().numpy().view(np.uint64))


def assert_tree_equal(got, want, where=""):
    assert got["matched_len"] == want.matched_len, where
    assert got["match_count"] == want.match_count, where
    assert got["n_nodes"] == want.n_nodes, where
    np.testing.assert_array_equal(got["draft_tokens"], want.draft_tokens, err_msg=where)
    np.testing.assert_array_equal(got["parent_idx"], want.parent_idx, err_msg=where)
    np.testing.assert_array_equal(got["pos_ids"], want.pos_ids, err_msg=where)
    np.testing.assert_array_equal(got["node_weight"], want.node_weight, err_msg=where)
    np.testing.assert_array_equal(got["tree_mask"], want.tree_mask, err_msg=where)


# ------------------------------------------------------------------ index build
@pytest.mark.parametrize("dtype,sa_bytes", [(np.int32, 4), (np.uint16, 8), (np.uint16, 4), (np.int32, 8)])
@pytest.mark.parametrize("n,vocab,seed", [(1, 3, 1), (2, 2, 2), (63, 2, 3), (4097, 3, 4), (20000, 2, 5), (50000, 30000, 6)])
def test_build_index_equals_oracle_sort(n, vocab, seed, dtype, sa_bytes):
    corpus = small_corpus(n, vocab, seed, dtype)
    idx = rest.rest_build_index(dev(corpus), sa_bytes)
    sa = idx.suffix_array().cpu().numpy()
    assert sa.dtype == (np.int32 if sa_bytes == 4 else np.int64)
    np.testing.assert_array_equal(sa.astype(np.int64), oracle.suffix_array(corpus))
    idx.destroy()


def test_build_index_closed_forms_and_motifs():
    n = 3000
    for corpus, want in [(np.full(n, 7, np.int32), np.arange(n - 1, -1, -1)), (np.arange(n, dtype=np.int32), np.arange(n))]:
        idx = rest.rest_build_index(dev(corpus), 4)
        np.testing.assert_array_equal(idx.suffix_array().cpu().numpy(), want)
    c = synth.make_corpus(300_000, seed=9, n_motifs=60, copies=50)
    idx = rest.rest_build_index(dev(c.tokens), 4)
    sa = idx.suffix_array().cpu().numpy()
    assert oracle.check_suffix_array(c.tokens, sa) == -1
    np.testing.assert_array_equal(sa.astype(np.int64), oracle.suffix_array(c.tokens))


@pytest.mark.parametrize("sa_bytes", [4, 8])
def test_build_index_streams_that_need_many_rounds(sa_bytes):
    """Streams whose suffixes stay tied for long, so that nearly every suffix is still in play in every doubling round
    (closed forms; the quadratic oracle sort would take hours on them)."""
    n = 300_001
    # one token throughout: the shorter suffix is the smaller one; 19 rounds
    idx = rest.rest_build_index(dev(np.full(n, 5, np.uint16)), sa_bytes)
    np.testing.assert_array_equal(idx.suffix_array().cpu().numpy(), np.arange(n - 1, -1, -1))
    # period two, "1 0 1 0 ... 1": suffixes starting with 0 (odd positions) come first, among the suffixes of one parity
    # the shorter is a prefix of the longer, hence smaller
    t = (1 - np.arange(n) % 2).astype(np.int32)
    idx = rest.rest_build_index(dev(t), sa_bytes)
    want = np.concatenate([np.arange(n - 2, 0, -2), np.arange(n - 1, -1, -2)])
    assert want.size == n and t[want[0]] == 0
    np.testing.assert_array_equal(idx.suffix_array().cpu().numpy(), want)
    m = 201                                            # the same closed form against the oracle's sort where that is quick
    np.testing.assert_array_equal(oracle.suffix_array(t[:m]), np.concatenate([np.arange(m - 2, 0, -2), np.arange(m - 1, -1, -2)]))
    # the depth-limited build of the constant stream: suffixes with at least 32 tokens left tie and stay in position
    # order, behind the 31 shorter ones
    lim = rest.rest_build_index_prefix(dev(np.full(n, 5, np.uint16)), sa_bytes, 32)
    assert lim.sort_depth == 32
    np.testing.assert_array_equal(lim.suffix_array().cpu().numpy(),
                                  np.concatenate([np.arange(n - 1, n - 32, -1), np.arange(0, n - 31)]))


# ------------------------------------------------------------------ retrieval
def run_retrieve_case(corpus, contexts, lens, prm, index=None):
    idx = index or rest.rest_index_from_sa(dev(corpus), dev(oracle.suffix_array(corpus).astype(np.int32)))
    B = contexts.shape[0]
    out = rest.Tree.empty(B, prm["max_nodes"], fill=-0x5A5A5A5B)       # poisoned: unwritten slots show up
    rest.rest_retrieve(idx, dev(contexts), dev(lens), out=out, **prm)
    torch.cuda.synchronize()
    for b in range(B):
        want = oracle.draft_tree(corpus, contexts[b, :lens[b]], prm["n_max"], prm["n_min"], prm["max_matches"],
                                 prm["cont_len"], prm["max_nodes"])
        assert_tree_equal(tree_to_numpy(out, b), want, where=f"context {b}")
    return idx


@pytest.mark.parametrize("dtype", [np.int32, np.uint16])
@pytest.mark.parametrize("n,vocab,seed", [(40, 2, 1), (300, 2, 2), (5000, 3, 3), (20000, 4, 4), (20000, 200, 5)])
def test_retrieve_small_corpora(n, vocab, seed, dtype):
    corpus = small_corpus(n, vocab, seed, dtype)
    B, stride = 24, 40
    ctx = np.zeros((B, stride), dtype=np.int32)
    lens = np.zeros(B, dtype=np.int32)
    for b in range(B):
        t = [0, 1, 2, 3, 7, 16, 17, 40][b % 8]
        lens[b] = t
        if b % 3 == 0 and t <= n:     # copied from the corpus; b == 0 .. also the very end of the stream
            e = n if b % 6 == 0 else int(synth.randint(seed + 70, [b], max(t, 1), n + 1)[0])
            ctx[b, :t] = corpus[e - t:e]
        else:
            ctx[b, :t] = small_corpus(t, vocab + (b % 2), seed * 131 + b)
    for prm in [dict(n_max=16, n_min=2, max_matches=1000, cont_len=10, max_nodes=32),
                dict(n_max=16, n_min=2, max_matches=7, cont_len=3, max_nodes=5),
                dict(n_max=5, n_min=1, max_matches=8192, cont_len=32, max_nodes=256),
                dict(n_max=16, n_min=16, max_matches=64, cont_len=1, max_nodes=64)]:
        run_retrieve_case(corpus, ctx, lens, prm)


@pytest.mark.parametrize("m,c", [(1, 64), (10, 3), (10, 64), (16, 256), (17, 40), (32, 256)])
def test_retrieve_around_64_kept_rows(m, c):
    """Up to 64 kept rows take a path of their own in the kernel (one wavefront, rows in lanes): a motif that occurs
    1 .. 130 times, followed by continuations over two tokens (so that Trie nodes are shared and weights differ), and
    a match cap that cuts the rows to 64 and to 63."""
    motif = np.arange(1000, 1006, dtype=np.int32)
    for k in (1, 2, 63, 64, 65, 130):
        parts = []
        for i in range(k):
            parts.append(small_corpus(40, 50, 900 + i))
            parts.append(motif)
            parts.append(small_corpus(3 + (i * 7) % 30, 2, 7000 + i) + 7)
        parts.append(small_corpus(25, 50, 999))
        parts.append(motif)                                   # one more occurrence at the very end: a row of length 0
        corpus = np.concatenate(parts).astype(np.int32)
        ctx = np.zeros((2, 12), dtype=np.int32)
        ctx[0, :6] = motif
        ctx[1, :3] = motif[3:]
        lens = np.array([6, 3], dtype=np.int32)
        idx = None
        for K in (8192, 64, 63):
            idx = run_retrieve_case(corpus, ctx, lens, dict(n_max=16, n_min=2, max_matches=K, cont_len=m, max_nodes=c), index=idx)


def test_retrieve_degenerate_streams():
    prm = dict(n_max=16, n_min=2, max_matches=1000, cont_len=10, max_nodes=32)
    same = np.full(500, 3, dtype=np.int32)            # every suffix length matches everywhere, rows reach the end
    ctx = np.full((3, 30), 3, dtype=np.int32)
    run_retrieve_case(same, ctx, np.array([30, 5, 2], np.int32), prm)
    one = np.array([9], dtype=np.int32)               # single-token stream: nothing of length >= 2 can match
    run_retrieve_case(one, np.full((1, 4), 9, np.int32), np.array([4], np.int32), prm)
    # B == 0 is a no-op
    idx = rest.rest_index_from_sa(dev(same), dev(oracle.suffix_array(same).astype(np.int32)))
    rest.rest_retrieve(idx, torch.zeros((0, 8), dtype=torch.int32, device="cuda"),
                       torch.zeros(0, dtype=torch.int32, device="cuda"), **prm)


def test_retrieve_rejects_bad_arguments():
    corpus = small_corpus(1000, 3, 1)
    idx = rest.rest_index_from_sa(dev(corpus), dev(oracle.suffix_array(corpus).astype(np.int32)))
    ctx, lens = dev(np.zeros((1, 8), np.int32)), dev(np.array([8], np.int32))
    for bad in [dict(n_max=17), dict(n_min=0), dict(n_min=5, n_max=4), dict(max_matches=0), dict(max_matches=8193),
                dict(cont_len=0), dict(cont_len=33), dict(max_nodes=0), dict(max_nodes=257)]:
        prm = dict(n_max=16, n_min=2, max_matches=100, cont_len=10, max_nodes=32)
        prm.update(bad)
        with pytest.raises(rest.RestError) as e:
            rest.rest_retrieve(idx, ctx, lens, **prm)
        assert e.value.status == rest.REST_INVALID_ARG
    with pytest.raises(rest.RestError):      # empty stream
        rest.rest_index_from_sa(dev(np.zeros(0, np.int32)), dev(np.zeros(0, np.int32)))
    with pytest.raises(rest.RestError):
        rest.rest_build_index(dev(np.zeros(0, np.int32)), 4)


def test_retrieve_tiny_config_with_gpu_built_index():
    """Config 'tiny': 10^6-token Zipf stream with planted motifs, 8 contexts of 64, K=1000, m=10, c=32."""
    w = synth.WORKLOADS["tiny"]
    c = synth.make_corpus(w.n_tokens, w.corpus_seed, w.n_motifs)
    ctx, lens = synth.make_contexts(c, w.batch, w.ctx_len, w.query_seed)
    d_corpus = dev(c.tokens)
    idx = rest.rest_build_index(d_corpus, 4)
    sa = idx.suffix_array().cpu().numpy()
    assert oracle.check_suffix_array(c.tokens, sa) == -1
    prm = dict(n_max=w.n_max, n_min=w.n_min, max_matches=w.max_matches, cont_len=w.cont_len, max_nodes=w.max_nodes)
    run_retrieve_case(c.tokens, ctx, lens, prm, index=idx)
    # a larger batch with more varied contexts
    ctx2, lens2 = synth.make_contexts(c, 64, 32, 99)
    run_retrieve_case(c.tokens, ctx2, lens2, prm, index=idx)


# ------------------------------------------------------------------ tree attention
def attention_case(Nb, H, T, P, seed, dtype="bf16", per_batch=False, num_splits=0, Tq_extra=0, tree="random", scales=True):
    Tq = T + Tq_extra
    if tree == "chain":
        par = np.arange(-1, T - 1, dtype=np.int32)
        mask = oracle.mask_from_parents(par, T)
    else:
        _, _, _, mask = synth.random_tree(T, seed) if T > 0 else (None, None, None, np.zeros((0, 1), np.uint64))
    words = max(1, (T + 63) // 64)
    mask = mask[:, :words]
    if Tq_extra:
        mask = np.vstack([np.zeros((Tq_extra, words), np.uint64), mask])
    if per_batch:
        masks = [mask]
        for nb in range(1, Nb):
            m2 = synth.random_tree(T, seed + 100 + nb)[3][:, :words]
            if Tq_extra:
                m2 = np.vstack([np.zeros((Tq_extra, words), np.uint64), m2])
            masks.append(m2)
        mask = np.stack(masks)
    if dtype == "bf16":
        qb = synth.normal_bf16_bits(seed, (Nb, H, Tq, 128))
        kb = synth.normal_bf16_bits(seed + 1, (Nb, H, P + T, 128))
        vb = synth.normal_bf16_bits(seed + 2, (Nb, H, P + T, 128))
        q, k, v = (synth.bf16_bits_to_f32(x) for x in (qb, kb, vb))
        dq, dk, dv = (dev(x.view(np.int16)).view(torch.bfloat16) for x in (qb, kb, vb))
    elif dtype == "fp8kv":
        # bf16 queries on an 8-bit cache: normal values divided by the slab's scale, then encoded by the oracle
        qb = synth.normal_bf16_bits(seed, (Nb, H, Tq, 128))
        q = synth.bf16_bits_to_f32(qb)
        dq = dev(qb.view(np.int16)).view(torch.bfloat16)
        k_scale = (0.25 + 2 * synth.uniform01(seed + 3, np.arange(Nb * H))).reshape(Nb, H).astype(np.float32)
        v_scale = (0.25 + 2 * synth.uniform01(seed + 4, np.arange(Nb * H))).reshape(Nb, H).astype(np.float32)
        if not scales:
            k_scale[:], v_scale[:] = 1.0, 1.0
        k8 = oracle.fp8_e4m3_encode(synth.normal_f32(seed + 1, (Nb, H, P + T, 128)) / k_scale[..., None, None])
        v8 = oracle.fp8_e4m3_encode(synth.normal_f32(seed + 2, (Nb, H, P + T, 128)) / v_scale[..., None, None])
        dk, dv = dev(k8), dev(v8)
    else:
        q = synth.normal_f32(seed, (Nb, H, Tq, 128))
        k = synth.normal_f32(seed + 1, (Nb, H, P + T, 128))
        v = synth.normal_f32(seed + 2, (Nb, H, P + T, 128))
        dq, dk, dv = dev(q), dev(k), dev(v)
    scale = 1.0 / np.sqrt(128.0)
    omask = mask[:, None] if per_batch else mask
    dmask = dev(mask.view(np.int64)) if T > 0 else torch.zeros((Tq, 1), dtype=torch.int64, device="cuda")
    out = torch.full_like(dq, float("nan"))
    if dtype == "fp8kv":
        want = oracle.tree_attention_fp8kv(q, k8, v8, k_scale, v_scale, omask, P, scale)
        rest.rest_tree_attention(dq, dk, dv, dmask, P, float(scale), out=out, num_splits=num_splits,
                                 k_scale=dev(k_scale) if scales else None, v_scale=dev(v_scale) if scales else None)
    else:
        want = oracle.tree_attention(q, k, v, omask, P, scale)
        rest.rest_tree_attention(dq, dk, dv, dmask, P, float(scale), out=out, num_splits=num_splits)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    if dtype in ("bf16", "fp8kv"):
        assert np.abs(got - want).max() <= 2e-2, np.abs(got - want).max()
    else:
        for nb in range(Nb):
            for h in range(H):
                rel = np.abs(got[nb, h] - want[nb, h]).max() / np.abs(want[nb, h]).max()
                assert rel <= 1e-3, rel
    return np.abs(got - want).max()


@pytest.mark.parametrize("T,P", [(1, 1), (16, 100), (32, 31), (33, 64), (64, 256), (64, 1000), (100, 77),
                                 (128, 513), (200, 5), (256, 300), (64, 0), (7, 2049)])
def test_tree_attention_bf16_shapes(T, P):
    attention_case(2, 3, T, P, seed=T * 1000 + P)


@pytest.mark.parametrize("ns", [1, 2, 3, 8, 64])
def test_tree_attention_bf16_split_counts(ns):
    attention_case(1, 2, 64, 1500, seed=5, num_splits=ns)
    attention_case(1, 2, 40, 3, seed=6, num_splits=ns)      # more waves than key blocks


@pytest.mark.parametrize("T,P,ns", [(128, 700, 3), (100, 31, 1), (256, 300, 5), (200, 1, 64), (130, 2050, 2)])
def test_tree_attention_bf16_wide_units_split(T, P, ns):
    """More than 64 queries: streams of four or eight wavefronts on tiles of 64 or 128 keys, with the unit cut
    between streams and merged."""
    attention_case(1, 2, T, P, seed=300 + T, num_splits=ns)
    attention_case(3, 1, T, P, seed=301 + T, num_splits=ns, per_batch=True)


def test_tree_attention_bf16_variants():
    attention_case(3, 2, 64, 200, seed=7, per_batch=True)
    attention_case(2, 2, 64, 200, seed=8, Tq_extra=1)        # extra root query row seeing the prefix only
    attention_case(1, 1, 64, 300, seed=9, tree="chain")      # chain tree = plain causal attention
    attention_case(1, 2, 0, 129, seed=10, Tq_extra=3)        # no draft keys at all
    attention_case(9, 5, 64, 64, seed=11)                    # streams not a multiple of 8
    attention_case(2, 2, 128, 200, seed=12, Tq_extra=1)      # 129 query rows: eight-wavefront streams, mostly idle rows
    attention_case(1, 3, 0, 300, seed=13, Tq_extra=100)      # 100 query rows and no draft keys
    attention_case(5, 7, 96, 1000, seed=14, tree="chain")    # 96 rows: four-wavefront streams with an idle wavefront


@pytest.mark.parametrize("Tq,Tk", [(7, 20), (32, 70), (20, 130), (32, 200), (31, 256), (64, 256), (100, 190)])
def test_tree_attention_arbitrary_masks_at_every_prefix_alignment(Tq, Tk):
    """Masks that are not trees (every bit drawn at random, rows independent of each other), few query rows against up
    to 256 draft keys, and the prefix ending at every offset 0..31 inside a block of 32 keys: the block that holds
    the prefix's end mixes always-visible keys with masked ones at every possible shift, and the draft keys cross the
    64-, 128- and 192-bit word boundaries of a mask row.  Both plans (units cut between workgroups with the partials
    combined in the kernel; streams over whole units) and the 8-bit cache."""
    scale = 1.0 / np.sqrt(128.0)
    words = (Tk + 63) // 64
    for r in range(32):
        P = 32 * (1 + (r * 7) % 9) + r                    # 8+ blocks of keys, prefix end at offset r of its block
        seed = 7000 + Tq * 300 + Tk + r
        bits = synth.randint(seed, np.arange(Tq * words * 64), 0, 2).reshape(Tq, words * 64).astype(np.uint64)
        bits[:, Tk:] = 0
        if r % 5 == 0:
            bits[r % Tq] = 0                               # a row that sees the prefix only
        mask = np.zeros((Tq, words), np.uint64)
        for j in range(words * 64):
            mask[:, j // 64] |= bits[:, j] << np.uint64(j % 64)
        qb = synth.normal_bf16_bits(seed + 1, (1, 2, Tq, 128))
        kb = synth.normal_bf16_bits(seed + 2, (1, 2, P + Tk, 128))
        vb = synth.normal_bf16_bits(seed + 3, (1, 2, P + Tk, 128))
        q, k, v = (synth.bf16_bits_to_f32(x) for x in (qb, kb, vb))
        dq, dk, dv = (dev(x.view(np.int16)).view(torch.bfloat16) for x in (qb, kb, vb))
        want = oracle.tree_attention(q, k, v, mask, P, scale)
        dmask = dev(mask.view(np.int64))
        for ns in (0, 1):
            out = torch.full_like(dq, float("nan"))
            rest.rest_tree_attention(dq, dk, dv, dmask, P, float(scale), out=out, num_splits=ns)
            torch.cuda.synchronize()
            err = np.abs(out.float().cpu().numpy() - want).max()
            assert err <= 2e-2, (P, ns, err)
        if r % 4 == 0:
            k8, v8 = oracle.fp8_e4m3_encode(k), oracle.fp8_e4m3_encode(v)
            want8 = oracle.tree_attention_fp8kv(q, k8, v8, np.ones((1, 2)), np.ones((1, 2)), mask, P, scale)
            out = torch.full_like(dq, float("nan"))
            rest.rest_tree_attention(dq, dev(k8), dev(v8), dmask, P, float(scale), out=out)
            torch.cuda.synchronize()
            assert np.abs(out.float().cpu().numpy() - want8).max() <= 2e-2, (P, "e4m3")


@pytest.mark.parametrize("Nb,H,T,P,dtype", [(22, 50, 64, 100, "bf16"), (35, 41, 64, 36, "bf16"), (42, 50, 64, 70, "bf16"),
                                            (7, 150, 33, 300, "fp8kv"), (20, 30, 128, 300, "bf16"), (10, 30, 256, 200, "bf16"),
                                            (40, 40, 64, 50, "bf16"), (31, 50, 40, 64, "fp8kv"), (30, 28, 128, 200, "bf16"),
                                            (7, 100, 256, 100, "bf16"), (45, 57, 64, 8, "bf16")])
def test_tree_attention_more_units_than_streams(Nb, H, T, P, dtype):
    """More units than the streams one launch runs (1024, 512 or 256 by the width of a unit) and not a multiple of
    them: one or two whole rounds, then either the remaining units cut into spans and merged, or -- half a round or
    more of them, 64 queries at most, 16-bit cache -- one more whole unit for that many streams; every slab is
    compared."""
    attention_case(Nb, H, T, P, seed=Nb * 100 + H, dtype=dtype, per_batch=True)


def test_tree_attention_bf16_tiny_config():
    """Config 'tiny': 1 layer x 32 heads x 128, KV length 256, the 32-node cap."""
    attention_case(1, 32, 32, 256, seed=22)


@pytest.mark.parametrize("T,P,ns", [(1, 1, 0), (16, 100, 0), (33, 64, 0), (64, 256, 0), (64, 1000, 3), (64, 2048, 0), (100, 77, 0),
                                     (128, 700, 3), (256, 300, 5), (200, 1, 64), (130, 2050, 2), (64, 0, 0), (40, 3, 8)])
def test_tree_attention_on_8bit_cache(T, P, ns):
    """K and V as E4M3 bytes with per-(batch, head) scales: two-, four- and eight-wavefront streams, whole units and
    units cut between streams, ragged last tiles."""
    attention_case(2, 3, T, P, seed=500 + T + P, dtype="fp8kv", num_splits=ns)


def test_tree_attention_on_8bit_cache_variants():
    attention_case(3, 2, 64, 200, seed=507, dtype="fp8kv", per_batch=True)
    attention_case(2, 2, 64, 200, seed=508, dtype="fp8kv", Tq_extra=1, scales=False)
    attention_case(1, 2, 0, 129, seed=510, dtype="fp8kv", Tq_extra=3)            # no draft keys
    attention_case(9, 5, 64, 64, seed=511, dtype="fp8kv")                         # streams not a multiple of 8
    attention_case(5, 7, 96, 1000, seed=514, dtype="fp8kv", tree="chain")
    attention_case(1, 32, 32, 256, seed=522, dtype="fp8kv")
    # token-major cache [Nb, L, H, D] viewed as [Nb, H, L, D], every code (NaN excepted) present, extreme magnitudes
    Nb, H, T, P = 2, 4, 64, 300
    qb = synth.normal_bf16_bits(1, (Nb, H, T, 128))
    codes = synth.randint(31, np.arange(2 * Nb * (P + T) * H * 128), 0, 256).astype(np.uint8).reshape(2, Nb, P + T, H, 128)
    codes[(codes & 0x7F) == 0x7F] = 0x38
    codes[0] = np.where((codes[0] & 0x78) > 0x48, codes[0] & 0xC7 | 0x30, codes[0])    # keys: |k| < 4 keeps the softmax soft
    k_scale = np.full((Nb, H), 0.5, np.float32)
    v_scale = np.full((Nb, H), 2.0 ** -6, np.float32)
    mask = synth.random_tree(T, 5)[3]
    dq = dev(qb.view(np.int16)).view(torch.bfloat16)
    dk, dv = dev(codes[0]).permute(0, 2, 1, 3), dev(codes[1]).permute(0, 2, 1, 3)
    out = rest.rest_tree_attention(dq, dk, dv, dev(mask.view(np.int64)), P, 0.088, k_scale=dev(k_scale), v_scale=dev(v_scale))
    torch.cuda.synchronize()
    want = oracle.tree_attention_fp8kv(synth.bf16_bits_to_f32(qb), codes[0].transpose(0, 2, 1, 3), codes[1].transpose(0, 2, 1, 3),
                                       k_scale, v_scale, mask, P, 0.088)
    err = np.abs(out.float().cpu().numpy() - want)
    assert (err <= 2e-2 * np.maximum(1.0, np.abs(want))).all(), err.max()
    # refused before anything is launched: fp32 queries on an 8-bit cache; cache strides that are not multiples of 16
    d = rest.make_attn_desc(dq, dk, dv, out, P, 0.088, False)
    args = (dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), dev(mask.view(np.int64)).data_ptr(), out.data_ptr())
    ws = torch.empty(max(rest.rest_tree_attention_workspace_bytes(d), 16), dtype=torch.uint8, device="cuda")
    tail = (ctypes.byref(d), ws.data_ptr(), ws.numel(), None)
    assert rest._lib.rest_tree_attention(*args, *tail) == rest.REST_OK
    d.dtype = rest.REST_FP32
    assert rest._lib.rest_tree_attention(*args, *tail) == rest.REST_INVALID_ARG
    d.dtype = rest.REST_BF16
    d.k_stride[2] = H * 128 + 8
    assert rest._lib.rest_tree_attention(*args, *tail) == rest.REST_INVALID_ARG
    torch.cuda.synchronize()


@pytest.mark.parametrize("T,P,ns", [(1, 3, 1), (64, 256, 1), (33, 200, 4), (130, 77, 2), (32, 31, 0), (64, 2048, 0), (100, 77, 0),
                                    (130, 1000, 0), (256, 300, 3), (200, 1, 64), (20, 5000, 0), (64, 0, 0)])
def test_tree_attention_fp32(T, P, ns):
    attention_case(2, 2, T, P, seed=40 + T, dtype="fp32", num_splits=ns)


def test_tree_attention_fp32_variants():
    attention_case(3, 5, 64, 515, seed=71, dtype="fp32", per_batch=True)           # a mask per batch entry
    attention_case(1, 2, 20, 130, seed=72, dtype="fp32", Tq_extra=12)              # more query rows than draft tokens
    attention_case(1, 3, 256, 40, seed=73, dtype="fp32", tree="chain")             # every draft token sees all before it
    attention_case(40, 16, 16, 100, seed=74, dtype="fp32")                         # more groups than workgroups wanted: no split


def test_tree_attention_strided_layout_and_errors():
    # K/V stored [Nb, L, H, D] (token-major cache) and viewed as [Nb, H, L, D]
    Nb, H, T, P = 2, 4, 64, 300
    qb = synth.normal_bf16_bits(1, (Nb, H, T, 128))
    kb = synth.normal_bf16_bits(2, (Nb, P + T, H, 128))
    vb = synth.normal_bf16_bits(3, (Nb, P + T, H, 128))
    mask = synth.random_tree(T, 5)[3]
    dq = dev(qb.view(np.int16)).view(torch.bfloat16)
    dk = dev(kb.view(np.int16)).view(torch.bfloat16).permute(0, 2, 1, 3)
    dv = dev(vb.view(np.int16)).view(torch.bfloat16).permute(0, 2, 1, 3)
    out = rest.rest_tree_attention(dq, dk, dv, dev(mask.view(np.int64)), P, 0.088)
    torch.cuda.synchronize()
    want = oracle.tree_attention(synth.bf16_bits_to_f32(qb), synth.bf16_bits_to_f32(kb).transpose(0, 2, 1, 3),
                                 synth.bf16_bits_to_f32(vb).transpose(0, 2, 1, 3), mask, P, 0.088)
    assert np.abs(out.float().cpu().numpy() - want).max() <= 2e-2
    with pytest.raises(rest.RestError):
        rest.rest_tree_attention(dq, dk, dv, dev(mask.view(np.int64)), P, -1.0)
    with pytest.raises(rest.RestError):
        rest.rest_tree_attention(dq[..., :64].contiguous(), dk[..., :64].contiguous(), dv[..., :64].contiguous(),
                                 dev(mask.view(np.int64)), P, 0.1)


@pytest.mark.parametrize("dtype,Hkv,g,T,P,per_batch", [("bf16", 2, 4, 16, 100, False), ("bf16", 3, 4, 64, 515, True),
                                                       ("bf16", 8, 2, 33, 64, False), ("fp32", 2, 3, 20, 40, False),
                                                       ("bf16", 2, 8, 64, 300, False), ("bf16", 1, 16, 64, 100, True),
                                                       ("bf16", 3, 6, 100, 77, False), ("fp32", 1, 8, 40, 50, False)])
def test_grouped_query_attention_as_a_view(dtype, Hkv, g, T, P, per_batch):
    """g query heads per K/V head: the call sees H = Hkv heads with g*T query rows each and mask_rows = T."""
    Nb = 2
    masks = np.stack([synth.random_tree(T, 60 + nb)[3] for nb in range(Nb)])
    mask = masks if per_batch else masks[0]
    if dtype == "bf16":
        qb = synth.normal_bf16_bits(71, (Nb, Hkv * g, T, 128))
        kb = synth.normal_bf16_bits(72, (Nb, Hkv, P + T, 128))
        vb = synth.normal_bf16_bits(73, (Nb, Hkv, P + T, 128))
        q, k, v = (synth.bf16_bits_to_f32(x) for x in (qb, kb, vb))
        dq, dk, dv = (dev(x.view(np.int16)).view(torch.bfloat16) for x in (qb, kb, vb))
    else:
        q, k, v = (synth.normal_f32(71 + i, shp) for i, shp in enumerate([(Nb, Hkv * g, T, 128), (Nb, Hkv, P + T, 128),
                                                                        (Nb, Hkv, P + T, 128)]))
        dq, dk, dv = dev(q), dev(k), dev(v)
    scale = 1.0 / np.sqrt(128.0)
    out = torch.full_like(dq, float("nan"))
    rest.rest_tree_attention(dq.view(Nb, Hkv, g * T, 128), dk, dv, dev(mask.view(np.int64)), P, float(scale),
                             out=out.view(Nb, Hkv, g * T, 128), mask_rows=T)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy().astype(np.float64)
    for nb in range(Nb):
        for h in range(Hkv * g):
            want = oracle.tree_attention(q[nb, h], k[nb, h // g], v[nb, h // g], masks[nb] if per_batch else masks[0], P, scale)
            if dtype == "bf16":
                assert np.abs(got[nb, h] - want).max() <= 2e-2
            else:
                assert np.abs(got[nb, h] - want).max() / np.abs(want).max() <= 1e-3


@pytest.mark.parametrize("n_seq,m,c,seed", [(8, 8, 64, 1), (8, 8, 16, 2), (3, 5, 64, 3), (64, 10, 256, 4), (1, 16, 64, 5)])
def test_random_selection_strategy_matches_oracle(n_seq, m, c, seed):
    corp = synth.make_corpus(200_000, 6, 60)
    ctx, lens = synth.make_contexts(corp, 24, 64, 17)
    index = rest.rest_build_index(dev(corp.tokens), 4)
    out = rest.rest_retrieve(index, dev(ctx), dev(lens), max_matches=700, cont_len=m, max_nodes=c, random_seqs=n_seq,
                             seed=seed)
    torch.cuda.synchronize()
    words = (c + 63) // 64
    rich = 0
    for b in range(24):
        want = oracle.draft_tree(corp.tokens, ctx[b], 16, 2, 700, m, c, random_seqs=n_seq, seed=seed, ctx_index=b)
        assert (int(out.matched_len[b]), int(out.match_count[b]), int(out.n_nodes[b])) == \
            (want.matched_len, want.match_count, want.n_nodes), b
        np.testing.assert_array_equal(out.draft_tokens[b].cpu().numpy(), want.draft_tokens)
        np.testing.assert_array_equal(out.parent_idx[b].cpu().numpy(), want.parent_idx)
        np.testing.assert_array_equal(out.pos_ids[b].cpu().numpy(), want.pos_ids)
        np.testing.assert_array_equal(out.node_weight[b].cpu().numpy(), want.node_weight)
        np.testing.assert_array_equal(out.tree_mask[b].cpu().numpy().view(np.uint64).reshape(c, words), want.tree_mask)
        rich += want.n_nodes > m
    assert rich >= 3 or n_seq == 1


@pytest.mark.parametrize("K,m,c,n_seq,sa_bytes", [(1, 10, 64, 0, 4), (7, 10, 64, 0, 4), (64, 10, 64, 0, 8), (300, 16, 256, 0, 4),
                                                  (100, 8, 64, 8, 4), (8192, 10, 64, 0, 4)])
def test_evenly_spaced_match_sample_matches_oracle(K, m, c, n_seq, sa_bytes):
    """More occurrences than max_matches: the kept ones are spread over the whole sorted range."""
    corp = synth.make_corpus(200_000, 8, 40)
    ctx, lens = synth.make_contexts(corp, 24, 64, 23)
    t = corp.tokens.astype(np.int64)      # eight contexts end in the most frequent pairs: hundreds to thousands of occurrences
    pairs, cnt = np.unique(t[:-1] * 65536 + t[1:], return_counts=True)
    top = pairs[np.argsort(-cnt, kind="stable")[:8]]
    ctx[:8, -2] = top >> 16
    ctx[:8, -1] = top & 65535
    ctx[:8, -3] = 31_999
    index = rest.rest_build_index(dev(corp.tokens), sa_bytes)
    out = rest.rest_retrieve(index, dev(ctx), dev(lens), max_matches=K, cont_len=m, max_nodes=c, random_seqs=n_seq, seed=9,
                             strided=True)
    head = rest.rest_retrieve(index, dev(ctx), dev(lens), max_matches=K, cont_len=m, max_nodes=c, random_seqs=n_seq, seed=9)
    torch.cuda.synchronize()
    words = (c + 63) // 64
    capped = differs = 0
    for b in range(24):
        want = oracle.draft_tree(corp.tokens, ctx[b], 16, 2, K, m, c, random_seqs=n_seq, seed=9, ctx_index=b, strided=True)
        assert (int(out.matched_len[b]), int(out.match_count[b]), int(out.n_nodes[b])) == \
            (want.matched_len, want.match_count, want.n_nodes), b
        np.testing.assert_array_equal(out.draft_tokens[b].cpu().numpy(), want.draft_tokens)
        np.testing.assert_array_equal(out.parent_idx[b].cpu().numpy(), want.parent_idx)
        np.testing.assert_array_equal(out.pos_ids[b].cpu().numpy(), want.pos_ids)
        np.testing.assert_array_equal(out.node_weight[b].cpu().numpy(), want.node_weight)
        np.testing.assert_array_equal(out.tree_mask[b].cpu().numpy().view(np.uint64).reshape(c, words), want.tree_mask)
        if want.match_count > K:
            capped += 1
            differs += not torch.equal(out.node_weight[b], head.node_weight[b]) or \
                not torch.equal(out.draft_tokens[b], head.draft_tokens[b])
        else:                               # nothing dropped: the option changes nothing
            assert torch.equal(out.draft_tokens[b], head.draft_tokens[b])
            assert torch.equal(out.node_weight[b], head.node_weight[b])
    if K < 8192:
        assert capped >= 6 and (differs >= 3 or K == 1), (capped, differs)


@pytest.mark.parametrize("n,dtype,sa_bytes,depth", [(5_000, np.int32, 4, 2), (40_000, np.uint16, 4, 8), (150_000, np.int32, 8, 32),
                                                     (150_000, np.int32, 4, 26), (70_001, np.int32, 4, 1)])
def test_depth_limited_index_matches_oracle_order(n, dtype, sa_bytes, depth):
    """Few distinct tokens and planted repeats, so that many positions share their first `depth` tokens."""
    rng_tokens = synth.randint(61, np.arange(n), 0, 3).astype(dtype)
    rng_tokens[n // 2:n // 2 + n // 5] = rng_tokens[:n // 5]          # a long repeat: full doubling would need many rounds
    index = rest.rest_build_index_prefix(dev(rng_tokens), sa_bytes, depth)
    used = index.sort_depth
    assert used >= max(depth, 2) and used < 2 * max(depth, 2) and used & (used - 1) == 0
    got = index.suffix_array().cpu().numpy()
    np.testing.assert_array_equal(got, oracle.prefix_sorted_array(rng_tokens, used))
    assert got.dtype == (np.int32 if sa_bytes == 4 else np.int64)
    # a depth the repeats do not reach: the suffix array itself, marked as such
    plain = synth.randint(62, np.arange(3000), 0, 30_000).astype(np.int32)
    full = rest.rest_build_index_prefix(dev(plain), 4, 16)
    assert full.sort_depth == 0 and oracle.check_suffix_array(plain, full.suffix_array().cpu().numpy()) == -1


def test_depth_limited_index_serves_retrieval_like_the_suffix_array(tmp_path):
    corp = synth.make_corpus(300_000, 12, 30)
    toks = corp.tokens.copy()
    toks[200_000:260_000] = toks[10_000:70_000]                         # duplicated "document"
    d_corpus = dev(toks)
    full = rest.rest_build_index(d_corpus, 4)
    lim = rest.rest_build_index_prefix(d_corpus, 4, 32)
    assert full.sort_depth == 0 and lim.sort_depth == 32
    assert not torch.equal(full.suffix_array(), lim.suffix_array())
    ctx, lens = synth.make_contexts(corp, 32, 64, 13)
    ctx[:8, :] = toks[30_000 - 64 + np.arange(8)[:, None] * 500 + np.arange(64)[None, :]]   # contexts inside the duplicate
    for kw in (dict(max_matches=5000, cont_len=16, max_nodes=64), dict(max_matches=7, cont_len=10, max_nodes=64, strided=True),
               dict(max_matches=300, cont_len=8, max_nodes=256, random_seqs=8, seed=4)):
        a = rest.rest_retrieve(full, dev(ctx), dev(lens), **kw)
        b = rest.rest_retrieve(lim, dev(ctx), dev(lens), **kw)
        torch.cuda.synchronize()
        for name in ("draft_tokens", "parent_idx", "pos_ids", "node_weight", "tree_mask", "n_nodes", "matched_len", "match_count"):
            assert torch.equal(getattr(a, name), getattr(b, name)), (name, kw)
        assert int(a.n_nodes.sum()) > 100
    for bi in range(0, 32, 5):                                           # and the oracle's definition directly
        want = oracle.draft_tree(toks, ctx[bi], 16, 2, 5000, 16, 64)
        got = rest.rest_retrieve(lim, dev(ctx[bi:bi + 1]), dev(lens[bi:bi + 1]), max_matches=5000, cont_len=16, max_nodes=64)
        np.testing.assert_array_equal(got.draft_tokens[0].cpu().numpy(), want.draft_tokens)
        np.testing.assert_array_equal(got.node_weight[0].cpu().numpy(), want.node_weight)
    # the limit is enforced: a 16-token index cannot serve n_max + cont_len = 26
    short = rest.rest_build_index_prefix(d_corpus, 4, 16)
    assert short.sort_depth == 16
    with pytest.raises(rest.RestError) as e:
        rest.rest_retrieve(short, dev(ctx), dev(lens), max_matches=100, cont_len=10, max_nodes=64)
    assert e.value.status == rest.REST_UNSUPPORTED
    rest.rest_retrieve(short, dev(ctx), dev(lens), n_max=8, max_matches=100, cont_len=8, max_nodes=64)
    # the file keeps the depth
    p = str(tmp_path / "lim.restsa")
    rest.rest_index_save(lim, p)
    assert oracle.read_index_file(p)[5] == 32
    back = rest.rest_index_load(p, d_corpus)
    assert back.sort_depth == 32 and torch.equal(back.suffix_array(), lim.suffix_array())
    oracle.write_index_file(p, toks, oracle.prefix_sorted_array(toks, 32).astype(np.int32), sort_depth=32)
    theirs = rest.rest_index_load(p, d_corpus)
    assert theirs.sort_depth == 32 and torch.equal(theirs.suffix_array(), lim.suffix_array())
    torch.cuda.synchronize()


def test_datastore_in_pinned_host_memory():
    """A datastore that does not fit the GPU stays in pinned host memory; retrieval reads it in place."""
    corp = synth.make_corpus(400_000, 14, 40)
    ctx, lens = synth.make_contexts(corp, 16, 64, 29)
    sa = oracle.suffix_array(corp.tokens).astype(np.int32)
    h_corpus = torch.empty(corp.tokens.shape, dtype=torch.int32, pin_memory=True)
    h_corpus.copy_(torch.from_numpy(corp.tokens))
    h_sa = torch.empty(sa.shape, dtype=torch.int32, pin_memory=True)
    h_sa.copy_(torch.from_numpy(sa))
    index = rest.rest_index_from_sa(h_corpus, h_sa)        # refuses memory the device cannot address
    out = rest.rest_retrieve(index, dev(ctx), dev(lens), max_matches=1000, cont_len=10, max_nodes=64)
    torch.cuda.synchronize()
    some = 0
    for b in range(16):
        want = oracle.draft_tree(corp.tokens, ctx[b], 16, 2, 1000, 10, 64)
        assert_tree_equal(tree_to_numpy(out, b), want, f"context {b}")
        some += want.n_nodes > 0
    assert some >= 6
    with pytest.raises(TypeError):                         # ordinary host memory is not accepted
        rest.rest_index_from_sa(torch.from_numpy(corp.tokens), torch.from_numpy(sa))


def test_index_file_round_trip_and_exchange_with_the_oracle(tmp_path):
    corp = synth.make_corpus(300_000, 4, 30)
    d_corpus = dev(corp.tokens)
    index = rest.rest_build_index(d_corpus, 4)
    p = str(tmp_path / "a.restsa")
    rest.rest_index_save(index, p)
    # the oracle reads what the library wrote: header, fingerprint, and the array is the suffix array by definition
    n, tb, sb, fp, sa, depth = oracle.read_index_file(p)
    assert (n, tb, sb) == (300_000, 4, 4) and fp == oracle.corpus_fingerprint(corp.tokens)
    assert oracle.check_suffix_array(corp.tokens, sa) == -1
    # the library reads its own file back: same array, same retrieval results
    loaded = rest.rest_index_load(p, d_corpus)
    assert torch.equal(loaded.suffix_array(), index.suffix_array())
    ctx, lens = synth.make_contexts(corp, 16, 64, 9)
    a = rest.rest_retrieve(index, dev(ctx), dev(lens), max_matches=500, cont_len=8, max_nodes=32)
    b = rest.rest_retrieve(loaded, dev(ctx), dev(lens), max_matches=500, cont_len=8, max_nodes=32)
    torch.cuda.synchronize()
    for name in ("draft_tokens", "parent_idx", "pos_ids", "node_weight", "tree_mask", "n_nodes", "matched_len", "match_count"):
        assert torch.equal(getattr(a, name), getattr(b, name)), name
    # the library reads a file the oracle wrote (uint16 tokens, 64-bit entries)
    small = synth.make_corpus(5000, 5, 3, dtype=np.uint16)
    q = str(tmp_path / "b.restsa")
    oracle.write_index_file(q, small.tokens, oracle.suffix_array(small.tokens).astype(np.int64))
    from_oracle = rest.rest_index_load(q, dev(small.tokens))
    np.testing.assert_array_equal(from_oracle.suffix_array().cpu().numpy(), oracle.suffix_array(small.tokens))
    # wrong stream, damaged and truncated files
    other = corp.tokens.copy()
    other[12345] ^= 1
    with pytest.raises(rest.RestError) as e:
        rest.rest_index_load(p, dev(other))
    assert e.value.status == rest.REST_BAD_FILE
    with pytest.raises(rest.RestError) as e:
        rest.rest_index_load(p, dev(corp.tokens[:-1].copy()))
    assert e.value.status == rest.REST_BAD_FILE
    raw = open(p, "rb").read()
    open(p, "wb").write(b"RESTSA02" + raw[8:])
    with pytest.raises(rest.RestError) as e:
        rest.rest_index_load(p, d_corpus)
    assert e.value.status == rest.REST_BAD_FILE
    open(p, "wb").write(raw[:-100])
    with pytest.raises(rest.RestError) as e:
        rest.rest_index_load(p, d_corpus)
    assert e.value.status == rest.REST_IO_ERROR
    with pytest.raises(rest.RestError) as e:
        rest.rest_index_save(index, str(tmp_path / "no-such-dir" / "c.restsa"))
    assert e.value.status == rest.REST_IO_ERROR


# ------------------------------------------------------------------ acceptance
def test_results_repeat_bit_for_bit():
    """The same call on the same inputs, many times: every output identical to the first run's (sums are taken in
    a fixed order everywhere; nothing depends on which workgroup arrives first)."""
    corp = synth.make_corpus(300_000, seed=17, n_motifs=60, copies=50)
    d_corpus = dev(corp.tokens)
    sa0 = rest.rest_build_index(d_corpus, 4).suffix_array().clone()
    index = rest.rest_build_index(d_corpus, 4)
    assert torch.equal(index.suffix_array(), sa0)
    ctx, lens = synth.make_contexts(corp, 16, 64, 3)
    d_ctx, d_lens = dev(ctx), dev(lens)
    prm = dict(n_max=16, n_min=2, max_matches=5000, cont_len=16, max_nodes=64)
    first = rest.rest_retrieve(index, d_ctx, d_lens, **prm)
    fields = ("draft_tokens", "parent_idx", "pos_ids", "node_weight", "tree_mask", "n_nodes", "matched_len", "match_count")
    keep = [getattr(first, f).clone() for f in fields]
    for _ in range(50):
        again = rest.rest_retrieve(index, d_ctx, d_lens, **prm)
        for f, want in zip(fields, keep):
            assert torch.equal(getattr(again, f), want), f
    g = torch.Generator(device="cuda")
    g.manual_seed(8)
    mask = first.tree_mask[0]
    # one layer cut into spans and merged; more units than streams with a cut remainder; with a whole extra round
    for Nb, H, P in [(1, 32, 2048), (22, 50, 100), (40, 40, 50)]:
        q = torch.randn((Nb, H, 64, 128), generator=g, device="cuda").to(torch.bfloat16)
        k = torch.randn((Nb, H, P + 64, 128), generator=g, device="cuda").to(torch.bfloat16)
        v = torch.randn((Nb, H, P + 64, 128), generator=g, device="cuda").to(torch.bfloat16)
        want = rest.rest_tree_attention(q, k, v, mask, P, 0.0884).clone()
        for _ in range(30):
            assert torch.equal(rest.rest_tree_attention(q, k, v, mask, P, 0.0884), want), (Nb, H, P)
    logits = torch.randn((65, 32000), generator=g, device="cuda") * 3
    u = torch.rand(65, generator=g, device="cuda")
    want = rest.rest_sample_ids(logits, u, 0.7, 0.95).clone()
    for _ in range(20):
        assert torch.equal(rest.rest_sample_ids(logits, u, 0.7, 0.95), want)


def test_calls_from_several_host_threads():
    """Four host threads, each on its own stream with its own outputs and workspaces, drive retrieval (with
    parameters of different LDS needs), attention and acceptance at once; every result equals the one a single
    thread got before."""
    import threading
    corp = synth.make_corpus(200_000, seed=31, n_motifs=40, copies=50)
    ctx, lens = synth.make_contexts(corp, 8, 64, 9)
    d_ctx, d_lens = dev(ctx), dev(lens)
    index = rest.rest_build_index(dev(corp.tokens), 4)
    prms = [dict(n_max=16, n_min=2, max_matches=K, cont_len=m, max_nodes=c)
            for K, m, c in [(100, 4, 16), (1000, 10, 64), (5000, 16, 64), (8192, 32, 256)]]
    H, P = 4, 300
    g = torch.Generator(device="cuda")
    g.manual_seed(3)
    scale = float(1 / np.sqrt(128.0))

    def one_pass(prm, seed):
        c = prm["max_nodes"]
        tree = rest.rest_retrieve(index, d_ctx, d_lens, **prm)
        gg = torch.Generator(device="cuda")
        gg.manual_seed(seed)
        q = torch.randn((8, H, c, 128), generator=gg, device="cuda").to(torch.bfloat16)
        k = torch.randn((8, H, P + c, 128), generator=gg, device="cuda").to(torch.bfloat16)
        v = torch.randn((8, H, P + c, 128), generator=gg, device="cuda").to(torch.bfloat16)
        out = rest.rest_tree_attention(q, k, v, tree.tree_mask, P, scale)
        ids = torch.randint(0, 32000, (8, 1 + c), generator=gg, device="cuda", dtype=torch.int32)
        ids[:, 0] = tree.draft_tokens[:, 0]                      # the first draft token is accepted where there is one
        alen, apath, nxt = rest.rest_accept(ids, tree, prm["cont_len"])
        return [tree.draft_tokens, tree.parent_idx, tree.tree_mask, tree.n_nodes, out, alen, apath, nxt]

    want = []
    for i, prm in enumerate(prms):
        want.append([t.clone() for t in one_pass(prm, 100 + i)])
    torch.cuda.synchronize()
    failures = []

    def worker(i):
        try:
            with torch.cuda.stream(torch.cuda.Stream()):
                for rep in range(10):
                    j = (i + rep) % len(prms)
                    got = one_pass(prms[j], 100 + j)
                    torch.cuda.current_stream().synchronize()
                    for a, b in zip(got, want[j]):
                        if not torch.equal(a, b):
                            failures.append((i, rep, j))
        except Exception as e:                                   # noqa: BLE001 - reported below
            failures.append((i, repr(e)))

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(4)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not failures, failures[:5]
    assert int(want[1][3].max()) > 8 and int(want[1][5].max()) >= 1


def test_accept_matches_oracle_on_random_trees():
    B, c, cap = 40, 64, 16
    tree = rest.Tree.empty(B, c, fill=0)
    toks = np.full((B, c), -1, np.int32)
    pars = np.full((B, c), -1, np.int32)
    nn = np.zeros(B, np.int32)
    ids = np.zeros((B, 1 + c), np.int32)
    for b in range(B):
        T = [0, 1, 5, 33, 64][b % 5]
        if T:
            par, dep, tok, _ = synth.random_tree(T, 300 + b)
            toks[b, :T], pars[b, :T] = tok, par
        nn[b] = T
        ids[b] = synth.sampled_ids(500 + b, toks[b], pars[b], T, vocab=30000, p_follow=0.85)
    tree.draft_tokens.copy_(dev(toks))
    tree.parent_idx.copy_(dev(pars))
    tree.n_nodes.copy_(dev(nn))
    for path_cap in (cap, 2):
        alen, apath, nxt = rest.rest_accept(dev(ids), tree, path_cap)
        torch.cuda.synchronize()
        some = 0
        for b in range(B):
            n, path, nt = oracle.accept(ids[b], toks[b], pars[b], int(nn[b]), path_cap)
            assert int(alen[b]) == n and int(nxt[b]) == nt
            np.testing.assert_array_equal(apath[b].cpu().numpy(), path)
            some += n
        assert some > 0


def test_gpu_rest_loop_reproduces_greedy_decoding():
    """Drafts from rest_retrieve + rest_accept on the GPU drive a decoding loop whose output must equal plain
    greedy decoding with the same deterministic toy model (the lossless property of the acceptance rule)."""
    corp = synth.make_corpus(30000, seed=2, n_motifs=40, copies=20, vocab=500)
    corpus = corp.tokens
    succ = {}
    for a, b, c3 in zip(corpus[:-2], corpus[1:-1], corpus[2:]):
        succ[(int(a), int(b))] = int(c3)

    def model(seq):
        key = (seq[-2], seq[-1])
        h = (seq[-1] * 1000003 + seq[-2] * 10007 + seq[-3] * 101) % 7
        return succ[key] if key in succ and h != 0 else (seq[-1] * 31 + seq[-2] * 17 + seq[-3]) % 500

    o = int(corp.motif_offsets[0, 0])
    prompt = corpus[o:o + 6].astype(np.int32).tolist()
    want = oracle.greedy_decode(model, prompt, 50)
    idx = rest.rest_build_index(dev(corpus), 4)
    c, m = 24, 8
    seq, steps = list(prompt), 0
    buf = torch.zeros((1, 128), dtype=torch.int32, device="cuda")
    while len(seq) - len(prompt) < 50:
        t = len(seq)
        buf[0, :t] = torch.tensor(seq, dtype=torch.int32)
        tree = rest.rest_retrieve(idx, buf, torch.tensor([t], dtype=torch.int32, device="cuda"),
                                  max_matches=200, cont_len=m, max_nodes=c)
        T = int(tree.n_nodes[0])
        toks, pars = tree.draft_tokens[0].cpu().numpy(), tree.parent_idx[0].cpu().numpy()
        ids = np.zeros((1, 1 + c), np.int32)
        ids[0, 0] = model(seq)
        for i in range(T):
            path, v = [], i
            while v != -1:
                path.append(int(toks[v]))
                v = int(pars[v])
            ids[0, 1 + i] = model(seq + path[::-1])
        alen, apath, nxt = rest.rest_accept(dev(ids), tree, m)
        for j in range(int(alen[0])):
            seq.append(int(toks[int(apath[0, j])]))
        seq.append(int(nxt[0]))
        steps += 1
    assert seq[len(prompt):len(prompt) + 50] == want
    assert steps < 50
