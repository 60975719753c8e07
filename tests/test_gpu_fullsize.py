"""Full-size GPU parity: the benchmark's own shapes and launch configuration, checked on sampled outputs the
oracle can compute one by one (whole contexts for retrieval, whole (layer, head) slabs for attention) and on
the suffix array's defining property; attention on every (layer or context, head) slab of each launch."""
from concurrent.futures import ThreadPoolExecutor

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


def check_retrieval(corp, index, w, n_contexts, seed, sample):
    ctx, lens = synth.make_contexts(corp, n_contexts, w.ctx_len, seed)
    prm = dict(n_max=w.n_max, n_min=w.n_min, max_matches=w.max_matches, cont_len=w.cont_len, max_nodes=w.max_nodes)
    out = rest.Tree.empty(n_contexts, w.max_nodes, fill=-0x5A5A5A5B)
    rest.rest_retrieve(index, dev(ctx), dev(lens), out=out, **prm)
    torch.cuda.synchronize()
    tok, par = out.draft_tokens.cpu().numpy(), out.parent_idx.cpu().numpy()
    pos, wgt = out.pos_ids.cpu().numpy(), out.node_weight.cpu().numpy()
    msk = out.tree_mask.cpu().numpy().view(np.uint64)
    nn, ml, mc = out.n_nodes.cpu().numpy(), out.matched_len.cpu().numpy(), out.match_count.cpu().numpy()
    lens_seen = set()
    sample = list(sample)
    # Algorithm 1 of the oracle is one scan of the whole stream per context: the scans (C code, no shared state) run
    # side by side in threads; Algorithm 2 and the layout follow one context at a time, as oracle.draft_tree does
    with ThreadPoolExecutor(max_workers=min(16, len(sample))) as pool:
        found = list(pool.map(lambda b: oracle.retrieve(corp.tokens, ctx[b], w.n_max, w.n_min, w.max_matches, w.cont_len,
                                                        one_pass=True), sample))
    for b, got in zip(sample, found):
        want = oracle.select_drafts(got.rows, got.row_len, w.max_nodes, np.argsort(got.row_pos, kind="stable").astype(np.int64))
        want.matched_len, want.match_count = got.matched_len, got.match_count
        assert (int(ml[b]), int(mc[b]), int(nn[b])) == (want.matched_len, want.match_count, want.n_nodes), b
        np.testing.assert_array_equal(tok[b], want.draft_tokens)
        np.testing.assert_array_equal(par[b], want.parent_idx)
        np.testing.assert_array_equal(pos[b], want.pos_ids)
        np.testing.assert_array_equal(wgt[b], want.node_weight)
        np.testing.assert_array_equal(msk[b], want.tree_mask)
        lens_seen.add(want.matched_len)
    # properties that hold for every context at any size
    T = nn.astype(np.int64)
    cols = np.arange(w.max_nodes)[None, :]
    live = cols < T[:, None]
    assert ((par < cols) | ~live).all() and (par[~live] == -1).all() and (tok[~live] == -1).all()
    assert ((pos >= 1) & (pos <= w.cont_len))[live].all() and (pos[~live] == 0).all()
    assert (mc >= 0).all() and ((ml == 0) == (mc == 0)).all() and (ml <= w.n_max).all()
    return lens_seen


def attention_check_all_slabs(Nb, H, T, P, seed, mask_np, kv8=False):
    """Inputs from torch's seeded GPU generator (as bench.py does), one launch over all Nb x H slabs, and every slab
    of the output against the float64 oracle, one batch entry (a layer or a context: H slabs) at a time.  mask_np:
    [T, words], shared, or [Nb, T, words], one per batch entry.  kv8: K and V as E4M3 bytes with a scale per slab."""
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    q = torch.randn((Nb, H, T, 128), generator=g, device="cuda").to(torch.bfloat16)
    scale = 1.0 / np.sqrt(128.0)
    ks = vs = None
    if kv8:
        ks = 0.25 + torch.rand((Nb, H), generator=g, device="cuda")
        vs = 0.25 + torch.rand((Nb, H), generator=g, device="cuda")
        k = (torch.randn((Nb, H, P + T, 128), generator=g, device="cuda") / ks[..., None, None]).to(torch.float8_e4m3fn).view(torch.uint8)
        v = (torch.randn((Nb, H, P + T, 128), generator=g, device="cuda") / vs[..., None, None]).to(torch.float8_e4m3fn).view(torch.uint8)
    else:
        k = torch.randn((Nb, H, P + T, 128), generator=g, device="cuda").to(torch.bfloat16)
        v = torch.randn((Nb, H, P + T, 128), generator=g, device="cuda").to(torch.bfloat16)
    out = torch.full_like(q, float("nan"))
    rest.rest_tree_attention(q, k, v, dev(mask_np.view(np.int64)), P, float(scale), out=out, k_scale=ks, v_scale=vs)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    worst = 0.0
    for nb in range(Nb):
        m = mask_np[nb] if mask_np.ndim == 3 else mask_np
        if kv8:
            ref = oracle.tree_attention_fp8kv(q[nb].float().cpu().numpy()[None], k[nb].cpu().numpy()[None], v[nb].cpu().numpy()[None],
                                              ks[nb].cpu().numpy()[None], vs[nb].cpu().numpy()[None], m, P, scale)[0]
        else:
            ref = oracle.tree_attention(q[nb].float().cpu().numpy(), k[nb].float().cpu().numpy(), v[nb].float().cpu().numpy(),
                                        m, P, scale)
        err = float(np.abs(out[nb].float().cpu().numpy() - ref).max())
        assert err <= 2e-2, (nb, err)
        worst = max(worst, err)
    return worst


def test_llama7b_index_retrieval_attention_at_benchmark_shape():
    w = synth.WORKLOADS["llama7b"]
    corp = synth.make_corpus(w.n_tokens, w.corpus_seed, w.n_motifs)
    d_corpus = dev(corp.tokens)
    index = rest.rest_build_index(d_corpus, 4)
    sa = index.suffix_array().cpu().numpy()
    assert oracle.check_suffix_array(corp.tokens, sa) == -1          # permutation + strictly increasing suffixes
    del sa
    # the 16 contexts the benchmark rotates over: every one of them against the oracle
    seen = check_retrieval(corp, index, w, 16, w.query_seed, range(16))
    assert 16 in seen and min(seen) <= 4                              # long planted matches and short fallbacks
    # the batched throughput set: 4096 contexts in one launch, a sample of them against the oracle
    check_retrieval(corp, index, w, 4096, w.query_seed + 1, [0, 1, 2, 3, 1000, 2047, 4094, 4095])
    # attention in the benchmark's launch configuration, with the tree of context 0
    tree = oracle.draft_tree(corp.tokens, synth.make_contexts(corp, 1, w.ctx_len, w.query_seed)[0][0],
                             w.n_max, w.n_min, w.max_matches, w.cont_len, w.max_nodes, one_pass=True)
    attention_check_all_slabs(w.layers, w.heads, w.max_nodes, w.kv_len, w.qkv_seed, tree.tree_mask)


def test_llama7b_cache_steps_at_benchmark_shape():
    """rest_rope_append and rest_kv_compact over all 32 layers x 32 heads in one call each, as bench.py times them;
    sampled (layer, head) slabs against the oracle."""
    w = synth.WORKLOADS["llama7b"]
    Nb, H, T, P = w.layers, w.heads, w.max_nodes, w.kv_len
    g = torch.Generator(device="cuda")
    g.manual_seed(w.qkv_seed + 7)
    q, kn, vn = (torch.randn((Nb, H, T, 128), generator=g, device="cuda").to(torch.bfloat16) for _ in range(3))
    kc, vc = (torch.randn((Nb, H, P + T, 128), generator=g, device="cuda").to(torch.bfloat16) for _ in range(2))
    par, dep, tok, mask = synth.random_tree(T, 77)
    q0, kc0, vc0 = q.clone(), kc.clone(), vc.clone()
    rest.rest_rope_append(q, kn, vn, kc, vc, dev(dep.astype(np.int32)), P)
    leaf = int(np.argmax(dep))
    path = []
    v = leaf
    while v != -1:
        path.append(v)
        v = int(par[v])
    path = np.array(path[::-1] + [-1] * (w.cont_len - len(path)), dtype=np.int32)
    A = int(dep[leaf])
    kc1, vc1 = kc.clone(), vc.clone()
    rest.rest_kv_compact(kc, vc, dev(path[None]), dev(np.array([A], dtype=np.int32)), T, P)
    torch.cuda.synchronize()
    f64 = lambda t: t.float().cpu().numpy().astype(np.float64)
    rng = np.random.default_rng(5)
    picks = {(0, 0), (Nb - 1, H - 1)}
    while len(picks) < 12:
        picks.add((int(rng.integers(Nb)), int(rng.integers(H))))
    for a, b in sorted(picks):
        q_ref, k_ref, v_ref = oracle.rope_append(f64(q0[a, b]), f64(kn[a, b]), f64(vn[a, b]), f64(kc0[a, b]), f64(vc0[a, b]),
                                                 dep, P - 1, P)
        for got, ref, src in ((f64(q[a, b]), q_ref, f64(q0[a, b])), (f64(kc1[a, b])[P:], k_ref[P:], f64(kn[a, b]))):
            mag = np.abs(src[:, :64]) + np.abs(src[:, 64:])
            bound = 2.0 ** -8 * np.abs(ref) + 2.0 ** -21 * np.concatenate([mag, mag], axis=-1)
            assert (np.abs(got - ref) <= bound).all()
        np.testing.assert_array_equal(f64(kc1[a, b])[:P], f64(kc0[a, b])[:P])
        np.testing.assert_array_equal(f64(vc1[a, b]), v_ref)
        np.testing.assert_array_equal(f64(kc[a, b]), oracle.kv_compact(f64(kc1[a, b]), P, path, A))
        np.testing.assert_array_equal(f64(vc[a, b]), oracle.kv_compact(f64(vc1[a, b]), P, path, A))


def test_llama7b_attention_on_8bit_cache_at_benchmark_shape():
    """The 8-bit cache in the benchmark's launch configuration (32 layers x 32 heads in one call, 2048 + 64 keys):
    every (layer, head) slab against the oracle."""
    w = synth.WORKLOADS["llama7b"]
    attention_check_all_slabs(w.layers, w.heads, w.max_nodes, w.kv_len, w.qkv_seed + 11, synth.random_tree(w.max_nodes, 78)[3], kv8=True)


@pytest.mark.parametrize("P", [1024, 4096, 8192])
@pytest.mark.parametrize("T", [16, 64, 128, 256])
def test_sweep_shapes_random_trees(T, P):
    """Tree-size / KV-length sweep at the 7B head shape with random tries (branching <= 8, depth <= 16)."""
    mask = synth.random_tree(T, 14 + T)[3]
    attention_check_all_slabs(32, 32, T, P, 100 + T + P, mask)


def test_llama13b_shape():
    w = synth.WORKLOADS["llama13b"]
    corp = synth.make_corpus(w.n_tokens, w.corpus_seed, w.n_motifs)
    index = rest.rest_build_index(dev(corp.tokens), 4)
    sa = index.suffix_array().cpu().numpy()
    assert oracle.check_suffix_array(corp.tokens, sa) == -1
    del sa
    check_retrieval(corp, index, w, 8, w.query_seed, range(8))
    mask = synth.random_tree(w.max_nodes, 3)[3]
    attention_check_all_slabs(w.layers, w.heads, w.max_nodes, w.kv_len, w.qkv_seed, mask)


def batched_uint16_int64(n_tokens, n_motifs, sample):
    """The batched workload's step on a datastore of n_tokens 16-bit tokens with 64-bit suffix-array entries: index
    by its definition, 32 contexts of 1024 tokens in one retrieval launch, one layer of attention over the 32
    contexts with a mask per context."""
    w = synth.WORKLOADS["batched2b"]
    corp = synth.make_corpus(n_tokens, w.corpus_seed, n_motifs, dtype=np.uint16, workers=16)
    index = rest.rest_build_index(dev(corp.tokens), 8)
    sa = index.suffix_array().cpu().numpy()
    assert sa.dtype == np.int64
    assert oracle.check_suffix_array(corp.tokens, sa) == -1
    del sa
    check_retrieval(corp, index, w, w.batch, w.query_seed, sample)
    Nb, H, T, P = w.batch, w.heads, w.max_nodes, w.kv_len
    masks = np.stack([synth.random_tree(T, 500 + i)[3] for i in range(Nb)])
    attention_check_all_slabs(Nb, H, T, P, w.qkv_seed, masks)


def test_batched_uint16_int64_on_a_tenth_of_the_datastore():
    w = synth.WORKLOADS["batched2b"]
    batched_uint16_int64(w.n_tokens // 10, w.n_motifs // 10, range(w.batch))


def test_batched_2b_uint16_int64():
    """The full datastore: 2 * 10^9 tokens, suffix-array entries beyond 2^31, all 32 contexts against the oracle."""
    w = synth.WORKLOADS["batched2b"]
    batched_uint16_int64(w.n_tokens, w.n_motifs, range(w.batch))
