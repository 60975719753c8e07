"""GPU parity of rest_rope_append and rest_kv_compact against the CPU oracle.

Rotated values: the library forms angles in fp64 and rotates in fp32, so a result differs from the oracle's
float64 value by the final rounding to bf16 (half a unit in the last place, relative 2^-9) plus fp32 rounding of the
two products (2^-23 of their magnitudes, which matters only where the products cancel).  The bound asserted is
2^-8 |ref| + 2^-21 (|a| + |b|).  Values and moved rows are compared bit for bit."""
import numpy as np
import pytest
import torch

import oracle
import synth

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2311_08252_amd as rest


def bf16_tensor(shape, seed):
    bits = synth.normal_bf16_bits(seed, shape)
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16), synth.bf16_bits_to_f32(bits).astype(np.float64)


def to_np(t):
    return t.float().cpu().numpy().astype(np.float64)


def assert_rotated(got, ref, src):
    """src: the unrotated input rows; |a| + |b| per plane bounds the products' rounding."""
    h = src.shape[-1] // 2
    mag = np.abs(src[..., :h]) + np.abs(src[..., h:])
    mag = np.concatenate([mag, mag], axis=-1)
    bound = 2.0 ** -8 * np.abs(ref) + 2.0 ** -21 * mag
    err = np.abs(got - ref)
    assert (err <= bound).all(), float((err - bound).max())


@pytest.mark.parametrize("Nb,H,T,P,extra,per_batch,theta", [
    (2, 3, 5, 7, 0, False, 10000.0),
    (1, 8, 64, 200, 3, False, 10000.0),
    (3, 5, 33, 100, 9, True, 1000000.0),
    (4, 32, 64, 4096, 0, True, 500000.0),
    (1, 1, 1, 0, 0, False, 10000.0),
    (2, 9, 256, 17, 5, False, 10000.0),
])
def test_rope_append_matches_oracle(Nb, H, T, P, extra, per_batch, theta):
    L = P + T + extra
    q, q_np = bf16_tensor((Nb, H, T, 128), 1)
    kn, kn_np = bf16_tensor((Nb, H, T, 128), 2)
    vn, vn_np = bf16_tensor((Nb, H, T, 128), 3)
    kc, kc_np = bf16_tensor((Nb, H, L, 128), 4)
    vc, vc_np = bf16_tensor((Nb, H, L, 128), 5)
    rng = np.random.default_rng(T + P)
    pos_np = rng.integers(0, 17, size=(Nb, T) if per_batch else (T,)).astype(np.int32)
    pos_b = pos_np[:, None, :] if per_batch else pos_np
    off = P - 1 if P else 41
    q_ref, k_ref, v_ref = oracle.rope_append(q_np, kn_np, vn_np, kc_np, vc_np,
                                             np.broadcast_to(pos_b, (Nb, H, T)) if per_batch else pos_np, off, P, theta)
    rest.rest_rope_append(q, kn, vn, kc, vc, torch.from_numpy(pos_np).cuda(), P, off, theta)
    torch.cuda.synchronize()
    assert_rotated(to_np(q), q_ref, q_np)
    assert_rotated(to_np(kc)[:, :, P:P + T], k_ref[:, :, P:P + T], kn_np)
    # untouched rows and the appended values are exact
    np.testing.assert_array_equal(to_np(kc)[:, :, :P], kc_np[:, :, :P])
    np.testing.assert_array_equal(to_np(kc)[:, :, P + T:], kc_np[:, :, P + T:])
    np.testing.assert_array_equal(to_np(vc), v_ref)
    # the inputs k_new / v_new are not modified
    np.testing.assert_array_equal(to_np(kn), kn_np)


def test_rope_append_strided_inputs_from_a_fused_projection():
    """q, k, v as slices of one [Nb, T, 3, H, D] projection output; caches with padded rows."""
    Nb, H, T, P = 2, 4, 10, 12
    fused, fused_np = bf16_tensor((Nb, T, 3, H, 128), 7)
    q, kn, vn = (fused[:, :, i].permute(0, 2, 1, 3) for i in range(3))
    q_np, kn_np, vn_np = (fused_np[:, :, i].transpose(0, 2, 1, 3) for i in range(3))
    big_k, big_k_np = bf16_tensor((Nb, H, P + T, 256), 8)
    big_v, big_v_np = bf16_tensor((Nb, H, P + T, 256), 9)
    kc, vc = big_k[..., :128], big_v[..., 128:]
    pos = np.arange(1, T + 1, dtype=np.int32)
    q_ref, k_ref, v_ref = oracle.rope_append(q_np, kn_np, vn_np, big_k_np[..., :128], big_v_np[..., 128:], pos, P - 1, P)
    rest.rest_rope_append(q, kn, vn, kc, vc, torch.from_numpy(pos).cuda(), P)
    torch.cuda.synchronize()
    assert_rotated(to_np(q), q_ref, q_np)
    assert_rotated(to_np(kc)[:, :, P:], k_ref[:, :, P:], kn_np)
    np.testing.assert_array_equal(to_np(vc), v_ref)
    # the halves of the padded rows that do not belong to the caches are untouched
    np.testing.assert_array_equal(to_np(big_k[..., 128:]), big_k_np[..., 128:])
    np.testing.assert_array_equal(to_np(big_v[..., :128]), big_v_np[..., :128])


@pytest.mark.parametrize("Nb,H,T,P,cap,paths", [
    (1, 2, 6, 3, 4, [[1, 3, -1, -1]]),
    (2, 3, 8, 5, 5, [[0, 1, 2, 3, 4]]),                  # chain accepted in full: already in place
    (2, 3, 8, 5, 5, [[1, 2, 5, -1, -1]]),                # row P+1 is read by move 0 and written by move 1
    (3, 4, 16, 9, 6, [[2, 5, 9, 15, -1, -1], [-1] * 6, [0, 3, 4, 7, 8, 11]]),     # per batch, one empty
    (1, 32, 64, 2048, 16, [[0, 2, 7, 12, 20, 33, 41, 63] + [-1] * 8]),
    (1, 1, 40, 0, 32, [list(range(8, 40))]),             # the longest path the call takes
    (2, 2, 8, 3, 4, [[2, 0, 1, -1]]),                    # not increasing (no tree gives this): old rows move all the same
])
def test_kv_compact_matches_oracle_bit_for_bit(Nb, H, T, P, cap, paths):
    kc, kc_np = bf16_tensor((Nb, H, P + T + 2, 128), 11)
    vc, vc_np = bf16_tensor((Nb, H, P + T + 2, 128), 12)
    path = np.array(paths, dtype=np.int32)
    lens = np.array([sum(1 for x in row if x >= 0) for row in paths], dtype=np.int32)
    k_ref, v_ref = kc_np.copy(), vc_np.copy()
    for nb in range(Nb):
        row = nb if len(paths) > 1 else 0
        k_ref[nb] = oracle.kv_compact(kc_np[nb], P, path[row], lens[row])
        v_ref[nb] = oracle.kv_compact(vc_np[nb], P, path[row], lens[row])
    rest.rest_kv_compact(kc, vc, torch.from_numpy(path).cuda(), torch.from_numpy(lens).cuda(), T, P)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_np(kc), k_ref)
    np.testing.assert_array_equal(to_np(vc), v_ref)


def test_kv_compact_stops_at_an_entry_that_is_no_draft_row():
    Nb, H, T, P = 1, 2, 8, 4
    kc, kc_np = bf16_tensor((Nb, H, P + T, 128), 13)
    vc, vc_np = bf16_tensor((Nb, H, P + T, 128), 14)
    path = np.array([[3, 9, 5, -1]], dtype=np.int32)     # 9 >= T: only the first move is made, although len says 3
    rest.rest_kv_compact(kc, vc, torch.from_numpy(path).cuda(), torch.tensor([3], dtype=torch.int32).cuda(), T, P)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_np(kc)[0], oracle.kv_compact(kc_np[0], P, path[0], 1))
    np.testing.assert_array_equal(to_np(vc)[0], oracle.kv_compact(vc_np[0], P, path[0], 1))


def codes(shape, seed):
    """seeded E4M3 bytes (every finite code) as a device tensor and a numpy array"""
    c = synth.randint(seed, np.arange(int(np.prod(shape))), 0, 256).astype(np.uint8).reshape(shape)
    c[(c & 0x7F) == 0x7F] = 0x3A
    return torch.from_numpy(c).cuda(), c


def assert_codes(got, want, exact):
    """E4M3 codes written by the library against the oracle's.  The library forms rotation and quotient in fp32, so
    where the exact quotient lies within 2^-16 (relative) of the midpoint of two neighbouring values either neighbour
    is right; everywhere else the codes are equal."""
    diff = got != want
    if diff.any():
        g, w, x = oracle.fp8_e4m3_decode(got[diff]), oracle.fp8_e4m3_decode(want[diff]), exact[diff]
        mid = 0.5 * (g + w)
        step = np.abs(g - w)
        assert (step <= 2.0 ** (np.floor(np.log2(np.maximum(np.abs(x), 2.0 ** -6))) - 3) * 1.001).all()    # neighbours
        assert (np.abs(x - mid) <= 2.0 ** -16 * np.maximum(np.abs(x), 2.0 ** -9)).all(), float(np.abs(x - mid).max())
    return int(diff.sum())


@pytest.mark.parametrize("Nb,H,T,P,extra,per_batch,scales", [
    (2, 3, 5, 7, 0, False, True), (1, 8, 64, 200, 3, False, True), (3, 5, 33, 100, 9, True, True),
    (4, 32, 64, 4096, 0, True, False), (1, 1, 1, 0, 0, False, True), (2, 9, 256, 17, 5, False, True)])
def test_rope_append_on_8bit_cache(Nb, H, T, P, extra, per_batch, scales):
    L = P + T + extra
    q, q_np = bf16_tensor((Nb, H, T, 128), 1)
    kn, kn_np = bf16_tensor((Nb, H, T, 128), 2)
    vn, vn_np = bf16_tensor((Nb, H, T, 128), 3)
    kc, kc_np = codes((Nb, H, L, 128), 4)
    vc, vc_np = codes((Nb, H, L, 128), 5)
    ks = (0.05 + 0.5 * synth.uniform01(6, np.arange(Nb * H))).reshape(Nb, H).astype(np.float32)
    vs = (0.05 + 0.5 * synth.uniform01(7, np.arange(Nb * H))).reshape(Nb, H).astype(np.float32)
    vs.flat[0] = 0.002                                                   # most values of this slab saturate
    if not scales:
        ks[:], vs[:] = 1.0, 1.0
    rng = np.random.default_rng(T + P)
    pos_np = rng.integers(0, 17, size=(Nb, T) if per_batch else (T,)).astype(np.int32)
    off = P - 1 if P else 41
    q_ref, k_ref, v_ref, kx, vx = oracle.rope_append_fp8kv(q_np, kn_np, vn_np, kc_np, vc_np, ks, vs, pos_np, off, P, 10000.0)
    rest.rest_rope_append(q, kn, vn, kc, vc, torch.from_numpy(pos_np).cuda(), P, off, 10000.0,
                          k_scale=torch.from_numpy(ks).cuda() if scales else None,
                          v_scale=torch.from_numpy(vs).cuda() if scales else None)
    torch.cuda.synchronize()
    assert_rotated(to_np(q), q_ref, q_np)
    got_k, got_v = kc.cpu().numpy(), vc.cpu().numpy()
    flips = assert_codes(got_k[:, :, P:P + T], k_ref[:, :, P:P + T], kx)
    assert flips <= 1 + kx.size // 20000, flips
    # a value is a bf16 number divided once: only the fp32 quotient can differ from the exact one
    assert_codes(got_v[:, :, P:P + T], v_ref[:, :, P:P + T], vx)
    if scales:
        assert ((v_ref[0, 0, P:P + T] & 0x7F) == 0x7E).mean() > 0.2     # saturated values were among the cases
    for got, old in ((got_k, kc_np), (got_v, vc_np)):                   # rows outside P .. P+T-1 keep their bytes
        np.testing.assert_array_equal(got[:, :, :P], old[:, :, :P])
        np.testing.assert_array_equal(got[:, :, P + T:], old[:, :, P + T:])


def test_kv_compact_on_8bit_cache_is_bit_exact():
    for Nb, H, T, P, paths in [(2, 3, 8, 5, [[1, 2, 5, -1, -1]]), (3, 4, 16, 9, [[2, 5, 9, 15, -1, -1], [-1] * 6, [0, 3, 4, 7, 8, 11]]),
                               (1, 32, 64, 2048, [[0, 2, 7, 12, 20, 33, 41, 63] + [-1] * 8])]:
        big_k, big_k_np = codes((Nb, H, P + T + 2, 256), 11)             # caches as halves of wider rows
        big_v, big_v_np = codes((Nb, H, P + T + 2, 256), 12)
        kc, vc = big_k[..., :128], big_v[..., 128:]
        path = np.array(paths, dtype=np.int32)
        lens = np.array([sum(1 for x in row if x >= 0) for row in paths], dtype=np.int32)
        k_ref, v_ref = big_k_np.copy(), big_v_np.copy()
        for nb in range(Nb):
            row = nb if len(paths) > 1 else 0
            k_ref[nb, ..., :128] = oracle.kv_compact(big_k_np[nb, ..., :128], P, path[row], lens[row])
            v_ref[nb, ..., 128:] = oracle.kv_compact(big_v_np[nb, ..., 128:], P, path[row], lens[row])
        rest.rest_kv_compact(kc, vc, torch.from_numpy(path).cuda(), torch.from_numpy(lens).cuda(), T, P)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(big_k.cpu().numpy(), k_ref)
        np.testing.assert_array_equal(big_v.cpu().numpy(), v_ref)


def test_layer_step_on_an_8bit_cache():
    """append (quantising) -> tree attention on the 8-bit cache -> compact, against the oracle's chain of the same
    steps; a code that differs at a rounding boundary moves one key element by one grid step, far inside the
    attention tolerance."""
    Nb, H, T, P = 2, 4, 48, 333
    par, dep, tok, mask = synth.random_tree(T, 9)
    q, q_np = bf16_tensor((Nb, H, T, 128), 31)
    kn, kn_np = bf16_tensor((Nb, H, T, 128), 32)
    vn, vn_np = bf16_tensor((Nb, H, T, 128), 33)
    ks = (0.2 + 0.3 * synth.uniform01(34, np.arange(Nb * H))).reshape(Nb, H).astype(np.float32)
    vs = (0.2 + 0.3 * synth.uniform01(35, np.arange(Nb * H))).reshape(Nb, H).astype(np.float32)
    k8 = oracle.fp8_e4m3_encode(synth.normal_f32(36, (Nb, H, P + T, 128)) / ks[..., None, None])
    v8 = oracle.fp8_e4m3_encode(synth.normal_f32(37, (Nb, H, P + T, 128)) / vs[..., None, None])
    kc, vc = torch.from_numpy(k8).cuda(), torch.from_numpy(v8).cuda()
    d_ks, d_vs = torch.from_numpy(ks).cuda(), torch.from_numpy(vs).cuda()
    pos = dep.astype(np.int32)
    rest.rest_rope_append(q, kn, vn, kc, vc, torch.from_numpy(pos).cuda(), P, k_scale=d_ks, v_scale=d_vs)
    out = rest.rest_tree_attention(q, kc, vc, torch.from_numpy(mask.view(np.int64)).cuda(), P, 0.088, k_scale=d_ks, v_scale=d_vs)
    path = np.array([[0, 1, 2, 3, -1, -1]], dtype=np.int32)
    rest.rest_kv_compact(kc, vc, torch.from_numpy(path).cuda(), torch.tensor([4], dtype=torch.int32).cuda(), T, P)
    torch.cuda.synchronize()
    q_ref, k_ref, v_ref, _, _ = oracle.rope_append_fp8kv(q_np, kn_np, vn_np, k8, v8, ks, vs, pos, P - 1, P)
    want = oracle.tree_attention_fp8kv(q_ref, k_ref, v_ref, ks, vs, mask, P, 0.088)
    assert np.abs(to_np(out) - want).max() <= 2e-2
    k_fin = oracle.kv_compact(k_ref, P, path[0], 4)
    assert (kc.cpu().numpy() != k_fin).sum() <= 2
    np.testing.assert_array_equal(vc.cpu().numpy()[:, :, :P], v8[:, :, :P])


def test_layer_step_on_the_gpu_equals_plain_decoding_of_the_accepted_tokens():
    """retrieve -> rope_append -> tree attention -> accept -> compact, all on the GPU, against the oracle's
    token-by-token decoding of the accepted path (positions P, P+1, ...; causal attention)."""
    w = synth.WORKLOADS["tiny"]
    corp = synth.make_corpus(w.n_tokens, w.corpus_seed, w.n_motifs)
    ctx, lens = synth.make_contexts(corp, 8, w.ctx_len, w.query_seed)
    index = rest.rest_build_index(torch.from_numpy(corp.tokens).cuda(), 4)
    c, m, H, P = w.max_nodes, w.cont_len, 4, 64
    done = 0
    for b in range(8):
        tree = rest.rest_retrieve(index, torch.from_numpy(ctx[b:b + 1]).cuda(), torch.from_numpy(lens[b:b + 1]).cuda(),
                                  n_max=w.n_max, n_min=w.n_min, max_matches=w.max_matches, cont_len=m, max_nodes=c)
        torch.cuda.synchronize()
        n = int(tree.n_nodes[0])
        if n < 3:
            continue
        tok, par = tree.draft_tokens[0].cpu().numpy(), tree.parent_idx[0].cpu().numpy()
        ids = synth.sampled_ids(900 + b, tok, par, n)
        q, q_np = bf16_tensor((1, H, c, 128), 20 + b)
        kn, kn_np = bf16_tensor((1, H, c, 128), 30 + b)
        vn, vn_np = bf16_tensor((1, H, c, 128), 40 + b)
        kc, kc_np = bf16_tensor((1, H, P + c, 128), 50 + b)
        vc, vc_np = bf16_tensor((1, H, P + c, 128), 60 + b)
        scale = 1.0 / np.sqrt(128.0)
        rest.rest_rope_append(q, kn, vn, kc, vc, tree.pos_ids[0], P)
        out = rest.rest_tree_attention(q, kc, vc, tree.tree_mask[0], P, float(scale))
        alen, apath, nxt = rest.rest_accept(torch.from_numpy(ids[None]).cuda(), tree, m)
        rest.rest_kv_compact(kc, vc, apath, alen, c, P)
        torch.cuda.synchronize()
        A = int(alen[0])
        path = apath[0].cpu().numpy()[:A]
        k_plain, v_plain = kc_np[0].copy(), vc_np[0].copy()
        for i, node in enumerate(path):
            pos = np.array([P + i])
            # the cache holds bf16: plain decoding would store the rotated key rounded the same way
            k_plain[:, P + i] = oracle.rope(kn_np[0, :, node:node + 1], pos)[:, 0]
            v_plain[:, P + i] = vn_np[0, :, node]
            assert_rotated(to_np(kc)[0, :, P + i], k_plain[:, P + i], kn_np[0, :, node])
            k_plain[:, P + i] = to_np(kc)[0, :, P + i]
            np.testing.assert_array_equal(to_np(vc)[0, :, P + i], v_plain[:, P + i])
            qi = to_np(q)[0, :, node:node + 1]
            s = scale * np.einsum("hqd,hkd->hqk", qi, k_plain[:, :P + i + 1])
            p = np.exp(s - s.max(-1, keepdims=True))
            p /= p.sum(-1, keepdims=True)
            o = np.einsum("hqk,hkd->hqd", p, v_plain[:, :P + i + 1])
            assert np.abs(to_np(out)[0, :, node] - o[:, 0]).max() <= 2e-2
        done += A > 0
    assert done >= 2


def test_whole_step_replays_as_a_hip_graph():
    """The per-step calls only enqueue kernels on the given stream (no allocation, no synchronisation, no memset), so
    a step can be captured once and replayed: every replay, with eager work and synchronisations in between, must
    reproduce the eager results bit for bit."""
    if rest.rest_version().endswith("(bounds-checked build)"):
        pytest.skip("the bounds-checked build waits for its kernels in every call, which a stream capture does not allow")
    w = synth.WORKLOADS["tiny"]
    corp = synth.make_corpus(w.n_tokens, w.corpus_seed, w.n_motifs)
    ctx, lens = synth.make_contexts(corp, 8, w.ctx_len, w.query_seed)
    index = rest.rest_build_index(torch.from_numpy(corp.tokens).cuda(), 4)
    c, m, H, P, V = w.max_nodes, w.cont_len, 4, 96, 4000
    d_ctx, d_len = torch.from_numpy(ctx).cuda(), torch.from_numpy(lens).cuda()
    tree = rest.Tree.empty(8, c)
    q0, _ = bf16_tensor((8, H, c, 128), 70)
    kn, _ = bf16_tensor((8, H, c, 128), 71)
    vn, _ = bf16_tensor((8, H, c, 128), 72)
    kc0, _ = bf16_tensor((8, H, P + c, 128), 73)
    vc0, _ = bf16_tensor((8, H, P + c, 128), 74)
    q, kc, vc = q0.clone(), kc0.clone(), vc0.clone()
    out = torch.empty_like(q)
    g = torch.Generator(device="cuda")
    g.manual_seed(5)
    logits = torch.randn((8 * (1 + c), V), generator=g, device="cuda") * 3
    u = torch.rand(8 * (1 + c), generator=g, device="cuda")
    ids = torch.empty(8 * (1 + c), dtype=torch.int32, device="cuda")
    alen = torch.empty(8, dtype=torch.int32, device="cuda")
    apath = torch.empty((8, m), dtype=torch.int32, device="cuda")
    nxt = torch.empty(8, dtype=torch.int32, device="cuda")
    desc = rest.make_attn_desc(q, kc, vc, out, P, 0.088, True)
    ws = torch.empty(max(rest.rest_tree_attention_workspace_bytes(desc), 16), dtype=torch.uint8, device="cuda")
    ws_sample = torch.empty(rest.rest_sample_ids_workspace_bytes(8 * (1 + c), V), dtype=torch.uint8, device="cuda")

    def step():
        q.copy_(q0)
        kc.copy_(kc0)
        vc.copy_(vc0)
        rest.rest_retrieve(index, d_ctx, d_len, out=tree, n_max=w.n_max, n_min=w.n_min, max_matches=w.max_matches,
                           cont_len=m, max_nodes=c)
        rest.rest_rope_append(q, kn, vn, kc, vc, tree.pos_ids, P)
        rest.rest_tree_attention(q, kc, vc, tree.tree_mask, P, 0.088, out=out, workspace=ws)
        rest.rest_sample_ids(logits, u, 0.8, 0.95, out=ids, workspace=ws_sample)
        rest.rest_accept(ids.view(8, 1 + c), tree, m, alen, apath, nxt)
        rest.rest_kv_compact(kc, vc, apath, alen, c, P)

    step()                       # eager: also raises the kernels' LDS limits, which cannot be done under capture
    torch.cuda.synchronize()
    want = [t.clone() for t in (tree.draft_tokens, tree.tree_mask, out, ids, alen, apath, nxt, kc, vc)]
    s = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(s):
        with torch.cuda.graph(graph, stream=s):
            step()
    torch.cuda.synchronize()
    for replay in range(3):
        for t in (tree.draft_tokens, out, ids, alen, kc):
            t.zero_()                       # eager work between replays; also proves the replay rewrites everything
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = (tree.draft_tokens, tree.tree_mask, out, ids, alen, apath, nxt, kc, vc)
        for a, b in zip(got, want):
            assert torch.equal(a, b), replay
