"""Seeded sweeps over randomly drawn configurations: every call of the library against the oracle on many small,
irregular cases (sizes, caps, options and layouts drawn from a counter-based generator, so the cases never change)."""
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


def draw(seed, k, lo, hi):
    return int(synth.randint(seed, [k], lo, hi)[0])


@pytest.mark.parametrize("case", range(40))
def test_retrieve_random_configuration(case):
    s = 9000 + case
    n = [1, 2, 3, 17, 64, 65, 300, 1000, 4097, 30000][draw(s, 0, 0, 10)]
    vocab = [1, 2, 3, 5, 50, 30000][draw(s, 1, 0, 6)]
    dtype = [np.int32, np.uint16][draw(s, 2, 0, 2)]
    sa_bytes = [4, 8][draw(s, 3, 0, 2)]
    corpus = synth.randint(s, 100 + np.arange(n), 0, vocab).astype(dtype)
    n_max = draw(s, 4, 1, 17)
    n_min = draw(s, 5, 1, n_max + 1)
    K = [1, 2, 5, 63, 64, 65, 1000, 8192][draw(s, 6, 0, 8)]
    m = draw(s, 7, 1, 33)
    c = [1, 2, 7, 63, 64, 65, 128, 256][draw(s, 8, 0, 8)]
    strided = bool(draw(s, 9, 0, 2))
    n_seq = [0, 0, 1, 8, 64][draw(s, 10, 0, 5)]
    depth = [0, 0, n_max + m][draw(s, 11, 0, 3)]
    B, stride = draw(s, 12, 1, 9), 24
    ctx = np.zeros((B, stride), np.int32)
    lens = np.zeros(B, np.int32)
    for b in range(B):
        t = draw(s, 20 + b, 0, stride + 1)
        lens[b] = t
        if b % 2 == 0 and t <= n and t > 0:          # copied from the stream, so that long suffixes match
            e = draw(s, 40 + b, t, n + 1)
            ctx[b, :t] = corpus[e - t:e]
        else:
            ctx[b, :t] = synth.randint(s, 1000 + 100 * b + np.arange(t), 0, vocab + 1)
    d_corpus = dev(corpus)
    index = rest.rest_build_index_prefix(d_corpus, sa_bytes, depth) if depth else rest.rest_build_index(d_corpus, sa_bytes)
    out = rest.Tree.empty(B, c, fill=-0x5A5A5A5B)
    rest.rest_retrieve(index, dev(ctx), dev(lens), out=out, n_max=n_max, n_min=n_min, max_matches=K, cont_len=m, max_nodes=c,
                       random_seqs=n_seq, seed=s, strided=strided)
    torch.cuda.synchronize()
    words = (c + 63) // 64
    for b in range(B):
        want = oracle.draft_tree(corpus, ctx[b, :lens[b]], n_max, n_min, K, m, c, random_seqs=n_seq, seed=s, ctx_index=b,
                                 strided=strided)
        where = f"case {case} context {b}: n={n} vocab={vocab} n_max={n_max} n_min={n_min} K={K} m={m} c={c} " \
                f"strided={strided} n_seq={n_seq} depth={depth}"
        assert (int(out.matched_len[b]), int(out.match_count[b]), int(out.n_nodes[b])) == \
            (want.matched_len, want.match_count, want.n_nodes), where
        for name in ("draft_tokens", "parent_idx", "pos_ids", "node_weight"):
            np.testing.assert_array_equal(getattr(out, name)[b].cpu().numpy(), getattr(want, name), err_msg=where + " " + name)
        np.testing.assert_array_equal(out.tree_mask[b].cpu().numpy().view(np.uint64).reshape(c, words), want.tree_mask,
                                      err_msg=where)


@pytest.mark.parametrize("case", range(40))
def test_attention_random_configuration(case):
    s = 9500 + case
    Nb, H = draw(s, 0, 1, 5), draw(s, 1, 1, 6)
    T = [0, 1, 5, 31, 32, 33, 64, 65, 100, 128, 129, 200, 256][draw(s, 2, 0, 13)]
    P = [0, 1, 15, 16, 31, 32, 33, 63, 64, 100, 257, 1000][draw(s, 3, 0, 12)]
    if T == 0 and P == 0:
        P = 7
    g = [1, 1, 2, 4][draw(s, 4, 0, 4)] if 0 < T <= 128 else 1          # grouped query heads as a view
    extra = [0, 0, 1, 3][draw(s, 5, 0, 4)] if g == 1 else 0               # query rows that see the prefix only
    if T == 0:
        extra = max(extra, 1)
    ns = [0, 0, 1, 2, 5, 64][draw(s, 6, 0, 6)]
    per_batch = bool(draw(s, 7, 0, 2)) and T > 0
    kv8 = bool(draw(s, 8, 0, 2))
    scale = [0.088, 0.5, 0.01][draw(s, 9, 0, 3)]
    token_major = bool(draw(s, 10, 0, 2))                                 # cache stored [Nb, L, H, D]
    L = P + T
    words = max(1, (T + 63) // 64)
    masks = []
    for nb in range(Nb if per_batch else 1):
        m_ = synth.random_tree(T, s + nb)[3][:, :words] if T > 0 else np.zeros((0, 1), np.uint64)
        masks.append(np.vstack([np.zeros((extra, words), np.uint64), m_]))
    mask = np.stack(masks) if per_batch else masks[0]
    rows = T + extra
    Tq = g * rows
    qb = synth.normal_bf16_bits(s, (Nb, H, Tq, 128))
    q = synth.bf16_bits_to_f32(qb)
    dq = dev(qb.view(np.int16)).view(torch.bfloat16)
    kv_shape = (Nb, L, H, 128) if token_major else (Nb, H, L, 128)
    if kv8:
        ks = (0.25 + synth.uniform01(s + 1, np.arange(Nb * H))).reshape(Nb, H).astype(np.float32)
        vs = (0.25 + synth.uniform01(s + 2, np.arange(Nb * H))).reshape(Nb, H).astype(np.float32)
        kraw = oracle.fp8_e4m3_encode(synth.normal_f32(s + 3, kv_shape))
        vraw = oracle.fp8_e4m3_encode(synth.normal_f32(s + 4, kv_shape))
        dk, dv = dev(kraw), dev(vraw)
    else:
        kbits, vbits = synth.normal_bf16_bits(s + 3, kv_shape), synth.normal_bf16_bits(s + 4, kv_shape)
        kraw, vraw = synth.bf16_bits_to_f32(kbits), synth.bf16_bits_to_f32(vbits)
        dk, dv = (dev(x.view(np.int16)).view(torch.bfloat16) for x in (kbits, vbits))
    if token_major:
        dk, dv = dk.permute(0, 2, 1, 3), dv.permute(0, 2, 1, 3)
        kraw, vraw = kraw.transpose(0, 2, 1, 3), vraw.transpose(0, 2, 1, 3)
    dmask = dev(mask.view(np.int64)) if rows > 0 and T > 0 else torch.zeros((max(rows, 1), 1), dtype=torch.int64, device="cuda")
    out = torch.full_like(dq, float("nan"))
    kw = dict(k_scale=dev(ks), v_scale=dev(vs)) if kv8 else {}
    rest.rest_tree_attention(dq, dk, dv, dmask, P, scale, out=out, num_splits=ns, mask_rows=rows if g > 1 else 0, **kw)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy().astype(np.float64)
    # the oracle sees the grouped heads unstacked: head (h, j) = rows j*rows .. of slab h
    qo = q.reshape(Nb, H, g, rows, 128)
    omask = mask[:, None, None] if per_batch else mask
    if kv8:
        k64 = oracle.fp8_e4m3_decode(kraw) * ks[..., None, None].astype(np.float64)
        v64 = oracle.fp8_e4m3_decode(vraw) * vs[..., None, None].astype(np.float64)
    else:
        k64, v64 = kraw.astype(np.float64), vraw.astype(np.float64)
    with np.errstate(invalid="ignore"):
        want = oracle.tree_attention(qo, k64[:, :, None], v64[:, :, None], omask, P, scale).reshape(Nb, H, Tq, 128)
    if P == 0 and extra > 0:            # rows without any visible key: 0/0 by the definition, zeros by the library's contract
        assert np.isnan(want).any()
        want = np.nan_to_num(want, nan=0.0)
    where = f"case {case}: Nb={Nb} H={H} T={T} P={P} g={g} extra={extra} ns={ns} per_batch={per_batch} kv8={kv8} " \
            f"scale={scale} token_major={token_major}"
    assert np.isfinite(got).all(), where
    assert np.abs(got - want).max() <= 2e-2, (where, float(np.abs(got - want).max()))


@pytest.mark.parametrize("case", range(30))
def test_sampling_random_configuration(case):
    """rest_sample_ids against the oracle: equal token ids."""
    s = 9800 + case
    V = [1, 2, 63, 64, 65, 513, 1000, 4097, 32000, 50257][draw(s, 0, 0, 10)]
    R = draw(s, 1, 1, 7)
    temperature = [0.1, 0.7, 0.8, 1.0, 2.5][draw(s, 2, 0, 5)]
    top_p = [0.05, 0.5, 0.8, 0.95, 1.0][draw(s, 3, 0, 5)]
    kind = draw(s, 4, 0, 4)
    x = synth.normal_f32(s, (R, V)) * 2.0
    if kind == 1:                       # many exactly equal logits
        x = np.round(x * 2.0) / 2.0
    elif kind == 2:                     # a few dominant tokens
        for r in range(R):
            x[r, synth.randint(s + r, np.arange(min(V, 4)), 0, V)] += 9.0
    elif kind == 3:                     # part of the vocabulary switched off
        x[:, ::3] = -np.inf
        x[:, 0] = 0.0
    x = x.astype(np.float32)
    u = synth.uniform01(s + 50, np.arange(R)).astype(np.float32)
    stride = V + [0, 0, 3, 64][draw(s, 5, 0, 4)]
    big = torch.full((R, stride), 5.0, dtype=torch.float32, device="cuda")
    big[:, :V] = torch.from_numpy(x).cuda()
    ids = rest.rest_sample_ids(big[:, :V], torch.from_numpy(u).cuda(), temperature, top_p)
    torch.cuda.synchronize()
    got = ids.cpu().numpy()
    want, _ = oracle.sample_ids(x, np.float32(temperature), np.float32(top_p), u)
    np.testing.assert_array_equal(got, want, err_msg=str((case, V, temperature, top_p, kind)))
