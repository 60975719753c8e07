"""GPU parity of rest_sample_ids against the CPU oracle: the drawn token ids must be equal.

The definition of the draw carries probability masses as integers and fixes every rounding of the exponential, so
there is one right token per row whatever order an implementation adds in (oracle: sort and cumulative sum; kernels:
histograms of masses filled with atomic adds -- by one workgroup that holds the row in registers up to 32768 tokens,
by several workgroups per row beyond)."""
import numpy as np
import pytest
import torch

import oracle
import synth

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2311_08252_amd as rest


def check(logits, u, temperature, top_p, stride=None, first=0):
    """first: the rows start that many floats into their allocation (rows that are not 16-byte aligned)."""
    R, V = logits.shape
    if stride is None and first == 0:
        d_logits = torch.from_numpy(logits).cuda()
    else:
        big = torch.full((R, first + (stride or V)), 7.0, dtype=torch.float32, device="cuda")
        big[:, first:first + V] = torch.from_numpy(logits).cuda()
        d_logits = big[:, first:first + V]
    out = torch.full((R,), -77, dtype=torch.int32, device="cuda")
    # the workspace needs no initialisation: hand over one full of ones
    ws = torch.full((rest.rest_sample_ids_workspace_bytes(R, V),), 0xFF, dtype=torch.uint8, device="cuda")
    ids = rest.rest_sample_ids(d_logits, torch.from_numpy(u.astype(np.float32)).cuda(), temperature, top_p, out=out, workspace=ws)
    torch.cuda.synchronize()
    got = ids.cpu().numpy()
    want, _ = oracle.sample_ids(logits, np.float32(temperature), np.float32(top_p), u.astype(np.float32))
    np.testing.assert_array_equal(got, want)
    return got


@pytest.mark.parametrize("V,R,temperature,top_p,seed", [
    (32000, 65, 0.8, 0.95, 0),        # the paper's code-generation setting, one row per position of a 64-node tree
    (32000, 65, 0.7, 0.8, 1),         # the paper's chat setting
    (32016, 9, 1.0, 1.0, 2),          # whole distribution
    (32768, 4, 0.8, 0.95, 3),         # the longest row one workgroup keeps in registers
    (32769, 4, 0.8, 0.95, 13),        # the shortest that is cut into slices
    (4097, 6, 0.8, 0.95, 14),         # one token into the second group of four registers
    (131072, 3, 0.8, 0.95, 9),        # largest vocabulary the call takes: sixteen workgroups per row
    (128256, 5, 0.7, 0.9, 10),        # a current vocabulary, last slice ragged
    (8192, 7, 1.0, 0.9, 11),          # exactly one slice
    (8193, 7, 1.0, 0.9, 12),          # one token into the second slice
    (1000, 130, 0.8, 0.95, 4),        # ragged: most threads hold padding
    (5, 40, 1.0, 0.8, 5),
    (1, 3, 1.0, 0.5, 6),
    (32000, 33, 0.05, 0.95, 7),       # nearly greedy
    (32000, 33, 5.0, 0.999, 8),       # nearly flat: the nucleus holds almost every token
])
def test_matches_oracle(V, R, temperature, top_p, seed):
    rng = np.random.default_rng(seed)
    # logits like a language model's: a heavy head over a broad body
    logits = (rng.standard_normal((R, V)) * 2.0).astype(np.float32)
    head = rng.integers(0, V, size=(R, min(V, 6)))
    for r in range(R):
        logits[r, head[r]] += rng.uniform(4, 12, size=head.shape[1]).astype(np.float32)
    u = rng.random(R)
    u[0] = 0.0
    u[-1] = np.float32(1.0) - np.float32(2.0 ** -24)       # the largest float32 below 1
    check(logits, u, temperature, top_p)


def test_ties_go_by_ascending_token_id():
    V = 4096
    logits = np.full((64, V), -3.0, dtype=np.float32)       # every row: all tokens equally likely
    logits[32:, 100:200] = 1.5                               # or a plateau of 100 equal leaders
    u = (128.0 * (np.arange(64) % 32) + 64.4) / 4096.0       # off the boundaries k / 4096 of a flat row
    got = check(logits, u, 1.0, 1.0)
    # flat rows: the draw is token floor(u * V)
    np.testing.assert_array_equal(got[:32], np.floor(u[:32] * V).astype(np.int32))
    # -0.0 and +0.0 are one logit
    z = np.zeros((2, 8), dtype=np.float32)
    z[0, ::2] = -0.0
    np.testing.assert_array_equal(check(z, np.array([0.3, 0.3]), 1.0, 1.0), [2, 2])


def test_plateaus_larger_than_the_kernels_token_list():
    """Thousands of exactly equal logits land in one cell of the kernel's first search level; beyond 1024 of them the
    kernel searches the row itself instead of a list in LDS.  Flat rows, a plateau of 6000 leaders, a plateau in the
    body (the nucleus boundary or the draw falls into it), logits with few distinct values."""
    V = 20000
    rng = np.random.default_rng(21)
    rows = [np.full(V, 0.25, dtype=np.float32) for _ in range(6)]
    rows[2][3000:9000] = 4.0
    rows[3][3000:9000] = 4.0
    rows[4] = (rng.standard_normal(V) * 2).astype(np.float32)
    rows[4][rng.permutation(V)[:7000]] = 1.0
    rows[5] = np.round(rng.standard_normal(V) * 2).astype(np.float32)          # about twenty distinct values
    logits = np.stack(rows)
    u = np.array([0.0, 0.73519, 0.41, 0.999, 0.6, 0.35])
    got = check(logits, u, 1.0, 1.0)
    assert got[0] == 0 and got[1] == int(np.floor(np.float32(0.73519) * V))    # flat rows: token floor(u V)
    for top_p, temperature in ((0.9, 0.8), (0.5, 1.3), (0.999, 0.3)):
        check(logits, rng.random(6), temperature, top_p)
    # the same in rows of 40000 tokens, which several workgroups share
    wide = np.concatenate([logits, np.full((6, 20000), -9.0, dtype=np.float32)], axis=1)
    wide[1, 20000:] = 0.25
    for top_p, temperature in ((1.0, 1.0), (0.9, 0.8)):
        check(wide, u, temperature, top_p)


@pytest.mark.parametrize("size", [3, 16, 17, 32, 33, 64, 65, 128, 129, 256, 300, 512, 513, 1000, 1024, 1025, 1500])
def test_plateau_sizes_around_the_list_phases_group_widths(size):
    """The tokens of the crossing cell are ordered by groups of 64, 32, ... 1 threads per listed token, as many as the
    workgroup has for that many tokens, and by the search in memory beyond 1024: a plateau of `size` equal logits holds
    the nucleus boundary and most draws, a few leaders and a random body around it."""
    V, R = 9000, 12
    rng = np.random.default_rng(size)
    logits = (rng.standard_normal((R, V)) * 0.5 - 6.0).astype(np.float32)
    for r in range(R):
        where = rng.permutation(V)
        logits[r, where[:size]] = np.float32(1.0 + 0.125 * r)          # the plateau, scattered over the row
        logits[r, where[size:size + 2]] = np.float32(3.0)              # two leaders above it
    u = rng.random(R)
    u[0] = 0.0
    check(logits, u, 1.0, 0.9)
    check(logits, rng.random(R), 0.6, 0.97)


def test_minus_infinity_logits_and_strided_rows():
    rng = np.random.default_rng(11)
    logits = rng.standard_normal((20, 3000)).astype(np.float32)
    logits[:, rng.integers(0, 3000, 2500)] = -np.inf          # masked-out tokens
    got = check(logits, rng.random(20), 0.9, 0.9, stride=3100)
    assert np.isfinite(logits[np.arange(20), got]).all()


@pytest.mark.parametrize("V,stride,first", [(3000, 3001, 0), (3000, 3004, 1), (32000, 32002, 3), (40000, 40001, 2)])
def test_rows_that_are_not_16_byte_aligned(V, stride, first):
    """Aligned rows are read as groups of four floats; these cannot be."""
    rng = np.random.default_rng(V + stride)
    logits = (rng.standard_normal((9, V)) * 2.0).astype(np.float32)
    logits[:, :5] += 8.0
    check(logits, rng.random(9), 0.8, 0.95, stride=stride, first=first)


def test_sampled_acceptance_on_the_gpu():
    """sample ids for the root and every node, then the usual walk: equals the oracle's sample + walk."""
    w = synth.WORKLOADS["tiny"]
    corp = synth.make_corpus(w.n_tokens, w.corpus_seed, w.n_motifs)
    ctx, lens = synth.make_contexts(corp, 8, w.ctx_len, w.query_seed)
    index = rest.rest_build_index(torch.from_numpy(corp.tokens).cuda(), 4)
    c, m, V = w.max_nodes, w.cont_len, 32000
    tree = rest.rest_retrieve(index, torch.from_numpy(ctx).cuda(), torch.from_numpy(lens).cuda(), n_max=w.n_max,
                              n_min=w.n_min, max_matches=w.max_matches, cont_len=m, max_nodes=c)
    torch.cuda.synchronize()
    rng = np.random.default_rng(3)
    tok, par, nn = tree.draft_tokens.cpu().numpy(), tree.parent_idx.cpu().numpy(), tree.n_nodes.cpu().numpy()
    logits = rng.standard_normal((8, 1 + c, V)).astype(np.float32)
    for b in range(8):            # make the model agree with some child at most positions
        for pos in range(1 + int(nn[b])):
            kids = [i for i in range(int(nn[b])) if par[b, i] == pos - 1]
            if kids and rng.random() < 0.8:
                logits[b, pos, tok[b, kids[rng.integers(len(kids))]]] += 14.0
    u = rng.random((8, 1 + c)).astype(np.float32)
    ids = rest.rest_sample_ids(torch.from_numpy(logits.reshape(-1, V)).cuda(), torch.from_numpy(u.reshape(-1)).cuda(), 0.8, 0.95)
    alen, apath, nxt = rest.rest_accept(ids.view(8, 1 + c), tree, m)
    torch.cuda.synchronize()
    accepted = 0
    for b in range(8):
        want_ids, _ = oracle.sample_ids(logits[b], np.float32(0.8), np.float32(0.95), u[b])
        np.testing.assert_array_equal(ids.view(8, 1 + c)[b].cpu().numpy(), want_ids)
        a, path, nx = oracle.accept(want_ids, tok[b], par[b], int(nn[b]), m)
        assert (int(alen[b]), int(nxt[b])) == (a, nx)
        np.testing.assert_array_equal(apath[b].cpu().numpy(), path)
        accepted += a
    assert accepted >= 4
