"""GPU parity of rest_sample_ids against the CPU oracle.

Both sides compute in float64 from the same fp32 logits; their exponentials and the order of their sums differ at
rounding level, so a drawn token may legitimately differ only where a decision threshold (top_p, or u times the nucleus
mass) falls within rounding of a cumulative sum.  The oracle lists, per row, every token such a perturbation (1e-9 in
probability mass) could produce -- one token for nearly every row -- and the GPU's id must be in that list."""
import numpy as np
import pytest
import torch

import oracle
import synth

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2311_08252_amd as rest


def check(logits, u, temperature, top_p, stride=None):
    R, V = logits.shape
    if stride is None:
        d_logits = torch.from_numpy(logits).cuda()
    else:
        big = torch.full((R, stride), 7.0, dtype=torch.float32, device="cuda")
        big[:, :V] = torch.from_numpy(logits).cuda()
        d_logits = big[:, :V]
    ids = rest.rest_sample_ids(d_logits, torch.from_numpy(u.astype(np.float32)).cuda(), temperature, top_p)
    torch.cuda.synchronize()
    got = ids.cpu().numpy()
    want, _ = oracle.sample_ids(logits, np.float32(temperature), np.float32(top_p), u.astype(np.float32))
    single = 0
    for r in range(R):
        cands = oracle.nucleus_candidates(logits[r], np.float32(temperature), np.float32(top_p), np.float32(u[r]))
        assert int(want[r]) in cands
        assert int(got[r]) in cands, (r, int(got[r]), int(want[r]), cands)
        single += len(cands) == 1
    assert single >= 0.9 * R - 1
    return got


@pytest.mark.parametrize("V,R,temperature,top_p,seed", [
    (32000, 65, 0.8, 0.95, 0),        # the paper's code-generation setting, one row per position of a 64-node tree
    (32000, 65, 0.7, 0.8, 1),         # the paper's chat setting
    (32016, 9, 1.0, 1.0, 2),          # whole distribution
    (32768, 4, 0.8, 0.95, 3),         # largest vocabulary the call takes
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


def test_minus_infinity_logits_and_strided_rows():
    rng = np.random.default_rng(11)
    logits = rng.standard_normal((20, 3000)).astype(np.float32)
    logits[:, rng.integers(0, 3000, 2500)] = -np.inf          # masked-out tokens
    got = check(logits, rng.random(20), 0.9, 0.9, stride=3100)
    assert np.isfinite(logits[np.arange(20), got]).all()


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
        assert all(len(oracle.nucleus_candidates(logits[b, r], np.float32(0.8), np.float32(0.95), u[b, r])) == 1
                   for r in range(1 + c))
        np.testing.assert_array_equal(ids.view(8, 1 + c)[b].cpu().numpy(), want_ids)
        a, path, nx = oracle.accept(want_ids, tok[b], par[b], int(nn[b]), m)
        assert (int(alen[b]), int(nxt[b])) == (a, nx)
        np.testing.assert_array_equal(apath[b].cpu().numpy(), path)
        accepted += a
    assert accepted >= 4
