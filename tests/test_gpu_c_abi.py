"""The library driven from plain C: tests/c_abi_driver.c is compiled with gcc (build() does it), linked against
the shared library and the HIP runtime, and run as a process of its own with no Python in it.  One step --
index build, retrieval, attention with the mask retrieval left on the device, acceptance -- against the oracle."""
import os
import subprocess

import numpy as np
import pytest

import oracle
import synth

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
EXE = os.path.join(ROOT, "tests", "_build", "c_abi_driver")


def driver():
    if not os.path.exists(EXE):           # a one-second gcc run; the library itself is never built here
        import __graft_entry__
        __graft_entry__.build_c_driver()
    return EXE


@pytest.mark.parametrize("depth", [0, 32])
def test_one_step_from_a_c_program(tmp_path, depth):
    n, B, stride, K, m, c, cap, H, P = 300_000, 6, 48, 1000, 10, 64, 10, 3, 150
    corp = synth.make_corpus(n, seed=21, n_motifs=60, copies=50)
    ctx, lens = synth.make_contexts(corp, B, stride, 5)
    lens[B - 1] = 1                                                   # too short to match: an empty tree
    want = [oracle.draft_tree(corp.tokens, ctx[b][:lens[b]], 16, 2, K, m, c) for b in range(B)]
    ids = np.stack([synth.sampled_ids(40 + b, w.draft_tokens, w.parent_idx, w.n_nodes) for b, w in enumerate(want)])
    q = synth.bf16_bits_to_f32(synth.normal_bf16_bits(61, (B, H, c, 128)))
    k = synth.bf16_bits_to_f32(synth.normal_bf16_bits(62, (B, H, P + c, 128)))
    v = synth.bf16_bits_to_f32(synth.normal_bf16_bits(63, (B, H, P + c, 128)))
    src, dst = tmp_path / "in.bin", tmp_path / "out.bin"
    with open(src, "wb") as f:
        f.write(np.array([n, B, stride, K, m, c, cap, H, P, depth], np.int64).tobytes())
        for a in (corp.tokens.astype(np.int32), ctx.astype(np.int32), lens.astype(np.int32), ids.astype(np.int32),
                  q.astype(np.float32), k.astype(np.float32), v.astype(np.float32)):
            f.write(np.ascontiguousarray(a).tobytes())
    run = subprocess.run([driver(), str(src), str(dst)], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0, run.stderr[-2000:]

    words = (c + 63) // 64
    raw = open(dst, "rb").read()
    at = 0

    def take(dtype, *shape):
        nonlocal at
        count = int(np.prod(shape))
        a = np.frombuffer(raw, dtype, count, at).reshape(shape)
        at += count * np.dtype(dtype).itemsize
        return a

    tok, par, pos, wgt = (take(np.int32, B, c) for _ in range(4))
    msk = take(np.uint64, B, c, words)
    nn, ml, mc = take(np.int32, B), take(np.int32, B), take(np.int64, B)
    alen, apath, nxt = take(np.int32, B), take(np.int32, B, cap), take(np.int32, B)
    out = take(np.float32, B, H, c, 128)
    assert at == len(raw)

    for b, w in enumerate(want):
        assert (int(nn[b]), int(ml[b]), int(mc[b])) == (w.n_nodes, w.matched_len, w.match_count), b
        np.testing.assert_array_equal(tok[b], w.draft_tokens)
        np.testing.assert_array_equal(par[b], w.parent_idx)
        np.testing.assert_array_equal(pos[b], w.pos_ids)
        np.testing.assert_array_equal(wgt[b], w.node_weight)
        np.testing.assert_array_equal(msk[b], w.tree_mask)
        n_acc, path, nt = oracle.accept(ids[b], w.draft_tokens, w.parent_idx, w.n_nodes, cap)
        assert (int(alen[b]), int(nxt[b])) == (n_acc, nt)
        np.testing.assert_array_equal(apath[b], path)
    assert nn[B - 1] == 0 and max(nn) > 8 and max(alen) >= 1
    masks = np.stack([w.tree_mask for w in want])[:, None]
    ref = oracle.tree_attention(q, k, v, masks, P, 1.0 / np.sqrt(128.0))
    for b in range(B):
        for h in range(H):
            assert np.abs(out[b, h] - ref[b, h]).max() <= 1e-3 * np.abs(ref[b, h]).max(), (b, h)
