"""Pins for the oracle's tree attention (no GPU): a library attention routine
for the chain-shaped tree, closed forms, and special cases with known answers."""
import numpy as np
import pytest
import torch

import oracle
import synth


def chain_mask(T):
    par = np.arange(-1, T - 1, dtype=np.int32)
    return oracle.mask_from_parents(par, T)


def star_mask(T):
    return oracle.mask_from_parents(np.full(T, -1, dtype=np.int32), T)


def qkv(H, T, P, D, seed):
    q = synth.normal_f32(seed, (H, T, D)).astype(np.float64)
    k = synth.normal_f32(seed + 1, (H, P + T, D)).astype(np.float64)
    v = synth.normal_f32(seed + 2, (H, P + T, D)).astype(np.float64)
    return q, k, v


@pytest.mark.parametrize("T,P,D", [(1, 5, 8), (7, 0, 16), (64, 40, 32), (70, 129, 128)])
def test_chain_tree_is_causal_attention_library(T, P, D):
    """A chain-shaped tree is ordinary causal decoding of T tokens after a
    P-token prefix: compare with torch's scaled_dot_product_attention in
    float64 given the explicit causal mask."""
    q, k, v = qkv(3, T, P, D, 5)
    scale = 1.0 / np.sqrt(D)
    got = oracle.tree_attention(q, k, v, chain_mask(T), P, scale)
    allow = torch.ones(T, P + T, dtype=torch.bool).tril(diagonal=P)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q), torch.from_numpy(k), torch.from_numpy(v), attn_mask=allow, scale=scale)
    np.testing.assert_allclose(got, ref.numpy(), rtol=1e-11, atol=1e-12)


@pytest.mark.parametrize("seed,T,P", [(1, 5, 3), (2, 9, 0), (3, 66, 2)])
def test_matches_explicit_loops_on_random_trees(seed, T, P):
    par, dep, tok, mask = synth.random_tree(T, seed, max_children=3, max_depth=6)
    q, k, v = qkv(1, T, P, 4, seed + 20)
    got = oracle.tree_attention(q[0], k[0], v[0], mask, P, 0.37)
    ref = oracle.tree_attention_loops(q[0], k[0], v[0], mask, P, 0.37)
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-13)


def test_star_tree_sees_prefix_and_self_only():
    T, P, D = 6, 4, 8
    q, k, v = qkv(2, T, P, D, 9)
    got = oracle.tree_attention(q, k, v, star_mask(T), P, 0.5)
    for h in range(2):
        for i in range(T):
            keys = np.concatenate([k[h, :P], k[h, P + i:P + i + 1]])
            vals = np.concatenate([v[h, :P], v[h, P + i:P + i + 1]])
            w = np.exp(0.5 * keys @ q[h, i])
            np.testing.assert_allclose(got[h, i], (w / w.sum()) @ vals, rtol=1e-12)


def test_closed_forms():
    T, P, D = 10, 6, 16
    q, k, v = qkv(2, T, P, D, 13)
    par, dep, tok, mask = synth.random_tree(T, 4)
    # constant V -> the output is that constant (softmax rows sum to 1)
    vc = np.broadcast_to(np.linspace(-1, 1, D), v.shape).copy()
    out = oracle.tree_attention(q, k, vc, mask, P, 0.3)
    np.testing.assert_allclose(out, np.broadcast_to(np.linspace(-1, 1, D), out.shape), atol=1e-14)
    # one visible key -> the output is its value row
    out = oracle.tree_attention(q, k[:, P:], v[:, P:], star_mask(T), 0, 0.3)
    np.testing.assert_allclose(out, v[:, P:], atol=1e-14)
    # zero queries -> uniform average over the visible keys
    out = oracle.tree_attention(np.zeros_like(q), k, v, mask, P, 0.3)
    for i in range(T):
        anc = [j for j in range(T) if (int(mask[i, 0]) >> j) & 1]
        want = (v[:, :P].sum(1) + v[:, [P + j for j in anc]].sum(1)) / (P + len(anc))
        np.testing.assert_allclose(out[:, i], want, rtol=1e-12)
    # a hidden key cannot influence the output, a visible one does
    k2, v2 = k.copy(), v.copy()
    hidden = [j for j in range(T) if not (int(mask[T - 1, 0]) >> j) & 1]
    assert hidden
    k2[:, P + hidden[0]] += 100.0
    v2[:, P + hidden[0]] -= 50.0
    out2 = oracle.tree_attention(q, k2, v2, mask, P, 0.3)
    base = oracle.tree_attention(q, k, v, mask, P, 0.3)
    np.testing.assert_array_equal(out2[:, T - 1], base[:, T - 1])
    v3 = v.copy()
    v3[:, 0] += 1.0
    assert np.abs(oracle.tree_attention(q, k, v3, mask, P, 0.3) - base).max() > 1e-3
    # scale matters and is applied to the logits: doubling q equals doubling scale
    np.testing.assert_allclose(oracle.tree_attention(2 * q, k, v, mask, P, 0.3),
                               oracle.tree_attention(q, k, v, mask, P, 0.6), rtol=1e-12)


def test_per_batch_masks_and_tq_not_equal_tk():
    Tk, P, D = 5, 3, 4
    q, k, v = qkv(2, Tk + 1, P, D, 17)
    k, v = k[:, :P + Tk], v[:, :P + Tk]
    m0 = np.vstack([np.zeros((1, 1), np.uint64), chain_mask(Tk)])      # extra root row sees the prefix only
    m1 = np.vstack([np.zeros((1, 1), np.uint64), star_mask(Tk)])
    both = oracle.tree_attention(q, k, v, np.stack([m0, m1]), P, 0.4)
    np.testing.assert_allclose(both[0], oracle.tree_attention(q[0], k[0], v[0], m0, P, 0.4))
    np.testing.assert_allclose(both[1], oracle.tree_attention(q[1], k[1], v[1], m1, P, 0.4))
    root = oracle.tree_attention(q[0, :1], k[0, :P], v[0, :P], np.zeros((1, 1), np.uint64), P, 0.4)
    np.testing.assert_allclose(both[0, 0], root[0])
