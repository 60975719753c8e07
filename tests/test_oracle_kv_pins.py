"""Pins for the oracle's rotary embedding, key/value append and post-acceptance compaction (CPU only).

None of the expected values below comes from the oracle's own formula: they are literal constants, a complex-number
route to the same rotation, algebraic properties a rotation must have, and the equivalence that gives compaction its
meaning (verifying a draft tree and then keeping the accepted path must leave exactly what plain one-token-at-a-time
decoding of those tokens would have produced)."""
import numpy as np
import pytest

import oracle
import synth

COS1, SIN1 = 0.5403023058681398, 0.8414709848078965      # cos(1), sin(1)


def test_rope_plane_rotation_literal():
    # D = 2: one plane, frequency theta^0 = 1, position 1 -> rotation by one radian
    out = oracle.rope(np.array([[2.0, 3.0]]), np.array([1]), theta=10000.0)
    np.testing.assert_allclose(out, [[2 * COS1 - 3 * SIN1, 2 * SIN1 + 3 * COS1]], rtol=0, atol=1e-15)


def test_rope_frequency_exponent_literal():
    # D = 4, theta = 10000: plane 1 = components (1, 3) has frequency 10000^(-2/4) = 0.01, so position 100 is one
    # radian there; plane 0 = components (0, 2) turns by 100 radians
    x = np.array([[1.0, 2.0, 3.0, 4.0]])
    out = oracle.rope(x, np.array([100]), theta=10000.0)
    c100, s100 = 0.8623188722876839, -0.5063656411097588     # cos(100), sin(100)
    want = [1 * c100 - 3 * s100, 2 * COS1 - 4 * SIN1, 1 * s100 + 3 * c100, 2 * SIN1 + 4 * COS1]
    np.testing.assert_allclose(out[0], want, rtol=0, atol=1e-12)


def test_rope_equals_complex_multiplication():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((3, 5, 7, 128))
    pos = rng.integers(0, 5000, size=7)
    z = (x[..., :64] + 1j * x[..., 64:]) * np.exp(1j * pos[:, None] * 500000.0 ** (-np.arange(64) / 64.0))
    out = oracle.rope(x, pos, theta=500000.0)
    np.testing.assert_allclose(out[..., :64], z.real, rtol=0, atol=1e-11)
    np.testing.assert_allclose(out[..., 64:], z.imag, rtol=0, atol=1e-11)


def test_rope_rotation_properties():
    rng = np.random.default_rng(1)
    q, k = rng.standard_normal((6, 128)), rng.standard_normal((6, 128))
    p, r = rng.integers(0, 3000, 6), rng.integers(0, 3000, 6)
    # position 0 is the identity
    np.testing.assert_array_equal(oracle.rope(q, np.zeros(6, dtype=int)), q)
    # every plane keeps its length
    a = oracle.rope(q, p)
    np.testing.assert_allclose(a[:, :64] ** 2 + a[:, 64:] ** 2, q[:, :64] ** 2 + q[:, 64:] ** 2, rtol=1e-12)
    # rotations add
    np.testing.assert_allclose(oracle.rope(oracle.rope(q, p), r), oracle.rope(q, p + r), rtol=0, atol=1e-10)
    # the score of a query and a key depends on their distance only
    for shift in (1, 17, 1234):
        s0 = np.sum(oracle.rope(q, p) * oracle.rope(k, r), axis=-1)
        s1 = np.sum(oracle.rope(q, p + shift) * oracle.rope(k, r + shift), axis=-1)
        np.testing.assert_allclose(s1, s0, rtol=0, atol=1e-9)


def test_rope_per_slab_positions_broadcast():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((4, 3, 5, 16))
    pos = rng.integers(0, 50, size=(4, 1, 5))
    out = oracle.rope(x, np.broadcast_to(pos, (4, 3, 5)))
    for a in range(4):
        np.testing.assert_array_equal(out[a], oracle.rope(x[a], pos[a, 0]))


def test_append_places_rows_and_leaves_the_rest():
    rng = np.random.default_rng(3)
    P, T, D = 5, 3, 8
    kc, vc = rng.standard_normal((2, P + T + 2, D)), rng.standard_normal((2, P + T + 2, D))
    q, kn, vn = (rng.standard_normal((2, T, D)) for _ in range(3))
    pos_ids = np.array([1, 1, 2])
    qr, k2, v2 = oracle.rope_append(q, kn, vn, kc, vc, pos_ids, P - 1, P, theta=100.0)
    np.testing.assert_array_equal(k2[:, :P], kc[:, :P])
    np.testing.assert_array_equal(k2[:, P + T:], kc[:, P + T:])
    np.testing.assert_array_equal(v2[:, P:P + T], vn)
    np.testing.assert_array_equal(v2[:, :P], vc[:, :P])
    # depth-1 nodes sit one position behind the last context token (position P-1), i.e. at position P
    z = (kn[:, 0, :4] + 1j * kn[:, 0, 4:]) * np.exp(1j * P * 100.0 ** (-np.arange(4) / 4.0))
    np.testing.assert_allclose(k2[:, P, :4], z.real, atol=1e-12)
    np.testing.assert_allclose(k2[:, P, 4:], z.imag, atol=1e-12)
    np.testing.assert_allclose(qr[:, 2], oracle.rope(q[:, 2:3], np.array([P + 1]), 100.0)[:, 0], atol=0)


def test_compact_hand_case_and_identity():
    P = 2
    cache = np.arange(7, dtype=np.float64)[:, None] * np.ones((1, 3))        # row r holds the value r
    out = oracle.kv_compact(cache, P, np.array([1, 3, -1, -1]), 2)
    np.testing.assert_array_equal(out[:, 0], [0, 1, 3, 5, 4, 5, 6])          # tree rows 1 and 3 move up, rest untouched
    # a chain accepted in full is already in place
    np.testing.assert_array_equal(oracle.kv_compact(cache, P, np.arange(5), 5), cache)
    # nothing accepted: nothing moves
    np.testing.assert_array_equal(oracle.kv_compact(cache, P, np.full(4, -1), 0), cache)
    # a source row may be another move's destination (path [1, 2]: row P+1 is read by move 0 and written by move 1)
    out = oracle.kv_compact(cache, P, np.array([1, 2]), 2)
    np.testing.assert_array_equal(out[:, 0], [0, 1, 3, 4, 4, 5, 6])
    # the definition reads the cache as it was: a path that is not increasing (no tree produces one) still moves the
    # old rows -- new P+0 = old P+2, new P+1 = old P+0, new P+2 = old P+1 --, not rows an earlier move has written
    out = oracle.kv_compact(cache, P, np.array([2, 0, 1]), 3)
    np.testing.assert_array_equal(out[:, 0], [0, 1, 4, 2, 3, 5, 6])


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_verify_then_compact_equals_plain_decoding(seed):
    """Tree verification followed by compaction must leave what token-by-token decoding of the accepted tokens
    leaves: the same cache rows, and for every accepted node the attention output plain causal attention gives."""
    rng = np.random.default_rng(seed)
    P, T, D, H = 9, 24, 16, 2
    par, dep, tok, mask = synth.random_tree(T, 40 + seed)
    leaf = int(np.argmax(dep))                      # accept the path to a deepest node
    path = []
    v = leaf
    while v != -1:
        path.append(v)
        v = int(par[v])
    path = path[::-1]
    A = len(path)
    assert A == dep[leaf] and A >= 2
    kc = rng.standard_normal((H, P + T, D))
    vc = rng.standard_normal((H, P + T, D))
    q, kn, vn = (rng.standard_normal((H, T, D)) for _ in range(3))
    scale = 0.25
    # REST's way: embed + append all T nodes, verify with the tree mask, keep the accepted rows
    qr, k2, v2 = oracle.rope_append(q, kn, vn, kc, vc, dep, P - 1, P, theta=10000.0)
    out_tree = oracle.tree_attention(qr, k2, v2, mask, P, scale)
    k3 = oracle.kv_compact(k2, P, np.array(path), A)
    v3 = oracle.kv_compact(v2, P, np.array(path), A)
    # plain decoding of the same tokens: position P, P+1, ... one at a time, causal attention
    k_plain, v_plain = kc.copy(), vc.copy()
    for i, node in enumerate(path):
        pos = np.array([P + i])
        k_plain[:, P + i] = oracle.rope(kn[:, node:node + 1], pos)[:, 0]
        v_plain[:, P + i] = vn[:, node]
        qi = oracle.rope(q[:, node:node + 1], pos)
        s = scale * np.einsum("hqd,hkd->hqk", qi, k_plain[:, :P + i + 1])
        p = np.exp(s - s.max(-1, keepdims=True))
        p /= p.sum(-1, keepdims=True)
        o = np.einsum("hqk,hkd->hqd", p, v_plain[:, :P + i + 1])
        np.testing.assert_allclose(out_tree[:, node], o[:, 0], rtol=0, atol=1e-12)
    np.testing.assert_allclose(k3[:, :P + A], k_plain[:, :P + A], rtol=0, atol=1e-13)
    np.testing.assert_array_equal(v3[:, :P + A], v_plain[:, :P + A])
