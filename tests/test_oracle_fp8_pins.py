"""Pins of the oracle's 8-bit (OCP E4M3) KV-cache functions against the published format, torch's CPU conversion of
the same format, brute force, and the algebra that ties attention on a scaled 8-bit cache to plain attention."""
import numpy as np
import torch

import oracle
import synth


def test_decode_matches_the_format_and_torch():
    d = oracle.fp8_e4m3_decode(np.arange(256))
    # values the format's specification names: one, the largest finite, the smallest normal and subnormal, zeros, NaN
    assert d[0x38] == 1.0 and d[0x7E] == 448.0 and d[0x08] == 2.0 ** -6 and d[0x01] == 2.0 ** -9 and d[0x07] == 7 * 2.0 ** -9
    assert d[0x00] == 0.0 and d[0x80] == 0.0 and np.signbit(d[0x80]) and np.isnan(d[0x7F]) and np.isnan(d[0xFF])
    assert d[0x40] == 2.0 and d[0x3C] == 1.5 and d[0xB8] == -1.0 and d[0x78] == 256.0
    assert (np.diff(d[:0x7F]) > 0).all() and np.array_equal(d[0x80:0xFF], -d[:0x7F])
    # an independent implementation of the same format
    t = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    np.testing.assert_array_equal(np.nan_to_num(d, nan=12345.0), np.nan_to_num(t, nan=12345.0))


def test_encode_is_nearest_even_and_saturates():
    d = oracle.fp8_e4m3_decode(np.arange(256))
    finite = [c for c in range(256) if not np.isnan(d[c])]
    # every representable value encodes to itself (the two zeros keep their signs)
    np.testing.assert_array_equal(oracle.fp8_e4m3_encode(d[finite]), np.array(finite, dtype=np.uint8))
    # ties: halfway between 1 and 1.125 goes down to the even mantissa, between 1.125 and 1.25 up; likewise subnormals
    assert oracle.fp8_e4m3_encode(np.array([1.0625, 1.1875, -1.0625, 2.0 ** -10, 3 * 2.0 ** -10])).tolist() == \
        [0x38, 0x3A, 0xB8, 0x00, 0x02]
    assert oracle.fp8_e4m3_encode(np.array([448.0, 449.0, 1e9, -1e9, np.inf, np.nan])).tolist() == \
        [0x7E, 0x7E, 0x7E, 0xFE, 0x7E, 0x7F]
    # brute force: no other finite code is closer
    x = synth.normal_f32(3, (4000,)).astype(np.float64) * np.exp(synth.normal_f32(4, (4000,)).astype(np.float64) * 3)
    got = oracle.fp8_e4m3_encode(x)
    grid = d[finite]
    best = np.abs(grid[None, :] - x[:, None]).min(axis=1)
    np.testing.assert_array_equal(np.abs(d[got] - x), best)
    # torch's conversion of in-range values rounds the same way
    inr = np.abs(x) <= 448
    t = torch.from_numpy(x[inr]).to(torch.float32).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    x32 = x[inr].astype(np.float32).astype(np.float64)        # torch rounds from float32
    np.testing.assert_array_equal(oracle.fp8_e4m3_encode(x32), t)


def test_attention_on_an_8bit_cache_is_plain_attention_on_the_decoded_values():
    Nb, H, T, P, D = 2, 3, 9, 21, 16
    par, dep, tok, mask = synth.random_tree(T, 5)
    q = synth.normal_f32(11, (Nb, H, T, D)).astype(np.float64)
    k = synth.normal_f32(12, (Nb, H, P + T, D)).astype(np.float64)
    v = synth.normal_f32(13, (Nb, H, P + T, D)).astype(np.float64)
    k8, v8 = oracle.fp8_e4m3_encode(k), oracle.fp8_e4m3_encode(v)
    one = np.ones((Nb, H))
    got = oracle.tree_attention_fp8kv(q, k8, v8, one, one, mask, P, 0.3)
    want = oracle.tree_attention(q, oracle.fp8_e4m3_decode(k8), oracle.fp8_e4m3_decode(v8), mask, P, 0.3)
    np.testing.assert_array_equal(got, want)
    # close to attention on the unquantised values (3 mantissa bits: relative step 1/16 per element)
    full = oracle.tree_attention(q, k, v, mask, P, 0.3)
    assert 1e-4 < np.abs(got - full).max() < 0.15
    # the scales factor out: k_scale multiplies the logits, v_scale the output, per (batch, head)
    ks = 0.5 + synth.uniform01(14, np.arange(Nb * H)).reshape(Nb, H)
    vs = 0.5 + synth.uniform01(15, np.arange(Nb * H)).reshape(Nb, H)
    got = oracle.tree_attention_fp8kv(q, k8, v8, ks, vs, mask, P, 0.3)
    for nb in range(Nb):
        for h in range(H):
            ref = oracle.tree_attention_loops(q[nb, h], oracle.fp8_e4m3_decode(k8[nb, h]), oracle.fp8_e4m3_decode(v8[nb, h]),
                                              mask, P, 0.3 * ks[nb, h]) * vs[nb, h]
            np.testing.assert_allclose(got[nb, h], ref, rtol=1e-12, atol=1e-14)


def test_append_to_an_8bit_cache():
    Nb, H, T, P, L, D = 2, 3, 6, 5, 14, 16
    q = synth.normal_f32(21, (Nb, H, T, D)).astype(np.float64)
    kn = synth.normal_f32(22, (Nb, H, T, D)).astype(np.float64)
    vn = synth.normal_f32(23, (Nb, H, T, D)).astype(np.float64)
    kc = synth.randint(24, np.arange(Nb * H * L * D), 0, 0x7F).astype(np.uint8).reshape(Nb, H, L, D)
    vc = synth.randint(25, np.arange(Nb * H * L * D), 0, 0x7F).astype(np.uint8).reshape(Nb, H, L, D)
    ks = 0.25 + synth.uniform01(26, np.arange(Nb * H)).reshape(Nb, H)
    vs = 0.25 + synth.uniform01(27, np.arange(Nb * H)).reshape(Nb, H)
    pos = np.array([1, 1, 2, 2, 3, 4])
    qr, k8, v8, kx, vx = oracle.rope_append_fp8kv(q, kn, vn, kc, vc, ks, vs, pos, P - 1, P, 10000.0)
    # the 16-bit definition gives the values that are quantised; q is embedded as there
    q_ref, k_ref, v_ref = oracle.rope_append(q, kn, vn, np.zeros((Nb, H, L, D)), np.zeros((Nb, H, L, D)), pos, P - 1, P, 10000.0)
    np.testing.assert_array_equal(qr, q_ref)
    np.testing.assert_allclose(kx * ks[..., None, None], k_ref[:, :, P:P + T], rtol=1e-15, atol=0)
    np.testing.assert_allclose(vx * vs[..., None, None], v_ref[:, :, P:P + T], rtol=1e-15, atol=0)
    # stored codes are within half a grid step of the quotient (grid step = 2^(exponent - 3), 2^-9 below 2^-6)
    for x, c8 in ((kx, k8), (vx, v8)):
        new = oracle.fp8_e4m3_decode(c8[:, :, P:P + T])
        step = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(x), 2.0 ** -6))) - 3)
        assert (np.abs(new - x) <= step / 2).all() and (np.sign(new) * np.sign(x) >= 0).all()
    # rows outside P .. P+T-1 keep their codes
    for old, c8 in ((kc, k8), (vc, v8)):
        np.testing.assert_array_equal(c8[:, :, :P], old[:, :, :P])
        np.testing.assert_array_equal(c8[:, :, P + T:], old[:, :, P + T:])
    # representable values at position 0 (no rotation) and unit scales come back as their own codes; a per-batch
    # position array gives every batch entry its own angles
    codes = synth.randint(28, np.arange(Nb * H * T * D), 0, 0x7F).astype(np.uint8).reshape(Nb, H, T, D)
    one = np.ones((Nb, H))
    _, k8, v8, _, _ = oracle.rope_append_fp8kv(q, oracle.fp8_e4m3_decode(codes), -oracle.fp8_e4m3_decode(codes), kc, vc, one, one,
                                               np.zeros(T, np.int64), 0, P)
    np.testing.assert_array_equal(k8[:, :, P:P + T], codes)
    np.testing.assert_array_equal(v8[:, :, P:P + T] & 0x7F, codes & 0x7F)
    pos2 = np.stack([pos, pos[::-1]])
    _, k8b, _, _, _ = oracle.rope_append_fp8kv(q, kn, vn, kc, vc, ks, vs, pos2, P - 1, P)
    _, k8r, _, _, _ = oracle.rope_append_fp8kv(q[1:], kn[1:], vn[1:], kc[1:], vc[1:], ks[1:], vs[1:], pos[::-1], P - 1, P)
    np.testing.assert_array_equal(k8b[1], k8r[0])
    # saturation: a scale far too small stores the largest magnitude
    _, ksat, _, _, _ = oracle.rope_append_fp8kv(q, kn * 1e12, vn, kc, vc, one, one, pos, P - 1, P)
    assert set(np.unique(ksat[:, :, P:P + T] & 0x7F)) == {0x7E}
