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
