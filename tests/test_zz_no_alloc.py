"""rest_tree_attention_noalloc (partial results in the library's own fixed device array) against rest_tree_attention
with a caller's workspace: same kernels, so the outputs must agree bit for bit -- on two calls in a row, the second
with a smaller input, so that what the first call left in the array is shown not to matter."""
import ctypes

import numpy as np
import pytest
import torch

import synth

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2311_08252_amd as rest


def inputs(Nb, H, T, P, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    q = torch.randn((Nb, H, T, 128), generator=g, device="cuda").to(torch.bfloat16)
    k = torch.randn((Nb, H, P + T, 128), generator=g, device="cuda").to(torch.bfloat16)
    v = torch.randn((Nb, H, P + T, 128), generator=g, device="cuda").to(torch.bfloat16)
    mask = torch.from_numpy(synth.random_tree(T, seed)[3].view(np.int64)).cuda()
    return q, k, v, mask


def test_noalloc_entry_point_equals_the_workspace_one_on_two_calls_in_a_row():
    scale = float(1 / np.sqrt(128.0))
    # one layer of the 7B shape (32 units cut into 528 spans: 35 MB of partials), then a smaller, ragged one
    cases = [(1, 32, 64, 2048, 0), (1, 8, 33, 300, 0), (2, 3, 130, 777, 5), (1, 32, 64, 2048, 3)]
    prepared = []
    for i, (Nb, H, T, P, splits) in enumerate(cases):
        q, k, v, mask = inputs(Nb, H, T, P, 900 + i)
        want = torch.full_like(q, float("nan"))
        desc = rest.make_attn_desc(q, k, v, want, P, scale, False, splits)
        assert 0 < rest.rest_tree_attention_workspace_bytes(desc) <= rest.REST_STATIC_SCRATCH_BYTES
        rest.rest_tree_attention(q, k, v, mask, P, scale, out=want, num_splits=splits)
        prepared.append((q, k, v, mask, P, splits, want, torch.full_like(q, float("nan"))))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    for q, k, v, mask, P, splits, want, got in prepared:          # back to back on one stream, no allocation between
        rest.rest_tree_attention_noalloc(q, k, v, mask, P, scale, out=got, num_splits=splits)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    for q, k, v, mask, P, splits, want, got in prepared:
        assert torch.isfinite(got.float()).all()
        assert torch.equal(got.view(torch.int16), want.view(torch.int16))


def test_noalloc_entry_point_refuses_what_does_not_fit():
    # 64 forced splits of 512 units: 16384 streams x 2 slots x 64 rows x 130 floats = 1.09 GB of partials
    q, k, v, mask = inputs(1, 2, 64, 300, 7)
    big_q = q.expand(256, 2, 64, 128)
    big_k, big_v = k.expand(256, 2, 364, 128), v.expand(256, 2, 364, 128)
    out = torch.empty((256, 2, 64, 128), dtype=torch.bfloat16, device="cuda")
    desc = rest.make_attn_desc(big_q, big_k, big_v, out, 300, 0.088, False, 64)
    assert rest.rest_tree_attention_workspace_bytes(desc) > rest.REST_STATIC_SCRATCH_BYTES
    with pytest.raises(rest.RestError) as e:
        rest.rest_tree_attention_noalloc(big_q, big_k, big_v, mask, 300, 0.088, out=out, num_splits=64)
    assert e.value.status == rest.REST_WORKSPACE_TOO_SMALL
    # no workspace needed at all: nothing is asked of the runtime, the call just runs
    q, k, v, mask = inputs(32, 32, 64, 500, 8)
    want = rest.rest_tree_attention(q, k, v, mask, 500, 0.088)
    got = torch.empty_like(q)
    assert rest.rest_tree_attention_workspace_bytes(rest.make_attn_desc(q, k, v, got, 500, 0.088, False)) == 0
    rest.rest_tree_attention_noalloc(q, k, v, mask, 500, 0.088, out=got)
    torch.cuda.synchronize()
    assert torch.equal(got.view(torch.int16), want.view(torch.int16))
    st = rest._lib.rest_tree_attention_noalloc(None, None, None, None, None, ctypes.byref(desc), None)
    assert st == rest.REST_WORKSPACE_TOO_SMALL or st == rest.REST_INVALID_ARG
