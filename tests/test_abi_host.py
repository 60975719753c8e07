"""CPU-side checks of the C ABI: the library loads, exports every function include/rest.h declares, and
its host-only logic (status strings, argument validation, workspace sizing) behaves as documented.
No kernel is launched here."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2311_08252_amd", "librest_gfx950.so")


@pytest.fixture(scope="module")
def rest():
    if not os.path.exists(LIB):
        from paper_2311_08252_amd.build import build   # noqa: WPS433 (build.py imports nothing from the package)
        build()
    import paper_2311_08252_amd as mod
    return mod


def declared_functions():
    text = open(os.path.join(ROOT, "include", "rest.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rest_[a-z_0-9]+)\s*\(", text)))


def test_header_functions_are_exported(rest):
    names = declared_functions()
    assert len(names) == 20 and "rest_retrieve" in names and "rest_tree_attention" in names
    lib = ctypes.CDLL(LIB)
    for n in names:
        assert getattr(lib, n) is not None
    assert sorted(rest.EXPORTS) == names


def test_status_strings_and_version(rest):
    assert rest.rest_status_string(0) == "ok"
    assert "workspace" in rest.rest_status_string(rest.REST_WORKSPACE_TOO_SMALL)
    assert "file" in rest.rest_status_string(rest.REST_IO_ERROR) and "file" in rest.rest_status_string(rest.REST_BAD_FILE)
    assert rest.rest_status_string(12345) == "unknown status"
    assert rest.rest_version().startswith("rest-gfx950")


def test_limits_match_header(rest):
    text = open(os.path.join(ROOT, "include", "rest.h")).read()
    for name in ["REST_MAX_SUFFIX_LEN", "REST_MAX_CONT_LEN", "REST_MAX_MATCHES", "REST_MAX_NODES", "REST_MAX_QUERY_ROWS"]:
        val = int(re.search(rf"#define {name} (\d+)", text).group(1))
        assert getattr(rest, name) == val


def make_desc(rest, **over):
    d = rest.rest_attn_desc()
    d.Nb, d.H, d.Tq, d.Tk, d.P, d.D = 32, 32, 64, 64, 2048, 128
    d.dtype, d.scale = rest.REST_BF16, 0.088
    L = 2112
    d.q_stride[:] = [32 * 64 * 128, 64 * 128, 128]
    d.o_stride[:] = [32 * 64 * 128, 64 * 128, 128]
    d.k_stride[:] = [32 * L * 128, L * 128, 128]
    d.v_stride[:] = [32 * L * 128, L * 128, 128]
    for k, v in over.items():
        setattr(d, k, v)
    return d


def test_attention_workspace_sizing_is_host_only(rest):
    # sixteen grouped query heads of 64 draft tokens are the most one slab takes: four groups of 256 rows over 1024
    # units, every stream a whole unit; one row more is refused (size 0 = invalid description)
    wide = make_desc(rest, Nb=8, Tq=1024, mask_rows=64)
    wide.q_stride[:] = [32 * 1024 * 128, 1024 * 128, 128]
    wide.o_stride[:] = [32 * 1024 * 128, 1024 * 128, 128]
    assert rest.rest_tree_attention_workspace_bytes(wide) == 0
    lib = ctypes.CDLL(LIB)
    p16 = ctypes.c_void_p(16)
    wide.Tq = 1025
    assert lib.rest_tree_attention(p16, p16, p16, p16, p16, ctypes.byref(wide), None, 0, None) == rest.REST_INVALID_ARG
    # 1024 (layer, head) units over 1024 streams: every stream owns whole units, no partial results
    assert rest.rest_tree_attention_workspace_bytes(make_desc(rest)) == 0
    # one layer: 32 units, the split plan with 256 / 32 = 8 workgroups per unit: 32 tickets, then per workgroup
    # 64 rows x (reference, sum as floats + 128 bf16 outputs)
    one_layer = make_desc(rest, Nb=1)
    assert rest.rest_tree_attention_workspace_bytes(one_layer) == 256 + 32 * 8 * 64 * (8 + 256)
    # few key blocks: every key group of a workgroup needs one, so 9 blocks allow two workgroups per unit; below 8, stream-K
    assert rest.rest_tree_attention_workspace_bytes(make_desc(rest, Nb=1, P=224)) == 256 + 32 * 2 * 64 * (8 + 256)
    short = make_desc(rest, Nb=1, P=150)
    assert rest.rest_tree_attention_workspace_bytes(short) == (32 * 7 // 4) * 2 * 64 * (128 + 2) * 4
    forced = make_desc(rest, Nb=1, num_splits=4)
    assert rest.rest_tree_attention_workspace_bytes(forced) == 32 * 4 * 2 * 64 * 130 * 4
    # 128 queries: streams of four wavefronts on 64-key tiles: 32 units x 33 tiles over 264 streams, 128 rows per slot
    wide = make_desc(rest, Nb=1, Tq=128, Tk=128, P=1984)
    assert rest.rest_tree_attention_workspace_bytes(wide) == 264 * 2 * 128 * (128 + 2) * 4
    # 13B shape: 1600 units, 1024 streams: one whole unit each, and 576 >= 512 of them a second one: nothing is cut
    big = make_desc(rest, Nb=40, H=40, P=4096)
    assert rest.rest_tree_attention_workspace_bytes(big) == 0
    # 1280 units: the 256 < 512 left over after the whole round are cut into 1024 spans
    cut = make_desc(rest, Nb=40, H=32, P=4096)
    assert rest.rest_tree_attention_workspace_bytes(cut) == 1024 * 2 * 64 * 130 * 4
    fp32 = make_desc(rest, Nb=1, dtype=rest.REST_FP32, num_splits=3)
    assert rest.rest_tree_attention_workspace_bytes(fp32) == 32 * 3 * 64 * 130 * 4
    for bad in [dict(D=64), dict(Tq=0), dict(Tq=257), dict(Tk=257), dict(scale=0.0), dict(dtype=7), dict(num_splits=65),
                dict(Nb=0), dict(P=-1), dict(mask_rows=-1), dict(mask_rows=65)]:
        assert rest.rest_tree_attention_workspace_bytes(make_desc(rest, **bad)) == 0


def test_calls_reject_null_and_bad_arguments_before_touching_the_gpu(rest):
    lib = rest._lib
    d = make_desc(rest)
    assert lib.rest_tree_attention(None, None, None, None, None, ctypes.byref(d), None, 0, None) == rest.REST_INVALID_ARG
    h = ctypes.c_void_p()
    assert lib.rest_build_index(None, 10, 4, 4, None, ctypes.byref(h)) == rest.REST_INVALID_ARG
    assert lib.rest_build_index(ctypes.c_void_p(16), 10, 3, 4, None, ctypes.byref(h)) == rest.REST_INVALID_ARG
    assert lib.rest_build_index(ctypes.c_void_p(16), 1 << 31, 4, 4, None, ctypes.byref(h)) == rest.REST_INVALID_ARG
    assert lib.rest_build_index(ctypes.c_void_p(16), 0, 4, 8, None, ctypes.byref(h)) == rest.REST_INVALID_ARG
    assert lib.rest_index_from_sa(ctypes.c_void_p(16), None, 10, 4, 4, None, ctypes.byref(h)) == rest.REST_INVALID_ARG
    assert lib.rest_build_index_prefix(ctypes.c_void_p(16), 10, 4, 4, -1, None, ctypes.byref(h)) == rest.REST_INVALID_ARG
    assert lib.rest_build_index_prefix(None, 10, 4, 4, 32, None, ctypes.byref(h)) == rest.REST_INVALID_ARG
    assert lib.rest_index_sort_depth(None) == -1
    assert lib.rest_index_view(None, None, None, None, None, None) == rest.REST_INVALID_ARG
    lib.rest_index_destroy(None)
    prm = rest.rest_retrieve_params(16, 2, 100, 10, 64, 0, 0, 0, 0)
    tree = rest.rest_tree()
    assert lib.rest_retrieve(None, None, None, 1, 8, ctypes.byref(prm), ctypes.byref(tree), None, 0, None) == rest.REST_INVALID_ARG
    assert lib.rest_accept(None, ctypes.byref(tree), 1, 64, 10, None, None, None, None) == rest.REST_INVALID_ARG
    assert rest.rest_retrieve_workspace_bytes(4) == 0
    p16 = ctypes.c_void_p(16)
    big = ctypes.c_size_t(1 << 30)
    assert lib.rest_sample_ids(None, 100, p16, 1, 100, 1.0, 0.9, p16, p16, big, None) == rest.REST_INVALID_ARG
    assert lib.rest_sample_ids(p16, 99, p16, 1, 100, 1.0, 0.9, p16, p16, big, None) == rest.REST_INVALID_ARG        # stride < V
    assert lib.rest_sample_ids(p16, 100, p16, 1, 100, 0.0, 0.9, p16, p16, big, None) == rest.REST_INVALID_ARG       # temperature
    assert lib.rest_sample_ids(p16, 100, p16, 1, 100, 1.0, 0.0, p16, p16, big, None) == rest.REST_INVALID_ARG       # top_p
    assert lib.rest_sample_ids(p16, 100, p16, 1, 100, 1.0, 1.5, p16, p16, big, None) == rest.REST_INVALID_ARG
    assert lib.rest_sample_ids(p16, 200000, p16, 1, 200000, 1.0, 0.9, p16, p16, big, None) == rest.REST_UNSUPPORTED
    assert lib.rest_sample_ids(p16, 100, p16, 0, 100, 1.0, 0.9, p16, None, 0, None) == rest.REST_OK                 # nothing to do
    need = rest.rest_sample_ids_workspace_bytes(65, 32000)
    assert need == 65 * (2048 + 32) * 8 and rest.rest_sample_ids_workspace_bytes(65, 131072) == need
    assert rest.rest_sample_ids_workspace_bytes(1, 131073) == 0
    assert lib.rest_sample_ids(p16, 32000, p16, 65, 32000, 1.0, 0.9, p16, p16, need - 1, None) == rest.REST_WORKSPACE_TOO_SMALL
    assert lib.rest_sample_ids(p16, 32000, p16, 65, 32000, 1.0, 0.9, p16, None, need, None) == rest.REST_WORKSPACE_TOO_SMALL
    assert lib.rest_sample_ids(p16, 32000, p16, 65, 32000, 1.0, 0.9, p16, ctypes.c_void_p(20), need, None) == rest.REST_INVALID_ARG
    hh = ctypes.c_void_p()
    assert lib.rest_index_save(None, b"/tmp/x", None) == rest.REST_INVALID_ARG
    assert lib.rest_index_load(None, p16, 10, 4, None, ctypes.byref(hh)) == rest.REST_INVALID_ARG
    assert lib.rest_index_load(b"/tmp/x", None, 10, 4, None, ctypes.byref(hh)) == rest.REST_INVALID_ARG
    assert lib.rest_index_load(b"/tmp/x", p16, 10, 3, None, ctypes.byref(hh)) == rest.REST_INVALID_ARG
    # a file that is not there is reported before anything touches the GPU
    assert lib.rest_index_load(b"/nonexistent-dir/none.restsa", p16, 10, 4, None, ctypes.byref(hh)) == rest.REST_IO_ERROR
    kd = rest.rest_kv_desc()
    kd.Nb, kd.H, kd.T, kd.D, kd.P, kd.pos_offset, kd.dtype, kd.theta = 2, 4, 8, 128, 16, 15, rest.REST_BF16, 10000.0
    for name in ("q_stride", "kn_stride", "vn_stride"):
        getattr(kd, name)[:] = [4 * 8 * 128, 8 * 128, 128]
    for name in ("kc_stride", "vc_stride"):
        getattr(kd, name)[:] = [4 * 32 * 128, 32 * 128, 128]
    p16 = ctypes.c_void_p(16)
    assert lib.rest_rope_append(None, p16, p16, p16, p16, p16, ctypes.byref(kd), None) == rest.REST_INVALID_ARG
    assert lib.rest_rope_append(p16, p16, p16, p16, p16, None, ctypes.byref(kd), None) == rest.REST_INVALID_ARG
    assert lib.rest_rope_append(ctypes.c_void_p(8), p16, p16, p16, p16, p16, ctypes.byref(kd), None) == rest.REST_INVALID_ARG
    assert lib.rest_kv_compact(p16, p16, None, p16, 10, ctypes.byref(kd), None) == rest.REST_INVALID_ARG
    assert lib.rest_kv_compact(p16, p16, p16, p16, 33, ctypes.byref(kd), None) == rest.REST_INVALID_ARG
    for field, bad in (("D", 64), ("T", 0), ("T", 257), ("theta", 1.0), ("P", -1), ("Nb", 0)):
        keep = getattr(kd, field)
        setattr(kd, field, bad)
        assert lib.rest_rope_append(p16, p16, p16, p16, p16, p16, ctypes.byref(kd), None) == rest.REST_INVALID_ARG
        assert lib.rest_kv_compact(p16, p16, p16, p16, 10, ctypes.byref(kd), None) == rest.REST_INVALID_ARG
        setattr(kd, field, keep)
    kd.kc_stride[2] = 100          # rows must be 16-byte aligned and at least D long
    assert lib.rest_kv_compact(p16, p16, p16, p16, 10, ctypes.byref(kd), None) == rest.REST_INVALID_ARG
    kd.kc_stride[2] = 128
    kd.dtype = rest.REST_FP32
    assert lib.rest_kv_compact(p16, p16, p16, p16, 10, ctypes.byref(kd), None) == rest.REST_UNSUPPORTED


def test_header_is_plain_c_and_struct_layouts_match_the_binding(tmp_path, rest):
    """include/rest.h compiles as C99 and as C++17 on its own, and the sizes / field offsets a C compiler gives the
    parameter structs are the ones the ctypes binding marshals."""
    import subprocess
    structs = {"rest_retrieve_params": rest.rest_retrieve_params, "rest_attn_desc": rest.rest_attn_desc,
               "rest_kv_desc": rest.rest_kv_desc, "rest_tree": rest.rest_tree}
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "rest.h"', 'int main(void) {']
    for name, cls in structs.items():
        lines.append(f'  printf("{name} %zu\\n", sizeof({name}));')
        for field, _ in cls._fields_:
            lines.append(f'  printf("{name}.{field} %zu\\n", offsetof({name}, {field}));')
    lines += ['  return 0;', '}']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    inc = os.path.join(ROOT, "include")
    subprocess.check_call(["g++", "-std=c++17", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-x", "c++", "-I", inc, str(src)])
    exe = tmp_path / "layout"
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", inc, str(src), "-o", str(exe)])
    out = dict(line.split() for line in subprocess.check_output([str(exe)], text=True).splitlines())
    for name, cls in structs.items():
        assert int(out[name]) == ctypes.sizeof(cls), name
        for field, _ in cls._fields_:
            assert int(out[f"{name}.{field}"]) == getattr(cls, field).offset, (name, field)


def test_binding_rejects_buffers_that_do_not_fit_the_call(rest):
    """The kernels index every buffer from the sizes in the call, so the binding compares shapes and dtypes with those
    sizes before a pointer goes anywhere (host tensors suffice: the shape checks come first)."""
    import torch
    bf = torch.bfloat16
    q, k, v = torch.zeros((4, 2, 8, 128), dtype=bf), torch.zeros((4, 2, 40, 128), dtype=bf), torch.zeros((4, 2, 40, 128), dtype=bf)
    ok_mask = torch.zeros((8, 1), dtype=torch.int64)

    def attn(**over):
        a = dict(q=q, k=k, v=v, mask=ok_mask, prefix_len=32, scale=0.1)
        a.update(over)
        return rest.rest_tree_attention(**a)

    # a single tree's [1, c, words] mask with four batch entries would be read as one mask per entry, three past its end
    with pytest.raises(ValueError, match="mask"):
        attn(mask=torch.zeros((1, 8, 1), dtype=torch.int64))
    for bad in (torch.zeros((7, 1), dtype=torch.int64), torch.zeros((8, 2), dtype=torch.int64),
                torch.zeros((8, 1), dtype=torch.int32), torch.zeros((8, 2), dtype=torch.int64)[:, :1]):
        with pytest.raises(ValueError, match="mask"):
            attn(mask=bad)
    with pytest.raises(ValueError, match="mask_rows"):
        attn(mask_rows=9)
    with pytest.raises(ValueError, match="mask"):
        attn(mask_rows=4)                                              # then the mask has four rows, not eight
    with pytest.raises(ValueError):
        attn(v=torch.zeros((4, 2, 39, 128), dtype=bf))
    with pytest.raises(ValueError):
        attn(k=torch.zeros((4, 3, 40, 128), dtype=bf), v=torch.zeros((4, 3, 40, 128), dtype=bf))
    with pytest.raises(ValueError):
        attn(k=k.float(), v=v.float())
    with pytest.raises(ValueError, match="out"):
        attn(out=torch.zeros((4, 2, 7, 128), dtype=bf))
    with pytest.raises(ValueError, match="out"):
        attn(out=torch.zeros((4, 2, 8, 128), dtype=torch.float32))
    with pytest.raises(ValueError, match="prefix_len"):
        attn(prefix_len=41)
    with pytest.raises(ValueError):
        attn(q=q.transpose(2, 3))
    with pytest.raises(ValueError, match="scale"):
        attn(k=k.view(torch.uint8)[..., :128].contiguous(), v=v.view(torch.uint8)[..., :128].contiguous(),
             k_scale=torch.ones(7))
    with pytest.raises(TypeError):                                     # shapes fit; host tensors are then refused as such
        attn()

    class FakeIndex:
        handle = None

    ctx, ln = torch.zeros((3, 16), dtype=torch.int32), torch.zeros(3, dtype=torch.int32)
    with pytest.raises(ValueError, match="ctx_len"):
        rest.rest_retrieve(FakeIndex(), ctx, ln[:2], max_nodes=8)
    small = rest.Tree.empty(3, 4, device="cpu")                        # room for four nodes, eight asked for
    with pytest.raises(ValueError, match="tree"):
        rest.rest_retrieve(FakeIndex(), ctx, ln, out=small, max_nodes=8)
    few = rest.Tree.empty(2, 8, device="cpu")
    with pytest.raises(ValueError, match="tree"):
        rest.rest_retrieve(FakeIndex(), ctx, ln, out=few, max_nodes=8)
    wrong = rest.Tree.empty(3, 8, device="cpu")
    wrong.match_count = wrong.match_count.to(torch.int32)
    with pytest.raises(ValueError, match="match_count"):
        rest.rest_retrieve(FakeIndex(), ctx, ln, out=wrong, max_nodes=8)

    tree = rest.Tree.empty(3, 8, device="cpu")
    with pytest.raises(ValueError, match="tree"):                      # ids for a capacity of 16 against a tree of 8
        rest.rest_accept(torch.zeros((3, 17), dtype=torch.int32), tree, 10)
    with pytest.raises(ValueError, match="tree"):
        rest.rest_accept(torch.zeros((2, 9), dtype=torch.int32), tree, 10)
    with pytest.raises(ValueError, match="accept_path"):
        rest.rest_accept(torch.zeros((3, 9), dtype=torch.int32), tree, 10, accept_path=torch.zeros((3, 9), dtype=torch.int32))
    with pytest.raises(ValueError, match="path_cap"):
        rest.rest_accept(torch.zeros((3, 9), dtype=torch.int32), tree, 33)
    with pytest.raises(TypeError):
        rest.rest_accept(torch.zeros((3, 9), dtype=torch.int32), tree, 10)
