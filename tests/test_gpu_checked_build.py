"""The bounds-checked build of the library (librest_gfx950_checked.so, the same sources with -DREST_BOUNDS_CHECK):
indices that depend on data or on the launch plan are clamped into their arrays, a violation makes the call return
REST_BOUNDS_VIOLATION, and no kernel traps.  The binding loads it when REST_LIBRARY=checked, one library per process,
so it is exercised in child processes: a slice of the parity suite must pass under it unchanged (no index of the
product's own making leaves its array), and a suffix array whose entries point outside the stream must be reported."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_checked(args, timeout):
    env = dict(os.environ, REST_LIBRARY="checked")
    return subprocess.run([sys.executable] + args, cwd=ROOT, env=env, capture_output=True, text=True, timeout=timeout)


def test_parity_slice_passes_under_the_bounds_checked_build():
    pick = ("build_index_equals_oracle_sort or retrieve_small_corpora or retrieve_degenerate or bf16_shapes or "
            "bf16_split_counts or wide_units_split or arbitrary_masks or on_8bit_cache or accept_matches")
    r = run_checked(["-m", "pytest", "tests/test_gpu_parity.py", "-m", "gpu", "-x", "-q", "-k", pick, "-p", "no:cacheprovider"], 600)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-2000:]
    assert " passed" in r.stdout and "failed" not in r.stdout


VIOLATION_SCRIPT = r"""
import numpy as np, torch
import oracle, synth
import paper_2311_08252_amd as rest
assert rest.rest_version().endswith("(bounds-checked build)")
corpus = synth.randint(3, np.arange(5000), 0, 4).astype(np.int32)
sa = oracle.suffix_array(corpus).astype(np.int32)
d_corpus = torch.from_numpy(corpus).cuda()
ok = rest.rest_index_from_sa(d_corpus, torch.from_numpy(sa).cuda())          # a sound array passes
ctx = torch.from_numpy(corpus[100:140][None].copy()).cuda()
ln = torch.tensor([40], dtype=torch.int32, device="cuda")
rest.rest_retrieve(ok, ctx, ln)
bad = sa.copy()
bad[:] = 5000 + 12345                                                          # every entry points past the stream
try:
    rest.rest_index_from_sa(d_corpus, torch.from_numpy(bad).cuda())
    print("NOT REPORTED")
except rest.RestError as e:
    print("STATUS", e.status)
# the library is usable afterwards
tree = rest.rest_retrieve(ok, ctx, ln)
torch.cuda.synchronize()
print("NODES", int(tree.n_nodes[0]))
"""


def test_entries_outside_the_stream_are_reported_not_followed():
    r = run_checked(["-c", VIOLATION_SCRIPT], 300)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]
    assert "STATUS -8" in r.stdout and "NODES" in r.stdout, r.stdout
