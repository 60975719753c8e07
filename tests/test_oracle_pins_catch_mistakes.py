"""Do the pins pin?  Each case plants one plausible mistake in the CPU oracle -- a dropped factor, a wrong sign or
index, swapped operands, an inclusive bound for an exclusive one, a tie broken the other way -- and runs the pin tests
of that part of the oracle against the damaged copy: at least one of them has to fail.  Nothing here touches the GPU
path; the mistakes live in copies of the oracle's functions on the CPU and are undone after each case.

Python parts of the oracle are damaged in their source text (one replacement, which must apply exactly once); the
parts written in C are wrapped (arguments or results altered the way the mistake would alter them)."""
import importlib.util
import inspect
import os
import textwrap

import numpy as np
import pytest

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))
SLOW = {"test_c_oracle_under_address_and_undefined_behaviour_sanitizers"}      # compiles C; no oracle function in it


def pin_module(name):
    spec = importlib.util.spec_from_file_location("pins_" + name, os.path.join(HERE, f"test_oracle_{name}_pins.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def first_failing_pin(mod, tmp_path):
    """Calls the module's test functions, parametrisations expanded, and returns the name of the first that fails."""
    for name, fn in list(vars(mod).items()):
        if not name.startswith("test_") or name in SLOW or not callable(fn):
            continue
        cases = [{}]
        for mark in getattr(fn, "pytestmark", []):
            if mark.name != "parametrize":
                continue
            names = [s.strip() for s in mark.args[0].split(",")]
            cases = [{**c, **dict(zip(names, vals if len(names) > 1 else (vals,)))} for c in cases for vals in mark.args[1]]
        for kw in cases:
            if "tmp_path" in inspect.signature(fn).parameters:
                kw = {**kw, "tmp_path": tmp_path}
            try:
                fn(**kw)
            except Exception:                      # noqa: BLE001 - an assertion, or a crash the mistake causes
                return name
    return None


def edited(fn, old, new):
    """The oracle function with `old` replaced by `new` in its source."""
    src = textwrap.dedent(inspect.getsource(fn))
    assert src.count(old) == 1, (fn.__name__, old, src.count(old))
    scope = dict(vars(oracle))
    exec(compile(src.replace(old, new), f"<{fn.__name__} with a mistake>", "exec"), scope)
    return scope[fn.__name__]


# ---------------------------------------------------------------- mistakes in the Python parts: (function, old, new)
EDITS = {
    "attention: softmax scale dropped": ("attention", "tree_attention", "s = scale * np.matmul(", "s = np.matmul("),
    "attention: K used for V": ("attention", "tree_attention", "return np.matmul(p, v)", "return np.matmul(p, k)"),
    "attention: mask bit index off by one": ("attention", "tree_attention", ">> np.uint64(j % 64)", ">> np.uint64((j + 1) % 64)"),
    "attention: last cached key hidden": ("attention", "tree_attention", "bits[..., :P] = True", "bits[..., :max(P - 1, 0)] = True"),
    "attention: mask ignored": ("attention", "tree_attention", "s = np.where(bits, s, -np.inf)", "s = s + 0.0"),
    "attention: normalised over queries": ("attention", "tree_attention", "p = p / np.sum(p, axis=-1, keepdims=True)",
                                           "p = p / np.sum(p, axis=-2, keepdims=True)"),
    "rope: frequency exponent i/D": ("kv", "rope", "theta ** (-2.0 * np.arange", "theta ** (-1.0 * np.arange"),
    "rope: rotation the other way": ("kv", "rope", "[a * c - b * s, a * s + b * c]", "[a * c + b * s, b * c - a * s]"),
    "rope: adjacent pairs instead of half-split": ("kv", "rope", "a, b = x[..., :h], x[..., h:]", "a, b = x[..., 0::2], x[..., 1::2]"),
    "append: position offset forgotten": ("kv", "rope_append", "+ int(pos_offset)", "+ 0"),
    "append: V rotated as well": ("kv", "rope_append", "vc[..., P:P + T, :] = np.asarray(v_new, dtype=np.float64)",
                                  "vc[..., P:P + T, :] = rope(v_new, pos, theta)"),
    "append: rows one place early": ("kv", "rope_append", "kc[..., P:P + T, :] = rope(k_new, pos, theta)",
                                     "kc[..., P - 1:P + T - 1, :] = rope(k_new, pos, theta)"),
    "compact: reads the rows it has already overwritten": ("kv", "kv_compact", "= cache[..., P + int(accept_path[i]), :]",
                                                           "= out[..., P + int(accept_path[i]), :]"),
    "compact: rows land one place late": ("kv", "kv_compact", "out[..., P + i, :] =", "out[..., P + i + 1, :] ="),
    "sampling: nucleus must exceed top_p": ("sampling", "nucleus_sample", "np.nonzero(cum.astype(np.float64) >= thr)", "np.nonzero(cum.astype(np.float64) > thr)"),
    "sampling: draw at cumulative mass >= target": ("sampling", "nucleus_sample", "np.nonzero(cum.astype(np.float64) > target)", "np.nonzero(cum.astype(np.float64) >= target)"),
    "sampling: logits times temperature": ("sampling", "nucleus_weights", "c = np.float64(_LOG2E) / np.float64(np.float32(temperature))",
                                           "c = np.float64(_LOG2E) * np.float64(np.float32(temperature))"),
    "sampling: ties by descending id": ("sampling", "nucleus_sample", "np.lexsort((np.arange(x.size), -x))",
                                        "np.lexsort((-np.arange(x.size), -x))"),
    "sampling: u not scaled by the nucleus mass": ("sampling", "nucleus_sample", "* np.float64(mass)", "* np.float64(total)"),
    "sampling: natural exponent taken for base two": ("sampling", "nucleus_weights", "t = (y - n) * np.float64(_LN2)", "t = (y - n)"),
    "sampling: polynomial one term short of the constant": ("sampling", "nucleus_weights", "for k in range(12, -1, -1):", "for k in range(12, 0, -1):"),
    "sampling: weights in units of 2^-35": ("sampling", "nucleus_weights", "(n + SAMPLE_WEIGHT_BITS).astype(np.int32)", "(n + SAMPLE_WEIGHT_BITS - 1).astype(np.int32)"),
    "mask: a node does not see itself": ("integer", "mask_from_parents", "        v = i\n", "        v = int(parent_idx[i])\n"),
    "mask: parent only, no further ancestors": ("integer", "mask_from_parents", "while v != -1:", "for _ in range(2 if v != -1 else 0):\n            if v == -1:\n                break"),
    "attention: only the first mask word read": ("attention", "tree_attention", "mask[..., j // 64]", "mask[..., 0]"),
    "attention: 8-bit cache, V scaled by the K scale": ("fp8", "tree_attention_fp8kv", "fp8_e4m3_decode(v8) * np.asarray(v_scale,",
                                                       "fp8_e4m3_decode(v8) * np.asarray(k_scale,"),
    "append: queries not rotated": ("kv", "rope_append", "qr = rope(q, pos, theta)", "qr = np.asarray(q, dtype=np.float64)"),
    "append: 8-bit cache, multiplied by the scale": ("fp8", "rope_append_fp8kv", "kx = rope(k_new, pos, theta) / np.asarray(",
                                                    "kx = rope(k_new, pos, theta) * np.asarray("),
    "compact: last accepted row not moved": ("kv", "kv_compact", "for i in range(int(accept_len)):", "for i in range(int(accept_len) - 1):"),
    "retrieve: evenly spaced sample rounded up": ("integer", "retrieve", "pick = np.array([(i * S) // K for i in range(K)]",
                                                  "pick = np.array([min((i * S + K - 1) // K, S - 1) for i in range(K)]"),
    "random selection: draw by remainder": ("integer", "random_rows", "(_mix64(h + G * (1 + j)) * n_rows) >> 64", "_mix64(h + G * (1 + j)) % n_rows"),
    "random selection: draws counted from zero": ("integer", "random_rows", "_mix64(h + G * (1 + j))", "_mix64(h + G * j)"),
    "depth-limited order: equal prefixes by descending position": ("integer", "prefix_sorted_array", "return np.lexsort(columns[::-1])",
                                                                   "return np.lexsort([-np.arange(n)] + columns[::-1])"),
    "depth-limited order: end of the stream largest": ("integer", "prefix_sorted_array", "np.zeros(depth, dtype=np.int64)]",
                                                       "np.full(depth, 1 << 40, dtype=np.int64)]"),
    "index file: fingerprint without the position": ("integer", "corpus_fingerprint", "z = tok + (np.arange(", "z = tok + 0 * (np.arange("),
    "decoding loop: bonus token left out": ("integer", "rest_decode", "        seq.append(int(nxt))\n", "        seq.append(int(nxt)) if n_acc == 0 else None\n"),
    "fp8: truncation instead of nearest": ("fp8", "fp8_e4m3_encode", "code = np.where(d_lo < d_hi, lo, np.where(d_hi < d_lo, hi, np.where(lo % 2 == 0, lo, hi)))",
                                           "code = lo + (d_hi == 0)"),
    "fp8: ties away from zero": ("fp8", "fp8_e4m3_encode", "np.where(lo % 2 == 0, lo, hi)", "hi"),
    "fp8: exponent bias 8": ("fp8", "fp8_e4m3_decode", "- 7))", "- 8))"),
    "fp8: subnormals read as normals": ("fp8", "fp8_e4m3_decode", "np.where(e == 0, m * 2.0 ** -9,", "np.where(e < 0, m * 2.0 ** -9,"),
}


# ---------------------------------------------------------------- mistakes in the C parts, as wrappers
def retrieve_with(change):
    orig = oracle.retrieve

    def f(corpus, context, n_max=16, n_min=2, max_matches=5000, cont_len=10, one_pass=False, strided=False):
        if change == "n_min ignored":
            return orig(corpus, context, n_max, 1, max_matches, cont_len, one_pass, strided)
        if change == "longest length never tried":
            return orig(corpus, context, max(n_max - 1, 1), n_min, max_matches, cont_len, one_pass, strided)
        got = orig(corpus, context, n_max, n_min, max_matches, cont_len, one_pass, strided)
        if change == "count capped at K":
            got.match_count = min(got.match_count, int(max_matches))
        elif change == "continuation starts at the last matched token" and got.matched_len:
            for r, pos in enumerate(got.row_pos):
                seg = np.asarray(corpus[int(pos) + got.matched_len - 1:int(pos) + got.matched_len - 1 + cont_len], np.int32)
                got.rows[r, :] = -1
                got.rows[r, :seg.shape[0]] = seg
                got.row_len[r] = seg.shape[0]
        elif change == "occurrences without a continuation dropped":
            keep = got.row_len > 0
            got = oracle.Retrieved(got.matched_len if keep.any() else 0, got.match_count - int((~keep).sum()),
                                   got.row_pos[keep], got.rows[keep], got.row_len[keep])
        elif change == "keeps the last K of the range" and got.match_count > max_matches > 0 and not strided:
            full = orig(corpus, context, n_max, n_min, got.match_count, cont_len, one_pass, False)
            keep = slice(got.match_count - int(max_matches), got.match_count)
            got = oracle.Retrieved(full.matched_len, full.match_count, full.row_pos[keep], full.rows[keep], full.row_len[keep])
        return got
    return f


def select_with(change):
    orig = oracle.select_drafts

    def f(rows, row_len, max_nodes, order=None):
        if change == "one node too few":
            t = orig(rows, row_len, max(int(max_nodes) - 1, 0), order)
            c = int(max_nodes)
            pad = lambda a, fill: np.concatenate([a, np.full((c - a.shape[0],) + a.shape[1:], fill, a.dtype)])   # noqa: E731
            words = max(1, (c + 63) // 64)
            mask = np.zeros((c, words), np.uint64)
            mask[:t.tree_mask.shape[0], :t.tree_mask.shape[1]] = t.tree_mask
            return oracle.DraftTree(t.n_nodes, pad(t.draft_tokens, -1), pad(t.parent_idx, -1), pad(t.pos_ids, 0),
                                    pad(t.node_weight, 0), mask, 0, 0, t.total_trie_nodes)
        t = orig(rows, row_len, max_nodes, order)
        live = np.arange(t.draft_tokens.shape[0]) < t.n_nodes
        if change == "depths counted from zero":
            t.pos_ids = np.where(live, t.pos_ids - 1, t.pos_ids).astype(np.int32)
        elif change == "weights one too high":
            t.node_weight = np.where(live, t.node_weight + 1, t.node_weight).astype(np.int32)
        elif change == "rows beyond their length counted":
            full = np.full_like(np.asarray(row_len), np.asarray(rows).shape[1] if np.asarray(rows).ndim == 2 else 0)
            return orig(np.where(np.asarray(rows) < 0, 0, rows), full, max_nodes, order)
        elif change == "siblings in descending token order" and t.n_nodes > 1:
            # the first level reversed, subtrees moving with their roots: a relabelling of the nodes
            n = t.n_nodes
            top = [i for i in range(n) if t.parent_idx[i] == -1]
            rank = {i: k for k, i in enumerate(reversed(top))}
            root = np.zeros(n, np.int64)
            for i in range(n):
                root[i] = rank[i] if t.parent_idx[i] == -1 else root[t.parent_idx[i]]
            perm = sorted(range(n), key=lambda i: (t.pos_ids[i], root[i], i))      # new place -> old node
            where = {old: new for new, old in enumerate(perm)}
            tok, par, pos, wgt = t.draft_tokens.copy(), t.parent_idx.copy(), t.pos_ids.copy(), t.node_weight.copy()
            for new, old in enumerate(perm):
                tok[new], pos[new], wgt[new] = t.draft_tokens[old], t.pos_ids[old], t.node_weight[old]
                par[new] = -1 if t.parent_idx[old] == -1 else where[int(t.parent_idx[old])]
            t.draft_tokens, t.parent_idx, t.pos_ids, t.node_weight = tok, par, pos, wgt
            t.tree_mask = oracle.mask_from_parents(par, n, t.tree_mask.shape[1])
        return t
    return f


def python_select(rows, row_len, max_nodes, order=None, tie="as defined", layout="as defined"):
    """Algorithm 2 and the layout once more, on Python tuples, with the order of equal weights and the order inside
    a depth open to a mistake."""
    from collections import Counter
    rows, row_len = np.asarray(rows), np.asarray(row_len)
    weight = Counter()
    for r in range(rows.shape[0]):
        for d in range(1, int(row_len[r]) + 1):
            weight[tuple(int(x) for x in rows[r, :d])] += 1
    rank = {"as defined": lambda p: (-weight[p], len(p), p),
            "deeper first": lambda p: (-weight[p], -len(p), p),
            "larger token first": lambda p: (-weight[p], len(p), tuple(-x for x in p))}[tie]
    c = int(max_nodes)
    kept = sorted(weight, key=rank)[:c]
    place = {"as defined": lambda p: (len(p), p), "heavier first": lambda p: (len(p), -weight[p], p)}[layout]
    kept.sort(key=place)
    index = {p: i for i, p in enumerate(kept)}
    tok = np.full(c, -1, np.int32)
    par = np.full(c, -1, np.int32)
    pos = np.zeros(c, np.int32)
    wgt = np.zeros(c, np.int32)
    for i, p in enumerate(kept):
        tok[i], pos[i], wgt[i] = p[-1], len(p), weight[p]
        par[i] = index.get(p[:-1], -1) if len(p) > 1 else -1
    words = max(1, (c + 63) // 64)
    mask = np.zeros((c, words), np.uint64)
    for i, p in enumerate(kept):
        for d in range(1, len(p) + 1):
            j = index.get(p[:d])
            if j is not None:
                mask[i, j // 64] |= np.uint64(1) << np.uint64(j % 64)
    return oracle.DraftTree(len(kept), tok, par, pos, wgt, mask, 0, 0, len(weight))


def test_the_python_selection_is_the_oracles_when_no_mistake_is_planted():
    rng = np.random.default_rng(4)
    for _ in range(30):
        R, m, c = int(rng.integers(1, 40)), int(rng.integers(1, 7)), int(rng.integers(1, 40))
        rows = rng.integers(0, 3, (R, m)).astype(np.int32)
        row_len = rng.integers(0, m + 1, R).astype(np.int32)
        rows[np.arange(m)[None, :] >= row_len[:, None]] = -1
        a, b = python_select(rows, row_len, c), oracle.select_drafts(rows, row_len, c)
        assert a.n_nodes == b.n_nodes and a.total_trie_nodes == b.total_trie_nodes
        for f in ("draft_tokens", "parent_idx", "pos_ids", "node_weight", "tree_mask"):
            np.testing.assert_array_equal(getattr(a, f), getattr(b, f), err_msg=f)


def accept_with(change):
    orig = oracle.accept

    def f(ids, draft_tokens, parent_idx, n_nodes, path_cap):
        n, path, nxt = orig(ids, draft_tokens, parent_idx, n_nodes, path_cap)
        if change == "bonus token is the last accepted draft token" and n > 0:
            nxt = int(draft_tokens[path[n - 1]])
        elif change == "stops one token early" and n > 0:
            path = path.copy()
            path[n - 1] = -1
            n -= 1
            nxt = int(ids[0] if n == 0 else ids[1 + path[n - 1]])
        elif change == "the model's token read at the child":
            # walks on while the child's own prediction, not the current position's, names the child
            cur, n, path = -1, 0, np.full(max(path_cap, 1), -1, np.int32)[:path_cap]
            while n < path_cap:
                kids = [i for i in range(n_nodes) if parent_idx[i] == cur and draft_tokens[i] == ids[1 + i]]
                if not kids:
                    break
                cur = kids[0]
                path[n] = cur
                n += 1
            nxt = int(ids[1 + cur])
        return n, path, nxt
    return f


def suffix_array_with(change):
    def f(corpus):
        toks = [int(x) for x in corpus]
        if change == "end of the stream sorts last":
            big = max(toks, default=0) + 1
            order = sorted(range(len(toks)), key=lambda i: tuple(toks[i:]) + (big,) * (len(toks) + 1 - (len(toks) - i)))
        else:                                   # "ordered by the first token only"
            order = sorted(range(len(toks)), key=lambda i: (toks[i], i))
        return np.array(order, dtype=np.int64)
    return f


WRAPS = {f"retrieve: {c}": ("integer", "retrieve", retrieve_with, c) for c in
         ["n_min ignored", "longest length never tried", "count capped at K",
          "continuation starts at the last matched token", "keeps the last K of the range",
          "occurrences without a continuation dropped"]}
WRAPS.update({f"select: {c}": ("integer", "select_drafts", select_with, c) for c in
              ["one node too few", "depths counted from zero", "weights one too high", "rows beyond their length counted",
               "siblings in descending token order"]})
WRAPS.update({f"select: equal weights, {t}": ("integer", "select_drafts",
                                               lambda t: (lambda rows, row_len, max_nodes, order=None: python_select(rows, row_len, max_nodes, order, tie=t)), t)
              for t in ["deeper first", "larger token first"]})
WRAPS["select: a depth laid out heavier first"] = ("integer", "select_drafts",
                                                   lambda _: (lambda rows, row_len, max_nodes, order=None: python_select(rows, row_len, max_nodes, order, layout="heavier first")), "")
WRAPS.update({f"accept: {c}": ("integer", "accept", accept_with, c) for c in
              ["bonus token is the last accepted draft token", "stops one token early", "the model's token read at the child"]})
WRAPS.update({f"suffix array: {c}": ("integer", "suffix_array", suffix_array_with, c) for c in
              ["end of the stream sorts last", "ordered by the first token only"]})


@pytest.mark.parametrize("part", ["integer", "attention", "kv", "sampling", "fp8"])
def test_the_harness_runs_the_pins_and_they_pass_on_the_oracle_as_it_is(part, tmp_path):
    assert first_failing_pin(pin_module(part), tmp_path) is None


@pytest.mark.parametrize("mistake", sorted(EDITS))
def test_a_mistake_in_the_python_part_fails_a_pin(mistake, monkeypatch, tmp_path):
    part, fn, old, new = EDITS[mistake]
    monkeypatch.setattr(oracle, fn, edited(getattr(oracle, fn), old, new))
    assert first_failing_pin(pin_module(part), tmp_path) is not None, f"no pin notices: {mistake}"


@pytest.mark.parametrize("mistake", sorted(WRAPS))
def test_a_mistake_in_the_c_part_fails_a_pin(mistake, monkeypatch, tmp_path):
    part, fn, make, change = WRAPS[mistake]
    monkeypatch.setattr(oracle, fn, make(change))
    assert first_failing_pin(pin_module(part), tmp_path) is not None, f"no pin notices: {mistake}"
