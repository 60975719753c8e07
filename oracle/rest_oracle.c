/*
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, single-threaded CPU statement of what
 * the integer half of REST's draft-and-verify step computes, written from the
 * paper (arXiv 2311.08252).  Nothing in the product path may call into this
 * file; it shares no code with the GPU library.
 *
 * Every function works on host memory.  Tokens are non-negative integers stored
 * as int32 (token_bytes == 4) or uint16 (token_bytes == 2).
 *
 * Readings taken where the paper is silent (each repeated at its use):
 *  - the datastore is one flat token stream; the context c_i of position i is
 *    the stream up to i and its continuation t_i the tokens after it
 *    ("Datastore construction");
 *  - suffixes are ordered lexicographically with the end of the stream smaller
 *    than every token, which makes the suffix array unique;
 *  - Algorithm 1 stops at a smallest suffix length n_min instead of running
 *    down to the empty suffix;
 *  - of a large candidate set only the first K in suffix-array order are kept;
 *  - ties among equal Trie weights are broken by (depth ascending, prefix
 *    lexicographic ascending) so the kept set is closed under taking parents.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    const void *base;
    int tb;
    uint64_t n;
} corpus_t;

static inline int64_t tok_at(const corpus_t *c, uint64_t i)
{
    return c->tb == 2 ? (int64_t)((const uint16_t *)c->base)[i]
                      : (int64_t)((const int32_t *)c->base)[i];
}

/* Lexicographic order of two suffixes of the stream; a suffix that runs off the
 * end of the stream first is the smaller one. */
static int suffix_cmp(const corpus_t *c, uint64_t a, uint64_t b)
{
    if (a == b) return 0;
    while (a < c->n && b < c->n) {
        int64_t x = tok_at(c, a), y = tok_at(c, b);
        if (x != y) return x < y ? -1 : 1;
        a++;
        b++;
    }
    return a == c->n ? -1 : 1;
}

/* ---------------------------------------------------------------------------
 * Suffix array (the exact-match index the paper uses, "Retrieving from the
 * datastore", citing Manber & Myers): the permutation of 0..N-1 that sorts all
 * suffixes.  Written as the definition: sort positions by suffix_cmp.
 * ------------------------------------------------------------------------- */
static const corpus_t *g_sort_corpus;

static int sa_qsort_cmp(const void *pa, const void *pb)
{
    uint64_t a = (uint64_t)(*(const int64_t *)pa), b = (uint64_t)(*(const int64_t *)pb);
    return suffix_cmp(g_sort_corpus, a, b);
}

int oracle_suffix_array(const void *corpus, uint64_t n, int token_bytes, int64_t *sa_out)
{
    corpus_t c = { corpus, token_bytes, n };
    if (token_bytes != 2 && token_bytes != 4) return -1;
    for (uint64_t i = 0; i < n; i++) sa_out[i] = (int64_t)i;
    g_sort_corpus = &c;
    qsort(sa_out, n, sizeof(int64_t), sa_qsort_cmp);
    return 0;
}

/* Checks a claimed suffix array against the definition: it is a permutation of
 * 0..N-1 and every adjacent pair is strictly increasing in suffix order.
 * Returns -1 if it holds, else the first offending rank i (pair i, i+1, or the
 * rank of a repeated / out-of-range entry).  sa_bytes is 4 (int32) or 8. */
int64_t oracle_check_suffix_array(const void *corpus, uint64_t n, int token_bytes,
                                  const void *sa, int sa_bytes)
{
    corpus_t c = { corpus, token_bytes, n };
    uint8_t *seen = (uint8_t *)calloc(n ? n : 1, 1);
    int64_t bad = -1;
    for (uint64_t i = 0; i < n && bad < 0; i++) {
        int64_t p = sa_bytes == 4 ? (int64_t)((const int32_t *)sa)[i] : ((const int64_t *)sa)[i];
        if (p < 0 || (uint64_t)p >= n || seen[p]) bad = (int64_t)i;
        else seen[p] = 1;
    }
    for (uint64_t i = 0; i + 1 < n && bad < 0; i++) {
        int64_t p = sa_bytes == 4 ? (int64_t)((const int32_t *)sa)[i] : ((const int64_t *)sa)[i];
        int64_t q = sa_bytes == 4 ? (int64_t)((const int32_t *)sa)[i + 1] : ((const int64_t *)sa)[i + 1];
        if (suffix_cmp(&c, (uint64_t)p, (uint64_t)q) >= 0) bad = (int64_t)i;
    }
    free(seen);
    return bad;
}

/* ---------------------------------------------------------------------------
 * Algorithm 1, Retrieve(D, s): the longest suffix q of the context s, of
 * length n from min(n_max, t) down to n_min, that occurs in the stream, and
 * the continuations of all its occurrences.
 *
 * An occurrence at position p means corpus[p .. p+n) == q; its continuation is
 * corpus[p+n .. p+n+m) cut at the end of the stream (possibly empty; it still
 * counts as an occurrence).  match_count is the number of occurrences.  Of
 * them, the K smallest in suffix order (order of corpus[p ..]) are kept, and
 * are reported in that order: row_pos[r] = p, rows[r*m ..] = continuation,
 * row_len[r] = its length.
 *
 * Two ways of finding the occurrences are provided; both are the definition:
 *  mode 0: for each n, scan every position and compare n tokens (the loop of
 *          Algorithm 1 taken literally);
 *  mode 1: one scan that, for every end position e, measures how many tokens
 *          before e agree with the end of s (capped at n_max); the longest
 *          matching suffix is the largest such length >= n_min, and its
 *          occurrences are the positions reaching it.  Needed for streams of
 *          10^9 tokens where 15 scans per context are too slow.
 * ------------------------------------------------------------------------- */
typedef struct {
    int64_t *pos;
    int64_t size, cap;
} keep_t;

/* keep the `cap` smallest suffixes seen so far, sorted ascending */
static void keep_offer(keep_t *k, const corpus_t *c, int64_t p)
{
    if (k->cap == 0) return;
    if (k->size == k->cap && suffix_cmp(c, (uint64_t)p, (uint64_t)k->pos[k->size - 1]) > 0) return;
    int64_t lo = 0, hi = k->size;
    while (lo < hi) {
        int64_t mid = (lo + hi) / 2;
        if (suffix_cmp(c, (uint64_t)k->pos[mid], (uint64_t)p) < 0) lo = mid + 1;
        else hi = mid;
    }
    int64_t last = k->size < k->cap ? k->size : k->cap - 1;
    memmove(&k->pos[lo + 1], &k->pos[lo], (size_t)(last - lo) * sizeof(int64_t));
    k->pos[lo] = p;
    if (k->size < k->cap) k->size++;
}

static int occurs_at(const corpus_t *c, uint64_t p, const int32_t *q, int n)
{
    if (p + (uint64_t)n > c->n) return 0;
    for (int j = 0; j < n; j++)
        if (tok_at(c, p + j) != (int64_t)q[j]) return 0;
    return 1;
}

int oracle_retrieve(const void *corpus, uint64_t n_tokens, int token_bytes,
                    const int32_t *s, int32_t t,
                    int32_t n_max, int32_t n_min, int64_t K, int32_t m, int32_t mode,
                    int32_t *matched_len, int64_t *match_count, int64_t *n_rows,
                    int64_t *row_pos, int32_t *rows, int32_t *row_len)
{
    corpus_t c = { corpus, token_bytes, n_tokens };
    if (token_bytes != 2 && token_bytes != 4) return -1;
    if (n_min < 1 || n_max < n_min || K < 0 || m < 0 || t < 0) return -1;
    *matched_len = 0;
    *match_count = 0;
    *n_rows = 0;
    keep_t keep = { (int64_t *)malloc((size_t)(K + 1) * sizeof(int64_t)), 0, K };
    int n_start = t < n_max ? t : n_max;
    int found_n = 0;
    int64_t count = 0;

    if (mode == 0) {
        for (int n = n_start; n >= n_min && !found_n; n--) {
            const int32_t *q = s + (t - n);
            count = 0;
            keep.size = 0;
            for (uint64_t p = 0; p + (uint64_t)n <= n_tokens; p++) {
                if (occurs_at(&c, p, q, n)) {
                    count++;
                    keep_offer(&keep, &c, (int64_t)p);
                }
            }
            if (count > 0) found_n = n;
        }
    } else {
        /* agree(e) = number of tokens ending at stream index e-1 that equal the
         * tokens ending at s[t-1], capped at n_start */
        int64_t hist[64];
        memset(hist, 0, sizeof hist);
        if (n_start > 63) { free(keep.pos); return -1; }
        for (uint64_t e = 1; e <= n_tokens; e++) {
            int a = 0;
            while (a < n_start && (uint64_t)a < e && tok_at(&c, e - 1 - a) == (int64_t)s[t - 1 - a]) a++;
            hist[a]++;
        }
        for (int n = n_start; n >= n_min && !found_n; n--) {
            int64_t tot = 0;
            for (int a = n; a <= n_start; a++) tot += hist[a];
            if (tot > 0) { found_n = n; count = tot; }
        }
        if (found_n) {
            for (uint64_t e = (uint64_t)found_n; e <= n_tokens; e++) {
                int a = 0;
                while (a < found_n && tok_at(&c, e - 1 - a) == (int64_t)s[t - 1 - a]) a++;
                if (a == found_n) keep_offer(&keep, &c, (int64_t)(e - found_n));
            }
        }
    }

    if (found_n) {
        *matched_len = found_n;
        *match_count = count;
        *n_rows = keep.size;
        for (int64_t r = 0; r < keep.size; r++) {
            uint64_t start = (uint64_t)keep.pos[r] + (uint64_t)found_n;
            int len = 0;
            while (len < m && start + (uint64_t)len < n_tokens) {
                rows[r * m + len] = (int32_t)tok_at(&c, start + len);
                len++;
            }
            for (int j = len; j < m; j++) rows[r * m + j] = -1;
            row_len[r] = len;
            row_pos[r] = keep.pos[r];
        }
    }
    free(keep.pos);
    return 0;
}

/* ---------------------------------------------------------------------------
 * Algorithm 2, draft selection with a Trie, followed by the breadth-first
 * pseudo sequence and its attention mask ("Draft verification").
 *
 * Every non-empty prefix of every candidate is inserted into a pointer Trie;
 * a node's weight is the number of candidates having that prefix.  Candidates
 * are inserted in the order given by `order` (the caller passes stream
 * position order, not sorted order, so nothing here relies on sortedness).
 * The c heaviest nodes are kept -- the text's "top c nodes with the highest
 * weights"; the listing's heap pops the smallest until c remain, the same
 * set -- with ties resolved by (depth ascending, prefix lexicographic
 * ascending).  Kept nodes are laid out breadth first: by depth, then by prefix
 * lexicographic order (siblings by ascending token).
 *
 * Outputs (arrays of length c, padded past n_nodes with token -1, parent -1,
 * pos 0, weight 0, empty mask row):
 *   draft_tokens, parent_idx (-1: child of the context's last token),
 *   pos_ids (depth, 1-based), node_weight,
 *   tree_mask [c][mask_words] uint64: bit j of row i set iff j == i or node j
 *   is an ancestor of node i (a token sees exactly its own draft sequence).
 * total_trie_nodes (optional) receives the size of the whole Trie.
 * ------------------------------------------------------------------------- */
typedef struct {
    int32_t token, parent, weight, depth, first_child, next_sibling;
} tnode_t;

static tnode_t *g_nodes;

static int path_of(const tnode_t *nodes, int32_t v, int32_t *out)
{
    int d = nodes[v].depth;
    for (int k = d - 1; k >= 0; k--) {
        out[k] = nodes[v].token;
        v = nodes[v].parent;
    }
    return d;
}

static int prefix_lex_cmp(int32_t a, int32_t b)
{
    int32_t pa[256], pb[256];
    int da = path_of(g_nodes, a, pa), db = path_of(g_nodes, b, pb);
    int d = da < db ? da : db;
    for (int k = 0; k < d; k++)
        if (pa[k] != pb[k]) return pa[k] < pb[k] ? -1 : 1;
    return (da > db) - (da < db);
}

static int by_weight_cmp(const void *x, const void *y)
{
    int32_t a = *(const int32_t *)x, b = *(const int32_t *)y;
    if (g_nodes[a].weight != g_nodes[b].weight) return g_nodes[a].weight > g_nodes[b].weight ? -1 : 1;
    if (g_nodes[a].depth != g_nodes[b].depth) return g_nodes[a].depth < g_nodes[b].depth ? -1 : 1;
    return prefix_lex_cmp(a, b);
}

static int by_bfs_cmp(const void *x, const void *y)
{
    int32_t a = *(const int32_t *)x, b = *(const int32_t *)y;
    if (g_nodes[a].depth != g_nodes[b].depth) return g_nodes[a].depth < g_nodes[b].depth ? -1 : 1;
    return prefix_lex_cmp(a, b);
}

int oracle_select_drafts(const int32_t *rows, const int32_t *row_len, const int64_t *order,
                         int64_t n_rows, int32_t m, int32_t c, int32_t mask_words,
                         int32_t *n_nodes, int32_t *draft_tokens, int32_t *parent_idx,
                         int32_t *pos_ids, int32_t *node_weight, uint64_t *tree_mask,
                         int64_t *total_trie_nodes)
{
    if (m > 255 || c < 0 || mask_words * 64 < c) return -1;
    int64_t cap = n_rows * (int64_t)m + 1;
    tnode_t *nodes = (tnode_t *)malloc((size_t)cap * sizeof(tnode_t));
    int64_t n_alloc = 1;
    nodes[0] = (tnode_t){ -1, -1, 0, 0, -1, -1 };  /* root: the empty prefix */
    for (int64_t k = 0; k < n_rows; k++) {
        int64_t r = order ? order[k] : k;
        int32_t cur = 0;
        nodes[0].weight++;
        for (int d = 0; d < row_len[r]; d++) {
            int32_t tkn = rows[r * m + d];
            int32_t ch = nodes[cur].first_child;
            while (ch != -1 && nodes[ch].token != tkn) ch = nodes[ch].next_sibling;
            if (ch == -1) {
                ch = (int32_t)n_alloc++;
                nodes[ch] = (tnode_t){ tkn, cur, 0, nodes[cur].depth + 1, -1, nodes[cur].first_child };
                nodes[cur].first_child = ch;
            }
            nodes[ch].weight++;
            cur = ch;
        }
    }
    int64_t n_trie = n_alloc - 1;
    if (total_trie_nodes) *total_trie_nodes = n_trie;

    int32_t *ids = (int32_t *)malloc((size_t)(n_trie + 1) * sizeof(int32_t));
    for (int64_t i = 0; i < n_trie; i++) ids[i] = (int32_t)(i + 1);
    g_nodes = nodes;
    qsort(ids, (size_t)n_trie, sizeof(int32_t), by_weight_cmp);
    int32_t T = (int32_t)(n_trie < c ? n_trie : c);
    qsort(ids, (size_t)T, sizeof(int32_t), by_bfs_cmp);

    int32_t *out_index = (int32_t *)malloc((size_t)n_alloc * sizeof(int32_t));
    for (int64_t i = 0; i < n_alloc; i++) out_index[i] = -1;
    for (int32_t i = 0; i < T; i++) out_index[ids[i]] = i;

    memset(tree_mask, 0, (size_t)c * (size_t)mask_words * sizeof(uint64_t));
    for (int32_t i = 0; i < c; i++) {
        if (i < T) {
            const tnode_t *nd = &nodes[ids[i]];
            draft_tokens[i] = nd->token;
            parent_idx[i] = nd->parent == 0 ? -1 : out_index[nd->parent];
            pos_ids[i] = nd->depth;
            node_weight[i] = nd->weight;
            int32_t v = ids[i];
            while (v != 0) {
                int32_t j = out_index[v];
                if (j < 0) { free(nodes); free(ids); free(out_index); return -2; }
                tree_mask[(size_t)i * mask_words + j / 64] |= (uint64_t)1 << (j % 64);
                v = nodes[v].parent;
            }
        } else {
            draft_tokens[i] = -1;
            parent_idx[i] = -1;
            pos_ids[i] = 0;
            node_weight[i] = 0;
        }
    }
    *n_nodes = T;
    free(nodes);
    free(ids);
    free(out_index);
    return 0;
}

/* ---------------------------------------------------------------------------
 * Draft acceptance ("Draft acceptance of REST"): starting at the context's
 * last token, follow the draft tree while the model's own token at the
 * current position equals the token of one of its children; everything after
 * the first disagreement is rejected.  ids[0] is the model's token after the
 * context, ids[1+i] its token after draft node i.  Returns the number of
 * accepted draft tokens, their node indices (path, padded with -1 to m) and
 * the model's token at the last accepted position (the next real token).
 * ------------------------------------------------------------------------- */
int oracle_accept(const int32_t *ids, const int32_t *draft_tokens, const int32_t *parent_idx,
                  int32_t n_nodes, int32_t m,
                  int32_t *accept_len, int32_t *accept_path, int32_t *next_token)
{
    int32_t cur = -1, len = 0;
    for (int j = 0; j < m; j++) accept_path[j] = -1;
    for (;;) {
        int32_t want = ids[cur + 1], hit = -1;
        for (int32_t i = 0; i < n_nodes; i++)
            if (parent_idx[i] == cur && draft_tokens[i] == want) { hit = i; break; }
        if (hit < 0 || len >= m) break;
        accept_path[len++] = hit;
        cur = hit;
    }
    *accept_len = len;
    *next_token = ids[cur + 1];
    return 0;
}
