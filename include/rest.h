/*
 * rest.h -- C ABI of the MI355X (gfx950) implementation of REST's per-step
 * draft-and-verify hot path (Retrieval-Based Speculative Decoding,
 * arXiv 2311.08252).
 *
 * The four main calls follow the paper's problem statement:
 *   rest_build_index   "Datastore construction" + the suffix array used for
 *                      exact match ("Retrieving from the datastore")
 *   rest_retrieve      Algorithm 1 (longest matching suffix, its continuations)
 *                      + Algorithm 2 (Trie weights, top-c nodes)
 *                      + the breadth-first pseudo sequence and tree attention
 *                      mask of "Draft verification"
 *   rest_tree_attention  the attention of the verification forward pass under
 *                      that mask ("Draft verification")
 *   rest_accept        "Draft acceptance": accept draft tokens from the start
 *                      while they equal the model's own tokens
 * rest_sample_ids draws the model's token per position for nucleus sampling
 * ("Sampling strategies"); rest_rope_append and rest_kv_compact are the cache
 * steps before and after verification that "Draft acceptance" implies.
 * rest_index_save / rest_index_load keep the index as a file and
 * rest_build_index_prefix builds one ordered by a bounded number of tokens.
 *
 * Conventions
 *  - Every pointer whose name starts with d_ (and every pointer inside
 *    rest_tree) is DEVICE memory owned by the caller; the library never frees
 *    or reallocates it.  Pointers to parameter structs are HOST memory and are
 *    read before the call returns.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    rest_retrieve, rest_tree_attention, rest_accept, rest_sample_ids,
 *    rest_rope_append and rest_kv_compact only enqueue work on it and never
 *    synchronise; rest_build_index allocates scratch memory and
 *    may synchronise.
 *  - All calls return a rest_status; no call aborts, throws or prints.  On an
 *    error nothing has been enqueued and output buffers are untouched.
 *  - The library keeps no state between calls apart from the rest_index
 *    handles: calls may come from several host threads and on several streams at
 *    once as long as they share no output buffer and no workspace; any number
 *    of rest_retrieve calls may read one index concurrently.
 *  - Tokens are non-negative.  A corpus stores them as int32 (token_bytes 4)
 *    or uint16 (token_bytes 2); contexts and draft tokens are always int32.
 */
#ifndef REST_H
#define REST_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t rest_status;
enum {
    REST_OK = 0,
    REST_INVALID_ARG = -1,        /* null pointer, size out of range, bad enum */
    REST_UNSUPPORTED = -2,        /* legal request this build has no kernel for */
    REST_WORKSPACE_TOO_SMALL = -3,
    REST_OUT_OF_MEMORY = -4,      /* hipMalloc failed (index build / handle creation only) */
    REST_HIP_ERROR = -5,          /* a HIP runtime call or kernel launch failed */
    REST_IO_ERROR = -6,           /* a file could not be opened, read or written in full */
    REST_BAD_FILE = -7,           /* not an index file, or not the index of this token stream */
    REST_BOUNDS_VIOLATION = -8    /* bounds-checked build of the library only: a kernel formed an index outside its
                                     array (the access was redirected inside it); the call's results mean nothing */
};

/* Compile-time limits of the retrieval kernels (rest_retrieve rejects larger values). */
#define REST_MAX_SUFFIX_LEN 16      /* n_max <= 16: the paper's setting, "Hyperparameters" */
#define REST_MAX_CONT_LEN 32        /* m */
#define REST_MAX_MATCHES 8192       /* K */
#define REST_MAX_NODES 256          /* c */
#define REST_MAX_QUERY_ROWS 1024    /* query rows of one rest_tree_attention slab (grouped heads stacked) */

const char* rest_status_string(rest_status s);
/* Library version string, e.g. "rest-gfx950 0.2"; the bounds-checked build says so here. */
const char* rest_version(void);

/* ------------------------------------------------------------------------
 * Index: the token stream plus its suffix array, both resident in HBM.
 *
 * The datastore of the paper, D = {(c_i, t_i)}, holds for every position i of
 * a corpus the context ending there and the continuation that follows
 * ("Datastore construction").  It is represented by the flat token stream; a
 * suffix array over it answers "which contexts end with q" exactly
 * ("Retrieving from the datastore").  Suffix order: lexicographic by token
 * value, the end of the stream smaller than every token (this makes the
 * array unique).
 * ---------------------------------------------------------------------- */
typedef struct rest_index rest_index;

/* Builds the suffix array of d_corpus[0 .. n_tokens) on the GPU (prefix
 * doubling with radix sorts) and returns a handle that owns the suffix array
 * and a small search table, and BORROWS d_corpus (it must stay valid and
 * unchanged until rest_index_destroy).
 *   token_bytes 2|4; sa_bytes 4 (int32 entries, needs n_tokens < 2^31) or 8.
 *   n_tokens must be in [1, 2^32 - 2].
 * Synchronises `stream` before returning. */
rest_status rest_build_index(const void* d_corpus, uint64_t n_tokens, int32_t token_bytes,
                             int32_t sa_bytes, void* stream, rest_index** out);

/* The same with a depth limit: positions are ordered by their first `depth`
 * tokens only (depth is rounded up to a power of two >= 2; 0 = no limit), and
 * positions whose prefixes of that length are equal stay in ascending position
 * order.  Algorithm 1 reads at most n_max tokens of a suffix and Algorithm 2
 * the cont_len after them, so every call of rest_retrieve with
 * n_max + cont_len <= depth returns what it returns on the full suffix array
 * (others are refused with REST_UNSUPPORTED), while streams with long repeats
 * (duplicated documents) need far fewer doubling rounds.  If the rounds leave
 * no two equal prefixes the result is the suffix array and is marked so. */
rest_status rest_build_index_prefix(const void* d_corpus, uint64_t n_tokens, int32_t token_bytes,
                                    int32_t sa_bytes, int32_t depth, void* stream, rest_index** out);

/* Number of tokens the handle's array is ordered by; 0 = a full suffix array;
 * -1 for a NULL handle. */
int32_t rest_index_sort_depth(const rest_index* index);

/* Wraps a caller-supplied suffix array (e.g. one built elsewhere or loaded
 * from disk); both arrays are borrowed.  The array is trusted, not checked.
 * Only the small search table is computed (synchronises `stream`).
 * Here d_corpus and d_sa may also be host memory that the device addresses
 * directly (hipHostMalloc): a datastore larger than the GPU's memory stays on
 * the host and rest_retrieve reads it over the host link (a few hundred small
 * reads per context; same results, about twice the latency of one context). */
rest_status rest_index_from_sa(const void* d_corpus, const void* d_sa, uint64_t n_tokens,
                               int32_t token_bytes, int32_t sa_bytes, void* stream, rest_index** out);

/* Read-only view of what the handle holds (any out pointer may be NULL). */
rest_status rest_index_view(const rest_index* index, const void** d_corpus, const void** d_sa,
                            uint64_t* n_tokens, int32_t* token_bytes, int32_t* sa_bytes);

/* Datastore persistence ("Datastore construction": the index is built once and
 * reused).  rest_index_save writes the suffix array behind a 64-byte header
 * ("RESTSA01", n_tokens u64, token_bytes i32, sa_bytes i32, a 64-bit
 * fingerprint of the token stream, the sort depth i32, zero padding; little endian) to the host
 * file `path`.  rest_index_load reads such a file for the stream at d_corpus
 * (borrowed, as in rest_build_index): length, token width and fingerprint
 * must agree with the file's, else REST_BAD_FILE; the handle owns the array.
 * Both synchronise `stream`. */
rest_status rest_index_save(const rest_index* index, const char* path, void* stream);
rest_status rest_index_load(const char* path, const void* d_corpus, uint64_t n_tokens, int32_t token_bytes,
                            void* stream, rest_index** out);

/* Frees what the handle owns.  NULL is allowed. */
void rest_index_destroy(rest_index* index);

/* ------------------------------------------------------------------------
 * rest_retrieve: contexts -> draft trees.
 *
 * For each of the B contexts s = d_contexts[b*ctx_stride .. + d_ctx_len[b]):
 *  1. Algorithm 1: for n = min(n_max, len) down to n_min, q = last n tokens
 *     of s; the first n for which q occurs in the stream is matched_len and
 *     match_count its number of occurrences (0 / 0 if none, or if len < n_min).
 *     The paper's loop has no lower bound; n_min >= 1 supplies one.
 *  2. Of the occurrences, the first max_matches in suffix-array order are kept
 *     (the paper gives no rule for a large match set; see `strided` below for
 *     the other rule offered); the candidate of an occurrence is the cont_len
 *     tokens following it, cut at the end of the stream ("Hyperparameters": m).
 *  3. Algorithm 2: the Trie of all non-empty candidate prefixes, node weight =
 *     number of candidates with that prefix; the max_nodes heaviest nodes are
 *     kept, ties broken by (depth ascending, prefix lexicographically
 *     ascending), which keeps the set closed under taking parents.
 *  4. "Draft verification": the kept nodes in breadth-first order (depth, then
 *     prefix order, i.e. siblings by ascending token) form the pseudo
 *     sequence; tree_mask row i has bit j set iff j == i or node j is an
 *     ancestor of node i.
 *
 * Outputs, row stride max_nodes per context; slots i >= n_nodes hold
 * draft_tokens -1, parent_idx -1, pos_ids 0, node_weight 0, mask row 0.
 * ---------------------------------------------------------------------- */
typedef struct {
    int32_t n_max;        /* longest suffix tried, 1..REST_MAX_SUFFIX_LEN (paper: 16) */
    int32_t n_min;        /* shortest suffix tried, 1..n_max */
    int32_t max_matches;  /* K, 1..REST_MAX_MATCHES */
    int32_t cont_len;     /* m, 1..REST_MAX_CONT_LEN (paper: 10) */
    int32_t max_nodes;    /* c, 1..REST_MAX_NODES (paper: 64) */
    /* The draft strategy the paper compares the Trie with ("Effect of draft token selecting
     * strategies": at most eight randomly sampled candidates, each cut to eight tokens).
     * random_seqs == 0: the Trie over all kept candidates (steps 2-3 above).  random_seqs in
     * 1..64: step 3 runs on random_seqs candidates drawn from the kept ones instead (cont_len is the
     * cut).  Draw j of context b is candidate floor(U_j * R / 2^64), R = number of kept candidates,
     * U_j = mix(mix(seed + G*(1 + b)) + G*(1 + j)), G = 0x9E3779B97F4A7C15, mix = the splitmix64
     * finaliser; equal draws collapse. */
    int32_t random_seqs;
    uint64_t seed;
    /* 0: keep the first max_matches occurrences in suffix-array order.  1: of S > max_matches
     * occurrences keep an evenly spaced sample of the sorted range, number i (0-based) of the K kept
     * being occurrence floor(i*S/K), so that node weights estimate the frequencies over all
     * occurrences and not over the lexicographically smallest ones.  No difference when S <= K. */
    int32_t strided;
    int32_t reserved_;    /* set to 0 */
} rest_retrieve_params;

typedef struct {
    int32_t* draft_tokens;   /* [B, c] token of node i */
    int32_t* parent_idx;     /* [B, c] index of the parent node, -1 = the context's last token */
    int32_t* pos_ids;        /* [B, c] depth of node i, 1-based (position offset after the context) */
    int32_t* node_weight;    /* [B, c] Trie weight of node i */
    uint64_t* tree_mask;     /* [B, c, ceil(c/64)] ancestor-or-self bit rows */
    int32_t* n_nodes;        /* [B] */
    int32_t* matched_len;    /* [B] */
    int64_t* match_count;    /* [B] */
} rest_tree;

/* Bytes of device workspace rest_retrieve needs for B contexts (0 on bad params). */
size_t rest_retrieve_workspace_bytes(int32_t B, const rest_retrieve_params* params);

rest_status rest_retrieve(const rest_index* index, const int32_t* d_contexts, const int32_t* d_ctx_len,
                          int32_t B, int32_t ctx_stride, const rest_retrieve_params* params,
                          const rest_tree* out, void* d_workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------
 * rest_tree_attention: masked softmax attention of the draft tokens against
 * the KV cache ("Draft verification": each token must see exactly its own
 * draft sequence).
 *
 * For every batch entry nb (a layer or a context) and head h, query row i:
 *   O[i] = sum_j softmax_j(scale * q_i . k_j) v_j over the visible keys j:
 *   keys 0..P-1 (the cached context) are always visible, key P+j (draft token
 *   j) is visible iff bit j of mask row i is set.
 * A row with no visible key (P == 0 and an empty mask row) yields zeros.
 *
 * Layout: q, out [Nb, H, Tq, D]; k, v [Nb, H, P+Tk, D]; D contiguous; the
 * strides (in elements) of the Nb, H and row axes are given per tensor.
 * d_mask: [Tq, ceil(Tk/64)] uint64 when mask_per_batch == 0 (shared by all Nb),
 * else [Nb, Tq, ceil(Tk/64)].  Heads share K/V one-to-one (multi-head attention).
 * Grouped-query attention (g query heads per K/V head) is the same call on a view: H = number
 * of K/V heads, the g query heads of a group stacked along the row axis (Tq = g * T, row
 * h_in_group * T + t; a plain reshape when the query heads are contiguous) and
 * mask_rows = T, so that all g copies of node t use mask row t; each K/V byte is then read once
 * per group.
 * dtype: REST_BF16 (bf16 in/out, fp32 accumulation and softmax, probabilities
 * rounded to bf16 for the second product) or REST_FP32 (fp32 in/out and math).
 * D must be 128.  Tk <= REST_MAX_NODES (Tk may be 0); Tq <= REST_MAX_QUERY_ROWS, so that up to 16
 * grouped query heads of 64 draft tokens fit one call.  Query rows are worked on in groups of at most 256,
 * each of which reads the slab's K and V once.
 *
 * 8-bit cache (an extension; the paper's models keep a 16-bit cache): with
 * kv_dtype = REST_KV_FP8_E4M3 (dtype must be REST_BF16) d_k and d_v hold one
 * byte per element in the OCP 8-bit floating point format E4M3 (1 sign,
 * 4 exponent bits with bias 7, 3 mantissa bits, no infinities), strides in
 * elements = bytes and multiples of 16, and the attention is, by definition,
 * the one above on k = d_k_scale[nb*H + h] * decode(d_k), v = d_v_scale[nb*H + h]
 * * decode(d_v) (device arrays of Nb*H floats; NULL = all ones).  Decoding is
 * exact, so q.k and the result differ from that definition only as the bf16
 * path's do.  A NaN code poisons its row as a NaN in a 16-bit cache would.
 * ---------------------------------------------------------------------- */
enum { REST_BF16 = 0, REST_FP32 = 1 };
enum { REST_KV_AS_DTYPE = 0, REST_KV_FP8_E4M3 = 1 };

typedef struct {
    int32_t Nb, H, Tq, Tk, P, D;
    int32_t dtype;
    float scale;
    int64_t q_stride[3];     /* elements: Nb, H, row */
    int64_t k_stride[3];
    int64_t v_stride[3];
    int64_t o_stride[3];
    int32_t mask_per_batch;
    int32_t num_splits;      /* 0 = let the library choose; else KV splits per (Nb, H) */
    int32_t mask_rows;       /* 0 = Tq; else rows of one mask: query row i uses mask row i % mask_rows */
    int32_t kv_dtype;        /* REST_KV_AS_DTYPE: K, V have `dtype`; REST_KV_FP8_E4M3: one E4M3 byte per element */
    const float* d_k_scale;  /* 8-bit cache: [Nb*H] device floats, NULL = 1 */
    const float* d_v_scale;
} rest_attn_desc;

/* Bytes of device workspace (partial results of the KV splits, 16-byte aligned; it needs no initialisation and its
 * contents after a call mean nothing to the caller). */
size_t rest_tree_attention_workspace_bytes(const rest_attn_desc* desc);

rest_status rest_tree_attention(const void* d_q, const void* d_k, const void* d_v, const uint64_t* d_mask,
                                void* d_out, const rest_attn_desc* desc,
                                void* d_workspace, size_t workspace_bytes, void* stream);

/* rest_tree_attention for callers that cannot allocate device memory or bring a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (minus the workspace), same
 * kernels, same results bit for bit; the partial results of the KV splits go to a device array of
 * REST_STATIC_SCRATCH_BYTES that is part of the library's image on each GPU (held until the process ends).  The
 * call allocates nothing and frees nothing.  A description whose rest_tree_attention_workspace_bytes exceeds
 * REST_STATIC_SCRATCH_BYTES is refused with REST_WORKSPACE_TOO_SMALL (64 MiB covers one layer of 32 heads at any
 * KV length, i.e. single-context decoding; launches with many (batch, head) slabs need no partials at all unless
 * num_splits forces them).  All calls on one GPU share that GPU's array: calls that overlap in time on one GPU
 * (two streams, two host threads) race on it and must be serialised by the caller; calls in stream order on one
 * stream are safe.  The first call on a device asks the runtime for the array's address there (do that call
 * outside a graph capture). */
#define REST_STATIC_SCRATCH_BYTES (64 * 1024 * 1024)
rest_status rest_tree_attention_noalloc(const void* d_q, const void* d_k, const void* d_v, const uint64_t* d_mask,
                                        void* d_out, const rest_attn_desc* desc, void* stream);

/* ------------------------------------------------------------------------
 * rest_accept ("Draft acceptance"): d_ids[b, 0] is the model's token after the
 * context, d_ids[b, 1+i] its token after draft node i (greedy: the argmax).
 * Starting at the context's last token, step to the child whose token equals
 * the model's token at the current position, until none does or path_cap
 * tokens are accepted.  Siblings have distinct tokens, so the walk is unique.
 *   d_accept_len[b]   number of accepted draft tokens
 *   d_accept_path[b, path_cap]  their node indices, -1 padded
 *   d_next_token[b]   the model's token at the last accepted position
 * `tree` rows have stride c (= the max_nodes used by rest_retrieve); d_ids has
 * row stride 1 + c.
 * ---------------------------------------------------------------------- */
rest_status rest_accept(const int32_t* d_ids, const rest_tree* tree, int32_t B, int32_t c, int32_t path_cap,
                        int32_t* d_accept_len, int32_t* d_accept_path, int32_t* d_next_token, void* stream);

/* ------------------------------------------------------------------------
 * rest_sample_ids ("Sampling strategies"): nucleus sampling of the model's token
 * at R positions (the context's last token and every draft node), so that
 * rest_accept can compare sampled tokens, not arg-max tokens, with the drafts.
 * The paper gives temperature and top-p, not the mechanics; this definition
 * fixes the drawn token to the last bit, whatever order an implementation adds in:
 *  - row r, token i weighs w_i = floor(2^36 * E((x_i - x_max) * c)), an integer,
 *    with x = d_logits[r, :], c = log2(e) / temperature formed in fp64 and
 *    E(y) = 2^y evaluated as: n = floor(y), t = (y - n) * ln 2, E = 2^n * P(t),
 *    P = the Taylor polynomial of exp of degree 13 in Horner form, every
 *    multiplication and addition a separate correctly rounded fp64 operation;
 *    tokens below 2^-64 of the largest weigh 0 (so does a logit of -inf);
 *  - tokens are ordered by logit, highest first (+0 = -0), equal logits by
 *    ascending token id;
 *  - the nucleus is the shortest prefix of that order whose mass C_k satisfies
 *    (double)C_k >= (double)top_p * (double)W, W the row's total mass;
 *  - d_ids[r] = the first token of the order whose cumulative mass satisfies
 *    (double)C_j > (double)d_u[r] * (double)M, M the nucleus mass.
 * d_u[r] in [0, 1) is the caller's random number for that position: tie it to
 * the position in the sequence and decoding with drafts emits exactly what
 * one-token-at-a-time sampling emits.  Logits are finite or -inf, at least one
 * finite per row; d_logits [R, row_stride >= V] fp32.  V <= 131072
 * (REST_UNSUPPORTED above: masses are summed exactly in 53 bits); temperature > 0;
 * 0 < top_p <= 1.  d_workspace: rest_sample_ids_workspace_bytes(R, V) bytes of
 * device memory, 8-byte aligned, no initialisation needed (rows of at most
 * 32768 logits are handled without touching it; it is asked for all the same).
 * Rows that start at multiples of 16 bytes (d_logits and row_stride * 4) and
 * hold a multiple of 4 logits are read fastest.
 * ---------------------------------------------------------------------- */
size_t rest_sample_ids_workspace_bytes(int32_t R, int32_t V);
rest_status rest_sample_ids(const float* d_logits, int64_t row_stride, const float* d_u, int32_t R, int32_t V,
                            float temperature, float top_p, int32_t* d_ids, void* d_workspace, size_t workspace_bytes,
                            void* stream);

/* ------------------------------------------------------------------------
 * The steps either side of verification inside one model layer.  The paper
 * implies them ("Draft acceptance": accepted draft tokens become context; the
 * pseudo sequence of "Draft verification" needs positions that reflect each
 * token's place in its own draft) without describing them; the definitions
 * below are this library's reading for models with rotary position embedding
 * and a key/value cache.
 *
 * rest_rope_append, before rest_tree_attention: draft node t (depth
 * d_pos_ids[t], as emitted by rest_retrieve) gets position
 * pos_offset + d_pos_ids[t]; pos_offset is the position of the context's last
 * token (P - 1 when the cache holds the whole context).  Its query and key are
 * rotated by the rotary embedding of that position -- half-split layout: with
 * h = D/2, components (i, i+h) form a plane vector turned by the angle
 * position * theta^(-2i/D) -- in fp32 with angles formed in fp64, and rounded to
 * bf16.  The query is rewritten in place; the rotated key and the value are
 * written to row P + t of the caches.
 *   d_q, d_k_new, d_v_new  [Nb, H, T, D] bf16
 *   d_k_cache, d_v_cache   [Nb, H, >= P + T, D] bf16
 *   d_pos_ids              [T] int32 (per_batch == 0) or [Nb, T]
 *
 * rest_kv_compact, after rest_accept: for i < accept_len, cache row P + i
 * becomes what row P + accept_path[i] was (all reads happen before any write);
 * rows from P + accept_len on are dead afterwards.
 *   d_accept_path  [path_cap] int32 (per_batch == 0) or [Nb, path_cap]
 *   d_accept_len   [1] or [Nb] int32; entries outside [0, T) end the moves
 * path_cap <= REST_MAX_CONT_LEN.
 *
 * D must be 128; strides are in elements for the Nb, H and row axes, D
 * contiguous, rows 16-byte aligned.  Both calls only enqueue work on `stream`.
 *
 * 8-bit cache (cache_dtype = REST_KV_FP8_E4M3, see rest_tree_attention): the
 * caches hold one E4M3 byte per element, strides in bytes and multiples of 16.
 * rest_rope_append then stores, for slab (nb, h), the codes nearest to
 * rotated key / d_k_scale[nb*H + h] and value / d_v_scale[nb*H + h] (ties to
 * the even code, magnitudes beyond 448 saturate; the quotients are formed in
 * fp32); d_q, d_k_new and d_v_new stay bf16.  rest_kv_compact moves bytes.
 * ---------------------------------------------------------------------- */
typedef struct {
    int32_t Nb, H, T, D;
    int32_t P;
    int32_t pos_offset;
    int32_t per_batch;       /* 0: one d_pos_ids / d_accept_path row for all Nb; 1: one per Nb */
    int32_t dtype;           /* REST_BF16 */
    double theta;            /* rotary base, e.g. 10000 */
    int64_t q_stride[3];
    int64_t kn_stride[3];
    int64_t vn_stride[3];
    int64_t kc_stride[3];
    int64_t vc_stride[3];
    int32_t cache_dtype;     /* REST_KV_AS_DTYPE or REST_KV_FP8_E4M3 */
    int32_t reserved_;       /* set to 0 */
    const float* d_k_scale;  /* 8-bit cache: [Nb*H] device floats, NULL = 1 */
    const float* d_v_scale;
} rest_kv_desc;

rest_status rest_rope_append(void* d_q, const void* d_k_new, const void* d_v_new, void* d_k_cache, void* d_v_cache,
                             const int32_t* d_pos_ids, const rest_kv_desc* desc, void* stream);

rest_status rest_kv_compact(void* d_k_cache, void* d_v_cache, const int32_t* d_accept_path,
                            const int32_t* d_accept_len, int32_t path_cap, const rest_kv_desc* desc, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* REST_H */
