/* One draft-and-verify step driven from plain C99 through the library's C ABI: no Python, no torch in the process.
 * The GPU test writes a seeded problem to a file, runs this program and compares what it wrote back with the CPU oracle.
 *
 *   c_abi_driver <in> <out>
 *
 * <in>:  int64 header {n_tokens, B, ctx_stride, K, m, c, path_cap, H, P, depth}, then
 *        int32 corpus[n_tokens], int32 contexts[B*ctx_stride], int32 ctx_len[B], int32 ids[B*(1+c)],
 *        float q[B*H*c*128], float k[B*H*(P+c)*128], float v[B*H*(P+c)*128]
 * <out>: int32 draft_tokens[B*c], parent_idx[B*c], pos_ids[B*c], node_weight[B*c], uint64 tree_mask[B*c*words],
 *        int32 n_nodes[B], matched_len[B], int64 match_count[B], int32 accept_len[B], accept_path[B*path_cap],
 *        next_token[B], float out[B*H*c*128]
 * depth = 0 builds the full index, otherwise the index ordered by `depth` tokens.
 * The mask rest_tree_attention reads is the one rest_retrieve wrote: it never leaves the device.
 * Exit status: 0, or 1 with a message on stderr. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <hip/hip_runtime_api.h>

#include "rest.h"

#define CHECK_HIP(call)                                                                         \
    do {                                                                                        \
        hipError_t e_ = (call);                                                                 \
        if (e_ != hipSuccess) {                                                                 \
            fprintf(stderr, "%s:%d: %s: %s\n", __FILE__, __LINE__, #call, hipGetErrorString(e_)); \
            return 1;                                                                           \
        }                                                                                       \
    } while (0)
#define CHECK_REST(call)                                                              \
    do {                                                                              \
        rest_status s_ = (call);                                                      \
        if (s_ != 0) {                                                                \
            fprintf(stderr, "%s:%d: %s: status %d\n", __FILE__, __LINE__, #call, (int)s_); \
            return 1;                                                                 \
        }                                                                             \
    } while (0)

static void* read_block(FILE* f, size_t bytes) {
    void* p = malloc(bytes ? bytes : 1);
    if (!p || fread(p, 1, bytes, f) != bytes) {
        fprintf(stderr, "short read (%zu bytes wanted)\n", bytes);
        exit(1);
    }
    return p;
}

static int to_device(void** d, const void* h, size_t bytes) {
    CHECK_HIP(hipMalloc(d, bytes ? bytes : 1));
    CHECK_HIP(hipMemcpy(*d, h, bytes, hipMemcpyHostToDevice));
    return 0;
}

static int write_back(FILE* f, const void* d, size_t bytes) {
    void* h = malloc(bytes ? bytes : 1);
    if (!h) return 1;
    CHECK_HIP(hipMemcpy(h, d, bytes, hipMemcpyDeviceToHost));
    const int bad = fwrite(h, 1, bytes, f) != bytes;
    free(h);
    return bad;
}

int main(int argc, char** argv) {
    if (argc != 3) {
        fprintf(stderr, "usage: %s <in> <out>\n", argv[0]);
        return 1;
    }
    FILE* in = fopen(argv[1], "rb");
    if (!in) { perror(argv[1]); return 1; }
    int64_t* hdr = (int64_t*)read_block(in, 10 * sizeof(int64_t));
    const uint64_t n = (uint64_t)hdr[0];
    const int32_t B = (int32_t)hdr[1], stride = (int32_t)hdr[2], K = (int32_t)hdr[3], m = (int32_t)hdr[4];
    const int32_t c = (int32_t)hdr[5], cap = (int32_t)hdr[6], H = (int32_t)hdr[7], P = (int32_t)hdr[8];
    const int32_t depth = (int32_t)hdr[9];
    const int32_t words = (c + 63) / 64, D = 128;
    const size_t q_elems = (size_t)B * H * c * D, kv_elems = (size_t)B * H * (P + c) * D;

    int32_t* corpus = (int32_t*)read_block(in, n * 4);
    int32_t* ctx = (int32_t*)read_block(in, (size_t)B * stride * 4);
    int32_t* len = (int32_t*)read_block(in, (size_t)B * 4);
    int32_t* ids = (int32_t*)read_block(in, (size_t)B * (1 + c) * 4);
    float* q = (float*)read_block(in, q_elems * 4);
    float* k = (float*)read_block(in, kv_elems * 4);
    float* v = (float*)read_block(in, kv_elems * 4);
    fclose(in);

    void *d_corpus, *d_ctx, *d_len, *d_ids, *d_q, *d_k, *d_v;
    if (to_device(&d_corpus, corpus, n * 4) || to_device(&d_ctx, ctx, (size_t)B * stride * 4) ||
        to_device(&d_len, len, (size_t)B * 4) || to_device(&d_ids, ids, (size_t)B * (1 + c) * 4) ||
        to_device(&d_q, q, q_elems * 4) || to_device(&d_k, k, kv_elems * 4) || to_device(&d_v, v, kv_elems * 4))
        return 1;

    hipStream_t stream;
    CHECK_HIP(hipStreamCreate(&stream));

    /* the datastore index, once */
    rest_index* index = NULL;
    if (depth > 0)
        CHECK_REST(rest_build_index_prefix(d_corpus, n, 4, 4, depth, stream, &index));
    else
        CHECK_REST(rest_build_index(d_corpus, n, 4, 4, stream, &index));
    if (rest_index_sort_depth(index) != depth) {
        fprintf(stderr, "sort depth %d, wanted %d\n", (int)rest_index_sort_depth(index), (int)depth);
        return 1;
    }

    /* retrieval and the draft tree */
    rest_retrieve_params prm;
    memset(&prm, 0, sizeof prm);
    prm.n_max = 16;
    prm.n_min = 2;
    prm.max_matches = K;
    prm.cont_len = m;
    prm.max_nodes = c;
    rest_tree tree;
    const size_t bc = (size_t)B * c;
    CHECK_HIP(hipMalloc((void**)&tree.draft_tokens, bc * 4));
    CHECK_HIP(hipMalloc((void**)&tree.parent_idx, bc * 4));
    CHECK_HIP(hipMalloc((void**)&tree.pos_ids, bc * 4));
    CHECK_HIP(hipMalloc((void**)&tree.node_weight, bc * 4));
    CHECK_HIP(hipMalloc((void**)&tree.tree_mask, bc * words * 8));
    CHECK_HIP(hipMalloc((void**)&tree.n_nodes, (size_t)B * 4));
    CHECK_HIP(hipMalloc((void**)&tree.matched_len, (size_t)B * 4));
    CHECK_HIP(hipMalloc((void**)&tree.match_count, (size_t)B * 8));
    const size_t ws_r = rest_retrieve_workspace_bytes(B, &prm);
    void* d_ws_r = NULL;
    CHECK_HIP(hipMalloc(&d_ws_r, ws_r ? ws_r : 1));
    CHECK_REST(rest_retrieve(index, (const int32_t*)d_ctx, (const int32_t*)d_len, B, stride, &prm, &tree, d_ws_r, ws_r, stream));

    /* verification attention of one layer: context b is batch entry b, with the mask retrieval just wrote */
    rest_attn_desc ad;
    memset(&ad, 0, sizeof ad);
    ad.Nb = B; ad.H = H; ad.Tq = c; ad.Tk = c; ad.P = P; ad.D = D;
    ad.dtype = REST_FP32;
    ad.scale = 0.08838834764831845f;     /* 1 / sqrt(128) */
    ad.q_stride[0] = (int64_t)H * c * D;       ad.q_stride[1] = (int64_t)c * D;       ad.q_stride[2] = D;
    ad.k_stride[0] = (int64_t)H * (P + c) * D; ad.k_stride[1] = (int64_t)(P + c) * D; ad.k_stride[2] = D;
    memcpy(ad.v_stride, ad.k_stride, sizeof ad.k_stride);
    memcpy(ad.o_stride, ad.q_stride, sizeof ad.q_stride);
    ad.mask_per_batch = 1;
    const size_t ws_a = rest_tree_attention_workspace_bytes(&ad);
    void *d_ws_a = NULL, *d_out = NULL;
    CHECK_HIP(hipMalloc(&d_ws_a, ws_a ? ws_a : 1));
    CHECK_HIP(hipMalloc(&d_out, q_elems * 4));
    CHECK_REST(rest_tree_attention(d_q, d_k, d_v, tree.tree_mask, d_out, &ad, d_ws_a, ws_a, stream));

    /* acceptance against the model's tokens */
    int32_t *d_alen, *d_apath, *d_next;
    CHECK_HIP(hipMalloc((void**)&d_alen, (size_t)B * 4));
    CHECK_HIP(hipMalloc((void**)&d_apath, (size_t)B * cap * 4));
    CHECK_HIP(hipMalloc((void**)&d_next, (size_t)B * 4));
    CHECK_REST(rest_accept((const int32_t*)d_ids, &tree, B, c, cap, d_alen, d_apath, d_next, stream));
    CHECK_HIP(hipStreamSynchronize(stream));

    FILE* out = fopen(argv[2], "wb");
    if (!out) { perror(argv[2]); return 1; }
    if (write_back(out, tree.draft_tokens, bc * 4) || write_back(out, tree.parent_idx, bc * 4) ||
        write_back(out, tree.pos_ids, bc * 4) || write_back(out, tree.node_weight, bc * 4) ||
        write_back(out, tree.tree_mask, bc * words * 8) || write_back(out, tree.n_nodes, (size_t)B * 4) ||
        write_back(out, tree.matched_len, (size_t)B * 4) || write_back(out, tree.match_count, (size_t)B * 8) ||
        write_back(out, d_alen, (size_t)B * 4) || write_back(out, d_apath, (size_t)B * cap * 4) ||
        write_back(out, d_next, (size_t)B * 4) || write_back(out, d_out, q_elems * 4)) {
        fprintf(stderr, "writing %s failed\n", argv[2]);
        return 1;
    }
    if (fclose(out) != 0) { perror(argv[2]); return 1; }

    rest_index_destroy(index);
    CHECK_HIP(hipStreamDestroy(stream));
    return 0;
}
