// Draft acceptance ("Draft acceptance of REST", arXiv 2311.08252): accept draft tokens from the start of
// the tree while they equal the model's own token at that position; everything after the first
// disagreement is rejected, so the emitted sequence equals ordinary autoregressive decoding.
//
// One wavefront per context.  At each step the 64 lanes scan the nodes for the child of the current node
// whose token equals the model's token; siblings carry distinct tokens, so at most one lane group hits.
#include "common.h"

namespace {

__global__ __launch_bounds__(64) void accept_kernel(const int32_t* ids, const int32_t* draft_tokens,
                                                    const int32_t* parent_idx, const int32_t* n_nodes, int32_t c,
                                                    int32_t path_cap, int32_t* accept_len, int32_t* accept_path,
                                                    int32_t* next_token) {
    const int b = blockIdx.x, lane = threadIdx.x;
    const int32_t* id = ids + (int64_t)b * (1 + c);
    const int32_t* tok = draft_tokens + (int64_t)b * c;
    const int32_t* par = parent_idx + (int64_t)b * c;
    int n = n_nodes[b];
    n = n < 0 ? 0 : (n > c ? c : n);
    int cur = -1, len = 0;
    while (len < path_cap) {
        const int want = id[cur + 1];
        int hit = 0x7fffffff;
        for (int i = lane; i < n; i += 64)
            if (par[i] == cur && tok[i] == want) hit = min(hit, i);
        for (int off = 32; off > 0; off >>= 1) hit = min(hit, __shfl_xor(hit, off, 64));
        if (hit == 0x7fffffff) break;
        if (lane == 0) accept_path[(int64_t)b * path_cap + len] = hit;
        cur = hit;
        len++;
    }
    for (int i = len + lane; i < path_cap; i += 64) accept_path[(int64_t)b * path_cap + i] = -1;
    if (lane == 0) {
        accept_len[b] = len;
        next_token[b] = id[cur + 1];
    }
}

}  // namespace

extern "C" __attribute__((visibility("default"))) rest_status rest_accept(const int32_t* d_ids, const rest_tree* tree, int32_t B, int32_t c, int32_t path_cap,
                                   int32_t* d_accept_len, int32_t* d_accept_path, int32_t* d_next_token, void* stream) {
    if (!d_ids || !tree || !tree->draft_tokens || !tree->parent_idx || !tree->n_nodes) return REST_INVALID_ARG;
    if (!d_accept_len || !d_accept_path || !d_next_token) return REST_INVALID_ARG;
    if (B < 0 || c < 1 || c > REST_MAX_NODES || path_cap < 1 || path_cap > REST_MAX_NODES) return REST_INVALID_ARG;
    if (B == 0) return REST_OK;
    hipLaunchKernelGGL(accept_kernel, dim3(B), dim3(64), 0, (hipStream_t)stream, d_ids, tree->draft_tokens,
                       tree->parent_idx, tree->n_nodes, c, path_cap, d_accept_len, d_accept_path, d_next_token);
    REST_HIP_TRY(hipGetLastError());
    return REST_OK;
}
