// Draft acceptance ("Draft acceptance of REST", arXiv 2311.08252): accept draft tokens from the start of
// the tree while they equal the model's own token at that position; everything after the first
// disagreement is rejected, so the emitted sequence equals ordinary autoregressive decoding.
//
// One wavefront per context.  The tree (parents, tokens) and the model's tokens are read once -- nodes into registers,
// four per lane, the model's tokens into LDS --, so that a step of the walk is an LDS read and a ballot: the child of
// the current node whose token equals the model's token (siblings carry distinct tokens, so at most one node hits;
// the lowest index is taken).
#include "common.h"

namespace {

constexpr int kPerLane = REST_MAX_NODES / 64;

__global__ __launch_bounds__(64) void accept_kernel(const int32_t* ids, const int32_t* draft_tokens,
                                                    const int32_t* parent_idx, const int32_t* n_nodes, int32_t c,
                                                    int32_t path_cap, int32_t* accept_len, int32_t* accept_path,
                                                    int32_t* next_token) {
    __shared__ int32_t s_id[REST_MAX_NODES + 1];
    const int b = blockIdx.x, lane = threadIdx.x;
    const int32_t* id = ids + (int64_t)b * (1 + c);
    const int32_t* tok = draft_tokens + (int64_t)b * c;
    const int32_t* par = parent_idx + (int64_t)b * c;
    // all reads at once: the tree's c slots are read whatever the number of nodes turns out to be (it arrives with
    // them), and the slots beyond it are struck out afterwards
    int n = n_nodes[b];
    int32_t my_par[kPerLane], my_tok[kPerLane];
#pragma unroll
    for (int k = 0; k < kPerLane; k++) {
        const int i = 64 * k + lane;            // node 64 k + lane
        my_par[k] = i < c ? par[i] : -2;        // -2: never a parent
        my_tok[k] = i < c ? tok[i] : 0;
    }
    for (int i = lane; i <= c; i += 64) s_id[i] = id[i];
    n = n < 0 ? 0 : (n > c ? c : n);
#pragma unroll
    for (int k = 0; k < kPerLane; k++)
        if (64 * k + lane >= n) my_par[k] = -2;
    __syncthreads();
    int cur = -1, len = 0;
    while (len < path_cap) {
        const int32_t want = s_id[cur + 1];
        int hit = -1;
#pragma unroll
        for (int k = kPerLane - 1; k >= 0; k--) {
            const uint64_t m = __ballot(my_par[k] == cur && my_tok[k] == want);
            if (m) hit = 64 * k + __builtin_ctzll(m);
        }
        if (hit < 0) break;
        if (lane == 0) accept_path[(int64_t)b * path_cap + len] = hit;
        cur = hit;
        len++;
    }
    for (int i = len + lane; i < path_cap; i += 64) accept_path[(int64_t)b * path_cap + i] = -1;
    if (lane == 0) {
        accept_len[b] = len;
        next_token[b] = s_id[cur + 1];
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
