// Shared host/device helpers for the gfx950 REST library (internal, not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/rest.h"

#define REST_HIP_TRY(expr)                         \
    do {                                           \
        hipError_t e__ = (expr);                   \
        if (e__ != hipSuccess) {                   \
            (void)hipGetLastError();               \
            return REST_HIP_ERROR;                 \
        }                                          \
    } while (0)

#define REST_WAVE 64

struct rest_index {
    const void* d_corpus;   // borrowed
    const void* d_sa;       // owned iff owns_sa
    int32_t* d_top_keys;    // owned: table of top_count sampled suffixes (ranks and first REST_MAX_SUFFIX_LEN tokens,
                            // -1 past the end), in the layout the retrieval kernel copies to LDS
    uint64_t n_tokens;
    int32_t token_bytes;
    int32_t sa_bytes;
    int32_t top_count;      // number of sampled suffix-array ranks in d_top_keys
    int32_t owns_sa;
    int32_t sort_depth;     // 0: d_sa is the suffix array; else positions are ordered by their first sort_depth tokens only
};

// Rank of the i-th sampled suffix (i in [0, top_count)): the ranks split [0, n) into top_count + 1 near-equal parts.
__host__ __device__ inline uint64_t rest_top_rank(uint64_t n, int32_t top_count, int32_t i) {
    // n < 2^32 and top_count < 2^11, so the product fits 64 bits
    return (n * (uint64_t)(i + 1)) / (uint64_t)(top_count + 1);
}

rest_status rest_internal_make_top_table(rest_index* idx, hipStream_t stream);
