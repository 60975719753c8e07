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

// Bounds-checked build (-DREST_BOUNDS_CHECK, librest_gfx950_checked.so): every index into the token stream, the
// suffix array, the rank and list arrays of the index build and the K/V/Q/output rows of the attention kernels that
// depends on data or on the launch plan goes through REST_IDX(index, size, site).  An index that is not below size is
// replaced by the last valid one -- the access stays inside the array, the kernel never traps or faults -- and bit
// (site % 32) of a device word is set; after its launches the call waits for the stream, reads the word and returns
// REST_BOUNDS_VIOLATION if it is not zero (the results of such a call mean nothing).  The product build compiles
// REST_IDX to the bare index.  Each translation unit has its own word and reads it in its own entry points.
#ifdef REST_BOUNDS_CHECK
static __device__ unsigned int rest_bounds_word;
__device__ inline uint64_t rest_checked_index(uint64_t i, uint64_t n, unsigned int site) {
    if (i < n) return i;
    atomicOr(&rest_bounds_word, 1u << (site & 31u));
    return n ? n - 1 : 0;
}
#define REST_IDX(i, n, site) rest_checked_index((uint64_t)(i), (uint64_t)(n), (site))
static inline rest_status rest_bounds_epilogue(hipStream_t stream) {
    unsigned int w = 0, zero = 0;
    if (hipStreamSynchronize(stream) != hipSuccess) return REST_HIP_ERROR;
    if (hipMemcpyFromSymbol(&w, HIP_SYMBOL(rest_bounds_word), sizeof(w)) != hipSuccess) return REST_HIP_ERROR;
    if (w == 0) return REST_OK;
    (void)hipMemcpyToSymbol(HIP_SYMBOL(rest_bounds_word), &zero, sizeof(zero));
    return REST_BOUNDS_VIOLATION;
}
#define REST_BOUNDS_EPILOGUE(stream)                                  \
    do {                                                              \
        const rest_status b__ = rest_bounds_epilogue((hipStream_t)(stream)); \
        if (b__ != REST_OK) return b__;                               \
    } while (0)
#else
#define REST_IDX(i, n, site) (i)
#define REST_BOUNDS_EPILOGUE(stream) do { } while (0)
#endif

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
