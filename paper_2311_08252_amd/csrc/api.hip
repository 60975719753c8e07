// Handle management and small utilities of the C ABI.
#include "common.h"
#include <new>

extern "C" __attribute__((visibility("default"))) const char* rest_status_string(rest_status s) {
    switch (s) {
        case REST_OK: return "ok";
        case REST_INVALID_ARG: return "invalid argument";
        case REST_UNSUPPORTED: return "unsupported";
        case REST_WORKSPACE_TOO_SMALL: return "workspace too small";
        case REST_OUT_OF_MEMORY: return "out of device memory";
        case REST_HIP_ERROR: return "HIP runtime error";
        case REST_IO_ERROR: return "file input/output error";
        case REST_BAD_FILE: return "not an index file of this token stream";
        case REST_BOUNDS_VIOLATION: return "index out of bounds inside a kernel (bounds-checked build)";
        default: return "unknown status";
    }
}

extern "C" __attribute__((visibility("default"))) const char* rest_version(void) {
#ifdef REST_BOUNDS_CHECK
    return "rest-gfx950 0.2 (bounds-checked build)";
#else
    return "rest-gfx950 0.2";
#endif
}

extern "C" __attribute__((visibility("default"))) rest_status rest_index_from_sa(const void* d_corpus, const void* d_sa, uint64_t n_tokens, int32_t token_bytes,
                                          int32_t sa_bytes, void* stream, rest_index** out) {
    if (!d_corpus || !d_sa || !out) return REST_INVALID_ARG;
    if (token_bytes != 2 && token_bytes != 4) return REST_INVALID_ARG;
    if (sa_bytes != 4 && sa_bytes != 8) return REST_INVALID_ARG;
    if (n_tokens < 1 || n_tokens > 0xFFFFFFFEull) return REST_INVALID_ARG;
    if (sa_bytes == 4 && n_tokens >= (1ull << 31)) return REST_INVALID_ARG;
    rest_index* idx = new (std::nothrow) rest_index();
    if (!idx) return REST_OUT_OF_MEMORY;
    idx->d_corpus = d_corpus;
    idx->d_sa = d_sa;
    idx->d_top_keys = nullptr;
    idx->n_tokens = n_tokens;
    idx->token_bytes = token_bytes;
    idx->sa_bytes = sa_bytes;
    idx->top_count = 0;
    idx->owns_sa = 0;
    idx->sort_depth = 0;
    rest_status st = rest_internal_make_top_table(idx, (hipStream_t)stream);
    if (st != REST_OK) {
        rest_index_destroy(idx);
        return st;
    }
    *out = idx;
    return REST_OK;
}

extern "C" __attribute__((visibility("default"))) rest_status rest_index_view(const rest_index* index, const void** d_corpus, const void** d_sa,
                                       uint64_t* n_tokens, int32_t* token_bytes, int32_t* sa_bytes) {
    if (!index) return REST_INVALID_ARG;
    if (d_corpus) *d_corpus = index->d_corpus;
    if (d_sa) *d_sa = index->d_sa;
    if (n_tokens) *n_tokens = index->n_tokens;
    if (token_bytes) *token_bytes = index->token_bytes;
    if (sa_bytes) *sa_bytes = index->sa_bytes;
    return REST_OK;
}

extern "C" __attribute__((visibility("default"))) int32_t rest_index_sort_depth(const rest_index* index) {
    return index ? index->sort_depth : -1;
}

extern "C" __attribute__((visibility("default"))) void rest_index_destroy(rest_index* index) {
    if (!index) return;
    if (index->owns_sa && index->d_sa) (void)hipFree((void*)index->d_sa);
    if (index->d_top_keys) (void)hipFree(index->d_top_keys);
    delete index;
}
