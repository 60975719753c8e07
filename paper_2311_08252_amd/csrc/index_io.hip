// Datastore persistence: the suffix array of a token stream is built once ("Datastore construction", REST,
// arXiv 2311.08252) and reused by every later run, so it can be written to and read from a host file.
//
// File layout (little endian): 64-byte header
//     bytes  0.. 7  "RESTSA01"
//     bytes  8..15  n_tokens        uint64
//     bytes 16..19  token_bytes     int32 (2 or 4)
//     bytes 20..23  sa_bytes        int32 (4 or 8)
//     bytes 24..31  fingerprint     uint64 of the token stream the array belongs to
//     bytes 32..35  sort depth      int32: 0 = a suffix array, else the positions are ordered by that many tokens
//     bytes 36..63  zero
// followed by n_tokens suffix-array entries of sa_bytes each.
// fingerprint = sum over i of mix(token_i + (i + 1) * 0x9E3779B97F4A7C15) modulo 2^64, mix = the splitmix64 finaliser;
// a sum, so it can be formed in any order.  The array moves through a pinned 64 MB staging buffer.
#include "common.h"
#include <cstdio>
#include <cstring>
#include <new>

namespace {

constexpr size_t kHeader = 64;
constexpr size_t kStage = 64u << 20;
const char kMagic[8] = {'R', 'E', 'S', 'T', 'S', 'A', '0', '1'};

__device__ inline uint64_t mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

template <typename TokT>
__global__ __launch_bounds__(256) void fingerprint_kernel(const TokT* tok, uint64_t n, unsigned long long* out) {
    uint64_t acc = 0;
    for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (uint64_t)gridDim.x * 256)
        acc += mix64((uint64_t)tok[i] + (i + 1) * 0x9E3779B97F4A7C15ull);
    for (int off = 32; off > 0; off >>= 1) {
        const uint32_t lo = __shfl_xor((uint32_t)acc, off, 64), hi = __shfl_xor((uint32_t)(acc >> 32), off, 64);
        acc += ((uint64_t)hi << 32) | lo;
    }
    if ((threadIdx.x & 63) == 0) atomicAdd(out, (unsigned long long)acc);
}

// fingerprint of the stream; synchronises `stream`
rest_status fingerprint(const void* d_corpus, uint64_t n, int token_bytes, hipStream_t stream, uint64_t* fp) {
    unsigned long long* d_fp = nullptr;
    if (hipMalloc((void**)&d_fp, sizeof(*d_fp)) != hipSuccess) {
        (void)hipGetLastError();
        return REST_OUT_OF_MEMORY;
    }
    rest_status st = REST_OK;
    const int blocks = (int)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
    if (hipMemsetAsync(d_fp, 0, sizeof(*d_fp), stream) != hipSuccess) st = REST_HIP_ERROR;
    if (st == REST_OK) {
        if (token_bytes == 2)
            hipLaunchKernelGGL(fingerprint_kernel<uint16_t>, dim3(blocks), dim3(256), 0, stream, (const uint16_t*)d_corpus, n, d_fp);
        else
            hipLaunchKernelGGL(fingerprint_kernel<int32_t>, dim3(blocks), dim3(256), 0, stream, (const int32_t*)d_corpus, n, d_fp);
        unsigned long long h = 0;
        if (hipGetLastError() != hipSuccess || hipMemcpyAsync(&h, d_fp, sizeof(h), hipMemcpyDeviceToHost, stream) != hipSuccess ||
            hipStreamSynchronize(stream) != hipSuccess)
            st = REST_HIP_ERROR;
        *fp = h;
    }
    (void)hipFree(d_fp);
    if (st != REST_OK) (void)hipGetLastError();
    return st;
}

struct Stage {
    void* p = nullptr;
    ~Stage() { if (p) (void)hipHostFree(p); }
    bool alloc() { if (hipHostMalloc(&p, kStage, hipHostMallocDefault) != hipSuccess) { (void)hipGetLastError(); p = nullptr; } return p != nullptr; }
};

struct File {
    FILE* f = nullptr;
    ~File() { if (f) fclose(f); }
};

}  // namespace

extern "C" __attribute__((visibility("default"))) rest_status rest_index_save(const rest_index* index, const char* path, void* stream_) {
    if (!index || !path || !index->d_sa || !index->d_corpus) return REST_INVALID_ARG;
    hipStream_t stream = (hipStream_t)stream_;
    File file;
    file.f = fopen(path, "wb");
    if (!file.f) return REST_IO_ERROR;
    uint64_t fp = 0;
    rest_status st = fingerprint(index->d_corpus, index->n_tokens, index->token_bytes, stream, &fp);
    if (st != REST_OK) return st;
    unsigned char header[kHeader];
    memset(header, 0, sizeof(header));
    memcpy(header, kMagic, 8);
    memcpy(header + 8, &index->n_tokens, 8);
    memcpy(header + 16, &index->token_bytes, 4);
    memcpy(header + 20, &index->sa_bytes, 4);
    memcpy(header + 24, &fp, 8);
    memcpy(header + 32, &index->sort_depth, 4);
    if (fwrite(header, 1, kHeader, file.f) != kHeader) return REST_IO_ERROR;
    Stage stage;
    if (!stage.alloc()) return REST_OUT_OF_MEMORY;
    const size_t total = (size_t)index->n_tokens * (size_t)index->sa_bytes;
    for (size_t off = 0; off < total; off += kStage) {
        const size_t len = total - off < kStage ? total - off : kStage;
        REST_HIP_TRY(hipMemcpyAsync(stage.p, (const char*)index->d_sa + off, len, hipMemcpyDeviceToHost, stream));
        REST_HIP_TRY(hipStreamSynchronize(stream));
        if (fwrite(stage.p, 1, len, file.f) != len) return REST_IO_ERROR;
    }
    if (fflush(file.f) != 0) return REST_IO_ERROR;
    return REST_OK;
}

extern "C" __attribute__((visibility("default"))) rest_status rest_index_load(const char* path, const void* d_corpus, uint64_t n_tokens, int32_t token_bytes,
                                       void* stream_, rest_index** out) {
    if (!path || !d_corpus || !out) return REST_INVALID_ARG;
    if (token_bytes != 2 && token_bytes != 4) return REST_INVALID_ARG;
    if (n_tokens < 1 || n_tokens > 0xFFFFFFFEull) return REST_INVALID_ARG;
    hipStream_t stream = (hipStream_t)stream_;
    File file;
    file.f = fopen(path, "rb");
    if (!file.f) return REST_IO_ERROR;
    unsigned char header[kHeader];
    if (fread(header, 1, kHeader, file.f) != kHeader) return REST_IO_ERROR;
    uint64_t n = 0, fp_file = 0;
    int32_t tb = 0, sb = 0, depth = 0;
    memcpy(&n, header + 8, 8);
    memcpy(&tb, header + 16, 4);
    memcpy(&sb, header + 20, 4);
    memcpy(&fp_file, header + 24, 8);
    memcpy(&depth, header + 32, 4);
    if (memcmp(header, kMagic, 8) != 0 || (sb != 4 && sb != 8) || (sb == 4 && n >= (1ull << 31))) return REST_BAD_FILE;
    if (n != n_tokens || tb != token_bytes || depth < 0) return REST_BAD_FILE;
    uint64_t fp = 0;
    rest_status st = fingerprint(d_corpus, n_tokens, token_bytes, stream, &fp);
    if (st != REST_OK) return st;
    if (fp != fp_file) return REST_BAD_FILE;
    Stage stage;
    if (!stage.alloc()) return REST_OUT_OF_MEMORY;
    const size_t total = (size_t)n * (size_t)sb;
    void* d_sa = nullptr;
    if (hipMalloc(&d_sa, total) != hipSuccess) {
        (void)hipGetLastError();
        return REST_OUT_OF_MEMORY;
    }
    st = REST_OK;
    for (size_t off = 0; off < total && st == REST_OK; off += kStage) {
        const size_t len = total - off < kStage ? total - off : kStage;
        if (fread(stage.p, 1, len, file.f) != len) st = REST_IO_ERROR;
        else if (hipMemcpyAsync((char*)d_sa + off, stage.p, len, hipMemcpyHostToDevice, stream) != hipSuccess ||
                 hipStreamSynchronize(stream) != hipSuccess)
            st = REST_HIP_ERROR;
    }
    rest_index* idx = nullptr;
    if (st == REST_OK) st = rest_index_from_sa(d_corpus, d_sa, n_tokens, token_bytes, sb, stream_, &idx);
    if (st != REST_OK) {
        (void)hipFree(d_sa);
        (void)hipGetLastError();
        return st;
    }
    idx->owns_sa = 1;
    idx->sort_depth = depth;
    *out = idx;
    return REST_OK;
}
