// rest_build_index for gfx950: the suffix array of the token stream ("Datastore construction" and the
// suffix-array exact match of "Retrieving from the datastore", REST, arXiv 2311.08252), built on the GPU
// by prefix doubling (Manber & Myers' idea) where every round is an LSD radix sort.
//
// Round with step h: rank[i] orders suffix i by its first h tokens (0 = past the end of the stream, which
// makes the end smaller than every token).  Sorting positions by the 64-bit key (rank[i], rank[i+h])
// orders them by their first 2h tokens; new ranks are the index of the first member of each run of equal
// keys.  The first round uses token + 1 as rank.  A suffix whose key is unique has its final rank; only the
// others (kept as a list, in sorted order) go into the next round, where the first key half -- the rank of
// their group, i.e. one plus the group's first place in the final array -- keeps the groups apart and in
// place.  On text, and on the synthetic streams, four fifths of the suffixes remain after the first round,
// an eighth after the second, under one per cent after the third.  Rounds stop when no suffix is left.
//
// Radix sort: 8-bit digits, three kernels per digit (per-tile digit histogram, exclusive scan over
// (digit, tile), stable scatter).  Inside a wavefront, lanes holding the same digit find each other with
// eight ballots, so ranking needs no LDS atomics.  No kernel spins on another workgroup.
#include "common.h"

namespace {

constexpr int kSortThreads = 256;
constexpr int kScanChunk = 2048;

template <typename TokT>
__global__ void init_rank_kernel(const TokT* corpus, uint64_t n, uint32_t* rank, uint32_t* max_out) {
    uint32_t mx = 0;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (uint64_t)gridDim.x * blockDim.x) {
        const uint32_t r = (uint32_t)corpus[i] + 1u;
        rank[i] = r;
        mx = r > mx ? r : mx;
    }
    __shared__ uint32_t part[4];
    for (int off = 32; off > 0; off >>= 1) {
        uint32_t y = __shfl_xor(mx, off, 64);
        mx = y > mx ? y : mx;
    }
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = mx;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 4; w++) mx = part[w] > mx ? part[w] : mx;
        atomicMax(max_out, mx);
    }
}

// keys of the m suffixes still in play: list[j] (or j itself in the first round, list == null)
__global__ void make_keys_kernel(const uint32_t* rank, uint64_t n, uint64_t h, const uint32_t* list, uint64_t m,
                                 uint64_t* key, uint32_t* val) {
    for (uint64_t j = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; j < m; j += (uint64_t)gridDim.x * blockDim.x) {
        const uint64_t i = REST_IDX(list ? (uint64_t)list[j] : j, n, 8);      // a listed suffix is a position of the stream
        const uint32_t second = i + h < n ? rank[i + h] : 0u;
        key[j] = ((uint64_t)rank[i] << 32) | second;
        val[j] = (uint32_t)i;
    }
}

// lanes of the wavefront that are valid and hold the same 8-bit digit as this lane
__device__ inline uint64_t match_digit(uint32_t digit, bool valid) {
    uint64_t m = __ballot(valid);
#pragma unroll
    for (int b = 0; b < 8; b++) {
        const bool bit = (digit >> b) & 1u;
        const uint64_t bb = __ballot(bit);
        m &= bit ? bb : ~bb;
    }
    return m;
}

// per-tile digit histogram, stored digit-major: hist[digit * ntiles + tile]
__global__ __launch_bounds__(kSortThreads) void radix_hist_kernel(const uint64_t* key, uint64_t n, int shift,
                                                                   uint32_t tile, uint32_t ntiles, uint32_t* hist) {
    __shared__ uint32_t cnt[256];
    const int tid = threadIdx.x, lane = tid & 63;
    cnt[tid] = 0;
    __syncthreads();
    const uint64_t base = (uint64_t)blockIdx.x * tile;
    // eight reads in flight per thread (tile is a multiple of 256, not of 2048: the last group may be ragged)
    for (uint32_t s = 0; s < tile; s += 8 * kSortThreads) {
        uint64_t k[8];
#pragma unroll
        for (int r = 0; r < 8; r++) {
            const uint64_t i = base + s + r * kSortThreads + tid;
            k[r] = (s + r * kSortThreads < tile && i < n) ? key[i] : 0ull;
        }
#pragma unroll
        for (int r = 0; r < 8; r++) {
            const uint64_t i = base + s + r * kSortThreads + tid;
            const bool valid = s + r * kSortThreads < tile && i < n;
            const uint32_t d = (uint32_t)(k[r] >> shift) & 255u;
            const uint64_t m = match_digit(d, valid);
            if (valid && (m & ((1ull << lane) - 1ull)) == 0) atomicAdd(&cnt[d], (uint32_t)__popcll(m));
        }
    }
    __syncthreads();
    hist[(uint64_t)tid * ntiles + blockIdx.x] = cnt[tid];
}

// ---- exclusive scan (add) / inclusive scan (max) over uint32 arrays, three kernels, no spinning
template <bool IS_MAX>
__device__ inline uint32_t op(uint32_t a, uint32_t b) { return IS_MAX ? (a > b ? a : b) : a + b; }

template <bool IS_MAX>
__global__ __launch_bounds__(256) void scan_sums_kernel(const uint32_t* x, uint64_t n, uint32_t* sums) {
    __shared__ uint32_t red[256];
    const uint64_t base = (uint64_t)blockIdx.x * kScanChunk;
    uint32_t a = 0;
    for (int i = threadIdx.x; i < kScanChunk; i += 256)
        if (base + i < n) a = op<IS_MAX>(a, x[base + i]);
    red[threadIdx.x] = a;
    __syncthreads();
    for (int st = 128; st > 0; st >>= 1) {
        if ((int)threadIdx.x < st) red[threadIdx.x] = op<IS_MAX>(red[threadIdx.x], red[threadIdx.x + st]);
        __syncthreads();
    }
    if (threadIdx.x == 0) sums[blockIdx.x] = red[0];
}

// exclusive scan of `sums` in place by one workgroup (each thread owns a contiguous run)
template <bool IS_MAX>
__global__ __launch_bounds__(1024) void scan_top_kernel(uint32_t* sums, uint64_t n) {
    __shared__ uint32_t tot[1024];
    const uint64_t per = (n + 1023) / 1024;
    const uint64_t b0 = (uint64_t)threadIdx.x * per;
    uint32_t a = 0;
    for (uint64_t i = 0; i < per; i++)
        if (b0 + i < n) a = op<IS_MAX>(a, sums[b0 + i]);
    tot[threadIdx.x] = a;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t run = 0;
        for (int i = 0; i < 1024; i++) {
            const uint32_t v = tot[i];
            tot[i] = run;
            run = op<IS_MAX>(run, v);
        }
    }
    __syncthreads();
    uint32_t run = tot[threadIdx.x];
    for (uint64_t i = 0; i < per; i++)
        if (b0 + i < n) {
            const uint32_t v = sums[b0 + i];
            sums[b0 + i] = run;
            run = op<IS_MAX>(run, v);
        }
}

// add: x becomes its exclusive prefix sum; max: x becomes its inclusive prefix maximum
template <bool IS_MAX>
__global__ __launch_bounds__(256) void scan_apply_kernel(uint32_t* x, uint64_t n, const uint32_t* sums) {
    __shared__ uint32_t part[256];
    const uint64_t base = (uint64_t)blockIdx.x * kScanChunk;
    constexpr int per = kScanChunk / 256;
    const uint64_t b0 = base + (uint64_t)threadIdx.x * per;
    uint32_t v[per];
    uint32_t a = 0;
#pragma unroll
    for (int i = 0; i < per; i++) {
        v[i] = b0 + i < n ? x[b0 + i] : 0u;
        a = op<IS_MAX>(a, v[i]);
    }
    part[threadIdx.x] = a;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t run = sums[blockIdx.x];
        for (int i = 0; i < 256; i++) {
            const uint32_t t = part[i];
            part[i] = run;
            run = op<IS_MAX>(run, t);
        }
    }
    __syncthreads();
    uint32_t run = part[threadIdx.x];
#pragma unroll
    for (int i = 0; i < per; i++) {
        if (IS_MAX) {
            run = op<true>(run, v[i]);
            if (b0 + i < n) x[b0 + i] = run;
        } else {
            if (b0 + i < n) x[b0 + i] = run;
            run += v[i];
        }
    }
}

// Stable scatter of one tile by digit.  The tile goes through LDS in chunks of kChunk elements: a chunk is first put
// in digit order inside LDS (wavefront w ranks elements [1024 w, 1024 w + 1024) of the chunk, 64 at a time, with a
// running count per digit; a scan over (digit, wavefront) turns the ranks into LDS positions), then written out in
// that order, so that the elements of one digit leave as one contiguous run instead of one 12-byte write each.
constexpr int kChunk = 4096;
constexpr int kPerLane = kChunk / kSortThreads;     // 16 elements per thread and chunk

__global__ __launch_bounds__(kSortThreads) void radix_scatter_kernel(const uint64_t* key_in, const uint32_t* val_in,
                                                                      uint64_t* key_out, uint32_t* val_out, uint64_t n,
                                                                      int shift, uint32_t tile, uint32_t ntiles,
                                                                      const uint32_t* offsets) {
    __shared__ uint64_t skey[kChunk];
    __shared__ uint32_t sval[kChunk];
    __shared__ uint32_t base[256];            // global position of the next element of each digit
    __shared__ uint32_t wcnt[4][256];         // running count per (wavefront, digit), then its LDS start
    __shared__ uint32_t dstart[256];          // LDS position of a digit's first element in the chunk
    __shared__ uint32_t scan[256];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    base[tid] = offsets[(uint64_t)tid * ntiles + blockIdx.x];
    const uint64_t tbase = (uint64_t)blockIdx.x * tile;
    for (uint32_t c0 = 0; c0 < tile; c0 += kChunk) {
#pragma unroll
        for (int w = 0; w < 4; w++) wcnt[w][tid] = 0;
        __syncthreads();
        // ---- rank: element e of the chunk is handled by wavefront e / 1024, round (e % 1024) / 64, lane e % 64
        uint64_t k[kPerLane];
        uint32_t v[kPerLane];
        uint32_t rank[kPerLane];              // rank among the wavefront's elements of the same digit
        const uint32_t climit = tile - c0 < (uint32_t)kChunk ? tile - c0 : (uint32_t)kChunk;
        // all of the chunk's reads are issued before the first is needed
#pragma unroll
        for (int r = 0; r < kPerLane; r++) {
            const uint32_t e = (uint32_t)wave * (kChunk / 4) + r * 64 + lane;
            const uint64_t i = tbase + c0 + e;
            k[r] = 0;
            v[r] = 0;
            if (e < climit && i < n) { k[r] = key_in[i]; v[r] = val_in[i]; }
        }
#pragma unroll
        for (int r = 0; r < kPerLane; r++) {
            const uint32_t e = (uint32_t)wave * (kChunk / 4) + r * 64 + lane;
            const bool valid = e < climit && tbase + c0 + e < n;
            const uint32_t d = (uint32_t)(k[r] >> shift) & 255u;
            const uint64_t m = match_digit(d, valid);
            const uint32_t before = (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
            // all lanes of a digit read the running count, then the first of them moves it on
            const uint32_t old = valid ? wcnt[wave][d] : 0u;
            rank[r] = valid ? old + before : 0xffffffffu;
            if (valid && before == 0) wcnt[wave][d] = old + (uint32_t)__popcll(m);
        }
        __syncthreads();
        // ---- LDS start of every (digit, wavefront) group: digits ascending, wavefronts ascending within a digit
        uint32_t c[4], tot = 0;
#pragma unroll
        for (int w = 0; w < 4; w++) { c[w] = wcnt[w][tid]; tot += c[w]; }
        scan[tid] = tot;
        __syncthreads();
        for (int off = 1; off < 256; off <<= 1) {
            const uint32_t y = tid >= off ? scan[tid - off] : 0u;
            __syncthreads();
            scan[tid] += y;
            __syncthreads();
        }
        uint32_t run = scan[tid] - tot;       // exclusive
        dstart[tid] = run;
#pragma unroll
        for (int w = 0; w < 4; w++) { wcnt[w][tid] = run; run += c[w]; }
        __syncthreads();
        // ---- place
#pragma unroll
        for (int r = 0; r < kPerLane; r++) {
            if (rank[r] != 0xffffffffu) {
                const uint32_t d = (uint32_t)(k[r] >> shift) & 255u;
                const uint32_t pos = wcnt[wave][d] + rank[r];
                skey[pos] = k[r];
                sval[pos] = v[r];
            }
        }
        __syncthreads();
        // ---- write out in LDS order: position p of digit d goes to base[d] + (p - dstart[d])
        const uint32_t count = scan[255];
        for (uint32_t pp = tid; pp < count; pp += kSortThreads) {
            const uint64_t kk = skey[pp];
            const uint32_t d = (uint32_t)(kk >> shift) & 255u;
            const uint32_t dst = (uint32_t)REST_IDX(base[d] + (pp - dstart[d]), n, 9);      // scattered inside the sorted array
            key_out[dst] = kk;
            val_out[dst] = sval[pp];
        }
        __syncthreads();
        base[tid] += tot;
        __syncthreads();
    }
}

// Sorted keys of the suffixes in play: run[j] = j where a run of equal keys starts, grp[j] = j where a group (equal
// first half, i.e. one group of the previous round) starts, else 0; an inclusive max-scan turns both into "start of
// my run / of my group".  In the first round the first halves are tokens, not ranks: everything is one group.
// Counts the runs.
__global__ __launch_bounds__(256) void marks_kernel(const uint64_t* key, uint64_t m, int first_round, uint32_t* run, uint32_t* grp,
                                                    unsigned long long* n_runs) {
    uint32_t local = 0;
    for (uint64_t j = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; j < m; j += (uint64_t)gridDim.x * blockDim.x) {
        const uint64_t k = key[j], prev = j ? key[j - 1] : 0ull;
        const bool head = j == 0 || k != prev;
        const bool ghead = j > 0 && !first_round && (k >> 32) != (prev >> 32);
        run[j] = head ? (uint32_t)j : 0u;
        grp[j] = ghead ? (uint32_t)j : 0u;
        local += head ? 1u : 0u;
    }
    // one atomic per workgroup: a quarter of a million of them on one address would take longer than the pass itself
    __shared__ uint32_t part[4];
    for (int off = 32; off > 0; off >>= 1) local += __shfl_xor(local, off, 64);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = local;
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t sum = part[0] + part[1] + part[2] + part[3];
        if (sum) atomicAdd(n_runs, (unsigned long long)sum);
    }
}

// New rank of suffix val[j]: the rank of its group (first key half; 1 in the first round) plus the offset of its run
// inside the group.  In the last round of a depth-limited build every suffix gets its own place instead (offset of j
// itself): equal keys then stay in the order they have, which is ascending position.
__global__ void assign_rank_kernel(const uint64_t* key, const uint32_t* val, const uint32_t* run_start, const uint32_t* grp_start,
                                   uint64_t m, int first_round, int spread, uint32_t* rank, uint64_t n) {
    for (uint64_t j = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; j < m; j += (uint64_t)gridDim.x * blockDim.x) {
        const uint32_t base = first_round ? 1u : (uint32_t)(key[j] >> 32);
        const uint32_t at = spread ? (uint32_t)j : run_start[j];
        rank[REST_IDX(val[j], n, 10)] = base + (at - grp_start[j]);
    }
}

// flag[j] = 1 if suffix j of the sorted list shares its key with a neighbour (it stays in play), else 0; counts them
__global__ __launch_bounds__(256) void unsettled_kernel(const uint32_t* run_start, uint64_t m, uint32_t* flag, unsigned long long* count) {
    uint32_t local = 0;
    for (uint64_t j = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; j < m; j += (uint64_t)gridDim.x * blockDim.x) {
        const bool alone = run_start[j] == (uint32_t)j && (j + 1 == m || run_start[j + 1] == (uint32_t)(j + 1));
        flag[j] = alone ? 0u : 1u;
        local += alone ? 0u : 1u;
    }
    __shared__ uint32_t part[4];
    for (int off = 32; off > 0; off >>= 1) local += __shfl_xor(local, off, 64);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = local;
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t sum = part[0] + part[1] + part[2] + part[3];
        if (sum) atomicAdd(count, (unsigned long long)sum);
    }
}

// the suffixes that stay in play, in their sorted order: pos = exclusive prefix sum of the flags
__global__ void compact_kernel(const uint32_t* val, const uint32_t* run_start, const uint32_t* pos, uint64_t m, uint32_t* list) {
    for (uint64_t j = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; j < m; j += (uint64_t)gridDim.x * blockDim.x) {
        const bool alone = run_start[j] == (uint32_t)j && (j + 1 == m || run_start[j + 1] == (uint32_t)(j + 1));
        if (!alone) list[REST_IDX(pos[j], m, 11)] = val[j];
    }
}

// final ranks are a permutation of 1..n: the suffix array is its inverse
template <typename SaT>
__global__ void invert_kernel(const uint32_t* rank, uint64_t n, SaT* sa) {
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (uint64_t)gridDim.x * blockDim.x) {
        const uint32_t r = rank[i];
        (void)REST_IDX((uint64_t)r - 1u, n, 12);           // final ranks are 1 .. n (a rank outside is skipped, and noted)
        if (r >= 1u && (uint64_t)r <= n) sa[r - 1u] = (SaT)i;
    }
}

template <bool IS_MAX>
rest_status scan_u32(uint32_t* x, uint64_t n, uint32_t* sums, hipStream_t st) {
    const uint64_t chunks = (n + kScanChunk - 1) / kScanChunk;
    hipLaunchKernelGGL(scan_sums_kernel<IS_MAX>, dim3((unsigned)chunks), dim3(256), 0, st, x, n, sums);
    hipLaunchKernelGGL(scan_top_kernel<IS_MAX>, dim3(1), dim3(1024), 0, st, sums, chunks);
    hipLaunchKernelGGL(scan_apply_kernel<IS_MAX>, dim3((unsigned)chunks), dim3(256), 0, st, x, n, sums);
    REST_HIP_TRY(hipGetLastError());
    return REST_OK;
}

int bit_length(uint64_t x) {
    int b = 0;
    while (x) { b++; x >>= 1; }
    return b;
}

struct Scratch {
    uint64_t* key[2] = {nullptr, nullptr};
    uint32_t* val[2] = {nullptr, nullptr};
    uint32_t* rank = nullptr;
    uint32_t* list = nullptr;
    uint32_t* hist = nullptr;
    uint32_t* sums = nullptr;
    unsigned long long* counters = nullptr;
    void* sa = nullptr;
    ~Scratch() {
        for (int i = 0; i < 2; i++) { if (key[i]) (void)hipFree(key[i]); if (val[i]) (void)hipFree(val[i]); }
        if (rank) (void)hipFree(rank);
        if (list) (void)hipFree(list);
        if (hist) (void)hipFree(hist);
        if (sums) (void)hipFree(sums);
        if (counters) (void)hipFree(counters);
        if (sa) (void)hipFree(sa);
    }
};

#define REST_ALLOC(ptr, bytes)                                   \
    do {                                                         \
        if (hipMalloc((void**)&(ptr), (bytes)) != hipSuccess) {  \
            (void)hipGetLastError();                             \
            return REST_OUT_OF_MEMORY;                           \
        }                                                        \
    } while (0)

}  // namespace

extern "C" __attribute__((visibility("default"))) rest_status rest_build_index(const void* d_corpus, uint64_t n, int32_t token_bytes, int32_t sa_bytes,
                                        void* stream_, rest_index** out) {
    return rest_build_index_prefix(d_corpus, n, token_bytes, sa_bytes, 0, stream_, out);
}

// depth > 0: doubling stops once the positions are ordered by their first 2h >= depth tokens; every round sorts
// (position order, key) pairs stably from scratch, so positions with equal prefixes stay in ascending order.
extern "C" __attribute__((visibility("default"))) rest_status rest_build_index_prefix(const void* d_corpus, uint64_t n, int32_t token_bytes, int32_t sa_bytes,
                                               int32_t depth, void* stream_, rest_index** out) {
    if (!d_corpus || !out) return REST_INVALID_ARG;
    if (depth < 0 || depth > (1 << 30)) return REST_INVALID_ARG;
    if (token_bytes != 2 && token_bytes != 4) return REST_INVALID_ARG;
    if (sa_bytes != 4 && sa_bytes != 8) return REST_INVALID_ARG;
    if (n < 1 || n > 0xFFFFFFFEull) return REST_INVALID_ARG;
    if (sa_bytes == 4 && n >= (1ull << 31)) return REST_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream_;

    // tiles of the radix passes: multiples of 256 elements, at most 32768 of them; sized per round for the m suffixes
    // still in play, so the buffers sized here for m = n hold every round
    auto tile_of = [](uint64_t m) {
        uint64_t t = (m + 32767) / 32768;
        t = ((t + kSortThreads - 1) / kSortThreads) * kSortThreads;
        return (uint32_t)(t < 4096 ? 4096 : t);
    };
    // a round with m <= n suffixes uses ceil(m / tile_of(m)) tiles: never more than 32768, nor than ceil(n / 4096)
    const uint64_t max_tiles = (n + 4095) / 4096 < 32768 ? (n + 4095) / 4096 : 32768;
    const uint64_t hist_cap = (uint64_t)256 * max_tiles;
    const uint64_t sums_n = ((n > hist_cap ? n : hist_cap) + kScanChunk - 1) / kScanChunk;

    Scratch s;
    for (int i = 0; i < 2; i++) { REST_ALLOC(s.key[i], n * 8); REST_ALLOC(s.val[i], n * 4); }
    REST_ALLOC(s.rank, n * 4);
    REST_ALLOC(s.list, n * 4);
    REST_ALLOC(s.hist, hist_cap * 4);
    REST_ALLOC(s.sums, sums_n * 4);
    REST_ALLOC(s.counters, 16);
    REST_ALLOC(s.sa, n * (uint64_t)sa_bytes);

    auto blocks_for = [](uint64_t m, unsigned cap) { return (unsigned)((m + 255) / 256 < cap ? (m + 255) / 256 : cap); };
    REST_HIP_TRY(hipMemsetAsync(s.counters, 0, 16, st));
    if (token_bytes == 2)
        hipLaunchKernelGGL(init_rank_kernel<uint16_t>, dim3(blocks_for(n, 4096)), dim3(256), 0, st, (const uint16_t*)d_corpus, n, s.rank, (uint32_t*)s.counters);
    else
        hipLaunchKernelGGL(init_rank_kernel<int32_t>, dim3(blocks_for(n, 4096)), dim3(256), 0, st, (const int32_t*)d_corpus, n, s.rank, (uint32_t*)s.counters);
    REST_HIP_TRY(hipGetLastError());
    uint32_t max_rank = 0;
    REST_HIP_TRY(hipMemcpyAsync(&max_rank, s.counters, 4, hipMemcpyDeviceToHost, st));
    REST_HIP_TRY(hipStreamSynchronize(st));

    int32_t sorted_by = 0;   // tokens the final order looks at; 0 = all of them
    uint64_t m = n;          // suffixes still in play, listed in s.list in sorted order (first round: all, no list)
    for (uint64_t h = 1;; h *= 2) {
        const bool first_round = h == 1;
        const unsigned gs = blocks_for(m, 65536), gs_reduce = blocks_for(m, 4096);
        const uint32_t tile = tile_of(m);
        const uint32_t ntiles = (uint32_t)((m + tile - 1) / tile);
        const uint64_t hist_n = (uint64_t)256 * ntiles;
        const int passes_half = (bit_length(max_rank) + 7) / 8;
        hipLaunchKernelGGL(make_keys_kernel, dim3(gs), dim3(256), 0, st, s.rank, n, h, first_round ? nullptr : s.list, m, s.key[0], s.val[0]);
        REST_HIP_TRY(hipGetLastError());
        int cur = 0;
        for (int half = 0; half < 2; half++) {
            for (int ps = 0; ps < passes_half; ps++) {
                const int shift = half * 32 + ps * 8;
                hipLaunchKernelGGL(radix_hist_kernel, dim3(ntiles), dim3(kSortThreads), 0, st, s.key[cur], m, shift, tile, ntiles, s.hist);
                REST_HIP_TRY(hipGetLastError());
                rest_status rs = scan_u32<false>(s.hist, hist_n, s.sums, st);
                if (rs != REST_OK) return rs;
                hipLaunchKernelGGL(radix_scatter_kernel, dim3(ntiles), dim3(kSortThreads), 0, st, s.key[cur], s.val[cur],
                                   s.key[cur ^ 1], s.val[cur ^ 1], m, shift, tile, ntiles, s.hist);
                REST_HIP_TRY(hipGetLastError());
                cur ^= 1;
            }
        }
        // runs of equal keys and groups of equal first halves -> new ranks.  The other key and value buffers are free now.
        uint32_t* run = s.val[cur ^ 1];
        uint32_t* grp = (uint32_t*)s.key[cur ^ 1];
        uint32_t* flag = grp + m;
        REST_HIP_TRY(hipMemsetAsync(s.counters, 0, 16, st));
        hipLaunchKernelGGL(marks_kernel, dim3(gs_reduce), dim3(256), 0, st, s.key[cur], m, first_round ? 1 : 0, run, grp, s.counters);
        REST_HIP_TRY(hipGetLastError());
        unsigned long long runs = 0;
        REST_HIP_TRY(hipMemcpyAsync(&runs, s.counters, 8, hipMemcpyDeviceToHost, st));
        rest_status rs = scan_u32<true>(run, m, s.sums, st);
        if (rs != REST_OK) return rs;
        rs = scan_u32<true>(grp, m, s.sums, st);
        if (rs != REST_OK) return rs;
        REST_HIP_TRY(hipStreamSynchronize(st));
        // the last round of a depth-limited build (or, as a guard, a step that already spans the stream) gives every
        // suffix a place of its own
        const bool limit = depth > 0 && 2 * h >= (uint64_t)depth;
        const bool spread = runs < m && (limit || h >= n);
        hipLaunchKernelGGL(assign_rank_kernel, dim3(gs), dim3(256), 0, st, s.key[cur], s.val[cur], run, grp, m, first_round ? 1 : 0,
                           spread ? 1 : 0, s.rank, n);
        REST_HIP_TRY(hipGetLastError());
        if (runs == m) break;                               // every suffix distinct: the suffix array
        if (spread) { sorted_by = limit ? (int32_t)(2 * h) : 0; break; }
        // the suffixes that still share a key go on
        REST_HIP_TRY(hipMemsetAsync(s.counters, 0, 16, st));
        hipLaunchKernelGGL(unsettled_kernel, dim3(gs_reduce), dim3(256), 0, st, run, m, flag, s.counters);
        REST_HIP_TRY(hipGetLastError());
        unsigned long long left = 0;
        REST_HIP_TRY(hipMemcpyAsync(&left, s.counters, 8, hipMemcpyDeviceToHost, st));
        rs = scan_u32<false>(flag, m, s.sums, st);
        if (rs != REST_OK) return rs;
        hipLaunchKernelGGL(compact_kernel, dim3(gs), dim3(256), 0, st, s.val[cur], run, flag, m, s.list);
        REST_HIP_TRY(hipGetLastError());
        REST_HIP_TRY(hipStreamSynchronize(st));
        if (left == 0) break;                               // cannot happen while runs < m; a guard
        m = left;
        max_rank = (uint32_t)n;
    }

    const unsigned gn = blocks_for(n, 65536);
    if (sa_bytes == 4) hipLaunchKernelGGL(invert_kernel<int32_t>, dim3(gn), dim3(256), 0, st, s.rank, n, (int32_t*)s.sa);
    else hipLaunchKernelGGL(invert_kernel<int64_t>, dim3(gn), dim3(256), 0, st, s.rank, n, (int64_t*)s.sa);
    REST_HIP_TRY(hipGetLastError());
    REST_HIP_TRY(hipStreamSynchronize(st));
    REST_BOUNDS_EPILOGUE(st);

    rest_index* idx = nullptr;
    rest_status rs = rest_index_from_sa(d_corpus, s.sa, n, token_bytes, sa_bytes, stream_, &idx);
    if (rs != REST_OK) return rs;
    idx->owns_sa = 1;
    idx->sort_depth = sorted_by;
    s.sa = nullptr;   // ownership moved to the handle
    *out = idx;
    return REST_OK;
}
