// Nucleus sampling of the model's token at every position of the verification pass (REST, arXiv 2311.08252,
// "Sampling strategies"; temperature and top-p as in the caption of the main speed table).  REST accepts a draft
// token only if it equals the token sampled at its position, so the ids written here feed rest_accept unchanged.
//
// Definition (the paper fixes the parameters, not the mechanics; this one fixes the result to the last bit):
//  * probability masses are integers: token i weighs w_i = floor(2^36 * E((x_i - x_max) * c)), c = log2(e) /
//    temperature, with E(y) = 2^y evaluated by a fixed sequence of correctly rounded fp64 operations (weight_of
//    below); sums of weights are exact, so they do not depend on the order of summation;
//  * tokens are ordered by logit, highest first (+0 and -0 are one value), equal logits by ascending token id;
//  * the nucleus is the shortest prefix of that order whose mass C_k satisfies double(C_k) >= double(top_p) * double(W),
//    W the row's total mass; the draw is the first token whose cumulative mass satisfies double(C_j) > double(u) *
//    double(M), M the nucleus mass, u in [0, 1) given by the caller.
//
// Nothing is sorted.  "The place in the order where the cumulative mass crosses a threshold" is found by descending
// the order-preserving 32-bit key of the logit: 11 bits, 11 bits, 10 bits.  The first level's histogram of masses is
// built by all workgroups of a row together (each adds its slice of the row into LDS, then its non-empty buckets into
// the row's histogram in memory; integer adds, any order); the workgroup that arrives last at the row's ticket does
// the rest alone: crossing bucket of level one, then two passes over the row for the lower levels (only the few
// elements of the chosen bucket are weighed again), the rank among equal logits by integer arithmetic, the same
// for the draw, and one pass to find the token of that rank.  No workgroup waits for another.
//
// A row of at most 32768 logits takes a shorter way (sample_row_kernel): one workgroup per row holds the whole row in
// registers (32 logits per thread), so the maximum, the weights, the level-one histogram and both descents happen in
// one launch without a word of workspace, a device-scope atomic or a second walk over memory.
#include "common.h"

namespace {

typedef unsigned long long u64;

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / 64;
constexpr int kMaxSlices = 16;             // workgroups that share a row in the histogram phase, at most
constexpr int kBatch = 16;                 // reads a thread has in flight when it walks over a row
constexpr int kCap = 1024;                 // tokens of one level-one cell that the list in LDS holds: one per thread
constexpr int kMaxVocab = 1 << 17;         // sums of up to 2^17 weights of at most 2^36 stay below 2^53
constexpr int kWeightBits = 36;
constexpr int kL1 = 2048, kL2 = 2048, kL3 = 1024;     // buckets per level: key bits 31..21, 20..10, 9..0
constexpr int kRowWords = kL1 + 32;        // per row in the workspace: the level-one histogram, then 32 words: slice
                                           // maxima (floats, two to a word, up to kMaxSlices) and the ticket

// A row is cut into slices of slice_len tokens, one workgroup each: as many as keep all workgroups of the launch on
// the chip at once (256 compute units, one workgroup of 1024 threads each), at least 2048 tokens long.
struct Slicing { int slices, slice_len; };
inline Slicing slicing_of(int R, int V) {
    int s = 256 / (R > 0 ? R : 1);
    if (s > kMaxSlices) s = kMaxSlices;
    if (s > (V + 2047) / 2048) s = (V + 2047) / 2048;
    if (s < 1) s = 1;
    Slicing out;
    out.slice_len = ((V + s - 1) / s + 63) / 64 * 64;
    out.slices = (V + out.slice_len - 1) / out.slice_len;
    return out;
}

__device__ inline uint32_t key_of(float x) {
    if (x == 0.f) x = 0.f;               // -0 and +0 are the same logit
    const uint32_t b = __builtin_bit_cast(uint32_t, x);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

__device__ inline float logit_of_key(uint32_t k) {
    return __builtin_bit_cast(float, (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

// Level one of the search: 2048 cells, linear in how far a logit lies below the row's largest one (cell 0 holds the
// largest), scaled so that cell 2047 starts where the weights have long been zero.  Any function that never grows
// with the logit would do -- the cells only have to respect the order --; a linear one keeps the cell around the
// nucleus boundary small (tens of tokens of a 32000-token row), which is what the second stage costs by.
__device__ inline int cell_of(float x, float top, float scale) {
    const float d = (top - x) * scale;        // >= 0; +inf for a logit of -inf
    return d < 2047.f ? (int)d : 2047;
}

// w = floor(2^36 * E((x - top) * c)): n = floor(y), f = y - n, t = f * ln 2, E = 2^n * P(t) with P the Taylor polynomial
// of exp of degree 13 in Horner form; every step is one multiplication and one addition, each correctly rounded (no
// fused multiply-add), so the value is the same on every machine that computes in IEEE fp64.
__device__ inline u64 weight_of(float x, float top, double c) {
#pragma clang fp contract(off)
    // Below 2^-36 of the largest the floor is zero (the definition's own limit of 2^-64 lies further down).  Nothing
    // branches on that: y is held at -47 (fmax also turns -inf and NaN into -47), and the shift at the end gives zero.
    const double y = fmax(((double)x - (double)top) * c, -47.0);
    const double n = floor(y);
    const double t = (y - n) * 0x1.62e42fefa39efp-1;
    constexpr double k[14] = {0x1.0000000000000p+0,  0x1.0000000000000p+0,  0x1.0000000000000p-1,  0x1.5555555555555p-3,
                              0x1.5555555555555p-5,  0x1.1111111111111p-7,  0x1.6c16c16c16c17p-10, 0x1.a01a01a01a01ap-13,
                              0x1.a01a01a01a01ap-16, 0x1.71de3a556c734p-19, 0x1.27e4fb7789f5cp-22, 0x1.ae64567f544e4p-26,
                              0x1.1eed8eff8d898p-29, 0x1.6124613a86d09p-33};      // 1 / k!
    double p = k[13];
#pragma unroll
    for (int i = 12; i >= 0; i--) {
        p = p * t;
        p = p + k[i];
    }
    // p is in [1, 2) and n + 36 in [-11, 36]: floor(p * 2^(n + 36)) is p's significand (its bits with the exponent
    // field 0x3ff turned into the leading one) moved right by 16 ... 63 places; 53 or more leave nothing
    const u64 sig = (u64)__double_as_longlong(p) - 0x3fe0000000000000ull;
    return sig >> (52 - kWeightBits - (int)n);
}

// Calls fn(index, logit) for every token in [begin, end) of row g, the workgroup's threads side by side.  A thread's
// reads come in batches that are all issued before the first is used: a walk is bound by the latency of a read
// (the row sits in the L2 cache by then), so the number of reads in flight sets its time.
template <typename Fn>
__device__ inline void for_each_token(const float* g, int begin, int end, Fn fn) {
    for (int base = begin; base < end; base += kThreads * kBatch) {
        float xs[kBatch];
#pragma unroll
        for (int j = 0; j < kBatch; j++) {
            const int i = base + j * kThreads + (int)threadIdx.x;
            xs[j] = i < end ? g[i] : 0.f;
        }
#pragma unroll
        for (int j = 0; j < kBatch; j++) {
            const int i = base + j * kThreads + (int)threadIdx.x;
            if (i < end) fn(i, xs[j]);
        }
    }
}

// The value of another lane by the data-parallel-primitive path of the vector unit (no trip through LDS): kCtrl
// 0x110 + n = the lane n places below within its row of 16, 0x142 / 0x143 = lane 15 of the row below / lane 31 of the
// lower half, for the rows in kRows (other values of kCtrl: the permutations group_sum names); a lane with no such
// source, or in a row not named, gets `none`.
template <int kCtrl, int kRows>
__device__ inline uint32_t from_lane_below(uint32_t v, uint32_t none) {
    return (uint32_t)__builtin_amdgcn_update_dpp((int)none, (int)v, kCtrl, kRows, 0xf, false);
}

template <int kCtrl, int kRows>
__device__ inline u64 scan_step(u64 v) {
    const uint32_t lo = from_lane_below<kCtrl, kRows>((uint32_t)v, 0u), hi = from_lane_below<kCtrl, kRows>((uint32_t)(v >> 32), 0u);
    return v + (((u64)hi << 32) | lo);
}

// inclusive prefix sum over the 64 lanes of a wavefront: within rows of 16, then row 0 into 1 and 2 into 3, then the
// lower half into the upper
__device__ inline u64 wave_inclusive_scan(u64 v) {
    v = scan_step<0x111, 0xf>(v);
    v = scan_step<0x112, 0xf>(v);
    v = scan_step<0x114, 0xf>(v);
    v = scan_step<0x118, 0xf>(v);
    v = scan_step<0x142, 0xa>(v);
    v = scan_step<0x143, 0xc>(v);
    return v;
}

template <int kCtrl, int kRows>
__device__ inline float max_step(float v) {
    return fmaxf(v, __builtin_bit_cast(float, from_lane_below<kCtrl, kRows>(__builtin_bit_cast(uint32_t, v), 0xff800000u)));
}

// the largest value of the wavefront's 64 lanes, in every lane
__device__ inline float wave_max(float v) {
    v = max_step<0x111, 0xf>(v);
    v = max_step<0x112, 0xf>(v);
    v = max_step<0x114, 0xf>(v);
    v = max_step<0x118, 0xf>(v);
    v = max_step<0x142, 0xa>(v);
    v = max_step<0x143, 0xc>(v);
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

template <int kCtrl>
__device__ inline u64 swap_add(u64 v) {
    const uint32_t lo = from_lane_below<kCtrl, 0xf>((uint32_t)v, 0u), hi = from_lane_below<kCtrl, 0xf>((uint32_t)(v >> 32), 0u);
    return v + (((u64)hi << 32) | lo);
}

// Sum over each aligned group of 2^shift neighbouring lanes (shift <= 6), in every lane of the group: lane ^ 1 and
// lane ^ 2 by permutations within four lanes, then the mirror image within 8 and within 16 lanes (after the steps
// before, all lanes of the mirrored half hold one value), the last two steps through LDS.
__device__ inline u64 group_sum(u64 v, int shift) {
    if (shift > 0) v = swap_add<0xb1>(v);           // quad_perm [1, 0, 3, 2]
    if (shift > 1) v = swap_add<0x4e>(v);           // quad_perm [2, 3, 0, 1]
    if (shift > 2) v = swap_add<0x141>(v);          // row_half_mirror
    if (shift > 3) v = swap_add<0x140>(v);          // row_mirror
    for (int off = 16; off < (1 << shift); off <<= 1) {
        const uint32_t lo = __shfl_xor((uint32_t)v, off, 64), hi = __shfl_xor((uint32_t)(v >> 32), off, 64);
        v += ((u64)hi << 32) | lo;
    }
    return v;
}

// exclusive prefix sum over the workgroup's threads in thread order; `total` = sum over all threads
__device__ __forceinline__ u64 block_exclusive_scan(u64 v, u64* wave_sums /* LDS, kWaves + 1 */, u64& total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const u64 incl = wave_inclusive_scan(v);
    __syncthreads();                       // the previous use of wave_sums is over
    if (lane == 63) wave_sums[wave] = incl;
    __syncthreads();
    u64 before = 0, all = 0;
    for (int w = 0; w < kWaves; w++) {
        if (w < wave) before += wave_sums[w];
        all += wave_sums[w];
    }
    total = all;
    return before + incl - v;
}

struct Found {
    int bucket;      // first bucket (walking from the highest down) at which the cumulative mass meets the condition
    u64 above;       // mass of everything before that bucket, `base` included
};

// The buckets of `hist` (LDS, nb of them) are walked in the order of falling logits -- from the highest bucket down
// (descending) or from bucket 0 up -- starting at cumulative mass `base`; the crossing is the first bucket whose
// inclusive cumulative mass C has double(C) >= thr (strict: > thr).  Every thread returns the same answer; bucket =
// -1 if no bucket meets the condition (the callers never ask for that).
__device__ __forceinline__ Found find_crossing(const u64* hist, int nb, bool descending, u64 base, double thr, bool strict,
                                      u64* wave_sums, int* out_bucket, u64* out_above) {
    const int per = nb / kThreads, tid = threadIdx.x;
    // this thread's buckets, in walking order: first, first + step, ...
    const int first = descending ? nb - 1 - tid * per : tid * per, step = descending ? -1 : 1;
    u64 mine = 0;
    for (int i = 0; i < per; i++) mine += hist[first + i * step];
    u64 total;
    u64 cum = base + block_exclusive_scan(mine, wave_sums, total);
    auto met = [&](u64 c) { return strict ? (double)c > thr : (double)c >= thr; };
    if (tid == 0) *out_bucket = -1;
    __syncthreads();
    if (!met(cum) && met(cum + mine)) {    // the crossing lies in this thread's buckets: exactly one thread gets here
        for (int i = 0; i < per; i++) {
            const u64 next = cum + hist[first + i * step];
            if (met(next)) {
                *out_bucket = first + i * step;
                *out_above = cum;
                break;
            }
            cum = next;
        }
    }
    __syncthreads();
    Found f;
    f.bucket = *out_bucket;
    f.above = *out_above;
    return f;
}

// smallest r in [1, ties] with met(above + r * each); the caller knows that r = ties meets it
__device__ inline u64 rank_among_equals(u64 above, u64 each, u64 ties, double thr, bool strict) {
    auto met = [&](u64 r) { const u64 c = above + r * each; return strict ? (double)c > thr : (double)c >= thr; };
    const double gap = thr - (double)above;
    u64 r = 1;
    if (gap > 0.0) {
        const double q = gap / (double)each;
        r = q >= (double)ties ? ties : (u64)q;
    }
    r = r < 1 ? 1 : (r > ties ? ties : r);
    while (r > 1 && met(r - 1)) r--;
    while (r < ties && !met(r)) r++;
    return r;
}

// Masses of the tokens of cell `cell` by a field of their keys (nb buckets from bit `shift`), among the tokens whose key
// bits from want_shift up equal `want` (want_shift 32: all of them), straight from the row: the path for a cell
// with more tokens than the list in LDS holds (thousands of equal or nearly equal logits).  Every token is weighed
// again here; kept out of line so that the usual path does not carry its code.
__device__ __forceinline__ void fill_from_row(u64* hist, int nb, int shift, uint32_t want, int want_shift, const float* g, int V,
                                           int cell, float top, float scale, double c) {
    for (int i = threadIdx.x; i < V; i += kThreads) {
        const float x = g[i];
        const uint32_t k = key_of(x);
        if (cell_of(x, top, scale) == cell && (want_shift >= 32 || (k >> want_shift) == want)) {
            const u64 wt = weight_of(x, top, c);
            if (wt) atomicAdd(&hist[(k >> shift) & (uint32_t)(nb - 1)], wt);
        }
    }
}

struct SampleParams {
    const float* logits;
    int64_t stride;
    const float* u;
    int32_t* ids;
    u64* ws;              // [R][kRowWords]
    int32_t R, V, slices, slice_len;
    double c;             // log2(e) / temperature
    float scale;          // cells per unit of logit: c * 2047 / 36.5 (weights are zero from 36 binary orders below the top)
    double top_p;
};

// Phase 0: slice maxima, and the row's histogram and ticket put to zero (the workspace needs no initialisation).
__global__ __launch_bounds__(kThreads) void sample_prepare_kernel(SampleParams p) {
    __shared__ float red[kWaves];
    const int row = blockIdx.x / p.slices, slice = blockIdx.x % p.slices, tid = threadIdx.x;
    const float* g = p.logits + (int64_t)row * p.stride;
    u64* w = p.ws + (int64_t)row * kRowWords;
    float mx = -INFINITY;
    for_each_token(g, slice * p.slice_len, min(p.V, (slice + 1) * p.slice_len), [&](int, float x) { mx = fmaxf(mx, x); });
    mx = wave_max(mx);
    if ((tid & 63) == 0) red[tid >> 6] = mx;
    // this workgroup's share of the histogram's buckets
    const int share = (kL1 + p.slices - 1) / p.slices;
    for (int b = slice * share + tid; b < min(kL1, (slice + 1) * share); b += kThreads) w[b] = 0ull;
    __syncthreads();
    if (tid == 0) {
        for (int i = 1; i < kWaves; i++) mx = fmaxf(mx, red[i]);
        ((float*)(w + kL1))[slice] = mx;
        if (slice == 0) w[kL1 + 31] = 0ull;                   // the ticket
    }
}

// LDS of the kernels that search a row
struct SelectLds {
    u64 h1[kL1];                    // masses per cell
    u64 h2[kL2];                    // (large cells only) masses by key bits
    u64 h3[kL3];
    int cnt[kMaxVocab / 64];        // (large cells only) per group of 64 tokens: matches, then their prefix sum
    uint32_t list_k[kCap];          // the tokens of one cell, in no particular order: key, index, weight
    int list_i[kCap];
    u64 list_w[kCap];
    u64 wave_sums[kWaves + 1];
    // per descent (0: nucleus, 1: draw), so that no thread still reads the first's while the second's are set:
    u64 above[2];
    u64 mass[2];                    // cumulative mass up to and including the crossing token
    int bucket[2];
    int n[2];                       // tokens in the cell
    int found[2];                   // index of the crossing token, -1: none
    int last;
    float red[kWaves];
};

// A cell with more tokens than the list holds (thousands of equal or nearly equal logits): three levels of key bits
// inside the cell, masses straight from the row in memory, then the rank among equal logits by integer arithmetic and
// (want_token) the token of that rank.  false: a step that cannot fail did.
__device__ __forceinline__ bool descend_large_cell(const SampleParams& p, const float* g, SelectLds& l, int cell, float top,
                                                u64 above, double thr, bool strict, int pass, u64& mass, int& token) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t want = 0;
    bool ok = true;
    for (int level = 0; level < 3 && ok; level++) {
        u64* hist = level < 2 ? l.h2 : l.h3;
        const int nb = level < 2 ? kL2 : kL3, shift = level == 0 ? 21 : (level == 1 ? 10 : 0);
        const int want_shift = level == 0 ? 32 : (level == 1 ? 21 : 10);
        for (int b = tid; b < nb; b += kThreads) hist[b] = 0ull;
        __syncthreads();
        fill_from_row(hist, nb, shift, want, want_shift, g, p.V, cell, top, p.scale, p.c);
        __syncthreads();
        const Found f = find_crossing(hist, nb, true, above, thr, strict, l.wave_sums, &l.bucket[pass], &l.above[pass]);
        ok = f.bucket >= 0;
        above = f.above;
        want = level == 0 ? (uint32_t)f.bucket : (level == 1 ? (want << 11) | (uint32_t)f.bucket : (want << 10) | (uint32_t)f.bucket);
    }
    if (!ok) return false;
    const uint32_t key = want;
    const u64 each = weight_of(logit_of_key(key), top, p.c);  // equal keys are equal logits, hence equal weights
    const u64 ties = each ? l.h3[key & (kL3 - 1)] / each : 0ull;
    __syncthreads();                              // h3 is read above by every thread before anyone reuses it
    if (ties == 0) return false;
    const u64 r = rank_among_equals(above, each, ties, thr, strict);
    mass = above + r * each;
    if (pass == 0) return true;
    // the token: the r-th smallest index among the tokens with this key.  Matches are counted per group of 64
    // consecutive tokens, the counts are scanned, and the match of that rank reports itself.
    for (int j = tid; j < kMaxVocab / 64; j += kThreads) l.cnt[j] = 0;
    __syncthreads();
    for (int step = 0; step < 2; step++) {
        for (int i0 = wave * 64; i0 < p.V; i0 += kThreads) {
            const int i = i0 + lane;
            const bool m = i < p.V && key_of(g[i]) == key;
            const u64 ballot = __ballot(m);
            if (step == 0) {
                if (lane == 0) l.cnt[i0 >> 6] = __popcll(ballot);
            } else if (m && (u64)(l.cnt[i0 >> 6] + __popcll(ballot & ((1ull << lane) - 1ull))) + 1 == r) {
                l.found[1] = i;
            }
        }
        __syncthreads();
        if (step == 0) {
            constexpr int kPer = (kMaxVocab / 64) / kThreads;          // 2
            u64 mine = 0;
            for (int j = 0; j < kPer; j++) mine += (u64)l.cnt[tid * kPer + j];
            u64 all;
            u64 run = block_exclusive_scan(mine, l.wave_sums, all);
            for (int j = 0; j < kPer; j++) {
                const int c = l.cnt[tid * kPer + j];
                l.cnt[tid * kPer + j] = (int)run;
                run += (u64)c;
            }
            __syncthreads();
        }
    }
    if (l.found[1] < 0) return false;
    token = l.found[1];
    return true;
}

// Two descents by the same code, first the nucleus (the shortest prefix with mass >= top_p * total), then the draw
// (the first token with cumulative mass > u * nucleus mass).  A descent finds the cell in which the cumulative
// mass (highest logit first) meets the threshold -- cross(thr, strict), the same answer in every thread --, gathers
// that cell's tokens -- tens of them, as a rule -- into the list in LDS -- gather(cell, pass); l.n[pass] counts them,
// also those beyond the list's end --, weighs them, and lets every listed token add up the mass of the listed tokens that come
// before it in the order (higher logit, or equal logit and smaller index): the crossing token is the one whose own
// weight carries the cumulative mass over the threshold.  Returns the draw, or 0 if a step that cannot fail did; with
// kStopAtLargeCell, -1 as soon as a cell has more tokens than the list holds (the caller then starts again by
// descents_from_memory, whose code and registers the usual path does not have to carry).
template <bool kStopAtLargeCell, typename Cross, typename Gather>
__device__ __forceinline__ int two_descents(const SampleParams& p, const float* g, float u, SelectLds& l, float top, u64 total,
                                            Cross cross, Gather gather) {
    const int tid = threadIdx.x;
    __syncthreads();                                      // whoever read these words before is done with them
    if (tid < 2) {
        l.n[tid] = 0;
        l.found[tid] = -1;
        l.bucket[tid] = -1;
    }
    __syncthreads();
    double thr = p.top_p * (double)total;
    bool strict = false;
    int token = 0;
    for (int pass = 0; pass < 2; pass++) {
        auto met = [&](u64 cm) { return strict ? (double)cm > thr : (double)cm >= thr; };
        const Found f1 = cross(pass, thr, strict);
        if (f1.bucket < 0) break;                         // cannot happen: the thresholds used here are always met
        const int cell = f1.bucket;
        gather(cell, pass);
        __syncthreads();
        const int n = l.n[pass];
        u64 mass = 0;
        if (n <= kCap) {
            if (tid < n) l.list_w[tid] = weight_of(logit_of_key(l.list_k[tid]), top, p.c);
            __syncthreads();
            // listed token e = tid / group: the group's threads share the walk over the list (a power of two of
            // neighbouring lanes, as many as 1024 threads allow for n tokens, so a group never leaves its wavefront)
            int shift = 0;                                // group = 2^shift threads
            while (shift < 6 && (n << (shift + 1)) <= kThreads) shift++;
            const int e = tid >> shift, sub = tid & ((1 << shift) - 1);
            u64 before = 0;
            uint32_t k = 0;
            int i = 0;
            if (e < n) {
                k = l.list_k[e];
                i = l.list_i[e];
                for (int f = sub; f < n; f += 1 << shift) {
                    const uint32_t kf = l.list_k[f];
                    if (kf > k || (kf == k && l.list_i[f] < i)) before += l.list_w[f];
                }
            }
            before = group_sum(before, shift);
            if (e < n && sub == 0) {
                before += f1.above;
                const u64 mine = l.list_w[e];
                if (!met(before) && met(before + mine)) {
                    l.found[pass] = i;
                    l.mass[pass] = before + mine;
                }
            }
            __syncthreads();
            if (l.found[pass] < 0) break;                 // cannot happen
            token = l.found[pass];
            mass = l.mass[pass];
        } else if (kStopAtLargeCell) {
            return -1;
        } else if (!descend_large_cell(p, g, l, cell, top, f1.above, thr, strict, pass, mass, token)) {
            break;
        }
        if (pass == 0) {
            thr = (double)u * (double)mass;               // mass: the nucleus mass
            strict = true;
            token = 0;
        }
    }
    return token;
}

// Both descents with the row read from memory: l.h1 holds the row's masses per cell, `total` their sum.
__device__ __forceinline__ int descents_from_memory(const SampleParams& p, const float* g, float u, SelectLds& l, float top, u64 total) {
    const int tid = threadIdx.x, lane = tid & 63;
    return two_descents<false>(
        p, g, u, l, top, total,
        [&](int pass, double thr, bool strict) {
            return find_crossing(l.h1, kL1, false, 0ull, thr, strict, l.wave_sums, &l.bucket[pass], &l.above[pass]);
        },
        [&](int cell, int pass) {                         // one walk over the row
            for (int base = 0; base < p.V; base += kThreads * kBatch) {
                float xs[kBatch];
#pragma unroll
                for (int j = 0; j < kBatch; j++) {
                    const int i = base + j * kThreads + tid;
                    xs[j] = i < p.V ? g[i] : 0.f;
                }
#pragma unroll
                for (int j = 0; j < kBatch; j++) {
                    const int i = base + j * kThreads + tid;
                    const bool m = i < p.V && cell_of(xs[j], top, p.scale) == cell;
                    const u64 ballot = __ballot(m);
                    if (ballot) {                          // one counter update per wavefront and step
                        int start = 0;
                        if (lane == 0) start = atomicAdd(&l.n[pass], __popcll(ballot));
                        start = __shfl(start, 0, 64);
                        const int pos = start + __popcll(ballot & ((1ull << lane) - 1ull));
                        if (m && pos < kCap) {
                            l.list_k[pos] = key_of(xs[j]);
                            l.list_i[pos] = i;
                        }
                    }
                }
            }
        });
}

__global__ __launch_bounds__(kThreads) void sample_select_kernel(SampleParams p) {
    __shared__ SelectLds l;
    const int row = blockIdx.x / p.slices, slice = blockIdx.x % p.slices, tid = threadIdx.x, lane = tid & 63;
    const float* g = p.logits + (int64_t)row * p.stride;
    u64* w = p.ws + (int64_t)row * kRowWords;

    float top = -INFINITY;
    {
        float tops[kMaxSlices];                           // all reads in flight together
#pragma unroll
        for (int sidx = 0; sidx < kMaxSlices; sidx++) tops[sidx] = sidx < p.slices ? ((const float*)(w + kL1))[sidx] : -INFINITY;
#pragma unroll
        for (int sidx = 0; sidx < kMaxSlices; sidx++) top = fmaxf(top, tops[sidx]);
    }

    // ---- all workgroups: masses of this slice per cell, into LDS, then the non-empty cells into the row's histogram
    // in memory
    for (int b = tid; b < kL1; b += kThreads) l.h1[b] = 0ull;
    __syncthreads();
    for_each_token(g, slice * p.slice_len, min(p.V, (slice + 1) * p.slice_len), [&](int, float x) {
        const u64 wt = weight_of(x, top, p.c);
        if (wt) atomicAdd(&l.h1[cell_of(x, top, p.scale)], wt);
    });
    __syncthreads();
    for (int b = tid; b < kL1; b += kThreads) {
        const u64 v = l.h1[b];
        if (v) (void)__hip_atomic_fetch_add(w + b, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    // The adds above are device-scope atomics (performed where every compute unit sees them); each wavefront waits
    // until its own have been acknowledged, the workgroup meets, and only then its arrival is counted: whoever counts
    // the last arrival finds every slice's masses in the histogram.
    __builtin_amdgcn_s_waitcnt(0x0F70);                 // vmcnt(0)
    __syncthreads();
    if (tid == 0) {
        const u64 old = __hip_atomic_fetch_add(w + kL1 + 31, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        l.last = old + 1 == (u64)p.slices ? 1 : 0;
    }
    __syncthreads();
    if (!l.last) return;

    // ---- the row's last workgroup
    u64 part = 0;
    for (int b = tid; b < kL1; b += kThreads) {
        const u64 v = __hip_atomic_load(w + b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        l.h1[b] = v;
        part += v;
    }
    u64 total;
    (void)block_exclusive_scan(part, l.wave_sums, total);
    __syncthreads();

    const int token = descents_from_memory(p, g, p.u[row], l, top, total);
    if (tid == 0) p.ids[row] = token;
}

// ---- a row of at most kRowCap logits: one workgroup, the row in registers.  Thread t holds the tokens
// 4 (t + 1024 j) + e, j < 8, e < 4 (row_index), read as 16-byte groups when the rows' addresses and length allow it
// (kAligned: rows start at multiples of 16 bytes and hold a multiple of 4 tokens).
constexpr int kRowVec = 8;
constexpr int kRowPer = 4 * kRowVec;
constexpr int kRowCap = kThreads * kRowPer;       // 32768

__device__ inline int row_index(int tid, int k) { return 4 * (tid + kThreads * (k >> 2)) + (k & 3); }

template <bool kAligned>
__global__ __launch_bounds__(kThreads) void sample_row_kernel(SampleParams p) {
    __shared__ SelectLds l;
    const int row = blockIdx.x, tid = threadIdx.x;
    const float* g = p.logits + (int64_t)row * p.stride;

    const float u = p.u[row];                   // needed late, read early
    // Every read is unconditional and lands inside the row (a place beyond the row's end reads the row's last group or
    // token instead and then holds -inf), so that all of them are in flight together.
    float x[kRowPer];
#pragma unroll
    for (int j = 0; j < kRowVec; j++) {
        const int i0 = row_index(tid, 4 * j);
        if (kAligned) {                             // V is a multiple of 4 here: a group lies inside the row or outside
            const float4 v = *(const float4*)(g + min(i0, p.V - 4));
            const bool in = i0 < p.V;
            x[4 * j] = in ? v.x : -INFINITY;
            x[4 * j + 1] = in ? v.y : -INFINITY;
            x[4 * j + 2] = in ? v.z : -INFINITY;
            x[4 * j + 3] = in ? v.w : -INFINITY;
        } else {
#pragma unroll
            for (int e = 0; e < 4; e++) {
                const float v = g[min(i0 + e, p.V - 1)];
                x[4 * j + e] = i0 + e < p.V ? v : -INFINITY;
            }
        }
    }
    for (int b = tid; b < kL1; b += kThreads) l.h1[b] = 0ull;

    // the row's largest logit
    float top = -INFINITY;
#pragma unroll
    for (int k = 0; k < kRowPer; k++) top = fmaxf(top, x[k]);
    top = wave_max(top);
    if ((tid & 63) == 0) l.red[tid >> 6] = top;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kWaves; i++) top = fmaxf(top, l.red[i]);

    // weights into the cells' masses; every token's cell is kept, two to a register.  A place beyond the row's end
    // holds -inf: no weight, and the last cell, which has no mass and is never searched.
    uint32_t cells[kRowPer / 2];
#pragma unroll
    for (int k = 0; k < kRowPer; k++) {
        uint32_t cell = kL1 - 1;
        if (row_index(0, k & ~3) < p.V) {       // (the same for all threads) this group of 4096 places holds tokens at all
            cell = (uint32_t)cell_of(x[k], top, p.scale);
            const u64 wt = weight_of(x[k], top, p.c);
            if (wt) atomicAdd(&l.h1[cell], wt);
        }
        cells[k >> 1] = (k & 1) ? (cells[k >> 1] | (cell << 16)) : cell;
        __builtin_amdgcn_sched_barrier(0);      // one token after the other: interleaved, their fp64 temporaries do not fit the registers
    }
    __syncthreads();

    // cumulative masses, once for both descents: this thread's cells are 2 tid and 2 tid + 1
    const u64 c0 = l.h1[2 * tid], c1 = l.h1[2 * tid + 1];
    u64 total;
    const u64 before = block_exclusive_scan(c0 + c1, l.wave_sums, total);

    int token = two_descents<true>(
        p, g, u, l, top, total,
        [&](int pass, double thr, bool strict) {
            auto met = [&](u64 cm) { return strict ? (double)cm > thr : (double)cm >= thr; };
            if (!met(before) && met(before + c0 + c1)) {      // exactly one thread gets here
                const bool first = met(before + c0);
                l.bucket[pass] = 2 * tid + (first ? 0 : 1);
                l.above[pass] = first ? before : before + c0;
            }
            __syncthreads();
            Found f;
            f.bucket = l.bucket[pass];
            f.above = l.above[pass];
            return f;
        },
        [&](int cell, int pass) {
            const uint32_t both = (uint32_t)cell * 0x10001u;
            auto put = [&](int k) {                        // rare: kept out of the way of the 32 comparisons
                float xv = x[k];
                asm volatile("" : "+v"(xv));               // (nothing of this is worked out ahead for all 32 tokens)
                const int pos = atomicAdd(&l.n[pass], 1);
                if (pos < kCap) {
                    l.list_k[pos] = key_of(xv);
                    l.list_i[pos] = row_index(tid, k);
                }
            };
#pragma unroll
            for (int j = 0; j < kRowPer / 2; j++) {
                const uint32_t t = cells[j] ^ both;        // a half that is zero: that token lies in the cell
                if ((uint16_t)t == 0) put(2 * j);
                if (t < 0x10000u) put(2 * j + 1);
            }
        });
    if (token < 0) token = descents_from_memory(p, g, u, l, top, total);      // a cell of thousands of tokens
    if (tid == 0) p.ids[row] = token;
}

}  // namespace

extern "C" __attribute__((visibility("default"))) size_t rest_sample_ids_workspace_bytes(int32_t R, int32_t V) {
    if (R < 0 || V < 1 || V > kMaxVocab) return 0;
    return (size_t)R * kRowWords * sizeof(u64);
}

extern "C" __attribute__((visibility("default"))) rest_status rest_sample_ids(const float* d_logits, int64_t row_stride, const float* d_u, int32_t R,
                                       int32_t V, float temperature, float top_p, int32_t* d_ids, void* d_workspace,
                                       size_t workspace_bytes, void* stream) {
    if (!d_logits || !d_u || !d_ids) return REST_INVALID_ARG;
    if (R < 0 || V < 1 || row_stride < V) return REST_INVALID_ARG;
    if (!(temperature > 0.f) || !(temperature < 1e30f) || !(top_p > 0.f) || !(top_p <= 1.f)) return REST_INVALID_ARG;
    if (V > kMaxVocab) return REST_UNSUPPORTED;
    if (R == 0) return REST_OK;
    const size_t need = rest_sample_ids_workspace_bytes(R, V);
    if (!d_workspace || workspace_bytes < need) return REST_WORKSPACE_TOO_SMALL;
    if ((uintptr_t)d_workspace & 7) return REST_INVALID_ARG;
    const Slicing sl = slicing_of(R, V);
    if ((int64_t)R * sl.slices > 0x7fffffff) return REST_INVALID_ARG;
    SampleParams p;
    p.logits = d_logits;
    p.stride = row_stride;
    p.u = d_u;
    p.ids = d_ids;
    p.ws = (u64*)d_workspace;
    p.R = R;
    p.V = V;
    p.slices = sl.slices;
    p.slice_len = sl.slice_len;
    p.c = 0x1.71547652b82fep+0 / (double)temperature;         // log2(e) / temperature, one fp64 division
    p.scale = (float)(p.c * (2047.0 / 36.5));
    p.top_p = (double)top_p;
    if (V <= kRowCap) {                                       // the row fits one workgroup's registers
        if (((uintptr_t)d_logits & 15) == 0 && (row_stride & 3) == 0 && (V & 3) == 0)
            hipLaunchKernelGGL(sample_row_kernel<true>, dim3(R), dim3(kThreads), 0, (hipStream_t)stream, p);
        else
            hipLaunchKernelGGL(sample_row_kernel<false>, dim3(R), dim3(kThreads), 0, (hipStream_t)stream, p);
        REST_HIP_TRY(hipGetLastError());
        return REST_OK;
    }
    hipLaunchKernelGGL(sample_prepare_kernel, dim3(R * p.slices), dim3(kThreads), 0, (hipStream_t)stream, p);
    REST_HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL(sample_select_kernel, dim3(R * p.slices), dim3(kThreads), 0, (hipStream_t)stream, p);
    REST_HIP_TRY(hipGetLastError());
    return REST_OK;
}
