// Nucleus sampling of the model's token at every position of the verification pass (REST, arXiv 2311.08252,
// "Sampling strategies"; temperature and top-p as in the caption of the main speed table).  REST accepts a draft
// token only if it equals the token sampled at its position, so the ids written here feed rest_accept unchanged.
//
// Definition (the paper fixes the parameters, not the mechanics): probabilities = softmax(logits / temperature);
// tokens ordered by probability, highest first, equal probabilities by ascending token id; the nucleus is the
// shortest prefix of that order whose mass reaches top_p; the draw is the first token whose cumulative mass
// exceeds u times the nucleus mass, u in [0, 1) given by the caller.
//
// One 512-thread workgroup per position; a thread keeps its 64 logits (as order-preserving 32-bit keys) and their
// exponentials (fp64) in registers.  Nothing is sorted: "the place in the sorted order where the cumulative mass
// crosses a threshold" is found by descending the key four bits at a time.  At each level every thread adds its
// matching elements into 16 private fp64 slots in LDS (no atomics, no conflicts), each bucket is summed over the
// threads by one wavefront in a fixed order, and every thread walks the 16 bucket masses from the top.  Eight levels pin the key;
// equal keys are then resolved arithmetically (their masses are equal) and by ascending token id through ballots.
// All sums have a fixed order, so results repeat bit for bit from run to run.
#include <mutex>

#include "common.h"

namespace {

constexpr int kThreads = 512;            // 8 wavefronts: 256 VGPRs each, room for 64 keys and 64 fp64 masses
constexpr int kPer = 64;                 // elements per thread: V <= 32768
constexpr int kWaves = kThreads / 64;

__device__ inline uint32_t key_of(float x) {
    if (x == 0.f) x = 0.f;               // -0 and +0 are the same logit
    const uint32_t b = __builtin_bit_cast(uint32_t, x);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ inline float float_of(uint32_t k) {
    const uint32_t b = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
    return __builtin_bit_cast(float, b);
}

struct Crossing {
    uint32_t key;       // key of the element at which the cumulative mass crosses the target
    double above;       // mass of all elements with a larger key
    long long rank;     // 1-based position of the crossing element among those with this key
    long long ties;     // number of elements with this key
    double each;        // mass of one of them
    bool found;
};

__global__ __launch_bounds__(kThreads) void sample_kernel(const float* logits, int64_t stride, const float* u, int V,
                                                          double temperature, double top_p, int32_t* ids) {
    extern __shared__ double acc[];                    // [16][kThreads]
    __shared__ double level_mass[8][16];   // bucket masses of the first descent, per level
    __shared__ double scratch_mass[16];
    __shared__ uint32_t level_prefix[8];
    __shared__ float red_f[kWaves];
    __shared__ int red_i[kWaves];
    __shared__ int row_cnt[kPer][kWaves];
    __shared__ int pick[3];
    if (threadIdx.x == 0) { pick[0] = 0; pick[1] = 0; pick[2] = 1; }
    const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float* g = logits + (int64_t)row * stride;

    uint32_t key[kPer];
    double e[kPer];
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < kPer; i++) {
        const int j = i * kThreads + tid;
        const float x = j < V ? g[j] : -INFINITY;
        key[i] = j < V ? key_of(x) : 0u;       // key 0 (a NaN pattern) marks padding: mass 0, never a crossing key
        mx = fmaxf(mx, x);
    }
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
    if (lane == 0) red_f[wave] = mx;
    __syncthreads();
    for (int w = 0; w < kWaves; w++) mx = fmaxf(mx, red_f[w]);
    const double zmax = (double)mx / temperature;
#pragma unroll
    for (int i = 0; i < kPer; i++) {
        const int j = i * kThreads + tid;
        e[i] = j < V ? exp((double)float_of(key[i]) / temperature - zmax) : 0.0;
    }

    // descends the key to the element where the cumulative mass (largest key first) first reaches (strict: exceeds)
    // `target`.  A recording descent keeps the bucket masses of its levels (1 KB); a later descent reuses them for as
    // long as it follows the same prefix -- usually through the first levels (sign and exponent bits), which are the
    // expensive ones because nearly every element takes part in them.
    int levels_kept = 0;                           // same value in every thread
    auto select = [&](double target, bool strict, bool record) -> Crossing {
        Crossing c{};
        uint32_t prefix = 0;
        double cum = 0.0;
        c.found = true;
        bool follow = true;
        for (int lvl = 0; lvl < 8; lvl++) {
            const double* masses = &level_mass[lvl][0];
            follow = follow && lvl < levels_kept && level_prefix[lvl] == prefix;
            if (!follow) {
#pragma unroll
                for (int d = 0; d < 16; d++) acc[d * kThreads + tid] = 0.0;
                const int sh = 28 - 4 * lvl;
#pragma unroll
                for (int i = 0; i < kPer; i++) {
                    const bool match = lvl == 0 || (key[i] >> (sh + 4)) == prefix;
                    // a private slot: the atomic is only a read-modify-write the wavefront need not wait for
                    if (match)
                        __hip_atomic_fetch_add(&acc[((key[i] >> sh) & 15u) * kThreads + tid], e[i], __ATOMIC_RELAXED,
                                               __HIP_MEMORY_SCOPE_WORKGROUP);
                }
                __syncthreads();
                double* dst = record ? &level_mass[lvl][0] : &scratch_mass[0];
                for (int b = wave; b < 16; b += kWaves) {
                    double s = 0.0;
#pragma unroll
                    for (int t = 0; t < kThreads / 64; t++) s += acc[b * kThreads + lane + 64 * t];
                    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
                    if (lane == 0) dst[b] = s;
                }
                if (record) {
                    if (tid == 0) level_prefix[lvl] = prefix;
                    levels_kept = lvl + 1;          // deeper kept levels belonged to another prefix
                }
                __syncthreads();
                masses = dst;
            }
            int d = 15;
            for (; d >= 0; d--) {
                const double next = cum + masses[d];
                if (strict ? next > target : next >= target) break;
                cum = next;
            }
            if (d < 0) {            // rounding left the total just under the target
                c.found = false;
                c.above = cum;
                return c;
            }
            prefix = (prefix << 4) | (uint32_t)d;
        }
        c.key = prefix;
        c.above = cum;
        // elements with this key: how many, and which of them is the crossing one
        int n = 0;
#pragma unroll
        for (int i = 0; i < kPer; i++) n += __popcll(__ballot(key[i] == prefix));
        if (lane == 0) red_i[wave] = n;
        __syncthreads();
        long long ties = 0;
        for (int w = 0; w < kWaves; w++) ties += red_i[w];
        __syncthreads();
        c.ties = ties;
        c.each = exp((double)float_of(prefix) / temperature - zmax);
        long long r = 1;
        if (c.each > 0.0) {
            const double q = (target - cum) / c.each;
            r = strict ? (long long)floor(q) + 1 : (long long)ceil(q);
        }
        r = r < 1 ? 1 : (r > ties ? ties : r);
        auto reached = [&](long long k) { const double m = cum + (double)k * c.each; return strict ? m > target : m >= target; };
        while (r > 1 && reached(r - 1)) r--;
        while (r < ties && !reached(r)) r++;
        c.rank = r;
        return c;
    };

    // the nucleus and its mass.  The total is the sum of the level-0 bucket masses in the order of a descent's walk,
    // so the first descent is run with an unreachable target and stops after that level.
    const double total = select(INFINITY, false, true).above;
    // the nucleus descent reuses level 0 and records its own deeper levels; the draw follows it while it can
    const Crossing nuc = select(top_p * total, false, true);
    const double mass = nuc.found ? nuc.above + (double)nuc.rank * nuc.each : nuc.above;
    Crossing hit = select((double)u[row] * mass, true, false);
    if (!hit.found) hit = nuc;                         // cannot happen for u < 1 except through rounding
    if (!hit.found) {                                  // nor this: the total is positive
        if (tid == 0) ids[row] = 0;
        return;
    }

    // token id = the hit.rank-th smallest index among the elements with key hit.key; index = i * kThreads + tid
#pragma unroll
    for (int i = 0; i < kPer; i++) {
        const uint64_t b = __ballot(key[i] == hit.key);
        if (lane == 0) row_cnt[i][wave] = __popcll(b);
    }
    __syncthreads();
    if (wave == 0) {
        // kPer * kWaves = 512 counts in index order (i major, wavefront minor), 8 per lane
        static_assert(kPer * kWaves == 512, "eight counts per lane");
        const int* flat = &row_cnt[0][0];
        int mine = 0;
        for (int t = 0; t < 8; t++) mine += flat[lane * 8 + t];
        int incl = mine;
        for (int off = 1; off < 64; off <<= 1) {
            const int y = __shfl_up(incl, off, 64);
            if (lane >= off) incl += y;
        }
        const int before = incl - mine;
        const long long want = hit.rank;
        if ((long long)before < want && want <= (long long)incl) {
            int run = before;
            for (int t = 0; t < 8; t++) {
                const int c = flat[lane * 8 + t];
                if ((long long)(run + c) >= want) {
                    pick[0] = (lane * 8 + t) / kWaves;        // i
                    pick[1] = (lane * 8 + t) % kWaves;        // wavefront
                    pick[2] = (int)(want - run);               // 1-based among that ballot's set bits
                    break;
                }
                run += c;
            }
        }
    }
    __syncthreads();
    if (wave == pick[1]) {
        const int i_star = pick[0];
        bool m = false;
#pragma unroll
        for (int i = 0; i < kPer; i++)
            if (i == i_star) m = key[i] == hit.key;
        const uint64_t b = __ballot(m);
        const int below = __popcll(b & ((1ull << lane) - 1ull));
        if (m && below == pick[2] - 1) ids[row] = i_star * kThreads + tid;
    }
}

}  // namespace

extern "C" __attribute__((visibility("default"))) rest_status rest_sample_ids(const float* d_logits, int64_t row_stride, const float* d_u, int32_t R,
                                       int32_t V, float temperature, float top_p, int32_t* d_ids, void* stream) {
    if (!d_logits || !d_u || !d_ids) return REST_INVALID_ARG;
    if (R < 0 || V < 1 || row_stride < V) return REST_INVALID_ARG;
    if (!(temperature > 0.f) || !(temperature < 1e30f) || !(top_p > 0.f) || !(top_p <= 1.f)) return REST_INVALID_ARG;
    if (V > kThreads * kPer) return REST_UNSUPPORTED;
    if (R == 0) return REST_OK;
    const size_t lds = (size_t)16 * kThreads * sizeof(double);
    static bool granted[64] = {false};
    static std::mutex granted_lock;                 // host threads may call at once
    int dev = 0;
    REST_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return REST_UNSUPPORTED;
    {
        std::lock_guard<std::mutex> hold(granted_lock);
        if (!granted[dev]) {
            REST_HIP_TRY(hipFuncSetAttribute((const void*)sample_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
            granted[dev] = true;
        }
    }
    hipLaunchKernelGGL(sample_kernel, dim3(R), dim3(kThreads), lds, (hipStream_t)stream, d_logits, row_stride, d_u, V,
                       (double)temperature, (double)top_p, d_ids);
    REST_HIP_TRY(hipGetLastError());
    return REST_OK;
}
