// Tree-masked verification attention for gfx950 ("Draft verification" of REST, arXiv 2311.08252):
// every draft token attends to the whole cached context and, among the draft tokens, to itself and
// its ancestors only.
//
// bf16 kernel design (HBM-bound: ~T flop per KV byte, far below the chip's balance point):
//  * a unit is one (batch, head, group of 64 queries); its keys are cut into blocks of 32.  W streams share the
//    work, a stream being a workgroup of two wavefronts (wavefront w owns queries 32w .. 32w+31 of the unit).
//    (Described for up to 64 query rows; 128 / 256 rows per unit run on streams of four / eight wavefronts and
//    tiles of two / four blocks, see the kernel's template comment.  An 8-bit cache changes the fetch only.)
//    Stream s first takes whole units s, s + W, ... and writes their output directly; the blocks of the units
//    that are left over (fewer than W) are cut into equal contiguous spans, one per stream (stream-K), so every
//    stream gets the same number of blocks whatever the number of units.  Only a span that starts or ends inside
//    a unit leaves an fp32 partial (reference, sum, O), and a small second kernel merges those.  After at least
//    one whole round, W/2 or more units left over are not cut (two-wavefront streams on a 16-bit cache only): that
//    many streams take one more whole unit;
//  * a block's K and V (8 KB each) are fetched with coalesced 16-byte non-temporal loads one block ahead of the
//    arithmetic -- each wavefront fetches half of the tile --, wait in registers while in flight, and are then
//    parked in one of two LDS tiles shared by the two wavefronts (one workgroup barrier per block); the XOR
//    swizzle that keeps the LDS reads conflict free is applied by choosing which 16-byte piece of a row each
//    lane fetches, so the parking stores are plain lane-linear 16-byte writes;
//  * the query fragments stay in registers for a whole unit;
//  * S^T = K Q^T and O^T += V^T P^T run on v_mfma_f32_32x32x16_bf16.  With keys on the MFMA row axis a
//    lane owns one query column, so the softmax statistics are per lane; V^T fragments come out of LDS
//    through ds_read_b64_tr_b16; the probabilities go from the S accumulator straight into the B
//    operand of the second product (the key permutation this implies is applied to V^T as well);
//  * the softmax reference is only moved when a block's maximum exceeds it by more than 2^8, so the O
//    accumulators are rescaled a handful of times per unit instead of once per block (the result does not
//    depend on the reference);
//  * tree-mask bit rows are held in LDS and only consulted for blocks that reach past the prefix.
#include "common.h"
#include <mutex>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kD = 128;            // head dim
constexpr int kBlk = 32;           // keys per block
constexpr int kSubBytes = kBlk * kD * 2;    // 8 KB: K or V of one 32-key block in bf16
constexpr float kNegBig = -1.0e30f;
constexpr float kLazy = 8.0f;      // log2 units the running maximum may exceed the softmax reference
constexpr int kMaxWaves = 2048;    // wavefronts in flight: eight on each of 256 compute units
#ifdef REST_BOUNDS_CHECK
constexpr bool kBoundsChecked = true;    // K/V rows always go through the path that clamps them to the last key
#else
constexpr bool kBoundsChecked = false;
#endif

struct AttnParams {
    const __bf16* q;
    const __bf16* k;
    const __bf16* v;
    const uint64_t* mask;
    __bf16* out;
    float* ws_o;      // bf16 path: [W][2][QT*32][128] partial O; fp32 path: [rows][128]
    float* ws_ml;     // bf16 path: [W][2][QT*32][2] (reference in log2 units, sum); fp32 path: [rows][2]
    const float* k_scale;   // 8-bit cache only: [Nb*H] factors of the decoded K and V values, or null for 1
    const float* v_scale;
    int32_t Nb, H, Tq, Tk, P, Lk;
    int32_t nsplit, qgroups, mask_words, mask_per_batch;
    int32_t mask_rows;   // rows of one mask: query row i uses mask row i % mask_rows
    int32_t nblk;     // tiles per unit: ceil(Lk / (16 * wavefronts per stream))
    int32_t units;    // Nb * H * qgroups
    int32_t n_streams;  // W: streams (workgroups) that share the work
    // Work of stream w: whole units w, w + W, ... (dp_rounds of them), then its span of the tail, i.e. of the
    // blocks of the last tail_units units, which are cut into tail_streams contiguous spans (stream-K).
    int32_t dp_rounds, tail_units, tail_streams;
    // or, instead of a tail: extra_units whole units more, one each for the first extra_units streams in the order
    // "even streams, then odd streams"
    int32_t extra_units;
    float c;          // scale * log2(e)
    int64_t qs[3], ks[3], vs[3], os[3];
    // split plan (few units): every unit is shared by split_s workgroups of four key groups each
    int32_t split_s;               // workgroups per unit
    int32_t split_rounds;          // most blocks any key group gets: ceil(nblk / (4 split_s))
    __bf16* ws_po;                 // [units][split_s][64][128] normalised partial outputs
    unsigned long long* tickets;   // [units] arrival counters
};

__device__ inline float wave_xor32(float x) { return __shfl_xor(x, 32, 64); }

// first block of stream w when `total` blocks are cut into `n` contiguous spans
__host__ __device__ inline int64_t span_begin(int64_t total, int32_t n, int64_t w) { return (total * w) / n; }
// the stream whose span contains block b
__host__ __device__ inline int32_t span_owner(int64_t total, int32_t n, int64_t b) {
    return (int32_t)(((b + 1) * n - 1) / total);
}

// One block of 32 keys for the 32 queries of a wavefront: S^T = K Q^T, the tree mask for keys past the prefix,
// softmax numerators against the lazily updated reference, O^T += V^T P^T.  ldsK / ldsV: the block's K and V rows in
// LDS (256-byte rows, swizzled as the parking stores leave them); ka0, va0, vsw: the lane's operand read offsets;
// qf: the query fragments; o, m_ref (log2 units), l_run: the running output, reference and sum of this lane's query
// column; key0: index of the block's first key; mw: the four mask words of this lane's query row (in LDS).
//
// kPrio > 0: the wavefront runs its matrix instructions at issue priority kPrio and everything else at 0, so that
// of the two wavefronts of a SIMD the one that is in a run of matrix instructions keeps that pipe while the other
// one's exponentials fill the vector pipe.  Measured: 4-5 % on grouped-query units of 512 queries, 1-2 % on 128
// and 256 queries, nothing on 64.
template <bool kPairSwap, int kPrio = 0>
__device__ __forceinline__ void attn_block(const unsigned char* ldsK, const unsigned char* ldsV, const uint32_t ka0,
                                           const uint32_t va0, const uint32_t vsw, const int hh, const bf16x8 (&qf)[8],
                                           f32x16 (&o)[4], float& m_ref, float& l_run, const float cu, const int key0,
                                           const int P, const int Tk, const uint64_t* mw) {
    // ---- S^T[key][query] = K Q^T
    f32x16 s;
#pragma unroll
    for (int r = 0; r < 16; r++) s[r] = 0.f;
    if constexpr (kPrio > 0) __builtin_amdgcn_s_setprio(kPrio);
#pragma unroll
    for (int ks = 0; ks < 8; ks++) {
        const bf16x8 a = *(const bf16x8*)(ldsK + (ka0 ^ (ks << 5) ^ (kPairSwap ? (ks >> 2) << 4 : 0)));
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], s, 0, 0, 0);
    }
    // keep two K fragments in flight: read, read, then (multiply, read) ..., so that an LDS read's latency
    // hides behind the previous matrix instruction
    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
#pragma unroll
    for (int ks = 0; ks < 6; ks++) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
    if constexpr (kPrio > 0) __builtin_amdgcn_s_setprio(0);

    // ---- visibility (only blocks that reach past the prefix): one 32-bit word per lane says which of
    // the block's 32 keys its query sees; bit i <-> key j*32 + i
    if (key0 + kBlk > P) {
        const int kb = key0 - P;              // draft-token index of the block's first key (may be < 0)
        const int end = Tk - kb;              // keys at block offset >= end are past the last key
        const uint32_t in_range = end >= 32 ? 0xffffffffu : (end > 0 ? (1u << end) - 1u : 0u);
        uint32_t vbits;
        if (kb < 0) {
            vbits = ((1u << (-kb)) - 1u) | ((uint32_t)mw[0] << (-kb));
        } else {
            const int w = kb >> 6, sh = kb & 63;
            const uint64_t lo = mw[w];
            const uint64_t hi = (w + 1 < 4) ? mw[w + 1] : 0ull;
            vbits = (uint32_t)(lo >> sh);
            if (sh > 32) vbits |= (uint32_t)(hi << (64 - sh));
        }
        vbits &= in_range;
        vbits >>= 4 * hh;
#pragma unroll
        for (int r = 0; r < 16; r++) {
            const bool vis = (vbits >> (8 * (r >> 2) + (r & 3))) & 1u;
            s[r] = vis ? s[r] : -INFINITY;
        }
    }

    // ---- softmax numerators against a lazily updated reference, per lane = per query column
    bf16x8 pf[2];
    {
        float mx = s[0];
#pragma unroll
        for (int r = 1; r < 16; r++) mx = fmaxf(mx, s[r]);
        mx = fmaxf(mx, wave_xor32(mx)) * cu;
        if (__any(mx > m_ref + kLazy)) {
            const float m_new = fmaxf(m_ref, mx);
            const float alpha = __builtin_amdgcn_exp2f(m_ref - m_new);
            m_ref = m_new;
            l_run *= alpha;
#pragma unroll
            for (int dt = 0; dt < 4; dt++)
#pragma unroll
                for (int r = 0; r < 16; r++) o[dt][r] *= alpha;
        }
        float sum = 0.f;
#pragma unroll
        for (int r = 0; r < 16; r++) {
            const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], cu, -m_ref));
            sum += e;
            pf[r >> 3][r & 7] = (__bf16)e;
        }
        l_run += sum;
    }

    // ---- O^T[d][query] += V^T P^T
    if constexpr (kPrio > 0) __builtin_amdgcn_s_setprio(kPrio);
#pragma unroll
    for (int ss = 0; ss < 2; ss++) {
#pragma unroll
        for (int dt = 0; dt < 4; dt++) {
            const unsigned char* a0 = ldsV + ((va0 + ss * 4096 + ((((uint32_t)dt << 2) ^ vsw) << 4)) ^ (kPairSwap ? (dt >> 1) << 4 : 0));
            s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)a0);
            s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(a0 + 8 * 256));
            union { struct { s16x4 lo, hi; } sp; bf16x8 v; } u;
            u.sp.lo = lo;
            u.sp.hi = hi;
            o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(u.v, pf[ss], o[dt], 0, 0, 0);
        }
    }
    __builtin_amdgcn_sched_group_barrier(0x100, 4, 1);
#pragma unroll
    for (int i = 0; i < 6; i++) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 1);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 1);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 2, 1);
    if constexpr (kPrio > 0) __builtin_amdgcn_s_setprio(0);
}

// One stream = one workgroup of NW wavefronts (2, 4 or 8) for a unit of 32 NW queries: wavefront w owns queries
// [32w, 32w+32).  All see the same K/V tile in LDS, NW/2 blocks = 16 NW keys long, of which each wavefront fetches
// its 1/NW: eight 16-byte pieces per lane and tile whatever NW is, so the bytes in flight per compute unit (eight
// wavefronts: 2 per SIMD) do not depend on the number of queries, and every K/V byte is read once per unit.
//
// KV8: the cache holds OCP E4M3 bytes (128-byte rows).  A lane still fetches 16-byte pieces -- half as many per
// tile --, and turns each into two pieces of bf16 (exact: every E4M3 value is a bf16 value) on the way into the
// same LDS layout, so everything after the parking store is the bf16 kernel; the per-(batch, head) scales are
// folded into the softmax scale and into the final division.
template <int NW, bool KV8>
__global__ __launch_bounds__(64 * NW, 2) void tree_attn_bf16_kernel(AttnParams p) {
    constexpr int kElt = KV8 ? 1 : 2;                  // bytes per cached element
    constexpr int kFetch = KV8 ? 2 : 4;                // 16-byte pieces of K (and of V) a lane fetches per tile
    constexpr bool kPairSwap = KV8;                    // LDS rows hold pieces 8..15 with the slots of each pair swapped
    constexpr int kSub = NW / 2;                       // 32-key blocks per tile
    constexpr int kTileKeys = kSub * kBlk;
    constexpr int kTileBytes = kSub * kSubBytes;       // K (or V) part of a tile
    __shared__ __attribute__((aligned(1024))) unsigned char lds_tile[2][2 * kTileBytes];   // [buffer][K | V]
    __shared__ uint64_t lds_mask[NW * 32 * 4];                                              // query rows x 4 words

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int hh = lane >> 5;      // which half of the wave (selects the k-slice of MFMA operands)
    const int col = lane & 31;     // MFMA column = query within this wave's 32-query tile
    const int lrow = lane >> 4, lpc = lane & 15;

    const int gw = blockIdx.x;     // stream index
    // this stream's span [tb, te) of the tail blocks (< 2^31 of them; tail coordinates count from the first tail
    // unit).  Recomputed where needed rather than kept: the block loop is short of scalar registers.
    auto tail_span = [&](int& tb, int& te) {
        const int64_t t_total = (int64_t)p.tail_units * p.nblk;
        tb = te = 0;
        if (gw < p.tail_streams) {
            tb = (int)span_begin(t_total, p.tail_streams, gw);
            te = (int)span_begin(t_total, p.tail_streams, gw + 1);
        }
    };
    int blocks_left;                                            // blocks still to be requested
    {
        int tb, te;
        tail_span(tb, te);
        blocks_left = p.dp_rounds * p.nblk + (te - tb);
    }
    // place of this stream in the order in which streams take an extra unit
    const int extra_rank = (gw & 1) ? ((p.n_streams + 1) >> 1) + (gw >> 1) : gw >> 1;
    if (extra_rank < p.extra_units) blocks_left += p.nblk;
    if (blocks_left == 0) return;

    // The stream's segments, in order: blocks [0, nblk) of units gw, gw + W, ... (dp_rounds of them), then its extra
    // unit if it has one, or the pieces of its tail span [tb, te), one per tail unit it touches.  Two cursors walk them, one for the loads and, one
    // block behind, one for the arithmetic; each is a handful of scalars (kept out of structs so that they stay in
    // registers: a cursor in scratch memory would tie every step to the outstanding K/V loads).
#define REST_SEGMENT_FIRST(unit, j, je, round, tail)                                  \
    do {                                                                              \
        round = 0;                                                                    \
        if (p.dp_rounds > 0) {                                                        \
            tail = false; unit = gw; j = 0; je = p.nblk;                              \
        } else {                                                                      \
            tail = true;                                                              \
            int tb_, te_;                                                             \
            tail_span(tb_, te_);                                                      \
            const int ut_ = tb_ / p.nblk;                                             \
            unit = p.dp_rounds * p.n_streams + ut_; j = tb_ - ut_ * p.nblk;           \
            const int rest_ = te_ - ut_ * p.nblk;                                     \
            je = rest_ < p.nblk ? rest_ : p.nblk;                                     \
        }                                                                             \
    } while (0)
    // to the next segment; the caller knows from its block count that there is one
#define REST_SEGMENT_NEXT(unit, j, je, round, tail)                                   \
    do {                                                                              \
        if (!tail && ++round < p.dp_rounds) {                                         \
            unit += p.n_streams; j = 0;                                               \
        } else if (p.extra_units > 0) {                                               \
            unit = p.dp_rounds * p.n_streams + extra_rank; j = 0;                     \
        } else {                                                                      \
            int tb_, te_;                                                             \
            tail_span(tb_, te_);                                                      \
            const int u0_ = p.dp_rounds * p.n_streams;                                \
            if (!tail) {                                                              \
                tail = true;                                                          \
                const int ut_ = tb_ / p.nblk;                                         \
                unit = u0_ + ut_; j = tb_ - ut_ * p.nblk;                             \
            } else {                                                                  \
                unit++; j = 0;                                                        \
            }                                                                         \
            const int rest_ = te_ - (unit - u0_) * p.nblk;                            \
            je = rest_ < p.nblk ? rest_ : p.nblk;                                     \
        }                                                                             \
    } while (0)

    uint64_t* const my_mask = lds_mask + wave * (32 * 4);
    const int64_t k_row_bytes = p.ks[2] * kElt, v_row_bytes = p.vs[2] * kElt;

    // Global -> registers -> LDS.  Chunk i of a tile is 4 rows x 256 B = 64 lanes x 16 B and is parked at
    // tile + i*1024 + lane*16, i.e. row i*4 + (lane >> 4), piece slot lane & 15.  The slot holds row piece
    // (slot ^ swizzle(row)), so that is the piece this lane fetches.  K: swizzle = row & 15; V: (row & 3) << 2.
    // Wavefront w moves chunks 4w .. 4w+3 of K and of V.
    // KV8: chunk i is 8 rows x 128 B; the lane fetches piece lane & 7 of row i*8 + (lane >> 3) as it lies in memory
    // and applies the swizzle when it parks the two bf16 pieces made from it.  Wavefront w moves chunks 2w, 2w+1.
    uint32_t k_off[4];
#pragma unroll
    for (int x = 0; x < 4; x++)
        k_off[x] = KV8 ? (uint32_t)((lane >> 3) * k_row_bytes) + ((lane & 7) << 4)
                       : (uint32_t)(lrow * k_row_bytes) + ((lpc ^ (x * 4 + lrow)) << 4);
    const uint32_t v_off = KV8 ? (uint32_t)((lane >> 3) * v_row_bytes) + ((lane & 7) << 4)
                               : (uint32_t)(lrow * v_row_bytes) + ((lpc ^ (lrow << 2)) << 4);

    auto unit_bases = [&](int unit, const char*& kp, const char*& vp) {
        unit = (int)REST_IDX(unit, p.units, 3);
        const int slab = unit / p.qgroups;
        const int h = slab % p.H, nb = slab / p.H;
        kp = (const char*)p.k + (nb * p.ks[0] + h * p.ks[1]) * kElt;
        vp = (const char*)p.v + (nb * p.vs[0] + h * p.vs[1]) * kElt;
    };

    // ---- load side: a cursor one block ahead of the arithmetic
    int ld_unit, ld_j, ld_je, ld_round;
    bool ld_tail;
    REST_SEGMENT_FIRST(ld_unit, ld_j, ld_je, ld_round, ld_tail);
    const char *ld_kp, *ld_vp;
    unit_bases(ld_unit, ld_kp, ld_vp);
    i32x4 kr[kFetch], vr[kFetch];
    constexpr int kChunkRows = KV8 ? 8 : 4;            // rows of a 1 KB chunk
    auto issue = [&]() {
        const int j = ld_j;
        (void)REST_IDX((int64_t)j * kTileKeys, p.Lk, 2);       // a tile starts at a key that exists (a plan error if not)
        if (!kBoundsChecked && (j + 1) * kTileKeys <= p.Lk) {
#pragma unroll
            for (int i = 0; i < kFetch; i++) {
                const int64_t row = (int64_t)j * kTileKeys + (kFetch * wave + i) * kChunkRows;
                kr[i] = __builtin_nontemporal_load((const i32x4*)(ld_kp + row * k_row_bytes + k_off[i]));
                vr[i] = __builtin_nontemporal_load((const i32x4*)(ld_vp + row * v_row_bytes + v_off));
            }
        } else {
            // last, partial tile of a unit: rows past the end re-read the last row; those keys are never visible
#pragma unroll
            for (int i = 0; i < kFetch; i++) {
                int64_t row = (int64_t)j * kTileKeys + (kFetch * wave + i) * kChunkRows + (KV8 ? lane >> 3 : lrow);
                row = row < p.Lk ? row : p.Lk - 1;
                const int sw_k = KV8 ? (lane & 7) << 4 : (lpc ^ (i * 4 + lrow)) << 4;
                const int sw_v = KV8 ? (lane & 7) << 4 : (lpc ^ (lrow << 2)) << 4;
                kr[i] = __builtin_nontemporal_load((const i32x4*)(ld_kp + row * k_row_bytes + sw_k));
                vr[i] = __builtin_nontemporal_load((const i32x4*)(ld_vp + row * v_row_bytes + sw_v));
            }
        }
        blocks_left--;
        if (++ld_j == ld_je && blocks_left > 0) {
            REST_SEGMENT_NEXT(ld_unit, ld_j, ld_je, ld_round, ld_tail);
            unit_bases(ld_unit, ld_kp, ld_vp);
        }
    };
    // eight E4M3 bytes (two dwords) -> one 16-byte piece of bf16
    auto widen = [](int lo, int hi) -> i32x4 {
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        union { bf16x2 h[4]; i32x4 v; } u;
        u.h[0] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, 1.0f, false);
        u.h[1] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, 1.0f, true);
        u.h[2] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, 1.0f, false);
        u.h[3] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, 1.0f, true);
        return u.v;
    };
    auto park = [&](unsigned char* tile) {
        if constexpr (KV8) {
#pragma unroll
            for (int i = 0; i < 2; i++) {
                // fetched piece g of tile row `row` becomes bf16 pieces 2g and 2g+1, parked in their swizzled slots.
                // The eight lanes of a row store eight pieces of one parity at a time, which would hit each bank
                // twice; swapping the slots of a pair in the upper half of the row (pieces 8..15) spreads one store
                // over all banks.  The operand reads below undo the swap (kPairSwap).
                const int row = (2 * wave + i) * 8 + (lane >> 3), pc = (2 * (lane & 7)) ^ ((lane & 7) >> 2);
                unsigned char* krow = tile + row * 256;
                unsigned char* vrow = tile + kTileBytes + row * 256;
                const int swk = row & 15, swv = (row & 3) << 2;
                *(i32x4*)(krow + ((pc ^ swk) << 4)) = widen(kr[i][0], kr[i][1]);
                *(i32x4*)(krow + (((pc ^ 1) ^ swk) << 4)) = widen(kr[i][2], kr[i][3]);
                *(i32x4*)(vrow + ((pc ^ swv) << 4)) = widen(vr[i][0], vr[i][1]);
                *(i32x4*)(vrow + (((pc ^ 1) ^ swv) << 4)) = widen(vr[i][2], vr[i][3]);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 4; i++) {
                *(i32x4*)(tile + (4 * wave + i) * 1024 + lane * 16) = kr[i];
                *(i32x4*)(tile + kTileBytes + (4 * wave + i) * 1024 + lane * 16) = vr[i];
            }
        }
    };

    // ---- LDS read addresses (byte offsets inside a K or V tile), loop invariant
    const uint32_t ka0 = col * 256 + ((hh ^ (col & 15)) << 4);                     // ^ (ks << 5) per k-step
    const int vq = (lane & 15) >> 2;                                                 // V row inside a 4-row group
    const uint32_t va0 = (4 * hh + vq) * 256 + ((2 * ((lane >> 4) & 1) + ((lane & 3) >> 1)) << 4) + (lane & 1) * 8;
    const uint32_t vsw = (uint32_t)vq << 2;                                          // V swizzle of that row

    int buf = 0;
    int unit, seg_j, seg_je, seg_round;
    bool seg_tail;
    REST_SEGMENT_FIRST(unit, seg_j, seg_je, seg_round, seg_tail);
    int todo = blocks_left;          // blocks still to be computed
    issue();
    while (true) {
        // ================= one segment: blocks [seg_j, seg_je) of `unit`
        const bool whole = seg_j == 0 && seg_je == p.nblk;
        // a partial segment is the first of this stream's tail span (slot 0) or its last (slot 1)
        bool first_seg = false;
        if (seg_tail) {
            int tb, te;
            tail_span(tb, te);
            first_seg = (unit - p.dp_rounds * p.n_streams) * p.nblk + seg_j == tb;
        }
        unit = (int)REST_IDX(unit, p.units, 3);
        const int qg = unit % p.qgroups, slab = unit / p.qgroups;
        const int h = slab % p.H, nb = slab / p.H;
        const int qi = qg * (32 * NW) + wave * 32 + col;        // this lane's query row
        // scale of the logits in log2 units, and of the output: the slab's K and V factors folded in
        const float cu = KV8 && p.k_scale ? p.c * p.k_scale[slab] : p.c;
        const float vu = KV8 && p.v_scale ? p.v_scale[slab] : 1.0f;

        // mask row of this lane's query -> LDS (the halves write words 0,1 / 2,3); only this wave reads it back
        {
            const uint64_t* mrow = p.mask + (p.mask_per_batch ? (int64_t)nb * p.mask_rows * p.mask_words : 0);
#pragma unroll
            for (int w = 0; w < 2; w++) {
                const int ww = 2 * hh + w;
                my_mask[col * 4 + ww] = (qi < p.Tq && ww < p.mask_words) ? mrow[(int64_t)(qi % p.mask_rows) * p.mask_words + ww] : 0ull;
            }
        }
        // Q fragments (B operand of S^T = K Q^T): lane holds query `col`, d = 16*ks + 8*hh .. +8
        bf16x8 qf[8];
        {
            const __bf16* qp = p.q + nb * p.qs[0] + h * p.qs[1];
#pragma unroll
            for (int ks = 0; ks < 8; ks++) {
                bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
                if (qi < p.Tq) z = *(const bf16x8*)(qp + qi * p.qs[2] + 16 * ks + 8 * hh);
                qf[ks] = z;
            }
        }
        // The query fragments (and the mask words) must have arrived before the block loop: inside it the only
        // outstanding vector loads are to be the K/V of the next block, which the arithmetic must not wait for.
        // s_waitcnt vmcnt(0), other counters untouched.
        __builtin_amdgcn_s_waitcnt(0x0F70);

        f32x16 o[4];
        float m_ref = kNegBig, l_run = 0.f;     // m_ref in log2 units (logit * c)
#pragma unroll
        for (int dt = 0; dt < 4; dt++)
#pragma unroll
            for (int r = 0; r < 16; r++) o[dt][r] = 0.f;

        for (int j = seg_j; j < seg_je; j++, buf ^= 1) {
            // my half of this block moves from the staging registers to tile `buf`, my half of the next one (possibly
            // of the next unit) is requested, and after the barrier the whole tile is visible to both waves.
            // Tile buf^1 may still be read by the other wave (previous block); tile `buf` was last read two
            // blocks ago, which both waves finished before the previous barrier.
            unsigned char* tile = lds_tile[buf];
            park(tile);
            if (blocks_left > 0) issue();
            __syncthreads();
            // the tile's 32-key blocks, one after the other
#pragma unroll
            for (int sb = 0; sb < kSub; sb++) {
                const int key0 = j * kTileKeys + sb * kBlk;        // first key of the block
                if (sb > 0 && key0 >= p.Lk) break;                 // the last tile of a unit may hold fewer blocks
                const unsigned char* ldsK = tile + sb * kSubBytes;
                const unsigned char* ldsV = tile + kTileBytes + sb * kSubBytes;
                attn_block<kPairSwap, 1>(ldsK, ldsV, ka0, va0, vsw, hh, qf, o, m_ref, l_run, cu, key0, p.P, p.Tk, &my_mask[col * 4]);
            }
        }

        // ================= end of segment: the two key halves of the wave hold disjoint keys
        l_run += wave_xor32(l_run);
        if (qi < p.Tq) {
            if (whole) {
                const float inv = l_run > 0.f ? vu / l_run : 0.f;
                __bf16* op = p.out + nb * p.os[0] + h * p.os[1] + qi * p.os[2];
#pragma unroll
                for (int dt = 0; dt < 4; dt++)
#pragma unroll
                    for (int gq = 0; gq < 4; gq++) {
                        bf16x4 w;
#pragma unroll
                        for (int e = 0; e < 4; e++) w[e] = (__bf16)(o[dt][4 * gq + e] * inv);
                        *(bf16x4*)(op + dt * 32 + 8 * gq + 4 * hh) = w;
                    }
            } else {
                const int64_t row = REST_IDX(((int64_t)gw * 2 + (first_seg ? 0 : 1)) * (32 * NW) + wave * 32 + col,
                                             (int64_t)p.tail_streams * 2 * (32 * NW), 4);
                float* wo = p.ws_o + row * kD;
#pragma unroll
                for (int dt = 0; dt < 4; dt++)
#pragma unroll
                    for (int gq = 0; gq < 4; gq++) {
                        f32x4 w;
#pragma unroll
                        for (int e = 0; e < 4; e++) w[e] = o[dt][4 * gq + e] * vu;
                        *(f32x4*)(wo + dt * 32 + 8 * gq + 4 * hh) = w;
                    }
                if (hh == 0) {
                    p.ws_ml[row * 2 + 0] = m_ref;
                    p.ws_ml[row * 2 + 1] = l_run;
                }
            }
        }
        todo -= seg_je - seg_j;
        if (todo == 0) break;
        REST_SEGMENT_NEXT(unit, seg_j, seg_je, seg_round, seg_tail);
    }
#undef REST_SEGMENT_FIRST
#undef REST_SEGMENT_NEXT
}

// Arrival of one workgroup at a unit's ticket; true for the one that completes the unit (the `need`-th arrival).
// The ticket word is (kTicketMagic << 8) | arrivals; the completing workgroup puts it back to "no arrivals" when it is
// done, so in the steady state an arrival is one fetch-and-add, a single trip to the memory side.  A word that
// does not carry the magic number -- the caller's workspace as it was allocated -- counts as "no arrivals yet" and
// is put right by compare-and-swap (an add that met such a word is thrown away with it), so the workspace needs no
// initialisation: a wrong start would take uninitialised memory that holds exactly these 56 bits.  No workgroup waits
// for another: every loop here ends as soon as no other arrival has changed the word in between.
constexpr unsigned long long kTicketMagic = 0x52455354747265ull;       // 56 bits
__device__ inline bool ticket_arrive(unsigned long long* t, int need) {
    unsigned long long old = __hip_atomic_fetch_add(t, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if ((old >> 8) == kTicketMagic) return (int)(old & 0xffull) + 1 == need;
    old = __hip_atomic_load(t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    unsigned long long want;
    do {
        want = (old >> 8) == kTicketMagic ? old + 1 : ((kTicketMagic << 8) | 1ull);
    } while (!__hip_atomic_compare_exchange_strong(t, &old, want, __ATOMIC_RELAXED, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    return (int)(want & 0xffull) == need;
}

// Split plan, for launches with so few units that whole units or long spans per stream would leave most of the chip
// idle (one layer of a single context: 32 heads).  A workgroup is eight wavefronts = four key groups x two query
// halves; split_s workgroups share a unit, so its key blocks are cut into 4 split_s contiguous runs, one per key
// group.  A key group is a two-wavefront stream as in the kernel above (own pair of LDS tiles, same fetch, same
// arithmetic).  The four partial results of a workgroup are combined through LDS (the tiles' space, free by then) into
// one partial per workgroup: the output normalised by its own sum, in bf16 (one more rounding of the size the final
// output has anyway), plus reference and sum in fp32.  The workgroup that arrives last at the unit's ticket combines
// the split_s partials, always in the order 0 .. split_s-1, so the result does not depend on who that is.
// Workgroup w works on unit w % units: workgroups are dealt to the eight XCDs in turn, so when the number of units is a
// multiple of eight all workgroups of a unit sit on one XCD and its queries and partials stay in that XCD's L2.
template <bool KV8>
__global__ __launch_bounds__(512, 1) void tree_attn_split_kernel(AttnParams p) {
    constexpr int G = 4;                               // key groups per workgroup
    constexpr int kElt = KV8 ? 1 : 2;
    constexpr int kFetch = KV8 ? 2 : 4;
    constexpr int kChunkRows = KV8 ? 8 : 4;
    constexpr int kTileBytes = kSubBytes;              // a tile is one block of 32 keys
    // [group][buffer][K | V]; afterwards the groups' fp32 outputs [group][64 queries][128]
    __shared__ __attribute__((aligned(1024))) unsigned char lds_tile[G * 2 * 2 * kTileBytes];
    __shared__ uint64_t lds_mask[2 * G * 32 * 4];
    __shared__ float lds_ml[G * 64 * 2];
    __shared__ int lds_last;
    static_assert(G * 2 * 2 * kTileBytes == G * 64 * kD * 4, "the outputs of the key groups reuse the tiles' space exactly");

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = wave >> 1, qw = wave & 1;            // key group; which 32 of the 64 queries
    const int hh = lane >> 5, col = lane & 31, lrow = lane >> 4, lpc = lane & 15;
    const int unit = blockIdx.x % p.units, part = (int)REST_IDX(blockIdx.x / p.units, p.split_s, 6);
    const int h = unit % p.H, nb = unit / p.H;
    // this key group's blocks [b0, b1) of the unit's nblk
    const int ngroups = G * p.split_s, gi = part * G + g;
    const int b0 = (p.nblk * gi) / ngroups, b1 = (p.nblk * (gi + 1)) / ngroups;
    const int my_rounds = b1 - b0;

    const int64_t k_row_bytes = p.ks[2] * kElt, v_row_bytes = p.vs[2] * kElt;
    const char* kp = (const char*)p.k + (nb * p.ks[0] + h * p.ks[1]) * kElt;
    const char* vp = (const char*)p.v + (nb * p.vs[0] + h * p.vs[1]) * kElt;
    uint32_t k_off[4];
#pragma unroll
    for (int x = 0; x < 4; x++)
        k_off[x] = KV8 ? (uint32_t)((lane >> 3) * k_row_bytes) + ((lane & 7) << 4)
                       : (uint32_t)(lrow * k_row_bytes) + ((lpc ^ (x * 4 + lrow)) << 4);
    const uint32_t v_off = KV8 ? (uint32_t)((lane >> 3) * v_row_bytes) + ((lane & 7) << 4)
                               : (uint32_t)(lrow * v_row_bytes) + ((lpc ^ (lrow << 2)) << 4);

    // the fetch and the parking stores of the kernel above, for tiles of one block and two wavefronts
    i32x4 kr[kFetch], vr[kFetch];
    auto issue = [&](int j) {
        (void)REST_IDX((int64_t)j * kBlk, p.Lk, 2);
        if (!kBoundsChecked && (j + 1) * kBlk <= p.Lk) {
#pragma unroll
            for (int i = 0; i < kFetch; i++) {
                const int64_t row = (int64_t)j * kBlk + (kFetch * qw + i) * kChunkRows;
                kr[i] = __builtin_nontemporal_load((const i32x4*)(kp + row * k_row_bytes + k_off[i]));
                vr[i] = __builtin_nontemporal_load((const i32x4*)(vp + row * v_row_bytes + v_off));
            }
        } else {
#pragma unroll
            for (int i = 0; i < kFetch; i++) {
                int64_t row = (int64_t)j * kBlk + (kFetch * qw + i) * kChunkRows + (KV8 ? lane >> 3 : lrow);
                row = row < p.Lk ? row : p.Lk - 1;
                const int sw_k = KV8 ? (lane & 7) << 4 : (lpc ^ (i * 4 + lrow)) << 4;
                const int sw_v = KV8 ? (lane & 7) << 4 : (lpc ^ (lrow << 2)) << 4;
                kr[i] = __builtin_nontemporal_load((const i32x4*)(kp + row * k_row_bytes + sw_k));
                vr[i] = __builtin_nontemporal_load((const i32x4*)(vp + row * v_row_bytes + sw_v));
            }
        }
    };
    auto widen = [](int lo, int hi) -> i32x4 {
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        union { bf16x2 h[4]; i32x4 v; } u;
        u.h[0] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, 1.0f, false);
        u.h[1] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, 1.0f, true);
        u.h[2] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, 1.0f, false);
        u.h[3] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, 1.0f, true);
        return u.v;
    };
    auto park = [&](unsigned char* tile) {
        if constexpr (KV8) {
#pragma unroll
            for (int i = 0; i < 2; i++) {
                const int row = (2 * qw + i) * 8 + (lane >> 3), pc = (2 * (lane & 7)) ^ ((lane & 7) >> 2);
                unsigned char* krow = tile + row * 256;
                unsigned char* vrow = tile + kTileBytes + row * 256;
                const int swk = row & 15, swv = (row & 3) << 2;
                *(i32x4*)(krow + ((pc ^ swk) << 4)) = widen(kr[i][0], kr[i][1]);
                *(i32x4*)(krow + (((pc ^ 1) ^ swk) << 4)) = widen(kr[i][2], kr[i][3]);
                *(i32x4*)(vrow + ((pc ^ swv) << 4)) = widen(vr[i][0], vr[i][1]);
                *(i32x4*)(vrow + (((pc ^ 1) ^ swv) << 4)) = widen(vr[i][2], vr[i][3]);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 4; i++) {
                *(i32x4*)(tile + (4 * qw + i) * 1024 + lane * 16) = kr[i];
                *(i32x4*)(tile + kTileBytes + (4 * qw + i) * 1024 + lane * 16) = vr[i];
            }
        }
    };

    if (my_rounds > 0) issue(b0);

    const int qi = qw * 32 + col;                       // this lane's query row
    const float cu = KV8 && p.k_scale ? p.c * p.k_scale[unit] : p.c;
    uint64_t* const my_mask = lds_mask + wave * (32 * 4);
    {
        const uint64_t* mrow = p.mask + (p.mask_per_batch ? (int64_t)nb * p.mask_rows * p.mask_words : 0);
#pragma unroll
        for (int w = 0; w < 2; w++) {
            const int ww = 2 * hh + w;
            my_mask[col * 4 + ww] = (qi < p.Tq && ww < p.mask_words) ? mrow[(int64_t)(qi % p.mask_rows) * p.mask_words + ww] : 0ull;
        }
    }
    bf16x8 qf[8];
    {
        const __bf16* qp = p.q + nb * p.qs[0] + h * p.qs[1];
#pragma unroll
        for (int ks = 0; ks < 8; ks++) {
            bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
            if (qi < p.Tq) z = *(const bf16x8*)(qp + qi * p.qs[2] + 16 * ks + 8 * hh);
            qf[ks] = z;
        }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);                 // vmcnt(0): queries, mask words and the first tile are here

    const uint32_t ka0 = col * 256 + ((hh ^ (col & 15)) << 4);
    const int vq = (lane & 15) >> 2;
    const uint32_t va0 = (4 * hh + vq) * 256 + ((2 * ((lane >> 4) & 1) + ((lane & 3) >> 1)) << 4) + (lane & 1) * 8;
    const uint32_t vsw = (uint32_t)vq << 2;

    f32x16 o[4];
    float m_ref = kNegBig, l_run = 0.f;
#pragma unroll
    for (int dt = 0; dt < 4; dt++)
#pragma unroll
        for (int r = 0; r < 16; r++) o[dt][r] = 0.f;

    // Every wavefront passes the same number of barriers: a key group with fewer blocks than split_rounds sits the
    // last rounds out.  Tile `buf` of a group was last read two rounds ago, which both of its wavefronts had finished
    // before the previous barrier.
    for (int r = 0; r < p.split_rounds; r++) {
        unsigned char* tile = lds_tile + (g * 2 + (r & 1)) * (2 * kTileBytes);
        if (r < my_rounds) {
            park(tile);
            if (r + 1 < my_rounds) issue(b0 + r + 1);
        }
        __syncthreads();
        if (r < my_rounds)
            attn_block<KV8>(tile, tile + kTileBytes, ka0, va0, vsw, hh, qf, o, m_ref, l_run, cu, (b0 + r) * kBlk, p.P, p.Tk,
                            &my_mask[col * 4]);
    }
    l_run += wave_xor32(l_run);                         // the two key halves of the wavefront hold disjoint keys

    // ---- the four key groups' results -> LDS.  Row q of group g: 32 pieces of four floats, piece c at slot c ^ (q & 31)
    __syncthreads();                                    // all tiles have been read
    float* const lds_o = (float*)lds_tile;
    {
        float* row = lds_o + (g * 64 + qi) * kD;
#pragma unroll
        for (int dt = 0; dt < 4; dt++)
#pragma unroll
            for (int gq = 0; gq < 4; gq++) {
                f32x4 w;
#pragma unroll
                for (int e = 0; e < 4; e++) w[e] = o[dt][4 * gq + e];
                const int piece = dt * 8 + 2 * gq + hh;
                *(f32x4*)(row + ((piece ^ (qi & 31)) << 2)) = w;
            }
        if (hh == 0) {
            lds_ml[(g * 64 + qi) * 2 + 0] = m_ref;
            lds_ml[(g * 64 + qi) * 2 + 1] = l_run;
        }
    }
    __syncthreads();

    // ---- thread t: query t / 8, output columns 8 (t % 8) .. +7 and 64 + 8 (t % 8) .. +7 (pieces of four columns:
    // 2 (t % 8), the next one, and the same two 16 further on), so that the eight threads of a query write and read
    // 128 consecutive bytes of its bf16 row with each 16-byte access
    const int q = tid >> 3, c0 = (tid & 7) * 8, c1 = 64 + c0;
    auto piece_of = [&](int i) { return (i < 2 ? 0 : 16) + 2 * (tid & 7) + (i & 1); };
    float acc[16];
    float m_all = kNegBig, l_all = 0.f;
    {
#pragma unroll
        for (int gg = 0; gg < G; gg++) m_all = fmaxf(m_all, lds_ml[(gg * 64 + q) * 2]);
#pragma unroll
        for (int i = 0; i < 16; i++) acc[i] = 0.f;
#pragma unroll
        for (int gg = 0; gg < G; gg++) {
            const float w = __builtin_amdgcn_exp2f(lds_ml[(gg * 64 + q) * 2] - m_all);
            l_all += w * lds_ml[(gg * 64 + q) * 2 + 1];
            const float* row = lds_o + (gg * 64 + q) * kD;
#pragma unroll
            for (int i = 0; i < 4; i++) {
                const f32x4 x = *(const f32x4*)(row + ((piece_of(i) ^ (q & 31)) << 2));
#pragma unroll
                for (int e = 0; e < 4; e++) acc[4 * i + e] += w * x[e];
            }
        }
    }
    // Partial of this workgroup: output normalised by its own sum (bf16), reference and sum (fp32).  The partials cross
    // from one XCD to another, whose L2 caches do not see each other's plain stores until a write-back of the whole
    // cache (what a release fence at device scope costs here: tens of microseconds when every wavefront pays it).
    // Instead every partial is written and read with device-scope atomic accesses (relaxed, 64 bits at a time), which
    // go through to the memory side, and the order "partials before arrival" is kept by hand: each wavefront waits
    // until all its stores are acknowledged, the workgroup meets at a barrier, and only then thread 0 counts the
    // arrival.  The completing workgroup issues its reads after its arrival has returned.
    typedef unsigned long long u64;
    {
        const float inv = l_all > 0.f ? 1.0f / l_all : 0.f;
        const int64_t prow = REST_IDX(((int64_t)unit * p.split_s + part) * 64 + q, (int64_t)p.units * p.split_s * 64, 5);
        union { bf16x8 h[2]; i32x4 v[2]; } pk;
#pragma unroll
        for (int e = 0; e < 8; e++) {
            pk.h[0][e] = (__bf16)(acc[e] * inv);
            pk.h[1][e] = (__bf16)(acc[8 + e] * inv);
        }
        // Two 16-byte stores at device scope (sc1, what the compiler puts on a device-scope atomic store); with each,
        // the eight threads of a row write one whole 128-byte line.  As 8-byte atomic stores the same rows cost four
        // times their size in write traffic (WRITE_SIZE 17.0 MB per launch against 4.8 MB of partials and output).
        __bf16* po = p.ws_po + prow * kD + c0;
        asm volatile("global_store_dwordx4 %0, %1, off sc1\n\tglobal_store_dwordx4 %0, %2, off offset:128 sc1"
                     :
                     : "v"(po), "v"(pk.v[0]), "v"(pk.v[1])
                     : "memory");
        if ((tid & 7) == 0) {
            union { float f[2]; u64 w; } ml;
            ml.f[0] = m_all;
            ml.f[1] = l_all;
            __hip_atomic_store((u64*)(p.ws_ml + prow * 2), ml.w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);                 // vmcnt(0): this wavefront's partial stores are acknowledged
    __syncthreads();
    if (tid == 0) lds_last = ticket_arrive(p.tickets + unit, p.split_s) ? 1 : 0;
    __syncthreads();
    if (!lds_last) return;

    // ---- the last workgroup of the unit: partials 0 .. split_s-1 in that order, eight at a time with all their reads
    // in flight together (one trip to the memory side per batch)
    float m_fin = kNegBig, l_fin = 0.f;
#pragma unroll
    for (int i = 0; i < 16; i++) acc[i] = 0.f;
    const int64_t prow0 = (int64_t)unit * p.split_s * 64 + q;
    for (int s0 = 0; s0 < p.split_s; s0 += 8) {
        union { float f[2]; u64 w; } ml[8];
        union { bf16x8 h[2]; u64 w[4]; } pk[8];
#pragma unroll
        for (int i = 0; i < 8; i++) {
            const int sidx = s0 + i < p.split_s ? s0 + i : p.split_s - 1;        // past the end: the last one again, unused
            const int64_t prow = prow0 + sidx * 64;
            ml[i].w = __hip_atomic_load((const u64*)(p.ws_ml + prow * 2), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const u64* po = (const u64*)(p.ws_po + prow * kD + c0);
#pragma unroll
            for (int j = 0; j < 4; j++)          // columns c0 .. c0+7, then c1 .. c1+7 (16 eight-byte words further on)
                pk[i].w[j] = __hip_atomic_load(po + (j & 1) + 16 * (j >> 1), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        float m_new = m_fin;
#pragma unroll
        for (int i = 0; i < 8; i++)
            if (s0 + i < p.split_s) m_new = fmaxf(m_new, ml[i].f[0]);
        const float resc = __builtin_amdgcn_exp2f(m_fin - m_new);
        m_fin = m_new;
        l_fin *= resc;
#pragma unroll
        for (int e = 0; e < 16; e++) acc[e] *= resc;
#pragma unroll
        for (int i = 0; i < 8; i++) {
            const float w = s0 + i < p.split_s ? __builtin_amdgcn_exp2f(ml[i].f[0] - m_fin) * ml[i].f[1] : 0.f;
            l_fin += w;
#pragma unroll
            for (int e = 0; e < 8; e++) {
                acc[e] += w * (float)pk[i].h[0][e];
                acc[8 + e] += w * (float)pk[i].h[1][e];
            }
        }
    }
    if (q < p.Tq) {
        const float vu = KV8 && p.v_scale ? p.v_scale[unit] : 1.0f;
        const float inv = l_fin > 0.f ? vu / l_fin : 0.f;
        bf16x8 w0, w1;
#pragma unroll
        for (int e = 0; e < 8; e++) {
            w0[e] = (__bf16)(acc[e] * inv);
            w1[e] = (__bf16)(acc[8 + e] * inv);
        }
        __bf16* op = p.out + nb * p.os[0] + h * p.os[1] + q * p.os[2];
        *(bf16x8*)(op + c0) = w0;
        *(bf16x8*)(op + c1) = w1;
    }
    if (tid == 0) __hip_atomic_store(p.tickets + unit, kTicketMagic << 8, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Merges the partials of every tail unit that was cut between streams.  A 256-thread block takes `rows` query rows
// of one tail unit, a wavefront one row at a time (a lane owns two of the 128 output columns) and walks the
// streams that hold a piece of the unit.
__global__ __launch_bounds__(256) void tree_attn_streamk_merge_kernel(AttnParams p, int rows, int unit_rows) {
    const int per_unit = unit_rows / rows;
    const int ut = blockIdx.x / per_unit;                   // unit in tail coordinates
    const int row0 = (blockIdx.x % per_unit) * rows;
    const int unit = p.dp_rounds * p.n_streams + ut;
    const int qg = unit % p.qgroups, slab = unit / p.qgroups;
    const int64_t t_total = (int64_t)p.tail_units * p.nblk;
    const int64_t ub = (int64_t)ut * p.nblk, ue = ub + p.nblk;
    const int w0 = span_owner(t_total, p.tail_streams, ub), w1 = span_owner(t_total, p.tail_streams, ue - 1);
    if (w0 == w1) return;     // one stream covered the whole unit and wrote the output itself
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    // Only the first stream can have started before this unit (its partial sits in slot 1); every later stream
    // starts inside the unit, so this is its first segment (slot 0).  Streams are never empty.
    const int slot0 = span_begin(t_total, p.tail_streams, w0) >= ub ? 0 : 1;
    const int h = slab % p.H, nb = slab / p.H;
    for (int ql = row0 + wv; ql < row0 + rows; ql += 4) {
        const int qi = qg * unit_rows + ql;
        if (qi >= p.Tq) break;
        float m = kNegBig, l = 0.f, a0 = 0.f, a1 = 0.f;
#pragma unroll 4
        for (int w = w0; w <= w1; w++) {
            const int64_t row = ((int64_t)w * 2 + (w == w0 ? slot0 : 0)) * unit_rows + ql;
            const float mi = p.ws_ml[row * 2], li = p.ws_ml[row * 2 + 1];
            const float2 oi = *(const float2*)(p.ws_o + row * kD + 2 * lane);
            const float m_new = fmaxf(m, mi);
            const float sa = __builtin_amdgcn_exp2f(m - m_new), sb = __builtin_amdgcn_exp2f(mi - m_new);
            l = l * sa + li * sb;
            a0 = a0 * sa + oi.x * sb;
            a1 = a1 * sa + oi.y * sb;
            m = m_new;
        }
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        const float inv = l > 0.f ? 1.0f / l : 0.f;
        const bf16x2 o2 = {(__bf16)(a0 * inv), (__bf16)(a1 * inv)};
        *(bf16x2*)(p.out + nb * p.os[0] + h * p.os[1] + qi * p.os[2] + 2 * lane) = o2;
    }
}

// ---------------------------------------------------------------------------------------------------------
// fp32 path: one workgroup of NW wavefronts per (batch, head, 32 NW queries) and key split; wavefront w owns
// queries [32w, 32w + 32) of the group, all share one 32-key K/V tile in LDS, so every K/V element is read once per
// group.  S^T = K Q^T and O^T += V^T P^T run on v_mfma_f32_32x32x2_f32 with keys (then head dimensions) on the row
// axis, as in the bf16 kernels: a lane holds the scores of ONE query, and P is used where it was produced.  The
// instruction contracts two k-values at a time, lanes 0-31 giving one and lanes 32-63 the other; which two is free
// as long as both operands agree: for K Q^T lane half h contributes dimensions 8j + 4h + i (one 16-byte LDS read
// per four instructions), for V^T P^T it contributes key 8a + 4h + b, the row of S it already holds.
// K rows are padded to 132 words in LDS so that the 32 lanes of a half, which read the same columns of 32 different
// rows, fall on different banks.  Rows are 16-byte aligned (the host checks pointers and strides).
constexpr int kF32KStride = kD + 4;
template <int NW>
__global__ __launch_bounds__(64 * NW, NW == 2 ? 2 : 1) void tree_attn_f32_tiled_kernel(const float* q, const float* k, const float* v,
                                                                      const uint64_t* mask, float* out, float* ws_o, float* ws_ml,
                                                                      AttnParams p) {
    __shared__ __attribute__((aligned(16))) float ldsK[kBlk * kF32KStride];
    __shared__ __attribute__((aligned(16))) float ldsV[kBlk * kD];
    constexpr int kThreadsWG = 64 * NW;
    constexpr int kChunks = 2 * kBlk * (kD / 4) / kThreadsWG;      // 16-byte pieces of a K/V tile per thread
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, col = lane & 31, hh = lane >> 5;
    const int qg = blockIdx.x % p.qgroups;
    const int64_t slab = blockIdx.x / p.qgroups;
    const int h = (int)(slab % p.H);
    const int64_t nb = slab / p.H;
    const int split = blockIdx.y;
    const int qi = (qg * NW + wave) * 32 + col;
    const bool q_on = qi < p.Tq;
    const float* kp = k + nb * p.ks[0] + h * p.ks[1];
    const float* vp = v + nb * p.vs[0] + h * p.vs[1];

    // my query's dimensions 8j + 4hh .. + 3, j = 0..15, and its mask row
    f32x4 qf[kD / 8];
    uint64_t mw[REST_MAX_NODES / 64] = {0, 0, 0, 0};
    {
        const float* qp = q + nb * p.qs[0] + h * p.qs[1] + (int64_t)(q_on ? qi : 0) * p.qs[2];
#pragma unroll
        for (int j = 0; j < kD / 8; j++) {
            qf[j] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (q_on) qf[j] = *(const f32x4*)(qp + 8 * j + 4 * hh);
        }
        if (q_on && p.Tk > 0) {
            const uint64_t* mrow = mask + (p.mask_per_batch ? nb * p.mask_rows * p.mask_words : 0) + (int64_t)(qi % p.mask_rows) * p.mask_words;
#pragma unroll
            for (int w = 0; w < REST_MAX_NODES / 64; w++)
                if (w < p.mask_words) mw[w] = mrow[w];
        }
    }
    // blocks of this split
    const int nblk = (p.Lk + kBlk - 1) / kBlk;
    const int per = (nblk + p.nsplit - 1) / p.nsplit;
    const int b0 = split * per, b1 = min(nblk, b0 + per);

    // A thread moves the same 16-byte column `ch` of rows row0, row0 + kStep, ... of K and of V: addresses differ by a
    // constant from piece to piece, and only the last block of a slab checks rows against the end
    constexpr int kHalf = kChunks / 2;             // pieces of K (and of V) per thread
    constexpr int kStep = kThreadsWG / (kD / 4);   // rows between two pieces of a thread
    const int row0 = tid / (kD / 4), ch = tid % (kD / 4);
    f32x4 stage[kChunks];
    auto fetch = [&](int jb) {
        const int key0 = jb * kBlk;
        const float* kb = kp + (int64_t)(key0 + row0) * p.ks[2] + 4 * ch;
        const float* vb = vp + (int64_t)(key0 + row0) * p.vs[2] + 4 * ch;
        if (!kBoundsChecked && key0 + kBlk <= p.Lk) {
#pragma unroll
            for (int i = 0; i < kHalf; i++) {
                stage[i] = *(const f32x4*)(kb + (int64_t)(i * kStep) * p.ks[2]);
                stage[kHalf + i] = *(const f32x4*)(vb + (int64_t)(i * kStep) * p.vs[2]);
            }
        } else {
#pragma unroll
            for (int i = 0; i < kHalf; i++) {
                stage[i] = stage[kHalf + i] = f32x4{0.f, 0.f, 0.f, 0.f};     // rows past the end: zeros (V must not be garbage)
                const int key = key0 + row0 + i * kStep;
                if (key < p.Lk) {
                    const int64_t kk = REST_IDX(key, p.Lk, 6);
                    stage[i] = *(const f32x4*)(kp + kk * p.ks[2] + 4 * ch);
                    stage[kHalf + i] = *(const f32x4*)(vp + kk * p.vs[2] + 4 * ch);
                }
            }
        }
    };
    auto park = [&]() {
#pragma unroll
        for (int i = 0; i < kHalf; i++) {
            *(f32x4*)(ldsK + (row0 + i * kStep) * kF32KStride + 4 * ch) = stage[i];
            *(f32x4*)(ldsV + (row0 + i * kStep) * kD + 4 * ch) = stage[kHalf + i];
        }
    };

    f32x16 o[4];
    float m_ref = kNegBig, l_run = 0.f;           // m_ref in log2 units (score * c)
#pragma unroll
    for (int dt = 0; dt < 4; dt++)
#pragma unroll
        for (int r = 0; r < 16; r++) o[dt][r] = 0.f;
    const float cu = p.c;

    if (b0 < b1) fetch(b0);
    for (int jb = b0; jb < b1; jb++) {
        __syncthreads();                           // everyone has left the previous tile
        park();
        __syncthreads();
        if (jb + 1 < b1) fetch(jb + 1);            // on its way during the arithmetic below
        const int key0 = jb * kBlk;

        // ---- S^T[key][query] = K Q^T
        f32x16 sc;
#pragma unroll
        for (int r = 0; r < 16; r++) sc[r] = 0.f;
#pragma unroll
        for (int j = 0; j < kD / 8; j++) {
            const f32x4 kv = *(const f32x4*)(ldsK + col * kF32KStride + 8 * j + 4 * hh);
#pragma unroll
            for (int i = 0; i < 4; i++) sc = __builtin_amdgcn_mfma_f32_32x32x2f32(kv[i], qf[j][i], sc, 0, 0, 0);
        }
        // ---- visibility: bit i of vbits <-> key key0 + i; prefix keys are visible to everyone
        if (key0 + kBlk > p.P) {
            const int kb = key0 - p.P;            // draft-token index of the block's first key (may be < 0)
            const int end = p.Tk - kb;            // keys at block offset >= end are past the last key
            const uint32_t in_range = end >= 32 ? 0xffffffffu : (end > 0 ? (1u << end) - 1u : 0u);
            uint32_t vbits;
            if (kb < 0) {
                vbits = ((1u << (-kb)) - 1u) | ((uint32_t)mw[0] << (-kb));
            } else {
                const int w = kb >> 6, sh = kb & 63;
                const uint64_t lo = w == 0 ? mw[0] : (w == 1 ? mw[1] : (w == 2 ? mw[2] : mw[3]));
                const uint64_t hi = w == 0 ? mw[1] : (w == 1 ? mw[2] : (w == 2 ? mw[3] : 0ull));
                vbits = (uint32_t)(lo >> sh);
                if (sh > 32) vbits |= (uint32_t)(hi << (64 - sh));
            }
            vbits &= in_range;
            vbits >>= 4 * hh;
#pragma unroll
            for (int r = 0; r < 16; r++) {
                const bool vis = (vbits >> (8 * (r >> 2) + (r & 3))) & 1u;
                sc[r] = vis ? sc[r] : -INFINITY;
            }
        }
        // ---- softmax numerators against a lazily updated reference, per lane = per query column
        {
            float mx = sc[0];
#pragma unroll
            for (int r = 1; r < 16; r++) mx = fmaxf(mx, sc[r]);
            mx = fmaxf(mx, wave_xor32(mx)) * cu;
            if (__any(mx > m_ref + kLazy)) {
                const float m_new = fmaxf(m_ref, mx);
                const float alpha = __builtin_amdgcn_exp2f(m_ref - m_new);
                m_ref = m_new;
                l_run *= alpha;
#pragma unroll
                for (int dt = 0; dt < 4; dt++)
#pragma unroll
                    for (int r = 0; r < 16; r++) o[dt][r] *= alpha;
            }
            float sum = 0.f;
#pragma unroll
            for (int r = 0; r < 16; r++) {
                sc[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[r], cu, -m_ref));
                sum += sc[r];
            }
            l_run += sum;
        }
        // ---- O^T[d][query] += V^T P^T: lane half hh brings key 8a + 4hh + b, whose probability is its sc[4a + b]
#pragma unroll
        for (int a = 0; a < 4; a++)
#pragma unroll
            for (int bb = 0; bb < 4; bb++) {
                const float* vrow = ldsV + (8 * a + 4 * hh + bb) * kD + col;
#pragma unroll
                for (int dt = 0; dt < 4; dt++)
                    o[dt] = __builtin_amdgcn_mfma_f32_32x32x2f32(vrow[32 * dt], sc[4 * a + bb], o[dt], 0, 0, 0);
            }
    }

    // ---- o[dt][4g + e] = O[query][d = 32 dt + 8 g + 4 hh + e]; the two halves of a query hold disjoint keys' sums
    l_run += wave_xor32(l_run);
    if (!q_on) return;
    if (p.nsplit == 1) {
        const float inv = l_run > 0.f ? 1.0f / l_run : 0.f;
        float* op = out + nb * p.os[0] + h * p.os[1] + (int64_t)qi * p.os[2];
#pragma unroll
        for (int dt = 0; dt < 4; dt++)
#pragma unroll
            for (int g = 0; g < 4; g++) {
                f32x4 w;
#pragma unroll
                for (int e = 0; e < 4; e++) w[e] = o[dt][4 * g + e] * inv;
                *(f32x4*)(op + 32 * dt + 8 * g + 4 * hh) = w;
            }
    } else {
        const int64_t row = (slab * p.nsplit + split) * p.Tq + qi;
        float* wo = ws_o + row * kD;
#pragma unroll
        for (int dt = 0; dt < 4; dt++)
#pragma unroll
            for (int g = 0; g < 4; g++) {
                f32x4 w;
#pragma unroll
                for (int e = 0; e < 4; e++) w[e] = o[dt][4 * g + e];
                *(f32x4*)(wo + 32 * dt + 8 * g + 4 * hh) = w;
            }
        if (hh == 0) {
            ws_ml[row * 2] = m_ref;
            ws_ml[row * 2 + 1] = l_run;
        }
    }
}

__global__ __launch_bounds__(128) void tree_attn_f32_merge_kernel(const float* ws_o, const float* ws_ml, float* out,
                                                                  int32_t H, int32_t Tq, int32_t nsplit,
                                                                  int64_t os0, int64_t os1, int64_t os2) {
    const int64_t rowid = blockIdx.x;            // (slab, qi)
    const int qi = (int)(rowid % Tq);
    const int64_t slab = rowid / Tq;
    const int h = (int)(slab % H);
    const int64_t nb = slab / H;
    const int d = threadIdx.x;
    float m = kNegBig;
    for (int s = 0; s < nsplit; s++) m = fmaxf(m, ws_ml[((slab * nsplit + s) * Tq + qi) * 2]);
    float l = 0.f, acc = 0.f;
    for (int s = 0; s < nsplit; s++) {
        const int64_t row = (slab * nsplit + s) * Tq + qi;
        const float w = __builtin_amdgcn_exp2f(ws_ml[row * 2] - m);       // references are in log2 units
        l += ws_ml[row * 2 + 1] * w;
        acc += ws_o[row * kD + d] * w;
    }
    out[nb * os0 + h * os1 + qi * os2 + d] = l > 0.f ? acc / l : 0.f;
}

// ---------------------------------------------------------------------------------------------------------
struct Plan {
    int qt, qgroups, nblk, units, n_streams, nsplit_f32;
    int dp_rounds, tail_units, tail_streams, extra_units, merge_rows;
    bool need_merge;
    int split_s;      // > 0: the split plan with that many workgroups per unit (then nothing above but nblk, units counts)
};

constexpr int kSplitGroups = 4;       // key groups of a split-plan workgroup
constexpr int kSplitMaxUnits = 128;   // the split plan is for launches with at most this many units
constexpr int kSplitMaxParts = 16;    // workgroups per unit, at most

Plan make_plan(const rest_attn_desc* d) {
    Plan pl{};
    const int Lk = d->P + d->Tk;
    pl.nblk = (Lk + kBlk - 1) / kBlk;
    if (d->dtype == REST_FP32) {
        // groups of 32 qt queries; with few groups the keys are split so that the launch has about two workgroups per
        // compute unit, every split with at least one block
        pl.qt = d->Tq <= 32 ? 1 : (d->Tq <= 64 ? 2 : (d->Tq <= 128 ? 4 : 8));
        pl.qgroups = (d->Tq + 32 * pl.qt - 1) / (32 * pl.qt);
        pl.units = d->Nb * d->H * pl.qgroups;
        int ns = d->num_splits;
        if (ns <= 0) {
            ns = (512 + pl.units - 1) / pl.units;
            if (ns > 64) ns = 64;
        }
        if (ns > pl.nblk) ns = pl.nblk > 0 ? pl.nblk : 1;
        pl.nsplit_f32 = ns;
        return pl;
    }
    // a stream of qt wavefronts covers 32 qt queries and moves tiles of 16 qt keys
    pl.qt = d->Tq <= 64 ? 2 : (d->Tq <= 128 ? 4 : 8);
    pl.qgroups = (d->Tq + 32 * pl.qt - 1) / (32 * pl.qt);
    pl.nblk = (Lk + 16 * pl.qt - 1) / (16 * pl.qt);
    pl.units = d->Nb * d->H * pl.qgroups;
    // Few units of at most 64 queries (one layer of a single context): the split plan.  One workgroup of four key
    // groups per compute unit, i.e. 256 / units workgroups per unit, every key group with at least one block.
    if (d->num_splits == 0 && pl.qt == 2 && pl.units <= kSplitMaxUnits && d->o_stride[0] % 8 == 0 && d->o_stride[1] % 8 == 0 &&
        d->o_stride[2] % 8 == 0) {
        int s = 256 / pl.units;
        if (s > kSplitMaxParts) s = kSplitMaxParts;
        if (s > pl.nblk / kSplitGroups) s = pl.nblk / kSplitGroups;
        if (s >= 2) {
            pl.split_s = s;
            return pl;
        }
    }
    const int64_t total = (int64_t)pl.units * pl.nblk;
    int64_t w;
    if (d->num_splits > 0) {
        w = (int64_t)pl.units * d->num_splits;       // explicit request: num_splits streams per unit
        if (w > 16384) w = 16384;
    } else {
        // eight wavefronts per compute unit, but at least four tiles per stream
        w = total / 4;
        if (w > kMaxWaves / pl.qt) w = kMaxWaves / pl.qt;
    }
    if (w > total) w = total;
    if (w < 1) w = 1;
    pl.n_streams = (int)w;
    // every stream takes dp_rounds whole units; the blocks of the units left over are cut into spans
    pl.dp_rounds = pl.units / pl.n_streams;
    pl.tail_units = pl.units - pl.dp_rounds * pl.n_streams;
    // Half a round or more left over: those units stay whole, one more for each of that many streams, and nothing
    // is cut or merged.  A stream runs faster when fewer run beside it, so the short-handed last round costs little
    // more than its share of a full one would; cutting the units would add a second start-up, the partials and the
    // merge.  The even streams go first: streams are dealt to the eight XCDs in turn, and with every XCD
    // saturating memory the even-numbered ones were measured to finish a round about 12 % earlier than the odd ones.
    // Only where memory is the limit (two-wavefront streams on a 16-bit cache): a stream bound by its own
    // instruction issue gains nothing from idle neighbours, and there the cut is the faster plan (measured).
    pl.extra_units = 0;
    if (d->num_splits == 0 && pl.qt == 2 && d->kv_dtype == REST_KV_AS_DTYPE && pl.dp_rounds > 0 &&
        2 * pl.tail_units >= pl.n_streams) {
        pl.extra_units = pl.tail_units;
        pl.tail_units = 0;
    }
    const int64_t t_total = (int64_t)pl.tail_units * pl.nblk;
    int64_t ts = d->num_splits > 0 ? w : t_total / 4;      // at least four blocks per tail span
    if (ts > w) ts = w;
    if (ts > t_total) ts = t_total;
    if (ts < 1 && t_total > 0) ts = 1;
    pl.tail_streams = (int)ts;
    pl.need_merge = false;
    for (int u = 0; u < pl.tail_units && !pl.need_merge; u++) {
        const int64_t ub = (int64_t)u * pl.nblk;
        if (span_owner(t_total, pl.tail_streams, ub) != span_owner(t_total, pl.tail_streams, ub + pl.nblk - 1)) pl.need_merge = true;
    }
    // rows of a unit per merge block: about a thousand blocks in all, a multiple of the four wavefronts
    pl.merge_rows = 32 * pl.qt;
    while (pl.merge_rows > 4 && (int64_t)pl.tail_units * (32 * pl.qt / pl.merge_rows) < 1024) pl.merge_rows /= 2;
    return pl;
}

bool desc_ok(const rest_attn_desc* d) {
    if (!d) return false;
    if (d->Nb < 1 || d->H < 1 || d->Tq < 1 || d->Tq > REST_MAX_QUERY_ROWS || d->Tk < 0 || d->Tk > REST_MAX_NODES) return false;
    if (d->P < 0 || d->P + d->Tk < 1 || d->D != kD) return false;
    if (d->dtype != REST_BF16 && d->dtype != REST_FP32) return false;
    if (d->kv_dtype != REST_KV_AS_DTYPE && d->kv_dtype != REST_KV_FP8_E4M3) return false;
    if (d->kv_dtype == REST_KV_FP8_E4M3 && d->dtype != REST_BF16) return false;
    if (!(d->scale > 0.f) || !(d->scale < 1e30f)) return false;
    if (d->num_splits < 0 || d->num_splits > 64) return false;
    if (d->mask_rows < 0 || d->mask_rows > d->Tq) return false;
    // units (a slab's query rows in groups of at most 256) and block counts are kept in 32 bits
    const int64_t slabs_q = (int64_t)d->Nb * d->H * ((d->Tq + 255) / 256);
    if (slabs_q * 64 > 0x7fffffff) return false;
    if ((slabs_q + 1) * ((d->P + d->Tk + kBlk - 1) / kBlk) > 0x7fffffff) return false;
    for (int i = 0; i < 3; i++)
        if (d->q_stride[i] < 0 || d->k_stride[i] < 0 || d->v_stride[i] < 0 || d->o_stride[i] < 0) return false;
    // rows are read with 16-byte vector loads
    const int64_t al = d->dtype == REST_BF16 ? 8 : 4;
    const int64_t al_kv = d->kv_dtype == REST_KV_FP8_E4M3 ? 16 : al;
    for (int i = 0; i < 3; i++)
        if (d->q_stride[i] % al || d->k_stride[i] % al_kv || d->v_stride[i] % al_kv || d->o_stride[i] % 4) return false;
    if (d->q_stride[2] < kD || d->k_stride[2] < kD || d->v_stride[2] < kD || d->o_stride[2] < kD) return false;
    // four consecutive rows are addressed with a 32-bit byte offset
    if (d->k_stride[2] > (1 << 26) || d->v_stride[2] > (1 << 26)) return false;
    return true;
}

}  // namespace

// workspace of the split plan: [tickets: one 64-bit word per unit, padded to 256 bytes][reference, sum: units x parts x
// 64 rows x 2 floats][normalised partial outputs: units x parts x 64 rows x 128 bf16]
static size_t split_ticket_bytes(int units) { return ((size_t)units * 8 + 255) / 256 * 256; }

extern "C" __attribute__((visibility("default"))) size_t rest_tree_attention_workspace_bytes(const rest_attn_desc* d) {
    if (!desc_ok(d)) return 0;
    const Plan pl = make_plan(d);
    if (d->dtype == REST_FP32) {
        if (pl.nsplit_f32 == 1) return 0;
        return (size_t)d->Nb * d->H * pl.nsplit_f32 * d->Tq * (kD + 2) * sizeof(float);
    }
    if (pl.split_s > 0) return split_ticket_bytes(pl.units) + (size_t)pl.units * pl.split_s * 64 * (2 * sizeof(float) + kD * 2);
    if (!pl.need_merge) return 0;
    return (size_t)pl.tail_streams * 2 * (pl.qt * 32) * (kD + 2) * sizeof(float);
}

// Checks the call and enqueues its kernels; the partial results of cut units go to d_workspace.
static rest_status enqueue_tree_attention(const void* d_q, const void* d_k, const void* d_v, const uint64_t* d_mask,
                                          void* d_out, const rest_attn_desc* d, void* d_workspace,
                                          size_t workspace_bytes, void* stream_) {
    if (!desc_ok(d) || !d_q || !d_k || !d_v || !d_out) return REST_INVALID_ARG;
    if (d->Tk > 0 && !d_mask) return REST_INVALID_ARG;
    if (((uintptr_t)d_q | (uintptr_t)d_k | (uintptr_t)d_v | (uintptr_t)d_out) & 15) return REST_INVALID_ARG;
    hipStream_t stream = (hipStream_t)stream_;
    const Plan pl = make_plan(d);
    const size_t need = rest_tree_attention_workspace_bytes(d);
    if (need > workspace_bytes || (need && !d_workspace)) return REST_WORKSPACE_TOO_SMALL;
    if (need && ((uintptr_t)d_workspace & 15)) return REST_INVALID_ARG;      // partials are moved 16 bytes at a time

    AttnParams p;
    p.q = (const __bf16*)d_q;
    p.k = (const __bf16*)d_k;
    p.v = (const __bf16*)d_v;
    // Tk == 0: the kernels never dereference mask rows beyond mask_words == 0, but give them a valid pointer
    p.mask = d_mask ? d_mask : (const uint64_t*)d_q;
    p.out = (__bf16*)d_out;
    p.Nb = d->Nb; p.H = d->H; p.Tq = d->Tq; p.Tk = d->Tk; p.P = d->P; p.Lk = d->P + d->Tk;
    p.mask_words = (d->Tk + 63) / 64;
    p.mask_per_batch = d->mask_per_batch ? 1 : 0;
    p.mask_rows = d->mask_rows > 0 ? d->mask_rows : d->Tq;
    p.nblk = pl.nblk;
    p.c = d->scale * 1.4426950408889634f;
    for (int i = 0; i < 3; i++) { p.qs[i] = d->q_stride[i]; p.ks[i] = d->k_stride[i]; p.vs[i] = d->v_stride[i]; p.os[i] = d->o_stride[i]; }
    p.ws_o = (float*)d_workspace;
    const bool kv8 = d->kv_dtype == REST_KV_FP8_E4M3;
    p.k_scale = kv8 ? d->d_k_scale : nullptr;
    p.v_scale = kv8 ? d->d_v_scale : nullptr;

    p.split_s = 0;
    p.split_rounds = 0;
    p.ws_po = nullptr;
    p.tickets = nullptr;
    if (d->dtype == REST_BF16 && pl.split_s > 0) {
        p.nsplit = 1;
        p.qgroups = 1;
        p.units = pl.units;
        p.n_streams = p.dp_rounds = p.tail_units = p.tail_streams = p.extra_units = 0;
        p.split_s = pl.split_s;
        const int ngroups = kSplitGroups * pl.split_s;
        p.split_rounds = (pl.nblk + ngroups - 1) / ngroups;
        p.tickets = (unsigned long long*)d_workspace;
        p.ws_ml = (float*)((char*)d_workspace + split_ticket_bytes(pl.units));
        p.ws_po = (__bf16*)(p.ws_ml + (size_t)pl.units * pl.split_s * 64 * 2);
        if (kv8)
            hipLaunchKernelGGL((tree_attn_split_kernel<true>), dim3(pl.units * pl.split_s), dim3(512), 0, stream, p);
        else
            hipLaunchKernelGGL((tree_attn_split_kernel<false>), dim3(pl.units * pl.split_s), dim3(512), 0, stream, p);
        REST_HIP_TRY(hipGetLastError());
    } else if (d->dtype == REST_BF16) {
        p.nsplit = 1;
        p.qgroups = pl.qgroups;
        p.units = pl.units;
        p.n_streams = pl.n_streams;
        p.dp_rounds = pl.dp_rounds;
        p.tail_units = pl.tail_units;
        p.tail_streams = pl.tail_streams;
        p.extra_units = pl.extra_units;
        const size_t rows = (size_t)pl.tail_streams * 2 * (pl.qt * 32);
        p.ws_ml = p.ws_o ? p.ws_o + rows * kD : nullptr;
        if (pl.qt == 2 && !kv8)
            hipLaunchKernelGGL((tree_attn_bf16_kernel<2, false>), dim3(pl.n_streams), dim3(128), 0, stream, p);
        else if (pl.qt == 4 && !kv8)
            hipLaunchKernelGGL((tree_attn_bf16_kernel<4, false>), dim3(pl.n_streams), dim3(256), 0, stream, p);
        else if (!kv8)
            hipLaunchKernelGGL((tree_attn_bf16_kernel<8, false>), dim3(pl.n_streams), dim3(512), 0, stream, p);
        else if (pl.qt == 2)
            hipLaunchKernelGGL((tree_attn_bf16_kernel<2, true>), dim3(pl.n_streams), dim3(128), 0, stream, p);
        else if (pl.qt == 4)
            hipLaunchKernelGGL((tree_attn_bf16_kernel<4, true>), dim3(pl.n_streams), dim3(256), 0, stream, p);
        else
            hipLaunchKernelGGL((tree_attn_bf16_kernel<8, true>), dim3(pl.n_streams), dim3(512), 0, stream, p);
        REST_HIP_TRY(hipGetLastError());
        if (pl.need_merge) {
            hipLaunchKernelGGL(tree_attn_streamk_merge_kernel, dim3(pl.tail_units * (32 * pl.qt / pl.merge_rows)), dim3(256), 0,
                               stream, p, pl.merge_rows, 32 * pl.qt);
            REST_HIP_TRY(hipGetLastError());
        }
    } else {
        const int ns = pl.nsplit_f32;
        p.nsplit = ns;
        p.units = 0;
        p.n_streams = 0;
        p.dp_rounds = p.tail_units = p.tail_streams = p.extra_units = 0;
        const size_t rows = (size_t)d->Nb * d->H * ns * d->Tq;
        p.ws_ml = p.ws_o ? p.ws_o + rows * kD : nullptr;
        p.qgroups = pl.qgroups;
        const dim3 grid(pl.units, ns);
        const float *fq = (const float*)d_q, *fk = (const float*)d_k, *fv = (const float*)d_v;
        if (pl.qt == 1)
            hipLaunchKernelGGL((tree_attn_f32_tiled_kernel<1>), grid, dim3(64), 0, stream, fq, fk, fv, p.mask, (float*)d_out, p.ws_o, p.ws_ml, p);
        else if (pl.qt == 2)
            hipLaunchKernelGGL((tree_attn_f32_tiled_kernel<2>), grid, dim3(128), 0, stream, fq, fk, fv, p.mask, (float*)d_out, p.ws_o, p.ws_ml, p);
        else if (pl.qt == 4)
            hipLaunchKernelGGL((tree_attn_f32_tiled_kernel<4>), grid, dim3(256), 0, stream, fq, fk, fv, p.mask, (float*)d_out, p.ws_o, p.ws_ml, p);
        else
            hipLaunchKernelGGL((tree_attn_f32_tiled_kernel<8>), grid, dim3(512), 0, stream, fq, fk, fv, p.mask, (float*)d_out, p.ws_o, p.ws_ml, p);
        REST_HIP_TRY(hipGetLastError());
        if (ns > 1) {
            hipLaunchKernelGGL(tree_attn_f32_merge_kernel, dim3(d->Nb * d->H * d->Tq), dim3(128), 0, stream,
                               p.ws_o, p.ws_ml, (float*)d_out, d->H, d->Tq, ns, p.os[0], p.os[1], p.os[2]);
            REST_HIP_TRY(hipGetLastError());
        }
    }
    REST_BOUNDS_EPILOGUE(stream);
    return REST_OK;
}

extern "C" __attribute__((visibility("default"))) rest_status rest_tree_attention(const void* d_q, const void* d_k, const void* d_v, const uint64_t* d_mask,
                                           void* d_out, const rest_attn_desc* d, void* d_workspace,
                                           size_t workspace_bytes, void* stream_) {
    return enqueue_tree_attention(d_q, d_k, d_v, d_mask, d_out, d, d_workspace, workspace_bytes, stream_);
}

// ---------------------------------------------------------------------------------------------------------
// rest_tree_attention for callers that cannot allocate: the partial results live in a device array that is part of
// the library's code object.  Each GPU holds its own copy at its own address; the array's name is only a handle in
// host code, so the address is asked of the runtime once per device and that pointer is what the kernels get.
namespace {
static __device__ __align__(256) unsigned char scratch[REST_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
void* g_scratch_ptr[kMaxDevices];      // per device: where `scratch` lives there (null = not asked yet)

rest_status static_scratch(void** out) {
    int dev = -1;
    REST_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return REST_UNSUPPORTED;
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        REST_HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return REST_HIP_ERROR;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return REST_OK;
}
}  // namespace

extern "C" __attribute__((visibility("default"))) rest_status rest_tree_attention_noalloc(const void* d_q, const void* d_k, const void* d_v,
                                                   const uint64_t* d_mask, void* d_out, const rest_attn_desc* d,
                                                   void* stream_) {
    if (!desc_ok(d)) return REST_INVALID_ARG;
    const size_t need = rest_tree_attention_workspace_bytes(d);
    if (need > (size_t)REST_STATIC_SCRATCH_BYTES) return REST_WORKSPACE_TOO_SMALL;
    void* ws = nullptr;
    if (need) {
        const rest_status st = static_scratch(&ws);
        if (st != REST_OK) return st;
    }
    // Every partial that the merge reads was written earlier in the same call, so nothing in the array has to start
    // at zero and what the last call left there is never seen.
    return enqueue_tree_attention(d_q, d_k, d_v, d_mask, d_out, d, ws, need, stream_);
}
