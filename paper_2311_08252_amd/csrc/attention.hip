// Tree-masked verification attention for gfx950 ("Draft verification" of REST, arXiv 2311.08252):
// every draft token attends to the whole cached context and, among the draft tokens, to itself and
// its ancestors only.
//
// bf16 kernel design (HBM-bound: ~T flop per KV byte, far below the chip's balance point):
//  * one wavefront = one independent stream over a contiguous range of 32-key blocks, for up to 64
//    queries; no workgroup barrier inside the streaming loop;
//  * a block's K and V (8 KB each) are fetched with coalesced 16-byte loads one block ahead of the
//    arithmetic, kept in registers while in flight, then parked in wave-private LDS with an XOR swizzle;
//  * S^T = K Q^T and O^T += V^T P^T run on v_mfma_f32_32x32x16_bf16.  With keys on the MFMA row axis a
//    lane owns one query column, so the softmax statistics are per lane; V^T fragments come out of LDS
//    through ds_read_b64_tr_b16; the probabilities go from the S accumulator straight into the B
//    operand of the second product (the key permutation this implies is applied to V^T as well);
//  * the four waves of a workgroup merge their (max, sum, O) through LDS; several workgroups per
//    (batch, head) write partials that a small second kernel merges.
//  * tree-mask bit rows are staged in LDS and only consulted for the blocks that reach past the prefix.
#include "common.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kD = 128;            // head dim
constexpr int kBlk = 32;           // keys per block
constexpr int kWaves = 4;          // waves per workgroup
constexpr int kTileBytes = kBlk * kD * 2;   // 8 KB: one K or V block in bf16
constexpr float kNegBig = -1.0e30f;

struct AttnParams {
    const __bf16* q;
    const __bf16* k;
    const __bf16* v;
    const uint64_t* mask;
    __bf16* out;
    float* ws_o;      // [streams][qrows][128] partial O (un-normalised), only when nsplit > 1
    float* ws_ml;     // [streams][qrows][2]   (max, sum)
    int32_t Nb, H, Tq, Tk, P, Lk;
    int32_t nsplit, qgroups, mask_words, mask_per_batch;
    int32_t nblk;     // ceil(Lk / 32)
    int32_t nstreams; // Nb * H * nsplit
    float c;          // scale * log2(e)
    int64_t qs[3], ks[3], vs[3], os[3];
};

__device__ inline float wave_xor32(float x) { return __shfl_xor(x, 32, 64); }

template <int QT>
__global__ __launch_bounds__(256) void tree_attn_bf16_kernel(AttnParams p) {
    __shared__ __attribute__((aligned(16))) unsigned char lds_stage[kWaves * 2 * kTileBytes];  // 64 KB
    __shared__ uint64_t lds_mask[QT * 32 * 4];   // QT*32 query rows x 4 mask words
    __shared__ float lds_ml[kWaves][QT][2][64];

    // ---- XCD-aware decode of the flat workgroup id: consecutive ids go to different XCDs, so the
    // q-groups that stream the same K/V are given ids that land on one XCD (shared L2).
    const int id = blockIdx.x;
    const int xcd = id & 7, slot = id >> 3;
    const int qg = slot % p.qgroups;
    const int stream = (slot / p.qgroups) * 8 + xcd;
    if (stream >= p.nstreams) return;
    const int split = stream % p.nsplit;
    const int slab = stream / p.nsplit;
    const int h = slab % p.H, nb = slab / p.H;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int hh = lane >> 5;      // which half of the wave (selects the k-slice of MFMA operands)
    const int col = lane & 31;     // MFMA column = query within a 32-query tile
    const int qbase = qg * (QT * 32);

    // ---- stage this q-group's mask rows in LDS
    {
        const uint64_t* mrow = p.mask + (p.mask_per_batch ? (int64_t)nb * p.Tq * p.mask_words : 0);
        for (int i = tid; i < QT * 32 * 4; i += 256) {
            int qi = qbase + (i >> 2), w = i & 3;
            lds_mask[i] = (qi < p.Tq && w < p.mask_words) ? mrow[(int64_t)qi * p.mask_words + w] : 0ull;
        }
    }

    // ---- Q fragments (B operand of S^T = K Q^T): lane holds query `col`, d = 16*ks + 8*hh .. +8
    bf16x8 qf[QT][8];
    {
        const __bf16* qp = p.q + nb * p.qs[0] + h * p.qs[1];
#pragma unroll
        for (int qt = 0; qt < QT; qt++) {
            int qi = qbase + qt * 32 + col;
#pragma unroll
            for (int ks = 0; ks < 8; ks++) {
                bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
                if (qi < p.Tq) z = *(const bf16x8*)(qp + qi * p.qs[2] + 16 * ks + 8 * hh);
                qf[qt][ks] = z;
            }
        }
    }
    __syncthreads();

    // ---- this wave's block range
    const int gw = split * kWaves + wave, nw = p.nsplit * kWaves;
    const int jb = (int)(((int64_t)p.nblk * gw) / nw), je = (int)(((int64_t)p.nblk * (gw + 1)) / nw);
    const int plain_end = p.P / kBlk;   // blocks below this hold prefix keys only

    const __bf16* kp = p.k + nb * p.ks[0] + h * p.ks[1];
    const __bf16* vp = p.v + nb * p.vs[0] + h * p.vs[1];
    unsigned char* ldsK = lds_stage + wave * 2 * kTileBytes;
    unsigned char* ldsV = ldsK + kTileBytes;

    f32x16 o[QT][4];
    float m_run[QT], l_run[QT];
#pragma unroll
    for (int qt = 0; qt < QT; qt++) {
        m_run[qt] = kNegBig;
        l_run[qt] = 0.f;
#pragma unroll
        for (int dt = 0; dt < 4; dt++)
#pragma unroll
            for (int r = 0; r < 16; r++) o[qt][dt][r] = 0.f;
    }

    i32x4 kr[8], vr[8];
    const int lrow = lane >> 4, lpc = lane & 15;
    auto issue = [&](int j) {
#pragma unroll
        for (int i = 0; i < 8; i++) {
            int row = j * kBlk + i * 4 + lrow;
            row = row < p.Lk ? row : p.Lk - 1;
            kr[i] = __builtin_nontemporal_load((const i32x4*)(kp + row * p.ks[2] + lpc * 8));
            vr[i] = __builtin_nontemporal_load((const i32x4*)(vp + row * p.vs[2] + lpc * 8));
        }
    };
    auto park = [&]() {
#pragma unroll
        for (int i = 0; i < 8; i++) {
            int r = i * 4 + lrow;
            *(i32x4*)(ldsK + r * 256 + ((lpc ^ (r & 15)) << 4)) = kr[i];
            *(i32x4*)(ldsV + r * 256 + ((lpc ^ ((r & 3) << 2)) << 4)) = vr[i];
        }
    };

    if (jb < je) issue(jb);
    for (int j = jb; j < je; j++) {
        park();
        if (j + 1 < je) issue(j + 1);

        // ---- S^T[key][query] = K Q^T
        f32x16 s[QT];
#pragma unroll
        for (int qt = 0; qt < QT; qt++)
#pragma unroll
            for (int r = 0; r < 16; r++) s[qt][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ks++) {
            bf16x8 a = *(const bf16x8*)(ldsK + col * 256 + (((2 * ks + hh) ^ (col & 15)) << 4));
#pragma unroll
            for (int qt = 0; qt < QT; qt++)
                s[qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[qt][ks], s[qt], 0, 0, 0);
        }

        // ---- visibility (only blocks that reach past the prefix): one 32-bit word per lane says which of
        // the block's 32 keys its query sees; bit i <-> key j*32 + i
        if (j >= plain_end) {
            const int kb = j * kBlk - p.P;          // draft-token index of the block's first key (may be < 0)
            const int end = p.Tk - kb;              // keys at block offset >= end are past the last key
            const uint32_t in_range = end >= 32 ? 0xffffffffu : (end > 0 ? (1u << end) - 1u : 0u);
#pragma unroll
            for (int qt = 0; qt < QT; qt++) {
                const uint64_t* mw = &lds_mask[(qt * 32 + col) * 4];
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
                    s[qt][r] = vis ? s[qt][r] : -INFINITY;
                }
            }
        }

        // ---- online softmax, per lane = per query column
        bf16x8 pf[QT][2];
#pragma unroll
        for (int qt = 0; qt < QT; qt++) {
            float mx = s[qt][0];
#pragma unroll
            for (int r = 1; r < 16; r++) mx = fmaxf(mx, s[qt][r]);
            mx = fmaxf(mx, wave_xor32(mx));
            float m_new = fmaxf(m_run[qt], mx);
            float alpha = __builtin_amdgcn_exp2f((m_run[qt] - m_new) * p.c);
            float mc = m_new * p.c;
            float sum = 0.f;
#pragma unroll
            for (int r = 0; r < 16; r++) {
                float e = __builtin_amdgcn_exp2f(__builtin_fmaf(s[qt][r], p.c, -mc));
                sum += e;
                pf[qt][r >> 3][r & 7] = (__bf16)e;
            }
            l_run[qt] = l_run[qt] * alpha + sum;
            m_run[qt] = m_new;
            if (__any(alpha != 1.0f)) {
#pragma unroll
                for (int dt = 0; dt < 4; dt++)
#pragma unroll
                    for (int r = 0; r < 16; r++) o[qt][dt][r] *= alpha;
            }
        }

        // ---- O^T[d][query] += V^T P^T
#pragma unroll
        for (int ss = 0; ss < 2; ss++) {
            const int rowA = 16 * ss + 4 * hh + ((lane & 15) >> 2);
            const int sw = (rowA & 3) << 2;
#pragma unroll
            for (int dt = 0; dt < 4; dt++) {
                const int pc = dt * 4 + 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
                const unsigned char* a0 = ldsV + rowA * 256 + ((pc ^ sw) << 4) + (lane & 1) * 8;
                s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)a0);
                s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(a0 + 8 * 256));
                union { struct { s16x4 lo, hi; } sp; bf16x8 v; } u;
                u.sp.lo = lo;
                u.sp.hi = hi;
#pragma unroll
                for (int qt = 0; qt < QT; qt++)
                    o[qt][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(u.v, pf[qt][ss], o[qt][dt], 0, 0, 0);
            }
        }
    }

    // ---- combine the two key halves of the wave
#pragma unroll
    for (int qt = 0; qt < QT; qt++) l_run[qt] += wave_xor32(l_run[qt]);

    // ---- merge the four waves through LDS: 1 -> 0 and 3 -> 2, then 2 -> 0
    float* xch = (float*)lds_stage;   // [2 slots][QT*4*16][64] floats: 32 KB per slot at QT = 2
    for (int round = 0; round < 2; round++) {
        __syncthreads();
        const bool sender = round == 0 ? (wave & 1) : (wave == 2);
        const bool receiver = round == 0 ? !(wave & 1) : (wave == 0);
        const int slotw = round == 0 ? (wave >> 1) : 0;
        float* xs = xch + slotw * (QT * 64 * 64);
        if (sender) {
#pragma unroll
            for (int qt = 0; qt < QT; qt++) {
                lds_ml[wave][qt][0][lane] = m_run[qt];
                lds_ml[wave][qt][1][lane] = l_run[qt];
#pragma unroll
                for (int dt = 0; dt < 4; dt++)
#pragma unroll
                    for (int r = 0; r < 16; r++) xs[((qt * 4 + dt) * 16 + r) * 64 + lane] = o[qt][dt][r];
            }
        }
        __syncthreads();
        if (receiver) {
            const int from = round == 0 ? wave + 1 : 2;
#pragma unroll
            for (int qt = 0; qt < QT; qt++) {
                float mo = lds_ml[from][qt][0][lane], lo = lds_ml[from][qt][1][lane];
                float m_new = fmaxf(m_run[qt], mo);
                float a = __builtin_amdgcn_exp2f((m_run[qt] - m_new) * p.c);
                float b = __builtin_amdgcn_exp2f((mo - m_new) * p.c);
                l_run[qt] = l_run[qt] * a + lo * b;
                m_run[qt] = m_new;
#pragma unroll
                for (int dt = 0; dt < 4; dt++)
#pragma unroll
                    for (int r = 0; r < 16; r++)
                        o[qt][dt][r] = o[qt][dt][r] * a + xs[((qt * 4 + dt) * 16 + r) * 64 + lane] * b;
            }
        }
    }

    // ---- wave 0 holds the workgroup's result
    if (wave != 0) return;
#pragma unroll
    for (int qt = 0; qt < QT; qt++) {
        const int qi = qbase + qt * 32 + col;
        if (qi >= p.Tq) continue;
        if (p.nsplit == 1) {
            const float inv = l_run[qt] > 0.f ? 1.0f / l_run[qt] : 0.f;
            __bf16* op = p.out + nb * p.os[0] + h * p.os[1] + qi * p.os[2];
#pragma unroll
            for (int dt = 0; dt < 4; dt++)
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    bf16x4 w;
#pragma unroll
                    for (int e = 0; e < 4; e++) w[e] = (__bf16)(o[qt][dt][4 * g + e] * inv);
                    *(bf16x4*)(op + dt * 32 + 8 * g + 4 * hh) = w;
                }
        } else {
            const int64_t row = (int64_t)stream * p.Tq + qi;
            float* wo = p.ws_o + row * kD;
#pragma unroll
            for (int dt = 0; dt < 4; dt++)
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    f32x4 w;
#pragma unroll
                    for (int e = 0; e < 4; e++) w[e] = o[qt][dt][4 * g + e];
                    *(f32x4*)(wo + dt * 32 + 8 * g + 4 * hh) = w;
                }
            if (hh == 0) {
                p.ws_ml[row * 2 + 0] = m_run[qt];
                p.ws_ml[row * 2 + 1] = l_run[qt];
            }
        }
    }
}

// Merges the partial (max, sum, O) of the KV splits of one (batch, head, query): one 128-thread block per row.
template <typename OutT>
__global__ __launch_bounds__(128) void tree_attn_merge_kernel(const float* ws_o, const float* ws_ml, OutT* out,
                                                              int32_t H, int32_t Tq, int32_t nsplit, float c,
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
        float w = __builtin_amdgcn_exp2f((ws_ml[row * 2] - m) * c);
        l += ws_ml[row * 2 + 1] * w;
        acc += ws_o[row * kD + d] * w;
    }
    out[nb * os0 + h * os1 + qi * os2 + d] = (OutT)(l > 0.f ? acc / l : 0.f);
}

// fp32 path: plain fp32 arithmetic, one 128-thread block per (batch, head, query), one KV split per
// blockIdx.y.  Exists for accuracy checks with fp32 inputs; not a throughput path.
__global__ __launch_bounds__(128) void tree_attn_f32_kernel(const float* q, const float* k, const float* v,
                                                            const uint64_t* mask, float* out, float* ws_o, float* ws_ml,
                                                            AttnParams p) {
    __shared__ float qs[kD];
    __shared__ float prob[128];
    __shared__ float red[128];
    const int64_t rowid = blockIdx.x;
    const int qi = (int)(rowid % p.Tq);
    const int64_t slab = rowid / p.Tq;
    const int h = (int)(slab % p.H);
    const int64_t nb = slab / p.H;
    const int split = blockIdx.y;
    const int tid = threadIdx.x;
    const float* qp = q + nb * p.qs[0] + h * p.qs[1] + qi * p.qs[2];
    const float* kp = k + nb * p.ks[0] + h * p.ks[1];
    const float* vp = v + nb * p.vs[0] + h * p.vs[1];
    const uint64_t* mrow = mask + (p.mask_per_batch ? nb * p.Tq * p.mask_words : 0) + (int64_t)qi * p.mask_words;
    qs[tid] = qp[tid];
    __syncthreads();
    const int chunk = (p.Lk + p.nsplit - 1) / p.nsplit;
    const int k0 = split * chunk, k1 = min(p.Lk, k0 + chunk);
    float m = kNegBig, l = 0.f, acc = 0.f;
    for (int base = k0; base < k1; base += 128) {
        const int key = base + tid;
        float sc = -INFINITY;
        if (key < k1) {
            const int t = key - p.P;
            bool vis = t < 0 || ((mrow[t >> 6] >> (t & 63)) & 1ull);
            if (vis) {
                float dot = 0.f;
                const float* kr = kp + key * p.ks[2];
                for (int d = 0; d < kD; d++) dot = __builtin_fmaf(qs[d], kr[d], dot);
                sc = dot;
            }
        }
        red[tid] = sc;
        __syncthreads();
        for (int st = 64; st > 0; st >>= 1) {
            if (tid < st) red[tid] = fmaxf(red[tid], red[tid + st]);
            __syncthreads();
        }
        const float m_new = fmaxf(m, red[0]);
        __syncthreads();
        const float e = __builtin_amdgcn_exp2f((sc - m_new) * p.c);
        prob[tid] = e;
        red[tid] = e;
        __syncthreads();
        for (int st = 64; st > 0; st >>= 1) {
            if (tid < st) red[tid] += red[tid + st];
            __syncthreads();
        }
        const float alpha = __builtin_amdgcn_exp2f((m - m_new) * p.c);
        l = l * alpha + red[0];
        acc *= alpha;
        const int nk = min(128, k1 - base);
        for (int jj = 0; jj < nk; jj++) acc = __builtin_fmaf(prob[jj], vp[(base + jj) * p.vs[2] + tid], acc);
        m = m_new;
        __syncthreads();
    }
    if (p.nsplit == 1) {
        out[nb * p.os[0] + h * p.os[1] + qi * p.os[2] + tid] = l > 0.f ? acc / l : 0.f;
    } else {
        const int64_t row = (slab * p.nsplit + split) * p.Tq + qi;
        ws_o[row * kD + tid] = acc;
        if (tid == 0) {
            ws_ml[row * 2] = m;
            ws_ml[row * 2 + 1] = l;
        }
    }
}

int choose_splits(const rest_attn_desc* d) {
    if (d->num_splits > 0) return d->num_splits;
    const int Lk = d->P + d->Tk;
    const int64_t slabs = (int64_t)d->Nb * d->H;
    if (d->dtype == REST_FP32) return 1;
    const int nblk = (Lk + kBlk - 1) / kBlk;
    // aim for about two workgroups per compute unit, but keep >= 4 key blocks per wavefront
    int want = (int)((512 + slabs - 1) / slabs);
    int cap = nblk / (kWaves * 4);
    if (want > cap) want = cap;
    if (want < 1) want = 1;
    if (want > 64) want = 64;
    return want;
}

bool desc_ok(const rest_attn_desc* d) {
    if (!d) return false;
    if (d->Nb < 1 || d->H < 1 || d->Tq < 1 || d->Tq > REST_MAX_NODES || d->Tk < 0 || d->Tk > REST_MAX_NODES) return false;
    if (d->P < 0 || d->P + d->Tk < 1 || d->D != kD) return false;
    if (d->dtype != REST_BF16 && d->dtype != REST_FP32) return false;
    if (!(d->scale > 0.f) || !(d->scale < 1e30f)) return false;
    if (d->num_splits < 0 || d->num_splits > 64) return false;
    if ((int64_t)d->Nb * d->H * 64 > 0x7fffffff) return false;
    for (int i = 0; i < 3; i++)
        if (d->q_stride[i] < 0 || d->k_stride[i] < 0 || d->v_stride[i] < 0 || d->o_stride[i] < 0) return false;
    // rows are read with 16-byte vector loads
    const int64_t al = d->dtype == REST_BF16 ? 8 : 4;
    for (int i = 0; i < 3; i++)
        if (d->q_stride[i] % al || d->k_stride[i] % al || d->v_stride[i] % al || d->o_stride[i] % 4) return false;
    if (d->q_stride[2] < kD || d->k_stride[2] < kD || d->v_stride[2] < kD || d->o_stride[2] < kD) return false;
    return true;
}

}  // namespace

extern "C" __attribute__((visibility("default"))) size_t rest_tree_attention_workspace_bytes(const rest_attn_desc* d) {
    if (!desc_ok(d)) return 0;
    const int ns = choose_splits(d);
    if (ns == 1) return 0;
    const size_t rows = (size_t)d->Nb * d->H * ns * d->Tq;
    return rows * (kD + 2) * sizeof(float);
}

extern "C" __attribute__((visibility("default"))) rest_status rest_tree_attention(const void* d_q, const void* d_k, const void* d_v, const uint64_t* d_mask,
                                           void* d_out, const rest_attn_desc* d, void* d_workspace,
                                           size_t workspace_bytes, void* stream_) {
    if (!desc_ok(d) || !d_q || !d_k || !d_v || !d_out) return REST_INVALID_ARG;
    if (d->Tk > 0 && !d_mask) return REST_INVALID_ARG;
    if (((uintptr_t)d_q | (uintptr_t)d_k | (uintptr_t)d_v | (uintptr_t)d_out) & 15) return REST_INVALID_ARG;
    hipStream_t stream = (hipStream_t)stream_;
    const int ns = choose_splits(d);
    const size_t need = rest_tree_attention_workspace_bytes(d);
    if (need > workspace_bytes || (need && !d_workspace)) return REST_WORKSPACE_TOO_SMALL;

    AttnParams p;
    p.q = (const __bf16*)d_q;
    p.k = (const __bf16*)d_k;
    p.v = (const __bf16*)d_v;
    // Tk == 0: the kernels never dereference mask rows beyond mask_words == 0, but give them a valid pointer
    p.mask = d_mask ? d_mask : (const uint64_t*)d_q;
    p.out = (__bf16*)d_out;
    p.Nb = d->Nb; p.H = d->H; p.Tq = d->Tq; p.Tk = d->Tk; p.P = d->P; p.Lk = d->P + d->Tk;
    p.nsplit = ns;
    p.mask_words = (d->Tk + 63) / 64;
    p.mask_per_batch = d->mask_per_batch ? 1 : 0;
    p.nblk = (p.Lk + kBlk - 1) / kBlk;
    p.nstreams = d->Nb * d->H * ns;
    p.c = d->scale * 1.4426950408889634f;
    for (int i = 0; i < 3; i++) { p.qs[i] = d->q_stride[i]; p.ks[i] = d->k_stride[i]; p.vs[i] = d->v_stride[i]; p.os[i] = d->o_stride[i]; }
    const size_t rows = (size_t)p.nstreams * d->Tq;
    p.ws_o = (float*)d_workspace;
    p.ws_ml = p.ws_o ? p.ws_o + rows * kD : nullptr;

    if (d->dtype == REST_BF16) {
        const int qt = d->Tq <= 32 ? 1 : 2;
        p.qgroups = (d->Tq + qt * 32 - 1) / (qt * 32);
        const int grid = ((p.nstreams + 7) / 8) * 8 * p.qgroups;
        if (qt == 1) hipLaunchKernelGGL(tree_attn_bf16_kernel<1>, dim3(grid), dim3(256), 0, stream, p);
        else hipLaunchKernelGGL(tree_attn_bf16_kernel<2>, dim3(grid), dim3(256), 0, stream, p);
        REST_HIP_TRY(hipGetLastError());
        if (ns > 1) {
            hipLaunchKernelGGL(tree_attn_merge_kernel<__bf16>, dim3(d->Nb * d->H * d->Tq), dim3(128), 0, stream,
                               p.ws_o, p.ws_ml, (__bf16*)d_out, d->H, d->Tq, ns, p.c, p.os[0], p.os[1], p.os[2]);
            REST_HIP_TRY(hipGetLastError());
        }
    } else {
        p.qgroups = 1;
        hipLaunchKernelGGL(tree_attn_f32_kernel, dim3(d->Nb * d->H * d->Tq, ns), dim3(128), 0, stream,
                           (const float*)d_q, (const float*)d_k, (const float*)d_v, p.mask, (float*)d_out, p.ws_o, p.ws_ml, p);
        REST_HIP_TRY(hipGetLastError());
        if (ns > 1) {
            hipLaunchKernelGGL(tree_attn_merge_kernel<float>, dim3(d->Nb * d->H * d->Tq), dim3(128), 0, stream,
                               p.ws_o, p.ws_ml, (float*)d_out, d->H, d->Tq, ns, p.c, p.os[0], p.os[1], p.os[2]);
            REST_HIP_TRY(hipGetLastError());
        }
    }
    return REST_OK;
}
