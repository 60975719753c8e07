// The cache steps either side of verification inside one layer, for models with rotary position embedding
// (REST, arXiv 2311.08252: "Draft verification" needs each draft token at the position it has in its own
// draft; "Draft acceptance" turns the accepted tokens into context).  The paper does not describe them; the
// definitions are stated in rest.h.
//
// rope_append_kernel: one workgroup owns four draft rows of one Nb index and walks over the heads.  Its 256
// angles (4 rows x 64 planes) are formed once, in fp64 (position * theta^(-2i/D), then sincos), kept in LDS as
// fp32, and reused for every head, so the kernel is a plain HBM stream: 3 x T x 256 B read and written per head.
// kv_compact_kernel: one workgroup per (Nb, head); all accepted rows are read into registers before any is
// written, because a row can be the source of one move and the destination of another.
#include "common.h"

namespace {

typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
constexpr int kD = 128;

struct KvParams {
    __bf16* q;
    const __bf16* kn;
    const __bf16* vn;
    __bf16* kc;
    __bf16* vc;
    const int32_t* pos_ids;
    const int32_t* path;
    const int32_t* path_len;
    const float* k_scale;   // 8-bit cache: [Nb*H] factors (stored code = value / factor), or null for 1
    const float* v_scale;
    int32_t Nb, H, T, P, pos_offset, per_batch, path_cap;
    double log2_theta;
    int64_t qs[3], kns[3], vns[3], kcs[3], vcs[3];
};

__device__ inline float bf16_lo(int32_t w) { return __builtin_bit_cast(float, (uint32_t)w << 16); }
__device__ inline float bf16_hi(int32_t w) { return __builtin_bit_cast(float, (uint32_t)w & 0xffff0000u); }
// two fp32 -> packed bf16 pair, round to nearest even
__device__ inline int32_t pack_bf16(float lo, float hi) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    bf16x2 p = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(int32_t, p);
}

// rotates the plane vectors (a[e], b[e]), e = 0..7, given as two 16-byte groups of bf16
__device__ inline void rotate8(i32x4& a, i32x4& b, const float (&c)[8], const float (&s)[8]) {
#pragma unroll
    for (int w = 0; w < 4; w++) {
        const float a0 = bf16_lo(a[w]), a1 = bf16_hi(a[w]), b0 = bf16_lo(b[w]), b1 = bf16_hi(b[w]);
        const float ra0 = a0 * c[2 * w] - b0 * s[2 * w], rb0 = a0 * s[2 * w] + b0 * c[2 * w];
        const float ra1 = a1 * c[2 * w + 1] - b1 * s[2 * w + 1], rb1 = a1 * s[2 * w + 1] + b1 * c[2 * w + 1];
        a[w] = pack_bf16(ra0, ra1);
        b[w] = pack_bf16(rb0, rb1);
    }
}

// rotated plane vectors as floats: ra[e], rb[e] from the bf16 groups a, b
__device__ inline void rotate8f(const i32x4& a, const i32x4& b, const float (&c)[8], const float (&s)[8], float (&ra)[8], float (&rb)[8]) {
#pragma unroll
    for (int w = 0; w < 4; w++) {
        const float a0 = bf16_lo(a[w]), a1 = bf16_hi(a[w]), b0 = bf16_lo(b[w]), b1 = bf16_hi(b[w]);
        ra[2 * w] = a0 * c[2 * w] - b0 * s[2 * w];
        rb[2 * w] = a0 * s[2 * w] + b0 * c[2 * w];
        ra[2 * w + 1] = a1 * c[2 * w + 1] - b1 * s[2 * w + 1];
        rb[2 * w + 1] = a1 * s[2 * w + 1] + b1 * c[2 * w + 1];
    }
}

// eight floats divided by `scale` -> eight E4M3 codes (nearest even, magnitudes beyond 448 saturate) in two dwords
typedef int32_t i32x2 __attribute__((ext_vector_type(2)));
__device__ inline i32x2 to_e4m3(const float (&x)[8], float scale) {
    int32_t w0, w1;
    float y[8];
#pragma unroll
    for (int e = 0; e < 8; e++) {
        const float q = x[e] / scale;
        y[e] = q == q ? fminf(fmaxf(q, -448.f), 448.f) : q;     // a NaN stays a NaN (code 0x7f)
    }
    w0 = __builtin_amdgcn_cvt_pk_fp8_f32(y[0], y[1], 0, false);
    w0 = __builtin_amdgcn_cvt_pk_fp8_f32(y[2], y[3], w0, true);
    w1 = __builtin_amdgcn_cvt_pk_fp8_f32(y[4], y[5], 0, false);
    w1 = __builtin_amdgcn_cvt_pk_fp8_f32(y[6], y[7], w1, true);
    return i32x2{w0, w1};
}

// C8: the caches hold one E4M3 byte per element (128-byte rows); q, k_new, v_new are bf16 either way
template <bool C8>
__global__ __launch_bounds__(256) void rope_append_kernel(KvParams p) {
    __shared__ float lds_c[4][64], lds_s[4][64];
    const int tid = threadIdx.x;
    const int nb = blockIdx.y;
    const int t0 = blockIdx.x * 4;
    {
        const int r = tid >> 6, i = tid & 63;
        const int t = t0 + r;
        float c = 1.f, s = 0.f;
        if (t < p.T) {
            const int pos = p.pos_ids[(p.per_batch ? (int64_t)nb * p.T : 0) + t] + p.pos_offset;
            const double freq = exp2(-(2.0 * i / kD) * p.log2_theta);
            double sd, cd;
            sincos((double)pos * freq, &sd, &cd);
            c = (float)cd;
            s = (float)sd;
        }
        lds_c[r][i] = c;
        lds_s[r][i] = s;
    }
    __syncthreads();
    const int sub = tid >> 5, r = (tid >> 3) & 3, o = tid & 7;
    const int t = t0 + r;
    if (t >= p.T) return;
    float c[8], s[8];
#pragma unroll
    for (int e = 0; e < 8; e++) { c[e] = lds_c[r][8 * o + e]; s[e] = lds_s[r][8 * o + e]; }
    for (int h = blockIdx.z * 8 + sub; h < p.H; h += 8 * gridDim.z) {
        __bf16* qp = p.q + nb * p.qs[0] + h * p.qs[1] + t * p.qs[2] + 8 * o;
        const __bf16* kp = p.kn + nb * p.kns[0] + h * p.kns[1] + t * p.kns[2] + 8 * o;
        const __bf16* vp = p.vn + nb * p.vns[0] + h * p.vns[1] + t * p.vns[2] + 8 * o;
        i32x4 qa = *(const i32x4*)qp, qb = *(const i32x4*)(qp + 64);
        i32x4 ka = *(const i32x4*)kp, kb = *(const i32x4*)(kp + 64);
        const i32x4 va = *(const i32x4*)vp, vb = *(const i32x4*)(vp + 64);
        rotate8(qa, qb, c, s);
        *(i32x4*)qp = qa;
        *(i32x4*)(qp + 64) = qb;
        if constexpr (!C8) {
            rotate8(ka, kb, c, s);
            __bf16* kd = p.kc + nb * p.kcs[0] + h * p.kcs[1] + (int64_t)(p.P + t) * p.kcs[2] + 8 * o;
            __bf16* vd = p.vc + nb * p.vcs[0] + h * p.vcs[1] + (int64_t)(p.P + t) * p.vcs[2] + 8 * o;
            *(i32x4*)kd = ka;
            *(i32x4*)(kd + 64) = kb;
            *(i32x4*)vd = va;
            *(i32x4*)(vd + 64) = vb;
        } else {
            const float ksc = p.k_scale ? p.k_scale[nb * p.H + h] : 1.f, vsc = p.v_scale ? p.v_scale[nb * p.H + h] : 1.f;
            float ra[8], rb[8], fa[8], fb[8];
            rotate8f(ka, kb, c, s, ra, rb);
#pragma unroll
            for (int w = 0; w < 4; w++) {
                fa[2 * w] = bf16_lo(va[w]); fa[2 * w + 1] = bf16_hi(va[w]);
                fb[2 * w] = bf16_lo(vb[w]); fb[2 * w + 1] = bf16_hi(vb[w]);
            }
            const i32x2 ka8 = to_e4m3(ra, ksc), kb8 = to_e4m3(rb, ksc), va8 = to_e4m3(fa, vsc), vb8 = to_e4m3(fb, vsc);
            unsigned char* kd = (unsigned char*)p.kc + nb * p.kcs[0] + h * p.kcs[1] + (int64_t)(p.P + t) * p.kcs[2] + 8 * o;
            unsigned char* vd = (unsigned char*)p.vc + nb * p.vcs[0] + h * p.vcs[1] + (int64_t)(p.P + t) * p.vcs[2] + 8 * o;
            *(i32x2*)kd = ka8;
            *(i32x2*)(kd + 64) = kb8;
            *(i32x2*)vd = va8;
            *(i32x2*)(vd + 64) = vb8;
        }
    }
}

// ELT: bytes per cached element (2: bf16, 1: E4M3); a row is 16 or 8 pieces of 16 bytes
template <int ELT>
__global__ __launch_bounds__(512) void kv_compact_kernel(KvParams p) {
    const int h = blockIdx.x, nb = blockIdx.y;
    const int i = threadIdx.x >> 4, piece = threadIdx.x & 15;
    const int row = p.per_batch ? nb : 0;
    // the path's entry is read together with the path's length, not after it (the array has path_cap entries a row)
    int n = p.path_len[row];
    int src = i < p.path_cap ? p.path[(int64_t)row * p.path_cap + i] : -1;
    n = n < 0 ? 0 : (n > p.path_cap ? p.path_cap : n);
    // the moves end at the first entry that is not a draft row
    bool live = i < n;
    if (!live) src = -1;
    live = live && src >= 0 && src < p.T;
    // a move is made only if every move before it is: the smallest offending index is agreed on through LDS
    __shared__ int first_bad;
    if (threadIdx.x == 0) first_bad = 0x7fffffff;
    __syncthreads();
    if (i < n && !live && piece == 0) atomicMin(&first_bad, i);
    __syncthreads();
    live = live && i < first_bad && piece * 16 < kD * ELT;
    unsigned char* kbase = (unsigned char*)p.kc + (nb * p.kcs[0] + h * p.kcs[1]) * ELT + 16 * piece;
    unsigned char* vbase = (unsigned char*)p.vc + (nb * p.vcs[0] + h * p.vcs[1]) * ELT + 16 * piece;
    i32x4 kv = {0, 0, 0, 0}, vv = {0, 0, 0, 0};
    if (live) {
        kv = *(const i32x4*)(kbase + (int64_t)(p.P + src) * p.kcs[2] * ELT);
        vv = *(const i32x4*)(vbase + (int64_t)(p.P + src) * p.vcs[2] * ELT);
    }
    __syncthreads();
    if (live) {
        *(i32x4*)(kbase + (int64_t)(p.P + i) * p.kcs[2] * ELT) = kv;
        *(i32x4*)(vbase + (int64_t)(p.P + i) * p.vcs[2] * ELT) = vv;
    }
}

bool strides_ok(const int64_t (&s)[3], int64_t multiple = 8) {
    for (int i = 0; i < 3; i++)
        if (s[i] < 0 || s[i] % multiple) return false;
    return s[2] >= kD;
}

bool desc_ok(const rest_kv_desc* d) {
    if (!d) return false;
    if (d->Nb < 1 || d->H < 1 || d->T < 1 || d->T > REST_MAX_NODES || d->D != kD || d->P < 0) return false;
    if (d->Nb > 65535) return false;                 // grid y
    if (!(d->theta > 1.0) || !(d->theta < 1e30)) return false;
    if ((int64_t)d->P + d->T > 0x7fffffff) return false;
    if (d->cache_dtype != REST_KV_AS_DTYPE && d->cache_dtype != REST_KV_FP8_E4M3) return false;
    // rows are moved in 16-byte pieces
    const int64_t mult = d->cache_dtype == REST_KV_FP8_E4M3 ? 16 : 8;
    return strides_ok(d->kc_stride, mult) && strides_ok(d->vc_stride, mult);
}

void fill(KvParams& p, const rest_kv_desc* d) {
    p.Nb = d->Nb; p.H = d->H; p.T = d->T; p.P = d->P; p.pos_offset = d->pos_offset;
    p.per_batch = d->per_batch ? 1 : 0;
    p.log2_theta = log2(d->theta);
    const bool c8 = d->cache_dtype == REST_KV_FP8_E4M3;
    p.k_scale = c8 ? d->d_k_scale : nullptr;
    p.v_scale = c8 ? d->d_v_scale : nullptr;
    for (int i = 0; i < 3; i++) {
        p.qs[i] = d->q_stride[i]; p.kns[i] = d->kn_stride[i]; p.vns[i] = d->vn_stride[i];
        p.kcs[i] = d->kc_stride[i]; p.vcs[i] = d->vc_stride[i];
    }
}

}  // namespace

extern "C" __attribute__((visibility("default"))) rest_status rest_rope_append(void* d_q, const void* d_k_new, const void* d_v_new, void* d_k_cache,
                                        void* d_v_cache, const int32_t* d_pos_ids, const rest_kv_desc* d, void* stream) {
    if (!desc_ok(d) || !d_q || !d_k_new || !d_v_new || !d_k_cache || !d_v_cache || !d_pos_ids) return REST_INVALID_ARG;
    if (!strides_ok(d->q_stride) || !strides_ok(d->kn_stride) || !strides_ok(d->vn_stride)) return REST_INVALID_ARG;
    if (((uintptr_t)d_q | (uintptr_t)d_k_new | (uintptr_t)d_v_new | (uintptr_t)d_k_cache | (uintptr_t)d_v_cache) & 15)
        return REST_INVALID_ARG;
    if (d->dtype != REST_BF16) return REST_UNSUPPORTED;
    KvParams p{};
    fill(p, d);
    p.q = (__bf16*)d_q; p.kn = (const __bf16*)d_k_new; p.vn = (const __bf16*)d_v_new;
    p.kc = (__bf16*)d_k_cache; p.vc = (__bf16*)d_v_cache;
    p.pos_ids = d_pos_ids;
    const int tg = (d->T + 3) / 4, hg = (d->H + 7) / 8;
    // enough workgroups to fill the chip, at most one per eight heads
    int gz = (int)((2048 + (int64_t)tg * d->Nb - 1) / ((int64_t)tg * d->Nb));
    gz = gz < 1 ? 1 : (gz > hg ? hg : gz);
    if (d->cache_dtype == REST_KV_FP8_E4M3)
        hipLaunchKernelGGL(rope_append_kernel<true>, dim3(tg, d->Nb, gz), dim3(256), 0, (hipStream_t)stream, p);
    else
        hipLaunchKernelGGL(rope_append_kernel<false>, dim3(tg, d->Nb, gz), dim3(256), 0, (hipStream_t)stream, p);
    REST_HIP_TRY(hipGetLastError());
    return REST_OK;
}

extern "C" __attribute__((visibility("default"))) rest_status rest_kv_compact(void* d_k_cache, void* d_v_cache, const int32_t* d_accept_path,
                                       const int32_t* d_accept_len, int32_t path_cap, const rest_kv_desc* d, void* stream) {
    if (!desc_ok(d) || !d_k_cache || !d_v_cache || !d_accept_path || !d_accept_len) return REST_INVALID_ARG;
    if (path_cap < 1 || path_cap > REST_MAX_CONT_LEN) return REST_INVALID_ARG;
    if (((uintptr_t)d_k_cache | (uintptr_t)d_v_cache) & 15) return REST_INVALID_ARG;
    if (d->dtype != REST_BF16) return REST_UNSUPPORTED;
    KvParams p{};
    fill(p, d);
    p.kc = (__bf16*)d_k_cache; p.vc = (__bf16*)d_v_cache;
    p.path = d_accept_path;
    p.path_len = d_accept_len;
    p.path_cap = path_cap;
    if (d->cache_dtype == REST_KV_FP8_E4M3)
        hipLaunchKernelGGL(kv_compact_kernel<1>, dim3(d->H, d->Nb), dim3(512), 0, (hipStream_t)stream, p);
    else
        hipLaunchKernelGGL(kv_compact_kernel<2>, dim3(d->H, d->Nb), dim3(512), 0, (hipStream_t)stream, p);
    REST_HIP_TRY(hipGetLastError());
    return REST_OK;
}
