// Window scoring for any shape and element type (Sec. 3.2, Eqs. barA, st, Dk).
//
// Plain-ALU kernels: one thread per key, the window-query rows broadcast from
// LDS eight at a time.  This is the path for fp32 inputs and for shapes the
// MFMA kernel does not cover; it favours generality over speed.
//
// Pass 1 (skipped when the caller supplies row_lse): per window-query row the
// running (max, sum exp) of its scaled logits over the visible keys, per key
// chunk, then a combine kernel turns the chunk partials into one log-sum-exp
// per row.  Pass 2: probabilities exp(x - lse), head mean, column sum s_t and
// the per-token entropy term.
#include "sablock_internal.h"

#include <hip/hip_bf16.h>

namespace sablock {
namespace {

constexpr int RG = 8;          // window-query rows held in LDS at a time
constexpr int NT = 256;        // threads per block
constexpr int MAX_W = 64;

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ inline void load8(const float *p, float out[8])
    {
        float4 a = *reinterpret_cast<const float4 *>(p), b = *reinterpret_cast<const float4 *>(p + 4);
        out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w;
        out[4] = b.x; out[5] = b.y; out[6] = b.z; out[7] = b.w;
    }
    static __device__ inline float load1(const float *p) { return *p; }
};
template <> struct Elem<uint16_t> {   // bf16 bit patterns
    static __device__ inline float cvt(uint32_t h) { return __uint_as_float(h << 16); }
    static __device__ inline void load8(const uint16_t *p, float out[8])
    {
        uint4 a = *reinterpret_cast<const uint4 *>(p);
        out[0] = cvt(a.x & 0xffffu); out[1] = cvt(a.x >> 16);
        out[2] = cvt(a.y & 0xffffu); out[3] = cvt(a.y >> 16);
        out[4] = cvt(a.z & 0xffffu); out[5] = cvt(a.z >> 16);
        out[6] = cvt(a.w & 0xffffu); out[7] = cvt(a.w >> 16);
    }
    static __device__ inline float load1(const uint16_t *p) { return cvt(*p); }
};

// stage rows r0 .. r0+RG-1 (row r = h_local * W + i) of the problem's window queries into LDS as float
template <typename T>
__device__ inline void stage_q_rows(const Dims &d, const T *q, int p, int r0, float *q_lds)
{
    for (int e = threadIdx.x; e < RG * d.D; e += blockDim.x) {
        int rr = e / d.D, dd = e - rr * d.D;
        int r = r0 + rr;
        float v = 0.f;
        if (r < d.M) v = Elem<T>::load1(q + q_row_offset(d, p, r / d.W, r % d.W) + dd);
        q_lds[e] = v;
    }
}

// x[rr] = <q_row(r0+rr), k_t> for the RG staged rows
template <typename T>
__device__ inline void dots(const Dims &d, const T *krow, const float *q_lds, float x[RG])
{
#pragma unroll
    for (int rr = 0; rr < RG; ++rr) x[rr] = 0.f;
    for (int dd = 0; dd < d.D; dd += 8) {
        float kv[8];
        Elem<T>::load8(krow + dd, kv);
#pragma unroll
        for (int rr = 0; rr < RG; ++rr) {
            const float *qr = q_lds + rr * d.D + dd;
#pragma unroll
            for (int j = 0; j < 8; ++j) x[rr] = fmaf(qr[j], kv[j], x[rr]);
        }
    }
}

// ---------------------------------------------------------------- pass 1
// grid (n_chunks, ceil(M/RG), P); partial[((p * n_chunks + chunk) * M + r) * 2 + {0,1}] = (max, sum exp)
template <typename T>
__global__ void __launch_bounds__(NT)
score_generic_stats(Dims d, const T *q, const T *k, int chunk_len, int n_chunks, float *partial)
{
    extern __shared__ float lds[];
    float *q_lds = lds;                       // RG * D
    float *red = lds + RG * d.D;              // (NT/64) * RG * 2
    const int p = blockIdx.z, r0 = blockIdx.y * RG, chunk = blockIdx.x;
    const float scale = 1.0f / sqrtf((float)d.D);
    stage_q_rows<T>(d, q, p, r0, q_lds);
    __syncthreads();

    const T *kp = k + k_problem_offset(d, p);
    const int lo = chunk * chunk_len;
    const int hi = min(lo + chunk_len, d.L);
    float m[RG], z[RG];
#pragma unroll
    for (int rr = 0; rr < RG; ++rr) { m[rr] = -INFINITY; z[rr] = 0.f; }

    for (int t = lo + threadIdx.x; t < hi; t += NT) {
        float x[RG];
        dots<T>(d, kp + (int64_t)t * d.ks[3], q_lds, x);
#pragma unroll
        for (int rr = 0; rr < RG; ++rr) {
            int r = r0 + rr;
            int i = r % d.W;
            bool vis = (r < d.M) && (t <= d.T + i);          // causal inside the window
            if (vis) {
                float xv = x[rr] * scale;
                float mn = fmaxf(m[rr], xv);
                z[rr] = z[rr] * expf(m[rr] - mn) + expf(xv - mn);   // exp(-inf) = 0 on the first key
                m[rr] = mn;
            }
        }
    }
    // reduce (m, z) over the block: wave shuffles, then across waves through LDS
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int rr = 0; rr < RG; ++rr) {
        for (int off = 32; off > 0; off >>= 1) {
            float mo = __shfl_xor(m[rr], off), zo = __shfl_xor(z[rr], off);
            float mn = fmaxf(m[rr], mo);
            float za = (m[rr] == -INFINITY) ? 0.f : z[rr] * expf(m[rr] - mn);
            float zb = (mo == -INFINITY) ? 0.f : zo * expf(mo - mn);
            m[rr] = mn; z[rr] = za + zb;
        }
        if (lane == 0) { red[(wave * RG + rr) * 2] = m[rr]; red[(wave * RG + rr) * 2 + 1] = z[rr]; }
    }
    __syncthreads();
    if (threadIdx.x < RG && r0 + threadIdx.x < d.M) {
        int rr = threadIdx.x;
        float mm = -INFINITY, zz = 0.f;
        for (int w = 0; w < NT / 64; ++w) {
            float mo = red[(w * RG + rr) * 2], zo = red[(w * RG + rr) * 2 + 1];
            float mn = fmaxf(mm, mo);
            float za = (mm == -INFINITY) ? 0.f : zz * expf(mm - mn);
            float zb = (mo == -INFINITY) ? 0.f : zo * expf(mo - mn);
            mm = mn; zz = za + zb;
        }
        float *o = partial + (((int64_t)p * n_chunks + chunk) * d.M + (r0 + rr)) * 2;
        o[0] = mm; o[1] = zz;
    }
}

// one thread per (problem, row): lse = max + ln(sum)
__global__ void score_generic_combine(Dims d, int n_chunks, const float *partial, float *lse)
{
    int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= (int64_t)d.P * d.M) return;
    int p = (int)(gid / d.M), r = (int)(gid % d.M);
    float mm = -INFINITY;
    for (int c = 0; c < n_chunks; ++c) mm = fmaxf(mm, partial[(((int64_t)p * n_chunks + c) * d.M + r) * 2]);
    float zz = 0.f;
    for (int c = 0; c < n_chunks; ++c) {
        const float *o = partial + (((int64_t)p * n_chunks + c) * d.M + r) * 2;
        if (o[0] != -INFINITY) zz += o[1] * expf(o[0] - mm);
    }
    lse[gid] = mm + logf(zz);
}

// ---------------------------------------------------------------- pass 2
// grid (ceil(L/NT), P); lse [P][M] natural-log sum-exp of the scaled logits
template <typename T>
__global__ void __launch_bounds__(NT)
score_generic_columns(Dims d, const T *q, const T *k, const float *lse, float eps, float *s_out, float *ent_out)
{
    extern __shared__ float lds[];
    float *q_lds = lds;                       // RG * D
    float *lse_lds = lds + RG * d.D;          // M
    const int p = blockIdx.y;
    const int t = blockIdx.x * NT + threadIdx.x;
    const bool live = t < d.L;
    const float scale = 1.0f / sqrtf((float)d.D);
    const T *krow = k + k_problem_offset(d, p) + (int64_t)(live ? t : 0) * d.ks[3];
    for (int r = threadIdx.x; r < d.M; r += NT) lse_lds[r] = lse[(int64_t)p * d.M + r];

    float abar[MAX_W];
    for (int i = 0; i < d.W; ++i) abar[i] = 0.f;

    for (int r0 = 0; r0 < d.M; r0 += RG) {
        __syncthreads();
        stage_q_rows<T>(d, q, p, r0, q_lds);
        __syncthreads();
        float x[RG];
        dots<T>(d, krow, q_lds, x);
#pragma unroll
        for (int rr = 0; rr < RG; ++rr) {
            int r = r0 + rr;
            if (r < d.M) {
                int i = r % d.W;
                if (live && t <= d.T + i) abar[i] += expf(x[rr] * scale - lse_lds[r]);
            }
        }
    }
    if (!live) return;
    float s = 0.f;
    const float inv_g = 1.0f / (float)d.G;
    for (int i = 0; i < d.W; ++i) { abar[i] *= inv_g; s += abar[i]; }       // Eq. barA, Eq. st
    float ent = 0.f;
    if (s > 0.f) {
        float inv_s = 1.0f / s;
        for (int i = 0; i < d.W; ++i) {
            float ah = abar[i] * inv_s;
            ent -= ah * logf(ah + eps);                                      // inner sum of Eq. Dk
        }
    }
    s_out[(int64_t)p * d.L + t] = s;
    ent_out[(int64_t)p * d.L + t] = ent;
}

int generic_chunks(const Dims &d, int *chunk_len)
{
    int target = 64;                                   // at most 64 chunk partials per row
    int len = (d.L + target - 1) / target;
    len = ((len + NT - 1) / NT) * NT;
    *chunk_len = len;
    return (d.L + len - 1) / len;
}

template <typename T>
hipError_t run(const Dims &d, const void *q, const void *k, const float *row_lse, float eps,
               float *s_out, float *ent_out, void *ws, hipStream_t st)
{
    const T *qq = static_cast<const T *>(q);
    const T *kk = static_cast<const T *>(k);
    const float *lse = row_lse;
    if (!lse) {
        int chunk_len, n_chunks = generic_chunks(d, &chunk_len);
        float *lse_ws = static_cast<float *>(ws);
        float *partial = reinterpret_cast<float *>(static_cast<char *>(ws) + align256((size_t)d.P * d.M * 4));
        size_t lds1 = (size_t)(RG * d.D + (NT / 64) * RG * 2) * sizeof(float);
        dim3 g1(n_chunks, (d.M + RG - 1) / RG, d.P);
        hipLaunchKernelGGL(score_generic_stats<T>, g1, dim3(NT), lds1, st, d, qq, kk, chunk_len, n_chunks, partial);
        int64_t rows = (int64_t)d.P * d.M;
        hipLaunchKernelGGL(score_generic_combine, dim3((unsigned)((rows + 255) / 256)), dim3(256), 0, st,
                           d, n_chunks, partial, lse_ws);
        lse = lse_ws;
    }
    size_t lds2 = (size_t)(RG * d.D + d.M) * sizeof(float);
    dim3 g2((d.L + NT - 1) / NT, d.P);
    hipLaunchKernelGGL(score_generic_columns<T>, g2, dim3(NT), lds2, st, d, qq, kk, lse, eps, s_out, ent_out);
    return hipGetLastError();
}

}  // namespace

size_t score_generic_ws_bytes(const Dims &d)
{
    int chunk_len, n_chunks = generic_chunks(d, &chunk_len);
    return align256((size_t)d.P * d.M * 4) + align256((size_t)d.P * n_chunks * d.M * 2 * 4);
}

hipError_t launch_score_generic(const Dims &d, const void *q, const void *k, const float *row_lse, float eps,
                                float *s_out, float *ent_out, void *ws, hipStream_t st)
{
    if (d.dtype == SABLOCK_F32) return run<float>(d, q, k, row_lse, eps, s_out, ent_out, ws, st);
    return run<uint16_t>(d, q, k, row_lse, eps, s_out, ent_out, ws, st);
}

}  // namespace sablock
