// Decode-time attention of one new token over a KV cache (Sec. 2.1 Eq. 1 for a single query position), for the
// compacted cache the compression path produces and for the full cache it replaces.  GQA: the G query heads of
// a KV head share its rows.  The work is one read of K and V, so the kernel is a plain streaming one:
//
//   decode_partial_kernel  grid (splits, P), 256 threads.  A row (D elements) is spread over D*elt/16 consecutive
//       lanes, 16 bytes each, so every load instruction of a wavefront covers whole consecutive rows; the lane
//       groups of a workgroup stride over the rows of the split.  Per group an online softmax (running maximum,
//       denominator, weighted sum of V) in the log2 domain, the scale 1/sqrt(D) folded into the query; four rows
//       are loaded before the first is used.  The groups' partial results are merged through LDS and written as
//       (maximum, denominator, numerator[D]) per (problem, split, head).
//   decode_merge_kernel    grid (P): merges the splits and divides.
#include "sablock_internal.h"

namespace sablock {
namespace {

constexpr int DT = 256;                    // threads per workgroup
constexpr int UNROLL = 4;                  // rows in flight per lane group
constexpr size_t MAX_LDS = 72 * 1024;      // merge buffer of the lane groups (largest: G = 8, D = 128, bf16)

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// 16 bytes that are read once: non-temporal
__device__ inline uint4 load16(const char *p)
{
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
    return make_uint4(v[0], v[1], v[2], v[3]);
}

// sum over the LPR consecutive lanes that hold one row (LPR a power of two, the group is LPR-aligned); every lane
// of the group gets the sum.  Up to 16 lanes the exchanges are DPP row operations, no LDS traffic.
template <int LPR>
__device__ inline float row_sum(float x)
{
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xF, 0xF, true));   // lane ^ 1
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xF, 0xF, true));   // lane ^ 2
    if (LPR >= 8) x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x141, 0xF, 0xF, true));  // mirror in 8
    if (LPR >= 16) x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x140, 0xF, 0xF, true)); // mirror in 16
    if (LPR >= 32) x += __shfl_xor(x, 16);
    if (LPR >= 64) x += __shfl_xor(x, 32);
    return x;
}

template <bool BF16> struct Chunk;         // 16 bytes of a row as floats
template <> struct Chunk<true> {
    static constexpr int N = 8;
    __device__ static void load(const char *p, float (&f)[8])
    {
        const uint4 u = load16(p);
        const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) { f[2 * i] = __uint_as_float(w[i] << 16); f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u); }
    }
};
template <> struct Chunk<false> {
    static constexpr int N = 4;
    __device__ static void load(const char *p, float (&f)[4])
    {
        const uint4 u = load16(p);
        f[0] = __uint_as_float(u.x); f[1] = __uint_as_float(u.y); f[2] = __uint_as_float(u.z); f[3] = __uint_as_float(u.w);
    }
};

struct DecodeArgs {
    Dims d;                 // d.L = rows of the cache buffers
    const char *q, *k, *v;
    const int32_t *n_sel;   // nullable; rows [n_sel[p], budget) of problem p hold nothing
    int budget;
    int rows_per_split, n_splits;
    int lpr;                // lanes per row = D * elt / 16, a power of two in [4, 64]
    float qscale;           // log2(e) / sqrt(D)
    float *part;            // [P][n_splits][G][2 + D]
    float *out;             // [n_seq][n_layers][Hq][D]
};

template <int G, bool BF16, int LPR>
__global__ void __launch_bounds__(DT)
decode_partial_kernel(DecodeArgs a)
{
    extern __shared__ float sh[];          // [groups][G][2 + D]
    constexpr int E = Chunk<BF16>::N;
    constexpr int ELT = BF16 ? 2 : 4;
    const Dims &d = a.d;
    const int p = blockIdx.y, split = blockIdx.x;
    constexpr int lpr = LPR, groups = DT / LPR;
    const int grp = threadIdx.x / lpr, sub = threadIdx.x % lpr;
    const int D = d.D;
    const int r0 = split * a.rows_per_split, r1 = min(r0 + a.rows_per_split, d.L);
    const int hole_lo = a.n_sel ? a.n_sel[p] : d.L, hole_hi = a.n_sel ? a.budget : d.L;   // rows without content
    const int head0 = head_of_problem(d, p) * G;
    const int64_t qbase = ((int64_t)(seq_of_problem(d, p) * d.n_layers + layer_of_problem(d, p)) * d.Hq + head0) * D;

    float qf[G][E];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        Chunk<BF16>::load(a.q + (qbase + (int64_t)g * D + sub * E) * ELT, qf[g]);
#pragma unroll
        for (int e = 0; e < E; ++e) qf[g][e] *= a.qscale;
    }
    float m[G], l[G], acc[G][E];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        m[g] = -INFINITY; l[g] = 0.f;
#pragma unroll
        for (int e = 0; e < E; ++e) acc[g][e] = 0.f;
    }
    const char *kp = a.k + k_problem_offset(d, p) * ELT + (int64_t)sub * 16;
    const char *vp = a.v + v_problem_offset(d, p) * ELT + (int64_t)sub * 16;
    const int64_t kstep = d.ks[3] * ELT, vstep = d.vs[3] * ELT;

    for (int rb = r0 + grp; rb < r1; rb += groups * UNROLL) {
        float kf[UNROLL][E], vf[UNROLL][E];
        bool live[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int r = rb + u * groups;
            live[u] = r < r1 && !(r >= hole_lo && r < hole_hi);
            const int rc = min(r, r1 - 1);                 // in bounds; the value is unused when not live
            Chunk<BF16>::load(kp + (int64_t)rc * kstep, kf[u]);
            Chunk<BF16>::load(vp + (int64_t)rc * vstep, vf[u]);
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float x = 0.f;
#pragma unroll
                for (int e = 0; e < E; ++e) x = fmaf(qf[g][e], kf[u][e], x);
                x = row_sum<LPR>(x);                               // every lane of the row holds the logit
                if (live[u]) {
                    const float mn = fmaxf(m[g], x);
                    const float corr = __builtin_amdgcn_exp2f(m[g] - mn);        // exp2(-inf) = 0 on the first row
                    const float pe = __builtin_amdgcn_exp2f(x - mn);
                    l[g] = l[g] * corr + pe;
#pragma unroll
                    for (int e = 0; e < E; ++e) acc[g][e] = fmaf(pe, vf[u][e], acc[g][e] * corr);
                    m[g] = mn;
                }
            }
        }
    }
    // merge the lane groups of the workgroup
    const int stride = 2 + D;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        float *o = sh + ((int64_t)grp * G + g) * stride;
        if (sub == 0) { o[0] = m[g]; o[1] = l[g]; }
#pragma unroll
        for (int e = 0; e < E; ++e) o[2 + sub * E + e] = acc[g][e];
    }
    __syncthreads();
    float *po = a.part + ((int64_t)p * a.n_splits + split) * G * stride;
    for (int i = threadIdx.x; i < G * stride; i += DT) {
        const int g = i / stride, c = i - g * stride;
        float mx = -INFINITY;
        for (int w = 0; w < groups; ++w) mx = fmaxf(mx, sh[((int64_t)w * G + g) * stride]);
        float val = 0.f;
        if (c == 0) val = mx;
        else if (mx > -INFINITY)
            for (int w = 0; w < groups; ++w) {
                const float *o = sh + ((int64_t)w * G + g) * stride;
                val += o[c] * __builtin_amdgcn_exp2f(o[0] - mx);
            }
        po[i] = val;
    }
}

// grid (P), G * D threads (<= 1024)
__global__ void decode_merge_kernel(DecodeArgs a, int G)
{
    const Dims &d = a.d;
    const int p = blockIdx.x, D = d.D, stride = 2 + D;
    const int g = threadIdx.x / D, c = threadIdx.x - g * D;
    if (g >= G) return;
    const float *pp = a.part + (int64_t)p * a.n_splits * G * stride + (int64_t)g * stride;
    float mx = -INFINITY;
    for (int s = 0; s < a.n_splits; ++s) mx = fmaxf(mx, pp[(int64_t)s * G * stride]);
    float num = 0.f, den = 0.f;
    if (mx > -INFINITY)
        for (int s = 0; s < a.n_splits; ++s) {
            const float *o = pp + (int64_t)s * G * stride;
            const float w = __builtin_amdgcn_exp2f(o[0] - mx);
            den += o[1] * w;
            num += o[2 + c] * w;
        }
    const int head0 = head_of_problem(d, p) * G;
    const int64_t obase = ((int64_t)(seq_of_problem(d, p) * d.n_layers + layer_of_problem(d, p)) * d.Hq + head0 + g) * D;
    a.out[obase + c] = den > 0.f ? num / den : 0.f;
}

int pick_splits(const Dims &d)
{
    // enough workgroups to fill 256 CUs many times over (short tail), at least 256 rows each
    int s = 1;
    while ((int64_t)d.P * s < 8192 && d.L / (s * 2) >= 256) s *= 2;
    return s;
}

}  // namespace

bool decode_supported(const Dims &d)
{
    const int elt = d.dtype == SABLOCK_F32 ? 4 : 2;
    const int lpr = d.D * elt / 16;
    const bool pow2 = lpr >= 4 && lpr <= 64 && (lpr & (lpr - 1)) == 0 && lpr * 16 == d.D * elt;
    const bool g_ok = d.G >= 1 && d.G <= 8;
    return pow2 && g_ok && d.G * d.D <= 1024 && (size_t)(DT / (pow2 ? lpr : 4)) * d.G * (2 + d.D) * 4 <= MAX_LDS;
}

size_t decode_ws_bytes(const Dims &d)
{
    return align256((size_t)d.P * pick_splits(d) * d.G * (2 + d.D) * 4);
}

hipError_t launch_decode(const Dims &d, const void *q, const void *k, const void *v, const int32_t *n_sel,
                         int32_t budget, float *out, void *ws, hipStream_t st)
{
    if (d.P <= 0) return hipSuccess;
    const int elt = d.dtype == SABLOCK_F32 ? 4 : 2;
    DecodeArgs a;
    a.d = d;
    a.q = static_cast<const char *>(q);
    a.k = static_cast<const char *>(k);
    a.v = static_cast<const char *>(v);
    a.n_sel = n_sel;
    a.budget = budget;
    a.n_splits = pick_splits(d);
    a.rows_per_split = (d.L + a.n_splits - 1) / a.n_splits;
    a.lpr = d.D * elt / 16;
    a.qscale = (float)(1.4426950408889634 / sqrt((double)d.D));
    a.part = static_cast<float *>(ws);
    a.out = out;
    const size_t lds = (size_t)(DT / a.lpr) * d.G * (2 + d.D) * 4;
    dim3 grid(a.n_splits, d.P);
    const bool bf = d.dtype == SABLOCK_BF16;
    // one instantiation per (G, dtype, lanes per row)
    using Kern = void (*)(DecodeArgs);
    Kern fn = nullptr;
#define SABLOCK_DECODE_L(GV, BV, LV) if (d.G == GV && bf == BV && a.lpr == LV) fn = decode_partial_kernel<GV, BV, LV>;
#define SABLOCK_DECODE_G(GV)                                                                                         \
    SABLOCK_DECODE_L(GV, true, 4) SABLOCK_DECODE_L(GV, true, 8) SABLOCK_DECODE_L(GV, true, 16) SABLOCK_DECODE_L(GV, true, 32) \
    SABLOCK_DECODE_L(GV, false, 4) SABLOCK_DECODE_L(GV, false, 8) SABLOCK_DECODE_L(GV, false, 16)                    \
    SABLOCK_DECODE_L(GV, false, 32) SABLOCK_DECODE_L(GV, false, 64)
    SABLOCK_DECODE_G(1) SABLOCK_DECODE_G(2) SABLOCK_DECODE_G(3) SABLOCK_DECODE_G(4) SABLOCK_DECODE_G(5) SABLOCK_DECODE_G(6)
    SABLOCK_DECODE_G(7) SABLOCK_DECODE_G(8)
#undef SABLOCK_DECODE_G
#undef SABLOCK_DECODE_L
    if (!fn) return hipErrorInvalidValue;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(fn), hipFuncAttributeMaxDynamicSharedMemorySize, (int)MAX_LDS);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(fn, grid, dim3(DT), lds, st, a);
    hipLaunchKernelGGL(decode_merge_kernel, dim3(d.P), dim3(d.G * d.D), 0, st, a, d.G);
    return hipGetLastError();
}

}  // namespace sablock
