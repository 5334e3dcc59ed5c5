// MFMA window scoring (Sec. 3.2, Eqs. barA, st, Dk) for bf16, D = 128, G = 4, W = 32.
//
// The 128 window-query rows of a KV head (4 query heads x 32 window queries)
// stay in registers as MFMA A operands; keys are the B operand, 32 per
// wavefront iteration ("subtile"), so in the 32x32 accumulator layout a lane
// owns ONE key column and 16 of the 32 queries of each head:
//   * the head mean (Eq. barA) is an in-lane add over the four accumulators,
//   * the column sum (Eq. st) is 16 in-lane adds plus one exchange between the
//     two lane halves, and so is the entropy term (inner sum of Eq. Dk),
//   * the per-row softmax statistics are kept per lane and only reduced across
//     lanes once per workgroup.
// Each wavefront streams its own keys: global -> LDS with direct-to-LDS loads
// (16 bytes per lane, fully coalesced 256-byte key rows) into a private
// four-deep ring, LDS -> registers with an XOR swizzle so the 16-byte reads of 32
// different key rows do not collide on banks.  No workgroup barrier in the loop.
//
// Softmax over all keys needs each row's log-sum-exp before any column is
// final, so scoring is two kernels unless the caller supplies row_lse:
//   pass 1  row statistics (running reference, sum of exp2) per key chunk,
//   combine chunk partials -> natural-log lse per row,
//   pass 2  probabilities, head mean, column sum, entropy term.
// Problems are processed in groups whose keys fit the memory-side cache, so the
// second read of K is served from it rather than from HBM.
#include "sablock_internal.h"

#include <cstdlib>

namespace sablock {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef const void __attribute__((address_space(1))) *gptr_t;
typedef void __attribute__((address_space(3))) *lptr_t;

constexpr int SUB = 32;                    // keys per wavefront iteration
constexpr int NBUF = 4;                    // ring depth (subtiles) per wavefront
constexpr int WAVES = 4;
constexpr int ROW_BYTES = 256;             // D = 128 bf16
constexpr int BUF_BYTES = SUB * ROW_BYTES; // 8 KiB
constexpr int RING_BYTES = NBUF * BUF_BYTES;
constexpr int M_ROWS = 128;
constexpr int LDS_BYTES = WAVES * RING_BYTES + WAVES * M_ROWS * 2 * 4;
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;
constexpr float RESCALE_AT = 64.f;         // pass 1 moves a row's reference when an exponent exceeds this

struct ScoreArgs {
    Dims d;
    const uint16_t *q, *k;
    int p0;                // first problem of the group
    int chunk_len;         // keys per workgroup, multiple of WAVES * SUB
    int n_chunks;          // workgroups per problem
    float c1;              // log2(e) / sqrt(D)
    float eps;
    float *partial;        // pass 1 out: [group problem][chunk][128][2] (reference, sum) in the log2 domain
    const float *lse;      // pass 2 in: [P][128] natural-log sum-exp per row
    float *s_out, *e_out;  // pass 2 out: [P][L]
};

__device__ inline uint32_t lds_addr(const void *p)
{
    return (uint32_t)(uintptr_t)(lptr_t)p;
}

// Window-query rows as A operands: qa[h][s] = Q[h][lane % 32][(2s + lane/32) * 8 .. +8]
__device__ inline void load_q(const Dims &d, const uint16_t *q, int p, int lane, bf16x8 qa[4][8])
{
    const int iq = lane & 31, hf = lane >> 5;
#pragma unroll
    for (int h = 0; h < 4; ++h) {
        const uint16_t *row = q + q_row_offset(d, p, h, iq);
#pragma unroll
        for (int s = 0; s < 8; ++s) qa[h][s] = *reinterpret_cast<const bf16x8 *>(row + (2 * s + hf) * 8);
    }
}

// Direct-to-LDS load of 32 key rows starting at t0 (rows past L-1 are clamped): 8 instructions of
// 1 KiB; LDS slot (row, pos) receives 16-byte chunk pos ^ (row & 15) of the row.
__device__ inline void issue_subtile(const uint16_t *kp, int64_t ks3, int t0, int L, char *buf, int lane)
{
    const int r4 = lane >> 4, pos = lane & 15;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int row = 4 * j + r4;
        const int t = min(t0 + row, L - 1);
        const uint16_t *g = kp + (int64_t)t * ks3 + ((pos ^ (row & 15)) << 3);
        __builtin_amdgcn_global_load_lds((gptr_t)g, (lptr_t)(buf + j * 1024), 16, 0, 0);
    }
}

// B operands of one subtile: kb[s] = K[key lane % 32][(2s + lane/32) * 8 .. +8]
__device__ inline void read_subtile(uint32_t buf_addr, const uint32_t xoff[8], bf16x8 kb[8])
{
#pragma unroll
    for (int s = 0; s < 8; ++s)
        asm volatile("ds_read_b128 %0, %1" : "=v"(kb[s]) : "v"(buf_addr + xoff[s]) : "memory");
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(kb[0]), "+v"(kb[1]), "+v"(kb[2]), "+v"(kb[3]), "+v"(kb[4]), "+v"(kb[5]), "+v"(kb[6]), "+v"(kb[7])
                 :
                 : "memory");
}

// wait until at most `loads_after` of this wavefront's vector-memory operations are outstanding
__device__ inline void wait_loads(int subtiles_after)
{
    if (subtiles_after >= 2) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
    else if (subtiles_after == 1) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

__device__ inline void qk_tile(const bf16x8 qa[4][8], const bf16x8 kb[8], floatx16 acc[4])
{
#pragma unroll
    for (int h = 0; h < 4; ++h)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[h][i] = 0.f;
#pragma unroll
    for (int s = 0; s < 8; ++s)
#pragma unroll
        for (int h = 0; h < 4; ++h) acc[h] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa[h][s], kb[s], acc[h], 0, 0, 0);
}

// window query owned by accumulator register i in lane half hf
__device__ inline int query_of(int i, int hf) { return 8 * (i >> 2) + 4 * hf + (i & 3); }

struct WaveWork {
    const uint16_t *kp;    // keys of the problem
    int p, pl, chunk;
    int first, n_sub;      // this wavefront's subtiles: keys [first + u * WAVES * SUB, +SUB), u < n_sub
};

__device__ inline WaveWork wave_work(const ScoreArgs &a, int wave)
{
    WaveWork w;
    w.pl = blockIdx.x / a.n_chunks;
    w.chunk = blockIdx.x - w.pl * a.n_chunks;
    w.p = a.p0 + w.pl;
    w.kp = a.k + k_problem_offset(a.d, w.p);
    const int lo = w.chunk * a.chunk_len;
    const int hi = min(lo + a.chunk_len, a.d.L);
    w.first = lo + wave * SUB;
    const int span = hi - w.first;
    w.n_sub = span > 0 ? (span + WAVES * SUB - 1) / (WAVES * SUB) : 0;
    return w;
}

// ------------------------------------------------------------------ pass 1
__global__ void __launch_bounds__(WAVES * 64)
score_mfma_stats(ScoreArgs a)
{
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 31, hf = lane >> 5;
    const Dims &d = a.d;
    char *ring = lds + wave * RING_BYTES;
    float *wg_red = reinterpret_cast<float *>(lds + WAVES * RING_BYTES);     // [WAVES][128][2]
    const WaveWork w = wave_work(a, wave);

    bf16x8 qa[4][8];
    load_q(d, a.q, w.p, lane, qa);
    uint32_t xoff[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) xoff[s] = n * ROW_BYTES + (((2 * s + hf) ^ (n & 15)) << 4);
    const uint32_t ring_addr = lds_addr(ring);

    float r[4][16], z[4][16];
#pragma unroll
    for (int h = 0; h < 4; ++h)
#pragma unroll
        for (int i = 0; i < 16; ++i) { r[h][i] = -INFINITY; z[h][i] = 0.f; }

    const int stride = WAVES * SUB;
    for (int u = 0; u < min(NBUF - 1, w.n_sub); ++u)
        issue_subtile(w.kp, d.ks[3], w.first + u * stride, d.L, ring + u * BUF_BYTES, lane);

    for (int u = 0; u < w.n_sub; ++u) {
        wait_loads(min(NBUF - 2, w.n_sub - 1 - u));
        bf16x8 kb[8];
        read_subtile(ring_addr + (u % NBUF) * BUF_BYTES, xoff, kb);
        if (u + NBUF - 1 < w.n_sub)
            issue_subtile(w.kp, d.ks[3], w.first + (u + NBUF - 1) * stride, d.L,
                          ring + ((u + NBUF - 1) % NBUF) * BUF_BYTES, lane);
        floatx16 acc[4];
        qk_tile(qa, kb, acc);

        const int t = w.first + u * stride + n;                // this lane's key
        const bool edge = w.first + u * stride + SUB > d.T;    // subtile touches the window keys or the end
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            float dd[16];
            float dmax = -INFINITY;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                float v = fmaf(acc[h][i], a.c1, -r[h][i]);
                if (edge && !(t < d.L && t <= d.T + query_of(i, hf))) v = -INFINITY;   // causal inside the window
                dd[i] = v;
                dmax = fmaxf(dmax, v);
            }
            if (__any(dmax > RESCALE_AT)) {
                // move the reference of the rows whose new logit is far above it (also the first visit: r = -inf)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    if (dd[i] > RESCALE_AT) {
                        z[h][i] *= __builtin_amdgcn_exp2f(-dd[i]);
                        r[h][i] = acc[h][i] * a.c1;
                        dd[i] = 0.f;
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) z[h][i] += __builtin_amdgcn_exp2f(dd[i]);
        }
    }

    // ---- reduce the lane-local (reference, sum) pairs: over the 32 lanes of a half through the wavefront's
    // ring (all loads have landed: the last iteration waited for everything), then over wavefronts
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    float *scr_r = reinterpret_cast<float *>(ring);            // [128][32]
    float *scr_z = scr_r + M_ROWS * 32;                        // [128][32]
#pragma unroll
    for (int h = 0; h < 4; ++h)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int row = h * 32 + query_of(i, hf);
            scr_r[row * 32 + n] = r[h][i];
            scr_z[row * 32 + n] = z[h][i];
        }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int rr = 0; rr < 2; ++rr) {
        const int row = lane + 64 * rr;
        float m = -INFINITY;
        for (int j = 0; j < 32; ++j) m = fmaxf(m, scr_r[row * 32 + ((j + lane) & 31)]);
        float zz = 0.f;
        for (int j = 0; j < 32; ++j) {
            const int c = (j + lane) & 31;
            const float rj = scr_r[row * 32 + c];
            if (rj != -INFINITY) zz += scr_z[row * 32 + c] * __builtin_amdgcn_exp2f(rj - m);
        }
        wg_red[(wave * M_ROWS + row) * 2] = m;
        wg_red[(wave * M_ROWS + row) * 2 + 1] = zz;
    }
    __syncthreads();
    if (threadIdx.x < M_ROWS) {
        const int row = threadIdx.x;
        float m = -INFINITY;
        for (int wv = 0; wv < WAVES; ++wv) m = fmaxf(m, wg_red[(wv * M_ROWS + row) * 2]);
        float zz = 0.f;
        for (int wv = 0; wv < WAVES; ++wv) {
            const float rj = wg_red[(wv * M_ROWS + row) * 2];
            if (rj != -INFINITY) zz += wg_red[(wv * M_ROWS + row) * 2 + 1] * __builtin_amdgcn_exp2f(rj - m);
        }
        float *o = a.partial + (((int64_t)w.pl * a.n_chunks + w.chunk) * M_ROWS + row) * 2;
        o[0] = m;
        o[1] = zz;
    }
}

// chunk partials (log2 domain) -> natural-log sum-exp per row; one thread per (group problem, row)
__global__ void score_mfma_combine(int n_rows, int n_chunks, int p0, const float *partial, float *lse)
{
    const int gid = blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= n_rows) return;
    const int pl = gid / M_ROWS, row = gid - pl * M_ROWS;
    float m = -INFINITY;
    for (int c = 0; c < n_chunks; ++c) m = fmaxf(m, partial[(((int64_t)pl * n_chunks + c) * M_ROWS + row) * 2]);
    float zz = 0.f;
    for (int c = 0; c < n_chunks; ++c) {
        const float *o = partial + (((int64_t)pl * n_chunks + c) * M_ROWS + row) * 2;
        if (o[0] != -INFINITY) zz += o[1] * exp2f(o[0] - m);
    }
    lse[(int64_t)(p0 + pl) * M_ROWS + row] = (m + log2f(zz)) * LN2;
}

// ------------------------------------------------------------------ pass 2
__global__ void __launch_bounds__(WAVES * 64)
score_mfma_columns(ScoreArgs a)
{
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 31, hf = lane >> 5;
    const Dims &d = a.d;
    char *ring = lds + wave * RING_BYTES;
    const WaveWork w = wave_work(a, wave);

    bf16x8 qa[4][8];
    load_q(d, a.q, w.p, lane, qa);
    uint32_t xoff[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) xoff[s] = n * ROW_BYTES + (((2 * s + hf) ^ (n & 15)) << 4);
    const uint32_t ring_addr = lds_addr(ring);

    // exponent offsets of this lane's rows: log2-domain lse plus log2(G), so that exp2 yields A / G
    float l2[4][16];
#pragma unroll
    for (int h = 0; h < 4; ++h)
#pragma unroll
        for (int i = 0; i < 16; ++i)
            l2[h][i] = a.lse[(int64_t)w.p * M_ROWS + h * 32 + query_of(i, hf)] * LOG2E + 2.0f;

    float *out = (hf == 0 ? a.s_out : a.e_out) + (int64_t)w.p * d.L;
    const int stride = WAVES * SUB;
    for (int u = 0; u < min(NBUF - 1, w.n_sub); ++u)
        issue_subtile(w.kp, d.ks[3], w.first + u * stride, d.L, ring + u * BUF_BYTES, lane);

    float pending = 0.f;          // result of the previous subtile, stored one iteration late
    int pending_t = -1;
    for (int u = 0; u < w.n_sub; ++u) {
        wait_loads(min(NBUF - 2, w.n_sub - 1 - u));
        bf16x8 kb[8];
        read_subtile(ring_addr + (u % NBUF) * BUF_BYTES, xoff, kb);
        if (pending_t >= 0 && pending_t < d.L) out[pending_t] = pending;
        if (u + NBUF - 1 < w.n_sub)
            issue_subtile(w.kp, d.ks[3], w.first + (u + NBUF - 1) * stride, d.L,
                          ring + ((u + NBUF - 1) % NBUF) * BUF_BYTES, lane);
        floatx16 acc[4];
        qk_tile(qa, kb, acc);

        const int t = w.first + u * stride + n;
        const bool edge = w.first + u * stride + SUB > d.T;
        float ab[16];                                          // Abar of this lane's 16 queries (Eq. barA)
        float s_part = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            float v = 0.f;
#pragma unroll
            for (int h = 0; h < 4; ++h) v += __builtin_amdgcn_exp2f(fmaf(acc[h][i], a.c1, -l2[h][i]));
            if (edge && !(t < d.L && t <= d.T + query_of(i, hf))) v = 0.f;
            ab[i] = v;
            s_part += v;
        }
        const float s = s_part + __shfl_xor(s_part, 32);      // Eq. st
        const float inv_s = s > 0.f ? __builtin_amdgcn_rcpf(s) : 0.f;
        float e_part = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float ah = ab[i] * inv_s;
            e_part = fmaf(ah, __builtin_amdgcn_logf(ah + a.eps), e_part);
        }
        const float ent = -LN2 * (e_part + __shfl_xor(e_part, 32));   // inner sum of Eq. Dk
        pending = hf == 0 ? s : ent;
        pending_t = t;
    }
    if (pending_t >= 0 && pending_t < d.L) out[pending_t] = pending;
}

struct Plan {
    int group;        // problems per launch pair
    int chunk_len;
    int n_chunks;
};

Plan make_plan(const Dims &d)
{
    // One launch covers `group` problems with about one workgroup per CU (256 of them), all of equal
    // length, so that no second, partial wave of workgroups trails the first.  group is a power of two.
    Plan pl;
    const int64_t bytes_per_problem = (int64_t)d.L * ROW_BYTES;
    int64_t cache_target = (int64_t)128 << 20;                // keys of one group: inside the memory-side cache
    if (const char *e = getenv("SABLOCK_SCORE_GROUP_MB")) { long v = atol(e); if (v > 0) cache_target = (int64_t)v << 20; }
    int g = 1;
    while (g * 2 <= 256 && g * 2 <= d.P && (int64_t)g * 2 * bytes_per_problem <= cache_target) g *= 2;
    pl.group = g;
    const int unit = WAVES * SUB;
    const int want_chunks = 256 / g;
    int len = (d.L + want_chunks - 1) / want_chunks;
    len = ((len + unit - 1) / unit) * unit;
    pl.chunk_len = len;
    pl.n_chunks = (d.L + len - 1) / len;
    return pl;
}

}  // namespace

bool score_mfma_supported(const Dims &d)
{
    return d.dtype == SABLOCK_BF16 && d.D == 128 && d.G == 4 && d.W == 32;
}

size_t score_mfma_ws_bytes(const Dims &d)
{
    Plan pl = make_plan(d);
    return align256((size_t)d.P * M_ROWS * 4) + align256((size_t)pl.group * pl.n_chunks * M_ROWS * 2 * 4);
}

hipError_t launch_score_mfma(const Dims &d, const void *q, const void *k, const float *row_lse, float eps,
                             float *s_out, float *ent_out, void *ws, hipStream_t st)
{
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(score_mfma_stats),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(score_mfma_columns),
                                hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    const Plan pl = make_plan(d);
    ScoreArgs a;
    a.d = d;
    a.q = static_cast<const uint16_t *>(q);
    a.k = static_cast<const uint16_t *>(k);
    a.chunk_len = pl.chunk_len;
    a.n_chunks = pl.n_chunks;
    a.c1 = (float)(1.4426950408889634 / sqrt((double)d.D));
    a.eps = eps;
    a.s_out = s_out;
    a.e_out = ent_out;
    float *lse_ws = static_cast<float *>(ws);
    a.partial = ws ? reinterpret_cast<float *>(static_cast<char *>(ws) + align256((size_t)d.P * M_ROWS * 4)) : nullptr;
    a.lse = row_lse ? row_lse : lse_ws;
    for (int p0 = 0; p0 < d.P; p0 += pl.group) {
        const int g = (d.P - p0 < pl.group) ? d.P - p0 : pl.group;
        a.p0 = p0;
        dim3 grid(g * pl.n_chunks);
        if (!row_lse) {
            hipLaunchKernelGGL(score_mfma_stats, grid, dim3(WAVES * 64), LDS_BYTES, st, a);
            const int rows = g * M_ROWS;
            hipLaunchKernelGGL(score_mfma_combine, dim3((rows + 255) / 256), dim3(256), 0, st, rows, pl.n_chunks, p0,
                               a.partial, lse_ws);
        }
        hipLaunchKernelGGL(score_mfma_columns, grid, dim3(WAVES * 64), LDS_BYTES, st, a);
    }
    return hipGetLastError();
}

}  // namespace sablock
