// Causal attention of the observation-window queries over all L keys (Sec. 2.1, Eq. 1), with the natural-log
// softmax denominators of its rows as a second output: the part of a prefill attention whose row statistics the
// scoring step (Sec. 3.2) needs.  With them sablock_score reads K once (its column pass alone).
//
// bf16, D = 128; W in {8, 16, 32, 64} with G * W in {32, 64, 128, 256} window-query rows per KV head.  The rows
// are ordered head * W + query and a wavefront is one block of 32 of them (one head, half of a head's window of
// 64, or several heads when W < 32), so a workgroup has one to eight wavefronts.  A workgroup owns a chunk
// of keys of one problem (sequence, layer, KV head).  K and V subtiles of 32 keys
// go global -> LDS by direct-to-LDS loads into a workgroup-wide ring of NSTAGE stages (each wavefront issues its
// share of a stage); one LDS-only barrier per subtile tells that the stage has landed and that the stage of
// the previous iteration is free to be refilled.  The score product, the exponentials and the second product of
// a subtile depend on each other, so a wavefront alone leaves its SIMD idle between them: the ring is kept to
// 64 KiB so that two workgroups share a CU, and a problem is split over at least two workgroups (partial results
// are merged by a second kernel).
//
// Scores are formed TRANSPOSED, S^T = K Q^T (the same operand registers as Q K^T with the MFMA's A and B swapped):
// a lane then owns ONE query (column) and 16 of the subtile's 32 keys, so the row maximum and the row sum are
// in-lane plus one exchange between the two lane halves, and the 16 probabilities of a lane are, eight at a
// time, exactly an A operand of the second product O += P V (rows = queries, k = keys; the order of the keys
// inside a k-step is a fixed permutation that the V operand follows).  V is needed with the keys contiguous per
// lane, i.e. transposed: `ds_read_b64_tr_b16` delivers that from the row-major V tile, four keys per read.
// Probabilities are taken relative to a per-query reference that is fixed at the first subtile and moved only when
// a logit exceeds it by more than 64 in the log2 domain (rare), so the output accumulators are not rescaled per
// subtile.
#include "sablock_internal.h"

#include <algorithm>
#include <cstdlib>

namespace sablock {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef void __attribute__((address_space(3))) *lptr_t;

constexpr int SUB = 32;                        // keys per subtile
constexpr int ROW_BYTES = 256;                 // D = 128 bf16
constexpr int TILE_BYTES = SUB * ROW_BYTES;    // 8 KiB: one K or V subtile
// with V: a stage of the ring is a K tile then a V tile; statistics only: a K tile
constexpr int stage_bytes(bool with_v) { return with_v ? 2 * TILE_BYTES : TILE_BYTES; }
constexpr int NSTAGE = 4;                      // 64 KiB ring per workgroup: two workgroups (8 wavefronts) per CU
constexpr int ROWS = 32;                       // window-query rows of a wavefront
constexpr int wa_lds(int nw, bool with_v = true) { return NSTAGE * stage_bytes(with_v) + nw * ROWS * 4; }   // ring + a 32-float exchange slice per wavefront
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;
constexpr float RESCALE_AT = 64.f;

struct WinArgs {
    Dims d;
    const uint16_t *q, *k, *v;
    int chunk_len, n_chunks;
    float c1;                  // log2(e) / sqrt(D)
    float *out;                // [P * G][W][D] fp32 (n_chunks == 1) ...
    float *lse;                // [P][G * W] natural log
    float *o_part;             // ... or partial results [P * NW][n_chunks][32][D], unnormalised (NW row blocks per problem)
    float *ml_part;            // [P * NW][n_chunks][32][2]: reference (log2 domain), sum
    float *stats;              // statistics-only kernel: [P][2 row blocks][n_chunks][128][2] (reference in the log2 domain, sum)
};

__device__ __forceinline__ uint32_t lds_addr(const void *p) { return (uint32_t)(uintptr_t)(lptr_t)p; }

__device__ __forceinline__ void dma_1k(uint32_t voff, const char *sbase, uint32_t lds_dst)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt" : : "v"(voff), "s"(sbase), "s"(lds_dst) : "memory", "m0");
}

// key row owned by accumulator register i in lane half hf (rows of an MFMA result tile)
__device__ __forceinline__ int row_of(int i, int hf) { return 8 * (i >> 2) + 4 * hf + (i & 3); }

__device__ __forceinline__ float other_half(float x, bool take_max)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    const float a = __uint_as_float(r[0]), b = __uint_as_float(r[1]);
    return take_max ? fmaxf(a, b) : a + b;
}

// all LDS traffic of this wavefront done, then the workgroup barrier (global loads stay in flight)
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// one 1 KiB piece (4 rows) of a K or V subtile whose first row is t0: rows past L-1 read row L-1 (masked later).
// LDS slot (row, pos) of a K tile receives the row's 16-byte chunk pos ^ (row & 15) (conflict-free 16-byte operand
// reads, one row per lane); of a V tile chunk pos ^ 4 ((row >> 1) & 3), i.e. the row's four 64-byte groups are
// rotated by the row pair: a transposing read touches one 64-byte group of 8 consecutive rows, which then fall on
// four different bank groups, two rows each: the two LDS passes that 512 bytes need anyway.
// FULL: the caller knows that the tile has all its 32 rows
template <bool IS_K, bool FULL = false>
__device__ __forceinline__ void issue_piece(const char *tile_base, int64_t row_bytes, int t0, int L, int j, int lane, uint32_t lds_dst)
{
    const int r4 = lane >> 4, pos = lane & 15, row = 4 * j + r4;
    const uint32_t chunk = IS_K ? (uint32_t)((pos ^ row) & 15) : (uint32_t)(pos ^ (4 * ((row >> 1) & 3)));
    if (FULL || t0 + SUB <= L) {
        dma_1k((uint32_t)(r4 * row_bytes) + (chunk << 4), tile_base + (int64_t)(4 * j) * row_bytes, lds_dst);
    } else {
        dma_1k((uint32_t)min(row, L - t0 - 1) * (uint32_t)row_bytes + (chunk << 4), tile_base, lds_dst);
    }
}

// NW: wavefronts = 32-row blocks per problem (G * W / 32).
// WITH_V = false: the row statistics alone (reference and sum of exponentials per window-query row and chunk of
// keys), i.e. the first pass of the scoring step with ONE read of K for all 256 rows: no V tiles, no second
// product, no output rows.
template <int NW, bool WITH_V>
__global__ void __launch_bounds__(NW * 64)
window_attention_kernel(WinArgs a)
{
    constexpr int STAGE_BYTES = stage_bytes(WITH_V);
    constexpr int KPIECES = 8 / NW;                            // K pieces per wavefront and stage (as many V pieces)
    constexpr int LOADS = WITH_V ? 2 * KPIECES : KPIECES;      // direct-to-LDS loads per wavefront and stage
    extern __shared__ __attribute__((aligned(8192))) char lds[];
    const Dims &d = a.d;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 31, hf = lane >> 5;                   // n: query (score tiles) or d column (output tiles)
    const int p = blockIdx.x / a.n_chunks, chunk = blockIdx.x - p * a.n_chunks;
    const int lo = chunk * a.chunk_len, hi = min(lo + a.chunk_len, d.L);
    const int n_sub = hi > lo ? (hi - lo + SUB - 1) / SUB : 0;                 // the same for all wavefronts
    // the problem's G * W rows in the order head * W + query; this lane's row of the wavefront's block of 32
    // (W >= 32: one head per block; W < 32: 32 / W heads per block)
    const int head = (ROWS * wave + n) / d.W, qoff = (ROWS * wave + n) - head * d.W - n;    // query of this lane = qoff + n
    const uint32_t ring = __builtin_amdgcn_readfirstlane(lds_addr(lds));
    float *fac = reinterpret_cast<float *>(lds + NSTAGE * STAGE_BYTES) + wave * ROWS;        // this wavefront's exchange slice
    const char *kp = reinterpret_cast<const char *>(a.k + k_problem_offset(d, p));
    const char *vp = WITH_V ? reinterpret_cast<const char *>(a.v + v_problem_offset(d, p)) : nullptr;
    const int64_t krow = d.ks[3] * 2, vrow = d.vs[3] * 2;

    // ---- loads: stage u % NSTAGE holds subtile u; this wavefront brings its share of the 8 K pieces and of the 8 V
    // pieces (both tiles are stored swizzled, see issue_piece)
    auto issue = [&](int u) {
        const int t0 = lo + u * SUB;                           // < L
        const uint32_t st = ring + (u % NSTAGE) * STAGE_BYTES;
#pragma unroll
        for (int jj = 0; jj < KPIECES; ++jj) {
            const int j = KPIECES * wave + jj;
            issue_piece<true>(kp + (int64_t)t0 * krow, krow, t0, d.L, j, lane, st + j * 1024);
        }
        if (WITH_V) {
#pragma unroll
            for (int jj = 0; jj < KPIECES; ++jj) {
                const int j = KPIECES * wave + jj;
                issue_piece<false>(vp + (int64_t)t0 * vrow, vrow, t0, d.L, j, lane, st + TILE_BYTES + j * 1024);
            }
        }
    };
    for (int u = 0; u < NSTAGE - 1 && u < n_sub; ++u) issue(u);

    // ---- this block's window queries: B operand of S^T = K Q^T, lane (query n, half hf) holds Q[n][(2s + hf) * 8 .. +8]
    bf16x8 qa[8];
    const bool real_row = ROWS * wave + n < d.G * d.W;         // rows behind the problem's G * W pad the last block(s)
    if (real_row) {
        const uint16_t *row = a.q + q_row_offset(d, p, head, qoff + n);
#pragma unroll
        for (int s = 0; s < 8; ++s) qa[s] = *reinterpret_cast<const bf16x8 *>(row + (2 * s + hf) * 8);
    } else {
#pragma unroll
        for (int s = 0; s < 8; ++s) qa[s] = bf16x8{};
    }

    floatx16 o[4];                                             // O[query][32 t + d], rows = queries
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[t][i] = 0.f;
    float r = 0.f;                                             // reference of this lane's query, in units of <q,k>
    float l = 0.f;                                             // sum of exp2(c1 * (<q,k> - r)) over this lane's keys
    const float lim = RESCALE_AT / a.c1;
    const uint32_t k_lane = (uint32_t)(n * ROW_BYTES + ((hf ^ (n & 15)) << 4));       // K operand reads (chunk 2s+hf: ^ (s << 5))
    // V operand reads: lane = 16 g + pp; receiver of column 16 (g % 2) + pp of the 32-column tile, key block kb = g / 2;
    // as a provider it points at row (pp / 4) of a 4-key group, columns 4 (pp % 4) .. +4 of its 16-column half
    const int g16 = lane >> 4, pp = lane & 15;
    uint32_t v_lane[4];                                        // per 32-column tile t: its 64-byte group sits at t ^ sw
    {
        const int sw = (2 * (g16 >> 1) + (pp >> 3)) & 3;       // ((row >> 1) & 3) of the rows this lane points at
#pragma unroll
        for (int t = 0; t < 4; ++t)
            v_lane[t] = (uint32_t)((4 * (g16 >> 1) + (pp >> 2)) * ROW_BYTES + 64 * (t ^ sw) + 32 * (g16 & 1) + 8 * (pp & 3));
    }

    // subtiles 1 .. n_fast - 1 have no masked key, and the subtile refilled while they are worked on exists and is full
    const int n_fast = min(min(n_sub, (d.L - lo) / SUB) - (NSTAGE - 1), (d.T - lo) / SUB);

    for (int u = 0; u < n_sub; ++u) {
        if constexpr (!WITH_V) {
            if (u == 1 && n_fast >= 3) {
                // ---- statistics, steady state: the products of subtile v + 1 are issued before the exponentials of
                // subtile v, in one basic block, so that the matrix pipe works in the shadow of the exponentials
                float nrc = -r * a.c1;
                auto products = [&](int v) -> floatx16 {
                    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * LOADS) : "memory");
                    lds_barrier();
                    {
                        const int w = v + NSTAGE - 1, t0 = lo + w * SUB;
#pragma unroll
                        for (int jj = 0; jj < KPIECES; ++jj) {
                            const int j = KPIECES * wave + jj;
                            issue_piece<true, true>(kp + (int64_t)t0 * krow, krow, t0, d.L, j, lane,
                                                    ring + (w % NSTAGE) * STAGE_BYTES + j * 1024);
                        }
                    }
                    const uint32_t st = ring + (v % NSTAGE) * STAGE_BYTES;
                    bf16x8 kb[8];
#pragma unroll
                    for (int s = 0; s < 8; ++s)
                        asm volatile("ds_read_b128 %0, %1" : "=v"(kb[s]) : "v"((st + k_lane) ^ (uint32_t)(s << 5)) : "memory");
                    asm volatile("s_waitcnt lgkmcnt(0)"
                                 : "+v"(kb[0]), "+v"(kb[1]), "+v"(kb[2]), "+v"(kb[3]), "+v"(kb[4]), "+v"(kb[5]), "+v"(kb[6]), "+v"(kb[7])
                                 :
                                 : "memory");
                    floatx16 acc;
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
                    for (int s = 0; s < 8; ++s) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kb[s], qa[s], acc, 0, 0, 0);
                    return acc;
                };
                // a logit may run ahead of the reference by any amount: the reference moves before the exponentials
                auto anchor = [&](const floatx16 &acc) {
                    float mx = acc[0];
#pragma unroll
                    for (int i = 1; i < 16; ++i) mx = fmaxf(mx, acc[i]);
                    if (__ballot(mx > r + lim) != 0ull) {
                        const float m2 = other_half(mx, true);
                        if (m2 > r + lim) {
                            l *= __builtin_amdgcn_exp2f(a.c1 * (r - m2));
                            r = m2;
                            nrc = -r * a.c1;
                        }
                    }
                };
                auto sums = [&](const floatx16 &acc) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) l += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[i], a.c1, nrc));
                };
                int v = 1;
                floatx16 sa = products(v), sb;
                while (v + 2 < n_fast) {
                    anchor(sa);
                    sb = products(v + 1);
                    sums(sa);
                    anchor(sb);
                    sa = products(v + 2);
                    sums(sb);
                    v += 2;
                }
                anchor(sa);
                sums(sa);
                u = v + 1;                                     // < n_sub: the generic step goes on from here
            }
        }
        // the pieces this wavefront issued for subtile u have landed (later stages: 4 loads each stay in flight) ...
        {
            static_assert(NSTAGE - 2 <= 2, "the wait below knows up to two later stages");
            const int after = min(NSTAGE - 2, n_sub - 1 - u);
            static_assert(2 * LOADS < 64, "vmcnt is a 6-bit counter");
            if (after >= 2) {
                asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * LOADS) : "memory");
            } else if (after == 1) {
                asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LOADS) : "memory");
            } else {
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            }
        }
        // ... and after the barrier so have everyone's; the stage of the previous iteration is free: refill it
        lds_barrier();
        if (u + NSTAGE - 1 < n_sub) issue(u + NSTAGE - 1);
        const uint32_t st = ring + (u % NSTAGE) * STAGE_BYTES;
        const int t0 = lo + u * SUB;

        // ---- S^T = K Q^T: acc[i] = <q_n, k_{t0 + row_of(i, hf)}> - r
        bf16x8 kb[8];
#pragma unroll
        for (int s = 0; s < 8; ++s)
            asm volatile("ds_read_b128 %0, %1" : "=v"(kb[s]) : "v"((st + k_lane) ^ (uint32_t)(s << 5)) : "memory");
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(kb[0]), "+v"(kb[1]), "+v"(kb[2]), "+v"(kb[3]), "+v"(kb[4]), "+v"(kb[5]), "+v"(kb[6]), "+v"(kb[7])
                     :
                     : "memory");
        floatx16 acc;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = -r;
#pragma unroll
        for (int s = 0; s < 8; ++s) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kb[s], qa[s], acc, 0, 0, 0);
        // keys this query does not see (causal inside the window, end of the sequence)
        const bool edge = t0 + SUB > d.T;
        if (edge) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int t = t0 + row_of(i, hf);
                if (!(t < d.L && t <= d.T + qoff + n)) acc[i] = -INFINITY;
            }
        }
        // ---- reference: anchored at the first subtile, moved when a logit runs more than `lim` ahead of it
        float mx = acc[0];
#pragma unroll
        for (int i = 1; i < 16; ++i) mx = fmaxf(mx, acc[i]);
        if (u == 0 || __ballot(mx > lim) != 0ull) {
            const float m2 = other_half(mx, true);             // over all 32 keys of the subtile
            float dlt = 0.f;                                   // how far the reference moves
            if (u == 0) dlt = m2 > -INFINITY ? m2 : 0.f;
            else if (m2 > lim) dlt = m2;
            const float f = u == 0 ? 1.f : __builtin_amdgcn_exp2f(-a.c1 * dlt);
            r += dlt;
            l *= f;
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] -= dlt;
            if (WITH_V) {
                // the output rows are queries: hand the per-query factors over through LDS
                if (hf == 0) fac[n] = f;
                __builtin_amdgcn_wave_barrier();
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float fi = fac[row_of(i, hf)];
#pragma unroll
                    for (int t = 0; t < 4; ++t) o[t][i] *= fi;
                }
                __builtin_amdgcn_wave_barrier();
            }
        }
        // ---- probabilities relative to the reference, their sum, and the two A operands of O += P V
        float pr[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) { pr[i] = __builtin_amdgcn_exp2f(acc[i] * a.c1); l += pr[i]; }
        if (!WITH_V) continue;
        bf16x8 pa[2];
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int j = 0; j < 8; ++j) pa[s][j] = (__bf16)pr[8 * s + j];
        // ---- O += P V: k-step s covers keys 16 s .. 16 s + 15 in the order of the accumulator rows, so lane half kb
        // needs V rows 16 s + 4 kb + (0..3) and 16 s + 8 + 4 kb + (0..3) of its column: two transposing reads
#pragma unroll
        for (int s = 0; s < 2; ++s) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const uint32_t va = st + TILE_BYTES + v_lane[t] + (uint32_t)(16 * s * ROW_BYTES);
                short4v v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4v *)(uintptr_t)va);
                short4v v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) short4v *)(uintptr_t)(va + 8 * ROW_BYTES));
                short8v vv = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
                o[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pa[s], __builtin_bit_cast(bf16x8, vv), o[t], 0, 0, 0);
            }
        }
    }

    // ---- results: the row sums of the two lane halves together; rows of O scaled by 1 / sum (one chunk) or stored
    // unnormalised with (reference, sum) for the merge
    const float l_tot = other_half(l, false);
    const float ref2 = r * a.c1;                               // log2 domain
    if (!WITH_V) {
        // where the column pass for 256 rows looks for a row's statistics: two blocks of 128 rows per problem
        // (W = 64: the window halves, rows head * 32 + query; G = 8: heads 0-3 and 4-7)
        const int blk = d.W > ROWS ? qoff / ROWS : head / 4;
        const int row = d.W > ROWS ? head * ROWS + n : (head & 3) * ROWS + n;
        if (hf == 0) {
            float *o2 = a.stats + ((((int64_t)p * (NW / 4) + blk) * a.n_chunks + chunk) * 128 + row) * 2;
            o2[0] = ref2;
            o2[1] = l_tot;
        }
        return;
    }
    const int pb = p * NW + wave;                              // (problem, row block)
    const int64_t out_row0 = (int64_t)p * d.G * d.W + ROWS * wave;             // first output row of this block
    const int rows_here = min(ROWS, d.G * d.W - ROWS * wave);  // real rows of this block (<= 0: all padding)
    if (a.n_chunks == 1) {
        if (hf == 0) {
            fac[n] = l_tot > 0.f ? 1.0f / l_tot : 0.f;
            if (real_row) a.lse[out_row0 + n] = (ref2 + __builtin_amdgcn_logf(l_tot)) * LN2;
        }
    } else if (hf == 0) {
        fac[n] = 1.f;
        float *ml = a.ml_part + (((int64_t)pb * a.n_chunks + chunk) * ROWS + n) * 2;
        ml[0] = ref2;
        ml[1] = l_tot;
    }
    __builtin_amdgcn_wave_barrier();
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    float *ob = a.n_chunks == 1 ? a.out + out_row0 * 128 : a.o_part + ((int64_t)pb * a.n_chunks + chunk) * ROWS * 128;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int qy = row_of(i, hf);
        const float fi = fac[qy];
#pragma unroll
        for (int t = 0; t < 4; ++t)
            if (a.n_chunks > 1 || qy < rows_here) ob[qy * 128 + 32 * t + n] = o[t][i] * fi;
    }
}

// merge of the chunks' partial results: one workgroup per output row (problem, head, window query), one thread per
// output column; the row's partial results sit in row block (head, window half) of its problem
__global__ void __launch_bounds__(128)
window_attention_merge_kernel(const float *o_part, const float *ml_part, int n_chunks, int G, int W, int nw, float *out,
                              float *lse)
{
    const int row = blockIdx.x;                                // (p * G + h) * W + i
    const int GW = G * W, p = row / GW, r = row - p * GW;      // r = h * W + i: blocks of 32 consecutive r
    const int pb = p * nw + r / ROWS, qy = r % ROWS;           // nw row blocks per problem (the last ones may be padding)
    float m = -INFINITY;
    for (int c = 0; c < n_chunks; ++c) {
        const float *ml = ml_part + (((int64_t)pb * n_chunks + c) * ROWS + qy) * 2;
        if (ml[1] > 0.f) m = fmaxf(m, ml[0]);
    }
    float acc = 0.f, z = 0.f;
    for (int c = 0; c < n_chunks; ++c) {
        const float *ml = ml_part + (((int64_t)pb * n_chunks + c) * ROWS + qy) * 2;
        if (ml[1] > 0.f) {
            const float w = __builtin_amdgcn_exp2f(ml[0] - m);
            z += ml[1] * w;
            acc += o_part[(((int64_t)pb * n_chunks + c) * ROWS + qy) * 128 + threadIdx.x] * w;
        }
    }
    out[(int64_t)row * 128 + threadIdx.x] = z > 0.f ? acc / z : 0.f;
    if (threadIdx.x == 0) lse[row] = (m + __builtin_amdgcn_logf(z)) * LN2;
}

// keys per workgroup: whole rounds of two workgroups per CU (two wavefronts per SIMD: while one waits for its
// LDS reads or an MFMA result the other computes), as few as keep a chunk within 131 072 keys
void wa_plan(const Dims &d, int *chunk_len, int *n_chunks, int wgs_per_cu)
{
    constexpr int MAX_CHUNK = 131072;
    const int64_t cus = wgs_per_cu * (int64_t)d.cus;
    const int64_t rounds = ((int64_t)d.P * d.L + cus * MAX_CHUNK - 1) / (cus * MAX_CHUNK);
    const int64_t per_problem = std::max<int64_t>(1, (cus * rounds + d.P / 2) / d.P);
    int len = (int)(((d.L + per_problem - 1) / per_problem + SUB - 1) / SUB) * SUB;
    if (d.tune.window_chunk >= SUB) len = (d.tune.window_chunk / SUB) * SUB;
    len = std::min(std::max(len, SUB), MAX_CHUNK);
    *chunk_len = len;
    *n_chunks = (d.L + len - 1) / len;
}

}  // namespace

// ---- the statistics alone for 256 window-query rows per KV head, as the first pass of the scoring step
bool row_stats_supported(const Dims &d)
{
    return d.dtype == SABLOCK_BF16 && d.D == 128 &&
           (((d.W == 32 || d.W == 64) && d.G * d.W > 128 && d.G * d.W <= 256) || (d.G == 4 && d.W == 32));
}

// 32 KiB rings: two 8-wavefront workgroups per CU, or four 4-wavefront ones (128 rows)
static int row_stats_wgs_per_cu(const Dims &d) { return d.G * d.W > 128 ? 2 : 4; }

int row_stats_chunks(const Dims &d)
{
    int len, nc;
    wa_plan(d, &len, &nc, row_stats_wgs_per_cu(d));
    return nc;
}

hipError_t launch_row_stats(const Dims &d, const void *q, const void *k, float *stats, hipStream_t st)
{
    static thread_local PerDeviceOnce attr_once;
    if (attr_once.needed()) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(window_attention_kernel<8, false>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, wa_lds(8, false));
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(window_attention_kernel<4, false>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, wa_lds(4, false));
        if (e != hipSuccess) return e;
        attr_once.done();
    }
    WinArgs a;
    a.d = d;
    a.q = static_cast<const uint16_t *>(q);
    a.k = static_cast<const uint16_t *>(k);
    a.v = nullptr;
    wa_plan(d, &a.chunk_len, &a.n_chunks, row_stats_wgs_per_cu(d));
    a.c1 = (float)(1.4426950408889634 / sqrt((double)d.D));
    a.out = a.lse = a.o_part = a.ml_part = nullptr;
    a.stats = stats;
    const dim3 grid((unsigned)((int64_t)d.P * a.n_chunks));
    if (d.G * d.W > 128) hipLaunchKernelGGL((window_attention_kernel<8, false>), grid, dim3(8 * 64), wa_lds(8, false), st, a);
    else hipLaunchKernelGGL((window_attention_kernel<4, false>), grid, dim3(4 * 64), wa_lds(4, false), st, a);
    return hipGetLastError();
}

bool window_attention_supported(const Dims &d)
{
    // blocks of 32 rows, each of whole heads or inside one head; up to 8 blocks
    return d.dtype == SABLOCK_BF16 && d.D == 128 && d.G * d.W <= 8 * ROWS &&
           (d.W == 8 || d.W == 16 || d.W == 32 || d.W == 64);
}

// wavefronts per workgroup: the problem's G * W rows in blocks of 32, rounded up to 1, 2, 4 or 8 blocks (the
// kernel splits a stage's eight key pieces evenly over its wavefronts); blocks behind the rows are padding
static int wa_blocks(const Dims &d)
{
    const int nb = (d.G * d.W + ROWS - 1) / ROWS;
    return nb <= 1 ? 1 : nb <= 2 ? 2 : nb <= 4 ? 4 : 8;
}

size_t window_attention_ws_bytes(const Dims &d)
{
    int len, nc;
    wa_plan(d, &len, &nc, wa_blocks(d) <= 4 ? 2 : 1);
    if (nc == 1) return 256;
    const size_t blocks = (size_t)d.P * wa_blocks(d);
    return align256(blocks * nc * ROWS * 128 * 4) + align256(blocks * nc * ROWS * 2 * 4);
}

hipError_t launch_window_attention(const Dims &d, const void *q, const void *k, const void *v, float *out, float *lse,
                                   void *ws, hipStream_t st)
{
    static thread_local PerDeviceOnce attr_once;
    if (attr_once.needed()) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(window_attention_kernel<1, true>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, wa_lds(1));
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(window_attention_kernel<2, true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, wa_lds(2));
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(window_attention_kernel<4, true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, wa_lds(4));
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(window_attention_kernel<8, true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, wa_lds(8));
        if (e != hipSuccess) return e;
        attr_once.done();
    }
    const int nw = wa_blocks(d);                               // 1, 2, 4 or 8 row blocks = wavefronts per workgroup
    WinArgs a;
    a.d = d;
    a.q = static_cast<const uint16_t *>(q);
    a.k = static_cast<const uint16_t *>(k);
    a.v = static_cast<const uint16_t *>(v);
    // workgroups of up to four wavefronts pair up on a CU; eight-wavefront ones already put two wavefronts on every SIMD
    wa_plan(d, &a.chunk_len, &a.n_chunks, nw <= 4 ? 2 : 1);
    a.c1 = (float)(1.4426950408889634 / sqrt((double)d.D));
    a.out = out;
    a.lse = lse;
    a.o_part = static_cast<float *>(ws);
    a.ml_part = reinterpret_cast<float *>(static_cast<char *>(ws) + align256((size_t)d.P * nw * a.n_chunks * ROWS * 128 * 4));
    const dim3 grid((unsigned)((int64_t)d.P * a.n_chunks));
    a.stats = nullptr;
    if (nw == 1) hipLaunchKernelGGL((window_attention_kernel<1, true>), grid, dim3(64), wa_lds(1), st, a);
    else if (nw == 2) hipLaunchKernelGGL((window_attention_kernel<2, true>), grid, dim3(2 * 64), wa_lds(2), st, a);
    else if (nw == 4) hipLaunchKernelGGL((window_attention_kernel<4, true>), grid, dim3(4 * 64), wa_lds(4), st, a);
    else hipLaunchKernelGGL((window_attention_kernel<8, true>), grid, dim3(8 * 64), wa_lds(8), st, a);
    if (a.n_chunks > 1)
        hipLaunchKernelGGL(window_attention_merge_kernel, dim3((unsigned)((int64_t)d.P * d.G * d.W)), dim3(128), 0, st,
                           a.o_part, a.ml_part, a.n_chunks, d.G, d.W, nw, out, lse);
    return hipGetLastError();
}

}  // namespace sablock
