// MFMA window scoring (Sec. 3.2, Eqs. barA, st, Dk) for bf16, D = 128 and (G, W) = (4, 32), (4, 64) or (8, 32).
//
// The window-query rows of a KV head (4 query heads x 32 window queries) stay in
// accumulation registers as MFMA A operands; keys are the B operand, 32 per
// wavefront iteration ("subtile"), so in the 32x32 accumulator layout a lane
// owns ONE key column and 16 of the 32 queries of each head:
//   * the head mean (Eq. barA) is an in-lane add over the four accumulators,
//   * the column sum (Eq. st) is 16 in-lane adds plus one exchange between the
//     two lane halves, and so is the entropy term (inner sum of Eq. Dk),
//   * the per-row softmax statistics are kept per lane and only reduced across
//     lanes once per workgroup.
// Each wavefront streams its own keys: global -> LDS with direct-to-LDS loads
// (16 bytes per lane, fully coalesced 256-byte key rows) into a private ring,
// LDS -> registers with an XOR swizzle so the 16-byte reads of 32 different key
// rows do not collide on banks.  No workgroup barrier in the loops.
//
// Softmax over all keys needs each row's log-sum-exp before any column is
// final, so scoring is two kernels unless the caller supplies row_lse:
//   pass 1  per row a reference (kept in LDS, shared by the 32 lanes that hold
//           the row) and per lane the sum of exp2 relative to it; the reference
//           enters the MFMA as its C operand, so the exponent is one multiply;
//   pass 2  the chunk partials are combined into the row log-sum-exp in the
//           prologue and fed as the MFMA C operand; probabilities, head mean,
//           column sum and entropy term follow in registers.
// In both passes the four heads rotate through two accumulators: head h is
// multiplied while head h-1 is exponentiated, which overlaps the matrix pipe
// with the exp/log work inside one wavefront (one wavefront per SIMD).
// One launch per pass covers every problem of the call.
//
// 256 window-query rows per KV head (G = 4 with W = 64, or G = 8 with W = 32).  The row statistics are
// independent per row, so pass 1 runs the same kernel on two blocks of 128 rows (the two halves of the window, or
// heads 0-3 and 4-7) as if they were two problems (K is streamed once per block).  Pass 2 needs all rows of a
// key together (head mean, column sum, entropy), so a variant of the column kernel keeps all eight 32-row tiles
// as A operands (256 accumulation registers), the keys in ordinary registers and the C operands in LDS.
#include "sablock_internal.h"

#include <algorithm>

namespace sablock {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef const void __attribute__((address_space(1))) *gptr_t;
typedef void __attribute__((address_space(3))) *lptr_t;

constexpr int SUB = 32;                    // keys per wavefront iteration
constexpr int ROW_BYTES = 256;             // D = 128 bf16
constexpr int BUF_BYTES = SUB * ROW_BYTES; // 8 KiB
constexpr int M_ROWS = 128;
constexpr int STREAMS = 4;                 // key streams per workgroup (subtile u of the chunk goes to stream u % 4)
constexpr int STRIDE = STREAMS * SUB;      // keys between consecutive subtiles of one stream

constexpr int P1_LDS = 4 * 4 * BUF_BYTES + 4 * M_ROWS * 2 * 4 + 4 * M_ROWS * 4;   // rings + cross-wave reduction + row references
constexpr int P2_LDS = 4 * 4 * BUF_BYTES + M_ROWS * 4 + 256 * 2 * 4;   // four rings + the rows' log-sum-exp + combine scratch

constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;
constexpr float RESCALE_AT = 64.f;         // pass 1 moves a row's reference when an exponent exceeds this

struct ScoreArgs {
    Dims d;
    const uint16_t *q, *k;
    int p0;                // first problem of the group
    int chunk_len;         // keys per workgroup, multiple of STRIDE
    int n_chunks;          // workgroups per problem
    int nv;                // 128-row blocks per problem in pass 1 (G * W / 128)
    int pc;                // (reference, sum) pairs per row that pass 2 reads: n_chunks, or 1 once they are merged
    float c1;              // log2(e) / sqrt(D)
    float log2_G;          // log2 of the heads per KV head (the head mean is folded into the rows' log-sum-exp)
    float eps;
    float *partial;        // pass 1 out: [problem][query block][chunk][128][2] (reference, sum), log2 domain
    const float *merged;   // pass 2 in: the same layout with pc chunks
    const float *lse;      // pass 2 in, optional: [P][G * W] natural-log sum-exp per row (NULL: use partial)
    float *s_out, *e_out;  // pass 2 out: [P][L]
    float *abar;           // pass 2 out of the all-head variant: head-group means [P][W / 4][L][4]
};

__device__ __forceinline__ uint32_t lds_addr(const void *p) { return (uint32_t)(uintptr_t)(lptr_t)p; }

// window query owned by accumulator register i in lane half hf
__device__ __forceinline__ int query_of(int i, int hf) { return 8 * (i >> 2) + 4 * hf + (i & 3); }

// Direct-to-LDS load of 32 key rows starting at t0: 8 instructions of 1 KiB (4 rows each); LDS slot
// (row, pos) receives 16-byte chunk pos ^ (row & 15) of the row.  The address is a wave-uniform 64-bit base
// (scalar registers) plus a per-lane 32-bit byte offset; M0 carries the LDS destination of each 1 KiB group.
__device__ __forceinline__ void dma_1k(uint32_t voff, const char *sbase, uint32_t lds_dst)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt" : : "v"(voff), "s"(sbase), "s"(lds_dst) : "memory", "m0");
}

// subtile entirely inside [0, L): one of four precomputed lane offsets
//   lane_off[j & 3] = (lane / 16) * row_bytes + (((lane & 15) ^ (lane / 16) ^ 4 (j & 3)) << 4),
// so issuing costs no vector ALU work
__device__ __forceinline__ void issue_subtile_fast(const char *base, int64_t row_bytes, const uint32_t (&lane_off)[4], uint32_t buf_lds)
{
#pragma unroll
    for (int j = 0; j < 8; ++j) dma_1k(lane_off[j & 3], base + (int64_t)(4 * j) * row_bytes, buf_lds + j * 1024);
}

// The same for dense rows (row_bytes = 256): four rows are then 1 KiB apart in memory as in LDS, and the
// instruction's immediate offset is added to the global address and to the LDS address alike, so four loads share
// one scalar base and one M0 value; the subtile takes two of each instead of eight.
__device__ __forceinline__ void dma_4k(const uint32_t (&lane_off)[4], const char *sbase, uint32_t lds_dst)
{
    asm volatile("s_mov_b32 m0, %5\n\ts_nop 0\n\t"
                 "global_load_lds_dwordx4 %0, %4 nt\n\t"
                 "global_load_lds_dwordx4 %1, %4 offset:1024 nt\n\t"
                 "global_load_lds_dwordx4 %2, %4 offset:2048 nt\n\t"
                 "global_load_lds_dwordx4 %3, %4 offset:3072 nt"
                 : : "v"(lane_off[0]), "v"(lane_off[1]), "v"(lane_off[2]), "v"(lane_off[3]), "s"(sbase), "s"(lds_dst) : "memory", "m0");
}
__device__ __forceinline__ void issue_subtile_dense(const char *base, const uint32_t (&lane_off)[4], uint32_t buf_lds)
{
    dma_4k(lane_off, base, buf_lds);
    dma_4k(lane_off, base + 4096, buf_lds + 4096);
}

// subtile that crosses L: rows past L-1 read row L-1 instead (their results are masked later); t0 < L
__device__ __forceinline__ void issue_subtile_clamped(const char *base, int64_t row_bytes, int rows_valid, uint32_t buf_lds, int lane)
{
    const int r4 = lane >> 4, pos = lane & 15;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int row = 4 * j + r4;
        const uint32_t voff = (uint32_t)min(row, rows_valid - 1) * (uint32_t)row_bytes + (uint32_t)(((pos ^ row) & 15) << 4);
        dma_1k(voff, base, buf_lds + j * 1024);
    }
}

// wait until this wavefront's direct-to-LDS loads issued before the last `subtiles_after` subtiles have landed
// (8 loads per subtile; later stores only make the wait longer, never shorter)
__device__ __forceinline__ void wait_loads(int subtiles_after)
{
    if (subtiles_after >= 3) asm volatile("s_waitcnt vmcnt(24)" ::: "memory");
    else if (subtiles_after == 2) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
    else if (subtiles_after == 1) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

struct WaveWork {
    const uint16_t *kp;    // keys of the problem
    int p, pl, chunk;
    int pv, qoff, hoff;    // pass 1: (problem, row block) index, the block's first window query and first head
    int first, n_sub;      // this stream's subtiles: keys [first + u * STRIDE, +SUB), u < n_sub
};

__device__ __forceinline__ WaveWork wave_work(const ScoreArgs &a, int stream)
{
    stream = __builtin_amdgcn_readfirstlane(stream);         // wave-uniform: addresses below stay in scalar registers
    WaveWork w;
    w.pl = blockIdx.x / a.n_chunks;
    w.chunk = blockIdx.x - w.pl * a.n_chunks;
    w.p = a.p0 + w.pl;
    w.pv = w.p;
    w.qoff = 0;
    w.hoff = 0;
    w.kp = a.k + k_problem_offset(a.d, w.p);
    const int lo = w.chunk * a.chunk_len;
    const int hi = min(lo + a.chunk_len, a.d.L);
    w.first = lo + stream * SUB;
    const int span = hi - w.first;
    w.n_sub = span > 0 ? (span + STRIDE - 1) / STRIDE : 0;
    return w;
}

// pass 1: workgroups are indexed by ((problem, query block), chunk)
__device__ __forceinline__ WaveWork wave_work_blocks(const ScoreArgs &a, int stream)
{
    WaveWork w = wave_work(a, stream);
    w.pv = a.p0 * a.nv + w.pl;
    w.p = w.pv / a.nv;
    const int v = w.pv - w.p * a.nv;
    w.qoff = a.d.W > 32 ? 32 * v : 0;                        // blocks are window halves ...
    w.hoff = a.d.W > 32 ? 0 : 4 * v;                         // ... or groups of four heads
    w.kp = a.k + k_problem_offset(a.d, w.p);
    return w;
}

// ------------------------------------------------------------------ shared pieces of both passes
// B operands of one subtile into accumulation registers: kb[s] = K[key lane % 32][(2s + lane/32) * 8 .. +8].
// lane_addr = buffer address + row * 256 + ((hf ^ (row & 15)) << 4); chunk 2s+hf sits at that address ^ (s << 5).
__device__ __forceinline__ void read_subtile_acc(uint32_t lane_addr, bf16x8 (&kb)[8])
{
#pragma unroll
    for (int s = 0; s < 8; ++s)
        asm volatile("ds_read_b128 %0, %1" : "=a"(kb[s]) : "v"(lane_addr ^ (uint32_t)(s << 5)) : "memory");
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+a"(kb[0]), "+a"(kb[1]), "+a"(kb[2]), "+a"(kb[3]), "+a"(kb[4]), "+a"(kb[5]), "+a"(kb[6]), "+a"(kb[7])
                 :
                 : "memory");
}

// the same into ordinary registers (for the kernel whose accumulation registers are all taken by A operands)
__device__ __forceinline__ void read_subtile_vgpr(uint32_t lane_addr, bf16x8 (&kb)[8])
{
#pragma unroll
    for (int s = 0; s < 8; ++s)
        asm volatile("ds_read_b128 %0, %1" : "=v"(kb[s]) : "v"(lane_addr ^ (uint32_t)(s << 5)) : "memory");
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(kb[0]), "+v"(kb[1]), "+v"(kb[2]), "+v"(kb[3]), "+v"(kb[4]), "+v"(kb[5]), "+v"(kb[6]), "+v"(kb[7])
                 :
                 : "memory");
}

// k-steps [S0, S1) of one head's 32x32 tile; the first step takes `c` as its C operand
template <int S0, int S1, int N>
__device__ __forceinline__ floatx16 chain(const bf16x8 (&qa)[N], const bf16x8 (&kb)[N], floatx16 c)
{
    static_assert(S1 <= N, "k-step outside the operands");
#pragma unroll
    for (int s = S0; s < S1; ++s) c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa[s], kb[s], c, 0, 0, 0);
    return c;
}

// Per-wavefront stream of subtiles through a ring of NBUF LDS buffers.  Subtile u lives in buffer u % NBUF; at
// the top of iteration u the stream waits for subtile u, reads it into registers, and immediately re-fills the
// same buffer with subtile u + NBUF, so NBUF subtiles (32 KiB per wavefront) are in flight or landed at any time.
template <int NBUF>
struct KeyStream {
    const uint16_t *kp;
    int64_t ks3;
    char *ring;
    uint32_t lane_addr0, ring_lds;
    uint32_t lane_off[4];
    int first, n_sub, L, lane;
    const char *next;                                          // keys of the next subtile to issue
    int64_t step;                                              // bytes between consecutive subtiles of this stream

    __device__ __forceinline__ void init(const uint16_t *kp_, int64_t ks3_, char *ring_, int first_, int n_sub_, int L_, int lane_)
    {
        kp = kp_; ks3 = ks3_; ring = ring_; first = first_; n_sub = n_sub_; L = L_; lane = lane_;
        next = reinterpret_cast<const char *>(kp) + (int64_t)first * ks3 * 2;
        step = (int64_t)STRIDE * ks3 * 2;
        const int n = lane & 31, hf = lane >> 5, r4 = lane >> 4, pos = lane & 15;
        ring_lds = __builtin_amdgcn_readfirstlane(lds_addr(ring));
        lane_addr0 = ring_lds + n * ROW_BYTES + ((hf ^ (n & 15)) << 4);
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) lane_off[jj] = (uint32_t)(r4 * ks3 * 2) + (uint32_t)(((pos ^ r4 ^ (4 * jj)) & 15) << 4);
    }
    __device__ __forceinline__ void issue(int u)
    {
        const int t0 = first + u * STRIDE;                     // wave-uniform, < L
        const char *base = next;                               // subtiles are issued in order: a running address
        next += step;
        const uint32_t buf_lds = ring_lds + (u % NBUF) * BUF_BYTES;
        if (t0 + SUB <= L) {
            if (ks3 == ROW_BYTES / 2) issue_subtile_dense(base, lane_off, buf_lds);
            else issue_subtile_fast(base, ks3 * 2, lane_off, buf_lds);
        } else issue_subtile_clamped(base, ks3 * 2, L - t0, buf_lds, lane);
    }
    __device__ __forceinline__ void prime()
    {
        for (int u = 0; u < min(NBUF, n_sub); ++u) issue(u);
    }
    __device__ __forceinline__ void fetch(int u, bf16x8 (&kb)[8])
    {
        wait_loads(min(NBUF - 1, n_sub - 1 - u));
        read_subtile_acc(lane_addr0 + (u % NBUF) * BUF_BYTES, kb);
        if (u + NBUF < n_sub) issue(u + NBUF);
    }
    __device__ __forceinline__ void fetch_vgpr(int u, bf16x8 (&kb)[8])
    {
        wait_loads(min(NBUF - 1, n_sub - 1 - u));
        read_subtile_vgpr(lane_addr0 + (u % NBUF) * BUF_BYTES, kb);
        if (u + NBUF < n_sub) issue(u + NBUF);
    }
};

// Keys of 64 elements (128-byte rows) for the kernels that take any row shape: no LDS staging.  A lane loads its
// own B operand (key lane % 32, elements (2s + lane / 32) * 8 .. +8 of k-step s: the two lane halves of a key read
// adjacent 16-byte pieces) straight into registers with ordinary loads, whose counter the compiler keeps; subtile
// u + 1 is requested before subtile u is worked on.  Keys past the end of the sequence read key L - 1 (their results
// are masked later, as in the staged stream).  Same interface as KeyStream.
template <int KS>
struct KeyStreamDirect {
    const uint16_t *kp;
    int64_t ks3;
    int first, n_sub, L, lane;
    bf16x8 nxt[KS];

    __device__ __forceinline__ void init(const uint16_t *kp_, int64_t ks3_, char *, int first_, int n_sub_, int L_, int lane_)
    {
        kp = kp_; ks3 = ks3_; first = first_; n_sub = n_sub_; L = L_; lane = lane_;
    }
    __device__ __forceinline__ void load(int u)
    {
        const int t = min(first + u * STRIDE + (lane & 31), L - 1);
        const uint16_t *row = kp + (int64_t)t * ks3 + (lane >> 5) * 8;
#pragma unroll
        for (int s = 0; s < KS; ++s) nxt[s] = *reinterpret_cast<const bf16x8 *>(row + 16 * s);
    }
    __device__ __forceinline__ void prime()
    {
        if (n_sub > 0) load(0);
    }
    __device__ __forceinline__ void fetch(int u, bf16x8 (&kb)[KS])
    {
#pragma unroll
        for (int s = 0; s < KS; ++s) kb[s] = nxt[s];
        if (u + 1 < n_sub) load(u + 1);
    }
};

// the key stream of the any-row-shape kernels by k-steps per key: 8 (D = 128) staged through LDS; 4 (D = 64), 6
// (D = 96) and 16 (D = 256, whose 512-byte rows would need a ring twice the LDS) direct
template <int KS> struct StreamFor { using type = KeyStream<4>; };
template <> struct StreamFor<4> { using type = KeyStreamDirect<4>; };
template <> struct StreamFor<6> { using type = KeyStreamDirect<6>; };
template <> struct StreamFor<16> { using type = KeyStreamDirect<16>; };

// A operands: the window queries of the four heads, query row `n`, k-slices (2s + hf) * 8 .. +8, into
// accumulation registers.  All 32 loads are issued before the first is consumed.
__device__ __forceinline__ void load_queries(bf16x8 (&qa)[4][8], const uint16_t *q, const Dims &d, int p, int h0, int n, int hf)
{
#pragma unroll
    for (int h = 0; h < 4; ++h) {
        if (h0 + h < d.G) {
            const uint16_t *row = q + q_row_offset(d, p, h0 + h, n);   // n: window query of this lane
#pragma unroll
            for (int s = 0; s < 8; ++s) qa[h][s] = *reinterpret_cast<const bf16x8 *>(row + (2 * s + hf) * 8);
        } else {                                                   // a head behind the group's last: padding, zero queries
#pragma unroll
            for (int s = 0; s < 8; ++s) qa[h][s] = bf16x8{};
        }
    }
#pragma unroll
    for (int h = 0; h < 4; ++h)
#pragma unroll
        for (int s = 0; s < 8; ++s) asm volatile("" : "+a"(qa[h][s]));
}

constexpr int NBUF = 4;
constexpr int WAVES = 4;
constexpr int RING_BYTES = NBUF * BUF_BYTES;

// ------------------------------------------------------------------ pass 1
// Row statistics.  Every window-query row keeps, per wavefront, ONE reference shared by the 32 lanes that hold
// the row (stored negated and divided by c1 in LDS, `cref`), and per lane the sum z of exp2(c1 * <q,k> - ref) over
// the lane's keys.  cref is the MFMA C operand, so acc = <q,k> - ref/c1 and the exponent is c1 * acc.  A row is
// anchored at the maximum over the wavefront's first 32 keys and re-anchored (rarely) when a later logit exceeds
// the reference by more than RESCALE_AT, so any finite logits are handled without overflow or total underflow.
//
// The loop over subtiles has two bodies.  The fast one assumes keys before the window (no causal mask) and no
// re-anchoring: per head a maximum over the raw accumulators guards the exponentials, and a head that fails the
// guard leaves the fast body BEFORE anything of it was added.  The careful one (first subtile, subtiles touching
// the window or the end of the sequence, and the rest of a subtile after a failed guard) masks, re-anchors and
// runs the heads one after the other.  Keeping the careful code out of the fast body keeps the fast body free
// of register copies at control-flow joins.

// C operand of head h for this lane half: 16 consecutive floats
__device__ __forceinline__ floatx16 load_cref(const float *cref, int h, int hf)
{
    return *reinterpret_cast<const floatx16 *>(cref + h * 32 + hf * 16);
}

template <int CTRL>
__device__ __forceinline__ float dpp_f(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), CTRL, 0xf, 0xf, false));
}

// careful reduction of one 32-row tile of the subtile whose lane key is t; qf(i) = window query of register i
template <typename QF>
__device__ __forceinline__ void stats_tile_careful(const floatx16 &acc, float (&z)[16], float *cref_h, float c1, bool first,
                                                   int t, int hf, int n, QF qf, int T, int L)
{
    float dd[16];
    float dmax = -INFINITY;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        float v = acc[i] * c1;
        if (!(t < L && t <= T + qf(i))) v = -INFINITY;                   // causal inside the window
        dd[i] = v;
        dmax = fmaxf(dmax, v);
    }
    if (first || __any(dmax > RESCALE_AT)) {
        const float inv_c1 = 1.0f / c1;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            // row maximum over the 32 lanes of this half: four DPP steps inside each row of 16 lanes (lane ^ 1,
            // lane ^ 2, mirror inside 8, mirror inside 16), then the other row of the half
            float rm = dd[i];
            rm = fmaxf(rm, dpp_f<0xB1>(rm));
            rm = fmaxf(rm, dpp_f<0x4E>(rm));
            rm = fmaxf(rm, dpp_f<0x141>(rm));
            rm = fmaxf(rm, dpp_f<0x140>(rm));
            rm = fmaxf(rm, __shfl_xor(rm, 16));
            const bool move = first ? (rm > -INFINITY) : (rm > RESCALE_AT);
            const float cshift = move ? rm * inv_c1 : 0.f;      // change of the C operand
            const float shift = cshift * c1;                    // and the matching change of the exponent
            z[i] *= __builtin_amdgcn_exp2f(-shift);
            dd[i] -= shift;
            if (n == 0 && move) cref_h[hf * 16 + i] -= cshift;
        }
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) z[i] += __builtin_amdgcn_exp2f(dd[i]);
}

// the same for a tile that is one head's 32 window queries
__device__ __forceinline__ void stats_head_careful(const floatx16 &acc, float (&z)[16], float *cref_h, float c1, bool first,
                                                   int t, int hf, int n, int T, int L)
{
    stats_tile_careful(acc, z, cref_h, c1, first, t, hf, n, [hf](int i) { return query_of(i, hf); }, T, L);
}

// guard of the fast body: true when some accumulator of the wavefront exceeds `lim` (= RESCALE_AT / c1)
__device__ __forceinline__ bool stats_guard(const floatx16 &acc, float lim)
{
    float m = fmaxf(acc[0], acc[1]);
#pragma unroll
    for (int i = 2; i < 16; i += 2) m = fmaxf(fmaxf(m, acc[i]), acc[i + 1]);
    return __any(m > lim);
}

__device__ __forceinline__ void stats_add(const floatx16 &acc, float (&z)[16], float c1)
{
#pragma unroll
    for (int i = 0; i < 16; ++i) z[i] += __builtin_amdgcn_exp2f(acc[i] * c1);
    // materialise the sums here: keeps the compiler from sinking this head's exponentials past the next heads
    asm volatile("" : "+v"(z[0]), "+v"(z[1]), "+v"(z[2]), "+v"(z[3]), "+v"(z[4]), "+v"(z[5]), "+v"(z[6]), "+v"(z[7]),
                      "+v"(z[8]), "+v"(z[9]), "+v"(z[10]), "+v"(z[11]), "+v"(z[12]), "+v"(z[13]), "+v"(z[14]), "+v"(z[15]));
}

constexpr int STATS_OK = -1;
constexpr int STATS_PREV = 3;              // the guard failed for head 3 of the previous subtile

// Fast body of one subtile.  Head h is multiplied into acc[h & 1] while head h-1 (head 3: of the previous
// subtile, waiting in acc[1]) is exponentiated from the other accumulator; the first two k-steps of a head are
// issued before the guard of the head before it, the other six after it, next to that head's exponentials.
// Returns STATS_OK, or which head failed its guard: STATS_PREV, or 0..2 = that head of this subtile (the heads
// before it were added, it and the ones after it were not).  Head 3 of this subtile is left waiting in acc[1].
__device__ __forceinline__ int stats_fast(const bf16x8 (&qa)[4][8], const bf16x8 (&kb)[8], floatx16 (&acc)[2],
                                          const floatx16 (&cr)[4], float (&z)[4][16], float c1, float lim)
{
    acc[0] = chain<0, 2>(qa[0], kb, cr[0]);
    if (stats_guard(acc[1], lim)) return STATS_PREV;
    acc[0] = chain<2, 8>(qa[0], kb, acc[0]);
    stats_add(acc[1], z[3], c1);
    acc[1] = chain<0, 2>(qa[1], kb, cr[1]);
    if (stats_guard(acc[0], lim)) return 0;
    acc[1] = chain<2, 8>(qa[1], kb, acc[1]);
    stats_add(acc[0], z[0], c1);
    acc[0] = chain<0, 2>(qa[2], kb, cr[2]);
    if (stats_guard(acc[1], lim)) return 1;
    acc[0] = chain<2, 8>(qa[2], kb, acc[0]);
    stats_add(acc[1], z[1], c1);
    acc[1] = chain<0, 2>(qa[3], kb, cr[3]);
    if (stats_guard(acc[0], lim)) return 2;
    acc[1] = chain<2, 8>(qa[3], kb, acc[1]);
    stats_add(acc[0], z[2], c1);
    return STATS_OK;
}

// Careful body: heads h_from..3 of the subtile in kb, one after the other, each multiplied afresh against the
// references as they are now.
__device__ __forceinline__ void stats_careful(const bf16x8 (&qa)[4][8], const bf16x8 (&kb)[8], float *cref, float (&z)[4][16],
                                              float c1, int h_from, bool first, int t, int hf, int n, int T, int L)
{
#pragma unroll
    for (int h = 0; h < 4; ++h) {
        if (h >= h_from) {
            const floatx16 a = chain<0, 8>(qa[h], kb, load_cref(cref, h, hf));
            stats_head_careful(a, z[h], cref + 32 * h, c1, first, t, hf, n, T, L);
        }
    }
}

__global__ void __launch_bounds__(WAVES * 64)
score_mfma_stats(ScoreArgs a)
{
    extern __shared__ __attribute__((aligned(8192))) char lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 31, hf = lane >> 5;
    const Dims &d = a.d;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    char *ring = lds + wave_u * RING_BYTES;
    float *wg_red = reinterpret_cast<float *>(lds + WAVES * RING_BYTES);       // [WAVES][128][2]
    float *cref = wg_red + WAVES * M_ROWS * 2 + wave_u * M_ROWS;               // [4 heads][2 halves][16], this wave's
    const WaveWork w = wave_work_blocks(a, wave);
    const int Tq = d.T + w.qoff;                               // causal limit of this block's query 0: key t is visible to query i iff t <= Tq + i

    KeyStream<NBUF> ks;
    ks.init(w.kp, d.ks[3], ring, w.first, w.n_sub, d.L, lane);
    ks.prime();

    bf16x8 qa[4][8];
    load_queries(qa, a.q, d, w.p, w.hoff, w.qoff + n, hf);
    cref[lane] = 0.f;
    cref[lane + 64] = 0.f;

    floatx16 acc[2];
    float z[4][16];
#pragma unroll
    for (int h = 0; h < 4; ++h)
#pragma unroll
        for (int i = 0; i < 16; ++i) { z[h][i] = 0.f; acc[h & 1][i] = -INFINITY; }

    // `waiting`: head 3 of subtile u-1 sits in acc[1], multiplied but not yet reduced (never of subtile 0, which
    // the careful body handles whole).  When nothing waits, acc[1] = -inf makes the fast body's first step add zeros.
    const float lim = RESCALE_AT / a.c1;
    floatx16 cr[4];                                            // the rows' references as MFMA C operands (copy of cref)
#pragma unroll
    for (int h = 0; h < 4; ++h)
#pragma unroll
        for (int i = 0; i < 16; ++i) cr[h][i] = 0.f;
    bool waiting = false;
    for (int u = 0; u < w.n_sub; ++u) {
        bf16x8 kb[8];
        ks.fetch(u, kb);
        const int t0 = w.first + u * STRIDE;
        int code = 0;
        const bool plain = u > 0 && t0 + SUB <= d.T;           // neither the anchoring subtile nor a masked one
        if (plain) code = stats_fast(qa, kb, acc, cr, z, a.c1, lim);
        if (code == STATS_OK) { waiting = true; continue; }
        if (waiting && (!plain || code == STATS_PREV))         // the waiting head was not reduced by the fast body
            stats_head_careful(acc[1], z[3], cref + 96, a.c1, false, t0 - STRIDE + n, hf, n, Tq, d.L);
        stats_careful(qa, kb, cref, z, a.c1, (plain && code != STATS_PREV) ? code : 0, u == 0, t0 + n, hf, n, Tq, d.L);
        waiting = false;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[1][i] = -INFINITY;
#pragma unroll
        for (int h = 0; h < 4; ++h) cr[h] = load_cref(cref, h, hf);     // the careful body may have moved references
    }
    if (waiting)
        stats_head_careful(acc[1], z[3], cref + 96, a.c1, false, w.first + (w.n_sub - 1) * STRIDE + n, hf, n, Tq, d.L);

    // ---- per row: add the 32 lane sums (same reference) through the wavefront's ring (every load has landed),
    // then combine the four wavefronts' (reference, sum) pairs
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    float *scr_z = reinterpret_cast<float *>(ring);            // [128 rows][32 lanes]
#pragma unroll
    for (int h = 0; h < 4; ++h)
#pragma unroll
        for (int i = 0; i < 16; ++i) scr_z[(h * 32 + query_of(i, hf)) * 32 + n] = z[h][i];
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int rr = 0; rr < 2; ++rr) {
        const int row = lane + 64 * rr;                         // row = h * 32 + query
        float zz = 0.f;
        for (int j = 0; j < 32; ++j) zz += scr_z[row * 32 + ((j + lane) & 31)];
        const int q = row & 31, hfq = (q >> 2) & 1, iq = ((q >> 3) << 2) | (q & 3);
        wg_red[(wave * M_ROWS + row) * 2] = -cref[(row >> 5) * 32 + hfq * 16 + iq] * a.c1;   // reference, log2 domain
        wg_red[(wave * M_ROWS + row) * 2 + 1] = zz;
    }
    __syncthreads();
    if (threadIdx.x < M_ROWS) {
        const int row = threadIdx.x;
        float m = -INFINITY;
        for (int wv = 0; wv < WAVES; ++wv) {
            const float *e = wg_red + (wv * M_ROWS + row) * 2;
            if (e[1] > 0.f) m = fmaxf(m, e[0]);
        }
        float zz = 0.f;
        for (int wv = 0; wv < WAVES; ++wv) {
            const float *e = wg_red + (wv * M_ROWS + row) * 2;
            if (e[1] > 0.f) zz += e[1] * __builtin_amdgcn_exp2f(e[0] - m);
        }
        float *o = a.partial + (((int64_t)w.pv * a.n_chunks + w.chunk) * M_ROWS + row) * 2;
        o[0] = m;
        o[1] = zz;
    }
}

// ------------------------------------------------------------------ pass 2
// acc = <q,k> - (lse2 + log2 G)/c1 per (head, query), so exp2(c1 * acc) = A / G
template <bool EDGE, bool ASSIGN>
__device__ __forceinline__ void columns_head(const floatx16 &acc, float (&ab)[16], float c1, int t, int hf, int T, int L)
{
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        float v = __builtin_amdgcn_exp2f(acc[i] * c1);
        if (EDGE && !(t < L && t <= T + query_of(i, hf))) v = 0.f;      // causal inside the window
        ab[i] = ASSIGN ? v : ab[i] + v;                                   // Eq. barA, accumulated over the heads
    }
}

// x of this lane plus x of the lane 32 away: one swap of the upper half of a register with the lower half of
// its copy, so both results hold (lower-half value, upper-half value) in every lane
__device__ __forceinline__ float add_other_half(float x)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// column sum (Eq. st, lane half 0) or entropy term (inner sum of Eq. Dk, lane half 1) from the lane's 16 Abar values
__device__ __forceinline__ float columns_finish(const float (&ab)[16], float eps, int hf)
{
    float s_part = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s_part += ab[i];
    const float s = add_other_half(s_part);
    const float inv_s = s > 0.f ? __builtin_amdgcn_rcpf(s) : 0.f;
    // sum_i Ahat_i log2(Ahat_i + eps) with Ahat_i = Abar_i / s: the division of the weights is applied once, to the sum
    float e_part = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) e_part = fmaf(ab[i], __builtin_amdgcn_logf(fmaf(ab[i], inv_s, eps)), e_part);
    const float ent = -LN2 * inv_s * add_other_half(e_part);
    return hf == 0 ? s : ent;
}

// One subtile: head h is multiplied into acc[h & 1] while head h-1 is exponentiated from the other accumulator;
// returns the output value of the PREVIOUS subtile.
template <bool EDGE>
__device__ __forceinline__ float columns_body(const bf16x8 (&qa)[4][8], const bf16x8 (&kb)[8], const floatx16 (&cinit)[4],
                                              floatx16 (&acc)[2], float (&ab)[16], float c1, float eps, int t_prev, int t_cur,
                                              int hf, int T, int L)
{
    acc[0] = chain<0, 8>(qa[0], kb, cinit[0]);
    columns_head<EDGE, false>(acc[1], ab, c1, t_prev, hf, T, L);       // last head of the previous subtile
    const float prev = columns_finish(ab, eps, hf);
    acc[1] = chain<0, 8>(qa[1], kb, cinit[1]);
    columns_head<EDGE, true>(acc[0], ab, c1, t_cur, hf, T, L);
    acc[0] = chain<0, 8>(qa[2], kb, cinit[2]);
    columns_head<EDGE, false>(acc[1], ab, c1, t_cur, hf, T, L);
    acc[1] = chain<0, 8>(qa[3], kb, cinit[3]);
    columns_head<EDGE, false>(acc[0], ab, c1, t_cur, hf, T, L);
    return prev;
}

__global__ void __launch_bounds__(WAVES * 64)
score_mfma_columns(ScoreArgs a)
{
    extern __shared__ __attribute__((aligned(8192))) char lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 31, hf = lane >> 5;
    const Dims &d = a.d;
    char *ring = lds + __builtin_amdgcn_readfirstlane(wave) * RING_BYTES;
    float *lse2 = reinterpret_cast<float *>(lds + WAVES * RING_BYTES);       // [128] log2-domain lse + log2 G
    float *comb = lse2 + M_ROWS;                                             // [256][2] combine scratch
    const WaveWork w = wave_work(a, wave);

    KeyStream<NBUF> ks;
    ks.init(w.kp, d.ks[3], ring, w.first, w.n_sub, d.L, lane);
    ks.prime();

    // row log-sum-exp: given by the caller, or combined here from the chunk partials of pass 1 (two threads per
    // row, each folding every other chunk with an online max / rescaled sum)
    {
        const int row = threadIdx.x & (M_ROWS - 1), half = threadIdx.x >> 7;
        float m = -INFINITY, zz = 0.f;
        if (a.lse) {
            m = a.lse[(int64_t)w.p * M_ROWS + row] * LOG2E;
            zz = half == 0 ? 1.f : 0.f;
        } else {
            const float *pp = a.merged + ((int64_t)w.p * a.pc * M_ROWS + row) * 2;
#pragma unroll 4
            for (int c = half; c < a.pc; c += 2) {
                const float2 e = *reinterpret_cast<const float2 *>(pp + (int64_t)c * M_ROWS * 2);
                if (e.y > 0.f) {
                    const float mn = fmaxf(m, e.x);
                    zz = zz * __builtin_amdgcn_exp2f(m - mn) + e.y * __builtin_amdgcn_exp2f(e.x - mn);
                    m = mn;
                }
            }
        }
        comb[threadIdx.x * 2] = m;
        comb[threadIdx.x * 2 + 1] = zz;
    }
    __syncthreads();
    if (threadIdx.x < M_ROWS) {
        const float m0 = comb[threadIdx.x * 2], z0 = comb[threadIdx.x * 2 + 1];
        const float m1 = comb[(threadIdx.x + M_ROWS) * 2], z1 = comb[(threadIdx.x + M_ROWS) * 2 + 1];
        const float mn = fmaxf(m0, m1);
        float zz = 0.f;
        if (z0 > 0.f) zz += z0 * __builtin_amdgcn_exp2f(m0 - mn);
        if (z1 > 0.f) zz += z1 * __builtin_amdgcn_exp2f(m1 - mn);
        lse2[threadIdx.x] = mn + __builtin_amdgcn_logf(zz) + 2.0f;        // + log2(G): exp2 then yields A / G
    }
    __syncthreads();

    bf16x8 qa[4][8];
    floatx16 cinit[4], acc[2];
    const float inv_c1 = 1.0f / a.c1;
    load_queries(qa, a.q, d, w.p, 0, n, hf);
#pragma unroll
    for (int h = 0; h < 4; ++h) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            cinit[h][i] = -lse2[h * 32 + query_of(i, hf)] * inv_c1;
            acc[h & 1][i] = -INFINITY;                         // makes the "previous subtile" of iteration 0 a no-op
        }
    }
    float ab[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) ab[i] = 0.f;
    float *out = (hf == 0 ? a.s_out : a.e_out) + (int64_t)w.p * d.L;

    // Results are stored one iteration late, at the top of the next iteration, so that the multiply/exponentiate
    // section of an iteration is a single straight-line region.  The subtiles before the window (no mask) and
    // the ones that touch the window or the end of the sequence run in two consecutive loops, which keeps the
    // masked body and its control-flow joins out of the hot loop.
    float pending = 0.f;
    int pending_t = -1;
    const int n_plain = w.first + SUB <= d.T ? min(w.n_sub, (d.T - SUB - w.first) / STRIDE + 1) : 0;
    int u = 0;
    for (; u < n_plain; ++u) {
        if (pending_t >= 0) out[pending_t] = pending;
        bf16x8 kb[8];
        ks.fetch(u, kb);
        const int t_cur = w.first + u * STRIDE + n;
        pending = columns_body<false>(qa, kb, cinit, acc, ab, a.c1, a.eps, t_cur - STRIDE, t_cur, hf, d.T, d.L);
        pending_t = u > 0 ? t_cur - STRIDE : -1;
    }
    for (; u < w.n_sub; ++u) {
        if (pending_t >= 0 && pending_t < d.L) out[pending_t] = pending;
        bf16x8 kb[8];
        ks.fetch(u, kb);
        const int t_cur = w.first + u * STRIDE + n;
        pending = columns_body<true>(qa, kb, cinit, acc, ab, a.c1, a.eps, t_cur - STRIDE, t_cur, hf, d.T, d.L);
        pending_t = u > 0 ? t_cur - STRIDE : -1;
    }
    if (pending_t >= 0 && pending_t < d.L) out[pending_t] = pending;
    if (w.n_sub > 0) {
        const int t_last = w.first + (w.n_sub - 1) * STRIDE + n;
        columns_head<true, false>(acc[1], ab, a.c1, t_last, hf, d.T, d.L);
        const float v = columns_finish(ab, a.eps, hf);
        if (t_last < d.L) out[t_last] = v;
    }
}

// ------------------------------------------------------------------ pass 2, 256 rows
// Eight 32-row tiles.  W = 64: tile j holds head j / 2, window queries 32 (j % 2) .. +32; W = 32: tile j holds
// head j.  Groups of fewer heads than the tiles hold (G = 5 .. 7 with W = 32, G = 3 with W = 64) leave the last
// tiles as padding: zero queries and an infinite log-sum-exp, so they add exact zeros.  Same pipeline as above with
// the tiles rotating through two accumulators; ab[b] collects the head mean of the window queries 32 b .. 32 b + 31.
template <int W> struct Tiles8 {
    static constexpr int NB = W / 32;                                        // 32-query blocks of the window
    __host__ __device__ static constexpr int head(int j) { return W == 64 ? j / 2 : j; }
    __host__ __device__ static constexpr int qoff(int j) { return W == 64 ? 32 * (j % 2) : 0; }
    __host__ __device__ static constexpr int blk(int j) { return W == 64 ? j % 2 : 0; }
    __host__ __device__ static constexpr bool first(int j) { return W == 64 ? j < 2 : j == 0; }   // first tile of its block
    // where pass 1 stored the statistics of tile j: (row block, 32-row group inside it)
    __host__ __device__ static constexpr int p1_block(int j) { return W == 64 ? j % 2 : j / 4; }
    __host__ __device__ static constexpr int p1_group(int j) { return W == 64 ? j / 2 : j % 4; }
};
constexpr int M_ROWS64 = 256;
constexpr int P2W_LDS = 4 * 4 * BUF_BYTES + M_ROWS64 * 4 + 8 * 32 * 4;   // rings + the rows' log-sum-exp + C operands

template <int NB>
__device__ __forceinline__ float columns_finish8t(const float (&ab)[NB][16], float eps, int hf)
{
    float s_part = 0.f;
#pragma unroll
    for (int v = 0; v < NB; ++v)
#pragma unroll
        for (int i = 0; i < 16; ++i) s_part += ab[v][i];
    const float s = add_other_half(s_part);
    const float inv_s = s > 0.f ? __builtin_amdgcn_rcpf(s) : 0.f;
    float e_part = 0.f;
#pragma unroll
    for (int v = 0; v < NB; ++v)
#pragma unroll
        for (int i = 0; i < 16; ++i) e_part = fmaf(ab[v][i], __builtin_amdgcn_logf(fmaf(ab[v][i], inv_s, eps)), e_part);
    const float ent = -LN2 * inv_s * add_other_half(e_part);
    return hf == 0 ? s : ent;
}

__device__ __forceinline__ floatx16 load_c64(const float *cmat, int j, int hf)
{
    return *reinterpret_cast<const floatx16 *>(cmat + j * 32 + hf * 16);
}

// One subtile; returns the output value of the PREVIOUS subtile (its last tile waits in acc[1])
template <int W, bool EDGE, int J>
__device__ __forceinline__ void columns_tile8t(const floatx16 &acc, float (&ab)[Tiles8<W>::NB][16], float c1, int t, int hf,
                                               int T, int L)
{
    using TL = Tiles8<W>;
    columns_head<EDGE, TL::first(J)>(acc, ab[TL::blk(J)], c1, t, hf, T + TL::qoff(J), L);
}

template <int W, bool EDGE>
__device__ __forceinline__ float columns_body8t(const bf16x8 (&qa)[8][8], const bf16x8 (&kb)[8], const float *cmat,
                                                floatx16 (&acc)[2], float (&ab)[Tiles8<W>::NB][16], float c1, float eps,
                                                int t_prev, int t_cur, int hf, int T, int L)
{
    using TL = Tiles8<W>;
    acc[0] = chain<0, 8>(qa[0], kb, load_c64(cmat, 0, hf));
    columns_head<EDGE, false>(acc[1], ab[TL::blk(7)], c1, t_prev, hf, T + TL::qoff(7), L);     // tile 7 of the previous subtile
    const float prev = columns_finish8t<TL::NB>(ab, eps, hf);
    acc[1] = chain<0, 8>(qa[1], kb, load_c64(cmat, 1, hf));
    columns_tile8t<W, EDGE, 0>(acc[0], ab, c1, t_cur, hf, T, L);
    acc[0] = chain<0, 8>(qa[2], kb, load_c64(cmat, 2, hf));
    columns_tile8t<W, EDGE, 1>(acc[1], ab, c1, t_cur, hf, T, L);
    acc[1] = chain<0, 8>(qa[3], kb, load_c64(cmat, 3, hf));
    columns_tile8t<W, EDGE, 2>(acc[0], ab, c1, t_cur, hf, T, L);
    acc[0] = chain<0, 8>(qa[4], kb, load_c64(cmat, 4, hf));
    columns_tile8t<W, EDGE, 3>(acc[1], ab, c1, t_cur, hf, T, L);
    acc[1] = chain<0, 8>(qa[5], kb, load_c64(cmat, 5, hf));
    columns_tile8t<W, EDGE, 4>(acc[0], ab, c1, t_cur, hf, T, L);
    acc[0] = chain<0, 8>(qa[6], kb, load_c64(cmat, 6, hf));
    columns_tile8t<W, EDGE, 5>(acc[1], ab, c1, t_cur, hf, T, L);
    acc[1] = chain<0, 8>(qa[7], kb, load_c64(cmat, 7, hf));
    columns_tile8t<W, EDGE, 6>(acc[0], ab, c1, t_cur, hf, T, L);
    return prev;
}

template <int W>
__global__ void __launch_bounds__(WAVES * 64)
score_mfma_columns8t(ScoreArgs a)
{
    using TL = Tiles8<W>;
    extern __shared__ __attribute__((aligned(8192))) char lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 31, hf = lane >> 5;
    const Dims &d = a.d;
    char *ring = lds + __builtin_amdgcn_readfirstlane(wave) * RING_BYTES;
    float *lse2 = reinterpret_cast<float *>(lds + WAVES * RING_BYTES);       // [256] log2-domain lse + log2 G, row h * W + i
    float *cmat = lse2 + M_ROWS64;                                           // [8 tiles][2 halves][16] C operands
    const WaveWork w = wave_work(a, wave);

    KeyStream<NBUF> ks;
    ks.init(w.kp, d.ks[3], ring, w.first, w.n_sub, d.L, lane);
    ks.prime();

    // one thread per row (h, i): its log-sum-exp, given by the caller or folded from the chunk partials of pass 1,
    // which are stored per 128-row block (see Tiles8::p1_block / p1_group)
    {
        const int r = threadIdx.x, h = r / W, i = r % W;
        const int j = W == 64 ? 2 * h + i / 32 : h;                           // the row's tile
        float m = -INFINITY, zz = 0.f;
        if (h >= d.G) {                                                       // padding row
            m = INFINITY;
            zz = 1.f;
        } else if (a.lse) {
            m = a.lse[(int64_t)w.p * d.G * W + r] * LOG2E;
            zz = 1.f;
        } else {
            const float *pp = a.merged + (((int64_t)(w.p * 2 + TL::p1_block(j)) * a.pc) * M_ROWS + TL::p1_group(j) * 32 + (i & 31)) * 2;
            for (int c = 0; c < a.pc; ++c) {
                const float2 e = *reinterpret_cast<const float2 *>(pp + (int64_t)c * M_ROWS * 2);
                if (e.y > 0.f) {
                    const float mn = fmaxf(m, e.x);
                    zz = zz * __builtin_amdgcn_exp2f(m - mn) + e.y * __builtin_amdgcn_exp2f(e.x - mn);
                    m = mn;
                }
            }
        }
        lse2[r] = m + __builtin_amdgcn_logf(zz) + a.log2_G;                   // + log2(G): exp2 then yields A / G
    }
    __syncthreads();
    {
        const float inv_c1 = 1.0f / a.c1;
        const int j = threadIdx.x >> 5, slot = threadIdx.x & 31;
        const int i = TL::qoff(j) + query_of(slot & 15, slot >> 4);
        cmat[threadIdx.x] = -lse2[TL::head(j) * W + i] * inv_c1;
    }
    __syncthreads();

    bf16x8 qa[8][8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        if (TL::head(j) < d.G) {
            const uint16_t *row = a.q + q_row_offset(d, w.p, TL::head(j), TL::qoff(j) + n);
#pragma unroll
            for (int s = 0; s < 8; ++s) qa[j][s] = *reinterpret_cast<const bf16x8 *>(row + (2 * s + hf) * 8);
        } else {
#pragma unroll
            for (int s = 0; s < 8; ++s) qa[j][s] = bf16x8{};
        }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int s = 0; s < 8; ++s) asm volatile("" : "+a"(qa[j][s]));       // all 256 accumulation registers

    floatx16 acc[2];
    float ab[TL::NB][16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        acc[0][i] = acc[1][i] = -INFINITY;
#pragma unroll
        for (int v = 0; v < TL::NB; ++v) ab[v][i] = 0.f;
    }
    float *out = (hf == 0 ? a.s_out : a.e_out) + (int64_t)w.p * d.L;

    float pending = 0.f;
    int pending_t = -1;
    const int n_plain = w.first + SUB <= d.T ? min(w.n_sub, (d.T - SUB - w.first) / STRIDE + 1) : 0;
    int u = 0;
    for (; u < n_plain; ++u) {
        if (pending_t >= 0) out[pending_t] = pending;
        bf16x8 kb[8];
        ks.fetch_vgpr(u, kb);
        const int t_cur = w.first + u * STRIDE + n;
        pending = columns_body8t<W, false>(qa, kb, cmat, acc, ab, a.c1, a.eps, t_cur - STRIDE, t_cur, hf, d.T, d.L);
        pending_t = u > 0 ? t_cur - STRIDE : -1;
    }
    for (; u < w.n_sub; ++u) {
        if (pending_t >= 0 && pending_t < d.L) out[pending_t] = pending;
        bf16x8 kb[8];
        ks.fetch_vgpr(u, kb);
        const int t_cur = w.first + u * STRIDE + n;
        pending = columns_body8t<W, true>(qa, kb, cmat, acc, ab, a.c1, a.eps, t_cur - STRIDE, t_cur, hf, d.T, d.L);
        pending_t = u > 0 ? t_cur - STRIDE : -1;
    }
    if (pending_t >= 0 && pending_t < d.L) out[pending_t] = pending;
    if (w.n_sub > 0) {
        const int t_last = w.first + (w.n_sub - 1) * STRIDE + n;
        columns_head<true, false>(acc[1], ab[TL::blk(7)], a.c1, t_last, hf, d.T + TL::qoff(7), d.L);
        const float v = columns_finish8t<TL::NB>(ab, a.eps, hf);
        if (t_last < d.L) out[t_last] = v;
    }
}

// ------------------------------------------------------------------ pass 2, all heads of a layer
// Head mean over all 32 heads of a layer with 8 KV heads (Eq. barA taken literally) without writing the
// per-KV-head means to memory.  A workgroup owns a chunk of keys of one (sequence, layer).  Wavefront w multiplies
// the keys of KV heads 2w and 2w+1 (two load streams interleaved in one ring) by those heads' 8 query heads (256
// accumulation registers of A operands) and adds exp2 over its 8 heads; the four partial sums of a subtile meet
// in LDS, where the wavefronts take turns (subtile u: wavefront u % 4) to add them and to form the column sum
// and the entropy term.  One barrier per subtile; it waits for LDS only, never for the loads in flight.
typedef float floatx4 __attribute__((ext_vector_type(4)));
constexpr int LAYER_KV = 8;                   // KV heads of a layer this kernel is built for (two per wavefront)
constexpr int XCH_BYTES = 16 * 64 * 4;        // one wavefront's partial sums of a subtile, [4][64 lanes][4]
constexpr int PL_LDS = WAVES * RING_BYTES + 2 * 3 * XCH_BYTES + WAVES * 8 * 32 * 4;   // rings + exchange + C operands

// Two key streams of one wavefront as one sequence of half-steps: element e = 2u + s is subtile u of stream s and
// lives in ring buffer e % NBUF, refilled with element e + NBUF right after it is read.  Subtile u covers keys
// [first + u * SUB, +SUB): here all wavefronts of a workgroup walk the same keys.
struct PairStream {
    const uint16_t *kp0, *kp1;
    int64_t ks3;
    uint32_t lane_addr0, ring_lds;
    uint32_t lane_off[4];
    int first, n_el, L, lane;

    __device__ __forceinline__ void init(const uint16_t *k0, const uint16_t *k1, int64_t ks3_, char *ring, int first_, int n_sub, int L_, int lane_)
    {
        kp0 = k0; kp1 = k1; ks3 = ks3_; first = first_; n_el = 2 * n_sub; L = L_; lane = lane_;
        const int n = lane & 31, hf = lane >> 5, r4 = lane >> 4, pos = lane & 15;
        ring_lds = __builtin_amdgcn_readfirstlane(lds_addr(ring));
        lane_addr0 = ring_lds + n * ROW_BYTES + ((hf ^ (n & 15)) << 4);
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) lane_off[jj] = (uint32_t)(r4 * ks3 * 2) + (uint32_t)(((pos ^ r4 ^ (4 * jj)) & 15) << 4);
    }
    __device__ __forceinline__ void issue(int e) const
    {
        const int t0 = first + (e >> 1) * SUB;                 // wave-uniform, < L
        const char *base = reinterpret_cast<const char *>((e & 1) ? kp1 : kp0) + (int64_t)t0 * ks3 * 2;
        const uint32_t buf_lds = ring_lds + (e % NBUF) * BUF_BYTES;
        if (t0 + SUB <= L) {
            if (ks3 == ROW_BYTES / 2) issue_subtile_dense(base, lane_off, buf_lds);
            else issue_subtile_fast(base, ks3 * 2, lane_off, buf_lds);
        } else issue_subtile_clamped(base, ks3 * 2, L - t0, buf_lds, lane);
    }
    __device__ __forceinline__ void prime() const
    {
#pragma unroll
        for (int e = 0; e < NBUF; ++e)
            if (e < n_el) issue(e);
    }
    __device__ __forceinline__ void fetch(int e, bf16x8 (&kb)[8]) const
    {
        wait_loads(min(NBUF - 1, n_el - 1 - e));
        read_subtile_vgpr(lane_addr0 + (e % NBUF) * BUF_BYTES, kb);
        if (e + NBUF < n_el) issue(e + NBUF);
    }
};

// this lane's 16 partial sums into an exchange slot / the sum of `ab` and the three slots of a buffer
__device__ __forceinline__ void xch_write(uint32_t addr, const float (&ab)[16])
{
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const floatx4 v = {ab[4 * j], ab[4 * j + 1], ab[4 * j + 2], ab[4 * j + 3]};
        asm volatile("ds_write_b128 %0, %1" : : "v"(addr + j * 1024), "v"(v) : "memory");
    }
}
__device__ __forceinline__ void xch_add(uint32_t addr, float (&ab)[16])
{
    floatx4 v[3][4];
#pragma unroll
    for (int sl = 0; sl < 3; ++sl)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            asm volatile("ds_read_b128 %0, %1" : "=v"(v[sl][j]) : "v"(addr + sl * XCH_BYTES + j * 1024) : "memory");
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(v[0][0]), "+v"(v[0][1]), "+v"(v[0][2]), "+v"(v[0][3]), "+v"(v[1][0]), "+v"(v[1][1]), "+v"(v[1][2]),
                   "+v"(v[1][3]), "+v"(v[2][0]), "+v"(v[2][1]), "+v"(v[2][2]), "+v"(v[2][3])
                 :
                 : "memory");
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int c = 0; c < 4; ++c) ab[4 * j + c] += v[0][j][c] + v[1][j][c] + v[2][j][c];
}
// all LDS writes of this wavefront done, then the workgroup barrier (global loads stay in flight)
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

struct LayerCtx {
    uint32_t xch_lds;      // exchange area
    int wave, lane, n, hf;
    int lo;                // first key of the chunk
    float c1, eps;
    int T, L;
    float *out;            // s (lane half 0) or entropy term (lane half 1) row of this (sequence, layer)
};

// the partial sums `ab` of subtile `up` are complete in every wavefront: hand them to wavefront up % 4 ...
__device__ __forceinline__ void layer_give(const LayerCtx &c, int up, const float (&ab)[16])
{
    const int fin = up & 3;
    if (c.wave != fin) xch_write(c.xch_lds + (uint32_t)(((up & 1) * 3 + ((c.wave - fin - 1) & 3)) * XCH_BYTES + c.lane * 16), ab);
}
// ... which, after the barrier, adds them up and stores the two results of its key
__device__ __forceinline__ void layer_take(const LayerCtx &c, int up, float (&ab)[16])
{
    if (c.wave != (up & 3)) return;
    xch_add(c.xch_lds + (uint32_t)((up & 1) * 3 * XCH_BYTES + c.lane * 16), ab);
    const float v = columns_finish(ab, c.eps, c.hf);
    const int t = c.lo + up * SUB + c.n;
    if (t < c.L) c.out[t] = v;
}

// One subtile u: tiles 0-3 (KV head 2w) then 4-7 (KV head 2w+1), rotating through two accumulators; tile 7 of the
// previous subtile is exponentiated first, which completes that subtile's partial sums (handed over mid-way).
template <bool EDGE>
__device__ __forceinline__ void layer_body(const LayerCtx &c, const bf16x8 (&qa)[8][8], const PairStream &ps, const float *cm,
                                           floatx16 (&acc)[2], float (&ab)[16], int u)
{
    const int t_cur = c.lo + u * SUB + c.n, t_prev = t_cur - SUB;
    bf16x8 kb[8];
    ps.fetch(2 * u, kb);
    acc[0] = chain<0, 8>(qa[0], kb, load_c64(cm, 0, c.hf));
    columns_head<EDGE, false>(acc[1], ab, c.c1, t_prev, c.hf, c.T, c.L);
    float abp[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) abp[i] = ab[i];
    if (u > 0) layer_give(c, u - 1, abp);
    acc[1] = chain<0, 8>(qa[1], kb, load_c64(cm, 1, c.hf));
    columns_head<EDGE, true>(acc[0], ab, c.c1, t_cur, c.hf, c.T, c.L);
    acc[0] = chain<0, 8>(qa[2], kb, load_c64(cm, 2, c.hf));
    columns_head<EDGE, false>(acc[1], ab, c.c1, t_cur, c.hf, c.T, c.L);
    acc[1] = chain<0, 8>(qa[3], kb, load_c64(cm, 3, c.hf));
    columns_head<EDGE, false>(acc[0], ab, c.c1, t_cur, c.hf, c.T, c.L);
    ps.fetch(2 * u + 1, kb);
    acc[0] = chain<0, 8>(qa[4], kb, load_c64(cm, 4, c.hf));
    columns_head<EDGE, false>(acc[1], ab, c.c1, t_cur, c.hf, c.T, c.L);
    if (u > 0) {                                               // u is uniform over the workgroup
        lds_barrier();
        layer_take(c, u - 1, abp);
    }
    acc[1] = chain<0, 8>(qa[5], kb, load_c64(cm, 5, c.hf));
    columns_head<EDGE, false>(acc[0], ab, c.c1, t_cur, c.hf, c.T, c.L);
    acc[0] = chain<0, 8>(qa[6], kb, load_c64(cm, 6, c.hf));
    columns_head<EDGE, false>(acc[1], ab, c.c1, t_cur, c.hf, c.T, c.L);
    acc[1] = chain<0, 8>(qa[7], kb, load_c64(cm, 7, c.hf));
    columns_head<EDGE, false>(acc[0], ab, c.c1, t_cur, c.hf, c.T, c.L);
}

__global__ void __launch_bounds__(WAVES * 64)
score_mfma_columns_layer(ScoreArgs a)
{
    extern __shared__ __attribute__((aligned(8192))) char lds[];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const Dims &d = a.d;
    char *ring = lds + wave * RING_BYTES;
    char *xch = lds + WAVES * RING_BYTES;                                     // [2 buffers][3 slots][4][64 lanes][4]
    float *cmat = reinterpret_cast<float *>(xch + 2 * 3 * XCH_BYTES);         // [wave][8 tiles][2 halves][16] C operands
    const int sl = blockIdx.x / a.n_chunks, chunk = blockIdx.x - sl * a.n_chunks;
    const int p_first = sl * LAYER_KV;                                        // the layer's first problem
    const int lo = chunk * a.chunk_len, hi = min(lo + a.chunk_len, d.L);
    const int n_sub = hi > lo ? (hi - lo + SUB - 1) / SUB : 0;                // the same for the four wavefronts

    PairStream ps;
    ps.init(a.k + k_problem_offset(d, p_first + 2 * wave), a.k + k_problem_offset(d, p_first + 2 * wave + 1), d.ks[3], ring, lo,
            n_sub, d.L, lane);
    ps.prime();

    // C operands: minus (row log-sum-exp + log2 of the number of heads) / c1, so that exp2(c1 * acc) = A / H.
    // Row R = kv * 128 + h * 32 + query; four rows per thread.
    {
        const float inv_c1 = 1.0f / a.c1, log2_heads = __builtin_amdgcn_logf((float)(d.G * LAYER_KV));
#pragma unroll
        for (int k4 = 0; k4 < 4; ++k4) {
            const int R = threadIdx.x + 256 * k4, kv = R >> 7, row = R & (M_ROWS - 1);
            float m = -INFINITY, zz = 0.f;
            if (a.lse) {
                m = a.lse[(int64_t)(p_first + kv) * M_ROWS + row] * LOG2E;
                zz = 1.f;
            } else {
                const float *pp = a.merged + ((int64_t)(p_first + kv) * a.pc * M_ROWS + row) * 2;
                for (int c = 0; c < a.pc; ++c) {
                    const float2 e = *reinterpret_cast<const float2 *>(pp + (int64_t)c * M_ROWS * 2);
                    if (e.y > 0.f) {
                        const float mn = fmaxf(m, e.x);
                        zz = zz * __builtin_amdgcn_exp2f(m - mn) + e.y * __builtin_amdgcn_exp2f(e.x - mn);
                        m = mn;
                    }
                }
            }
            const int qy = row & 31, j = (kv & 1) * 4 + (row >> 5);
            const int hq = (qy >> 2) & 1, iq = ((qy >> 3) << 2) | (qy & 3);   // inverse of query_of
            cmat[((kv >> 1) * 8 + j) * 32 + hq * 16 + iq] = -(m + __builtin_amdgcn_logf(zz) + log2_heads) * inv_c1;
        }
    }
    __syncthreads();

    LayerCtx c;
    c.xch_lds = __builtin_amdgcn_readfirstlane(lds_addr(xch));
    c.wave = wave; c.lane = lane; c.n = lane & 31; c.hf = lane >> 5;
    c.lo = lo; c.c1 = a.c1; c.eps = a.eps; c.T = d.T; c.L = d.L;
    c.out = (c.hf == 0 ? a.s_out : a.e_out) + (int64_t)sl * d.L;
    const float *cm = cmat + wave * 8 * 32;

    bf16x8 qa[8][8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uint16_t *row = a.q + q_row_offset(d, p_first + 2 * wave + j / 4, j % 4, c.n);
#pragma unroll
        for (int s = 0; s < 8; ++s) qa[j][s] = *reinterpret_cast<const bf16x8 *>(row + (2 * s + c.hf) * 8);
    }
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int s = 0; s < 8; ++s) asm volatile("" : "+a"(qa[j][s]));       // all 256 accumulation registers

    floatx16 acc[2];
    float ab[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) { acc[0][i] = acc[1][i] = -INFINITY; ab[i] = 0.f; }

    const int n_plain = lo + SUB <= d.T ? min(n_sub, (d.T - SUB - lo) / SUB + 1) : 0;
    int u = 0;
    for (; u < n_plain; ++u) layer_body<false>(c, qa, ps, cm, acc, ab, u);
    for (; u < n_sub; ++u) layer_body<true>(c, qa, ps, cm, acc, ab, u);
    if (n_sub > 0) {                                           // tile 7 of the last subtile, then its hand-over
        columns_head<true, false>(acc[1], ab, c.c1, lo + (n_sub - 1) * SUB + c.n, c.hf, c.T, c.L);
        layer_give(c, n_sub - 1, ab);
        lds_barrier();
        layer_take(c, n_sub - 1, ab);
    }
}

// ------------------------------------------------------------------ other head / window shapes
// Any G with G * W <= 128 rows, W = 8, 16, 32 or 64: NT = ceil(G * W / 32) tiles of 32 rows, row = head * W +
// window query; the rows behind the problem's G * W are padding (W < 32 and G not a multiple of 32 / W): zero
// queries, never written by pass 1 and given an infinite log-sum-exp in pass 2, so they add exact zeros.  For
// W < 32 a tile holds several heads, so the head mean adds REGISTERS of one accumulator (register i of lane half
// hf is row 8 (i / 4) + 4 hf + i % 4 of the tile); for W >= 32 it adds accumulators, as in the kernels above.
// These kernels run the tiles of a subtile one after the other (no rotation of accumulators): with at most the
// arithmetic of the 128-row case per key and usually far less they wait for memory anyway.
template <int NT_, int W> struct Rows {
    static constexpr int NT = NT_;                          // tiles
    static constexpr int MP = 32 * NT;                      // rows of the tiles (padding included)
    static constexpr int QB = W >= 32 ? W / 32 : 1;         // 32-query blocks of the window
    static constexpr int NS = W >= 32 ? 16 * QB : W / 2;    // head-mean values per lane
    static_assert(NT >= 1 && NT <= 4 && (W == 8 || W == 16 || W == 32 || W == 64) && NT % QB == 0, "unsupported shape");
    __device__ static int tile_row(int i, int hf) { return 8 * (i >> 2) + 4 * hf + (i & 3); }
    __device__ static int query(int J, int i, int hf) { return W >= 32 ? 32 * (J % QB) + tile_row(i, hf) : tile_row(i, hf) % W; }
    __host__ __device__ static constexpr int slot(int J, int i) { return W >= 32 ? 16 * (J % QB) + i : i % (W / 2); }
    // window query that head-mean value `s` of lane half hf belongs to
    __device__ static int slot_query(int s, int hf) { return W >= 32 ? 32 * (s / 16) + tile_row(s % 16, hf) : tile_row(s, hf) % W; }
};

// a lane's A operands: row `r` of the problem's window-query matrix, zeros for a padding row
template <int KS>
__device__ __forceinline__ void load_query_row(bf16x8 (&qa)[KS], const ScoreArgs &a, int p, int r, int W, int hf)
{
    if (r < a.d.G * W) {
        const uint16_t *row = a.q + q_row_offset(a.d, p, r / W, r % W);
#pragma unroll
        for (int s = 0; s < KS; ++s) qa[s] = *reinterpret_cast<const bf16x8 *>(row + (2 * s + hf) * 8);
    } else {
#pragma unroll
        for (int s = 0; s < KS; ++s) qa[s] = bf16x8{};
    }
}

template <int NT, int W, int KS>
__global__ void __launch_bounds__(WAVES * 64)
score_mfma_stats_g(ScoreArgs a)
{
    using R = Rows<NT, W>;
    constexpr int MP = R::MP;
    extern __shared__ __attribute__((aligned(8192))) char lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 31, hf = lane >> 5;
    const Dims &d = a.d;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    char *ring = lds + wave_u * RING_BYTES;
    float *wg_red = reinterpret_cast<float *>(lds + WAVES * RING_BYTES);       // [WAVES][MP][2]
    float *cref = wg_red + WAVES * MP * 2 + wave_u * MP;                         // [NT tiles][2 halves][16], this wave's
    const WaveWork w = wave_work(a, wave);
    const int M = d.G * W;                                                     // rows of the problem; [M, MP) is padding

    typename StreamFor<KS>::type ks;
    ks.init(w.kp, d.ks[3], ring, w.first, w.n_sub, d.L, lane);
    ks.prime();

    bf16x8 qa[NT][KS];
#pragma unroll
    for (int J = 0; J < NT; ++J) load_query_row(qa[J], a, w.p, 32 * J + n, W, hf);   // row of the window-query matrix
#pragma unroll
    for (int J = 0; J < NT; ++J)
#pragma unroll
        for (int s = 0; s < KS; ++s) asm volatile("" : "+a"(qa[J][s]));
    for (int i = lane; i < MP; i += 64) cref[i] = 0.f;

    float z[NT][16];
#pragma unroll
    for (int J = 0; J < NT; ++J)
#pragma unroll
        for (int i = 0; i < 16; ++i) z[J][i] = 0.f;
    const float lim = RESCALE_AT / a.c1;
    for (int u = 0; u < w.n_sub; ++u) {
        bf16x8 kb[KS];
        ks.fetch(u, kb);
        const int t0 = w.first + u * STRIDE;
        const bool plain = u > 0 && t0 + SUB <= d.T;
#pragma unroll
        for (int J = 0; J < NT; ++J) {
            const floatx16 acc = chain<0, KS>(qa[J], kb, load_cref(cref, J, hf));
            if (plain && !stats_guard(acc, lim)) stats_add(acc, z[J], a.c1);
            else stats_tile_careful(acc, z[J], cref + 32 * J, a.c1, u == 0, t0 + n, hf, n,
                                    [J, hf](int i) { return R::query(J, i, hf); }, d.T, d.L);
        }
    }

    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    float *scr_z = reinterpret_cast<float *>(ring);            // [MP rows][32 lanes]
#pragma unroll
    for (int J = 0; J < NT; ++J)
#pragma unroll
        for (int i = 0; i < 16; ++i) scr_z[(J * 32 + R::tile_row(i, hf)) * 32 + n] = z[J][i];
    __builtin_amdgcn_wave_barrier();
    for (int row = lane; row < MP; row += 64) {                 // row = 32 * tile + row in tile
        float zz = 0.f;
        for (int j = 0; j < 32; ++j) zz += scr_z[row * 32 + ((j + lane) & 31)];
        const int q = row & 31, hfq = (q >> 2) & 1, iq = ((q >> 3) << 2) | (q & 3);
        wg_red[(wave * MP + row) * 2] = -cref[(row >> 5) * 32 + hfq * 16 + iq] * a.c1;   // reference, log2 domain
        wg_red[(wave * MP + row) * 2 + 1] = zz;
    }
    __syncthreads();
    if (threadIdx.x < M) {
        const int row = threadIdx.x;
        float m = -INFINITY;
        for (int wv = 0; wv < WAVES; ++wv) {
            const float *e = wg_red + (wv * MP + row) * 2;
            if (e[1] > 0.f) m = fmaxf(m, e[0]);
        }
        float zz = 0.f;
        for (int wv = 0; wv < WAVES; ++wv) {
            const float *e = wg_red + (wv * MP + row) * 2;
            if (e[1] > 0.f) zz += e[1] * __builtin_amdgcn_exp2f(e[0] - m);
        }
        float *o = a.partial + (((int64_t)w.p * a.n_chunks + w.chunk) * M + row) * 2;
        o[0] = m;
        o[1] = zz;
    }
}

// STORE: instead of the column sum and entropy of the KV head, write the head-group mean Abar[query][key] itself
// (for the mean over ALL heads of a layer, which is formed across KV heads afterwards), four consecutive window
// queries of a key per 16-byte store, layout [problem][W / 4][L][4].
template <int NT, int W, bool STORE, int KS>
__global__ void __launch_bounds__(WAVES * 64)
score_mfma_columns_g(ScoreArgs a)
{
    using R = Rows<NT, W>;
    constexpr int MP = R::MP, NS = R::NS;
    extern __shared__ __attribute__((aligned(8192))) char lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 31, hf = lane >> 5;
    const Dims &d = a.d;
    char *ring = lds + __builtin_amdgcn_readfirstlane(wave) * RING_BYTES;
    float *lse2 = reinterpret_cast<float *>(lds + WAVES * RING_BYTES);       // [MP] log2-domain lse + log2 G, row head * W + query; +inf for padding rows
    const WaveWork w = wave_work(a, wave);
    const int M = d.G * W;                                                   // rows of the problem; [M, MP) is padding

    typename StreamFor<KS>::type ks;
    ks.init(w.kp, d.ks[3], ring, w.first, w.n_sub, d.L, lane);
    ks.prime();

    if (threadIdx.x >= M && threadIdx.x < MP) lse2[threadIdx.x] = INFINITY;
    if (threadIdx.x < M) {
        const int r = threadIdx.x;
        float m = -INFINITY, zz = 0.f;
        if (a.lse) {
            m = a.lse[(int64_t)w.p * M + r] * LOG2E;
            zz = 1.f;
        } else {
            const float *pp = a.merged + ((int64_t)w.p * a.pc * M + r) * 2;
            for (int c = 0; c < a.pc; ++c) {
                const float2 e = *reinterpret_cast<const float2 *>(pp + (int64_t)c * M * 2);
                if (e.y > 0.f) {
                    const float mn = fmaxf(m, e.x);
                    zz = zz * __builtin_amdgcn_exp2f(m - mn) + e.y * __builtin_amdgcn_exp2f(e.x - mn);
                    m = mn;
                }
            }
        }
        lse2[r] = m + __builtin_amdgcn_logf(zz) + a.log2_G;
    }
    __syncthreads();

    bf16x8 qa[NT][KS];
    floatx16 cinit[NT];
    const float inv_c1 = 1.0f / a.c1;
#pragma unroll
    for (int J = 0; J < NT; ++J) {
        load_query_row(qa[J], a, w.p, 32 * J + n, W, hf);
#pragma unroll
        for (int i = 0; i < 16; ++i) cinit[J][i] = -lse2[32 * J + R::tile_row(i, hf)] * inv_c1;
    }
#pragma unroll
    for (int J = 0; J < NT; ++J)
#pragma unroll
        for (int s = 0; s < KS; ++s) asm volatile("" : "+a"(qa[J][s]));
    float *out = (hf == 0 ? a.s_out : a.e_out) + (int64_t)w.p * d.L;

    for (int u = 0; u < w.n_sub; ++u) {
        bf16x8 kb[KS];
        ks.fetch(u, kb);
        const int t0 = w.first + u * STRIDE, t = t0 + n;
        const bool edge = t0 + SUB > d.T;
        float ab[NS];
#pragma unroll
        for (int i = 0; i < NS; ++i) ab[i] = 0.f;
#pragma unroll
        for (int J = 0; J < NT; ++J) {
            const floatx16 acc = chain<0, KS>(qa[J], kb, cinit[J]);
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                float v = __builtin_amdgcn_exp2f(acc[i] * a.c1);                        // A / G
                if (edge && !(t < d.L && t <= d.T + R::query(J, i, hf))) v = 0.f;       // causal inside the window
                ab[R::slot(J, i)] += v;                                                 // Eq. barA
            }
        }
        if (STORE) {
            if (t < d.L) {
#pragma unroll
                for (int j = 0; j < NS / 4; ++j) {
                    const int qd = R::slot_query(4 * j, hf) >> 2;                        // slots 4j .. 4j+3: four consecutive queries
                    float4 *dst = reinterpret_cast<float4 *>(a.abar) + ((int64_t)w.p * (W / 4) + qd) * d.L + t;
                    *dst = make_float4(ab[4 * j], ab[4 * j + 1], ab[4 * j + 2], ab[4 * j + 3]);
                }
            }
            continue;
        }
        float s_part = 0.f;
#pragma unroll
        for (int i = 0; i < NS; ++i) s_part += ab[i];
        const float sv = add_other_half(s_part);                                         // Eq. st
        const float inv_s = sv > 0.f ? __builtin_amdgcn_rcpf(sv) : 0.f;
        float e_part = 0.f;
#pragma unroll
        for (int i = 0; i < NS; ++i) {
            const float ah = ab[i] * inv_s;
            e_part = fmaf(ah, __builtin_amdgcn_logf(ah + a.eps), e_part);
        }
        const float ent = -LN2 * add_other_half(e_part);                                 // inner sum of Eq. Dk
        if (t < d.L) out[t] = hf == 0 ? sv : ent;
    }
}

template <int NT> constexpr int stats_g_lds() { return 4 * 4 * BUF_BYTES + 4 * 32 * NT * 2 * 4 + 4 * 32 * NT * 4; }
template <int NT> constexpr int columns_g_lds() { return 4 * 4 * BUF_BYTES + 32 * NT * 4; }

// Folds the chunk partials of pass 1 into one (reference, sum) pair per row, one wavefront per row, so that
// with many chunks per problem the workgroups of pass 2 do not each repeat the fold.
// partial [blocks][n_chunks][M][2] -> merged [blocks][M][2]; grid ceil(blocks * M / 4), 256 threads
__global__ void __launch_bounds__(256)
merge_partials_kernel(const float *partial, float *merged, int n_chunks, int M, int n_rows)
{
    const int lane = threadIdx.x & 63;
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= n_rows) return;
    const int blk = r / M, row = r - blk * M;
    const float *pp = partial + ((int64_t)blk * n_chunks * M + row) * 2;
    float m = -INFINITY, z = 0.f;
    for (int c = lane; c < n_chunks; c += 64) {
        const float2 e = *reinterpret_cast<const float2 *>(pp + (int64_t)c * M * 2);
        if (e.y > 0.f) {
            const float mn = fmaxf(m, e.x);
            z = z * __builtin_amdgcn_exp2f(m - mn) + e.y * __builtin_amdgcn_exp2f(e.x - mn);
            m = mn;
        }
    }
    for (int off = 32; off > 0; off >>= 1) {
        const float m2 = __shfl_xor(m, off), z2 = __shfl_xor(z, off);
        const float mn = fmaxf(m, m2);
        z = (z > 0.f ? z * __builtin_amdgcn_exp2f(m - mn) : 0.f) + (z2 > 0.f ? z2 * __builtin_amdgcn_exp2f(m2 - mn) : 0.f);
        m = mn;
    }
    if (lane == 0) {
        merged[(int64_t)r * 2] = m;
        merged[(int64_t)r * 2 + 1] = z;
    }
}

// enqueues the fold when pass 2 is to read merged pairs (a.pc == 1 with more than one chunk)
void launch_merge(const ScoreArgs &a, int blocks, int M, hipStream_t st)
{
    if (a.merged == a.partial) return;
    const int n_rows = blocks * M;
    hipLaunchKernelGGL(merge_partials_kernel, dim3((unsigned)((n_rows + 3) / 4)), dim3(256), 0, st,
                       a.partial, const_cast<float *>(a.merged), a.n_chunks, M, n_rows);
}

template <int NT, int W, bool STORE, int KS = 8>
hipError_t launch_score_g(const ScoreArgs &a, dim3 grid, bool with_stats, hipStream_t st)
{
    static thread_local PerDeviceOnce attr_once;
    if (attr_once.needed()) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(score_mfma_stats_g<NT, W, KS>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, stats_g_lds<NT>());
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(score_mfma_columns_g<NT, W, STORE, KS>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, columns_g_lds<NT>());
        if (e != hipSuccess) return e;
        attr_once.done();
    }
    constexpr int lds1 = stats_g_lds<NT>(), lds2 = columns_g_lds<NT>();
    if (with_stats) {
        hipLaunchKernelGGL((score_mfma_stats_g<NT, W, KS>), grid, dim3(WAVES * 64), lds1, st, a);
        launch_merge(a, a.d.P, a.d.G * W, st);
    }
    hipLaunchKernelGGL((score_mfma_columns_g<NT, W, STORE, KS>), grid, dim3(WAVES * 64), lds2, st, a);
    return hipGetLastError();
}

// Mean over the KV heads of a layer of the head-group means, then column sum and entropy term (Eqs. barA with
// all H heads, st, inner sum of Dk): one thread per key.  grid (ceil(L / 256), n_seq * n_layers)
template <int W>
__global__ void __launch_bounds__(256)
abar_reduce_kernel(const float *abar, int Hkv, int L, float eps, float *s_out, float *e_out)
{
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= L) return;
    const int sl = blockIdx.y;
    float ab[W];
#pragma unroll
    for (int i = 0; i < W; ++i) ab[i] = 0.f;
    for (int kv = 0; kv < Hkv; ++kv) {
        const float4 *src = reinterpret_cast<const float4 *>(abar) + ((int64_t)(sl * Hkv + kv) * (W / 4)) * L + t;
#pragma unroll
        for (int j = 0; j < W / 4; ++j) {
            const float4 v = src[(int64_t)j * L];
            ab[4 * j] += v.x; ab[4 * j + 1] += v.y; ab[4 * j + 2] += v.z; ab[4 * j + 3] += v.w;
        }
    }
    const float inv_h = 1.0f / (float)Hkv;
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < W; ++i) { ab[i] *= inv_h; s += ab[i]; }
    const float inv_s = s > 0.f ? 1.0f / s : 0.f;
    float e = 0.f;
#pragma unroll
    for (int i = 0; i < W; ++i) {
        const float ah = ab[i] * inv_s;
        e = fmaf(ah, __builtin_amdgcn_logf(ah + eps), e);
    }
    s_out[(int64_t)sl * L + t] = s;
    e_out[(int64_t)sl * L + t] = -LN2 * e;
}

// the (G, W) pairs served by the generic-row kernels
// (tiles, window) pairs of the any-row-shape kernels: tiles = ceil(G * W / 32) <= 4.  Four tiles of a 32-query
// window are G = 4, which has kernels of its own at D = 128, so that pair is listed apart.
#define SABLOCK_TILE_SHAPES(X) X(1, 8) X(2, 8) X(3, 8) X(4, 8) X(1, 16) X(2, 16) X(3, 16) X(4, 16) X(1, 32) X(2, 32) X(3, 32)
#define SABLOCK_TILE_SHAPES_W64(X) X(2, 64) X(4, 64)

bool tile_shape(const Dims &d)
{
    return (d.W == 8 || d.W == 16 || d.W == 32 || d.W == 64) && d.G >= 1 && d.G * d.W <= M_ROWS;
}
int tiles_of(const Dims &d) { return (d.G * d.W + 31) / 32; }
// 129 .. 256 rows of a window of 32 or 64 queries (G = 5 .. 8 / G = 3, 4): the eight-tile column kernels
bool wide_shape(const Dims &d)
{
    return (d.W == 32 || d.W == 64) && d.G * d.W > M_ROWS && d.G * d.W <= 2 * M_ROWS;
}

struct Plan {
    int chunk_len;    // keys per workgroup
    int n_chunks;     // workgroups per problem
    bool merge;       // fold the chunk partials in a kernel of its own between the passes
};

constexpr int MERGE_FROM = 8;       // chunks per problem from which the separate fold pays

Plan make_plan(const Dims &d)
{
    // One launch per pass covers every problem.  A workgroup owns chunk_len consecutive keys of one problem, and
    // one workgroup fills a CU (registers and the load ring).  Each round of workgroups costs a prologue and an
    // epilogue during which its CU loads nothing (measured: about 17 us per round and pass), so the plan aims at
    // a whole number of rounds, as few as keep a chunk at or under MAX_CHUNK keys.
    constexpr int MAX_CHUNK = 131072;
    Plan pl;
    int len;
    if (d.tune.score_chunk >= STRIDE) len = (d.tune.score_chunk / STRIDE) * STRIDE;
    else {
        const int64_t cus = d.cus;
        const int64_t rounds = ((int64_t)d.P * d.L + cus * MAX_CHUNK - 1) / (cus * MAX_CHUNK);
        const int64_t per_problem = std::max<int64_t>(1, (cus * rounds + d.P / 2) / d.P);     // chunks per problem
        len = (int)(((d.L + per_problem - 1) / per_problem + STRIDE - 1) / STRIDE) * STRIDE;
        len = std::min(std::max(len, STRIDE), MAX_CHUNK);
    }
    pl.chunk_len = len;
    pl.n_chunks = (d.L + len - 1) / len;
    pl.merge = pl.n_chunks >= MERGE_FROM;
    return pl;
}

// bytes of the chunk partials, and of their merged form behind them
// (more than 128 rows: two blocks of 128 rows, the second padded where G * W < 256)
int stat_rows(const Dims &d) { return d.G * d.W > M_ROWS ? 2 * M_ROWS : d.G * d.W; }
size_t partial_bytes(const Dims &d, const Plan &pl) { return align256((size_t)d.P * pl.n_chunks * stat_rows(d) * 2 * 4); }
size_t merged_bytes(const Dims &d) { return align256((size_t)d.P * stat_rows(d) * 2 * 4); }

// pass-1 bookkeeping of both entry points: where the partials go and what pass 2 reads
void plan_partials(ScoreArgs &a, const Dims &d, const Plan &pl, void *ws)
{
    a.chunk_len = pl.chunk_len;
    a.n_chunks = pl.n_chunks;
    a.partial = static_cast<float *>(ws);
    a.merged = a.partial;
    a.pc = pl.n_chunks;
    if (pl.merge) {
        a.merged = reinterpret_cast<float *>(static_cast<char *>(ws) + partial_bytes(d, pl));
        a.pc = 1;
    }
}

}  // namespace

bool score_mfma_supported(const Dims &d)
{
    if (d.dtype != SABLOCK_BF16) return false;
    if (d.D == 64 || d.D == 96) return tile_shape(d);                       // up to 128 rows, kernels for any row shape
    if (d.D == 256) return tile_shape(d) && tiles_of(d) <= 3;               // up to 96 rows: four tiles of 16 k-steps do not fit the registers
    return d.D == 128 && (tile_shape(d) || wide_shape(d));
}

// pass 1 for 256 rows by the transposed-score kernel (csrc/window_attn.hip): K is read once instead of once per
// block of 128 rows
static bool stats_by_rows(const Dims &d)
{
    if (!row_stats_supported(d) || d.tune.stats_per_key == 1) return false;
    return d.tune.stats_per_key == 2 || d.G * d.W > M_ROWS;
}
static size_t row_stats_bytes(const Dims &d) { return align256((size_t)d.P * 2 * row_stats_chunks(d) * M_ROWS * 2 * 4); }

size_t score_mfma_ws_bytes(const Dims &d)
{
    const Plan pl = make_plan(d);
    size_t part = partial_bytes(d, pl);
    if (stats_by_rows(d)) part = std::max(part, row_stats_bytes(d));
    return part + merged_bytes(d);
}

hipError_t launch_score_mfma(const Dims &d, const void *q, const void *k, const float *row_lse, float eps,
                             float *s_out, float *ent_out, void *ws, hipStream_t st)
{
    static thread_local PerDeviceOnce attr_once;
    if (attr_once.needed()) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(score_mfma_stats),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, P1_LDS);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(score_mfma_columns),
                                hipFuncAttributeMaxDynamicSharedMemorySize, P2_LDS);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(score_mfma_columns8t<64>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, P2W_LDS);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(score_mfma_columns8t<32>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, P2W_LDS);
        if (e != hipSuccess) return e;
        attr_once.done();
    }
    const Plan pl = make_plan(d);
    ScoreArgs a;
    a.d = d;
    a.q = static_cast<const uint16_t *>(q);
    a.k = static_cast<const uint16_t *>(k);
    plan_partials(a, d, pl, ws);
    a.c1 = (float)(1.4426950408889634 / sqrt((double)d.D));
    a.log2_G = (float)log2((double)d.G);
    a.eps = eps;
    a.s_out = s_out;
    a.e_out = ent_out;
    a.lse = row_lse;
    a.abar = nullptr;
    a.p0 = 0;
    a.nv = d.G * d.W > M_ROWS ? 2 : 1;
    dim3 grid((unsigned)((int64_t)d.P * pl.n_chunks));
    if (tile_shape(d)) {
        const int nt = tiles_of(d);
        if (d.D == 256) {
#define X(NTV, WV) if (nt == NTV && d.W == WV) return launch_score_g<NTV, WV, false, 16>(a, grid, !row_lse, st);
            X(1, 8) X(2, 8) X(3, 8) X(1, 16) X(2, 16) X(3, 16) X(1, 32) X(2, 32) X(3, 32) X(2, 64)
#undef X
        }
        if (d.D == 96) {
#define X(NTV, WV) if (nt == NTV && d.W == WV) return launch_score_g<NTV, WV, false, 6>(a, grid, !row_lse, st);
            SABLOCK_TILE_SHAPES(X)
            X(4, 32)
            SABLOCK_TILE_SHAPES_W64(X)
#undef X
        }
        if (d.D == 64) {
#define X(NTV, WV) if (nt == NTV && d.W == WV) return launch_score_g<NTV, WV, false, 4>(a, grid, !row_lse, st);
            SABLOCK_TILE_SHAPES(X)
            X(4, 32)
            SABLOCK_TILE_SHAPES_W64(X)
#undef X
        }
#define X(NTV, WV) if (nt == NTV && d.W == WV) return launch_score_g<NTV, WV, false>(a, grid, !row_lse, st);
        SABLOCK_TILE_SHAPES(X)
        SABLOCK_TILE_SHAPES_W64(X)
#undef X
    }
    dim3 grid1((unsigned)((int64_t)d.P * a.nv * pl.n_chunks));
    if (!row_lse && stats_by_rows(d)) {
        // a lane per window query: one read of K serves all 256 rows; the chunks of this pass are its own
        const int nc1 = row_stats_chunks(d);
        hipError_t e = launch_row_stats(d, q, k, a.partial, st);
        if (e != hipSuccess) return e;
        a.merged = a.partial;
        a.pc = nc1;
        if (nc1 >= MERGE_FROM) {
            float *merged = reinterpret_cast<float *>(static_cast<char *>(ws) + row_stats_bytes(d));
            const int n_rows = d.P * a.nv * M_ROWS;
            hipLaunchKernelGGL(merge_partials_kernel, dim3((unsigned)((n_rows + 3) / 4)), dim3(256), 0, st, a.partial, merged,
                               nc1, M_ROWS, n_rows);
            a.merged = merged;
            a.pc = 1;
        }
    } else if (!row_lse) {
        hipLaunchKernelGGL(score_mfma_stats, grid1, dim3(WAVES * 64), P1_LDS, st, a);
        launch_merge(a, d.P * a.nv, M_ROWS, st);
    }
    if (d.W == 64) hipLaunchKernelGGL(score_mfma_columns8t<64>, grid, dim3(WAVES * 64), P2W_LDS, st, a);
    else if (d.G > 4) hipLaunchKernelGGL(score_mfma_columns8t<32>, grid, dim3(WAVES * 64), P2W_LDS, st, a);
    else hipLaunchKernelGGL(score_mfma_columns, grid, dim3(WAVES * 64), P2_LDS, st, a);
    return hipGetLastError();
}

namespace {

// ---- measurement aid: the scoring kernels' key stream without their arithmetic
// Same chunk plan, same workgroups, same direct-to-LDS ring and waits as score_mfma_columns; per subtile a
// wavefront either only waits for the subtile and refills its buffer (READ_LDS = false), or also reads the whole
// subtile from LDS into registers as the scoring kernels do (READ_LDS = true).  With STORES it also writes what the
// column pass writes, 4 bytes per key into each of two [P][L] rows, with that kernel's store pattern (lanes 0..31 a
// row of s_out, lanes 32..63 a row of e_out, once per subtile).  What this kernel takes is what the memory system
// delivers to the scoring kernels' access pattern: the yardstick their times are compared with.
template <bool READ_LDS, bool STORES>
__global__ void __launch_bounds__(WAVES * 64)
stream_probe_kernel(ScoreArgs a, uint32_t *sink)
{
    extern __shared__ __attribute__((aligned(8192))) char lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    char *ring = lds + __builtin_amdgcn_readfirstlane(wave) * RING_BYTES;
    const WaveWork w = wave_work(a, wave);
    KeyStream<NBUF> ks;
    ks.init(w.kp, a.d.ks[3], ring, w.first, w.n_sub, a.d.L, lane);
    ks.prime();
    uint32_t x = 0;
    for (int u = 0; u < w.n_sub; ++u) {
        if (READ_LDS) {
            bf16x8 kb[8];
            ks.fetch_vgpr(u, kb);
#pragma unroll
            for (int s = 0; s < 8; ++s) x ^= ((const uint32_t *)&kb[s])[0] ^ ((const uint32_t *)&kb[s])[3];
        } else {
            wait_loads(min(NBUF - 1, w.n_sub - 1 - u));
            x ^= *reinterpret_cast<const volatile uint32_t *>(ring + (u % NBUF) * BUF_BYTES + lane * 4);
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            if (u + NBUF < w.n_sub) ks.issue(u + NBUF);
        }
        if (STORES) {
            const int t = w.first + u * STRIDE + (lane & 31);
            float *out = ((lane >> 5) == 0 ? a.s_out : a.e_out) + (int64_t)w.p * a.d.L;
            if (t < a.d.L) out[t] = __uint_as_float(x & 0x3fffffffu);
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (x == 0x5ab10c4bu) *sink = x;                           // keeps the reads alive; practically never taken
}

}  // namespace

bool stream_probe_supported(const Dims &d) { return d.dtype == SABLOCK_BF16 && d.D == 128; }

hipError_t launch_stream_probe(const Dims &d, const void *k, int read_lds, float *s_out, float *e_out, void *sink, hipStream_t st)
{
    static thread_local PerDeviceOnce attr_once;
    if (attr_once.needed()) {
#define X(R, S) { hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(stream_probe_kernel<R, S>), \
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, P2_LDS); \
                  if (e != hipSuccess) return e; }
        X(false, false) X(false, true) X(true, false) X(true, true)
#undef X
        attr_once.done();
    }
    const Plan pl = make_plan(d);
    ScoreArgs a = {};
    a.d = d;
    a.k = static_cast<const uint16_t *>(k);
    a.chunk_len = pl.chunk_len;
    a.n_chunks = pl.n_chunks;
    a.p0 = 0;
    a.s_out = s_out;
    a.e_out = e_out;
    dim3 grid((unsigned)((int64_t)d.P * pl.n_chunks));
    uint32_t *sk = static_cast<uint32_t *>(sink);
    const bool stores = s_out != nullptr;
#define X(R, S) if ((read_lds != 0) == R && stores == S) hipLaunchKernelGGL((stream_probe_kernel<R, S>), grid, dim3(WAVES * 64), P2_LDS, st, a, sk);
    X(false, false) X(false, true) X(true, false) X(true, true)
#undef X
    return hipGetLastError();
}

// ---- head mean over all query heads of a layer (Eq. barA, literal): shapes with up to 128 window-query rows
bool score_all_heads_supported(const Dims &d)
{
    return d.dtype == SABLOCK_BF16 && d.D == 128 && tile_shape(d) && d.W <= 32;
}

// the shape whose layers one workgroup can sum in registers and LDS (score_mfma_columns_layer)
static bool layer_kernel_shape(const Dims &d) { return d.G == 4 && d.W == 32 && d.Hkv == LAYER_KV; }

size_t score_all_heads_ws_bytes(const Dims &d)
{
    const Plan pl = make_plan(d);
    const size_t abar = layer_kernel_shape(d) ? 0 : align256((size_t)d.P * d.L * d.W * 4);
    return partial_bytes(d, pl) + merged_bytes(d) + abar;
}

hipError_t launch_score_all_heads(const Dims &d, const void *q, const void *k, const float *row_lse, float eps,
                                  float *s_out, float *ent_out, void *ws, hipStream_t st)
{
    const Plan pl = make_plan(d);
    ScoreArgs a;
    a.d = d;
    a.q = static_cast<const uint16_t *>(q);
    a.k = static_cast<const uint16_t *>(k);
    plan_partials(a, d, pl, ws);
    a.nv = 1;
    a.c1 = (float)(1.4426950408889634 / sqrt((double)d.D));
    a.log2_G = (float)log2((double)d.G);
    a.eps = eps;
    a.lse = row_lse;
    a.p0 = 0;
    a.abar = nullptr;
    dim3 grid((unsigned)((int64_t)d.P * pl.n_chunks));
    if (layer_kernel_shape(d)) {
        static thread_local PerDeviceOnce attr_once;
        if (attr_once.needed()) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(score_mfma_stats),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, P1_LDS);
            if (e != hipSuccess) return e;
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(score_mfma_columns_layer),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, PL_LDS);
            if (e != hipSuccess) return e;
            attr_once.done();
        }
        a.s_out = s_out;
        a.e_out = ent_out;
        if (!row_lse) {
            hipLaunchKernelGGL(score_mfma_stats, grid, dim3(WAVES * 64), P1_LDS, st, a);
            launch_merge(a, d.P, M_ROWS, st);
        }
        // pass 2 has its own decomposition: a workgroup walks a chunk of keys through all 8 KV heads of a layer,
        // again in whole rounds of one workgroup per CU
        constexpr int MAX_LAYER_CHUNK = 32768;
        const int64_t n_sl = (int64_t)d.n_seq * d.n_layers, cus = d.cus;
        const int64_t rounds = (n_sl * d.L + cus * MAX_LAYER_CHUNK - 1) / (cus * MAX_LAYER_CHUNK);
        const int64_t per_layer = std::max<int64_t>(1, (cus * rounds + n_sl / 2) / n_sl);
        int len = (int)(((d.L + per_layer - 1) / per_layer + SUB - 1) / SUB) * SUB;
        len = std::min(std::max(len, SUB), MAX_LAYER_CHUNK);
        ScoreArgs a2 = a;
        a2.chunk_len = len;
        a2.n_chunks = (d.L + len - 1) / len;
        hipLaunchKernelGGL(score_mfma_columns_layer, dim3((unsigned)(n_sl * a2.n_chunks)), dim3(WAVES * 64), PL_LDS, st, a2);
        return hipGetLastError();
    }
    // other shapes: every KV head's head-group means go to memory, a second kernel averages them over the KV heads
    a.s_out = nullptr;
    a.e_out = nullptr;
    a.abar = reinterpret_cast<float *>(static_cast<char *>(ws) + partial_bytes(d, pl) + merged_bytes(d));
    hipError_t e = hipErrorInvalidValue;
    const int nt = tiles_of(d);
#define X(NTV, WV) if (nt == NTV && d.W == WV) e = launch_score_g<NTV, WV, true>(a, grid, !row_lse, st);
    SABLOCK_TILE_SHAPES(X)
    X(4, 32)
#undef X
    if (e != hipSuccess) return e;
    dim3 rgrid((unsigned)((d.L + 255) / 256), (unsigned)(d.n_seq * d.n_layers));
#define X(WV) if (d.W == WV) hipLaunchKernelGGL(abar_reduce_kernel<WV>, rgrid, dim3(256), 0, st, a.abar, d.Hkv, d.L, eps, s_out, ent_out);
    X(8) X(16) X(32)
#undef X
    return hipGetLastError();
}

}  // namespace sablock
