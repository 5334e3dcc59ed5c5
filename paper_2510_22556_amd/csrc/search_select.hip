// Budget-driven block-size search and selection (Alg. 2; Eqs. topk,
// implicit_budget, rk, gk_star, final_selection).
//
// topb_kernel     one workgroup per problem: radix select of the min(B,T)-th best
//                 score (12 bits over the row, then 10 + 10 on an LDS candidate
//                 list), ties resolved by ascending index.
//                 Result: (ordered key v, index cut c); token t is in T_topB iff
//                 key(t) > v or (key(t) == v and t <= c).  Its last phase counts
//                 the Top-B tokens of every segment: the implicit budgets b_k.
// heavy_list_kernel one workgroup per problem: segments with b_k >= 2 are appended to
//                 ONE list for the whole call (only they need a search; b_k == 1
//                 means g_k* = 1, b_k == 0 means g_k* = 0).
// search_kernel   wavefronts stride over that list: Score_base of a segment, then
//                 the candidates largest first.
// seg_prefix_kernel one workgroup per problem: prefix sum of b_k (output offsets); the
//                 segments that retain anything are appended to one of two lists for
//                 the call: token-level ones (g_k* = 1) and the others.
// select_light_kernel sixteen lanes per token-level segment: its Top-B tokens in order.
// select_kernel   wavefronts stride over the other list: T_k(g_k*) written in
//                 ascending order at the segment's offset.
// A list entry carries everything its consumer needs (problem, segment bounds, budget,
// block size, output offset), so a consumer starts with one 32-byte load; the lists
// are filled through one atomic counter per call, their order does not matter.
//
// All quantities that decide an integer (block sums Phi, Score_k(g), Score_base,
// tau * Score_base) are fp64 and summed in ascending token order, one addition at
// a time, so that they are identical for identical fp32 inputs regardless of how
// the work is spread over lanes.  Rankings use (value descending, index ascending).
#include "sablock_internal.h"

#include <algorithm>
#include <cstdlib>

namespace sablock {
namespace {

// one unit of work of search_kernel / select_kernel
struct __attribute__((aligned(32))) SegRec {
    int32_t p, k;        // problem, segment
    int32_t a, b;        // token range of the segment
    int32_t bk;          // implicit budget b_k
    int32_t g;           // select: block size g_k*;  search: ordered key of the Top-B threshold
    int32_t pos;         // select: offset of the segment's tokens in the problem's idx_out row;  search: index cut
    int32_t out;         // search that also selects: offset of the segment's tokens in the problem's idx_out row
};

// LDS slices of a search/select wavefront: tokens whose scores are staged, blocks whose Phi / class are kept.
// Two sizes: the small one keeps many wavefronts resident for the bulk of the segments; segments longer than
// CAPT go to a second list that is served by the same kernels with the large slices.
constexpr int CAPT = 512, CAPB = 256;
constexpr int CAPT_LONG = 4096, CAPB_LONG = 2048;
constexpr int MAX_G = 64;           // largest candidate block size

// Wavefront reductions without LDS round trips: four DPP steps inside each row of 16 lanes (lane ^ 1, lane ^ 2,
// mirror inside 8, mirror inside 16: together they pair every lane with every other lane of its row), then the
// four row results are read as scalars.  The results are wave-uniform.
template <int CTRL>
__device__ inline int dpp_i(int v) { return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xf, 0xf, false); }
constexpr int DPP_XOR1 = 0xB1, DPP_XOR2 = 0x4E, DPP_HALF_MIRROR = 0x141, DPP_MIRROR = 0x140;

__device__ inline int wave_sum_i(int v)
{
    v += dpp_i<DPP_XOR1>(v);
    v += dpp_i<DPP_XOR2>(v);
    v += dpp_i<DPP_HALF_MIRROR>(v);
    v += dpp_i<DPP_MIRROR>(v);
    return __builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) + __builtin_amdgcn_readlane(v, 32) +
           __builtin_amdgcn_readlane(v, 48);
}
__device__ inline int wave_max_i(int v)
{
    v = max(v, dpp_i<DPP_XOR1>(v));
    v = max(v, dpp_i<DPP_XOR2>(v));
    v = max(v, dpp_i<DPP_HALF_MIRROR>(v));
    v = max(v, dpp_i<DPP_MIRROR>(v));
    return max(max(__builtin_amdgcn_readlane(v, 0), __builtin_amdgcn_readlane(v, 16)),
               max(__builtin_amdgcn_readlane(v, 32), __builtin_amdgcn_readlane(v, 48)));
}
// best (value descending, index ascending) of the lanes' (value, index) pairs
__device__ inline bool pair_better(double op, int om, double bp, int bm) { return op > bp || (op == bp && om < bm); }
template <int CTRL>
__device__ inline void argmax_step(double &bp, int &bm)
{
    const int olo = dpp_i<CTRL>(__double2loint(bp)), ohi = dpp_i<CTRL>(__double2hiint(bp)), om = dpp_i<CTRL>(bm);
    const double op = __hiloint2double(ohi, olo);
    if (pair_better(op, om, bp, bm)) { bp = op; bm = om; }
}
__device__ inline void wave_argmax(double &bp, int &bm)
{
    argmax_step<DPP_XOR1>(bp, bm);
    argmax_step<DPP_XOR2>(bp, bm);
    argmax_step<DPP_HALF_MIRROR>(bp, bm);
    argmax_step<DPP_MIRROR>(bp, bm);
    const int lo = __double2loint(bp), hi = __double2hiint(bp);
    double rp = __hiloint2double(__builtin_amdgcn_readlane(hi, 0), __builtin_amdgcn_readlane(lo, 0));
    int rm = __builtin_amdgcn_readlane(bm, 0);
#pragma unroll
    for (int r = 16; r < 64; r += 16) {
        const double op = __hiloint2double(__builtin_amdgcn_readlane(hi, r), __builtin_amdgcn_readlane(lo, r));
        const int om = __builtin_amdgcn_readlane(bm, r);
        if (pair_better(op, om, rp, rm)) { rp = op; rm = om; }
    }
    bp = rp;
    bm = rm;
}

// acc += v[j] for every set bit j of mask, ascending; mask and acc are wave-uniform
__device__ inline double add_in_order(double acc, unsigned long long mask, float v)
{
    while (mask) {
        const int j = __builtin_ctzll(mask);                 // wave-uniform, so the value comes by v_readlane
        acc += (double)__int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), j));
        mask &= mask - 1;
    }
    return acc;
}

// ------------------------------------------------------------------ Top-B
constexpr int TB_THREADS = 1024;
constexpr int TB_OFFS = 4096;              // segment offsets and per-segment counts kept in LDS while the implicit budgets are counted:
constexpr int TB_OFFS_MAX = 16384;         // the launch picks 4 096, 8 192 or 16 384 entries (dynamic LDS: two int32 arrays of that size)
constexpr int TB_HITS = 4096;              // Top-B tokens collected in LDS before they are assigned to segments
constexpr int TB_HITS_MAX = 16384;         // ... when the launch gives the list dynamic LDS (8 192 or 16 384 entries)
constexpr int TB_CAND = 4096;              // tokens of the threshold's 12-bit bin that the LDS candidate list holds

__device__ inline bool in_topb(float v, int t, uint32_t thr_key, int thr_cut)
{
    const uint32_t key = ordered_key(v);
    return key > thr_key || (key == thr_key && t <= thr_cut);
}

// segment of token t: the k with seg_off[k] <= t < seg_off[k+1], 0 <= k < K
__device__ inline int segment_of(const int32_t *off, int K, int t)
{
    int lo = 0, hi = K;                       // invariant: off[lo] <= t < off[hi]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (off[mid] <= t) lo = mid; else hi = mid;
    }
    return lo;
}

// f(t, s_tilde[t]) for every token of a row, in no particular order: 16-byte loads, four in flight per thread
// (the passes over a row are latency-bound), scalar loads for the unaligned head and the tail
template <typename F>
__device__ inline void scan_row(const float *sp, int T, int tid, F &&f)
{
    const int head = min(T, (int)(((16u - (uint32_t)((uintptr_t)sp & 15u)) & 15u) >> 2));
    const int nvec = (T - head) >> 2;
    const float4 *vp = reinterpret_cast<const float4 *>(sp + head);
    for (int i0 = tid; i0 < nvec; i0 += 4 * TB_THREADS) {
        float4 v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) { const int i = i0 + j * TB_THREADS; v[j] = vp[i < nvec ? i : nvec - 1]; }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int i = i0 + j * TB_THREADS;
            if (i < nvec) {
                const int t = head + 4 * i;
                f(t, v[j].x); f(t + 1, v[j].y); f(t + 2, v[j].z); f(t + 3, v[j].w);
            }
        }
    }
    if (tid < head) f(tid, sp[tid]);
    const int t_tail = head + 4 * nvec + tid;
    if (t_tail < T) f(t_tail, sp[t_tail]);
}

// Bin of the k-th entry counted from the top bin of hist[0 .. nbins): wavefront 0 scans, everyone gets
// (bin, entries in the bins above it).  nbins is a multiple of 64.  Ends with a barrier.
__device__ inline void find_bin_from_top(const uint32_t *hist, int nbins, uint32_t krem, uint32_t *sh_pair,
                                         uint32_t &bin, uint32_t &above)
{
    const int lane = threadIdx.x & 63;
    if ((threadIdx.x >> 6) == 0) {
        // position r counts bins from the top: r = nbins-1-bin; lane owns `per` consecutive positions
        const int per = nbins / 64;
        uint32_t mine = 0;
        for (int j = 0; j < per; ++j) mine += hist[nbins - 1 - (lane * per + j)];
        uint32_t incl = mine;
        for (int off = 1; off < 64; off <<= 1) {
            uint32_t o = __shfl_up(incl, off);
            if (lane >= off) incl += o;
        }
        const uint32_t excl = incl - mine;
        if (excl < krem && krem <= incl) {
            uint32_t run = excl;
            for (int j = 0; j < per; ++j) {
                const int bn = nbins - 1 - (lane * per + j);
                const uint32_t c = hist[bn];
                if (run + c >= krem) { sh_pair[0] = (uint32_t)bn; sh_pair[1] = run; break; }
                run += c;
            }
        }
    }
    __syncthreads();
    bin = sh_pair[0];
    above = sh_pair[1];
}

// grid (P).  With seg_budget != NULL the kernel also clears the problem's seg_budget / block_size rows, counts
// the implicit budgets (Eq. implicit_budget) into seg_budget, and workgroup 0 clears counter[0..1].
//
// Selection of the k-th best score, k = min(B, T).  Usual path, two passes over the row: a histogram of the
// keys' top 12 bits locates the bin of the k-th key; the second pass puts the tokens of higher bins straight
// into the list of Top-B tokens and the tokens of that bin (key, index) into a candidate list in LDS, on which
// the remaining 20 bits are resolved without touching global memory again.  If the bin holds more candidates
// than the list (or k exceeds the token list), three histogram passes over the row (11 + 11 + 10 bits) do it.
// Ties at the threshold are cut by ascending index with one ordered pass over the row.
//
// PLAN (the search that also selects; the host launches it only when 0 < B < T, B <= hit_cap and every sequence
// has fewer than `offs_cap` segments, so the Top-B tokens and the segment counters are in LDS): the same workgroup
// goes on to the exclusive prefix of b_k (each segment's offset in the problem's idx_out row), writes n_sel, the
// single token of every segment with b_k == 1 (g_k* = 1) straight to its place, and appends the segments with
// b_k >= 2 to the call's search lists with their output offset.  `counter` must then be zero on entry.
struct PlanArgs {
    SegRec *list, *list_long;
    int capacity;
    int32_t *idx_out, *n_sel_out;
    // results of the sliced passes over the rows (null: the workgroup scans its row itself)
    const uint32_t *pre_hist;    // [P][4096] histogram of the keys' top 12 bits
    const int32_t *pre_cnt;      // [P][2] entries of pre_hit, pre_cand
    const int32_t *pre_hit;      // [P][TB_HITS] tokens of the bins above the threshold's bin
    const uint32_t *pre_cand;    // [P][TB_CAND][2] (key, token) of the threshold's bin
};

// ---- the two passes over the rows with several workgroups per row (few problems in a call: one workgroup per
// row leaves most of the chip idle and is bound by the latency of its own loads).  grid (slices, P).
__device__ inline void slice_of_row(int T, int n_slices, int sl, int &a, int &b)
{
    const int per = ((T + n_slices - 1) / n_slices + 3) & ~3;
    a = min(sl * per, T);
    b = min(a + per, T);
}

// pass A: histogram of the top 12 key bits of a slice, added to the row's histogram (zero on entry)
__global__ void __launch_bounds__(TB_THREADS)
topb_hist_kernel(Dims d, const float *s_tilde, uint32_t *g_hist)
{
    __shared__ uint32_t hist[4096];
    const int p = blockIdx.y, tid = threadIdx.x;
    int a, b;
    slice_of_row(d.T, gridDim.x, blockIdx.x, a, b);
    for (int i = tid; i < 4096; i += TB_THREADS) hist[i] = 0;
    __syncthreads();
    scan_row(s_tilde + (int64_t)p * d.T + a, b - a, tid, [&](int, float v) { atomicAdd(&hist[ordered_key(v) >> 20], 1u); });
    __syncthreads();
    for (int i = tid; i < 4096; i += TB_THREADS) {
        const uint32_t c = hist[i];
        if (c) atomicAdd(&g_hist[(int64_t)p * 4096 + i], c);
    }
}

// pass B: every workgroup finds the threshold's bin from the row's histogram, splits its slice into sure Top-B
// tokens and candidates in LDS, reserves room in the row's two lists with one atomic each and copies them there.
// Does nothing when the lists cannot hold the row's entries (the per-row kernel then makes its own passes).
__global__ void __launch_bounds__(TB_THREADS)
topb_split_kernel(Dims d, const float *s_tilde, int budget, const uint32_t *g_hist, int32_t *g_cnt, int32_t *g_hit,
                  uint32_t *g_cand)
{
    __shared__ uint32_t hist[4096];              // the row's histogram, then this slice's sure tokens
    __shared__ uint32_t lc_key[TB_CAND];
    __shared__ int32_t lc_idx[TB_CAND];
    __shared__ int sh_nhit, sh_ncand, sh_base[2];
    __shared__ uint32_t sh_pair[2];
    const int p = blockIdx.y, tid = threadIdx.x, T = d.T;
    const int k = min(budget, T);
    int a, b;
    slice_of_row(T, gridDim.x, blockIdx.x, a, b);
    for (int i = tid; i < 4096; i += TB_THREADS) hist[i] = g_hist[(int64_t)p * 4096 + i];
    if (tid == 0) { sh_nhit = 0; sh_ncand = 0; }
    __syncthreads();
    uint32_t bin, above;
    find_bin_from_top(hist, 4096, (uint32_t)k, sh_pair, bin, above);
    const uint32_t n_bin = hist[bin];
    __syncthreads();                             // hist is reused below
    if (!(n_bin <= (uint32_t)TB_CAND && k <= TB_HITS)) return;
    int32_t *lc_hit = reinterpret_cast<int32_t *>(hist);
    scan_row(s_tilde + (int64_t)p * T + a, b - a, tid, [&](int t, float v) {
        const uint32_t key = ordered_key(v);
        const uint32_t kb = key >> 20;
        if (kb > bin) lc_hit[atomicAdd(&sh_nhit, 1)] = a + t;
        else if (kb == bin) { const int c = atomicAdd(&sh_ncand, 1); lc_key[c] = key; lc_idx[c] = a + t; }
    });
    __syncthreads();
    if (tid == 0) sh_base[0] = sh_nhit > 0 ? atomicAdd(&g_cnt[2 * p], sh_nhit) : 0;
    if (tid == 64) sh_base[1] = sh_ncand > 0 ? atomicAdd(&g_cnt[2 * p + 1], sh_ncand) : 0;
    __syncthreads();
    for (int i = tid; i < sh_nhit; i += TB_THREADS) g_hit[(int64_t)p * TB_HITS + sh_base[0] + i] = lc_hit[i];
    for (int i = tid; i < sh_ncand; i += TB_THREADS) {
        uint32_t *dst = g_cand + ((int64_t)p * TB_CAND + sh_base[1] + i) * 2;
        dst[0] = lc_key[i];
        dst[1] = (uint32_t)lc_idx[i];
    }
}

template <bool PLAN>
__global__ void __launch_bounds__(TB_THREADS)
topb_kernel(Dims d, const float *s_tilde, int budget, int32_t *thr, SegView sv, int32_t *seg_budget,
            int32_t *block_size, int32_t *counter, PlanArgs pa, int offs_cap, int hit_cap, int hist_ways_log2)
{
    __shared__ uint32_t hist[TB_HITS];           // pass-A histogram (4096 bins), later the list of Top-B tokens (hit_cap == TB_HITS)
    __shared__ uint32_t hist2[2048];             // histograms of the later passes
    extern __shared__ int32_t sh_u[];            // [2][offs_cap]: candidates (key, index) during selection, then offsets and
                                                 // counters; behind them [hit_cap] Top-B tokens when hit_cap > TB_HITS
    __shared__ int sh_nhit, sh_ncand;
    __shared__ uint32_t sh_pair[2];
    __shared__ int sh_wcnt[TB_THREADS / 64];
    __shared__ int sh_cut;
    static_assert(TB_HITS == 4096 && TB_CAND <= TB_OFFS, "LDS regions are shared between phases");
    int32_t *sh_hit = hit_cap > TB_HITS ? sh_u + 2 * offs_cap : reinterpret_cast<int32_t *>(hist);
    uint32_t *cand_key = reinterpret_cast<uint32_t *>(sh_u);
    int32_t *cand_idx = sh_u + offs_cap;
    int32_t *sh_off = sh_u, *sh_cnt = sh_u + offs_cap;
    const int p = blockIdx.x, T = d.T;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float *sp = s_tilde + (int64_t)p * T;
    const int k = min(budget, T);
    const int64_t row = (int64_t)p * sv.max_segments;
    if (seg_budget) {
        for (int i = tid; i < sv.max_segments; i += TB_THREADS) { seg_budget[row + i] = 0; block_size[row + i] = 0; }
        if (!PLAN && counter && p == 0 && tid < 2) counter[tid] = 0;
    }

    uint32_t prefix = 0, mask = 0, krem = (uint32_t)max(k, 0), n_eq = 0;
    int cut = T - 1;
    bool have_hits = false;                    // sh_hit[0 .. k) holds T_topB
    if (k <= 0) {
        prefix = 0xFFFFFFFFu;                  // nothing is inside
        cut = -1;
    } else if (k < T) {
        // ---- pass A: top 12 bits
        const bool sliced = PLAN && pa.pre_hist;               // the passes over the row were made by sliced kernels
        if (sliced) {
            for (int i = tid; i < 4096; i += TB_THREADS) hist[i] = pa.pre_hist[(int64_t)p * 4096 + i];
        } else {
            if (hist_ways_log2 > 0) {
                // The scores of a row crowd into a few bins, and LDS atomics of one instruction on one address run one
                // after the other: threads are dealt out over 2 or 4 copies of the histogram (in the dynamic region,
                // which holds nothing yet), added up afterwards.
                uint32_t *hw = reinterpret_cast<uint32_t *>(sh_u);
                const int sh = hist_ways_log2, way = tid & ((1 << sh) - 1);
                for (int i = tid; i < (4096 << sh); i += TB_THREADS) hw[i] = 0;
                __syncthreads();
                scan_row(sp, T, tid, [&](int, float v) { atomicAdd(&hw[((ordered_key(v) >> 20) << sh) | way], 1u); });
                __syncthreads();
                for (int i = tid; i < 4096; i += TB_THREADS) {
                    uint32_t c = 0;
                    for (int w2 = 0; w2 < (1 << sh); ++w2) c += hw[(i << sh) | w2];
                    hist[i] = c;
                }
            } else {
                for (int i = tid; i < 4096; i += TB_THREADS) hist[i] = 0;
                __syncthreads();
                scan_row(sp, T, tid, [&](int, float v) { atomicAdd(&hist[ordered_key(v) >> 20], 1u); });
            }
        }
        __syncthreads();
        uint32_t bin, above;
        find_bin_from_top(hist, 4096, krem, sh_pair, bin, above);
        const uint32_t n_bin = hist[bin];
        __syncthreads();                       // hist is reused below
        // the candidate list is as long as the LDS arrays it sits in (the sliced passes stage theirs in TB_CAND entries)
        const uint32_t cand_cap = sliced ? (uint32_t)TB_CAND : (uint32_t)offs_cap;
        if (n_bin <= cand_cap && k <= hit_cap) {
            // ---- pass B: split the row into sure Top-B tokens and candidates
            if (sliced) {
                const int nh = pa.pre_cnt[2 * p], nc = pa.pre_cnt[2 * p + 1];
                for (int i = tid; i < nh; i += TB_THREADS) sh_hit[i] = pa.pre_hit[(int64_t)p * TB_HITS + i];
                for (int i = tid; i < nc; i += TB_THREADS) {
                    const uint32_t *src = pa.pre_cand + ((int64_t)p * TB_CAND + i) * 2;
                    cand_key[i] = src[0];
                    cand_idx[i] = (int32_t)src[1];
                }
                if (tid == 0) { sh_nhit = nh; sh_ncand = nc; }
            } else {
                if (tid == 0) { sh_nhit = 0; sh_ncand = 0; }
                __syncthreads();
                scan_row(sp, T, tid, [&](int t, float v) {
                    const uint32_t key = ordered_key(v);
                    const uint32_t kb = key >> 20;
                    if (kb > bin) sh_hit[atomicAdd(&sh_nhit, 1)] = t;
                    else if (kb == bin) { const int c = atomicAdd(&sh_ncand, 1); cand_key[c] = key; cand_idx[c] = t; }
                });
            }
            __syncthreads();
            const int ncand = sh_ncand;
            krem -= above;
            prefix = bin << 20;
            mask = 0xFFF00000u;
            // ---- the remaining 20 bits on the candidate list
            for (int shift = 10; shift >= 0; shift -= 10) {
                for (int i = tid; i < 1024; i += TB_THREADS) hist2[i] = 0;
                __syncthreads();
                for (int c = tid; c < ncand; c += TB_THREADS)
                    if ((cand_key[c] & mask) == prefix) atomicAdd(&hist2[(cand_key[c] >> shift) & 1023u], 1u);
                __syncthreads();
                uint32_t b2, a2;
                find_bin_from_top(hist2, 1024, krem, sh_pair, b2, a2);
                krem -= a2;
                n_eq = hist2[b2];
                prefix |= b2 << shift;
                mask |= 1023u << shift;
                __syncthreads();
            }
            have_hits = true;
        } else {
            // ---- three histogram passes over the row
            const int shifts[3] = {21, 10, 0};
            const int bits[3] = {11, 11, 10};
            for (int pass = 0; pass < 3; ++pass) {
                const int nbins = 1 << bits[pass], shift = shifts[pass];
                for (int i = tid; i < nbins; i += TB_THREADS) hist2[i] = 0;
                __syncthreads();
                scan_row(sp, T, tid, [&](int, float v) {
                    const uint32_t key = ordered_key(v);
                    if ((key & mask) == prefix) atomicAdd(&hist2[(key >> shift) & (nbins - 1)], 1u);
                });
                __syncthreads();
                uint32_t b2, a2;
                find_bin_from_top(hist2, nbins, krem, sh_pair, b2, a2);
                krem -= a2;
                n_eq = hist2[b2];
                prefix |= b2 << shift;
                mask |= (uint32_t)(nbins - 1) << shift;
                __syncthreads();
            }
        }
        // prefix is the key v of the k-th best score; krem of its n_eq ties are inside, lowest indices first
        if (krem < n_eq) {
            int seen = 0;
            for (int c0 = 0; c0 < T; c0 += TB_THREADS) {
                const int t = c0 + tid;
                const bool tie = t < T && ordered_key(sp[t]) == prefix;
                const unsigned long long bal = __ballot(tie);
                if (lane == 0) sh_wcnt[wave] = __popcll(bal);
                __syncthreads();
                int before = 0, total = 0;
                for (int w = 0; w < TB_THREADS / 64; ++w) { int c = sh_wcnt[w]; if (w < wave) before += c; total += c; }
                const bool found = seen + total >= (int)krem;
                if (found && tie && seen + before + __popcll(bal & ((1ull << lane) - 1ull)) + 1 == (int)krem) sh_cut = t;
                __syncthreads();
                if (found) { cut = sh_cut; break; }
                seen += total;
            }
        }
        if (have_hits) {
            // candidates at or above the threshold complete the list of Top-B tokens
            const int ncand = sh_ncand;
            for (int c = tid; c < ncand; c += TB_THREADS) {
                const uint32_t key = cand_key[c];
                const int t = cand_idx[c];
                if (key > prefix || (key == prefix && t <= cut)) sh_hit[atomicAdd(&sh_nhit, 1)] = t;
            }
            __syncthreads();                   // sh_nhit == k; the candidate region is free again
        }
    }   // k < T; for k >= T everything is inside: key 0 is below every score's key, cut = T - 1
    if (tid == 0) { thr[2 * p] = (int32_t)prefix; thr[2 * p + 1] = cut; }
    if (!seg_budget || k <= 0) return;

    // ---- implicit budgets: every Top-B token adds one to its segment (rows cleared above; the barrier below
    // orders the clearing stores of all wavefronts before the first atomic)
    __syncthreads();
    const int seq = seq_of_problem(d, p);
    const int32_t *off = sv.seg_off + sv.seq_ptr[seq];
    const int K = sv.seq_ptr[seq + 1] - sv.seq_ptr[seq] - 1;
    if (k >= T) {
        for (int j = tid; j < K; j += TB_THREADS) seg_budget[row + j] = off[j + 1] - off[j];
        return;
    }
    if (!have_hits && k <= hit_cap) {
        // collect T_topB with one more pass over the row
        if (tid == 0) sh_nhit = 0;
        __syncthreads();
        scan_row(sp, T, tid, [&](int t, float v) {
            if (in_topb(v, t, prefix, cut)) sh_hit[atomicAdd(&sh_nhit, 1)] = t;      // exactly k of them
        });
        __syncthreads();
        have_hits = true;
    }
    if (have_hits && K + 1 <= offs_cap) {
        // assign the listed tokens to segments in parallel: binary search on an LDS copy of the offsets, LDS counters
        for (int j = tid; j <= K; j += TB_THREADS) { sh_off[j] = off[j]; sh_cnt[j] = 0; }
        __syncthreads();
        for (int i = tid; i < sh_nhit; i += TB_THREADS) atomicAdd(&sh_cnt[segment_of(sh_off, K, sh_hit[i])], 1);
        __syncthreads();
        for (int j = tid; j < K; j += TB_THREADS) seg_budget[row + j] = sh_cnt[j];
        if (PLAN) {
            // exclusive prefix of the counters in place (K + 1 entries: b_k = pos[k + 1] - pos[k]); offs_cap / 1024
            // consecutive entries per thread, wavefront scan, then the sixteen wavefront totals
            __syncthreads();
            constexpr int PER_MAX = TB_OFFS_MAX / TB_THREADS;
            const int per = offs_cap / TB_THREADS;
            const int j0 = per * tid;
            int c[PER_MAX], tot = 0;
#pragma unroll
            for (int i = 0; i < PER_MAX; ++i) { c[i] = (i < per && j0 + i < K) ? sh_cnt[j0 + i] : 0; tot += c[i]; }
            int incl = tot;
            for (int o = 1; o < 64; o <<= 1) { const int x = __shfl_up(incl, o); if (lane >= o) incl += x; }
            if (lane == 63) sh_wcnt[wave] = incl;
            __syncthreads();
            int run = incl - tot;
            for (int w = 0; w < wave; ++w) run += sh_wcnt[w];
#pragma unroll
            for (int i = 0; i < PER_MAX; ++i) { if (i < per && j0 + i <= K) sh_cnt[j0 + i] = run; run += c[i]; }
            __syncthreads();
            int32_t *out = pa.idx_out + (int64_t)p * budget;
            if (tid == 0) pa.n_sel_out[p] = k;                 // k = B < T here, so there is nothing to pad
            // the token of every single-token segment goes straight to its place
            for (int i = tid; i < sh_nhit; i += TB_THREADS) {
                const int t = sh_hit[i], sg = segment_of(sh_off, K, t);
                if (sh_cnt[sg + 1] - sh_cnt[sg] == 1) { out[sh_cnt[sg]] = t; block_size[row + sg] = 1; }
            }
            // the others to the search lists (as in heavy_list_kernel), with their output offset
            const int32_t thr_key = (int32_t)prefix;
            for (int c0 = 0; c0 < K; c0 += TB_THREADS) {
                const int sg = c0 + tid;
                const int bk = sg < K ? sh_cnt[sg + 1] - sh_cnt[sg] : 0;
                const int a = sg < K ? sh_off[sg] : 0, b = sg < K ? sh_off[sg + 1] : 0;
                const bool hv = bk >= 2 && b - a <= CAPT, hx = bk >= 2 && b - a > CAPT;
                const unsigned long long bal = __ballot(hv), bax = __ballot(hx);
                __syncthreads();                               // the previous round's sh_pair reads are done
                if (lane == 0) { sh_wcnt[wave] = __popcll(bal) | (__popcll(bax) << 16); }
                __syncthreads();
                int before = 0, total = 0, before_x = 0, total_x = 0;
                for (int w = 0; w < TB_THREADS / 64; ++w) {
                    const int n0 = sh_wcnt[w] & 0xffff, n1 = sh_wcnt[w] >> 16;
                    if (w < wave) { before += n0; before_x += n1; }
                    total += n0; total_x += n1;
                }
                if (tid == 0 && total > 0) sh_pair[0] = (uint32_t)atomicAdd(&counter[0], total);
                if (tid == 1 && total_x > 0) sh_pair[1] = (uint32_t)atomicAdd(&counter[1], total_x);
                __syncthreads();
                if (hv || hx) {
                    const unsigned long long lt = (1ull << lane) - 1ull;
                    const int pos = hv ? (int)sh_pair[0] + before + __popcll(bal & lt) : (int)sh_pair[1] + before_x + __popcll(bax & lt);
                    if (pos < pa.capacity) {
                        SegRec r;
                        r.p = p; r.k = sg; r.a = a; r.b = b; r.bk = bk; r.g = thr_key; r.pos = cut; r.out = sh_cnt[sg];
                        (hv ? pa.list : pa.list_long)[pos] = r;
                    }
                }
            }
        }
    } else if (have_hits) {
        for (int i = tid; i < sh_nhit; i += TB_THREADS) atomicAdd(&seg_budget[row + segment_of(off, K, sh_hit[i])], 1);
    } else {
        scan_row(sp, T, tid, [&](int t, float v) {
            if (in_topb(v, t, prefix, cut)) atomicAdd(&seg_budget[row + segment_of(off, K, t)], 1);
        });
    }
}

// ------------------------------------------------------------------ one segment, one block size
struct WaveScratch {
    double *phi;        // block sums
    uint8_t *cls;       // block classes: 0 not taken, 1 taken whole, 2 cut to its best tokens
    int capb;           // blocks that fit
};

// Phi of block m of segment [a,b) with block size g: ascending fp64 sum.  `val(t)` yields s_tilde of token t
// (from the wave's LDS copy of the segment when it fits, else from global memory).
template <typename V>
__device__ inline double block_sum(V val, int a, int b, int g, int m)
{
    const int lo = a + m * g, hi = min(lo + g, b);
    double phi = 0.0;
    for (int t = lo; t < hi; ++t) phi += (double)val(t);
    return phi;
}

// number of blocks ranked before block m
template <typename V>
__device__ inline int block_rank(V val, int a, int b, int g, int nb, int m, double phi_m,
                                 const double *phi_lds, bool fast)
{
    int r = 0;
#pragma unroll 4
    for (int o = 0; o < nb; ++o) {
        double po = fast ? phi_lds[o] : block_sum(val, a, b, g, o);
        r += (po > phi_m || (po == phi_m && o < m)) ? 1 : 0;
    }
    return r;
}

// T_k(g) for segment [a,b) with implicit budget bk (Alg. 2's inner loop).  Calls
// emit(c0, taken_mask, value) for each 64-token chunk in ascending order; lane l
// of the chunk starting at token c0 holds the value of token c0 + l.
// Requires 1 <= g <= MAX_G, g <= min(b - a, bk); all arguments wave-uniform.
template <typename V, typename F>
__device__ inline void segment_fill(V val, int a, int b, int g, int bk, WaveScratch ws, F &&emit)
{
    const int lane = threadIdx.x & 63;
    const int len = b - a;
    const int nb = (len + g - 1) / g;
    const int ts = len - (nb - 1) * g;                 // size of the last block, 1..g
    const bool fast = nb <= ws.capb;
    const int mt = nb - 1;

    if (fast) {
        for (int m = lane; m < nb; m += 64) ws.phi[m] = block_sum(val, a, b, g, m);
        __builtin_amdgcn_wave_barrier();
    }
    // blocks taken whole: the first rstar in rank order; all blocks have g tokens except a short last one,
    // whose rank q decides how many blocks fit
    int rstar, nwhole;
    if (ts == g) {
        rstar = min(nb, bk / g);
        nwhole = rstar * g;
    } else {
        const double phi_t = fast ? ws.phi[mt] : block_sum(val, a, b, g, mt);
        int cnt = 0;
        for (int o = lane; o < mt; o += 64) {
            double po = fast ? ws.phi[o] : block_sum(val, a, b, g, o);
            cnt += (po >= phi_t) ? 1 : 0;                // o < mt: an equal sum ranks first
        }
        const int q = wave_sum_i(cnt);
        const int c = bk / g, r = bk - c * g;
        if (q < c) {
            if (ts <= r) { rstar = c + 1; nwhole = c * g + ts; } else { rstar = c; nwhole = c * g - g + ts; }
        } else if (q == c) {
            if (ts <= r) { rstar = c + 1; nwhole = c * g + ts; } else { rstar = c; nwhole = c * g; }
        } else {
            rstar = c; nwhole = c * g;
        }
        rstar = min(rstar, nb);
    }
    const int rem = bk - nwhole;                         // tokens to take from the block ranked rstar

    // classify blocks; remember the cut block
    int mp_local = -1;
    const int picks = rstar + (rem > 0 ? 1 : 0);           // blocks to single out when rstar < nb
    if (fast && rstar < nb && (picks <= 8 || picks * 512 <= nb * nb)) {
        // few blocks are taken: pick them one by one, best first (sum descending, index ascending), instead of
        // ranking every block against every other
        for (int m = lane; m < nb; m += 64) ws.cls[m] = 0;
        __builtin_amdgcn_wave_barrier();
        for (int sel = 0; sel < picks; ++sel) {
            double bp = -INFINITY;
            int bm = 0x7fffffff;
            for (int m = lane; m < nb; m += 64) {
                const double pm = ws.phi[m];
                if (ws.cls[m] == 0 && (pm > bp || (pm == bp && m < bm))) { bp = pm; bm = m; }
            }
            wave_argmax(bp, bm);
            if (lane == 0) ws.cls[bm] = sel < rstar ? 1 : 2;
            if (sel == rstar) mp_local = bm;
            __builtin_amdgcn_wave_barrier();
        }
    } else if (fast) {
        for (int m = lane; m < nb; m += 64) {
            int rk = (rstar >= nb) ? 0 : block_rank(val, a, b, g, nb, m, ws.phi[m], ws.phi, true);
            uint8_t c = (rk < rstar) ? 1 : ((rk == rstar && rem > 0) ? 2 : 0);
            ws.cls[m] = c;
            if (c == 2) mp_local = m;
        }
        __builtin_amdgcn_wave_barrier();
    } else if (rem > 0 && rstar < nb) {
        for (int m = lane; m < nb; m += 64) {
            int rk = block_rank(val, a, b, g, nb, m, block_sum(val, a, b, g, m), nullptr, false);
            if (rk == rstar) mp_local = m;
        }
    }
    const int mp = wave_max_i(mp_local);

    // inside the cut block: its best rem tokens
    unsigned long long pmask = 0;
    int plo = 0;
    if (mp >= 0) {
        plo = a + mp * g;
        const int phi_hi = min(plo + g, b);
        const int sz = phi_hi - plo;
        bool tk = false;
        if (lane < sz) {
            const float v = val(plo + lane);
            int rk = 0;
            for (int j = 0; j < sz; ++j) {
                float o = val(plo + j);
                rk += (o > v || (o == v && j < lane)) ? 1 : 0;
            }
            tk = rk < rem;
        }
        pmask = __ballot(tk);
    }

    for (int c0 = a; c0 < b; c0 += 64) {
        const int t = c0 + lane;
        const bool live = t < b;
        float v = 0.f;
        bool take = false;
        if (live) {
            v = val(t);
            const int m = (t - a) / g;
            int c;
            if (fast) {
                c = ws.cls[m];
            } else {
                int rk = (rstar >= nb) ? 0 : block_rank(val, a, b, g, nb, m, block_sum(val, a, b, g, m), nullptr, false);
                c = (rk < rstar) ? 1 : ((m == mp) ? 2 : 0);
            }
            take = (c == 1) || (c == 2 && ((pmask >> (t - plo)) & 1ull));
        }
        emit(c0, __ballot(take), v);
    }
    __builtin_amdgcn_wave_barrier();
}

// ------------------------------------------------------------------ search
// One workgroup per problem: g_k* = 1 where b_k == 1 (the rows are zero elsewhere), and the segments with
// b_k >= 2 are appended to the call's search list.
constexpr int LIST_THREADS = 1024;         // threads of the per-problem list-building kernels: segments handled per step

__global__ void __launch_bounds__(LIST_THREADS)
heavy_list_kernel(Dims d, SegView sv, const int32_t *thr, const int32_t *seg_budget, int32_t *block_size,
                  SegRec *list, SegRec *list_long, int32_t *counters, int capacity)
{
    __shared__ int sh_w[LIST_THREADS / 64], sh_x[LIST_THREADS / 64];
    __shared__ int sh_base[2];
    const int p = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int seq = seq_of_problem(d, p);
    const int32_t *off = sv.seg_off + sv.seq_ptr[seq];
    const int K = sv.seq_ptr[seq + 1] - sv.seq_ptr[seq] - 1;
    const int64_t row = (int64_t)p * sv.max_segments;
    const int32_t thr_key = thr[2 * p], thr_cut = thr[2 * p + 1];
    for (int c0 = 0; c0 < K; c0 += LIST_THREADS) {
        const int k = c0 + tid;
        const int bk = k < K ? seg_budget[row + k] : 0;
        if (k < K && bk == 1) block_size[row + k] = 1;
        const int a = k < K ? off[k] : 0, b = k < K ? off[k + 1] : 0;
        const bool hv = bk >= 2 && b - a <= CAPT, hx = bk >= 2 && b - a > CAPT;
        const unsigned long long bal = __ballot(hv), bax = __ballot(hx);
        if (lane == 0) { sh_w[wave] = __popcll(bal); sh_x[wave] = __popcll(bax); }
        __syncthreads();
        int before = 0, total = 0, before_x = 0, total_x = 0;
        for (int w = 0; w < LIST_THREADS / 64; ++w) {
            if (w < wave) { before += sh_w[w]; before_x += sh_x[w]; }
            total += sh_w[w]; total_x += sh_x[w];
        }
        if (tid == 0 && total > 0) sh_base[0] = atomicAdd(&counters[0], total);
        if (tid == 1 && total_x > 0) sh_base[1] = atomicAdd(&counters[1], total_x);
        __syncthreads();
        if (hv || hx) {
            const unsigned long long lt = (1ull << lane) - 1ull;
            const int pos = hv ? sh_base[0] + before + __popcll(bal & lt) : sh_base[1] + before_x + __popcll(bax & lt);
            if (pos < capacity) {
                SegRec r;
                r.p = p; r.k = k; r.a = a; r.b = b; r.bk = bk; r.g = thr_key; r.pos = thr_cut; r.out = 0;
                (hv ? list : list_long)[pos] = r;
            }
        }
    }
}

// one wavefront per workgroup, striding over the call's search list
constexpr int SEARCH_WGS = 65536;

// EMIT: the wavefront also writes T_k(g_k*) in ascending order at the segment's offset in idx_out (the record's
// `out`), so that no select pass over the segment is needed.
template <int CT, int CB, bool EMIT>
__global__ void __launch_bounds__(64)
search_kernel(Dims d, const float *s_tilde, SegView sv, CandList cand, float tau,
              const SegRec *list, const int32_t *counter, int capacity, int32_t *block_size, int budget, int32_t *idx_out)
{
    __shared__ double sh_phi[CB];
    __shared__ float sh_val[CT];
    __shared__ uint8_t sh_cls[CB];
    __shared__ unsigned long long sh_mask[EMIT ? CT / 64 : 1];   // the taken tokens of the candidate just tried
    const int lane = threadIdx.x;
    int j = blockIdx.x;                                     // < capacity: the grid is no larger than the list can get
    SegRec r = list[j];                                     // fetched together with the list length
    const int n_list = min(*counter, capacity);
    for (; j < n_list; j += gridDim.x, r = list[min(j, capacity - 1)]) {
    const int p = r.p, a = r.a, b = r.b, bk = r.bk;
    const int64_t o = (int64_t)p * sv.max_segments + r.k;
    const float *sp = s_tilde + (int64_t)p * d.T;
    const uint32_t thr_key = (uint32_t)r.g;
    const int thr_cut = r.pos;

    // token-level baseline Score_base = sum over T_topB & S_k, ascending; segments that fit are copied to LDS
    // on the way so that the candidate loop never goes back to global memory
    const bool staged = b - a <= CT;
    double base = 0.0;
    for (int c0 = a; c0 < b; c0 += 64) {
        const int t = c0 + lane;
        float v = 0.f;
        bool in = false;
        if (t < b) {
            v = sp[t];
            in = in_topb(v, t, thr_key, thr_cut);
            if (staged) sh_val[t - a] = v;
        }
        base = add_in_order(base, __ballot(in), v);
    }
    __builtin_amdgcn_wave_barrier();
    int gstar = 0;
    const int gcap = min(b - a, bk);                        // G_k: g <= min(|S_k|, b_k, g_max)
    const double need = (double)tau * base;                // R_k(g) >= tau  <=>  Score_k(g) >= tau * Score_base
    WaveScratch ws{sh_phi, sh_cls, CB};
    auto run = [&](auto val) {
        for (int c = cand.n - 1; c >= 0; --c) {
            const int g = cand.g[c];
            if (g > gcap) continue;
            if (g == 1) { gstar = 1; break; }               // token level: the unconditional last resort
            double score = 0.0;
            segment_fill(val, a, b, g, bk, ws, [&](int c0, unsigned long long m, float v) {
                score = add_in_order(score, m, v);
                if (EMIT && staged && lane == 0) sh_mask[(c0 - a) >> 6] = m;
            });
            if (score >= need) { gstar = g; break; }        // Eq. gk_star: first accepted, largest first
        }
    };
    float *lv = sh_val;
    if (staged) run([lv, a](int t) { return lv[t - a]; });
    else run([sp](int t) { return sp[t]; });
    if (lane == 0) block_size[o] = gstar;
    if (EMIT) {
        int32_t *out = idx_out + (int64_t)p * budget;
        int pos = r.out;
        const unsigned long long lt = (1ull << lane) - 1ull;
        auto put = [&](int c0, unsigned long long m, float) {
            const int jo = pos + __popcll(m & lt);
            if (((m >> lane) & 1ull) && jo < budget) out[jo] = c0 + lane;
            pos += __popcll(m);
        };
        if (gstar == 1) {                                   // T_k(1) = T_topB & S_k (b_k is the implicit budget)
            for (int c0 = a; c0 < b; c0 += 64) {
                const int t = c0 + lane;
                const float v = staged ? lv[min(t, b - 1) - a] : sp[min(t, b - 1)];
                put(c0, __ballot(t < b && in_topb(v, t, thr_key, thr_cut)), 0.f);
            }
        } else if (gstar > 1) {
            if (staged) {                                   // the accepted candidate was the last one tried
                __builtin_amdgcn_wave_barrier();
                for (int c0 = a; c0 < b; c0 += 64) put(c0, sh_mask[(c0 - a) >> 6], 0.f);
            } else {
                segment_fill([sp](int t) { return sp[t]; }, a, b, gstar, bk, ws, put);
            }
        }
    }
    __builtin_amdgcn_wave_barrier();                        // the LDS slices are reused by the next segment
    }
}

// ------------------------------------------------------------------ select
__global__ void reset_counters_kernel(int32_t *counters)
{
    if (threadIdx.x < 3) counters[threadIdx.x] = 0;
}

// counters of the call's lists, and the rows' histograms and list lengths of the sliced Top-B passes
__global__ void __launch_bounds__(256)
reset_sliced_kernel(int32_t *counters, uint32_t *words, int64_t n_words)
{
    if (blockIdx.x == 0 && threadIdx.x < 3) counters[threadIdx.x] = 0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n_words; i += (int64_t)gridDim.x * 256) words[i] = 0u;
}

// One workgroup per problem: exclusive prefix of b_k over its segments (where each segment's tokens go in the
// problem's idx_out row), n_sel, the -1 padding of idx_out.  The segments that retain anything are appended to
// one of the call's three select lists: token-level ones (g_k* = 1) to `light`, the others to `full` or, when
// longer than CAPT tokens, to `full_long`.  counters[0..2] are the lengths of light / full / full_long.
__global__ void __launch_bounds__(LIST_THREADS)
seg_prefix_kernel(Dims d, SegView sv, const int32_t *seg_budget, const int32_t *block_size, int budget,
                  SegRec *light, SegRec *full, SegRec *full_long, int32_t *counters, int capacity, int32_t *idx_out,
                  int32_t *n_sel_out)
{
    __shared__ int sh_w[LIST_THREADS / 64], sh_l[LIST_THREADS / 64], sh_f[LIST_THREADS / 64], sh_x[LIST_THREADS / 64];
    __shared__ int sh_base[3];
    const int p = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int seq = seq_of_problem(d, p);
    const int32_t *off = sv.seg_off + sv.seq_ptr[seq];
    const int K = sv.seq_ptr[seq + 1] - sv.seq_ptr[seq] - 1;
    const int64_t row = (int64_t)p * sv.max_segments;
    const unsigned long long lt = (1ull << lane) - 1ull;
    int carry = 0;
    for (int c0 = 0; c0 < K; c0 += LIST_THREADS) {
        const int k = c0 + tid;
        const int v = (k < K) ? seg_budget[row + k] : 0;
        const int g = (k < K) ? block_size[row + k] : 0;
        const int sa = k < K ? off[k] : 0, sb = k < K ? off[k + 1] : 0;
        const bool is_light = v > 0 && g == 1;
        const bool is_full = v > 0 && g > 1 && sb - sa <= CAPT, is_long = v > 0 && g > 1 && sb - sa > CAPT;
        const unsigned long long bl = __ballot(is_light), bf = __ballot(is_full), bx = __ballot(is_long);
        int incl = v;
        for (int o = 1; o < 64; o <<= 1) { int x = __shfl_up(incl, o); if (lane >= o) incl += x; }
        if (lane == 63) sh_w[wave] = incl;
        if (lane == 0) { sh_l[wave] = __popcll(bl); sh_f[wave] = __popcll(bf); sh_x[wave] = __popcll(bx); }
        __syncthreads();
        int before = 0, total = 0, before_l = 0, total_l = 0, before_f = 0, total_f = 0, before_x = 0, total_x = 0;
        for (int w = 0; w < LIST_THREADS / 64; ++w) {
            if (w < wave) { before += sh_w[w]; before_l += sh_l[w]; before_f += sh_f[w]; before_x += sh_x[w]; }
            total += sh_w[w]; total_l += sh_l[w]; total_f += sh_f[w]; total_x += sh_x[w];
        }
        if (tid == 0 && total_l > 0) sh_base[0] = atomicAdd(&counters[0], total_l);
        if (tid == 1 && total_f > 0) sh_base[1] = atomicAdd(&counters[1], total_f);
        if (tid == 2 && total_x > 0) sh_base[2] = atomicAdd(&counters[2], total_x);
        __syncthreads();
        if (is_light || is_full || is_long) {
            const int slot = is_light ? sh_base[0] + before_l + __popcll(bl & lt)
                           : is_full ? sh_base[1] + before_f + __popcll(bf & lt)
                                     : sh_base[2] + before_x + __popcll(bx & lt);
            if (slot < capacity) {
                SegRec r;
                r.p = p; r.k = k; r.a = sa; r.b = sb; r.bk = v; r.g = g; r.pos = carry + before + incl - v; r.out = 0;
                (is_light ? light : is_full ? full : full_long)[slot] = r;
            }
        }
        carry += total;
    }
    const int n = min(carry, budget);
    if (tid == 0) n_sel_out[p] = n;
    for (int j = n + tid; j < budget; j += LIST_THREADS) idx_out[(int64_t)p * budget + j] = -1;
}

// Token-level segments, sixteen lanes each (most retaining segments hold one or two Top-B tokens, so a wavefront
// per segment would mostly idle): T_k(1) = T_topB & S_k when b_k is the implicit budget, written in ascending
// order.  A segment whose b_k is something else (a caller's own budgets) is passed on to one of the full lists.
constexpr int LIGHT_GROUP = 16;

__global__ void __launch_bounds__(256)
select_light_kernel(Dims d, const float *s_tilde, const int32_t *thr, const SegRec *light, SegRec *full,
                    SegRec *full_long, int32_t *counters, int capacity, int budget, int32_t *idx_out)
{
    const int sub = threadIdx.x & (LIGHT_GROUP - 1);
    const int j = blockIdx.x * (256 / LIGHT_GROUP) + threadIdx.x / LIGHT_GROUP;       // < capacity rounded up
    const int n_list = min(counters[0], capacity);
    if (j >= n_list) return;
    const SegRec r = light[j];
    const int p = r.p, a = r.a, b = r.b;
    const int bk = min(r.bk, b - a);
    const float *sp = s_tilde + (int64_t)p * d.T;
    int32_t *out = idx_out + (int64_t)p * budget;
    const uint32_t thr_key = (uint32_t)thr[2 * p];
    const int thr_cut = thr[2 * p + 1];
    const int shift = (threadIdx.x & 63) & ~(LIGHT_GROUP - 1);                          // first lane of this group
    int cnt = 0;
    // groups of one wavefront may run different trip counts: ballots are taken over the lanes still in the loop
    for (int c0 = a; c0 < b; c0 += LIGHT_GROUP) {
        const int t = c0 + sub;
        const bool in = t < b && in_topb(sp[t < b ? t : a], t, thr_key, thr_cut);
        const uint32_t gm = (uint32_t)(__ballot(in) >> shift) & ((1u << LIGHT_GROUP) - 1u);
        const int slot = cnt + __popc(gm & ((1u << sub) - 1u));
        if (in && slot < bk && r.pos + slot < budget) out[r.pos + slot] = t;
        cnt += __popc(gm);
    }
    if (cnt != bk && sub == 0) {
        const bool lng = b - a > CAPT;
        const int slot = atomicAdd(&counters[lng ? 2 : 1], 1);
        if (slot < capacity) (lng ? full_long : full)[slot] = r;
    }
}

// T_k(g_k*) of one listed segment, written in ascending order from its offset in idx_out
template <int CT, int CB>
__device__ inline void select_segment(const Dims &d, const float *s_tilde, const int32_t *thr, const SegRec &r,
                                      int budget, int32_t *idx_out, double (&sh_phi)[CB], float (&sh_val)[CT],
                                      uint8_t (&sh_cls)[CB])
{
    const int lane = threadIdx.x & 63;
    const int p = r.p, a = r.a, b = r.b;
    const int bk = min(r.bk, b - a);
    int g = r.g;
    if (bk <= 0 || g <= 0) return;
    g = min(min(g, MAX_G), bk);
    const float *sp = s_tilde + (int64_t)p * d.T;
    int32_t *out = idx_out + (int64_t)p * budget;
    int pos = r.pos;
    const unsigned long long lt = (1ull << lane) - 1ull;
    auto put = [&](int c0, unsigned long long m, float) {
        const int j = pos + __popcll(m & lt);
        if (((m >> lane) & 1ull) && j < budget) out[j] = c0 + lane;
        pos += __popcll(m);
    };
    if (g == 1) {
        // T_k(1) = T_topB & S_k whenever b_k is the implicit budget; otherwise rank the tokens
        const uint32_t thr_key = (uint32_t)thr[2 * p];
        const int thr_cut = thr[2 * p + 1];
        if (b - a <= 64) {
            const int t = a + lane;
            const unsigned long long m = __ballot(t < b && in_topb(sp[t < b ? t : a], t, thr_key, thr_cut));
            if (__popcll(m) == bk) { put(a, m, 0.f); return; }
        } else {
            int cnt = 0;
            for (int c0 = a; c0 < b; c0 += 64) {
                const int t = c0 + lane;
                cnt += (t < b && in_topb(sp[t], t, thr_key, thr_cut)) ? 1 : 0;
            }
            if (wave_sum_i(cnt) == bk) {
                for (int c0 = a; c0 < b; c0 += 64) {
                    const int t = c0 + lane;
                    put(c0, __ballot(t < b && in_topb(sp[t], t, thr_key, thr_cut)), 0.f);
                }
                return;
            }
        }
    }
    WaveScratch ws{sh_phi, sh_cls, CB};
    if (b - a <= CT) {
        float *lv = sh_val;
        for (int t = a + lane; t < b; t += 64) lv[t - a] = sp[t];
        __builtin_amdgcn_wave_barrier();
        auto val = [lv, a](int t) { return lv[t - a]; };
        segment_fill(val, a, b, g, bk, ws, put);
    } else {
        auto val = [sp](int t) { return sp[t]; };
        segment_fill(val, a, b, g, bk, ws, put);
    }
}

// one wavefront per workgroup, striding over the call's select list
constexpr int SELECT_WGS = 32768;

template <int CT, int CB>
__global__ void __launch_bounds__(64)
select_kernel(Dims d, const float *s_tilde, const int32_t *thr, const SegRec *list, const int32_t *counter,
              int capacity, int budget, int32_t *idx_out)
{
    __shared__ double sh_phi[CB];
    __shared__ float sh_val[CT];
    __shared__ uint8_t sh_cls[CB];
    int j = blockIdx.x;                                     // < capacity: the grid is no larger than the list can get
    SegRec r = list[j];                                     // fetched together with the list length
    const int n_list = min(*counter, capacity);
    for (; j < n_list; j += gridDim.x, r = list[min(j, capacity - 1)]) {
        select_segment<CT, CB>(d, s_tilde, thr, r, budget, idx_out, sh_phi, sh_val, sh_cls);
        __builtin_amdgcn_wave_barrier();                    // the LDS slices are reused by the next segment
    }
}

}  // namespace

// dynamic LDS of topb_kernel, and what a launch may take next to the kernel's 25 KiB of static LDS
static size_t topb_lds(int offs_cap, int hit_cap)
{
    return ((size_t)2 * offs_cap + (hit_cap > TB_HITS ? hit_cap : 0)) * sizeof(int32_t);
}
constexpr size_t TOPB_LDS_MAX = 128 * 1024;
static int topb_offs_cap(const SegView &sv)
{
    return sv.max_segments + 1 <= TB_OFFS ? TB_OFFS : sv.max_segments + 1 <= 2 * TB_OFFS ? 2 * TB_OFFS : TB_OFFS_MAX;
}
static int topb_hit_cap(int32_t budget) { return budget <= TB_HITS ? TB_HITS : budget <= 2 * TB_HITS ? 2 * TB_HITS : TB_HITS_MAX; }
// copies of the pass-A histogram (log2): as many as the launch's dynamic LDS holds anyway, and four (64 KiB) when
// there is at most one workgroup per compute unit, so that the extra LDS costs no occupancy
static int topb_hist_ways_log2(const Dims &d, size_t lds_needed) { return d.P <= d.cus || lds_needed >= 65536 ? 2 : 1; }
static size_t topb_lds_with_hist(size_t lds_needed, int ways_log2) { return std::max(lds_needed, (size_t)16384 << ways_log2); }

hipError_t launch_topb(const Dims &d, const float *s_tilde, int32_t budget, int32_t *thr, hipStream_t st)
{
    if (d.P <= 0) return hipSuccess;
    SegView none{};
    hipLaunchKernelGGL(topb_kernel<false>, dim3(d.P), dim3(TB_THREADS), topb_lds(TB_OFFS, TB_HITS), st, d, s_tilde, budget, thr, none,
                       (int32_t *)nullptr, (int32_t *)nullptr, (int32_t *)nullptr, PlanArgs{}, TB_OFFS, TB_HITS, 1);
    return hipGetLastError();
}

// upper bound of the search list: a listed segment holds at least two of the |T_topB| tokens
static size_t max_heavy_segments(const Dims &d, int32_t max_segments, int32_t budget)
{
    const int k = budget < d.T ? budget : d.T;
    const int h = k / 2 < max_segments ? k / 2 : max_segments;
    return (size_t)d.P * (size_t)(h > 0 ? h : 0);
}

constexpr int LONG_WGS = 8192;             // workgroups of the kernels that serve the lists of long segments

size_t search_ws_bytes(const Dims &d, int32_t max_segments, int32_t budget)
{
    const size_t cap = max_heavy_segments(d, max_segments, budget);
    return align256((size_t)d.P * 2 * 4) + align256(8) + 2 * align256((cap > 0 ? cap : 1) * sizeof(SegRec));
}

hipError_t launch_search(const Dims &d, const float *s_tilde, const SegView &sv, const CandList &cand,
                         int32_t budget, float tau, int32_t *seg_budget, int32_t *block_size, int32_t *topb_out,
                         void *ws, hipStream_t st)
{
    if (d.P <= 0 || sv.max_segments <= 0) return hipSuccess;
    const size_t cap = max_heavy_segments(d, sv.max_segments, budget);
    char *w = static_cast<char *>(ws);
    int32_t *thr = topb_out ? topb_out : reinterpret_cast<int32_t *>(w);
    w += align256((size_t)d.P * 2 * 4);
    int32_t *counters = reinterpret_cast<int32_t *>(w);
    w += align256(8);
    SegRec *list = reinterpret_cast<SegRec *>(w);
    w += align256((cap > 0 ? cap : 1) * sizeof(SegRec));
    SegRec *list_long = reinterpret_cast<SegRec *>(w);
    hipLaunchKernelGGL(topb_kernel<false>, dim3(d.P), dim3(TB_THREADS), topb_lds(TB_OFFS, TB_HITS), st, d, s_tilde, budget, thr, sv,
                       seg_budget, block_size, counters, PlanArgs{}, TB_OFFS, TB_HITS, 1);
    if (budget > 0 && d.T > 0) {
        hipLaunchKernelGGL(heavy_list_kernel, dim3(d.P), dim3(LIST_THREADS), 0, st, d, sv, thr, seg_budget, block_size,
                           list, list_long, counters, (int)cap);
        if (cap > 0) {
            hipLaunchKernelGGL((search_kernel<CAPT, CAPB, false>), dim3((unsigned)(cap < SEARCH_WGS ? cap : SEARCH_WGS)), dim3(64),
                               0, st, d, s_tilde, sv, cand, tau, list, counters, (int)cap, block_size, 0, (int32_t *)nullptr);
            hipLaunchKernelGGL((search_kernel<CAPT_LONG, CAPB_LONG, false>), dim3((unsigned)(cap < LONG_WGS ? cap : LONG_WGS)),
                               dim3(64), 0, st, d, s_tilde, sv, cand, tau, list_long, counters + 1, (int)cap, block_size, 0,
                               (int32_t *)nullptr);
        }
    }
    return hipGetLastError();
}

// upper bound of the select lists: a listed segment retains at least one token of its problem's budget
static size_t max_active_segments(const Dims &d, int32_t max_segments, int32_t budget)
{
    const int a = budget < max_segments ? budget : max_segments;
    return (size_t)d.P * (size_t)(a > 0 ? a : 0);
}

size_t select_ws_bytes(const Dims &d, int32_t max_segments, int32_t budget)
{
    const size_t cap = max_active_segments(d, max_segments, budget);
    return align256((size_t)d.P * 2 * 4) + align256(12) + 3 * align256((cap > 0 ? cap : 1) * sizeof(SegRec));
}

hipError_t launch_select(const Dims &d, const float *s_tilde, const SegView &sv, const int32_t *seg_budget,
                         const int32_t *block_size, const int32_t *topb, int32_t budget, int32_t *idx_out,
                         int32_t *n_sel_out, void *ws, hipStream_t st)
{
    if (d.P <= 0) return hipSuccess;
    const size_t cap = max_active_segments(d, sv.max_segments, budget);
    const size_t list_bytes = align256((cap > 0 ? cap : 1) * sizeof(SegRec));
    char *w = static_cast<char *>(ws);
    int32_t *thr_ws = reinterpret_cast<int32_t *>(w);
    w += align256((size_t)d.P * 2 * 4);
    int32_t *counters = reinterpret_cast<int32_t *>(w);
    w += align256(12);
    SegRec *light = reinterpret_cast<SegRec *>(w);
    SegRec *full = reinterpret_cast<SegRec *>(w + list_bytes);
    SegRec *full_long = reinterpret_cast<SegRec *>(w + 2 * list_bytes);
    const int32_t *thr = topb;
    if (!thr) {
        hipError_t e = launch_topb(d, s_tilde, budget, thr_ws, st);
        if (e != hipSuccess) return e;
        thr = thr_ws;
    }
    hipLaunchKernelGGL(reset_counters_kernel, dim3(1), dim3(64), 0, st, counters);
    hipLaunchKernelGGL(seg_prefix_kernel, dim3(d.P), dim3(LIST_THREADS), 0, st, d, sv, seg_budget, block_size, budget,
                       light, full, full_long, counters, (int)cap, idx_out, n_sel_out);
    if (cap > 0) {
        const unsigned per_wg = 256 / LIGHT_GROUP;
        hipLaunchKernelGGL(select_light_kernel, dim3((unsigned)((cap + per_wg - 1) / per_wg)), dim3(256), 0, st, d,
                           s_tilde, thr, light, full, full_long, counters, (int)cap, budget, idx_out);
        hipLaunchKernelGGL((select_kernel<CAPT, CAPB>), dim3((unsigned)(cap < SELECT_WGS ? cap : SELECT_WGS)), dim3(64), 0,
                           st, d, s_tilde, thr, full, counters + 1, (int)cap, budget, idx_out);
        hipLaunchKernelGGL((select_kernel<CAPT_LONG, CAPB_LONG>), dim3((unsigned)(cap < LONG_WGS ? cap : LONG_WGS)), dim3(64),
                           0, st, d, s_tilde, thr, full_long, counters + 2, (int)cap, budget, idx_out);
    }
    return hipGetLastError();
}

// ---- search and select in one sequence (same results as launch_search followed by launch_select)
bool search_select_fused(const Dims &d, const SegView &sv, int32_t budget)
{
    if (!(budget > 0 && budget < d.T && budget <= TB_HITS_MAX && sv.max_segments + 1 <= TB_OFFS_MAX)) return false;
    return topb_lds(topb_offs_cap(sv), topb_hit_cap(budget)) <= TOPB_LDS_MAX;
}

// Workgroups per row for the two Top-B passes of the one-call form: with few problems in a call (a layer at a
// time) one workgroup per row would leave most of the chip idle.  1: the per-row kernel scans its row itself.
static int topb_slices(const Dims &d, int32_t budget)
{
    if (budget > TB_HITS) return 1;                            // the sliced passes stage at most TB_HITS tokens per row
    if (const int v = d.tune.topb_slices; v >= 1) return (int64_t)v * 4096 <= d.T ? v : 1;
    int s = (int)std::min<int64_t>(16, (int64_t)d.cus / std::max(d.P, 1));
    s = std::min(s, d.T / 8192);                               // a slice is worth a workgroup from 8 192 tokens on
    return s >= 2 ? s : 1;
}
static size_t sliced_words(const Dims &d) { return (size_t)d.P * (4096 + 2); }          // histograms, then list lengths
static size_t sliced_bytes(const Dims &d)
{
    return align256(sliced_words(d) * 4) + align256((size_t)d.P * TB_HITS * 4) + align256((size_t)d.P * TB_CAND * 8);
}

size_t search_select_ws_bytes(const Dims &d, int32_t max_segments, int32_t budget)
{
    const size_t a = search_ws_bytes(d, max_segments, budget), b = select_ws_bytes(d, max_segments, budget);
    return (a > b ? a : b) + (topb_slices(d, budget) > 1 ? sliced_bytes(d) : 0);
}

hipError_t launch_search_select(const Dims &d, const float *s_tilde, const SegView &sv, const CandList &cand,
                                int32_t budget, float tau, int32_t *seg_budget, int32_t *block_size, int32_t *topb_out,
                                int32_t *idx_out, int32_t *n_sel_out, void *ws, hipStream_t st)
{
    if (d.P <= 0) return hipSuccess;
    if (!search_select_fused(d, sv, budget)) {
        hipError_t e = launch_search(d, s_tilde, sv, cand, budget, tau, seg_budget, block_size, topb_out, ws, st);
        if (e != hipSuccess) return e;
        // the select lists reuse the workspace of the search lists, which are consumed by then; the Top-B state
        // sits in front of both layouts
        const int32_t *thr = topb_out ? topb_out : static_cast<const int32_t *>(ws);
        return launch_select(d, s_tilde, sv, seg_budget, block_size, thr, budget, idx_out, n_sel_out, ws, st);
    }
    const size_t cap = max_heavy_segments(d, sv.max_segments, budget);
    char *w = static_cast<char *>(ws);
    int32_t *thr = topb_out ? topb_out : reinterpret_cast<int32_t *>(w);
    w += align256((size_t)d.P * 2 * 4);
    int32_t *counters = reinterpret_cast<int32_t *>(w);
    w += align256(8);
    SegRec *list = reinterpret_cast<SegRec *>(w);
    w += align256((cap > 0 ? cap : 1) * sizeof(SegRec));
    SegRec *list_long = reinterpret_cast<SegRec *>(w);
    PlanArgs pa{list, list_long, (int)cap, idx_out, n_sel_out, nullptr, nullptr, nullptr, nullptr};
    const int n_slices = topb_slices(d, budget);
    if (n_slices > 1) {
        // behind the larger of the search and select layouts
        const size_t base = search_select_ws_bytes(d, sv.max_segments, budget) - sliced_bytes(d);
        char *x = static_cast<char *>(ws) + base;
        uint32_t *g_hist = reinterpret_cast<uint32_t *>(x);
        int32_t *g_cnt = reinterpret_cast<int32_t *>(g_hist + (size_t)d.P * 4096);
        x += align256(sliced_words(d) * 4);
        int32_t *g_hit = reinterpret_cast<int32_t *>(x);
        x += align256((size_t)d.P * TB_HITS * 4);
        uint32_t *g_cand = reinterpret_cast<uint32_t *>(x);
        const int64_t n_words = (int64_t)sliced_words(d);
        hipLaunchKernelGGL(reset_sliced_kernel, dim3((unsigned)std::min<int64_t>((n_words + 1023) / 1024, 1024)), dim3(256), 0, st,
                           counters, g_hist, n_words);
        hipLaunchKernelGGL(topb_hist_kernel, dim3(n_slices, d.P), dim3(TB_THREADS), 0, st, d, s_tilde, g_hist);
        hipLaunchKernelGGL(topb_split_kernel, dim3(n_slices, d.P), dim3(TB_THREADS), 0, st, d, s_tilde, budget, g_hist, g_cnt,
                           g_hit, g_cand);
        pa.pre_hist = g_hist;
        pa.pre_cnt = g_cnt;
        pa.pre_hit = g_hit;
        pa.pre_cand = g_cand;
    } else {
        hipLaunchKernelGGL(reset_counters_kernel, dim3(1), dim3(64), 0, st, counters);
    }
    // counters and offsets of all segments of a sequence, and the Top-B tokens of a row, in LDS
    const int offs_cap = topb_offs_cap(sv), hit_cap = topb_hit_cap(budget);
    const int ways_log2 = topb_hist_ways_log2(d, topb_lds(offs_cap, hit_cap));
    const size_t lds = topb_lds_with_hist(topb_lds(offs_cap, hit_cap), ways_log2);
    if (lds > topb_lds(TB_OFFS, TB_HITS)) {
        static thread_local PerDeviceOnce attr_once;
        if (attr_once.needed()) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(topb_kernel<true>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)TOPB_LDS_MAX);
            if (e != hipSuccess) return e;
            attr_once.done();
        }
    }
    hipLaunchKernelGGL(topb_kernel<true>, dim3(d.P), dim3(TB_THREADS), lds, st, d, s_tilde, budget, thr,
                       sv, seg_budget, block_size, counters, pa, offs_cap, hit_cap, ways_log2);
    if (cap > 0) {
        hipLaunchKernelGGL((search_kernel<CAPT, CAPB, true>), dim3((unsigned)(cap < SEARCH_WGS ? cap : SEARCH_WGS)), dim3(64),
                           0, st, d, s_tilde, sv, cand, tau, list, counters, (int)cap, block_size, budget, idx_out);
        hipLaunchKernelGGL((search_kernel<CAPT_LONG, CAPB_LONG, true>), dim3((unsigned)(cap < LONG_WGS ? cap : LONG_WGS)),
                           dim3(64), 0, st, d, s_tilde, sv, cand, tau, list_long, counters + 1, (int)cap, block_size, budget,
                           idx_out);
    }
    return hipGetLastError();
}

}  // namespace sablock
