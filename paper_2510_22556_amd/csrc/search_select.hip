// Budget-driven block-size search and selection (Alg. 2; Eqs. topk,
// implicit_budget, rk, gk_star, final_selection).
//
// topb_kernel     one workgroup per problem: LDS radix select (11+11+10 bits) of
//                 the min(B,T)-th best score, ties resolved by ascending index.
//                 Result: (ordered key v, index cut c); token t is in T_topB iff
//                 key(t) > v or (key(t) == v and t <= c).
// seg_count_kernel  one thread per token: every Top-B token adds 1 to its segment's b_k.
// heavy_list_kernel one workgroup per problem: segments with b_k >= 2 are listed (only
//                 they need a search; b_k == 1 means g_k* = 1, b_k == 0 means g_k* = 0).
// search_kernel   one wavefront per listed (problem, segment): Score_base, then the
//                 candidates largest first.
// seg_prefix_kernel one workgroup per problem: prefix sum of b_k (output offsets) and the
//                 list of segments that retain anything.
// select_kernel   one wavefront per listed (problem, segment): T_k(g_k*) written in
//                 ascending order at the segment's offset.
//
// All quantities that decide an integer (block sums Phi, Score_k(g), Score_base,
// tau * Score_base) are fp64 and summed in ascending token order, one addition at
// a time, so that they are identical for identical fp32 inputs regardless of how
// the work is spread over lanes.  Rankings use (value descending, index ascending).
#include "sablock_internal.h"

namespace sablock {
namespace {

constexpr int WAVES = 1;            // wavefronts (segments) per workgroup in search/select: a slow segment holds no others back
constexpr int CAPB = 512;           // blocks per segment whose Phi/class fit the wave's LDS slice
constexpr int CAPT = 1024;          // tokens per segment whose scores are staged in the wave's LDS slice
constexpr int MAX_G = 64;           // largest candidate block size

__device__ inline int wave_sum_i(int v)
{
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}
__device__ inline int wave_max_i(int v)
{
    for (int off = 32; off > 0; off >>= 1) v = max(v, __shfl_xor(v, off));
    return v;
}

// acc += v[j] for every set bit j of mask, ascending; mask and acc are wave-uniform
__device__ inline double add_in_order(double acc, unsigned long long mask, float v)
{
    while (mask) {
        int j = __builtin_ctzll(mask);
        acc += (double)__shfl(v, j);
        mask &= mask - 1;
    }
    return acc;
}

// ------------------------------------------------------------------ Top-B
constexpr int TB_THREADS = 1024;

__global__ void __launch_bounds__(TB_THREADS)
topb_kernel(Dims d, const float *s_tilde, int budget, int32_t *thr, int32_t *zero_a, int32_t *zero_b, int row_len)
{
    __shared__ uint32_t hist[2048];
    __shared__ uint32_t sh_bin, sh_above;
    __shared__ int sh_wcnt[TB_THREADS / 64];
    __shared__ int sh_cut;
    const int p = blockIdx.x, T = d.T;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float *sp = s_tilde + (int64_t)p * T;
    const int k = min(budget, T);
    if (zero_a) {            // the search counts into / writes these rows later in the stream
        for (int i = tid; i < row_len; i += TB_THREADS) { zero_a[(int64_t)p * row_len + i] = 0; zero_b[(int64_t)p * row_len + i] = 0; }
    }
    if (k <= 0) { if (tid == 0) { thr[2 * p] = (int32_t)0xFFFFFFFFu; thr[2 * p + 1] = -1; } return; }
    if (k >= T) { if (tid == 0) { thr[2 * p] = 0; thr[2 * p + 1] = T - 1; } return; }

    uint32_t prefix = 0, mask = 0, krem = (uint32_t)k, n_eq = 0;
    const int shifts[3] = {21, 10, 0};
    const int bits[3] = {11, 11, 10};
    for (int pass = 0; pass < 3; ++pass) {
        const int nbins = 1 << bits[pass], shift = shifts[pass];
        for (int i = tid; i < nbins; i += TB_THREADS) hist[i] = 0;
        __syncthreads();
        // eight independent loads in flight per thread: the pass is latency-bound otherwise
        for (int t0 = tid; t0 < T; t0 += 8 * TB_THREADS) {
            float v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) { const int t = t0 + j * TB_THREADS; v[j] = sp[t < T ? t : T - 1]; }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint32_t key = ordered_key(v[j]);
                if (t0 + j * TB_THREADS < T && (key & mask) == prefix) atomicAdd(&hist[(key >> shift) & (nbins - 1)], 1u);
            }
        }
        __syncthreads();
        if (wave == 0) {
            // position r counts bins from the top: r = nbins-1-bin; lane owns `per` consecutive positions
            const int per = nbins / 64;
            uint32_t mine = 0;
            for (int j = 0; j < per; ++j) mine += hist[nbins - 1 - (lane * per + j)];
            uint32_t incl = mine;
            for (int off = 1; off < 64; off <<= 1) {
                uint32_t o = __shfl_up(incl, off);
                if (lane >= off) incl += o;
            }
            uint32_t excl = incl - mine;
            if (excl < krem && krem <= incl) {
                uint32_t run = excl;
                for (int j = 0; j < per; ++j) {
                    int bin = nbins - 1 - (lane * per + j);
                    uint32_t c = hist[bin];
                    if (run + c >= krem) { sh_bin = (uint32_t)bin; sh_above = run; break; }
                    run += c;
                }
            }
        }
        __syncthreads();
        const uint32_t bin = sh_bin;
        krem -= sh_above;
        n_eq = hist[bin];
        prefix |= bin << shift;
        mask |= (uint32_t)(nbins - 1) << shift;
        __syncthreads();
    }
    // prefix is the key v of the k-th best score; krem of its n_eq ties are inside, lowest indices first
    int cut = T - 1;
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
    if (tid == 0) { thr[2 * p] = (int32_t)prefix; thr[2 * p + 1] = cut; }
}

// ------------------------------------------------------------------ one segment, one block size
struct WaveScratch {
    double *phi;        // CAPB block sums
    uint8_t *cls;       // CAPB block classes: 0 not taken, 1 taken whole, 2 cut to its best tokens
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
    const bool fast = nb <= CAPB;
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
    if (fast) {
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

__device__ inline bool in_topb(float v, int t, uint32_t thr_key, int thr_cut)
{
    const uint32_t key = ordered_key(v);
    return key > thr_key || (key == thr_key && t <= thr_cut);
}

// ------------------------------------------------------------------ search
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

// implicit budgets (Eq. implicit_budget): grid (ceil(T / (256 * 8)), P); seg_budget rows are zero on entry.
// A workgroup covers 2048 consecutive tokens; the segments they fall in form a short range that is located once
// per workgroup, so a Top-B token finds its segment in a few steps.
__global__ void __launch_bounds__(256)
seg_count_kernel(Dims d, const float *s_tilde, SegView sv, const int32_t *thr, int32_t *seg_budget)
{
    __shared__ int sh_range[2];
    const int p = blockIdx.y, T = d.T;
    const float *sp = s_tilde + (int64_t)p * T;
    const uint32_t thr_key = (uint32_t)thr[2 * p];
    const int thr_cut = thr[2 * p + 1];
    const int seq = seq_of_problem(d, p);
    const int32_t *off = sv.seg_off + sv.seq_ptr[seq];
    const int K = sv.seq_ptr[seq + 1] - sv.seq_ptr[seq] - 1;
    const int base_t = blockIdx.x * (256 * 8);
    if (threadIdx.x < 2) sh_range[threadIdx.x] = segment_of(off, K, threadIdx.x == 0 ? base_t : min(base_t + 256 * 8, T) - 1);
    const int t0 = base_t + threadIdx.x;
    float v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) { const int t = t0 + j * 256; v[j] = sp[t < T ? t : T - 1]; }
    __syncthreads();
    const int k_lo = sh_range[0], k_hi = sh_range[1] + 1;          // off[k_lo] <= t < off[k_hi] for every token here
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int t = t0 + j * 256;
        if (t < T && in_topb(v[j], t, thr_key, thr_cut))
            atomicAdd(&seg_budget[(int64_t)p * sv.max_segments + k_lo + segment_of(off + k_lo, k_hi - k_lo, t)], 1);
    }
}

// one workgroup per problem: ordered list of the segments with b_k >= 2, and g_k* = 1 where b_k == 1
__global__ void __launch_bounds__(256)
heavy_list_kernel(Dims d, SegView sv, const int32_t *seg_budget, int32_t *block_size, int32_t *heavy,
                  int32_t *n_heavy, int max_heavy)
{
    __shared__ int sh_w[4];
    const int p = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int seq = seq_of_problem(d, p);
    const int K = sv.seq_ptr[seq + 1] - sv.seq_ptr[seq] - 1;
    const int64_t row = (int64_t)p * sv.max_segments;
    int carry = 0;
    for (int c0 = 0; c0 < K; c0 += 256) {
        const int k = c0 + tid;
        const int bk = k < K ? seg_budget[row + k] : 0;
        if (k < K && bk == 1) block_size[row + k] = 1;
        const bool hv = bk >= 2;
        const unsigned long long bal = __ballot(hv);
        if (lane == 0) sh_w[wave] = __popcll(bal);
        __syncthreads();
        int before = 0, total = 0;
        for (int w = 0; w < 4; ++w) { if (w < wave) before += sh_w[w]; total += sh_w[w]; }
        const int pos = carry + before + __popcll(bal & ((1ull << lane) - 1ull));
        if (hv && pos < max_heavy) heavy[(int64_t)p * max_heavy + pos] = k;
        carry += total;
        __syncthreads();
    }
    if (tid == 0) n_heavy[p] = min(carry, max_heavy);
}

// grid (SEARCH_GRID, P), one wavefront each, striding over the problem's list of segments with b_k >= 2
constexpr int SEARCH_GRID = 1024;

__global__ void __launch_bounds__(64)
search_kernel(Dims d, const float *s_tilde, SegView sv, CandList cand, float tau, const int32_t *thr,
              const int32_t *heavy, const int32_t *n_heavy, int max_heavy, const int32_t *seg_budget,
              int32_t *block_size)
{
    __shared__ double sh_phi[CAPB];
    __shared__ float sh_val[CAPT];
    __shared__ uint8_t sh_cls[CAPB];
    const int p = blockIdx.y;
    const int lane = threadIdx.x;
    const int n_list = n_heavy[p];
    for (int j = blockIdx.x; j < n_list; j += gridDim.x) {
    const int k = heavy[(int64_t)p * max_heavy + j];
    const int seq = seq_of_problem(d, p);
    const int sbase = sv.seq_ptr[seq];
    const int64_t o = (int64_t)p * sv.max_segments + k;
    const int a = sv.seg_off[sbase + k], b = sv.seg_off[sbase + k + 1];
    const int bk = seg_budget[o];
    const float *sp = s_tilde + (int64_t)p * d.T;
    const uint32_t thr_key = (uint32_t)thr[2 * p];
    const int thr_cut = thr[2 * p + 1];

    // token-level baseline Score_base = sum over T_topB & S_k, ascending; segments that fit are copied to LDS
    // on the way so that the candidate loop never goes back to global memory
    const bool staged = b - a <= CAPT;
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
    WaveScratch ws{sh_phi, sh_cls};
    auto run = [&](auto val) {
        for (int c = cand.n - 1; c >= 0; --c) {
            const int g = cand.g[c];
            if (g > gcap) continue;
            if (g == 1) { gstar = 1; break; }               // token level: the unconditional last resort
            double score = 0.0;
            segment_fill(val, a, b, g, bk, ws,
                         [&](int, unsigned long long m, float v) { score = add_in_order(score, m, v); });
            if (score >= need) { gstar = g; break; }        // Eq. gk_star: first accepted, largest first
        }
    };
    float *lv = sh_val;
    if (staged) run([lv, a](int t) { return lv[t - a]; });
    else run([sp](int t) { return sp[t]; });
    if (lane == 0) block_size[o] = gstar;
    __builtin_amdgcn_wave_barrier();                        // the LDS slices are reused by the next segment
    }
}

// ------------------------------------------------------------------ select
// exclusive prefix of b_k over the segments of one problem, the ordered list of segments that retain anything,
// n_sel and the -1 padding of idx_out
__global__ void __launch_bounds__(256)
seg_prefix_kernel(Dims d, SegView sv, const int32_t *seg_budget, const int32_t *block_size, int budget, int32_t *prefix,
                  int32_t *act, int32_t *n_act, int max_act, int32_t *idx_out, int32_t *n_sel_out)
{
    __shared__ int sh_w[4], sh_a[4];
    int carry_a = 0;
    const int p = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int seq = seq_of_problem(d, p);
    const int K = sv.seq_ptr[seq + 1] - sv.seq_ptr[seq] - 1;
    const int32_t *bp = seg_budget + (int64_t)p * sv.max_segments;
    int32_t *pp = prefix + (int64_t)p * sv.max_segments;
    int carry = 0;
    for (int c0 = 0; c0 < K; c0 += 256) {
        const int k = c0 + tid;
        const int v = (k < K) ? bp[k] : 0;
        const bool active = v > 0 && block_size[(int64_t)p * sv.max_segments + (k < K ? k : 0)] > 0;
        const unsigned long long bal = __ballot(active);
        int incl = v;
        for (int off = 1; off < 64; off <<= 1) { int o = __shfl_up(incl, off); if (lane >= off) incl += o; }
        if (lane == 63) sh_w[wave] = incl;
        if (lane == 0) sh_a[wave] = __popcll(bal);
        __syncthreads();
        int before = 0, total = 0, before_a = 0, total_a = 0;
        for (int w = 0; w < 4; ++w) {
            if (w < wave) { before += sh_w[w]; before_a += sh_a[w]; }
            total += sh_w[w]; total_a += sh_a[w];
        }
        if (k < K) pp[k] = carry + before + incl - v;
        const int pa = carry_a + before_a + __popcll(bal & ((1ull << lane) - 1ull));
        if (active && pa < max_act) act[(int64_t)p * max_act + pa] = k;
        carry += total;
        carry_a += total_a;
        __syncthreads();
    }
    const int n = min(carry, budget);
    if (tid == 0) { n_sel_out[p] = n; n_act[p] = min(carry_a, max_act); }
    for (int j = n + tid; j < budget; j += 256) idx_out[(int64_t)p * budget + j] = -1;
}

// T_k(g_k*) of one segment, written in ascending order from its offset in idx_out
__device__ inline void select_segment(const Dims &d, const float *s_tilde, const SegView &sv, const int32_t *thr,
                                      const int32_t *seg_budget, const int32_t *block_size, const int32_t *prefix,
                                      int budget, int32_t *idx_out, int p, int k, double (&sh_phi)[WAVES][CAPB],
                                      float (&sh_val)[WAVES][CAPT], uint8_t (&sh_cls)[WAVES][CAPB])
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int seq = seq_of_problem(d, p);
    const int sbase = sv.seq_ptr[seq];
    const int64_t o = (int64_t)p * sv.max_segments + k;
    const int a = sv.seg_off[sbase + k], b = sv.seg_off[sbase + k + 1];
    const int bk = min(seg_budget[o], b - a);
    int g = block_size[o];
    if (bk <= 0 || g <= 0) return;
    g = min(min(g, MAX_G), bk);
    const float *sp = s_tilde + (int64_t)p * d.T;
    int32_t *out = idx_out + (int64_t)p * budget;
    int pos = prefix[o];
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
    WaveScratch ws{sh_phi[wave], sh_cls[wave]};
    if (b - a <= CAPT) {
        float *lv = sh_val[wave];
        for (int t = a + lane; t < b; t += 64) lv[t - a] = sp[t];
        __builtin_amdgcn_wave_barrier();
        auto val = [lv, a](int t) { return lv[t - a]; };
        segment_fill(val, a, b, g, bk, ws, put);
    } else {
        auto val = [sp](int t) { return sp[t]; };
        segment_fill(val, a, b, g, bk, ws, put);
    }
}

// grid (SELECT_GRID, P), one wavefront each, striding over the problem's list of segments that retain anything
constexpr int SELECT_GRID = 2048;

__global__ void __launch_bounds__(WAVES * 64)
select_kernel(Dims d, const float *s_tilde, SegView sv, const int32_t *thr, const int32_t *seg_budget,
              const int32_t *block_size, const int32_t *prefix, const int32_t *act, const int32_t *n_act, int max_act,
              int budget, int32_t *idx_out)
{
    __shared__ double sh_phi[WAVES][CAPB];
    __shared__ float sh_val[WAVES][CAPT];
    __shared__ uint8_t sh_cls[WAVES][CAPB];
    const int p = blockIdx.y;
    const int n_list = n_act[p];
    for (int j = blockIdx.x; j < n_list; j += gridDim.x) {
        select_segment(d, s_tilde, sv, thr, seg_budget, block_size, prefix, budget, idx_out, p,
                       act[(int64_t)p * max_act + j], sh_phi, sh_val, sh_cls);
        __builtin_amdgcn_wave_barrier();                    // the LDS slices are reused by the next segment
    }
}

}  // namespace

hipError_t launch_topb(const Dims &d, const float *s_tilde, int32_t budget, int32_t *thr, hipStream_t st)
{
    if (d.P <= 0) return hipSuccess;
    hipLaunchKernelGGL(topb_kernel, dim3(d.P), dim3(TB_THREADS), 0, st, d, s_tilde, budget, thr,
                       (int32_t *)nullptr, (int32_t *)nullptr, 0);
    return hipGetLastError();
}

static int max_heavy_segments(const Dims &d, int32_t max_segments, int32_t budget)
{
    const int k = budget < d.T ? budget : d.T;             // |T_topB|; a listed segment holds at least two of them
    const int h = k / 2 < max_segments ? k / 2 : max_segments;
    return h > 0 ? h : 0;
}

size_t search_ws_bytes(const Dims &d, int32_t max_segments, int32_t budget)
{
    const int mh = max_heavy_segments(d, max_segments, budget);
    return align256((size_t)d.P * 2 * 4) + align256((size_t)d.P * (size_t)(mh > 0 ? mh : 1) * 4) + align256((size_t)d.P * 4);
}

hipError_t launch_search(const Dims &d, const float *s_tilde, const SegView &sv, const CandList &cand,
                         int32_t budget, float tau, int32_t *seg_budget, int32_t *block_size, int32_t *topb_out,
                         void *ws, hipStream_t st)
{
    if (d.P <= 0 || sv.max_segments <= 0) return hipSuccess;
    const int mh = max_heavy_segments(d, sv.max_segments, budget);
    char *w = static_cast<char *>(ws);
    int32_t *thr = topb_out ? topb_out : reinterpret_cast<int32_t *>(w);
    int32_t *heavy = reinterpret_cast<int32_t *>(w + align256((size_t)d.P * 2 * 4));
    int32_t *n_heavy = reinterpret_cast<int32_t *>(w + align256((size_t)d.P * 2 * 4) + align256((size_t)d.P * (size_t)(mh > 0 ? mh : 1) * 4));
    hipLaunchKernelGGL(topb_kernel, dim3(d.P), dim3(TB_THREADS), 0, st, d, s_tilde, budget, thr, seg_budget,
                       block_size, sv.max_segments);
    if (budget > 0 && d.T > 0) {
        dim3 gc((d.T + 256 * 8 - 1) / (256 * 8), d.P);
        hipLaunchKernelGGL(seg_count_kernel, gc, dim3(256), 0, st, d, s_tilde, sv, thr, seg_budget);
        hipLaunchKernelGGL(heavy_list_kernel, dim3(d.P), dim3(256), 0, st, d, sv, seg_budget, block_size, heavy,
                           n_heavy, mh);
        if (mh > 0)
            hipLaunchKernelGGL(search_kernel, dim3(mh < SEARCH_GRID ? mh : SEARCH_GRID, d.P), dim3(64), 0, st, d, s_tilde, sv, cand, tau, thr, heavy,
                               n_heavy, mh, seg_budget, block_size);
    }
    return hipGetLastError();
}

static int max_active_segments(int32_t max_segments, int32_t budget)
{
    const int a = budget < max_segments ? budget : max_segments;   // a listed segment retains at least one token
    return a > 0 ? a : 1;
}

size_t select_ws_bytes(const Dims &d, int32_t max_segments, int32_t budget)
{
    const size_t ms = (size_t)(max_segments > 0 ? max_segments : 1);
    return align256((size_t)d.P * 2 * 4) + align256((size_t)d.P * ms * 4) +
           align256((size_t)d.P * (size_t)max_active_segments(max_segments, budget) * 4) + align256((size_t)d.P * 4);
}

hipError_t launch_select(const Dims &d, const float *s_tilde, const SegView &sv, const int32_t *seg_budget,
                         const int32_t *block_size, const int32_t *topb, int32_t budget, int32_t *idx_out,
                         int32_t *n_sel_out, void *ws, hipStream_t st)
{
    if (d.P <= 0) return hipSuccess;
    const size_t ms = (size_t)(sv.max_segments > 0 ? sv.max_segments : 1);
    const int ma = max_active_segments(sv.max_segments, budget);
    char *w = static_cast<char *>(ws);
    int32_t *thr_ws = reinterpret_cast<int32_t *>(w);
    w += align256((size_t)d.P * 2 * 4);
    int32_t *prefix = reinterpret_cast<int32_t *>(w);
    w += align256((size_t)d.P * ms * 4);
    int32_t *act = reinterpret_cast<int32_t *>(w);
    w += align256((size_t)d.P * (size_t)ma * 4);
    int32_t *n_act = reinterpret_cast<int32_t *>(w);
    const int32_t *thr = topb;
    if (!thr) {
        hipError_t e = launch_topb(d, s_tilde, budget, thr_ws, st);
        if (e != hipSuccess) return e;
        thr = thr_ws;
    }
    hipLaunchKernelGGL(seg_prefix_kernel, dim3(d.P), dim3(256), 0, st, d, sv, seg_budget, block_size, budget, prefix,
                       act, n_act, ma, idx_out, n_sel_out);
    if (sv.max_segments > 0 && budget > 0) {
        dim3 grid(ma < SELECT_GRID ? ma : SELECT_GRID, d.P);
        hipLaunchKernelGGL(select_kernel, grid, dim3(WAVES * 64), 0, st, d, s_tilde, sv, thr, seg_budget,
                           block_size, prefix, act, n_act, ma, budget, idx_out);
    }
    return hipGetLastError();
}

}  // namespace sablock
