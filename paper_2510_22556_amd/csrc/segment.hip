// Punctuation-based segmentation of the compressible region (Sec. 3.1): a delimiter token closes the segment it
// belongs to, so a new segment starts after every delimiter that is not the region's last token.
//
// One 1024-thread workgroup per sequence walks the tokens in chunks of 4096 (16-byte loads where the row is
// aligned) and keeps a running count of boundaries; the offsets kernel writes boundary positions in order at
// carry + (block-wide exclusive prefix).  Segmentation runs once per prompt (all layers and heads share it), on
// 4 bytes per token, so the kernels are sized for simplicity, not for the last microsecond.
#include "sablock_internal.h"

namespace sablock {
namespace {

constexpr int SG_THREADS = 1024;
constexpr int SG_PER = 4;                  // tokens per thread and chunk

__device__ inline bool is_delim(int32_t tok, const DelimSet &ds)
{
    bool hit = false;
    for (int i = 0; i < ds.n; ++i) hit |= tok == ds.id[i];
    return hit;
}

// boundary flags of tokens t0 .. t0+3 (a boundary sits AFTER token t: t is a delimiter and t < T - 1)
__device__ inline int chunk_flags(const int32_t *row, int t0, int T, const DelimSet &ds)
{
    int f = 0;
#pragma unroll
    for (int j = 0; j < SG_PER; ++j) {
        const int t = t0 + j;
        if (t < T - 1 && is_delim(row[t], ds)) f |= 1 << j;
    }
    return f;
}

// exclusive prefix of v over the workgroup and the workgroup total; ends with a barrier
__device__ inline int block_exclusive(int v, int *sh_w, int &total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int incl = v;
    for (int o = 1; o < 64; o <<= 1) { int x = __shfl_up(incl, o); if (lane >= o) incl += x; }
    if (lane == 63) sh_w[wave] = incl;
    __syncthreads();
    int before = 0;
    total = 0;
    for (int w = 0; w < SG_THREADS / 64; ++w) { if (w < wave) before += sh_w[w]; total += sh_w[w]; }
    __syncthreads();
    return before + incl - v;
}

// grid (n_seq): seg_count[s] = 1 + number of boundaries
__global__ void __launch_bounds__(SG_THREADS)
segment_count_kernel(const int32_t *tok, int64_t stride, int T, DelimSet ds, int32_t *seg_count)
{
    __shared__ int sh_w[SG_THREADS / 64];
    const int32_t *row = tok + (int64_t)blockIdx.x * stride;
    int n = 0;
    for (int c0 = 0; c0 < T; c0 += SG_THREADS * SG_PER) n += __popc(chunk_flags(row, c0 + threadIdx.x * SG_PER, T, ds));
    int total;
    block_exclusive(n, sh_w, total);
    if (threadIdx.x == 0) seg_count[blockIdx.x] = total + 1;
}

// grid (n_seq): offsets 0, t+1 for every boundary t in ascending order, T
__global__ void __launch_bounds__(SG_THREADS)
segment_offsets_kernel(const int32_t *tok, int64_t stride, int T, DelimSet ds, SeqPtr sp, int32_t *seg_off)
{
    __shared__ int sh_w[SG_THREADS / 64];
    const int s = blockIdx.x;
    const int32_t *row = tok + (int64_t)s * stride;
    int32_t *out = seg_off + sp.ptr[s];
    const int n_out = sp.ptr[s + 1] - sp.ptr[s];         // offsets this sequence may write (segments + 1)
    if (threadIdx.x == 0 && n_out > 0) out[0] = 0;
    int carry = 1;                                        // next free slot
    for (int c0 = 0; c0 < T; c0 += SG_THREADS * SG_PER) {
        const int t0 = c0 + threadIdx.x * SG_PER;
        const int f = chunk_flags(row, t0, T, ds);
        int total;
        int pos = carry + block_exclusive(__popc(f), sh_w, total);
#pragma unroll
        for (int j = 0; j < SG_PER; ++j)
            if ((f >> j) & 1) { if (pos < n_out) out[pos] = t0 + j + 1; ++pos; }
        carry += total;
    }
    if (threadIdx.x == 0 && carry < n_out) out[carry] = T;
}

// grid (n_seq): bad[s] = number of offsets of sequence s that break "0 = off[0] < off[1] < ... < off[K] = T"
// (an entry counts when it is not above its predecessor; the first when it is not 0, the last also when it is not T)
__global__ void __launch_bounds__(SG_THREADS)
segment_check_kernel(const int32_t *seg_off, SeqPtr sp, int T, int32_t *bad)
{
    __shared__ int sh_w[SG_THREADS / 64];
    const int s = blockIdx.x;
    const int32_t *off = seg_off + sp.ptr[s];
    const int n = sp.ptr[s + 1] - sp.ptr[s];              // offsets of this sequence, >= 2
    int mine = 0;
    for (int j = threadIdx.x; j < n; j += SG_THREADS) {
        const int v = off[j];
        bool ok = j == 0 ? v == 0 : v > off[j - 1];
        if (j == n - 1) ok = ok && v == T;
        mine += !ok;
    }
    int total;
    block_exclusive(mine, sh_w, total);
    if (threadIdx.x == 0) bad[s] = total;
}

}  // namespace

hipError_t launch_segment_check(const int32_t *seg_off, int32_t n_seq, int32_t T, const SeqPtr &sp, int32_t *bad,
                                hipStream_t st)
{
    if (n_seq <= 0) return hipSuccess;
    hipLaunchKernelGGL(segment_check_kernel, dim3(n_seq), dim3(SG_THREADS), 0, st, seg_off, sp, T, bad);
    return hipGetLastError();
}

hipError_t launch_segment_count(const int32_t *tok, int64_t stride, int32_t n_seq, int32_t T, const DelimSet &ds,
                                int32_t *seg_count, hipStream_t st)
{
    if (n_seq <= 0) return hipSuccess;
    hipLaunchKernelGGL(segment_count_kernel, dim3(n_seq), dim3(SG_THREADS), 0, st, tok, stride, T, ds, seg_count);
    return hipGetLastError();
}

hipError_t launch_segment_offsets(const int32_t *tok, int64_t stride, int32_t n_seq, int32_t T, const DelimSet &ds,
                                  const SeqPtr &sp, int32_t *seg_off, hipStream_t st)
{
    if (n_seq <= 0) return hipSuccess;
    hipLaunchKernelGGL(segment_offsets_kernel, dim3(n_seq), dim3(SG_THREADS), 0, st, tok, stride, T, ds, sp, seg_off);
    return hipGetLastError();
}

}  // namespace sablock
