// Cache construction (end of Sec. 3.3): gather the retained K/V rows, then the
// observation-window rows, into a dense cache.  Pure bit copy, 16 bytes per lane,
// a row (D elements) per group of consecutive lanes so that both the gathered
// reads and the dense writes are coalesced row-wise.
#include "sablock_internal.h"

namespace sablock {
namespace {

constexpr int NT = 256;
constexpr int RPT = 4;            // output rows per thread: that many independent 16-byte gathers in flight

// grid (ceil(ceil(rows / RPT) * chunks / NT), P, 2): z = 0 copies K, z = 1 copies V.  A thread copies chunk `ch`
// of output rows r, r + R4, r + 2 R4, r + 3 R4 (R4 = ceil(rows / RPT)), so consecutive lanes still cover a row.
// idx_div = 1: every problem has its own index row; idx_div = Hkv: the KV heads of a (sequence, layer) share one
// (retained set chosen per layer)
__global__ void __launch_bounds__(NT)
compact_kernel(Dims d, const char *k, const char *v, const int32_t *idx, const int32_t *n_sel,
               int budget, int rows, int chunks, int elt, char *k_out, char *v_out, int idx_div)
{
    const int p = blockIdx.y;
    const int ip = p / idx_div;                         // row of idx / n_sel: the problem, or its (sequence, layer)
    const int r4 = (rows + RPT - 1) / RPT;
    const int e = blockIdx.x * NT + threadIdx.x;
    if (e >= r4 * chunks) return;
    const int row0 = e / chunks, ch = e - row0 * chunks;
    const bool is_v = blockIdx.z != 0;
    const char *src = (is_v ? v : k) + (is_v ? v_problem_offset(d, p) : k_problem_offset(d, p)) * elt + (int64_t)ch * 16;
    char *dst = (is_v ? v_out : k_out) + (int64_t)p * rows * ((int64_t)chunks * 16) + (int64_t)ch * 16;
    const int64_t tstride = (is_v ? d.vs[3] : d.ks[3]) * elt;
    const int ns = n_sel[ip];
    int t[RPT];
#pragma unroll
    for (int j = 0; j < RPT; ++j) {
        const int row = row0 + j * r4;
        t[j] = -1;
        if (row < budget) {
            if (row < ns) t[j] = idx[(int64_t)ip * budget + row];
        } else if (row < rows) {
            t[j] = d.T + (row - budget);                // the W most recent rows, in order
        }
    }
    uint4 val[RPT];
#pragma unroll
    for (int j = 0; j < RPT; ++j) {
        val[j] = make_uint4(0, 0, 0, 0);
        if (t[j] >= 0 && t[j] < d.L) val[j] = *reinterpret_cast<const uint4 *>(src + (int64_t)t[j] * tstride);
    }
#pragma unroll
    for (int j = 0; j < RPT; ++j) {
        const int row = row0 + j * r4;
        if (row < rows) *reinterpret_cast<uint4 *>(dst + (int64_t)row * ((int64_t)chunks * 16)) = val[j];
    }
}

}  // namespace

hipError_t launch_compact(const Dims &d, const void *k, const void *v, const int32_t *idx,
                          const int32_t *n_sel, int32_t budget, int32_t append_window,
                          void *k_out, void *v_out, int32_t shared_rows, hipStream_t st)
{
    const int elt = d.dtype == SABLOCK_F32 ? 4 : 2;
    const int rows = budget + (append_window ? d.W : 0);
    const int chunks = d.D * elt / 16;
    if (rows <= 0 || d.P <= 0) return hipSuccess;
    const int r4 = (rows + RPT - 1) / RPT;
    dim3 grid((unsigned)(((int64_t)r4 * chunks + NT - 1) / NT), d.P, 2);
    hipLaunchKernelGGL(compact_kernel, grid, dim3(NT), 0, st, d, static_cast<const char *>(k),
                       static_cast<const char *>(v), idx, n_sel, budget, rows, chunks, elt,
                       static_cast<char *>(k_out), static_cast<char *>(v_out), shared_rows ? d.Hkv : 1);
    return hipGetLastError();
}

}  // namespace sablock
