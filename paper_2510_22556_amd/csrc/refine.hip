// Segment-guided score refinement (Alg. 1; Eqs. Ik, Dk, omegak, st_tilde).
//
// A workgroup owns 16 consecutive segments of one problem, i.e. one contiguous token range.  It first streams
// the range's scores and entropy terms into LDS with fully coalesced loads (all of a thread's loads in flight
// at once: the kernel is a chain of a few memory round trips, so it is tuned for latency and occupancy), then
// sixteen lanes per segment accumulate the two segment sums in fp64 from LDS (shuffle reduction inside the
// 16-lane group) and rescale the segment's tokens.  Traffic is 12 bytes per token.  A range that does not fit
// in LDS (very long segments) is read from global memory by the lane groups directly.
#include "sablock_internal.h"

namespace sablock {
namespace {

constexpr int GROUP = 16;                  // lanes per segment
constexpr int NT = 256;                    // threads per workgroup: 16 segments at a time
constexpr int RSEG = NT / GROUP;           // segments per workgroup
constexpr int RPT = 8;                     // staged tokens per thread
constexpr int RCAP = RPT * NT;             // tokens per workgroup whose inputs are staged in LDS

// sum over the 16 lanes of a group = one DPP row: lane ^ 1, lane ^ 2, mirror inside 8, mirror inside 16 (no LDS
// round trips); every lane of the group gets the sum
template <int CTRL>
__device__ inline double dpp_add(double v)
{
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, 0xf, 0xf, false);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, 0xf, 0xf, false);
    return v + __hiloint2double(hi, lo);
}
__device__ inline double group_sum(double v)
{
    static_assert(GROUP == 16, "a group is one DPP row");
    v = dpp_add<0xB1>(v);
    v = dpp_add<0x4E>(v);
    v = dpp_add<0x141>(v);
    v = dpp_add<0x140>(v);
    return v;
}

// grid (ceil(max_segments / RSEG), P)
__global__ void __launch_bounds__(NT)
refine_kernel(Dims d, const float *s, const float *ent, SegView sv, sablock_hparams hp,
              float *s_tilde, float *omega)
{
    __shared__ float sh_s[RCAP], sh_e[RCAP];
    const int p = blockIdx.y;
    const int sub = threadIdx.x & (GROUP - 1), grp = threadIdx.x / GROUP;
    const int seq = seq_of_problem(d, p);
    const int base = sv.seq_ptr[seq];
    const int K = sv.seq_ptr[seq + 1] - base - 1;
    const int k0 = blockIdx.x * RSEG;
    const int k1 = min(k0 + RSEG, K);
    // rows of omega are max_segments wide: zero behind the sequence's last segment
    if (omega)
        for (int k = max(k0, K) + (int)threadIdx.x; k < min(k0 + RSEG, sv.max_segments); k += NT)
            omega[(int64_t)p * sv.max_segments + k] = 0.f;
    if (k0 >= K) return;
    const float *sp = s + (int64_t)p * d.L;
    const float *ep = ent + (int64_t)p * d.L;
    float *op = s_tilde + (int64_t)p * d.T;
    // this lane group's segment (its bounds are fetched together with the range's)
    const int k = k0 + grp;
    const bool mine = k < k1;
    const int a = sv.seg_off[base + (mine ? k : k0)], b = sv.seg_off[base + (mine ? k : k0) + 1];
    const int lo = sv.seg_off[base + k0], hi = sv.seg_off[base + k1];
    const bool staged = hi - lo <= RCAP;
    if (staged) {
        // only as many rounds of loads as the range has tokens (uniform over the workgroup), all in flight together
        const int nj = (hi - lo + NT - 1) / NT;
        float rs[RPT], re[RPT];
#pragma unroll
        for (int j = 0; j < RPT; ++j) {
            if (j < nj) {
                const int t = min(lo + j * NT + (int)threadIdx.x, hi - 1);
                rs[j] = sp[t];
                re[j] = ep[t];
            }
        }
#pragma unroll
        for (int j = 0; j < RPT; ++j) {
            const int i = j * NT + (int)threadIdx.x;
            if (j < nj && lo + i < hi) { sh_s[i] = rs[j]; sh_e[i] = re[j]; }
        }
        __syncthreads();
    }
    if (!mine) return;
    double sum_s = 0.0, sum_e = 0.0;
    if (staged) for (int t = a + sub; t < b; t += GROUP) { sum_s += (double)sh_s[t - lo]; sum_e += (double)sh_e[t - lo]; }
    else for (int t = a + sub; t < b; t += GROUP) { sum_s += (double)sp[t]; sum_e += (double)ep[t]; }
    sum_s = group_sum(sum_s);
    sum_e = group_sum(sum_e);
    const double n = (double)(b - a);
    const double Ik = sum_s / n;                                   // Eq. Ik
    const double Dk = sum_e / n;                                   // Eq. Dk
    const double wk = Ik * (1.0 + (double)hp.eta * Dk);            // Eq. omegak
    const double f = 1.0 + (double)hp.alpha * wk;
    if (staged) for (int t = a + sub; t < b; t += GROUP) op[t] = (float)((double)sh_s[t - lo] * f);   // Eq. st_tilde
    else for (int t = a + sub; t < b; t += GROUP) op[t] = (float)((double)sp[t] * f);
    if (omega && sub == 0) omega[(int64_t)p * sv.max_segments + k] = (float)wk;
}

}  // namespace

hipError_t launch_refine(const Dims &d, const float *s, const float *ent, const SegView &sv,
                         sablock_hparams hp, float *s_tilde, float *omega, hipStream_t st)
{
    if (sv.max_segments <= 0 || d.P <= 0) return hipSuccess;
    dim3 grid((sv.max_segments + RSEG - 1) / RSEG, d.P);
    hipLaunchKernelGGL(refine_kernel, grid, dim3(NT), 0, st, d, s, ent, sv, hp, s_tilde, omega);
    return hipGetLastError();
}

}  // namespace sablock
