// Segment-guided score refinement (Alg. 1; Eqs. Ik, Dk, omegak, st_tilde).
//
// Sixteen lanes per (problem, segment), four segments per wavefront: lanes stride over the segment's tokens, the
// two segment sums are accumulated in fp64 and reduced with shuffles inside the 16-lane group, then every lane
// rescales its tokens.  Traffic is 12 bytes per token; the kernel is latency-bound (a chain of three dependent
// memory round trips per segment), so several segments share a wavefront and all problems of a call share one launch.
#include "sablock_internal.h"

namespace sablock {
namespace {

constexpr int GROUP = 16;                  // lanes per segment
constexpr int NT = 256;                    // threads per workgroup: 16 segments

__device__ inline double group_sum(double v)
{
    for (int off = GROUP / 2; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

// grid (ceil(max_segments / 16), P)
__global__ void __launch_bounds__(NT)
refine_kernel(Dims d, const float *s, const float *ent, SegView sv, sablock_hparams hp,
              float *s_tilde, float *omega)
{
    const int p = blockIdx.y;
    const int sub = threadIdx.x & (GROUP - 1);
    const int k = blockIdx.x * (NT / GROUP) + threadIdx.x / GROUP;
    const int seq = seq_of_problem(d, p);
    const int base = sv.seq_ptr[seq];
    const int K = sv.seq_ptr[seq + 1] - base - 1;
    if (k >= sv.max_segments) return;
    if (k >= K) {
        if (omega && sub == 0) omega[(int64_t)p * sv.max_segments + k] = 0.f;
        return;
    }
    const int a = sv.seg_off[base + k], b = sv.seg_off[base + k + 1];
    const float *sp = s + (int64_t)p * d.L;
    const float *ep = ent + (int64_t)p * d.L;
    double sum_s = 0.0, sum_e = 0.0;
    for (int t = a + sub; t < b; t += GROUP) { sum_s += (double)sp[t]; sum_e += (double)ep[t]; }
    sum_s = group_sum(sum_s);
    sum_e = group_sum(sum_e);
    const double n = (double)(b - a);
    const double Ik = sum_s / n;                                   // Eq. Ik
    const double Dk = sum_e / n;                                   // Eq. Dk
    const double wk = Ik * (1.0 + (double)hp.eta * Dk);            // Eq. omegak
    const double f = 1.0 + (double)hp.alpha * wk;
    float *op = s_tilde + (int64_t)p * d.T;
    for (int t = a + sub; t < b; t += GROUP) op[t] = (float)((double)sp[t] * f);   // Eq. st_tilde
    if (omega && sub == 0) omega[(int64_t)p * sv.max_segments + k] = (float)wk;
}

}  // namespace

hipError_t launch_refine(const Dims &d, const float *s, const float *ent, const SegView &sv,
                         sablock_hparams hp, float *s_tilde, float *omega, hipStream_t st)
{
    if (sv.max_segments <= 0 || d.P <= 0) return hipSuccess;
    dim3 grid((sv.max_segments + NT / GROUP - 1) / (NT / GROUP), d.P);
    hipLaunchKernelGGL(refine_kernel, grid, dim3(NT), 0, st, d, s, ent, sv, hp, s_tilde, omega);
    return hipGetLastError();
}

}  // namespace sablock
