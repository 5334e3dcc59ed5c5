// Internal declarations shared by the host ABI layer and the kernel files.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/sablock.h"

namespace sablock {

// Host-validated view of one call; passed to kernels by value.
struct Dims {
    int32_t n_seq, n_layers, Hq, Hkv, G, D, L, W, T, M;   // M = G * W rows of the window-query matrix
    int32_t P;                                            // problems = n_seq * n_layers * Hkv
    int32_t dtype;
    int32_t cus;                                          // compute units the launch plans assume (never 0)
    sablock_tuning tune;                                  // the caller's launch parameters, validated (0 = plan)
    int64_t qs[4], ks[4], vs[4];
};

constexpr int MAX_SEQ = 64;
constexpr int MAX_CAND = 16;

struct SegView {
    const int32_t *seg_off;      // device, CSR
    int32_t seq_ptr[MAX_SEQ + 1];  // host copy of the CSR pointers, travels in the kernel arguments
    int32_t max_segments;
};

constexpr int MAX_DELIM = 64;

struct DelimSet {                  // delimiter token ids, by value in the kernel arguments
    int32_t n;
    int32_t id[MAX_DELIM];
};

struct SeqPtr {                    // host CSR pointers of the segment offsets, by value in the kernel arguments
    int32_t ptr[MAX_SEQ + 1];
};

struct CandList {
    int32_t n;
    int32_t g[MAX_CAND];
};

__host__ __device__ inline int32_t seq_of_problem(const Dims &d, int32_t p) { return p / (d.n_layers * d.Hkv); }
__host__ __device__ inline int32_t layer_of_problem(const Dims &d, int32_t p) { return (p / d.Hkv) % d.n_layers; }
__host__ __device__ inline int32_t head_of_problem(const Dims &d, int32_t p) { return p % d.Hkv; }

__host__ __device__ inline int64_t k_problem_offset(const Dims &d, int32_t p)
{
    return seq_of_problem(d, p) * d.ks[0] + layer_of_problem(d, p) * d.ks[1] + head_of_problem(d, p) * d.ks[2];
}
__host__ __device__ inline int64_t v_problem_offset(const Dims &d, int32_t p)
{
    return seq_of_problem(d, p) * d.vs[0] + layer_of_problem(d, p) * d.vs[1] + head_of_problem(d, p) * d.vs[2];
}
// offset of window-query row (h_local, i) of problem p
__host__ __device__ inline int64_t q_row_offset(const Dims &d, int32_t p, int32_t h_local, int32_t i)
{
    return seq_of_problem(d, p) * d.qs[0] + layer_of_problem(d, p) * d.qs[1] +
           (int64_t)(head_of_problem(d, p) * d.G + h_local) * d.qs[2] + (int64_t)i * d.qs[3];
}

// order-preserving map float -> uint32 (larger float <=> larger key; -0.0 and +0.0 share a key, as they compare equal)
__host__ __device__ inline uint32_t ordered_key(float f)
{
    uint32_t u;
#if defined(__HIP_DEVICE_COMPILE__)
    u = __float_as_uint(f);
#else
    __builtin_memcpy(&u, &f, 4);
#endif
    if (u == 0x80000000u) u = 0u;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// ---- kernel launchers (each returns the hipError_t of its launches) ----

// generic (any shape/dtype) scoring; row statistics go through ws
size_t score_generic_ws_bytes(const Dims &d);
hipError_t launch_score_generic(const Dims &d, const void *q, const void *k, const float *row_lse, float eps,
                                float *s_out, float *ent_out, void *ws, hipStream_t st);

// MFMA scoring for bf16, D = 128, G*W = 128
bool score_mfma_supported(const Dims &d);
size_t score_mfma_ws_bytes(const Dims &d);
hipError_t launch_score_mfma(const Dims &d, const void *q, const void *k, const float *row_lse, float eps,
                             float *s_out, float *ent_out, void *ws, hipStream_t st);

// measurement aid: K streamed through the scoring kernels' load ring with no arithmetic
bool stream_probe_supported(const Dims &d);
hipError_t launch_stream_probe(const Dims &d, const void *k, int read_lds, float *s_out, float *e_out, void *sink,
                               hipStream_t st);

// head mean over all query heads of a layer (one score row per layer)
bool score_all_heads_supported(const Dims &d);
size_t score_all_heads_ws_bytes(const Dims &d);
hipError_t launch_score_all_heads(const Dims &d, const void *q, const void *k, const float *row_lse, float eps,
                                  float *s_out, float *ent_out, void *ws, hipStream_t st);

hipError_t launch_refine(const Dims &d, const float *s, const float *ent, const SegView &sv,
                         sablock_hparams hp, float *s_tilde, float *omega, hipStream_t st);

// Top-B threshold per problem: thr[p] = {ordered key of the B-th best score, index cut among its ties}
hipError_t launch_topb(const Dims &d, const float *s_tilde, int32_t budget, int32_t *thr, hipStream_t st);

size_t search_ws_bytes(const Dims &d, int32_t max_segments, int32_t budget);
hipError_t launch_search(const Dims &d, const float *s_tilde, const SegView &sv, const CandList &cand,
                         int32_t budget, float tau, int32_t *seg_budget, int32_t *block_size, int32_t *topb_out,
                         void *ws, hipStream_t st);

size_t select_ws_bytes(const Dims &d, int32_t max_segments, int32_t budget);
hipError_t launch_select(const Dims &d, const float *s_tilde, const SegView &sv, const int32_t *seg_budget,
                         const int32_t *block_size, const int32_t *topb, int32_t budget, int32_t *idx_out,
                         int32_t *n_sel_out, void *ws, hipStream_t st);

// search and select in one sequence: same results as launch_search followed by launch_select; when the Top-B
// tokens and the segment counters of a problem fit on chip (search_select_fused) the Top-B kernel also plans the
// output rows and the search kernel writes the selected tokens, so no select kernel runs
bool search_select_fused(const Dims &d, const SegView &sv, int32_t budget);
size_t search_select_ws_bytes(const Dims &d, int32_t max_segments, int32_t budget);
hipError_t launch_search_select(const Dims &d, const float *s_tilde, const SegView &sv, const CandList &cand,
                                int32_t budget, float tau, int32_t *seg_budget, int32_t *block_size, int32_t *topb_out,
                                int32_t *idx_out, int32_t *n_sel_out, void *ws, hipStream_t st);

hipError_t launch_compact(const Dims &d, const void *k, const void *v, const int32_t *idx,
                          const int32_t *n_sel, int32_t budget, int32_t append_window,
                          void *k_out, void *v_out, int32_t shared_rows, hipStream_t st);

// punctuation-based segmentation (the step before the path)
hipError_t launch_segment_count(const int32_t *tok, int64_t stride, int32_t n_seq, int32_t T, const DelimSet &ds,
                                int32_t *seg_count, hipStream_t st);
hipError_t launch_segment_offsets(const int32_t *tok, int64_t stride, int32_t n_seq, int32_t T, const DelimSet &ds,
                                  const SeqPtr &sp, int32_t *seg_off, hipStream_t st);
hipError_t launch_segment_check(const int32_t *seg_off, int32_t n_seq, int32_t T, const SeqPtr &sp, int32_t *bad,
                                hipStream_t st);

// Opt-ins that hold per device (dynamic LDS above 64 KiB for a kernel) are made once per host thread and device:
//     static thread_local PerDeviceOnce once;  if (once.needed()) { ...; once.done(); }
// A thread that switches devices simply makes them again.
struct PerDeviceOnce {
    int done_dev = -1, cur = -1;
    bool needed()
    {
        if (hipGetDevice(&cur) != hipSuccess) cur = -1;
        return cur < 0 || cur != done_dev;
    }
    void done() { done_dev = cur; }
};

// row statistics of the scoring step for 256 window-query rows per KV head with one read of K (the attention
// kernel's first product alone): stats [P][2][row_stats_chunks][128][2] = (reference in the log2 domain, sum)
bool row_stats_supported(const Dims &d);
int row_stats_chunks(const Dims &d);
hipError_t launch_row_stats(const Dims &d, const void *q, const void *k, float *stats, hipStream_t st);

// attention of the window queries over all keys, with the rows' log-sum-exp (the producer of sablock_score's row_lse)
bool window_attention_supported(const Dims &d);
size_t window_attention_ws_bytes(const Dims &d);
hipError_t launch_window_attention(const Dims &d, const void *q, const void *k, const void *v, float *out, float *lse,
                                   void *ws, hipStream_t st);

// decode-time attention over a cache (the step after the path); d.L = rows of the cache buffers
bool decode_supported(const Dims &d);
size_t decode_ws_bytes(const Dims &d);
hipError_t launch_decode(const Dims &d, const void *q, const void *k, const void *v, const int32_t *n_sel,
                         int32_t budget, float *out, void *ws, hipStream_t st);

}  // namespace sablock
