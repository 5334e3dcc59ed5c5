// Host side of the C ABI: argument validation, workspace carving, kernel dispatch.
// Nothing here touches the device except kernel launches on the caller's stream.
#include "sablock_internal.h"

#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cstring>

using namespace sablock;

namespace {

thread_local char g_err[512] = "";

sablock_status fail(sablock_status st, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Compute units of the current device.  Asked once per device and remembered (the only thing the library
// remembers between calls); concurrent first calls store the same value.
constexpr int MAX_DEVICES = 64;
std::atomic<int> g_cus[MAX_DEVICES];

sablock_status current_device_cus(int32_t *out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0) {
        (void)hipGetLastError();
        return fail(SABLOCK_ERR_DEVICE, "no current HIP device (set shape.tuning.compute_units to plan without one)");
    }
    if (dev < MAX_DEVICES) {
        const int c = g_cus[dev].load(std::memory_order_relaxed);
        if (c > 0) { *out = c; return SABLOCK_OK; }
    }
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) {
        (void)hipGetLastError();
        return fail(SABLOCK_ERR_DEVICE, "cannot read the compute-unit count of device %d", dev);
    }
    if (dev < MAX_DEVICES) g_cus[dev].store(n, std::memory_order_relaxed);
    *out = n;
    return SABLOCK_OK;
}

// Scratch memory of sablock_score_static: one array per GPU, part of the library's code object, so it exists from
// the moment the library is loaded on a device until the process ends and no allocation call is ever made for
// it.  In host code the array's name is only a handle: the address a kernel can use comes from
// hipGetSymbolAddress, asked once per device with that device current (every GPU has its own copy at its own
// address) and remembered.
__device__ __align__(256) static unsigned char scratch[SABLOCK_STATIC_SCRATCH_BYTES];
std::atomic<void *> g_scratch_ptr[MAX_DEVICES];

sablock_status static_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0) {
        (void)hipGetLastError();
        return fail(SABLOCK_ERR_DEVICE, "sablock_score_static: no current HIP device");
    }
    if (dev >= MAX_DEVICES) return fail(SABLOCK_ERR_UNSUPPORTED, "sablock_score_static: device %d: at most %d devices", dev, MAX_DEVICES);
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            (void)hipGetLastError();
            return fail(SABLOCK_ERR_DEVICE, "sablock_score_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
        }
        g_scratch_ptr[dev].store(p, std::memory_order_release);     // concurrent first calls store the same address
    }
    *out = p;
    return SABLOCK_OK;
}

sablock_status make_dims(const sablock_shape *s, Dims *d)
{
    if (!s) return fail(SABLOCK_ERR_INVALID_ARG, "shape is NULL");
    if (s->n_seq < 1 || s->n_layers < 1 || s->n_kv_heads < 1 || s->n_q_heads < 1)
        return fail(SABLOCK_ERR_INVALID_ARG, "n_seq, n_layers, n_q_heads, n_kv_heads must be >= 1");
    if (s->n_q_heads % s->n_kv_heads != 0)
        return fail(SABLOCK_ERR_INVALID_ARG, "n_q_heads (%d) is not a multiple of n_kv_heads (%d)", s->n_q_heads, s->n_kv_heads);
    if (s->window < 1 || s->seq_len < 2 || s->window >= s->seq_len)
        return fail(SABLOCK_ERR_INVALID_ARG, "need 1 <= window < seq_len (window %d, seq_len %d)", s->window, s->seq_len);
    if (s->dtype != SABLOCK_F32 && s->dtype != SABLOCK_BF16)
        return fail(SABLOCK_ERR_INVALID_ARG, "unknown dtype %d", s->dtype);
    if (s->head_dim < 8 || s->head_dim > 256 || s->head_dim % 8 != 0)
        return fail(SABLOCK_ERR_UNSUPPORTED, "head_dim %d: need a multiple of 8 in [8, 256]", s->head_dim);
    if (s->window > 64) return fail(SABLOCK_ERR_UNSUPPORTED, "window %d: at most 64", s->window);
    if (s->n_seq > MAX_SEQ) return fail(SABLOCK_ERR_UNSUPPORTED, "n_seq %d: at most %d per call", s->n_seq, MAX_SEQ);
    const int64_t P = (int64_t)s->n_seq * s->n_layers * s->n_kv_heads;
    if (P > 65535) return fail(SABLOCK_ERR_UNSUPPORTED, "n_seq*n_layers*n_kv_heads = %lld: at most 65535 per call", (long long)P);
    if ((int64_t)s->n_q_heads / s->n_kv_heads * s->window > 1024)
        return fail(SABLOCK_ERR_UNSUPPORTED, "G*W > 1024");
    for (int a = 0; a < 4; ++a) {
        if (s->q_stride[a] < 0 || s->k_stride[a] < 0 || s->v_stride[a] < 0)
            return fail(SABLOCK_ERR_INVALID_ARG, "negative stride");
        if (s->q_stride[a] % 8 || s->k_stride[a] % 8 || s->v_stride[a] % 8)
            return fail(SABLOCK_ERR_UNSUPPORTED, "strides must be multiples of 8 elements (16-byte row alignment)");
    }
    if (s->q_stride[3] < s->head_dim || s->k_stride[3] < s->head_dim)
        return fail(SABLOCK_ERR_INVALID_ARG, "token stride smaller than head_dim");
    const sablock_tuning &tu = s->tuning;
    if (tu.compute_units < 0 || tu.compute_units > 65536)
        return fail(SABLOCK_ERR_INVALID_ARG, "tuning.compute_units %d: need 0 (ask the device) .. 65536", tu.compute_units);
    if (tu.score_chunk != 0 && (tu.score_chunk < 128 || tu.score_chunk > 131072))
        return fail(SABLOCK_ERR_INVALID_ARG, "tuning.score_chunk %d: need 0 or 128 .. 131072", tu.score_chunk);
    if (tu.window_chunk != 0 && (tu.window_chunk < 32 || tu.window_chunk > 131072))
        return fail(SABLOCK_ERR_INVALID_ARG, "tuning.window_chunk %d: need 0 or 32 .. 131072", tu.window_chunk);
    if (tu.topb_slices < 0 || tu.topb_slices > 64)
        return fail(SABLOCK_ERR_INVALID_ARG, "tuning.topb_slices %d: need 0 .. 64", tu.topb_slices);
    if (tu.stats_per_key < 0 || tu.stats_per_key > 2)
        return fail(SABLOCK_ERR_INVALID_ARG, "tuning.stats_per_key %d: need 0, 1 or 2", tu.stats_per_key);
    if (tu.reserved[0] || tu.reserved[1] || tu.reserved[2])
        return fail(SABLOCK_ERR_INVALID_ARG, "tuning.reserved must be 0");
    d->tune = tu;
    d->cus = tu.compute_units;
    if (d->cus == 0) {
        const sablock_status st = current_device_cus(&d->cus);
        if (st != SABLOCK_OK) return st;
    }
    d->n_seq = s->n_seq; d->n_layers = s->n_layers; d->Hq = s->n_q_heads; d->Hkv = s->n_kv_heads;
    d->G = s->n_q_heads / s->n_kv_heads; d->D = s->head_dim; d->L = s->seq_len; d->W = s->window;
    d->T = s->seq_len - s->window; d->M = d->G * d->W; d->P = (int32_t)P; d->dtype = s->dtype;
    for (int a = 0; a < 4; ++a) { d->qs[a] = s->q_stride[a]; d->ks[a] = s->k_stride[a]; d->vs[a] = s->v_stride[a]; }
    return SABLOCK_OK;
}

sablock_status make_segview(const Dims &d, const int32_t *seg_off, const int32_t *seg_ptr, int32_t max_segments,
                            SegView *sv)
{
    if (!seg_off || !seg_ptr) return fail(SABLOCK_ERR_INVALID_ARG, "seg_off or seg_ptr is NULL");
    if (max_segments < 0) return fail(SABLOCK_ERR_INVALID_ARG, "max_segments < 0");
    if (seg_ptr[0] < 0) return fail(SABLOCK_ERR_INVALID_ARG, "seg_ptr[0] < 0");
    for (int s = 0; s < d.n_seq; ++s) {
        const int n = seg_ptr[s + 1] - seg_ptr[s];
        if (n < 1) return fail(SABLOCK_ERR_INVALID_ARG, "sequence %d: seg_ptr must leave at least one offset", s);
        if (n - 1 > max_segments)
            return fail(SABLOCK_ERR_INVALID_ARG, "sequence %d has %d segments > max_segments %d", s, n - 1, max_segments);
    }
    sv->seg_off = seg_off;
    sv->max_segments = max_segments;
    memset(sv->seq_ptr, 0, sizeof(sv->seq_ptr));
    for (int s = 0; s <= d.n_seq; ++s) sv->seq_ptr[s] = seg_ptr[s];
    return SABLOCK_OK;
}

size_t score_ws(const Dims &d)
{
    size_t a = score_generic_ws_bytes(d);
    if (score_mfma_supported(d)) { size_t b = score_mfma_ws_bytes(d); if (b > a) a = b; }
    return a;
}

sablock_status dev(hipError_t e, const char *what)
{
    if (e == hipSuccess) return SABLOCK_OK;
    return fail(SABLOCK_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
}

}  // namespace

extern "C" {

const char *sablock_version(void) { return "sablock-gfx950 0.1"; }
const char *sablock_last_error(void) { return g_err; }

sablock_status sablock_workspace_bytes(const sablock_shape *shape, int32_t max_segments, int32_t budget,
                                       size_t *bytes_out)
{
    Dims d;
    sablock_status st = make_dims(shape, &d);
    if (st != SABLOCK_OK) return st;
    if (!bytes_out) return fail(SABLOCK_ERR_INVALID_ARG, "bytes_out is NULL");
    if (max_segments < 0 || budget < 0) return fail(SABLOCK_ERR_INVALID_ARG, "max_segments or budget < 0");
    size_t b = score_ws(d);
    size_t c = search_ws_bytes(d, max_segments, budget); if (c > b) b = c;
    c = select_ws_bytes(d, max_segments, budget); if (c > b) b = c;
    c = search_select_ws_bytes(d, max_segments, budget); if (c > b) b = c;
    *bytes_out = b + 256;
    return SABLOCK_OK;
}

// shared by sablock_score and sablock_score_static: everything but where the scratch memory comes from
static sablock_status score_checked(const char *who, const sablock_shape *shape, const void *q_win, const void *k,
                                    const float *row_lse, float eps, float *s_out, float *ent_out,
                                    Dims *d, size_t *need)
{
    sablock_status st = make_dims(shape, d);
    if (st != SABLOCK_OK) return st;
    if (!q_win || !k || !s_out || !ent_out) return fail(SABLOCK_ERR_INVALID_ARG, "%s: NULL tensor", who);
    if (!aligned16(q_win) || !aligned16(k)) return fail(SABLOCK_ERR_INVALID_ARG, "%s: Q/K must be 16-byte aligned", who);
    if (!(eps > 0.f)) return fail(SABLOCK_ERR_INVALID_ARG, "%s: eps must be > 0", who);
    *need = row_lse ? 0 : (score_mfma_supported(*d) ? score_mfma_ws_bytes(*d) : score_generic_ws_bytes(*d));
    return SABLOCK_OK;
}

static sablock_status score_launch(const char *who, const Dims &d, const void *q_win, const void *k, const float *row_lse,
                                   float eps, float *s_out, float *ent_out, void *ws, void *stream)
{
    hipStream_t hs = static_cast<hipStream_t>(stream);
    hipError_t e = score_mfma_supported(d) ? launch_score_mfma(d, q_win, k, row_lse, eps, s_out, ent_out, ws, hs)
                                           : launch_score_generic(d, q_win, k, row_lse, eps, s_out, ent_out, ws, hs);
    return dev(e, who);
}

sablock_status sablock_score(const sablock_shape *shape, const void *q_win, const void *k,
                             const float *row_lse, float eps, float *s_out, float *ent_out,
                             void *ws, size_t ws_bytes, void *stream)
{
    Dims d;
    size_t need = 0;
    sablock_status st = score_checked("sablock_score", shape, q_win, k, row_lse, eps, s_out, ent_out, &d, &need);
    if (st != SABLOCK_OK) return st;
    if (need && (!ws || ws_bytes < need))
        return fail(SABLOCK_ERR_WORKSPACE_TOO_SMALL, "sablock_score: workspace %zu < %zu bytes", ws_bytes, need);
    return score_launch("sablock_score", d, q_win, k, row_lse, eps, s_out, ent_out, ws, stream);
}

sablock_status sablock_score_static(const sablock_shape *shape, const void *q_win, const void *k,
                                    const float *row_lse, float eps, float *s_out, float *ent_out, void *stream)
{
    Dims d;
    size_t need = 0;
    sablock_status st = score_checked("sablock_score_static", shape, q_win, k, row_lse, eps, s_out, ent_out, &d, &need);
    if (st != SABLOCK_OK) return st;
    if (need > SABLOCK_STATIC_SCRATCH_BYTES)
        return fail(SABLOCK_ERR_UNSUPPORTED, "sablock_score_static: the row statistics of this call need %zu bytes of scratch, "
                    "the static array holds %zu; use sablock_score with a workspace, or fewer problems per call",
                    need, (size_t)SABLOCK_STATIC_SCRATCH_BYTES);
    void *ptr = nullptr;
    if (need) {
        st = static_scratch(&ptr);
        if (st != SABLOCK_OK) return st;
    }
    // every word of the statistics that the column pass reads is written by this call's own statistics kernels
    // first, so the previous call's contents need no clearing
    return score_launch("sablock_score_static", d, q_win, k, row_lse, eps, s_out, ent_out, ptr, stream);
}

sablock_status sablock_stream_probe(const sablock_shape *shape, const void *k, int32_t read_lds, float *s_out,
                                    float *ent_out, void *sink, void *stream)
{
    Dims d;
    sablock_status st = make_dims(shape, &d);
    if (st != SABLOCK_OK) return st;
    if (!k || !sink) return fail(SABLOCK_ERR_INVALID_ARG, "sablock_stream_probe: NULL argument");
    if ((s_out == nullptr) != (ent_out == nullptr))
        return fail(SABLOCK_ERR_INVALID_ARG, "sablock_stream_probe: s_out and ent_out must both be given or both be NULL");
    if (!aligned16(k)) return fail(SABLOCK_ERR_INVALID_ARG, "sablock_stream_probe: K must be 16-byte aligned");
    if (!stream_probe_supported(d)) return fail(SABLOCK_ERR_UNSUPPORTED, "sablock_stream_probe: needs bf16 and head_dim 128");
    return dev(launch_stream_probe(d, k, read_lds, s_out, ent_out, sink, static_cast<hipStream_t>(stream)),
               "sablock_stream_probe");
}

sablock_status sablock_refine(const sablock_shape *shape, const float *s, const float *ent,
                              const int32_t *seg_off, const int32_t *seg_ptr, int32_t max_segments,
                              const sablock_hparams *hp, float *s_tilde_out, float *omega_out,
                              void *ws, size_t ws_bytes, void *stream)
{
    (void)ws; (void)ws_bytes;
    Dims d;
    sablock_status st = make_dims(shape, &d);
    if (st != SABLOCK_OK) return st;
    if (!s || !ent || !s_tilde_out || !hp) return fail(SABLOCK_ERR_INVALID_ARG, "sablock_refine: NULL argument");
    if (!(hp->alpha >= 0.f) || !(hp->eta >= 0.f)) return fail(SABLOCK_ERR_INVALID_ARG, "sablock_refine: alpha, eta must be >= 0");
    SegView sv;
    st = make_segview(d, seg_off, seg_ptr, max_segments, &sv);
    if (st != SABLOCK_OK) return st;
    return dev(launch_refine(d, s, ent, sv, *hp, s_tilde_out, omega_out, static_cast<hipStream_t>(stream)),
               "sablock_refine");
}

// candidate block sizes: 1 = cand[0] < cand[1] < ... <= 64
static sablock_status make_candlist(const char *who, const int32_t *cand, int32_t n_cand, CandList *cl)
{
    if (n_cand < 1 || n_cand > MAX_CAND) return fail(SABLOCK_ERR_INVALID_ARG, "%s: n_cand must be in [1, %d]", who, MAX_CAND);
    if (cand[0] != 1) return fail(SABLOCK_ERR_INVALID_ARG, "%s: cand[0] must be 1", who);
    memset(cl, 0, sizeof(*cl));
    cl->n = n_cand;
    for (int c = 0; c < n_cand; ++c) {
        if (c && cand[c] <= cand[c - 1]) return fail(SABLOCK_ERR_INVALID_ARG, "%s: cand must be strictly ascending", who);
        if (cand[c] > 64) return fail(SABLOCK_ERR_UNSUPPORTED, "%s: block size %d > 64", who, cand[c]);
        cl->g[c] = cand[c];
    }
    return SABLOCK_OK;
}

sablock_status sablock_search_blocks(const sablock_shape *shape, const float *s_tilde,
                                     const int32_t *seg_off, const int32_t *seg_ptr, int32_t max_segments,
                                     const int32_t *cand, int32_t n_cand, int32_t budget, float tau,
                                     int32_t *seg_budget_out, int32_t *block_size_out, int32_t *topb_out,
                                     void *ws, size_t ws_bytes, void *stream)
{
    Dims d;
    sablock_status st = make_dims(shape, &d);
    if (st != SABLOCK_OK) return st;
    if (!s_tilde || !seg_budget_out || !block_size_out || !cand)
        return fail(SABLOCK_ERR_INVALID_ARG, "sablock_search_blocks: NULL argument");
    if (budget < 0) return fail(SABLOCK_ERR_INVALID_ARG, "sablock_search_blocks: budget < 0");
    if (!(tau >= 0.f)) return fail(SABLOCK_ERR_INVALID_ARG, "sablock_search_blocks: tau must be >= 0");
    CandList cl;
    st = make_candlist("sablock_search_blocks", cand, n_cand, &cl);
    if (st != SABLOCK_OK) return st;
    SegView sv;
    st = make_segview(d, seg_off, seg_ptr, max_segments, &sv);
    if (st != SABLOCK_OK) return st;
    const size_t need = search_ws_bytes(d, max_segments, budget);
    if (!ws || ws_bytes < need)
        return fail(SABLOCK_ERR_WORKSPACE_TOO_SMALL, "sablock_search_blocks: workspace %zu < %zu bytes", ws_bytes, need);
    hipError_t e = launch_search(d, s_tilde, sv, cl, budget, tau, seg_budget_out, block_size_out, topb_out, ws,
                                 static_cast<hipStream_t>(stream));
    return dev(e, "sablock_search_blocks");
}

sablock_status sablock_select(const sablock_shape *shape, const float *s_tilde,
                              const int32_t *seg_off, const int32_t *seg_ptr, int32_t max_segments,
                              const int32_t *seg_budget, const int32_t *block_size, const int32_t *topb,
                              int32_t budget, int32_t *idx_out, int32_t *n_sel_out, void *ws, size_t ws_bytes,
                              void *stream)
{
    Dims d;
    sablock_status st = make_dims(shape, &d);
    if (st != SABLOCK_OK) return st;
    if (!s_tilde || !seg_budget || !block_size || !n_sel_out || (!idx_out && budget > 0))
        return fail(SABLOCK_ERR_INVALID_ARG, "sablock_select: NULL argument");
    if (budget < 0) return fail(SABLOCK_ERR_INVALID_ARG, "sablock_select: budget < 0");
    SegView sv;
    st = make_segview(d, seg_off, seg_ptr, max_segments, &sv);
    if (st != SABLOCK_OK) return st;
    const size_t need = select_ws_bytes(d, max_segments, budget);
    if (!ws || ws_bytes < need)
        return fail(SABLOCK_ERR_WORKSPACE_TOO_SMALL, "sablock_select: workspace %zu < %zu bytes", ws_bytes, need);
    return dev(launch_select(d, s_tilde, sv, seg_budget, block_size, topb, budget, idx_out, n_sel_out, ws,
                             static_cast<hipStream_t>(stream)), "sablock_select");
}

sablock_status sablock_search_select(const sablock_shape *shape, const float *s_tilde,
                                     const int32_t *seg_off, const int32_t *seg_ptr, int32_t max_segments,
                                     const int32_t *cand, int32_t n_cand, int32_t budget, float tau,
                                     int32_t *seg_budget_out, int32_t *block_size_out, int32_t *topb_out,
                                     int32_t *idx_out, int32_t *n_sel_out, void *ws, size_t ws_bytes, void *stream)
{
    Dims d;
    sablock_status st = make_dims(shape, &d);
    if (st != SABLOCK_OK) return st;
    if (!s_tilde || !seg_budget_out || !block_size_out || !cand || !n_sel_out || (!idx_out && budget > 0))
        return fail(SABLOCK_ERR_INVALID_ARG, "sablock_search_select: NULL argument");
    if (budget < 0) return fail(SABLOCK_ERR_INVALID_ARG, "sablock_search_select: budget < 0");
    if (!(tau >= 0.f)) return fail(SABLOCK_ERR_INVALID_ARG, "sablock_search_select: tau must be >= 0");
    CandList cl;
    st = make_candlist("sablock_search_select", cand, n_cand, &cl);
    if (st != SABLOCK_OK) return st;
    SegView sv;
    st = make_segview(d, seg_off, seg_ptr, max_segments, &sv);
    if (st != SABLOCK_OK) return st;
    const size_t need = search_select_ws_bytes(d, max_segments, budget);
    if (!ws || ws_bytes < need)
        return fail(SABLOCK_ERR_WORKSPACE_TOO_SMALL, "sablock_search_select: workspace %zu < %zu bytes", ws_bytes, need);
    return dev(launch_search_select(d, s_tilde, sv, cl, budget, tau, seg_budget_out, block_size_out, topb_out, idx_out,
                                    n_sel_out, ws, static_cast<hipStream_t>(stream)), "sablock_search_select");
}

sablock_status sablock_compact(const sablock_shape *shape, const void *k, const void *v,
                               const int32_t *idx, const int32_t *n_sel, int32_t budget,
                               int32_t append_window, void *k_out, void *v_out, void *stream)
{
    Dims d;
    sablock_status st = make_dims(shape, &d);
    if (st != SABLOCK_OK) return st;
    if (budget < 0) return fail(SABLOCK_ERR_INVALID_ARG, "sablock_compact: budget < 0");
    if (!k || !v || !n_sel || (!idx && budget > 0)) return fail(SABLOCK_ERR_INVALID_ARG, "sablock_compact: NULL argument");
    const int rows = budget + (append_window ? d.W : 0);
    if (rows > 0 && (!k_out || !v_out)) return fail(SABLOCK_ERR_INVALID_ARG, "sablock_compact: NULL output");
    if (!aligned16(k) || !aligned16(v) || !aligned16(k_out) || !aligned16(v_out))
        return fail(SABLOCK_ERR_INVALID_ARG, "sablock_compact: K/V buffers must be 16-byte aligned");
    if (shape->v_stride[3] < d.D) return fail(SABLOCK_ERR_INVALID_ARG, "sablock_compact: V token stride smaller than head_dim");
    return dev(launch_compact(d, k, v, idx, n_sel, budget, append_window, k_out, v_out, 0,
                              static_cast<hipStream_t>(stream)), "sablock_compact");
}

sablock_status sablock_compact_shared(const sablock_shape *shape, const void *k, const void *v,
                                      const int32_t *idx, const int32_t *n_sel, int32_t budget,
                                      int32_t append_window, void *k_out, void *v_out, void *stream)
{
    Dims d;
    sablock_status st = make_dims(shape, &d);
    if (st != SABLOCK_OK) return st;
    if (budget < 0) return fail(SABLOCK_ERR_INVALID_ARG, "sablock_compact_shared: budget < 0");
    if (!k || !v || !n_sel || (!idx && budget > 0)) return fail(SABLOCK_ERR_INVALID_ARG, "sablock_compact_shared: NULL argument");
    const int rows = budget + (append_window ? d.W : 0);
    if (rows > 0 && (!k_out || !v_out)) return fail(SABLOCK_ERR_INVALID_ARG, "sablock_compact_shared: NULL output");
    if (!aligned16(k) || !aligned16(v) || !aligned16(k_out) || !aligned16(v_out))
        return fail(SABLOCK_ERR_INVALID_ARG, "sablock_compact_shared: K/V buffers must be 16-byte aligned");
    if (shape->v_stride[3] < d.D) return fail(SABLOCK_ERR_INVALID_ARG, "sablock_compact_shared: V token stride smaller than head_dim");
    return dev(launch_compact(d, k, v, idx, n_sel, budget, append_window, k_out, v_out, 1,
                              static_cast<hipStream_t>(stream)), "sablock_compact_shared");
}

sablock_status sablock_score_all_heads_workspace_bytes(const sablock_shape *shape, size_t *bytes_out)
{
    if (!bytes_out) return fail(SABLOCK_ERR_INVALID_ARG, "bytes_out is NULL");
    Dims d;
    sablock_status st = make_dims(shape, &d);
    if (st != SABLOCK_OK) return st;
    if (!score_all_heads_supported(d))
        return fail(SABLOCK_ERR_UNSUPPORTED, "sablock_score_all_heads: needs bf16, head_dim 128, a window of 8, 16 or 32 and at most 128 window-query rows per KV head");
    *bytes_out = score_all_heads_ws_bytes(d);
    return SABLOCK_OK;
}

sablock_status sablock_score_all_heads(const sablock_shape *shape, const void *q_win, const void *k,
                                       const float *row_lse, float eps, float *s_out, float *ent_out,
                                       void *ws, size_t ws_bytes, void *stream)
{
    Dims d;
    sablock_status st = make_dims(shape, &d);
    if (st != SABLOCK_OK) return st;
    if (!q_win || !k || !s_out || !ent_out) return fail(SABLOCK_ERR_INVALID_ARG, "sablock_score_all_heads: NULL argument");
    if (!aligned16(q_win) || !aligned16(k)) return fail(SABLOCK_ERR_INVALID_ARG, "sablock_score_all_heads: Q/K must be 16-byte aligned");
    if (!(eps > 0.f)) return fail(SABLOCK_ERR_INVALID_ARG, "sablock_score_all_heads: eps must be > 0");
    if (!score_all_heads_supported(d))
        return fail(SABLOCK_ERR_UNSUPPORTED, "sablock_score_all_heads: needs bf16, head_dim 128, a window of 8, 16 or 32 and at most 128 window-query rows per KV head");
    const size_t need = score_all_heads_ws_bytes(d);
    if (!ws || ws_bytes < need)
        return fail(SABLOCK_ERR_WORKSPACE_TOO_SMALL, "sablock_score_all_heads: workspace %zu < %zu bytes", ws_bytes, need);
    return dev(launch_score_all_heads(d, q_win, k, row_lse, eps, s_out, ent_out, ws, static_cast<hipStream_t>(stream)),
               "sablock_score_all_heads");
}

sablock_status sablock_window_attention_workspace_bytes(const sablock_shape *shape, size_t *bytes_out)
{
    if (!bytes_out) return fail(SABLOCK_ERR_INVALID_ARG, "bytes_out is NULL");
    Dims d;
    sablock_status st = make_dims(shape, &d);
    if (st != SABLOCK_OK) return st;
    if (!window_attention_supported(d))
        return fail(SABLOCK_ERR_UNSUPPORTED, "sablock_window_attention: needs bf16, head_dim 128, a window of 8, 16, 32 or 64 and 32, 64, 128 or 256 window-query rows per KV head");
    *bytes_out = window_attention_ws_bytes(d);
    return SABLOCK_OK;
}

sablock_status sablock_window_attention(const sablock_shape *shape, const void *q_win, const void *k, const void *v,
                                        float *out, float *row_lse_out, void *ws, size_t ws_bytes, void *stream)
{
    Dims d;
    sablock_status st = make_dims(shape, &d);
    if (st != SABLOCK_OK) return st;
    if (!q_win || !k || !v || !out || !row_lse_out) return fail(SABLOCK_ERR_INVALID_ARG, "sablock_window_attention: NULL argument");
    if (!aligned16(q_win) || !aligned16(k) || !aligned16(v))
        return fail(SABLOCK_ERR_INVALID_ARG, "sablock_window_attention: Q/K/V must be 16-byte aligned");
    if (shape->v_stride[3] < d.D) return fail(SABLOCK_ERR_INVALID_ARG, "sablock_window_attention: V token stride smaller than head_dim");
    if (!window_attention_supported(d))
        return fail(SABLOCK_ERR_UNSUPPORTED, "sablock_window_attention: needs bf16, head_dim 128, a window of 8, 16, 32 or 64 and 32, 64, 128 or 256 window-query rows per KV head");
    const size_t need = window_attention_ws_bytes(d);
    if (!ws || ws_bytes < need)
        return fail(SABLOCK_ERR_WORKSPACE_TOO_SMALL, "sablock_window_attention: workspace %zu < %zu bytes", ws_bytes, need);
    return dev(launch_window_attention(d, q_win, k, v, out, row_lse_out, ws, static_cast<hipStream_t>(stream)),
               "sablock_window_attention");
}

static sablock_status make_delims(const int32_t *delims, int32_t n_delim, DelimSet *ds)
{
    if (n_delim < 0 || (n_delim > 0 && !delims)) return fail(SABLOCK_ERR_INVALID_ARG, "delims is NULL or n_delim < 0");
    if (n_delim > MAX_DELIM) return fail(SABLOCK_ERR_UNSUPPORTED, "n_delim %d: at most %d", n_delim, MAX_DELIM);
    ds->n = n_delim;
    for (int i = 0; i < MAX_DELIM; ++i) ds->id[i] = i < n_delim ? delims[i] : 0;
    return SABLOCK_OK;
}

sablock_status sablock_segment_count(const int32_t *token_ids, int64_t token_stride, int32_t n_seq, int32_t n_tokens,
                                     const int32_t *delims, int32_t n_delim, int32_t *seg_count_out, void *stream)
{
    if (!token_ids || !seg_count_out) return fail(SABLOCK_ERR_INVALID_ARG, "sablock_segment_count: NULL argument");
    if (n_seq < 1 || n_tokens < 1 || token_stride < n_tokens)
        return fail(SABLOCK_ERR_INVALID_ARG, "sablock_segment_count: need n_seq >= 1, n_tokens >= 1, token_stride >= n_tokens");
    if (n_seq > MAX_SEQ) return fail(SABLOCK_ERR_UNSUPPORTED, "n_seq %d: at most %d per call", n_seq, MAX_SEQ);
    DelimSet ds;
    sablock_status st = make_delims(delims, n_delim, &ds);
    if (st != SABLOCK_OK) return st;
    return dev(launch_segment_count(token_ids, token_stride, n_seq, n_tokens, ds, seg_count_out,
                                    static_cast<hipStream_t>(stream)), "sablock_segment_count");
}

sablock_status sablock_segment_offsets(const int32_t *token_ids, int64_t token_stride, int32_t n_seq, int32_t n_tokens,
                                       const int32_t *delims, int32_t n_delim, const int32_t *seg_ptr,
                                       int32_t *seg_off_out, void *stream)
{
    if (!token_ids || !seg_ptr || !seg_off_out) return fail(SABLOCK_ERR_INVALID_ARG, "sablock_segment_offsets: NULL argument");
    if (n_seq < 1 || n_tokens < 1 || token_stride < n_tokens)
        return fail(SABLOCK_ERR_INVALID_ARG, "sablock_segment_offsets: need n_seq >= 1, n_tokens >= 1, token_stride >= n_tokens");
    if (n_seq > MAX_SEQ) return fail(SABLOCK_ERR_UNSUPPORTED, "n_seq %d: at most %d per call", n_seq, MAX_SEQ);
    SeqPtr sp;
    if (seg_ptr[0] < 0) return fail(SABLOCK_ERR_INVALID_ARG, "seg_ptr[0] < 0");
    for (int s = 0; s <= MAX_SEQ; ++s) sp.ptr[s] = seg_ptr[s < n_seq ? s : n_seq];
    for (int s = 0; s < n_seq; ++s) {
        const int n = seg_ptr[s + 1] - seg_ptr[s];
        if (n < 2 || n > n_tokens + 1)
            return fail(SABLOCK_ERR_INVALID_ARG, "sequence %d: seg_ptr leaves %d offsets, need 2 .. n_tokens + 1", s, n);
    }
    DelimSet ds;
    sablock_status st = make_delims(delims, n_delim, &ds);
    if (st != SABLOCK_OK) return st;
    return dev(launch_segment_offsets(token_ids, token_stride, n_seq, n_tokens, ds, sp, seg_off_out,
                                      static_cast<hipStream_t>(stream)), "sablock_segment_offsets");
}

sablock_status sablock_validate_segments(const int32_t *seg_off, const int32_t *seg_ptr, int32_t n_seq, int32_t n_tokens,
                                         int32_t *n_bad_out, void *stream)
{
    if (!seg_off || !seg_ptr || !n_bad_out) return fail(SABLOCK_ERR_INVALID_ARG, "sablock_validate_segments: NULL argument");
    if (n_seq < 1 || n_tokens < 1) return fail(SABLOCK_ERR_INVALID_ARG, "sablock_validate_segments: need n_seq >= 1, n_tokens >= 1");
    if (n_seq > MAX_SEQ) return fail(SABLOCK_ERR_UNSUPPORTED, "n_seq %d: at most %d per call", n_seq, MAX_SEQ);
    if (seg_ptr[0] < 0) return fail(SABLOCK_ERR_INVALID_ARG, "seg_ptr[0] < 0");
    SeqPtr sp;
    for (int s = 0; s <= MAX_SEQ; ++s) sp.ptr[s] = seg_ptr[s < n_seq ? s : n_seq];
    for (int s = 0; s < n_seq; ++s) {
        const int n = seg_ptr[s + 1] - seg_ptr[s];
        if (n < 2 || n > n_tokens + 1)
            return fail(SABLOCK_ERR_INVALID_ARG, "sequence %d: seg_ptr leaves %d offsets, need 2 .. n_tokens + 1", s, n);
    }
    return dev(launch_segment_check(seg_off, n_seq, n_tokens, sp, n_bad_out, static_cast<hipStream_t>(stream)),
               "sablock_validate_segments");
}

static sablock_status make_cache_dims(const sablock_shape *shape, Dims *d)
{
    if (!shape) return fail(SABLOCK_ERR_INVALID_ARG, "shape is NULL");
    if (shape->seq_len < 2) return fail(SABLOCK_ERR_INVALID_ARG, "decode: the cache needs at least 2 rows");
    sablock_shape s = *shape;
    s.window = 1;                                  // not used by the decode kernels
    s.q_stride[0] = (int64_t)s.n_layers * s.n_q_heads * s.head_dim;   // q is dense
    s.q_stride[1] = (int64_t)s.n_q_heads * s.head_dim;
    s.q_stride[2] = s.q_stride[3] = s.head_dim;
    sablock_status st = make_dims(&s, d);
    if (st != SABLOCK_OK) return st;
    if (!decode_supported(*d))
        return fail(SABLOCK_ERR_UNSUPPORTED, "decode: need G <= 8, head_dim * element size / 16 a power of two in [4, 64], G * head_dim <= 1024");
    return SABLOCK_OK;
}

sablock_status sablock_decode_workspace_bytes(const sablock_shape *shape, size_t *bytes_out)
{
    if (!bytes_out) return fail(SABLOCK_ERR_INVALID_ARG, "bytes_out is NULL");
    Dims d;
    sablock_status st = make_cache_dims(shape, &d);
    if (st != SABLOCK_OK) return st;
    *bytes_out = decode_ws_bytes(d);
    return SABLOCK_OK;
}

sablock_status sablock_decode_attention(const sablock_shape *shape, const void *q, const void *k_cache,
                                        const void *v_cache, const int32_t *n_sel, int32_t budget, float *out,
                                        void *ws, size_t ws_bytes, void *stream)
{
    Dims d;
    sablock_status st = make_cache_dims(shape, &d);
    if (st != SABLOCK_OK) return st;
    if (!q || !k_cache || !v_cache || !out) return fail(SABLOCK_ERR_INVALID_ARG, "sablock_decode_attention: NULL argument");
    if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache))
        return fail(SABLOCK_ERR_INVALID_ARG, "sablock_decode_attention: q/K/V must be 16-byte aligned");
    if (n_sel && (budget < 0 || budget > d.L)) return fail(SABLOCK_ERR_INVALID_ARG, "sablock_decode_attention: need 0 <= budget <= rows");
    if (shape->v_stride[3] < d.D) return fail(SABLOCK_ERR_INVALID_ARG, "sablock_decode_attention: V row stride smaller than head_dim");
    const size_t need = decode_ws_bytes(d);
    if (!ws || ws_bytes < need)
        return fail(SABLOCK_ERR_WORKSPACE_TOO_SMALL, "sablock_decode_attention: workspace %zu < %zu bytes", ws_bytes, need);
    return dev(launch_decode(d, q, k_cache, v_cache, n_sel, budget, out, ws, static_cast<hipStream_t>(stream)),
               "sablock_decode_attention");
}

}  // extern "C"
