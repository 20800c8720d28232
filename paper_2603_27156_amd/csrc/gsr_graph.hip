// Graph construction: adjacency A of Section 3 of the paper as a device CSR, its transpose
// for the backward pass (gradients flow through G^T), the symmetric GCN normalisation, and
// the split plan for very long rows.  Also: error strings, options, workspace carving.
#include "gsr_internal.h"

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <numeric>
#include <vector>

namespace gsr {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

gsr_status_t fail(gsr_status_t st, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}

Options& options() {
    static Options o;
    return o;
}

// ---- per-kernel timing ------------------------------------------------------------------------
struct ProfRec {
    int kc;
    hipEvent_t e0, e1;
};
static std::vector<ProfRec> g_prof_open;          // recorded, not yet read
static std::vector<std::pair<hipEvent_t, hipEvent_t>> g_prof_pool;
static double g_prof_ms[KC_COUNT];
static int64_t g_prof_n[KC_COUNT];

ProfScope::ProfScope(KernelClass kc, hipStream_t s) : slot(-1), stream(s) {
    if (!((options().profile >> kc) & 1)) return;
    ProfRec r;
    r.kc = kc;
    if (!g_prof_pool.empty()) {
        r.e0 = g_prof_pool.back().first;
        r.e1 = g_prof_pool.back().second;
        g_prof_pool.pop_back();
    } else if (hipEventCreate(&r.e0) != hipSuccess || hipEventCreate(&r.e1) != hipSuccess) {
        return;
    }
    if (hipEventRecord(r.e0, s) != hipSuccess) return;
    g_prof_open.push_back(r);
    slot = (int)g_prof_open.size() - 1;
}

ProfScope::~ProfScope() {
    if (slot >= 0) (void)hipEventRecord(g_prof_open[slot].e1, stream);
}

static void prof_collect() {
    for (ProfRec& r : g_prof_open) {
        float ms = 0.f;
        if (hipEventSynchronize(r.e1) == hipSuccess && hipEventElapsedTime(&ms, r.e0, r.e1) == hipSuccess) {
            g_prof_ms[r.kc] += ms;
            g_prof_n[r.kc] += 1;
        }
        g_prof_pool.emplace_back(r.e0, r.e1);
    }
    g_prof_open.clear();
}

// ---- normalisation kernels ----------------------------------------------------------------

// dinv[i] = 1/sqrt(stored length of row i), float32, correctly rounded divide and sqrt.
__global__ void k_dinv(int n, const int32_t* __restrict__ rp, float* __restrict__ dinv) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dinv[i] = 1.0f / sqrtf((float)(rp[i + 1] - rp[i]));
}

// a_ij = dinv_i * dinv_j for every stored entry; one thread per row chunk keeps it simple and
// the work is done once per graph.
__global__ void k_gcn_values(int n, const int32_t* __restrict__ rp, const int32_t* __restrict__ ci,
                             const float* __restrict__ dinv, float* __restrict__ av) {
    int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    int lane = threadIdx.x & 63;
    int nwaves = (gridDim.x * blockDim.x) >> 6;
    for (int i = wave; i < n; i += nwaves) {
        float di = dinv[i];
        for (int e = rp[i] + lane; e < rp[i + 1]; e += 64) av[e] = di * dinv[ci[e]];
    }
}

__global__ void k_fill(int64_t n, float v, float* __restrict__ out) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = v;
}

static gsr_status_t normalise_csr(const Csr& c, int64_t n, int64_t nnz, int32_t mode, hipStream_t s,
                                  float* dinv_scratch) {
    if (nnz == 0 || n == 0) return GSR_OK;
    if (mode == GSR_ADJ_UNIT) {
        hipLaunchKernelGGL(k_fill, dim3((unsigned)((nnz + 255) / 256)), dim3(256), 0, s, nnz, 1.0f, c.av);
    } else {
        hipLaunchKernelGGL(k_dinv, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, (int)n, c.rp, dinv_scratch);
        int blocks = (int)std::min<int64_t>((n + 3) / 4, 4096);
        hipLaunchKernelGGL(k_gcn_values, dim3(blocks), dim3(256), 0, s, (int)n, c.rp, c.ci, dinv_scratch, c.av);
    }
    GSR_HIP_CHECK(hipGetLastError());
    return GSR_OK;
}

// ---- host-side structure building -----------------------------------------------------------

struct HostCsr {
    std::vector<int32_t> rp;
    std::vector<int32_t> ci;
    std::vector<float> av;
};

static void free_csr(Csr& c) {
    if (c.rp) (void)hipFree(c.rp);
    if (c.ci) (void)hipFree(c.ci);
    if (c.av) (void)hipFree(c.av);
    if (c.hub.rows) (void)hipFree(c.hub.rows);
    if (c.hub.cptr) (void)hipFree(c.hub.cptr);
    if (c.hub.tile0) (void)hipFree(c.hub.tile0);
    if (c.hub.crow) (void)hipFree(c.hub.crow);
    if (c.hub.ce0) (void)hipFree(c.hub.ce0);
    if (c.hub.ce1) (void)hipFree(c.hub.ce1);
    if (c.heavy) (void)hipFree(c.heavy);
    c = Csr();
}

template <typename V>
static gsr_status_t upload(const std::vector<V>& h, V** d) {
    size_t bytes = std::max<size_t>(h.size(), 1) * sizeof(V);
    GSR_HIP_CHECK(hipMalloc((void**)d, bytes));
    if (!h.empty()) GSR_HIP_CHECK(hipMemcpy(*d, h.data(), h.size() * sizeof(V), hipMemcpyHostToDevice));
    return GSR_OK;
}

static gsr_status_t upload_csr(const HostCsr& h, int64_t n, int64_t threshold, int64_t chunk, Csr* out) {
    std::vector<int32_t> heavy;
    for (int64_t t0 = 0; t0 < n; t0 += 16) {
        int64_t e = 0;      // stored entries of the tile's rows that are not split
        for (int64_t r = t0; r < std::min<int64_t>(n, t0 + 16); ++r) {
            const int64_t d = h.rp[r + 1] - h.rp[r];
            e += d > threshold ? 0 : d;
        }
        if (e > kHeavyTileEdges) heavy.push_back((int32_t)(t0 / 16));
    }
    out->n_heavy = (int32_t)heavy.size();
    GSR_TRY(upload(heavy, &out->heavy));
    GSR_TRY(upload(h.rp, &out->rp));
    GSR_TRY(upload(h.ci, &out->ci));
    GSR_TRY(upload(h.av, &out->av));
    std::vector<int32_t> rows, cptr, crow, ce0, ce1, tile0;
    cptr.push_back(0);
    for (int64_t i = 0; i < n; ++i) {
        if ((i & 15) == 0) tile0.push_back((int32_t)rows.size());
        int64_t len = h.rp[i + 1] - h.rp[i];
        if (len <= threshold) continue;
        rows.push_back((int32_t)i);
        for (int64_t e = h.rp[i]; e < h.rp[i + 1]; e += chunk) {
            crow.push_back((int32_t)i);
            ce0.push_back((int32_t)e);
            ce1.push_back((int32_t)std::min<int64_t>(e + chunk, h.rp[i + 1]));
        }
        cptr.push_back((int32_t)crow.size());
    }
    tile0.push_back((int32_t)rows.size());
    out->hub.n_hub = (int32_t)rows.size();
    out->hub.n_chunks = (int32_t)crow.size();
    GSR_TRY(upload(tile0, &out->hub.tile0));
    GSR_TRY(upload(rows, &out->hub.rows));
    GSR_TRY(upload(cptr, &out->hub.cptr));
    GSR_TRY(upload(crow, &out->hub.crow));
    GSR_TRY(upload(ce0, &out->hub.ce0));
    GSR_TRY(upload(ce1, &out->hub.ce1));
    return GSR_OK;
}

// Sort the columns of every row, merge duplicates (values summed).
static void canonicalise(int64_t n, std::vector<int64_t>& rp64, std::vector<int32_t>& ci, std::vector<float>& av,
                         HostCsr* out) {
    out->rp.assign(n + 1, 0);
    out->ci.clear();
    out->av.clear();
    out->ci.reserve(ci.size());
    out->av.reserve(ci.size());
    std::vector<std::pair<int32_t, float>> row;
    for (int64_t i = 0; i < n; ++i) {
        row.clear();
        for (int64_t e = rp64[i]; e < rp64[i + 1]; ++e) row.emplace_back(ci[e], av[e]);
        std::stable_sort(row.begin(), row.end(),
                         [](const std::pair<int32_t, float>& a, const std::pair<int32_t, float>& b) {
                             return a.first < b.first;
                         });
        for (size_t p = 0; p < row.size(); ++p) {
            if (p > 0 && row[p].first == row[p - 1].first) {
                out->av.back() += row[p].second;
            } else {
                out->ci.push_back(row[p].first);
                out->av.push_back(row[p].second);
            }
        }
        out->rp[i + 1] = (int32_t)out->ci.size();
    }
}

static void transpose_host(int64_t n, const HostCsr& a, HostCsr* t) {
    int64_t nnz = (int64_t)a.ci.size();
    t->rp.assign(n + 1, 0);
    t->ci.assign(nnz, 0);
    t->av.assign(nnz, 0.f);
    for (int64_t e = 0; e < nnz; ++e) t->rp[a.ci[e] + 1]++;
    for (int64_t i = 0; i < n; ++i) t->rp[i + 1] += t->rp[i];
    std::vector<int32_t> fill(t->rp.begin(), t->rp.end() - 1);
    for (int64_t i = 0; i < n; ++i)
        for (int32_t e = a.rp[i]; e < a.rp[i + 1]; ++e) {
            int32_t p = fill[a.ci[e]]++;
            t->ci[p] = (int32_t)i;
            t->av[p] = a.av[e];
        }
}

// The tile counters of a graph's dynamic sweeps and, behind them, the nine counters its waves sign off
// in.  Both are zero between launches (clear when the graph is created; every launch clears them again).
void tile_counters(const gsr_graph_t* g, int** set, int** done) {
    *set = g->draws;
    *done = g->draws + kTileCounters;
}

LayerWs carve_layer(const gsr_config_t* cfg, const gsr_graph_t* g) {
    LayerWs w;
    memset(&w, 0, sizeof(w));
    size_t n = (size_t)cfg->n, dg = (size_t)(cfg->d / cfg->c), b = dtype_size(cfg->dtype);
    const int S = sub_planes(cfg);
    const size_t dgs = dg / S;                       // columns of a tile: 32 or 64
    size_t off = 0;
    for (int s = 0; s < cfg->c * S && s < kMaxRecordSlots; ++s) {
        w.rec_vals[s] = off;
        off += align_up(n * (size_t)cfg->k * b + 16);   // the record gather loads up to 16 bytes past a record
        w.rec_mask[s] = off;
        off += align_up(n * (dgs == 32 ? 4 : 8));
    }
    w.y0 = off;
    off += align_up(n * dg * b);
    w.dh = off;
    if (S > 1) off += align_up(n * dg * sizeof(float));
    w.dw_partial = off;
    off += align_up((size_t)g->grid * dgs * dgs * sizeof(float) * (size_t)(S * S));      // (wide groups: a set per block of dW_i)
    w.hub_partial = off;
    size_t chunks = (size_t)std::max(g->a.hub.n_chunks, g->at.hub.n_chunks);
    // (wide groups summed value by value: the partial rows of all S column blocks from one pass, [S][chunks][64])
    const bool wide_values = S > 1 && b == 4 && g->hub_values;
    off += align_up(std::max<size_t>(chunks, 1) * dgs * (wide_values ? S : 1) * sizeof(float));
    w.hub_partial2 = off;
    off += align_up(std::max<size_t>(chunks, 1) * dgs * sizeof(float));
    w.hub_cols = off;
    if (b == 4 && g->hub_values) off += align_up(n * (size_t)cfg->k + 16);
    w.hub_vals = off;
    if (wide_values) off += align_up(n * (size_t)cfg->k * sizeof(float) + 16);
    w.h = off;               // (not for 16-bit storage at 32 columns: that backward keeps H on chip)
    if ((b == 4 || dgs == 64) && g->split_backward) off += align_up(n * dgs * sizeof(float));
    w.total = off;
    return w;
}

StepWs carve_step(const gsr_config_t* cfg, const gsr_graph_t* g) {
    StepWs w;
    size_t n = (size_t)cfg->n, b = dtype_size(cfg->dtype);
    size_t off = 0;
    w.act = off;
    off += align_up(n * (size_t)cfg->d * b);
    w.grad = off;
    off += align_up(n * (size_t)cfg->d * b);
    w.head = off;
    off += align_up((size_t)g->grid * ((size_t)cfg->d + 2) * sizeof(float));
    w.layer = off;
    off += carve_layer(cfg, g).total;
    w.masks = off;
    const size_t segs = ((size_t)(cfg->l > 0 ? cfg->l : 0) + 1) * (size_t)cfg->c;
    if (cfg->save_indices == 1) off += align_up(segs * n * (size_t)(cfg->d / cfg->c / 8));
    w.tie_counts = w.tie_rows = w.tie_masks = off;
    w.tie_cap = 0;
    if (cfg->save_indices == 2) {
        w.tie_cap = (tie_capacity(cfg) + kTieSub - 1) / kTieSub;           // places per sub-list
        off += align_up(segs * kTieSub * kTieCounterStride * sizeof(int));
        w.tie_rows = off;
        off += align_up(segs * kTieSub * (size_t)w.tie_cap * sizeof(uint32_t));
        w.tie_masks = off;
        off += align_up(segs * kTieSub * (size_t)w.tie_cap * (size_t)(std::min(cfg->d / cfg->c, 64) / 8));
    }
    w.total = off;
    return w;
}

int64_t tie_capacity(const gsr_config_t* cfg) {
    if (cfg->tie_capacity > 0) return cfg->tie_capacity;
    return cfg->n / 32 + 1024;
}

gsr_status_t validate_config(const gsr_config_t* cfg, const gsr_graph_t* g, bool need_l) {
    if (!cfg || !g) return fail(GSR_ERR_INVALID_ARG, "null config or graph");
    if (cfg->n != g->n) return fail(GSR_ERR_INVALID_ARG, "config n=%lld differs from graph n=%lld",
                                    (long long)cfg->n, (long long)g->n);
    if (cfg->c < 2 || cfg->c > 8) return fail(GSR_ERR_UNSUPPORTED, "groups C=%d outside [2,8]", cfg->c);
    if (cfg->d <= 0 || cfg->d % cfg->c != 0) return fail(GSR_ERR_UNSUPPORTED, "D=%d not divisible by C=%d", cfg->d, cfg->c);
    int dg = cfg->d / cfg->c;
    if (dg != 32 && dg != 64 && dg != 128 && dg != 192 && dg != 256)
        return fail(GSR_ERR_UNSUPPORTED, "D/C=%d: 32, 64, 128, 192 and 256 are built", dg);
    if (dg > 64 && cfg->save_indices == 2)
        return fail(GSR_ERR_UNSUPPORTED, "save_indices = 2 is built for D/C <= 64; use 0 or 1 with D/C=%d", dg);
    if (cfg->k < 1 || cfg->k > dg) return fail(GSR_ERR_UNSUPPORTED, "k=%d outside [1, D/C=%d]", cfg->k, dg);
    if (cfg->dtype != GSR_F32 && cfg->dtype != GSR_BF16) return fail(GSR_ERR_UNSUPPORTED, "dtype %d", cfg->dtype);
    if (cfg->norm != GSR_NORM_NONE && cfg->norm != GSR_NORM_RMS) return fail(GSR_ERR_UNSUPPORTED, "norm %d", cfg->norm);
    if (cfg->layout != GSR_LAYOUT_ROW_MAJOR && cfg->layout != GSR_LAYOUT_GROUP_PLANAR)
        return fail(GSR_ERR_UNSUPPORTED, "layout %d", cfg->layout);
    if ((uint64_t)cfg->n * (uint64_t)cfg->k >= ((uint64_t)1 << 32))
        return fail(GSR_ERR_UNSUPPORTED, "n * k = %llu does not fit 32-bit record offsets", (unsigned long long)cfg->n * cfg->k);
    if (need_l && cfg->l < 1) return fail(GSR_ERR_INVALID_ARG, "layers L=%d", cfg->l);
    if (!(cfg->eps >= 0.f)) return fail(GSR_ERR_INVALID_ARG, "eps must be >= 0");
    if (cfg->save_indices < 0 || cfg->save_indices > 2) return fail(GSR_ERR_INVALID_ARG, "save_indices must be 0, 1 or 2");
    if (cfg->save_indices == 2 && (!(cfg->tie_tol >= 0.f) || cfg->tie_capacity < 0))
        return fail(GSR_ERR_INVALID_ARG, "tie_tol and tie_capacity must be >= 0");
    return GSR_OK;
}

}  // namespace gsr

using namespace gsr;

extern "C" {

const char* gsr_last_error(void) { return g_err; }
const char* gsr_version(void) { return "gsr-mi355x 0.1 (gfx950)"; }

gsr_status_t gsr_set_option(const char* key, int64_t value) {
    if (!key) return fail(GSR_ERR_INVALID_ARG, "null key");
    Options& o = options();
    if (!strcmp(key, "hub_threshold")) {
        if (value < 0) return fail(GSR_ERR_INVALID_ARG, "hub_threshold must be >= 0");
        o.hub_threshold = value;
    } else if (!strcmp(key, "hub_chunk")) {
        if (value < 0) return fail(GSR_ERR_INVALID_ARG, "hub_chunk must be >= 0");
        o.hub_chunk = value;
    } else if (!strcmp(key, "hub_values")) {
        if (value < 0 || value > 2) return fail(GSR_ERR_INVALID_ARG, "hub_values must be 0, 1 or 2");
        o.hub_values = value;
    } else if (!strcmp(key, "max_workgroups")) {
        if (value < 0 || value % 8 != 0) return fail(GSR_ERR_INVALID_ARG, "max_workgroups must be a multiple of 8");
        o.max_workgroups = value;
    } else if (!strcmp(key, "profile")) {
        if (value < 0 || value >= ((int64_t)1 << KC_COUNT)) return fail(GSR_ERR_INVALID_ARG, "profile mask out of range");
        o.profile = value;
    } else {
        return fail(GSR_ERR_INVALID_ARG, "unknown option '%s'", key);
    }
    return GSR_OK;
}

gsr_status_t gsr_profile_read(int32_t kernel_class, double* total_ms, int64_t* launches) {
    if (kernel_class < 0 || kernel_class >= KC_COUNT) return fail(GSR_ERR_INVALID_ARG, "kernel class %d", kernel_class);
    prof_collect();
    if (total_ms) *total_ms = g_prof_ms[kernel_class];
    if (launches) *launches = g_prof_n[kernel_class];
    return GSR_OK;
}

gsr_status_t gsr_profile_reset(void) {
    prof_collect();
    for (int i = 0; i < KC_COUNT; ++i) { g_prof_ms[i] = 0.0; g_prof_n[i] = 0; }
    return GSR_OK;
}

const char* gsr_profile_class_name(int32_t kernel_class) {
    static const char* names[KC_COUNT] = {"block_forward", "block_inverse", "block_backward", "grad", "group_sum",
                                          "hub_first_pass", "dw_reduce", "head", "layout_copy", "tie_fixup", "weight_gradient"};
    return (kernel_class >= 0 && kernel_class < KC_COUNT) ? names[kernel_class] : "";
}

static gsr_status_t graph_create_impl(gsr_graph_t** out, int64_t n, int64_t nnz, const void* rowptr,
                                      const int32_t* colidx, const float* vals, uint32_t flags, void* stream);

gsr_status_t gsr_graph_create(gsr_graph_t** out, int64_t n, int64_t nnz, const void* rowptr,
                              const int32_t* colidx, const float* vals, uint32_t flags, void* stream) {
    // the host-side preprocessing holds several arrays of nnz entries: running out of host memory is a status,
    // not an exception across the C boundary
    try {
        return graph_create_impl(out, n, nnz, rowptr, colidx, vals, flags, stream);
    } catch (const std::bad_alloc&) {
        if (out) *out = nullptr;
        return fail(GSR_ERR_INVALID_ARG, "out of host memory while preprocessing %lld rows / %lld entries", (long long)n, (long long)nnz);
    } catch (...) {
        if (out) *out = nullptr;
        return fail(GSR_ERR_INVALID_ARG, "unexpected failure while preprocessing the graph");
    }
}

static gsr_status_t graph_create_impl(gsr_graph_t** out, int64_t n, int64_t nnz, const void* rowptr,
                                      const int32_t* colidx, const float* vals, uint32_t flags, void* stream) {
    if (!out) return fail(GSR_ERR_INVALID_ARG, "out is null");
    *out = nullptr;
    if (n < 0 || nnz < 0) return fail(GSR_ERR_INVALID_ARG, "negative size");
    if (!rowptr || (nnz > 0 && !colidx)) return fail(GSR_ERR_INVALID_ARG, "null CSR array");
    if (n >= (int64_t)1 << 31) return fail(GSR_ERR_UNSUPPORTED, "n >= 2^31");
    if ((flags & GSR_GRAPH_GCN_NORM) && vals) return fail(GSR_ERR_INVALID_ARG, "GCN_NORM and explicit values are exclusive");

    // ---- validate and widen the input
    std::vector<int64_t> rp64(n + 1);
    for (int64_t i = 0; i <= n; ++i)
        rp64[i] = (flags & GSR_GRAPH_ROWPTR_I64) ? ((const int64_t*)rowptr)[i] : (int64_t)((const int32_t*)rowptr)[i];
    if (rp64[0] != 0 || rp64[n] != nnz) return fail(GSR_ERR_BAD_CSR, "rowptr[0]=%lld, rowptr[n]=%lld, nnz=%lld",
                                                    (long long)rp64[0], (long long)rp64[n], (long long)nnz);
    for (int64_t i = 0; i < n; ++i)
        if (rp64[i + 1] < rp64[i]) return fail(GSR_ERR_BAD_CSR, "row pointers decrease at row %lld", (long long)i);
    for (int64_t e = 0; e < nnz; ++e)
        if (colidx[e] < 0 || colidx[e] >= n) return fail(GSR_ERR_BAD_CSR, "column %d out of range at entry %lld", colidx[e], (long long)e);

    // ---- pattern transforms: symmetrise, self-loops
    std::vector<int64_t> rp2;
    std::vector<int32_t> ci2;
    std::vector<float> av2;
    const bool sym = flags & GSR_GRAPH_SYMMETRISE, loops = flags & GSR_GRAPH_ADD_SELF_LOOPS;
    if (sym || loops) {
        std::vector<int64_t> cnt(n + 1, 0);
        for (int64_t i = 0; i < n; ++i) {
            for (int64_t e = rp64[i]; e < rp64[i + 1]; ++e) {
                int32_t j = colidx[e];
                if (loops && j == i) continue;      // existing diagonal entries collapse into the one self-loop
                cnt[i + 1]++;
                if (sym && j != i) cnt[j + 1]++;
            }
            if (loops) cnt[i + 1]++;
        }
        for (int64_t i = 0; i < n; ++i) cnt[i + 1] += cnt[i];
        ci2.resize(cnt[n]);
        av2.resize(cnt[n]);
        std::vector<int64_t> fill(cnt.begin(), cnt.end() - 1);
        for (int64_t i = 0; i < n; ++i) {
            if (loops) { ci2[fill[i]] = (int32_t)i; av2[fill[i]++] = 1.0f; }
            for (int64_t e = rp64[i]; e < rp64[i + 1]; ++e) {
                int32_t j = colidx[e];
                if (loops && j == i) continue;
                float v = vals ? vals[e] : 1.0f;
                ci2[fill[i]] = j; av2[fill[i]++] = v;
                if (sym && j != i) { ci2[fill[j]] = (int32_t)i; av2[fill[j]++] = v; }
            }
        }
        rp2 = cnt;
    } else {
        rp2 = rp64;
        ci2.assign(colidx, colidx + nnz);
        av2.resize(nnz);
        for (int64_t e = 0; e < nnz; ++e) av2[e] = vals ? vals[e] : 1.0f;
    }
    if ((int64_t)ci2.size() >= ((int64_t)1 << 31)) return fail(GSR_ERR_UNSUPPORTED, "more than 2^31 stored entries");
    HostCsr a;
    canonicalise(n, rp2, ci2, av2, &a);
    // duplicates of a unit-weight pattern stay unit weight (pattern union, not a multigraph)
    if (!vals) std::fill(a.av.begin(), a.av.end(), 1.0f);
    std::vector<int64_t>().swap(rp2);
    std::vector<int32_t>().swap(ci2);
    std::vector<float>().swap(av2);

    HostCsr t;
    transpose_host(n, a, &t);
    bool symmetric = (a.rp == t.rp) && (a.ci == t.ci) && (a.av == t.av);

    gsr_graph_t* g = new (std::nothrow) gsr_graph_t();
    if (!g) return fail(GSR_ERR_INVALID_ARG, "out of host memory");
    g->n = n;
    g->nnz = (int64_t)a.ci.size();
    for (int64_t i = 0; i < n; ++i) g->max_degree = std::max<int64_t>(g->max_degree, a.rp[i + 1] - a.rp[i]);
    g->symmetric = symmetric;
    g->has_transpose = true;
    // Rows above the threshold are cut into chunks that a first pass sums, one wave per chunk.  Sparse graphs with a few
    // very long rows: 512 / 64.  Graphs whose mean row is long (the 49,600-node, 11.7M-entry workload shaped like the
    // paper's Table 1: 871 ms per step with 512 / 64, 661 with 64 / 64, 566 with 64 / 256) are better served when nearly
    // every row goes through the first pass, whose lanes add a row's entries in ordinary arithmetic instead of spending
    // a 16-row matrix product on them.  Every row of two entries or more, in fact: a launch of a tile kernel is one
    // tile per wave there, and it ended with the few tiles that still had short rows to gather themselves (that stage
    // 6 us at the median, 26 us at most; 503 ms per step with the cut at 64, 460 at 32, 445 at 8, 443 at 1).
    const bool long_rows = g->nnz >= 64 * n;
    g->long_rows = long_rows;

    hipError_t e = hipGetDevice(&g->device);
    if (e != hipSuccess) { delete g; return fail(GSR_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e)); }
    hipDeviceProp_t prop;
    e = hipGetDeviceProperties(&prop, g->device);
    if (e != hipSuccess) { delete g; return fail(GSR_ERR_HIP, "hipGetDeviceProperties: %s", hipGetErrorString(e)); }
    g->num_cus = prop.multiProcessorCount;
    int grid = options().max_workgroups > 0 ? (int)options().max_workgroups : g->num_cus * 4;
    g->grid = std::max(8, grid / 8 * 8);
    const int full_grid = g->grid;
    // A graph of a few hundred tiles is served best by a workgroup per two tiles (every workgroup of a layer kernel
    // first loads and splits W_i): on the 2,000-node workload, 125 tiles, the step takes 0.35 ms with 64 workgroups
    // per launch against 0.47 with 512, 0.37 with 256, 0.40 with 16.
    if (options().max_workgroups <= 0) {
        const int64_t by_tiles = std::max<int64_t>(64, ((n + 15) / 16 / 2 + 7) / 8 * 8);
        if (by_tiles < g->grid) g->grid = (int)by_tiles;
    }
    // Small graphs (fewer than four tiles per resident wave: a launch is as long as its longest tile, and the heavy
    // tiles are not dealt out first) are cut at 64 as well, with chunks of 64: on the 100k-node workload (6,250 tiles
    // for 4,096 waves, rows of up to 575 entries) the step takes 11.5 ms against 16.0 with the cut at 512, while the
    // 1M-node workload (15 tiles per wave) is best left at 512 (79.0 ms per 16 layers against 79.7 / 82.4 / 82.7 at
    // 256 / 128 / 64).
    // With fewer than two tiles per resident wave the cut at 16 is better still (the same workload: 9.4 ms against 10.6;
    // 12 / 8: 9.6 / 9.8; chunks of 32 instead of 64: 9.7).
    const bool few_tiles = (n + 15) / 16 < (int64_t)16 * full_grid, very_few_tiles = (n + 15) / 16 < (int64_t)8 * full_grid;
    const int64_t hub_threshold = options().hub_threshold > 0 ? options().hub_threshold
                                  : long_rows ? 1 : very_few_tiles ? 16 : few_tiles ? 64 : 512;
    const int64_t hub_chunk = options().hub_chunk > 0 ? options().hub_chunk : (long_rows ? 512 : 64);      // (Table-1-shaped graph, rows of up to 390 entries: 289 / 274 / 263 / 263 ms per step with chunks of 128 / 256 / 512 / 1,024)
    g->hub_threshold = (int32_t)hub_threshold;
    g->hub_values = options().hub_values == 1 ? 2 : (options().hub_values == 0 && long_rows) ? 1 : 0;
    g->split_backward = !(long_rows || (n + 15) / 16 < (int64_t)8 * full_grid);    // (not with fewer than two tiles per resident wave)

    gsr_status_t st = upload_csr(a, n, hub_threshold, hub_chunk, &g->a);
    if (st == GSR_OK) {
        if (symmetric) g->at = g->a;
        else st = upload_csr(t, n, hub_threshold, hub_chunk, &g->at);
    }
    if (st == GSR_OK) {
        const size_t chunks = (size_t)std::max(std::max(g->a.hub.n_chunks, g->at.hub.n_chunks), 1);
        e = hipMalloc((void**)&g->scratch, chunks * 64 * sizeof(float));
        const size_t draw_bytes = (size_t)kTileCounterSet * kTileCounterSets * sizeof(int);
        if (e == hipSuccess) e = hipMalloc((void**)&g->dinv, std::max<size_t>((size_t)n, 1) * sizeof(float));
        if (e == hipSuccess) e = hipMalloc((void**)&g->draws, draw_bytes);
        if (e == hipSuccess) e = hipMemset(g->draws, 0, draw_bytes);
        if (e != hipSuccess) st = fail(GSR_ERR_HIP, "hipMalloc: %s", hipGetErrorString(e));
    }
    if (st == GSR_OK && (flags & GSR_GRAPH_GCN_NORM)) st = gsr_graph_normalize(g, GSR_ADJ_GCN_SYM, stream);
    if (st == GSR_OK) {
        e = hipStreamSynchronize((hipStream_t)stream);
        if (e != hipSuccess) st = fail(GSR_ERR_HIP, "hipStreamSynchronize: %s", hipGetErrorString(e));
    }
    if (st != GSR_OK) { gsr_graph_destroy(g); return st; }
    *out = g;
    return GSR_OK;
}

gsr_status_t gsr_graph_normalize(gsr_graph_t* g, int32_t mode, void* stream) {
    if (!g) return fail(GSR_ERR_INVALID_ARG, "graph is null");
    if (mode != GSR_ADJ_UNIT && mode != GSR_ADJ_GCN_SYM) return fail(GSR_ERR_INVALID_ARG, "unknown normalisation %d", mode);
    if (mode == GSR_ADJ_GCN_SYM && !g->symmetric)
        return fail(GSR_ERR_UNSUPPORTED, "symmetric GCN normalisation needs a symmetric stored pattern");
    hipStream_t s = (hipStream_t)stream;
    // d^-1/2 goes through a buffer the graph owns: nothing is allocated here and the call only launches kernels
    gsr_status_t st = normalise_csr(g->a, g->n, g->nnz, mode, s, g->dinv);
    if (st == GSR_OK && !g->symmetric) st = normalise_csr(g->at, g->n, g->nnz, mode, s, g->dinv);
    return st;
}

gsr_status_t gsr_graph_info(const gsr_graph_t* g, int64_t* n, int64_t* nnz, int64_t* max_degree, int64_t* n_hub_rows) {
    if (!g) return fail(GSR_ERR_INVALID_ARG, "graph is null");
    if (n) *n = g->n;
    if (nnz) *nnz = g->nnz;
    if (max_degree) *max_degree = g->max_degree;
    if (n_hub_rows) *n_hub_rows = g->a.hub.n_hub;
    return GSR_OK;
}

gsr_status_t gsr_graph_export(const gsr_graph_t* g, int64_t* rowptr, int32_t* colidx, float* vals) {
    if (!g) return fail(GSR_ERR_INVALID_ARG, "graph is null");
    GSR_HIP_CHECK(hipDeviceSynchronize());
    if (rowptr) {
        std::vector<int32_t> rp(g->n + 1);
        GSR_HIP_CHECK(hipMemcpy(rp.data(), g->a.rp, (g->n + 1) * sizeof(int32_t), hipMemcpyDeviceToHost));
        for (int64_t i = 0; i <= g->n; ++i) rowptr[i] = rp[i];
    }
    if (colidx && g->nnz) GSR_HIP_CHECK(hipMemcpy(colidx, g->a.ci, g->nnz * sizeof(int32_t), hipMemcpyDeviceToHost));
    if (vals && g->nnz) GSR_HIP_CHECK(hipMemcpy(vals, g->a.av, g->nnz * sizeof(float), hipMemcpyDeviceToHost));
    return GSR_OK;
}

gsr_status_t gsr_graph_destroy(gsr_graph_t* g) {
    if (!g) return GSR_OK;
    if (!g->symmetric) free_csr(g->at);
    free_csr(g->a);
    if (g->scratch) (void)hipFree(g->scratch);
    if (g->draws) (void)hipFree(g->draws);
    if (g->dinv) (void)hipFree(g->dinv);
    delete g;
    return GSR_OK;
}

gsr_status_t gsr_workspace_size(const gsr_config_t* cfg, const gsr_graph_t* g, size_t* layer_bytes, size_t* step_bytes) {
    GSR_TRY(validate_config(cfg, g, false));
    if (layer_bytes) *layer_bytes = carve_layer(cfg, g).total;
    if (step_bytes) *step_bytes = carve_step(cfg, g).total;
    return GSR_OK;
}

}  // extern "C"
