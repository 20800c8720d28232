// Operators of the paper exposed on their own: GS(X, k) -> (V, I), the dense neighbour
// aggregation A X, and the aggregation of a compressed embedding A * scatter(V, I).
#include "gsr_internal.h"
#include "gsr_device.h"

#include <algorithm>

namespace gsr {

CsrView make_view(const gsr_graph_t* g, bool transpose);
CsrView make_view(const gsr_graph_t* g, bool transpose) {
    const Csr& c = transpose ? g->at : g->a;
    CsrView v;
    v.rp = c.rp; v.ci = c.ci; v.av = c.av;
    v.hub_rows = c.hub.rows; v.hub_cptr = c.hub.cptr; v.n_hub = c.hub.n_hub;
    v.hub_threshold = g->hub_threshold;
    return v;
}

// ---- GS operator, Section 4.1 -------------------------------------------------------------------
// One (sub-)wave per row, lanes beyond dg hold -inf-like padding that can never be selected
// ahead of a real column (padding compares below every finite value and sits at higher lanes).
template <typename T>
__global__ __launch_bounds__(256) void k_group_sparse(const T* __restrict__ x, int64_t n, int dg, int64_t ld, int k,
                                                      int norm, float eps, T* __restrict__ vals, int32_t* __restrict__ idx) {
    const int lane = lane_id();
    const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t row = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6; row < n; row += nwaves) {
        const bool real = lane < dg;
        const float v = real ? to_float(x[row * ld + lane]) : -__builtin_huge_valf();
        const float xs[1] = {v};
        bool sels[1];
        uint64_t masks[1];
        topk_select_multi<64, 1>(xs, k, lane, 0, sels, masks);
        const bool sel = sels[0];
        const uint64_t mask = masks[0];
        float scale = 1.f;
        if (norm == GSR_NORM_RMS) {
            const float ss = sub_sum<64>(real ? v * v : 0.f);
            scale = __builtin_amdgcn_rsqf(ss * (1.0f / (float)dg) + eps);
        }
        if (sel) {
            const int pos = __popcll(mask & (((uint64_t)1 << lane) - 1));
            vals[row * k + pos] = from_float<T>(norm == GSR_NORM_RMS ? v * scale : v);
            idx[row * k + pos] = lane;
        }
    }
}

// ---- dense aggregation Y = A X, eq. (2) -----------------------------------------------------------
__global__ __launch_bounds__(256) void k_spmm_dense(CsrView g, int64_t n, const float* __restrict__ x, int64_t ldx,
                                                    int width, float* __restrict__ y, int64_t ldy) {
    const int lane = lane_id();
    const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t row = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6; row < n; row += nwaves) {
        const int e0 = g.rp[row], e1 = g.rp[row + 1];
        for (int c0 = 0; c0 < width; c0 += 64) {
            const int c = c0 + lane;
            float acc = 0.f;
            if (c < width)
                for (int e = e0; e < e1; ++e) acc += g.av[e] * x[(int64_t)g.ci[e] * ldx + c];
            if (c < width) y[row * ldy + c] = acc;
        }
    }
}

// ---- (V, I int32, any slot order) -> record (values in ascending column order + column mask) -----
template <int DG, typename T>
__global__ void k_pack_records(int64_t n, int k, const T* __restrict__ v_in, const int32_t* __restrict__ i_in,
                               T* __restrict__ v_out, typename MaskOf<DG>::type* __restrict__ m_out) {
    using M = typename MaskOf<DG>::type;
    const int64_t row = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (row >= n) return;
    M mask = 0;
    for (int t = 0; t < k; ++t) mask |= (M)1 << i_in[row * k + t];
    for (int t = 0; t < k; ++t) {
        const int col = i_in[row * k + t];
        v_out[row * k + popc<DG>(mask & (((M)1 << col) - 1))] = v_in[row * k + t];
    }
    m_out[row] = mask;
}

template <int DG>
__global__ void k_check_indices(int64_t n, int k, const int32_t* __restrict__ idx, int* __restrict__ bad) {
    const int64_t row = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (row >= n) return;
    uint64_t mask = 0;
    for (int t = 0; t < k; ++t) {
        const int col = idx[row * k + t];
        if (col < 0 || col >= DG || ((mask >> col) & 1)) { *bad = 1; return; }
        mask |= (uint64_t)1 << col;
    }
}

template <int DG, typename T>
__global__ __launch_bounds__(256) void k_aggregate(CsrView g, int n, const T* __restrict__ vals,
                                                   const typename MaskOf<DG>::type* __restrict__ masks, int k,
                                                   const float* __restrict__ hub_part, float* __restrict__ h_out) {
    constexpr int G = 64 / DG;
    const int lane = lane_id(), c = lane % DG, sub = lane / DG;
    const int nwaves = (gridDim.x * blockDim.x) >> 6;
    for (int r0 = ((blockIdx.x * blockDim.x + threadIdx.x) >> 6) * G; r0 < n; r0 += nwaves * G) {
        const int row = r0 + sub;
        const bool ok = row < n;
        const float acc = row_records<DG, T>(g, vals, masks, k, hub_part, row, ok, c);
        if (ok) h_out[(size_t)row * DG + c] = acc;
    }
}

template <int DG, typename T>
static gsr_status_t aggregate_impl(const gsr_graph_t* g, const void* vals, const int32_t* idx, int k, float* h_out,
                                   void* ws, hipStream_t s) {
    using M = typename MaskOf<DG>::type;
    const int64_t n = g->n;
    char* p = (char*)ws;
    T* v_rec = (T*)p;
    p += align_up((size_t)n * k * sizeof(T));
    M* m_rec = (M*)p;
    p += align_up((size_t)n * sizeof(M));
    float* part = (float*)p;
    const unsigned rows_blocks = (unsigned)((n + 255) / 256);
    hipLaunchKernelGGL((k_pack_records<DG, T>), dim3(rows_blocks), dim3(256), 0, s, n, k, (const T*)vals, idx, v_rec, m_rec);
    CsrView v = make_view(g, false);
    if (g->a.hub.n_chunks > 0) {
        HubChunks hc{g->a.hub.ce0, g->a.hub.ce1, g->a.hub.n_chunks};
        hipLaunchKernelGGL((k_hub_records<DG, T>), dim3((unsigned)std::min(g->a.hub.n_chunks, 4096)), dim3(256), 0, s, v, hc,
                           (const T*)v_rec, (const M*)m_rec, k, part);
    }
    hipLaunchKernelGGL((k_aggregate<DG, T>), dim3((unsigned)g->grid * 2), dim3(256), 0, s, v, (int)n, (const T*)v_rec,
                       (const M*)m_rec, k, (const float*)part, h_out);
    GSR_HIP_CHECK(hipGetLastError());
    return GSR_OK;
}

}  // namespace gsr

using namespace gsr;

extern "C" {

gsr_status_t gsr_group_sparse(const void* x, int64_t n, int32_t dg, int64_t ld, int32_t k, int32_t dtype, int32_t norm,
                              float eps, void* vals_out, int32_t* idx_out, void* stream) {
    if (n < 0) return fail(GSR_ERR_INVALID_ARG, "negative n");
    if (dg < 1 || dg > 64) return fail(GSR_ERR_UNSUPPORTED, "dg=%d outside [1,64]", dg);
    if (k < 1 || k > dg) return fail(GSR_ERR_UNSUPPORTED, "k=%d outside [1, dg=%d]", k, dg);
    if (ld < dg) return fail(GSR_ERR_INVALID_ARG, "row stride %lld below dg=%d", (long long)ld, dg);
    if (dtype != GSR_F32 && dtype != GSR_BF16) return fail(GSR_ERR_UNSUPPORTED, "dtype %d", dtype);
    if (norm != GSR_NORM_NONE && norm != GSR_NORM_RMS) return fail(GSR_ERR_UNSUPPORTED, "norm %d", norm);
    if (n == 0) return GSR_OK;
    if (!x || !vals_out || !idx_out) return fail(GSR_ERR_INVALID_ARG, "null pointer");
    hipStream_t s = (hipStream_t)stream;
    const unsigned blocks = (unsigned)std::min<int64_t>((n + 3) / 4, 8192);
    if (dtype == GSR_F32)
        hipLaunchKernelGGL((k_group_sparse<float>), dim3(blocks), dim3(256), 0, s, (const float*)x, n, dg, ld, k, norm, eps,
                           (float*)vals_out, idx_out);
    else
        hipLaunchKernelGGL((k_group_sparse<bf16_t>), dim3(blocks), dim3(256), 0, s, (const bf16_t*)x, n, dg, ld, k, norm, eps,
                           (bf16_t*)vals_out, idx_out);
    GSR_HIP_CHECK(hipGetLastError());
    return GSR_OK;
}

gsr_status_t gsr_spmm(const gsr_graph_t* g, const float* x, int64_t ldx, int32_t width, float* y, int64_t ldy,
                      int32_t transpose, void* stream) {
    if (!g) return fail(GSR_ERR_INVALID_ARG, "graph is null");
    if (width < 1) return fail(GSR_ERR_INVALID_ARG, "width=%d", width);
    if (ldx < width || ldy < width) return fail(GSR_ERR_INVALID_ARG, "row stride below width");
    if (g->n == 0) return GSR_OK;
    if (!x || !y) return fail(GSR_ERR_INVALID_ARG, "null pointer");
    const unsigned blocks = (unsigned)std::min<int64_t>((g->n + 3) / 4, 8192);
    hipLaunchKernelGGL(k_spmm_dense, dim3(blocks), dim3(256), 0, (hipStream_t)stream, make_view(g, transpose != 0), g->n, x,
                       ldx, width, y, ldy);
    GSR_HIP_CHECK(hipGetLastError());
    return GSR_OK;
}

size_t gsr_spmm_compressed_workspace(const gsr_graph_t* g, int32_t k, int32_t dg) {
    if (!g || k < 1 || dg < 1) return 0;
    return align_up((size_t)g->n * k * 4) + align_up((size_t)g->n * 8) +
           align_up((size_t)std::max(g->a.hub.n_chunks, 1) * dg * sizeof(float)) + 256;
}

gsr_status_t gsr_spmm_compressed(const gsr_graph_t* g, const void* vals, const int32_t* idx, int32_t k, int32_t dg,
                                 int32_t dtype, float* h_out, void* workspace, size_t workspace_bytes, void* stream) {
    if (!g) return fail(GSR_ERR_INVALID_ARG, "graph is null");
    if (dg != 32 && dg != 64) return fail(GSR_ERR_UNSUPPORTED, "dg=%d: only 32 and 64 are built", dg);
    if (k < 1 || k > dg) return fail(GSR_ERR_UNSUPPORTED, "k=%d outside [1, dg=%d]", k, dg);
    if (dtype != GSR_F32 && dtype != GSR_BF16) return fail(GSR_ERR_UNSUPPORTED, "dtype %d", dtype);
    if (g->n == 0) return GSR_OK;
    if (!vals || !idx || !h_out || !workspace) return fail(GSR_ERR_INVALID_ARG, "null pointer");
    if (workspace_bytes < gsr_spmm_compressed_workspace(g, k, dg))
        return fail(GSR_ERR_WORKSPACE_TOO_SMALL, "workspace %zu < %zu", workspace_bytes, gsr_spmm_compressed_workspace(g, k, dg));
    hipStream_t s = (hipStream_t)stream;
    // indices come from the caller: reject out-of-range or repeated columns instead of reading wild
    int* bad = (int*)((char*)workspace + gsr_spmm_compressed_workspace(g, k, dg) - 256);
    GSR_HIP_CHECK(hipMemsetAsync(bad, 0, sizeof(int), s));
    const unsigned rows_blocks = (unsigned)((g->n + 255) / 256);
    if (dg == 32) hipLaunchKernelGGL((k_check_indices<32>), dim3(rows_blocks), dim3(256), 0, s, g->n, k, idx, bad);
    else hipLaunchKernelGGL((k_check_indices<64>), dim3(rows_blocks), dim3(256), 0, s, g->n, k, idx, bad);
    int bad_h = 0;
    GSR_HIP_CHECK(hipMemcpyAsync(&bad_h, bad, sizeof(int), hipMemcpyDeviceToHost, s));
    GSR_HIP_CHECK(hipStreamSynchronize(s));
    if (bad_h) return fail(GSR_ERR_INVALID_ARG, "idx holds a column outside [0,dg) or a repeated column");
    if (dg == 32 && dtype == GSR_F32) return aggregate_impl<32, float>(g, vals, idx, k, h_out, workspace, s);
    if (dg == 64 && dtype == GSR_F32) return aggregate_impl<64, float>(g, vals, idx, k, h_out, workspace, s);
    if (dg == 32) return aggregate_impl<32, bf16_t>(g, vals, idx, k, h_out, workspace, s);
    return aggregate_impl<64, bf16_t>(g, vals, idx, k, h_out, workspace, s);
}

}  // extern "C"
