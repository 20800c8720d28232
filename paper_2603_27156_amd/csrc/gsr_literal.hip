// The two-group pipeline of Algorithms 1 and 2 as the walk-throughs of Sections 4.3 and 4.4 print it.
// Its block places a row's sums in the row's OWN recorded columns,
//     block(V, I)[i, I[i,t]] = sum_j a_ij V[j,t],
// i.e. a product of A with the n x k matrix of kept values followed by a scatter to k columns; there
// are no weights.  The product runs through gsr_spmm (the k slots padded to 16, 32 or 64 columns so that
// it takes the tiled path on the matrix cores, split rows included; kept values that fill their width
// are its operand as they stand); the kernels here prepare its operand otherwise and combine its
// result with the planes.  float32 only.
#include "gsr_internal.h"

#include <algorithm>

namespace gsr {

// P[i][t] = vals[i][t] (dense == NULL) or dense[i][idx[i][t]] for t < k, 0 for k <= t < W.
// An index outside [0, dg) reads nothing (the slot becomes 0).
__global__ __launch_bounds__(256) void k_slots_prepare(int64_t n, int k, int W, int dg, const float* __restrict__ vals,
                                                       const float* __restrict__ dense, int64_t ld,
                                                       const int32_t* __restrict__ idx, float* __restrict__ P) {
    const int64_t total = n * W;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
        const int64_t i = e / W;
        const int t = (int)(e - i * W);
        float v = 0.f;
        if (t < k) {
            if (dense) {
                const int c = idx[i * k + t];
                if ((unsigned)c < (unsigned)dg) v = dense[i * ld + c];
            } else {
                v = vals[i * k + t];
            }
        }
        P[e] = v;
    }
}

// out[i][c] = beta * base[i][c] + sign * sum_t [idx_own[i][t] == c] S[i][t] + gamma * sum_t [idx_b[i][t] == c] Vb[i][t]
// A workgroup builds 64 rows in LDS: the base rows arrive coalesced, then one thread per row adds the
// row's slots in slot order (so repeated columns add up in a fixed order; a column outside [0, dg)
// is skipped), then the rows leave coalesced.  out may alias base.  Measured at 1M rows, dg 64, k 16:
// 185 - 270 us; staging the slots in LDS too and splitting a row over four threads was not faster.
constexpr int COMBINE_ROWS = 64;
__global__ __launch_bounds__(256) void k_slots_combine(int64_t n, int dg, int k, int W, float* out, int64_t ld_out, float beta,
                                                       const float* base, int64_t ld_base, float sign,
                                                       const float* __restrict__ S, const int32_t* __restrict__ idx_own,
                                                       float gamma, const float* __restrict__ Vb,
                                                       const int32_t* __restrict__ idx_b) {
    __shared__ float tile[COMBINE_ROWS * 65];
    const int64_t groups = (n + COMBINE_ROWS - 1) / COMBINE_ROWS;
    for (int64_t gidx = blockIdx.x; gidx < groups; gidx += gridDim.x) {
        const int64_t r0 = gidx * COMBINE_ROWS;
        const int rows = (int)(n - r0 < COMBINE_ROWS ? n - r0 : COMBINE_ROWS);
        __syncthreads();
        for (int e = threadIdx.x; e < rows * dg; e += 256) {
            const int r = e / dg, c = e - r * dg;
            tile[r * 65 + c] = beta != 0.f ? beta * base[(r0 + r) * ld_base + c] : 0.f;
        }
        __syncthreads();
        if ((int)threadIdx.x < rows) {
            const int r = threadIdx.x;
            const int64_t i = r0 + r;
            for (int t = 0; t < k; ++t) {
                const int c = idx_own[i * k + t];
                if ((unsigned)c < (unsigned)dg) tile[r * 65 + c] += sign * S[i * W + t];
            }
            if (Vb) {
                for (int t = 0; t < k; ++t) {
                    const int c = idx_b[i * k + t];
                    if ((unsigned)c < (unsigned)dg) tile[r * 65 + c] += gamma * Vb[i * k + t];
                }
            }
        }
        __syncthreads();
        for (int e = threadIdx.x; e < rows * dg; e += 256) {
            const int r = e / dg, c = e - r * dg;
            out[(r0 + r) * ld_out + c] = tile[r * 65 + c];
        }
    }
}

struct LiteralWs {
    size_t v1, i1, v2, i2, p, s, total;
};
static int slot_width(int k) { return k <= 16 ? 16 : k <= 32 ? 32 : 64; }
static LiteralWs carve_literal(int64_t n, int k) {
    const int W = slot_width(k);
    LiteralWs w;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t at = off; off += align_up(std::max<size_t>(bytes, 1)); return at; };
    w.v1 = take((size_t)n * k * 4); w.i1 = take((size_t)n * k * 4);
    w.v2 = take((size_t)n * k * 4); w.i2 = take((size_t)n * k * 4);
    w.p = take((size_t)n * W * 4);  w.s = take((size_t)n * W * 4);
    w.total = off;
    return w;
}

static unsigned blocks_for(int64_t elems) { return (unsigned)std::min<int64_t>(std::max<int64_t>((elems + 255) / 256, 1), 65536); }

struct Lit {
    const gsr_graph_t* g;
    int64_t n;
    int dg, k, W;
    hipStream_t s;
    float *v1, *v2, *P, *S;
    int32_t *i1, *i2;
};

static gsr_status_t lit_gs(const Lit& x, const float* plane, int64_t ld, float* v, int32_t* i) {
    return gsr_group_sparse(plane, x.n, x.dg, ld, x.k, GSR_F32, GSR_NORM_NONE, 0.f, v, i, x.s);
}
// S[:, 0..k) = A (or A^T) * slots, the slots being vals or dense[i, idx[i, t]]
static gsr_status_t lit_product(const Lit& x, const float* vals, const float* dense, int64_t ld, const int32_t* idx,
                                bool transpose) {
    if (vals && x.k == x.W) return gsr_spmm(x.g, vals, x.W, x.W, x.S, x.W, transpose ? 1 : 0, x.s);
    hipLaunchKernelGGL(k_slots_prepare, dim3(blocks_for(x.n * x.W)), dim3(256), 0, x.s, x.n, x.k, x.W, x.dg, vals, dense, ld, idx,
                       x.P);
    return gsr_spmm(x.g, x.P, x.W, x.W, x.S, x.W, transpose ? 1 : 0, x.s);
}
static void lit_combine(const Lit& x, float* out, int64_t ld_out, float beta, const float* base, int64_t ld_base, float sign,
                        const int32_t* idx_own, float gamma, const float* vb, const int32_t* idx_b) {
    hipLaunchKernelGGL(k_slots_combine, dim3((unsigned)std::min<int64_t>((x.n + COMBINE_ROWS - 1) / COMBINE_ROWS, 65536)), dim3(256), 0, x.s, x.n, x.dg, x.k, x.W, out, ld_out, beta,
                       base, ld_base, sign, (const float*)x.S, idx_own, gamma, vb, idx_b);
}

static gsr_status_t lit_check(const gsr_graph_t* g, int32_t dg, int32_t k, int64_t ld, const void* a, const void* b,
                              const void* ws, size_t ws_bytes, Lit* x, void* stream) {
    if (!g) return fail(GSR_ERR_INVALID_ARG, "graph is null");
    if (dg < 1 || dg > 64) return fail(GSR_ERR_UNSUPPORTED, "dg=%d outside [1,64]", dg);
    if (k < 1 || k > dg) return fail(GSR_ERR_UNSUPPORTED, "k=%d outside [1, dg=%d]", k, dg);
    if (ld < dg) return fail(GSR_ERR_INVALID_ARG, "row stride %lld below dg=%d", (long long)ld, dg);
    if (g->n == 0) return GSR_OK;
    if (!a || !b || !ws) return fail(GSR_ERR_INVALID_ARG, "null pointer");
    if ((uintptr_t)ws & 255) return fail(GSR_ERR_INVALID_ARG, "the workspace must be 256-byte aligned");
    const LiteralWs w = carve_literal(g->n, k);
    if (ws_bytes < w.total) return fail(GSR_ERR_WORKSPACE_TOO_SMALL, "workspace %zu < %zu bytes", ws_bytes, w.total);
    char* base = (char*)ws;
    x->g = g; x->n = g->n; x->dg = dg; x->k = k; x->W = slot_width(k); x->s = (hipStream_t)stream;
    x->v1 = (float*)(base + w.v1); x->i1 = (int32_t*)(base + w.i1);
    x->v2 = (float*)(base + w.v2); x->i2 = (int32_t*)(base + w.i2);
    x->P = (float*)(base + w.p); x->S = (float*)(base + w.s);
    return GSR_OK;
}

}  // namespace gsr

using namespace gsr;

extern "C" {

size_t gsr_walkthrough_workspace(const gsr_graph_t* g, int32_t k) {
    if (!g || k < 1 || k > 64) return 0;
    return carve_literal(g->n, k).total;
}

gsr_status_t gsr_slot_block(const gsr_graph_t* g, const float* vals, const int32_t* idx, int32_t k, int32_t dg,
                            int32_t transpose, float* out, int64_t ld, void* workspace, size_t workspace_bytes,
                            void* stream) {
    Lit x;
    GSR_TRY(lit_check(g, dg, k, ld, vals, out, workspace, workspace_bytes, &x, stream));
    if (g->n == 0) return GSR_OK;
    if (!idx) return fail(GSR_ERR_INVALID_ARG, "null pointer");
    if (transpose && !g->has_transpose) return fail(GSR_ERR_UNSUPPORTED, "graph has no transpose");
    GSR_TRY(lit_product(x, vals, nullptr, 0, idx, transpose != 0));
    lit_combine(x, out, ld, 0.f, nullptr, 0, 1.f, idx, 0.f, nullptr, nullptr);
    GSR_HIP_CHECK(hipGetLastError());
    return GSR_OK;
}

gsr_status_t gsr_alg1_layer_forward(const gsr_graph_t* g, int32_t dg, int32_t k, float* x1_inout, float* x2_inout, int64_t ld,
                                    void* workspace, size_t workspace_bytes, void* stream) {
    Lit x;
    GSR_TRY(lit_check(g, dg, k, ld, x1_inout, x2_inout, workspace, workspace_bytes, &x, stream));
    if (g->n == 0) return GSR_OK;
    GSR_TRY(lit_gs(x, x1_inout, ld, x.v1, x.i1));                                   // (V1, I1) = GS(X1)
    GSR_TRY(lit_product(x, x.v1, nullptr, 0, x.i1, false));                         // S = A V1
    lit_combine(x, x2_inout, ld, 1.f, x2_inout, ld, 1.f, x.i1, 0.f, nullptr, nullptr);   // Y2 = X2 + S placed at I1
    GSR_TRY(lit_gs(x, x2_inout, ld, x.v2, x.i2));                                   // (V2, I2) = GS(Y2)
    GSR_TRY(lit_product(x, x.v2, nullptr, 0, x.i2, false));                         // S = A V2
    lit_combine(x, x1_inout, ld, 0.f, nullptr, 0, 1.f, x.i2, 1.f, x.v1, x.i1);      // Y1 = scatter(V1, I1) + S placed at I2
    GSR_HIP_CHECK(hipGetLastError());
    return GSR_OK;
}

gsr_status_t gsr_alg2_layer_backward(const gsr_graph_t* g, int32_t dg, int32_t k, float* g1_inout, float* g2_inout, int64_t ld,
                                     void* workspace, size_t workspace_bytes, void* stream) {
    Lit x;
    GSR_TRY(lit_check(g, dg, k, ld, g1_inout, g2_inout, workspace, workspace_bytes, &x, stream));
    if (g->n == 0) return GSR_OK;
    if (!g->has_transpose) return fail(GSR_ERR_UNSUPPORTED, "graph has no transpose");
    GSR_TRY(lit_gs(x, g2_inout, ld, x.v2, x.i2));                                   // (V2, I2) = GS(G2)
    GSR_TRY(lit_product(x, x.v2, nullptr, 0, x.i2, false));
    lit_combine(x, g1_inout, ld, 1.f, g1_inout, ld, -1.f, x.i2, 0.f, nullptr, nullptr);  // M1 = G1 - block(V2, I2), kept in g1
    GSR_TRY(lit_gs(x, g1_inout, ld, x.v1, x.i1));                                   // (V1, I1) = GS(M1)
    GSR_TRY(lit_product(x, x.v1, nullptr, 0, x.i1, false));
    lit_combine(x, g2_inout, ld, 0.f, nullptr, 0, -1.f, x.i1, 1.f, x.v2, x.i2);     // M2 = scatter(V2, I2) - block(V1, I1), kept in g2
    GSR_TRY(lit_product(x, nullptr, g1_inout, ld, x.i1, true));                     // each M through its block's adjoint, in place
    lit_combine(x, g1_inout, ld, 0.f, nullptr, 0, 1.f, x.i1, 0.f, nullptr, nullptr);
    GSR_TRY(lit_product(x, nullptr, g2_inout, ld, x.i2, true));
    lit_combine(x, g2_inout, ld, 0.f, nullptr, 0, 1.f, x.i2, 0.f, nullptr, nullptr);
    GSR_HIP_CHECK(hipGetLastError());
    return GSR_OK;
}

}  // extern "C"
