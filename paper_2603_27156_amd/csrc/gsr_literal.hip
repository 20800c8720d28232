// The two-group pipeline of Algorithms 1 and 2 as the walk-throughs of Sections 4.3 and 4.4 print it.
// Its block places a row's sums in the row's OWN recorded columns,
//     block(V, I)[i, I[i,t]] = sum_j a_ij V[j,t],
// i.e. a product of A with the n x k matrix of kept values followed by a scatter to k columns; there
// are no weights.  The k slots are padded to W = 16, 32 or 64 columns (kept values that fill their width
// are the operand as they stand, otherwise k_slots_prepare builds it) and go through the same 16-row
// tiles on the matrix cores as gsr_spmm, split rows included; the tile's sums are placed in its rows' own
// columns and combined with the planes before they leave (k_slot_tile).  float32 only.
#include "gsr_internal.h"
#include "gsr_device.h"

#include <algorithm>

namespace gsr {

CsrView make_view(const gsr_graph_t* g, bool transpose);

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

// out[i][c] = beta * base[i][c] + sign * sum_t [idx_own[i][t] == c] S[i][t] + gamma * sum_t [idx_b[i][t] == c] Vb[i][t],
// S = A P (or A^T P) over the W-column operand P.  One wave per 16-row tile: S forms in the accumulators of the
// matrix-core gather and is parked in LDS; the tile's base rows arrive coalesced in a second LDS tile; one lane
// per row then adds the row's slots in slot order (so repeated columns add up in a fixed order; a column outside
// [0, dg) is skipped); the rows leave coalesced.  out may alias base; P may not alias out.
struct SlotArgs {
    CsrView g;
    int n, tiles, dg, k;
    const float* P;          // [n][W]
    float* out; int64_t ld_out;
    float beta; const float* base; int64_t ld_base;
    float sign; const int32_t* idx_own;
    float gamma; const float* vb; const int32_t* idx_b;
    const float* hub_part;
    int* draws; int* draws_done;
};
template <int W>
struct SlotLds {
    TileLds t;
    float s[16 * (W + 1)];   // the tile's sums, row stride W + 1
    float o[16 * 65];        // the tile's rows of the plane, row stride 65
    uint8_t col[16 * 64];    // recorded columns, 255 = skip
};

template <int W, bool DEAL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4))) void k_slot_tile(SlotArgs a) {
    constexpr int CPL = W / 16, SR = W + 1;
    __shared__ SlotLds<W> lds[4];
    SlotLds<W>& L = lds[threadIdx.x >> 6];
    const int lane = lane_id();
    TileWalk<DEAL> walk(a.g, a.tiles, a.draws, a.draws_done);
    while (walk.more()) {
        walk.ahead();
        const int r0 = walk.t * 16;
        wave_sync();          // the previous tile's rows have left the LDS tiles
        const int rpv = tile_rp_load(a.g, r0, a.n, lane);
        const bool has_hub = tile_begin(a.g, rpv, L.t.rp, lane);
        if (walk.dealt(a.g, rpv, L.t.rp, has_hub)) { walk.next(a.g); continue; }
        const int rows = a.n - r0 < 16 ? a.n - r0 : 16;
        // the plane's rows and the recorded columns are requested before the gather
        float b[16];
        int c[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const bool ok = r < rows;
            b[r] = (a.beta != 0.f && ok && lane < a.dg) ? a.base[(size_t)(r0 + r) * a.ld_base + lane] : 0.f;
            c[r] = (ok && lane < a.k) ? a.idx_own[(size_t)(r0 + r) * a.k + lane] : -1;
        }
        f32x4 acc[CPL];
#pragma unroll
        for (int cb = 0; cb < CPL; ++cb) acc[cb] = f32x4{0.f, 0.f, 0.f, 0.f};
        tile_ranges(a.g, has_hub, L.t.rp, [&](int e_a, int e_b) {
            gather_dense_mfma<W, float, 8>(a.g, a.P, W, __builtin_amdgcn_readfirstlane(e_a), __builtin_amdgcn_readfirstlane(e_b),
                                           L.t.rp, L.t.ebuf, lane, acc);
        });
#pragma unroll
        for (int cb = 0; cb < CPL; ++cb)
#pragma unroll
            for (int reg = 0; reg < 4; ++reg) L.s[(4 * (lane >> 4) + reg) * SR + CPL * (lane & 15) + cb] = acc[cb][reg];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            if (lane < a.dg) L.o[r * 65 + lane] = a.beta * b[r];
            if (lane < a.k) L.col[r * 64 + lane] = (unsigned)c[r] < (unsigned)a.dg ? (uint8_t)c[r] : (uint8_t)255;
        }
        wave_sync();
        if (has_hub) {        // split rows: the sum of their first-pass partial rows instead
            for (int r = 0; r < 16; ++r) {
                const bool hub = (L.t.rp[r + 1] - L.t.rp[r]) > a.g.hub_threshold;
                if (hub && lane < W) L.s[r * SR + lane] = hub_row_sum<W>(a.g, a.hub_part, r0 + r, lane);
            }
            wave_sync();
        }
        if (lane < rows) {
            for (int t = 0; t < a.k; ++t) {
                const int cc = L.col[lane * 64 + t];
                if (cc != 255) L.o[lane * 65 + cc] += a.sign * L.s[lane * SR + t];
            }
        }
        if (a.vb) {           // a second set of slots, placed as they are (no product)
            wave_sync();
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const bool ok = r < rows && lane < a.k;
                const float v = ok ? a.vb[(size_t)(r0 + r) * a.k + lane] : 0.f;
                const int cb2 = ok ? a.idx_b[(size_t)(r0 + r) * a.k + lane] : -1;
                if (lane < a.k) {
                    L.s[r * SR + lane] = v;
                    L.col[r * 64 + lane] = (unsigned)cb2 < (unsigned)a.dg ? (uint8_t)cb2 : (uint8_t)255;
                }
            }
            wave_sync();
            if (lane < rows) {
                for (int t = 0; t < a.k; ++t) {
                    const int cc = L.col[lane * 64 + t];
                    if (cc != 255) L.o[lane * 65 + cc] += a.gamma * L.s[lane * SR + t];
                }
            }
        }
        wave_sync();
        for (int r = 0; r < rows; ++r)
            if (lane < a.dg) a.out[(size_t)(r0 + r) * a.ld_out + lane] = L.o[r * 65 + lane];
        walk.next(a.g);
    }
    walk.finish();
}

struct LiteralWs {
    size_t v1, i1, v2, i2, p, total;
};
static int slot_width(int k) { return k <= 16 ? 16 : k <= 32 ? 32 : 64; }
static LiteralWs carve_literal(int64_t n, int k) {
    const int W = slot_width(k);
    LiteralWs w;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t at = off; off += align_up(std::max<size_t>(bytes, 1)); return at; };
    w.v1 = take((size_t)n * k * 4); w.i1 = take((size_t)n * k * 4);
    w.v2 = take((size_t)n * k * 4); w.i2 = take((size_t)n * k * 4);
    w.p = take((size_t)n * W * 4);
    w.total = off;
    return w;
}

static unsigned blocks_for(int64_t elems) { return (unsigned)std::min<int64_t>(std::max<int64_t>((elems + 255) / 256, 1), 65536); }

struct Lit {
    const gsr_graph_t* g;
    int64_t n;
    int dg, k, W;
    hipStream_t s;
    float *v1, *v2, *P;
    int32_t *i1, *i2;
};

static gsr_status_t lit_gs(const Lit& x, const float* plane, int64_t ld, float* v, int32_t* i) {
    return gsr_group_sparse(plane, x.n, x.dg, ld, x.k, GSR_F32, GSR_NORM_NONE, 0.f, v, i, x.s);
}
// S[:, 0..k) = A (or A^T) * slots, the slots being vals or dense[i, idx[i, t]]
template <int W>
static void launch_slot_tile(const Lit& x, const SlotArgs& a, const HubPlan& h) {
    if (h.n_chunks > 0) {
        HubChunks hc{h.ce0, h.ce1, h.n_chunks, x.g->long_rows};
        hipLaunchKernelGGL((k_hub_dense<W, float>), dim3(hub_grid(h.n_chunks)), dim3(256), 0, x.s, a.g, hc,
                           a.P, (int64_t)W, x.g->scratch);
    }
    // as many workgroups as stay resident with this much LDS, at most the graph's persistent grid
    const int per_cu = std::min<int>(4, (int)(160 * 1024 / (4 * sizeof(SlotLds<W>))));
    const unsigned grid = (unsigned)std::max(8, std::min(x.g->grid, x.g->num_cus * per_cu) / 8 * 8);
    if (heavy_first(a.g.n_heavy, a.tiles, grid)) hipLaunchKernelGGL((k_slot_tile<W, true>), dim3(grid), dim3(256), 0, x.s, a);
    else hipLaunchKernelGGL((k_slot_tile<W, false>), dim3(grid), dim3(256), 0, x.s, a);
}

// out = beta * base + sign * block(slots, idx) + gamma * scatter(vb, idx_b), the block over A or A^T with the
// slots being vals, or dense[i, idx[i, t]]
static void lit_block(const Lit& x, const float* vals, const float* dense, int64_t ld, const int32_t* idx, bool transpose,
                      float* out, int64_t ld_out, float beta, const float* base, int64_t ld_base, float sign, float gamma,
                      const float* vb, const int32_t* idx_b) {
    const float* P = vals;
    if (!(vals && x.k == x.W)) {
        hipLaunchKernelGGL(k_slots_prepare, dim3(blocks_for(x.n * x.W)), dim3(256), 0, x.s, x.n, x.k, x.W, x.dg, vals, dense, ld, idx,
                           x.P);
        P = x.P;
    }
    SlotArgs a;
    a.g = make_view(x.g, transpose);
    a.n = (int)x.n; a.tiles = (int)((x.n + 15) / 16); a.dg = x.dg; a.k = x.k;
    a.P = P;
    a.out = out; a.ld_out = ld_out;
    a.beta = beta; a.base = base; a.ld_base = ld_base;
    a.sign = sign; a.idx_own = idx;
    a.gamma = gamma; a.vb = vb; a.idx_b = idx_b;
    a.hub_part = x.g->scratch;
    tile_counters(x.g, &a.draws, &a.draws_done);
    const HubPlan& h = transpose ? x.g->at.hub : x.g->a.hub;
    if (x.W == 16) launch_slot_tile<16>(x, a, h);
    else if (x.W == 32) launch_slot_tile<32>(x, a, h);
    else launch_slot_tile<64>(x, a, h);
}

static gsr_status_t lit_check(const gsr_graph_t* g, int32_t dg, int32_t k, int64_t ld, const void* a, const void* b,
                              const void* ws, size_t ws_bytes, Lit* x, void* stream) {
    if (!g) return fail(GSR_ERR_INVALID_ARG, "graph is null");
    if (dg < 1 || dg > 64) return fail(GSR_ERR_UNSUPPORTED, "dg=%d outside [1,64]", dg);
    if (k < 1 || k > dg) return fail(GSR_ERR_UNSUPPORTED, "k=%d outside [1, dg=%d]", k, dg);
    if (ld < dg) return fail(GSR_ERR_INVALID_ARG, "row stride %lld below dg=%d", (long long)ld, dg);
    if (g->n == 0) return GSR_OK;
    if (g->n >= ((int64_t)1 << 31) || !g->scratch) return fail(GSR_ERR_UNSUPPORTED, "graph too large for the tiled product");
    if (!a || !b || !ws) return fail(GSR_ERR_INVALID_ARG, "null pointer");
    if ((uintptr_t)ws & 255) return fail(GSR_ERR_INVALID_ARG, "the workspace must be 256-byte aligned");
    const LiteralWs w = carve_literal(g->n, k);
    if (ws_bytes < w.total) return fail(GSR_ERR_WORKSPACE_TOO_SMALL, "workspace %zu < %zu bytes", ws_bytes, w.total);
    char* base = (char*)ws;
    x->g = g; x->n = g->n; x->dg = dg; x->k = k; x->W = slot_width(k); x->s = (hipStream_t)stream;
    x->v1 = (float*)(base + w.v1); x->i1 = (int32_t*)(base + w.i1);
    x->v2 = (float*)(base + w.v2); x->i2 = (int32_t*)(base + w.i2);
    x->P = (float*)(base + w.p);
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
    if (vals == out) return fail(GSR_ERR_INVALID_ARG, "out may not alias vals");
    lit_block(x, vals, nullptr, 0, idx, transpose != 0, out, ld, 0.f, nullptr, 0, 1.f, 0.f, nullptr, nullptr);
    GSR_HIP_CHECK(hipGetLastError());
    return GSR_OK;
}

gsr_status_t gsr_alg1_layer_forward(const gsr_graph_t* g, int32_t dg, int32_t k, float* x1_inout, float* x2_inout, int64_t ld,
                                    void* workspace, size_t workspace_bytes, void* stream) {
    Lit x;
    GSR_TRY(lit_check(g, dg, k, ld, x1_inout, x2_inout, workspace, workspace_bytes, &x, stream));
    if (g->n == 0) return GSR_OK;
    GSR_TRY(lit_gs(x, x1_inout, ld, x.v1, x.i1));                                   // (V1, I1) = GS(X1)
    lit_block(x, x.v1, nullptr, 0, x.i1, false, x2_inout, ld, 1.f, x2_inout, ld, 1.f, 0.f, nullptr, nullptr);   // Y2 = X2 + block(V1, I1)
    GSR_TRY(lit_gs(x, x2_inout, ld, x.v2, x.i2));                                   // (V2, I2) = GS(Y2)
    lit_block(x, x.v2, nullptr, 0, x.i2, false, x1_inout, ld, 0.f, nullptr, 0, 1.f, 1.f, x.v1, x.i1);            // Y1 = scatter(V1, I1) + block(V2, I2)
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
    lit_block(x, x.v2, nullptr, 0, x.i2, false, g1_inout, ld, 1.f, g1_inout, ld, -1.f, 0.f, nullptr, nullptr);  // M1 = G1 - block(V2, I2), kept in g1
    GSR_TRY(lit_gs(x, g1_inout, ld, x.v1, x.i1));                                   // (V1, I1) = GS(M1)
    lit_block(x, x.v1, nullptr, 0, x.i1, false, g2_inout, ld, 0.f, nullptr, 0, -1.f, 1.f, x.v2, x.i2);          // M2 = scatter(V2, I2) - block(V1, I1), kept in g2
    // each M through its block's adjoint, in place (the slots are copied out of the plane first)
    lit_block(x, nullptr, g1_inout, ld, x.i1, true, g1_inout, ld, 0.f, nullptr, 0, 1.f, 0.f, nullptr, nullptr);
    lit_block(x, nullptr, g2_inout, ld, x.i2, true, g2_inout, ld, 0.f, nullptr, 0, 1.f, 0.f, nullptr, nullptr);
    GSR_HIP_CHECK(hipGetLastError());
    return GSR_OK;
}

}  // extern "C"
