// Operators of the paper exposed on their own: GS(X, k) -> (V, I), the dense neighbour
// aggregation A X, and the aggregation of a compressed embedding A * scatter(V, I).
#include "gsr_internal.h"
#include "gsr_device.h"

#include <algorithm>
#include <mutex>

namespace gsr {

static_assert(TILE_COUNTERS == kTileCounters, "host and device disagree on the size of a counter set");
static_assert(TIE_SUB == kTieSub && TIE_COUNTER_STRIDE == kTieCounterStride, "host and device disagree on the near-tie sub-lists");

CsrView make_view(const gsr_graph_t* g, bool transpose);
CsrView make_view(const gsr_graph_t* g, bool transpose) {
    const Csr& c = transpose ? g->at : g->a;
    CsrView v;
    v.rp = c.rp; v.ci = c.ci; v.av = c.av;
    v.hub_rows = c.hub.rows; v.hub_cptr = c.hub.cptr; v.hub_tile0 = c.hub.tile0; v.n_hub = c.hub.n_hub;
    v.hub_threshold = g->hub_threshold;
    v.heavy = c.heavy; v.n_heavy = c.n_heavy; v.heavy_edges = kHeavyTileEdges;
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

// Rows of 65 to 256 columns: one wave per row, lane c owning columns c, c + 64, c + 128, c + 192 (those past dg hold
// padding that can never be kept ahead of a real column).  The k-th largest value is found by bisection on the
// order-preserving integer image of the values, count = the popcounts of up to four ballots; ties go to the lowest
// columns of the row.
template <typename T>
__global__ __launch_bounds__(256) void k_group_sparse_wide(const T* __restrict__ x, int64_t n, int dg, int64_t ld, int k,
                                                           int norm, float eps, T* __restrict__ vals, int32_t* __restrict__ idx) {
    const int lane = lane_id();
    const int ns = (dg + 63) / 64;
    const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t row = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6; row < n; row += nwaves) {
        float v[4];
        uint32_t key[4];
        float ss = 0.f;
        uint32_t top = 0u;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int c = 64 * s + lane;
            const bool real = s < ns && c < dg;
            v[s] = real ? to_float(x[row * ld + c]) : 0.f;
            ss += v[s] * v[s];
            uint32_t u = __float_as_uint(v[s]);
            if (u == 0x80000000u) u = 0u;                                   // -0 -> +0
            key[s] = real ? ((u & 0x80000000u) ? ~u : (u | 0x80000000u)) : 0u;      // padding: below every finite value
            top = max(top, key[s]);
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) top = max(top, (uint32_t)__shfl_xor((int)top, off, 64));
        auto count_ge = [&](uint32_t t) {
            int cnt = 0;
#pragma unroll
            for (int s = 0; s < 4; ++s) cnt += __popcll(ballot(key[s] >= t));
            return cnt;
        };
        uint32_t lo = 0u, hi = top + 1u;                 // at least k keys are >= lo, fewer than k are >= hi
        if (k < dg) {
            for (int round = 0; round < 33 && hi - lo > 1u; ++round) {
                const uint32_t mid = lo + ((hi - lo) >> 1);
                const int cnt = count_ge(mid);
                if (cnt >= k) lo = mid; else hi = mid;
                if (cnt == k) break;
            }
        }
        // kept: every key above lo, and of those equal to lo the lowest columns (padding keys are 0 = lo only when k >= dg,
        // where every real column is kept and none of the padding)
        int need = k;
        uint64_t gt[4], eq[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const bool real = s < ns && 64 * s + lane < dg;
            gt[s] = ballot(real && key[s] > lo);
            eq[s] = ballot(real && key[s] == lo);
            need -= __popcll(gt[s]);
        }
        const float scale = norm == GSR_NORM_RMS ? __builtin_amdgcn_rsqf(sub_sum<64>(ss) * (1.0f / (float)dg) + eps) : 1.f;
        const uint64_t below = ((uint64_t)1 << lane) - 1;
        int pos0 = 0;                                     // kept columns in the sub-rows before s
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int ties = __popcll(eq[s]);
            const int take = need < 0 ? 0 : (need < ties ? need : ties);
            // the `take` lowest lanes of eq[s]
            const bool tie_kept = ((eq[s] >> lane) & 1ull) && __popcll(eq[s] & below) < take;
            const uint64_t kept = gt[s] | ballot(tie_kept);
            if ((kept >> lane) & 1ull) {
                const int pos = pos0 + __popcll(kept & below);
                vals[row * k + pos] = from_float<T>(norm == GSR_NORM_RMS ? v[s] * scale : v[s]);
                idx[row * k + pos] = 64 * s + lane;
            }
            pos0 += __popcll(kept);
            need -= take;
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

// ---- the same operators on 16-row tiles (the forms the layer kernels use) -------------------------
// One wave per tile in a persistent sweep; neighbour data gathered as MFMA products (see
// gsr_device.h), results stored straight from the accumulators: lane (g, j) holds rows
// 4 g + reg and the CPL adjacent columns CPL j .. CPL j + CPL - 1, so every store instruction
// writes four whole rows.
template <int W>
__device__ __forceinline__ void store_acc_rows(const f32x4 (&acc)[W / 16], const CsrView& g, const float* __restrict__ hub_part,
                                               bool has_hub, int r0, int n, const int* s_rp, float* __restrict__ y,
                                               int64_t ldy, int lane) {
    constexpr int CPL = W / 16;
#pragma unroll
    for (int reg = 0; reg < 4; ++reg) {
        const int rr = 4 * (lane >> 4) + reg, row = r0 + rr;
        float v[CPL];
#pragma unroll
        for (int cb = 0; cb < CPL; ++cb) v[cb] = acc[cb][reg];
        const bool split = has_hub && (s_rp[rr + 1] - s_rp[rr]) > g.hub_threshold;     // written below instead
        if (row < n && !split) store_cols<CPL, float>(y + (size_t)row * ldy + CPL * (lane & 15), v);
    }
    if (has_hub) {
        for (int r = 0; r < 16; ++r) {
            const bool hub = (s_rp[r + 1] - s_rp[r]) > g.hub_threshold;
            if (hub && lane < W) y[(size_t)(r0 + r) * ldy + lane] = hub_row_sum<W>(g, hub_part, r0 + r, lane);
        }
    }
}

// Widths 32 and 64: the sums of a tile in ordinary arithmetic into an LDS tile (gather_dense_rows: on this chip the
// float32 matrix instructions do not run beside the vector pipe, and a 16-row product spends fifteen rows of every
// edge on zeros), rows stored from there; width 16: on the matrix cores, rows stored from the accumulators.
template <int W, bool DEAL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4))) void k_spmm_tile(CsrView g, int n, int tiles, const float* __restrict__ x, int64_t ldx,
                                                   float* __restrict__ y, int64_t ldy, const float* __restrict__ hub_part,
                                                   int* draws, int* draws_done) {
    constexpr int LR = W + 1, CPL = W / 16;
    constexpr bool ROWS = W >= 32;
    struct Wave {
        TileLds t;
        float st[ROWS ? 16 * LR : 1];
    };
    __shared__ Wave lds[4];
    Wave& Wv = lds[threadIdx.x >> 6];
    TileLds& L = Wv.t;
    const int lane = lane_id();
    TileWalk<DEAL> walk(g, tiles, draws, draws_done);
    while (walk.more()) {
        walk.ahead();
        const int r0 = walk.t * 16;
        wave_sync();
        const int rpv = tile_rp_load(g, r0, n, lane);
        const bool has_hub = tile_begin(g, rpv, L.rp, lane);
        if (walk.dealt(g, rpv, L.rp, has_hub)) { walk.next(g); continue; }
        if constexpr (ROWS) {
            tile_gather_rows<W>(g, hub_part, has_hub, r0, L.rp, Wv.st, lane, [&](int e_a, int e_b) {
                gather_dense_rows<W, 8>(g, x, ldx, __builtin_amdgcn_readfirstlane(e_a), __builtin_amdgcn_readfirstlane(e_b), L.rp,
                                        L.ebuf, lane, Wv.st);
            });
            wave_sync();
            // four rows per store instruction, CPL adjacent columns per lane
#pragma unroll
            for (int reg = 0; reg < 4; ++reg) {
                const int rr = 4 * reg + (lane >> 4), row = r0 + rr;
                float v[CPL];
#pragma unroll
                for (int cb = 0; cb < CPL; ++cb) v[cb] = Wv.st[rr * LR + CPL * (lane & 15) + cb];
                if (row < n) store_cols<CPL, float>(y + (size_t)row * ldy + CPL * (lane & 15), v);
            }
        } else {
            f32x4 acc[W / 16];
#pragma unroll
            for (int cb = 0; cb < W / 16; ++cb) acc[cb] = f32x4{0.f, 0.f, 0.f, 0.f};
            tile_ranges(g, has_hub, L.rp, [&](int e_a, int e_b) {
                gather_dense_mfma<W, float, 16>(g, x, ldx, __builtin_amdgcn_readfirstlane(e_a), __builtin_amdgcn_readfirstlane(e_b),
                                                L.rp, L.ebuf, lane, acc);
            });
            store_acc_rows<W>(acc, g, hub_part, has_hub, r0, n, L.rp, y, ldy, lane);
        }
        walk.next(g);
    }
    walk.finish();
}

// float32 records: the sums of a tile in ordinary arithmetic into an LDS tile (gather_records_rows), rows stored from
// there; 16-bit records: on the matrix cores, rows stored from the accumulators.
template <int DG, typename T, bool DEAL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4))) void k_aggregate_tile(CsrView g, int n, int tiles, const T* __restrict__ vals,
                                                        const typename MaskOf<DG>::type* __restrict__ masks, int k,
                                                        const float* __restrict__ hub_part, float* __restrict__ h_out,
                                                        int* draws, int* draws_done) {
    constexpr int LR = DG + 1;
    struct Wave {
        TileLds t;
        float st[sizeof(T) == 4 ? 16 * LR : 1];
    };
    __shared__ Wave lds[4];
    __shared__ typename std::conditional<sizeof(T) == 2, DealLut, DealLutF>::type dlut;
    if constexpr (sizeof(T) == 2) deal_lut_fill(dlut);
    else deal_lutf_fill(dlut);
    Wave& W = lds[threadIdx.x >> 6];
    TileLds& L = W.t;
    const int lane = lane_id();
    TileWalk<DEAL> walk(g, tiles, draws, draws_done);
    while (walk.more()) {
        walk.ahead();
        const int r0 = walk.t * 16;
        wave_sync();
        const int rpv = tile_rp_load(g, r0, n, lane);
        const bool has_hub = tile_begin(g, rpv, L.rp, lane);
        if (walk.dealt(g, rpv, L.rp, has_hub)) { walk.next(g); continue; }
        if constexpr (sizeof(T) == 4) {
            tile_gather_rows<DG>(g, hub_part, has_hub, r0, L.rp, W.st, lane, [&](int e_a, int e_b) {
                gather_records_rows<DG, 8, true>(g, vals, masks, k, __builtin_amdgcn_readfirstlane(e_a), __builtin_amdgcn_readfirstlane(e_b),
                                                 L.rp, reinterpret_cast<RecEdge*>(L.ebuf), L.rbuf, lane, W.st, &dlut);
            });
            wave_sync();
            const int rows = n - r0 < 16 ? n - r0 : 16;
            for (int r = 0; r < rows; ++r)
                if (lane < DG) __builtin_nontemporal_store(W.st[r * LR + lane], h_out + (size_t)(r0 + r) * DG + lane);
        } else {
            f32x4 acc[DG / 16];
#pragma unroll
            for (int cb = 0; cb < DG / 16; ++cb) acc[cb] = f32x4{0.f, 0.f, 0.f, 0.f};
            tile_ranges(g, has_hub, L.rp, [&](int e_a, int e_b) {
                gather_records_mfma<DG, T, 8>(g, vals, masks, k, __builtin_amdgcn_readfirstlane(e_a),
                                              __builtin_amdgcn_readfirstlane(e_b), L.rp, reinterpret_cast<RecEdge*>(L.ebuf), L.rbuf,
                                              lane, acc, &dlut);
            });
            store_acc_rows<DG>(acc, g, hub_part, has_hub, r0, n, L.rp, h_out, DG, lane);
        }
        walk.next(g);
    }
    walk.finish();
}

// GS of 16 rows per wave: rows are read four at a time into an LDS tile, then selected in the
// quarter layout (emit_tile), values and column numbers leave as contiguous blocks.
template <int DG, typename T>
__global__ __launch_bounds__(256) void k_gs_tile(const T* __restrict__ x, int n, int64_t ld, int k, int norm, float eps,
                                                 T* __restrict__ vals, int32_t* __restrict__ idx) {
    constexpr int LR = DG + 1, CPL = DG / 16;
    struct Wave {
        float st[16 * LR + 64];
        int ist[16 * DG];
    };
    __shared__ Wave lds[4];
    Wave& L = lds[threadIdx.x >> 6];
    const int lane = lane_id(), tg = lane >> 4, tj = lane & 15;
    const int nwaves = (gridDim.x * blockDim.x) >> 6, tiles = (n + 15) / 16;
    Record<DG, T> out;
    out.vals = vals;
    out.mask = nullptr;
    for (int t = (blockIdx.x * blockDim.x + threadIdx.x) >> 6; t < tiles; t += nwaves) {
        const int r0 = t * 16;
        float v[4][CPL];
#pragma unroll
        for (int reg = 0; reg < 4; ++reg) {
            const int row = r0 + 4 * reg + tg;
            load_cols<CPL, T>(x + (size_t)(row < n ? row : n - 1) * ld + CPL * tj, v[reg]);
        }
        wave_sync();          // the previous tile's results have left the scratch
#pragma unroll
        for (int reg = 0; reg < 4; ++reg)
#pragma unroll
            for (int cb = 0; cb < CPL; ++cb)
                L.st[(4 * reg + tg) * LR + CPL * tj + cb] = r0 + 4 * reg + tg < n ? v[reg][cb] : 0.f;
        wave_sync();
        emit_tile<DG, T>(L.st, r0, n, k, norm, eps, out, false, lane, idx, L.ist);
    }
}

// ---- (V, I int32, any slot order) -> record (values in ascending column order + column mask) -----
// kp lanes per row (kp: the power of two at or above k), 64 / kp rows per wave step, so that the
// [n][k] arrays are read and written in whole rows.  The row's mask is the OR over its lanes;
// a column outside [0, DG) or named twice sets *bad (the caller's indices are not trusted).
template <int DG, typename T>
__global__ __launch_bounds__(256) void k_pack_records(int64_t n, int k, int kp, const T* __restrict__ v_in,
                                                      const int32_t* __restrict__ i_in, T* __restrict__ v_out,
                                                      typename MaskOf<DG>::type* __restrict__ m_out, int* __restrict__ bad) {
    using M = typename MaskOf<DG>::type;
    const int lane = lane_id(), t = lane % kp, sub = lane / kp, per = 64 / kp;
    const int64_t nwaves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t r0 = (((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6) * per; r0 < n; r0 += nwaves * per) {
        const int64_t row = r0 + sub;
        const bool ok = row < n && t < k;
        const int col = ok ? i_in[row * k + t] : 0;
        const bool in_range = col >= 0 && col < DG;
        const M bit = (ok && in_range) ? (M)1 << col : (M)0;
        uint32_t lo = (uint32_t)bit, hi = DG == 64 ? (uint32_t)((uint64_t)bit >> 32) : 0u;
        for (int off = 1; off < kp; off <<= 1) {
            lo |= (uint32_t)__shfl_xor((int)lo, off, 64);
            if (DG == 64) hi |= (uint32_t)__shfl_xor((int)hi, off, 64);
        }
        const M mask = DG == 64 ? (M)(((uint64_t)hi << 32) | lo) : (M)lo;
        if (ok && (!in_range || popc<DG>(mask) != k)) *bad = 1;
        if (ok && in_range) v_out[row * k + popc<DG>(mask & (bit - 1))] = v_in[row * k + t];
        if (row < n && t == 0) m_out[row] = mask;
    }
}

template <int DG, typename T>
static gsr_status_t aggregate_impl(const gsr_graph_t* g, const void* vals, const int32_t* idx, int k, float* h_out,
                                   void* ws, int* bad, hipStream_t s) {
    using M = typename MaskOf<DG>::type;
    const int64_t n = g->n;
    char* p = (char*)ws;
    T* v_rec = (T*)p;
    p += align_up((size_t)n * k * sizeof(T) + 16);          // the record gather loads up to 16 bytes past a record
    M* m_rec = (M*)p;
    p += align_up((size_t)n * sizeof(M));
    float* part = (float*)p;
    // indices come from the caller: reject out-of-range or repeated columns instead of reading wild
    int kp = 1;
    while (kp < k) kp <<= 1;
    const int64_t steps = (n + 64 / kp - 1) / (64 / kp);
    GSR_HIP_CHECK(hipMemsetAsync(bad, 0, sizeof(int), s));
    hipLaunchKernelGGL((k_pack_records<DG, T>), dim3((unsigned)std::min<int64_t>((steps + 3) / 4, 16384)), dim3(256), 0, s, n, k,
                       kp, (const T*)vals, idx, v_rec, m_rec, bad);
    int bad_h = 0;
    GSR_HIP_CHECK(hipMemcpyAsync(&bad_h, bad, sizeof(int), hipMemcpyDeviceToHost, s));
    GSR_HIP_CHECK(hipStreamSynchronize(s));
    if (bad_h) return fail(GSR_ERR_INVALID_ARG, "idx holds a column outside [0,dg) or a repeated column");
    CsrView v = make_view(g, false);
    if (g->a.hub.n_chunks > 0) {
        HubChunks hc{g->a.hub.ce0, g->a.hub.ce1, g->a.hub.n_chunks, g->long_rows};
        hipLaunchKernelGGL((k_hub_records<DG, T>), dim3(hub_grid(g->a.hub.n_chunks)), dim3(256), 0, s, v, hc,
                           (const T*)v_rec, (const M*)m_rec, k, part);
    }
    int *dn, *dx;
    tile_counters(g, &dn, &dx);
    const int tiles = (int)((n + 15) / 16);
    if (heavy_first(v.n_heavy, tiles, (unsigned)g->grid))
        hipLaunchKernelGGL((k_aggregate_tile<DG, T, true>), dim3((unsigned)g->grid), dim3(256), 0, s, v, (int)n, tiles,
                           (const T*)v_rec, (const M*)m_rec, k, (const float*)part, h_out, dn, dx);
    else
        hipLaunchKernelGGL((k_aggregate_tile<DG, T, false>), dim3((unsigned)g->grid), dim3(256), 0, s, v, (int)n, tiles,
                           (const T*)v_rec, (const M*)m_rec, k, (const float*)part, h_out, dn, dx);
    GSR_HIP_CHECK(hipGetLastError());
    return GSR_OK;
}


// ---- gsr_spmm: argument checks and launches shared by its two entry points ------------------------------
static gsr_status_t spmm_check(const gsr_graph_t* g, const float* x, int64_t ldx, int32_t width, float* y, int64_t ldy,
                               int32_t transpose) {
    if (!g) return fail(GSR_ERR_INVALID_ARG, "graph is null");
    if (width < 1) return fail(GSR_ERR_INVALID_ARG, "width=%d", width);
    if (ldx < width || ldy < width) return fail(GSR_ERR_INVALID_ARG, "row stride below width");
    if (g->n == 0) return GSR_OK;
    if (!x || !y) return fail(GSR_ERR_INVALID_ARG, "null pointer");
    if (transpose && !g->has_transpose) return fail(GSR_ERR_UNSUPPORTED, "graph has no transpose");
    return GSR_OK;
}

// hub_part: first-pass sums of split rows, [chunks][64] floats; draws / done: a clear counter set (tile_draws)
static gsr_status_t spmm_launch(const gsr_graph_t* g, const float* x, int64_t ldx, int32_t width, float* y, int64_t ldy,
                                int32_t transpose, float* hub_part, int* draws, int* done, hipStream_t s) {
    const CsrView view = make_view(g, transpose != 0);
    // 16, 32 or 64 columns with aligned rows: 16-row tiles on the matrix cores; split rows go through a
    // first pass into hub_part
    const size_t piece = (size_t)(width / 16) * sizeof(float);
    if ((width == 16 || width == 32 || width == 64) && g->n < ((int64_t)1 << 31) && (ldx * sizeof(float)) % piece == 0 &&
        (ldy * sizeof(float)) % piece == 0 && ((uintptr_t)x % piece) == 0 && ((uintptr_t)y % piece) == 0 && hub_part) {
        const HubPlan& h = transpose ? g->at.hub : g->a.hub;
        const int tiles = (int)((g->n + 15) / 16);
        if (h.n_chunks > 0) {
            HubChunks hc{h.ce0, h.ce1, h.n_chunks, g->long_rows};
            const dim3 hg(hub_grid(h.n_chunks));
            if (width == 64) hipLaunchKernelGGL((k_hub_dense<64, float>), hg, dim3(256), 0, s, view, hc, x, ldx, hub_part);
            else if (width == 32) hipLaunchKernelGGL((k_hub_dense<32, float>), hg, dim3(256), 0, s, view, hc, x, ldx, hub_part);
            else hipLaunchKernelGGL((k_hub_dense<16, float>), hg, dim3(256), 0, s, view, hc, x, ldx, hub_part);
        }
        const bool deal = heavy_first(view.n_heavy, tiles, (unsigned)g->grid);
        auto launch = [&](auto kernel) {
            hipLaunchKernelGGL(kernel, dim3((unsigned)g->grid), dim3(256), 0, s, view, (int)g->n, tiles, x, ldx, y, ldy,
                               (const float*)hub_part, draws, done);
        };
        if (width == 64) deal ? launch(k_spmm_tile<64, true>) : launch(k_spmm_tile<64, false>);
        else if (width == 32) deal ? launch(k_spmm_tile<32, true>) : launch(k_spmm_tile<32, false>);
        else deal ? launch(k_spmm_tile<16, true>) : launch(k_spmm_tile<16, false>);
        GSR_HIP_CHECK(hipGetLastError());
        return GSR_OK;
    }
    const unsigned blocks = (unsigned)std::min<int64_t>((g->n + 3) / 4, 8192);
    hipLaunchKernelGGL(k_spmm_dense, dim3(blocks), dim3(256), 0, s, view, g->n, x, ldx, width, y, ldy);
    GSR_HIP_CHECK(hipGetLastError());
    return GSR_OK;
}

// ---- gsr_spmm_noalloc: the scratch of gsr_spmm in a fixed device array -------------------------------------
// For callers that cannot allocate.  Layout: one counter set of the dynamic tile sweep with its sign-off counters,
// then the first-pass sums of up to kNoAllocMaxChunks chunks of split rows.  Every GPU the library runs on holds its
// own copy of the array until the process ends; host code reaches it only through the address that
// hipGetSymbolAddress returns with that GPU current (the array's name is not a device address on the host).
constexpr int kNoAllocMaxChunks = 16384;
constexpr int kNoAllocCounterInts = kTileCounters + 9 * 32;
constexpr size_t kNoAllocCounterBytes = ((size_t)kNoAllocCounterInts * sizeof(int) + 255) / 256 * 256;
constexpr size_t kNoAllocBytes = kNoAllocCounterBytes + (size_t)kNoAllocMaxChunks * 64 * sizeof(float);
static __device__ __align__(256) unsigned char scratch[kNoAllocBytes];

constexpr int kNoAllocMaxDevices = 64;
static std::mutex g_noalloc_mutex;
static char* g_noalloc_ptr[kNoAllocMaxDevices];      // per device: the address of `scratch` there

// The address of the array on `device` (looked up once per device, with that device current).
static gsr_status_t noalloc_scratch(int device, char** out) {
    int cur = -1;
    GSR_HIP_CHECK(hipGetDevice(&cur));
    if (cur != device) return fail(GSR_ERR_INVALID_ARG, "the graph was built on device %d, the current device is %d", device, cur);
    if (device < 0 || device >= kNoAllocMaxDevices) return fail(GSR_ERR_UNSUPPORTED, "device index %d above %d", device, kNoAllocMaxDevices - 1);
    std::lock_guard<std::mutex> lock(g_noalloc_mutex);
    if (!g_noalloc_ptr[device]) {
        void* p = nullptr;
        GSR_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(GSR_ERR_HIP, "hipGetSymbolAddress returned a null address");
        g_noalloc_ptr[device] = static_cast<char*>(p);
    }
    *out = g_noalloc_ptr[device];
    return GSR_OK;
}

__global__ void k_clear_ints(int* p, int count) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = 0;
}

}  // namespace gsr

using namespace gsr;

extern "C" {

gsr_status_t gsr_group_sparse(const void* x, int64_t n, int32_t dg, int64_t ld, int32_t k, int32_t dtype, int32_t norm,
                              float eps, void* vals_out, int32_t* idx_out, void* stream) {
    if (n < 0) return fail(GSR_ERR_INVALID_ARG, "negative n");
    if (dg < 1 || dg > 256) return fail(GSR_ERR_UNSUPPORTED, "dg=%d outside [1,256]", dg);
    if (k < 1 || k > dg) return fail(GSR_ERR_UNSUPPORTED, "k=%d outside [1, dg=%d]", k, dg);
    if (ld < dg) return fail(GSR_ERR_INVALID_ARG, "row stride %lld below dg=%d", (long long)ld, dg);
    if (dtype != GSR_F32 && dtype != GSR_BF16) return fail(GSR_ERR_UNSUPPORTED, "dtype %d", dtype);
    if (norm != GSR_NORM_NONE && norm != GSR_NORM_RMS) return fail(GSR_ERR_UNSUPPORTED, "norm %d", norm);
    if (n == 0) return GSR_OK;
    if (!x || !vals_out || !idx_out) return fail(GSR_ERR_INVALID_ARG, "null pointer");
    hipStream_t s = (hipStream_t)stream;
    // whole groups of 32 or 64 columns with rows that can be moved in aligned pieces: 16 rows per wave
    const size_t piece = (size_t)(dg / 16) * dtype_size(dtype);
    if ((dg == 32 || dg == 64) && n < ((int64_t)1 << 31) && ((size_t)ld * dtype_size(dtype)) % piece == 0 &&
        ((uintptr_t)x % piece) == 0) {
        const unsigned tb = (unsigned)std::min<int64_t>((n + 63) / 64, 4096);
        if (dtype == GSR_F32 && dg == 64)
            hipLaunchKernelGGL((k_gs_tile<64, float>), dim3(tb), dim3(256), 0, s, (const float*)x, (int)n, ld, k, norm, eps,
                               (float*)vals_out, idx_out);
        else if (dtype == GSR_F32)
            hipLaunchKernelGGL((k_gs_tile<32, float>), dim3(tb), dim3(256), 0, s, (const float*)x, (int)n, ld, k, norm, eps,
                               (float*)vals_out, idx_out);
        else if (dg == 64)
            hipLaunchKernelGGL((k_gs_tile<64, bf16_t>), dim3(tb), dim3(256), 0, s, (const bf16_t*)x, (int)n, ld, k, norm, eps,
                               (bf16_t*)vals_out, idx_out);
        else
            hipLaunchKernelGGL((k_gs_tile<32, bf16_t>), dim3(tb), dim3(256), 0, s, (const bf16_t*)x, (int)n, ld, k, norm, eps,
                               (bf16_t*)vals_out, idx_out);
        GSR_HIP_CHECK(hipGetLastError());
        return GSR_OK;
    }
    const unsigned blocks = (unsigned)std::min<int64_t>((n + 3) / 4, 8192);
    if (dg > 64) {
        if (dtype == GSR_F32)
            hipLaunchKernelGGL((k_group_sparse_wide<float>), dim3(blocks), dim3(256), 0, s, (const float*)x, n, dg, ld, k, norm, eps,
                               (float*)vals_out, idx_out);
        else
            hipLaunchKernelGGL((k_group_sparse_wide<bf16_t>), dim3(blocks), dim3(256), 0, s, (const bf16_t*)x, n, dg, ld, k, norm, eps,
                               (bf16_t*)vals_out, idx_out);
        GSR_HIP_CHECK(hipGetLastError());
        return GSR_OK;
    }
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
    GSR_TRY(spmm_check(g, x, ldx, width, y, ldy, transpose));
    if (g->n == 0) return GSR_OK;
    int *draws, *done;
    tile_counters(g, &draws, &done);
    return spmm_launch(g, x, ldx, width, y, ldy, transpose, g->scratch, draws, done, (hipStream_t)stream);
}

gsr_status_t gsr_spmm_noalloc(const gsr_graph_t* g, const float* x, int64_t ldx, int32_t width, float* y, int64_t ldy,
                              int32_t transpose, void* stream) {
    GSR_TRY(spmm_check(g, x, ldx, width, y, ldy, transpose));
    if (g->n == 0) return GSR_OK;
    const HubPlan& h = transpose ? g->at.hub : g->a.hub;
    if (h.n_chunks > kNoAllocMaxChunks)
        return fail(GSR_ERR_UNSUPPORTED, "gsr_spmm_noalloc: the graph's split rows make %d first-pass chunks, the built-in scratch holds %d",
                    h.n_chunks, kNoAllocMaxChunks);
    char* base = nullptr;
    GSR_TRY(noalloc_scratch(g->device, &base));
    hipStream_t s = (hipStream_t)stream;
    int* draws = reinterpret_cast<int*>(base);
    // the array keeps the last call's contents: the counters must read zero when the sweep starts
    hipLaunchKernelGGL(k_clear_ints, dim3((kNoAllocCounterInts + 255) / 256), dim3(256), 0, s, draws, kNoAllocCounterInts);
    float* part = reinterpret_cast<float*>(base + kNoAllocCounterBytes);
    return spmm_launch(g, x, ldx, width, y, ldy, transpose, part, draws, draws + kTileCounters, s);
}

size_t gsr_spmm_compressed_workspace(const gsr_graph_t* g, int32_t k, int32_t dg) {
    if (!g || k < 1 || dg < 1) return 0;
    return align_up((size_t)g->n * k * 4 + 16) + align_up((size_t)g->n * 8) +
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
    if ((uint64_t)g->n * (uint64_t)k >= ((uint64_t)1 << 32)) return fail(GSR_ERR_UNSUPPORTED, "n * k does not fit 32 bits");
    if (((uintptr_t)workspace & 255) || ((uintptr_t)h_out & 15))
        return fail(GSR_ERR_INVALID_ARG, "the workspace must be 256-byte aligned and h_out 16-byte aligned");
    if (workspace_bytes < gsr_spmm_compressed_workspace(g, k, dg))
        return fail(GSR_ERR_WORKSPACE_TOO_SMALL, "workspace %zu < %zu", workspace_bytes, gsr_spmm_compressed_workspace(g, k, dg));
    hipStream_t s = (hipStream_t)stream;
    int* bad = (int*)((char*)workspace + gsr_spmm_compressed_workspace(g, k, dg) - 256);
    if (dg == 32 && dtype == GSR_F32) return aggregate_impl<32, float>(g, vals, idx, k, h_out, workspace, bad, s);
    if (dg == 64 && dtype == GSR_F32) return aggregate_impl<64, float>(g, vals, idx, k, h_out, workspace, bad, s);
    if (dg == 32) return aggregate_impl<32, bf16_t>(g, vals, idx, k, h_out, workspace, bad, s);
    return aggregate_impl<64, bf16_t>(g, vals, idx, k, h_out, workspace, bad, s);
}

}  // extern "C"
