// The grouped reversible layer (Section 3, eq. (6)/(7)), its backward fused with the inverse
// (Algorithm 2's structure; eq. (3), eq. (11)) and the whole training step.
//
// Kernels (persistent over 16-row tiles, one wave per tile, no cross-wave synchronisation inside
// the sweep):
//   k_block   H = A*scatter(V,I) of Y_{i-1} gathered from compressed records into an LDS tile;
//             O = H W_i on the matrix cores; Y_i = X_i + O (forward) or X_i = Y_i - O (inverse),
//             in place; the GS record of the row just written is emitted in the same pass.  With
//             WITH_DW it also accumulates dW_i += H^T dY_i, so the recomputed H is consumed
//             where it is rebuilt.
//   k_grad    (first: dW_i summed from the workgroup partials the kernel before left;) Q = A^T dY_i (dense-row gather); dH = Q W_i^T on the matrix cores; only the k
//             positions recorded by I are read; back through the RMS scale; dY_{i-1} += dZ.
//   k_sum     Y_0 = sum_{j>=2} X_j and/or the GS record of a plane.
//   k_head    scalar linear head, squared error, dX^L, partial sums for dw_out / db / loss.
#include "gsr_internal.h"
#include "gsr_device.h"

#include <algorithm>
#include <vector>

namespace gsr {

CsrView make_view(const gsr_graph_t* g, bool transpose);

// per-wave LDS: tile(s) of 16 x (DG+1) floats, 64 staged edges, 17 row pointers
template <int DG, int TILES>
struct WaveLds {
    float st[TILES][16 * (DG + 1) + 64];   // tile + 64 dump words for contributions that must not count
    EdgeRec ebuf[64];                      // 64 staged edges (RecEdge has the same size)
    int rp[20];                            // row pointers of the tile's 17 row boundaries
    uint8_t rbuf[64];                      // tile row of every staged edge
};

// ---- block: forward / inverse (+ weight gradient) ------------------------------------------------
template <int DG, typename T>
struct BlockArgs {
    CsrView g;
    int n, tiles;
    Record<DG, T> in;       // record of Y_{i-1}
    int k;
    const float* hub_part;  // first-pass partial rows of split rows
    const float* w;         // W_i [DG][DG], row stride ldw (DG, or D/C when the block is a part of a wider matrix)
    int ldw;
    T* plane;               // X_i on entry / Y_i on return (or the reverse), row stride ld
    int64_t ld;
    Record<DG, T> out;      // record of the row written (out.mask == NULL: none)
    bool out_given;         // out.mask holds the column sets to use (kept from the forward sweep)
    int norm;
    float eps;
    const T* dy;            // dY_i, row stride ldg            (WITH_DW)
    int64_t ldg;
    float* dw_partial;      // [gridDim.x][DG*DG]              (WITH_DW)
    int* draws;             // tile counters of the dynamic sweep and the sign-off counter (not WITH_DW)
    int* draws_done;
    TieSeg<DG> tie;         // where rows that select at a near-tie are listed (count == NULL: nowhere)
    float* h_out;           // [n][DG] float32: receives H = A scatter(V, I) of the block for k_dw (NULL: not kept)
    // YG (groups wider than a tile): blockIdx.y is the column block written, ob: W_i's block 64 columns on, the plane
    // and dY 64 elements on, the dW partials and the tile counters a set on
    size_t y_dw_partial;
    int y_draws;
};

// B3: the H W_i (and dW_i) products on the bf16 matrix pipe from three-term splits (mfma_tile_b3), with W_i kept
// split in LDS.  That copy is half as large again as the float32 one, so the kernels without dW accumulators run
// eight waves per workgroup on it to keep sixteen waves per compute unit resident.  Measured on the 1M-node workload:
// forward 345 -> 319 us, inverse + dW 516 -> 477 us per launch.  The forward kernel keeps a float32 variant (B3 =
// false, four waves per workgroup) for graphs whose rows nearly all go through the first pass, where a launch is a
// single short tile per wave and the variant with the larger workgroups took 121 us against 84.  Both inverse kernels
// always use the split form: the plain and the fused inverse must rebuild the same bits.
constexpr int block_waves(bool with_dw, bool b3) { return (!with_dw && b3) ? 8 : 4; }

template <int DG, typename T, int SIGN, bool WITH_DW, bool DEAL, bool B3 = true, bool YG = false>
__global__ __launch_bounds__(64 * block_waves(WITH_DW, B3)) __attribute__((amdgpu_waves_per_eu(WITH_DW ? 2 : 4))) void k_block(BlockArgs<DG, T> a) {
    static_assert(B3 || (SIGN > 0 && !WITH_DW), "only the forward kernel has a float32 variant");
    if constexpr (YG) {
        const int ob = blockIdx.y;
        a.w += 64 * ob;
        a.plane += 64 * ob;
        if (a.dy) a.dy += 64 * ob;
        a.dw_partial += (size_t)ob * a.y_dw_partial;
        if (a.draws) { a.draws += ob * a.y_draws; a.draws_done += ob * a.y_draws; }
        if (ob > 0) a.h_out = nullptr;          // (the same rows for every column block written)
    }
    constexpr int LR = DG + 1, CPL = DG / 16;
    __shared__ WaveLds<DG, 1> lds[block_waves(WITH_DW, B3)];
    const int lane = lane_id(), wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), tg = lane >> 4, tj = lane & 15;
    WaveLds<DG, 1>& L = lds[wave];
    float* st_h = L.st[0];
    __shared__ typename std::conditional<B3, WLdsB3<DG>, WLds<DG>>::type wl;
    __shared__ typename std::conditional<sizeof(T) == 2, DealLut, DealLutF>::type dlut;
    if constexpr (sizeof(T) == 2) deal_lut_fill(dlut);
    else deal_lutf_fill(dlut);
    if constexpr (B3) load_w_lds_b3<DG>(a.w, a.ldw, false, wl);
    else load_w_lds<DG>(a.w, a.ldw, false, wl);
    f32x4 dw[WITH_DW ? DG / 16 : 1][WITH_DW ? DG / 16 : 1];
    if constexpr (WITH_DW) {
#pragma unroll
        for (int mb = 0; mb < DG / 16; ++mb)
#pragma unroll
            for (int ob = 0; ob < DG / 16; ++ob) dw[mb][ob] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    // the weight gradient sums over the tiles a wave has seen: fixed sweep there, drawn tiles otherwise
    const TileSweep ts = tile_sweep(a.tiles);
    TileDraws td;
    TileDeal deal{0, 0, false};      // DEAL: the heavy tiles first (a variant of its own: the bookkeeping costs
    if constexpr (DEAL) deal = tile_deal(a.g);   // 3 % on a graph with 120 short tiles per wave even when it never fires)
    int requested = 0;     // the draw that is outstanding (dynamic sweep)
    int t = ts.first, t_end = ts.end;
    if constexpr (!WITH_DW) {
        td = tile_draws(a.tiles, a.draws, a.draws_done);
        requested = tile_request(td);
        t_end = td.end;
        if (!deal.on) t = tile_drawn(td, requested);
    }
    if constexpr (DEAL) {
        if (deal.on) { t = a.g.heavy[deal.at]; t_end = a.tiles; }
    }
    while (t < t_end) {
        if constexpr (!WITH_DW) {
            if (!DEAL || !deal.on) requested = tile_request(td);
        }
        const int r0 = t * 16;
        wave_sync();
        const int rpv = tile_rp_load(a.g, r0, a.n, lane);
        // The tile's own rows (X_i, and dY_i for the weight gradient), in the tile register layout.  Requested before
        // the gather they arrive while it runs, but hold sixteen registers through it; where the gather is short of
        // registers they are requested after it and arrive during the weight product (1M-node workload, float32:
        // forward 291 -> 274 us, inverse 326 -> 309 us, spilled registers 14 -> 4; measured per variant: the fused
        // inverse + dW kernel gains at D/C = 32 and loses at 64, the 16-bit forward kernel the other way round).
        constexpr bool OWN_LATE = WITH_DW ? DG == 32 : (sizeof(T) == 4 || DG == 64);
        float xy[4][CPL], gy[WITH_DW ? 4 : 1][CPL];
        auto own_rows = [&]() {
#pragma unroll
            for (int reg = 0; reg < 4; ++reg) {
                const int row = r0 + 4 * reg + tg;
                const size_t rowc = (size_t)(row < a.n ? row : a.n - 1);
                load_cols<CPL, T>(a.plane + rowc * a.ld + CPL * tj, xy[reg]);
                if constexpr (WITH_DW) load_cols<CPL, T>(a.dy + rowc * a.ldg + CPL * tj, gy[reg]);
            }
        };
        if constexpr (!OWN_LATE) own_rows();
        const bool has_hub = tile_begin(a.g, rpv, L.rp, lane);
        if constexpr (DEAL) {
            if (!deal.on && tile_is_heavy(a.g, rpv, L.rp, has_hub)) {      // dealt out before the sweep
                if constexpr (WITH_DW) t += ts.step;
                else t = tile_drawn(td, requested);
                continue;
            }
        }
        // float32: the sums in ordinary arithmetic (forward 329 us against 370 through the matrix cores on the 1M-node
        // workload), in the forward and in both inverse kernels alike, so that f_i is recomputed by the instructions that
        // computed it; four window loads in flight per lane group (eight cost registers: inverse 310 us against 297).
        if constexpr (sizeof(T) == 4) {
            tile_gather_rows<DG>(a.g, a.hub_part, has_hub, r0, L.rp, st_h, lane, [&](int e_a, int e_b) {
                gather_records_rows<DG, 4, true>(a.g, a.in.vals, a.in.mask, a.k, __builtin_amdgcn_readfirstlane(e_a),
                                                 __builtin_amdgcn_readfirstlane(e_b), L.rp, reinterpret_cast<RecEdge*>(L.ebuf),
                                                 L.rbuf, lane, st_h, &dlut);
            });
        } else {
            f32x4 hacc[DG / 16];
            tile_gather<DG>(a.g, a.hub_part, has_hub, r0, L.rp, st_h, lane, hacc, [&](int e_a, int e_b) {
                gather_records_mfma<DG, T, 8>(a.g, a.in.vals, a.in.mask, a.k, __builtin_amdgcn_readfirstlane(e_a),
                                              __builtin_amdgcn_readfirstlane(e_b), L.rp, reinterpret_cast<RecEdge*>(L.ebuf), L.rbuf,
                                              lane, hacc, &dlut);
            });
        }
        if constexpr (OWN_LATE) own_rows();
        if constexpr (WITH_DW) {
#pragma unroll
            for (int reg = 0; reg < 4; ++reg)
#pragma unroll
                for (int cb = 0; cb < CPL; ++cb) gy[reg][cb] = r0 + 4 * reg + tg < a.n ? gy[reg][cb] : 0.f;   // rows past the end
        }
        wave_sync();
        if constexpr (!WITH_DW) {
            if (a.h_out) {                                 // H leaves for the weight-gradient kernel, four rows per store
#pragma unroll
                for (int reg = 0; reg < 4; ++reg) {
                    const int rr = 4 * reg + tg, row = r0 + rr;
                    float hv[CPL];
#pragma unroll
                    for (int cb = 0; cb < CPL; ++cb) hv[cb] = st_h[rr * LR + CPL * tj + cb];
                    if (row < a.n) store_cols<CPL, float>(a.h_out + (size_t)row * DG + CPL * tj, hv);
                }
            }
        }
        f32x4 acc[CPL];
        if constexpr (B3) {
            mfma_tile_b3<DG>(st_h, wl, acc);               // O = H W_i in the tile register layout
            if constexpr (WITH_DW) mfma_outer_b3<DG>(st_h, gy, dw);
        } else {
            mfma_tile<DG>(st_h, wl, acc);
            if constexpr (WITH_DW) mfma_outer<DG>(st_h, gy, dw);
        }
        wave_sync();                                       // H has been read: the tile is free
        // residual: four rows per instruction, CPL adjacent elements per lane
#pragma unroll
        for (int reg = 0; reg < 4; ++reg) {
            const int rr = 4 * reg + tg, row = r0 + rr;
            const bool ok = row < a.n;
            T* p = a.plane + (size_t)(ok ? row : a.n - 1) * a.ld + CPL * tj;
            float y[CPL];
#pragma unroll
            for (int cb = 0; cb < CPL; ++cb) y[cb] = stored<T>(SIGN > 0 ? xy[reg][cb] + acc[cb][reg] : xy[reg][cb] - acc[cb][reg]);
            if (ok) store_cols<CPL, T>(p, y);
#pragma unroll
            for (int cb = 0; cb < CPL; ++cb) st_h[rr * LR + CPL * tj + cb] = ok ? y[cb] : 0.f;
        }
        if (a.out.mask) {
            wave_sync();
            emit_tile<DG, T>(st_h, r0, a.n, a.k, a.norm, a.eps, a.out, a.out_given, lane, nullptr, nullptr, a.tie);
        }
        if (DEAL && deal.on) {
            deal.at += deal.waves;
            deal.on = deal.at < a.g.n_heavy;
            if (deal.on) {
                t = a.g.heavy[deal.at];
            } else if constexpr (WITH_DW) {
                t = ts.first; t_end = ts.end;
            } else {
                t = tile_drawn(td, requested); t_end = td.end;
            }
        } else {
            if constexpr (WITH_DW) t += ts.step;
            else t = tile_drawn(td, requested);
        }
    }
    if constexpr (!WITH_DW) tile_finish(td);
    if constexpr (WITH_DW) {
        // workgroup partial of dW_i: the four waves add their accumulators in wave order
        float* red = reinterpret_cast<float*>(lds);
        static_assert(sizeof(lds) >= DG * DG * sizeof(float), "LDS too small for the dW reduction");
        for (int w = 0; w < 4; ++w) {
            __syncthreads();
            if (wave == w) {
#pragma unroll
                for (int mb = 0; mb < DG / 16; ++mb)
#pragma unroll
                    for (int ob = 0; ob < DG / 16; ++ob)
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const int m = 16 * mb + 4 * (lane >> 4) + r, o = CPL * (lane & 15) + ob;
                            if (w == 0) red[m * DG + o] = dw[mb][ob][r];
                            else red[m * DG + o] += dw[mb][ob][r];
                        }
            }
        }
        __syncthreads();
        for (int i = threadIdx.x; i < DG * DG; i += 256) a.dw_partial[(size_t)blockIdx.x * DG * DG + i] = red[i];
    }
}

// The records of listed rows, written again with the column sets kept from the forward sweep: a wave takes sixteen
// list entries in the quarter layout of emit_tile (lane = (entry, quarter of the row)) and forms the values exactly
// as emit_tile does when the set is given.  plane: the rows the record was just taken from, row stride ld.  Called by
// every wave of a grid of `nwaves` waves (a multiple of TIE_SUB): wave w takes sub-list w mod TIE_SUB.
template <int DG, typename T>
__device__ __forceinline__ void tie_fixup_rows(const TieSeg<DG>& tie, const T* __restrict__ plane, int64_t ld, int k, int norm, float eps,
                                               const Record<DG, T>& out, int wave, int nwaves) {
    using M = typename MaskOf<DG>::type;
    constexpr int QW = DG / 4;
    const int lane = lane_id(), r = lane & 15, q = lane >> 4;
    const int sub = wave & (TIE_SUB - 1);
    const int listed = tie.count[sub * TIE_COUNTER_STRIDE], cnt = listed < tie.cap ? listed : tie.cap;
    for (int e0 = (wave / TIE_SUB) * 16; e0 < cnt; e0 += (nwaves / TIE_SUB) * 16) {
        const bool ok = e0 + r < cnt;
        const int e = sub * tie.cap + (ok ? e0 + r : cnt - 1);
        const size_t row = tie.rows[e];
        const M m = tie.masks[e];
        float x[QW];
#pragma unroll
        for (int j = 0; j < QW; ++j) x[j] = to_float(plane[row * ld + q * QW + j]);
        const uint32_t msel = (uint32_t)(m >> (QW * q)) & ((1u << QW) - 1u);
        uint32_t all[4];
        quarter_all((uint32_t)__popc(msel), all);
        size_t slot = row * k;
#pragma unroll
        for (int i = 0; i < 3; ++i) slot += i < q ? all[i] : 0u;
        const float scale = record_scale<DG>(x, norm, eps);
#pragma unroll
        for (int j = 0; j < QW; ++j) {
            const bool bit = (msel >> j) & 1u;
            if (ok && bit) out.vals[slot] = from_float<T>(x[j] * scale);
            slot += bit ? 1 : 0;
        }
        if (ok && q == 0) out.mask[row] = m;
    }
}

// dW_i[e] = sum over workgroup partials, as a launch of its own (used when the gradient kernel that follows has too
// few tiles per wave to absorb the work, see layer_backward_impl).  A block of 256 threads owns 16 entries; its 16
// thread rows each sum a contiguous sixteenth of the partials in ascending order, then the 16 sums are added in order.
// (Blocks of 64 entries left three quarters of the compute units idle on a 64 x 64 matrix: 18 us per launch.)
constexpr int DW_REDUCE_ENTRIES = 16;
__device__ __forceinline__ void dw_reduce_block(int block, const float* __restrict__ partial, int nparts, int elems,
                                                float* __restrict__ out, int cols, int ld_out) {
    __shared__ float red[16][DW_REDUCE_ENTRIES];
    const int j = threadIdx.x & (DW_REDUCE_ENTRIES - 1), seg = threadIdx.x / DW_REDUCE_ENTRIES;
    const int e = block * DW_REDUCE_ENTRIES + j;
    const int per = (nparts + 15) / 16, p0 = seg * per, p1 = min(nparts, p0 + per);
    float acc = 0.f;
    if (e < elems) {
        int p = p0;
        for (; p + 8 <= p1; p += 8) {           // eight loads in flight, added in ascending order
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = partial[(size_t)(p + u) * elems + e];
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += v[u];
        }
        for (; p < p1; ++p) acc += partial[(size_t)p * elems + e];
    }
    red[seg][j] = acc;
    __syncthreads();
    if (seg == 0 && e < elems) {
        float s = red[0][j];
#pragma unroll
        for (int q = 1; q < 16; ++q) s += red[q][j];
        out[(size_t)(e / cols) * ld_out + e % cols] = s;       // entry (e / cols, e % cols) of a matrix of row stride ld_out
    }
}

// What a launch of k_tie_fixup may take along: the reduction of dW_i's workgroup partials (its workgroups from
// fix_blocks on do that; out == NULL: nothing), which saves a launch per block on small graphs.
struct DwReduceJob {
    const float* partial;
    int nparts, elems;
    float* out;
    int cols, ld_out;
    int fix_blocks;
};

template <int DG, typename T>
__global__ __launch_bounds__(256) void k_tie_fixup(TieSeg<DG> tie, const T* __restrict__ plane, int64_t ld, int k, int norm,
                                                   float eps, Record<DG, T> out, DwReduceJob red) {
    if (red.out && (int)blockIdx.x >= red.fix_blocks) {
        dw_reduce_block((int)blockIdx.x - red.fix_blocks, red.partial, red.nparts, red.elems, red.out, red.cols, red.ld_out);
        return;
    }
    const int blocks = red.out ? red.fix_blocks : (int)gridDim.x;
    tie_fixup_rows<DG, T>(tie, plane, ld, k, norm, eps, out, (int)((blockIdx.x * blockDim.x + threadIdx.x) >> 6),
                          (int)((blocks * blockDim.x) >> 6));
}

// dW_i = H^T dY_i as a pass of its own over H (left by the inverse kernel) and dY_i: a wave sums over the tiles of a
// fixed sweep (so the partial sums do not depend on timing), 64 x 64 accumulators in registers, products on the bf16
// pipe (mfma_outer_b3); workgroup partials as k_block writes them.  The inverse kernel then runs without the 64
// accumulator registers per lane, at sixteen waves per compute unit with the row-wise sums of the forward kernel.
template <int DG, typename T>
struct DwArgs {
    int n, tiles;
    const float* h;         // [n][DG]
    const T* dy;            // row stride ldg
    int64_t ldg;
    float* dw_partial;      // [gridDim.x][DG*DG]
    // mode 2 of the step: the record the inverse kernel has just taken again gets the kept column sets of its listed
    // rows back here (tie.count == NULL: nothing to do), which saves a launch per block
    TieSeg<DG> tie;
    const T* fix_plane;
    int64_t fix_ld;
    int k, norm;
    float eps;
    Record<DG, T> fix_out;
};

template <int DG, typename T>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void k_dw(DwArgs<DG, T> a) {
    if (a.tie.count)
        tie_fixup_rows<DG, T>(a.tie, a.fix_plane, a.fix_ld, a.k, a.norm, a.eps, a.fix_out, (int)((blockIdx.x * blockDim.x + threadIdx.x) >> 6),
                              (int)((gridDim.x * blockDim.x) >> 6));
    constexpr int LR = DG + 1, CPL = DG / 16;
    __shared__ float tile[4][16 * LR];
    const int lane = lane_id(), wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), tg = lane >> 4, tj = lane & 15;
    float* st = tile[wave];
    f32x4 dw[DG / 16][DG / 16];
#pragma unroll
    for (int mb = 0; mb < DG / 16; ++mb)
#pragma unroll
        for (int ob = 0; ob < DG / 16; ++ob) dw[mb][ob] = f32x4{0.f, 0.f, 0.f, 0.f};
    const TileSweep ts = tile_sweep(a.tiles);
    // the next tile's rows are requested while the present tile is multiplied
    float hv[4][CPL], gy[4][CPL];
    auto request = [&](int t) {
#pragma unroll
        for (int reg = 0; reg < 4; ++reg) {
            const int row = t * 16 + 4 * reg + tg;
            const size_t rowc = (size_t)(row < a.n ? row : a.n - 1);
            load_cols<CPL, float>(a.h + rowc * DG + CPL * tj, hv[reg]);
            load_cols<CPL, T>(a.dy + rowc * a.ldg + CPL * tj, gy[reg]);
        }
    };
    int t = ts.first;
    if (t < ts.end) request(t);
    while (t < ts.end) {
        const int r0 = t * 16;
        float g[4][CPL];
        wave_sync();          // the tile before has been read
#pragma unroll
        for (int reg = 0; reg < 4; ++reg) {
            const bool ok = r0 + 4 * reg + tg < a.n;
#pragma unroll
            for (int cb = 0; cb < CPL; ++cb) {
                st[(4 * reg + tg) * LR + CPL * tj + cb] = ok ? hv[reg][cb] : 0.f;
                g[reg][cb] = ok ? gy[reg][cb] : 0.f;          // rows past the end
            }
        }
        t += ts.step;
        if (t < ts.end) request(t);
        wave_sync();
        mfma_outer_b3<DG>(st, g, dw);
    }
    // workgroup partial of dW_i: the four waves add their accumulators in wave order
    __shared__ float red[DG * DG];
    for (int w = 0; w < 4; ++w) {
        __syncthreads();
        if (wave == w) {
#pragma unroll
            for (int mb = 0; mb < DG / 16; ++mb)
#pragma unroll
                for (int ob = 0; ob < DG / 16; ++ob)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int m = 16 * mb + 4 * (lane >> 4) + r, o = CPL * (lane & 15) + ob;
                        if (w == 0) red[m * DG + o] = dw[mb][ob][r];
                        else red[m * DG + o] += dw[mb][ob][r];
                    }
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < DG * DG; i += 256) a.dw_partial[(size_t)blockIdx.x * DG * DG + i] = red[i];
}

// blockIdx.y (groups wider than a tile: the S x S blocks of dW_i in one launch): set y of the partials starts
// y * set_stride floats on, and goes to block (y / sets_per_row, y % sets_per_row) of the output, 64 rows and 64 columns apart.
__global__ __launch_bounds__(256) void k_dw_reduce(const float* __restrict__ partial, int nparts, int elems,
                                                   float* __restrict__ out, int cols, int ld_out, size_t set_stride = 0,
                                                   int sets_per_row = 1) {
    partial += (size_t)blockIdx.y * set_stride;
    out += (size_t)(blockIdx.y / sets_per_row) * 64 * ld_out + (size_t)(blockIdx.y % sets_per_row) * 64;
    dw_reduce_block((int)blockIdx.x, partial, nparts, elems, out, cols, ld_out);
}

// ---- block: data gradient ---------------------------------------------------------------------------
template <int DG, typename T>
struct GradArgs {
    using M = typename MaskOf<DG>::type;
    CsrView gt;             // A^T
    int n, tiles;
    const T* dy;            // dY_i (complete), row stride ldg
    int64_t ldg;
    const float* hub_part;
    const float* w;         // W_i, row stride ldw
    int ldw;
    const M* own_mask;      // columns recorded for Y_{i-1}
    const T* z;             // Y_{i-1} rows (RMS only), row stride ldz
    int64_t ldz;
    int norm;
    float eps;
    T* dst;                 // dY_{i-1} plane(s): ndst planes, dst_gs apart, row stride ldd
    int64_t ldd, dst_gs;
    int ndst;
    int* draws;             // tile counters of the dynamic sweep and the sign-off counter
    int* draws_done;
    // dW_i of the same block, left as workgroup partials by the inverse + dW kernel just before: summed here by
    // the first workgroups before they start on tiles, which saves a launch per block (dw_out == NULL: nothing to do)
    const float* dw_partial;
    int dw_parts;
    float* dw_out;
    // ACC (groups wider than one tile: the gradient of a block is summed over its column blocks before the epilogue):
    // dh [n][DG] float32 receives dH = Q W^T (dh_first) or has it added
    float* dh;
    bool dh_first;
    // ACC: blockIdx.y is the block mb of dH written: W_i's block 64 rows on, dh a plane of [n][64] on, the tile counters a set on
    int y_draws;
};

// dW_i[e] = sum over the workgroup partials, in a fixed order: a workgroup takes 64 entries at a time; its four
// waves each sum a contiguous quarter of the partials in ascending order (sixteen loads in flight), then the four
// sums are added in order.
template <int ELEMS>
__device__ __forceinline__ void dw_reduce_slices(const float* __restrict__ partial, int nparts, float* __restrict__ out,
                                                 float* red /* 256 floats of LDS */) {
    const int col = threadIdx.x & 63, seg = threadIdx.x >> 6;
    const int per = (nparts + 3) / 4, p0 = seg * per, p1 = min(nparts, p0 + per);
    // the last workgroups take the slices: when there are fewer tiles than waves they are the ones without a tile
    for (int slice = gridDim.x - 1 - blockIdx.x; slice < ELEMS / 64; slice += gridDim.x) {
        const float* src = partial + slice * 64 + col;
        float acc = 0.f;
        int p = p0;
        for (; p + 16 <= p1; p += 16) {
            float v[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) v[u] = src[(size_t)(p + u) * ELEMS];
#pragma unroll
            for (int u = 0; u < 16; ++u) acc += v[u];
        }
        for (; p < p1; ++p) acc += src[(size_t)p * ELEMS];
        __syncthreads();
        if (seg < 4) red[seg * 64 + col] = acc;
        __syncthreads();
        if (seg == 0) out[slice * 64 + col] = ((red[col] + red[64 + col]) + red[128 + col]) + red[192 + col];
    }
    __syncthreads();
}

// Waves per workgroup of k_grad (they share one copy of W^T in LDS).  Measured at 1M rows, Dg = 64, float32 product:
// 4 and 8 waves (16 resident waves per compute unit either way) take the same time; 6 and 10
// waves, which would allow 18 and 20 resident waves, are 20 % and 10 % slower.
// B3 as in k_block: dH = Q W^T on the bf16 pipe with eight waves per workgroup (322 -> 309 us on the 1M-node
// workload), or the float32 product with four (graphs whose rows nearly all go through the first pass: 106 us
// against 132).
constexpr int grad_waves(bool b3) { return b3 ? 8 : 4; }

template <int DG, typename T, bool DEAL, bool B3, bool ACC = false>
__global__ __launch_bounds__(64 * grad_waves(B3)) __attribute__((amdgpu_waves_per_eu(4))) void k_grad(GradArgs<DG, T> a) {
    constexpr int CPL = DG / 16;
    constexpr int GRAD_WAVES = grad_waves(B3);
    if constexpr (ACC) {
        const int mb = blockIdx.y;
        a.w += (size_t)mb * 64 * a.ldw;
        a.dh += (size_t)mb * a.n * 64;
        a.draws += mb * a.y_draws;
        a.draws_done += mb * a.y_draws;
    }
    // the partial rows of a tile's split rows requested together (hub_rows_fill) only where that spills no register:
    // these kernels sit at their 128 registers
    constexpr bool FILL_FAST = ACC || (!DEAL && sizeof(T) == 4 && DG == 64);
    __shared__ WaveLds<DG, 1> lds[GRAD_WAVES];
    const int lane = lane_id(), wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), tg = lane >> 4, tj = lane & 15;
    WaveLds<DG, 1>& L = lds[wave];
    float* st = L.st[0];
    __shared__ typename std::conditional<B3, WLdsB3<DG>, WLds<DG>>::type wl;
    static_assert(GRAD_WAVES >= 4 && sizeof(lds) >= 256 * sizeof(float), "dw_reduce_slices works with the first 256 threads");
    if (a.dw_out) dw_reduce_slices<DG * DG>(a.dw_partial, a.dw_parts, a.dw_out, reinterpret_cast<float*>(lds));
    if constexpr (B3) load_w_lds_b3<DG>(a.w, a.ldw, true, wl);
    else load_w_lds<DG>(a.w, a.ldw, true, wl);
    TileDraws td = tile_draws(a.tiles, a.draws, a.draws_done);
    TileDeal deal{0, 0, false};
    if constexpr (DEAL) deal = tile_deal(a.gt);
    int requested = tile_request(td);      // the draw that is outstanding
    int t_end = td.end;
    int t = 0;
    if (DEAL && deal.on) { t = a.gt.heavy[deal.at]; t_end = a.tiles; }
    else t = tile_drawn(td, requested);
    while (t < t_end) {
        if (!DEAL || !deal.on) requested = tile_request(td);
        const int r0 = t * 16;
        wave_sync();
        const int rpv = tile_rp_load(a.gt, r0, a.n, lane);
        // what the epilogue needs of the tile's own rows is requested first
        typename MaskOf<DG>::type own[4];
        float z[4][CPL];
#pragma unroll
        for (int reg = 0; reg < 4; ++reg) {
            const int row = r0 + 4 * reg + tg;
            const size_t rowc = (size_t)(row < a.n ? row : a.n - 1);
            if constexpr (!ACC) {
                own[reg] = a.own_mask[rowc];
                if (a.norm == GSR_NORM_RMS) load_cols<CPL, T>(a.z + rowc * a.ldz + CPL * tj, z[reg]);
            }
        }
        const bool has_hub = tile_begin(a.gt, rpv, L.rp, lane);
        if constexpr (DEAL) {
            if (!deal.on && tile_is_heavy(a.gt, rpv, L.rp, has_hub)) {    // dealt out before the sweep
                t = tile_drawn(td, requested);
                continue;
            }
        }
        // float32: Q in ordinary arithmetic, a run of the staged edges per lane group (322 us against 378 through the
        // matrix cores on the 1M-node workload; sixteen steps in flight instead of eight spill)
        if constexpr (sizeof(T) == 4) {
            tile_gather_rows<DG, FILL_FAST>(a.gt, a.hub_part, has_hub, r0, L.rp, st, lane, [&](int e_a, int e_b) {
                gather_dense_rows<DG, 8>(a.gt, a.dy, a.ldg, __builtin_amdgcn_readfirstlane(e_a),
                                               __builtin_amdgcn_readfirstlane(e_b), L.rp, L.ebuf, lane, st);
            });
        } else {
            f32x4 qacc[DG / 16];
            tile_gather<DG, FILL_FAST>(a.gt, a.hub_part, has_hub, r0, L.rp, st, lane, qacc, [&](int e_a, int e_b) {
                gather_dense_mfma<DG, T, (sizeof(T) == 4 || DG == 32) ? 16 : 8>(a.gt, a.dy, a.ldg, __builtin_amdgcn_readfirstlane(e_a),
                                         __builtin_amdgcn_readfirstlane(e_b), L.rp, L.ebuf, lane, qacc);
            });
        }
        wave_sync();
        f32x4 acc[CPL];
        if constexpr (B3) mfma_tile_b3<DG>(st, wl, acc);          // dH = Q W^T in the tile register layout
        else mfma_tile<DG>(st, wl, acc);
        // epilogue on registers: row 4 reg + tg, columns CPL tj + cb
        float dz[4][CPL];
#pragma unroll
        for (int reg = 0; reg < 4; ++reg) {
            const int row = r0 + 4 * reg + tg;
            const bool ok = row < a.n;
            if constexpr (ACC) {
#pragma unroll
                for (int cb = 0; cb < CPL; ++cb) dz[reg][cb] = acc[cb][reg];
                continue;
            }
            const uint32_t bits = ok ? (uint32_t)(own[reg] >> (CPL * tj)) & ((1u << CPL) - 1u) : 0u;
            if (a.norm == GSR_NORM_RMS) {
                // V = Z[I] * rinv, rinv = (mean Z^2 + eps)^-1/2:
                // dZ_c = [c in I] g_c rinv - Z_c (sum_t g_t Z_{I_t}) rinv^3 / DG
                float ss = 0.f, dot = 0.f;
#pragma unroll
                for (int cb = 0; cb < CPL; ++cb) {
                    ss += z[reg][cb] * z[reg][cb];
                    dot += ((bits >> cb) & 1u) ? acc[cb][reg] * z[reg][cb] : 0.f;
                }
                ss = group16_sum(ss);
                dot = group16_sum(dot);
                const float rinv = __builtin_amdgcn_rsqf(ss * (1.0f / (float)DG) + a.eps);
                const float coef = dot * (rinv * rinv * rinv) * (1.0f / (float)DG);
#pragma unroll
                for (int cb = 0; cb < CPL; ++cb) dz[reg][cb] = (((bits >> cb) & 1u) ? acc[cb][reg] * rinv : 0.f) - z[reg][cb] * coef;
            } else {
#pragma unroll
                for (int cb = 0; cb < CPL; ++cb) dz[reg][cb] = ((bits >> cb) & 1u) ? acc[cb][reg] : 0.f;
            }
        }
        // the planes that receive dZ (or the float32 sum of dH): the four rows of a plane are requested together
        if constexpr (ACC) {
            float g[4][CPL];
#pragma unroll
            for (int reg = 0; reg < 4; ++reg) {
                const int row = r0 + 4 * reg + tg;
                const int rowc = row < a.n ? row : a.n - 1;
#pragma unroll
                for (int cb = 0; cb < CPL; ++cb) g[reg][cb] = 0.f;
                if (!a.dh_first) load_cols<CPL, float>(a.dh + (size_t)rowc * DG + CPL * tj, g[reg]);
            }
#pragma unroll
            for (int reg = 0; reg < 4; ++reg) {
                const int row = r0 + 4 * reg + tg;
#pragma unroll
                for (int cb = 0; cb < CPL; ++cb) g[reg][cb] += dz[reg][cb];
                if (row < a.n) store_cols<CPL, float>(a.dh + (size_t)row * DG + CPL * tj, g[reg]);
            }
        } else {
            // JC planes at a time: all their rows are requested before the first is written back (block 1 updates C - 1
            // planes; one plane after the other took 3.2 ms against 1.2 ms for a one-plane launch at 8M rows, C = 8)
            constexpr int JC = CPL <= 2 ? 4 : 2;
            if (a.ndst == 1) {          // the common case on its own, so that it requests nothing twice
                float g[4][CPL];
#pragma unroll
                for (int reg = 0; reg < 4; ++reg) {
                    const int row = r0 + 4 * reg + tg;
                    const int rowc = row < a.n ? row : a.n - 1;
                    load_cols<CPL, T>(a.dst + (size_t)rowc * a.ldd + CPL * tj, g[reg]);
                }
#pragma unroll
                for (int reg = 0; reg < 4; ++reg) {
                    const int row = r0 + 4 * reg + tg;
#pragma unroll
                    for (int cb = 0; cb < CPL; ++cb) g[reg][cb] = stored<T>(g[reg][cb] + dz[reg][cb]);
                    if (row < a.n) store_cols<CPL, T>(a.dst + (size_t)row * a.ldd + CPL * tj, g[reg]);
                }
            } else
            for (int j0 = 0; j0 < a.ndst; j0 += JC) {
                float g[JC][4][CPL];
#pragma unroll
                for (int jj = 0; jj < JC; ++jj) {
                    const int j = j0 + jj < a.ndst ? j0 + jj : a.ndst - 1;
#pragma unroll
                    for (int reg = 0; reg < 4; ++reg) {
                        const int row = r0 + 4 * reg + tg;
                        const int rowc = row < a.n ? row : a.n - 1;
                        load_cols<CPL, T>(a.dst + (size_t)j * a.dst_gs + (size_t)rowc * a.ldd + CPL * tj, g[jj][reg]);
                    }
                }
#pragma unroll
                for (int jj = 0; jj < JC; ++jj) {
                    const int j = j0 + jj;
#pragma unroll
                    for (int reg = 0; reg < 4; ++reg) {
                        const int row = r0 + 4 * reg + tg;
#pragma unroll
                        for (int cb = 0; cb < CPL; ++cb) g[jj][reg][cb] = stored<T>(g[jj][reg][cb] + dz[reg][cb]);
                        if (row < a.n && j < a.ndst) store_cols<CPL, T>(a.dst + (size_t)j * a.dst_gs + (size_t)row * a.ldd + CPL * tj, g[jj][reg]);
                    }
                }
            }
        }
        if (DEAL && deal.on) {
            deal.at += deal.waves;
            deal.on = deal.at < a.gt.n_heavy;
            if (deal.on) t = a.gt.heavy[deal.at];
            else { t = tile_drawn(td, requested); t_end = td.end; }
        } else {
            t = tile_drawn(td, requested);
        }
    }
    tile_finish(td);
}

// ---- group sum / record of a plane --------------------------------------------------------------------
template <int DG, typename T>
struct SumArgs {
    int n;
    const T* src;           // nsrc planes, src_gs apart, row stride ld
    int64_t ld, src_gs;
    int nsrc;
    T* y0;                  // dense [n][DG] copy of the sum (NULL: not kept)
    int k, norm;
    float eps;
    Record<DG, T> out;
    bool out_given;         // out.mask holds the column sets to use
    TieSeg<DG> tie;         // where rows that select at a near-tie are listed (count == NULL: nowhere)
};

__global__ void k_zero_ints(int* p, int count) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = 0;
}

template <int DG, typename T>
__global__ __launch_bounds__(256) void k_sum(SumArgs<DG, T> a) {
    constexpr int LR = DG + 1, CPL = DG / 16;
    __shared__ float tile[4][16 * LR + 64];
    const int lane = lane_id(), tg = lane >> 4, tj = lane & 15;
    float* st = tile[threadIdx.x >> 6];
    const int nwaves = (gridDim.x * blockDim.x) >> 6, tiles = (a.n + 15) / 16;
    for (int t = (blockIdx.x * blockDim.x + threadIdx.x) >> 6; t < tiles; t += nwaves) {
        const int r0 = t * 16;
        float y[4][CPL];
#pragma unroll
        for (int reg = 0; reg < 4; ++reg) {
            const int row = r0 + 4 * reg + tg;
            load_cols<CPL, T>(a.src + (size_t)(row < a.n ? row : a.n - 1) * a.ld + CPL * tj, y[reg]);
        }
        for (int j = 1; j < a.nsrc; ++j) {
            float v[4][CPL];
#pragma unroll
            for (int reg = 0; reg < 4; ++reg) {
                const int row = r0 + 4 * reg + tg;
                load_cols<CPL, T>(a.src + (size_t)j * a.src_gs + (size_t)(row < a.n ? row : a.n - 1) * a.ld + CPL * tj, v[reg]);
            }
#pragma unroll
            for (int reg = 0; reg < 4; ++reg)
#pragma unroll
                for (int cb = 0; cb < CPL; ++cb) y[reg][cb] += v[reg][cb];
        }
        wave_sync();          // the previous tile's records have left the scratch
#pragma unroll
        for (int reg = 0; reg < 4; ++reg) {
            const int rr = 4 * reg + tg, row = r0 + rr;
            const bool ok = row < a.n;
#pragma unroll
            for (int cb = 0; cb < CPL; ++cb) y[reg][cb] = stored<T>(y[reg][cb]);
            if (ok && a.y0) store_cols<CPL, T>(a.y0 + (size_t)row * DG + CPL * tj, y[reg]);
#pragma unroll
            for (int cb = 0; cb < CPL; ++cb) st[rr * LR + CPL * tj + cb] = ok ? y[reg][cb] : 0.f;
        }
        wave_sync();
        emit_tile<DG, T>(st, r0, a.n, a.k, a.norm, a.eps, a.out, a.out_given, lane, nullptr, nullptr, a.tie);
    }
}

// ---- groups wider than one tile: D/C = 64 S, S = 2, 3 or 4 ---------------------------------------------------
// Such a group is handled as S column blocks of 64 ("sub-planes": block s of a row starts 64 s elements into it).  The
// aggregation is column-wise, so every sub-plane has a record of its own in the 64-column format (the kept values that
// fall into it, at most k, and its 64-bit mask) and the 64-column block kernels compute Y_i[:, ob] (+)= H_mb W_i[mb][ob]
// one pair (mb, ob) per launch.  What couples the sub-planes is GS, which selects over the whole row (Section 4.1),
// and the scale and the backward through it: those are the two kernels below.

template <int S, typename T>
struct WideGsArgs {
    int n;
    const T* src;           // nsrc groups, src_gs apart, row stride ld; sub-plane s of a row starts at + 64 s
    int64_t ld, src_gs;
    int nsrc;
    T* y0;                  // [S][n][64]: the sum, sub-plane by sub-plane (NULL: not kept)
    int k, norm;
    float eps;
    Record<64, T> out[S];
    bool out_given;         // out[s].mask hold the column sets to use
};

// GS of a 16-row tile of a wide group, lane (r, q) holding the q-th quarter (16 columns) of every sub-plane of row r:
// the same search as select_quarter over 16 S keys per lane; ties go to the lowest column of the whole row (sub-plane,
// then quarter, then column).  Records leave sub-plane by sub-plane in the layout emit_tile writes.
template <int S, typename T>
__global__ __launch_bounds__(256) void k_gs_wide(WideGsArgs<S, T> a) {
    constexpr int DGW = 64 * S, LRW = DGW + 1;
    constexpr int KS = sizeof(T) == 2 ? 16 : 0;
    __shared__ float tile[4][16 * LRW + 64];
    const int lane = lane_id(), tg = lane >> 4, tj = lane & 15, r = lane & 15, q = lane >> 4;
    float* st = tile[threadIdx.x >> 6];
    const int nwaves = (gridDim.x * blockDim.x) >> 6, tiles = (a.n + 15) / 16;
    for (int t = (blockIdx.x * blockDim.x + threadIdx.x) >> 6; t < tiles; t += nwaves) {
        const int r0 = t * 16;
        wave_sync();          // the previous tile's records have left the scratch
#pragma unroll
        for (int s = 0; s < S; ++s) {
            float y[4][4];
#pragma unroll
            for (int reg = 0; reg < 4; ++reg) {
                const int row = r0 + 4 * reg + tg;
                load_cols<4, T>(a.src + (size_t)(row < a.n ? row : a.n - 1) * a.ld + 64 * s + 4 * tj, y[reg]);
            }
            for (int j = 1; j < a.nsrc; ++j) {
#pragma unroll
                for (int reg = 0; reg < 4; ++reg) {
                    const int row = r0 + 4 * reg + tg;
                    float v[4];
                    load_cols<4, T>(a.src + (size_t)j * a.src_gs + (size_t)(row < a.n ? row : a.n - 1) * a.ld + 64 * s + 4 * tj, v);
#pragma unroll
                    for (int cb = 0; cb < 4; ++cb) y[reg][cb] += v[cb];
                }
            }
#pragma unroll
            for (int reg = 0; reg < 4; ++reg) {
                const int rr = 4 * reg + tg, row = r0 + rr;
                const bool ok = row < a.n;
#pragma unroll
                for (int cb = 0; cb < 4; ++cb) y[reg][cb] = stored<T>(y[reg][cb]);
                if (ok && a.y0) store_cols<4, T>(a.y0 + ((size_t)s * a.n + row) * 64 + 4 * tj, y[reg]);
#pragma unroll
                for (int cb = 0; cb < 4; ++cb) st[rr * LRW + 64 * s + 4 * tj + cb] = ok ? y[reg][cb] : 0.f;
            }
        }
        wave_sync();
        const bool valid = r0 + r < a.n;
        float x[S][16];
        uint32_t key[S][16];
        uint32_t top = 0u;
        float ss = 0.f;
#pragma unroll
        for (int s = 0; s < S; ++s)
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                x[s][j] = st[r * LRW + 64 * s + 16 * q + j];
                ss += x[s][j] * x[s][j];
                const uint32_t u = __float_as_uint(x[s][j]);
                uint32_t kk = u ^ ((uint32_t)((int32_t)u >> 31) | 0x80000000u);
                kk = kk == 0x7FFFFFFFu ? 0x80000000u : kk;          // -0 -> +0
                key[s][j] = kk >> KS;
                top = max(top, key[s][j]);
            }
        uint32_t msel[S];
        if (a.out_given) {
#pragma unroll
            for (int s = 0; s < S; ++s) msel[s] = (uint32_t)(a.out[s].mask[valid ? r0 + r : a.n - 1] >> (16 * q)) & 0xFFFFu;
        } else {
            top = quarter_max(top);
            auto count_ge = [&](uint32_t th) {
                uint32_t cnt = 0u;
#pragma unroll
                for (int s = 0; s < S; ++s)
#pragma unroll
                    for (int j = 0; j < 16; ++j) cnt += key[s][j] >= th ? 1u : 0u;
                return quarter_sum(cnt);
            };
            constexpr uint32_t span = (4u << 23) >> KS;
            const uint32_t uk = (uint32_t)a.k;
            uint32_t lo = top > span ? top - span : 0u, hi = top + 1u;
            {
                const uint32_t cnt = count_ge(lo);
                lo = (cnt >= uk && a.k < DGW) ? lo : 0u;
                uint32_t open = (cnt != uk && a.k < DGW && valid) ? 1u : 0u;
                for (int round = 0; round < 33 && ballot(open != 0u) != 0ull; ++round) {
                    const uint32_t mid = lo + ((hi - lo) >> 1);
                    const uint32_t c2 = count_ge(mid);
                    lo = c2 >= uk ? mid : lo;
                    hi = c2 >= uk ? hi : mid;
                    open = (c2 == uk || hi - lo <= 1u) ? 0u : open;
                }
            }
            // kept: every key above the threshold, and of those at the threshold the lowest columns of the row
            uint32_t mgt[S], meq[S];
            int ngt = 0;
#pragma unroll
            for (int s = 0; s < S; ++s) {
                mgt[s] = meq[s] = 0u;
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    mgt[s] |= key[s][j] > lo ? 1u << j : 0u;
                    meq[s] |= key[s][j] == lo ? 1u << j : 0u;
                }
                ngt += __popc(mgt[s]);
            }
            int need = a.k - (int)quarter_sum((uint32_t)ngt);      // ties to take, in column order
#pragma unroll
            for (int s = 0; s < S; ++s) {
                uint32_t all[4];
                quarter_all((uint32_t)__popc(meq[s]), all);
                int before = 0;
#pragma unroll
                for (int i = 0; i < 3; ++i) before += i < q ? (int)all[i] : 0;
                int take = min(max(need - before, 0), (int)__popc(meq[s]));
                msel[s] = mgt[s];
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const uint32_t sbit = ((meq[s] >> j) & 1u) & (take > 0 ? 1u : 0u);
                    msel[s] |= sbit << j;
                    take -= (int)sbit;
                }
                need -= (int)(all[0] + all[1] + all[2] + all[3]);
            }
        }
        float scale = 1.f;
        if (a.norm == GSR_NORM_RMS) scale = __builtin_amdgcn_rsqf(quarter_sum(ss) * (1.0f / (float)DGW) + a.eps);
        const int rows = min(16, a.n - r0), total = rows * a.k;
#pragma unroll
        for (int s = 0; s < S; ++s) {
            uint32_t all[4];
            quarter_all(msel[s] | (uint32_t)__popc(msel[s]) << 16, all);
            int slot = r * a.k;
#pragma unroll
            for (int i = 0; i < 3; ++i) slot += i < q ? (int)(all[i] >> 16) : 0;
            const uint64_t mask = (uint64_t)(all[0] & 0xFFFFu) | (uint64_t)(all[1] & 0xFFFFu) << 16 |
                                  (uint64_t)(all[2] & 0xFFFFu) << 32 | (uint64_t)(all[3] & 0xFFFFu) << 48;
            wave_sync();   // every lane holds its values (s = 0) / the previous sub-plane's record has left the scratch
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const uint32_t bit = (msel[s] >> j) & 1u;
                st[bit ? slot : 16 * LRW + lane] = x[s][j] * scale;      // dropped columns go to the dump words
                slot += (int)bit;
            }
            wave_sync();
            T* dst = a.out[s].vals + (size_t)r0 * a.k;
            for (int i = lane; i < total; i += 64) dst[i] = from_float<T>(st[i]);
            if (!a.out_given && q == 0 && r < rows) a.out[s].mask[r0 + r] = mask;
        }
    }
}

// Backward through GS and its scale for a wide group, after dH = sum over column blocks of Q W^T has been summed into
// dh [S][n][64]: one wave per row, lane c holding column c of every sub-plane.  dZ_c = [c in I] g_c / r - Z_c (sum_t g_t
// Z_{I_t}) / (D/C r^3) with g = dH at the recorded positions (eq. (11): only those are read); dst planes += dZ.
template <int S, typename T>
struct WideEpiArgs {
    int n;
    const float* dh;                    // [S][n][64]
    const uint64_t* mask[S];            // column sets recorded for the block's input
    const T* z;                         // rows of the block's input (RMS only): row stride ldz, sub-plane s at + s * z_sub
    int64_t ldz, z_sub;
    int norm;
    float eps;
    T* dst;                             // ndst groups, dst_gs apart, row stride ldd
    int64_t ldd, dst_gs;
    int ndst;
};

template <int S, typename T>
__global__ __launch_bounds__(256) void k_grad_epi_wide(WideEpiArgs<S, T> a) {
    constexpr int DGW = 64 * S;
    const int lane = lane_id();
    const int nwaves = (gridDim.x * blockDim.x) >> 6;
    for (int row = (blockIdx.x * blockDim.x + threadIdx.x) >> 6; row < a.n; row += nwaves) {
        float g[S], zz[S];
        bool kept[S];
        float ss = 0.f, dot = 0.f;
#pragma unroll
        for (int s = 0; s < S; ++s) {
            g[s] = a.dh[((size_t)s * a.n + row) * 64 + lane];
            kept[s] = (a.mask[s][row] >> lane) & 1ull;
            zz[s] = a.norm == GSR_NORM_RMS ? to_float(a.z[(size_t)row * a.ldz + (size_t)s * a.z_sub + lane]) : 0.f;
            ss += zz[s] * zz[s];
            dot += kept[s] ? g[s] * zz[s] : 0.f;
        }
        float rinv = 1.f, coef = 0.f;
        if (a.norm == GSR_NORM_RMS) {
            ss = sub_sum<64>(ss);
            dot = sub_sum<64>(dot);
            rinv = __builtin_amdgcn_rsqf(ss * (1.0f / (float)DGW) + a.eps);
            coef = dot * (rinv * rinv * rinv) * (1.0f / (float)DGW);
        }
#pragma unroll
        for (int s = 0; s < S; ++s) {
            const float dz = (kept[s] ? g[s] * rinv : 0.f) - zz[s] * coef;
            for (int j = 0; j < a.ndst; ++j) {
                T* p = a.dst + (size_t)j * a.dst_gs + (size_t)row * a.ldd + 64 * s + lane;
                *p = from_float<T>(to_float(*p) + dz);
            }
        }
    }
}

// ---- head: yhat = X w + b, loss = mean (yhat - t)^2 ----------------------------------------------------
template <typename T>
struct HeadArgs {
    int n, d, dg;
    const T* act;           // element (row, grp, c) at grp*gs + row*ld + c
    T* grad;                // same layout
    int64_t ld, gs;
    const float* w_out;
    const float* b_out;
    const float* target;
    float* yhat;            // may be NULL
    float* partial;         // [gridDim.x][d + 2]: dw (d), db, sum of squared errors
};

constexpr int HEAD_MAXQ = 8;  // d <= 512

template <typename T>
__global__ __launch_bounds__(256) void k_head(HeadArgs<T> a) {
    __shared__ float red[4][HEAD_MAXQ * 64 + 2];
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int nq = (a.d + 63) / 64;
    float wv[HEAD_MAXQ], dwacc[HEAD_MAXQ];
    size_t off[HEAD_MAXQ];
#pragma unroll
    for (int q = 0; q < HEAD_MAXQ; ++q) {
        const int cc = q * 64 + lane;
        const bool in = q < nq && cc < a.d;
        wv[q] = in ? a.w_out[cc] : 0.f;
        dwacc[q] = 0.f;
        off[q] = in ? (size_t)(cc / a.dg) * a.gs + (cc % a.dg) : 0;
    }
    const float bias = a.b_out[0];
    float db = 0.f, sse = 0.f;
    const int nwaves = (gridDim.x * blockDim.x) >> 6;
    for (int row = (blockIdx.x * blockDim.x + threadIdx.x) >> 6; row < a.n; row += nwaves) {
        float xv[HEAD_MAXQ];
        float dot = 0.f;
#pragma unroll
        for (int q = 0; q < HEAD_MAXQ; ++q) {
            const bool in = q < nq && q * 64 + lane < a.d;
            xv[q] = in ? to_float(a.act[off[q] + (size_t)row * a.ld]) : 0.f;
            dot += xv[q] * wv[q];
        }
        const float y = sub_sum<64>(dot) + bias;
        const float e = y - a.target[row];
        const float gy = 2.0f * e / (float)a.n;
        if (lane == 0 && a.yhat) a.yhat[row] = y;
        db += gy;
        sse += e * e;
#pragma unroll
        for (int q = 0; q < HEAD_MAXQ; ++q) {
            const bool in = q < nq && q * 64 + lane < a.d;
            dwacc[q] += xv[q] * gy;
            if (in) a.grad[off[q] + (size_t)row * a.ld] = from_float<T>(gy * wv[q]);
        }
    }
#pragma unroll
    for (int q = 0; q < HEAD_MAXQ; ++q) red[wave][q * 64 + lane] = dwacc[q];
    if (lane == 0) { red[wave][HEAD_MAXQ * 64] = db; red[wave][HEAD_MAXQ * 64 + 1] = sse; }
    __syncthreads();
    for (int i = threadIdx.x; i < a.d + 2; i += 256) {
        const int src = i < a.d ? i : HEAD_MAXQ * 64 + (i - a.d);
        a.partial[(size_t)blockIdx.x * (a.d + 2) + i] = ((red[0][src] + red[1][src]) + red[2][src]) + red[3][src];
    }
}

// One wave per output element: lane l adds partials l, l + 64, .. in that order, then the 64 lane sums are
// added in a fixed tree.  (One thread per element walking all partials in turn took 240 us whatever the size.)
__global__ __launch_bounds__(256) void k_head_reduce(const float* __restrict__ partial, int nparts, int d, int n,
                                                     float* __restrict__ dw_out, float* __restrict__ db_out,
                                                     float* __restrict__ loss_out) {
    const int i = (int)((blockIdx.x * blockDim.x + threadIdx.x) >> 6), lane = lane_id();
    if (i >= d + 2) return;
    float acc = 0.f;
    for (int p = lane; p < nparts; p += 64) acc += partial[(size_t)p * (d + 2) + i];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (lane != 0) return;
    if (i < d) dw_out[i] = acc;
    else if (i == d) db_out[0] = acc;
    else loss_out[0] = acc / (float)n;
}

// ---- layout copy: (row, grp, c) between two stride sets ---------------------------------------------------
template <typename T>
__global__ void k_copy_planes(int64_t n, int dg, int ngroups, const T* __restrict__ src, int64_t s_ld, int64_t s_gs,
                              T* __restrict__ dst, int64_t d_ld, int64_t d_gs) {
    const int64_t total = n * dg * ngroups;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int c = (int)(i % dg);
        const int64_t t = i / dg;
        const int grp = (int)(t % ngroups);
        const int64_t row = t / ngroups;
        dst[grp * d_gs + row * d_ld + c] = src[grp * s_gs + row * s_ld + c];
    }
}

// ======================================== host orchestration ===============================================

template <typename T>
struct Planes {
    T* base;
    int64_t ld, gs;
    T* grp(int i) const { return base + (size_t)i * gs; }
};

template <typename T>
static Planes<T> caller_planes(void* p, const gsr_config_t* cfg) {
    const int dg = cfg->d / cfg->c;
    if (cfg->layout == GSR_LAYOUT_ROW_MAJOR) return Planes<T>{(T*)p, (int64_t)cfg->d, (int64_t)dg};
    return Planes<T>{(T*)p, (int64_t)dg, (int64_t)cfg->n * dg};
}

template <int DG, typename T>
struct Ctx {
    using M = typename MaskOf<DG>::type;
    const gsr_graph_t* g;
    const gsr_config_t* cfg;
    hipStream_t s;
    char* ws;
    LayerWs lw;
    int tiles;
    int S;          // sub-planes of a group: 1, or D/C / 64 for groups wider than a tile (then DG = 64)
    M* saved;       // [L+1][C][S][n] column masks kept from the forward sweep, or NULL
    // rows kept because they selected at a near-tie (cfg->save_indices == 2), per segment (layer, slot), or NULL
    int* tie_counts;
    uint32_t* tie_rows;
    M* tie_masks;
    int tie_cap;
    TieSeg<DG> tie_seg(int layer, int slot) const {
        if (!tie_counts || layer < 0) return TieSeg<DG>{nullptr, nullptr, nullptr, 0, 0.f};
        const size_t seg = (size_t)layer * cfg->c + slot;
        return TieSeg<DG>{tie_counts + seg * TIE_SUB * TIE_COUNTER_STRIDE, tie_rows + seg * TIE_SUB * tie_cap,
                          tie_masks + seg * TIE_SUB * tie_cap, tie_cap, cfg->tie_tol};
    }
    // Record slot `slot` of layer `layer`: the values always live in the slot (they are rebuilt),
    // the mask in the slot, or in the kept store when indices are saved.
    Record<DG, T> rec(int slot, int layer = 0, int sub = 0) const {
        Record<DG, T> r;
        if (slot < 0) { r.vals = nullptr; r.mask = nullptr; return r; }
        r.vals = (T*)(ws + lw.rec_vals[slot * S + sub]);
        r.mask = saved ? saved + (((size_t)layer * cfg->c + slot) * S + sub) * (size_t)cfg->n : (M*)(ws + lw.rec_mask[slot * S + sub]);
        return r;
    }
    T* y0() const { return (T*)(ws + lw.y0); }
    float* dh() const { return (float*)(ws + lw.dh); }
    float* hplane() const { return (float*)(ws + lw.h); }
    float* dw_partial() const { return (float*)(ws + lw.dw_partial); }
    float* hub_part() const { return (float*)(ws + lw.hub_partial); }
    float* hub_part2() const { return (float*)(ws + lw.hub_partial2); }
    uint8_t* hub_cols() const { return (uint8_t*)(ws + lw.hub_cols); }
    float* hub_vals() const { return (float*)(ws + lw.hub_vals); }
    bool hub_by_value() const { return g->hub_values == 2 || (g->hub_values == 1 && 2 * cfg->k <= DG); }
};

// Workgroups of 256 threads one CU keeps resident for a kernel, and the persistent grid that
// fills the chip with them: a multiple of 8 (one share per XCD), never above g->grid, which
// sizes the per-workgroup partial buffers.
static int resident_blocks(const void* kernel, int threads = 256) {
    int nb = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, kernel, threads, 0) != hipSuccess || nb < 1) nb = 1;
    return nb;
}
static unsigned persistent_grid(const gsr_graph_t* g, int per_cu) {
    int grid = g->num_cus * per_cu / 8 * 8;
    if (grid > g->grid) grid = g->grid;
    if (grid < 8) grid = 8;
    return (unsigned)grid;
}

template <int DG, typename T>
static void launch_sum(const Ctx<DG, T>& x, const T* src, int64_t ld, int64_t gs, int nsrc, T* y0,
                       const Record<DG, T>& out, bool out_given = false,
                       TieSeg<DG> tie = TieSeg<DG>{nullptr, nullptr, nullptr, 0, 0.f}) {
    SumArgs<DG, T> a;
    a.tie = tie;
    a.n = (int)x.cfg->n; a.src = src; a.ld = ld; a.src_gs = gs; a.nsrc = nsrc; a.y0 = y0;
    a.k = x.cfg->k; a.norm = x.cfg->norm; a.eps = x.cfg->eps;
    a.out = out; a.out_given = out_given;
    ProfScope prof(KC_SUM, x.s);
    hipLaunchKernelGGL((k_sum<DG, T>), dim3((unsigned)x.g->grid * 2), dim3(256), 0, x.s, a);
}

template <int DG, typename T>
static void launch_hub_records(const Ctx<DG, T>& x, const Record<DG, T>& in) {
    const HubPlan& h = x.g->a.hub;
    if (h.n_chunks == 0) return;
    HubChunks hc{h.ce0, h.ce1, h.n_chunks, x.g->long_rows};
    ProfScope prof(KC_HUB, x.s);
    if constexpr (sizeof(T) == 4) {
        if (x.hub_by_value()) {
            hipLaunchKernelGGL((k_record_columns<DG>), dim3((unsigned)((x.cfg->n + 255) / 256)), dim3(256), 0, x.s, (int)x.cfg->n,
                               x.cfg->k, (const typename MaskOf<DG>::type*)in.mask, x.hub_cols());
            hub_values_variant(x.cfg->k, [&](auto lg, auto kq) {
                hipLaunchKernelGGL((k_hub_values<DG, decltype(lg)::value, decltype(kq)::value>),
                                   dim3(hub_grid(h.n_chunks)), dim3(256), 0, x.s, make_view(x.g, false), hc,
                                   (const float*)in.vals, (const uint8_t*)x.hub_cols(), x.cfg->k, x.hub_part());
            });
            return;
        }
    }
    hipLaunchKernelGGL((k_hub_records<DG, T>), dim3(hub_grid(h.n_chunks)), dim3(256), 0, x.s,
                       make_view(x.g, false), hc, (const T*)in.vals, (const typename MaskOf<DG>::type*)in.mask, x.cfg->k,
                       x.hub_part());
}

template <int DG, typename T>
static void launch_hub_dense(const Ctx<DG, T>& x, const T* plane, int64_t ld) {
    const HubPlan& h = x.g->at.hub;
    if (h.n_chunks == 0) return;
    HubChunks hc{h.ce0, h.ce1, h.n_chunks, x.g->long_rows};
    ProfScope prof(KC_HUB, x.s);
    hipLaunchKernelGGL((k_hub_dense<DG, T>), dim3(hub_grid(h.n_chunks)), dim3(256), 0, x.s,
                       make_view(x.g, true), hc, plane, ld, x.hub_part());
}

// Both first passes of a block's backward (records over A into hub_part, dY rows over A^T into hub_part2).
// Returns false if there is nothing to do.
template <int DG, typename T>
static bool launch_hub_both(const Ctx<DG, T>& x, const Record<DG, T>& in, const T* dy, int64_t ldg) {
    const HubPlan &ha = x.g->a.hub, &ht = x.g->at.hub;
    if (ha.n_chunks == 0 && ht.n_chunks == 0) return false;
    HubChunks ca{ha.ce0, ha.ce1, ha.n_chunks, x.g->long_rows}, ct{ht.ce0, ht.ce1, ht.n_chunks, x.g->long_rows};
    ProfScope prof(KC_HUB, x.s);
    const unsigned gx = hub_grid(std::max(ha.n_chunks, ht.n_chunks));
    if constexpr (sizeof(T) == 4) {
        if (x.hub_by_value()) {
            hipLaunchKernelGGL((k_record_columns<DG>), dim3((unsigned)((x.cfg->n + 255) / 256)), dim3(256), 0, x.s, (int)x.cfg->n,
                               x.cfg->k, (const typename MaskOf<DG>::type*)in.mask, x.hub_cols());
            // (two launches: as the two rows of one grid, as the dealing variant runs them, they took 50 us longer on the
            // Table-1-shaped graph than one after the other)
            if (ha.n_chunks > 0)
                hub_values_variant(x.cfg->k, [&](auto lg, auto kq) {
                    hipLaunchKernelGGL((k_hub_values<DG, decltype(lg)::value, decltype(kq)::value>),
                                       dim3(hub_grid(ha.n_chunks)), dim3(256), 0, x.s, make_view(x.g, false),
                                       ca, (const float*)in.vals, (const uint8_t*)x.hub_cols(), x.cfg->k, x.hub_part());
                });
            if (ht.n_chunks > 0)
                hipLaunchKernelGGL((k_hub_dense<DG, T>), dim3(hub_grid(ht.n_chunks)), dim3(256), 0, x.s,
                                   make_view(x.g, true), ct, dy, ldg, x.hub_part2());
            return true;
        }
    }
    hipLaunchKernelGGL((k_hub_both<DG, T>), dim3(gx, 2), dim3(256), 0, x.s, make_view(x.g, false), ca, (const T*)in.vals,
                       (const typename MaskOf<DG>::type*)in.mask, x.cfg->k, x.hub_part(), make_view(x.g, true), ct, dy, ldg,
                       x.hub_part2());
    return true;
}

// How the backward of a block takes dW_i.  float32: the inverse kernel (sixteen waves per compute unit, row-wise sums as
// in the forward kernel, so f_i is recomputed in the arithmetic it was computed in) leaves H in memory and k_dw takes
// H^T dY_i in a pass of its own: 476 -> 320 + 112 us per block on the 1M-node workload (-3.8 % on the step) for 512 more
// bytes per row.  bf16 storage at D/C = 64: split as well (240 + 81 us against 340 fused at 1M nodes once the inverse
// requested its own rows after the gather; 253 + 80 against 337 before).  bf16 storage at D/C = 32: the fused kernel
// (inverse + dW accumulators at eight waves per compute unit), whose neighbour sums hide on the bf16 pipe: 1,243 + 228 us
// split against 1,205 fused at 8M nodes (1,150 fused now).
// Graphs with fewer than two tiles per resident wave, or with all rows in the first pass (a launch there is one or two
// short tiles per wave, and two more launches per block cost more than the occupancy gains: 0.56 against 0.70 ms per
// step on the 2,000-node workload, 487 against 496 ms on the Table-1-shaped one, 8.7 against 9.0 ms on the 100k-node
// one - which was better split, 12.0 against 12.3 ms, while a tile's split rows still cost a memory round trip each)
// keep the fused kernel in float32 as well; it uses the same row-wise sums, so whichever way a block's backward runs
// it rebuilds the bits the plain inverse rebuilds.
template <int DG, typename T>
static bool split_dw(const gsr_graph_t* g) { return (sizeof(T) == 4 || DG == 64) && g->split_backward; }

// mode 0: forward (+), 1: inverse (-), 2: inverse (-) with dW
template <int DG, typename T>
static unsigned launch_block(const Ctx<DG, T>& x, int mode, const Record<DG, T>& in, const float* w, T* plane, int64_t ld,
                             const Record<DG, T>& out, bool out_given, const T* dy, int64_t ldg, bool first_pass_done = false,
                             TieSeg<DG> tie = TieSeg<DG>{nullptr, nullptr, nullptr, 0, 0.f}, int ldw = DG, float* h_out = nullptr,
                             const float* hub_part = nullptr, float* dw_partial = nullptr, int ygrid = 1) {
    if (!first_pass_done) launch_hub_records<DG, T>(x, in);
    BlockArgs<DG, T> a;
    a.tie = tie;
    a.h_out = h_out;
    a.g = make_view(x.g, false);
    a.n = (int)x.cfg->n; a.tiles = x.tiles;
    a.in = in; a.k = x.cfg->k;
    a.hub_part = hub_part ? hub_part : x.hub_part(); a.w = w; a.ldw = ldw; a.plane = plane; a.ld = ld;
    a.out = out; a.out_given = out_given;
    a.norm = x.cfg->norm; a.eps = x.cfg->eps; a.dy = dy; a.ldg = ldg; a.dw_partial = dw_partial ? dw_partial : x.dw_partial();
    if (mode != 2) tile_counters(x.g, &a.draws, &a.draws_done);
    else a.draws = a.draws_done = nullptr;
    const bool b3 = mode != 0 || !x.g->long_rows;       // (see k_block)
    const dim3 block(64 * block_waves(mode == 2, b3));
    ProfScope prof(mode == 0 ? KC_BLOCK_FWD : mode == 1 ? KC_BLOCK_INV : KC_BLOCK_BWD, x.s);
    unsigned grid = 0;
    a.y_dw_partial = (size_t)x.g->grid * DG * DG;
    a.y_draws = kTileCounterSet;
    auto go = [&](auto plain, auto deal, int per_cu) {
        grid = persistent_grid(x.g, per_cu);
        // (ygrid column blocks written by one launch: the resident workgroups are shared out between them)
        if (ygrid > 1) grid = std::max(8u, grid / (unsigned)ygrid / 8 * 8);
        if (heavy_first(a.g.n_heavy, x.tiles, grid * (block.x / 64) / 4)) hipLaunchKernelGGL(deal, dim3(grid, (unsigned)ygrid), block, 0, x.s, a);
        else hipLaunchKernelGGL(plain, dim3(grid, (unsigned)ygrid), block, 0, x.s, a);
    };
    if constexpr (DG == 64) {
        if (ygrid > 1) {
            if (mode == 0 && b3) {
                static const int per_cu = resident_blocks((const void*)k_block<DG, T, +1, false, false, true, true>, 512);
                go(k_block<DG, T, +1, false, false, true, true>, k_block<DG, T, +1, false, true, true, true>, per_cu);
            } else if (mode == 0) {
                static const int per_cu = resident_blocks((const void*)k_block<DG, T, +1, false, false, false, true>, 256);
                go(k_block<DG, T, +1, false, false, false, true>, k_block<DG, T, +1, false, true, false, true>, per_cu);
            } else if (mode == 1) {
                static const int per_cu = resident_blocks((const void*)k_block<DG, T, -1, false, false, true, true>, 512);
                go(k_block<DG, T, -1, false, false, true, true>, k_block<DG, T, -1, false, true, true, true>, per_cu);
            } else {
                static const int per_cu = resident_blocks((const void*)k_block<DG, T, -1, true, false, true, true>, 256);
                go(k_block<DG, T, -1, true, false, true, true>, k_block<DG, T, -1, true, true, true, true>, per_cu);
            }
            return grid;
        }
    }
    if (mode == 0 && b3) {
        static const int per_cu = resident_blocks((const void*)k_block<DG, T, +1, false, false, true>, 512);
        go(k_block<DG, T, +1, false, false, true>, k_block<DG, T, +1, false, true, true>, per_cu);
    } else if (mode == 0) {
        static const int per_cu = resident_blocks((const void*)k_block<DG, T, +1, false, false, false>, 256);
        go(k_block<DG, T, +1, false, false, false>, k_block<DG, T, +1, false, true, false>, per_cu);
    } else if (mode == 1) {
        static const int per_cu = resident_blocks((const void*)k_block<DG, T, -1, false, false, true>, 512);
        go(k_block<DG, T, -1, false, false, true>, k_block<DG, T, -1, false, true, true>, per_cu);
    } else {
        static const int per_cu = resident_blocks((const void*)k_block<DG, T, -1, true, false, true>, 256);
        go(k_block<DG, T, -1, true, false, true>, k_block<DG, T, -1, true, true, true>, per_cu);
    }
    return grid;
}

template <int DG, typename T>
static void launch_grad(const Ctx<DG, T>& x, const T* dy, int64_t ldg, const float* w,
                        const typename MaskOf<DG>::type* own_mask, const T* z,
                        int64_t ldz, T* dst, int64_t ldd, int64_t dst_gs, int ndst, int dw_parts, float* dw_out,
                        bool first_pass_done = false) {
    if (!first_pass_done) launch_hub_dense<DG, T>(x, dy, ldg);
    GradArgs<DG, T> a;
    a.ldw = DG; a.dh = nullptr; a.dh_first = false;
    a.gt = make_view(x.g, true);
    a.n = (int)x.cfg->n; a.tiles = x.tiles; a.dy = dy; a.ldg = ldg; a.hub_part = first_pass_done ? x.hub_part2() : x.hub_part();
    a.w = w;
    a.own_mask = own_mask; a.z = z; a.ldz = ldz; a.norm = x.cfg->norm; a.eps = x.cfg->eps;
    a.dst = dst; a.ldd = ldd; a.dst_gs = dst_gs; a.ndst = ndst;
    a.dw_partial = x.dw_partial(); a.dw_parts = dw_parts; a.dw_out = dw_out;
    tile_counters(x.g, &a.draws, &a.draws_done);
    ProfScope prof(KC_GRAD, x.s);
    auto go = [&](auto plain, auto deal, int per_cu, unsigned threads) {
        const unsigned grid = persistent_grid(x.g, per_cu);
        if (heavy_first(a.gt.n_heavy, x.tiles, grid * (threads / 64) / 4)) hipLaunchKernelGGL(deal, dim3(grid), dim3(threads), 0, x.s, a);
        else hipLaunchKernelGGL(plain, dim3(grid), dim3(threads), 0, x.s, a);
    };
    if (!x.g->long_rows) {
        static const int per_cu = resident_blocks((const void*)k_grad<DG, T, false, true>, 512);
        go(k_grad<DG, T, false, true>, k_grad<DG, T, true, true>, per_cu, 512u);
    } else {
        static const int per_cu = resident_blocks((const void*)k_grad<DG, T, false, false>, 256);
        go(k_grad<DG, T, false, false>, k_grad<DG, T, true, false>, per_cu, 256u);
    }
}

// After a record was taken again from rebuilt rows during the inverse sweep: the rows listed for that application of
// GS in the forward sweep get their kept column sets back (values from the same rebuilt rows).
template <int DG, typename T>
// (red: a reduction of dW_i's partials for the launch to take along, or NULL; returns whether it was taken)
static bool launch_tie_fixup(const Ctx<DG, T>& x, const TieSeg<DG>& tie, const T* plane, int64_t ld, const Record<DG, T>& out,
                             const DwReduceJob* red = nullptr) {
    if (!tie.count) return false;
    ProfScope prof(KC_TIE, x.s);
    const unsigned blocks = (unsigned)std::min((TIE_SUB * tie.cap + 63) / 64 / 4 * 4 + 4, 1024);     // 4 waves each: a multiple of TIE_SUB waves
    DwReduceJob job{nullptr, 0, 0, nullptr, 0, 0, 0};
    unsigned more = 0;
    if (red) {
        job = *red;
        job.fix_blocks = (int)blocks;
        more = (unsigned)((job.elems + DW_REDUCE_ENTRIES - 1) / DW_REDUCE_ENTRIES);
    }
    hipLaunchKernelGGL((k_tie_fixup<DG, T>), dim3(blocks + more), dim3(256), 0, x.s, tie, plane, ld, x.cfg->k, x.cfg->norm, x.cfg->eps, out, job);
    return red != nullptr;
}

// dW_i's workgroup partials from H (in x.hplane()) and dY_i; returns their number
template <int DG, typename T>
static unsigned launch_dw(const Ctx<DG, T>& x, const T* dy, int64_t ldg, const TieSeg<DG>& tie = TieSeg<DG>{nullptr, nullptr, nullptr, 0, 0.f},
                          const T* fix_plane = nullptr, int64_t fix_ld = 0, const Record<DG, T>* fix_out = nullptr,
                          float* dw_partial = nullptr) {
    DwArgs<DG, T> a;
    a.n = (int)x.cfg->n; a.tiles = x.tiles; a.h = x.hplane(); a.dy = dy; a.ldg = ldg;
    a.dw_partial = dw_partial ? dw_partial : x.dw_partial();
    a.tie = fix_out ? tie : TieSeg<DG>{nullptr, nullptr, nullptr, 0, 0.f};
    a.fix_plane = fix_plane; a.fix_ld = fix_ld; a.k = x.cfg->k; a.norm = x.cfg->norm; a.eps = x.cfg->eps;
    a.fix_out = fix_out ? *fix_out : x.rec(-1);
    ProfScope prof(KC_DW, x.s);
    static const int per_cu = resident_blocks((const void*)k_dw<DG, T>, 256);
    const unsigned grid = persistent_grid(x.g, per_cu);
    hipLaunchKernelGGL((k_dw<DG, T>), dim3(grid), dim3(256), 0, x.s, a);
    return grid;
}

// ---- groups wider than one tile (see k_gs_wide): D/C = 64 S as S sub-planes of 64 columns -----------------------
// Sub-plane s of group i of a plane set p starts 64 s elements into the group's rows (both caller layouts and the
// step's arena keep a group's columns adjacent in a row), so the 64-column kernels work on it in place with the row
// stride of the set.  W_i is D/C x D/C row-major; its block (mb, ob) starts at w + 64 mb D/C + 64 ob with row stride D/C.

// dH_mb (+)= (A^T dY_ob) W_i[mb][ob]^T: the gradient kernel without its epilogue (always the bf16-pipe variant)
template <typename T>
static void launch_grad_acc(const Ctx<64, T>& x, const T* dy, int64_t ldg, const float* w, int ldw, float* dh, bool first,
                            bool first_pass_done, int ygrid = 1) {
    if (!first_pass_done) launch_hub_dense<64, T>(x, dy, ldg);
    GradArgs<64, T> a;
    a.gt = make_view(x.g, true);
    a.n = (int)x.cfg->n; a.tiles = x.tiles; a.dy = dy; a.ldg = ldg; a.hub_part = x.hub_part();
    a.w = w; a.ldw = ldw;
    a.own_mask = nullptr; a.z = nullptr; a.ldz = 0; a.norm = x.cfg->norm; a.eps = x.cfg->eps;
    a.dst = nullptr; a.ldd = 0; a.dst_gs = 0; a.ndst = 0;
    a.dw_partial = nullptr; a.dw_parts = 0; a.dw_out = nullptr;
    a.dh = dh; a.dh_first = first;
    a.y_draws = kTileCounterSet;
    tile_counters(x.g, &a.draws, &a.draws_done);
    ProfScope prof(KC_GRAD, x.s);
    static const int per_cu = resident_blocks((const void*)k_grad<64, T, false, true, true>, 512);
    unsigned grid = persistent_grid(x.g, per_cu);
    // (ygrid blocks of dH from one launch, blockIdx.y = mb: the resident workgroups are shared out between them)
    if (ygrid > 1) grid = std::max(8u, grid / (unsigned)ygrid / 8 * 8);
    if (heavy_first(a.gt.n_heavy, x.tiles, grid * 2)) hipLaunchKernelGGL((k_grad<64, T, true, true, true>), dim3(grid, (unsigned)ygrid), dim3(512), 0, x.s, a);
    else hipLaunchKernelGGL((k_grad<64, T, false, true, true>), dim3(grid, (unsigned)ygrid), dim3(512), 0, x.s, a);
}

// GS over the whole rows of a wide group (sum of nsrc groups first when nsrc > 1), records of slot `slot`
template <int S, typename T>
static void launch_gs_wide_s(const Ctx<64, T>& x, const T* src, int64_t ld, int64_t gs, int nsrc, T* y0, int slot, int layer,
                             bool given) {
    WideGsArgs<S, T> a;
    a.n = (int)x.cfg->n; a.src = src; a.ld = ld; a.src_gs = gs; a.nsrc = nsrc; a.y0 = y0;
    a.k = x.cfg->k; a.norm = x.cfg->norm; a.eps = x.cfg->eps;
    for (int s = 0; s < S; ++s) a.out[s] = x.rec(slot, layer, s);
    a.out_given = given;
    ProfScope prof(KC_SUM, x.s);
    hipLaunchKernelGGL((k_gs_wide<S, T>), dim3((unsigned)x.g->grid * 2), dim3(256), 0, x.s, a);
}
template <typename T>
static void launch_gs_wide(const Ctx<64, T>& x, const T* src, int64_t ld, int64_t gs, int nsrc, T* y0, int slot, int layer,
                           bool given = false) {
    if (x.S == 2) launch_gs_wide_s<2, T>(x, src, ld, gs, nsrc, y0, slot, layer, given);
    else if (x.S == 3) launch_gs_wide_s<3, T>(x, src, ld, gs, nsrc, y0, slot, layer, given);
    else launch_gs_wide_s<4, T>(x, src, ld, gs, nsrc, y0, slot, layer, given);
}

template <int S, typename T>
static void launch_epi_wide_s(const Ctx<64, T>& x, int slot, int layer, const T* z, int64_t ldz, int64_t z_sub, T* dst, int64_t ldd,
                              int64_t dst_gs, int ndst) {
    WideEpiArgs<S, T> a;
    a.n = (int)x.cfg->n; a.dh = x.dh();
    for (int s = 0; s < S; ++s) a.mask[s] = x.rec(slot, layer, s).mask;
    a.z = z; a.ldz = ldz; a.z_sub = z_sub; a.norm = x.cfg->norm; a.eps = x.cfg->eps;
    a.dst = dst; a.ldd = ldd; a.dst_gs = dst_gs; a.ndst = ndst;
    ProfScope prof(KC_GRAD, x.s);
    hipLaunchKernelGGL((k_grad_epi_wide<S, T>), dim3((unsigned)x.g->grid * 4), dim3(256), 0, x.s, a);
}
template <typename T>
static void launch_epi_wide(const Ctx<64, T>& x, int slot, int layer, const T* z, int64_t ldz, int64_t z_sub, T* dst, int64_t ldd,
                            int64_t dst_gs, int ndst) {
    if (x.S == 2) launch_epi_wide_s<2, T>(x, slot, layer, z, ldz, z_sub, dst, ldd, dst_gs, ndst);
    else if (x.S == 3) launch_epi_wide_s<3, T>(x, slot, layer, z, ldz, z_sub, dst, ldd, dst_gs, ndst);
    else launch_epi_wide_s<4, T>(x, slot, layer, z, ldz, z_sub, dst, ldd, dst_gs, ndst);
}

// First pass over the records of a wide group's S column blocks in one launch, value by value (float32 records, S = 2
// or 3, 2 k <= D/C, a graph whose first pass runs that way): the row's k kept values are collected from the S records
// with their columns in the whole row (k_record_columns_wide), and one pass sums them into rows of D/C sums per
// chunk, written as S arrays of partial rows [chunks][64].  Returns false where it does not apply (then each column
// block has a first pass of its own).
template <typename T>
static bool launch_hub_values_wide(const Ctx<64, T>& x, int in_slot, int layer) {
    if constexpr (sizeof(T) != 4) {
        return false;
    } else {
        const HubPlan& h = x.g->a.hub;
        const int S = x.S, k = x.cfg->k;
        if (!x.g->hub_values || S < 2 || S > 3 || 2 * k > 64 * S || h.n_chunks == 0) return false;
        HubChunks hc{h.ce0, h.ce1, h.n_chunks, x.g->long_rows};
        ProfScope prof(KC_HUB, x.s);
        const unsigned rows_grid = (unsigned)((x.cfg->n + 255) / 256);
        auto go = [&](auto sc) {
            constexpr int SS = decltype(sc)::value;
            WideRecords<SS> r;
            for (int sub = 0; sub < SS; ++sub) {
                const Record<64, T> rec = x.rec(in_slot, layer, sub);
                r.vals[sub] = (const float*)rec.vals;
                r.mask[sub] = (const uint64_t*)rec.mask;
            }
            hipLaunchKernelGGL((k_record_columns_wide<SS>), dim3(rows_grid), dim3(256), 0, x.s, (int)x.cfg->n, k, r, x.hub_vals(),
                               x.hub_cols());
            hub_values_variant_wide(k, [&](auto lg, auto kq) {
                hipLaunchKernelGGL((k_hub_values<64 * SS, decltype(lg)::value, decltype(kq)::value>), dim3(hub_grid(h.n_chunks)),
                                   dim3(256), 0, x.s, make_view(x.g, false), hc, (const float*)x.hub_vals(),
                                   (const uint8_t*)x.hub_cols(), k, x.hub_part());
            });
        };
        if (S == 2) go(std::integral_constant<int, 2>{});
        else go(std::integral_constant<int, 3>{});
        return true;
    }
}

// plane (+/-)= f_i(Y_{i-1}) for one group: the S x S products of 64 x 64 blocks as S launches of the 64-column block
// kernel.  mode as launch_block; dw_i (mode 2): D/C x D/C, receives dW_i.
template <typename T>
static void wide_block(const Ctx<64, T>& x, int mode, int in_slot, int layer, const float* wi, T* plane, int64_t ld, const T* dy,
                       int64_t ldg, float* dw_i) {
    const int S = x.S, dgw = 64 * S;
    const Record<64, T> none = x.rec(-1);
    const TieSeg<64> no_tie{nullptr, nullptr, nullptr, 0, 0.f};
    // the first pass over the records of all S column blocks at once where it runs value by value (float32, two or
    // three blocks): the partial rows of block mb are then at hub_part + mb * chunks * 64
    const bool one_pass = launch_hub_values_wide<T>(x, in_slot, layer);
    const size_t part_stride = (size_t)x.g->a.hub.n_chunks * 64;
    const size_t dw_set = (size_t)x.g->grid * 64 * 64;
    unsigned nparts = 0;
    // One launch per input block mb writes all S column blocks (blockIdx.y = ob: W_i's block, the plane's and dY's
    // columns, the dW partials and the tile counters move on with it), sharing the resident waves out between them:
    // a launch per pair (mb, ob) is one short tile per wave on a long-row graph and as long as its slowest wave.
    // (Without the one first pass for all blocks, the pass over block mb's records comes first, inside launch_block.)
    const bool split = mode == 2 && split_dw<64, T>(x.g);
    for (int mb = 0; mb < S; ++mb) {
        const float* part = one_pass ? x.hub_part() + mb * part_stride : nullptr;
        const float* wmb = wi + (size_t)mb * 64 * dgw;
        if (split) {
            // the inverse of all column blocks, leaving H_mb (written once, by the workgroups of ob = 0), then dW_i's
            // blocks (mb, ob) = H_mb^T dY_i[:, ob], a pass over H_mb each, into partial sets of their own
            launch_block<64, T>(x, 1, x.rec(in_slot, layer, mb), wmb, plane, ld, none, false, nullptr, 0, one_pass, no_tie, dgw,
                                x.hplane(), part, nullptr, S);
            for (int ob = 0; ob < S; ++ob)
                nparts = launch_dw<64, T>(x, dy + 64 * ob, ldg, no_tie, nullptr, 0, nullptr,
                                          x.dw_partial() + (size_t)(mb * S + ob) * dw_set);
        } else {
            nparts = launch_block<64, T>(x, mode, x.rec(in_slot, layer, mb), wmb, plane, ld, none, false, dy, ldg, one_pass, no_tie,
                                         dgw, nullptr, part, x.dw_partial() + (size_t)(mb * S) * dw_set, S);
        }
    }
    // dW_i: its S x S blocks from their partial sets in one launch (every launch of a kind has the same grid)
    if (mode == 2) {
        ProfScope prof(KC_DW_REDUCE, x.s);
        hipLaunchKernelGGL(k_dw_reduce, dim3(64 * 64 / DW_REDUCE_ENTRIES, (unsigned)(S * S)), dim3(256), 0, x.s, (const float*)x.dw_partial(),
                           (int)nparts, 64 * 64, dw_i, 64, dgw, dw_set, S);
    }
}

template <typename T>
static void wide_forward(const Ctx<64, T>& x, const float* w, const Planes<T>& p, bool slot0_ready, int layer) {
    const int C = x.cfg->c, dgw = 64 * x.S;
    if (!slot0_ready) launch_gs_wide<T>(x, p.grp(1), p.ld, p.gs, C - 1, nullptr, 0, layer);
    for (int i = 1; i <= C; ++i) {
        wide_block<T>(x, 0, i - 1, layer, w + (size_t)(i - 1) * dgw * dgw, p.grp(i - 1), p.ld, nullptr, 0, nullptr);
        if (i < C) launch_gs_wide<T>(x, p.grp(i - 1), p.ld, p.gs, 1, nullptr, i, layer);
        else if (C == 2) launch_gs_wide<T>(x, p.grp(i - 1), p.ld, p.gs, 1, nullptr, 0, layer + 1);
    }
}

template <typename T>
static void wide_inverse(const Ctx<64, T>& x, const float* w, const Planes<T>& p) {
    const int C = x.cfg->c, dgw = 64 * x.S;
    for (int i = 1; i < C; ++i) launch_gs_wide<T>(x, p.grp(i - 1), p.ld, p.gs, 1, nullptr, i, 0);
    for (int i = C; i >= 1; --i) {
        if (i == 1 && C > 2) launch_gs_wide<T>(x, p.grp(1), p.ld, p.gs, C - 1, nullptr, 0, 0);
        wide_block<T>(x, 1, i - 1, 0, w + (size_t)(i - 1) * dgw * dgw, p.grp(i - 1), p.ld, nullptr, 0, nullptr);
        if (i == 2 && C == 2) launch_gs_wide<T>(x, p.grp(1), p.ld, p.gs, 1, nullptr, 0, 0);
    }
}

// as layer_backward_impl
template <typename T>
static void wide_backward(const Ctx<64, T>& x, const float* w, const Planes<T>& y, const Planes<T>& dy, float* dw_out, bool slots_ready,
                          int layer, bool in_step) {
    const int C = x.cfg->c, S = x.S, dgw = 64 * S;
    const int64_t n = x.cfg->n;
    const bool given = x.saved != nullptr;
    if (!slots_ready)
        for (int i = 1; i < C; ++i) launch_gs_wide<T>(x, y.grp(i - 1), y.ld, y.gs, 1, nullptr, i, layer, given);
    for (int i = C; i >= 1; --i) {
        const float* wi = w + (size_t)(i - 1) * dgw * dgw;
        const T* z;          // rows of Y_{i-1}: row stride ldz, sub-plane s at + s * z_sub
        int64_t ldz, z_sub;
        if (i >= 2) { z = y.grp(i - 2); ldz = y.ld; z_sub = 64; }
        else if (C == 2) { z = y.grp(1); ldz = y.ld; z_sub = 64; }      // Y_0 = X_2, rebuilt just before
        else {
            launch_gs_wide<T>(x, y.grp(1), y.ld, y.gs, C - 1, x.y0(), 0, layer, given);
            z = x.y0(); ldz = 64; z_sub = n * 64;
        }
        wide_block<T>(x, 2, i - 1, layer, wi, y.grp(i - 1), y.ld, dy.grp(i - 1), dy.ld, dw_out + (size_t)(i - 1) * dgw * dgw);
        // the record of the rebuilt X_i, where the next block or the layer below needs it
        if (i < C) {
            if (!(in_step && layer == 0)) launch_gs_wide<T>(x, y.grp(i - 1), y.ld, y.gs, 1, nullptr, i, given ? layer - 1 : 0, given);
        } else if (C == 2) {
            launch_gs_wide<T>(x, y.grp(i - 1), y.ld, y.gs, 1, nullptr, 0, layer, given);      // X_2 = Y_0 of this layer
        }
        // dH_mb = sum_ob (A^T dY_i[:, ob]) W_i[mb][ob]^T, then back through GS of the whole row
        // (one launch per column block ob of dY_i for all S blocks of dH: blockIdx.y = mb)
        for (int ob = 0; ob < S; ++ob)
            launch_grad_acc<T>(x, dy.grp(i - 1) + 64 * ob, dy.ld, wi + 64 * ob, dgw, x.dh(), ob == 0, false, S);
        if (i >= 2) launch_epi_wide<T>(x, i - 1, layer, z, ldz, z_sub, dy.grp(i - 2), dy.ld, dy.gs, 1);
        else launch_epi_wide<T>(x, 0, layer, z, ldz, z_sub, dy.grp(1), dy.ld, dy.gs, C - 1);
    }
}

// eq. (6).  slot0_ready: the record of Y_0 is already in slot 0 (C = 2: it is the record of the
// previous layer's Y_2, emitted when that plane was written).  `layer`: index of the layer inside
// a step (selects the kept masks when indices are saved; 0 otherwise).
template <int DG, typename T>
static void layer_forward_impl(const Ctx<DG, T>& x, const float* w, const Planes<T>& p, bool slot0_ready, int layer = 0) {
    if constexpr (DG == 64) {
        if (x.S > 1) { wide_forward<T>(x, w, p, slot0_ready, layer); return; }
    }
    const int C = x.cfg->c;
    if (!slot0_ready) launch_sum<DG, T>(x, p.grp(1), p.ld, p.gs, C - 1, nullptr, x.rec(0, layer), false, x.tie_seg(layer, 0));
    for (int i = 1; i <= C; ++i) {
        const Record<DG, T> out = i < C ? x.rec(i, layer) : (C == 2 ? x.rec(0, layer + 1) : x.rec(-1));
        const TieSeg<DG> tie = i < C ? x.tie_seg(layer, i) : (C == 2 ? x.tie_seg(layer + 1, 0) : x.tie_seg(-1, 0));
        launch_block<DG, T>(x, 0, x.rec(i - 1, layer), w + (size_t)(i - 1) * DG * DG, p.grp(i - 1), p.ld, out, false, nullptr, 0,
                            false, out.mask ? tie : TieSeg<DG>{nullptr, nullptr, nullptr, 0, 0.f});
    }
}

// eq. (7)
template <int DG, typename T>
static void layer_inverse_impl(const Ctx<DG, T>& x, const float* w, const Planes<T>& p) {
    if constexpr (DG == 64) {
        if (x.S > 1) { wide_inverse<T>(x, w, p); return; }
    }
    const int C = x.cfg->c;
    for (int i = 1; i < C; ++i) launch_sum<DG, T>(x, p.grp(i - 1), p.ld, p.gs, 1, nullptr, x.rec(i));
    for (int i = C; i >= 1; --i) {
        if (i == 1 && C > 2) launch_sum<DG, T>(x, p.grp(1), p.ld, p.gs, C - 1, nullptr, x.rec(0));
        const Record<DG, T> out = (i == 2 && C == 2) ? x.rec(0) : x.rec(-1);
        launch_block<DG, T>(x, 1, x.rec(i - 1), w + (size_t)(i - 1) * DG * DG, p.grp(i - 1), p.ld, out, false, nullptr, 0);
    }
}

// Backward fused with the inverse.  slots_ready: slots 1..C-1 already hold the records of
// Y_1..Y_{C-1} of this layer (left by the forward sweep, or by the layer above while it rebuilt
// its input).  On return slots 1..C-1 hold the records of X_1..X_{C-1}, i.e. of the layer below
// (not written for the lowest layer of a step, `layer` = 0 with `in_step`).  When indices are
// saved, every record written here takes its column set from the kept masks of the layer it
// belongs to instead of selecting again.
template <int DG, typename T>
static void layer_backward_impl(const Ctx<DG, T>& x, const float* w, const Planes<T>& y, const Planes<T>& dy, float* dw_out,
                                bool slots_ready, int layer = 0, bool in_step = false) {
    if constexpr (DG == 64) {
        if (x.S > 1) { wide_backward<T>(x, w, y, dy, dw_out, slots_ready, layer, in_step); return; }
    }
    const int C = x.cfg->c;
    const bool given = x.saved != nullptr;
    if (!slots_ready)
        for (int i = 1; i < C; ++i) launch_sum<DG, T>(x, y.grp(i - 1), y.ld, y.gs, 1, nullptr, x.rec(i, layer), given);
    for (int i = C; i >= 1; --i) {
        const float* wi = w + (size_t)(i - 1) * DG * DG;
        const T* z;      // rows of Y_{i-1}
        int64_t ldz;
        if (i >= 2) { z = y.grp(i - 2); ldz = y.ld; }
        else if (C == 2) { z = y.grp(1); ldz = y.ld; }      // Y_0 = X_2, rebuilt just before
        else {
            launch_sum<DG, T>(x, y.grp(1), y.ld, y.gs, C - 1, x.y0(), x.rec(0, layer), given);
            launch_tie_fixup<DG, T>(x, x.tie_seg(layer, 0), x.y0(), DG, x.rec(0, layer));
            z = x.y0(); ldz = DG;
        }
        Record<DG, T> out = x.rec(-1);
        TieSeg<DG> out_tie = x.tie_seg(-1, 0);       // the segment that listed rows of `out` in the forward sweep
        if (i < C) {
            if (!(in_step && layer == 0)) {
                out = x.rec(i, given ? layer - 1 : 0);                                 // record of Y_i of the layer below
                if (in_step) out_tie = x.tie_seg(layer - 1, i);
            }
        } else if (C == 2) {
            out = x.rec(0, layer);                                                     // X_2 = Y_0 of this layer
            if (in_step) out_tie = x.tie_seg(layer, 0);
        }
        launch_hub_both<DG, T>(x, x.rec(i - 1, layer), dy.grp(i - 1), dy.ld);
        unsigned nparts;
        const bool own_reduce = x.tiles < 4 * 4 * x.g->grid;
        bool dw_reduced = false;
        if (split_dw<DG, T>(x.g)) {
            // X_i = Y_i - f_i(Y_{i-1}) with H kept for the weight gradient, then dW_i = H^T dY_i
            launch_block<DG, T>(x, 1, x.rec(i - 1, layer), wi, y.grp(i - 1), y.ld, out, given, nullptr, 0, true,
                                TieSeg<DG>{nullptr, nullptr, nullptr, 0, 0.f}, DG, x.hplane());
            nparts = launch_dw<DG, T>(x, dy.grp(i - 1), dy.ld, out_tie, y.grp(i - 1), y.ld, out.mask ? &out : nullptr);
        } else {
            nparts = launch_block<DG, T>(x, 2, x.rec(i - 1, layer), wi, y.grp(i - 1), y.ld, out, given, dy.grp(i - 1), dy.ld, true);
            // (on a small graph the launch that restores the listed rows' column sets also sums dW_i's partials)
            const DwReduceJob job{x.dw_partial(), (int)nparts, DG * DG, dw_out + (size_t)(i - 1) * DG * DG, DG, DG, 0};
            if (out.mask) dw_reduced = launch_tie_fixup<DG, T>(x, out_tie, y.grp(i - 1), y.ld, out, own_reduce ? &job : nullptr);
        }
        // dW_i is summed from the partials by the first job of the gradient kernel that follows, unless that kernel
        // has so few tiles per wave that it could not make up for the late start of those workgroups (measured on
        // a 49,600-node graph with 3,100 tiles: +80 us on a 405 us kernel): then by a launch of its own
        float* dwi = dw_out + (size_t)(i - 1) * DG * DG;
        if (dw_reduced) {
            dwi = nullptr;
        } else if (own_reduce) {
            ProfScope prof(KC_DW_REDUCE, x.s);
            hipLaunchKernelGGL(k_dw_reduce, dim3((DG * DG + DW_REDUCE_ENTRIES - 1) / DW_REDUCE_ENTRIES), dim3(256), 0, x.s, (const float*)x.dw_partial(),
                               (int)nparts, DG * DG, dwi, DG, DG);
            dwi = nullptr;
        }
        const typename MaskOf<DG>::type* own = x.rec(i - 1, layer).mask;
        if (i >= 2) launch_grad<DG, T>(x, dy.grp(i - 1), dy.ld, wi, own, z, ldz, dy.grp(i - 2), dy.ld, dy.gs, 1, (int)nparts, dwi, true);
        else launch_grad<DG, T>(x, dy.grp(0), dy.ld, wi, own, z, ldz, dy.grp(1), dy.ld, dy.gs, C - 1, (int)nparts, dwi, true);
    }
}

template <int DG, typename T>
static Ctx<DG, T> make_ctx(const gsr_graph_t* g, const gsr_config_t* cfg, void* ws, hipStream_t s) {
    Ctx<DG, T> x;
    x.g = g; x.cfg = cfg; x.s = s; x.ws = (char*)ws; x.lw = carve_layer(cfg, g);
    x.tiles = (int)((cfg->n + 15) / 16);
    x.S = sub_planes(cfg);
    x.saved = nullptr;
    x.tie_counts = nullptr; x.tie_rows = nullptr; x.tie_masks = nullptr; x.tie_cap = 0;
    return x;
}

enum LayerOp { OP_FWD, OP_INV, OP_BWD };

template <int DG, typename T>
static gsr_status_t layer_call(LayerOp op, const gsr_graph_t* g, const gsr_config_t* cfg, const float* w, void* y, void* dy,
                               float* dw, void* ws, hipStream_t s) {
    Ctx<DG, T> x = make_ctx<DG, T>(g, cfg, ws, s);
    Planes<T> py = caller_planes<T>(y, cfg);
    if (op == OP_FWD) layer_forward_impl<DG, T>(x, w, py, false);
    else if (op == OP_INV) layer_inverse_impl<DG, T>(x, w, py);
    else layer_backward_impl<DG, T>(x, w, py, caller_planes<T>(dy, cfg), dw, false);
    GSR_HIP_CHECK(hipGetLastError());
    return GSR_OK;
}

// rows are moved in pieces of up to 16 bytes
static bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

static gsr_status_t layer_dispatch(LayerOp op, const gsr_graph_t* g, const gsr_config_t* cfg, const float* w, void* y, void* dy,
                                   float* dw, void* ws, size_t ws_bytes, void* stream) {
    GSR_TRY(validate_config(cfg, g, false));
    if (cfg->n == 0) return GSR_OK;
    if (!w || !y || !ws || (op == OP_BWD && (!dy || !dw))) return fail(GSR_ERR_INVALID_ARG, "null pointer");
    if (op == OP_BWD && !g->has_transpose) return fail(GSR_ERR_UNSUPPORTED, "graph has no transpose");
    const size_t need = carve_layer(cfg, g).total;
    if (ws_bytes < need) return fail(GSR_ERR_WORKSPACE_TOO_SMALL, "workspace %zu < %zu bytes", ws_bytes, need);
    if (!aligned16(y) || !aligned16(dy) || ((uintptr_t)ws & 255))
        return fail(GSR_ERR_INVALID_ARG, "planes must be 16-byte aligned and the workspace 256-byte aligned");
    hipStream_t s = (hipStream_t)stream;
    const int dg = cfg->d / cfg->c;
    if (cfg->dtype == GSR_F32) {
        if (dg == 32) return layer_call<32, float>(op, g, cfg, w, y, dy, dw, ws, s);
        return layer_call<64, float>(op, g, cfg, w, y, dy, dw, ws, s);
    }
    if (dg == 32) return layer_call<32, bf16_t>(op, g, cfg, w, y, dy, dw, ws, s);
    return layer_call<64, bf16_t>(op, g, cfg, w, y, dy, dw, ws, s);
}

template <int DG, typename T>
static gsr_status_t step_impl(const gsr_graph_t* g, const gsr_config_t* cfg, const void* x0, const float* w_all,
                              const float* w_out, const float* b_out, const float* target, float* loss_out, float* yhat_out,
                              float* dw_all, float* dw_out, float* db_out, void* dx0_out, void* x0_rebuilt_out, void* xl_out,
                              void* ws, hipStream_t s) {
    const StepWs sw = carve_step(cfg, g);
    char* base = (char*)ws;
    Ctx<DG, T> x = make_ctx<DG, T>(g, cfg, base + sw.layer, s);
    if (cfg->save_indices == 1) x.saved = (typename MaskOf<DG>::type*)(base + sw.masks);
    const int C = cfg->c, L = cfg->l;
    if (cfg->save_indices == 2) {
        x.tie_counts = (int*)(base + sw.tie_counts);
        x.tie_rows = (uint32_t*)(base + sw.tie_rows);
        x.tie_masks = (typename MaskOf<DG>::type*)(base + sw.tie_masks);
        x.tie_cap = (int)sw.tie_cap;
        const int ints = (L + 1) * C * TIE_SUB * TIE_COUNTER_STRIDE;
        hipLaunchKernelGGL(k_zero_ints, dim3((ints + 255) / 256), dim3(256), 0, s, x.tie_counts, ints);
    }
    const int64_t n = cfg->n;
    const int dgw = DG * x.S;            // columns of a group (DG, or 64 S for the groups handled as sub-planes)
    const Planes<T> act{(T*)(base + sw.act), (int64_t)dgw, n * dgw};
    const Planes<T> grad{(T*)(base + sw.grad), (int64_t)dgw, n * dgw};
    const Planes<T> in = caller_planes<T>(const_cast<void*>(x0), cfg);
    const dim3 cgrid((unsigned)g->grid * 4), cblock(256);
    auto copy = [&](const Planes<T>& from, const Planes<T>& to) {
        ProfScope prof(KC_COPY, s);
        hipLaunchKernelGGL((k_copy_planes<T>), cgrid, cblock, 0, s, n, dgw, C, (const T*)from.base, from.ld, from.gs, to.base,
                           to.ld, to.gs);
    };
    copy(in, act);
    const size_t wl = (size_t)C * dgw * dgw;
    for (int l = 0; l < L; ++l) layer_forward_impl<DG, T>(x, w_all + l * wl, act, C == 2 && l > 0, l);
    if (xl_out) copy(act, caller_planes<T>(xl_out, cfg));
    HeadArgs<T> h;
    h.n = (int)n; h.d = cfg->d; h.dg = dgw; h.act = act.base; h.grad = grad.base; h.ld = act.ld; h.gs = act.gs;
    h.w_out = w_out; h.b_out = b_out; h.target = target; h.yhat = yhat_out; h.partial = (float*)(base + sw.head);
    {
        ProfScope prof(KC_HEAD, s);
        hipLaunchKernelGGL((k_head<T>), dim3((unsigned)g->grid), dim3(256), 0, s, h);
        hipLaunchKernelGGL(k_head_reduce, dim3((cfg->d + 2 + 3) / 4), dim3(256), 0, s, (const float*)h.partial, g->grid,
                           cfg->d, (int)n, dw_out, db_out, loss_out);
    }
    for (int l = L - 1; l >= 0; --l) layer_backward_impl<DG, T>(x, w_all + l * wl, act, grad, dw_all + l * wl, true, l, true);
    if (dx0_out) copy(grad, caller_planes<T>(dx0_out, cfg));
    if (x0_rebuilt_out) copy(act, caller_planes<T>(x0_rebuilt_out, cfg));
    GSR_HIP_CHECK(hipGetLastError());
    return GSR_OK;
}

}  // namespace gsr

using namespace gsr;

extern "C" {

gsr_status_t gsr_layer_forward(const gsr_graph_t* g, const gsr_config_t* cfg, const float* w, void* x_inout, void* workspace,
                               size_t workspace_bytes, void* stream) {
    return layer_dispatch(OP_FWD, g, cfg, w, x_inout, nullptr, nullptr, workspace, workspace_bytes, stream);
}

gsr_status_t gsr_layer_inverse(const gsr_graph_t* g, const gsr_config_t* cfg, const float* w, void* y_inout, void* workspace,
                               size_t workspace_bytes, void* stream) {
    return layer_dispatch(OP_INV, g, cfg, w, y_inout, nullptr, nullptr, workspace, workspace_bytes, stream);
}

gsr_status_t gsr_layer_backward(const gsr_graph_t* g, const gsr_config_t* cfg, const float* w, void* y_inout, void* dy_inout,
                                float* dw_out, void* workspace, size_t workspace_bytes, void* stream) {
    return layer_dispatch(OP_BWD, g, cfg, w, y_inout, dy_inout, dw_out, workspace, workspace_bytes, stream);
}

gsr_status_t gsr_step(const gsr_graph_t* g, const gsr_config_t* cfg, const void* x0, const float* w_all, const float* w_out,
                      const float* b_out, const float* target, float* loss_out, float* yhat_out, float* dw_all, float* dw_out,
                      float* db_out, void* dx0_out, void* x0_rebuilt_out, void* xl_out, void* workspace, size_t workspace_bytes,
                      void* stream) {
    GSR_TRY(validate_config(cfg, g, true));
    if (cfg->d > HEAD_MAXQ * 64) return fail(GSR_ERR_UNSUPPORTED, "D=%d above %d", cfg->d, HEAD_MAXQ * 64);
    if (!x0 || !w_all || !w_out || !b_out || !target || !loss_out || !dw_all || !dw_out || !db_out || !workspace)
        return fail(GSR_ERR_INVALID_ARG, "null pointer");
    if (!g->has_transpose) return fail(GSR_ERR_UNSUPPORTED, "graph has no transpose");
    const size_t need = carve_step(cfg, g).total;
    if (workspace_bytes < need) return fail(GSR_ERR_WORKSPACE_TOO_SMALL, "workspace %zu < %zu bytes", workspace_bytes, need);
    if (cfg->n == 0) return fail(GSR_ERR_INVALID_ARG, "empty graph");
    if ((uintptr_t)workspace & 255) return fail(GSR_ERR_INVALID_ARG, "the workspace must be 256-byte aligned");
    hipStream_t s = (hipStream_t)stream;
    const int dg = cfg->d / cfg->c;
#define GSR_STEP(DGV, TV)                                                                                            \
    return step_impl<DGV, TV>(g, cfg, x0, w_all, w_out, b_out, target, loss_out, yhat_out, dw_all, dw_out, db_out, \
                              dx0_out, x0_rebuilt_out, xl_out, workspace, s)
    if (cfg->dtype == GSR_F32) {
        if (dg == 32) GSR_STEP(32, float);
        GSR_STEP(64, float);
    }
    if (dg == 32) GSR_STEP(32, bf16_t);
    GSR_STEP(64, bf16_t);
#undef GSR_STEP
}

gsr_status_t gsr_step_tie_stats(const gsr_graph_t* g, const gsr_config_t* cfg, const void* workspace, int64_t* listed,
                                int64_t* max_per_block, int64_t* dropped, void* stream) {
    GSR_TRY(validate_config(cfg, g, true));
    if (!workspace) return fail(GSR_ERR_INVALID_ARG, "null pointer");
    if (cfg->save_indices != 2) return fail(GSR_ERR_INVALID_ARG, "cfg->save_indices is not 2: nothing was listed");
    const StepWs sw = carve_step(cfg, g);
    const int segs = cfg->l * cfg->c;      // (the set listed for a layer above the last is never used)
    std::vector<int> counts((size_t)segs * TIE_SUB * TIE_COUNTER_STRIDE);
    GSR_HIP_CHECK(hipStreamSynchronize((hipStream_t)stream));
    GSR_HIP_CHECK(hipMemcpy(counts.data(), (const char*)workspace + sw.tie_counts, counts.size() * sizeof(int), hipMemcpyDeviceToHost));
    int64_t total = 0, most = 0, lost = 0;
    for (int seg = 0; seg < segs; ++seg) {
        int64_t in_block = 0;
        for (int sub = 0; sub < TIE_SUB; ++sub) {
            const int64_t c = counts[((size_t)seg * TIE_SUB + sub) * TIE_COUNTER_STRIDE];
            in_block += c;
            total += std::min<int64_t>(c, sw.tie_cap);
            lost += std::max<int64_t>(0, c - sw.tie_cap);
        }
        most = std::max(most, in_block);
    }
    if (listed) *listed = total;
    if (max_per_block) *max_per_block = most;
    if (dropped) *dropped = lost;
    return GSR_OK;
}

gsr_status_t gsr_step_tie_export(const gsr_graph_t* g, const gsr_config_t* cfg, const void* workspace, int32_t layer,
                                 int32_t block, int32_t* rows_out, uint64_t* masks_out, int64_t* count_out, void* stream) {
    GSR_TRY(validate_config(cfg, g, true));
    if (!workspace || !rows_out || !masks_out || !count_out) return fail(GSR_ERR_INVALID_ARG, "null pointer");
    if (cfg->save_indices != 2) return fail(GSR_ERR_INVALID_ARG, "cfg->save_indices is not 2: nothing was listed");
    if (layer < 0 || layer >= cfg->l || block < 1 || block > cfg->c) return fail(GSR_ERR_INVALID_ARG, "layer %d / block %d out of range", layer, block);
    const StepWs sw = carve_step(cfg, g);
    const size_t seg = (size_t)layer * cfg->c + (block - 1);
    const char* base = (const char*)workspace;
    GSR_HIP_CHECK(hipStreamSynchronize((hipStream_t)stream));
    std::vector<int> counts((size_t)TIE_SUB * TIE_COUNTER_STRIDE);
    GSR_HIP_CHECK(hipMemcpy(counts.data(), base + sw.tie_counts + seg * counts.size() * sizeof(int), counts.size() * sizeof(int), hipMemcpyDeviceToHost));
    const int dg = std::min(cfg->d / cfg->c, 64);
    const size_t mbytes = dg == 64 ? 8 : 4;
    int64_t written = 0;
    for (int sub = 0; sub < TIE_SUB; ++sub) {
        const int64_t take = std::min<int64_t>(counts[(size_t)sub * TIE_COUNTER_STRIDE], sw.tie_cap);
        if (take == 0) continue;
        const size_t at = (seg * TIE_SUB + sub) * (size_t)sw.tie_cap;
        GSR_HIP_CHECK(hipMemcpy(rows_out + written, base + sw.tie_rows + at * sizeof(uint32_t), (size_t)take * sizeof(uint32_t), hipMemcpyDeviceToHost));
        if (mbytes == 8) {
            GSR_HIP_CHECK(hipMemcpy(masks_out + written, base + sw.tie_masks + at * 8, (size_t)take * 8, hipMemcpyDeviceToHost));
        } else {
            std::vector<uint32_t> m32((size_t)take);
            GSR_HIP_CHECK(hipMemcpy(m32.data(), base + sw.tie_masks + at * 4, (size_t)take * 4, hipMemcpyDeviceToHost));
            for (int64_t i = 0; i < take; ++i) masks_out[written + i] = m32[(size_t)i];
        }
        written += take;
    }
    *count_out = written;
    return GSR_OK;
}

}  // extern "C"
