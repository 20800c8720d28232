// Internal declarations shared by the translation units of libgsr (host side).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "gsr.h"

namespace gsr {

// ---- error plumbing -------------------------------------------------------------------
void set_error(const char* fmt, ...);
gsr_status_t fail(gsr_status_t st, const char* fmt, ...);

#define GSR_HIP_CHECK(expr)                                                                  \
    do {                                                                                     \
        hipError_t _e = (expr);                                                              \
        if (_e != hipSuccess)                                                                \
            return gsr::fail(GSR_ERR_HIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(_e), \
                             __FILE__, __LINE__);                                            \
    } while (0)

#define GSR_TRY(expr)                          \
    do {                                       \
        gsr_status_t _s = (expr);              \
        if (_s != GSR_OK) return _s;           \
    } while (0)

// ---- tunables (gsr_set_option) ----------------------------------------------------------
struct Options {
    int64_t hub_threshold = 0;    // rows longer than this are reduced in two passes (0: chosen per graph)
    int64_t hub_chunk = 0;        // neighbours per first-pass partial (0: chosen per graph)
    int64_t max_workgroups = 0;   // 0: derive from the device (multiple of 8)
    int64_t profile = 0;          // bit i set: time kernel class i with HIP events
    int64_t hub_values = 0;       // first pass over float32 records value by value: 0 on long-row graphs, 1 always, 2 never
};
Options& options();

// ---- per-kernel timing (gsr_set_option("profile", mask)) -----------------------------------
enum KernelClass {
    KC_BLOCK_FWD = 0,  // k_block, forward
    KC_BLOCK_INV,      // k_block, inverse only
    KC_BLOCK_BWD,      // k_block, inverse + weight gradient
    KC_GRAD,           // k_grad
    KC_SUM,            // k_sum (group sum / record of a plane)
    KC_HUB,            // first pass over hub rows
    KC_DW_REDUCE,
    KC_HEAD,
    KC_COPY,
    KC_TIE,            // records of listed rows written again with their kept column sets
    KC_DW,             // k_dw: dW_i = H^T dY_i
    KC_COUNT
};
// Records a HIP event on `s` before and after the launches made while it is alive, if the
// class is enabled.  Durations are collected by gsr_profile_read.
struct ProfScope {
    ProfScope(KernelClass kc, hipStream_t s);
    ~ProfScope();
    int slot;
    hipStream_t stream;
};

// ---- CSR on the device --------------------------------------------------------------------
// Rows longer than `hub_threshold` ("hub" rows: clock/reset-like nets) are cut into chunks of
// `hub_chunk` neighbours.  A first kernel reduces every chunk to one partial row, the main
// kernel then adds a hub row's partials in chunk order, so the summation order is fixed.
struct HubPlan {
    int32_t n_hub = 0;        // hub rows
    int32_t n_chunks = 0;     // chunks over all hub rows
    int32_t* rows = nullptr;  // device [n_hub]    ascending row ids
    int32_t* cptr = nullptr;  // device [n_hub+1]  first chunk of each hub row
    int32_t* tile0 = nullptr; // device [tiles+1]  hub rows before row 16 t (the place in `rows` of tile t's first hub row)
    int32_t* crow = nullptr;  // device [n_chunks] row of the chunk
    int32_t* ce0 = nullptr;   // device [n_chunks] first edge
    int32_t* ce1 = nullptr;   // device [n_chunks] one past the last edge
};

// 16-row tiles with more than this many stored entries in rows that are not split are listed per matrix; the
// layer kernels deal them out to their waves, one each, before their sweep, so that the long tiles start first
// and no wave meets several of them.  Measured on the 1M-node workload (median tile 63 entries, 1 % of the tiles
// around 1,300): inverse + dW kernel 546 us without, 495 - 498 us with 512 / 768 / 1,024, 531 us with 1,100.
constexpr int kHeavyTileEdges = 512;

struct Csr {
    int32_t* rp = nullptr;  // device [n+1]
    int32_t* ci = nullptr;  // device [nnz]
    float* av = nullptr;    // device [nnz]
    HubPlan hub;
    int32_t* heavy = nullptr;  // device [n_heavy]: the heavy tiles, ascending
    int32_t n_heavy = 0;
};

}  // namespace gsr

struct gsr_graph {
    int64_t n = 0, nnz = 0, max_degree = 0;
    gsr::Csr a;              // A
    gsr::Csr at;             // A^T (aliases `a` when symmetric)
    bool symmetric = false;
    bool has_transpose = false;
    bool split_backward = true;   // float32: the backward of a block as inverse kernel + k_dw (large graphs), else fused
    bool long_rows = false;  // the mean row has 64 stored entries or more: nearly every row goes through the first pass
    int hub_values = 0;      // the first pass over float32 records runs value by value (k_hub_values): 0 never, 1 while
                             // 2 k <= D/C (beyond that the dealing of the tile kernels is faster: 650 against 490 ms per step
                             // at k = D/C = 64 on the Table-1-shaped graph, 464 against 473 at k = 32), 2 always
    int32_t hub_threshold = 512;
    int device = 0;
    int num_cus = 256;
    int grid = 512;          // workgroups of the persistent row-tile kernels (multiple of 8)
    int* draws = nullptr;     // device: tile counters of the dynamic sweeps + their sign-off counter (see tile_draws)
    float* dinv = nullptr;    // device [n]: d^-1/2 while the values are being normalised
    float* scratch = nullptr; // device [max(chunks of A, chunks of A^T, 1)][64]: first-pass sums of split rows for gsr_spmm
};

namespace gsr {

// gsr_graph.hip
gsr_status_t validate_config(const gsr_config_t* cfg, const gsr_graph_t* g, bool need_l);

// Workspace carving shared by gsr_workspace_size and the layer / step calls.
constexpr int kMaxRecordSlots = 32;   // groups (at most 8) x sub-planes of a group (at most 4)
struct LayerWs {
    size_t rec_vals[kMaxRecordSlots];  // per slot and sub-plane: compressed values  [n][k] of T
    size_t rec_mask[kMaxRecordSlots];  // per slot and sub-plane: column bit mask    [n] of uint32 (32 columns) / uint64 (64)
    size_t y0;           // Y_0 plane [n][dg] of T (C > 2); wide groups: [S][n][64]
    size_t h;            // [n][min(dg, 64)] float: H of the block being inverted, for the weight-gradient kernel
    size_t dh;           // wide groups only: [S][n][64] float, the block gradient summed over column blocks
    size_t dw_partial;   // [grid][dg*dg] float; wide groups: [S*S][grid][64*64]
    size_t hub_partial;  // [max(n_chunks A, n_chunks A^T)][dg] float
    size_t hub_partial2; // same size: the backward's two first passes of a block run as one launch
    size_t hub_cols;     // [n][k] bytes: column of every record value, for the value-by-value first pass (float32)
    size_t hub_vals;     // wide groups, same pass: [n][k] float, the kept values of a whole row side by side
    size_t total;
};
struct StepWs {
    size_t act;   // [C][n][dg] of T
    size_t grad;  // [C][n][dg] of T
    size_t head;  // [grid][D + 2] float
    size_t layer; // LayerWs starts here
    size_t masks; // [L+1][C][n] column masks kept from the forward sweep (cfg->save_indices == 1), else unused
    // cfg->save_indices == 2: per segment (layer in 0..L, slot in 0..C-1) kTieSub sub-lists of up to tie_cap kept rows
    size_t tie_counts;  // [(L+1)*C][kTieSub] counters, kTieCounterStride ints apart
    size_t tie_rows;    // [(L+1)*C][kTieSub][tie_cap] uint32
    size_t tie_masks;   // [(L+1)*C][kTieSub][tie_cap] column masks
    int64_t tie_cap;    // places per sub-list
    size_t total;
};
LayerWs carve_layer(const gsr_config_t* cfg, const gsr_graph_t* g);
int64_t tie_capacity(const gsr_config_t* cfg);
constexpr int kTieSub = 16, kTieCounterStride = 32;     // (device code: TIE_SUB, TIE_COUNTER_STRIDE)

// Tile counters of the dynamic sweeps (device code: tile_draws): 8 XCDs x 64 queues, 128 bytes apart.
constexpr int kTileCounters = 8 * 64 * 32;
constexpr int kTileCounterSet = kTileCounters + 9 * 32;    // a counter set with its sign-off counters
constexpr int kTileCounterSets = 4;                        // a graph holds this many (launches whose blockIdx.y is a column block of a wide group use one each)
void tile_counters(const gsr_graph_t* g, int** set, int** done);
StepWs carve_step(const gsr_config_t* cfg, const gsr_graph_t* g);

// Whether a launch of `grid` workgroups of four waves deals the heavy tiles out first (TileDeal).  Measured: on the
// 1M-node workload (15 - 30 tiles per wave, 1.6 % of them heavy) it shortens every layer kernel by 10 - 16 %, and
// on a 49,600-node graph whose tiles are all heavy the forward kernel by 17 %.  On the 100k-node workload (1.5
// tiles per wave) the gradient kernel gets 19 % longer, and on the 8M-node workload (120 - 240 tiles per wave) all
// kernels get 6 - 10 % longer: there a late heavy tile is a small part of the kernel, while taking the heavy tiles
// out of the order of the sweep takes their neighbours out of the cached window.  So: only with a moderate number
// of tiles per wave, or when most tiles are heavy anyway.
inline bool heavy_first(int n_heavy, int tiles, unsigned grid) {
    const int64_t waves = (int64_t)4 * grid;
    return n_heavy > 0 && ((tiles >= 4 * waves && tiles < 64 * waves) || 2 * (int64_t)n_heavy >= tiles);
}

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }
// Workgroups of four waves for a first pass over n_chunks chunks: a wave per chunk up to 4,096 workgroups, a whole
// number of eights (the kernels give every XCD one contiguous eighth of the chunk list).
inline unsigned hub_grid(int n_chunks) {
    const int wgs = (n_chunks + 3) / 4 < 4096 ? (n_chunks + 3) / 4 : 4096;
    return (unsigned)((wgs + 7) / 8 * 8);
}
// A group wider than one 64-column tile is handled as D/C / 64 sub-planes of 64 columns.
inline int sub_planes(const gsr_config_t* cfg) { const int dg = cfg->d / cfg->c; return dg > 64 ? dg / 64 : 1; }
inline size_t dtype_size(int32_t dtype) { return dtype == GSR_BF16 ? 2 : 4; }

}  // namespace gsr
