// Internal declarations shared by the translation units of the library (not installed).
#ifndef GNN_INTERNAL_H
#define GNN_INTERNAL_H

#include <stddef.h>
#include <stdint.h>

#include "gnn.h"

namespace gnn {

constexpr uint32_t kMagic = 0x474e4e41u;  // "GNNA"
constexpr int kWaveSize = 64;
constexpr int kNumXcd = 8;
#ifndef GNN_XCD_RUN
#define GNN_XCD_RUN 32
#endif
constexpr int kXcdRun = GNN_XCD_RUN;  // consecutive tiles that the aggregation kernels keep on one XCD
constexpr int kMaxWavesPerBlock = 16;
constexpr size_t kAlign = 256;
constexpr size_t kMaxLdsBytes = 64 * 1024;  // per block, keeps several blocks per CU inside the 160 KB LDS

// First 256 bytes of the workspace (device memory).  Written by the partition kernels.
struct WsHeader {
    uint32_t magic;
    int32_t n;
    int64_t nnz;
    int32_t ngs;
    int32_t status;  // GNN_OK or the error a kernel recorded
    int64_t num_ng;  // number of neighbor groups
    int64_t ng_capacity;
    uint64_t rowptr_addr;
};

// One neighbor group (Sec. 4.1): target node, CSR range [start, end), flags.
// flags bit 0: first group of its node, bit 1: last group of its node.
struct alignas(16) NgEntry {
    int32_t node;
    int32_t start;
    int32_t end;
    int32_t flags;
};

struct WsLayout {
    size_t header;   // offset of WsHeader
    size_t ngptr;    // int32[n+1]: id of the first neighbor group of node v; [n] = num_ng
    size_t cnt;      // int32[n]: arrival counters of the ordered flush; zero between calls
    size_t scan;     // int32[scan_blocks + 1]
    size_t ng;       // NgEntry[ng_capacity]
    size_t tmp;      // float[n * max_dim]
    size_t total;
    int64_t ng_capacity;
    int64_t scan_blocks;
};

constexpr int kScanTile = 2048;  // nodes per block in the partition scan

inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// Upper bound on the number of neighbor groups: every group holds >= 1 entry, and a row of
// d entries makes ceil(d/ngs) <= d/ngs + 1 groups.
inline int64_t ng_upper_bound(int32_t n, int64_t nnz, int32_t ngs)
{
    int64_t a = nnz;
    int64_t b = nnz / (ngs > 0 ? ngs : 1) + (int64_t)n;
    return a < b ? a : b;
}

inline WsLayout ws_layout(int32_t n, int64_t nnz, int32_t max_dim, int32_t ngs_for_capacity)
{
    WsLayout L;
    L.ng_capacity = ng_upper_bound(n, nnz, ngs_for_capacity > 0 ? ngs_for_capacity : 1);
    L.scan_blocks = ((int64_t)n + kScanTile - 1) / kScanTile;
    size_t off = 0;
    L.header = off;
    off += align_up(sizeof(WsHeader));
    L.ngptr = off;
    off += align_up(sizeof(int32_t) * ((size_t)n + 1));
    L.cnt = off;
    off += align_up(sizeof(int32_t) * ((size_t)n + 1));
    L.scan = off;
    off += align_up(sizeof(int32_t) * ((size_t)L.scan_blocks + 1));
    L.ng = off;
    off += align_up(sizeof(NgEntry) * (size_t)(L.ng_capacity > 0 ? L.ng_capacity : 1));
    L.tmp = off;
    off += align_up(sizeof(float) * (size_t)n * (size_t)(max_dim > 0 ? max_dim : 0));
    L.total = off;
    return L;
}

// Ordered flush (the default when the workspace has room, required by GNN_FLAG_DETERMINISTIC): every
// block may leave up to two partial rows (the node of its first and of its last neighbor group) in
// scratch memory behind the caller's own use of the workspace.  The workspace-size functions allow
// for blocks of at least kPartMinTile groups.
constexpr int kPartMinTile = 16;
// groups that one wave of the wave-tile form of the fused GIN layer serves (its unit of the ordered flush)
// (8 measured slower: half-empty MFMA tiles double the time on the matrix units, which does not hide)
constexpr int kFusedWaveTile = 16;
static_assert(kFusedWaveTile >= kPartMinTile, "the workspace allows partial rows for tiles of kPartMinTile groups");

inline size_t part_rows_bytes(int64_t ng_capacity, int tile, int32_t dim)
{
    if (dim <= 0) return 0;
    const int64_t tiles = (ng_capacity + tile - 1) / tile;
    return align_up(sizeof(float) * 2 * (size_t)(tiles > 0 ? tiles : 1) * (size_t)dim);
}

// LDS bytes of one block of the one-block-per-tile aggregation kernel: the staged column indices (and
// weights) of the block's T groups of up to ngs entries plus kStagePad entries that a batch of reads may
// run over, one slot of dim floats per wave (the part of a node's sum that a wave hands to the node's
// leader, Sec. 5.2), two flags per wave, and a 64-entry list of rows without entries per wave.
// T = waves_per_block * 64 / dw.
constexpr int kStagePad = 8;

inline size_t agg_lds_bytes(int T, int32_t ngs, int32_t dim, int wpb, bool weighted)
{
    size_t b = ((size_t)T * ngs + kStagePad) * (weighted ? 2 : 1) * 4;
    b = (b + 15) & ~(size_t)15;
    b += (size_t)wpb * dim * 4;
    b += (size_t)2 * kMaxWavesPerBlock * 4;
    b += (size_t)wpb * 64 * 4;
    return b;
}

// Request to fuse the Update GEMM into a GIN aggregation (gnn_layer_forward); done tells the caller
// whether the fused kernel was used.
struct FuseSpec {
    const float *W;
    const float *b;
    float *out;
    int M;
    int relu;
    bool done;
};

// Host-side record of the last failing HIP status of this thread.
void set_last_hip_error(int e);

// Widest per-lane vector (floats) that the row length and the two pointers' alignment allow.
inline int pick_vec(int32_t dim, const void *a, const void *b)
{
    const uintptr_t al = (uintptr_t)a | (uintptr_t)b;
    if (dim % 4 == 0 && al % 16 == 0) return 4;
    if (dim % 2 == 0 && al % 8 == 0) return 2;
    return 1;
}

// Model defaults shared by gnn_decide and the entry points (0 = auto).
void decide_defaults(int32_t n, int64_t nnz, int32_t max_degree, int32_t dim, int vec, int32_t *ngs,
                     int32_t *dw, int32_t *wpb);

}  // namespace gnn

#define GNN_HIP_TRY(expr)                                   \
    do {                                                    \
        hipError_t e__ = (expr);                            \
        if (e__ != hipSuccess) {                            \
            ::gnn::set_last_hip_error((int)e__);            \
            return GNN_EHIP;                                \
        }                                                   \
    } while (0)

#endif
