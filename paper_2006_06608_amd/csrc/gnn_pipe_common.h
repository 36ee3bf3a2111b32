// Tile view shared by the persistent kernels: what one wave derives about the tile it works on
// from the tile's tuples (one per lane), without talking to the other waves.
#ifndef GNN_PIPE_COMMON_H
#define GNN_PIPE_COMMON_H

#include "gnn_agg_common.h"

namespace gnn {

constexpr int kPipeIdxLoads = 8;  // index (and weight) prefetch registers per lane

// What one wave knows about the tile it works on.
struct TileView {
    NgEntry e;        // tuple of this lane's team
    int slot;         // Algorithm 1 slot of the team's target node inside the block
    int ws0, ws1;     // CSR range covered by this wave's teams
    bool valid;       // the team has a neighbor group
    bool leader;      // Algorithm 1 leader flag of the team
    int nslots;       // distinct target nodes of the tile (slots in use)
};

// tl: lane i holds the tuple of neighbor group i of the tile (node = -1 beyond the end).
__device__ __forceinline__ TileView derive_tile(const NgEntry &tl, int dwl_log2, int T)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int G = 64 >> dwl_log2;
    const int team = wave * G + (lane >> dwl_log2);
    const bool v_i = tl.node >= 0;
    const int prev = __shfl_up(tl.node, 1);
    const bool leader_i = v_i && (lane == 0 || tl.node != prev);
    const unsigned long long lmask = __ballot(leader_i);
    const unsigned long long vmask = __ballot(v_i);
    const int nvalid = __popcll(vmask);  // valid groups are a prefix of the tile
    TileView V;
    V.e.node = __shfl(tl.node, team);
    V.e.start = __shfl(tl.start, team);
    V.e.end = __shfl(tl.end, team);
    V.e.flags = __shfl(tl.flags, team);
    V.valid = team < nvalid && team < T;
    V.leader = ((lmask >> team) & 1ull) != 0;
    V.slot = __popcll(lmask & ((2ull << team) - 1ull)) - 1;
    const int f = wave * G;
    int nv = nvalid - f;
    nv = nv < 0 ? 0 : (nv > G ? G : nv);
    const int s0 = __shfl(tl.start, f < 64 ? f : 63);
    const int s1 = __shfl(tl.end, nv > 0 ? f + nv - 1 : 0);
    V.ws0 = nv > 0 ? s0 : 0;
    V.ws1 = nv > 0 ? s1 : 0;
    V.nslots = __popcll(lmask);
    return V;
}

}  // namespace gnn
#endif
