// Device helpers shared by the aggregation kernels and the layout export kernel.
#ifndef GNN_DEVICE_H
#define GNN_DEVICE_H

#include <hip/hip_runtime.h>

#include "gnn_internal.h"

namespace gnn {

// A wavefront of 64 lanes is cut into teams of dwl = 2^dwl_log2 lanes (the dimension workers of
// Sec. 4.2).  A team is the paper's "warp": it serves one neighbor group.  A block of W waves
// therefore serves T = W * 64/dwl consecutive neighbor groups (Algorithm 1's warpPerBlock).
struct BlockLayout {
    int64_t g;                       // id of this team's neighbor group
    NgEntry e;                       // its tuple (node, start, end, flags)
    unsigned long long leader_mask;  // ballot over the wave: bit set at the first lane of every leader team
    int team;                        // team index inside the block
    bool valid;                      // g < number of groups
    bool leader;                     // Algorithm 1: first team of its (block, node) pair
};

// Step 1 of Algorithm 1 for the calling lane's team; every thread of the block must call it.
// s_wave_cnt: int[blockDim.x / 64] in LDS, receives the number of leaders of each wave.
__device__ __forceinline__ BlockLayout block_layout(const NgEntry *__restrict__ ng, int64_t g0, int64_t num_ng,
                                                    int dwl_log2, int *s_wave_cnt)
{
    BlockLayout L;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int team_in_wave = lane >> dwl_log2;
    const int tlane = lane & ((1 << dwl_log2) - 1);
    L.team = wave * (64 >> dwl_log2) + team_in_wave;
    L.g = g0 + L.team;
    L.valid = L.g < num_ng;
    NgEntry e;
    e.node = -1;
    e.start = e.end = e.flags = 0;
    int prev = -1;
    if (L.valid) {
        e = ng[L.g];
        if (L.team > 0) prev = ng[L.g - 1].node;
    }
    L.e = e;
    // the team at the front of a block is always a leader; inside the block a team leads when its
    // target node differs from its predecessor's
    L.leader = L.valid && (L.team == 0 || e.node != prev);
    L.leader_mask = __ballot(L.leader && tlane == 0);
    if (lane == 0) s_wave_cnt[wave] = __popcll(L.leader_mask);
    return L;
}

// Step 2, after a __syncthreads(): slot index of the team's target node = number of leaders up
// to and including this team, minus one (the local counter of Algorithm 1).
__device__ __forceinline__ int block_layout_slot(const BlockLayout &L, int dwl_log2, const int *s_wave_cnt)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int base = 0;
    for (int w = 0; w < wave; ++w) base += s_wave_cnt[w];
    const int head_lane = (lane >> dwl_log2) << dwl_log2;
    const unsigned long long upto = (2ull << head_lane) - 1ull;  // bits 0..head_lane (all ones when head_lane = 63)
    return base + __popcll(L.leader_mask & upto) - 1;
}

}  // namespace gnn
#endif
