// Pieces shared by the aggregation kernels: launch parameters, vector load/store, epilogue.
#ifndef GNN_AGG_COMMON_H
#define GNN_AGG_COMMON_H

#include <hip/hip_runtime.h>

#include "gnn_device.h"
#include "gnn_internal.h"

namespace gnn {

struct AggParams {
    WsHeader *hdr;
    const NgEntry *ng;
    const int *ngptr;
    const int *colidx;
    const float *ew;
    const float *X;
    float *out;
    const float *bias;  // epilogue: out = act(sum + bias); may be null
    float self_scale;   // 1 + eps (GIN)
    int relu;
    int n;
    int dim;
    int ngs;
    int dwl_log2;
    int T;           // neighbor groups per block
    int iter_total;  // chunks of dwl*VEC floats per row
    int xcd_remap;
    int do_empty;    // 1: the main kernel writes the rows without entries; 0: the init kernel does
    int64_t nnz;
};

template <int VEC>
__device__ __forceinline__ void load_vec(float (&r)[VEC], const float *p)
{
    if constexpr (VEC == 4) {
        const float4 v = *reinterpret_cast<const float4 *>(p);
        r[0] = v.x; r[1] = v.y; r[2] = v.z; r[3] = v.w;
    } else if constexpr (VEC == 2) {
        const float2 v = *reinterpret_cast<const float2 *>(p);
        r[0] = v.x; r[1] = v.y;
    } else {
        r[0] = *p;
    }
}

template <int VEC>
__device__ __forceinline__ void store_vec(float *p, const float (&r)[VEC])
{
    if constexpr (VEC == 4) {
        *reinterpret_cast<float4 *>(p) = make_float4(r[0], r[1], r[2], r[3]);
    } else if constexpr (VEC == 2) {
        *reinterpret_cast<float2 *>(p) = make_float2(r[0], r[1]);
    } else {
        *p = r[0];
    }
}

__device__ __forceinline__ bool header_ok(const WsHeader *hdr, const AggParams &p)
{
    return hdr->magic == kMagic && hdr->status == GNN_OK && hdr->ngs == p.ngs && hdr->n == p.n && hdr->nnz == p.nnz;
}

__device__ __forceinline__ float epilogue(float v, const float *bias, int d, int relu)
{
    if (bias) v += bias[d];
    if (relu) v = fmaxf(v, 0.0f);
    return v;
}

}  // namespace gnn
#endif
