// Vanilla distributed AMSGrad without compression (Section 3): gbar = (1/n) sum_i g_i in ascending
// worker order, then the AMSGrad update.  One workgroup per tile of 4096 coordinates (chunk: tile_of_block's;
// workgroups past the last tile leave at once).
// Traffic: 4 B per (worker, coordinate) + 32 B per coordinate.
#pragma once
#include "device_utils.h"

namespace cams {

constexpr int kPlainBatch = 4;   // workers whose gradients are in flight together

template <typename G, bool kStreamState>   // G: float, uint16_t (bfloat16 bits) or f16bits
__global__ __launch_bounds__(kThreads) void plain_update(const G *__restrict__ g, int64_t d, int n,
                                                         float *__restrict__ theta, float *__restrict__ m,
                                                         float *__restrict__ v, float *__restrict__ vhat, AmsParams p, int chunk,
                                                         int n_tiles)
{
    const int tid = threadIdx.x;
    const int t = tile_of_block(blockIdx.x, chunk);
    if (t >= n_tiles) return;
    const int64_t base = (int64_t)t * kTile;
    float acc[4][4];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[r][c] = 0.f;
    for (int i0 = 0; i0 < n; i0 += kPlainBatch) {
        float4 gv[kPlainBatch][4];
#pragma unroll
        for (int u = 0; u < kPlainBatch; ++u)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                gv[u][r] = i0 + u < n ? load_grad4(g + (int64_t)(i0 + u) * d, base + 4 * (tid + kThreads * r), d)
                                      : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int u = 0; u < kPlainBatch; ++u)
            if (i0 + u < n) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    acc[r][0] = fadd(acc[r][0], gv[u][r].x);
                    acc[r][1] = fadd(acc[r][1], gv[u][r].y);
                    acc[r][2] = fadd(acc[r][2], gv[u][r].z);
                    acc[r][3] = fadd(acc[r][3], gv[u][r].w);
                }
            }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int64_t j = base + 4 * (tid + kThreads * r);
        float4 th = ld4_state<kStreamState>(theta + j), mm = ld4_state<kStreamState>(m + j), vv = ld4_state<kStreamState>(v + j), vh = ld4_state<kStreamState>(vhat + j);
        // padding coordinates take no gradient (load_grad4 gives 0 past d)
        const float4 gbar = make_float4(fdiv(acc[r][0], p.n_workers), fdiv(acc[r][1], p.n_workers),
                                        fdiv(acc[r][2], p.n_workers), fdiv(acc[r][3], p.n_workers));
        amsgrad_update4(th, mm, vv, vh, gbar, p);
        st4_state<kStreamState>(theta + j, th);
        st4_state<kStreamState>(m + j, mm);
        st4_state<kStreamState>(v + j, vv);
        st4_state<kStreamState>(vhat + j, vh);
    }
}

}  // namespace cams
