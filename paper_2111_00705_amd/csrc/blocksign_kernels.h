// Scaled-sign compression per contiguous block (Appendix A, "Scaled sign"), with error feedback
// (Section 4), the server average and the AMSGrad update (Section 3) fused behind it.
//
// General path (any block table), three launches:
//   bs_partial   per (segment, worker): fp64 sum of |g+e| over one piece (<= 4096) of a block
//   bs_scale     per (block, worker):   fixed-order fp64 sum of the pieces, s = fl32(S / len)
//   bs_apply     per 1024 coordinates:  loop over workers in ascending order,
//                x = g+e, c = copysign(s,x), e = x-c, acc += c; then gbar = acc/n and AMSGrad
// Fused path (uniform blocks that fit one workgroup's registers), one launch:
//   bs_fused     per block: for each worker, hold x of the whole block in registers, reduce
//                sum|x| in the workgroup, then finish as above - g and e are read once and e is
//                written once, which is the algorithmic minimum of 12 bytes per (worker, coordinate).
#pragma once
#include "device_utils.h"

namespace cams {

// Block table on the device.  Segments cut every block into pieces of at most kTile
// coordinates, counted from the block's own start.
struct BsTable {
    const int32_t *offsets;      // [n_blocks+1] block boundaries
    const int32_t *seg_lo;       // [n_segs] first coordinate of a segment
    const int32_t *seg_hi;       // [n_segs] one past its last coordinate
    const int32_t *block_seg0;   // [n_blocks+1] first segment of each block
    const int32_t *tile_block;   // [ld/1024] block that holds coordinate 1024*t (clamped to the last block)
    int32_t n_blocks;
    int32_t n_segs;
    int32_t uniform;             // >0: all blocks have this length (the last may be shorter)
};

__global__ __launch_bounds__(kThreads) void bs_partial(const float *__restrict__ g, const float *__restrict__ e,
                                                       int64_t d, int64_t ld, BsTable tb,
                                                       double *__restrict__ partial)
{
    __shared__ double scratch[4];
    const int s = blockIdx.x;
    const int i = blockIdx.y;
    const int lo = tb.seg_lo[s], hi = tb.seg_hi[s];
    const float *grow = g + (int64_t)i * d;
    const float *erow = e + (int64_t)i * ld;
    const int q1 = (hi + 3) >> 2;
    double acc = 0.0;
    for (int q = (lo >> 2) + (int)threadIdx.x; q < q1; q += kThreads) {
        const int j = q << 2;
        const float4 gv = load_grad4(grow, j, d);
        const float4 ev = ld4(erow + j);
        const float x0 = fadd(gv.x, ev.x), x1 = fadd(gv.y, ev.y);
        const float x2 = fadd(gv.z, ev.z), x3 = fadd(gv.w, ev.w);
        if (j >= lo && j < hi) acc += (double)fabsf(x0);
        if (j + 1 >= lo && j + 1 < hi) acc += (double)fabsf(x1);
        if (j + 2 >= lo && j + 2 < hi) acc += (double)fabsf(x2);
        if (j + 3 >= lo && j + 3 < hi) acc += (double)fabsf(x3);
    }
    const double S = block_sum(acc, scratch);
    if (threadIdx.x == 0) partial[(int64_t)i * tb.n_segs + s] = S;
}

// One wavefront per (block, worker).
__global__ __launch_bounds__(kWave) void bs_scale(const double *__restrict__ partial, BsTable tb,
                                                  float *__restrict__ scales)
{
    const int b = blockIdx.x;
    const int i = blockIdx.y;
    const int s0 = tb.block_seg0[b], s1 = tb.block_seg0[b + 1];
    const double *row = partial + (int64_t)i * tb.n_segs;
    double acc = 0.0;
    for (int s = s0 + (int)threadIdx.x; s < s1; s += kWave) acc += row[s];
    const double S = wave_sum(acc);
    if (threadIdx.x == 0) {
        const double len = (double)(tb.offsets[b + 1] - tb.offsets[b]);
        scales[(int64_t)i * tb.n_blocks + b] = (float)(S / len);
    }
}

__device__ __forceinline__ int block_of(const BsTable &tb, int j, int hint)
{
    if (tb.uniform > 0) {
        const int b = j / tb.uniform;
        return b < tb.n_blocks ? b : tb.n_blocks - 1;
    }
    int b = hint;
    while (b + 1 < tb.n_blocks && j >= tb.offsets[b + 1]) ++b;
    return b;
}

constexpr int kBsUnroll = 4;   // workers whose loads are in flight together in bs_apply

__global__ __launch_bounds__(kThreads) void bs_apply(const float *__restrict__ g, float *__restrict__ e, int64_t d,
                                                     int64_t ld, int n, BsTable tb,
                                                     const float *__restrict__ scales, float *__restrict__ theta,
                                                     float *__restrict__ m, float *__restrict__ v,
                                                     float *__restrict__ vhat, AmsParams p)
{
    const int64_t j = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * 4;   // < ld by construction of the grid
    const int jj = (int)j;
    const int hint = tb.uniform > 0 ? 0 : tb.tile_block[blockIdx.x];
    const int b0 = block_of(tb, jj, hint);
    const int b1 = block_of(tb, jj + 1, b0);
    const int b2 = block_of(tb, jj + 2, b1);
    const int b3 = block_of(tb, jj + 3, b2);
    const bool ok0 = j < d, ok1 = j + 1 < d, ok2 = j + 2 < d, ok3 = j + 3 < d;

    // state loads go out first; they are not needed until the worker loop is over
    float4 th = ld4(theta + j), mm = ld4(m + j), vv = ld4(v + j), vh = ld4(vhat + j);
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);

    for (int i0 = 0; i0 < n; i0 += kBsUnroll) {
        float4 gv[kBsUnroll], ev[kBsUnroll], sc[kBsUnroll];
#pragma unroll
        for (int u = 0; u < kBsUnroll; ++u) {
            const int i = i0 + u;
            if (i < n) {
                gv[u] = load_grad4(g + (int64_t)i * d, j, d);
                ev[u] = ld4(e + (int64_t)i * ld + j);
                const float *srow = scales + (int64_t)i * tb.n_blocks;
                const float s0 = srow[b0];
                sc[u] = make_float4(s0, b1 == b0 ? s0 : srow[b1], b2 == b0 ? s0 : srow[b2],
                                    b3 == b0 ? s0 : srow[b3]);
            }
        }
#pragma unroll
        for (int u = 0; u < kBsUnroll; ++u) {
            const int i = i0 + u;
            if (i < n) {
                const float x0 = fadd(gv[u].x, ev[u].x), x1 = fadd(gv[u].y, ev[u].y);
                const float x2 = fadd(gv[u].z, ev[u].z), x3 = fadd(gv[u].w, ev[u].w);
                // C(x) = s * sign(x), sign taken from the IEEE sign bit; nothing at padding coordinates
                const float c0 = ok0 ? copysignf(sc[u].x, x0) : 0.f;
                const float c1 = ok1 ? copysignf(sc[u].y, x1) : 0.f;
                const float c2 = ok2 ? copysignf(sc[u].z, x2) : 0.f;
                const float c3 = ok3 ? copysignf(sc[u].w, x3) : 0.f;
                st4(e + (int64_t)i * ld + j, make_float4(fsub(x0, c0), fsub(x1, c1), fsub(x2, c2),
                                                         fsub(x3, c3)));
                acc.x = fadd(acc.x, c0);
                acc.y = fadd(acc.y, c1);
                acc.z = fadd(acc.z, c2);
                acc.w = fadd(acc.w, c3);
            }
        }
    }
    const float4 gbar = make_float4(fdiv(acc.x, p.n_workers), fdiv(acc.y, p.n_workers),
                                    fdiv(acc.z, p.n_workers), fdiv(acc.w, p.n_workers));
    amsgrad_update4(th, mm, vv, vh, gbar, p);
    st4(theta + j, th);
    st4(m + j, mm);
    st4(v + j, vv);
    st4(vhat + j, vh);
}

}  // namespace cams
