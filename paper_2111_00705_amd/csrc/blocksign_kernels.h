// Scaled-sign compression per contiguous block (Appendix A, "Scaled sign"), with error feedback
// (Section 4), the server average and the AMSGrad update (Section 3).
//
// The error memory is kept in deferred form.  After a step the library stores x_i = g_i + e_i (the
// vector that was compressed) together with that step's block scales s_i; the error itself,
//     e_i[j] = fl32( x_i[j] - copysign(s_i[block(j)], x_i[j]) ),
// is formed on the fly when the next step (or a getter) reads x_i.  The arithmetic is exactly the
// one of the definition, but one step needs a single pass over g and the stored vector:
//
//   bs_pass     per (tile of 4096 coordinates, worker): e = stored x minus its sign compression
//               (previous scales), x = g + e, store x, write the sign bits of x (1 bit per
//               coordinate), fp64 partial sums of |x| per piece (tile x block)
//   bs_scale    per (block, worker): fixed-order fp64 sum of the pieces, s = fl32(S / block length)
//               (skipped when every tile lies in one block of at most 8 pieces: bs_update then
//               adds the pieces itself)
//   bs_update   per tile: gbar[j] = (sum_i +-s_i[block(j)]) / n, signs from the stored bits, workers
//               in ascending order; then the AMSGrad update of theta, m, v, vhat
//
// Traffic per (worker, coordinate): 4 B g + 4 B stored x read + 4 B x written + 2 x 1/8 B of sign
// bits, for any block size; plus 32 B per coordinate of optimiser state.
#pragma once
#include "device_utils.h"

namespace cams {

// Block table on the device.  A "piece" is the intersection of one block with one 4096-aligned
// tile; pieces are numbered in coordinate order, so the pieces of a tile and the pieces of a
// block are both contiguous ranges.
struct BsTable {
    const int32_t *offsets;      // [n_blocks+1] block boundaries
    const int32_t *piece_hi;     // [n_pieces]   one past the last coordinate of a piece
    const int32_t *piece_blk;    // [n_pieces]   block of a piece
    const int32_t *tile_piece0;  // [n_tiles+1]  first piece of a tile
    const int32_t *block_piece0; // [n_blocks+1] first piece of a block
    int32_t n_blocks;
    int32_t n_pieces;
    int32_t uniform_tiles;       // >0: every block spans this many whole tiles (the last block may be shorter),
                                 // so tile t is piece t of block t / uniform_tiles: no table look-ups needed
};

// Sign bits: per worker, per tile, one 16-bit word per thread of the workgroup.  Bit r*4 + c of
// word `tid` is the sign of the coordinate  tile*4096 + 4*(tid + 256*r) + c,  i.e. of the c-th
// component of the r-th float4 that thread tid handles in the tile (same mapping in bs_pass and
// bs_update).
constexpr int kMaxFusedPieces = 8;   // bs_update adds up to this many pieces of a block itself

__device__ __forceinline__ float deferred_sign_error(float xs, float s_prev)
{
    return fsub(xs, copysignf(s_prev, xs));
}

template <bool kPending>
__global__ __launch_bounds__(kThreads) void bs_pass(const float *__restrict__ g, float *__restrict__ xs,
                                                    int64_t d, int64_t ld, BsTable tb,
                                                    const float *__restrict__ s_prev,
                                                    uint16_t *__restrict__ signs,
                                                    double *__restrict__ partial)
{
    __shared__ double scratch[4];
    const int t = blockIdx.x;
    const int i = blockIdx.y;
    const int tid = threadIdx.x;
    const int64_t base = (int64_t)t * kTile;
    const float *grow = g + (int64_t)i * d;
    float *xrow = xs + (int64_t)i * ld;
    const bool uni = tb.uniform_tiles > 0;
    const int p0 = uni ? t : tb.tile_piece0[t], p1 = uni ? t + 1 : tb.tile_piece0[t + 1];
    const float *sp = s_prev + (int64_t)i * tb.n_blocks;

    float4 gv[4], xv[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int64_t j = base + 4 * (tid + kThreads * r);
        gv[r] = load_grad4(grow, j, d);
        xv[r] = ld4(xrow + j);
    }
    float x[4][4];
    uint32_t sign_bits = 0;
    const bool single = (p1 - p0 == 1);
    const float s_single = (kPending && single) ? sp[uni ? t / tb.uniform_tiles : tb.piece_blk[p0]] : 0.f;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int64_t j = base + 4 * (tid + kThreads * r);
        const float gg[4] = {gv[r].x, gv[r].y, gv[r].z, gv[r].w};
        const float xx[4] = {xv[r].x, xv[r].y, xv[r].z, xv[r].w};
        int p = p0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            float e = xx[c];
            if (kPending) {
                float s = s_single;
                if (!single) {
                    while (p + 1 < p1 && j + c >= tb.piece_hi[p]) ++p;
                    s = sp[tb.piece_blk[p]];
                }
                e = deferred_sign_error(xx[c], s);
            }
            x[r][c] = (j + c < d) ? fadd(gg[c], e) : 0.f;
        }
        st4(xrow + j, make_float4(x[r][0], x[r][1], x[r][2], x[r][3]));
#pragma unroll
        for (int c = 0; c < 4; ++c) sign_bits |= (__float_as_uint(x[r][c]) >> 31) << (r * 4 + c);
    }
    signs[((int64_t)i * (ld / kTile) + t) * kThreads + tid] = (uint16_t)sign_bits;

    if (single) {
        double acc = 0.0;
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int c = 0; c < 4; ++c) acc += (double)fabsf(x[r][c]);   // padding coordinates hold 0
        const double S = block_sum(acc, scratch);
        if (tid == 0) partial[(int64_t)i * tb.n_pieces + p0] = S;
    } else {
        for (int p = p0; p < p1; ++p) {
            const int lo = (p == p0) ? (int)base : tb.piece_hi[p - 1];
            const int hi = tb.piece_hi[p];
            double acc = 0.0;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int j = (int)base + 4 * (tid + kThreads * r);
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (j + c >= lo && j + c < hi) acc += (double)fabsf(x[r][c]);
            }
            const double S = block_sum(acc, scratch);
            if (tid == 0) partial[(int64_t)i * tb.n_pieces + p] = S;
        }
    }
}

// One wavefront per (block, worker).
__global__ __launch_bounds__(kWave) void bs_scale(const double *__restrict__ partial, BsTable tb,
                                                  float *__restrict__ scales)
{
    const int b = blockIdx.x;
    const int i = blockIdx.y;
    const int q0 = tb.block_piece0[b], q1 = tb.block_piece0[b + 1];
    const double *row = partial + (int64_t)i * tb.n_pieces;
    double acc = 0.0;
    for (int q = q0 + (int)threadIdx.x; q < q1; q += kWave) acc += row[q];
    const double S = wave_sum(acc);
    if (threadIdx.x == 0) {
        const double len = (double)(tb.offsets[b + 1] - tb.offsets[b]);
        scales[(int64_t)i * tb.n_blocks + b] = (float)(S / len);
    }
}

// copysign(s, x) for the coordinate whose sign is bit `k` of `bits`; s >= 0.
__device__ __forceinline__ float signed_scale(float s, uint32_t bits, int k)
{
    return __uint_as_float(__float_as_uint(s) | ((bits << (31 - k)) & 0x80000000u));
}

constexpr int kScaleChunk = 1024;   // workers whose scales are staged in LDS at a time
constexpr int kSignBatch = 8;       // workers whose sign words are loaded together

// kFusedScale: every tile lies inside one block of at most kMaxFusedPieces pieces; the block's
// scale is formed here from the partial sums (and stored by the tile at the block's start).
// kEarlyState: load theta, m, v, vhat at the start (small grids: nothing else would hide that
// latency); otherwise after the worker loop (large grids: fewer live registers, more workgroups
// per compute unit).
template <bool kFusedScale, bool kEarlyState>
__global__ __launch_bounds__(kThreads) void bs_update(int64_t d, int64_t ld, int n, BsTable tb,
                                                      const double *__restrict__ partial,
                                                      float *__restrict__ scales,
                                                      const uint16_t *__restrict__ signs,
                                                      float *__restrict__ theta, float *__restrict__ m,
                                                      float *__restrict__ v, float *__restrict__ vhat, AmsParams p)
{
    __shared__ float s_lds[kScaleChunk];
    const int t = blockIdx.x;
    const int tid = threadIdx.x;
    const int64_t base = (int64_t)t * kTile;
    const int n_tiles = (int)(ld / kTile);

    float4 th[4], mm[4], vv[4], vh[4];
    if (kEarlyState) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int64_t j = base + 4 * (tid + kThreads * r);
            th[r] = ld4(theta + j);
            mm[r] = ld4(m + j);
            vv[r] = ld4(v + j);
            vh[r] = ld4(vhat + j);
        }
    }
    float acc[16];
#pragma unroll
    for (int q = 0; q < 16; ++q) acc[q] = 0.f;
    const uint16_t *srow = signs + (int64_t)t * kThreads + tid;
    const int64_t sstride = (int64_t)n_tiles * kThreads;

    // sign words of the first workers go out before anything waits
    uint32_t bits[kSignBatch];
#pragma unroll
    for (int u = 0; u < kSignBatch; ++u) bits[u] = (u < n) ? srow[u * sstride] : 0u;

    int p0, p1, b_single;
    if (tb.uniform_tiles > 0) {
        p0 = t;
        p1 = t + 1;
        b_single = t / tb.uniform_tiles;
    } else {
        p0 = tb.tile_piece0[t];
        p1 = tb.tile_piece0[t + 1];
        b_single = tb.piece_blk[p0];
    }
    const bool single = kFusedScale || (p1 - p0 == 1);

    if (single) {
        int q0 = 0, q1 = 0;
        double len = 1.0;
        if (kFusedScale) {
            if (tb.uniform_tiles > 0) {
                q0 = b_single * tb.uniform_tiles;
                q1 = min(q0 + tb.uniform_tiles, n_tiles);
                len = (double)min((int64_t)tb.uniform_tiles * kTile, d - (int64_t)q0 * kTile);
            } else {
                q0 = tb.block_piece0[b_single];
                q1 = tb.block_piece0[b_single + 1];
                len = (double)(tb.offsets[b_single + 1] - tb.offsets[b_single]);
            }
        }
        for (int c0 = 0; c0 < n; c0 += kScaleChunk) {
            const int cn = min(kScaleChunk, n - c0);
            __syncthreads();
            // one thread per worker: the scale of this tile's block
            for (int u = tid; u < cn; u += kThreads) {
                const int i = c0 + u;
                float s;
                if (kFusedScale) {
                    const double *prow = partial + (int64_t)i * tb.n_pieces;
                    double S = 0.0;
                    for (int q = q0; q < q1; ++q) S += prow[q];
                    s = (float)(S / len);
                    if (q0 == p0) scales[(int64_t)i * tb.n_blocks + b_single] = s;   // this tile starts the block
                } else {
                    s = scales[(int64_t)i * tb.n_blocks + b_single];
                }
                s_lds[u] = s;
            }
            __syncthreads();
            for (int u0 = 0; u0 < cn; u0 += kSignBatch) {
                if (c0 + u0 > 0) {
#pragma unroll
                    for (int u = 0; u < kSignBatch; ++u) bits[u] = (u0 + u < cn) ? srow[(c0 + u0 + u) * sstride] : 0u;
                }
#pragma unroll
                for (int u = 0; u < kSignBatch; ++u) {
                    if (u0 + u < cn) {
                        const float s = s_lds[u0 + u];
#pragma unroll
                        for (int q = 0; q < 16; ++q) acc[q] = fadd(acc[q], signed_scale(s, bits[u], q));
                    }
                }
            }
        }
    } else {
        // several blocks meet in this tile: look up the block of every coordinate
        int blk[16];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int j = (int)base + 4 * (tid + kThreads * r);
            int q = p0;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                while (q + 1 < p1 && j + c >= tb.piece_hi[q]) ++q;
                blk[r * 4 + c] = tb.piece_blk[q];
            }
        }
        for (int i = 0; i < n; ++i) {
            const uint32_t w = srow[i * sstride];
            const float *sc = scales + (int64_t)i * tb.n_blocks;
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[q] = fadd(acc[q], signed_scale(sc[blk[q]], w, q));
        }
    }
    if (!kEarlyState) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int64_t j = base + 4 * (tid + kThreads * r);
            th[r] = ld4(theta + j);
            mm[r] = ld4(m + j);
            vv[r] = ld4(v + j);
            vh[r] = ld4(vhat + j);
        }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int64_t j = base + 4 * (tid + kThreads * r);
        // padding coordinates take no gradient
        const float4 gbar = make_float4(j < d ? fdiv(acc[r * 4], p.n_workers) : 0.f,
                                        j + 1 < d ? fdiv(acc[r * 4 + 1], p.n_workers) : 0.f,
                                        j + 2 < d ? fdiv(acc[r * 4 + 2], p.n_workers) : 0.f,
                                        j + 3 < d ? fdiv(acc[r * 4 + 3], p.n_workers) : 0.f);
        amsgrad_update4(th[r], mm[r], vv[r], vh[r], gbar, p);
        st4(theta + j, th[r]);
        st4(m + j, mm[r]);
        st4(v + j, vv[r]);
        st4(vhat + j, vh[r]);
    }
}

// e_i of one worker in its defined form, from the stored x and the pending scales.
template <bool kPending>
__global__ __launch_bounds__(kThreads) void bs_materialize_error(const float *__restrict__ xrow, int64_t d,
                                                                 BsTable tb, const float *__restrict__ sp,
                                                                 float *__restrict__ out)
{
    const int64_t j = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (j >= d) return;
    float e = xrow[j];
    if (kPending) {
        const int t = (int)(j / kTile);
        int q = tb.tile_piece0[t];
        const int q1 = tb.tile_piece0[t + 1];
        while (q + 1 < q1 && j >= tb.piece_hi[q]) ++q;
        e = deferred_sign_error(e, sp[tb.piece_blk[q]]);
    }
    out[j] = e;
}

}  // namespace cams
