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
//               coordinate), fp64 partial sums of |x| per piece (tile x block); a block that lies
//               inside one tile of several pieces gets its scale here
//   bs_scale    per (other block, worker): fixed-order fp64 sum of the pieces, s = fl32(S / block
//               length) (skipped when every tile lies in one block of at most 8 pieces: bs_update
//               then adds the pieces itself)
//   bs_update   per tile: gbar[j] = (sum_i +-s_i[block(j)]) / n, signs from the stored bits, workers
//               in ascending order; then the AMSGrad update of theta, m, v, vhat
//
// Traffic per (worker, coordinate): 4 B g + 4 B stored x read + 4 B x written + 2 x 1/8 B of sign
// bits, for any block size; plus 32 B per coordinate of optimiser state.
//
// CD-Adam (Section 5, Algorithm 1) runs on the same kernels.  The worker's Markov sequence ghat_i
// takes the place of the error memory, again in deferred form: the library stores ghat_i of the step
// before, and c_i = copysign(s_i[block], sign bit) is added when the next step (or a getter) reads
// it.  The sign bits of c_i cannot be read off the stored vector here, so the step reads the old
// sign word before it writes the new one.
//
//   bs_pass<.., kBsCd>   ghat_i += pending c_i, u = g - ghat_i, store ghat_i, sign bits and piece sums of u
//   bs_scale             as above
//   bs_update<.., kMarkov = true>  mean of the c_i as above, ghat += mean, w = ghat - gtilde, sign bits and piece
//                        sums of w (the server's compression, lines 8-9 of Algorithm 1)
//   bs_scale             once more, for the single vector w
//   bs_apply             gtilde += copysign(s, w), then the AMSGrad update with gtilde
//
// Traffic: 12 B per (worker, coordinate) as above, plus 12 B + 40 B per coordinate.
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
    int32_t stream_rows;         // the stored rows are too large to stay cached between steps: bs_pass loads them as a stream
    const int32_t *scale_list;   // [n_scale_list] the blocks whose scale bs_scale forms from the piece sums: all but
    int32_t n_scale_list;        // those that lie inside one tile next to other pieces (bs_pass writes their scale)
    int32_t xcd_chunk;           // bs_pass: tile_of_block's chunk
};

// Sign bits: per worker, per tile, one 16-bit word per thread of the workgroup.  Bit r*4 + c of
// word `tid` is the sign of the coordinate  tile*4096 + 4*(tid + 256*r) + c,  i.e. of the c-th
// component of the r-th float4 that thread tid handles in the tile (same mapping in bs_pass and
// bs_update).
constexpr int kMaxFusedPieces = 8;   // bs_update adds up to this many pieces of a block itself
constexpr unsigned kPassTileLds = kTile * (sizeof(float) + sizeof(uint16_t));   // dynamic LDS bs_pass needs for a
                                                                                // tile of several pieces

__device__ __forceinline__ float deferred_sign_error(float xs, float s_prev)
{
    return fsub(xs, copysignf(s_prev, xs));
}

// copysign(s, x) for the coordinate whose sign is bit `k` of `bits`; s >= 0.
__device__ __forceinline__ float signed_scale(float s, uint32_t bits, int k)
{
    return __uint_as_float(__float_as_uint(s) | ((bits << (31 - k)) & 0x80000000u));
}

// The pieces of a tile of several pieces, in LDS: bound[q] = end of piece p0 + q relative to the tile
// (1 .. 4096), q < p1 - p0.  Inside a tile consecutive pieces belong to consecutive blocks (a new piece starts
// where a block ends), so the block of piece p0 + q is piece_blk[p0] + q and no table is read per coordinate.
// Ends with a barrier.
__device__ __forceinline__ void stage_piece_bounds(uint16_t *bound, int p0, int p1, const BsTable &tb, int64_t base)
{
    for (int q = threadIdx.x; q < p1 - p0; q += kThreads) bound[q] = (uint16_t)(tb.piece_hi[p0 + q] - (int)base);
    __syncthreads();
}
// Index of the piece that holds coordinate l of the tile: the first q with l < bound[q], the last piece for the
// padding past d.  P >= 1 pieces.
__device__ __forceinline__ int piece_index(const uint16_t *bound, int P, int l)
{
    int lo = 0, hi = P - 1;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (l < (int)bound[mid]) hi = mid; else lo = mid + 1;
    }
    return lo;
}

// Fixed-order fp64 sums of |x| over the pieces p0 .. p1-1 of the tile at `base`, one result per piece written
// to out[p].  x: the 16 values of this thread (padding holds 0).
// A tile that is one piece is summed by the whole workgroup.  A tile of several pieces stages |x| in LDS in
// coordinate order (absx, kTile floats) and sums 16 pieces at a time, each by a team of 16 lanes (strided
// partial sums, then a fixed butterfly) - one workgroup reduction per piece made tiles of many short blocks
// tens of times slower.  scales_row (may be null): a block that is a single piece of such a tile lies inside
// the tile, so its scale is complete here and is written at once (bs_scale does not visit it).
// bound: the tile's piece ends as stage_piece_bounds leaves them (only read for a tile of several pieces).
__device__ __forceinline__ void piece_sums(const float (&x)[4][4], int64_t base, int p0, int p1, const BsTable &tb,
                                           double *scratch, float *absx, const uint16_t *bound,
                                           double *__restrict__ out, float *scales_row)
{
    const int tid = threadIdx.x;
    if (p1 - p0 == 1) {
        double acc = 0.0;
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int c = 0; c < 4; ++c) acc += (double)fabsf(x[r][c]);
        const double S = block_sum(acc, scratch);
        if (tid == 0) out[p0] = S;
        return;
    }
#pragma unroll
    for (int r = 0; r < 4; ++r)
        st4(absx + 4 * (tid + kThreads * r), make_float4(fabsf(x[r][0]), fabsf(x[r][1]), fabsf(x[r][2]), fabsf(x[r][3])));
    __syncthreads();
    constexpr int kTeam = 16;
    const int team = tid / kTeam, tl = tid % kTeam;
    const int b0 = tb.piece_blk[p0];
    for (int pb = p0; pb < p1; pb += kThreads / kTeam) {          // uniform over the workgroup
        const int p = pb + team;
        double acc = 0.0;
        int lo = 0, hi = 0;
        if (p < p1) {
            lo = (p == p0) ? 0 : (int)bound[p - p0 - 1];
            hi = (int)bound[p - p0];
            for (int j = lo + tl; j < hi; j += kTeam) acc += (double)absx[j];
        }
#pragma unroll
        for (int off = kTeam / 2; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, kWave);   // stays inside the team
        if (p < p1 && tl == 0) {
            out[p] = acc;
            if (scales_row) {
                // a piece between two others is a whole block; the first and the last may be parts of longer ones
                const int b = b0 + (p - p0);
                const bool inner = p > p0 && p + 1 < p1;
                if (inner || tb.block_piece0[b + 1] - tb.block_piece0[b] == 1) scales_row[b] = (float)(acc / (double)(hi - lo));
            }
        }
    }
}

// kMode: kBsEf error feedback; kBsCd CD-Adam's worker stage (see the head of this file); kBsNaive naive
// compression (Section 4): x = g, nothing is read from or written to the stored rows.
enum { kBsEf = 0, kBsCd = 1, kBsNaive = 2 };

// G: element type of the gradients, float or uint16_t (bfloat16 bits).
template <bool kPending, int kMode, typename G>
__global__ __launch_bounds__(kThreads) void bs_pass(const G *__restrict__ g, float *__restrict__ xs,
                                                    int64_t d, int64_t ld, BsTable tb,
                                                    float *scales,          // [n][n_blocks]: the previous step's are
                                                                            // read; blocks inside a tile get their new one
                                                    uint16_t *__restrict__ signs,
                                                    double *__restrict__ partial)
{
    __shared__ double scratch[4];
    // dynamic LDS, kPassTileLds bytes when the table has tiles of several pieces (only those use it): the staged
    // |x| and the piece ends.  The host may ask for more: the amount also sets how many workgroups share a
    // compute unit, which this kernel is sensitive to (see pass_lds_bytes in the host code).
    extern __shared__ __align__(16) unsigned char pass_lds[];
    float *absx = reinterpret_cast<float *>(pass_lds);
    uint16_t *bound = reinterpret_cast<uint16_t *>(pass_lds + kTile * sizeof(float));
    const float *s_prev = scales;
    const int t = tile_of_block(blockIdx.x, tb.xcd_chunk);
    if (t >= (int)(ld / kTile)) return;
    const int i = blockIdx.y;
    const int tid = threadIdx.x;
    const int64_t base = (int64_t)t * kTile;
    const G *grow = g + (int64_t)i * d;
    float *xrow = xs + (int64_t)i * ld;
    const bool uni = tb.uniform_tiles > 0;
    const int p0 = uni ? t : tb.tile_piece0[t], p1 = uni ? t + 1 : tb.tile_piece0[t + 1];
    const float *sp = s_prev + (int64_t)i * tb.n_blocks;

    float4 gv[4], xv[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int64_t j = base + 4 * (tid + kThreads * r);
        gv[r] = load_grad4(grow, j, d);
        xv[r] = kMode == kBsNaive ? make_float4(0.f, 0.f, 0.f, 0.f) : ld4_row(xrow + j, tb.stream_rows);
    }
    uint16_t *word = signs + ((int64_t)i * (ld / kTile) + t) * kThreads + tid;
    const uint32_t old_bits = (kMode == kBsCd && kPending) ? (uint32_t)*word : 0u;   // sign bits of the pending c_i
    float x[4][4];
    uint32_t sign_bits = 0;
    const bool single = (p1 - p0 == 1);
    const int P = p1 - p0;
    const int b0 = (uni || (single && !kPending)) ? 0 : tb.piece_blk[p0];     // block of the tile's first piece
    const float s_single = (kPending && single) ? sp[uni ? t / tb.uniform_tiles : b0] : 0.f;
    if (!single) stage_piece_bounds(bound, p0, p1, tb, base);               // uniform over the workgroup
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int64_t j = base + 4 * (tid + kThreads * r);
        const int l0 = 4 * (tid + kThreads * r);
        const float gg[4] = {gv[r].x, gv[r].y, gv[r].z, gv[r].w};
        const float xx[4] = {xv[r].x, xv[r].y, xv[r].z, xv[r].w};
        float keep[4];     // what goes back to the stored vector
        int q = (kPending && !single) ? piece_index(bound, P, l0) : 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            float s = s_single;
            if (kPending && !single) {
                while (q + 1 < P && l0 + c >= (int)bound[q]) ++q;
                s = sp[b0 + q];
            }
            if (kMode == kBsCd) {
                // ghat_i = ghat_i + c_i (Algorithm 1, line 6, of the step before); u = g - ghat_i (line 5)
                float gh = xx[c];
                if (kPending && j + c < d) gh = fadd(gh, signed_scale(s, old_bits, r * 4 + c));
                keep[c] = gh;
                x[r][c] = (j + c < d) ? fsub(gg[c], gh) : 0.f;
            } else if (kMode == kBsNaive) {
                x[r][c] = (j + c < d) ? gg[c] : 0.f;
                keep[c] = 0.f;
            } else {
                const float e = kPending ? deferred_sign_error(xx[c], s) : xx[c];
                x[r][c] = (j + c < d) ? fadd(gg[c], e) : 0.f;
                keep[c] = x[r][c];
            }
        }
        if (kMode != kBsNaive) st4_stream(xrow + j, make_float4(keep[0], keep[1], keep[2], keep[3]));
#pragma unroll
        for (int c = 0; c < 4; ++c) sign_bits |= (__float_as_uint(x[r][c]) >> 31) << (r * 4 + c);
    }
    *word = (uint16_t)sign_bits;
    // every thread has read the scales it needs (the loop above) before any is rewritten (after the barrier inside)
    piece_sums(x, base, p0, p1, tb, scratch, absx, bound, partial + (int64_t)i * tb.n_pieces,
               scales + (int64_t)i * tb.n_blocks);
}

// One wavefront per (listed block, worker): see BsTable::scale_list.
__global__ __launch_bounds__(kWave) void bs_scale(const double *__restrict__ partial, BsTable tb,
                                                  float *__restrict__ scales)
{
    const int b = tb.scale_list[blockIdx.x];
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

constexpr int kScaleChunk = 1024;   // workers whose scales are staged in LDS at a time
constexpr int kSignBatch = 8;       // workers whose sign words are loaded together

// kFusedScale: every tile lies inside one block of at most kMaxFusedPieces pieces; the block's
// scale is formed here from the partial sums (and stored by the tile at the block's start).
// kEarlyState: load theta, m, v, vhat at the start (small grids: nothing else would hide that
// latency); otherwise after the worker loop (large grids: fewer live registers, more workgroups
// per compute unit).
// kMarkov: CD-Adam's server stage instead of the AMSGrad update: the mean of the c_i goes into
// ghat (Algorithm 1, line 8), w = ghat - gtilde is formed, and its sign bits and piece sums are
// written for the second compression (line 9).  The arrays of the Markov struct are only touched
// then; theta, m, v, vhat only otherwise.
// kStreamState: theta, m, v, vhat are loaded and stored as streams (see ld4_state).
struct BsMarkov {
    float *ghat;            // [ld] the server's aggregate
    float *gtil;            // [ld] gtilde of the step before (rewritten here only when whole_blocks is set)
    uint16_t *signs;        // [n_tiles][256] sign bits of w
    double *partial;        // [n_pieces] piece sums of |w|
    float *scales;          // [n_blocks] scales of the server's message
    int32_t whole_blocks;   // every tile is exactly one block: the block's scale of w is known inside the
                            // workgroup, so lines 9-16 of Algorithm 1 follow at once (no bs_scale, no bs_apply)
};

template <bool kFusedScale, bool kEarlyState, bool kMarkov, bool kStreamState>
__global__ __launch_bounds__(kThreads) void bs_update(int64_t d, int64_t ld, int n, BsTable tb,
                                                      const double *__restrict__ partial,
                                                      float *__restrict__ scales,
                                                      const uint16_t *__restrict__ signs,
                                                      float *__restrict__ theta, float *__restrict__ m,
                                                      float *__restrict__ v, float *__restrict__ vhat, AmsParams p,
                                                      BsMarkov mk)
{
    __shared__ float s_lds[kScaleChunk];
    __shared__ double scratch[4];
    __shared__ float absx[kMarkov ? kTile : 1];      // piece_sums of the server's vector
    __shared__ uint16_t bound[kTile];                // piece ends of a tile where several blocks meet
    const int t = blockIdx.x;
    const int tid = threadIdx.x;
    const int64_t base = (int64_t)t * kTile;
    const int n_tiles = (int)(ld / kTile);

    float4 th[4], mm[4], vv[4], vh[4];
    if (kEarlyState && !kMarkov) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int64_t j = base + 4 * (tid + kThreads * r);
            th[r] = ld4_state<kStreamState>(theta + j);
            mm[r] = ld4_state<kStreamState>(m + j);
            vv[r] = ld4_state<kStreamState>(v + j);
            vh[r] = ld4_state<kStreamState>(vhat + j);
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
                // the sign words of the batch after this one go out before this one is used
                uint32_t next[kSignBatch];
                const int w1 = c0 + u0 + kSignBatch;       // first worker of the next batch (may be in the next chunk)
#pragma unroll
                for (int u = 0; u < kSignBatch; ++u) next[u] = (w1 + u < n) ? srow[(w1 + u) * sstride] : 0u;
#pragma unroll
                for (int u = 0; u < kSignBatch; ++u) {
                    if (u0 + u < cn) {
                        const float s = s_lds[u0 + u];
#pragma unroll
                        for (int q = 0; q < 16; ++q) acc[q] = fadd(acc[q], signed_scale(s, bits[u], q));
                    }
                }
#pragma unroll
                for (int u = 0; u < kSignBatch; ++u) bits[u] = next[u];
            }
        }
    } else {
        // several blocks meet in this tile: find the block of every coordinate
        stage_piece_bounds(bound, p0, p1, tb, base);
        const int P = p1 - p0;
        int blk[16];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int l0 = 4 * (tid + kThreads * r);
            int q = piece_index(bound, P, l0);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                while (q + 1 < P && l0 + c >= (int)bound[q]) ++q;
                blk[r * 4 + c] = b_single + q;            // b_single: the block of the tile's first piece
            }
        }
        for (int i = 0; i < n; ++i) {
            const uint32_t w = srow[i * sstride];
            const float *sc = scales + (int64_t)i * tb.n_blocks;
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[q] = fadd(acc[q], signed_scale(sc[blk[q]], w, q));
        }
    }
    if (kMarkov) {
        float w[4][4];
        uint32_t sign_bits = 0;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int64_t j = base + 4 * (tid + kThreads * r);
            const float4 gh4 = ld4(mk.ghat + j), gt4 = ld4(mk.gtil + j);
            const float gh[4] = {gh4.x, gh4.y, gh4.z, gh4.w}, gt[4] = {gt4.x, gt4.y, gt4.z, gt4.w};
            float nh[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                // padding coordinates stay 0
                nh[c] = (j + c < d) ? fadd(gh[c], fdiv(acc[r * 4 + c], p.n_workers)) : gh[c];
                w[r][c] = (j + c < d) ? fsub(nh[c], gt[c]) : 0.f;
                sign_bits |= (__float_as_uint(w[r][c]) >> 31) << (r * 4 + c);
            }
            st4(mk.ghat + j, make_float4(nh[0], nh[1], nh[2], nh[3]));
        }
        mk.signs[(int64_t)t * kThreads + tid] = (uint16_t)sign_bits;
        __syncthreads();   // s_lds readers are done before scratch is used (separate arrays; keeps phases apart)
        if (!mk.whole_blocks) {
            piece_sums(w, base, p0, p1, tb, scratch, absx, bound, mk.partial, mk.scales);
            return;
        }
        // c = C(w) with the scale of this tile's block, gtilde += c, AMSGrad with gtilde
        double a64 = 0.0;
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int c = 0; c < 4; ++c) a64 += (double)fabsf(w[r][c]);
        const double S = block_sum(a64, scratch);
        const double blen = (double)min((int64_t)kTile, d - base);
        const float s = (float)(S / blen);
        if (tid == 0) mk.scales[b_single] = s;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int64_t j = base + 4 * (tid + kThreads * r);
            const float4 gt4 = ld4(mk.gtil + j);       // in cache: read a moment ago
            const float gt[4] = {gt4.x, gt4.y, gt4.z, gt4.w};
            float nt[4];
#pragma unroll
            for (int c = 0; c < 4; ++c)
                nt[c] = (j + c < d) ? fadd(gt[c], signed_scale(s, sign_bits, r * 4 + c)) : gt[c];   // padding stays 0
            const float4 g4 = make_float4(nt[0], nt[1], nt[2], nt[3]);
            float4 th4 = ld4_state<kStreamState>(theta + j), m4 = ld4_state<kStreamState>(m + j), v4 = ld4_state<kStreamState>(v + j), vh4 = ld4_state<kStreamState>(vhat + j);
            amsgrad_update4(th4, m4, v4, vh4, g4, p);
            st4(mk.gtil + j, g4);
            st4_state<kStreamState>(theta + j, th4);
            st4_state<kStreamState>(m + j, m4);
            st4_state<kStreamState>(v + j, v4);
            st4_state<kStreamState>(vhat + j, vh4);
        }
        return;
    }
    if (!kEarlyState) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int64_t j = base + 4 * (tid + kThreads * r);
            th[r] = ld4_state<kStreamState>(theta + j);
            mm[r] = ld4_state<kStreamState>(m + j);
            vv[r] = ld4_state<kStreamState>(v + j);
            vh[r] = ld4_state<kStreamState>(vhat + j);
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
        st4_state<kStreamState>(theta + j, th[r]);
        st4_state<kStreamState>(m + j, mm[r]);
        st4_state<kStreamState>(v + j, vv[r]);
        st4_state<kStreamState>(vhat + j, vh[r]);
    }
}

// ---------------------------------------------------------------------------------------------
// Error feedback with uniform blocks of whole tiles (at most kMaxFusedPieces each), one launch per step.
// The AMSGrad update of a step depends on nothing but that step's sign words and piece sums, and the next step's
// pass reads neither theta, m, v nor vhat: so the update of step t is deferred and runs inside the pass kernel of
// step t + 1, as extra workgroups that are dispatched first (blockIdx.y < 4: the four quarters of every tile;
// blockIdx.y >= 4: the pass of worker blockIdx.y - 4).  On small models the update alone is a chain of latencies
// on a mostly idle chip (293 workgroups for 1.2 M coordinates); inside the pass it costs its bytes.  Sign words
// and piece sums exist twice and alternate: the pass of step t + 1 writes one set while the update of step t reads
// the other.  The scales of step t are formed from its piece sums where they are needed - by the pass (the
// deferred error of the stored rows) and by the update - with the same arithmetic: the fp64 sum of the block's
// pieces in coordinate order, one division, one rounding.
struct BsDeferred {
    const uint16_t *signs_prev;     // [n][n_tiles][256] sign words of the step whose update is pending
    const double *partial_prev;     // [n][n_pieces] its piece sums (also what the pass takes the pending scales from)
    float *scales_out;              // [n][n_blocks] the update writes that step's scales here (for the getters)
    float *theta, *m, *v, *vhat;
    AmsParams p;                    // hyper-parameters of the step whose update is pending
    int32_t do_update;              // 0: nothing is pending (first step, or the update has been run on its own)
};

// The scale of block b = the tile's block for worker i from that worker's piece sums (uniform tiles).
__device__ __forceinline__ float fused_block_scale(const double *__restrict__ prow, int b, const BsTable &tb, int n_tiles,
                                                   int64_t d)
{
    const int q0 = b * tb.uniform_tiles, q1 = min(q0 + tb.uniform_tiles, n_tiles);
    const double len = (double)min((int64_t)tb.uniform_tiles * kTile, d - (int64_t)q0 * kTile);
    double S = 0.0;
    for (int q = q0; q < q1; ++q) S += prow[q];
    return (float)(S / len);
}

template <bool kPending, typename G, bool kStreamState>
__global__ __launch_bounds__(kThreads) void bs_pass_update(const G *__restrict__ g, float *__restrict__ xs, int64_t d,
                                                           int64_t ld, int n, BsTable tb,
                                                           uint16_t *__restrict__ signs, double *__restrict__ partial,
                                                           BsDeferred df)
{
    __shared__ double scratch[4];
    __shared__ float s_lds[kScaleChunk];
    // dynamic LDS: none is used; the amount only sets how many workgroups share a compute unit (see bs_pass)
    const int n_tiles = (int)(ld / kTile);
    const int t = tile_of_block(blockIdx.x, tb.xcd_chunk);
    if (t >= n_tiles) return;
    const int tid = threadIdx.x;
    const int64_t base = (int64_t)t * kTile;
    const int b = t / tb.uniform_tiles;

    if (blockIdx.y < 4) {
        // ---- the pending update of quarter r of tile t: coordinates base + 4 (tid + 256 r) + c
        if (!df.do_update) return;
        const int r = blockIdx.y;
        const int64_t j = base + 4 * (tid + kThreads * r);
        const float4 th0 = ld4_state<kStreamState>(df.theta + j), m0 = ld4_state<kStreamState>(df.m + j),
                     v0 = ld4_state<kStreamState>(df.v + j), vh0 = ld4_state<kStreamState>(df.vhat + j);
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
        const uint16_t *srow = df.signs_prev + (int64_t)t * kThreads + tid;
        const int64_t sstride = (int64_t)n_tiles * kThreads;
        const bool first_tile = (t == b * tb.uniform_tiles);
        for (int c0 = 0; c0 < n; c0 += kScaleChunk) {
            const int cn = min(kScaleChunk, n - c0);
            __syncthreads();
            for (int u = tid; u < cn; u += kThreads) {          // one thread per worker: the scale of this tile's block
                const float s = fused_block_scale(df.partial_prev + (int64_t)(c0 + u) * tb.n_pieces, b, tb, n_tiles, d);
                s_lds[u] = s;
                if (first_tile && r == 0) df.scales_out[(int64_t)(c0 + u) * tb.n_blocks + b] = s;
            }
            __syncthreads();
            for (int u0 = 0; u0 < cn; u0 += kSignBatch) {
                uint32_t bits[kSignBatch];
#pragma unroll
                for (int u = 0; u < kSignBatch; ++u) bits[u] = (u0 + u < cn) ? (uint32_t)srow[(c0 + u0 + u) * sstride] : 0u;
#pragma unroll
                for (int u = 0; u < kSignBatch; ++u) {
                    if (u0 + u < cn) {
                        const float s = s_lds[u0 + u];
#pragma unroll
                        for (int c = 0; c < 4; ++c) acc[c] = fadd(acc[c], signed_scale(s, bits[u], r * 4 + c));
                    }
                }
            }
        }
        // padding coordinates take no gradient
        const float4 gbar = make_float4(j < d ? fdiv(acc[0], df.p.n_workers) : 0.f, j + 1 < d ? fdiv(acc[1], df.p.n_workers) : 0.f,
                                        j + 2 < d ? fdiv(acc[2], df.p.n_workers) : 0.f, j + 3 < d ? fdiv(acc[3], df.p.n_workers) : 0.f);
        float4 th = th0, mm = m0, vv = v0, vh = vh0;
        amsgrad_update4(th, mm, vv, vh, gbar, df.p);
        st4_state<kStreamState>(df.theta + j, th);
        st4_state<kStreamState>(df.m + j, mm);
        st4_state<kStreamState>(df.v + j, vv);
        st4_state<kStreamState>(df.vhat + j, vh);
        return;
    }

    // ---- the pass of worker i over tile t (one piece: the tile lies inside block b)
    const int i = blockIdx.y - 4;
    const G *grow = g + (int64_t)i * d;
    float *xrow = xs + (int64_t)i * ld;
    float4 gv[4], xv[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int64_t j = base + 4 * (tid + kThreads * r);
        gv[r] = load_grad4(grow, j, d);
        xv[r] = ld4_row(xrow + j, tb.stream_rows);
    }
    const float s_prev = kPending ? fused_block_scale(df.partial_prev + (int64_t)i * tb.n_pieces, b, tb, n_tiles, d) : 0.f;
    float x[4][4];
    uint32_t sign_bits = 0;
    double a64 = 0.0;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int64_t j = base + 4 * (tid + kThreads * r);
        const float gg[4] = {gv[r].x, gv[r].y, gv[r].z, gv[r].w};
        const float xx[4] = {xv[r].x, xv[r].y, xv[r].z, xv[r].w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const float e = kPending ? deferred_sign_error(xx[c], s_prev) : xx[c];
            x[r][c] = (j + c < d) ? fadd(gg[c], e) : 0.f;
        }
        st4_stream(xrow + j, make_float4(x[r][0], x[r][1], x[r][2], x[r][3]));
#pragma unroll
        for (int c = 0; c < 4; ++c) sign_bits |= (__float_as_uint(x[r][c]) >> 31) << (r * 4 + c);
    }
    signs[((int64_t)i * n_tiles + t) * kThreads + tid] = (uint16_t)sign_bits;
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c) a64 += (double)fabsf(x[r][c]);
    const double S = block_sum(a64, scratch);
    if (tid == 0) partial[(int64_t)i * tb.n_pieces + t] = S;
}

// Wire form of the sign bits of one vector: output word q holds the coordinates 32 q .. 32 q + 31, bit
// j % 32 for coordinate j (set = negative), zero past d.  Those 32 coordinates are eight consecutive
// float4 of one row r of the tile, i.e. the r-th nibble of eight consecutive sign words.
__global__ __launch_bounds__(kThreads) void bs_pack_signs(const uint16_t *__restrict__ words, int64_t d,
                                                          uint32_t *__restrict__ out)
{
    const int64_t q = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (q * 32 >= d) return;
    const int64_t t = (q * 32) / kTile;
    const int vec0 = (int)((q * 32) % kTile) / 4;            // first of the eight float4
    const int r = vec0 / kThreads, tid0 = vec0 % kThreads;
    uint32_t bits = 0;
#pragma unroll
    for (int u = 0; u < 8; ++u)
        bits |= (((uint32_t)words[t * kThreads + tid0 + u] >> (r * 4)) & 0xfu) << (4 * u);
    const int64_t left = d - q * 32;
    if (left < 32) bits &= (1u << left) - 1u;
    out[q] = bits;
}

// e_i of one worker in its defined form, from the stored x and the pending scales.  out may be xrow itself
// (every thread reads its own element before it writes it).
template <bool kPending>
__global__ __launch_bounds__(kThreads) void bs_materialize_error(const float *xrow, int64_t d, BsTable tb,
                                                                 const float *__restrict__ sp, float *out)
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

// CD-Adam, Algorithm 1, lines 10 and 12-16: gtilde += c with c = copysign(s[block], w) from the
// server's sign bits and scales, then the AMSGrad update with gtilde.  One workgroup per tile.
template <bool kStreamState>
__global__ __launch_bounds__(kThreads) void bs_apply(int64_t d, BsTable tb, const float *__restrict__ scales,
                                                     const uint16_t *__restrict__ signs, float *__restrict__ gtil,
                                                     float *__restrict__ theta, float *__restrict__ m,
                                                     float *__restrict__ v, float *__restrict__ vhat, AmsParams p)
{
    __shared__ uint16_t bound[kTile];                // piece ends of a tile where several blocks meet
    const int t = blockIdx.x;
    const int tid = threadIdx.x;
    const int64_t base = (int64_t)t * kTile;
    const uint32_t bits = signs[(int64_t)t * kThreads + tid];
    float4 gt[4], th[4], mm[4], vv[4], vh[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int64_t j = base + 4 * (tid + kThreads * r);
        gt[r] = ld4(gtil + j);
        th[r] = ld4_state<kStreamState>(theta + j);
        mm[r] = ld4_state<kStreamState>(m + j);
        vv[r] = ld4_state<kStreamState>(v + j);
        vh[r] = ld4_state<kStreamState>(vhat + j);
    }
    int p0, p1;
    if (tb.uniform_tiles > 0) {
        p0 = t;
        p1 = t + 1;
    } else {
        p0 = tb.tile_piece0[t];
        p1 = tb.tile_piece0[t + 1];
    }
    const bool single = (p1 - p0 == 1);
    const int P = p1 - p0;
    const int b0 = tb.uniform_tiles > 0 ? t / tb.uniform_tiles : tb.piece_blk[p0];   // block of the tile's first piece
    const float s_single = single ? scales[b0] : 0.f;
    if (!single) stage_piece_bounds(bound, p0, p1, tb, base);                         // uniform over the workgroup
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int64_t j = base + 4 * (tid + kThreads * r);
        const int l0 = 4 * (tid + kThreads * r);
        const float old[4] = {gt[r].x, gt[r].y, gt[r].z, gt[r].w};
        float nt[4];
        int q = single ? 0 : piece_index(bound, P, l0);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            float s = s_single;
            if (!single) {
                while (q + 1 < P && l0 + c >= (int)bound[q]) ++q;
                s = scales[b0 + q];
            }
            nt[c] = (j + c < d) ? fadd(old[c], signed_scale(s, bits, r * 4 + c)) : old[c];   // padding stays 0
        }
        const float4 g4 = make_float4(nt[0], nt[1], nt[2], nt[3]);
        amsgrad_update4(th[r], mm[r], vv[r], vh[r], g4, p);
        st4(gtil + j, g4);
        st4_state<kStreamState>(theta + j, th[r]);
        st4_state<kStreamState>(m + j, mm[r]);
        st4_state<kStreamState>(v + j, vv[r]);
        st4_state<kStreamState>(vhat + j, vh[r]);
    }
}

// ghat_i of one worker in its defined form: the stored vector plus the pending c_i.  out may be xrow itself.
template <bool kPending>
__global__ __launch_bounds__(kThreads) void bs_materialize_markov(const float *xrow, int64_t d, BsTable tb,
                                                                  const float *__restrict__ sp,
                                                                  const uint16_t *__restrict__ signs_row, float *out)
{
    const int64_t j = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (j >= d) return;
    float gh = xrow[j];
    if (kPending) {
        const int t = (int)(j / kTile);
        int q = tb.tile_piece0[t];
        const int q1 = tb.tile_piece0[t + 1];
        while (q + 1 < q1 && j >= tb.piece_hi[q]) ++q;
        // coordinate 4 * (tid + 256 * r) + c of the tile is bit r * 4 + c of the word of thread tid
        const int l = (int)(j - (int64_t)t * kTile);
        const int vec = l >> 2, c = l & 3;
        const uint32_t bits = signs_row[(int64_t)t * kThreads + (vec & (kThreads - 1))];
        gh = fadd(gh, signed_scale(sp[tb.piece_blk[q]], bits, (vec / kThreads) * 4 + c));
    }
    out[j] = gh;
}

}  // namespace cams
