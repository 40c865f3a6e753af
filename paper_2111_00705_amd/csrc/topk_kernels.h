// Top-k compression (Appendix A, "Top-k") with error feedback (Section 4), server average and
// AMSGrad update (Section 3).
//
// Selection is an exact radix select, not a sort.  Every element gets the composite key
//     comp = (magnitude_bits << IB) | (2^IB - 1 - index),     magnitude_bits = bits(x) & 0x7fffffff,
// IB = number of bits of d-1.  comp is unique per element and its descending order is
// "larger magnitude first, lower index first among equals", so Top-k is { comp >= Tc } where Tc is
// the k-th largest comp.  Tc is found digit by digit from the top:
//
//   tk_pass1    streams g and e once: x = g+e is written over e, an LDS histogram of the top 11
//               magnitude bits goes to a per-worker global histogram, and elements whose bin is at
//               least the worker's guess (carried over from the previous step) are listed as
//               candidates, per (worker, tile), as 16-bit positions inside the tile
//   tk_findbin  per worker: the bin b* that holds the k-th largest and the rank left inside it;
//               checks the guess (guess <= b* means the candidates cover every possible pick)
//   tk_collect  only for workers whose guess failed (always on the first step): re-reads x and
//               lists the elements with bin >= b*
//   tk_scan / tk_find   one pair per further digit (<= 12 bits): histogram of that digit over the
//               candidates that match the digits fixed so far, then pick the digit of the k-th
//   tk_final    per tile, all workers: candidates with comp >= Tc are the kept coordinates; their
//               values are summed into an LDS copy of the tile in ascending worker order, their
//               error entries are zeroed, the kept (position, value) pairs are recorded, and the
//               tile's theta, m, v, vhat are updated from gbar = acc / n
//
// Apart from the candidates (a few per cent of the elements) g and e are read once and e is
// written once.
#pragma once
#include "device_utils.h"

namespace cams {

constexpr int kBins1 = 2048;      // pass-1 digit: top 11 of the 31 magnitude bits
constexpr int kShift1 = 20;
constexpr int kDigitBits = 12;    // later digits
constexpr int kBins2 = 1 << kDigitBits;
constexpr uint32_t kNoGuess = kBins1;   // guess that lists nothing (before the first step)

struct TkWorker {
    uint64_t prefix;        // digits of Tc fixed so far, right-aligned
    uint64_t tc;            // threshold composite, valid once done != 0
    uint32_t rank;          // 1-based rank (from the top) of Tc among elements matching prefix
    uint32_t bstar;         // pass-1 bin of the k-th largest magnitude
    uint32_t guess;         // pass 1 lists elements with bin >= guess
    uint32_t need_collect;  // the guess was above b*: candidates must be rebuilt
    uint32_t done;          // Tc is final
    uint32_t pad;
};

struct TkGeom {
    int64_t d, ld;
    int32_t n, n_tiles;
    int32_t idx_bits;       // IB
    uint32_t k;
};

__device__ __forceinline__ uint64_t composite(float x, uint32_t j, int idx_bits)
{
    const uint64_t inv = ((1ull << idx_bits) - 1ull) - (uint64_t)j;
    return ((uint64_t)mag_key(x) << idx_bits) | inv;
}

// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void tk_pass1(const float *__restrict__ g, float *__restrict__ e, TkGeom ge,
                                                     const TkWorker *__restrict__ ws,
                                                     uint32_t *__restrict__ hist1,
                                                     uint16_t *__restrict__ cand_idx,
                                                     uint32_t *__restrict__ cand_cnt)
{
    __shared__ uint32_t lh[kBins1];
    __shared__ uint32_t lcnt;
    const int i = blockIdx.y;
    const uint32_t guess = ws[i].guess;
    const float *grow = g + (int64_t)i * ge.d;
    float *erow = e + (int64_t)i * ge.ld;
    for (int b = threadIdx.x; b < kBins1; b += kThreads) lh[b] = 0;

    for (int t = blockIdx.x; t < ge.n_tiles; t += gridDim.x) {
        if (threadIdx.x == 0) lcnt = 0;
        __syncthreads();   // also orders the histogram reset before the first tile
        const int64_t base = (int64_t)t * kTile;
        uint16_t *seg = cand_idx + (((int64_t)i * ge.n_tiles + t) << 12);
        float4 gv[4], ev[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int64_t j = base + 4 * (threadIdx.x + kThreads * r);
            gv[r] = load_grad4(grow, j, ge.d);
            ev[r] = ld4(erow + j);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int l = 4 * (threadIdx.x + kThreads * r);
            const int64_t j = base + l;
            float x[4] = {fadd(gv[r].x, ev[r].x), fadd(gv[r].y, ev[r].y), fadd(gv[r].z, ev[r].z),
                          fadd(gv[r].w, ev[r].w)};
            st4(erow + j, make_float4(x[0], x[1], x[2], x[3]));
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (j + c < ge.d) {
                    const uint32_t bin = mag_key(x[c]) >> kShift1;
                    atomicAdd(&lh[bin], 1u);
                    if (bin >= guess) {
                        const uint32_t slot = atomicAdd(&lcnt, 1u);   // < kTile: one slot per element
                        seg[slot] = (uint16_t)(l + c);
                    }
                }
            }
        }
        __syncthreads();
        if (threadIdx.x == 0) cand_cnt[(int64_t)i * ge.n_tiles + t] = lcnt;
    }
    __syncthreads();
    for (int b = threadIdx.x; b < kBins1; b += kThreads) {
        const uint32_t c = lh[b];
        if (c) atomicAdd(&hist1[(int64_t)i * kBins1 + b], c);
    }
}

// Finds, in a histogram row of `bins` counters held in LDS, the bin of the element of 1-based rank
// `rank` counted from the top bin downwards.  Exactly one thread gets true and receives the bin,
// the number of elements in higher bins and the bin's own count.  Requires 1 <= rank <= total.
// `part` holds kThreads counters of LDS; bins is a multiple of kThreads.
__device__ __forceinline__ bool find_rank_bin(const uint32_t *lh, uint32_t *part, int bins, uint32_t rank,
                                              uint32_t &bin_out, uint32_t &above_out, uint32_t &count_out)
{
    const int per = bins / kThreads;
    uint32_t mine = 0;
    for (int q = 0; q < per; ++q) mine += lh[threadIdx.x * per + q];
    part[threadIdx.x] = mine;
    __syncthreads();
    uint32_t above = 0;
    for (int c = threadIdx.x + 1; c < kThreads; ++c) above += part[c];
    bool found = false;
    if (above < rank && above + mine >= rank) {
        for (int q = per - 1; q >= 0; --q) {
            const uint32_t c = lh[threadIdx.x * per + q];
            if (above + c >= rank) {
                bin_out = threadIdx.x * per + q;
                above_out = above;
                count_out = c;
                found = true;
                break;
            }
            above += c;
        }
    }
    return found;
}

__global__ __launch_bounds__(kThreads) void tk_findbin(TkGeom ge, TkWorker *__restrict__ ws,
                                                       uint32_t *__restrict__ hist1)
{
    __shared__ uint32_t lh[kBins1];
    __shared__ uint32_t part[kThreads];
    const int i = blockIdx.x;
    uint32_t *row = hist1 + (int64_t)i * kBins1;
    for (int b = threadIdx.x; b < kBins1; b += kThreads) {
        lh[b] = row[b];
        row[b] = 0;   // consumed: ready for the next step
    }
    __syncthreads();
    uint32_t bin, above, count;
    if (find_rank_bin(lh, part, kBins1, ge.k, bin, above, count)) {
        TkWorker w = ws[i];
        w.bstar = bin;
        w.prefix = bin;
        w.rank = ge.k - above;
        w.need_collect = (w.guess > bin) ? 1u : 0u;
        w.done = (count == w.rank) ? 1u : 0u;                    // the whole bin is kept
        w.tc = (uint64_t)bin << (kShift1 + ge.idx_bits);
        w.guess = bin >= 2 ? bin - 2 : 0;                        // next step: a quarter octave of slack
        ws[i] = w;
    }
}

__global__ __launch_bounds__(kThreads) void tk_collect(const float *__restrict__ e, TkGeom ge,
                                                       const TkWorker *__restrict__ ws,
                                                       uint16_t *__restrict__ cand_idx,
                                                       uint32_t *__restrict__ cand_cnt)
{
    __shared__ uint32_t lcnt;
    const int i = blockIdx.y;
    if (!ws[i].need_collect) return;   // uniform over the workgroup
    const uint32_t bstar = ws[i].bstar;
    const float *erow = e + (int64_t)i * ge.ld;
    for (int t = blockIdx.x; t < ge.n_tiles; t += gridDim.x) {
        if (threadIdx.x == 0) lcnt = 0;
        __syncthreads();
        const int64_t base = (int64_t)t * kTile;
        uint16_t *seg = cand_idx + (((int64_t)i * ge.n_tiles + t) << 12);
        float4 xv[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) xv[r] = ld4(erow + base + 4 * (threadIdx.x + kThreads * r));
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int l = 4 * (threadIdx.x + kThreads * r);
            const float x[4] = {xv[r].x, xv[r].y, xv[r].z, xv[r].w};
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (base + l + c < ge.d && (mag_key(x[c]) >> kShift1) >= bstar) {
                    const uint32_t slot = atomicAdd(&lcnt, 1u);
                    seg[slot] = (uint16_t)(l + c);
                }
            }
        }
        __syncthreads();
        if (threadIdx.x == 0) cand_cnt[(int64_t)i * ge.n_tiles + t] = lcnt;
    }
}

// One digit of Tc: histogram of bits [s_lo, s_hi) of comp over the candidates whose bits above
// s_hi equal the prefix.  One wavefront per tile.
__global__ __launch_bounds__(kThreads) void tk_scan(const float *__restrict__ e, TkGeom ge,
                                                    const TkWorker *__restrict__ ws,
                                                    const uint16_t *__restrict__ cand_idx,
                                                    const uint32_t *__restrict__ cand_cnt,
                                                    uint32_t *__restrict__ hist2, int s_hi, int s_lo)
{
    __shared__ uint32_t lh[kBins2];
    const int i = blockIdx.y;
    if (ws[i].done) return;
    const uint64_t prefix = ws[i].prefix;
    const uint32_t mask = (1u << (s_hi - s_lo)) - 1u;
    const float *erow = e + (int64_t)i * ge.ld;
    for (int b = threadIdx.x; b < kBins2; b += kThreads) lh[b] = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int t = blockIdx.x * 4 + wave; t < ge.n_tiles; t += gridDim.x * 4) {
        const uint32_t cnt = cand_cnt[(int64_t)i * ge.n_tiles + t];
        const uint16_t *seg = cand_idx + (((int64_t)i * ge.n_tiles + t) << 12);
        for (uint32_t q = lane; q < cnt; q += kWave) {
            const uint32_t j = (uint32_t)t * kTile + seg[q];
            const uint64_t comp = composite(erow[j], j, ge.idx_bits);
            if ((comp >> s_hi) == prefix) atomicAdd(&lh[(uint32_t)(comp >> s_lo) & mask], 1u);
        }
    }
    __syncthreads();
    for (int b = threadIdx.x; b < kBins2; b += kThreads) {
        const uint32_t c = lh[b];
        if (c) atomicAdd(&hist2[(int64_t)i * kBins2 + b], c);
    }
}

__global__ __launch_bounds__(kThreads) void tk_find(TkGeom ge, TkWorker *__restrict__ ws,
                                                    uint32_t *__restrict__ hist2, int s_hi, int s_lo)
{
    __shared__ uint32_t lh[kBins2];
    __shared__ uint32_t part[kThreads];
    const int i = blockIdx.x;
    if (ws[i].done) return;
    uint32_t *row = hist2 + (int64_t)i * kBins2;
    for (int b = threadIdx.x; b < kBins2; b += kThreads) {
        lh[b] = row[b];
        row[b] = 0;
    }
    __syncthreads();
    const uint32_t rank = ws[i].rank;
    uint32_t bin, above, count;
    if (find_rank_bin(lh, part, kBins2, rank, bin, above, count)) {
        TkWorker w = ws[i];
        w.prefix = (w.prefix << (s_hi - s_lo)) | bin;
        w.rank = rank - above;
        if (s_lo == 0 || count == w.rank) {   // last digit, or everything under this prefix is kept
            w.done = 1;
            w.tc = w.prefix << s_lo;
        }
        ws[i] = w;
    }
}

// ---------------------------------------------------------------------------------------------
constexpr int kFinChunk = 2048;   // candidates staged in LDS at a time
constexpr int kFinGroup = 32;     // workers whose candidate lists are flattened together

__global__ __launch_bounds__(kThreads) void tk_final(float *__restrict__ e, TkGeom ge,
                                                     const TkWorker *__restrict__ ws,
                                                     uint16_t *__restrict__ cand_idx, float *__restrict__ cand_val,
                                                     const uint32_t *__restrict__ cand_cnt,
                                                     uint32_t *__restrict__ sel_cnt, float *__restrict__ theta,
                                                     float *__restrict__ m, float *__restrict__ v,
                                                     float *__restrict__ vhat, AmsParams p)
{
    __shared__ float acc[kTile];
    __shared__ float lst_v[kFinChunk];
    __shared__ uint16_t lst_l[kFinChunk];
    __shared__ uint16_t lst_w[kFinChunk];   // worker within the group, bit 15 = kept
    __shared__ uint32_t pre[kFinGroup + 1];
    __shared__ uint32_t selc[kFinGroup];
    __shared__ uint64_t tcs[kFinGroup];

    const int t = blockIdx.x;
    const int64_t base = (int64_t)t * kTile;
    const int tid = threadIdx.x;

    // state loads first: independent of the selection
    float4 th[4], mm[4], vv[4], vh[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int64_t j = base + 4 * (tid + kThreads * r);
        th[r] = ld4(theta + j);
        mm[r] = ld4(m + j);
        vv[r] = ld4(v + j);
        vh[r] = ld4(vhat + j);
    }
    for (int l = tid; l < kTile; l += kThreads) acc[l] = 0.f;

    for (int w0 = 0; w0 < ge.n; w0 += kFinGroup) {
        const int nw = min(kFinGroup, ge.n - w0);
        __syncthreads();
        if (tid < nw) {
            pre[tid + 1] = cand_cnt[(int64_t)(w0 + tid) * ge.n_tiles + t];
            selc[tid] = 0;
            tcs[tid] = ws[w0 + tid].tc;
        }
        __syncthreads();
        if (tid == 0) {
            pre[0] = 0;
            for (int w = 0; w < nw; ++w) pre[w + 1] += pre[w];
        }
        __syncthreads();
        const uint32_t total = pre[nw];

        for (uint32_t c0 = 0; c0 < total; c0 += kFinChunk) {
            const uint32_t cn = min((uint32_t)kFinChunk, total - c0);
            // 1. read the candidates of this chunk, decide which are kept
            for (uint32_t q = tid; q < cn; q += kThreads) {
                const uint32_t gq = c0 + q;
                int lo = 0, hi = nw;                       // largest w with pre[w] <= gq
                while (hi - lo > 1) {
                    const int mid = (lo + hi) >> 1;
                    if (pre[mid] <= gq) lo = mid; else hi = mid;
                }
                const int w = lo;
                const int i = w0 + w;
                const int64_t seg = ((int64_t)i * ge.n_tiles + t) << 12;
                const uint32_t l = cand_idx[seg + (gq - pre[w])];
                const uint32_t j = (uint32_t)base + l;
                const float x = e[(int64_t)i * ge.ld + j];
                const bool keep = composite(x, j, ge.idx_bits) >= tcs[w];
                lst_l[q] = (uint16_t)l;
                lst_v[q] = x;
                lst_w[q] = (uint16_t)(w | (keep ? 0x8000 : 0));
            }
            __syncthreads();
            // 2. add kept values into the tile, one worker at a time, ascending
            int wa = 0, wb = nw - 1;
            while (pre[wa + 1] <= c0) ++wa;
            while (pre[wb] >= c0 + cn) --wb;
            for (int w = wa; w <= wb; ++w) {
                const uint16_t tag = (uint16_t)(w | 0x8000);
                for (uint32_t q = tid; q < cn; q += kThreads)
                    if (lst_w[q] == tag) acc[lst_l[q]] = fadd(acc[lst_l[q]], lst_v[q]);
                __syncthreads();
            }
            // 3. e = x - C(x) = +0 at kept coordinates; record (position, value) of the kept ones
            //    over the front of the candidate segment (slots already consumed)
            for (uint32_t q = tid; q < cn; q += kThreads) {
                const uint16_t wt = lst_w[q];
                if (wt & 0x8000) {
                    const int w = wt & 0x7fff;
                    const int i = w0 + w;
                    const uint32_t l = lst_l[q];
                    e[(int64_t)i * ge.ld + base + l] = 0.f;
                    const uint32_t slot = atomicAdd(&selc[w], 1u);
                    const int64_t seg = ((int64_t)i * ge.n_tiles + t) << 12;
                    cand_idx[seg + slot] = (uint16_t)l;
                    cand_val[seg + slot] = lst_v[q];
                }
            }
            __syncthreads();
        }
        if (tid < nw) sel_cnt[(int64_t)(w0 + tid) * ge.n_tiles + t] = selc[tid];
    }
    __syncthreads();

#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int l = 4 * (tid + kThreads * r);
        const int64_t j = base + l;
        const float4 gbar = make_float4(fdiv(acc[l], p.n_workers), fdiv(acc[l + 1], p.n_workers),
                                        fdiv(acc[l + 2], p.n_workers), fdiv(acc[l + 3], p.n_workers));
        amsgrad_update4(th[r], mm[r], vv[r], vh[r], gbar, p);
        st4(theta + j, th[r]);
        st4(m + j, mm[r]);
        st4(v + j, vv[r]);
        st4(vhat + j, vh[r]);
    }
}

// Copies the kept (index, value) pairs of one worker out of the per-tile records into dense
// arrays; `offs` is the exclusive prefix sum of the worker's per-tile counts.  One wavefront per tile.
__global__ __launch_bounds__(kWave) void tk_gather_selected(TkGeom ge, int worker,
                                                            const uint16_t *__restrict__ cand_idx,
                                                            const float *__restrict__ cand_val,
                                                            const uint32_t *__restrict__ sel_cnt,
                                                            const uint32_t *__restrict__ offs,
                                                            uint32_t *__restrict__ out_idx,
                                                            float *__restrict__ out_val)
{
    const int t = blockIdx.x;
    const uint32_t cnt = sel_cnt[(int64_t)worker * ge.n_tiles + t];
    const int64_t seg = ((int64_t)worker * ge.n_tiles + t) << 12;
    const uint32_t o = offs[t];
    for (uint32_t q = threadIdx.x; q < cnt; q += kWave) {
        if (o + q < ge.k) {
            out_idx[o + q] = (uint32_t)t * kTile + cand_idx[seg + q];
            out_val[o + q] = cand_val[seg + q];
        }
    }
}

}  // namespace cams
