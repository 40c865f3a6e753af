// Top-k compression (Appendix A, "Top-k") with error feedback (Section 4), server average and
// AMSGrad update (Section 3).
//
// Selection is an exact radix select, not a sort.  Every element gets the composite key
//     comp = (magnitude_bits << IB) | (2^IB - 1 - index),     magnitude_bits = bits(x) & 0x7fffffff,
// IB = number of bits of d-1.  comp is unique per element and its descending order is
// "larger magnitude first, lower index first among equals", so Top-k is { comp >= Tc } where Tc is
// the k-th largest comp.  Tc is found digit by digit from the top (11 bits, then 12 at a time).
//
// The error memory is kept in deferred form: after a step the library stores x_i = g_i + e_i and
// the worker's threshold Tc_i; e_i[j] = (comp(x_i[j], j) >= Tc_i) ? +0 : x_i[j] is formed on the fly
// when the next step (or a getter) reads x_i, so kept coordinates are never zeroed by scattered
// writes and one step needs a single pass over g and the stored vector.  Five launches per step,
// ordered only by kernel boundaries (no fences, no waiting inside a kernel):
//
//   tk_pass1    streams g and the stored x once and writes the new x; counts every element in a
//               per-worker histogram of its top 11 magnitude bits ("coarse" bin, an eighth of an
//               octave) and, for the two coarse bins around the worker's guess, of its top 17 bits
//               ("fine" bin, 0.2 % wide); lists "candidates" - elements whose fine bin is >= the
//               guess, which is carried over from the previous step's threshold minus a little
//               slack - as (index, value) pairs in one dense list per (worker, workgroup,
//               wavefront), with a directory entry (offset, count) per (worker, tile, wavefront)
//   tk_pick     one workgroup per worker: the coarse (and if covered, fine) bin of the k-th
//               largest, from the histograms
//   tk_compact  if the guess was above that bin (always on the first step) the worker's
//               candidates are listed again from the stored x; candidates in that bin are
//               copied, as comp values, to one dense list per worker
//   tk_resolve  one workgroup per worker: the remaining digits of Tc over the dense list, and
//               the guess for the next step
//   tk_final    per tile, all workers: candidates with comp >= Tc are the kept coordinates; their
//               values are added into an LDS copy of the tile in ascending worker order; then
//               gbar = acc / n and the AMSGrad update of the tile's theta, m, v, vhat
//
// Traffic per (worker, coordinate): 4 B g + 4 B stored x read + 4 B x written, plus the candidates
// (a few per cent of the elements, 8 B each, written once and read twice).
#pragma once
#include "device_utils.h"

namespace cams {

constexpr int kBins1 = 2048;      // coarse bin: top 11 of the 31 magnitude bits
constexpr int kShift1 = 20;
constexpr int kFineShift = 14;    // fine bin: top 17 bits; 64 fine bins per coarse bin
constexpr int kFinePerCoarse = 1 << (kShift1 - kFineShift);
constexpr int kFineWindow = 2 * kFinePerCoarse;   // fine bins counted: the guess's coarse bin and the next
constexpr int kDigitBits = 12;    // digits of the dense-list search
constexpr int kBins2 = 1 << kDigitBits;
constexpr int kSub = kTile / 4;   // coordinates of a tile that one wavefront handles
constexpr int kResolveThreads = 1024;
constexpr uint32_t kNoGuess = 1u << 17;      // fine-bin guess that lists nothing (before the first step)
constexpr uint64_t kNoThreshold = ~0ull;     // Tc that keeps nothing (no pending selection)
constexpr uint32_t kMinSlack = 8, kMaxSlack = 512, kFirstSlack = 8;   // in fine bins (0.2 % each)

struct TkWorker {
    uint64_t tc;            // threshold composite of the last finished step (pending selection)
    uint32_t guess;         // pass 1 lists elements with fine bin >= guess
    uint32_t slack;         // fine bins kept between the threshold and the next guess
    // leading digits of the running step's Tc, written by tk_compact, read by tk_resolve
    uint32_t prefix;        // magnitude bits above pshift
    uint32_t pshift;        // kShift1 (coarse bin known) or kFineShift (fine bin known)
    uint32_t rank;          // 1-based rank (from the top) of the k-th largest among elements with this prefix
    uint32_t whole;         // all elements with this prefix are kept: Tc needs no further digit
    uint32_t relisted;      // the guess was above the threshold: candidates were listed again
    uint32_t pad;
};

struct TkGeom {
    int64_t d, ld;
    int32_t n, n_tiles;
    int32_t idx_bits;       // IB
    uint32_t k;
    int32_t wgs;            // workgroups per worker in tk_pass1 / tk_compact; tile t belongs to t % wgs
    int32_t list_cap;       // capacity of one candidate list = ceil(n_tiles / wgs) * kSub
};

__device__ __forceinline__ uint64_t composite(float x, uint32_t j, int idx_bits)
{
    const uint64_t inv = ((1ull << idx_bits) - 1ull) - (uint64_t)j;
    return ((uint64_t)mag_key(x) << idx_bits) | inv;
}

// Finds, in a histogram held in LDS (`bins` counters, a multiple of the workgroup size), the bin
// of the element of 1-based rank `rank` counted from the top bin downwards, and leaves
// {bin, elements in higher bins, the bin's count} in res[0..2] for every thread (res[3] = 1 if
// found, which needs 1 <= rank <= total).  `part` holds one LDS counter per wavefront.
__device__ __forceinline__ void find_rank_bin(const uint32_t *lh, uint32_t *part, uint32_t *res, int bins,
                                              uint32_t rank)
{
    const int nt = blockDim.x;
    const int per = bins / nt;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t mine = 0;
    for (int q = 0; q < per; ++q) mine += lh[threadIdx.x * per + q];
    uint32_t suffix = mine;                       // sum over lanes >= this one
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const uint32_t t = __shfl_down(suffix, off, kWave);
        if (lane + off < kWave) suffix += t;
    }
    if (lane == 0) part[wave] = suffix;
    if (threadIdx.x == 0) res[3] = 0;
    __syncthreads();
    uint32_t above = suffix - mine;
    for (int w = wave + 1; w < (nt >> 6); ++w) above += part[w];
    if (above < rank && above + mine >= rank) {
        for (int q = per - 1; q >= 0; --q) {
            const uint32_t c = lh[threadIdx.x * per + q];
            if (above + c >= rank) {
                res[0] = threadIdx.x * per + q;
                res[1] = above;
                res[2] = c;
                res[3] = 1;
                break;
            }
            above += c;
        }
    }
    __syncthreads();
}

// Appends this wavefront's flagged lanes to a list: returns the slot of the calling lane (valid
// where flag is set) and advances count (uniform over the wavefront).
__device__ __forceinline__ uint32_t wave_append(bool flag, uint32_t &count)
{
    const uint64_t mask = __ballot(flag);
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t slot = count + __popcll(mask & ((1ull << lane) - 1ull));
    count += __popcll(mask);
    return slot;
}

// ---------------------------------------------------------------------------------------------
// Pending selection of the previous step in 32-bit form: the coordinate j with magnitude bits
// `key` was kept iff  key > tkey  or  (key == tkey and j <= tj).
struct KeptTest {
    uint32_t tkey, tj;
};
__device__ __forceinline__ KeptTest kept_test(uint64_t tc, int idx_bits)
{
    const uint32_t imask = (uint32_t)((1ull << idx_bits) - 1ull);
    KeptTest k;
    k.tkey = (uint32_t)(tc >> idx_bits);            // kNoThreshold gives 0xffffffff: above every key
    k.tj = imask - ((uint32_t)tc & imask);
    return k;
}
__device__ __forceinline__ bool was_kept(const KeptTest &k, uint32_t key, uint32_t j)
{
    return key >= k.tkey && (key > k.tkey || j <= k.tj);
}

// One tile of tk_pass1 for one workgroup.  kFull: the whole tile lies below d.
template <bool kFull>
__device__ __forceinline__ void pass1_tile(const float *__restrict__ grow, float *__restrict__ xrow, uint32_t base,
                                           uint32_t d, const KeptTest &kt, uint32_t guess, uint32_t wbase,
                                           uint32_t *lh, uint32_t *lf, uint2 *__restrict__ list, uint32_t &count)
{
    const int tid = threadIdx.x;
    float4 gv[4], xv[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const uint32_t j = base + 4 * (tid + kThreads * r);
        gv[r] = load_grad4(grow, j, d);
        xv[r] = ld4(xrow + j);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const uint32_t j = base + 4 * (tid + kThreads * r);
        const float gg[4] = {gv[r].x, gv[r].y, gv[r].z, gv[r].w};
        const float xo[4] = {xv[r].x, xv[r].y, xv[r].z, xv[r].w};
        float x[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            // e = x_old - C(x_old): +0 where the previous step kept the coordinate
            const float e = was_kept(kt, mag_key(xo[c]), j + c) ? 0.f : xo[c];
            x[c] = (kFull || j + c < d) ? fadd(gg[c], e) : 0.f;
        }
        st4(xrow + j, make_float4(x[0], x[1], x[2], x[3]));
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const bool valid = kFull || j + c < d;
            const uint32_t fine = mag_key(x[c]) >> kFineShift;
            if (valid) {
                atomicAdd(&lh[fine >> (kShift1 - kFineShift)], 1u);
                if (fine - wbase < (uint32_t)kFineWindow) atomicAdd(&lf[fine - wbase], 1u);
            }
            const bool hit = valid && fine >= guess;
            const uint32_t slot = wave_append(hit, count);   // < list_cap: kSub coordinates per tile
            if (hit) list[slot] = make_uint2(j + c, __float_as_uint(x[c]));
        }
    }
}

__global__ __launch_bounds__(kThreads) void tk_pass1(const float *__restrict__ g, float *__restrict__ xs, TkGeom ge,
                                                     const TkWorker *__restrict__ ws,
                                                     uint32_t *__restrict__ hist1,
                                                     uint32_t *__restrict__ histf, uint2 *__restrict__ cand,
                                                     uint2 *__restrict__ cand_dir,
                                                     uint32_t *__restrict__ list_len)
{
    __shared__ uint32_t lh[kBins1];
    __shared__ uint32_t lf[kFineWindow];
    const int i = blockIdx.y;
    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const uint32_t guess = ws[i].guess;
    const uint32_t wbase = guess & ~(uint32_t)(kFinePerCoarse - 1);   // first fine bin of the guess's coarse bin
    const KeptTest kt = kept_test(ws[i].tc, ge.idx_bits);
    const uint32_t d = (uint32_t)ge.d;
    const float *grow = g + (int64_t)i * ge.d;
    float *xrow = xs + (int64_t)i * ge.ld;
    const int64_t list_id = ((int64_t)i * ge.wgs + blockIdx.x) * 4 + wave;
    uint2 *list = cand + list_id * ge.list_cap;
    for (int b = tid; b < kBins1; b += kThreads) lh[b] = 0;
    if (tid < kFineWindow) lf[tid] = 0;
    __syncthreads();

    uint32_t count = 0;   // length of this wavefront's list so far
    for (int t = blockIdx.x; t < ge.n_tiles; t += ge.wgs) {
        const uint32_t base = (uint32_t)t * kTile;
        const uint32_t first = count;
        if (base + kTile <= d)
            pass1_tile<true>(grow, xrow, base, d, kt, guess, wbase, lh, lf, list, count);
        else
            pass1_tile<false>(grow, xrow, base, d, kt, guess, wbase, lh, lf, list, count);
        if ((tid & 63) == 0) cand_dir[((int64_t)i * ge.n_tiles + t) * 4 + wave] = make_uint2(first, count - first);
    }
    if ((tid & 63) == 0) list_len[list_id] = count;
    __syncthreads();
    uint32_t *row = hist1 + (int64_t)i * kBins1;
    for (int b = tid; b < kBins1; b += kThreads) {
        const uint32_t c = lh[b];
        if (c) atomicAdd(row + b, c);
    }
    if (tid < kFineWindow && lf[tid]) atomicAdd(histf + (int64_t)i * kFineWindow + tid, lf[tid]);
}

// ---------------------------------------------------------------------------------------------
// One workgroup per worker: the leading digits of Tc from the histograms of tk_pass1.
__global__ __launch_bounds__(kThreads) void tk_pick(TkGeom ge, TkWorker *__restrict__ ws,
                                                    const uint32_t *__restrict__ hist1,
                                                    const uint32_t *__restrict__ histf)
{
    __shared__ uint32_t lh[kBins1];
    __shared__ uint32_t part[kThreads / kWave];
    __shared__ uint32_t res[4];
    __shared__ uint32_t fres[3];
    const int i = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const uint32_t *row = hist1 + (int64_t)i * kBins1;
    for (int b = tid; b < kBins1; b += kThreads) lh[b] = row[b];
    __syncthreads();
    find_rank_bin(lh, part, res, kBins1, ge.k);
    if (!res[3]) return;                            // cannot happen: the histogram holds d >= k elements
    const uint32_t guess = ws[i].guess;
    uint32_t prefix = res[0];                       // coarse bin of the k-th largest
    uint32_t pshift = kShift1;
    uint32_t rank = ge.k - res[1];
    uint32_t count = res[2];
    const uint32_t wb = guess >> (kShift1 - kFineShift);      // first coarse bin of the fine window
    if (prefix - wb < 2u) {
        // the fine histogram covers this coarse bin: pick the fine bin as well (one wavefront)
        if (wave == 0) {
            const uint32_t c = histf[(int64_t)i * kFineWindow + (prefix - wb) * kFinePerCoarse + lane];
            uint32_t suffix = c;                    // elements of this coarse bin in fine bins >= lane
#pragma unroll
            for (int off = 1; off < kWave; off <<= 1) {
                const uint32_t t = __shfl_down(suffix, off, kWave);
                if (lane + off < kWave) suffix += t;
            }
            const uint64_t reach = __ballot(suffix >= rank);  // lane 0 always reaches: suffix(0) = count >= rank
            const int top = reach ? 63 - __builtin_clzll(reach) : 0;
            if (lane == top) {
                fres[0] = (uint32_t)lane;
                fres[1] = suffix - c;
                fres[2] = c;
            }
        }
        __syncthreads();
        prefix = (prefix << (kShift1 - kFineShift)) | fres[0];
        pshift = kFineShift;
        rank -= fres[1];
        count = fres[2];
    }
    if (tid == 0) {
        ws[i].prefix = prefix;
        ws[i].pshift = pshift;
        ws[i].rank = rank;
        ws[i].whole = (count == rank) ? 1u : 0u;
        // candidates are complete iff every element at or above the prefix was listed
        ws[i].relisted = (((uint64_t)guess << kFineShift) > ((uint64_t)prefix << pshift)) ? 1u : 0u;
    }
}

// Lists the worker's candidates again if the guess was too high, and copies the candidates that
// carry the prefix, as comp values, to the "dense" region of their list (same shape as the
// candidate lists; typically a handful per list).  No atomics: tk_resolve walks the regions.
__global__ __launch_bounds__(kThreads) void tk_compact(const float *__restrict__ xs, TkGeom ge,
                                                       const TkWorker *__restrict__ ws,
                                                       uint2 *__restrict__ cand, uint2 *__restrict__ cand_dir,
                                                       uint32_t *__restrict__ list_len,
                                                       uint64_t *__restrict__ dense, uint32_t *__restrict__ dense_len)
{
    const int i = blockIdx.y;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const uint32_t prefix = ws[i].prefix, pshift = ws[i].pshift;
    const bool whole = ws[i].whole != 0, relist = ws[i].relisted != 0;
    if (whole && !relist) return;

    const int64_t list_id = ((int64_t)i * ge.wgs + blockIdx.x) * 4 + wave;
    uint2 *list = cand + list_id * ge.list_cap;
    uint64_t *out = dense + list_id * ge.list_cap;
    uint32_t kept = 0;   // entries of this wavefront's dense region
    if (relist) {
        // list this workgroup's candidates again, now from the prefix up; those with the prefix
        // itself go to the dense region on the way
        const float *xrow = xs + (int64_t)i * ge.ld;
        uint32_t filled = 0;
        for (int t = blockIdx.x; t < ge.n_tiles; t += ge.wgs) {
            const int64_t base = (int64_t)t * kTile;
            const uint32_t first = filled;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const uint32_t j = (uint32_t)base + 4 * (tid + kThreads * r);
                const float4 xv = ld4(xrow + j);
                const float x[4] = {xv.x, xv.y, xv.z, xv.w};
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const uint32_t top = mag_key(x[c]) >> pshift;
                    const bool hit = j + c < ge.d && top >= prefix;
                    const uint32_t slot = wave_append(hit, filled);
                    if (hit) list[slot] = make_uint2(j + c, __float_as_uint(x[c]));
                    const bool eq = hit && top == prefix && !whole;
                    const uint32_t at = wave_append(eq, kept);
                    if (eq) out[at] = composite(x[c], j + c, ge.idx_bits);
                }
            }
            if (lane == 0) cand_dir[((int64_t)i * ge.n_tiles + t) * 4 + wave] = make_uint2(first, filled - first);
        }
        if (lane == 0) list_len[list_id] = filled;
    } else {
        const uint32_t len = list_len[list_id];
        for (uint32_t q0 = 0; q0 < len; q0 += kWave) {
            const uint32_t q = q0 + lane;
            bool eq = false;
            uint2 c = make_uint2(0u, 0u);
            if (q < len) {
                c = list[q];
                eq = ((c.y & 0x7fffffffu) >> pshift) == prefix;
            }
            const uint32_t at = wave_append(eq, kept);
            if (eq) out[at] = composite(__uint_as_float(c.y), c.x, ge.idx_bits);
        }
    }
    if (lane == 0) dense_len[list_id] = kept;
}

// ---------------------------------------------------------------------------------------------
// One workgroup of 1024 threads per worker: the digits of Tc below the prefix, over the worker's
// dense regions.  Also hands the next step its guess and clears the histogram rows.
__global__ __launch_bounds__(kResolveThreads) void tk_resolve(TkGeom ge, TkWorker *__restrict__ ws,
                                                              uint32_t *__restrict__ hist1,
                                                              uint32_t *__restrict__ histf,
                                                              const uint64_t *__restrict__ dense,
                                                              const uint32_t *__restrict__ dense_len)
{
    __shared__ uint32_t lh[kBins2];
    __shared__ uint32_t pre[kResolveThreads + 1];   // exclusive prefix of the region lengths of a chunk of lists
    __shared__ uint32_t part[kResolveThreads / kWave];
    __shared__ uint32_t res[4];
    const int i = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const TkWorker w = ws[i];
    uint64_t prefix = w.prefix;
    uint32_t rank = w.rank;
    int s_hi = (int)w.pshift + ge.idx_bits;
    bool done = w.whole != 0;
    uint64_t tc = prefix << s_hi;
    const int n_lists = ge.wgs * 4;
    const int64_t list0 = (int64_t)i * n_lists;

    while (!done) {
        const int s_lo = max(s_hi - kDigitBits, 0);
        const uint32_t mask = (1u << (s_hi - s_lo)) - 1u;
        for (int b = tid; b < kBins2; b += kResolveThreads) lh[b] = 0;
        for (int c0 = 0; c0 < n_lists; c0 += kResolveThreads) {
            // lengths of up to 1024 regions -> exclusive prefix sums in LDS
            const uint32_t len = (c0 + tid < n_lists) ? dense_len[list0 + c0 + tid] : 0u;
            uint32_t incl = len;
#pragma unroll
            for (int off = 1; off < kWave; off <<= 1) {
                const uint32_t up = __shfl_up(incl, off, kWave);
                if (lane >= off) incl += up;
            }
            __syncthreads();                       // previous chunk's readers of pre/part are done
            if (lane == kWave - 1) part[wave] = incl;
            __syncthreads();
            uint32_t before = 0;
            for (int v = 0; v < wave; ++v) before += part[v];
            pre[tid] = before + incl - len;
            if (tid == kResolveThreads - 1) pre[kResolveThreads] = before + incl;
            __syncthreads();
            const uint32_t total = pre[kResolveThreads];
            for (uint32_t q = tid; q < total; q += kResolveThreads) {
                int lo = 0, hi = kResolveThreads;              // largest l with pre[l] <= q
                while (hi - lo > 1) {
                    const int mid = (lo + hi) >> 1;
                    if (pre[mid] <= q) lo = mid; else hi = mid;
                }
                const uint64_t comp = dense[(list0 + c0 + lo) * ge.list_cap + (q - pre[lo])];
                if ((comp >> s_hi) == prefix) atomicAdd(&lh[(uint32_t)(comp >> s_lo) & mask], 1u);
            }
        }
        __syncthreads();
        find_rank_bin(lh, part, res, kBins2, rank);
        if (!res[3]) break;                                    // cannot happen: rank <= matching elements
        prefix = (prefix << (s_hi - s_lo)) | res[0];
        rank -= res[1];
        if (s_lo == 0 || res[2] == rank) {                     // last digit, or all under this prefix are kept
            done = true;
            tc = prefix << s_lo;
        }
        s_hi = s_lo;
        __syncthreads();
    }
    if (tid == 0) {
        ws[i].tc = tc;
        // next step lists from a few fine bins below this threshold; more after a miss
        const uint32_t slack = w.relisted ? min(w.slack * 2u, kMaxSlack) : max(w.slack - 1u, kMinSlack);
        const uint32_t fine = (uint32_t)(tc >> ge.idx_bits) >> kFineShift;
        ws[i].slack = slack;
        ws[i].guess = fine > slack ? fine - slack : 0u;
    }
    uint32_t *row = hist1 + (int64_t)i * kBins1;
    for (int b = tid; b < kBins1; b += kResolveThreads) row[b] = 0;
    if (tid < kFineWindow) histf[(int64_t)i * kFineWindow + tid] = 0;
}

// ---------------------------------------------------------------------------------------------
constexpr int kFinChunk = 1024;   // candidates staged in LDS at a time
constexpr int kFinGroup = 32;     // workers whose candidate lists are flattened together

__global__ __launch_bounds__(kThreads) void tk_final(TkGeom ge, const TkWorker *__restrict__ ws,
                                                     const uint2 *__restrict__ cand,
                                                     const uint2 *__restrict__ cand_dir,
                                                     float *__restrict__ theta, float *__restrict__ m,
                                                     float *__restrict__ v, float *__restrict__ vhat, AmsParams p)
{
    __shared__ float acc[kTile];
    __shared__ float lst_v[kFinChunk];
    __shared__ uint16_t lst_l[kFinChunk];
    __shared__ uint16_t lst_w[kFinChunk];   // worker within the group, bit 15 = kept
    __shared__ uint32_t pre[kFinGroup * 4 + 1];
    __shared__ uint32_t first[kFinGroup * 4];   // offset of each sub-list inside its wavefront's list
    __shared__ uint64_t tcs[kFinGroup];

    const int t = blockIdx.x;
    const int64_t base = (int64_t)t * kTile;
    const int tid = threadIdx.x;

    for (int l = tid; l < kTile; l += kThreads) acc[l] = 0.f;

    for (int w0 = 0; w0 < ge.n; w0 += kFinGroup) {
        const int nw = min(kFinGroup, ge.n - w0);
        const int ns = nw * 4;                      // (worker, wavefront) sub-lists in this group
        __syncthreads();
        if (tid < ns) {
            const uint2 dir = cand_dir[((int64_t)(w0 + (tid >> 2)) * ge.n_tiles + t) * 4 + (tid & 3)];
            first[tid] = dir.x;
            pre[tid + 1] = dir.y;
        }
        if (tid < nw) tcs[tid] = ws[w0 + tid].tc;
        __syncthreads();
        if (tid < kWave) {
            // inclusive prefix sum of the (at most 128) sub-list lengths, two per lane
            const uint32_t a = (2 * tid < ns) ? pre[2 * tid + 1] : 0u;
            const uint32_t b = (2 * tid + 1 < ns) ? pre[2 * tid + 2] : 0u;
            uint32_t incl = a + b;
#pragma unroll
            for (int off = 1; off < kWave; off <<= 1) {
                const uint32_t up = __shfl_up(incl, off, kWave);
                if (tid >= off) incl += up;
            }
            const uint32_t excl = incl - (a + b);
            if (2 * tid < ns) pre[2 * tid + 1] = excl + a;
            if (2 * tid + 1 < ns) pre[2 * tid + 2] = excl + a + b;
            if (tid == 0) pre[0] = 0;
        }
        __syncthreads();
        const uint32_t total = pre[ns];

        for (uint32_t c0 = 0; c0 < total; c0 += kFinChunk) {
            const uint32_t cn = min((uint32_t)kFinChunk, total - c0);
            // 1. read the candidates of this chunk, decide which are kept
            for (uint32_t q = tid; q < cn; q += kThreads) {
                const uint32_t gq = c0 + q;
                int lo = 0, hi = ns;                       // largest s with pre[s] <= gq
                while (hi - lo > 1) {
                    const int mid = (lo + hi) >> 1;
                    if (pre[mid] <= gq) lo = mid; else hi = mid;
                }
                const int w = lo >> 2;
                const int64_t list_id = ((int64_t)(w0 + w) * ge.wgs + (t % ge.wgs)) * 4 + (lo & 3);
                const uint2 c = cand[list_id * ge.list_cap + first[lo] + (gq - pre[lo])];
                const uint32_t l = c.x - (uint32_t)base;
                const float x = __uint_as_float(c.y);
                const bool keep = composite(x, c.x, ge.idx_bits) >= tcs[w];
                lst_l[q] = (uint16_t)l;
                lst_v[q] = x;
                lst_w[q] = (uint16_t)(w | (keep ? 0x8000 : 0));
            }
            __syncthreads();
            // 2. add kept values into the tile, one worker at a time, ascending
            int sa = 0, sb = ns - 1;
            while (pre[sa + 1] <= c0) ++sa;
            while (pre[sb] >= c0 + cn) --sb;
            for (int w = sa >> 2; w <= (sb >> 2); ++w) {
                const uint16_t tag = (uint16_t)(w | 0x8000);
                for (uint32_t q = tid; q < cn; q += kThreads)
                    if (lst_w[q] == tag) acc[lst_l[q]] = fadd(acc[lst_l[q]], lst_v[q]);
                __syncthreads();
            }
        }
    }
    __syncthreads();

    // the state is loaded only now: fewer live registers above, and the other workgroups resident
    // on the compute unit cover this latency
    float4 th[4], mm[4], vv[4], vh[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int64_t j = base + 4 * (tid + kThreads * r);
        th[r] = ld4(theta + j);
        mm[r] = ld4(m + j);
        vv[r] = ld4(v + j);
        vh[r] = ld4(vhat + j);
    }
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

// Getter support -------------------------------------------------------------------------------

// e_i of one worker in its defined form, from the stored x and the pending threshold.
__global__ __launch_bounds__(kThreads) void tk_materialize_error(const float *__restrict__ xrow, TkGeom ge,
                                                                 const TkWorker *__restrict__ w,
                                                                 float *__restrict__ out)
{
    const int64_t j = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (j >= ge.d) return;
    const float x = xrow[j];
    out[j] = was_kept(kept_test(w->tc, ge.idx_bits), mag_key(x), (uint32_t)j) ? 0.f : x;
}

// The kept (index, value) pairs of one worker, in no particular order: candidates with
// comp >= Tc.  *count must be 0 on entry and ends at k.  One wavefront per candidate list.
__global__ __launch_bounds__(kThreads) void tk_gather_selected(TkGeom ge, int worker,
                                                               const TkWorker *__restrict__ ws,
                                                               const uint2 *__restrict__ cand,
                                                               const uint32_t *__restrict__ list_len,
                                                               uint32_t *__restrict__ count,
                                                               uint32_t *__restrict__ out_idx,
                                                               float *__restrict__ out_val)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t tc = ws[worker].tc;
    const int64_t list_id = ((int64_t)worker * ge.wgs + blockIdx.x) * 4 + wave;
    const uint32_t len = list_len[list_id];
    for (uint32_t q = lane; q < len; q += kWave) {
        const uint2 c = cand[list_id * ge.list_cap + q];
        if (composite(__uint_as_float(c.y), c.x, ge.idx_bits) >= tc) {
            const uint32_t slot = atomicAdd(count, 1u);
            if (slot < ge.k) {
                out_idx[slot] = c.x;
                out_val[slot] = __uint_as_float(c.y);
            }
        }
    }
}

}  // namespace cams
