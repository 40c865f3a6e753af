// Top-k compression (Appendix A, "Top-k") with error feedback (Section 4), server average and
// AMSGrad update (Section 3).
//
// Selection is an exact radix select, not a sort.  Every element gets the composite key
//     comp = (magnitude_bits << IB) | (2^IB - 1 - index),     magnitude_bits = bits(x) & 0x7fffffff,
// IB = number of bits of d-1.  comp is unique per element and its descending order is
// "larger magnitude first, lower index first among equals", so Top-k is { comp >= Tc } where Tc is
// the k-th largest comp.  Tc is found digit by digit from the top.
//
// The error memory is kept in deferred form: after a step the library stores x_i = g_i + e_i and
// the worker's threshold Tc_i; e_i[j] = (comp(x_i[j], j) >= Tc_i) ? +0 : x_i[j] is formed on the fly
// when the next step (or a getter) reads x_i, so kept coordinates are never zeroed by scattered
// writes and one step needs a single pass over g and the stored vector.  Six launches per step,
// ordered only by kernel boundaries (no fences, no waiting inside a kernel):
//
//   tk_pass1    one workgroup per (tile, worker): streams g and the stored x once and writes the new
//               x; lists "candidates" - elements whose fine magnitude bin (top 17 bits, 0.2 % wide)
//               is >= the worker's guess, which is the previous step's threshold minus a little
//               slack - as (index, value) pairs, staged in LDS (value and place in the tile, 6 bytes)
//               and appended densely to one of 64 regions of the worker (one atomic add per tile).
//               A workgroup per tile (instead of a loop over tiles) matters: on this chip a wave
//               that loops must wait for its stores before it can use its next loads.
//   tk_hist     histograms of the candidates: coarse bins (top 11 bits) and the fine bins of the
//               eight coarse bins from the guess's on; with fewer than k candidates (always on the first
//               step) the guess was too high: then the workgroups count the whole vector into a
//               full coarse histogram instead
//   tk_pick     coarse and fine bin of the k-th largest (one workgroup per worker); after such a
//               miss: the coarse bin from the full histogram, and the candidates are listed again
//               from the stored x (many workgroups)
//   tk_compact  candidates in the threshold bin are copied, as comp values, to dense pieces (one
//               per wavefront)
//   tk_resolve  one workgroup per worker: the remaining digits of Tc over those pieces, and the
//               guess for the next step
//   tk_final    per tile, all workers: candidates with comp >= Tc are the kept coordinates; their
//               values are added into an LDS copy of the tile in ascending worker order; then
//               gbar = acc / n and the AMSGrad update of the tile's theta, m, v, vhat
//
// Traffic per (worker, coordinate): 4 B g + 4 B stored x read + 4 B x written, plus the candidates
// (about 1.2 k per worker, 8 B each, written once, read three times).
//
// The candidate regions are bounded (see region_base): a region that fills up is detected, and the step then
// goes the way of a guess that was too high (whole-vector count, lists made anew) and, if the lists still do not
// fit, selects without lists inside tk_resolve (exact_select).  Vectors of at most 16 tiles take three launches: tk_pass1,
// tk_small_select, tk_final.
//
// Exact zeros under error feedback: when fewer than k coordinates are non-zero the k-th largest is a zero and
// zeros are selected by lower index.  They are never listed as candidates (millions of equal keys would be);
// tk_pass1 counts them per tile, and tk_resolve places the threshold among them from those counts
// (zero_tail_threshold).  The other methods list zeros like any other value.
//
// Rand-k (Appendix A, "Rand-k") runs through the same kernels: the 31 magnitude bits are replaced by a
// 31-bit pseudo-random score of (seed, step, worker, index), see SelKey; everything after the key -
// bins, digits, thresholds, the deferred error - is unchanged.
#pragma once
#include "device_utils.h"

namespace cams {

constexpr int kBins1 = 2048;      // coarse bin: top 11 of the 31 magnitude bits
constexpr int kShift1 = 20;
constexpr int kFineShift = 14;    // fine bin: top 17 bits; 64 fine bins per coarse bin
constexpr int kFinePerCoarse = 1 << (kShift1 - kFineShift);
constexpr int kWindowCoarse = 8;  // coarse bins whose fine bins are counted, from the guess's on: one octave of
                                  // magnitudes.  In the first steps of a run the threshold climbs by tens of fine
                                  // bins per step; beyond the window only the coarse bin is known and the threshold
                                  // bin holds 64 times the elements (with two coarse bins, n = 8, d = 110 M: steps
                                  // 1 to 6 spent 65-200 us in tk_resolve instead of 15)
constexpr int kFineWindow = kWindowCoarse * kFinePerCoarse;
constexpr int kDigitBits = 12;    // digits of the dense-array search
constexpr int kBins2 = 1 << kDigitBits;
constexpr int kFirstBits = 10;    // first digit below the prefix, counted by tk_compact while it copies: narrower,
                                  // since every one of its workgroups clears and flushes the bins
constexpr int kBinsFirst = 1 << kFirstBits;
constexpr int kPieceWords = kBinsFirst / 32;   // words of a dense piece's bitmap: which first digits occur in it
constexpr int kSub = kTile / 4;   // coordinates of a tile that one wavefront handles = capacity of its staged list
constexpr int kMinSlices = 64;    // candidate regions per vector: a power of two in [kMinSlices, kMaxSlices]
                                  // (fewer for a vector of fewer tiles than that)
constexpr int kMaxSlices = 512;
constexpr int kMaxParts = 8;      // pieces a region is cut into for tk_hist / tk_compact, at most
constexpr int kResolveThreads = 1024;
constexpr uint32_t kNoGuess = 1u << 17;      // fine-bin guess that lists nothing (before the first step)
constexpr uint64_t kNoThreshold = ~0ull;     // Tc that keeps nothing (no pending selection)
constexpr uint32_t kMinSlack = 8, kMaxSlack = 512, kFirstSlack = 8;   // in fine bins (0.2 % each)
constexpr uint32_t kZeroTail = 2;            // value of TkWorker::whole
constexpr uint32_t kExact = 3;               // value of TkWorker::whole: exact_select has found Tc and listed the kept set


struct TkWorker {
    uint64_t tc;            // threshold composite of the last finished step (pending selection)
    uint32_t guess;         // pass 1 lists elements with fine bin >= guess
    uint32_t slack;         // fine bins kept between the threshold and the next guess
    // leading digits of the running step's Tc, written by tk_pick, read by the kernels after it
    uint32_t prefix;        // magnitude bits above pshift
    uint32_t pshift;        // kFineShift or kShift1: how many low magnitude bits are still open
    uint32_t rank;          // 1-based rank (from the top) of the k-th largest among elements with this prefix
    uint32_t whole;         // 1: all elements with this prefix are kept, Tc needs no further digit; kZeroTail: all
                            // candidates are kept and `rank` zeros besides (see zero_tail_threshold)
    uint32_t relisted;      // the guess was above the threshold: candidates are listed again
    uint32_t last_fine;     // fine bin of the previous threshold (to see how far thresholds move)
    uint32_t step_word;     // Rand-k: TkRand::step_now of the step that left tc - the draw the deferred error memory
                            // must be read with.  Kept in device memory, not in a kernel argument, so that a step
                            // replayed from a HIP graph (which repeats its draw) still reads its predecessor's.
    uint32_t overflow;      // tk_pass1 found a candidate region full: the lists are incomplete, tk_hist counts the
                            // whole vector instead (as after a guess that was too high)
    uint32_t overflow2;     // listing anew, tk_pick found a region full as well: tk_resolve selects without lists
                            // (exact_select)
    uint32_t pad_;
};
static_assert(sizeof(TkWorker) == 56, "TkWorker is copied between host and device as plain bytes");

// Rand-k: what the score of a coordinate depends on besides its index and the vector's number.
struct TkRand {
    uint32_t on;          // 0: Top-k (keys are magnitudes)
    uint32_t seed_hi;     // upper half of the 64-bit seed
    uint32_t step_now;    // mix32(lower half of the seed + draw * 0x9e3779b9) for the running step's draw (the draw of
                          // the step whose selection is still pending is TkWorker::step_word)
    uint32_t who0;        // number of vector 0 of this geometry: 0 for the workers, n for CD-Adam's server
    uint32_t min_slack;   // Rand-k: least slack of the guess, in fine bins (0: kMinSlack).  The k-th largest score
                          // of a fresh draw scatters by sqrt(k (1 - k/d)) / d of the key range around (1 - k/d).
};

struct TkGeom {
    int64_t d, ld;
    int32_t n, n_tiles;
    int32_t idx_bits;       // IB
    uint32_t k;
    int32_t slices;         // candidate regions per vector (see region_base)
    int32_t slice_tiles;    // tiles that append to one candidate region = ceil(n_tiles / slices)
    uint32_t region_cap;    // entries a candidate region holds (see region_base)
    int32_t parts;          // tk_hist / tk_compact: workgroups per region
    int32_t relist_wgs;     // workgroups per worker in tk_pick (after a miss each loops over tiles; else all but one leave)
    int32_t stream_rows;    // the stored rows are too large to stay cached between steps: tk_pass1 loads them as a stream
    int32_t xcd_chunk;      // tk_pass1: tile_of_block's chunk
    TkRand rand;
};

// The 31-bit key that orders the coordinates of one vector: the magnitude bits (Top-k), or the score
//     mix32(mix32(j + a) ^ b) >> 1,   a = mix32(step ^ seed_hi ^ who * 0x85ebca6b),  b = mix32(a + 0xc2b2ae35)
// (Rand-k), mix32 being the 32-bit finaliser of MurmurHash3.  For a fixed vector and step the score is a
// bijection of the index followed by a shift, so at most two coordinates share it.
struct SelKey {
    uint32_t on, a, b;
};
__device__ __forceinline__ uint32_t mix32(uint32_t h)
{
    h ^= h >> 16;
    h *= 0x85ebca6bu;
    h ^= h >> 13;
    h *= 0xc2b2ae35u;
    h ^= h >> 16;
    return h;
}
__device__ __forceinline__ SelKey sel_key_of(const TkRand &r, uint32_t per_step, int vec)
{
    SelKey s;
    s.on = r.on;
    s.a = mix32(per_step ^ r.seed_hi ^ ((r.who0 + (uint32_t)vec) * 0x85ebca6bu));
    s.b = mix32(s.a + 0xc2b2ae35u);
    return s;
}
__device__ __forceinline__ uint32_t sel_key(const SelKey &s, float x, uint32_t j)
{
    return s.on ? mix32(mix32(j + s.a) ^ s.b) >> 1 : mag_key(x);
}

__device__ __forceinline__ uint64_t composite(uint32_t key, uint32_t j, int idx_bits)
{
    const uint64_t inv = ((1ull << idx_bits) - 1ull) - (uint64_t)j;
    return ((uint64_t)key << idx_bits) | inv;
}

// Pending selection of the previous step in 32-bit form: the coordinate j with key
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

// Exclusive prefix sum of one value per thread over a 256-thread workgroup, left in pre[0..256]
// (pre[256] = total).  `part` holds 4 LDS counters.  Three barriers.
__device__ __forceinline__ void block_prefix(uint32_t v, uint32_t *pre, uint32_t *part)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t incl = v;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const uint32_t up = __shfl_up(incl, off, kWave);
        if (lane >= off) incl += up;
    }
    __syncthreads();                       // readers of an earlier pre/part are done
    if (lane == kWave - 1) part[wave] = incl;
    __syncthreads();
    uint32_t before = 0;
    for (int w = 0; w < wave; ++w) before += part[w];
    pre[threadIdx.x] = before + incl - v;
    if (threadIdx.x == kThreads - 1) pre[kThreads] = before + incl;
    __syncthreads();
}

// ---------------------------------------------------------------------------------------------
// Where candidates live.  Each worker owns ge.slices regions of ge.region_cap entries in the candidate array,
// one after the other; tile t appends to region t mod slices, so workgroups that run at the same time
// (neighbouring tiles) use different cursors.  Atomic adds on one cursor serialise at about a microsecond
// each, so a kernel of T tiles per vector lasts at least T / slices microseconds: a single long vector
// (CD-Adam's server) takes more regions than each of many workers.  A tile takes its space with one atomic add
// on the region's cursor and records {offset from the worker's first region, counts of its four wavefronts,
// zeros} in the tile directory; inside the tile's space the candidates stand wavefront by wavefront.  The
// order of the tiles inside a region depends on timing; nothing downstream depends on it (comp values are
// unique, the selection is a set).  Appending densely matters: per-tile fixed slots made the same kernel
// 10 - 20 % slower (8-byte pieces scattered over gigabytes).
//
// A region holds a bounded number of entries (the host sizes a worker's regions for twice max(4 k, d / 64)
// candidates in all; 1.2 k are listed in steady state), not every coordinate of its tiles.  A tile that does not
// fit sets the worker's overflow flag and stores nothing: the worker's lists are then incomplete and the step
// goes on as after a guess that was too high - tk_hist counts the whole vector and tk_pick lists again with
// the coarse bin of the k-th largest; if that does not fit either (thousands of equal magnitudes: nothing
// narrower than the whole composite key separates them), tk_resolve selects without lists (exact_select).
__device__ __forceinline__ int64_t worker_base(const TkGeom &ge, int worker)
{
    return (int64_t)worker * ge.slices * ge.region_cap;
}
__device__ __forceinline__ int64_t region_base(const TkGeom &ge, int worker, int slice)
{
    return ((int64_t)worker * ge.slices + slice) * ge.region_cap;
}

// Takes `total` entries of region (i, t mod slices) for tile t and writes the tile's directory record; one
// thread calls this.  cnt: the candidates of the tile's four wavefronts (each below 2^16: a wavefront owns
// kSub = 1024 coordinates).  Returns the offset of the tile's space from the worker's first region, or
// kNoSpace when the region is full - the record then says that nothing is stored and *overflow_flag is set.
constexpr uint32_t kNoSpace = 0xffffffffu;
__device__ __forceinline__ uint32_t take_space(const uint32_t (&cnt)[4], uint32_t zeros, const TkGeom &ge, int i, int t,
                                               uint32_t *__restrict__ cursor, uint4 *__restrict__ tile_dir,
                                               uint32_t *overflow_flag)
{
    const uint32_t total = cnt[0] + cnt[1] + cnt[2] + cnt[3];
    const int slice = t & (ge.slices - 1);
    uint32_t at = 0;
    if (total) {
        at = atomicAdd(cursor + i * ge.slices + slice, total);
        if (at > ge.region_cap || total > ge.region_cap - at) {
            *overflow_flag = 1u;
            tile_dir[(int64_t)i * ge.n_tiles + t] = make_uint4(0u, 0u, 0u, zeros);
            return kNoSpace;
        }
    }
    at += (uint32_t)slice * ge.region_cap;
    tile_dir[(int64_t)i * ge.n_tiles + t] = make_uint4(at, cnt[0] | (cnt[1] << 16), cnt[2] | (cnt[3] << 16), zeros);
    return at;
}

// First half of moving a tile's staged candidates (count per wavefront, in LDS) to its region: the
// thread `allocator` takes the space.  sh: 9 LDS words.  zeros: the wavefront's count of exact zeros (the
// tile's sum goes into the directory record).  Ends before the barrier so that the caller can put other
// work between the atomic and its use.
__device__ __forceinline__ void flush_begin(uint32_t count, uint32_t zeros, uint32_t *sh, int allocator, const TkGeom &ge,
                                            int i, int t, uint32_t *__restrict__ cursor, uint4 *__restrict__ tile_dir,
                                            uint32_t *overflow_flag)
{
    const int tid = threadIdx.x;
    if ((tid & 63) == 0) {
        sh[tid >> 6] = count;
        sh[5 + (tid >> 6)] = zeros;
    }
    __syncthreads();
    if (tid == allocator) {
        const uint32_t cnt[4] = {sh[0], sh[1], sh[2], sh[3]};
        sh[4] = take_space(cnt, sh[5] + sh[6] + sh[7] + sh[8], ge, i, t, cursor, tile_dir, overflow_flag);
    }
}
__device__ __forceinline__ void flush_end(const uint2 *stage, uint32_t count, const uint32_t *sh, const TkGeom &ge,
                                          int i, uint2 *__restrict__ cand)
{
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t off = sh[4];
    if (off == kNoSpace) return;
    for (int w = 0; w < wave; ++w) off += sh[w];
    uint2 *dst = cand + worker_base(ge, i) + off;
    // the wavefront reads back its own LDS writes: no barrier needed for those
    for (uint32_t q = lane; q < count; q += kWave) dst[q] = stage[q];
}

// A wavefront's staged candidates in tk_pass1: the value and the coordinate's place inside the tile, 6 bytes per
// entry instead of the 8 of an (index, value) pair.  With room for every coordinate of the wavefront (so the list
// cannot overflow) a workgroup's four lists take 24 KB, and six workgroups fit a compute unit where 32 KB allowed
// four: the passes that only read (CD-Adam, naive compression) run 3-5 % faster with the additional loads in flight.
// (Staging the places alone and reading the values again when the list is copied out - possible where the vector is
// g itself, naive compression - was built: eight workgroups per unit, and slower, n = 16, d = 11.2 M 158 -> 202 us:
// the scattered re-reads cost more than the workgroups bring.)
struct Stage {
    float *val;          // [kSub]
    uint16_t *at;        // [kSub] index - first index of the tile
};

// Stages one element of the vector that is compressed as a candidate if its fine bin reaches the guess.
// base: first index of the tile.
// kSkipZeros (error feedback with magnitude keys): exact zeros are never listed but counted (zeros, uniform
// over the wavefront) - when fewer than k coordinates are non-zero the threshold lies among the zeros, which
// are ordered by index alone, and is placed from these counts instead (see zero_tail_threshold).
template <bool kSkipZeros>
__device__ __forceinline__ void consider(float x, uint32_t j, uint32_t base, bool valid, uint32_t guess, const SelKey &sk,
                                         const Stage &stage, uint32_t &count, uint32_t &zeros)
{
    bool hit = valid && (sel_key(sk, x, j) >> kFineShift) >= guess;
    if (kSkipZeros && !sk.on) {
        const bool zero = valid && mag_key(x) == 0u;
        zeros += (uint32_t)__popcll(__ballot(zero));
        hit = hit && !zero;
    }
    const uint32_t slot = wave_append(hit, count);
    if (hit) {
        stage.val[slot] = x;
        stage.at[slot] = (uint16_t)(j - base);
    }
}

// One tile of one worker.  kFull: the whole tile lies below d.  Candidates are staged in LDS (one
// list per wavefront, which owns kSub coordinates of the tile, so it cannot overflow).
// Modes: kPassEf  error feedback: x = g + e, written back over the stored vector;
//        kPassCd  CD-Adam worker (Algorithm 1, line 5): u = g - ghat_i, nothing written back (ghat_i
//                 changes only where c_i is not zero; tk_merge does that);
//        kPassDiff  CD-Adam server (line 9): w = ghat - gtilde, both padded rows, nothing written back;
//        kPassNaive  naive compression (Section 4): x = g, the stored rows are not touched.
enum { kPassEf = 0, kPassCd = 1, kPassDiff = 2, kPassNaive = 3 };

template <bool kFull, int kMode, typename G>
__device__ __forceinline__ uint32_t pass1_tile(const G *__restrict__ grow, float *__restrict__ xrow,
                                               uint32_t base, uint32_t d, const KeptTest &kt, uint32_t guess,
                                               const SelKey &sk, const SelKey &sk_prev, const Stage &stage,
                                               int stream_rows, uint32_t &zeros)
{
    const int tid = threadIdx.x;
    float4 gv[4], xv[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const uint32_t j = base + 4 * (tid + kThreads * r);
        if constexpr (kMode == kPassDiff)
            gv[r] = ld4_row(grow + j, stream_rows);
        else
            gv[r] = load_grad4(grow, j, d);
        xv[r] = kMode == kPassNaive ? make_float4(0.f, 0.f, 0.f, 0.f) : ld4_row(xrow + j, stream_rows);
    }
    uint32_t count = 0;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const uint32_t j = base + 4 * (tid + kThreads * r);
        const float gg[4] = {gv[r].x, gv[r].y, gv[r].z, gv[r].w};
        const float xo[4] = {xv[r].x, xv[r].y, xv[r].z, xv[r].w};
        float x[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (kMode == kPassNaive) {
                x[c] = (kFull || j + c < d) ? gg[c] : 0.f;
            } else if (kMode != kPassEf) {
                x[c] = (kFull || j + c < d) ? fsub(gg[c], xo[c]) : 0.f;
            } else {
                // e = x_old - C(x_old): +0 where the previous step kept the coordinate
                const float e = was_kept(kt, sel_key(sk_prev, xo[c], j + c), j + c) ? 0.f : xo[c];
                x[c] = (kFull || j + c < d) ? fadd(gg[c], e) : 0.f;
            }
        }
        if (kMode == kPassEf) st4_stream(xrow + j, make_float4(x[0], x[1], x[2], x[3]));
#pragma unroll
        for (int c = 0; c < 4; ++c)
            consider<kMode == kPassEf>(x[c], j + c, base, kFull || j + c < d, guess, sk, stage, count, zeros);
    }
    return count;
}

// End of a tile in tk_pass1.  No workgroup barrier: a wavefront that is done registers itself, and
// whichever of the four comes last does the rest for the whole tile - takes the tile's space in its
// region (one atomic add), writes the directory record and copies all staged candidates.  The other
// three leave at once instead of waiting for the atomic.
// sh: 9 LDS words, sh[4] zeroed (with a barrier after it) before the first wavefront can get here.
// zeros: this wavefront's count of exact zeros; the tile's sum goes into the directory record's last word.
__device__ __forceinline__ void finish_tile(const float (*stage_val)[kSub], const uint16_t (*stage_at)[kSub], uint32_t *sh,
                                            uint32_t count, uint32_t zeros,
                                            const TkGeom &ge, int i, int t, uint2 *__restrict__ cand,
                                            uint32_t *__restrict__ cursor, uint4 *__restrict__ tile_dir,
                                            uint32_t *overflow_flag)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // this wavefront's staged candidates are complete before it registers
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    uint32_t arrived = 0;
    if (lane == 0) {
        sh[wave] = count;
        sh[5 + wave] = zeros;
        arrived = __hip_atomic_fetch_add(&sh[4], 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    arrived = __builtin_amdgcn_readfirstlane(arrived);
    if (arrived != 3) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");

    const uint32_t cnt[4] = {sh[0], sh[1], sh[2], sh[3]};
    uint32_t at = 0;
    if (lane == 0) at = take_space(cnt, sh[5] + sh[6] + sh[7] + sh[8], ge, i, t, cursor, tile_dir, overflow_flag);
    at = __builtin_amdgcn_readfirstlane(at);
    if (at == kNoSpace) return;
    uint2 *dst = cand + worker_base(ge, i) + at;
    const uint32_t base = (uint32_t)t * kTile;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        for (uint32_t q = lane; q < cnt[w]; q += kWave)
            dst[q] = make_uint2(base + stage_at[w][q], __float_as_uint(stage_val[w][q]));
        dst += cnt[w];
    }
}

// G: element type of g - float, or uint16_t (bfloat16 bits) for gradients handed over as bfloat16.
template <int kMode, typename G>
__global__ __launch_bounds__(kThreads) void tk_pass1(const G *__restrict__ g, float *__restrict__ xs, TkGeom ge,
                                                     TkWorker *ws, uint2 *__restrict__ cand,
                                                     uint32_t *__restrict__ cursor, uint4 *__restrict__ tile_dir)
{
    __shared__ float stage_val[4][kSub];
    __shared__ uint16_t stage_at[4][kSub];
    __shared__ uint32_t sh[9];
    const int t = tile_of_block(blockIdx.x, ge.xcd_chunk);
    if (t >= ge.n_tiles) return;
    const int i = blockIdx.y;
    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const uint32_t guess = ws[i].guess;
    const KeptTest kt = kept_test(ws[i].tc, ge.idx_bits);
    const SelKey sk = sel_key_of(ge.rand, ge.rand.step_now, i);
    const SelKey sk_prev = sel_key_of(ge.rand, ws[i].step_word, i);
    const uint32_t d = (uint32_t)ge.d;
    const uint32_t base = (uint32_t)t * kTile;
    if (tid == 0) sh[4] = 0;
    __syncthreads();
    uint32_t count, zeros = 0;
    const G *grow = g + (int64_t)i * (kMode == kPassDiff ? ge.ld : ge.d);
    const Stage stage{stage_val[wave], stage_at[wave]};
    if (base + kTile <= d)
        count = pass1_tile<true, kMode, G>(grow, xs + (int64_t)i * ge.ld, base, d, kt, guess, sk, sk_prev,
                                           stage, ge.stream_rows, zeros);
    else
        count = pass1_tile<false, kMode, G>(grow, xs + (int64_t)i * ge.ld, base, d, kt, guess, sk, sk_prev,
                                            stage, ge.stream_rows, zeros);
    finish_tile(stage_val, stage_at, sh, count, zeros, ge, i, t, cand, cursor, tile_dir, &ws[i].overflow);
}

// ---------------------------------------------------------------------------------------------
// The kept values of a tile, summed over the workers, and the AMSGrad update of the tile (tk_final's work).
//
// A coordinate of a tile belongs to one wavefront - the same one in tk_pass1, tk_pick's listing and here -
// and a tile's candidates are stored wavefront by wavefront, so each wavefront can sum the kept values
// of its own coordinates without looking at the others: no workgroup barrier, and the ascending worker
// order of the sum is just the order of its own instructions (within one worker the coordinates of
// the kept candidates are distinct).
constexpr int kFinBatch = 8;   // workers whose candidates a wavefront has in flight at a time

// Adds, for the calling wavefront's coordinates of tile t, the kept values (comp >= Tc_i) of all
// workers into acc (LDS, kTile floats, zeroed by the caller for these coordinates) in ascending
// worker order.  ws: the records that hold the selection's thresholds (and, for Rand-k, the draw they were made
// with).  kScatter (CD-Adam, Algorithm 1, line 6): the kept value u = c_i[j] is also added to
// ghat_i[j] in `rows` ([n][ld]); the old values are fetched for a whole batch before they are used.
template <bool kScatter>
__device__ __forceinline__ void sum_kept_tile(float *acc, const TkGeom &ge, const TkWorker *__restrict__ ws,
                                              const uint2 *__restrict__ cand, const uint4 *__restrict__ tile_dir,
                                              int t, float *__restrict__ rows)
{
    const uint32_t base = (uint32_t)t * kTile;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int w0 = 0; w0 < ge.n; w0 += kWave) {
        const int nw = min(kWave, ge.n - w0);
        // lane l: where worker w0 + l keeps this wavefront's candidates of the tile, and its threshold
        uint32_t my_start = 0, my_count = 0;
        uint64_t my_tc = kNoThreshold;
        SelKey my_sk = {0u, 0u, 0u};
        if (lane < nw) {
            const uint4 rec = tile_dir[(int64_t)(w0 + lane) * ge.n_tiles + t];
            const uint32_t c[4] = {rec.y & 0xffffu, rec.y >> 16, rec.z & 0xffffu, rec.z >> 16};
            my_start = rec.x;
            for (int q = 0; q < wave; ++q) my_start += c[q];
            my_count = c[wave];
            my_tc = ws[w0 + lane].tc;
            my_sk = sel_key_of(ge.rand, ws[w0 + lane].step_word, w0 + lane);
        }
        for (int wb = 0; wb < nw; wb += kFinBatch) {
            uint2 e[kFinBatch];
            uint32_t cnt[kFinBatch];
            bool keep[kFinBatch];
            float old[kFinBatch];
#pragma unroll
            for (int u = 0; u < kFinBatch; ++u) {
                const int w = min(wb + u, nw - 1);           // clamped: the copies past nw are not used
                cnt[u] = wb + u < nw ? (uint32_t)__shfl((int)my_count, w, kWave) : 0u;
                const uint32_t start = (uint32_t)__shfl((int)my_start, w, kWave);
                e[u] = make_uint2(0u, 0u);
                if ((uint32_t)lane < cnt[u]) e[u] = cand[worker_base(ge, w0 + w) + start + lane];
            }
#pragma unroll
            for (int u = 0; u < kFinBatch; ++u) {
                const int w = min(wb + u, nw - 1);
                const uint32_t tc_lo = (uint32_t)__shfl((int)(uint32_t)my_tc, w, kWave);
                const uint32_t tc_hi = (uint32_t)__shfl((int)(uint32_t)(my_tc >> 32), w, kWave);
                const uint64_t tc = ((uint64_t)tc_hi << 32) | tc_lo;
                SelKey sk = {0u, 0u, 0u};
                if (ge.rand.on) sk = {1u, (uint32_t)__shfl((int)my_sk.a, w, kWave), (uint32_t)__shfl((int)my_sk.b, w, kWave)};
                keep[u] = (uint32_t)lane < cnt[u] &&
                          composite(sel_key(sk, __uint_as_float(e[u].y), e[u].x), e[u].x, ge.idx_bits) >= tc;
                old[u] = 0.f;
                if (kScatter && keep[u]) old[u] = rows[(int64_t)(w0 + w) * ge.ld + e[u].x];
            }
#pragma unroll
            for (int u = 0; u < kFinBatch; ++u) {
                const int w = min(wb + u, nw - 1);
                if (keep[u]) {
                    const float x = __uint_as_float(e[u].y);
                    const uint32_t l = e[u].x - base;
                    acc[l] = fadd(acc[l], x);
                    if (kScatter) rows[(int64_t)(w0 + w) * ge.ld + e[u].x] = fadd(old[u], x);
                }
                if (cnt[u] > (uint32_t)kWave) {
                    // more than 64 candidates of this worker in the wavefront's quarter of the tile (rare)
                    const uint32_t tc_lo = (uint32_t)__shfl((int)(uint32_t)my_tc, w, kWave);
                    const uint32_t tc_hi = (uint32_t)__shfl((int)(uint32_t)(my_tc >> 32), w, kWave);
                    const uint64_t tc = ((uint64_t)tc_hi << 32) | tc_lo;
                    const uint32_t start = (uint32_t)__shfl((int)my_start, w, kWave);
                    const SelKey sk = {ge.rand.on, (uint32_t)__shfl((int)my_sk.a, w, kWave),
                                       (uint32_t)__shfl((int)my_sk.b, w, kWave)};
                    const uint2 *src = cand + worker_base(ge, w0 + w) + start;
                    for (uint32_t q = kWave + lane; q < cnt[u]; q += kWave) {
                        const uint2 c = src[q];
                        const float x = __uint_as_float(c.y);
                        if (composite(sel_key(sk, x, c.x), c.x, ge.idx_bits) >= tc) {
                            const uint32_t l = c.x - base;
                            acc[l] = fadd(acc[l], x);
                            if (kScatter) {
                                float *gh = rows + (int64_t)(w0 + w) * ge.ld + c.x;
                                *gh = fadd(*gh, x);
                            }
                        }
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // next worker's adds come after these
            }
        }
    }
}

// Server average and AMSGrad update, one workgroup per tile.
template <bool kStreamState>
__global__ __launch_bounds__(kThreads) void tk_final(TkGeom ge, const TkWorker *__restrict__ ws,
                                                     const uint2 *__restrict__ cand,
                                                     const uint4 *__restrict__ tile_dir,
                                                     float *__restrict__ theta, float *__restrict__ m,
                                                     float *__restrict__ v, float *__restrict__ vhat, AmsParams p)
{
    __shared__ float acc[kTile];
    const int t = blockIdx.x;
    const int64_t base = (int64_t)t * kTile;
    const int tid = threadIdx.x;

#pragma unroll
    for (int r = 0; r < 4; ++r) st4(acc + 4 * (tid + kThreads * r), make_float4(0.f, 0.f, 0.f, 0.f));
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    sum_kept_tile<false>(acc, ge, ws, cand, tile_dir, t, nullptr);

    // the state is loaded only now: fewer live registers above (more workgroups per compute unit),
    // which measured faster than loading it first
    float4 th[4], mm[4], vv[4], vh[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int64_t j = base + 4 * (tid + kThreads * r);
        th[r] = ld4_state<kStreamState>(theta + j);
        mm[r] = ld4_state<kStreamState>(m + j);
        vv[r] = ld4_state<kStreamState>(v + j);
        vh[r] = ld4_state<kStreamState>(vhat + j);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int l = 4 * (tid + kThreads * r);
        const int64_t j = base + l;
        const float4 a = ld4(acc + l);
        const float4 gbar = make_float4(fdiv(a.x, p.n_workers), fdiv(a.y, p.n_workers), fdiv(a.z, p.n_workers),
                                        fdiv(a.w, p.n_workers));
        const float4 vh0 = vh[r];
        amsgrad_update4(th[r], mm[r], vv[r], vh[r], gbar, p);
        st4_state<kStreamState>(theta + j, th[r]);
        st4_state<kStreamState>(m + j, mm[r]);
        st4_state<kStreamState>(v + j, vv[r]);
        // with a sparse average vhat = max(vhat, v) moves at few coordinates (v only decays elsewhere)
        st4_if_changed<kStreamState>(vhat + j, vh[r], vh0);
    }
}

// ---------------------------------------------------------------------------------------------
// How the workgroups of tk_hist and tk_compact share a worker's candidates: blockIdx.x = slice *
// parts + part, and a part is a contiguous piece of the slice's region.
struct Piece {
    int slice;
    uint32_t q0, q1;     // entries [q0, q1) of the region
};
__device__ __forceinline__ Piece piece_of(const TkGeom &ge, const uint32_t *__restrict__ cursor, int worker)
{
    Piece p;
    p.slice = blockIdx.x / ge.parts;
    const uint32_t part = blockIdx.x % ge.parts;
    const uint32_t count = min(cursor[worker * ge.slices + p.slice], ge.region_cap);
    const uint32_t chunk = (count + ge.parts - 1) / ge.parts;
    p.q0 = min(part * chunk, count);
    p.q1 = min(p.q0 + chunk, count);
    return p;
}

// ---------------------------------------------------------------------------------------------
// How a kernel forms the vector that is compressed again from what is stored:
//   kSrcStored  the stored x itself (error feedback)
//   kSrcGrad    g - ghat_i, a = g (rows of d floats, any 4-byte alignment), b = ghat_i (CD-Adam workers)
//   kSrcDiff    a - b, both padded rows (CD-Adam server: ghat - gtilde)
//   kSrcGradOnly  a = g itself (naive compression)
enum { kSrcStored = 0, kSrcGrad = 1, kSrcDiff = 2, kSrcGradOnly = 3 };

// The 16 values of this thread in the tile at `base` (coordinates base + 4 (tid + 256 r) + c).
// a: for kSrcGrad / kSrcGradOnly row i of the gradients (elements of type G), else a padded float row.
template <int kSrc, typename G>
__device__ __forceinline__ void load_source_tile(float (&x)[4][4], const void *__restrict__ a, int i, const TkGeom &ge,
                                                 const float *__restrict__ brow, uint32_t base, uint32_t d)
{
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const uint32_t j = base + 4 * (threadIdx.x + kThreads * r);
        float4 av;
        if constexpr (kSrc == kSrcGrad || kSrc == kSrcGradOnly)
            av = load_grad4(static_cast<const G *>(a) + (int64_t)i * ge.d, j, d);
        else
            av = ld4(static_cast<const float *>(a) + (int64_t)i * ge.ld + j);
        x[r][0] = av.x;
        x[r][1] = av.y;
        x[r][2] = av.z;
        x[r][3] = av.w;
        if (kSrc == kSrcGrad || kSrc == kSrcDiff) {
            const float4 bv = ld4(brow + j);
            x[r][0] = fsub(x[r][0], bv.x);
            x[r][1] = fsub(x[r][1], bv.y);
            x[r][2] = fsub(x[r][2], bv.z);
            x[r][3] = fsub(x[r][3], bv.w);
        }
    }
}

// Which way a worker's selection goes in this step, from what the listing pass left (the same test in tk_hist and
// tk_pick, which see the same cursors and flags):
//   kCaseListed    every element at or above the guess is listed and there are at least k of them: the k-th largest
//                  is a candidate, the candidate histograms locate it;
//   kCaseZeroTail  error feedback with magnitude keys, a guess of 0 (every non-zero element is listed) and fewer
//                  than k candidates: the k-th largest is a zero (see zero_tail_threshold);
//   kCaseMiss      the guess was too high (always on the first step, else when the threshold fell through the slack),
//                  or a candidate region was full: nothing below the guess is known, the whole vector is counted.
enum { kCaseListed = 0, kCaseZeroTail = 1, kCaseMiss = 2 };
template <int kSrc>
__device__ __forceinline__ int selection_case(const TkGeom &ge, uint32_t total, uint32_t guess, bool overflow)
{
    if (total >= ge.k && !overflow) return kCaseListed;
    if (kSrc == kSrcStored && !ge.rand.on && guess == 0u && !overflow) return kCaseZeroTail;
    return kCaseMiss;
}

// Number of candidates of worker i = sum of its region cursors.  Wavefront 0 adds them up; total_sh: one LDS
// word; ends with a barrier.  All threads of the workgroup call this.
__device__ __forceinline__ uint32_t candidates_listed(const TkGeom &ge, const uint32_t *__restrict__ cursor, int i,
                                                      uint32_t *total_sh)
{
    const int lane = threadIdx.x & 63;
    if ((threadIdx.x >> 6) == 0) {
        uint32_t c = 0;
        for (int q = lane; q < ge.slices; q += kWave) c += cursor[i * ge.slices + q];
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) c += __shfl_xor(c, off, kWave);
        if (lane == 0) *total_sh = c;
    }
    __syncthreads();
    return *total_sh;
}

// First kernel of the selection.  Grid (slices * parts, n).
// Usual case (kCaseListed): histograms of the candidates of a worker - coarse bins, and the fine bins of the
// kWindowCoarse coarse bins that start with the guess's.  Loads are issued four at a time.
// After a miss (kCaseMiss) the workgroups of the worker count the whole vector, re-formed from what is stored
// (a, b: see load_source_tile), into the worker's full coarse histogram instead; tk_pick takes the coarse bin of
// the k-th largest from it and lists again.  Bin 0 (zeros and the smallest denormals) is not counted there but
// taken as the remainder: in a sparse vector it would draw most LDS atomics of a tile to one word.
template <int kSrc, typename G>
__global__ __launch_bounds__(kThreads) void tk_hist(TkGeom ge, const TkWorker *__restrict__ ws,
                                                    const uint2 *__restrict__ cand,
                                                    const uint32_t *__restrict__ cursor,
                                                    uint32_t *__restrict__ hist1, uint32_t *__restrict__ histf,
                                                    uint32_t *__restrict__ hist_full, const void *__restrict__ a,
                                                    const float *__restrict__ b)
{
    __shared__ uint32_t lh[kBins1];
    __shared__ uint32_t lf[kFineWindow];
    __shared__ uint32_t total_sh;
    const int i = blockIdx.y;
    const int tid = threadIdx.x;
    const uint32_t guess = ws[i].guess;
    const uint32_t total = candidates_listed(ge, cursor, i, &total_sh);
    const int which = selection_case<kSrc>(ge, total, guess, ws[i].overflow != 0u);
    if (which == kCaseZeroTail) return;
    const Piece pc = piece_of(ge, cursor, i);
    if (which == kCaseListed && pc.q0 >= pc.q1) return;
    const SelKey sk = sel_key_of(ge.rand, ge.rand.step_now, i);
    for (int q = tid; q < kBins1; q += kThreads) lh[q] = 0;
    if (which == kCaseMiss) {
        __syncthreads();
        const uint32_t d = (uint32_t)ge.d;
        const float *brow = (kSrc == kSrcGrad || kSrc == kSrcDiff) ? b + (int64_t)i * ge.ld : nullptr;
        for (int t = blockIdx.x; t < ge.n_tiles; t += gridDim.x) {
            const uint32_t base = (uint32_t)t * kTile;
            float x[4][4];
            load_source_tile<kSrc, G>(x, a, i, ge, brow, base, d);
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const uint32_t j = base + 4 * (tid + kThreads * r) + c;
                    const uint32_t bin = sel_key(sk, x[r][c], j) >> kShift1;
                    if (bin != 0 && j < d) atomicAdd(&lh[bin], 1u);
                }
        }
        __syncthreads();
        for (int q = tid; q < kBins1; q += kThreads) {
            const uint32_t c = lh[q];
            if (c) atomicAdd(hist_full + (int64_t)i * kBins1 + q, c);
        }
        return;
    }
    for (int q = tid; q < kFineWindow; q += kThreads) lf[q] = 0;
    __syncthreads();
    const uint32_t wbase = guess & ~(uint32_t)(kFinePerCoarse - 1);   // first fine bin of the guess's coarse bin
    const uint2 *src = cand + region_base(ge, i, pc.slice);
    for (uint32_t qb = pc.q0; qb < pc.q1; qb += 4 * kThreads) {
        uint2 y[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t q = qb + u * kThreads + tid;
            y[u] = q < pc.q1 ? src[q] : make_uint2(0u, 0u);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (qb + u * kThreads + tid < pc.q1) {
                const uint32_t fine = sel_key(sk, __uint_as_float(y[u].y), y[u].x) >> kFineShift;
                atomicAdd(&lh[fine >> (kShift1 - kFineShift)], 1u);
                if (fine - wbase < (uint32_t)kFineWindow) atomicAdd(&lf[fine - wbase], 1u);
            }
        }
    }
    __syncthreads();
    for (int b1 = tid; b1 < kBins1; b1 += kThreads) {
        const uint32_t c = lh[b1];
        if (c) atomicAdd(hist1 + (int64_t)i * kBins1 + b1, c);
    }
    for (int q = tid; q < kFineWindow; q += kThreads)
        if (lf[q]) atomicAdd(histf + (int64_t)i * kFineWindow + q, lf[q]);
}

// Second kernel of the selection: the leading digits of Tc.  Grid (ge.relist_wgs, n).
// Usual case (kCaseListed): workgroup 0 of the worker finds the coarse and (if the window covers it) fine bin of
// the k-th largest from the candidate histograms, and the other workgroups return at once.
// After a miss tk_hist has counted the whole vector into the worker's full coarse histogram: every workgroup takes
// the coarse bin of the k-th largest from it (each works it out for itself; workgroup 0 records it) and lists the
// elements in that bin or above, tile by tile, into the worker's regions - through the second set of cursors
// (cursor_b, all zero here), since the first still holds the counts this kernel's workgroups decide by.  The
// worker is flagged `relisted`: tk_compact then reads cursor_b, and tk_resolve clears both.  A region that fills up
// there as well sets overflow2: tk_resolve then selects without lists (exact_select).
// Consumes (and clears) the candidate histograms.
template <int kSrc, typename G>
__global__ __launch_bounds__(kThreads) void tk_pick(TkGeom ge, TkWorker *__restrict__ ws,
                                                    uint32_t *__restrict__ hist1, uint32_t *__restrict__ histf,
                                                    const uint32_t *__restrict__ cursor,
                                                    uint32_t *__restrict__ cursor_b,
                                                    const uint32_t *__restrict__ hist_full,
                                                    const void *__restrict__ a, const float *__restrict__ b,
                                                    uint2 *__restrict__ cand, uint4 *__restrict__ tile_dir)
{
    __shared__ uint2 stage[4][kSub];
    __shared__ uint32_t lh[kBins1];
    __shared__ uint32_t part[kThreads / kWave];
    __shared__ uint32_t res[4];
    __shared__ uint32_t fres[3];
    __shared__ uint32_t sh[9];
    __shared__ uint32_t total_sh;
    const int i = blockIdx.y;
    const int bx = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const uint32_t guess = ws[i].guess;
    const uint32_t total = candidates_listed(ge, cursor, i, &total_sh);
    const int which = selection_case<kSrc>(ge, total, guess, ws[i].overflow != 0u);
    uint32_t *row = hist1 + (int64_t)i * kBins1;
    uint32_t *frow = histf + (int64_t)i * kFineWindow;

    if (which == kCaseListed) {
        if (bx != 0) return;
        for (int q = tid; q < kBins1; q += kThreads) lh[q] = row[q];
        __syncthreads();
        find_rank_bin(lh, part, res, kBins1, ge.k);
        uint32_t prefix = res[0];                   // coarse bin of the k-th largest
        uint32_t pshift = kShift1;
        uint32_t rank = ge.k - res[1];
        uint32_t count = res[2];
        const uint32_t wb = guess >> (kShift1 - kFineShift);      // first coarse bin of the fine window
        if (prefix - wb < (uint32_t)kWindowCoarse) {
            // the fine histogram covers this coarse bin: pick the fine bin as well (one wavefront)
            if (wave == 0) {
                const uint32_t c = frow[(prefix - wb) * kFinePerCoarse + lane];
                uint32_t suffix = c;                // candidates of this coarse bin in fine bins >= lane
#pragma unroll
                for (int off = 1; off < kWave; off <<= 1) {
                    const uint32_t t = __shfl_down(suffix, off, kWave);
                    if (lane + off < kWave) suffix += t;
                }
                const uint64_t reach = __ballot(suffix >= rank);  // lane 0 reaches: suffix(0) = count >= rank
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
        __syncthreads();   // every thread has read the histograms before they are cleared
        if (tid == 0) {
            ws[i].prefix = prefix;
            ws[i].pshift = pshift;
            ws[i].rank = rank;
            ws[i].whole = (count == rank) ? 1u : 0u;
            ws[i].relisted = 0u;
        }
        for (int q = tid; q < kBins1; q += kThreads) row[q] = 0;
        for (int q = tid; q < kFineWindow; q += kThreads) frow[q] = 0;
        return;
    }

    if (which == kCaseZeroTail) {
        // all candidates are kept; tk_resolve places the threshold among the zeros, which are ordered by index
        // alone, from the zero counts of the tiles
        if (bx != 0) return;
        if (tid == 0) {
            ws[i].prefix = 0u;
            ws[i].pshift = kShift1;
            ws[i].rank = ge.k - total;          // so many zeros are kept, the lowest indices first
            ws[i].whole = kZeroTail;
            ws[i].relisted = 0u;
        }
        return;
    }

    // after a miss: the coarse bin of the k-th largest from the full histogram, and the lists anew
    const uint32_t d = (uint32_t)ge.d;
    {
        uint32_t counted = 0;
        for (int q = tid; q < kBins1; q += kThreads) {
            const uint32_t c = hist_full[(int64_t)i * kBins1 + q];
            lh[q] = c;
            counted += c;
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) counted += __shfl_xor(counted, off, kWave);
        if (lane == 0) part[wave] = counted;
        __syncthreads();
        if (tid == 0) lh[0] = d - (part[0] + part[1] + part[2] + part[3]);   // bin 0 is the remainder
        __syncthreads();
        find_rank_bin(lh, part, res, kBins1, ge.k);        // the histogram holds all d >= k elements
    }
    const uint32_t prefix = res[0];
    const SelKey sk = sel_key_of(ge.rand, ge.rand.step_now, i);
    if (bx == 0 && tid == 0) {
        ws[i].prefix = prefix;
        ws[i].pshift = kShift1;
        ws[i].rank = ge.k - res[1];
        ws[i].whole = (res[2] == ge.k - res[1]) ? 1u : 0u;
        ws[i].relisted = 1u;
    }
    const float *brow = (kSrc == kSrcGrad || kSrc == kSrcDiff) ? b + (int64_t)i * ge.ld : nullptr;
    for (int t = bx; t < ge.n_tiles; t += gridDim.x) {
        const uint32_t base = (uint32_t)t * kTile;
        float x[4][4];
        load_source_tile<kSrc, G>(x, a, i, ge, brow, base, d);
        uint32_t count = 0, zeros = 0;
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t j = base + 4 * (tid + kThreads * r) + c;
                bool hit = j < d && (sel_key(sk, x[r][c], j) >> kShift1) >= prefix;
                if (kSrc == kSrcStored && !sk.on) {          // zeros are counted, not listed (as in tk_pass1)
                    const bool zero = j < d && mag_key(x[r][c]) == 0u;
                    zeros += (uint32_t)__popcll(__ballot(zero));
                    hit = hit && !zero;
                }
                const uint32_t slot = wave_append(hit, count);
                if (hit) stage[wave][slot] = make_uint2(j, __float_as_uint(x[r][c]));
            }
        flush_begin(count, zeros, sh, 0, ge, i, t, cursor_b, tile_dir, &ws[i].overflow2);
        flush_end(stage[wave], count, sh, ge, i, cand);
        __syncthreads();   // sh and stage are reused by the next tile
    }
}

// Copies the candidates that carry the prefix, as comp values, to the dense storage.  Each wavefront
// takes a quarter of the workgroup's piece and writes its hits from the start of that quarter
// onwards (as many slots as it reads, so it cannot overflow), and records {start, count} relative to
// the worker's first region; no atomics, tk_resolve walks the records.  While copying, the workgroup counts the
// next kFirstBits bits of comp below the prefix (hist2: [n][kBinsFirst], added to with atomics, emptied by
// tk_resolve) and every wavefront notes which of those digits occur in its piece (piece_bits: kPieceWords words
// per piece, written whole).  Grid (slices * parts, n).  Nothing to do for a worker whose threshold needs no
// further digit, or whose lists did not fit (tk_resolve then selects without lists).
__global__ __launch_bounds__(kThreads) void tk_compact(TkGeom ge, const TkWorker *__restrict__ ws,
                                                       const uint2 *__restrict__ cand,
                                                       const uint32_t *__restrict__ cursor,
                                                       const uint32_t *__restrict__ cursor_b,
                                                       uint64_t *__restrict__ dense, uint2 *__restrict__ dense_dir,
                                                       uint32_t *__restrict__ hist2, uint32_t *__restrict__ piece_bits)
{
    __shared__ uint32_t lh2[kBinsFirst];
    __shared__ uint32_t bits[kThreads / kWave][kPieceWords];
    const int per = gridDim.x;
    const int i = blockIdx.y;
    const int bx = blockIdx.x;
    if (ws[i].whole || ws[i].overflow2) return;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const uint32_t prefix = ws[i].prefix, pshift = ws[i].pshift;
    // the digit of comp right below the prefix (tk_resolve's first digit)
    const int s_lo = (int)pshift + ge.idx_bits - kFirstBits;      // pshift >= kFineShift > kFirstBits
    for (int b = tid; b < kBinsFirst; b += kThreads) lh2[b] = 0;
    if (lane < kPieceWords) bits[wave][lane] = 0;
    __syncthreads();
    const SelKey sk = sel_key_of(ge.rand, ge.rand.step_now, i);
    const Piece pc = piece_of(ge, ws[i].relisted ? cursor_b : cursor, i);   // lists made anew count in cursor_b
    const uint32_t quarter = (pc.q1 - pc.q0 + 3) / 4;
    const uint32_t w0 = min(pc.q0 + wave * quarter, pc.q1), w1 = min(w0 + quarter, pc.q1);
    const int64_t rbase = region_base(ge, i, pc.slice);
    const uint2 *src = cand + rbase;
    uint64_t *out = dense + rbase + w0;
    uint32_t count = 0;
    for (uint32_t qb = w0; qb < w1; qb += 4 * kWave) {
        uint2 c[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t q = qb + u * kWave + lane;
            c[u] = q < w1 ? src[q] : make_uint2(0u, 0u);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t key = sel_key(sk, __uint_as_float(c[u].y), c[u].x);
            const bool hit = qb + u * kWave + lane < w1 && (key >> pshift) == prefix;
            const uint32_t slot = wave_append(hit, count);
            if (hit) {
                const uint64_t comp = composite(key, c[u].x, ge.idx_bits);
                out[slot] = comp;
                const uint32_t digit = (uint32_t)(comp >> s_lo) & (uint32_t)(kBinsFirst - 1);
                atomicAdd(&lh2[digit], 1u);
                atomicOr(&bits[wave][digit >> 5], 1u << (digit & 31u));
            }
        }
    }
    const int64_t rec = ((int64_t)i * per + bx) * 4 + wave;
    if (lane == 0) dense_dir[rec] = make_uint2((uint32_t)(rbase - worker_base(ge, i)) + w0, count);
    // the piece's bitmap, written whole every step (the wavefront reads back its own LDS atomics)
    if (lane < kPieceWords) piece_bits[rec * kPieceWords + lane] = bits[wave][lane];
    __syncthreads();
    for (int b = tid; b < kBinsFirst; b += kThreads) {
        const uint32_t c = lh2[b];
        if (c) atomicAdd(hist2 + (int64_t)i * kBinsFirst + b, c);
    }
}

// ---------------------------------------------------------------------------------------------
// One workgroup of 1024 threads per worker: the digits of Tc below the prefix, over the pieces
// tk_compact filled (slices * parts * 4 <= 2 * kResolveThreads of them).  Hands the next step its
// guess and empties the worker's region cursors for it.
constexpr int kMaxPieces = 2048;   // slices * parts * 4 never exceeds this (the host picks parts accordingly)
constexpr int kFew = 256;         // at most this many elements are ranked directly instead of by further digits
                                  // (1024 measured slower: ranking a thousand elements against each other costs
                                  // more than one more digit over a threshold bin of a few thousand)
static_assert(kMaxPieces <= 2 * kResolveThreads, "two pieces per thread in the prefix sum");

constexpr int kScanUnroll = 4;    // independent loads per thread in the scans of the dense set

// LDS of the digit search, shared by tk_resolve and tk_select.
struct ResolveLds {
    uint32_t lh[kBins2];
    uint32_t part[kResolveThreads / kWave];
    uint32_t res[4];
    uint64_t few[kFew];
    uint32_t n_few;
    uint64_t tc_sh;
};

// The digits of Tc below `prefix` (which leaves s_hi low bits of comp open), 12 bits at a time, over the
// cnt comp values that fetch(q, comp) delivers kScanUnroll at a time (comp[u] = element q[u], anything for
// q[u] >= cnt; q ascends with u), of which the one of 1-based rank `rank` (from the top) among those that
// carry the prefix is wanted.  Once at most kFew elements carry the prefix they are fetched and
// ranked against each other directly.  All threads of the workgroup (256 or 1024) call this; returns Tc.
// kWholeBins: a digit whose bin holds exactly the elements still wanted ends the search with the bin's lower edge as
// Tc - right when every element of the vector that could fall into that bin is among the cnt delivered (the
// threshold bin of tk_compact is), wrong when the elements are only those above some bound that may cut the bin
// (the candidate list of tk_small_pass): then the search goes on to the k-th largest comp value itself.
// have_first: the first digit has kFirstBits bits and its counts are in L.lh[0 .. kBinsFirst) already (with a
// barrier after them); the first scan is not made.
template <bool kWholeBins = true, class Fetch>
__device__ __forceinline__ uint64_t resolve_digits(Fetch fetch, uint32_t cnt, uint64_t prefix, uint32_t rank, int s_hi,
                                                   ResolveLds &L, bool have_first = false)
{
    const int tid = threadIdx.x;
    const int nt = (int)blockDim.x;
    uint64_t tc = prefix << s_hi;
    bool done = false;
    while (!done) {
        const int s_lo = max(s_hi - (have_first ? kFirstBits : kDigitBits), 0);
        const uint32_t mask = (1u << (s_hi - s_lo)) - 1u;
        if (!have_first) {
            for (int b = tid; b < kBins2; b += nt) L.lh[b] = 0;
            __syncthreads();
            for (uint32_t qb = 0; qb < cnt; qb += kScanUnroll * nt) {
                uint32_t q[kScanUnroll];
                uint64_t comp[kScanUnroll];
#pragma unroll
                for (int u = 0; u < kScanUnroll; ++u) q[u] = qb + u * nt + tid;
                fetch(q, comp);                                 // independent loads: all in flight at once
#pragma unroll
                for (int u = 0; u < kScanUnroll; ++u)
                    if (q[u] < cnt && (comp[u] >> s_hi) == prefix)
                        atomicAdd(&L.lh[(uint32_t)(comp[u] >> s_lo) & mask], 1u);
            }
            __syncthreads();
        }
        find_rank_bin(L.lh, L.part, L.res, have_first ? kBinsFirst : kBins2, rank);
        have_first = false;
        if (!L.res[3]) break;                                  // cannot happen: rank <= matching elements
        prefix = (prefix << (s_hi - s_lo)) | L.res[0];
        rank -= L.res[1];
        const uint32_t left = L.res[2];                        // elements that carry the new prefix
        s_hi = s_lo;
        if (s_lo == 0 || (kWholeBins && left == rank)) {       // last digit, or all under this prefix are kept
            done = true;
            tc = prefix << s_lo;
        } else if (left <= (uint32_t)min(kFew, nt)) {
            if (tid == 0) L.n_few = 0;
            __syncthreads();
            for (uint32_t qb = 0; qb < cnt; qb += kScanUnroll * nt) {
                uint32_t q[kScanUnroll];
                uint64_t comp[kScanUnroll];
#pragma unroll
                for (int u = 0; u < kScanUnroll; ++u) q[u] = qb + u * nt + tid;
                fetch(q, comp);
#pragma unroll
                for (int u = 0; u < kScanUnroll; ++u)
                    if (q[u] < cnt && (comp[u] >> s_hi) == prefix)
                        L.few[atomicAdd(&L.n_few, 1u)] = comp[u];
            }
            __syncthreads();
            if ((uint32_t)tid < left) {
                const uint64_t mine = L.few[tid];
                uint32_t greater = 0;
                for (uint32_t u = 0; u < left; ++u) greater += L.few[u] > mine ? 1u : 0u;
                if (greater + 1 == rank) L.tc_sh = mine;      // comp values are unique: exactly one thread
            }
            __syncthreads();
            done = true;
            tc = L.tc_sh;
        }
        __syncthreads();
    }
    return tc;
}

// Records the finished selection of a worker and prepares the next step's guess: a few fine bins
// below this threshold - at least twice the distance the threshold just fell (a rising threshold needs
// no slack), never less than kMinSlack, shrinking by one bin per quiet step, doubled after a miss.
// w: the record as the step found it (its slack and last threshold bin).  The flags of the running step are
// cleared for the next one.  One thread calls this.
__device__ __forceinline__ void finish_worker(TkWorker *ws, int i, const TkWorker &w, uint64_t tc, const TkGeom &ge,
                                              bool missed)
{
    ws[i].tc = tc;
    ws[i].step_word = ge.rand.step_now;
    const uint32_t fine = (uint32_t)(tc >> ge.idx_bits) >> kFineShift;
    const uint32_t fell = (w.last_fine != kNoGuess && w.last_fine > fine) ? w.last_fine - fine : 0u;
    uint32_t slack = missed ? w.slack * 2u : w.slack - 1u;
    slack = max(slack, 2u * fell + 2u);
    slack = min(max(slack, max(kMinSlack, ge.rand.min_slack)), kMaxSlack);
    ws[i].slack = slack;
    ws[i].last_fine = fine;
    ws[i].guess = fine > slack ? fine - slack : 0u;
    ws[i].overflow = 0u;
    ws[i].overflow2 = 0u;
}

// Exclusive prefix sum of one value per thread over the 1024 threads of tk_resolve; returns the exclusive sum,
// leaves the total in *total_sh.  part: 16 LDS words.  Two barriers.
__device__ __forceinline__ uint32_t resolve_scan(uint32_t v, uint32_t *part, uint32_t *total_sh)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t incl = v;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const uint32_t up = __shfl_up(incl, off, kWave);
        if (lane >= off) incl += up;
    }
    __syncthreads();                       // readers of an earlier part are done
    if (lane == kWave - 1) part[wave] = incl;
    __syncthreads();
    uint32_t before = 0;
    for (int q = 0; q < wave; ++q) before += part[q];
    if (threadIdx.x == kResolveThreads - 1) *total_sh = before + incl;
    return before + incl - v;
}

// Error feedback with fewer than k non-zero coordinates: the threshold is the comp value of the R-th zero of
// the stored row in index order (zeros tie, the lower index wins), found from the tiles' zero counts: first
// the tile that holds it, then its place inside that tile.  All kResolveThreads threads call this; R >= 1 and
// the row holds at least R zeros below d.
__device__ __forceinline__ uint64_t zero_tail_threshold(const uint4 *__restrict__ dir_row, const float *__restrict__ xrow,
                                                        const TkGeom &ge, uint32_t R, ResolveLds &L)
{
    const int tid = threadIdx.x;
    if (tid == 0) {                              // what is read below if the counts held fewer than R zeros
        L.res[0] = 0u;
        L.res[1] = 0u;
        L.tc_sh = (1ull << ge.idx_bits) - 1ull;
    }
    const int chunk = (ge.n_tiles + kResolveThreads - 1) / kResolveThreads;
    const int t0 = min(tid * chunk, ge.n_tiles), t1 = min(t0 + chunk, ge.n_tiles);
    uint32_t mine = 0;
    for (int t = t0; t < t1; ++t) mine += dir_row[t].w;
    uint32_t before = resolve_scan(mine, L.part, &L.res[3]);
    if (before < R && R <= before + mine) {
        for (int t = t0; t < t1; ++t) {
            const uint32_t z = dir_row[t].w;
            if (before + z >= R) {
                L.res[0] = (uint32_t)t;           // the tile of the R-th zero ...
                L.res[1] = R - before;            // ... which is this tile's res[1]-th zero
                break;
            }
            before += z;
        }
    }
    __syncthreads();
    const uint32_t base = L.res[0] * (uint32_t)kTile, r = L.res[1];
    // the tile in coordinate order: thread tid holds the coordinates base + 4 tid .. + 3 (padding is not counted)
    const float4 v = ld4(xrow + base + 4 * tid);
    const float x[4] = {v.x, v.y, v.z, v.w};
    uint32_t zc = 0;
#pragma unroll
    for (int c = 0; c < 4; ++c) zc += (base + 4 * tid + c < (uint32_t)ge.d && mag_key(x[c]) == 0u) ? 1u : 0u;
    uint32_t seen = resolve_scan(zc, L.part, &L.res[3]);
    if (seen < r && r <= seen + zc) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (base + 4 * tid + c < (uint32_t)ge.d && mag_key(x[c]) == 0u && ++seen == r)
                L.tc_sh = ((1ull << ge.idx_bits) - 1ull) - (uint64_t)(base + 4 * tid + c);   // key part 0
        }
    }
    __syncthreads();
    return L.tc_sh;
}

// ---------------------------------------------------------------------------------------------
// Selection without lists, for a vector whose candidates fit no region even when listed anew (so many elements
// share the leading bits of the k-th largest that only the whole composite key tells them apart - all-equal
// input is the extreme).  The worker's workgroup of tk_resolve does it alone: the digits of Tc by counting over
// the whole vector, re-formed element by element from what is stored (kDigitBits bits per sweep), then one more
// sweep that lists exactly the kept elements - k of them, which always fit: a worker's regions hold at least 8 k
// entries in all, and this list is written as one run from the worker's first region (no cursors; a tile's
// record holds its offset in that run, its candidates stand by owning wavefront as everywhere).  Slow - one
// compute unit reads the vector up to six times - and meant to be: it only has to be right.
//
// How the vector is re-formed (src: kSrcStored ... kSrcGradOnly; gtype: element type of the gradients, 0 fp32,
// 1 bfloat16, 2 half) is decided at run time here: one scalar load per element and operand.
struct ExactSource {
    int32_t src, gtype;
    const void *a;
    const float *b;
};
__device__ __forceinline__ float exact_value(const ExactSource &e, const TkGeom &ge, int i, uint32_t j)
{
    float av;
    if (e.src == kSrcGrad || e.src == kSrcGradOnly) {
        const int64_t at = (int64_t)i * ge.d + j;
        av = e.gtype == 0   ? static_cast<const float *>(e.a)[at]
             : e.gtype == 1 ? bf16_to_float(static_cast<const uint16_t *>(e.a)[at])
                            : f16_to_float(static_cast<const uint16_t *>(e.a)[at]);
    } else {
        av = static_cast<const float *>(e.a)[(int64_t)i * ge.ld + j];
    }
    if (e.src == kSrcGrad || e.src == kSrcDiff) av = fsub(av, e.b[(int64_t)i * ge.ld + j]);
    return av;
}

struct ExactLds {
    uint2 stage[4][kSub];      // the kept elements of a tile by owning wavefront
    uint32_t cnt[4];
    uint32_t zeros;
};

// The digits of Tc by counting over the whole vector.  All threads of the workgroup (256 or 1024) call this.
__device__ __forceinline__ uint64_t exact_threshold(const ExactSource &es, const TkGeom &ge, int i, ResolveLds &L)
{
    const int tid = threadIdx.x, nt = (int)blockDim.x;
    const uint32_t d = (uint32_t)ge.d;
    const SelKey sk = sel_key_of(ge.rand, ge.rand.step_now, i);
    int s_hi = 31 + ge.idx_bits;                                    // bits of comp still open
    uint64_t prefix = 0;
    uint32_t rank = ge.k;
    while (true) {
        const int s_lo = max(s_hi - kDigitBits, 0);
        const uint32_t mask = (1u << (s_hi - s_lo)) - 1u;
        for (int q = tid; q < kBins2; q += nt) L.lh[q] = 0;
        __syncthreads();
        for (int t = 0; t < ge.n_tiles; ++t) {
            for (int T = tid; T < kTile / 4; T += nt) {
                const uint32_t j0 = (uint32_t)t * kTile + 4u * (uint32_t)T;
                float x[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) x[c] = j0 + c < d ? exact_value(es, ge, i, j0 + c) : 0.f;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const uint64_t comp = composite(sel_key(sk, x[c], j0 + c), j0 + c, ge.idx_bits);
                    if (j0 + c < d && (comp >> s_hi) == prefix) atomicAdd(&L.lh[(uint32_t)(comp >> s_lo) & mask], 1u);
                }
            }
        }
        __syncthreads();
        find_rank_bin(L.lh, L.part, L.res, kBins2, rank);          // rank <= elements under the prefix
        prefix = (prefix << (s_hi - s_lo)) | L.res[0];
        rank -= L.res[1];
        const uint32_t left = L.res[2];
        __syncthreads();
        if (s_lo == 0 || left == rank) return prefix << s_lo;      // last digit, or all under this prefix are kept
        s_hi = s_lo;
    }
}

// Lists the kept elements (comp >= tc) of the vector, tile by tile, as one run from the start of the worker's
// space, and writes every tile's record.  Coordinate 4 T + c of a tile (T = 0 .. 1023) belongs to the wavefront
// (T mod 256) / 64 of the listing pass.  All threads of the workgroup (256 or 1024) call this.
__device__ __forceinline__ void list_kept(const ExactSource &es, const TkGeom &ge, int i, uint64_t tc,
                                          uint2 *__restrict__ cand, uint4 *__restrict__ tile_dir, ExactLds &E)
{
    const int tid = threadIdx.x, nt = (int)blockDim.x;
    const int lane = tid & 63;
    const uint32_t d = (uint32_t)ge.d;
    const SelKey sk = sel_key_of(ge.rand, ge.rand.step_now, i);
    const bool skip_zeros = (es.src == kSrcStored && !sk.on);      // zeros are counted, not listed (as in tk_pass1)
    uint32_t run = 0;                                               // uniform over the workgroup
    if (tid < 4) E.cnt[tid] = 0;
    if (tid == 0) E.zeros = 0;
    __syncthreads();
    for (int t = 0; t < ge.n_tiles; ++t) {
        for (int T = tid; T < kTile / 4; T += nt) {                 // the same number of rounds for every thread
            const int owner = (T & (kThreads - 1)) >> 6;            // uniform over a wavefront
            const uint32_t j0 = (uint32_t)t * kTile + 4u * (uint32_t)T;
            float x[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) x[c] = j0 + c < d ? exact_value(es, ge, i, j0 + c) : 0.f;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t j = j0 + c;
                bool hit = j < d && composite(sel_key(sk, x[c], j), j, ge.idx_bits) >= tc;
                if (skip_zeros) {
                    const bool zero = j < d && mag_key(x[c]) == 0u;
                    const uint64_t zm = __ballot(zero);
                    if (lane == 0 && zm) atomicAdd(&E.zeros, (uint32_t)__popcll(zm));
                    hit = hit && !zero;
                }
                const uint64_t hm = __ballot(hit);
                uint32_t at = 0;
                if (lane == 0 && hm) at = atomicAdd(&E.cnt[owner], (uint32_t)__popcll(hm));
                at = __builtin_amdgcn_readfirstlane(at) + __popcll(hm & ((1ull << lane) - 1ull));
                if (hit) E.stage[owner][at] = make_uint2(j, __float_as_uint(x[c]));
            }
        }
        __syncthreads();
        const uint32_t cnt[4] = {E.cnt[0], E.cnt[1], E.cnt[2], E.cnt[3]};
        if (tid == 0)
            tile_dir[(int64_t)i * ge.n_tiles + t] = make_uint4(run, cnt[0] | (cnt[1] << 16), cnt[2] | (cnt[3] << 16), E.zeros);
        uint2 *dst = cand + worker_base(ge, i) + run;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            for (uint32_t q = tid; q < cnt[w]; q += nt) dst[q] = E.stage[w][q];
            dst += cnt[w];
        }
        run += cnt[0] + cnt[1] + cnt[2] + cnt[3];
        __syncthreads();
        if (tid < 4) E.cnt[tid] = 0;
        if (tid == 0) E.zeros = 0;
        __syncthreads();
    }
}

__device__ __forceinline__ uint64_t exact_select(const ExactSource &es, const TkGeom &ge, int i, uint2 *__restrict__ cand,
                                                 uint4 *__restrict__ tile_dir, ResolveLds &L, ExactLds &E)
{
    const uint64_t tc = exact_threshold(es, ge, i, L);
    list_kept(es, ge, i, tc, cand, tile_dir, E);
    return tc;
}

// xs: the stored rows under error feedback with magnitude keys (where zeros are counted instead of listed and
// the threshold may lie among them), else null.  es: how the compressed vector is re-formed, for a worker whose
// lists did not fit.
__global__ __launch_bounds__(kResolveThreads) void tk_resolve(TkGeom ge, TkWorker *__restrict__ ws,
                                                              const uint64_t *__restrict__ dense,
                                                              const uint2 *__restrict__ dense_dir,
                                                              uint32_t *__restrict__ cursor,
                                                              uint32_t *__restrict__ cursor_b,
                                                              uint32_t *__restrict__ hist_full,
                                                              uint32_t *__restrict__ hist2,
                                                              const uint32_t *__restrict__ piece_bits,
                                                              uint2 *__restrict__ cand, uint4 *__restrict__ tile_dir,
                                                              const float *__restrict__ xs, ExactSource es)
{
    __shared__ ResolveLds L;
    // the piece table of the usual path and the staging lists of exact_select are never needed together
    union Either {
        struct {
            uint32_t rpre[kMaxPieces + 1];
            uint32_t rstart[kMaxPieces];
            uint32_t plist[kFew];        // pieces that hold an element with the first digit of Tc
            uint32_t n_plist;
        } pieces;
        ExactLds exact;
    };
    __shared__ Either U;
    uint32_t *rpre = U.pieces.rpre, *rstart = U.pieces.rstart;
    const int i = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const TkWorker w = ws[i];
    const int s_hi = (int)w.pshift + ge.idx_bits;
    uint64_t tc = (uint64_t)w.prefix << s_hi;
    const uint4 *dir_row = tile_dir + (int64_t)i * ge.n_tiles;
    if (w.overflow2) {
        tc = exact_select(es, ge, i, cand, tile_dir, L, U.exact);
        if (tid == 0) ws[i].whole = kExact;          // for the records (comp_ams_get_selection_info)
    } else if (w.whole == kZeroTail) {
        tc = zero_tail_threshold(dir_row, xs + (int64_t)i * ge.ld, ge, w.rank, L);
    } else if (!w.whole) {
        // tk_compact counted the first digit below the prefix while it copied: take its counts (and leave the
        // worker's row of hist2 empty for the next step)
        for (int b = tid; b < kBinsFirst; b += kResolveThreads) {
            uint32_t *at = hist2 + (int64_t)i * kBinsFirst + b;
            L.lh[b] = *at;
            *at = 0u;
        }
        const int pieces = ge.slices * ge.parts * 4;
        const uint64_t *wdense = dense + region_base(ge, i, 0);
        // exclusive prefix sum of the piece counts, two pieces per thread
        const uint2 a = (2 * tid < pieces) ? dense_dir[(int64_t)i * pieces + 2 * tid] : make_uint2(0u, 0u);
        const uint2 b = (2 * tid + 1 < pieces) ? dense_dir[(int64_t)i * pieces + 2 * tid + 1] : make_uint2(0u, 0u);
        uint32_t incl = a.y + b.y;
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
            const uint32_t up = __shfl_up(incl, off, kWave);
            if (lane >= off) incl += up;
        }
        if (lane == kWave - 1) L.part[wave] = incl;
        __syncthreads();
        uint32_t before = 0;
        for (int q = 0; q < wave; ++q) before += L.part[q];
        const uint32_t excl = before + incl - (a.y + b.y);
        if (2 * tid < pieces) {
            rpre[2 * tid] = excl;
            rstart[2 * tid] = a.x;
        }
        if (2 * tid + 1 < pieces) {
            rpre[2 * tid + 1] = excl + a.y;
            rstart[2 * tid + 1] = b.x;
        }
        if (tid == kResolveThreads - 1) rpre[pieces] = before + incl;   // threads past the pieces add 0
        __syncthreads();
        const uint32_t cnt = rpre[pieces];
        // Elements q[u] of the worker's dense set, found through the prefix sums of the piece counts: the piece of
        // q is the last one that starts at or before it.  The searches of a batch advance together, one bit of the
        // piece number per round and without branches, so that a round's LDS reads are independent: one search
        // after the other leaves a scan waiting on kScanUnroll chains of dependent LDS reads per batch.
        int top = 1;
        while (2 * top < pieces) top *= 2;
        auto fetch = [&](const uint32_t (&q)[kScanUnroll], uint64_t (&comp)[kScanUnroll]) {
            if (q[0] >= cnt) return;                       // nothing for this thread in the batch
            int r[kScanUnroll];
#pragma unroll
            for (int u = 0; u < kScanUnroll; ++u) r[u] = 0;
            for (int bit = top; bit > 0; bit >>= 1) {
                uint32_t start[kScanUnroll];
#pragma unroll
                for (int u = 0; u < kScanUnroll; ++u) start[u] = rpre[min(r[u] + bit, pieces)];   // rpre[pieces] = cnt
#pragma unroll
                for (int u = 0; u < kScanUnroll; ++u) r[u] = (start[u] <= q[u] && r[u] + bit < pieces) ? r[u] + bit : r[u];
            }
            uint32_t at[kScanUnroll];
#pragma unroll
            for (int u = 0; u < kScanUnroll; ++u) at[u] = rstart[r[u]] + (q[u] - rpre[r[u]]);
#pragma unroll
            for (int u = 0; u < kScanUnroll; ++u) comp[u] = q[u] < cnt ? wdense[at[u]] : 0ull;
        };
        if (xs != nullptr && w.prefix == 0u && w.rank > cnt)
            // the threshold bin is the one of the smallest keys and the k-th largest lies below its listed
            // (non-zero) elements: among the zeros
            tc = zero_tail_threshold(dir_row, xs + (int64_t)i * ge.ld, ge, w.rank - cnt, L);
        else {
            // The first digit below the prefix from tk_compact's counts.  Usually at most kFew elements carry it:
            // they sit in at most as many pieces, which the pieces' bitmaps name, so only those pieces are read
            // (a few hundred elements instead of the whole threshold bin) and the elements ranked directly.
            const int s_lo = s_hi - kFirstBits;
            find_rank_bin(L.lh, L.part, L.res, kBinsFirst, w.rank);          // barriers since L.lh was filled
            const uint32_t digit = L.res[0], left = L.res[2], rank1 = w.rank - L.res[1];
            const bool found = L.res[3] != 0u;
            const uint64_t prefix1 = ((uint64_t)w.prefix << kFirstBits) | digit;
            if (found && left == rank1) {
                tc = prefix1 << s_lo;                                         // all under this prefix are kept
            } else if (found && left <= (uint32_t)min(kFew, kResolveThreads)) {
                if (tid == 0) {
                    U.pieces.n_plist = 0;
                    L.n_few = 0;
                }
                __syncthreads();
                for (int p = tid; p < pieces; p += kResolveThreads) {
                    const uint32_t word = piece_bits[((int64_t)i * pieces + p) * kPieceWords + (digit >> 5)];
                    if ((word >> (digit & 31u)) & 1u) {
                        const uint32_t slot = atomicAdd(&U.pieces.n_plist, 1u);
                        if (slot < (uint32_t)kFew) U.pieces.plist[slot] = (uint32_t)p;     // always: see n_listed
                    }
                }
                __syncthreads();
                const uint32_t n_listed = min(U.pieces.n_plist, (uint32_t)kFew);   // <= left: each names an element
                for (uint32_t q = wave; q < n_listed; q += kResolveThreads / kWave) {
                    const uint32_t p = U.pieces.plist[q];
                    const uint32_t first = rstart[p], count = rpre[p + 1] - rpre[p];
                    for (uint32_t e = lane; e < count; e += kWave) {
                        const uint64_t comp = wdense[first + e];
                        if ((comp >> s_lo) == prefix1) {
                            const uint32_t slot = atomicAdd(&L.n_few, 1u);
                            if (slot < (uint32_t)kFew) L.few[slot] = comp;
                        }
                    }
                }
                __syncthreads();
                if ((uint32_t)tid < left) {
                    const uint64_t mine = L.few[tid];
                    uint32_t greater = 0;
                    for (uint32_t u = 0; u < left; ++u) greater += L.few[u] > mine ? 1u : 0u;
                    if (greater + 1 == rank1) L.tc_sh = mine;                 // comp values are unique: exactly one thread
                }
                __syncthreads();
                tc = L.tc_sh;
            } else {
                tc = resolve_digits(fetch, cnt, w.prefix, w.rank, s_hi, L, true);
            }
        }
    }
    if (tid < ge.slices) cursor[i * ge.slices + tid] = 0;      // tk_compact was their last reader (slices <= 1024 threads)
    if (w.relisted) {                                          // tk_pick was the last reader of the full histogram
        if (tid < ge.slices) cursor_b[i * ge.slices + tid] = 0;
        for (int q = tid; q < kBins1; q += kResolveThreads) hist_full[(int64_t)i * kBins1 + q] = 0;
    }
    if (tid == 0) finish_worker(ws, i, w, tc, ge, w.relisted != 0);
}


// ---------------------------------------------------------------------------------------------
// Short vectors (at most kSmallTiles tiles) under error feedback: the selection in one launch.
// On such a vector every kernel of the selection chain is a launch on an idle chip, and five of them cost more
// than the work.  The listing pass is tk_pass1 itself with a single candidate region per worker (few tiles share
// its cursor); then one workgroup per worker finds the threshold from the list by itself - the digits of Tc over
// the listed comp values, or, when the list does not hold the k-th largest (first step, a guess that was too high,
// a full region), by counting over the stored row (exact_select).  The tile directory and the list have the
// usual form, so tk_final and the getters follow unchanged.  (Finding the threshold inside the listing pass, by
// the workgroup that finishes a worker's last tile, was built and measured: the device-scope fences it needs on
// this multi-XCD part cost more than the launch they save - 21.6 us against 6 + 5.)
constexpr int kSmallTiles = 16;

// sge: the handle's geometry with slices = 1 and region_cap = all of a worker's space.  count: [n] entries listed
// (cleared here for the next step).
__global__ __launch_bounds__(kResolveThreads) void tk_small_select(TkGeom sge, TkWorker *__restrict__ ws,
                                                                   uint2 *__restrict__ cand, uint32_t *__restrict__ count,
                                                                   uint4 *__restrict__ tile_dir, const float *__restrict__ xs)
{
    __shared__ ResolveLds L;
    __shared__ ExactLds E;
    const int i = blockIdx.x;
    const int tid = threadIdx.x;
    const TkWorker w = ws[i];
    const SelKey sk = sel_key_of(sge.rand, sge.rand.step_now, i);
    const uint32_t total = count[i];
    const ExactSource es{kSrcStored, 0, xs, nullptr};
    uint64_t tc;
    bool missed = false;
    if (!w.overflow && total >= sge.k) {
        // every element at or above the guess is listed and there are at least k: Tc is the k-th largest of the
        // list (the comp value itself: a digit's bin may reach below the guess, where nothing is listed)
        const uint2 *list = cand + worker_base(sge, i);
        auto fetch = [&](const uint32_t (&q)[kScanUnroll], uint64_t (&comp)[kScanUnroll]) {
#pragma unroll
            for (int u = 0; u < kScanUnroll; ++u) {
                comp[u] = 0ull;
                if (q[u] < total) {
                    const uint2 e = list[q[u]];
                    comp[u] = composite(sel_key(sk, __uint_as_float(e.y), e.x), e.x, sge.idx_bits);
                }
            }
        };
        tc = resolve_digits<false>(fetch, total, 0ull, sge.k, 31 + sge.idx_bits, L);
    } else if (!w.overflow && !sk.on && w.guess == 0u) {
        // magnitude keys, every non-zero element is listed and they are fewer than k: the threshold lies among the
        // zeros, which the list leaves out - all candidates are kept, and Tc comes from counting over the row
        tc = exact_threshold(es, sge, i, L);
    } else {
        missed = true;
        tc = exact_select(es, sge, i, cand, tile_dir, L, E);
    }
    if (tid == 0) {
        ws[i].relisted = missed ? 1u : 0u;
        ws[i].whole = missed ? kExact : 0u;
        finish_worker(ws, i, w, tc, sge, missed);
        count[i] = 0;
    }
}

// CD-Adam (Algorithm 1): selection buffers of the server's own Top-k - the same structures as the
// workers', for a single vector.
struct TkSide {
    TkGeom ge;                 // n = 1
    TkWorker *ws;
    uint2 *cand;
    uint32_t *cursor;
    uint4 *tile_dir;
};

// Per tile: ghat_i += c_i (line 6) and ghat += mean of the c_i (line 8).  The server's vector
// w = ghat - gtilde (line 9) is then listed by tk_pass1<kPassDiff>.
__global__ __launch_bounds__(kThreads) void tk_merge(TkGeom ge, const TkWorker *__restrict__ ws,
                                                     const uint2 *__restrict__ cand,
                                                     const uint4 *__restrict__ tile_dir,
                                                     float *__restrict__ ghat_rows, float *__restrict__ ghat,
                                                     float n_workers)
{
    __shared__ float acc[kTile];
    const int t = blockIdx.x;
    const int64_t base = (int64_t)t * kTile;
    const int tid = threadIdx.x;
#pragma unroll
    for (int r = 0; r < 4; ++r) st4(acc + 4 * (tid + kThreads * r), make_float4(0.f, 0.f, 0.f, 0.f));
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    sum_kept_tile<true>(acc, ge, ws, cand, tile_dir, t, ghat_rows);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int l = 4 * (tid + kThreads * r);
        const float4 a = ld4(acc + l), gh = ld4(ghat + base + l);
        // padding coordinates: 0 + 0 / n; ghat moves only where some worker kept a coordinate
        st4_if_changed<false>(ghat + base + l,
                              make_float4(fadd(gh.x, fdiv(a.x, n_workers)), fadd(gh.y, fdiv(a.y, n_workers)),
                                          fadd(gh.z, fdiv(a.z, n_workers)), fadd(gh.w, fdiv(a.w, n_workers))), gh);
    }
}

// CD-Adam (Algorithm 1), lines 10 and 12-16: gtilde += c, c = the kept coordinates of w, then the
// AMSGrad update with gtilde.  Per tile; each wavefront handles its own coordinates.
template <bool kStreamState>
__global__ __launch_bounds__(kThreads) void tk_apply(TkSide sv, float *__restrict__ gtil, float *__restrict__ theta,
                                                     float *__restrict__ m, float *__restrict__ v,
                                                     float *__restrict__ vhat, AmsParams p)
{
    __shared__ float acc[kTile];
    const int t = blockIdx.x;
    const int64_t base = (int64_t)t * kTile;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int r = 0; r < 4; ++r) st4(acc + 4 * (tid + kThreads * r), make_float4(0.f, 0.f, 0.f, 0.f));
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    {
        const uint4 rec = sv.tile_dir[t];
        const uint32_t c[4] = {rec.y & 0xffffu, rec.y >> 16, rec.z & 0xffffu, rec.z >> 16};
        uint32_t start = rec.x;
        for (int q = 0; q < wave; ++q) start += c[q];
        const uint64_t tc = sv.ws[0].tc;
        const SelKey sk = sel_key_of(sv.ge.rand, sv.ws[0].step_word, 0);
        const uint2 *src = sv.cand + start;          // a single vector: its space starts the array
        for (uint32_t q = lane; q < c[wave]; q += kWave) {
            const uint2 e = src[q];
            const float x = __uint_as_float(e.y);
            if (composite(sel_key(sk, x, e.x), e.x, sv.ge.idx_bits) >= tc) acc[e.x - (uint32_t)base] = x;   // distinct coordinates
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
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
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int l = 4 * (tid + kThreads * r);
        const int64_t j = base + l;
        const float4 c4 = ld4(acc + l);
        // c is +0 where nothing was kept; gtilde + 0 = gtilde
        const float4 g4 = make_float4(fadd(gt[r].x, c4.x), fadd(gt[r].y, c4.y), fadd(gt[r].z, c4.z),
                                      fadd(gt[r].w, c4.w));
        amsgrad_update4(th[r], mm[r], vv[r], vh[r], g4, p);
        st4_if_changed<false>(gtil + j, g4, gt[r]);      // gtilde moves at the k kept coordinates only
        st4_state<kStreamState>(theta + j, th[r]);
        st4_state<kStreamState>(m + j, mm[r]);
        st4_state<kStreamState>(v + j, vv[r]);
        st4_state<kStreamState>(vhat + j, vh[r]);
    }
}

// Getter support -------------------------------------------------------------------------------

// e_i of one worker in its defined form, from the stored x and the pending threshold.
__global__ __launch_bounds__(kThreads) void tk_materialize_error(const float *xrow, TkGeom ge, int worker,
                                                                 const TkWorker *__restrict__ w, float *out)
{
    const int64_t j = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (j >= ge.d) return;
    const float x = xrow[j];
    const SelKey sk = sel_key_of(ge.rand, w->step_word, worker);
    out[j] = was_kept(kept_test(w->tc, ge.idx_bits), sel_key(sk, x, (uint32_t)j), (uint32_t)j) ? 0.f : x;
}

// The kept (index, value) pairs of one worker, in no particular order: candidates with
// comp >= Tc.  *count must be 0 on entry and ends at k.  One workgroup per tile; one atomic add
// per wavefront that found something.
__global__ __launch_bounds__(kThreads) void tk_gather_selected(TkGeom ge, int worker,
                                                               const TkWorker *__restrict__ ws,
                                                               const uint2 *__restrict__ cand,
                                                               const uint4 *__restrict__ tile_dir,
                                                               uint32_t *__restrict__ count,
                                                               uint32_t *__restrict__ out_idx,
                                                               float *__restrict__ out_val)
{
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x;
    const uint64_t tc = ws[worker].tc;
    const SelKey sk = sel_key_of(ge.rand, ws[worker].step_word, worker);
    const uint4 rec = tile_dir[(int64_t)worker * ge.n_tiles + t];
    const uint2 *src = cand + worker_base(ge, worker) + rec.x;
    const uint32_t total = (rec.y & 0xffffu) + (rec.y >> 16) + (rec.z & 0xffffu) + (rec.z >> 16);
    for (uint32_t q0 = 0; q0 < total; q0 += kThreads) {      // uniform over the workgroup
        const uint32_t q = q0 + threadIdx.x;
        uint2 c = make_uint2(0u, 0u);
        bool keep = false;
        if (q < total) {
            c = src[q];
            keep = composite(sel_key(sk, __uint_as_float(c.y), c.x), c.x, ge.idx_bits) >= tc;
        }
        const uint64_t km = __ballot(keep);
        if (km) {
            uint32_t at = 0;
            if (lane == 0) at = atomicAdd(count, (uint32_t)__popcll(km));
            at = __shfl(at, 0, kWave) + __popcll(km & ((1ull << lane) - 1ull));
            if (keep && at < ge.k) {
                out_idx[at] = c.x;
                out_val[at] = __uint_as_float(c.y);
            }
        }
    }
}

// The kept zeros of one worker's stored row when the threshold lies among them (key part of Tc is 0): the
// zeros at indices up to Tc's, appended to the pairs tk_gather_selected has written.
__global__ __launch_bounds__(kThreads) void tk_gather_zero_tail(const float *__restrict__ xrow, TkGeom ge,
                                                                const TkWorker *__restrict__ w,
                                                                uint32_t *__restrict__ count,
                                                                uint32_t *__restrict__ out_idx,
                                                                float *__restrict__ out_val)
{
    const KeptTest kt = kept_test(w->tc, ge.idx_bits);
    if (kt.tkey != 0u) return;
    const int64_t j = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const bool keep = j < ge.d && j <= (int64_t)kt.tj && mag_key(xrow[min(j, ge.d - 1)]) == 0u;
    const uint64_t km = __ballot(keep);
    if (km) {
        const int lane = threadIdx.x & 63;
        uint32_t at = 0;
        if (lane == 0) at = atomicAdd(count, (uint32_t)__popcll(km));
        at = __shfl(at, 0, kWave) + __popcll(km & ((1ull << lane) - 1ull));
        if (keep && at < ge.k) {
            out_idx[at] = (uint32_t)j;
            out_val[at] = xrow[j];
        }
    }
}

// Wire form of a sparse message: (index, value bits) pairs.
__global__ __launch_bounds__(kThreads) void tk_pack_pairs(const uint32_t *__restrict__ idx, const float *__restrict__ val,
                                                          uint32_t k, uint2 *__restrict__ out)
{
    const uint32_t r = blockIdx.x * kThreads + threadIdx.x;
    if (r < k) out[r] = make_uint2(idx[r], __float_as_uint(val[r]));
}

}  // namespace cams
