// Device helpers shared by the gfx950 kernels: vector loads of caller-owned gradient rows
// of any alignment, wavefront reductions with a fixed tree, and the AMSGrad update line.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

namespace cams {

// Which tile a workgroup works on.  The hardware hands the workgroups of a launch to the chip's eight XCDs in
// turn (linear workgroup id modulo 8), so with tile = block id every XCD walks over every page of a row.  With
// chunk > 0 the blocks are taken in groups of 8 * chunk, and inside a group XCD x works through the contiguous
// tiles [x * chunk, (x + 1) * chunk) of the group.  Such a grid has a multiple of 8 * chunk blocks in x
// (grid_blocks); blocks whose tile is past the last one leave at once.  chunk = 0: tile = block id.
__device__ __forceinline__ int tile_of_block(unsigned b, int chunk)
{
    if (chunk <= 0) return (int)b;
    const unsigned span = 8u * (unsigned)chunk, within = b % span;
    return (int)(b - within + (within & 7u) * (unsigned)chunk + (within >> 3));
}

constexpr int kWave = 64;          // CDNA wavefront
constexpr int kThreads = 256;      // workgroup size of every streaming kernel (4 waves)
constexpr int kTile = 4096;        // coordinates per tile; rows of library-owned arrays are padded to it

// fp32 operations with one IEEE rounding each.  The translation unit is built with
// -ffp-contract=off and the pragma below repeats it, so a*b+c is never fused; `/` and sqrtf are
// the correctly rounded forms (hipcc's default for fp32; the __fsqrt_rn intrinsic is NOT: it maps
// to the approximate native square root).
#pragma clang fp contract(off)
__device__ __forceinline__ float fadd(float a, float b) { return a + b; }
__device__ __forceinline__ float fsub(float a, float b) { return a - b; }
__device__ __forceinline__ float fmul(float a, float b) { return a * b; }
__device__ __forceinline__ float fdiv(float a, float b) { return a / b; }
__device__ __forceinline__ float fsqrt(float a) { return sqrtf(a); }

// Hyper-parameters of the AMSGrad recursion (Section 3), fp32, prepared on the host.
struct AmsParams {
    float beta1, beta2, omb1, omb2;   // omb = 1 - beta, rounded once to fp32
    float eps, lr;
    int32_t eps_mode;                 // 0: sqrt(vhat)+eps   1: sqrt(vhat+eps)
    float n_workers;                  // divisor of the server average
    int32_t stream_state;             // theta, m, v, vhat are loaded and stored as streams (non-temporal): the host
                                      // launches the kStreamState = true variants of the update kernels
};

// m, v, vhat, theta update on one coordinate; every operation rounds to fp32 on its own
// (no fused multiply-add).
__device__ __forceinline__ void amsgrad_update(float &theta, float &m, float &v, float &vhat, float gbar,
                                               const AmsParams &p)
{
    m = fadd(fmul(p.beta1, m), fmul(p.omb1, gbar));
    v = fadd(fmul(p.beta2, v), fmul(p.omb2, fmul(gbar, gbar)));
    vhat = fmaxf(vhat, v);
    float den = p.eps_mode ? fsqrt(fadd(vhat, p.eps)) : fadd(fsqrt(vhat), p.eps);
    theta = fsub(theta, fdiv(fmul(p.lr, m), den));
}

__device__ __forceinline__ void amsgrad_update4(float4 &th, float4 &m, float4 &v, float4 &vh, const float4 &g,
                                                const AmsParams &p)
{
    amsgrad_update(th.x, m.x, v.x, vh.x, g.x, p);
    amsgrad_update(th.y, m.y, v.y, vh.y, g.y, p);
    amsgrad_update(th.z, m.z, v.z, vh.z, g.z, p);
    amsgrad_update(th.w, m.w, v.w, vh.w, g.w, p);
}

typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));

// Streaming (read-once) loads: the gradient is never read again by the same step.
__device__ __forceinline__ float4 stream_load4(const float *p)
{
    const v4f t = __builtin_nontemporal_load(reinterpret_cast<const v4f *>(p));
    return make_float4(t.x, t.y, t.z, t.w);
}
__device__ __forceinline__ float2 stream_load2(const float *p)
{
    const v2f t = __builtin_nontemporal_load(reinterpret_cast<const v2f *>(p));
    return make_float2(t.x, t.y);
}

// Four consecutive gradient coordinates row[j..j+3], j a multiple of 4.  The row is caller
// memory of length d whose start may be 16-, 8- or 4-byte aligned (row i of a dense [n][d]
// array starts at i*d floats); coordinates at or beyond d read as zero.  The alignment test is
// uniform across a wavefront.
__device__ __forceinline__ float4 load_grad4(const float *__restrict__ row, int64_t j, int64_t d)
{
    const float *p = row + j;
    if (j + 4 <= d) {
        const uintptr_t a = reinterpret_cast<uintptr_t>(p) & 15u;
        if (a == 0) return stream_load4(p);
        if (a == 8) {
            const float2 lo = stream_load2(p);
            const float2 hi = stream_load2(p + 2);
            return make_float4(lo.x, lo.y, hi.x, hi.y);
        }
        return make_float4(p[0], p[1], p[2], p[3]);
    }
    float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
    if (j < d) r.x = p[0];
    if (j + 1 < d) r.y = p[1];
    if (j + 2 < d) r.z = p[2];
    if (j + 3 < d) r.w = p[3];
    return r;
}

// Gradients handed over as bfloat16 (the upper 16 bits of the fp32 value): widened exactly, so every
// formula downstream sees the same fp32 numbers as with an fp32 copy of them.  Rows start at any 2-byte
// alignment; 8-/4-/2-byte aligned groups of four take a 64-/32-/16-bit load path.
typedef uint32_t v2u __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float bf16_to_float(uint32_t h) { return __uint_as_float(h << 16); }

__device__ __forceinline__ float4 load_grad4(const uint16_t *__restrict__ row, int64_t j, int64_t d)
{
    const uint16_t *p = row + j;
    if (j + 4 <= d) {
        const uintptr_t a = reinterpret_cast<uintptr_t>(p) & 7u;
        if (a == 0) {
            const v2u t = __builtin_nontemporal_load(reinterpret_cast<const v2u *>(p));
            return make_float4(__uint_as_float(t.x << 16), __uint_as_float(t.x & 0xffff0000u),
                               __uint_as_float(t.y << 16), __uint_as_float(t.y & 0xffff0000u));
        }
        if (a == 4) {
            const uint32_t lo = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(p));
            const uint32_t hi = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(p + 2));
            return make_float4(__uint_as_float(lo << 16), __uint_as_float(lo & 0xffff0000u),
                               __uint_as_float(hi << 16), __uint_as_float(hi & 0xffff0000u));
        }
        return make_float4(bf16_to_float(p[0]), bf16_to_float(p[1]), bf16_to_float(p[2]), bf16_to_float(p[3]));
    }
    float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
    if (j < d) r.x = bf16_to_float(p[0]);
    if (j + 1 < d) r.y = bf16_to_float(p[1]);
    if (j + 2 < d) r.z = bf16_to_float(p[2]);
    if (j + 3 < d) r.w = bf16_to_float(p[3]);
    return r;
}

// Gradients handed over as IEEE half precision: same layout and load paths as bfloat16, widened exactly
// by the hardware conversion.  The wrapper type only tells the two 16-bit formats apart.
struct f16bits {
    uint16_t v;
};
static_assert(sizeof(f16bits) == 2, "f16bits is a plain 16-bit value");

__device__ __forceinline__ float f16_to_float(uint32_t h) { return __half2float(__ushort_as_half((unsigned short)h)); }

__device__ __forceinline__ float4 load_grad4(const f16bits *__restrict__ row, int64_t j, int64_t d)
{
    const uint16_t *p = reinterpret_cast<const uint16_t *>(row) + j;
    if (j + 4 <= d) {
        const uintptr_t a = reinterpret_cast<uintptr_t>(p) & 7u;
        uint32_t lo, hi;
        if (a == 0) {
            const v2u t = __builtin_nontemporal_load(reinterpret_cast<const v2u *>(p));
            lo = t.x;
            hi = t.y;
        } else if (a == 4) {
            lo = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(p));
            hi = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(p + 2));
        } else {
            lo = (uint32_t)p[0] | ((uint32_t)p[1] << 16);
            hi = (uint32_t)p[2] | ((uint32_t)p[3] << 16);
        }
        return make_float4(f16_to_float(lo & 0xffffu), f16_to_float(lo >> 16), f16_to_float(hi & 0xffffu),
                           f16_to_float(hi >> 16));
    }
    float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
    if (j < d) r.x = f16_to_float(p[0]);
    if (j + 1 < d) r.y = f16_to_float(p[1]);
    if (j + 2 < d) r.z = f16_to_float(p[2]);
    if (j + 3 < d) r.w = f16_to_float(p[3]);
    return r;
}

__device__ __forceinline__ float4 ld4(const float *p) { return *reinterpret_cast<const float4 *>(p); }
__device__ __forceinline__ void st4(float *p, const float4 &v) { *reinterpret_cast<float4 *>(p) = v; }

// Streaming (write-once) store: what a step writes to the stored rows and to theta, m, v, vhat is not
// read again before the next step.  Marking these accesses (and the matching loads) non-temporal keeps
// them from displacing what the step does reuse - candidates, sign words, scales - and measured 7 - 11 %
// off the whole step on the large workloads.
__device__ __forceinline__ void st4_stream(float *p, const float4 &v)
{
    const v4f t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, reinterpret_cast<v4f *>(p));
}
// A stored row (error memory / Markov sequence) is read once per step.  Rows that together are far
// larger than the caches cannot survive from one step to the next, so they are loaded as a stream; small
// ones (stream == 0) are loaded normally, since part of them is still cached from the step before.  (They
// are stored as a stream in both cases: that measured faster or equal at every size.)
__device__ __forceinline__ float4 ld4_row(const float *p, int stream) { return stream ? stream_load4(p) : ld4(p); }
// theta, m, v, vhat are read and written once per step: streamed when they are too large to stay in the
// memory-side cache until the next step (AmsParams::stream_state).
// A compile-time choice: with a run-time flag the compiler merges the two stores and drops the hint.
template <bool kStream>
__device__ __forceinline__ float4 ld4_state(const float *p)
{
    if constexpr (kStream) return stream_load4(p); else return ld4(p);
}
template <bool kStream>
__device__ __forceinline__ void st4_state(float *p, const float4 &v)
{
    if constexpr (kStream) st4_stream(p, v); else st4(p, v);
}

// st4_state (kStream) or st4, unless the location already holds v: `old` is what this thread loaded from p.  Skipping such a
// store leaves memory as it is, so results are the same bit for bit.  Lanes that share a line of kLineLanes * 16
// bytes decide together, so that a line is written whole or not at all.  All lanes of the wavefront must call
// this together (it uses a ballot).
constexpr int kLineLanes = 8;
template <bool kStream>
__device__ __forceinline__ void st4_if_changed(float *p, const float4 &v, const float4 &old)
{
    const bool changed = __float_as_uint(v.x) != __float_as_uint(old.x) || __float_as_uint(v.y) != __float_as_uint(old.y) ||
                         __float_as_uint(v.z) != __float_as_uint(old.z) || __float_as_uint(v.w) != __float_as_uint(old.w);
    const uint64_t b = __ballot(changed);
    const int lane = threadIdx.x & (kWave - 1);
    if ((b >> (lane & ~(kLineLanes - 1))) & ((1ull << kLineLanes) - 1ull)) st4_state<kStream>(p, v);
}

__device__ __forceinline__ uint32_t mag_key(float x) { return __float_as_uint(x) & 0x7fffffffu; }

// Sum over the 64 lanes with a fixed butterfly; every lane receives the same result, and the
// result depends only on the lane values, not on timing.
__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// Sum over a 256-thread workgroup in a fixed order; valid in every thread.  `scratch` holds
// at least 4 doubles of LDS.  Contains two barriers.
__device__ __forceinline__ double block_sum(double v, double *scratch)
{
    v = wave_sum(v);
    const int wave = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) scratch[wave] = v;
    __syncthreads();
    return ((scratch[0] + scratch[1]) + scratch[2]) + scratch[3];
}

// Plain streaming copy, 16 bytes per lane, four independent loads per thread, one 16 KB piece per
// workgroup, non-temporal on both sides: the yardstick for the HBM counters (it moves exactly the bytes it
// is given) and for the bandwidth a simple kernel reaches on this chip.  chunk: tile_of_block's, over the
// pieces; blocks past the last piece do nothing.
__global__ __launch_bounds__(kThreads) void probe_copy(float *__restrict__ dst, const float *__restrict__ src,
                                                       int64_t vecs, int chunk)
{
    const int64_t q0 = (int64_t)tile_of_block(blockIdx.x, chunk) * (4 * kThreads) + threadIdx.x;
    float4 v[4];
#pragma unroll
    for (int r = 0; r < 4; ++r)
        if (q0 + r * kThreads < vecs) v[r] = stream_load4(src + 4 * (q0 + r * kThreads));
#pragma unroll
    for (int r = 0; r < 4; ++r)
        if (q0 + r * kThreads < vecs) st4_stream(dst + 4 * (q0 + r * kThreads), v[r]);
}

// The access pattern of the streaming passes with nothing else: x[i][j] = x[i][j] + g[i][j] in place, rows of d
// floats (d a multiple of 4, rows 16-byte aligned), one 16 KB piece of a row per workgroup, non-temporal on all
// three streams.  What this reaches is the practical ceiling for a kernel that reads two arrays and writes one of
// them back on this chip; the passes are measured against it.  chunk: tile_of_block's, over the pieces of a row.
__global__ __launch_bounds__(kThreads) void probe_update(float *__restrict__ x, const float *__restrict__ g, int64_t d,
                                                         int pieces, int chunk)
{
    const int t = tile_of_block(blockIdx.x, chunk);
    if (t >= pieces) return;
    const int64_t row = (int64_t)blockIdx.y * d;
    const int64_t j0 = (int64_t)t * kTile + 4 * threadIdx.x;
    float4 a[4], b[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int64_t j = j0 + 4 * kThreads * r;
        if (j < d) {
            a[r] = stream_load4(g + row + j);
            b[r] = stream_load4(x + row + j);
        }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int64_t j = j0 + 4 * kThreads * r;
        if (j < d) st4_stream(x + row + j, make_float4(fadd(a[r].x, b[r].x), fadd(a[r].y, b[r].y), fadd(a[r].z, b[r].z),
                                                       fadd(a[r].w, b[r].w)));
    }
}

}  // namespace cams
