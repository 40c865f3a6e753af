// Host side of the C ABI declared in include/comp_ams.h: handle, argument validation, device
// memory, kernel launches.  Every step of the method runs in the kernels of the two *_kernels.h
// files; nothing is computed on the host.
#include "../../include/comp_ams.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <utility>
#include <vector>

#include "blocksign_kernels.h"
#include "topk_kernels.h"

using namespace cams;

namespace {

thread_local std::string g_create_error;

}  // namespace

struct comp_ams {
    int64_t d = 0, ld = 0;
    int32_t n = 0, compressor = 0;
    int64_t k = 0, block = 0;
    AmsParams params{};
    int device = 0;
    hipStream_t stream = nullptr;
    uint64_t steps = 0;
    std::string err;
    std::vector<void *> allocs;

    float *theta = nullptr, *m = nullptr, *v = nullptr, *vhat = nullptr, *e = nullptr;

    // block sign
    BsTable tb{};
    std::vector<void *> tb_allocs;
    double *partial = nullptr;
    float *scales = nullptr;

    // Top-k
    TkGeom ge{};
    TkWorker *ws = nullptr;
    uint32_t *hist1 = nullptr, *hist2 = nullptr;
    uint16_t *cand_idx = nullptr;
    float *cand_val = nullptr;
    uint32_t *cand_cnt = nullptr, *sel_cnt = nullptr;
    uint32_t *sel_offs = nullptr, *sel_out_idx = nullptr;
    float *sel_out_val = nullptr;
    std::vector<std::pair<int, int>> levels;   // (s_hi, s_lo) of each digit after the first
    int grid_rows = 1;                         // workgroups per worker in the row-streaming kernels
    int grid_scan = 1;

    // optional per-kernel timing with HIP events on the step's stream
    bool prof_on = false;
    std::vector<std::vector<std::pair<hipEvent_t, hipEvent_t>>> prof;   // [slot] -> recorded pairs
};

namespace {

enum ProfSlot { P_BS_PARTIAL, P_BS_SCALE, P_BS_APPLY, P_TK_PASS1, P_TK_FINDBIN, P_TK_COLLECT, P_TK_SCAN, P_TK_FIND,
                P_TK_FINAL, P_SLOTS };
const char *const kProfNames[P_SLOTS] = {"bs_partial", "bs_scale", "bs_apply", "tk_pass1", "tk_findbin",
                                         "tk_collect", "tk_scan", "tk_find", "tk_final"};

// Runs `launch` (one kernel launch on st); with profiling on, brackets it with two events.
template <typename F>
void launch_timed(comp_ams *h, int slot, hipStream_t st, F &&launch)
{
    if (!h->prof_on) {
        launch();
        return;
    }
    hipEvent_t a = nullptr, b = nullptr;
    if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) {
        if (a) (void)hipEventDestroy(a);
        launch();
        return;
    }
    (void)hipEventRecord(a, st);
    launch();
    (void)hipEventRecord(b, st);
    h->prof[slot].emplace_back(a, b);
}

void prof_clear(comp_ams *h)
{
    for (auto &slot : h->prof)
        for (auto &pr : slot) {
            (void)hipEventDestroy(pr.first);
            (void)hipEventDestroy(pr.second);
        }
    h->prof.assign(P_SLOTS, {});
}

int fail(comp_ams *h, int code, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (h) h->err = buf; else g_create_error = buf;
    return code;
}

#define HIP_TRY(h, call)                                                                              \
    do {                                                                                              \
        hipError_t err__ = (call);                                                                    \
        if (err__ != hipSuccess) {                                                                    \
            int code__ = (err__ == hipErrorOutOfMemory) ? COMP_AMS_ENOMEM : COMP_AMS_EDEVICE;         \
            return fail(h, code__, "%s failed: %s", #call, hipGetErrorString(err__));                 \
        }                                                                                             \
    } while (0)

int dev_alloc(comp_ams *h, std::vector<void *> &owner, void **out, size_t bytes, bool zero)
{
    void *p = nullptr;
    if (bytes == 0) bytes = 16;
    HIP_TRY(h, hipMalloc(&p, bytes));
    owner.push_back(p);
    if (zero) HIP_TRY(h, hipMemset(p, 0, bytes));
    *out = p;
    return COMP_AMS_OK;
}

template <typename T>
int dev_alloc_t(comp_ams *h, std::vector<void *> &owner, T **out, size_t count, bool zero = true)
{
    return dev_alloc(h, owner, reinterpret_cast<void **>(out), count * sizeof(T), zero);
}

void free_all(std::vector<void *> &owner)
{
    for (void *p : owner) (void)hipFree(p);
    owner.clear();
}

// Builds the device block table from host offsets[0..nb] (already validated).
int build_block_table(comp_ams *h, const std::vector<int64_t> &off, int64_t uniform)
{
    const int nb = (int)off.size() - 1;
    std::vector<int32_t> off32(nb + 1), seg_lo, seg_hi, block_seg0(nb + 1);
    for (int b = 0; b <= nb; ++b) off32[b] = (int32_t)off[b];
    for (int b = 0; b < nb; ++b) {
        block_seg0[b] = (int32_t)seg_lo.size();
        for (int64_t s = off[b]; s < off[b + 1]; s += kTile) {
            seg_lo.push_back((int32_t)s);
            seg_hi.push_back((int32_t)std::min<int64_t>(s + kTile, off[b + 1]));
        }
    }
    block_seg0[nb] = (int32_t)seg_lo.size();
    const int64_t n_apply_tiles = h->ld / 1024;
    std::vector<int32_t> tile_block(n_apply_tiles);
    {
        int b = 0;
        for (int64_t t = 0; t < n_apply_tiles; ++t) {
            const int64_t j = t * 1024;
            while (b + 1 < nb && j >= off[b + 1]) ++b;
            tile_block[t] = b;
        }
    }
    std::vector<void *> fresh;
    int32_t *d_off = nullptr, *d_lo = nullptr, *d_hi = nullptr, *d_s0 = nullptr, *d_tb = nullptr;
    double *d_partial = nullptr;
    float *d_scales = nullptr;
    int rc;
    auto upload = [&](int32_t **dst, const std::vector<int32_t> &src) -> int {
        int r = dev_alloc_t(h, fresh, dst, src.size(), false);
        if (r != COMP_AMS_OK) return r;
        HIP_TRY(h, hipMemcpy(*dst, src.data(), src.size() * sizeof(int32_t), hipMemcpyHostToDevice));
        return COMP_AMS_OK;
    };
    if ((rc = upload(&d_off, off32)) || (rc = upload(&d_lo, seg_lo)) || (rc = upload(&d_hi, seg_hi)) ||
        (rc = upload(&d_s0, block_seg0)) || (rc = upload(&d_tb, tile_block)) ||
        (rc = dev_alloc_t(h, fresh, &d_partial, (size_t)h->n * seg_lo.size())) ||
        (rc = dev_alloc_t(h, fresh, &d_scales, (size_t)h->n * nb))) {
        free_all(fresh);
        return rc;
    }
    free_all(h->tb_allocs);
    h->tb_allocs = std::move(fresh);
    h->tb.offsets = d_off;
    h->tb.seg_lo = d_lo;
    h->tb.seg_hi = d_hi;
    h->tb.block_seg0 = d_s0;
    h->tb.tile_block = d_tb;
    h->tb.n_blocks = nb;
    h->tb.n_segs = (int32_t)seg_lo.size();
    h->tb.uniform = (int32_t)std::min<int64_t>(uniform, INT32_MAX);
    h->partial = d_partial;
    h->scales = d_scales;
    return COMP_AMS_OK;
}

int check_handle(comp_ams *h)
{
    if (!h) return fail(nullptr, COMP_AMS_EINVAL, "handle is NULL");
    hipError_t e = hipSetDevice(h->device);
    if (e != hipSuccess) return fail(h, COMP_AMS_EDEVICE, "hipSetDevice(%d) failed: %s", h->device, hipGetErrorString(e));
    return COMP_AMS_OK;
}

int copy_out(comp_ams *h, float *dst, const float *src_dev, size_t count, int on_device)
{
    if (!dst) return fail(h, COMP_AMS_EINVAL, "output pointer is NULL");
    HIP_TRY(h, hipMemcpyAsync(dst, src_dev, count * sizeof(float),
                              on_device ? hipMemcpyDeviceToDevice : hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    return COMP_AMS_OK;
}

int copy_in(comp_ams *h, float *dst_dev, const float *src, size_t count, int on_device)
{
    HIP_TRY(h, hipMemcpyAsync(dst_dev, src, count * sizeof(float),
                              on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    return COMP_AMS_OK;
}

int step_blocksign(comp_ams *h, const float *g, hipStream_t st)
{
    const BsTable &tb = h->tb;
    launch_timed(h, P_BS_PARTIAL, st, [&] {
        bs_partial<<<dim3(tb.n_segs, h->n), kThreads, 0, st>>>(g, h->e, h->d, h->ld, tb, h->partial);
    });
    launch_timed(h, P_BS_SCALE, st, [&] {
        bs_scale<<<dim3(tb.n_blocks, h->n), kWave, 0, st>>>(h->partial, tb, h->scales);
    });
    launch_timed(h, P_BS_APPLY, st, [&] {
        bs_apply<<<dim3((unsigned)(h->ld / 1024)), kThreads, 0, st>>>(g, h->e, h->d, h->ld, h->n, tb, h->scales,
                                                                      h->theta, h->m, h->v, h->vhat, h->params);
    });
    return COMP_AMS_OK;
}

int step_topk(comp_ams *h, const float *g, hipStream_t st)
{
    const TkGeom &ge = h->ge;
    const dim3 rows(h->grid_rows, h->n);
    launch_timed(h, P_TK_PASS1, st, [&] {
        tk_pass1<<<rows, kThreads, 0, st>>>(g, h->e, ge, h->ws, h->hist1, h->cand_idx, h->cand_cnt);
    });
    launch_timed(h, P_TK_FINDBIN, st, [&] { tk_findbin<<<h->n, kThreads, 0, st>>>(ge, h->ws, h->hist1); });
    launch_timed(h, P_TK_COLLECT, st, [&] {
        tk_collect<<<rows, kThreads, 0, st>>>(h->e, ge, h->ws, h->cand_idx, h->cand_cnt);
    });
    for (const auto &lv : h->levels) {
        launch_timed(h, P_TK_SCAN, st, [&] {
            tk_scan<<<dim3(h->grid_scan, h->n), kThreads, 0, st>>>(h->e, ge, h->ws, h->cand_idx, h->cand_cnt,
                                                                  h->hist2, lv.first, lv.second);
        });
        launch_timed(h, P_TK_FIND, st, [&] {
            tk_find<<<h->n, kThreads, 0, st>>>(ge, h->ws, h->hist2, lv.first, lv.second);
        });
    }
    launch_timed(h, P_TK_FINAL, st, [&] {
        tk_final<<<ge.n_tiles, kThreads, 0, st>>>(h->e, ge, h->ws, h->cand_idx, h->cand_val, h->cand_cnt,
                                                  h->sel_cnt, h->theta, h->m, h->v, h->vhat, h->params);
    });
    return COMP_AMS_OK;
}

}  // namespace

extern "C" {

int comp_ams_create(comp_ams_t **out, int64_t d, int32_t n, int32_t compressor, int64_t k_or_block, float beta1,
                    float beta2, float eps, float lr)
{
    if (!out) return fail(nullptr, COMP_AMS_EINVAL, "out is NULL");
    if (d < 1 || d >= (int64_t)1 << 31) return fail(nullptr, COMP_AMS_EINVAL, "d=%lld must be in [1, 2^31)", (long long)d);
    if (n < 1 || n > 65535) return fail(nullptr, COMP_AMS_EINVAL, "n=%d must be in [1, 65535]", n);
    if ((int64_t)n * d >= (int64_t)1 << 40) return fail(nullptr, COMP_AMS_EINVAL, "n*d must be below 2^40");
    if (compressor != COMP_AMS_TOPK && compressor != COMP_AMS_BLOCKSIGN)
        return fail(nullptr, COMP_AMS_EINVAL, "unknown compressor %d", compressor);
    if (compressor == COMP_AMS_TOPK && (k_or_block < 1 || k_or_block > d))
        return fail(nullptr, COMP_AMS_EINVAL, "Top-k needs 1 <= k <= d, got k=%lld d=%lld", (long long)k_or_block, (long long)d);
    if (compressor == COMP_AMS_BLOCKSIGN && k_or_block < 1)
        return fail(nullptr, COMP_AMS_EINVAL, "block length %lld must be >= 1", (long long)k_or_block);
    if (!(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f))
        return fail(nullptr, COMP_AMS_EINVAL, "beta1, beta2 must be in [0, 1)");
    if (!(eps > 0.f) || !std::isfinite(eps)) return fail(nullptr, COMP_AMS_EINVAL, "eps must be positive and finite");
    if (!(lr > 0.f) || !std::isfinite(lr)) return fail(nullptr, COMP_AMS_EINVAL, "lr must be positive and finite");

    comp_ams *h = new (std::nothrow) comp_ams;
    if (!h) return fail(nullptr, COMP_AMS_ENOMEM, "host allocation failed");
    h->d = d;
    h->n = n;
    h->compressor = compressor;
    h->ld = (d + kTile - 1) / kTile * kTile;
    h->params.beta1 = beta1;
    h->params.beta2 = beta2;
    h->params.omb1 = 1.0f - beta1;
    h->params.omb2 = 1.0f - beta2;
    h->params.eps = eps;
    h->params.lr = lr;
    h->params.eps_mode = 0;
    h->params.n_workers = (float)n;
    h->prof.assign(P_SLOTS, {});

    auto bail = [&](int rc) {
        g_create_error = h->err;
        free_all(h->allocs);
        free_all(h->tb_allocs);
        delete h;
        return rc;
    };
    {
        hipError_t e = hipGetDevice(&h->device);
        if (e != hipSuccess) {
            fail(h, COMP_AMS_EDEVICE, "hipGetDevice failed: %s", hipGetErrorString(e));
            return bail(COMP_AMS_EDEVICE);
        }
    }
    int rc;
    const size_t ld = (size_t)h->ld;
    if ((rc = dev_alloc_t(h, h->allocs, &h->theta, ld)) || (rc = dev_alloc_t(h, h->allocs, &h->m, ld)) ||
        (rc = dev_alloc_t(h, h->allocs, &h->v, ld)) || (rc = dev_alloc_t(h, h->allocs, &h->vhat, ld)) ||
        (rc = dev_alloc_t(h, h->allocs, &h->e, ld * (size_t)n)))
        return bail(rc);

    if (compressor == COMP_AMS_BLOCKSIGN) {
        const int64_t B = std::min<int64_t>(k_or_block, d);
        h->block = B;
        std::vector<int64_t> off;
        for (int64_t s = 0; s < d; s += B) off.push_back(s);
        off.push_back(d);
        if ((rc = build_block_table(h, off, B))) return bail(rc);
    } else {
        h->k = k_or_block;
        TkGeom &ge = h->ge;
        ge.d = d;
        ge.ld = h->ld;
        ge.n = n;
        ge.n_tiles = (int32_t)(h->ld / kTile);
        ge.k = (uint32_t)k_or_block;
        int ib = 1;
        while (((int64_t)1 << ib) < d) ++ib;
        ge.idx_bits = ib;
        for (int s_hi = kShift1 + ib; s_hi > 0;) {
            const int s_lo = std::max(s_hi - kDigitBits, 0);
            h->levels.emplace_back(s_hi, s_lo);
            s_hi = s_lo;
        }
        h->grid_rows = (int)std::min<int64_t>(ge.n_tiles, std::max(1, 2048 / n));
        h->grid_scan = (int)std::min<int64_t>((ge.n_tiles + 3) / 4, std::max(1, 2048 / n));
        const size_t segs = (size_t)n * ge.n_tiles;
        if ((rc = dev_alloc_t(h, h->allocs, &h->ws, (size_t)n)) ||
            (rc = dev_alloc_t(h, h->allocs, &h->hist1, (size_t)n * kBins1)) ||
            (rc = dev_alloc_t(h, h->allocs, &h->hist2, (size_t)n * kBins2)) ||
            (rc = dev_alloc_t(h, h->allocs, &h->cand_idx, segs * kTile, false)) ||
            (rc = dev_alloc_t(h, h->allocs, &h->cand_val, segs * kTile, false)) ||
            (rc = dev_alloc_t(h, h->allocs, &h->cand_cnt, segs)) ||
            (rc = dev_alloc_t(h, h->allocs, &h->sel_cnt, segs)) ||
            (rc = dev_alloc_t(h, h->allocs, &h->sel_offs, (size_t)ge.n_tiles)) ||
            (rc = dev_alloc_t(h, h->allocs, &h->sel_out_idx, (size_t)ge.k)) ||
            (rc = dev_alloc_t(h, h->allocs, &h->sel_out_val, (size_t)ge.k)))
            return bail(rc);
        std::vector<TkWorker> init((size_t)n);
        for (auto &w : init) {
            std::memset(&w, 0, sizeof w);
            w.guess = kNoGuess;
        }
        hipError_t e = hipMemcpy(h->ws, init.data(), init.size() * sizeof(TkWorker), hipMemcpyHostToDevice);
        if (e != hipSuccess) {
            fail(h, COMP_AMS_EDEVICE, "hipMemcpy failed: %s", hipGetErrorString(e));
            return bail(COMP_AMS_EDEVICE);
        }
    }
    {
        hipError_t e = hipDeviceSynchronize();
        if (e != hipSuccess) {
            fail(h, COMP_AMS_EDEVICE, "hipDeviceSynchronize failed: %s", hipGetErrorString(e));
            return bail(COMP_AMS_EDEVICE);
        }
    }
    *out = h;
    return COMP_AMS_OK;
}

void comp_ams_destroy(comp_ams_t *h)
{
    if (!h) return;
    if (hipSetDevice(h->device) == hipSuccess) {
        (void)hipStreamSynchronize(h->stream);
        prof_clear(h);
        free_all(h->allocs);
        free_all(h->tb_allocs);
    }
    delete h;
}

int comp_ams_set_blocks(comp_ams_t *h, const int64_t *offsets_host, int32_t n_blocks)
{
    int rc = check_handle(h);
    if (rc) return rc;
    if (h->compressor != COMP_AMS_BLOCKSIGN) return fail(h, COMP_AMS_ESTATE, "set_blocks needs a BLOCKSIGN handle");
    if (!offsets_host) return fail(h, COMP_AMS_EINVAL, "offsets is NULL");
    if (n_blocks < 1 || (int64_t)n_blocks > h->d) return fail(h, COMP_AMS_EINVAL, "n_blocks=%d must be in [1, d]", n_blocks);
    if (offsets_host[0] != 0 || offsets_host[n_blocks] != h->d)
        return fail(h, COMP_AMS_EINVAL, "offsets must start at 0 and end at d");
    for (int b = 0; b < n_blocks; ++b)
        if (offsets_host[b + 1] <= offsets_host[b]) return fail(h, COMP_AMS_EINVAL, "offsets must be strictly increasing (block %d)", b);
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    std::vector<int64_t> off(offsets_host, offsets_host + n_blocks + 1);
    return build_block_table(h, off, 0);
}

int comp_ams_set_theta(comp_ams_t *h, const float *theta, int on_device)
{
    int rc = check_handle(h);
    if (rc) return rc;
    if (!theta) return fail(h, COMP_AMS_EINVAL, "theta is NULL");
    return copy_in(h, h->theta, theta, (size_t)h->d, on_device);
}

int comp_ams_set_lr(comp_ams_t *h, float lr)
{
    if (!h) return fail(nullptr, COMP_AMS_EINVAL, "handle is NULL");
    if (!(lr > 0.f) || !std::isfinite(lr)) return fail(h, COMP_AMS_EINVAL, "lr must be positive and finite");
    h->params.lr = lr;
    return COMP_AMS_OK;
}

int comp_ams_set_eps_mode(comp_ams_t *h, int32_t mode)
{
    if (!h) return fail(nullptr, COMP_AMS_EINVAL, "handle is NULL");
    if (mode != 0 && mode != 1) return fail(h, COMP_AMS_EINVAL, "eps mode must be 0 or 1");
    h->params.eps_mode = mode;
    return COMP_AMS_OK;
}

int comp_ams_step(comp_ams_t *h, const float *grads_dev, void *hip_stream)
{
    int rc = check_handle(h);
    if (rc) return rc;
    if (!grads_dev) return fail(h, COMP_AMS_EINVAL, "grads is NULL");
    if (reinterpret_cast<uintptr_t>(grads_dev) & 3u) return fail(h, COMP_AMS_EINVAL, "grads must be 4-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (st != h->stream) {
        // work of earlier steps on another stream must be finished before this stream touches the state
        HIP_TRY(h, hipStreamSynchronize(h->stream));
        h->stream = st;
    }
    rc = (h->compressor == COMP_AMS_TOPK) ? step_topk(h, grads_dev, st) : step_blocksign(h, grads_dev, st);
    if (rc) return rc;
    HIP_TRY(h, hipGetLastError());
    ++h->steps;
    return COMP_AMS_OK;
}

int comp_ams_get_theta(comp_ams_t *h, float *out, int on_device)
{
    int rc = check_handle(h);
    return rc ? rc : copy_out(h, out, h->theta, (size_t)h->d, on_device);
}
int comp_ams_get_m(comp_ams_t *h, float *out, int on_device)
{
    int rc = check_handle(h);
    return rc ? rc : copy_out(h, out, h->m, (size_t)h->d, on_device);
}
int comp_ams_get_v(comp_ams_t *h, float *out, int on_device)
{
    int rc = check_handle(h);
    return rc ? rc : copy_out(h, out, h->v, (size_t)h->d, on_device);
}
int comp_ams_get_vhat(comp_ams_t *h, float *out, int on_device)
{
    int rc = check_handle(h);
    return rc ? rc : copy_out(h, out, h->vhat, (size_t)h->d, on_device);
}

int comp_ams_get_error(comp_ams_t *h, int32_t worker, float *out, int on_device)
{
    int rc = check_handle(h);
    if (rc) return rc;
    if (worker < 0 || worker >= h->n) return fail(h, COMP_AMS_EINVAL, "worker %d out of [0, %d)", worker, h->n);
    return copy_out(h, out, h->e + (size_t)worker * (size_t)h->ld, (size_t)h->d, on_device);
}

int comp_ams_get_selected(comp_ams_t *h, int32_t worker, uint32_t *idx_host, float *val_host)
{
    int rc = check_handle(h);
    if (rc) return rc;
    if (h->compressor != COMP_AMS_TOPK) return fail(h, COMP_AMS_ESTATE, "get_selected needs a TOPK handle");
    if (h->steps == 0) return fail(h, COMP_AMS_ESTATE, "no step has run yet");
    if (worker < 0 || worker >= h->n) return fail(h, COMP_AMS_EINVAL, "worker %d out of [0, %d)", worker, h->n);
    const TkGeom &ge = h->ge;
    const size_t nt = (size_t)ge.n_tiles, k = (size_t)ge.k;
    std::vector<uint32_t> cnt(nt), offs(nt);
    HIP_TRY(h, hipMemcpyAsync(cnt.data(), h->sel_cnt + (size_t)worker * nt, nt * sizeof(uint32_t), hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    uint64_t total = 0;
    for (size_t t = 0; t < nt; ++t) {
        offs[t] = (uint32_t)total;
        total += cnt[t];
    }
    if (total != k) return fail(h, COMP_AMS_EDEVICE, "internal: %llu coordinates recorded, expected k=%zu", (unsigned long long)total, k);
    HIP_TRY(h, hipMemcpyAsync(h->sel_offs, offs.data(), nt * sizeof(uint32_t), hipMemcpyHostToDevice, h->stream));
    tk_gather_selected<<<ge.n_tiles, kWave, 0, h->stream>>>(ge, worker, h->cand_idx, h->cand_val, h->sel_cnt,
                                                           h->sel_offs, h->sel_out_idx, h->sel_out_val);
    std::vector<uint32_t> idx(k);
    std::vector<float> val(k);
    HIP_TRY(h, hipMemcpyAsync(idx.data(), h->sel_out_idx, k * sizeof(uint32_t), hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(h, hipMemcpyAsync(val.data(), h->sel_out_val, k * sizeof(float), hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    std::vector<uint32_t> order(k);
    for (size_t r = 0; r < k; ++r) order[r] = (uint32_t)r;
    std::sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) { return idx[a] < idx[b]; });
    for (size_t r = 0; r < k; ++r) {
        if (idx_host) idx_host[r] = idx[order[r]];
        if (val_host) val_host[r] = val[order[r]];
    }
    return COMP_AMS_OK;
}

int comp_ams_get_scales(comp_ams_t *h, float *out_host)
{
    int rc = check_handle(h);
    if (rc) return rc;
    if (h->compressor != COMP_AMS_BLOCKSIGN) return fail(h, COMP_AMS_ESTATE, "get_scales needs a BLOCKSIGN handle");
    if (h->steps == 0) return fail(h, COMP_AMS_ESTATE, "no step has run yet");
    return copy_out(h, out_host, h->scales, (size_t)h->n * (size_t)h->tb.n_blocks, 0);
}

int32_t comp_ams_n_blocks(comp_ams_t *h)
{
    if (!h) return fail(nullptr, COMP_AMS_EINVAL, "handle is NULL");
    return h->compressor == COMP_AMS_BLOCKSIGN ? h->tb.n_blocks : 0;
}

int comp_ams_set_state(comp_ams_t *h, const float *m, const float *v, const float *vhat, const float *e, int on_device)
{
    int rc = check_handle(h);
    if (rc) return rc;
    const size_t d = (size_t)h->d;
    if (m && (rc = copy_in(h, h->m, m, d, on_device))) return rc;
    if (v && (rc = copy_in(h, h->v, v, d, on_device))) return rc;
    if (vhat && (rc = copy_in(h, h->vhat, vhat, d, on_device))) return rc;
    if (e) {
        HIP_TRY(h, hipMemcpy2DAsync(h->e, (size_t)h->ld * sizeof(float), e, d * sizeof(float), d * sizeof(float),
                                    (size_t)h->n, on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice,
                                    h->stream));
        HIP_TRY(h, hipStreamSynchronize(h->stream));
    }
    return COMP_AMS_OK;
}

int comp_ams_sync(comp_ams_t *h)
{
    int rc = check_handle(h);
    if (rc) return rc;
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    return COMP_AMS_OK;
}

int comp_ams_profile(comp_ams_t *h, int enable)
{
    int rc = check_handle(h);
    if (rc) return rc;
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    prof_clear(h);
    h->prof_on = enable != 0;
    return COMP_AMS_OK;
}

int comp_ams_profile_read(comp_ams_t *h, int32_t slot, const char **name, double *total_ms, int64_t *launches)
{
    int rc = check_handle(h);
    if (rc) return rc;
    if (slot < 0) return fail(h, COMP_AMS_EINVAL, "slot must be >= 0");
    if (slot >= P_SLOTS) return 1;
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    double total = 0.0;
    for (const auto &pr : h->prof[slot]) {
        float ms = 0.f;
        HIP_TRY(h, hipEventElapsedTime(&ms, pr.first, pr.second));
        total += ms;
    }
    if (name) *name = kProfNames[slot];
    if (total_ms) *total_ms = total;
    if (launches) *launches = (int64_t)h->prof[slot].size();
    return COMP_AMS_OK;
}

const char *comp_ams_last_error(const comp_ams_t *h) { return h ? h->err.c_str() : g_create_error.c_str(); }

}  // extern "C"
