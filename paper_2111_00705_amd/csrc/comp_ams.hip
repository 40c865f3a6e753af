// Host side of the C ABI declared in include/comp_ams.h: handle, argument validation, device
// memory, kernel launches.  Every step of the method runs in the kernels of the two *_kernels.h
// files; nothing is computed on the host.
#include "../../include/comp_ams.h"
#include "../../include/comp_ams_tuning.h"

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <tuple>
#include <type_traits>
#include <utility>
#include <vector>

#include "blocksign_kernels.h"
#include "topk_kernels.h"
#include "plain_kernels.h"

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
    int32_t rows_choice = -1, state_choice = -1;   // comp_ams_set_streaming: -1 by size, 0 cached, 1 streamed
    int32_t chunk_choice = -1;                     // comp_ams_set_tile_order: -1 by size
    int32_t lds_choice = -1;                       // comp_ams_set_pass_lds: -1 by size, method and gradient type
    unsigned pass_lds = 0, pass_lds16 = 0;         // dynamic LDS of bs_pass for gradients of 32 / 16 bits (see pass_lds_bytes)
    bool has_split_tiles = false;                  // some tile holds several pieces
    bool mostly_split_tiles = false;               // more than one tile in eight does
    uint64_t rand_seed = 0;                    // Rand-k: the generator's seed and the number of the next draw
    uint32_t draw = 0;
    std::string err;
    std::vector<void *> allocs;

    float *theta = nullptr, *m = nullptr, *v = nullptr, *vhat = nullptr, *e = nullptr;

    float *row_tmp = nullptr;                  // d floats: staging for getters that materialise e_i

    // block sign: e holds x = g + e of the last step; `pending` says its scales still have to be
    // subtracted (deferred error, see blocksign_kernels.h)
    BsTable tb{};
    std::vector<void *> tb_allocs;
    double *partial = nullptr;
    float *scales = nullptr;
    uint16_t *signs = nullptr;                 // [n][n_tiles][256] sign bits of the stored x
    // sign words and piece sums exist twice and alternate while the update is deferred (step_blocksign_deferred);
    // signs / partial always point at the set of the most recent step
    uint16_t *signs2[2] = {nullptr, nullptr};
    double *partial2[2] = {nullptr, nullptr};
    int bs_set = 0;
    bool pending = false;
    bool fused_scale = false;                  // bs_update forms the scales itself (see kMaxFusedPieces)

    // CD-Adam (Algorithm 1): e then holds the workers' Markov sequences ghat_i (deferred by one c_i while
    // `pending`), and the server keeps its aggregate, gtilde and the buffers of its own compression
    int32_t method = COMP_AMS_METHOD_EF;
    float *ghat_srv = nullptr, *gtil = nullptr;   // [ld] each
    uint16_t *signs_srv = nullptr;                // [n_tiles][256] sign bits of ghat - gtilde
    double *partial_srv = nullptr;                // [n_pieces]
    float *scales_srv = nullptr;                  // [n_blocks]

    // An update that the most recent step left to the next one (see step_blocksign), and the hyper-parameters it
    // must run with (those of its own step)
    bool final_pending = false;
    AmsParams pending_params{};

    // Top-k
    TkGeom ge{};
    TkWorker *ws = nullptr;
    uint2 *cand = nullptr;                     // [n][slices][region_cap] candidate (index, value bits)
    uint32_t *cursor = nullptr;                // [n][slices] entries in each region (zero between steps)
    uint4 *tile_dir = nullptr;                 // [n][n_tiles] {offset in the worker's space, counts per wavefront, zeros}
    uint32_t *hist_full = nullptr;             // [n][2048] coarse-bin counts of the whole vector (only after a miss)
    uint32_t *hist1 = nullptr;                 // [n][2048] coarse-bin counts of the candidates
    uint32_t *histf = nullptr;                 // [n][512] fine-bin counts from the guess's coarse bin on
    uint32_t *cursor_b = nullptr;              // [n][slices] the cursors that lists made anew after a miss count in
    uint32_t *piece_bits = nullptr;            // [n][64 * parts * 4][32] which first digits occur in each dense piece
    uint32_t *hist2 = nullptr;                 // [n][1024] threshold bin: counts of the first digit below the prefix
    uint64_t *dense = nullptr;                 // laid out like cand: comp of the candidates in the threshold bin

    uint2 *dense_dir = nullptr;                // [n][64 * parts * 4] {start, count} of each wavefront's piece
    uint32_t *small_ctr = nullptr;             // [n] short vectors (step_topk_small): entries listed
    uint32_t *sel_count = nullptr, *sel_out_idx = nullptr;
    float *sel_out_val = nullptr;
    // CD-Adam with Top-k: the same selection structures once more, for the server's single vector
    TkSide srv{};
    uint32_t *hist1_s = nullptr, *histf_s = nullptr, *hist_full_s = nullptr, *hist2_s = nullptr, *cursor_b_s = nullptr,
             *piece_bits_s = nullptr;
    uint64_t *dense_s = nullptr;
    uint2 *dense_dir_s = nullptr;

    // optional per-kernel timing with HIP events on the step's stream
    bool prof_on = false;
    std::vector<std::vector<std::pair<hipEvent_t, hipEvent_t>>> prof;   // [slot] -> recorded pairs
};

// What a step touches once per step - the n stored rows; theta, m, v, vhat - is accessed as a stream
// (see ld4_row, ld4_state) when it cannot stay in the 256 MB memory-side cache until the next step anyway.
// Measured with 16 workers from 1.2 M to 25 M coordinates: rows of 183 MB in total are faster cached
// (110 against 118 us per step), rows of 275 MB faster streamed (176 against 188 us).  The state is faster
// cached when it fits and the rows stream past it (11.2 M coordinates, 179 MB: tk_final 70 -> 62 us), faster
// streamed when it does not fit, and also when the rows are cached and it would compete with them (1.2 M
// coordinates: 52.2 against 52.9 us per step).
// With CD-Adam the server's ghat and gtilde are read and written next to the state; the six arrays then
// compete for the cache together (11.2 M coordinates: 268 MB, and streaming the state is 8 % faster).
constexpr size_t kCacheResidentBytes = (size_t)224 << 20;
inline bool rows_exceed_caches(const comp_ams *h) { return (size_t)h->n * (size_t)h->ld * sizeof(float) > kCacheResidentBytes; }
inline bool state_exceeds_caches(const comp_ams *h)
{
    const size_t arrays = h->method == COMP_AMS_METHOD_CD ? 6 : 4;
    return arrays * (size_t)h->ld * sizeof(float) > kCacheResidentBytes;
}
// Dynamic LDS of bs_pass.  Tiles of several pieces need kPassTileLds.  Beyond that the amount is a knob that sets
// how many workgroups share a compute unit, and the pass responds to it by a few per cent (one session, same
// build).  Where most tiles are whole (blocks of a tile, or layers): once the rows are well beyond the caches,
// 40 KB - three workgroups per unit - measured best over n = 4 to 64 and d = 11 M to 110 M (n = 32, d = 25.6 M:
// 1.63 ms, against 1.70 ms at 16 KB, 1.65 ms at 32 KB and 1.77 ms at 64 KB; CD-Adam's worker stage on the same
// workload: 1.63 ms at 32 KB, 1.65 ms at 24 and at 40 KB); below about a GiB of rows up to 16 KB is best (n = 16,
// d = 1.2 M: 36.4 us, against 37.7 at 24 KB and 42.1 at 40 KB; n = 8, d = 11.2 M: 177 against 184 us).  Where many
// tiles hold several pieces (short blocks) they pass through barriers, more workgroups per unit hide those, and
// the table gets just what it needs (n = 16, d = 11.2 M, blocks of 256: 0.37 ms at 24 KB, 0.43 at 32 KB, 0.51 at
// 40 KB).  The block-to-tile mapping below does not move these optima.  Gradients of 16 bits are another matter:
// that pass issues more instructions per byte and wants the workgroups (n = 32, d = 25.6 M, bfloat16 or half:
// 1.32 ms up to 24 KB, 1.54 ms at 32 KB, 1.83 ms at 40 KB), so it never gets more than 16 KB beyond its need.
inline unsigned pass_lds_bytes(const comp_ams *h, bool grads16)
{
    const unsigned need = h->has_split_tiles ? kPassTileLds : 0u;
    if (h->lds_choice >= 0) return std::max(need, (unsigned)h->lds_choice);
    if (h->mostly_split_tiles) return need;
    if (grads16) return std::max(need, 16u * 1024u);
    // (with the tile order of xcd_chunk_for the larger amount pays from about half a GiB of rows: n = 16, d = 11.2 M
    // 354 against 358-360 us, n = 8, d = 25.6 M 393-395 against 410 us)
    const bool far_beyond_caches = (size_t)h->n * h->ld * sizeof(float) > ((size_t)512 << 20);
    // naive compression reads g only and wants the workgroups as well (n = 32, d = 25.6 M: 0.55 ms up to 24 KB,
    // 0.66 ms at 32 KB, 0.78 ms at 40 KB)
    const unsigned large = h->method == COMP_AMS_METHOD_EF ? 40u * 1024u
                           : h->method == COMP_AMS_METHOD_CD ? 32u * 1024u : 16u * 1024u;
    return std::max(need, far_beyond_caches ? large : 16u * 1024u);
}

// The streaming passes' block-to-tile mapping (tile_of_block).  Measured with rows far beyond the caches (one
// session; n = 32, d = 25.6 M block sign and n = 8, d = 110 M Top-k): chunks of 16 tiles - each XCD takes 256 KB of
// every 2 MB in turn - make the pass 3 % faster (1.60 -> 1.55 ms, 1.72 -> 1.67 ms), 8 tiles 1.5-2.5 %, 32 tiles
// 1-2 %, 12 and 24 tiles nothing, one eighth of the row per XCD 1.3 %, 512 tiles are 3-15 % slower.  Rows of
// 715 MB (n = 16, d = 11.2 M) gain nothing (+-1 %), rows that stay cached lose 4-20 % (the few tiles of a short
// row then also fall on few XCDs), and the kernels with one workgroup per tile (the updates) do not respond.
// CD-Adam's passes gain 0.5-2 %; naive compression (g only) gains nothing or loses 0.5-3 %, and so does the
// Top-k pass with 16-bit gradients (block sign with 16-bit gradients gains 2 %): those keep the plain order.
// Rows of 11 M coordinates, half a GiB to 1.5 GiB in all, do gain 1-3 % with chunks of 8 tiles once the pass runs
// three workgroups per unit (block sign, n = 16: 354 against 358 us; n = 32: 697 against 709 us with chunks of 16;
// Top-k under CD-Adam, n = 16: 254 against 257 us), so shorter rows get 8 from half a GiB on.
inline int xcd_chunk_for(const comp_ams *h)
{
    if (h->method != COMP_AMS_METHOD_EF && h->method != COMP_AMS_METHOD_CD) return 0;
    if ((size_t)h->n * h->ld * sizeof(float) <= ((size_t)512 << 20)) return 0;
    return h->d < ((int64_t)16 << 20) ? 8 : 16;
}

// The error-feedback listing pass of Top-k / Rand-k on 32-bit gradients has its own optimum, which goes with the
// length of a row rather than with the total (one session; pass times with four workgroups per unit and no chunks /
// the choice below): rows of 11 M coordinates, n = 8, 12, 16, 24, 32: 179 / 173, 266 / 259, 353 / 341, 527 / 513,
// 700 / 688 us with five workgroups per unit and chunks of 8 tiles (chunks of 4, 12 or 32 lose, 16 gains half as
// much); 25 M coordinates, n = 16: 783 / 763 us; rows of 110 M coordinates want four workgroups and chunks of 16
// or 8 (n = 8: 1.68 ms against 1.69-1.71 ms with five; n = 4: 846-850 against 860 us).
inline bool tk_long_rows(const comp_ams *h) { return h->d >= ((int64_t)64 << 20); }
inline int tk_ef_chunk_for(const comp_ams *h)
{
    if (!rows_exceed_caches(h)) return 0;
    return tk_long_rows(h) ? 16 : 8;
}

// Grid of a kernel with one workgroup per tile (in x) under tile_of_block's mapping.
inline unsigned grid_blocks(int64_t n_tiles, int chunk)
{
    if (chunk <= 0) return (unsigned)n_tiles;
    const int64_t span = 8 * (int64_t)chunk;
    return (unsigned)((n_tiles + span - 1) / span * span);
}

// Applies the caller's choices (comp_ams_set_streaming; -1 = by size) to the kernel parameters.
inline void apply_streaming(comp_ams *h)
{
    const int rows = h->rows_choice < 0 ? (rows_exceed_caches(h) ? 1 : 0) : h->rows_choice;
    h->tb.stream_rows = rows;
    h->ge.stream_rows = rows;
    h->pass_lds = pass_lds_bytes(h, false);
    h->pass_lds16 = pass_lds_bytes(h, true);
    h->tb.xcd_chunk = h->ge.xcd_chunk = h->chunk_choice < 0 ? xcd_chunk_for(h) : h->chunk_choice;
    if (h->chunk_choice < 0 && h->method == COMP_AMS_METHOD_EF) h->ge.xcd_chunk = tk_ef_chunk_for(h);
    h->srv.ge.xcd_chunk = 0;   // the server's single vector: not measured, left alone
    // the state stays cached if it fits - except under error feedback with cached rows, where it would
    // compete with them (CD-Adam with cached rows measured the other way: 55.9 against 58.0 us per step with
    // 1.2 M coordinates; methods without memory do not touch the rows at all)
    const bool rows_cached = rows == 0 && h->method == COMP_AMS_METHOD_EF;
    h->params.stream_state = h->state_choice < 0 ? ((state_exceeds_caches(h) || rows_cached) ? 1 : 0) : h->state_choice;
}

// Geometry handed to tk_pass1 for gradients of type G: with 16-bit gradients the automatic tile order is the
// plain one unless the method is error feedback (n = 8, d = 110 M, bfloat16: error feedback 1.44 -> 1.38 ms with
// chunks of 16, CD-Adam 1.09 -> 1.10 ms); a caller's choice holds for every type.
template <typename G>
inline TkGeom pass_geometry(const comp_ams *h)
{
    TkGeom ge = h->ge;
    if (sizeof(G) == 2 && h->chunk_choice < 0 && h->method != COMP_AMS_METHOD_EF) ge.xcd_chunk = 0;
    return ge;
}

// Top-k and Rand-k share every buffer and kernel (the key differs, see SelKey).
inline bool is_sparse(const comp_ams *h) { return h->compressor != COMP_AMS_BLOCKSIGN; }

// Rand-k: fixes the draws of the step about to run (workers: who = 0..n-1; server of Algorithm 1: who = n)
// and keeps the previous step's, which the deferred error memory still needs.
inline uint32_t host_mix32(uint32_t h)
{
    h ^= h >> 16;
    h *= 0x85ebca6bu;
    h ^= h >> 13;
    h *= 0xc2b2ae35u;
    h ^= h >> 16;
    return h;
}
inline uint32_t per_step_word(const comp_ams *h, uint32_t draw) { return host_mix32((uint32_t)h->rand_seed + draw * 0x9e3779b9u); }

namespace {

enum ProfSlot { P_BS_PASS, P_BS_SCALE, P_BS_UPDATE, P_TK_PASS1, P_TK_HIST, P_TK_PICK, P_TK_COMPACT,
                P_TK_RESOLVE, P_TK_FINAL, P_BS_SERVER, P_BS_SCALE_SERVER, P_BS_APPLY, P_TK_MERGE, P_TK_PASS1_SERVER,
                P_TK_SELECT_SERVER, P_TK_APPLY, P_PLAIN_UPDATE, P_BS_PASS_UPDATE, P_SLOTS };
const char *const kProfNames[P_SLOTS] = {"bs_pass", "bs_scale", "bs_update", "tk_pass1", "tk_hist", "tk_pick",
                                         "tk_compact", "tk_resolve", "tk_final", "bs_server",
                                         "bs_scale_server", "bs_apply", "tk_merge", "tk_pass1_server", "tk_select_server",
                                         "tk_apply", "plain_update", "bs_pass_update"};

// Kernel launches of a step go through KLAUNCH.  With profiling on, launch_timed hands the launch a
// pair of events through t_ev0 / t_ev1 and the kernel is started with hipExtLaunchKernel, which stamps
// them with the begin and end of the kernel itself (two hipEventRecord calls around a launch also time
// the gaps before and after it, about 3 us); otherwise the launch is the ordinary one.
thread_local hipEvent_t t_ev0 = nullptr, t_ev1 = nullptr;

template <typename... P, typename... A, size_t... I>
void launch_ext_impl(void (*kernel)(P...), dim3 grid, dim3 block, unsigned lds, hipStream_t st,
                     std::index_sequence<I...>, A &&...args)
{
    std::tuple<P...> params{static_cast<P>(std::forward<A>(args))...};   // the kernel's own parameter types
    void *ptrs[] = {static_cast<void *>(&std::get<I>(params))...};
    (void)hipExtLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, ptrs, lds, st, t_ev0, t_ev1, 0);
}
template <typename... P, typename... A>
void launch_ext(void (*kernel)(P...), dim3 grid, dim3 block, unsigned lds, hipStream_t st, A &&...args)
{
    launch_ext_impl(kernel, grid, block, lds, st, std::index_sequence_for<P...>{}, std::forward<A>(args)...);
}
// lds: bytes of dynamic LDS
#define KLAUNCH_LDS(kern, grid, block, lds, st, ...)                  \
    do {                                                              \
        if (t_ev0)                                                    \
            launch_ext(kern, grid, block, lds, st, __VA_ARGS__);      \
        else                                                          \
            kern<<<grid, block, lds, st>>>(__VA_ARGS__);              \
    } while (0)
#define KLAUNCH(kern, grid, block, st, ...) KLAUNCH_LDS(kern, grid, block, 0u, st, __VA_ARGS__)

// Calls f with std::true_type or std::false_type: turns a run-time choice into a template argument.
template <typename F>
void by_flag(bool flag, F &&f)
{
    if (flag) f(std::true_type{}); else f(std::false_type{});
}

// Runs `launch` (exactly one KLAUNCH on st); with profiling on, the kernel's begin and end are recorded.
template <typename F>
void launch_timed(comp_ams *h, int slot, hipStream_t st, F &&launch)
{
    (void)st;
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
    t_ev0 = a;
    t_ev1 = b;
    launch();
    t_ev0 = t_ev1 = nullptr;
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
            /* the failure is reported through the status code: the runtime's "last error" is cleared, */ \
            /* or the caller's next HIP call (or its framework's error check) would trip over it */    \
            (void)hipGetLastError();                                                                  \
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
int build_block_table(comp_ams *h, const std::vector<int64_t> &off, int64_t uniform_len)
{
    const int nb = (int)off.size() - 1;
    const int64_t n_tiles = h->ld / kTile;
    std::vector<int32_t> off32(nb + 1), piece_hi, piece_blk, tile_piece0(n_tiles + 1), block_piece0(nb + 1);
    for (int b = 0; b <= nb; ++b) off32[b] = (int32_t)off[b];
    // pieces = blocks cut at every multiple of kTile, in coordinate order
    {
        int b = 0;
        int64_t pos = 0;
        block_piece0[0] = 0;
        for (int64_t t = 0; t < n_tiles; ++t) {
            tile_piece0[t] = (int32_t)piece_hi.size();
            const int64_t tile_end = std::min<int64_t>((t + 1) * kTile, h->d);
            while (pos < tile_end) {
                const int64_t hi = std::min(tile_end, off[b + 1]);
                piece_hi.push_back((int32_t)hi);
                piece_blk.push_back(b);
                pos = hi;
                if (pos == off[b + 1] && b + 1 < nb) {
                    ++b;
                    block_piece0[b] = (int32_t)piece_hi.size();
                }
            }
        }
        tile_piece0[n_tiles] = (int32_t)piece_hi.size();
        block_piece0[nb] = (int32_t)piece_hi.size();
    }
    // blocks whose scale bs_scale forms: all but those that are one piece of a tile with several pieces (the
    // pass kernels write the scale of such a block themselves)
    std::vector<int32_t> scale_list;
    for (int b = 0; b < nb; ++b) {
        bool direct = false;
        if (block_piece0[b + 1] - block_piece0[b] == 1) {
            const int64_t t = off[b] / kTile;
            direct = tile_piece0[t + 1] - tile_piece0[t] > 1;
        }
        if (!direct) scale_list.push_back(b);
    }
    const int32_t n_scale_list = (int32_t)scale_list.size();
    if (scale_list.empty()) scale_list.push_back(0);
    std::vector<void *> fresh;
    int32_t *d_off = nullptr, *d_hi = nullptr, *d_blk = nullptr, *d_tp = nullptr, *d_bp = nullptr, *d_sl = nullptr;
    double *d_partial = nullptr, *d_partial_b = nullptr, *d_partial_srv = nullptr;
    float *d_scales = nullptr, *d_scales_srv = nullptr;
    int rc;
    auto upload = [&](int32_t **dst, const std::vector<int32_t> &src) -> int {
        int r = dev_alloc_t(h, fresh, dst, src.size(), false);
        if (r != COMP_AMS_OK) return r;
        HIP_TRY(h, hipMemcpy(*dst, src.data(), src.size() * sizeof(int32_t), hipMemcpyHostToDevice));
        return COMP_AMS_OK;
    };
    if ((rc = upload(&d_off, off32)) || (rc = upload(&d_hi, piece_hi)) || (rc = upload(&d_blk, piece_blk)) ||
        (rc = upload(&d_tp, tile_piece0)) || (rc = upload(&d_bp, block_piece0)) || (rc = upload(&d_sl, scale_list)) ||
        (rc = dev_alloc_t(h, fresh, &d_partial, (size_t)h->n * piece_hi.size())) ||
        (rc = dev_alloc_t(h, fresh, &d_partial_b, (size_t)h->n * piece_hi.size())) ||
        (rc = dev_alloc_t(h, fresh, &d_scales, (size_t)h->n * nb)) ||
        (rc = dev_alloc_t(h, fresh, &d_partial_srv, piece_hi.size())) ||
        (rc = dev_alloc_t(h, fresh, &d_scales_srv, (size_t)nb))) {
        free_all(fresh);
        return rc;
    }
    free_all(h->tb_allocs);
    h->tb_allocs = std::move(fresh);
    h->tb.offsets = d_off;
    h->tb.piece_hi = d_hi;
    h->tb.piece_blk = d_blk;
    h->tb.tile_piece0 = d_tp;
    h->tb.block_piece0 = d_bp;
    h->tb.scale_list = d_sl;
    h->tb.n_scale_list = n_scale_list;
    h->has_split_tiles = (size_t)piece_hi.size() > (size_t)n_tiles;
    int64_t split = 0;
    for (int64_t t = 0; t < n_tiles; ++t) split += tile_piece0[t + 1] - tile_piece0[t] > 1;
    h->mostly_split_tiles = split * 8 > n_tiles;
    h->tb.n_blocks = nb;
    h->tb.n_pieces = (int32_t)piece_hi.size();
    h->tb.uniform_tiles = (uniform_len > 0 && uniform_len % kTile == 0) ? (int32_t)(uniform_len / kTile) : 0;
    apply_streaming(h);
    {
        bool ok = true;
        for (int64_t t = 0; t < n_tiles && ok; ++t) ok = (tile_piece0[t + 1] - tile_piece0[t] == 1);
        for (int b = 0; b < nb && ok; ++b) ok = (block_piece0[b + 1] - block_piece0[b] <= kMaxFusedPieces);
        h->fused_scale = ok;
    }
    h->partial2[0] = d_partial;
    h->partial2[1] = d_partial_b;
    h->partial = h->partial2[h->bs_set];
    h->scales = d_scales;
    h->partial_srv = d_partial_srv;
    h->scales_srv = d_scales_srv;
    return COMP_AMS_OK;
}

// Makes the handle's GPU the current device for the duration of an entry point and gives the caller its
// own current device back on the way out (also on every error return).
struct DeviceScope {
    int prev = -1;
    bool switched = false;
    int enter(comp_ams *h)
    {
        if (!h) return fail(nullptr, COMP_AMS_EINVAL, "handle is NULL");
        hipError_t e = hipGetDevice(&prev);
        if (e != hipSuccess) return fail(h, COMP_AMS_EDEVICE, "hipGetDevice failed: %s", hipGetErrorString(e));
        if (prev == h->device) return COMP_AMS_OK;
        e = hipSetDevice(h->device);
        if (e != hipSuccess) return fail(h, COMP_AMS_EDEVICE, "hipSetDevice(%d) failed: %s", h->device, hipGetErrorString(e));
        switched = true;
        return COMP_AMS_OK;
    }
    ~DeviceScope()
    {
        if (switched) (void)hipSetDevice(prev);
    }
};
// First lines of an entry point that touches the device: validates the handle, selects its GPU.
#define ENTER_DEVICE(h)        \
    DeviceScope device_scope__; \
    int rc = device_scope__.enter(h)
// The same for an entry point that reads or replaces state: an update that the last step left pending is
// launched first.
int flush_pending(comp_ams *h);
#define ENTER_STATE(h)          \
    DeviceScope device_scope__; \
    int rc = device_scope__.enter(h); \
    if (!rc) rc = flush_pending(h)

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

// bs_update for the sign words, piece sums and scales of the most recent step, with the hyper-parameters p.
void launch_bs_update(comp_ams *h, hipStream_t st, const AmsParams &p)
{
    const BsTable &tb = h->tb;
    const unsigned ugrid = (unsigned)(h->ld / kTile);
    launch_timed(h, P_BS_UPDATE, st, [&] {
        // few tiles: nothing hides the state loads, so issue them first; many tiles: load late, run more
        // workgroups per compute unit
        const bool early = h->ld / kTile < 2048;
#define CAMS_BS_UPDATE(F, E)                                                                                  \
    by_flag(h->params.stream_state, [&](auto ss) {                                                            \
        KLAUNCH((bs_update<F, E, false, decltype(ss)::value>), ugrid, kThreads, st, h->d, h->ld, h->n, tb,   \
                h->partial, h->scales, h->signs, h->theta, h->m, h->v, h->vhat, p, BsMarkov{});               \
    })
        if (h->fused_scale) {
            if (early) CAMS_BS_UPDATE(true, true); else CAMS_BS_UPDATE(true, false);
        } else {
            if (early) CAMS_BS_UPDATE(false, true); else CAMS_BS_UPDATE(false, false);
        }
#undef CAMS_BS_UPDATE
    });
}

template <typename G>
int step_blocksign(comp_ams *h, const G *g, hipStream_t st)
{
    const BsTable &tb = h->tb;
    const dim3 grid(grid_blocks(h->ld / kTile, tb.xcd_chunk), h->n);
    const unsigned lds = sizeof(G) == 2 ? h->pass_lds16 : h->pass_lds;
    launch_timed(h, P_BS_PASS, st, [&] {
        if (h->method == COMP_AMS_METHOD_NAIVE)   // C(g_i) itself: the stored rows are not touched
            KLAUNCH_LDS((bs_pass<false, kBsNaive, G>), grid, kThreads, lds, st, g, h->e, h->d, h->ld, tb, h->scales,
                    h->signs, h->partial);
        else if (h->pending)
            KLAUNCH_LDS((bs_pass<true, kBsEf, G>), grid, kThreads, lds, st, g, h->e, h->d, h->ld, tb, h->scales, h->signs,
                    h->partial);
        else
            KLAUNCH_LDS((bs_pass<false, kBsEf, G>), grid, kThreads, lds, st, g, h->e, h->d, h->ld, tb, h->scales, h->signs,
                    h->partial);
    });
    if (!h->fused_scale && tb.n_scale_list > 0)
        launch_timed(h, P_BS_SCALE, st, [&] {
            KLAUNCH((bs_scale), dim3(tb.n_scale_list, h->n), kWave, st, h->partial, tb, h->scales);
        });
    launch_bs_update(h, st, h->params);
    h->pending = (h->method == COMP_AMS_METHOD_EF);
    return COMP_AMS_OK;
}

// Error feedback where every block is a run of at most kMaxFusedPieces whole tiles (uniform blocks of a multiple of
// 4096 coordinates): one launch per step.  The update of a step is left pending and runs inside the next step's
// pass kernel (bs_pass_update); whatever reads the state first launches a pending update on its own
// (flush_pending).  Not used while the stream is being captured: a recorded step must be self-contained.
inline bool can_defer_blocksign(const comp_ams *h)
{
    // the grid's second dimension holds the workers and four rows of update workgroups
    return h->method == COMP_AMS_METHOD_EF && h->fused_scale && h->tb.uniform_tiles > 0 && h->n + 4 <= 65535;
}

template <typename G>
int step_blocksign_deferred(comp_ams *h, const G *g, hipStream_t st)
{
    const BsTable &tb = h->tb;
    const int prev = h->bs_set, cur = 1 - prev;
    const dim3 grid(grid_blocks(h->ld / kTile, tb.xcd_chunk), h->n + 4);
    const unsigned lds = sizeof(G) == 2 ? h->pass_lds16 : h->pass_lds;
    BsDeferred df{};
    df.signs_prev = h->signs2[prev];
    df.partial_prev = h->partial2[prev];
    df.scales_out = h->scales;
    df.theta = h->theta;
    df.m = h->m;
    df.v = h->v;
    df.vhat = h->vhat;
    df.p = h->pending_params;
    df.do_update = h->final_pending ? 1 : 0;
    launch_timed(h, P_BS_PASS_UPDATE, st, [&] {
        by_flag(h->params.stream_state, [&](auto ss) {
            if (h->pending)
                KLAUNCH_LDS((bs_pass_update<true, G, decltype(ss)::value>), grid, kThreads, lds, st, g, h->e, h->d, h->ld, h->n,
                            tb, h->signs2[cur], h->partial2[cur], df);
            else
                KLAUNCH_LDS((bs_pass_update<false, G, decltype(ss)::value>), grid, kThreads, lds, st, g, h->e, h->d, h->ld, h->n,
                            tb, h->signs2[cur], h->partial2[cur], df);
        });
    });
    h->bs_set = cur;
    h->signs = h->signs2[cur];
    h->partial = h->partial2[cur];
    h->pending = true;
    h->final_pending = true;
    h->pending_params = h->params;
    return COMP_AMS_OK;
}

// One iteration of Algorithm 1 (CD-Adam) with the block-wise scaled sign, five launches.
template <typename G>
int step_blocksign_cd(comp_ams *h, const G *g, hipStream_t st)
{
    const BsTable &tb = h->tb;
    const dim3 grid(grid_blocks(h->ld / kTile, tb.xcd_chunk), h->n);
    const unsigned ugrid = (unsigned)(h->ld / kTile);
    const unsigned lds = sizeof(G) == 2 ? h->pass_lds16 : h->pass_lds;
    launch_timed(h, P_BS_PASS, st, [&] {
        if (h->pending)
            KLAUNCH_LDS((bs_pass<true, kBsCd, G>), grid, kThreads, lds, st, g, h->e, h->d, h->ld, tb, h->scales, h->signs,
                    h->partial);
        else
            KLAUNCH_LDS((bs_pass<false, kBsCd, G>), grid, kThreads, lds, st, g, h->e, h->d, h->ld, tb, h->scales, h->signs,
                    h->partial);
    });
    // every tile exactly one block (uniform blocks of one tile): the worker scales and the server's own
    // scale are formed inside bs_update, which then also applies the server's message - two launches in all
    const bool whole = h->fused_scale && tb.n_pieces == tb.n_blocks;
    if (!whole && tb.n_scale_list > 0)
        launch_timed(h, P_BS_SCALE, st, [&] {
            KLAUNCH((bs_scale), dim3(tb.n_scale_list, h->n), kWave, st, h->partial, tb, h->scales);
        });
    launch_timed(h, P_BS_SERVER, st, [&] {
        const BsMarkov mk{h->ghat_srv, h->gtil, h->signs_srv, h->partial_srv, h->scales_srv, whole ? 1 : 0};
        if (whole)
            by_flag(h->params.stream_state, [&](auto ss) {
                KLAUNCH((bs_update<true, false, true, decltype(ss)::value>), ugrid, kThreads, st, h->d, h->ld,
                        h->n, tb, h->partial, h->scales, h->signs, h->theta, h->m, h->v, h->vhat, h->params, mk);
            });
        else
            by_flag(h->params.stream_state, [&](auto ss) {
                KLAUNCH((bs_update<false, false, true, decltype(ss)::value>), ugrid, kThreads, st, h->d, h->ld,
                        h->n, tb, h->partial, h->scales, h->signs, h->theta, h->m, h->v, h->vhat, h->params, mk);
            });
    });
    if (!whole) {
        if (tb.n_scale_list > 0)
            launch_timed(h, P_BS_SCALE_SERVER, st, [&] {
                KLAUNCH((bs_scale), dim3(tb.n_scale_list, 1), kWave, st, h->partial_srv, tb, h->scales_srv);
            });
        launch_timed(h, P_BS_APPLY, st, [&] {
            by_flag(h->params.stream_state, [&](auto ss) {
                KLAUNCH((bs_apply<decltype(ss)::value>), ugrid, kThreads, st, h->d, tb, h->scales_srv,
                        h->signs_srv, h->gtil, h->theta, h->m, h->v, h->vhat, h->params);
            });
        });
    }
    h->pending = true;
    return COMP_AMS_OK;
}

// The four selection launches between the listing pass and the kernel that uses Tc: candidate histograms (after
// a miss: the whole vector's), leading digits (after a miss: and the lists anew), compaction of the threshold bin,
// last digits (or, rarest, the selection without lists).  kSrc / a / b say how the compressed vector is formed
// again where that is needed.  cursor_b: the second set of region cursors, which the lists made anew count in.
template <int kSrc, typename G>
void launch_select(comp_ams *h, hipStream_t st, const TkGeom &ge, TkWorker *ws, uint2 *cand, uint32_t *cursor,
                   uint32_t *cursor_b, uint4 *tile_dir, uint32_t *hist1, uint32_t *histf, uint32_t *hist_full,
                   uint32_t *hist2, uint32_t *piece_bits, uint64_t *dense, uint2 *dense_dir, const void *a,
                   const float *b, const int (&slot)[4])
{
    const dim3 shared(ge.slices * ge.parts, ge.n);
    // tk_pick: one workgroup per vector does the work in the usual case; the others (needed only to list the
    // vector again after a miss) are kept to about four per compute unit in total
    const dim3 pick((unsigned)std::min<int>(ge.relist_wgs, std::max(1, 1024 / ge.n)), ge.n);
    launch_timed(h, slot[0], st, [&] {
        KLAUNCH((tk_hist<kSrc, G>), shared, kThreads, st, ge, ws, cand, cursor, hist1, histf, hist_full, a, b);
    });
    launch_timed(h, slot[1], st, [&] {
        KLAUNCH((tk_pick<kSrc, G>), pick, kThreads, st, ge, ws, hist1, histf, cursor, cursor_b, hist_full, a, b, cand,
                tile_dir);
    });
    launch_timed(h, slot[2], st, [&] {
        KLAUNCH((tk_compact), shared, kThreads, st, ge, ws, cand, cursor, cursor_b, dense, dense_dir, hist2, piece_bits);
    });
    launch_timed(h, slot[3], st, [&] {
        // error feedback with magnitude keys counts zeros instead of listing them: tk_resolve may need the rows
        const float *rows = (kSrc == kSrcStored && !ge.rand.on) ? static_cast<const float *>(a) : nullptr;
        const ExactSource es{kSrc, std::is_same<G, float>::value ? 0 : std::is_same<G, uint16_t>::value ? 1 : 2, a, b};
        KLAUNCH((tk_resolve), ge.n, kResolveThreads, st, ge, ws, dense, dense_dir, cursor, cursor_b, hist_full, hist2,
                piece_bits, cand, tile_dir, rows, es);
    });
}

constexpr int kWorkerSelectSlots[4] = {P_TK_HIST, P_TK_PICK, P_TK_COMPACT, P_TK_RESOLVE};
constexpr int kServerSelectSlots[4] = {P_TK_SELECT_SERVER, P_TK_SELECT_SERVER, P_TK_SELECT_SERVER, P_TK_SELECT_SERVER};

void launch_final(comp_ams *h, hipStream_t st)
{
    launch_timed(h, P_TK_FINAL, st, [&] {
        by_flag(h->params.stream_state, [&](auto ss) {
            KLAUNCH((tk_final<decltype(ss)::value>), h->ge.n_tiles, kThreads, st, h->ge, h->ws, h->cand, h->tile_dir,
                    h->theta, h->m, h->v, h->vhat, h->params);
        });
    });
}

// Dynamic LDS handed to tk_pass1 beyond its own 24 KB of staging lists: unused by the kernel, it only sets how many
// workgroups share a compute unit (six without it).  The passes that only read want all six (n = 16, d = 11.2 M,
// CD-Adam: 245 against 257 us with four; n = 8, d = 110 M: 1.134 against 1.173 ms).  The error-feedback pass, which
// also writes the row back, is best with four or five on 32-bit gradients (n = 8, d = 110 M: 1.67-1.68 ms, 1.70 with
// six, 1.74 with eight) and gets 9 KB, which leaves four (five for shorter rows, see tk_ef_chunk_for); on 16-bit
// gradients it issues more instructions per byte and wants the six as well (same shape, bfloat16: 1.44 against
// 1.76 ms).  comp_ams_set_pass_lds overrides.
inline unsigned tk_pass_lds(const comp_ams *h, size_t grad_bytes)
{
    if (h->lds_choice >= 0) return (unsigned)h->lds_choice;
    if (h->method != COMP_AMS_METHOD_EF || grad_bytes != 4) return 0u;
    // five workgroups per unit for rows that stream and are not long (see tk_ef_chunk_for), else four
    return rows_exceed_caches(h) && !tk_long_rows(h) ? 7000u : 9u * 1024u;
}

// Error feedback on a short vector: listing pass, one selection kernel (tk_small_select), update - three launches.
template <typename G>
int step_topk_small(comp_ams *h, const G *g, hipStream_t st)
{
    TkGeom sge = h->ge;
    sge.region_cap = (uint32_t)sge.slices * sge.region_cap;      // one region per worker: all of its space
    sge.slices = 1;
    sge.slice_tiles = sge.n_tiles;
    sge.xcd_chunk = 0;
    launch_timed(h, P_TK_PASS1, st, [&] {
        KLAUNCH((tk_pass1<kPassEf, G>), dim3(sge.n_tiles, h->n), kThreads, st, g, h->e, sge, h->ws, h->cand, h->small_ctr,
                h->tile_dir);
    });
    launch_timed(h, P_TK_RESOLVE, st, [&] {
        KLAUNCH((tk_small_select), (unsigned)h->n, kResolveThreads, st, sge, h->ws, h->cand, h->small_ctr, h->tile_dir, h->e);
    });
    launch_final(h, st);
    return COMP_AMS_OK;
}

template <typename G>
int step_topk(comp_ams *h, const G *g, hipStream_t st)
{
    if (h->ge.n_tiles <= kSmallTiles) return step_topk_small(h, g, st);
    const TkGeom &ge = h->ge;
    const TkGeom pge = pass_geometry<G>(h);
    launch_timed(h, P_TK_PASS1, st, [&] {
        KLAUNCH_LDS((tk_pass1<kPassEf, G>), dim3(grid_blocks(ge.n_tiles, pge.xcd_chunk), h->n), kThreads, tk_pass_lds(h, sizeof(G)), st, g, h->e, pge, h->ws,
                h->cand, h->cursor, h->tile_dir);
    });
    launch_select<kSrcStored, float>(h, st, ge, h->ws, h->cand, h->cursor, h->cursor_b, h->tile_dir, h->hist1, h->histf,
                                     h->hist_full, h->hist2, h->piece_bits, h->dense, h->dense_dir, h->e, nullptr, kWorkerSelectSlots);
    launch_final(h, st);
    return COMP_AMS_OK;
}

// Naive compression (Section 4) with Top-k: pass, selection and update on g itself, one set of buffers.
template <typename G>
int step_topk_naive(comp_ams *h, const G *g, hipStream_t st)
{
    const TkGeom &ge = h->ge;
    const TkGeom pge = pass_geometry<G>(h);
    launch_timed(h, P_TK_PASS1, st, [&] {
        KLAUNCH_LDS((tk_pass1<kPassNaive, G>), dim3(grid_blocks(ge.n_tiles, pge.xcd_chunk), h->n), kThreads, tk_pass_lds(h, sizeof(G)), st, g, h->e, pge, h->ws,
                h->cand, h->cursor, h->tile_dir);
    });
    launch_select<kSrcGradOnly, G>(h, st, ge, h->ws, h->cand, h->cursor, h->cursor_b, h->tile_dir, h->hist1, h->histf,
                                   h->hist_full, h->hist2, h->piece_bits, h->dense, h->dense_dir, g, nullptr, kWorkerSelectSlots);
    launch_final(h, st);
    return COMP_AMS_OK;
}

// Vanilla distributed AMSGrad (Section 3): no compression.
template <typename G>
int step_plain(comp_ams *h, const G *g, hipStream_t st)
{
    // Tile order: with many gradient rows far beyond the caches each XCD working through 16 consecutive tiles of
    // every row measured 9 % faster (n = 32, d = 25.6 M: 797 -> 726 us); n = 16, d = 11.2 M does not respond, and
    // with n = 8, d = 110 M chunks of 16 to 256 tiles gave -3 to +5 % without a pattern, so few rows keep the plain
    // order.
    const int n_tiles = (int)(h->ld / kTile);
    const bool many_long_rows = h->n >= 16 && (size_t)h->n * (size_t)h->d * sizeof(G) > ((size_t)1 << 30);
    const int chunk = h->chunk_choice >= 0 ? h->chunk_choice : many_long_rows ? 16 : 0;
    launch_timed(h, P_PLAIN_UPDATE, st, [&] {
        by_flag(h->params.stream_state, [&](auto ss) {
            KLAUNCH((plain_update<G, decltype(ss)::value>), grid_blocks(n_tiles, chunk), kThreads, st, g, h->d, h->n,
                    h->theta, h->m, h->v, h->vhat, h->params, chunk, n_tiles);
        });
    });
    return COMP_AMS_OK;
}

// One iteration of Algorithm 1 (CD-Adam) with Top-k in both directions, twelve launches.
template <typename G>
int step_topk_cd(comp_ams *h, const G *g, hipStream_t st)
{
    const TkGeom &ge = h->ge;
    const TkGeom pge = pass_geometry<G>(h);
    const TkSide &sv = h->srv;
    launch_timed(h, P_TK_PASS1, st, [&] {
        KLAUNCH_LDS((tk_pass1<kPassCd, G>), dim3(grid_blocks(ge.n_tiles, pge.xcd_chunk), h->n), kThreads, tk_pass_lds(h, sizeof(G)), st, g, h->e, pge, h->ws,
                h->cand, h->cursor, h->tile_dir);
    });
    launch_select<kSrcGrad, G>(h, st, ge, h->ws, h->cand, h->cursor, h->cursor_b, h->tile_dir, h->hist1, h->histf,
                               h->hist_full, h->hist2, h->piece_bits, h->dense, h->dense_dir, g, h->e, kWorkerSelectSlots);
    launch_timed(h, P_TK_MERGE, st, [&] {
        KLAUNCH((tk_merge), ge.n_tiles, kThreads, st, ge, h->ws, h->cand, h->tile_dir, h->e, h->ghat_srv,
                                                  h->params.n_workers);
    });
    launch_timed(h, P_TK_PASS1_SERVER, st, [&] {
        KLAUNCH((tk_pass1<kPassDiff, float>), dim3(grid_blocks(ge.n_tiles, sv.ge.xcd_chunk), 1), kThreads, st, h->ghat_srv,
                h->gtil, sv.ge, sv.ws, sv.cand, sv.cursor, sv.tile_dir);
    });
    launch_select<kSrcDiff, float>(h, st, sv.ge, sv.ws, sv.cand, sv.cursor, h->cursor_b_s, sv.tile_dir, h->hist1_s, h->histf_s,
                                   h->hist_full_s, h->hist2_s, h->piece_bits_s, h->dense_s, h->dense_dir_s, h->ghat_srv, h->gtil,
                                   kServerSelectSlots);
    launch_timed(h, P_TK_APPLY, st, [&] {
        by_flag(h->params.stream_state, [&](auto ss) {
            KLAUNCH((tk_apply<decltype(ss)::value>), ge.n_tiles, kThreads, st, sv, h->gtil, h->theta, h->m, h->v,
                    h->vhat, h->params);
        });
    });
    return COMP_AMS_OK;
}

// Candidate regions per vector and what follows from it: tiles per region, and the pieces a region
// is cut into for tk_hist / tk_compact - about 4096 candidates per workgroup when 1.5 k of them are
// listed, within the kMaxPieces records tk_resolve can walk.
void set_slices(TkGeom &ge, int slices)
{
    ge.slices = slices;
    ge.slice_tiles = (ge.n_tiles + slices - 1) / slices;
    const int64_t want = (3 * (int64_t)ge.k / 2 + (int64_t)slices * 4096 - 1) / ((int64_t)slices * 4096);
    ge.parts = (int32_t)std::min<int64_t>({(int64_t)kMaxParts, (int64_t)kMaxPieces / (4 * slices), std::max<int64_t>(1, want)});
    // Entries per region.  A vector's regions together hold twice max(4 k, d / 64) candidates: 1.2 k are listed in
    // steady state (error feedback piles mass up just below the threshold), a first step or a step after a miss lists
    // the coarse bin of the k-th largest and above (an eighth of an octave of magnitudes: about a hundredth of the
    // coordinates of a gradient spread over several decades), and the factor two covers uneven regions.  What does
    // not fit is found without lists (exact_select), which needs k entries in all: 8 k are there.  Never more than
    // every coordinate of the region's tiles.
    const int64_t full = (int64_t)ge.slice_tiles * kTile;
    const int64_t cands = std::max<int64_t>(4 * (int64_t)ge.k, ge.d / 64);
    const int64_t per_region = ((2 * cands + slices - 1) / slices + 1023) / 1024 * 1024;
    ge.region_cap = (uint32_t)std::min<int64_t>(full, std::max<int64_t>(per_region, 2048));
}

// Initial selection records: no pending threshold, no guess.
void fresh_tk_workers(std::vector<TkWorker> &init)
{
    for (auto &w : init) {
        std::memset(&w, 0, sizeof w);
        w.guess = kNoGuess;
        w.slack = kFirstSlack;
        w.last_fine = kNoGuess;
        w.tc = kNoThreshold;
    }
}

// Resets the per-worker selection records: no pending threshold, no guess.
int reset_topk_workers(comp_ams *h)
{
    std::vector<TkWorker> init((size_t)h->n);
    fresh_tk_workers(init);
    HIP_TRY(h, hipMemcpy(h->ws, init.data(), init.size() * sizeof(TkWorker), hipMemcpyHostToDevice));
    HIP_TRY(h, hipMemset(h->cursor, 0, (size_t)h->n * h->ge.slices * sizeof(uint32_t)));
    HIP_TRY(h, hipMemset(h->cursor_b, 0, (size_t)h->n * h->ge.slices * sizeof(uint32_t)));
    HIP_TRY(h, hipMemset(h->small_ctr, 0, (size_t)h->n * sizeof(uint32_t)));
    if (h->srv.ws) {
        HIP_TRY(h, hipMemcpy(h->srv.ws, init.data(), sizeof(TkWorker), hipMemcpyHostToDevice));
        HIP_TRY(h, hipMemset(h->srv.cursor, 0, (size_t)h->srv.ge.slices * sizeof(uint32_t)));
        HIP_TRY(h, hipMemset(h->cursor_b_s, 0, (size_t)h->srv.ge.slices * sizeof(uint32_t)));
    }
    return COMP_AMS_OK;
}

// Launches the update that the most recent step left pending (see step_topk, step_blocksign), on the handle's
// stream.  Every entry point that reads or replaces state calls this first.
int flush_pending(comp_ams *h)
{
    if (!h->final_pending) return COMP_AMS_OK;
    launch_bs_update(h, h->stream, h->pending_params);
    HIP_TRY(h, hipGetLastError());
    h->final_pending = false;
    return COMP_AMS_OK;
}

// Writes e_i (error feedback) or ghat_i (CD-Adam) in its defined form to dst (device memory, d floats)
// on the handle's stream.
void launch_materialize(comp_ams *h, int worker, float *dst)
{
    const float *xrow = h->e + (size_t)worker * (size_t)h->ld;
    const unsigned blocks = (unsigned)((h->d + kThreads - 1) / kThreads);
    if (is_sparse(h) && h->method == COMP_AMS_METHOD_CD) {
        // ghat_i is stored as it is (tk_merge has already added c_i)
        (void)hipMemcpyAsync(dst, xrow, (size_t)h->d * sizeof(float), hipMemcpyDeviceToDevice, h->stream);
    } else if (is_sparse(h)) {
        tk_materialize_error<<<blocks, kThreads, 0, h->stream>>>(xrow, h->ge, worker, h->ws + worker, dst);
    } else if (h->method == COMP_AMS_METHOD_CD) {
        const uint16_t *srow = h->signs + (size_t)worker * (size_t)(h->ld / kTile) * kThreads;
        if (h->pending)
            bs_materialize_markov<true><<<blocks, kThreads, 0, h->stream>>>(
                xrow, h->d, h->tb, h->scales + (size_t)worker * (size_t)h->tb.n_blocks, srow, dst);
        else
            bs_materialize_markov<false><<<blocks, kThreads, 0, h->stream>>>(xrow, h->d, h->tb, h->scales, srow, dst);
    } else if (h->pending) {
        bs_materialize_error<true><<<blocks, kThreads, 0, h->stream>>>(
            xrow, h->d, h->tb, h->scales + (size_t)worker * (size_t)h->tb.n_blocks, dst);
    } else {
        bs_materialize_error<false><<<blocks, kThreads, 0, h->stream>>>(xrow, h->d, h->tb, h->scales, dst);
    }
}

template <typename G>
int step_any(comp_ams *h, const G *grads_dev, void *hip_stream)
{
    ENTER_DEVICE(h);
    if (rc) return rc;
    if (!grads_dev) return fail(h, COMP_AMS_EINVAL, "grads is NULL");
    if (reinterpret_cast<uintptr_t>(grads_dev) & (sizeof(G) - 1))
        return fail(h, COMP_AMS_EINVAL, "grads must be %zu-byte aligned", sizeof(G));
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    bool capturing = false;
    {
        hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(st, &cs) == hipSuccess)
            capturing = (cs == hipStreamCaptureStatusActive);
        else
            (void)hipGetLastError();
    }
    if (capturing && h->final_pending)
        return fail(h, COMP_AMS_ESTATE, "the update of the last step is still pending: call comp_ams_sync (or any getter) "
                                        "before recording a step into a graph");
    if (st != h->stream) {
        // work of earlier steps on another stream must be finished before this stream touches the state
        if ((rc = flush_pending(h))) return rc;
        HIP_TRY(h, hipStreamSynchronize(h->stream));
        h->stream = st;
    }
    if (h->compressor == COMP_AMS_RANDK) {
        for (TkGeom *ge : {&h->ge, &h->srv.ge}) {
            ge->rand.on = 1u;
            ge->rand.seed_hi = (uint32_t)(h->rand_seed >> 32);
            ge->rand.step_now = per_step_word(h, h->draw);
        }
        h->ge.rand.who0 = 0u;
        h->srv.ge.rand.who0 = (uint32_t)h->n;
        // thresholds of independent draws differ by sqrt(2) standard deviations on average: six of those
        const double kd = (double)h->k / (double)h->d;
        const double sd_bins = std::sqrt((double)h->k * (1.0 - kd)) / (double)h->d * (double)(1u << 17);
        h->ge.rand.min_slack = h->srv.ge.rand.min_slack = (uint32_t)std::min(512.0, std::ceil(6.0 * 1.4143 * sd_bins));
    }
    if (h->method == COMP_AMS_METHOD_NONE)
        rc = step_plain(h, grads_dev, st);
    else if (is_sparse(h))
        rc = (h->method == COMP_AMS_METHOD_CD)      ? step_topk_cd(h, grads_dev, st)
             : (h->method == COMP_AMS_METHOD_NAIVE) ? step_topk_naive(h, grads_dev, st)
                                                    : step_topk(h, grads_dev, st);
    else
        rc = (h->method == COMP_AMS_METHOD_CD)            ? step_blocksign_cd(h, grads_dev, st)
             : (!capturing && can_defer_blocksign(h))     ? step_blocksign_deferred(h, grads_dev, st)
                                                           : step_blocksign(h, grads_dev, st);
    if (rc) return rc;
    HIP_TRY(h, hipGetLastError());
    ++h->steps;
    ++h->draw;
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
    if (compressor != COMP_AMS_TOPK && compressor != COMP_AMS_BLOCKSIGN && compressor != COMP_AMS_RANDK)
        return fail(nullptr, COMP_AMS_EINVAL, "unknown compressor %d", compressor);
    if (compressor != COMP_AMS_BLOCKSIGN && (k_or_block < 1 || k_or_block > d))
        return fail(nullptr, COMP_AMS_EINVAL, "Top-k / Rand-k need 1 <= k <= d, got k=%lld d=%lld", (long long)k_or_block, (long long)d);
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
        (rc = dev_alloc_t(h, h->allocs, &h->e, ld * (size_t)n)) ||
        (rc = dev_alloc_t(h, h->allocs, &h->row_tmp, (size_t)d)))
        return bail(rc);

    if (compressor == COMP_AMS_BLOCKSIGN) {
        const int64_t B = std::min<int64_t>(k_or_block, d);
        h->block = B;
        std::vector<int64_t> off;
        for (int64_t s = 0; s < d; s += B) off.push_back(s);
        off.push_back(d);
        if ((rc = dev_alloc_t(h, h->allocs, &h->signs2[0], ld / 16 * (size_t)n)) ||
            (rc = dev_alloc_t(h, h->allocs, &h->signs2[1], ld / 16 * (size_t)n)))
            return bail(rc);
        h->signs = h->signs2[0];
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
        // more regions per worker measured no faster (n workers already spread the cursors); fewer when the
        // vector has fewer tiles than that, so that many workers with a small model do not reserve 64 empty regions each
        int slices = kMinSlices;
        while (slices > 1 && slices / 2 >= ge.n_tiles) slices /= 2;
        set_slices(ge, slices);
        ge.relist_wgs = (int32_t)std::min<int64_t>(ge.n_tiles, std::max(1, 2048 / n));
        const size_t segs = (size_t)n * ge.n_tiles;
        const size_t region_entries = (size_t)n * ge.slices * (size_t)ge.region_cap;
        if ((rc = dev_alloc_t(h, h->allocs, &h->ws, (size_t)n)) ||
            (rc = dev_alloc_t(h, h->allocs, &h->cand, region_entries, false)) ||
            (rc = dev_alloc_t(h, h->allocs, &h->cursor, (size_t)n * ge.slices)) ||
            (rc = dev_alloc_t(h, h->allocs, &h->cursor_b, (size_t)n * ge.slices)) ||
            (rc = dev_alloc_t(h, h->allocs, &h->tile_dir, segs)) ||
            (rc = dev_alloc_t(h, h->allocs, &h->hist_full, (size_t)n * kBins1)) ||
            (rc = dev_alloc_t(h, h->allocs, &h->hist1, (size_t)n * kBins1)) ||
            (rc = dev_alloc_t(h, h->allocs, &h->histf, (size_t)n * kFineWindow)) ||
            (rc = dev_alloc_t(h, h->allocs, &h->hist2, (size_t)n * kBinsFirst)) ||
            (rc = dev_alloc_t(h, h->allocs, &h->dense, region_entries, false)) ||
            (rc = dev_alloc_t(h, h->allocs, &h->dense_dir, (size_t)n * ge.slices * ge.parts * 4)) ||
            (rc = dev_alloc_t(h, h->allocs, &h->piece_bits, (size_t)n * ge.slices * ge.parts * 4 * kPieceWords, false)) ||
            (rc = dev_alloc_t(h, h->allocs, &h->small_ctr, (size_t)n)) ||
            (rc = dev_alloc_t(h, h->allocs, &h->sel_count, 1)) ||
            (rc = dev_alloc_t(h, h->allocs, &h->sel_out_idx, (size_t)ge.k)) ||
            (rc = dev_alloc_t(h, h->allocs, &h->sel_out_val, (size_t)ge.k)))
            return bail(rc);
        if ((rc = reset_topk_workers(h))) return bail(rc);
    }
    apply_streaming(h);
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
    {
        DeviceScope scope;
        if (scope.enter(h) == COMP_AMS_OK) {
            (void)hipStreamSynchronize(h->stream);
            prof_clear(h);
            free_all(h->allocs);
            free_all(h->tb_allocs);
        }
    }
    delete h;
}

int comp_ams_set_blocks(comp_ams_t *h, const int64_t *offsets_host, int32_t n_blocks)
{
    ENTER_STATE(h);
    if (rc) return rc;
    if (h->compressor != COMP_AMS_BLOCKSIGN) return fail(h, COMP_AMS_ESTATE, "set_blocks needs a BLOCKSIGN handle");
    if (!offsets_host) return fail(h, COMP_AMS_EINVAL, "offsets is NULL");
    if (n_blocks < 1 || (int64_t)n_blocks > h->d) return fail(h, COMP_AMS_EINVAL, "n_blocks=%d must be in [1, d]", n_blocks);
    if (offsets_host[0] != 0 || offsets_host[n_blocks] != h->d)
        return fail(h, COMP_AMS_EINVAL, "offsets must start at 0 and end at d");
    for (int b = 0; b < n_blocks; ++b)
        if (offsets_host[b + 1] <= offsets_host[b]) return fail(h, COMP_AMS_EINVAL, "offsets must be strictly increasing (block %d)", b);
    if (h->pending) {
        // the stored vectors still owe the subtraction of the old blocks' scales: do it in place
        for (int i = 0; i < h->n; ++i) launch_materialize(h, i, h->e + (size_t)i * (size_t)h->ld);
        HIP_TRY(h, hipGetLastError());
        h->pending = false;
    }
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    std::vector<int64_t> off(offsets_host, offsets_host + n_blocks + 1);
    return build_block_table(h, off, 0);
}

int comp_ams_set_theta(comp_ams_t *h, const float *theta, int on_device)
{
    ENTER_STATE(h);
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

int comp_ams_set_streaming(comp_ams_t *h, int32_t rows, int32_t state)
{
    if (!h) return fail(nullptr, COMP_AMS_EINVAL, "handle is NULL");
    if (rows < -1 || rows > 1 || state < -1 || state > 1)
        return fail(h, COMP_AMS_EINVAL, "streaming choices are -1 (automatic), 0 (cached) or 1 (streamed)");
    h->rows_choice = rows;
    h->state_choice = state;
    apply_streaming(h);
    return COMP_AMS_OK;
}

int comp_ams_set_tile_order(comp_ams_t *h, int32_t chunk)
{
    if (!h) return fail(nullptr, COMP_AMS_EINVAL, "handle is NULL");
    if (chunk < -1 || chunk > 65536) return fail(h, COMP_AMS_EINVAL, "chunk is -1 (automatic) or 0 .. 65536 tiles");
    h->chunk_choice = chunk;
    apply_streaming(h);
    return COMP_AMS_OK;
}

int comp_ams_set_pass_lds(comp_ams_t *h, int32_t bytes)
{
    if (!h) return fail(nullptr, COMP_AMS_EINVAL, "handle is NULL");
    if (bytes < -1 || bytes > 61440) return fail(h, COMP_AMS_EINVAL, "bytes is -1 (automatic) or 0 .. 61440");
    h->lds_choice = bytes;
    apply_streaming(h);
    return COMP_AMS_OK;
}

int comp_ams_set_rand(comp_ams_t *h, uint64_t seed, uint32_t draw)
{
    if (!h) return fail(nullptr, COMP_AMS_EINVAL, "handle is NULL");
    if (h->compressor != COMP_AMS_RANDK) return fail(h, COMP_AMS_ESTATE, "set_rand needs a RANDK handle");
    if (h->steps != 0) return fail(h, COMP_AMS_ESTATE, "the draws can only be set before the first step");
    h->rand_seed = seed;
    h->draw = draw;
    return COMP_AMS_OK;
}

int comp_ams_set_eps_mode(comp_ams_t *h, int32_t mode)
{
    if (!h) return fail(nullptr, COMP_AMS_EINVAL, "handle is NULL");
    if (mode != 0 && mode != 1) return fail(h, COMP_AMS_EINVAL, "eps mode must be 0 or 1");
    h->params.eps_mode = mode;
    return COMP_AMS_OK;
}

int comp_ams_step(comp_ams_t *h, const float *grads_dev, void *hip_stream) { return step_any(h, grads_dev, hip_stream); }

int comp_ams_step_bf16(comp_ams_t *h, const uint16_t *grads_bf16_dev, void *hip_stream)
{
    return step_any(h, grads_bf16_dev, hip_stream);
}

int comp_ams_step_f16(comp_ams_t *h, const uint16_t *grads_f16_dev, void *hip_stream)
{
    return step_any(h, reinterpret_cast<const f16bits *>(grads_f16_dev), hip_stream);
}

int comp_ams_get_theta(comp_ams_t *h, float *out, int on_device)
{
    ENTER_STATE(h);
    return rc ? rc : copy_out(h, out, h->theta, (size_t)h->d, on_device);
}
int comp_ams_get_m(comp_ams_t *h, float *out, int on_device)
{
    ENTER_STATE(h);
    return rc ? rc : copy_out(h, out, h->m, (size_t)h->d, on_device);
}
int comp_ams_get_v(comp_ams_t *h, float *out, int on_device)
{
    ENTER_STATE(h);
    return rc ? rc : copy_out(h, out, h->v, (size_t)h->d, on_device);
}
int comp_ams_get_vhat(comp_ams_t *h, float *out, int on_device)
{
    ENTER_STATE(h);
    return rc ? rc : copy_out(h, out, h->vhat, (size_t)h->d, on_device);
}

int comp_ams_get_error(comp_ams_t *h, int32_t worker, float *out, int on_device)
{
    ENTER_STATE(h);
    if (rc) return rc;
    if (h->method != COMP_AMS_METHOD_EF)
        return fail(h, COMP_AMS_ESTATE, "this method keeps no error memory (CD-Adam: see comp_ams_get_ghat_worker)");
    if (worker < 0 || worker >= h->n) return fail(h, COMP_AMS_EINVAL, "worker %d out of [0, %d)", worker, h->n);
    if (!out) return fail(h, COMP_AMS_EINVAL, "output pointer is NULL");
    launch_materialize(h, worker, on_device ? out : h->row_tmp);
    HIP_TRY(h, hipGetLastError());
    if (!on_device) return copy_out(h, out, h->row_tmp, (size_t)h->d, 0);
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    return COMP_AMS_OK;
}

namespace {
// The kept (index, value) pairs of one vector's last selection, sorted by index, to host arrays.
// Leaves the kept (index, value) pairs of one vector in sel_out_idx / sel_out_val and their number in sel_count
// (device memory), on the handle's stream.  worker_row: the worker whose stored row holds the vector under error
// feedback with magnitude keys (zeros are then not among the candidates and come from the row), else -1.
int launch_gather(comp_ams *h, const TkGeom &ge, int vec, const TkWorker *ws, const uint2 *cand,
                  const uint4 *tile_dir, int worker_row)
{
    HIP_TRY(h, hipMemsetAsync(h->sel_count, 0, sizeof(uint32_t), h->stream));
    tk_gather_selected<<<ge.n_tiles, kThreads, 0, h->stream>>>(ge, vec, ws, cand, tile_dir, h->sel_count,
                                                              h->sel_out_idx, h->sel_out_val);
    if (worker_row >= 0)
        tk_gather_zero_tail<<<(unsigned)((h->d + kThreads - 1) / kThreads), kThreads, 0, h->stream>>>(
            h->e + (size_t)worker_row * (size_t)h->ld, ge, ws + vec, h->sel_count, h->sel_out_idx, h->sel_out_val);
    HIP_TRY(h, hipGetLastError());
    return COMP_AMS_OK;
}

// The row that holds worker `w`'s compressed vector when zeros are counted instead of listed, else -1.
int zero_row_of(const comp_ams *h, int w, bool server)
{
    return (!server && h->method == COMP_AMS_METHOD_EF && h->compressor == COMP_AMS_TOPK) ? w : -1;
}

int gather_selected(comp_ams *h, const TkGeom &ge, int worker, const TkWorker *ws, const uint2 *cand,
                    const uint4 *tile_dir, uint32_t *idx_host, float *val_host, int worker_row)
{
    const size_t k = (size_t)ge.k;
    int rc = launch_gather(h, ge, worker, ws, cand, tile_dir, worker_row);
    if (rc) return rc;
    uint32_t total = 0;
    std::vector<uint32_t> idx(k);
    std::vector<float> val(k);
    HIP_TRY(h, hipMemcpyAsync(&total, h->sel_count, sizeof(uint32_t), hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(h, hipMemcpyAsync(idx.data(), h->sel_out_idx, k * sizeof(uint32_t), hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(h, hipMemcpyAsync(val.data(), h->sel_out_val, k * sizeof(float), hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    if (total != k) return fail(h, COMP_AMS_EDEVICE, "internal: %u coordinates kept, expected k=%zu", total, k);
    std::vector<uint32_t> order(k);
    for (size_t r = 0; r < k; ++r) order[r] = (uint32_t)r;
    std::sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) { return idx[a] < idx[b]; });
    for (size_t r = 0; r < k; ++r) {
        if (idx_host) idx_host[r] = idx[order[r]];
        if (val_host) val_host[r] = val[order[r]];
    }
    return COMP_AMS_OK;
}
}  // namespace

int comp_ams_get_selected(comp_ams_t *h, int32_t worker, uint32_t *idx_host, float *val_host)
{
    ENTER_STATE(h);
    if (rc) return rc;
    if (!is_sparse(h)) return fail(h, COMP_AMS_ESTATE, "get_selected needs a TOPK handle");
    if (h->method == COMP_AMS_METHOD_NONE) return fail(h, COMP_AMS_ESTATE, "this handle does not compress");
    if (h->steps == 0) return fail(h, COMP_AMS_ESTATE, "no step has run yet");
    if (worker < 0 || worker >= h->n) return fail(h, COMP_AMS_EINVAL, "worker %d out of [0, %d)", worker, h->n);
    return gather_selected(h, h->ge, worker, h->ws, h->cand, h->tile_dir, idx_host, val_host,
                           zero_row_of(h, worker, false));
}

int comp_ams_get_server_selected(comp_ams_t *h, uint32_t *idx_host, float *val_host)
{
    ENTER_STATE(h);
    if (rc) return rc;
    if (!is_sparse(h) || h->method != COMP_AMS_METHOD_CD)
        return fail(h, COMP_AMS_ESTATE, "get_server_selected needs a TOPK handle set to CD-Adam");
    if (h->steps == 0) return fail(h, COMP_AMS_ESTATE, "no step has run yet");
    return gather_selected(h, h->srv.ge, 0, h->srv.ws, h->srv.cand, h->srv.tile_dir, idx_host, val_host, -1);
}

int comp_ams_get_scales(comp_ams_t *h, float *out_host)
{
    ENTER_STATE(h);
    if (rc) return rc;
    if (h->compressor != COMP_AMS_BLOCKSIGN) return fail(h, COMP_AMS_ESTATE, "get_scales needs a BLOCKSIGN handle");
    if (h->method == COMP_AMS_METHOD_NONE) return fail(h, COMP_AMS_ESTATE, "this handle does not compress");
    if (h->steps == 0) return fail(h, COMP_AMS_ESTATE, "no step has run yet");
    return copy_out(h, out_host, h->scales, (size_t)h->n * (size_t)h->tb.n_blocks, 0);
}

int comp_ams_get_signs(comp_ams_t *h, int32_t worker, uint8_t *bits_host)
{
    ENTER_STATE(h);
    if (rc) return rc;
    if (h->compressor != COMP_AMS_BLOCKSIGN) return fail(h, COMP_AMS_ESTATE, "get_signs needs a BLOCKSIGN handle");
    if (h->method == COMP_AMS_METHOD_NONE) return fail(h, COMP_AMS_ESTATE, "this handle does not compress");
    if (h->steps == 0) return fail(h, COMP_AMS_ESTATE, "no step has run yet");
    const bool server = (h->method == COMP_AMS_METHOD_CD && worker == h->n);
    if (!server && (worker < 0 || worker >= h->n)) return fail(h, COMP_AMS_EINVAL, "worker %d out of range", worker);
    if (!bits_host) return fail(h, COMP_AMS_EINVAL, "output pointer is NULL");
    // the wire order (bit j % 8 of byte j / 8 = coordinate j) is what bs_pack_signs writes as 32-bit words;
    // row_tmp (d floats) holds the (d + 31) / 32 words
    const size_t words = (size_t)h->ld / 16;
    const uint16_t *src = server ? h->signs_srv : h->signs + (size_t)worker * words;
    const int64_t out_words = (h->d + 31) / 32;
    uint32_t *packed = reinterpret_cast<uint32_t *>(h->row_tmp);
    bs_pack_signs<<<(unsigned)((out_words + kThreads - 1) / kThreads), kThreads, 0, h->stream>>>(src, h->d, packed);
    HIP_TRY(h, hipGetLastError());
    HIP_TRY(h, hipMemcpyAsync(bits_host, packed, ((size_t)h->d + 7) / 8, hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    return COMP_AMS_OK;
}

int comp_ams_message_bytes(comp_ams_t *h, uint64_t *bytes)
{
    if (!h) return fail(nullptr, COMP_AMS_EINVAL, "handle is NULL");
    if (!bytes) return fail(h, COMP_AMS_EINVAL, "output pointer is NULL");
    if (h->method == COMP_AMS_METHOD_NONE)
        *bytes = 4ull * (uint64_t)h->d;
    else if (is_sparse(h))
        *bytes = 8ull * (uint64_t)h->k;
    else
        *bytes = 4ull * (uint64_t)h->tb.n_blocks + 4ull * (uint64_t)((h->d + 31) / 32);
    return COMP_AMS_OK;
}

int comp_ams_pack_message(comp_ams_t *h, int32_t who, void *buf_dev, uint64_t capacity, uint64_t *bytes)
{
    ENTER_STATE(h);
    if (rc) return rc;
    if (h->method == COMP_AMS_METHOD_NONE) return fail(h, COMP_AMS_ESTATE, "this handle does not compress");
    if (h->steps == 0) return fail(h, COMP_AMS_ESTATE, "no step has run yet");
    const bool server = (h->method == COMP_AMS_METHOD_CD && who == h->n);
    if (!server && (who < 0 || who >= h->n)) return fail(h, COMP_AMS_EINVAL, "vector %d out of range", who);
    uint64_t need = 0;
    (void)comp_ams_message_bytes(h, &need);
    if (bytes) *bytes = need;
    if (!buf_dev) return fail(h, COMP_AMS_EINVAL, "buffer is NULL");
    if (reinterpret_cast<uintptr_t>(buf_dev) & 7u) return fail(h, COMP_AMS_EINVAL, "buffer must be 8-byte aligned");
    if (capacity < need)
        return fail(h, COMP_AMS_EINVAL, "buffer of %llu bytes, the message takes %llu", (unsigned long long)capacity,
                    (unsigned long long)need);
    if (is_sparse(h)) {
        const TkGeom &ge = server ? h->srv.ge : h->ge;
        if ((rc = launch_gather(h, ge, server ? 0 : who, server ? h->srv.ws : h->ws, server ? h->srv.cand : h->cand,
                                server ? h->srv.tile_dir : h->tile_dir, zero_row_of(h, who, server))))
            return rc;
        tk_pack_pairs<<<(unsigned)((ge.k + kThreads - 1) / kThreads), kThreads, 0, h->stream>>>(
            h->sel_out_idx, h->sel_out_val, ge.k, static_cast<uint2 *>(buf_dev));
    } else {
        const size_t words = (size_t)h->ld / 16;
        const size_t nb = (size_t)h->tb.n_blocks;
        const float *sc = server ? h->scales_srv : h->scales + (size_t)who * nb;
        const uint16_t *sw = server ? h->signs_srv : h->signs + (size_t)who * words;
        HIP_TRY(h, hipMemcpyAsync(buf_dev, sc, nb * sizeof(float), hipMemcpyDeviceToDevice, h->stream));
        const int64_t out_words = (h->d + 31) / 32;
        bs_pack_signs<<<(unsigned)((out_words + kThreads - 1) / kThreads), kThreads, 0, h->stream>>>(
            sw, h->d, reinterpret_cast<uint32_t *>(static_cast<float *>(buf_dev) + nb));
    }
    HIP_TRY(h, hipGetLastError());
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    return COMP_AMS_OK;
}

}  // extern "C"

// ---------------------------------------------------------------------------------------------------------
// comp_ams_pack_message_noalloc: the gather of a Top-k / Rand-k message runs in a fixed array in device memory
// instead of the handle's buffers.  Every GPU the library runs on holds its own copy of the array, at its own
// address, until the process ends; the name below is only a host-side stand-in, and host code reaches the memory
// through the per-device address from hipGetSymbolAddress (scratch_on_current_device).
namespace {
constexpr uint32_t kScratchMaxK = 1u << 20;                  // largest k the no-alloc entry point accepts
constexpr size_t kScratchHeader = 256;                       // the kept-pairs counter, alone on its lines
constexpr size_t kScratchBytes = kScratchHeader + 2 * sizeof(uint32_t) * (size_t)kScratchMaxK;   // 8 MiB + 256 B
}  // namespace
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

// Address of `scratch` on the current device (which must be device `dev`); looked up once per device.
int scratch_on_current_device(comp_ams *h, int dev, unsigned char **out)
{
    if (dev < 0 || dev >= kMaxDevices) return fail(h, COMP_AMS_EDEVICE, "device %d: only devices 0..%d are supported here", dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        HIP_TRY(h, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(h, COMP_AMS_EDEVICE, "hipGetSymbolAddress gave no address for the scratch array");
        g_scratch_ptr[dev] = p;
    }
    *out = static_cast<unsigned char *>(g_scratch_ptr[dev]);
    return COMP_AMS_OK;
}

__global__ void fill_words(uint32_t *dst, uint32_t value, uint32_t count)
{
    const uint32_t q = blockIdx.x * blockDim.x + threadIdx.x;
    if (q < count) dst[q] = value;
}
}  // namespace

extern "C" {

int comp_ams_pack_message_noalloc(comp_ams_t *h, int32_t who, void *buf_dev, uint64_t capacity, uint64_t *bytes)
{
    ENTER_STATE(h);
    if (rc) return rc;
    if (h->method == COMP_AMS_METHOD_NONE) return fail(h, COMP_AMS_ESTATE, "this handle does not compress");
    if (h->steps == 0) return fail(h, COMP_AMS_ESTATE, "no step has run yet");
    const bool server = (h->method == COMP_AMS_METHOD_CD && who == h->n);
    if (!server && (who < 0 || who >= h->n)) return fail(h, COMP_AMS_EINVAL, "vector %d out of range", who);
    uint64_t need = 0;
    (void)comp_ams_message_bytes(h, &need);
    if (bytes) *bytes = need;
    if (!buf_dev) return fail(h, COMP_AMS_EINVAL, "buffer is NULL");
    if (reinterpret_cast<uintptr_t>(buf_dev) & 7u) return fail(h, COMP_AMS_EINVAL, "buffer must be 8-byte aligned");
    if (capacity < need)
        return fail(h, COMP_AMS_EINVAL, "buffer of %llu bytes, the message takes %llu", (unsigned long long)capacity,
                    (unsigned long long)need);
    if (is_sparse(h)) {
        if ((uint64_t)h->k > kScratchMaxK)
            return fail(h, COMP_AMS_EINVAL, "k=%lld exceeds the %u pairs the fixed scratch array holds (use comp_ams_pack_message)",
                        (long long)h->k, kScratchMaxK);
        unsigned char *sp = nullptr;
        if ((rc = scratch_on_current_device(h, h->device, &sp))) return rc;
        uint32_t *count = reinterpret_cast<uint32_t *>(sp);
        uint32_t *idx = reinterpret_cast<uint32_t *>(sp + kScratchHeader);
        float *val = reinterpret_cast<float *>(sp + kScratchHeader + sizeof(uint32_t) * (size_t)kScratchMaxK);
        const TkGeom &ge = server ? h->srv.ge : h->ge;
        const int vec = server ? 0 : who;
        const TkWorker *ws = server ? h->srv.ws : h->ws;
        // the array keeps the last call's contents: the counter must start at zero (a kernel, not a memset node,
        // so that the call can also be recorded into a graph)
        fill_words<<<1, kWave, 0, h->stream>>>(count, 0u, 1u);
        tk_gather_selected<<<ge.n_tiles, kThreads, 0, h->stream>>>(ge, vec, ws, server ? h->srv.cand : h->cand,
                                                                  server ? h->srv.tile_dir : h->tile_dir, count, idx, val);
        const int zrow = zero_row_of(h, who, server);
        if (zrow >= 0)
            tk_gather_zero_tail<<<(unsigned)((h->d + kThreads - 1) / kThreads), kThreads, 0, h->stream>>>(
                h->e + (size_t)zrow * (size_t)h->ld, ge, ws + vec, count, idx, val);
        tk_pack_pairs<<<(unsigned)((ge.k + kThreads - 1) / kThreads), kThreads, 0, h->stream>>>(
            idx, val, ge.k, static_cast<uint2 *>(buf_dev));
    } else {
        // scaled sign: scales and sign words go straight from the handle's side buffers to the caller's buffer
        const size_t words = (size_t)h->ld / 16;
        const size_t nb = (size_t)h->tb.n_blocks;
        const float *sc = server ? h->scales_srv : h->scales + (size_t)who * nb;
        const uint16_t *sw = server ? h->signs_srv : h->signs + (size_t)who * words;
        HIP_TRY(h, hipMemcpyAsync(buf_dev, sc, nb * sizeof(float), hipMemcpyDeviceToDevice, h->stream));
        const int64_t out_words = (h->d + 31) / 32;
        bs_pack_signs<<<(unsigned)((out_words + kThreads - 1) / kThreads), kThreads, 0, h->stream>>>(
            sw, h->d, reinterpret_cast<uint32_t *>(static_cast<float *>(buf_dev) + nb));
    }
    HIP_TRY(h, hipGetLastError());
    return COMP_AMS_OK;
}

int32_t comp_ams_n_blocks(comp_ams_t *h)
{
    if (!h) return fail(nullptr, COMP_AMS_EINVAL, "handle is NULL");
    return h->compressor == COMP_AMS_BLOCKSIGN ? h->tb.n_blocks : 0;
}

int comp_ams_set_state(comp_ams_t *h, const float *m, const float *v, const float *vhat, const float *e, int on_device)
{
    ENTER_STATE(h);
    if (rc) return rc;
    const size_t d = (size_t)h->d;
    if (m && (rc = copy_in(h, h->m, m, d, on_device))) return rc;
    if (v && (rc = copy_in(h, h->v, v, d, on_device))) return rc;
    if (vhat && (rc = copy_in(h, h->vhat, vhat, d, on_device))) return rc;
    if (e && h->method != COMP_AMS_METHOD_EF)
        return fail(h, COMP_AMS_ESTATE, "this method keeps no error memory (CD-Adam: see comp_ams_set_markov_state)");
    if (e) {
        HIP_TRY(h, hipMemcpy2DAsync(h->e, (size_t)h->ld * sizeof(float), e, d * sizeof(float), d * sizeof(float),
                                    (size_t)h->n, on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice,
                                    h->stream));
        HIP_TRY(h, hipStreamSynchronize(h->stream));
        // the rows now hold e itself: nothing is pending on them
        h->pending = false;
        if (is_sparse(h) && (rc = reset_topk_workers(h))) return rc;
    }
    return COMP_AMS_OK;
}

int comp_ams_sync(comp_ams_t *h)
{
    ENTER_STATE(h);
    if (rc) return rc;
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    return COMP_AMS_OK;
}

int comp_ams_profile(comp_ams_t *h, int enable)
{
    ENTER_STATE(h);
    if (rc) return rc;
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    prof_clear(h);
    h->prof_on = enable != 0;
    return COMP_AMS_OK;
}

int comp_ams_profile_read(comp_ams_t *h, int32_t slot, const char **name, double *total_ms, int64_t *launches)
{
    ENTER_STATE(h);
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

int comp_ams_get_selection_info(comp_ams_t *h, int32_t worker, uint32_t *out_host)
{
    ENTER_STATE(h);
    if (rc) return rc;
    if (!is_sparse(h)) return fail(h, COMP_AMS_ESTATE, "get_selection_info needs a TOPK handle");
    if (worker < 0 || worker >= h->n) return fail(h, COMP_AMS_EINVAL, "worker %d out of [0, %d)", worker, h->n);
    if (!out_host) return fail(h, COMP_AMS_EINVAL, "output pointer is NULL");
    TkWorker w;
    HIP_TRY(h, hipMemcpyAsync(&w, h->ws + worker, sizeof w, hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    out_host[0] = w.guess;
    out_host[1] = w.slack;
    out_host[2] = w.relisted;
    out_host[3] = w.pshift;
    out_host[4] = w.prefix;
    out_host[5] = w.rank;
    out_host[6] = w.whole;
    out_host[7] = (uint32_t)(w.tc >> (h->ge.idx_bits + kFineShift));
    return COMP_AMS_OK;
}

int comp_ams_set_method(comp_ams_t *h, int32_t method)
{
    ENTER_STATE(h);
    if (rc) return rc;
    if (method < COMP_AMS_METHOD_EF || method > COMP_AMS_METHOD_NONE) return fail(h, COMP_AMS_EINVAL, "unknown method %d", method);
    if (method == h->method) return COMP_AMS_OK;
    if (h->steps != 0) return fail(h, COMP_AMS_ESTATE, "the method can only be chosen before the first step");
    if (method == COMP_AMS_METHOD_CD && !h->ghat_srv) {
        const size_t ld = (size_t)h->ld;
        if ((rc = dev_alloc_t(h, h->allocs, &h->ghat_srv, ld)) || (rc = dev_alloc_t(h, h->allocs, &h->gtil, ld)))
            return rc;
        if (h->compressor == COMP_AMS_BLOCKSIGN) {
            if ((rc = dev_alloc_t(h, h->allocs, &h->signs_srv, ld / 16))) return rc;
        } else {
            TkSide &sv = h->srv;
            sv.ge = h->ge;
            sv.ge.n = 1;
            // ghat and gtilde are reused within the step if they are small enough to stay cached
            sv.ge.stream_rows = 2 * (size_t)h->ld * sizeof(float) > kCacheResidentBytes ? 1 : 0;
            sv.ge.relist_wgs = (int32_t)std::min<int64_t>(sv.ge.n_tiles, 2048);
            // one vector, all tiles: enough regions that a cursor sees few tens of atomic adds
            int slices = kMinSlices;
            while (slices < kMaxSlices && sv.ge.n_tiles / slices > 32) slices *= 2;
            set_slices(sv.ge, slices);
            const size_t tiles = (size_t)sv.ge.n_tiles;
            const size_t region_entries = (size_t)sv.ge.slices * (size_t)sv.ge.region_cap;
            if ((rc = dev_alloc_t(h, h->allocs, &sv.ws, 1)) ||
                (rc = dev_alloc_t(h, h->allocs, &sv.cand, region_entries, false)) ||
                (rc = dev_alloc_t(h, h->allocs, &sv.cursor, (size_t)sv.ge.slices)) ||
                (rc = dev_alloc_t(h, h->allocs, &h->cursor_b_s, (size_t)sv.ge.slices)) ||
                (rc = dev_alloc_t(h, h->allocs, &sv.tile_dir, tiles)) ||
                (rc = dev_alloc_t(h, h->allocs, &h->hist_full_s, (size_t)kBins1)) ||
                (rc = dev_alloc_t(h, h->allocs, &h->hist1_s, (size_t)kBins1)) ||
                (rc = dev_alloc_t(h, h->allocs, &h->histf_s, (size_t)kFineWindow)) ||
                (rc = dev_alloc_t(h, h->allocs, &h->hist2_s, (size_t)kBinsFirst)) ||
                (rc = dev_alloc_t(h, h->allocs, &h->dense_s, region_entries, false)) ||
                (rc = dev_alloc_t(h, h->allocs, &h->dense_dir_s, (size_t)sv.ge.slices * sv.ge.parts * 4)) ||
                (rc = dev_alloc_t(h, h->allocs, &h->piece_bits_s, (size_t)sv.ge.slices * sv.ge.parts * 4 * kPieceWords,
                                  false)))
                return rc;
        }
    }
    if (is_sparse(h) && (rc = reset_topk_workers(h))) return rc;
    // the stored rows change their meaning (error memory <-> Markov sequence): start both from zero
    HIP_TRY(h, hipMemsetAsync(h->e, 0, (size_t)h->ld * (size_t)h->n * sizeof(float), h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    h->pending = false;
    h->method = method;
    apply_streaming(h);
    return COMP_AMS_OK;
}

namespace {
int need_cd(comp_ams *h)
{
    return h->method == COMP_AMS_METHOD_CD ? COMP_AMS_OK : fail(h, COMP_AMS_ESTATE, "needs a handle set to CD-Adam");
}
}  // namespace

int comp_ams_get_ghat_worker(comp_ams_t *h, int32_t worker, float *out, int on_device)
{
    ENTER_STATE(h);
    if (rc || (rc = need_cd(h))) return rc;
    if (worker < 0 || worker >= h->n) return fail(h, COMP_AMS_EINVAL, "worker %d out of [0, %d)", worker, h->n);
    if (!out) return fail(h, COMP_AMS_EINVAL, "output pointer is NULL");
    launch_materialize(h, worker, on_device ? out : h->row_tmp);
    HIP_TRY(h, hipGetLastError());
    if (!on_device) return copy_out(h, out, h->row_tmp, (size_t)h->d, 0);
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    return COMP_AMS_OK;
}

int comp_ams_get_ghat_server(comp_ams_t *h, float *out, int on_device)
{
    ENTER_STATE(h);
    if (rc || (rc = need_cd(h))) return rc;
    return copy_out(h, out, h->ghat_srv, (size_t)h->d, on_device);
}

int comp_ams_get_gtilde(comp_ams_t *h, float *out, int on_device)
{
    ENTER_STATE(h);
    if (rc || (rc = need_cd(h))) return rc;
    return copy_out(h, out, h->gtil, (size_t)h->d, on_device);
}

int comp_ams_get_server_scales(comp_ams_t *h, float *out_host)
{
    ENTER_STATE(h);
    if (rc || (rc = need_cd(h))) return rc;
    if (h->compressor != COMP_AMS_BLOCKSIGN) return fail(h, COMP_AMS_ESTATE, "get_server_scales needs a BLOCKSIGN handle");
    if (h->steps == 0) return fail(h, COMP_AMS_ESTATE, "no step has run yet");
    return copy_out(h, out_host, h->scales_srv, (size_t)h->tb.n_blocks, 0);
}

int comp_ams_set_markov_state(comp_ams_t *h, const float *ghat_workers, const float *ghat_server, const float *gtilde,
                              int on_device)
{
    ENTER_STATE(h);
    if (rc || (rc = need_cd(h))) return rc;
    const size_t d = (size_t)h->d;
    if (ghat_server && (rc = copy_in(h, h->ghat_srv, ghat_server, d, on_device))) return rc;
    if (gtilde && (rc = copy_in(h, h->gtil, gtilde, d, on_device))) return rc;
    if (ghat_workers) {
        HIP_TRY(h, hipMemcpy2DAsync(h->e, (size_t)h->ld * sizeof(float), ghat_workers, d * sizeof(float),
                                    d * sizeof(float), (size_t)h->n,
                                    on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice, h->stream));
        HIP_TRY(h, hipStreamSynchronize(h->stream));
        h->pending = false;   // the rows hold ghat_i itself
    }
    return COMP_AMS_OK;   // the Top-k guesses are left as they are: a guess is only a hint
}

int comp_ams_message_bits(comp_ams_t *h, uint64_t *uplink_per_worker, uint64_t *downlink)
{
    if (!h) return fail(nullptr, COMP_AMS_EINVAL, "handle is NULL");
    const uint64_t dense = 32ull * (uint64_t)h->d;
    const uint64_t packed = is_sparse(h) ? 64ull * (uint64_t)h->k
                                                           : (uint64_t)h->d + 32ull * (uint64_t)h->tb.n_blocks;
    if (uplink_per_worker) *uplink_per_worker = h->method == COMP_AMS_METHOD_NONE ? dense : packed;
    if (downlink) *downlink = h->method == COMP_AMS_METHOD_CD ? packed : dense;
    return COMP_AMS_OK;
}

int comp_ams_probe_copy(float *dst_dev, const float *src_dev, int64_t count, void *hip_stream)
{
    if (!dst_dev || !src_dev) return fail(nullptr, COMP_AMS_EINVAL, "probe_copy: NULL pointer");
    if (count < 4 || (count & 3) || ((reinterpret_cast<uintptr_t>(dst_dev) | reinterpret_cast<uintptr_t>(src_dev)) & 15u))
        return fail(nullptr, COMP_AMS_EINVAL, "probe_copy: count must be a positive multiple of 4 and the pointers 16-byte aligned");
    const int64_t vecs = count / 4;
    if (vecs > (int64_t)1 << 40) return fail(nullptr, COMP_AMS_EINVAL, "probe_copy: count too large");
    const int64_t pieces = (vecs + 4 * kThreads - 1) / (4 * kThreads);
    // The launch shape a plain copy measured fastest with (1 GiB to 1 GiB, one session): two workgroups per compute
    // unit (60 KB of LDS reserved, none used) and the XCD-aware piece order with chunks of 16 - 6.75 TB/s, against
    // 6.0 TB/s with neither, 6.35 with the LDS alone and 5.7 with the order alone.  Small copies keep the plain shape.
    const bool large = vecs * 16 >= ((int64_t)256 << 20);
    const int chunk = large ? 16 : 0;
    const unsigned lds = large ? 61440u : 0u;
    probe_copy<<<grid_blocks(pieces, chunk), kThreads, lds, static_cast<hipStream_t>(hip_stream)>>>(dst_dev, src_dev,
                                                                                                      vecs, chunk);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(nullptr, COMP_AMS_EDEVICE, "probe_copy launch failed: %s", hipGetErrorString(e));
    return COMP_AMS_OK;
}

int comp_ams_probe_update(float *x_dev, const float *g_dev, int64_t rows, int64_t d, void *hip_stream)
{
    if (!x_dev || !g_dev) return fail(nullptr, COMP_AMS_EINVAL, "probe_update: NULL pointer");
    if (rows < 1 || rows > 65535 || d < 4 || (d & 3) || d >= (int64_t)1 << 40 ||
        ((reinterpret_cast<uintptr_t>(x_dev) | reinterpret_cast<uintptr_t>(g_dev)) & 15u))
        return fail(nullptr, COMP_AMS_EINVAL, "probe_update: 1 <= rows <= 65535, d a positive multiple of 4, pointers 16-byte aligned");
    const int64_t pieces = (d + kTile - 1) / kTile;
    if (pieces > (int64_t)1 << 30) return fail(nullptr, COMP_AMS_EINVAL, "probe_update: rows too long");
    // The launch shape this pattern measured fastest with on rows far beyond the caches (8 rows of 110 M floats, one
    // session: 16 KB per workgroup, 256 or 512 threads, 0 - 60 KB of LDS reserved, chunks of 0 - 32 pieces): three
    // workgroups per compute unit (40 KB of LDS reserved, none used) and chunks of 32 - 6.43 TB/s, against 5.96 TB/s
    // in the plain shape and 5.35 TB/s with ordinary loads and stores.  Small problems keep the plain shape.
    const bool large = rows * d * (int64_t)sizeof(float) >= ((int64_t)256 << 20);
    const int chunk = large ? 32 : 0;
    const unsigned lds = large ? 40960u : 0u;
    probe_update<<<dim3(grid_blocks(pieces, chunk), (unsigned)rows), kThreads, lds, static_cast<hipStream_t>(hip_stream)>>>(
        x_dev, g_dev, d, (int)pieces, chunk);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(nullptr, COMP_AMS_EDEVICE, "probe_update launch failed: %s", hipGetErrorString(e));
    return COMP_AMS_OK;
}

const char *comp_ams_last_error(const comp_ams_t *h) { return h ? h->err.c_str() : g_create_error.c_str(); }

}  // extern "C"
