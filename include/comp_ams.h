/*
 * comp_ams.h - C ABI of the MI355X (gfx950) library for communication-compressed
 * AMSGrad with error feedback, n workers simulated as a batch on one GPU.
 *
 * One step (comp_ams_step) computes, for gradients g_i (i = 0..n-1), each of d fp32:
 *   x_i     = g_i + e_i                      error feedback, Section 4 ("Error feedback for SGD")
 *   ghat_i  = C(x_i)                         Top-k or scaled sign, Appendix A
 *   e_i     = x_i - ghat_i                   Section 4
 *   gbar    = (1/n) sum_i ghat_i             server aggregation, Section 3
 *   m       = beta1 m + (1-beta1) gbar       AMSGrad, Section 3 / Algorithm 1 update lines
 *   v       = beta2 v + (1-beta2) gbar^2
 *   vhat    = max(vhat, v)
 *   theta   = theta - lr m / (sqrt(vhat) + eps)        [eps mode 0]
 *           = theta - lr m / sqrt(vhat + eps)          [eps mode 1, the paper's Vhat = diag(vhat + nu)]
 * All arithmetic is fp32, one rounding per operation, no fused multiply-add; the sum over
 * workers runs in ascending worker order.  There is no bias correction (the paper has none).
 *
 * Conventions
 *  - Every function returns a status code; nothing throws or aborts.  On failure outputs
 *    are left untouched and comp_ams_last_error() describes the reason.
 *  - The handle owns all optimiser state and scratch in device memory.  It is allocated in
 *    comp_ams_create (and comp_ams_set_blocks); comp_ams_step allocates nothing.
 *  - "dev" pointers are device pointers on the GPU that was current when the handle was
 *    created; "host" pointers are ordinary host memory.  An entry point that takes a handle makes
 *    that GPU current while it runs and restores the caller's current device before it returns.  Where a function takes
 *    `on_device`, 0 means the buffer is host memory and non-zero means device memory.
 *  - comp_ams_step is asynchronous on the given HIP stream.  Getters and setters run on the
 *    stream of the most recent step (the null stream before the first) and return after
 *    their copy has completed.
 *  - A step may leave the last part of its work - the AMSGrad update, which nothing in the next
 *    step's compression depends on - to be launched together with the next step (block sign with
 *    uniform blocks of a multiple of 4096 coordinates does: one launch per step instead of two).
 *    The difference cannot be observed through this interface: every call that reads or replaces
 *    state first launches what is pending, with the hyper-parameters of the step it belongs to,
 *    and comp_ams_sync waits for it.  A caller that only synchronises its own stream has waited
 *    for everything but that pending update.
 *  - A handle must not be used from two threads at once.
 *  - Arguments are validated on the host before any device call, so invalid arguments are
 *    reported as COMP_AMS_EINVAL also on a machine without a GPU.
 */
#ifndef COMP_AMS_H
#define COMP_AMS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct comp_ams comp_ams_t;

enum { COMP_AMS_TOPK = 0, COMP_AMS_BLOCKSIGN = 1, COMP_AMS_RANDK = 2 };

/* How the compressor is used: classical error feedback (Section 4; the step described above);
 * CD-Adam (Section 5, Algorithm 1): Markov compression in both directions; naive compression
 * (Section 4, "Naive compression": ghat_i = C(g_i), nothing is remembered); or not at all (vanilla
 * distributed AMSGrad, Section 3: gbar = (1/n) sum_i g_i) - the arms of the paper's comparison. */
enum { COMP_AMS_METHOD_EF = 0, COMP_AMS_METHOD_CD = 1, COMP_AMS_METHOD_NAIVE = 2, COMP_AMS_METHOD_NONE = 3 };

enum {
    COMP_AMS_OK = 0,
    COMP_AMS_EINVAL = -1,  /* bad argument (range, NULL, inconsistent block table) */
    COMP_AMS_ENOMEM = -2,  /* device or host allocation failed */
    COMP_AMS_EDEVICE = -3, /* a HIP call failed (no device, launch error, copy error) */
    COMP_AMS_ESTATE = -4   /* call does not apply to this handle (wrong compressor kind, no step yet) */
};

/*
 * Problem statement of Section 3: model dimension d >= 1, n >= 1 workers; hyper-parameters of
 * Algorithm 1's input line: beta1, beta2 in [0,1), eps (the paper's nu) > 0, lr (alpha) > 0.
 *   compressor = COMP_AMS_TOPK:      k_or_block = k, 1 <= k <= d  (Appendix A, "Top-k").
 *   compressor = COMP_AMS_BLOCKSIGN: k_or_block = B >= 1, contiguous blocks of B coordinates,
 *                                    the last one partial; B >= d is the whole-vector scaled
 *                                    sign of Appendix A.
 *   compressor = COMP_AMS_RANDK:     k_or_block = k, 1 <= k <= d  (Appendix A, "Rand-k"): a random
 *                                    set of k coordinates, drawn anew for every step and worker
 *                                    (see comp_ams_set_rand).  Every call that names a TOPK handle
 *                                    below also serves a RANDK handle.
 * d < 2^31 and n*d < 2^40.
 * theta starts at zero until comp_ams_set_theta; m, v, vhat and every e_i start at zero.
 * On success *out receives the handle.
 */
int comp_ams_create(comp_ams_t **out, int64_t d, int32_t n, int32_t compressor, int64_t k_or_block,
                    float beta1, float beta2, float eps, float lr);

/* Frees the handle and everything it owns (waits for pending work).  NULL is a no-op. */
void comp_ams_destroy(comp_ams_t *h);

/*
 * Replace the uniform blocks of a BLOCKSIGN handle by n_blocks contiguous blocks of arbitrary
 * length ("per-layer" scaled sign): host array offsets[0..n_blocks] with offsets[0] = 0,
 * strictly increasing, offsets[n_blocks] = d.  Each block is compressed by Appendix A's scaled
 * sign with the block's own length as divisor.  ESTATE on a TOPK handle.
 */
int comp_ams_set_blocks(comp_ams_t *h, const int64_t *offsets_host, int32_t n_blocks);

/* Initial model x_1 (d floats, copied). */
int comp_ams_set_theta(comp_ams_t *h, const float *theta, int on_device);

/* Step size alpha_t for the following steps (Algorithm 1 allows a non-increasing schedule). */
int comp_ams_set_lr(comp_ams_t *h, float lr);

/* 0 (default): theta -= lr m/(sqrt(vhat)+eps).  1: theta -= lr m/sqrt(vhat+eps), Section 3. */
int comp_ams_set_eps_mode(comp_ams_t *h, int32_t mode);

/*
 * Rand-k (Appendix A, "Rand-k") only, before the first step: the seed of the draws and the number of
 * the next draw (default 0, 0; a resumed run passes the number of steps already taken).  The paper
 * leaves the drawing of S open.  Here coordinate j of the vector `who` (worker i: who = i; the
 * server's vector in Algorithm 1: who = n) gets, at draw t (t grows by one per step), the 31-bit score
 *     mix(mix(j + a) ^ b) >> 1,   a = mix(mix(lo(seed) + t * 0x9e3779b9) ^ hi(seed) ^ who * 0x85ebca6b),
 *                                 b = mix(a + 0xc2b2ae35),
 * mix = the 32-bit finaliser of MurmurHash3 (h ^= h >> 16; h *= 0x85ebca6b; h ^= h >> 13;
 * h *= 0xc2b2ae35; h ^= h >> 16), all in arithmetic mod 2^32, and S is the k coordinates of largest
 * score, the lower index first among equal scores.  S depends on (seed, t, who) only, so a receiver
 * that knows them needs no indices.  A step recorded into a HIP graph repeats its draw when replayed.
 */
int comp_ams_set_rand(comp_ams_t *h, uint64_t seed, uint32_t draw);

/*
 * One optimisation step on grads_dev: n*d floats in device memory, row-major [n][d]
 * (worker i at grads_dev + i*d), read-only, owned by the caller and borrowed until the work
 * enqueued on `hip_stream` (a hipStream_t, NULL = the null stream) has completed.
 * The base pointer must be 4-byte aligned; 16-byte alignment gives the fast path.
 * The call only launches kernels (no allocation, no memset, no wait while the stream stays the
 * same), so it may be recorded into a HIP graph; record after at least one ordinary step on the same
 * stream (the first step of a handle launches a different variant of the first kernel than the later
 * ones) and after comp_ams_sync or any getter (a recorded step is self-contained, so nothing of an
 * earlier step may be pending when recording starts: COMP_AMS_ESTATE otherwise).
 */
int comp_ams_step(comp_ams_t *h, const float *grads_dev, void *hip_stream);

/*
 * The same step with the gradients handed over as bfloat16: grads_bf16_dev holds n*d 16-bit values,
 * [n][d] row-major, each the upper half of an fp32 number (device memory, 2-byte aligned, borrowed
 * and not modified).  They are widened exactly, so the step computes what comp_ams_step computes on
 * the fp32 copy of the same numbers; it reads 2 instead of 4 bytes per gradient element.
 */
int comp_ams_step_bf16(comp_ams_t *h, const uint16_t *grads_bf16_dev, void *hip_stream);

/*
 * The same with IEEE half precision gradients (1 sign, 5 exponent, 10 fraction bits, subnormals
 * included; every finite half value is an fp32 value, so the widening is exact).  Same layout,
 * alignment and ownership as comp_ams_step_bf16.
 */
int comp_ams_step_f16(comp_ams_t *h, const uint16_t *grads_f16_dev, void *hip_stream);

/* State getters: d floats each, copied to `out` (host or device memory per on_device). */
int comp_ams_get_theta(comp_ams_t *h, float *out, int on_device);
int comp_ams_get_m(comp_ams_t *h, float *out, int on_device);
int comp_ams_get_v(comp_ams_t *h, float *out, int on_device);
int comp_ams_get_vhat(comp_ams_t *h, float *out, int on_device);

/* Error memory e_i of worker i in [0,n): d floats. */
int comp_ams_get_error(comp_ams_t *h, int32_t worker, float *out, int on_device);

/*
 * TOPK handles, after at least one step: the k coordinates worker i kept in the last step, as
 * host arrays idx_host[k] (ascending) and val_host[k] (the kept values x_i[idx]); either may be
 * NULL.  Among equal magnitudes the lower index is kept; magnitude order is the order of the
 * fp32 bit pattern with the sign bit cleared.
 */
int comp_ams_get_selected(comp_ams_t *h, int32_t worker, uint32_t *idx_host, float *val_host);

/* BLOCKSIGN handles, after at least one step: the scales of the last step, host array
 * [n][n_blocks] row-major, scale = (sum over the block of |x|) / block length. */
int comp_ams_get_scales(comp_ams_t *h, float *out_host);

/*
 * BLOCKSIGN handles, after at least one step: the sign bits of worker i's message of the last step,
 * packed in coordinate order into (d + 7) / 8 host bytes (bit j % 8 of byte j / 8 is set iff
 * coordinate j is negative, by the IEEE sign bit; the unused high bits of the last byte are 0).
 * Together with the worker's row of comp_ams_get_scales this is the whole message:
 * C(x)_j = (bit ? -1 : +1) * scale[block(j)] (Appendix A, "Scaled sign"; 1 bit per coordinate plus
 * 32 bits per scale).  worker = n on a CD handle gives the server's message instead (with
 * comp_ams_get_server_scales).
 */
int comp_ams_get_signs(comp_ams_t *h, int32_t worker, uint8_t *bits_host);

/* Number of blocks of a BLOCKSIGN handle (0 for TOPK, negative status on error). */
int32_t comp_ams_n_blocks(comp_ams_t *h);

/* Restore optimiser state (checkpoint resume): m, v, vhat of d floats and e of n*d floats
 * ([n][d] row-major); any pointer may be NULL to leave that array as it is. */
int comp_ams_set_state(comp_ams_t *h, const float *m, const float *v, const float *vhat, const float *e,
                       int on_device);

/*
 * Chooses the method of a handle before its first step (COMP_AMS_ESTATE afterwards).
 * COMP_AMS_METHOD_NAIVE and COMP_AMS_METHOD_NONE run the step described at the top with e_i = 0
 * throughout, respectively with ghat_i = g_i (the compressor of the handle is then not used);
 * both leave no error memory to read or restore (COMP_AMS_ESTATE), and NONE has no kept
 * coordinates or scales either.
 * CD-Adam, Section 5, Algorithm 1.  With
 * COMP_AMS_METHOD_CD one comp_ams_step computes, with the handle's compressor C in both directions,
 *   c_i     = C(g_i - ghat_i) ;  ghat_i = ghat_i + c_i          workers, lines 5-6
 *   ghat    = ghat + (1/n) sum_i c_i                            server, line 8 (ascending i, one division)
 *   c       = C(ghat - gtilde) ;  gtilde = gtilde + c           server and workers, lines 9-12
 *   m, v, vhat, theta: the AMSGrad update of the step above with gtilde in the place of gbar
 * starting from ghat_i = ghat = gtilde = 0 (line 1: both compressors map 0 to 0).  Algorithm 1
 * places nu inside the root: that is eps mode 1, which this call does not select by itself.
 * Allocates the server's vectors (2 d floats) and the buffers of its compression (d/8 bytes of sign
 * bits, or a second set of Top-k selection buffers); the rows that held the error memory are
 * cleared and hold ghat_i from then on, so comp_ams_get_error and the e argument of
 * comp_ams_set_state answer COMP_AMS_ESTATE on such a handle.  comp_ams_get_selected then gives the
 * kept coordinates of c_i (values of g_i - ghat_i).
 */
int comp_ams_set_method(comp_ams_t *h, int32_t method);

/* CD handles: ghat_i of worker i in [0,n), the server's aggregate ghat, and gtilde: d floats each. */
int comp_ams_get_ghat_worker(comp_ams_t *h, int32_t worker, float *out, int on_device);
int comp_ams_get_ghat_server(comp_ams_t *h, float *out, int on_device);
int comp_ams_get_gtilde(comp_ams_t *h, float *out, int on_device);

/* CD handles with BLOCKSIGN, after at least one step: the n_blocks scales of the server's message
 * c of the last step (host array); comp_ams_get_scales gives those of the workers' c_i. */
int comp_ams_get_server_scales(comp_ams_t *h, float *out_host);

/* CD handles with TOPK, after at least one step: the k coordinates the server kept in the last step
 * (host arrays, ascending index; values of ghat - gtilde), as comp_ams_get_selected does for a worker. */
int comp_ams_get_server_selected(comp_ams_t *h, uint32_t *idx_host, float *val_host);

/* CD handles, checkpoint resume: ghat_i as [n][d] row-major, ghat and gtilde of d floats; any
 * pointer may be NULL to leave that array as it is (m, v, vhat go through comp_ams_set_state). */
int comp_ams_set_markov_state(comp_ams_t *h, const float *ghat_workers, const float *ghat_server,
                              const float *gtilde, int on_device);

/*
 * One compressed message of the last step in its wire form, written to device memory (what a worker
 * would hand to an all-gather; the paper's accounting of bits, Section 5 and the table of total
 * bits, counts exactly these fields).  who = worker i in [0, n), or n on a CD handle for the
 * server's message.  buf_dev: device memory, 8-byte aligned, `capacity` bytes; *bytes (may be NULL)
 * receives the size of the message, also when the buffer is too small (EINVAL, nothing written).
 *   BLOCKSIGN:     n_blocks fp32 scales, then (d + 31) / 32 words of sign bits in coordinate order
 *                  (bit j % 32 of word j / 32 is set iff coordinate j is negative; zero past d):
 *                  C(x)_j = (bit ? -1 : +1) * scale[block(j)].
 *   TOPK / RANDK:  k pairs {uint32 index, fp32 value} in no particular order.
 * comp_ams_message_bytes gives the size alone (4 d for a handle that does not compress) and needs no
 * GPU.  Waits for the step to finish.
 */
int comp_ams_message_bytes(comp_ams_t *h, uint64_t *bytes);
int comp_ams_pack_message(comp_ams_t *h, int32_t who, void *buf_dev, uint64_t capacity, uint64_t *bytes);

/*
 * comp_ams_pack_message for callers that cannot allocate or wait: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same bytes in buf_dev (the pairs of a TOPK / RANDK
 * message again in no particular order).  It calls no hipMalloc / hipFree or other allocating routine and does
 * not wait: the kernels are enqueued on the stream of the last step and the message is complete when that
 * stream's work is (comp_ams_sync).  The gather of a TOPK / RANDK message works in a fixed array of device memory
 * inside the library (8 MiB + 256 B, present on every GPU the library runs on until the process ends) instead
 * of buffers of the handle; k above 2^20 = 1048576 pairs does not fit and is answered with COMP_AMS_EINVAL
 * (nothing written).  All handles on one GPU share that array: two such calls that overlap in time on one GPU
 * (different streams) race; calls on one stream, or separated by a wait, do not.  A BLOCKSIGN message needs no
 * scratch and is copied straight from the handle's side buffers.
 */
int comp_ams_pack_message_noalloc(comp_ams_t *h, int32_t who, void *buf_dev, uint64_t capacity, uint64_t *bytes);

/*
 * Communication cost of one step in bits, by the accounting of Section 5 (footnote to the
 * algorithm overview) and of the table "Average runtime and total bits": a scaled-sign message costs
 * 1 bit per coordinate plus 32 bits per scale (32 + d for the whole vector), a Top-k message 32 bits
 * of index plus 32 bits of value per kept coordinate, an uncompressed vector 32 d.
 * *uplink_per_worker: what one worker sends.  *downlink: what the server sends back to each worker -
 * a compressed message with CD-Adam, the dense average (32 d) with every other method (error
 * feedback and naive compression compress the workers' messages only).  Either pointer may be NULL.
 * Needs no GPU.
 */
int comp_ams_message_bits(comp_ams_t *h, uint64_t *uplink_per_worker, uint64_t *downlink);

/* Launches an update that the last step left pending and waits until all work enqueued by this handle has
 * completed. */
int comp_ams_sync(comp_ams_t *h);

/* Message of the last failure on this handle (or of the last failed comp_ams_create when
 * h is NULL).  The string stays valid until the next failing call. */
const char *comp_ams_last_error(const comp_ams_t *h);

#ifdef __cplusplus
}
#endif
#endif /* COMP_AMS_H */
