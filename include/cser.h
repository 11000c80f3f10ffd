/*
 * cser.h -- C ABI of the MI355X-native CSER optimizer update (arxiv 2007.13221).
 *
 * One call of cser_step() is one iteration t of the paper's Algorithm 3 (M-CSER, Section 3.2;
 * Algorithm 2 when momentum = 0) for all n = W workers at once, from the point where the
 * stochastic gradients g_{i,t} are known:
 *
 *     m_i <- beta m_i + g_i ;  p_i <- eta (beta m_i + g_i)              (Get_p, Appendix A.4)
 *     p'_i, r_i <- PSync(p_i, C_step)                                    (Algorithm PSync, Section 3.1)
 *     x_i <- x_i - p'_i ;  e_i <- e_i - r_i
 *     if t mod H = 0:  e'_i, e_i <- PSync(e_i, C_reset) ;  x_i <- x_i - e_i(old) + e'_i     (error reset)
 *
 * C_step and C_reset are globally-randomized blockwise sparsifiers (GRBS, Definition 2,
 * Section 3.3): the flat d-vector is cut into B = ceil(d / block) blocks and every worker keeps
 * the same k = ceil(B / R) randomly drawn blocks, a pure function of (seed, t).  C_step is the
 * compressor the paper calls C_2 (ratio R_C2, used every iteration), C_reset the one it calls
 * C_1 (ratio R_C1, used every H iterations); the names used here say what they do because the
 * paper's numbering is easy to swap.
 *
 * All W worker states live on ONE GPU as row-major fp32 matrices [W][ld]; the worker average
 * inside PSync is a reduction over the rows, not a collective.
 *
 * Conventions for every entry point
 *   - returns CSER_OK (0) or a negative cser_status; nothing is thrown, nothing aborts;
 *   - "device" pointers are HIP device addresses, "host" pointers ordinary memory;
 *   - kernels are enqueued on the hipStream_t passed as `void* hip_stream` (NULL = the null
 *     stream) and the call returns without waiting for them;
 *   - a context is bound to the device that was current at cser_create() and must be used with
 *     that device current (cser_step and cser_error_reset return CSER_EINVAL otherwise); calls on one context
 *     must not overlap each other.
 */
#ifndef CSER_H
#define CSER_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif
#if defined(__GNUC__)
#pragma GCC visibility push(default) /* the library is built with hidden visibility: only these entry points are exported */
#endif

typedef enum cser_status {
  CSER_OK = 0,
  CSER_EINVAL = -1,  /* null pointer, zero size, ld < d, R_reset = 0, beta outside [0,1), non-finite eta ... */
  CSER_EALIGN = -2,  /* a device pointer is not 4-byte aligned                                            */
  CSER_ENOMEM = -3,  /* host or device allocation failed                                                  */
  CSER_EHIP = -4,    /* a HIP runtime call failed; cser_last_hip_error() names it                          */
  CSER_ERANGE = -5   /* a size is beyond what the kernels index (B >= 2^32, d/4 >= 2^32, W * ceil(d/256) >= 2^31) */
} cser_status;

typedef struct cser_ctx cser_ctx; /* opaque, host-side */

typedef struct cser_config {
  uint64_t d;        /* parameters per worker, >= 1                                                       */
  uint64_t ld;       /* row stride of x, e, m, g in elements, >= d; a multiple of 1024 (4 KiB rows) is fastest */
  uint32_t W;        /* number of workers n, >= 1 (Section 3)                                             */
  uint32_t block;    /* elements per GRBS block, >= 1; B = ceil(d / block) (Definition 2)                 */
  uint32_t R_step;   /* ratio of the per-iteration compressor (paper: R_C2): keeps ceil(B / R_step)
                        blocks; 1 = identity; 0 = the delta = 0 compressor C(v) = 0 (Section 3)          */
  uint32_t R_reset;  /* ratio of the error-reset compressor (paper: R_C1), >= 1; 1 = full reset           */
  uint32_t H;        /* error-reset interval (Algorithm 3 input); 0 = cser_step never resets              */
  float lr;          /* eta                                                                               */
  float momentum;    /* beta in [0, 1); 0 gives Algorithm 2                                               */
  uint64_t seed;     /* the synchronized random seed of Section 3.3                                       */
} cser_config;

/*
 * Create a context (Algorithm 3, "Initialize").
 *   x  device [W][ld] fp32, in/out: the caller has written the same x_hat_0 into every row.
 *   e  device [W][ld] fp32 or NULL.  Non-NULL: implementation I; cser_create zero-fills it.
 *      NULL: implementation II of Appendix A.4 (no residual buffer; the reset averages x itself).
 *   m  device [W][ld] fp32 or NULL.  Non-NULL: zero-filled here.  NULL is allowed only with
 *      momentum = 0 (Algorithm 2 keeps no momentum) and removes the m traffic.
 * The buffers stay owned by the caller, must outlive the context and are never freed here.  The
 * context owns a few small device arrays (block masks and index lists), all allocated here: no later
 * call allocates device memory.  hip_stream is the stream the zero fills of e and m are enqueued on
 * (an addition to the four-call interface the method's statement suggests: the fills are device work
 * and must be ordered with the caller's own initialisation of x).  128-bit accesses are used whenever block is a multiple of 4 columns, whatever
 * ld and the base addresses are (rows that start on 16-byte boundaries, i.e. ld % 4 == 0 and aligned
 * bases, are faster, and ld a multiple of 1024 is fastest); other block sizes run element-wise kernels with the same
 * results.  On failure *out is NULL.
 */
int cser_create(const cser_config* cfg, float* x, float* e, float* m, void* hip_stream, cser_ctx** out);

/*
 * One iteration: t <- t + 1; block selection for (seed, stream 0, t); the fused local step,
 * partial synchronisation and residual bookkeeping (the four statements of Algorithm 3 before
 * its "if"); then, when H > 0 and t mod H = 0, the error reset (same result as cser_error_reset();
 * by default it is carried out inside the same kernel pass).
 *   g  device [W][ld] fp32, read-only: this iteration's stochastic gradients, one row per worker.
 * Arithmetic: beta*m+g and beta*m_new+g are single fused multiply-adds, the worker mean is the
 * left-to-right sum over i = 0..W-1 divided by W, everything in fp32.
 */
int cser_step(cser_ctx* ctx, const float* g, void* hip_stream);

/*
 * The error-reset branch of Algorithm 3 at the current t: block selection for (seed, stream 1,
 * t), then on the selected blocks  ebar = mean_i e_i ;  x_i <- (x_i - e_i) + ebar ;  e_i <- +0.
 * (Implementation II: x_i <- mean_i x_i on the selected blocks.)  Exposed so that a caller can
 * force a reset at any t.
 */
int cser_error_reset(cser_ctx* ctx, void* hip_stream);

/* Free the context and its device arrays (not x, e, m).  cser_destroy(NULL) returns CSER_OK. */
int cser_destroy(cser_ctx* ctx);

/*
 * Run the block selector (Definition 2; shared seed, Section 3.3) for iteration t and copy the
 * result to host memory.  Synchronous, on a stream of the context's own (the caller's streams are not
 * waited for); the context's state is not changed.  which: 0 = C_step's stream, 1 = C_reset's stream.
 *   idx_host   host, >= k entries or NULL: the chosen block ids in draw order pi(0..k-1)
 *   mask_host  host, B bytes or NULL: 1 where the block is chosen
 *   k_out      host or NULL: receives k
 */
int cser_select_blocks(const cser_ctx* ctx, int which, uint64_t t, uint32_t* idx_host, uint8_t* mask_host,
                       uint32_t* k_out);

/* Sizes derived from the configuration: B, k_step = ceil(B/R_step), k_reset = ceil(B/R_reset). */
int cser_block_counts(const cser_ctx* ctx, uint64_t* B, uint32_t* k_step, uint32_t* k_reset);

/*
 * The special cases of Appendix A.1 as settings of a configuration (host only, no device work):
 *   cser_preset_csea     C_step(v) = 0 and H = 1: SGD with error assimilation (CSEA); R_reset is its one compressor
 *   cser_preset_cser_pl  C_step(v) = 0: partial-local SGD (CSER-PL); with R_reset = 1 it is local SGD with period H
 * Both only overwrite R_step (and H); every other field is left as the caller set it.
 */
int cser_preset_csea(cser_config* cfg);
int cser_preset_cser_pl(cser_config* cfg);

/*
 * Overall compression ratio of a configuration, Section 5.1:  R = 1 / (1/R_step + 1/(R_reset * H)),
 * with 1/R_step = 0 for R_step = 0 and the second term 0 for H = 0.  *ratio = +inf if nothing is ever sent.
 */
int cser_overall_ratio(const cser_config* cfg, double* ratio);

/* Learning-rate schedules (Section 5.1): takes effect from the next cser_step. */
int cser_set_lr(cser_ctx* ctx, float lr);

/* The iteration counter t (0 after create; the state of a run is x, e, m, t and the seed). */
int cser_get_step(const cser_ctx* ctx, uint64_t* t);
int cser_set_step(cser_ctx* ctx, uint64_t t);

/*
 * n iterations in one call: the same as calling cser_step(ctx, g_list[0], hip_stream), ...,
 * cser_step(ctx, g_list[n-1], hip_stream) one after the other (Algorithm 3's loop over t with the
 * gradients already known, e.g. a recorded run that is replayed).  Meant for small d, where the
 * time of an iteration is the host's cost of making the call rather than the kernel's.
 *   g_list  host array of n device pointers, each [W][ld] fp32, read-only.
 * Stops at the first failing iteration and returns its status; *done (host, may be NULL) receives
 * the number of iterations enqueued.
 */
int cser_step_many(cser_ctx* ctx, const float* const* g_list, uint32_t n, void* hip_stream, uint32_t* done);

/*
 * cser_step() for callers that cannot allocate: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  No context: the call carries out iteration t of the configuration
 * *cfg on the caller's buffers (same meaning, layout and arithmetic as cser_create + cser_step; e and m
 * may be NULL as there; nothing is zero-filled, the caller keeps t) and allocates nothing, on the host
 * or on the device.  The block masks of C_step (and, when H > 0 and t mod H = 0, of C_reset) are drawn
 * into a fixed device array of 2 * CSER_STATIC_MAX_BLOCKS bytes that the library holds on every GPU it
 * has run on until the process ends; a configuration with more than CSER_STATIC_MAX_BLOCKS blocks
 * returns CSER_ERANGE.  All calls on one GPU share that array: calls that overlap on one GPU (different
 * streams, different threads) race; calls on one stream are ordered.  The first call on a device looks up
 * the array's address and the launch shapes for that device.
 */
#define CSER_STATIC_MAX_BLOCKS 524288u
int cser_step_static(const cser_config* cfg, uint64_t t, float* x, float* e, float* m, const float* g,
                     void* hip_stream);

const char* cser_strerror(int status);
const char* cser_last_hip_error(void); /* text of the last HIP error seen by this thread, "" if none */

#if defined(__GNUC__)
#pragma GCC visibility pop
#endif
#ifdef __cplusplus
}
#endif
#endif /* CSER_H */
