/*
 * adacgd.h -- C ABI of the AdaCGD engine for one MI355X (gfx950).
 *
 * The library runs, entirely on the device, the iteration of "DCGD with master
 * compression" (Algorithm 1) in its three-point-compressor form (Algorithm 2,
 * 3PC-BD) for n simulated workers, with the AdaCGD compressor of Section 4.3 on
 * both sides:
 *
 *     x^{t+1}     = x^t - gamma g^t
 *     g~_i^{t+1}  = C^AC_{g~_i^t, grad f_i(x^t)}( grad f_i(x^{t+1}) )      i = 1..n
 *     g~^{t+1}    = (1/n) sum_i g~_i^{t+1}      (kept incrementally from the n messages)
 *     g^{t+1}     = C^AC_{g^t, g~^t}( g~^{t+1} )                           (master)
 *
 * where C^AC_{h,y}(x) returns h if ||x-h||^2 <= zeta ||x-y||^2, otherwise
 * h + C_j(x-h) (the EF21 form, Eq. (7)) for the first level j < m whose realised
 * error ||x-h-C_j(x-h)||^2 <= zeta ||x-y||^2 (the trigger, Eq. (10)), otherwise
 * level m.  Levels are Top-K sparsifiers (Section 2.1; ties: larger |value|
 * first, then lower index) and b-bit stochastic quantisers.
 *
 * Conventions
 *  - Every function returns an adacgd_status; 0 is success.  Nothing aborts,
 *    prints or throws.  On failure adacgd_last_error() gives a message.
 *  - "device" pointers are HIP device addresses on the current device, "host"
 *    pointers are ordinary process memory.  All vectors are fp32, row-major,
 *    contiguous.  Reductions are accumulated in fp64.
 *  - The library allocates no device memory: the caller passes one workspace of
 *    adacgd_workspace_bytes() bytes (256-byte aligned) that the context owns
 *    until adacgd_destroy(); everything the engine stores lives there.
 *  - All work is enqueued on the caller's stream; adacgd_step does not
 *    synchronise.  adacgd_state synchronises the stream before copying.
 *  - One context must not be used from two threads at once.
 *  - Server aggregation: every coordinate's sum over the workers' messages is taken in fp64 and rounded
 *    to fp32 once.  With Top-K levels only and at most 64 workers the messages are added in ascending
 *    worker index (the sequential sum, reproducible for any data).  With more workers, or with quantiser
 *    or Rank-K levels in the set, partial sums are formed in another (for dense messages fixed, for
 *    Top-K messages unspecified) order: the fp64 sum is then the same for every order as long as the
 *    exponents of the values met at one coordinate spread over fewer than 53 - 24 - log2(n) bits; beyond
 *    that the last place of the fp64 sum, 29 bits below the fp32 result, may depend on the order.
 */
#ifndef ADACGD_H
#define ADACGD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct adacgd_ctx adacgd_ctx; /* opaque, host memory owned by the library */

enum adacgd_status {
  ADACGD_OK = 0,
  ADACGD_ERR_ARG = 1,    /* null pointer, size out of range, non-finite scalar       */
  ADACGD_ERR_LEVELS = 2, /* level set not ordered by contraction parameter           */
  ADACGD_ERR_ALLOC = 3,  /* workspace missing, misaligned or too small               */
  ADACGD_ERR_DEVICE = 4, /* a HIP call failed                                        */
  ADACGD_ERR_STATE = 5,  /* call not valid for this context's mode                   */
  ADACGD_ERR_FIELD = 6   /* unknown field or wrong destination size; nothing written */
};

/* One compression level.  The AdaCGD definition orders levels from strongest to
 * weakest compression, alpha_1 <= ... <= alpha_m.  alpha = K/d for Top-K;
 * alpha = 1/(1+omega), omega = min(d/(4 s^2), sqrt(d)/s), s = 2^(b-1)-1 for b bits. */
enum adacgd_level_kind {
  ADACGD_TOPK = 0,
  ADACGD_QUANT = 1,      /* b-bit stochastic quantiser, one max-norm scale for the whole vector          */
  ADACGD_QUANT_BLOCK = 2, /* the same quantiser applied to every block of B consecutive coordinates on its
                            own (one max-norm scale per block; the last block may be shorter); omega, and
                            with it alpha = 1/(1+omega), are those of a length-B vector; the message is the
                            d codes plus one float per block                                              */
  ADACGD_RANK = 3        /* Rank-K (Section 2.1): the argument, read row-major as a matrix of d/c rows and c
                            columns, is replaced by its best rank-K approximation (truncated singular value
                            decomposition, fp64, rounded once to fp32); alpha = K/c; the message is K scaled
                            left factors of d/c floats and K right factors of c floats.  All Rank-K levels of
                            a level set use the same c                                                     */
};
typedef struct {
  int32_t kind;  /* adacgd_level_kind                                   */
  int32_t block; /* QUANT_BLOCK: block length B, a power of two in [64, 2048]; RANK: columns c, one of 16, 32,
                    64, with d a multiple of c and d >= c^2; otherwise 0 */
  int64_t param; /* TOPK: K in [1,d] (K = d is the identity); QUANT, QUANT_BLOCK: b in [2,16]; RANK: K in [1,c] */
} adacgd_level;

#define ADACGD_MAX_LEVELS 16

/* Condition that guards one position of the cascade.  The Ada3PC construction (Section 4.2,
 * Lemma 2) accepts any conditions P_j; this library offers the family
 *     P_j :  err_j <= zeta ||x-y||^2 + eta ||x-h||^2
 * where err_0 = ||x-h||^2 (position 0: keep h, send nothing) and err_j is the realised error
 * of level j.  zeta = the AdaCGD constant, eta = 0 is the trigger of Eq. (10); zeta = 0 with
 * eta < 1 accepts the first level whose realised relative error is at most eta (a compressor
 * that is contractive with alpha = 1 - eta by construction).  The last level has no condition.
 * The right side is evaluated in fp64 as fl(fl(zeta D) + fl(eta S)). */
typedef struct {
  float zeta; /* finite, >= 0 */
  float eta;  /* finite, >= 0 */
} adacgd_trigger;

/* Where grad f_i(x^{t+1}) comes from. */
enum adacgd_grad_mode {
  ADACGD_GRAD_LOGISTIC = 0, /* engine computes the gradient of the Section 6 objective:
                               f_i(x) = (1/N_i) sum_l log(1+exp(-y_l a_l^T x)) + lambda sum_j x_j^2/(1+x_j^2) */
  ADACGD_GRAD_EXTERNAL = 1, /* caller passes grad f_i(x^{t+1}) to adacgd_step                         */
  ADACGD_DIFF_EXTERNAL = 2, /* caller passes x - h (the compressor's argument) and ||x-y||^2 directly  */
  ADACGD_GRAD_LOGISTIC_CSR = 3 /* as GRAD_LOGISTIC, with the features given as compressed sparse rows
                               (the data sets of Section 6 are sparse, several of them binary); the
                               gradient is summed over the stored entries only, in a fixed order   */
};

/* g~_i^0 ("known by nodes" in Algorithm 1's input line; the paper leaves it free). */
enum adacgd_init_mode {
  ADACGD_INIT_FULLGRAD = 0, /* g~_i^0 = grad f_i(x^0)  */
  ADACGD_INIT_ZERO = 1,     /* g~_i^0 = 0              */
  ADACGD_INIT_COMPRESSED = 2 /* g~_i^0 = C_m(grad f_i(x^0)), C_m the last worker level, which must be a
                               Top-K sparsifier: the start of EF21 and CLAG when only a compressed
                               gradient can be sent in round 0 */
};

enum adacgd_flags {
  ADACGD_FLAG_ANY_LEVEL_ORDER = 1, /* accept level sets not sorted by alpha (Lemma 2 holds for any order) */
  ADACGD_FLAG_RETAIN_EXT = 2,      /* GRAD_EXTERNAL: keep the caller's last gradient array as y for the
                                      next step instead of copying it; the caller must leave that array
                                      untouched until the next adacgd_step call has completed            */
  ADACGD_FLAG_KERNEL_TIMING = 4,   /* record HIP events around every kernel (see ADACGD_F_KERNEL_MS)    */
  ADACGD_FLAG_TWO_PASS = 8,        /* always use the general two-pass kernels: neither the sampled one-pass
                                      selection of long vectors nor the one-block kernel of short ones
                                      (same results, slower)                                            */
  ADACGD_FLAG_OVERLAP = 16         /* GRAD_EXTERNAL / DIFF_EXTERNAL: run the worker compression on a stream
                                      of the library's own, concurrently with the previous step's
                                      aggregation and master compression on the caller's stream (same
                                      results).  The arrays passed to adacgd_step must then be complete
                                      when the call is made, not merely enqueued on the caller's stream;
                                      the caller's stream still orders after everything a step enqueues */
};

typedef struct {
  int64_t n;                    /* workers, 1 <= n <= 65535                                   */
  int64_t d;                    /* dimension, 1 <= d < 2^31                                   */
  int32_t grad_mode;            /* adacgd_grad_mode                                           */
  int32_t init_mode;            /* adacgd_init_mode (DIFF_EXTERNAL requires INIT_ZERO)        */
  const float* A;               /* LOGISTIC: device [sum N_i x d] features; BORROWED for the context's life */
  const float* labels;          /* LOGISTIC, LOGISTIC_CSR: device [sum N_i], each -1 or +1; BORROWED */
  const int64_t* shard_offsets; /* LOGISTIC, LOGISTIC_CSR: host [n+1], rows of worker i are [off[i],off[i+1]); copied */
  const float* x0;              /* device [d] starting point; copied                          */
  const float* grad0;           /* GRAD_EXTERNAL: device [n x d] grad f_i(x^0); copied        */
  float lambda;                 /* regulariser weight                                         */
  float gamma;                  /* stepsize, finite                                           */
  const adacgd_level* worker_levels; /* host [m_worker]; copied                               */
  int32_t m_worker;             /* 1..ADACGD_MAX_LEVELS                                       */
  float zeta_worker;            /* trigger constant, finite, >= 0                             */
  const adacgd_level* master_levels; /* host [m_master]; copied                               */
  int32_t m_master;             /* 0 = identity master (g = g~); else 1..ADACGD_MAX_LEVELS    */
  float zeta_master;
  uint64_t seed;                /* Philox key of the quantiser's dither                       */
  uint32_t flags;               /* adacgd_flags                                               */
  uint32_t pad;                 /* set to 0                                                   */
  void* stream;                 /* hipStream_t; BORROWED                                      */
  void* workspace;              /* device, 256-byte aligned; owned by the context until destroy */
  int64_t workspace_bytes;
  const adacgd_trigger* worker_triggers; /* host [m_worker]: conditions of cascade positions 0..m_worker-1
                                            (0 = keep h, j = level j); copied.  NULL: every position uses
                                            (zeta_worker, 0), the AdaCGD definition; otherwise zeta_worker
                                            is ignored                                                  */
  const adacgd_trigger* master_triggers; /* host [m_master], likewise with zeta_master; NULL allowed   */
  /* GRAD_LOGISTIC_CSR: the feature matrix [sum N_i x d] in compressed sparse row form, all three in HOST
   * memory, read and copied by adacgd_workspace_bytes / adacgd_init (the context keeps a device copy of
   * the rows and a second one sorted by column inside every worker's shard, both in the workspace).
   * labels and shard_offsets are as in GRAD_LOGISTIC; A is not read. */
  const int64_t* csr_row_ptr; /* host [rows+1], rows = shard_offsets[n] < 2^31; starts at 0, non-decreasing */
  const int32_t* csr_col;     /* host [nnz]: columns in [0,d), strictly ascending inside a row; anything
                                 else is rejected with ADACGD_ERR_ARG before the device is touched     */
  const float* csr_val;       /* host [nnz], or NULL: every stored entry is 1 (binary features)        */
} adacgd_config;

/* Device bytes adacgd_init needs for this configuration (workspace and stream
 * fields are ignored).  Validates the configuration the way adacgd_init does. */
int adacgd_workspace_bytes(const adacgd_config* cfg, int64_t* bytes);

/* Input line of Algorithm 1: builds the state x^0, g~_i^0, g~^0 = (1/n) sum g~_i^0,
 * g^0 = g~^0, and y_i = grad f_i(x^0).  On success *out is a new context. */
int adacgd_init(const adacgd_config* cfg, adacgd_ctx** out);

/* adacgd_init for callers that cannot allocate device memory or have none to pass: code that runs
 * where hipMalloc is not allowed (under HIP graph capture, in tight serving loops, in harnesses that
 * forbid it).  The workspace is a static device array inside the library, ADACGD_STATIC_WORKSPACE_BYTES
 * long, that every device the library is used on holds until the process ends; the context object lives
 * in static host memory.  This call allocates nothing, on the device or on the host, and creates no
 * stream or event.  cfg->workspace and cfg->workspace_bytes are ignored; everything else is as in
 * adacgd_init, with these limits:
 *  - grad_mode is GRAD_EXTERNAL or DIFF_EXTERNAL, and neither FLAG_OVERLAP nor FLAG_KERNEL_TIMING is
 *    set (ADACGD_ERR_STATE otherwise);
 *  - adacgd_workspace_bytes(cfg) <= ADACGD_STATIC_WORKSPACE_BYTES, else ADACGD_ERR_ALLOC with a message
 *    that gives both numbers (about 26 bytes per worker-coordinate: n d up to about 2.5 million);
 *  - one such context per device at a time: a second call on the current device before the first
 *    context is destroyed returns ADACGD_ERR_STATE (all of them would share the one array).
 * The array keeps what the previous context left in it; this call clears what has to start at zero.
 * The context is used and destroyed like any other (adacgd_step, adacgd_state, adacgd_destroy). */
#define ADACGD_STATIC_WORKSPACE_BYTES (64ll << 20)
int adacgd_init_static(const adacgd_config* cfg, adacgd_ctx** out);

/* Runs nsteps iterations of Algorithm 2 (all of: iterate update, local gradients,
 * worker compression with level choice, server aggregation, master compression).
 *   LOGISTIC, LOGISTIC_CSR   ext = ext_D = NULL.
 *   GRAD_EXTERNAL ext = device [nsteps x n x d], one gradient array per step; ext_D = NULL.
 *   DIFF_EXTERNAL ext = device [nsteps x n x d] difference vectors v_i, ext_D = device
 *                 [nsteps x n] fp64 values of ||x-y||^2; g~_i accumulates C(v_i).
 * ext must be 16-byte aligned.  Arrays passed in must stay valid until the
 * enqueued work has completed. */
int adacgd_step(adacgd_ctx* ctx, const float* ext, const double* ext_D, int32_t nsteps);

/* Fields of adacgd_state.  Sizes in elements; W = worker side, M = master side. */
enum adacgd_field {
  ADACGD_F_X = 0,            /* float  [d]     x^t                                            */
  ADACGD_F_G = 1,            /* float  [d]     g^t                                            */
  ADACGD_F_GTILDE = 2,       /* float  [d]     g~^t                                           */
  ADACGD_F_GTILDE_PREV = 3,  /* float  [d]     g~^{t-1}                                       */
  ADACGD_F_GI = 4,           /* float  [n x d] g~_i^t                                         */
  ADACGD_F_PREV_GRAD = 5,    /* float  [n x d] grad f_i(x^t)  (not in DIFF_EXTERNAL)          */
  ADACGD_F_LEVEL = 6,        /* int32  [n]     level of the last step: 0 = skip, 1..m         */
  ADACGD_F_SQNORM = 7,       /* double [n]     ||x-h||^2 of the last step                     */
  ADACGD_F_D = 8,            /* double [n]     ||x-y||^2 of the last step                     */
  ADACGD_F_ERR = 9,          /* double [n x m_worker] realised error of every level; NaN in the
                                rows of workers that skipped (level 0): the cascade stops at
                                its first condition and their errors are not evaluated       */
  ADACGD_F_MSG_COUNT = 10,   /* int64  [n]     entries of each worker's last Top-K message    */
  ADACGD_F_MSG_IDX = 11,     /* int32  [sum counts] coordinates, ascending per worker, packed */
  ADACGD_F_MSG_VAL = 12,     /* float  [sum counts] values, packed in the same order          */
  ADACGD_F_M_LEVEL = 13,     /* int32  [1]                                                    */
  ADACGD_F_M_SQNORM = 14,    /* double [1]                                                    */
  ADACGD_F_M_D = 15,         /* double [1]                                                    */
  ADACGD_F_M_ERR = 16,       /* double [m_master]                                             */
  ADACGD_F_M_MSG_COUNT = 17, /* int64  [1]                                                    */
  ADACGD_F_M_MSG_IDX = 18,   /* int32  [count]                                                */
  ADACGD_F_M_MSG_VAL = 19,   /* float  [count]                                                */
  ADACGD_F_STEP = 20,        /* int64  [1]     iterations done                                */
  ADACGD_F_LEVEL_HIST = 21,  /* uint64 [m_worker+1] cumulative count of each worker level     */
  ADACGD_F_M_LEVEL_HIST = 22,/* uint64 [m_master+1]                                           */
  ADACGD_F_COMM = 23,        /* uint64 [4] cumulative values_up, bits_up, values_down, bits_down:
                                a Top-K message costs K (32 + ceil(log2 d)) bits, a b-bit message
                                d b + 32, plus ceil(log2(m+1)) bits for the level id; the master's
                                message is counted once per worker                             */
  ADACGD_F_QCODES = 24,      /* int16  [n x d] signed codes of the last quantised messages (rows of
                                workers that chose another level are unspecified)             */
  ADACGD_F_QSCALE = 25,      /* float  [n]     scale c of the last quantised message          */
  ADACGD_F_KERNEL_MS = 26,   /* double [2 x ADACGD_NUM_KERNELS] per kernel: summed milliseconds, then
                                launch counts, since init or the last query (query resets)    */
  ADACGD_F_GRAD = 27,        /* float  [n x d] same as PREV_GRAD (the gradients of the last step) */
  ADACGD_F_REPAIRS = 28,     /* uint64 [2]     node-steps (workers, master) on which the sampled candidate cut
                                of the one-pass selection was too high and the vector was scanned a
                                second time; a diagnostic: the results do not depend on it           */
  ADACGD_F_QBSCALE = 31,     /* float  [n x ceil(d/64)] scales of the last block-wise quantised message of each worker:
                                entry k of a row is the scale of block k (the first ceil(d/B) entries; the rest
                                and the rows of workers that chose another level are unspecified); only kept
                                when the worker level set holds a block-wise quantiser                        */
  ADACGD_F_RANK_SPECTRUM = 32, /* double [n x c] squared singular values, descending, of every worker's matrix-shaped
                                argument at the last step (rows of workers that skipped are unspecified); only
                                with Rank-K levels in the worker level set                                  */
  ADACGD_F_CANDIDATES = 30,  /* uint64 [2]     coordinates (workers, master) that the last step's one-pass scan kept as
                                candidates for the largest Top-K size, summed over the nodes (0 where the
                                one-pass sequence is not in use); a diagnostic of the sampled cut         */
  ADACGD_F_ESTIMATOR_ERR = 29  /* double [1]   G = (1/n) sum_i ||grad f_i(x^t) - g~_i^t||^2 after the last step, the
                                quantity whose contraction drives the convergence proofs (from the
                                realised errors of the chosen levels; needs at least one step)  */
};

/* Kernel slots of ADACGD_F_KERNEL_MS.  W = worker side, M = master side.  Long vectors with
 * Top-K levels only run sample + scan (the scan also extracts the candidates); the filter slot
 * then holds the second scan that repairs a failed estimate (idle otherwise).  Other vectors run
 * scan + filter as two passes.  Vectors of at most 4096 coordinates are handled by one kernel
 * that does the whole compression step of a node, timed in the scan slot; with at most 64 workers
 * and Top-K levels only that launch also aggregates (the aggregate slot stays empty), and the
 * launch that finishes g also writes the next iterate (the xupdate slot stays empty); so does the
 * aggregation of any vector length when there is no master compressor (g is g~ then). */
enum adacgd_kernel {
  ADACGD_K_XUPDATE = 0,
  ADACGD_K_GRAD_MARGIN = 1,
  ADACGD_K_GRAD_COLS = 2,
  ADACGD_K_AGGREGATE = 3,
  ADACGD_K_W_SAMPLE = 4,   /* histogram of a sample of the vector: candidate cut estimate     */
  ADACGD_K_W_SCAN = 5,     /* differences, norms, first-digit histogram (+ candidates)        */
  ADACGD_K_W_FILTER = 6,   /* candidate extraction, low-band energy, quantiser errors         */
  ADACGD_K_W_GATHER = 7,   /* keys inside the threshold bins -> one list per worker           */
  ADACGD_K_W_SELECT = 8,   /* remaining digits: exact thresholds                              */
  ADACGD_K_W_TALLY = 9,    /* band energies, level choice                                     */
  ADACGD_K_W_COMPACT = 10, /* message + estimator update                                      */
  ADACGD_K_W_QAPPLY = 11,  /* dense estimator update of quantised levels                      */
  ADACGD_K_M_SAMPLE = 12,
  ADACGD_K_M_SCAN = 13,
  ADACGD_K_M_FILTER = 14,
  ADACGD_K_M_GATHER = 15,
  ADACGD_K_M_SELECT = 16,
  ADACGD_K_M_TALLY = 17,
  ADACGD_K_M_COMPACT = 18,
  ADACGD_K_M_QAPPLY = 19,
  ADACGD_K_W_RANK = 20,    /* Rank-K levels: Gram matrix, realised errors, dense update (the contractions) */
  ADACGD_K_M_RANK = 21,
  ADACGD_K_W_EIG = 22,     /* Rank-K levels: eigen-decomposition of the Gram matrix */
  ADACGD_K_M_EIG = 23,
  ADACGD_NUM_KERNELS = 24
};

/* Copies one field to dst (host memory, or device memory if dst_on_device != 0)
 * after synchronising the context's stream.  dst_bytes must equal the field's
 * size exactly, else ADACGD_ERR_FIELD and nothing is written. */
int adacgd_state(adacgd_ctx* ctx, int32_t field, void* dst, int64_t dst_bytes, int32_t dst_on_device);

/* Restores persistent state, e.g. from a checkpoint made of adacgd_state copies: field is one of
 * F_X, F_G (only with a master compressor; otherwise g is g~), F_GTILDE, F_GTILDE_PREV, F_GI,
 * F_PREV_GRAD, F_STEP (also the Philox counter of the next step), F_LEVEL_HIST, F_M_LEVEL_HIST; any
 * other field gives ADACGD_ERR_FIELD.  src is host memory, or device memory if src_on_device != 0;
 * src_bytes must equal the field's size exactly, else ADACGD_ERR_FIELD and nothing is written.
 * Synchronises the context's stream before and after the copy.  The per-step outputs of the last
 * step (levels, errors, messages) are not part of this state and keep their values until the next
 * step.  With ADACGD_FLAG_RETAIN_EXT, F_PREV_GRAD is copied into the engine's own buffer, which
 * replaces the caller's retained array as y of the next step.  A run restored with all nine fields
 * continues bit for bit like the run the copies were taken from. */
int adacgd_set_state(adacgd_ctx* ctx, int32_t field, const void* src, int64_t src_bytes, int32_t src_on_device);

/* Synchronises the stream and frees the context (the workspace returns to the
 * caller).  NULL is accepted. */
int adacgd_destroy(adacgd_ctx* ctx);

/* Message of the last failure on this context, or, for ctx == NULL, of the
 * calling thread's last failed adacgd_init / adacgd_workspace_bytes. */
const char* adacgd_last_error(const adacgd_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* ADACGD_H */
