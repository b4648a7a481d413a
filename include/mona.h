/*
 * libmona -- the MONA optimizer step (Muon with an acceleration term built from
 * an EMA of gradient differences) for lists of weight matrices on one AMD
 * MI355X (gfx950) GPU.
 *
 * What one step computes, per matrix W (m x n), in the order of the paper's
 * Algorithm 1:
 *
 *     D_k   = G_k - G_{k-1}                          Alg. 1, difference line (Eq. alto_diff)
 *     A_k   = beta_a A_{k-1} + (1 - beta_a) D_k      Eq. alto_accel
 *     Gt_k  = G_k + alpha A_k                        Eq. alto_grad
 *     M_k   = mu M_{k-1} + Gt_k                      Eq. muon_momentum, fed with Gt_k
 *     X_0   = M_k / (||M_k||_F + eps)                Sec. 3.2, start of the Newton-Schulz iteration
 *     X_t+1 = a X_t + b (X_t X_t^T) X_t + c (X_t X_t^T)^2 X_t,   t = 0..T-1     Eq. newton_schulz
 *     O_k   = X_T
 *     W_k+1 = W_k - eta (gamma O_k + lambda W_k),  gamma = gamma_coeff sqrt(max(m, n))    Eq. muon_update
 *     G_{k-1} <- G_k                                 Alg. 1, last line of the loop
 *
 * with M_0 = A_0 = G_0 = 0 (Alg. 1, initialisation line).
 *
 * Conventions
 *   - plain C ABI; every pointer argument says whether it is HOST or DEVICE memory;
 *   - every function returns MONA_OK (0) or a negative mona_status and never throws;
 *     mona_last_error() gives a thread-local description of the last failure (a successful
 *     mona_step may leave a warning there: see mona_step);
 *   - nothing here synchronises the stream unless stated; work is enqueued on the
 *     stream the caller passes (a hipStream_t cast to void*, NULL = the null stream);
 *   - the library allocates no device memory for state or workspace: the caller hands
 *     it one arena (e.g. a torch uint8 tensor) sized by mona_state_size(); the library
 *     owns only host-side bookkeeping and a few small pinned host tables.
 */
#ifndef MONA_H
#define MONA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum mona_status {
  MONA_OK = 0,
  MONA_EINVAL = -1,       /* null pointer, size < 1, hyper-parameter out of range, misaligned pointer */
  MONA_ESHAPE = -2,       /* matrix list differs from the one given to mona_init_state            */
  MONA_ENOMEM = -3,       /* arena too small / host allocation failed                              */
  MONA_EHIP = -4,         /* a HIP runtime call failed (text in mona_last_error)                   */
  MONA_EUNSUPPORTED = -5  /* valid request this build does not implement                           */
} mona_status;

typedef enum mona_dtype { MONA_F32 = 0, MONA_BF16 = 1 } mona_dtype;

/* One weight matrix.  The caller owns w and g (DEVICE memory, row-major, contiguous,
 * m rows of n elements, 16-byte aligned).  w is updated in place (round-to-nearest-even
 * when bf16); g is only read. */
typedef struct mona_matrix {
  void* w;            /* DEVICE: W_k in, W_{k+1} out                    */
  const void* g;      /* DEVICE: G_k                                    */
  int32_t m, n;       /* 1 <= m, n <= 2^30; m * n < 2^31                */
  int32_t w_dtype;    /* mona_dtype                                     */
  int32_t g_dtype;    /* mona_dtype                                     */
} mona_matrix;

/* Alg. 1, REQUIRE line.  Passed per step because schedules change eta. */
typedef struct mona_hparams {
  float lr;            /* eta                                                            */
  float momentum;      /* mu in [0, 1)                                                   */
  float beta_a;        /* acceleration EMA coefficient in [0, 1)                         */
  float alpha;         /* acceleration coefficient; 0 gives plain Muon (Sec. 3.2)        */
  float weight_decay;  /* lambda, decoupled, acts on W_k, scaled by eta                  */
  int32_t ns_steps;    /* T >= 0 (5 in the paper); 0 gives O = X_0                       */
  float ns_a, ns_b, ns_c; /* 3.4445, -4.7750, 2.0315 (text under Eq. newton_schulz)      */
  float ns_eps;        /* X_0 = M / (||M||_F + ns_eps); the paper uses 0                 */
  float gamma_coeff;   /* 0.2 in gamma = 0.2 sqrt(max(m, n))                             */
  uint32_t flags;      /* MONA_FLAG_* bits                                               */
} mona_hparams;

/* At the first step after mona_init_state take D_1 = 0 instead of D_1 = G_1 - 0, i.e.
 * behave as if the previous-gradient buffer already held G_1.  Off by default
 * (Alg. 1 initialises G_0 = 0). */
#define MONA_FLAG_FIRST_DIFF_ZERO 0x1u
/* Keep O_k = X_T readable through mona_state_view(MONA_VIEW_O) after the step (costs one
 * extra store of the matrix in the update kernel). */
#define MONA_FLAG_KEEP_O 0x2u
/* Plain Muon step (Sec. 3.2, Eqs. muon_momentum / muon_ns / muon_update): M_k = mu M_{k-1} + G_k;
 * alpha and beta_a are ignored and the buffers G_{k-1} and A are neither read nor written.  This is
 * the baseline the paper's overhead figure (App. C) compares MONA with. */
#define MONA_FLAG_MUON_ONLY 0x4u

/* Fixed when the state is built. */
typedef struct mona_options {
  int32_t ns_precision; /* 0: bf16 operands, fp32 accumulation (MFMA bf16);
                           1: fp32 operands and accumulation (MFMA fp32)                     */
  int32_t state_dtype;  /* mona_dtype of the stored G_{k-1} and A_k: MONA_F32 (Sec. 6.3,
                           "full precision") or MONA_BF16 (the MONA-Lite variant, Sec. 6.3);
                           M_k is always fp32                                                */
  int32_t accel_form;   /* how the acceleration term (Eqs. alto_diff / alto_accel) is carried:
                           MONA_ACCEL_TWO_BUFFER (0): G_{k-1} and A_k are stored, as Alg. 1 writes it;
                           MONA_ACCEL_ONE_BUFFER (1): only C_{k+1} = beta_a A_k - (1 - beta_a) G_k is
                           stored and A_k = C_k + (1 - beta_a) G_k (the same A_k in exact arithmetic).
                           No previous-gradient buffer exists -- the aim of the streaming variant of
                           Sec. 6.3, reached without borrowing the caller's gradient slot -- and the
                           elementwise pass moves 22 instead of 30 bytes per element.  beta_a must
                           then stay the same from step to step (MONA_EINVAL otherwise)            */
  int32_t max_streams;  /* matrices of different shapes are orthogonalised independently; their launch
                           chains run on up to this many streams (the caller's plus side streams the
                           state owns, forked after the elementwise pass and joined before mona_step
                           returns, all at default priority).  0 = default (4), 1 = caller's stream only */
  int32_t ns_schedule;  /* how the T iterations of Eq. newton_schulz are laid out as matrix products (the
                           polynomial of X_0 they compute is the same; rounding differs):
                           MONA_NS_SCHEDULE_LITERAL (1): per iteration S = X X^T, B = b S + c S S, X <- a X + B X;
                           MONA_NS_SCHEDULE_FUSED (2): iterations in chunks of three, then two.  With
                             Q_t = a I + b S_t + c S_t^2 an iteration is X_{t+1} = Q_t X_t and S_{t+1} = S_t Q_t^2,
                             so a chunk forms S once, advances it on the p x p side and applies the product of its
                             Q_t to X once: fewer flop whenever the long side exceeds the short one;
                           MONA_NS_SCHEDULE_PAIRS (3): the same in chunks of two;
                           MONA_NS_SCHEDULE_AUTO (0): per shape group, for bf16 groups whose long side q is at
                             least 1.5 times the short side p: chunks of three then two where
                             1 / sqrt(p) + 1 / sqrt(q) <= 0.0438 (e.g. 1536 x 4096, 2048 x 8192: there the fused
                             form measured as accurate as the literal one or better), chunks of two where the
                             padded short side is at least 1024 (e.g. 1024 x 2048), literal otherwise    */
  int32_t overlap;      /* MONA_OVERLAP_OFF (0): one elementwise pass over every matrix, then the products.
                           MONA_OVERLAP_LATE_GROUP (1): when several large shape groups run one after the
                           other, the elementwise pass (HBM-bound) of the one with the most elements runs on a
                           stream confined to a quarter of the CUs, beside the matrix products (bound by the
                           matrix units) of the other groups, which keep to the remaining CUs; its own products
                           come last.  Results are bit-identical either way.  Takes effect only when the step
                           is enqueued on a stream other than the null stream (HIP creates CU-masked streams
                           as blocking ones, with which the null stream synchronises), not under stream
                           capture, and only where the other groups' products last about as long as the
                           slowed-down pass.  Off by default: measured on the 388-matrix MoE layer it takes
                           3.6 % off the step but costs the products 10 % (fewer CUs, shared HBM), and on
                           four such layers the step gets 5 % longer                                    */
  int32_t reserved[2];  /* must be 0 */
} mona_options;

#define MONA_OVERLAP_OFF 0
#define MONA_OVERLAP_LATE_GROUP 1

#define MONA_NS_SCHEDULE_AUTO 0
#define MONA_NS_SCHEDULE_LITERAL 1
#define MONA_NS_SCHEDULE_FUSED 2
#define MONA_NS_SCHEDULE_PAIRS 3

#define MONA_ACCEL_TWO_BUFFER 0
#define MONA_ACCEL_ONE_BUFFER 1
/* The streaming variant as Sec. 6.3 describes it: the arithmetic of Alg. 1 unchanged, but the library
 * keeps no G_{k-1} of its own -- the difference is taken against a gradient slot the CALLER keeps from
 * step to step, and the slot is overwritten with G_k.  Steps of such a state go through
 * mona_step_streaming(); the saving is memory (one state array less), not traffic. */
#define MONA_ACCEL_CALLER_SLOT 2

typedef struct mona_state mona_state;   /* opaque, HOST */

/* Bytes of DEVICE arena needed for `count` matrices (shapes and dtypes are read from
 * mats; the w/g pointers are ignored and may be NULL).  Host-only: touches no GPU.
 *   mats  HOST  array of count descriptors        opts  HOST (NULL = all zero)
 *   bytes_out HOST                                                              */
int mona_state_size(const mona_matrix* mats, int32_t count, const mona_options* opts,
                    size_t* bytes_out);

/* Alg. 1, initialisation line: lay the state {G_{k-1}, A, M} (or {C, M}) of every matrix and the
 * Newton-Schulz workspace out in `arena`, zero it (on `stream`, which is synchronised once
 * before returning), set k = 0 and build the launch plan (same-shape matrices are grouped
 * and orthogonalised together).
 *   arena  DEVICE, 256-byte aligned, arena_bytes >= mona_state_size(); stays the caller's
 *          and must outlive the state
 *   out    HOST   receives the handle; release with mona_free_state                  */
int mona_init_state(const mona_matrix* mats, int32_t count, const mona_options* opts,
                    void* arena, size_t arena_bytes, void* stream, mona_state** out);

/* Alg. 1, one pass of the loop body for every matrix: enqueues the kernels on `stream`
 * and returns without waiting.  `mats` must list the same shapes and dtypes, in the same
 * order, as at init (else MONA_ESHAPE); w and g pointers may differ from step to step.
 * Successive steps on one state must be issued on the same stream or be ordered by the
 * caller.
 * Graph capture: with profiling off and the same w / g pointers as in the previous call
 * (so that no pointer table is uploaded) the call enqueues only kernel launches and the
 * event record / wait pairs that fork and join its side streams -- no memset, no copy --
 * and may be recorded into a HIP graph on a capturing stream.
 * The hyper-parameters are baked into the recorded launches, and the host-side step
 * counter counts calls, not replays (it only matters for MONA_FLAG_FIRST_DIFF_ZERO at
 * the first step).
 * The convergence theorem (Theorem 1) assumes |alpha| < 1 / (1 - beta_a).  A step outside that range
 * is taken all the same and returns MONA_OK; mona_last_error() then holds a warning that says so.
 * If a HIP call fails after the first kernel of a step was enqueued, the state arrays are half updated:
 * the call returns MONA_EHIP and every later step on this state does, until a checkpoint is imported. */
int mona_step(mona_state* st, const mona_matrix* mats, int32_t count,
              const mona_hparams* hp, void* stream);

/* The step of a state built with MONA_ACCEL_CALLER_SLOT (Sec. 6.3, streaming gradient computation).
 *   slots  HOST array of `count` DEVICE pointers; slots[i] is an m x n array of the state dtype
 *          (mona_options.state_dtype), 16-byte aligned, owned by the caller, which must keep its
 *          contents from one step to the next: it holds G_{k-1} on entry (all zero before the
 *          first step: Alg. 1 starts from G_0 = 0) and G_k on return.
 * Everything else as mona_step; mona_step itself returns MONA_EINVAL on such a state, and this
 * function does on any other. */
int mona_step_streaming(mona_state* st, const mona_matrix* mats, void* const* slots, int32_t count,
                        const mona_hparams* hp, void* stream);

/* For callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  One step of Alg. 1 for ONE matrix whose state arrays the caller keeps, with no state
 * handle and no arena: the workspace mona_step finds in the arena (working copies, p x p matrices, partial
 * sums, tables) is a static device array of MONA_NOALLOC_SCRATCH_BYTES inside the library, which every GPU
 * the library runs on holds until the process ends.  The call allocates nothing (no hipMalloc, no pinned
 * host memory, no events or streams), copies nothing from host memory and enqueues only kernels on `stream`.
 *   mat     HOST    one descriptor; w and g DEVICE as for mona_step
 *   opts    HOST    NULL = all zero; accel_form must be MONA_ACCEL_TWO_BUFFER
 *   g_prev  DEVICE  G_{k-1}: m x n of opts->state_dtype, in/out (all zero before the first step)
 *   acc     DEVICE  A_{k-1} in, A_k out: m x n of opts->state_dtype
 *   mom     DEVICE  M_{k-1} in, M_k out: m x n fp32        (all three 16-byte aligned, caller-owned)
 *   k       number of steps this matrix has taken before (only MONA_FLAG_FIRST_DIFF_ZERO looks at it)
 * Results are those of mona_step on a state that holds this one matrix, bit for bit.
 * MONA_ENOMEM if the matrix needs more workspace than the static array holds (roughly: padded m x n up to
 * 2 M elements with a short side up to 1024).  All calls on one GPU share that GPU's array: calls that
 * overlap in time on one GPU (different streams, different threads) race; order them. */
#define MONA_NOALLOC_SCRATCH_BYTES ((size_t)32 << 20)
int mona_step_noalloc(const mona_matrix* mat, const mona_options* opts, void* g_prev, void* acc, void* mom,
                      const mona_hparams* hp, int64_t k, void* stream);

/* Release host bookkeeping (waits for the state's pinned tables to be idle).  The arena
 * is not touched. */
int mona_free_state(mona_state* st);

typedef enum mona_view_kind {
  MONA_VIEW_G_PREV = 0,  /* G_{k-1}: m x n, state dtype (MONA_EUNSUPPORTED when the caller keeps it) */
  MONA_VIEW_A = 1,       /* A_k:     m x n, state dtype                                */
  MONA_VIEW_M = 2,       /* M_k:     m x n, fp32                                       */
  MONA_VIEW_NORM = 3,    /* ||M_k||_F of the last step: 1 x 1 fp32                      */
  MONA_VIEW_O = 4,       /* O_k of the last step (needs MONA_FLAG_KEEP_O): m x n with a
                            leading dimension ld >= n, bf16 (ns_precision 0) or fp32 (1) */
  MONA_VIEW_C = 5        /* one-buffer form only: C_{k+1}, m x n, state dtype.  There
                            MONA_VIEW_G_PREV and MONA_VIEW_A return MONA_EUNSUPPORTED, and
                            here MONA_VIEW_C does                                        */
} mona_view_kind;

typedef struct mona_view {
  void* ptr;             /* DEVICE, inside the arena                                    */
  int32_t rows, cols;
  int32_t ld;            /* elements between consecutive rows                           */
  int32_t dtype;         /* mona_dtype                                                  */
} mona_view;

/* Where a piece of matrix i's state lives (test and checkpoint hook).  The caller may
 * read it, or write it between steps, after synchronising the stream. */
int mona_state_view(mona_state* st, int32_t i, int32_t kind, mona_view* out);

/* Checkpointing.  The persistent state is one contiguous block of the arena holding
 * {G_{k-1}, A, M} (one-buffer form: {C, M}) of every matrix; export copies it to dst, import copies it back
 * (both DEVICE-to-DEVICE, asynchronous on `stream`), and the step counter travels
 * separately.  A state imported into a fresh mona_init_state of the same matrix list
 * continues bit-identically. */
int mona_state_export_size(mona_state* st, size_t* bytes_out);
int mona_state_export(mona_state* st, void* dst, size_t dst_bytes, void* stream);
int mona_state_import(mona_state* st, const void* src, size_t src_bytes, int64_t step_count,
                      void* stream);
int mona_state_step_count(mona_state* st, int64_t* k_out);

/* Per-matrix status bits of the last step, copied to HOST after synchronising `stream`:
 * bit 0: ||M||_F + eps == 0 (O = 0, only weight decay applied);
 * bit 1: ||M||_F not finite (the matrix's W was left unchanged). */
#define MONA_STATUS_ZERO_NORM 0x1u
#define MONA_STATUS_NONFINITE 0x2u
/* bit 2 (informative): ||M||_F lay outside [2^-40, 2^40], so the working copy of M was rescaled by a power
 * of two before the products (the result is unaffected: Sec. 3.2's X_0 = M / ||M||_F is scale-free). */
#define MONA_STATUS_RESCALED 0x4u
int mona_state_status(mona_state* st, uint32_t* host_out, int32_t count, void* stream);

/* Elapsed GPU time of the phases of the last mona_step, from HIP events recorded on the
 * stream the step ran on.  Enabled with mona_set_profiling(st, 1); waits for the step.
 *   ms_out HOST float[4]: elementwise state + norm, Newton-Schulz products,
 *                         update (0 when fused into the last product), whole step.
 * With a late group (mona_options.overlap) the first figure covers the pass of the other groups only and
 * the second runs from there to the last product, the late pass hidden inside it; at level 2 everything
 * runs in one row on the caller's stream and the figures are those of the phases one after the other. */
int mona_set_profiling(mona_state* st, int32_t level /* 0 off, 1 phases, 2 every launch */);
int mona_last_step_times(mona_state* st, float* ms_out);
/* The same four figures averaged over the profiled steps since mona_set_profiling was last called (the
 * last 32 of them if there were more); *steps_out says over how many.  Waits for those steps. */
int mona_mean_step_times(mona_state* st, float* ms_out, int32_t* steps_out);

/* With mona_set_profiling(st, 2) every Newton-Schulz product launch of a step is bracketed
 * by its own pair of events.  mona_last_step_launches waits for the step and fills up to
 * max_records entries (out may be NULL to query the count).
 *   kind: 0 = Gram (X X^T), 1 = poly (b S + c S S [+ a I]), 2 = apply (a X + B X, or R X),
 *         3 = product of two commuting symmetric p x p matrices (fused schedule)
 *   tile:  block tile of the kernel, rows * 1000 + columns (e.g. 256128)
 *   flops: MFMA flop the launch issues (tiles x 2 x rows x columns x K), padding included */
typedef struct mona_launch_time {
  int32_t kind, group, iter, tile;
  int32_t m, n, count;   /* shape of the group's matrices and how many there are */
  float ms;
  double flops;
} mona_launch_time;
int mona_last_step_launches(mona_state* st, mona_launch_time* out, int32_t max_records,
                            int32_t* n_out);

/* Number of kernel launches and executed MFMA flop of the Newton-Schulz part of one
 * step under the current plan (host-only bookkeeping, for roofline reporting). */
int mona_plan_info(mona_state* st, int32_t ns_steps, int64_t* launches_out,
                   double* ns_flops_executed_out, double* elementwise_bytes_out);

/* ---------------------------------------------------------------------------------------
 * AdamW for the parameters that are not matrices (Sec. 4.1, text above Alg. 1: embeddings,
 * biases, norm gains "fall back to AdamW").  The paper prints no formula of its own; this
 * is the published decoupled-weight-decay Adam, with m_0 = v_0 = 0 and t counted from 1:
 *
 *     m_t = beta1 m_{t-1} + (1 - beta1) g_t          v_t = beta2 v_{t-1} + (1 - beta2) g_t^2
 *     w_t = w_{t-1} - eta ( (m_t / (1 - beta1^t)) / (sqrt(v_t / (1 - beta2^t)) + eps)
 *                           + lambda w_{t-1} )
 *
 * Same conventions as above: the caller owns w, g, the arena and the stream; nothing here
 * allocates device memory; all tensors of the list are updated by one fused pass.
 * ------------------------------------------------------------------------------------- */
typedef struct mona_vector {
  void* w;            /* DEVICE: parameter, n contiguous elements, 16-byte aligned; in/out  */
  const void* g;      /* DEVICE: gradient, n contiguous elements, 16-byte aligned; read     */
  int64_t n;          /* 1 <= n <= 2^40 (any shape: the update is elementwise)              */
  int32_t w_dtype;    /* mona_dtype; bf16 parameters are stored round-to-nearest-even       */
  int32_t g_dtype;    /* mona_dtype                                                         */
} mona_vector;

typedef struct mona_adamw_hparams {
  float lr;            /* eta                                   */
  float beta1, beta2;  /* in [0, 1)                             */
  float eps;           /* >= 0, added to sqrt(vhat)             */
  float weight_decay;  /* lambda, decoupled, acts on w_{t-1}    */
} mona_adamw_hparams;

typedef struct mona_adamw_state mona_adamw_state;   /* opaque, HOST */

/* Bytes of DEVICE arena for the moments {m, v} (fp32) of `count` tensors plus small tables.
 * Host-only.  vecs HOST (w / g ignored, may be NULL); bytes_out HOST. */
int mona_adamw_state_size(const mona_vector* vecs, int32_t count, size_t* bytes_out);
/* Lays {m, v} out in `arena` (DEVICE, 256-byte aligned, stays the caller's), zeroes them on
 * `stream` (synchronised once before returning) and sets t = 0. */
int mona_adamw_init_state(const mona_vector* vecs, int32_t count, void* arena, size_t arena_bytes,
                          void* stream, mona_adamw_state** out);
/* One AdamW step for every tensor, enqueued on `stream`, no wait.  Sizes and dtypes must
 * match init (MONA_ESHAPE otherwise); w and g pointers may change from step to step.
 * Not for graph replay: the bias corrections 1 / (1 - beta^t) are computed on the host
 * for this call's t and passed as launch arguments. */
int mona_adamw_step(mona_adamw_state* st, const mona_vector* vecs, int32_t count,
                    const mona_adamw_hparams* hp, void* stream);
int mona_adamw_free_state(mona_adamw_state* st);

#define MONA_ADAMW_VIEW_M 0
#define MONA_ADAMW_VIEW_V 1
/* DEVICE address (inside the arena) and element count of tensor i's fp32 m or v. */
int mona_adamw_state_view(mona_adamw_state* st, int32_t i, int32_t kind, void** dev_ptr,
                          int64_t* n_out);
/* Checkpointing: {m, v} of every tensor is one contiguous block; t travels separately. */
int mona_adamw_state_export_size(mona_adamw_state* st, size_t* bytes_out);
int mona_adamw_state_export(mona_adamw_state* st, void* dst, size_t dst_bytes, void* stream);
int mona_adamw_state_import(mona_adamw_state* st, const void* src, size_t src_bytes,
                            int64_t step_count, void* stream);
int mona_adamw_state_step_count(mona_adamw_state* st, int64_t* t_out);

const char* mona_last_error(void);
const char* mona_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MONA_H */
