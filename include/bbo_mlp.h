/*
 * bbo_mlp.h — C ABI of the batched MLP cross-validation evaluator for MI355X.
 *
 * One call evaluates a whole list of hyper-parameter suggestions the way the
 * suggest-observe loop of the paper's Algorithm 1 needs it: suggestions in,
 * one cross-validation score per suggestion out (Section 2 defines the
 * objective as a model's cross-validation score on a dataset under a loss;
 * Table 1 lists the MLP-adam / MLP-sgd models and the nll / acc / mse
 * metrics).  Every (suggestion, fold) pair is one small MLP; all of them are
 * trained and scored by HIP kernels inside a single call.
 *
 * Conventions
 *   - "device" pointers are HIP device memory on the current device; "host"
 *     pointers are ordinary host memory.  The caller owns every buffer.  The
 *     library allocates no device memory and keeps no state between calls
 *     (it keeps a small pinned host staging buffer per host thread and
 *     device; bbo_mlp_cv_eval_static is the one call that brings its own
 *     device workspace, a static array inside the library).
 *   - Work is enqueued on the caller's stream and the call returns without
 *     waiting for it; outputs are valid once the stream has been synchronised.
 *   - Every function returns BBO_OK or an error code; bbo_mlp_last_error()
 *     gives the message of the calling thread's last failure.  Nothing throws
 *     or aborts across this boundary.  A training run that blows up
 *     numerically is not an error: its score is left non-finite and its
 *     status entry is set to 1; other suggestions are unaffected.
 */
#ifndef BBO_MLP_H
#define BBO_MLP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BBO_MAX_HIDDEN 4     /* hidden layers per model */
#define BBO_MAX_WIDTH 1024   /* units per hidden layer */
#define BBO_MAX_FEATURES 4096
#define BBO_MAX_CLASSES 256

enum {
  BBO_OK = 0,
  BBO_INVALID_ARG = 1,
  BBO_UNSUPPORTED = 2,         /* shape beyond the compiled maxima above */
  BBO_WORKSPACE_TOO_SMALL = 3,
  BBO_DEVICE_ERROR = 4
};

enum { BBO_ADAM = 0, BBO_SGD = 1 };
enum { BBO_F32 = 0, BBO_BF16 = 1 };

/* One suggestion (Algorithm 1: an element of params_list).  POD, host memory. */
typedef struct bbo_mlp_hparams {
  int32_t n_hidden;               /* 0..BBO_MAX_HIDDEN; 0 is a linear model */
  int32_t hidden[BBO_MAX_HIDDEN]; /* widths, 1..BBO_MAX_WIDTH */
  int32_t solver;                 /* BBO_ADAM | BBO_SGD */
  int32_t nesterov;               /* SGD only */
  int32_t batch_size;             /* rows per step; <=0 or larger than the fold's
                                     training rows => full batch */
  int32_t epochs;                 /* >= 0; 0 scores the initial weights */
  float lr, alpha, momentum, beta1, beta2, eps;
  float power_t;                  /* SGD only: learning rate of epoch e =
                                     lr / (1 + e * n_train)^power_t; 0 = constant */
  uint64_t seed;                  /* initial weights and minibatch order */
  float tol;                      /* plateau stop, active when n_iter_no_change > 0: */
  int32_t n_iter_no_change;       /* training ends once the epoch's mean data loss has
                                     failed to beat the best so far by tol for more
                                     than this many epochs in a row; `epochs` stays
                                     the upper limit.  Switched off in a traced call
                                     that resumes from state_in. */
  float validation_fraction;      /* early stopping on held-out rows (the option the
                                     benchmark's MLP-adam / MLP-sgd of Table 1 are
                                     tuned with), active when > 0 and
                                     n_iter_no_change > 0: floor(fraction * n_train)
                                     rows (at least 1, at most n_train - 1) of the
                                     fold's training rows, chosen by a seeded
                                     shuffle, are never trained on, and the rule
                                     above watches THEIR loss (cross-entropy, or the
                                     plain mean squared error) after every epoch
                                     instead of the training loss.  The parameters
                                     of the epoch with the lowest such loss are kept
                                     aside, and when training ends (by the rule or
                                     at `epochs`) they are the model that is scored. */
  int32_t reserved;               /* 0 */
} bbo_mlp_hparams;

/*
 * Bytes of device workspace bbo_mlp_cv_eval needs for this problem.
 * hp: host, [B].  dtype: BBO_F32 | BBO_BF16.  Writes *out.
 * Errors: BBO_INVALID_ARG, BBO_UNSUPPORTED.
 */
int bbo_mlp_workspace_bytes(int64_t n, int32_t d, int32_t n_classes, int32_t n_folds,
                            const bbo_mlp_hparams* hp, int32_t B, int32_t dtype, size_t* out);

/*
 * evaluate(params_list) -> scores (Algorithm 1; Section 2).
 *
 *   X         device, row-major [n][d]; float32 (BBO_F32) or bfloat16 (BBO_BF16)
 *   y         device, [n]; int32 class ids 0..n_classes-1 if n_classes >= 2,
 *             int32 labels 0/1 if n_classes == 1 (one logit), float32 targets
 *             if n_classes == 0 (regression)
 *   fold_idx  device, int32 [n]; row i validates in fold fold_idx[i] and trains
 *             in every other fold; a negative value leaves the row unused
 *   hp        host, [B] suggestions
 *   scores    device, float32 [B][2]: {mean over folds of nll | mse,
 *             mean over folds of accuracy | mean absolute error}
 *   status    device, int32 [B]: 0 ok, 1 the first score is not finite
 *   per_fold  device, float32 [B][n_folds][2], or NULL
 *   workspace device, >= bbo_mlp_workspace_bytes() bytes, 256-byte aligned;
 *             contents are scratch
 *   stream    hipStream_t (NULL = default stream)
 *
 * Model: layers z = a W + b with ReLU between them; softmax cross-entropy over
 * n_classes outputs (n_classes >= 2), the logistic loss log(1 + e^z) - y z on
 * a single output (n_classes == 1; the second score is the accuracy of the
 * rule z > 0), or half squared error (n_classes == 0); penalty
 * alpha/(2 m) * |W|^2 with m the rows of the step; Adam (bias corrections in
 * the step size, eps added to sqrt(v)) or SGD with (Nesterov) momentum;
 * constant learning rate; exactly `epochs` passes in a seeded order; a short
 * last minibatch is kept.  BBO_BF16 rounds GEMM operands (inputs, weights,
 * hidden activations, deltas) to bfloat16 and keeps master weights, moments
 * and accumulation in float32.
 *
 * Errors: BBO_INVALID_ARG (null pointer, n < 0, d < 1, n_classes < 0,
 * n_folds < 1, bad hparams), BBO_UNSUPPORTED, BBO_WORKSPACE_TOO_SMALL,
 * BBO_DEVICE_ERROR (a HIP call failed).  B == 0 is a no-op returning BBO_OK.
 */
int bbo_mlp_cv_eval(const void* X, const void* y, int64_t n, int32_t d, int32_t n_classes,
                    const int32_t* fold_idx, int32_t n_folds, const bbo_mlp_hparams* hp,
                    int32_t B, int32_t dtype, float* scores, int32_t* status, float* per_fold,
                    void* workspace, size_t workspace_bytes, void* stream);

/*
 * bbo_mlp_cv_eval for callers that cannot allocate device memory (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc):
 * the workspace is a static device array inside the library, so the call takes
 * no workspace and makes no allocation of any kind on the device or in pinned
 * host memory (the item list travels as kernel arguments).  Same arguments,
 * same kernels and bit-identical results otherwise.
 *   limit   the problem's bbo_mlp_workspace_bytes() must not exceed
 *           BBO_STATIC_SCRATCH_BYTES, and its item records (a few hundred
 *           bytes per suggestion and fold) BBO_STATIC_MAX_ITEM_BYTES; beyond
 *           that the call returns BBO_WORKSPACE_TOO_SMALL and enqueues nothing.
 *   sharing every call on a device uses that device's one array: calls that
 *           overlap in time on one device (different streams or threads) race.
 *           Calls one after the other on one stream are fine; nothing is
 *           assumed about the array's contents.
 * Each device the library runs on holds the array until the process ends.
 */
#define BBO_STATIC_SCRATCH_BYTES (32u << 20)
#define BBO_STATIC_MAX_ITEM_BYTES (1u << 20)
int bbo_mlp_cv_eval_static(const void* X, const void* y, int64_t n, int32_t d, int32_t n_classes,
                           const int32_t* fold_idx, int32_t n_folds, const bbo_mlp_hparams* hp,
                           int32_t B, int32_t dtype, float* scores, int32_t* status, float* per_fold,
                           void* stream);

/*
 * Same evaluation, additionally recording the training steps
 * [step_begin, step_end) (counted over all epochs) of the single model
 * (trace_b, trace_fold) for parity checks of the per-step arithmetic.
 *   trace_out  device, float32 [step_end-step_begin][1 + 2P]: training loss of
 *              the step, its gradient, and the parameters after the update,
 *              packed per layer as W[in][out] then b[out]; P = parameter count
 *   trace_floats  capacity of trace_out in floats
 *   state_in   device, float32 [3P] or NULL.  When given, the traced model does
 *              not start from its initial weights: it resumes at step_begin
 *              from these parameters, first moments (or SGD velocities) and
 *              second moments, each packed like the parameters.  This isolates
 *              the arithmetic of single steps from the drift of a long run.
 * Errors: as bbo_mlp_cv_eval, plus BBO_INVALID_ARG for a window or item out of
 * range or a trace buffer that is too small.
 */
int bbo_mlp_cv_eval_traced(const void* X, const void* y, int64_t n, int32_t d,
                           int32_t n_classes, const int32_t* fold_idx, int32_t n_folds,
                           const bbo_mlp_hparams* hp, int32_t B, int32_t dtype, float* scores,
                           int32_t* status, float* per_fold, void* workspace,
                           size_t workspace_bytes, void* stream, int32_t trace_b,
                           int32_t trace_fold, int64_t step_begin, int64_t step_end,
                           float* trace_out, size_t trace_floats, const float* state_in);

/*
 * The hold-out (generalization) score (Section 6.2, Figure 2(b): the score of
 * the held-out test data, which the optimizers never see).  Each suggestion is
 * trained once on every row that belongs to a fold (fold_idx >= 0) and scored
 * on the rows that belong to none (fold_idx < 0), with the same training and
 * scoring arithmetic as bbo_mlp_cv_eval.  The model is keyed as fold -1: its
 * initial weights and minibatch order are independent of the suggestion's
 * cross-validation models.
 *   X, y, fold_idx, hp, dtype, status, workspace, stream: as for bbo_mlp_cv_eval
 *   scores     device, float32 [B][2] = {nll | mse, accuracy | mae} on the held
 *              rows; NaN (status 1) when no row is held out
 *   workspace  at least bbo_mlp_workspace_bytes(..., n_folds = 1, ...) bytes
 * Returns BBO_OK after enqueueing, or an error code as bbo_mlp_cv_eval does.
 */
int bbo_mlp_holdout_eval(const void* X, const void* y, int64_t n, int32_t d, int32_t n_classes,
                         const int32_t* fold_idx, const bbo_mlp_hparams* hp, int32_t B,
                         int32_t dtype, float* scores, int32_t* status, void* workspace,
                         size_t workspace_bytes, void* stream);

/*
 * The cross-validation split as the kernels see it (Section 2: k-fold
 * cross-validation score).  For each fold f the ascending list of training
 * rows (fold_idx not in {f, negative}) and of held rows (fold_idx == f).
 *   train_idx, val_idx  device, int32 [n_folds][n] (only the first count
 *                       entries of each row are written)
 *   counts              device, int32 [n_folds][2] = {n_train, n_val}
 */
int bbo_mlp_fold_lists(const int32_t* fold_idx, int64_t n, int32_t n_folds, int32_t* train_idx,
                       int32_t* val_idx, int32_t* counts, void* stream);

/*
 * The hold-out split as the kernels see it (Section 6.2): the ascending list
 * of the rows of all folds (fold_idx >= 0, training) and of the rows of none
 * (fold_idx < 0, scored).
 *   train_idx, val_idx  device, int32 [n]; counts device, int32 [2]
 */
int bbo_mlp_holdout_lists(const int32_t* fold_idx, int64_t n, int32_t* train_idx, int32_t* val_idx,
                          int32_t* counts, void* stream);

/*
 * The rows of minibatch `step` of `epoch` for suggestion hp[0] in fold `fold`,
 * from train_idx / counts as written by bbo_mlp_fold_lists; fold = -1 is the
 * hold-out model, with train_idx / counts from bbo_mlp_holdout_lists.
 * step = -1 asks for the rows the model sets aside for early stopping instead
 * (none unless validation_fraction and n_iter_no_change are both positive).
 *   rows_out  device, int32 [batch rows]; n_rows_out device int32 [1]
 */
int bbo_mlp_minibatch_rows(const int32_t* train_idx, const int32_t* counts, int64_t n,
                           const bbo_mlp_hparams* hp, int32_t fold, int32_t epoch, int64_t step,
                           int32_t* rows_out, int32_t* n_rows_out, void* stream);

/*
 * Initial parameters of suggestion hp[0] in fold `fold` (-1: the hold-out
 * model), Glorot-uniform from the counter-based generator, packed per layer as
 * W[in][out] then b[out].
 *   theta_out  device, float32 [P]
 */
int bbo_mlp_init_params(int32_t d, int32_t n_classes, const bbo_mlp_hparams* hp, int32_t fold,
                        float* theta_out, void* stream);

/* Number of parameters P of suggestion hp[0]; negative on invalid input. */
int64_t bbo_mlp_param_count(int32_t d, int32_t n_classes, const bbo_mlp_hparams* hp);

/*
 * Which training kernel suggestion hp[0] runs on for a data set of n rows (host
 * logic only, no device call): 0 the LDS-tiled bf16 kernel, 1 the LDS-resident
 * fp32 kernel, 2 the wavefront-per-model kernel (no hidden layer), 3 the
 * generic kernel, 4 the wider LDS-resident fp32 kernel (one hidden layer, up to
 * 127 inputs and 16 outputs); negative on invalid input.  Every suggestion of a call gets
 * the kernel this returns for it, whatever else the call holds (Algorithm 1's
 * evaluate(params_list) treats the suggestions independently).
 */
int bbo_mlp_kernel_class(int64_t n, int32_t d, int32_t n_classes, const bbo_mlp_hparams* hp,
                         int32_t dtype);

/* Message of the calling thread's last error ("" if none). */
const char* bbo_mlp_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* BBO_MLP_H */
