/*
 * CPU oracle for the batched cross-validated MLP evaluation.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what
 * the evaluation step of the suggest-observe loop computes.  The paper's
 * Section 2 defines the objective handed to an optimizer as a model's
 * cross-validation score on a dataset under a loss; Algorithm 1 calls it once
 * per iteration on the whole list of suggestions and gets one score back per
 * suggestion; Table 1 names the MLP-adam / MLP-sgd models and the nll / acc /
 * mse metrics.  It shares no code with the GPU library.  Only the tests, the
 * smoke check and the reported CPU baseline may call it.
 *
 * The paper is silent about the MLP's arithmetic; the readings taken here
 * (scikit-learn-style conventions) are:
 *   - layers z_l = a_{l-1} W_l + b_l, ReLU on hidden layers, identity output
 *     for regression, softmax over n_classes outputs for classification
 *     (binary included); n_classes == 1 is the other binary form, the one
 *     scikit-learn-style MLPs use: ONE output z, labels 0/1, p = 1/(1+e^-z),
 *     loss log(1 + e^z) - y z (the cross-entropy of p against y), output
 *     delta p - y, accuracy = mean[(z > 0) == y];
 *   - training loss = mean cross-entropy, or half the mean squared error,
 *     plus alpha/(2 m) * sum of squared weights (biases unpenalised), m being
 *     the number of rows of the minibatch actually used (a short last
 *     minibatch is kept);
 *   - ReLU derivative at 0 is 0;
 *   - Adam in the form with the bias corrections folded into the step size
 *     and eps added to sqrt(v); SGD with momentum, optionally Nesterov;
 *     constant learning rate, exactly `epochs` passes unless a stopping rule
 *     is switched on (see train_and_score);
 *   - scores on the held fold: nll = -mean log softmax(z)[y] (no clipping),
 *     acc = mean[argmax z == y] with ties to the lowest class, mse =
 *     mean (yhat - y)^2;  the CV score is the unweighted mean over folds.
 *
 * Arithmetic: parameters and optimizer state hold fp32 values; every dot
 * product / batch reduction is accumulated in fp64 and rounded once to fp32;
 * elementwise operations are rounded to fp32 after each operation.  With
 * prec=1 no rounding happens anywhere (pure fp64), which the gradient and
 * closed-form pins use.  prec=2 is a sensitivity probe (see accum()): fp32
 * running sums in the four contractions, everything else as prec=0.  With dtype=1 the GEMM operands (inputs, weights,
 * hidden activations, deltas) are rounded to bfloat16 (round to nearest even)
 * at the points marked BF below; master weights, moments and accumulation
 * stay fp32.
 *
 * Random numbers: a counter-based generator built on the SplitMix64 output
 * mixer (Steele, Lea, Flood 2014).  Initial weights are Glorot-uniform from a
 * 24-bit draw per element; the minibatch order of an epoch is a keyed
 * bijection of [0, n_train): a 4-round balanced Feistel network on an even
 * number of bits with cycle walking.
 *
 * Parity unpinned: the final CV scores of the benchmark configurations have
 * no published value; they are compared GPU <-> oracle only.  The two tie
 * rules of the accuracy (equal logits go to the lowest class; a single logit
 * of exactly zero counts as class 0) need exactly equal logits, which no
 * input of this interface produces on purpose: they are unpinned as well.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_MAX_HIDDEN 4
#define GOLDEN 0x9E3779B97F4A7C15ULL

typedef struct oracle_hparams {
  int32_t n_hidden;
  int32_t hidden[ORACLE_MAX_HIDDEN];
  int32_t solver;   /* 0 adam, 1 sgd */
  int32_t nesterov; /* sgd only */
  int32_t batch_size; /* 0 => full batch; clipped to the fold's train rows */
  int32_t epochs;
  float lr, alpha, momentum, beta1, beta2, eps;
  float power_t; /* sgd only: learning rate of epoch e = lr / (1 + e * n_train)^power_t; 0 = constant */
  uint64_t seed;
  float tol;                /* with n_iter_no_change > 0: training stops once the epoch's mean data loss */
  int32_t n_iter_no_change; /* has failed to improve on the best so far by tol more than this many epochs in a row */
  float validation_fraction; /* with n_iter_no_change > 0 and this > 0: that share of the fold's training rows is
                                set aside, never trained on, and the rule watches ITS loss after every epoch;
                                the model that is scored is the one of the epoch with the lowest such loss */
  int32_t reserved;
} oracle_hparams;

/* ------------------------------------------------------------------ */
/* counter-based random numbers                                        */
/* ------------------------------------------------------------------ */

/* SplitMix64 output function. */
uint64_t oracle_mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
  return z ^ (z >> 31);
}

/* Fold a counter into a key: the SplitMix64 stream started at h, read at
 * position v. */
uint64_t oracle_combine(uint64_t h, uint64_t v) {
  return oracle_mix64(h + (v + 1) * GOLDEN);
}

static uint64_t model_key(uint64_t seed, int fold) {
  return oracle_combine(oracle_combine(seed, 0x4D4C50ULL), (uint64_t)fold);
}

static uint64_t epoch_key(uint64_t seed, int fold, int epoch) {
  return oracle_combine(oracle_combine(model_key(seed, fold), 1), (uint64_t)epoch);
}

/* Keyed bijection of [0, n): position p of the epoch -> index into the
 * fold's ascending list of training rows. */
static int64_t perm_index(uint64_t key, int64_t n, int64_t p) {
  if (n <= 1) return 0;
  int bits = 0;
  while (((int64_t)1 << bits) < n) bits++;
  if (bits & 1) bits++;
  if (bits < 2) bits = 2;
  int hb = bits / 2;
  uint64_t mask = ((uint64_t)1 << hb) - 1;
  uint64_t x = (uint64_t)p;
  do {
    uint64_t L = x >> hb, R = x & mask;
    for (uint64_t r = 0; r < 4; r++) {
      uint64_t F = oracle_combine(key, (r << 32) | R) & mask;
      uint64_t t = L ^ F;
      L = R;
      R = t;
    }
    x = (L << hb) | R;
  } while ((int64_t)x >= n);
  return (int64_t)x;
}

int64_t oracle_perm_index(uint64_t seed, int32_t fold, int32_t epoch, int64_t n, int64_t p) {
  return perm_index(epoch_key(seed, fold, epoch), n, p);
}

/* ------------------------------------------------------------------ */
/* rounding helpers                                                    */
/* ------------------------------------------------------------------ */

static inline double rnd(double x, int prec) { return prec == 1 ? x : (double)(float)x; }

/* One term of a dot product.  prec 0 and 1 accumulate in fp64 (the definition).  prec 2 is a PROBE, not a
 * definition: the running sum is rounded to fp32 after every term, the way a single-precision pipeline
 * sums, so that comparing its final scores with those of prec 0 tells how far rounding at the level of an
 * fp32 accumulator moves this particular training run (its sensitivity, used by the tests to tell stable
 * runs from chaotic ones). */
static inline double accum(double acc, double term, int prec) {
  return prec == 2 ? (double)(float)(acc + (double)(float)term) : acc + term;
}

/* float -> bfloat16 bits, round to nearest even; NaN stays NaN (quiet). */
uint16_t oracle_bf16_bits(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

static inline double bf16_to_double(uint16_t h) {
  uint32_t u = (uint32_t)h << 16;
  float f;
  memcpy(&f, &u, 4);
  return (double)f;
}

/* BF: value -> nearest bfloat16 when the bf16 configuration is on. */
static inline double opnd(double x, int dtype) {
  return dtype ? bf16_to_double(oracle_bf16_bits((float)x)) : x;
}

/* ------------------------------------------------------------------ */
/* model description                                                   */
/* ------------------------------------------------------------------ */

typedef struct {
  int L;                            /* number of weight layers */
  int dims[ORACLE_MAX_HIDDEN + 2];  /* d, h..., c_out */
  int64_t w_off[ORACLE_MAX_HIDDEN + 1], b_off[ORACLE_MAX_HIDDEN + 1];
  int64_t P;
  int n_classes; /* 0 = regression */
} net_t;

static int net_build(net_t* net, int d, int n_classes, const oracle_hparams* hp) {
  if (hp->n_hidden < 0 || hp->n_hidden > ORACLE_MAX_HIDDEN) return -1;
  net->L = hp->n_hidden + 1;
  net->dims[0] = d;
  for (int i = 0; i < hp->n_hidden; i++) {
    if (hp->hidden[i] < 1) return -1;
    net->dims[i + 1] = hp->hidden[i];
  }
  net->dims[net->L] = n_classes >= 2 ? n_classes : 1;
  net->n_classes = n_classes;
  int64_t off = 0;
  for (int l = 0; l < net->L; l++) {
    net->w_off[l] = off;
    off += (int64_t)net->dims[l] * net->dims[l + 1];
    net->b_off[l] = off;
    off += net->dims[l + 1];
  }
  net->P = off;
  return 0;
}

int64_t oracle_param_count(int32_t d, int32_t n_classes, const oracle_hparams* hp) {
  net_t net;
  if (net_build(&net, d, n_classes, hp)) return -1;
  return net.P;
}

/* Glorot-uniform initial parameters, packed per layer as W[in][out] then
 * b[out].  The bound is sqrt(6/(fan_in+fan_out)) rounded to fp32; the draw
 * is (k - 2^23)/2^23 with k the top 24 bits of the element's hash. */
static void init_params(const net_t* net, uint64_t seed, int fold, double* theta) {
  uint64_t km = model_key(seed, fold);
  for (int l = 0; l < net->L; l++) {
    int fi = net->dims[l], fo = net->dims[l + 1];
    double bound = rnd(sqrt(6.0 / (double)(fi + fo)), 0);
    for (int t = 0; t < 2; t++) {
      uint64_t kt = oracle_combine(km, (uint64_t)(16 + 2 * l + t));
      int64_t cnt = t == 0 ? (int64_t)fi * fo : fo;
      double* dst = theta + (t == 0 ? net->w_off[l] : net->b_off[l]);
      for (int64_t i = 0; i < cnt; i++) {
        uint64_t k24 = oracle_combine(kt, (uint64_t)i) >> 40;
        double frac = ((double)k24 - 8388608.0) / 8388608.0;
        dst[i] = rnd(bound * frac, 0); /* initial values are fp32 in every mode */
      }
    }
  }
}

int oracle_init_params(int32_t d, int32_t n_classes, const oracle_hparams* hp, int32_t fold,
                       double* theta_out) {
  net_t net;
  if (net_build(&net, d, n_classes, hp)) return -1;
  init_params(&net, hp->seed, fold, theta_out);
  return 0;
}

/* ------------------------------------------------------------------ */
/* data access                                                         */
/* ------------------------------------------------------------------ */

typedef struct {
  const void* X; /* float32 [n][d] (dtype 0) or bfloat16 bits [n][d] (dtype 1) */
  const void* y; /* int32 [n] (classification) or float32 [n] (regression) */
  int64_t n;
  int d;
  int dtype;
} data_t;

static inline double x_at(const data_t* D, int64_t row, int col) {
  if (D->dtype) return bf16_to_double(((const uint16_t*)D->X)[row * D->d + col]);
  return (double)((const float*)D->X)[row * D->d + col];
}

/* ------------------------------------------------------------------ */
/* forward / loss / backward on one set of rows                        */
/* ------------------------------------------------------------------ */

typedef struct {
  double* a[ORACLE_MAX_HIDDEN + 2];     /* a[0] = inputs, a[l] = activations [m][dims[l]] */
  double* delta[ORACLE_MAX_HIDDEN + 2]; /* delta[l] for layer output l (1..L) */
  double* wop;                          /* GEMM-operand copy of the parameters */
  int64_t cap_rows;
} scratch_t;

static int scratch_alloc(scratch_t* s, const net_t* net, int64_t rows) {
  memset(s, 0, sizeof(*s));
  s->cap_rows = rows;
  for (int l = 0; l <= net->L; l++) {
    s->a[l] = (double*)malloc(sizeof(double) * (size_t)(rows > 0 ? rows : 1) * net->dims[l]);
    s->delta[l] = (double*)malloc(sizeof(double) * (size_t)(rows > 0 ? rows : 1) * net->dims[l]);
    if (!s->a[l] || !s->delta[l]) return -1;
  }
  s->wop = (double*)malloc(sizeof(double) * (size_t)net->P);
  return s->wop ? 0 : -1;
}

static void scratch_free(scratch_t* s, const net_t* net) {
  for (int l = 0; l <= net->L; l++) {
    free(s->a[l]);
    free(s->delta[l]);
  }
  free(s->wop);
}

/* Forward pass over `m` rows; leaves pre-softmax outputs z_L in a[L]. */
static void forward(const net_t* net, const data_t* D, const int32_t* rows, int64_t m,
                    const double* theta, scratch_t* s, int prec) {
  int dt = D->dtype;
  for (int64_t i = 0; i < net->P; i++) s->wop[i] = opnd(theta[i], dt); /* BF: weights */
  for (int64_t r = 0; r < m; r++)
    for (int k = 0; k < net->dims[0]; k++) s->a[0][r * net->dims[0] + k] = x_at(D, rows[r], k);
  for (int l = 0; l < net->L; l++) {
    int fi = net->dims[l], fo = net->dims[l + 1];
    const double* W = s->wop + net->w_off[l];
    const double* b = theta + net->b_off[l]; /* bias is added in fp32, not a GEMM operand */
    for (int64_t r = 0; r < m; r++) {
      for (int j = 0; j < fo; j++) {
        double acc = 0.0;
        for (int k = 0; k < fi; k++) acc = accum(acc, s->a[l][r * fi + k] * W[(int64_t)k * fo + j], prec);
        double z = rnd(acc + b[j], prec);
        if (l + 1 < net->L) {
          z = z > 0.0 ? z : 0.0;
          z = opnd(z, dt); /* BF: hidden activations */
        }
        s->a[l + 1][r * fo + j] = z;
      }
    }
  }
}

/* Mean data loss over the rows, and the output-layer delta (already divided
 * by m) in delta[L] when want_delta. */
static double data_loss(const net_t* net, const data_t* D, const int32_t* rows, int64_t m,
                        scratch_t* s, int prec, int want_delta, int half_sq) {
  int c = net->dims[net->L];
  double total = 0.0;
  for (int64_t r = 0; r < m; r++) {
    const double* z = s->a[net->L] + r * c;
    double* dl = s->delta[net->L] + r * c;
    if (net->n_classes >= 2) {
      int yr = ((const int32_t*)D->y)[rows[r]];
      double mx = z[0];
      for (int j = 1; j < c; j++) mx = z[j] > mx ? z[j] : mx;
      double se = 0.0;
      for (int j = 0; j < c; j++) se += exp(z[j] - mx);
      double lse = mx + log(se);
      total += rnd(lse - z[yr], prec);
      if (want_delta)
        for (int j = 0; j < c; j++) {
          double p = rnd(exp(z[j] - lse), prec);
          double g = rnd(p - (j == yr ? 1.0 : 0.0), prec);
          dl[j] = opnd(rnd(g / (double)m, prec), D->dtype); /* BF: deltas */
        }
    } else if (net->n_classes == 1) {
      /* single-logit binary head: log(1 + e^z) - y z in the form that cannot overflow */
      double yr = (double)((const int32_t*)D->y)[rows[r]];
      double az = z[0] < 0.0 ? -z[0] : z[0];
      double sp = (z[0] > 0.0 ? z[0] : 0.0) + log1p(exp(-az));
      total += rnd(sp - yr * z[0], prec);
      if (want_delta) {
        double p = rnd(1.0 / (1.0 + exp(-z[0])), prec);
        double g = rnd(p - yr, prec);
        dl[0] = opnd(rnd(g / (double)m, prec), D->dtype); /* BF: deltas */
      }
    } else {
      double yr = (double)((const float*)D->y)[rows[r]];
      double e = rnd(z[0] - yr, prec);
      total += (half_sq ? 0.5 : 1.0) * e * e;
      if (want_delta) dl[0] = opnd(rnd(e / (double)m, prec), D->dtype); /* BF: deltas */
    }
  }
  return m > 0 ? rnd(total / (double)m, prec) : NAN;
}

/* Training loss (data loss + L2 penalty) and its gradient on one minibatch. */
static double loss_grad(const net_t* net, const data_t* D, const int32_t* rows, int64_t m,
                        const double* theta, double alpha, double* grad, scratch_t* s,
                        int prec, double* data_part) {
  int dt = D->dtype;
  forward(net, D, rows, m, theta, s, prec);
  double loss = data_loss(net, D, rows, m, s, prec, 1, 1);
  if (data_part) *data_part = loss;
  double pen = 0.0;
  for (int l = 0; l < net->L; l++) {
    const double* W = theta + net->w_off[l];
    int64_t cnt = (int64_t)net->dims[l] * net->dims[l + 1];
    for (int64_t i = 0; i < cnt; i++) pen += W[i] * W[i];
  }
  loss = rnd(loss + rnd(0.5 * alpha * pen / (double)m, prec), prec);

  for (int l = net->L - 1; l >= 0; l--) {
    int fi = net->dims[l], fo = net->dims[l + 1];
    const double* dl = s->delta[l + 1];
    const double* W = theta + net->w_off[l];
    const double* Wop = s->wop + net->w_off[l];
    double* gW = grad + net->w_off[l];
    double* gb = grad + net->b_off[l];
    double am = alpha / (double)m;
    for (int k = 0; k < fi; k++)
      for (int j = 0; j < fo; j++) {
        double acc = 0.0;
        for (int64_t r = 0; r < m; r++) acc = accum(acc, s->a[l][r * fi + k] * dl[r * fo + j], prec);
        gW[(int64_t)k * fo + j] = rnd(acc + am * W[(int64_t)k * fo + j], prec);
      }
    for (int j = 0; j < fo; j++) {
      double acc = 0.0;
      for (int64_t r = 0; r < m; r++) acc = accum(acc, dl[r * fo + j], prec);
      gb[j] = rnd(acc, prec);
    }
    if (l > 0) {
      double* dp = s->delta[l];
      for (int64_t r = 0; r < m; r++)
        for (int k = 0; k < fi; k++) {
          double v = 0.0;
          if (s->a[l][r * fi + k] > 0.0) {
            double acc = 0.0;
            for (int j = 0; j < fo; j++) acc = accum(acc, dl[r * fo + j] * Wop[(int64_t)k * fo + j], prec);
            v = opnd(rnd(acc, prec), dt); /* BF: deltas */
          }
          dp[r * fi + k] = v;
        }
    }
  }
  return loss;
}

/* Public wrapper used by the gradient pins: params and grads are packed
 * W[in][out], b[out] per layer. */
int oracle_loss_grad(const void* X, const void* y, int64_t n, int32_t d, int32_t n_classes,
                     const int32_t* rows, int64_t m, const oracle_hparams* hp,
                     const double* theta, int32_t dtype, int32_t prec, double* loss_out,
                     double* grad_out) {
  net_t net;
  if (net_build(&net, d, n_classes, hp)) return -1;
  data_t D = {X, y, n, d, dtype};
  scratch_t s;
  if (scratch_alloc(&s, &net, m)) return -2;
  *loss_out = loss_grad(&net, &D, rows, m, theta, (double)hp->alpha, grad_out, &s, prec, NULL);
  scratch_free(&s, &net);
  return 0;
}

/* ------------------------------------------------------------------ */
/* optimizers                                                          */
/* ------------------------------------------------------------------ */

typedef struct {
  double *m, *v; /* adam moments, or m = sgd velocity */
  int64_t t;
} opt_t;

static void adam_step(const oracle_hparams* hp, int64_t P, double* theta, const double* g,
                      opt_t* o, int prec) {
  double b1 = hp->beta1, b2 = hp->beta2, lr = hp->lr, eps = hp->eps;
  o->t += 1;
  double lr_t = rnd(lr * sqrt(1.0 - pow(b2, (double)o->t)) / (1.0 - pow(b1, (double)o->t)), prec);
  double omb1 = rnd(1.0 - b1, prec), omb2 = rnd(1.0 - b2, prec);
  for (int64_t i = 0; i < P; i++) {
    o->m[i] = rnd(rnd(b1 * o->m[i], prec) + rnd(omb1 * g[i], prec), prec);
    o->v[i] = rnd(rnd(b2 * o->v[i], prec) + rnd(omb2 * rnd(g[i] * g[i], prec), prec), prec);
    double den = rnd(rnd(sqrt(o->v[i]), prec) + eps, prec);
    theta[i] = rnd(theta[i] - rnd(rnd(lr_t * o->m[i], prec) / den, prec), prec);
  }
}

static void sgd_step(const oracle_hparams* hp, double lr, int64_t P, double* theta, const double* g,
                     opt_t* o, int prec) {
  double mu = hp->momentum;
  for (int64_t i = 0; i < P; i++) {
    double u = rnd(rnd(mu * o->m[i], prec) - rnd(lr * g[i], prec), prec);
    o->m[i] = u;
    if (hp->nesterov)
      theta[i] = rnd(theta[i] + rnd(rnd(mu * u, prec) - rnd(lr * g[i], prec), prec), prec);
    else
      theta[i] = rnd(theta[i] + u, prec);
  }
}

/* Public single-step wrappers for the optimizer pins. */
int oracle_opt_step(const oracle_hparams* hp, int64_t P, double* theta, const double* g,
                    double* m, double* v, int64_t* t, int32_t prec) {
  opt_t o = {m, v, *t};
  if (hp->solver == 0)
    adam_step(hp, P, theta, g, &o, prec);
  else {
    sgd_step(hp, (double)hp->lr, P, theta, g, &o, prec);
    o.t += 1;
  }
  *t = o.t;
  return 0;
}

/* ------------------------------------------------------------------ */
/* fold lists, minibatch rows                                          */
/* ------------------------------------------------------------------ */

/* Ascending lists of the rows that train (fold_idx not in {f, negative}) and
 * validate (fold_idx == f) for fold f.  f < 0 is the hold-out split of the
 * generalization score (Section 6.2, Figure 2(b)): every row that belongs to a
 * fold trains, the rows outside all folds (fold_idx < 0) are scored.  Returns
 * counts through n_tr / n_va.  Either output list may be NULL to only count. */
void oracle_fold_lists(const int32_t* fold_idx, int64_t n, int32_t f, int32_t* train,
                       int32_t* val, int64_t* n_tr, int64_t* n_va) {
  int64_t a = 0, b = 0;
  for (int64_t i = 0; i < n; i++) {
    if (fold_idx[i] < 0 && f >= 0) continue;
    if (f >= 0 ? fold_idx[i] == f : fold_idx[i] < 0) {
      if (val) val[b] = (int32_t)i;
      b++;
    } else {
      if (train) train[a] = (int32_t)i;
      a++;
    }
  }
  *n_tr = a;
  *n_va = b;
}

static int64_t eff_batch(const oracle_hparams* hp, int64_t n_tr) {
  int64_t bs = hp->batch_size;
  if (bs <= 0 || bs > n_tr) bs = n_tr;
  return bs;
}

/* Early stopping on a validation fraction (the scikit-learn-style option the benchmark's MLP-adam / MLP-sgd
 * of Table 1 are tuned with).  Active when n_iter_no_change > 0 and validation_fraction > 0 and the fold has
 * at least two training rows.  The fold's ascending training list is cut by a keyed bijection of its own
 * (key = model key folded with 2): list[pi_split(p)] for p < n_fit are the rows the model is fitted on, in
 * that order; p >= n_fit are the n_hold = floor(fraction * n_train) rows (at least 1, at most n_train - 1)
 * it never trains on.  After every epoch the held rows' loss is taken; the parameters of the epoch with the
 * lowest loss so far are kept aside, and when training ends (by the rule or by reaching `epochs`) they are
 * the model that is scored, as scikit-learn-style early stopping hands back its best iterate.
 * Returns n_hold (0: the rule is off). */
static int64_t hold_count(const oracle_hparams* hp, int64_t n_tr) {
  if (hp->n_iter_no_change <= 0 || !(hp->validation_fraction > 0.0f) || n_tr < 2) return 0;
  int64_t h = (int64_t)floor((double)hp->validation_fraction * (double)n_tr);
  if (h < 1) h = 1;
  if (h > n_tr - 1) h = n_tr - 1;
  return h;
}

static uint64_t split_key(uint64_t seed, int fold) { return oracle_combine(model_key(seed, fold), 2); }

/* Index into the fold's training list of position p of epoch `key`'s order over the fitted rows. */
static int64_t fit_index(const oracle_hparams* hp, int fold, uint64_t key, int64_t n_tr, int64_t n_hold, int64_t p) {
  int64_t q = perm_index(key, n_tr - n_hold, p);
  return n_hold ? perm_index(split_key(hp->seed, fold), n_tr, q) : q;
}

/* The rows set aside for early stopping of fold f's model (empty when the rule is off); returns the count. */
int64_t oracle_early_stop_rows(const int32_t* fold_idx, int64_t n, const oracle_hparams* hp, int32_t f,
                               int32_t* rows_out) {
  int32_t* tr = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
  int64_t n_tr, n_va;
  oracle_fold_lists(fold_idx, n, f, tr, NULL, &n_tr, &n_va);
  int64_t n_hold = hold_count(hp, n_tr), n_fit = n_tr - n_hold;
  for (int64_t i = 0; i < n_hold; i++) rows_out[i] = tr[perm_index(split_key(hp->seed, f), n_tr, n_fit + i)];
  free(tr);
  return n_hold;
}

/* Rows of minibatch `step` of `epoch` for fold f; returns the row count. */
int64_t oracle_minibatch_rows(const int32_t* fold_idx, int64_t n, const oracle_hparams* hp,
                              int32_t f, int32_t epoch, int64_t step, int32_t* rows_out) {
  int32_t* tr = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
  int64_t n_tr, n_va;
  oracle_fold_lists(fold_idx, n, f, tr, NULL, &n_tr, &n_va);
  int64_t n_hold = hold_count(hp, n_tr), n_fit = n_tr - n_hold;
  int64_t bs = eff_batch(hp, n_fit);
  int64_t lo = step * bs, hi = lo + bs > n_fit ? n_fit : lo + bs, cnt = 0;
  uint64_t key = epoch_key(hp->seed, f, epoch);
  for (int64_t p = lo; p < hi; p++) rows_out[cnt++] = tr[fit_index(hp, f, key, n_tr, n_hold, p)];
  free(tr);
  return cnt;
}

/* ------------------------------------------------------------------ */
/* one model: train on a fold's training rows, score on its held rows  */
/* ------------------------------------------------------------------ */

typedef struct {
  int64_t step_begin, step_end; /* global step window, [begin, end) */
  double* out;                  /* per step: loss, grad[P], theta_after[P], m_after[P], v_after[P] */
  int stop_after;               /* stop training once the window is recorded */
} trace_t;

static int train_and_score(const net_t* net, const data_t* D, const oracle_hparams* hp, int fold,
                           const int32_t* tr, int64_t n_tr, const int32_t* va, int64_t n_va,
                           int prec, double out[2], trace_t* trace, double* theta_out) {
  int64_t P = net->P;
  int64_t n_hold = hold_count(hp, n_tr), n_fit = n_tr - n_hold;
  int64_t bs = eff_batch(hp, n_fit);
  int64_t max_rows = bs > n_va ? bs : n_va;
  if (n_hold > max_rows) max_rows = n_hold;
  scratch_t s;
  double* theta = (double*)malloc(sizeof(double) * (size_t)P * 5);
  int32_t* rows = (int32_t*)malloc(sizeof(int32_t) * (size_t)(bs > 0 ? bs : 1));
  int32_t* held = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n_hold > 0 ? n_hold : 1));
  if (!theta || !rows || !held || scratch_alloc(&s, net, max_rows)) return -2;
  for (int64_t i = 0; i < n_hold; i++) held[i] = tr[perm_index(split_key(hp->seed, fold), n_tr, n_fit + i)];
  double *grad = theta + P, *m = theta + 2 * P, *v = theta + 3 * P, *theta_best = theta + 4 * P;
  int have_best = 0;
  memset(grad, 0, sizeof(double) * (size_t)P * 3);
  opt_t o = {m, v, 0};
  init_params(net, hp->seed, fold, theta);

  int64_t steps = n_fit > 0 ? (n_fit + bs - 1) / bs : 0, gstep = 0;
  int done = 0, stalled = 0, stop = 0;
  float best = INFINITY;
  for (int e = 0; e < hp->epochs && !done && !stop; e++) {
    uint64_t key = epoch_key(hp->seed, fold, e);
    /* inverse-scaling schedule of the sgd solver: the rate falls with the rows seen before the epoch */
    double lr_e = (double)hp->lr;
    if (hp->solver != 0 && hp->power_t != 0.0f)
      lr_e = rnd(lr_e / pow(1.0 + (double)e * (double)n_fit, (double)hp->power_t), prec);
    double esum = 0.0;
    for (int64_t st = 0; st < steps && !done; st++, gstep++) {
      int64_t lo = st * bs, hi = lo + bs > n_fit ? n_fit : lo + bs, mb = hi - lo;
      for (int64_t p = lo; p < hi; p++) rows[p - lo] = tr[fit_index(hp, fold, key, n_tr, n_hold, p)];
      double data = 0.0;
      double loss = loss_grad(net, D, rows, mb, theta, (double)hp->alpha, grad, &s, prec, &data);
      esum += data * (double)mb;
      if (hp->solver == 0)
        adam_step(hp, P, theta, grad, &o, prec);
      else
        sgd_step(hp, lr_e, P, theta, grad, &o, prec);
      if (trace && gstep >= trace->step_begin && gstep < trace->step_end) {
        double* rec = trace->out + (gstep - trace->step_begin) * (1 + 4 * P);
        rec[0] = loss;
        memcpy(rec + 1, grad, sizeof(double) * (size_t)P);
        memcpy(rec + 1 + P, theta, sizeof(double) * (size_t)P);
        memcpy(rec + 1 + 2 * P, m, sizeof(double) * (size_t)P);
        memcpy(rec + 1 + 3 * P, v, sizeof(double) * (size_t)P);
        if (trace->stop_after && gstep + 1 == trace->step_end) done = 1;
      }
    }
    /* stopping rule, decided in single precision: without a validation fraction it watches the epoch's mean
     * data loss over the steps just taken; with one, the loss of the rows set aside (the same loss the final
     * score reports: cross-entropy, or the plain mean squared error), under the weights the epoch ends with */
    if (hp->n_iter_no_change > 0 && steps > 0 && !done) {
      float le = (float)(esum / (double)n_fit);
      if (n_hold > 0) {
        forward(net, D, held, n_hold, theta, &s, prec);
        le = (float)data_loss(net, D, held, n_hold, &s, prec, 0, 0);
      }
      stalled = le > best - hp->tol ? stalled + 1 : 0;
      if (le < best) {
        best = le;
        if (n_hold > 0) { /* the best iterate so far on the held rows */
          memcpy(theta_best, theta, sizeof(double) * (size_t)P);
          have_best = 1;
        }
      }
      if (stalled > hp->n_iter_no_change) stop = 1;
    }
  }
  if (have_best && !done) memcpy(theta, theta_best, sizeof(double) * (size_t)P);

  out[0] = NAN;
  out[1] = NAN;
  if (n_va > 0 && !done) {
    forward(net, D, va, n_va, theta, &s, prec);
    out[0] = data_loss(net, D, va, n_va, &s, prec, 0, 0);
    if (net->n_classes >= 2) {
      int c = net->dims[net->L];
      int64_t hit = 0;
      for (int64_t r = 0; r < n_va; r++) {
        const double* z = s.a[net->L] + r * c;
        int best = 0;
        for (int j = 1; j < c; j++)
          if (z[j] > z[best]) best = j;
        hit += best == ((const int32_t*)D->y)[va[r]];
      }
      out[1] = rnd((double)hit / (double)n_va, prec);
    } else if (net->n_classes == 1) {
      int64_t hit = 0;
      for (int64_t r = 0; r < n_va; r++)
        hit += (s.a[net->L][r] > 0.0 ? 1 : 0) == ((const int32_t*)D->y)[va[r]];
      out[1] = rnd((double)hit / (double)n_va, prec);
    } else {
      /* mean absolute error, the other regression metric of Section 2 */
      double sa = 0.0;
      for (int64_t r = 0; r < n_va; r++)
        sa += fabs(s.a[net->L][r] - (double)((const float*)D->y)[va[r]]);
      out[1] = rnd(sa / (double)n_va, prec);
    }
  }
  if (theta_out) memcpy(theta_out, theta, sizeof(double) * (size_t)P);
  scratch_free(&s, net);
  free(theta);
  free(rows);
  free(held);
  return 0;
}

/* Train one (suggestion, fold) model; optionally record a window of steps
 * and/or return the final parameters and the fold's two scores. */
int oracle_train_one(const void* X, const void* y, int64_t n, int32_t d, int32_t n_classes,
                     const int32_t* fold_idx, const oracle_hparams* hp, int32_t fold,
                     int32_t dtype, int32_t prec, int64_t step_begin, int64_t step_end,
                     int32_t stop_after, double* trace_out, double* theta_out,
                     double* score_out) {
  net_t net;
  if (net_build(&net, d, n_classes, hp)) return -1;
  data_t D = {X, y, n, d, dtype};
  int32_t* tr = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1) * 2);
  int32_t* va = tr + (n > 0 ? n : 1);
  int64_t n_tr, n_va;
  oracle_fold_lists(fold_idx, n, fold, tr, va, &n_tr, &n_va);
  trace_t trc = {step_begin, step_end, trace_out, stop_after};
  double sc[2];
  int rc = train_and_score(&net, &D, hp, fold, tr, n_tr, va, n_va, prec, sc,
                           trace_out ? &trc : NULL, theta_out);
  if (score_out) {
    score_out[0] = sc[0];
    score_out[1] = sc[1];
  }
  free(tr);
  return rc;
}

/* The evaluation call: B suggestions x n_folds folds.  scores[B][2] =
 * {mean nll | mse, mean acc | mae}; status[b] = 1 when the first score is not
 * finite; per_fold (optional) [B][n_folds][2].  Models run one per OpenMP
 * thread. */
int oracle_mlp_cv_eval(const void* X, const void* y, int64_t n, int32_t d, int32_t n_classes,
                       const int32_t* fold_idx, int32_t n_folds, const oracle_hparams* hp,
                       int32_t B, int32_t dtype, int32_t prec, float* scores, int32_t* status,
                       double* per_fold, int32_t n_threads) {
  if (n < 0 || d < 1 || n_folds < 1 || B < 0 || n_classes < 0) return -1;
  for (int b = 0; b < B; b++) {
    net_t net;
    if (net_build(&net, d, n_classes, &hp[b])) return -1;
  }
  int64_t nn = n > 0 ? n : 1;
  int32_t* lists = (int32_t*)malloc(sizeof(int32_t) * (size_t)nn * 2 * n_folds);
  int64_t* cnt = (int64_t*)malloc(sizeof(int64_t) * 2 * n_folds);
  double* pf = (double*)malloc(sizeof(double) * 2 * (size_t)(B > 0 ? B : 1) * n_folds);
  for (int f = 0; f < n_folds; f++)
    oracle_fold_lists(fold_idx, n, f, lists + (int64_t)2 * f * nn, lists + ((int64_t)2 * f + 1) * nn,
                      &cnt[2 * f], &cnt[2 * f + 1]);
  data_t D = {X, y, n, d, dtype};
  int err = 0;
  int64_t items = (int64_t)B * n_folds;
  if (n_threads < 1) n_threads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(n_threads)
  for (int64_t it = 0; it < items; it++) {
    int b = (int)(it / n_folds), f = (int)(it % n_folds);
    net_t net;
    net_build(&net, d, n_classes, &hp[b]);
    int rc = train_and_score(&net, &D, &hp[b], f, lists + (int64_t)2 * f * nn, cnt[2 * f],
                             lists + ((int64_t)2 * f + 1) * nn, cnt[2 * f + 1], prec,
                             pf + 2 * it, NULL, NULL);
    if (rc) {
#pragma omp atomic write
      err = rc;
    }
  }
  for (int b = 0; b < B; b++) {
    double s0 = 0.0, s1 = 0.0;
    for (int f = 0; f < n_folds; f++) {
      s0 += pf[2 * ((int64_t)b * n_folds + f)];
      s1 += pf[2 * ((int64_t)b * n_folds + f) + 1];
    }
    scores[2 * b] = (float)(s0 / n_folds);
    scores[2 * b + 1] = (float)(s1 / n_folds);
    status[b] = isfinite(scores[2 * b]) ? 0 : 1;
  }
  if (per_fold) memcpy(per_fold, pf, sizeof(double) * 2 * (size_t)items);
  free(lists);
  free(cnt);
  free(pf);
  return err;
}

/* The hold-out (generalization) score of Section 6.2: each suggestion is
 * trained once on all rows that belong to a fold and scored on the rows that
 * belong to none (fold_idx < 0).  The model is keyed as fold -1, so it shares
 * no random stream with the cross-validation models of the same suggestion.
 * scores[B][2] = {nll | mse, acc | mae}; status[b] = 1 when the first score is
 * not finite. */
int oracle_mlp_holdout_eval(const void* X, const void* y, int64_t n, int32_t d, int32_t n_classes,
                            const int32_t* fold_idx, const oracle_hparams* hp, int32_t B,
                            int32_t dtype, int32_t prec, float* scores, int32_t* status,
                            int32_t n_threads) {
  if (n < 0 || d < 1 || B < 0 || n_classes < 0) return -1;
  for (int b = 0; b < B; b++) {
    net_t net;
    if (net_build(&net, d, n_classes, &hp[b])) return -1;
  }
  int64_t nn = n > 0 ? n : 1;
  int32_t* lists = (int32_t*)malloc(sizeof(int32_t) * (size_t)nn * 2);
  int64_t n_tr, n_va;
  oracle_fold_lists(fold_idx, n, -1, lists, lists + nn, &n_tr, &n_va);
  data_t D = {X, y, n, d, dtype};
  int err = 0;
  if (n_threads < 1) n_threads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(n_threads)
  for (int b = 0; b < B; b++) {
    net_t net;
    net_build(&net, d, n_classes, &hp[b]);
    double sc[2];
    int rc = train_and_score(&net, &D, &hp[b], -1, lists, n_tr, lists + nn, n_va, prec, sc, NULL, NULL);
    scores[2 * b] = (float)sc[0];
    scores[2 * b + 1] = (float)sc[1];
    status[b] = isfinite(scores[2 * b]) ? 0 : 1;
    if (rc) {
#pragma omp atomic write
      err = rc;
    }
  }
  free(lists);
  return err;
}
