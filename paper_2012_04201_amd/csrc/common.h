// Shared declarations of the evaluator's kernels: counter-based random
// numbers, item descriptors, kernel parameters and small device helpers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/bbo_mlp.h"

namespace {

constexpr int MAXL = BBO_MAX_HIDDEN + 1;  // weight layers
constexpr int NTHREADS = 256;
constexpr uint64_t GOLDEN = 0x9E3779B97F4A7C15ull;

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------
// Counter-based random numbers: SplitMix64 output mixer over (key, counter).
// ---------------------------------------------------------------------------
__host__ __device__ inline uint64_t mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
__host__ __device__ inline uint64_t key_fold(uint64_t h, uint64_t v) { return mix64(h + (v + 1) * GOLDEN); }
__host__ __device__ inline uint64_t key_model(uint64_t seed, int fold) {
  return key_fold(key_fold(seed, 0x4D4C50ull), (uint64_t)fold);
}
__host__ __device__ inline uint64_t key_epoch(uint64_t kmodel, int epoch) {
  return key_fold(key_fold(kmodel, 1), (uint64_t)epoch);
}

// Position p of an epoch -> index into the fold's training list: 4-round
// balanced Feistel permutation on an even number of bits, cycle-walked into
// [0, n).
__device__ inline uint32_t perm_index(uint64_t key, uint32_t n, uint32_t p) {
  if (n <= 1) return 0;
  int bits = 32 - __builtin_clz(n - 1);
  bits += bits & 1;
  if (bits < 2) bits = 2;
  const int hb = bits >> 1;
  const uint32_t mask = (1u << hb) - 1;
  uint32_t x = p;
  do {
    uint32_t Lh = x >> hb, Rh = x & mask;
#pragma unroll
    for (uint32_t r = 0; r < 4; r++) {
      uint32_t F = (uint32_t)key_fold(key, ((uint64_t)r << 32) | Rh) & mask;
      uint32_t t = Lh ^ F;
      Lh = Rh;
      Rh = t;
    }
    x = (Lh << hb) | Rh;
  } while (x >= n);
  return x;
}

// Early stopping on a validation fraction: the fold's ascending training list is cut by a keyed bijection of
// its own (key = model key folded with 2): list[pi_split(p)], p < n_fit, are the rows the model is fitted on,
// in that order; p >= n_fit are the n_hold = floor(fraction * n_train) rows (at least 1, at most n_train - 1)
// it never trains on and whose loss the stopping rule watches.  n_hold = 0: no cut.
struct RowSplit {
  uint64_t ksplit;
  int n_tr, n_fit, n_hold;
};
__device__ inline RowSplit row_split(uint64_t kmodel, int patience, float frac, int n_tr) {
  RowSplit s{key_fold(kmodel, 2), n_tr, n_tr, 0};
  if (patience > 0 && frac > 0.f && n_tr >= 2) {
    int h = (int)floor((double)frac * (double)n_tr);
    h = h < 1 ? 1 : h;
    h = h > n_tr - 1 ? n_tr - 1 : h;
    s.n_hold = h;
    s.n_fit = n_tr - h;
  }
  return s;
}
// index into the training list of position p of the epoch whose key is ke
__device__ inline uint32_t fit_index(const RowSplit& s, uint64_t ke, uint32_t p) {
  const uint32_t q = perm_index(ke, (uint32_t)s.n_fit, p);
  return s.n_hold ? perm_index(s.ksplit, (uint32_t)s.n_tr, q) : q;
}
// index into the training list of the i-th row set aside
__device__ inline uint32_t held_index(const RowSplit& s, uint32_t i) {
  return perm_index(s.ksplit, (uint32_t)s.n_tr, (uint32_t)s.n_fit + i);
}
// Which rows a pass works on: the positions of a training epoch, the rows set aside, or a list as it stands.
enum RowMode { ROWS_EPOCH = 0, ROWS_HELD = 1, ROWS_PLAIN = 2 };
__device__ inline uint32_t row_index(const RowSplit& s, int mode, uint64_t ke, uint32_t p) {
  return mode == ROWS_EPOCH ? fit_index(s, ke, p) : (mode == ROWS_HELD ? held_index(s, p) : p);
}

// The permutation's domain for callers that walk many positions at once with a table of the
// round function (which sees the round and one half of the position only): n >= 2.
struct PermDomain {
  int hb;
  uint32_t mask;
};
__device__ inline PermDomain perm_domain(uint32_t n) {
  int bits = 32 - __builtin_clz(n - 1);
  bits += bits & 1;
  if (bits < 2) bits = 2;
  return PermDomain{bits >> 1, (1u << (bits >> 1)) - 1};
}

// ---------------------------------------------------------------------------
// Item description and per-item memory layout
// ---------------------------------------------------------------------------
struct ItemDesc {
  uint64_t seed;
  int32_t b, fold, L, solver, nesterov, batch_size, epochs, rows_cap;
  float lr, alpha, momentum, beta1, beta2, eps;
  float power_t, tol;
  int32_t patience;
  float val_frac;  // early stopping on held-out rows when > 0 (and patience > 0)
  int32_t dims[MAXL + 1];
  float bound[MAXL];
};

__host__ __device__ inline int rup(int x, int m) { return (x + m - 1) / m * m; }

struct Layout {
  int32_t L, rows;
  int32_t dims[MAXL + 1];
  int32_t ld[MAXL + 1];    // row length of W_l ([out][ld]): roundup(dims+1, kstep)
  int32_t kp[MAXL + 1];    // dims rounded up to the K step
  int32_t p16[MAXL + 1];   // dims rounded up to 16
  int32_t p16a[MAXL + 1];  // dims+1 rounded up to 16
  int32_t cw[MAXL], cb[MAXL];  // offsets in the packed W[in][out], b[out] order
  int32_t P;
  uint64_t w[MAXL], m[MAXL], v[MAXL], oi[MAXL], io[MAXL], best[MAXL];
  uint64_t A[MAXL], AT[MAXL], D[MAXL + 1], DT[MAXL + 1], Z, rowlist, total;
};

// Byte offsets of everything one item keeps in its slot.  Used by the host to
// size slots and by the device to address them.
__host__ __device__ inline void make_layout(Layout& y, const int32_t* dims, int L, int rows, int kstep,
                                            int opsz) {
  y.L = L;
  y.rows = rows;
  int c = 0;
  for (int l = 0; l <= L; l++) {
    y.dims[l] = dims[l];
    y.ld[l] = rup(dims[l] + 1, kstep);
    y.kp[l] = rup(dims[l], kstep);
    y.p16[l] = rup(dims[l], 16);
    y.p16a[l] = rup(dims[l] + 1, 16);
  }
  for (int l = 0; l < L; l++) {
    y.cw[l] = c;
    c += dims[l] * dims[l + 1];
    y.cb[l] = c;
    c += dims[l + 1];
  }
  y.P = c;
  uint64_t off = 0;
  auto take = [&](uint64_t bytes) {
    uint64_t o = off;
    off += (bytes + 255) & ~(uint64_t)255;
    return o;
  };
  for (int l = 0; l < L; l++) {
    uint64_t wn = (uint64_t)y.p16[l + 1] * y.ld[l];
    y.w[l] = take(wn * 4);
    y.m[l] = take(wn * 4);
    y.v[l] = take(wn * 4);
    y.best[l] = take(wn * 4);  // the parameters of the best epoch so far under early stopping on held-out rows
    y.oi[l] = opsz == 4 ? y.w[l] : take(wn * opsz);
    y.io[l] = l >= 1 ? take((uint64_t)y.p16[l] * y.kp[l + 1] * opsz) : 0;
    y.A[l] = take((uint64_t)rows * y.kp[l] * opsz);
    y.AT[l] = take((uint64_t)y.p16a[l] * rows * opsz);
  }
  y.D[0] = y.DT[0] = 0;
  for (int l = 1; l <= L; l++) {
    y.D[l] = take((uint64_t)rows * y.kp[l] * opsz);
    y.DT[l] = take((uint64_t)y.p16[l] * rows * opsz);
  }
  y.Z = take((uint64_t)rows * y.p16[L] * 4);
  y.rowlist = take((uint64_t)rows * 4);
  y.total = off;
}

struct TrainParams {
  const void* X;
  const void* y;
  const int32_t* train_idx;
  const int32_t* val_idx;
  const int32_t* counts;
  const void* items;  // ItemDesc[] (generic kernel) or TItem[] (tiled kernel), most expensive first
  int32_t* queue;
  float* item_out;  // [B*K][2]
  char* slots;
  uint64_t slot_bytes;
  int64_t n;
  int32_t d, n_classes, n_folds, n_items;
  int32_t fold_base;  // fold of list 0: 0 for cross-validation, -1 for the hold-out split
  // trace
  int32_t trace_item;  // b*K+fold or -1
  int64_t step_begin, step_end;
  float* trace_out;
  const float* state_in;  // optional [3P]: parameters, m, v of the traced item before step_begin
  int32_t x_bf16;         // wavefront-per-model kernel: X holds bfloat16 and the products take bfloat16 operands
};

__device__ inline double block_sum(double v, double* red) {
  for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if (lane == 0) red[wave] = v;
  __syncthreads();
  double t = 0.0;
  for (int w = 0; w < nw; w++) t += red[w];
  return t;
}


__device__ inline int eff_batch(int bs, int n_tr) { return (bs <= 0 || bs > n_tr) ? n_tr : bs; }

// Inverse-scaling schedule of the SGD solver: the rate of epoch e is lr / (1 + e * n_tr)^power_t
// (n_tr rows seen per epoch); single-precision exp2 / log2, a few 1e-6 relative.
__device__ inline float epoch_lr(float lr, float power_t, int e, int n_tr) {
  if (power_t == 0.f) return lr;
  return lr * exp2f(-power_t * log2f(1.f + (float)e * (float)n_tr));
}

// Plateau stop: the epoch's mean data loss against the best so far, decided in single precision.
struct Plateau {
  float best = INFINITY;
  int stalled = 0;
  bool improved = false;  // the last loss given was the lowest so far
  __device__ bool stop_after(float epoch_loss, float tol, int patience) {
    stalled = epoch_loss > best - tol ? stalled + 1 : 0;
    improved = epoch_loss < best;
    if (improved) best = epoch_loss;
    return stalled > patience;
  }
};

}  // namespace
