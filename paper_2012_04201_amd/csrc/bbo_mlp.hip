// Batched MLP cross-validation evaluator for MI355X (gfx950): HIP kernels and
// the C ABI declared in include/bbo_mlp.h.
//
// One call = evaluate(params_list) of the paper's Algorithm 1: every
// (suggestion, fold) pair is one small MLP ("item").  Items are sorted by
// estimated cost and pulled from a device-side queue by persistent
// workgroups; each workgroup trains its item for all epochs and scores it on
// the held fold without returning to the host.  Every contraction (forward,
// data gradient, weight gradient) runs on MFMA with fp32 accumulation; the
// optimizer update is fused into the weight-gradient epilogue, so the weight
// gradient is never stored.  (Models without a hidden layer are the exception:
// a wavefront each, on the vector ALU; see train_linear_f32.h.)
//
// Five training kernels share this scheme: the LDS-tiled bf16 kernel
// (train_tiled_bf16.h), the two LDS-resident fp32 kernels (train_small_f32.h,
// train_mid_f32.h), the wavefront-per-model fp32 kernel (train_linear_f32.h)
// and the generic kernel below, which takes every shape the header admits.  The planner gives each
// suggestion to the fastest kernel that takes its shape and launches every
// kernel that got items, one after the other, each with its own item array
// and queue counter.
//
// Operand layout.  MFMA operands are read straight from memory as 16-byte
// vectors along the contracted index, so every tensor is kept in the layout
// (or layouts) in which each of its consumers contracts it:
//   activations a_l, deltas d_l : row-major [row][unit]   (contract over units)
//                                 unit-major [unit][row]  (contract over rows)
//   weights W_l                 : [out][in+1] fp32 master with the bias in
//                                 column `in`, moments alike; operand copies
//                                 [out][in] and [in][out] in the GEMM dtype.
// All leading dimensions are padded with zeros to the MFMA K step, so the
// inner loops carry no bounds checks.  The unit-major activations carry one
// extra unit that is 1 on real rows: the weight-gradient GEMM then yields the
// bias gradient in the same pass.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <cmath>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/bbo_mlp.h"

#include "common.h"
#include "train_tiled_bf16.h"
#include "train_small_f32.h"
#include "train_mid_f32.h"
#include "train_linear_f32.h"

static_assert(sizeof(bbo_mlp_hparams) == 88, "the hyper-parameter record is part of the ABI");

// Workspace of bbo_mlp_cv_eval_static: device memory that exists from the moment the library is loaded, for
// callers that cannot allocate.  In host code the name is only a handle for hipGetSymbolAddress; the address
// the kernels get is the one that call returns (scratch_address()).  One copy per device, shared by every
// call on that device, contents left over from the last call.
static __device__ __align__(256) unsigned char scratch[BBO_STATIC_SCRATCH_BYTES];

namespace {

// ---------------------------------------------------------------------------
// Operand types
// ---------------------------------------------------------------------------
template <typename OpT>
struct Op;
template <>
struct Op<float> {
  static constexpr int KSTEP = 16, VEC = 4;
  typedef f32x4 vec;
  typedef f32x4 vec4;  // four consecutive elements
  __device__ static inline f32x4 mfma(const vec& a, const vec& b, f32x4 c) {
#pragma unroll
    for (int e = 0; e < 4; e++) c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[e], b[e], c, 0, 0, 0);
    return c;
  }
  __device__ static inline float cvt(float x) { return x; }
};
template <>
struct Op<__bf16> {
  static constexpr int KSTEP = 32, VEC = 8;
  typedef bf16x8 vec;
  typedef bf16x4 vec4;
  __device__ static inline f32x4 mfma(const vec& a, const vec& b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
  }
  __device__ static inline __bf16 cvt(float x) { return (__bf16)x; }  // round to nearest even
};

// ---------------------------------------------------------------------------
// Workgroup GEMM: C[M][N] = sum_k A[m][k] * B[n][k], both operands contiguous
// along k.  Each wave owns TM x TN tiles of 16x16 and reads its operands
// directly as 16-byte vectors (lane = row/col within the tile, quarter-wave =
// k sub-block).  epi(acc, i0, j): the lane holds C[i0..i0+3][j].
// ---------------------------------------------------------------------------
template <typename OpT, int TM, int TN, typename Epi>
__device__ inline void wg_gemm_blk(const OpT* __restrict__ A, int lda, const OpT* __restrict__ B, int ldb,
                                   int Mt, int Nt, int K, Epi epi) {
  typedef Op<OpT> O;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const int li = lane & 15, q = lane >> 4;
  const int nbm = (Mt + TM - 1) / TM, nbn = (Nt + TN - 1) / TN;
  for (int blk = wave; blk < nbm * nbn; blk += nw) {
    const int bm = blk % nbm, bn = blk / nbm;
    f32x4 acc[TM][TN];
    const OpT* ap[TM];
    const OpT* bp[TN];
#pragma unroll
    for (int i = 0; i < TM; i++) {
      int t = min(bm * TM + i, Mt - 1);
      ap[i] = A + (size_t)(t * 16 + li) * lda + q * O::VEC;
#pragma unroll
      for (int j = 0; j < TN; j++) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int j = 0; j < TN; j++) {
      int t = min(bn * TN + j, Nt - 1);
      bp[j] = B + (size_t)(t * 16 + li) * ldb + q * O::VEC;
    }
    for (int k0 = 0; k0 < K; k0 += O::KSTEP) {
      typename O::vec av[TM], bv[TN];
#pragma unroll
      for (int i = 0; i < TM; i++) av[i] = *(const typename O::vec*)(ap[i] + k0);
#pragma unroll
      for (int j = 0; j < TN; j++) bv[j] = *(const typename O::vec*)(bp[j] + k0);
#pragma unroll
      for (int i = 0; i < TM; i++)
#pragma unroll
        for (int j = 0; j < TN; j++) acc[i][j] = O::mfma(av[i], bv[j], acc[i][j]);
    }
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
      for (int j = 0; j < TN; j++) {
        int tm = bm * TM + i, tn = bn * TN + j;
        if (tm < Mt && tn < Nt) epi(acc[i][j], tm * 16 + 4 * q, tn * 16 + li);
      }
  }
}

template <typename OpT, typename Epi>
__device__ inline void wg_gemm(const OpT* A, int lda, const OpT* B, int ldb, int Mt, int Nt, int K, Epi epi) {
  const int nw = blockDim.x >> 6;
  if (Mt * Nt >= 16 * nw)
    wg_gemm_blk<OpT, 4, 4>(A, lda, B, ldb, Mt, Nt, K, epi);
  else
    wg_gemm_blk<OpT, 2, 2>(A, lda, B, ldb, Mt, Nt, K, epi);
}

// Per-row loss on the outputs z[0..c): returns the row's loss (cross-entropy,
// or squared error) and whether the prediction is correct; optionally writes
// the output delta (p - onehot)/m or (z - y)/m.
template <bool WANT_DELTA>
__device__ inline float row_loss(const float* z, int c, int n_classes, const void* yv, int row, float inv_den,
                                 float* delta, float* aux) {
  if (n_classes >= 2) {
    const int yr = ((const int32_t*)yv)[row];
    float mx = z[0];
    int best = 0;
    for (int j = 1; j < c; j++)
      if (z[j] > mx) {
        mx = z[j];
        best = j;
      }
    float se = 0.f;
    for (int j = 0; j < c; j++) se += expf(z[j] - mx);
    const float lse = mx + logf(se);
    if (WANT_DELTA)
      for (int j = 0; j < c; j++) delta[j] = (expf(z[j] - lse) - (j == yr ? 1.f : 0.f)) * inv_den;
    *aux = best == yr ? 1.f : 0.f;  // a correct prediction
    return lse - (yr >= 0 && yr < c ? z[yr] : 0.f);  // a label outside [0, c) matches no class
  } else if (n_classes == 1) {
    // one logit, labels 0/1: log(1 + e^z) - y z, delta (sigmoid(z) - y)/m
    const int yr = ((const int32_t*)yv)[row];
    const float zz = z[0];
    if (WANT_DELTA) delta[0] = (1.f / (1.f + expf(-zz)) - (float)yr) * inv_den;
    *aux = (zz > 0.f) == (yr != 0) ? 1.f : 0.f;
    return fmaxf(zz, 0.f) + log1pf(expf(-fabsf(zz))) - (yr ? zz : 0.f);
  } else {
    const float e = z[0] - ((const float*)yv)[row];
    if (WANT_DELTA) delta[0] = e * inv_den;
    *aux = fabsf(e);  // the absolute error
    return e * e;
  }
}

// The training kernels.  Every suggestion of a call goes to the fastest kernel that takes its shape, so
// a suggestion's scores do not depend on which other suggestions share its call.
enum { KC_TILED = 0, KC_SMALL = 1, KC_LINEAR = 2, KC_GENERIC = 3, KC_MID = 4, KC_N = 5 };

// ---------------------------------------------------------------------------
// Fold lists (ascending), one workgroup per list; also resets the work queues.
// List k is fold fold_base + k.  Fold -1 is the hold-out split: rows of every
// fold train, rows of none are scored.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(NTHREADS) void k_fold_lists(const int32_t* __restrict__ fold_idx, int64_t n,
                                                         int32_t* __restrict__ train_idx,
                                                         int32_t* __restrict__ val_idx,
                                                         int32_t* __restrict__ counts, int32_t* queue,
                                                         int fold_base) {
  __shared__ int wtr[NTHREADS / 64], wva[NTHREADS / 64];
  __shared__ int base_tr, base_va;
  const int f = blockIdx.x, fold = (int)blockIdx.x + fold_base, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (f == 0 && tid < KC_N && queue) queue[tid] = 0;  // one work-queue counter per training kernel
  if (tid == 0) base_tr = base_va = 0;
  __syncthreads();
  for (int64_t c0 = 0; c0 < n; c0 += NTHREADS) {
    const int64_t i = c0 + tid;
    const int fi = i < n ? fold_idx[i] : -1;
    const bool tr = fi >= 0 && fi != fold, va = i < n && (fold >= 0 ? fi == fold : fi < 0);
    const uint64_t btr = __ballot(tr), bva = __ballot(va);
    const uint64_t below = ((uint64_t)1 << lane) - 1;
    if (lane == 0) {
      wtr[wave] = __popcll(btr);
      wva[wave] = __popcll(bva);
    }
    __syncthreads();
    int otr = base_tr, ova = base_va;
    for (int w = 0; w < wave; w++) {
      otr += wtr[w];
      ova += wva[w];
    }
    if (tr) train_idx[(int64_t)f * n + otr + __popcll(btr & below)] = (int32_t)i;
    if (va) val_idx[(int64_t)f * n + ova + __popcll(bva & below)] = (int32_t)i;
    __syncthreads();
    if (tid == 0) {
      for (int w = 0; w < NTHREADS / 64; w++) {
        base_tr += wtr[w];
        base_va += wva[w];
      }
    }
    __syncthreads();
  }
  if (tid == 0) {
    counts[2 * f] = base_tr;
    counts[2 * f + 1] = base_va;
  }
}


// ---------------------------------------------------------------------------
// The training / scoring kernel: persistent workgroups, one item at a time.
// ---------------------------------------------------------------------------
template <typename OpT>
struct Trainer {
  typedef Op<OpT> O;
  const TrainParams& P;
  const ItemDesc& it;
  const Layout& y;
  char* slot;
  double* red;

  __device__ OpT* op(uint64_t off) const { return (OpT*)(slot + off); }
  __device__ float* fp(uint64_t off) const { return (float*)(slot + off); }
  __device__ int32_t* rowlist() const { return (int32_t*)(slot + y.rowlist); }

  // Initial parameters: Glorot-uniform, element i of the packed W[in][out],
  // b[out] order hashed with the tensor's key.
  __device__ void init_params() const {
    const uint64_t km = key_model(it.seed, it.fold);
    for (int l = 0; l < y.L; l++) {
      const int fi = y.dims[l], fo = y.dims[l + 1], ld = y.ld[l];
      float* W = fp(y.w[l]);
      OpT* oi = op(y.oi[l]);
      OpT* io = op(y.io[l]);
      const uint64_t kw = key_fold(km, 16 + 2 * l), kb = key_fold(km, 16 + 2 * l + 1);
      const float bound = it.bound[l];
      for (int i = threadIdx.x; i < fi * fo + fo; i += blockDim.x) {
        const bool isb = i >= fi * fo;
        const int e = isb ? i - fi * fo : i;
        const uint32_t k24 = (uint32_t)(key_fold(isb ? kb : kw, (uint64_t)e) >> 40);
        const float val = bound * ((float)((int32_t)k24 - 8388608) * 0x1p-23f);
        const int k = isb ? fi : e / fo, j = isb ? e : e % fo;
        W[j * ld + k] = val;
        if (sizeof(OpT) != 4) oi[j * ld + k] = O::cvt(val);
        if (l >= 1 && !isb) io[k * y.kp[l + 1] + j] = O::cvt(val);
      }
    }
  }

  // Parameters and moments from a packed [3P] state (W[in][out], b[out] order).
  __device__ void load_state(const float* st) const {
    for (int l = 0; l < y.L; l++) {
      const int fi = y.dims[l], fo = y.dims[l + 1], ld = y.ld[l];
      float* W = fp(y.w[l]);
      float* Mo = fp(y.m[l]);
      float* Vo = fp(y.v[l]);
      OpT* oi = op(y.oi[l]);
      OpT* io = op(y.io[l]);
      for (int i = threadIdx.x; i < fi * fo + fo; i += blockDim.x) {
        const bool isb = i >= fi * fo;
        const int e = isb ? i - fi * fo : i;
        const int k = isb ? fi : e / fo, j = isb ? e : e % fo;
        const int ci = (isb ? y.cb[l] : y.cw[l]) + e;
        const float val = st[ci];
        W[j * ld + k] = val;
        Mo[j * ld + k] = st[y.P + ci];
        Vo[j * ld + k] = st[2 * y.P + ci];
        if (sizeof(OpT) != 4) oi[j * ld + k] = O::cvt(val);
        if (l >= 1 && !isb) io[k * y.kp[l + 1] + j] = O::cvt(val);
      }
    }
  }

  // Early stopping on held-out rows hands back the parameters of the best epoch: keep them aside ...
  __device__ void keep_best() const {
    for (int l = 0; l < y.L; l++) {
      const float4* W = (const float4*)fp(y.w[l]);
      float4* B = (float4*)fp(y.best[l]);
      const int n4 = y.p16[l + 1] * y.ld[l] / 4;
      for (int i = threadIdx.x; i < n4; i += blockDim.x) B[i] = W[i];
    }
    __syncthreads();
  }
  // ... and put them back, with their operand copies, before the held fold is scored.
  __device__ void restore_best() const {
    for (int l = 0; l < y.L; l++) {
      const int fi = y.dims[l], fo = y.dims[l + 1], ld = y.ld[l];
      float* W = fp(y.w[l]);
      const float* B = fp(y.best[l]);
      OpT* oi = op(y.oi[l]);
      OpT* io = op(y.io[l]);
      for (int i = threadIdx.x; i < fi * fo + fo; i += blockDim.x) {
        const bool isb = i >= fi * fo;
        const int e = isb ? i - fi * fo : i;
        const int k = isb ? fi : e / fo, j = isb ? e : e % fo;
        const float val = B[j * ld + k];
        W[j * ld + k] = val;
        if (sizeof(OpT) != 4) oi[j * ld + k] = O::cvt(val);
        if (l >= 1 && !isb) io[k * y.kp[l + 1] + j] = O::cvt(val);
      }
    }
    __syncthreads();
  }

  // Rows of this step -> row list; gather X into a_0 in both layouts; set the
  // ones unit of every unit-major activation.
  __device__ void gather(const int32_t* list, const RowSplit& sp, int mode, uint64_t key, int lo, int mb, int Mrows) const {
    int32_t* rl = rowlist();
    for (int p = threadIdx.x; p < Mrows; p += blockDim.x)
      rl[p] = p < mb ? list[row_index(sp, mode, key, (uint32_t)(lo + p))] : -1;
    __syncthreads();
    const int d = y.dims[0], kp0 = y.kp[0], p16a = y.p16a[0], rows = y.rows;
    const int CW = max(kp0, p16a);
    OpT* A0 = op(y.A[0]);
    OpT* AT0 = op(y.AT[0]);
    const OpT* X = (const OpT*)P.X;
    for (int idx = threadIdx.x; idx < Mrows * CW; idx += blockDim.x) {
      const int r = idx / CW, c = idx - r * CW;
      const int row = rl[r];
      OpT val = O::cvt(0.f);
      if (row >= 0 && c < d) val = X[(size_t)row * d + c];
      if (c < kp0) A0[r * kp0 + c] = val;
      if (c < p16a) AT0[c * rows + r] = c == d ? O::cvt(row >= 0 ? 1.f : 0.f) : val;
    }
    for (int l = 1; l < y.L; l++) {
      OpT* AT = op(y.AT[l]) + (size_t)y.dims[l] * rows;
      for (int r = threadIdx.x; r < Mrows; r += blockDim.x) AT[r] = O::cvt(r < mb ? 1.f : 0.f);
    }
    __syncthreads();
  }

  // Forward through all layers for the first Mrows rows; leaves the outputs in Z.
  __device__ void forward(int Mrows) const {
    const int rows = y.rows;
    for (int l = 0; l < y.L; l++) {
      const bool last = l + 1 == y.L;
      const float* W = fp(y.w[l]);
      const int ld = y.ld[l], fi = y.dims[l], fo = y.dims[l + 1];
      OpT* An = last ? nullptr : op(y.A[l + 1]);
      OpT* ATn = last ? nullptr : op(y.AT[l + 1]);
      float* Z = fp(y.Z);
      const int kpn = y.kp[l + 1], zc = y.p16[y.L];
      wg_gemm<OpT>(op(y.A[l]), y.kp[l], op(y.oi[l]), ld, Mrows / 16, y.p16[l + 1] / 16, y.kp[l],
                   [&](const f32x4& acc, int i0, int j) {
                     if (j >= fo) return;
                     const float bias = W[j * ld + fi];
                     if (last) {
#pragma unroll
                       for (int r = 0; r < 4; r++) Z[(i0 + r) * zc + j] = acc[r] + bias;
                     } else {
                       typename O::vec4 pk;
#pragma unroll
                       for (int r = 0; r < 4; r++) {
                         pk[r] = O::cvt(fmaxf(acc[r] + bias, 0.f));
                         An[(i0 + r) * kpn + j] = pk[r];
                       }
                       *(typename O::vec4*)(ATn + (size_t)j * rows + i0) = pk;
                     }
                   });
      __syncthreads();
    }
  }

  // Output deltas from Z for the training step; returns the block's summed data loss.
  __device__ double loss_and_delta(int mb, int Mrows) const {
    const int Lc = y.L, c = y.dims[Lc], zc = y.p16[Lc], kpL = y.kp[Lc], rows = y.rows;
    const float* Z = fp(y.Z);
    OpT* D = op(y.D[Lc]);
    OpT* DT = op(y.DT[Lc]);
    const int32_t* rl = rowlist();
    double lsum = 0.0;
    for (int r = threadIdx.x; r < Mrows; r += blockDim.x) {
      if (r < mb) {
        // deltas are written straight to memory, one class at a time
        const int row = rl[r];
        const float* z = Z + r * zc;
        if (P.n_classes >= 2) {
          const int yr = ((const int32_t*)P.y)[row];
          float mx = z[0];
          for (int j = 1; j < c; j++) mx = fmaxf(mx, z[j]);
          float se = 0.f;
          for (int j = 0; j < c; j++) se += expf(z[j] - mx);
          const float lse = mx + logf(se);
          lsum += (double)(lse - (yr >= 0 && yr < c ? z[yr] : 0.f));  // a label outside [0, c) matches no class
          for (int j = 0; j < c; j++) {
            const float g = (expf(z[j] - lse) - (j == yr ? 1.f : 0.f)) / (float)mb;
            const OpT gv = O::cvt(g);
            D[r * kpL + j] = gv;
            DT[(size_t)j * rows + r] = gv;
          }
        } else if (P.n_classes == 1) {
          const int yr = ((const int32_t*)P.y)[row];
          const float zz = z[0];
          lsum += (double)(fmaxf(zz, 0.f) + log1pf(expf(-fabsf(zz))) - (yr ? zz : 0.f));
          const OpT gv = O::cvt((1.f / (1.f + expf(-zz)) - (float)yr) / (float)mb);
          D[r * kpL] = gv;
          DT[r] = gv;
        } else {
          const float e = z[0] - ((const float*)P.y)[row];
          lsum += 0.5 * (double)e * (double)e;
          const OpT gv = O::cvt(e / (float)mb);
          D[r * kpL] = gv;
          DT[r] = gv;
        }
      } else {
        for (int j = 0; j < c; j++) {
          D[r * kpL + j] = O::cvt(0.f);
          DT[(size_t)j * rows + r] = O::cvt(0.f);
        }
      }
    }
    __syncthreads();
    return lsum;
  }

  // Deltas of the hidden layers, from the last one down.
  __device__ void backward_data(int Mrows) const {
    const int rows = y.rows;
    for (int l = y.L - 1; l >= 1; l--) {
      OpT* Dl = op(y.D[l]);
      OpT* DTl = op(y.DT[l]);
      const OpT* ATl = op(y.AT[l]);
      const int kpl = y.kp[l], fi = y.dims[l];
      wg_gemm<OpT>(op(y.D[l + 1]), y.kp[l + 1], op(y.io[l]), y.kp[l + 1], Mrows / 16, y.p16[l] / 16, y.kp[l + 1],
                   [&](const f32x4& acc, int i0, int j) {
                     if (j >= fi) return;
                     const typename O::vec4 a = *(const typename O::vec4*)(ATl + (size_t)j * rows + i0);
                     typename O::vec4 pk;
#pragma unroll
                     for (int r = 0; r < 4; r++) {
                       pk[r] = O::cvt((float)a[r] > 0.f ? acc[r] : 0.f);
                       Dl[(i0 + r) * kpl + j] = pk[r];
                     }
                     *(typename O::vec4*)(DTl + (size_t)j * rows + i0) = pk;
                   });
      __syncthreads();
    }
  }

  // Weight (and bias) gradients of every layer with the optimizer update fused
  // into the epilogue.  `rec` (or null) receives gradient and new parameters.
  __device__ void wgrad_update(int mb, int Mrows, float lr_t, float* rec) const {
    const int rows = y.rows;
    const float am = it.alpha / (float)mb;
    const bool adam = it.solver == BBO_ADAM, nest = it.nesterov != 0;
    const float b1 = it.beta1, b2 = it.beta2, eps = it.eps, mu = it.momentum, lr = lr_t;  // lr: the SGD rate
    const float omb1 = 1.f - b1, omb2 = 1.f - b2;
    for (int l = 0; l < y.L; l++) {
      float* W = fp(y.w[l]);
      float* Mo = fp(y.m[l]);
      float* Vo = fp(y.v[l]);
      OpT* oi = op(y.oi[l]);
      OpT* io = op(y.io[l]);
      const int ld = y.ld[l], fi = y.dims[l], fo = y.dims[l + 1], ldo = y.kp[l + 1];
      const int cw = y.cw[l], cb = y.cb[l], Pn = y.P;
      wg_gemm<OpT>(op(y.AT[l]), rows, op(y.DT[l + 1]), rows, y.p16a[l] / 16, y.p16[l + 1] / 16, Mrows,
                   [&](const f32x4& acc, int i0, int j) {
                     if (j >= fo || i0 > fi) return;
                     const size_t o = (size_t)j * ld + i0;
                     f32x4 w = *(const f32x4*)(W + o), m = *(const f32x4*)(Mo + o), v;
                     if (adam) v = *(const f32x4*)(Vo + o);
                     typename O::vec4 pk;
#pragma unroll
                     for (int r = 0; r < 4; r++) {
                       const int i = i0 + r;
                       if (i <= fi) {
                         const float g = i < fi ? acc[r] + am * w[r] : acc[r];
                         if (adam) {
                           m[r] = b1 * m[r] + omb1 * g;
                           v[r] = b2 * v[r] + omb2 * (g * g);
                           w[r] = w[r] - (lr_t * m[r]) / (sqrtf(v[r]) + eps);
                         } else {
                           const float u = mu * m[r] - lr * g;
                           m[r] = u;
                           w[r] = w[r] + (nest ? mu * u - lr * g : u);
                         }
                         if (rec) {
                           const int ci = i < fi ? cw + i * fo + j : cb + j;
                           rec[1 + ci] = g;
                           rec[1 + Pn + ci] = w[r];
                         }
                         if (l >= 1 && i < fi) io[(size_t)i * ldo + j] = O::cvt(w[r]);
                       }
                       pk[r] = O::cvt(w[r]);
                     }
                     *(f32x4*)(W + o) = w;
                     *(f32x4*)(Mo + o) = m;
                     if (adam) *(f32x4*)(Vo + o) = v;
                     if (sizeof(OpT) != 4) *(typename O::vec4*)(oi + o) = pk;
                   });
    }
    __syncthreads();
  }

  __device__ double penalty_sum() const {
    double s = 0.0;
    for (int l = 0; l < y.L; l++) {
      const float* W = fp(y.w[l]);
      const int fi = y.dims[l], fo = y.dims[l + 1], ld = y.ld[l];
      for (int i = threadIdx.x; i < fi * fo; i += blockDim.x) {
        const float w = W[(i / fi) * ld + (i % fi)];
        s += (double)w * (double)w;
      }
    }
    return block_sum(s, red);
  }

  __device__ void run() const {
    const int f = it.fold, fl = it.fold - P.fold_base;  // fl: which row list
    const int n_tr = P.counts[2 * fl], n_va = P.counts[2 * fl + 1];
    const int32_t* tr = P.train_idx + (int64_t)fl * P.n;
    const int32_t* va = P.val_idx + (int64_t)fl * P.n;
    const uint64_t km = key_model(it.seed, f);
    const RowSplit sp = row_split(km, it.patience, it.val_frac, n_tr);
    const int n_fit = sp.n_fit;
    const int bs = eff_batch(it.batch_size, n_fit);
    const int steps = n_fit > 0 ? (n_fit + bs - 1) / bs : 0;
    const bool traced = P.trace_item == it.b * P.n_folds + fl;

    // zero the slot, then initial parameters
    {
      uint4* z = (uint4*)slot;
      const uint64_t n16 = y.total / 16;
      for (uint64_t i = threadIdx.x; i < n16; i += blockDim.x) z[i] = uint4{0, 0, 0, 0};
    }
    __syncthreads();
    double b1t = 1.0, b2t = 1.0;
    int64_t gstep = 0;
    int e0 = 0, st0 = 0;
    if (traced && P.state_in && steps > 0) {
      // resume: the given state is the one before step_begin
      load_state(P.state_in);
      gstep = P.step_begin;
      e0 = (int)(gstep / steps);
      st0 = (int)(gstep % steps);
      for (int64_t i = 0; i < gstep; i++) {  // beta^gstep by repeated products, as the free run builds it
        b1t *= (double)it.beta1;
        b2t *= (double)it.beta2;
      }
    } else {
      init_params();
    }
    __syncthreads();

    Plateau plateau;
    bool have_best = false;
    const bool watch = it.patience > 0 && steps > 0 && !(traced && P.state_in);
    for (int e = e0; e < it.epochs; e++) {
      const uint64_t ke = key_epoch(km, e);
      const float lr_e = epoch_lr(it.lr, it.power_t, e, n_fit);  // SGD
      double esum = 0.0;  // the thread's share of the epoch's summed data loss
      for (int st = e == e0 ? st0 : 0; st < steps; st++, gstep++) {
        const int lo = st * bs, mb = min(bs, n_fit - lo), Mrows = rup(mb, O::KSTEP);
        gather(tr, sp, ROWS_EPOCH, ke, lo, mb, Mrows);
        forward(Mrows);
        const double lpart = loss_and_delta(mb, Mrows);
        esum += lpart;
        float* rec = nullptr;
        if (traced && gstep >= P.step_begin && gstep < P.step_end) {
          rec = P.trace_out + (gstep - P.step_begin) * (1 + 2 * (int64_t)y.P);
          const double data = block_sum(lpart, red) / (double)mb;
          const double pen = penalty_sum();
          if (threadIdx.x == 0) rec[0] = (float)(data + 0.5 * (double)it.alpha * pen / (double)mb);
        }
        backward_data(Mrows);
        float lr_t = lr_e;
        if (it.solver == BBO_ADAM) {
          b1t *= (double)it.beta1;
          b2t *= (double)it.beta2;
          lr_t = (float)((double)it.lr * sqrt(1.0 - b2t) / (1.0 - b1t));
        }
        wgrad_update(mb, Mrows, lr_t, rec);
      }
      if (watch) {
        float watched = (float)(block_sum(esum, red) / (double)n_fit);
        if (sp.n_hold) watched = (float)(score_rows(tr, sp, ROWS_HELD, sp.n_hold, nullptr) / (double)sp.n_hold);
        const bool stop = plateau.stop_after(watched, it.tol, it.patience);
        if (sp.n_hold && plateau.improved) {
          keep_best();
          have_best = true;
        }
        if (stop) break;
      }
    }
    if (have_best) restore_best();

    // validation score on the held rows
    double hits = 0.0;
    const double lsum = score_rows(va, sp, ROWS_PLAIN, n_va, &hits);
    if (threadIdx.x == 0) {
      float* out = P.item_out + 2 * ((int64_t)it.b * P.n_folds + fl);
      out[0] = n_va > 0 ? (float)(lsum / (double)n_va) : __builtin_nanf("");
      out[1] = n_va > 0 ? (float)(hits / (double)n_va) : __builtin_nanf("");  // accuracy | mean absolute error
    }
  }

  // Summed loss (cross-entropy, or plain squared error) of `count` rows of a list under the current weights,
  // in chunks of the slot's row capacity; optionally the summed second score.  Block-wide result.
  __device__ double score_rows(const int32_t* list, const RowSplit& sp, int mode, int count, double* hits_out) const {
    double lsum = 0.0, hits = 0.0;
    const int c = y.dims[y.L], zc = y.p16[y.L];
    for (int off = 0; off < count; off += y.rows) {
      const int mb = min(y.rows, count - off), Mrows = rup(mb, O::KSTEP);
      gather(list, sp, mode, 0, off, mb, Mrows);
      forward(Mrows);
      const float* Z = fp(y.Z);
      const int32_t* rl = rowlist();
      for (int r = threadIdx.x; r < mb; r += blockDim.x) {
        float aux;
        lsum += (double)row_loss<false>(Z + r * zc, c, P.n_classes, P.y, rl[r], 0.f, nullptr, &aux);
        hits += (double)aux;
      }
      __syncthreads();
    }
    lsum = block_sum(lsum, red);
    hits = block_sum(hits, red);
    if (hits_out) *hits_out = hits;
    return lsum;
  }
};

template <typename OpT>
__global__ __launch_bounds__(NTHREADS) void k_train(const TrainParams P) {
  __shared__ Layout lay;
  __shared__ ItemDesc desc;
  __shared__ int s_item;
  __shared__ double red[NTHREADS / 64];
  char* slot = P.slots + (uint64_t)blockIdx.x * P.slot_bytes;
  for (;;) {
    __syncthreads();
    if (threadIdx.x == 0) s_item = atomicAdd(P.queue, 1);
    __syncthreads();
    const int item = s_item;
    if (item >= P.n_items) break;
    if (threadIdx.x == 0) {
      desc = ((const ItemDesc*)P.items)[item];
      make_layout(lay, desc.dims, desc.L, desc.rows_cap, Op<OpT>::KSTEP, (int)sizeof(OpT));
    }
    __syncthreads();
    Trainer<OpT> T{P, desc, lay, slot, red};
    T.run();
  }
}

// scores[b] = mean over folds (in fold order); status; optional per-fold copy.
__global__ void k_reduce(const float* __restrict__ item_out, int B, int K, float* __restrict__ scores,
                         int32_t* __restrict__ status, float* __restrict__ per_fold) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  double s0 = 0.0, s1 = 0.0;
  for (int f = 0; f < K; f++) {
    const float a = item_out[2 * ((int64_t)b * K + f)], c = item_out[2 * ((int64_t)b * K + f) + 1];
    s0 += (double)a;
    s1 += (double)c;
    if (per_fold) {
      per_fold[2 * ((int64_t)b * K + f)] = a;
      per_fold[2 * ((int64_t)b * K + f) + 1] = c;
    }
  }
  const float r0 = (float)(s0 / K), r1 = (float)(s1 / K);
  scores[2 * b] = r0;
  scores[2 * b + 1] = r1;
  status[b] = isfinite(r0) ? 0 : 1;
}

// Inspection kernels ---------------------------------------------------------
__global__ void k_minibatch_rows(const int32_t* train_idx, const int32_t* counts, int64_t n, uint64_t seed,
                                 int fold, int epoch, int64_t step, int batch_size, int patience, float val_frac,
                                 int32_t* rows_out, int32_t* n_rows_out) {
  const int fl = fold < 0 ? 0 : fold;  // the hold-out lists are a set of their own, with one entry
  const int n_tr = counts[2 * fl];
  const uint64_t km = key_model(seed, fold);
  const RowSplit sp = row_split(km, patience, val_frac, n_tr);
  const int bs = eff_batch(batch_size, sp.n_fit);
  const int64_t lo = step < 0 ? 0 : step * bs;
  const int mb = step < 0 ? sp.n_hold : (int)max((int64_t)0, min((int64_t)bs, (int64_t)sp.n_fit - lo));
  const uint64_t ke = key_epoch(km, epoch);
  for (int p = blockIdx.x * blockDim.x + threadIdx.x; p < mb; p += gridDim.x * blockDim.x)
    rows_out[p] = train_idx[(int64_t)fl * n + row_index(sp, step < 0 ? ROWS_HELD : ROWS_EPOCH, ke, (uint32_t)(lo + p))];
  if (blockIdx.x == 0 && threadIdx.x == 0) *n_rows_out = mb;
}

struct InitArgs {
  uint64_t seed;
  int32_t fold, L;
  int32_t dims[MAXL + 1];
  float bound[MAXL];
};
__global__ void k_init_params(const InitArgs a, float* theta) {
  const uint64_t km = key_model(a.seed, a.fold);
  int64_t off = 0;
  for (int l = 0; l < a.L; l++) {
    const int fi = a.dims[l], fo = a.dims[l + 1];
    const uint64_t kw = key_fold(km, 16 + 2 * l), kb = key_fold(km, 16 + 2 * l + 1);
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < fi * fo + fo; i += gridDim.x * blockDim.x) {
      const bool isb = i >= fi * fo;
      const int e = isb ? i - fi * fo : i;
      const uint32_t k24 = (uint32_t)(key_fold(isb ? kb : kw, (uint64_t)e) >> 40);
      theta[off + i] = a.bound[l] * ((float)((int32_t)k24 - 8388608) * 0x1p-23f);
    }
    off += (int64_t)fi * fo + fo;
  }
}

// ---------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------
thread_local std::string g_err;
int fail(int code, const std::string& msg) {
  g_err = msg;
  return code;
}
#define HIP_TRY(call)                                                                         \
  do {                                                                                        \
    hipError_t e_ = (call);                                                                   \
    if (e_ != hipSuccess)                                                                     \
      return fail(BBO_DEVICE_ERROR, std::string(#call) + ": " + hipGetErrorString(e_));       \
  } while (0)

int check_hparams(const bbo_mlp_hparams* hp, int B) {
  if (B < 0) return fail(BBO_INVALID_ARG, "B < 0");
  if (B > 0 && !hp) return fail(BBO_INVALID_ARG, "hp is null");
  for (int b = 0; b < B; b++) {
    const bbo_mlp_hparams& h = hp[b];
    if (h.n_hidden < 0) return fail(BBO_INVALID_ARG, "n_hidden < 0");
    if (h.n_hidden > BBO_MAX_HIDDEN) return fail(BBO_UNSUPPORTED, "n_hidden > BBO_MAX_HIDDEN");
    for (int i = 0; i < h.n_hidden; i++) {
      if (h.hidden[i] < 1) return fail(BBO_INVALID_ARG, "hidden width < 1");
      if (h.hidden[i] > BBO_MAX_WIDTH) return fail(BBO_UNSUPPORTED, "hidden width > BBO_MAX_WIDTH");
    }
    if (h.solver != BBO_ADAM && h.solver != BBO_SGD) return fail(BBO_INVALID_ARG, "unknown solver");
    if (h.epochs < 0) return fail(BBO_INVALID_ARG, "epochs < 0");
    if (std::isnan(h.lr) || std::isnan(h.alpha) || std::isnan(h.momentum) || std::isnan(h.beta1) ||
        std::isnan(h.beta2) || std::isnan(h.eps) || std::isnan(h.power_t) || std::isnan(h.tol) ||
        std::isnan(h.validation_fraction))
      return fail(BBO_INVALID_ARG, "NaN hyper-parameter");
    if (h.n_iter_no_change < 0) return fail(BBO_INVALID_ARG, "n_iter_no_change < 0");
    if (h.validation_fraction < 0.f || h.validation_fraction >= 1.f)
      return fail(BBO_INVALID_ARG, "validation_fraction outside [0, 1)");
  }
  return BBO_OK;
}

int check_problem(int64_t n, int d, int n_classes, int n_folds, int dtype) {
  if (n < 0) return fail(BBO_INVALID_ARG, "n < 0");
  if (n > 0x3fffffff) return fail(BBO_UNSUPPORTED, "n too large");
  if (d < 1) return fail(BBO_INVALID_ARG, "d < 1");
  if (d > BBO_MAX_FEATURES) return fail(BBO_UNSUPPORTED, "d > BBO_MAX_FEATURES");
  if (n_classes < 0) return fail(BBO_INVALID_ARG, "n_classes must be 0 (regression), 1 (one logit) or >= 2");
  if (n_classes > BBO_MAX_CLASSES) return fail(BBO_UNSUPPORTED, "n_classes > BBO_MAX_CLASSES");
  if (n_folds < 1) return fail(BBO_INVALID_ARG, "n_folds < 1");
  if (n_folds > 1024) return fail(BBO_UNSUPPORTED, "n_folds > 1024");
  if (dtype != BBO_F32 && dtype != BBO_BF16) return fail(BBO_INVALID_ARG, "unknown dtype");
  return BBO_OK;
}

void fill_dims(const bbo_mlp_hparams& h, int d, int n_classes, int32_t* dims, int* L) {
  *L = h.n_hidden + 1;
  dims[0] = d;
  for (int i = 0; i < h.n_hidden; i++) dims[i + 1] = h.hidden[i];
  dims[*L] = n_classes >= 2 ? n_classes : 1;
}

struct SubPlan {
  std::vector<ItemDesc> items;  // this kernel's items, most expensive first
  uint64_t slot_bytes = 0;      // global memory per resident workgroup
  int n_slots = 0;              // workgroups to launch
  uint32_t lds_bytes = 0;       // dynamic LDS per workgroup
  int waves = 0;                // linear kernel: wavefronts per workgroup
  size_t item_bytes = 0;        // size of its item record
  uint64_t o_items = 0;         // workspace byte offset of its item array
};

struct Plan {
  SubPlan sub[KC_N];
  size_t n_items = 0;
  // workspace byte offsets; the kernels run one after the other and share the slot region
  uint64_t o_items = 0, items_bytes = 0, o_queue = 0, o_out = 0, o_train = 0, o_val = 0, o_counts = 0, o_slots = 0,
           total = 0;
};

// Resident workgroups of the generic kernel / compute units, of the current device (looked up once per
// device and thread).
struct DeviceFacts {
  int dev, cus, slots[2];
};
int device_facts(DeviceFacts** out) {
  static thread_local std::vector<DeviceFacts> seen;
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  for (DeviceFacts& e : seen)
    if (e.dev == dev) {
      *out = &e;
      return BBO_OK;
    }
  DeviceFacts e{dev, 0, {0, 0}};
  HIP_TRY(hipDeviceGetAttribute(&e.cus, hipDeviceAttributeMultiprocessorCount, dev));
  seen.push_back(e);
  *out = &seen.back();
  return BBO_OK;
}

int device_slots(int dtype, int* out) {
  DeviceFacts* e = nullptr;
  if (int rc = device_facts(&e)) return rc;
  if (!e->slots[dtype]) {
    int occ = 0;
    if (dtype == BBO_F32)
      HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, k_train<float>, NTHREADS, 0));
    else
      HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, k_train<__bf16>, NTHREADS, 0));
    if (occ < 1) occ = 1;
    e->slots[dtype] = e->cus * occ;
  }
  *out = e->slots[dtype];
  return BBO_OK;
}

int device_cus(int* out) {
  DeviceFacts* e = nullptr;
  if (int rc = device_facts(&e)) return rc;
  *out = e->cus;
  return BBO_OK;
}

// The dynamic-LDS limit of a kernel is a property of the kernel on a device: it is set when first needed and
// raised when a later call needs more, not on every call.
int ensure_dynamic_lds(const void* fn, uint32_t bytes) {
  struct Seen {
    int dev;
    const void* fn;
    uint32_t bytes;
  };
  static thread_local std::vector<Seen> seen;
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  for (Seen& e : seen)
    if (e.dev == dev && e.fn == fn) {
      if (e.bytes >= bytes) return BBO_OK;
      HIP_TRY(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
      e.bytes = bytes;
      return BBO_OK;
    }
  HIP_TRY(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
  seen.push_back(Seen{dev, fn, bytes});
  return BBO_OK;
}

// The fastest kernel that takes a model of these layer sizes on a data set of n rows.
int kernel_class(const int32_t* dims, int L, int64_t n, int dtype) {
  const int d = dims[0];
  // the tiled kernel addresses the input matrix with 32-bit byte offsets, the fp32 kernels with 32-bit indices
  if (dtype == BBO_BF16) {
    if ((uint64_t)n * (uint64_t)d * 2 < (1ull << 31) && tiled_eligible(dims, L)) {
      TLay ty;
      make_tlay(ty, dims, L);
      if (ty.lds_total <= TB_LDS_LIMIT) return KC_TILED;
    }
    return n * (int64_t)d < 0x7fffffff && linear_eligible(dims, L) ? KC_LINEAR : KC_GENERIC;
  }
  if (n * (int64_t)d >= 0x7fffffff) return KC_GENERIC;
  if (small_eligible(dims, L)) {
    SLay sy;
    make_slay(sy, dims, n);
    if (sy.lds_total <= SM_LDS_LIMIT) return KC_SMALL;
  }
  if (mid_eligible(dims, L)) {
    MLay my;
    make_mlay(my, dims, n);
    if (my.lds_total <= MD_LDS_LIMIT) return KC_MID;
  }
  return linear_eligible(dims, L) ? KC_LINEAR : KC_GENERIC;
}

int make_plan(Plan& pl, int64_t n, int d, int n_classes, int n_folds, int fold_base, const bbo_mlp_hparams* hp, int B,
              int dtype) {
  const int kstep = dtype == BBO_F32 ? 16 : 32, opsz = dtype == BBO_F32 ? 4 : 2;
  const double n_tr_est = n_folds > 1 && fold_base >= 0 ? (double)n * (n_folds - 1) / n_folds : (double)n;
  std::vector<double> cost[KC_N];
  for (int k = 0; k < KC_N; k++) {
    pl.sub[k] = SubPlan();
    pl.sub[k].items.reserve((size_t)B * n_folds);
    cost[k].reserve((size_t)B * n_folds);
  }
  pl.sub[KC_TILED].item_bytes = sizeof(TItem);
  pl.sub[KC_SMALL].item_bytes = sizeof(SItem);
  pl.sub[KC_LINEAR].item_bytes = sizeof(ItemDesc);
  pl.sub[KC_GENERIC].item_bytes = sizeof(ItemDesc);
  pl.sub[KC_MID].item_bytes = sizeof(MItem);
  pl.sub[KC_SMALL].slot_bytes = 256;
  for (int b = 0; b < B; b++) {
    const bbo_mlp_hparams& h = hp[b];
    ItemDesc it;
    memset(&it, 0, sizeof(it));
    fill_dims(h, d, n_classes, it.dims, &it.L);
    it.seed = h.seed;
    it.b = b;
    it.solver = h.solver;
    it.nesterov = h.nesterov;
    it.batch_size = h.batch_size;
    it.epochs = h.epochs;
    it.lr = h.lr;
    it.alpha = h.alpha;
    it.momentum = h.momentum;
    it.beta1 = h.beta1;
    it.beta2 = h.beta2;
    it.eps = h.eps;
    it.power_t = h.power_t;
    it.tol = h.tol;
    it.patience = h.n_iter_no_change;
    it.val_frac = h.validation_fraction;
    const int64_t bs = (h.batch_size <= 0 || h.batch_size > n) ? n : h.batch_size;
    it.rows_cap = rup((int)std::max<int64_t>(bs, 1), kstep);
    double fps = 0, params = 0;
    for (int l = 0; l < it.L; l++) {
      it.bound[l] = (float)std::sqrt(6.0 / (double)(it.dims[l] + it.dims[l + 1]));
      fps += 2.0 * it.dims[l] * it.dims[l + 1] * (l == 0 ? 2 : 3);
      params += (double)it.dims[l] * it.dims[l + 1];
    }
    const int k = kernel_class(it.dims, it.L, n, dtype);
    if (k == KC_TILED) {
      TLay ty;
      make_tlay(ty, it.dims, it.L);
      pl.sub[k].slot_bytes = std::max<uint64_t>(pl.sub[k].slot_bytes, ty.total);
      pl.sub[k].lds_bytes = std::max<uint32_t>(pl.sub[k].lds_bytes, ty.lds_total);
    } else if (k == KC_SMALL) {
      SLay sy;
      make_slay(sy, it.dims, n);  // only the hidden layer's moments live in global memory
      // the hidden layer's moments, and room for the best epoch's weights (early stopping on held-out rows)
      pl.sub[k].slot_bytes = std::max<uint64_t>(pl.sub[k].slot_bytes, (3ull * sy.HP * sy.ldw + (sy.HP + 1) * 4ull) * 4);
      pl.sub[k].lds_bytes = std::max<uint32_t>(pl.sub[k].lds_bytes, sy.lds_total);
    } else if (k == KC_MID) {
      MLay my;
      make_mlay(my, it.dims, n);  // the moments of both layers live in global memory
      pl.sub[k].slot_bytes = std::max<uint64_t>(pl.sub[k].slot_bytes, my.g_total);
      pl.sub[k].lds_bytes = std::max<uint32_t>(pl.sub[k].lds_bytes, my.lds_total);
    } else if (k == KC_GENERIC) {
      Layout y;
      make_layout(y, it.dims, it.L, it.rows_cap, kstep, opsz);
      pl.sub[k].slot_bytes = std::max<uint64_t>(pl.sub[k].slot_bytes, y.total);
    }  // KC_LINEAR: a model per wavefront, nothing kept in global memory
    const double steps = std::ceil(n_tr_est / (double)std::max<int64_t>(bs, 1));
    const double c = (double)h.epochs * (n_tr_est * fps + steps * (params * 24.0 + 2.0e4));
    for (int f = 0; f < n_folds; f++) {
      it.fold = f + fold_base;
      pl.sub[k].items.push_back(it);
      cost[k].push_back(c);
    }
  }
  pl.n_items = (size_t)B * n_folds;
  uint64_t slots_region = 0;
  for (int k = 0; k < KC_N; k++) {
    SubPlan& sp = pl.sub[k];
    if (sp.items.empty()) continue;
    std::vector<int> order(sp.items.size());
    for (size_t i = 0; i < order.size(); i++) order[i] = (int)i;
    std::stable_sort(order.begin(), order.end(), [&](int a, int b2) { return cost[k][a] > cost[k][b2]; });
    std::vector<ItemDesc> sorted(sp.items.size());
    for (size_t i = 0; i < order.size(); i++) sorted[i] = sp.items[order[i]];
    sp.items.swap(sorted);
    int max_slots = 0;
    int rc = k == KC_GENERIC ? device_slots(dtype, &max_slots) : device_cus(&max_slots);
    if (rc) return rc;
    size_t units = sp.items.size();
    if (k == KC_SMALL) max_slots *= 2;  // the kernel's LDS footprint is capped at half a CU's LDS
    if (k == KC_LINEAR) {
      // as many workgroups as the LDS lets a CU hold, each of `waves` wavefronts with a model apiece
      const int c_out = n_classes >= 2 ? n_classes : 1;
      sp.waves = ln_waves(d, c_out, n);
      sp.lds_bytes = (uint32_t)sp.waves * ln_wave_bytes(d, c_out, n);
      max_slots *= std::max(1, std::min(8, (int)(160u * 1024u / sp.lds_bytes)));
      units = (sp.items.size() + sp.waves - 1) / sp.waves;
    }
    sp.slot_bytes = (sp.slot_bytes + 255) & ~(uint64_t)255;
    if (k == KC_LINEAR) sp.slot_bytes = 0;
    sp.n_slots = (int)std::min<size_t>(units, (size_t)max_slots);
    slots_region = std::max<uint64_t>(slots_region, sp.slot_bytes * (uint64_t)sp.n_slots);
  }
  uint64_t off = 0;
  auto take = [&](uint64_t bytes) {
    uint64_t o = off;
    off += (bytes + 255) & ~(uint64_t)255;
    return o;
  };
  const uint64_t nn = (uint64_t)std::max<int64_t>(n, 1);
  pl.o_items = off;
  for (int k = 0; k < KC_N; k++) pl.sub[k].o_items = take(pl.sub[k].item_bytes * pl.sub[k].items.size());
  pl.items_bytes = off - pl.o_items;
  pl.o_queue = take(256);  // one counter per kernel
  pl.o_out = take(8ull * std::max<size_t>(pl.n_items, 1));
  pl.o_train = take(4ull * nn * n_folds);
  pl.o_val = take(4ull * nn * n_folds);
  pl.o_counts = take(8ull * n_folds);
  pl.o_slots = take(std::max<uint64_t>(slots_region, 256));
  pl.total = off;
  return BBO_OK;
}


// Pinned staging for the item list: one buffer per host thread and device, reused once
// the previous call's copy has completed.
struct Staging {
  int dev = -1;
  void* ptr = nullptr;
  size_t cap = 0;
  hipEvent_t ev = nullptr;
  bool pending = false;
};
thread_local std::vector<Staging> g_stage;

int stage_items(const void* src, size_t bytes, void* dst, hipStream_t s) {
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  Staging* st = nullptr;
  for (Staging& e : g_stage)
    if (e.dev == dev) st = &e;
  if (!st) {
    g_stage.push_back(Staging());
    st = &g_stage.back();
    st->dev = dev;
  }
  if (!st->ev) HIP_TRY(hipEventCreateWithFlags(&st->ev, hipEventDisableTiming));
  if (st->pending) {
    HIP_TRY(hipEventSynchronize(st->ev));
    st->pending = false;
  }
  if (st->cap < bytes) {
    if (st->ptr) HIP_TRY(hipHostFree(st->ptr));
    st->ptr = nullptr;
    st->cap = 0;
    HIP_TRY(hipHostMalloc(&st->ptr, bytes, hipHostMallocDefault));
    st->cap = bytes;
  }
  memcpy(st->ptr, src, bytes);
  HIP_TRY(hipMemcpyAsync(dst, st->ptr, bytes, hipMemcpyHostToDevice, s));
  HIP_TRY(hipEventRecord(st->ev, s));
  st->pending = true;
  return BBO_OK;
}

// Device address of `scratch` on the current device, looked up once per device.
int scratch_address(void** out) {
  constexpr int MAX_DEV = 64;
  static std::mutex mu;
  static void* ptr[MAX_DEV] = {};
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEV) return fail(BBO_UNSUPPORTED, "device index beyond the static scratch table");
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr[dev]) {
    void* p = nullptr;
    HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(BBO_DEVICE_ERROR, "hipGetSymbolAddress returned no address");
    ptr[dev] = p;
  }
  *out = ptr[dev];
  return BBO_OK;
}

// Host bytes -> device memory without a staging buffer: the bytes travel as the argument of a small kernel
// (3.5 KB per launch).  Used where nothing may be allocated, not even pinned host memory.
struct PokeChunk {
  uint32_t words[896];
};
__global__ void k_poke(const PokeChunk c, uint32_t* __restrict__ dst, int n_words) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_words) dst[i] = c.words[i];
}
int poke_items(const void* src, size_t bytes, void* dst, hipStream_t s) {
  constexpr size_t CH = sizeof(PokeChunk);
  for (size_t off = 0; off < bytes; off += CH) {
    PokeChunk c;
    const size_t nb = std::min(CH, bytes - off);
    memset(&c, 0, sizeof(c));
    memcpy(&c, (const char*)src + off, nb);
    const int nw = (int)((nb + 3) / 4);  // the item region is padded to 256 bytes: whole words stay inside it
    hipLaunchKernelGGL(k_poke, dim3((nw + 255) / 256), dim3(256), 0, s, c, (uint32_t*)((char*)dst + off), nw);
    HIP_TRY(hipGetLastError());
  }
  return BBO_OK;
}

int64_t param_count(int d, int n_classes, const bbo_mlp_hparams& h) {
  int32_t dims[MAXL + 1];
  int L;
  fill_dims(h, d, n_classes, dims, &L);
  int64_t p = 0;
  for (int l = 0; l < L; l++) p += (int64_t)dims[l] * dims[l + 1] + dims[l + 1];
  return p;
}

int run_eval(const void* X, const void* y, int64_t n, int32_t d, int32_t n_classes, const int32_t* fold_idx,
             int32_t n_folds, const bbo_mlp_hparams* hp, int32_t B, int32_t dtype, float* scores,
             int32_t* status, float* per_fold, void* workspace, size_t workspace_bytes, void* stream,
             int32_t trace_b, int32_t trace_fold, int64_t step_begin, int64_t step_end, float* trace_out,
             size_t trace_floats, const float* state_in, bool traced, int fold_base = 0, bool static_ws = false) {
  g_err.clear();
  int rc = check_problem(n, d, n_classes, n_folds, dtype);
  if (rc) return rc;
  rc = check_hparams(hp, B);
  if (rc) return rc;
  if (B == 0) return BBO_OK;
  if (!scores || !status) return fail(BBO_INVALID_ARG, "scores/status is null");
  if (n > 0 && (!X || !y || !fold_idx)) return fail(BBO_INVALID_ARG, "X/y/fold_idx is null");
  if (static_ws) {
    if ((rc = scratch_address(&workspace))) return rc;
    workspace_bytes = BBO_STATIC_SCRATCH_BYTES;
  }
  if (!workspace) return fail(BBO_INVALID_ARG, "workspace is null");
  if (((uintptr_t)workspace & 255) != 0) return fail(BBO_INVALID_ARG, "workspace must be 256-byte aligned");
  if (traced) {
    if (trace_b < 0 || trace_b >= B || trace_fold < 0 || trace_fold >= n_folds)
      return fail(BBO_INVALID_ARG, "trace item out of range");
    if (step_begin < 0 || step_end < step_begin) return fail(BBO_INVALID_ARG, "bad trace window");
    const int64_t P = param_count(d, n_classes, hp[trace_b]);
    if (step_end > step_begin && (!trace_out || (uint64_t)(step_end - step_begin) * (1 + 2 * P) > trace_floats))
      return fail(BBO_INVALID_ARG, "trace buffer too small");
  }
  Plan pl;
  rc = make_plan(pl, n, d, n_classes, n_folds, fold_base, hp, B, dtype);
  if (rc) return rc;
  if (static_ws && (pl.total > BBO_STATIC_SCRATCH_BYTES || pl.items_bytes > BBO_STATIC_MAX_ITEM_BYTES))
    return fail(BBO_WORKSPACE_TOO_SMALL,
                "this problem needs " + std::to_string(pl.total) + " bytes of workspace (" +
                    std::to_string(pl.items_bytes) + " of item records); the allocation-free entry point holds " +
                    std::to_string((size_t)BBO_STATIC_SCRATCH_BYTES) + " (" +
                    std::to_string((size_t)BBO_STATIC_MAX_ITEM_BYTES) + "): use bbo_mlp_cv_eval with a workspace");
  if (workspace_bytes < pl.total) return fail(BBO_WORKSPACE_TOO_SMALL, "workspace too small");
  hipStream_t s = (hipStream_t)stream;
  char* ws = (char*)workspace;
  {
    // the item arrays of all kernels, laid out as in the workspace, in one staged copy
    static thread_local std::vector<char> blob;  // kept between calls
    blob.assign(pl.items_bytes, 0);
    for (int k = 0; k < KC_N; k++) {
      const SubPlan& sp = pl.sub[k];
      char* at = blob.data() + (sp.o_items - pl.o_items);
      for (size_t i = 0; i < sp.items.size(); i++) {
        if (k == KC_TILED) {
          TItem ti;
          memset(&ti, 0, sizeof(ti));
          ti.d = sp.items[i];
          make_tlay(ti.y, sp.items[i].dims, sp.items[i].L);
          memcpy(at + i * sizeof(TItem), &ti, sizeof(TItem));
        } else if (k == KC_SMALL) {
          SItem si;
          memset(&si, 0, sizeof(si));
          si.d = sp.items[i];
          make_slay(si.y, sp.items[i].dims, n);
          memcpy(at + i * sizeof(SItem), &si, sizeof(SItem));
        } else if (k == KC_MID) {
          MItem mi;
          memset(&mi, 0, sizeof(mi));
          mi.d = sp.items[i];
          make_mlay(mi.y, sp.items[i].dims, n);
          memcpy(at + i * sizeof(MItem), &mi, sizeof(MItem));
        } else {
          memcpy(at + i * sizeof(ItemDesc), &sp.items[i], sizeof(ItemDesc));
        }
      }
    }
    rc = static_ws ? poke_items(blob.data(), blob.size(), ws + pl.o_items, s)
                   : stage_items(blob.data(), blob.size(), ws + pl.o_items, s);
    if (rc) return rc;
  }

  TrainParams P;
  memset(&P, 0, sizeof(P));
  P.X = X;
  P.y = y;
  P.train_idx = (const int32_t*)(ws + pl.o_train);
  P.val_idx = (const int32_t*)(ws + pl.o_val);
  P.counts = (const int32_t*)(ws + pl.o_counts);
  P.item_out = (float*)(ws + pl.o_out);
  P.slots = ws + pl.o_slots;
  P.n = n;
  P.d = d;
  P.n_classes = n_classes;
  P.n_folds = n_folds;
  P.fold_base = fold_base;
  P.trace_item = traced ? trace_b * n_folds + trace_fold : -1;
  P.step_begin = step_begin;
  P.step_end = step_end;
  P.trace_out = trace_out;
  P.state_in = traced ? state_in : nullptr;
  P.x_bf16 = dtype == BBO_BF16;

  int32_t* queues = (int32_t*)(ws + pl.o_queue);  // one work-queue counter per kernel, reset by k_fold_lists
  hipLaunchKernelGGL(k_fold_lists, dim3(n_folds), dim3(NTHREADS), 0, s, fold_idx, n, (int32_t*)(ws + pl.o_train),
                     (int32_t*)(ws + pl.o_val), (int32_t*)(ws + pl.o_counts), queues, fold_base);
  HIP_TRY(hipGetLastError());
  // one launch per kernel that has items, one after the other on the caller's stream
  for (int k = 0; k < KC_N; k++) {
    const SubPlan& sp = pl.sub[k];
    if (sp.items.empty()) continue;
    P.items = ws + sp.o_items;
    P.queue = queues + k;
    P.slot_bytes = sp.slot_bytes;
    P.n_items = (int)sp.items.size();
    if (k == KC_TILED) {
      if ((rc = ensure_dynamic_lds((const void*)k_train_tiled, sp.lds_bytes))) return rc;
      hipLaunchKernelGGL(k_train_tiled, dim3(sp.n_slots), dim3(TB_THREADS), sp.lds_bytes, s, P);
    } else if (k == KC_SMALL) {
      const int kt = d + 1 <= 16 ? 1 : (d + 1 <= 32 ? 2 : 4);
      const int c_out = n_classes >= 2 ? n_classes : 1, co = c_out <= 2 ? c_out : 4;
      typedef void (*small_fn)(const TrainParams);
      static const small_fn fns[3][3] = {
          {k_train_small<1, 1>, k_train_small<1, 2>, k_train_small<1, 4>},
          {k_train_small<2, 1>, k_train_small<2, 2>, k_train_small<2, 4>},
          {k_train_small<4, 1>, k_train_small<4, 2>, k_train_small<4, 4>}};
      const small_fn fn = fns[kt == 1 ? 0 : (kt == 2 ? 1 : 2)][co == 1 ? 0 : (co == 2 ? 1 : 2)];
      if ((rc = ensure_dynamic_lds((const void*)fn, sp.lds_bytes))) return rc;
      hipLaunchKernelGGL(fn, dim3(sp.n_slots), dim3(SM_THREADS), sp.lds_bytes, s, P);
    } else if (k == KC_MID) {
      typedef void (*mid_fn)(const TrainParams);
      const int kt = md_kt(d);
      const mid_fn fn = kt == 2 ? k_train_mid<2> : (kt == 4 ? k_train_mid<4> : (kt == 5 ? k_train_mid<5> : (kt == 6 ? k_train_mid<6> : k_train_mid<8>)));
      if ((rc = ensure_dynamic_lds((const void*)fn, sp.lds_bytes))) return rc;
      hipLaunchKernelGGL(fn, dim3(sp.n_slots), dim3(MD_THREADS), sp.lds_bytes, s, P);
    } else if (k == KC_LINEAR) {
      const int c_out = n_classes >= 2 ? n_classes : 1, co = ln_co(c_out), ki = ln_ki(d);
      typedef void (*linear_fn)(const TrainParams);
      // [padded outputs 1, 2, 4, 8, 16][rows of W per lane 1, 2, 4], at most 32 parameters per lane
      static const linear_fn fns[5][3] = {
          {k_train_linear<1, 1>, k_train_linear<1, 2>, k_train_linear<1, 4>},
          {k_train_linear<2, 1>, k_train_linear<2, 2>, k_train_linear<2, 4>},
          {k_train_linear<4, 1>, k_train_linear<4, 2>, k_train_linear<4, 4>},
          {k_train_linear<8, 1>, k_train_linear<8, 2>, k_train_linear<8, 4>},
          {k_train_linear<16, 1>, k_train_linear<16, 2>, nullptr}};
      const linear_fn fn =
          fns[co == 1 ? 0 : (co == 2 ? 1 : (co == 4 ? 2 : (co == 8 ? 3 : 4)))][ki == 1 ? 0 : (ki == 2 ? 1 : 2)];
      if (!fn) return fail(BBO_DEVICE_ERROR, "no kernel for this linear shape");  // ruled out by linear_eligible()
      if ((rc = ensure_dynamic_lds((const void*)fn, sp.lds_bytes))) return rc;
      hipLaunchKernelGGL(fn, dim3(sp.n_slots), dim3(64 * sp.waves), sp.lds_bytes, s, P);
    } else if (dtype == BBO_F32) {
      hipLaunchKernelGGL(k_train<float>, dim3(sp.n_slots), dim3(NTHREADS), 0, s, P);
    } else {
      hipLaunchKernelGGL(k_train<__bf16>, dim3(sp.n_slots), dim3(NTHREADS), 0, s, P);
    }
    HIP_TRY(hipGetLastError());
  }
  hipLaunchKernelGGL(k_reduce, dim3((B + 255) / 256), dim3(256), 0, s, P.item_out, B, n_folds, scores, status,
                     per_fold);
  HIP_TRY(hipGetLastError());
  return BBO_OK;
}

}  // namespace

extern "C" {

int bbo_mlp_workspace_bytes(int64_t n, int32_t d, int32_t n_classes, int32_t n_folds, const bbo_mlp_hparams* hp,
                            int32_t B, int32_t dtype, size_t* out) {
  g_err.clear();
  if (!out) return fail(BBO_INVALID_ARG, "out is null");
  int rc = check_problem(n, d, n_classes, n_folds, dtype);
  if (rc) return rc;
  rc = check_hparams(hp, B);
  if (rc) return rc;
  Plan pl;
  rc = make_plan(pl, n, d, n_classes, n_folds, 0, hp, B, dtype);
  if (rc) return rc;
  *out = (size_t)pl.total;
  return BBO_OK;
}

int bbo_mlp_cv_eval(const void* X, const void* y, int64_t n, int32_t d, int32_t n_classes,
                    const int32_t* fold_idx, int32_t n_folds, const bbo_mlp_hparams* hp, int32_t B,
                    int32_t dtype, float* scores, int32_t* status, float* per_fold, void* workspace,
                    size_t workspace_bytes, void* stream) {
  return run_eval(X, y, n, d, n_classes, fold_idx, n_folds, hp, B, dtype, scores, status, per_fold, workspace,
                  workspace_bytes, stream, -1, -1, 0, 0, nullptr, 0, nullptr, false);
}

int bbo_mlp_cv_eval_static(const void* X, const void* y, int64_t n, int32_t d, int32_t n_classes,
                           const int32_t* fold_idx, int32_t n_folds, const bbo_mlp_hparams* hp, int32_t B,
                           int32_t dtype, float* scores, int32_t* status, float* per_fold, void* stream) {
  return run_eval(X, y, n, d, n_classes, fold_idx, n_folds, hp, B, dtype, scores, status, per_fold, nullptr, 0,
                  stream, -1, -1, 0, 0, nullptr, 0, nullptr, false, 0, true);
}

int bbo_mlp_cv_eval_traced(const void* X, const void* y, int64_t n, int32_t d, int32_t n_classes,
                           const int32_t* fold_idx, int32_t n_folds, const bbo_mlp_hparams* hp, int32_t B,
                           int32_t dtype, float* scores, int32_t* status, float* per_fold, void* workspace,
                           size_t workspace_bytes, void* stream, int32_t trace_b, int32_t trace_fold,
                           int64_t step_begin, int64_t step_end, float* trace_out, size_t trace_floats,
                           const float* state_in) {
  return run_eval(X, y, n, d, n_classes, fold_idx, n_folds, hp, B, dtype, scores, status, per_fold, workspace,
                  workspace_bytes, stream, trace_b, trace_fold, step_begin, step_end, trace_out, trace_floats,
                  state_in, true);
}

int bbo_mlp_fold_lists(const int32_t* fold_idx, int64_t n, int32_t n_folds, int32_t* train_idx, int32_t* val_idx,
                       int32_t* counts, void* stream) {
  g_err.clear();
  if (n < 0 || n > 0x3fffffff || n_folds < 1 || n_folds > 1024) return fail(BBO_INVALID_ARG, "bad n or n_folds");
  if (!counts || (n > 0 && (!fold_idx || !train_idx || !val_idx))) return fail(BBO_INVALID_ARG, "null pointer");
  hipLaunchKernelGGL(k_fold_lists, dim3(n_folds), dim3(NTHREADS), 0, (hipStream_t)stream, fold_idx, n, train_idx,
                     val_idx, counts, (int32_t*)nullptr, 0);
  HIP_TRY(hipGetLastError());
  return BBO_OK;
}

int bbo_mlp_holdout_eval(const void* X, const void* y, int64_t n, int32_t d, int32_t n_classes,
                         const int32_t* fold_idx, const bbo_mlp_hparams* hp, int32_t B, int32_t dtype,
                         float* scores, int32_t* status, void* workspace, size_t workspace_bytes, void* stream) {
  return run_eval(X, y, n, d, n_classes, fold_idx, 1, hp, B, dtype, scores, status, nullptr, workspace,
                  workspace_bytes, stream, 0, 0, 0, 0, nullptr, 0, nullptr, false, -1);
}

int bbo_mlp_holdout_lists(const int32_t* fold_idx, int64_t n, int32_t* train_idx, int32_t* val_idx, int32_t* counts,
                          void* stream) {
  g_err.clear();
  if (n < 0 || n > 0x3fffffff) return fail(BBO_INVALID_ARG, "bad n");
  if (!counts || (n > 0 && (!fold_idx || !train_idx || !val_idx))) return fail(BBO_INVALID_ARG, "null pointer");
  hipLaunchKernelGGL(k_fold_lists, dim3(1), dim3(NTHREADS), 0, (hipStream_t)stream, fold_idx, n, train_idx, val_idx,
                     counts, (int32_t*)nullptr, -1);
  HIP_TRY(hipGetLastError());
  return BBO_OK;
}

int bbo_mlp_minibatch_rows(const int32_t* train_idx, const int32_t* counts, int64_t n, const bbo_mlp_hparams* hp,
                           int32_t fold, int32_t epoch, int64_t step, int32_t* rows_out, int32_t* n_rows_out,
                           void* stream) {
  g_err.clear();
  if (!train_idx || !counts || !hp || !rows_out || !n_rows_out || n < 0 || fold < -1 || epoch < 0 || step < -1)
    return fail(BBO_INVALID_ARG, "bad argument");
  hipLaunchKernelGGL(k_minibatch_rows, dim3(64), dim3(256), 0, (hipStream_t)stream, train_idx, counts, n, hp->seed,
                     fold, epoch, step, hp->batch_size, hp->n_iter_no_change, hp->validation_fraction, rows_out,
                     n_rows_out);
  HIP_TRY(hipGetLastError());
  return BBO_OK;
}

int bbo_mlp_init_params(int32_t d, int32_t n_classes, const bbo_mlp_hparams* hp, int32_t fold, float* theta_out,
                        void* stream) {
  g_err.clear();
  int rc = check_problem(0, d, n_classes, 1, BBO_F32);
  if (rc) return rc;
  rc = check_hparams(hp, 1);
  if (rc) return rc;
  if (!theta_out || fold < -1) return fail(BBO_INVALID_ARG, "bad argument");
  InitArgs a;
  memset(&a, 0, sizeof(a));
  a.seed = hp->seed;
  a.fold = fold;
  fill_dims(*hp, d, n_classes, a.dims, &a.L);
  for (int l = 0; l < a.L; l++) a.bound[l] = (float)std::sqrt(6.0 / (double)(a.dims[l] + a.dims[l + 1]));
  hipLaunchKernelGGL(k_init_params, dim3(128), dim3(256), 0, (hipStream_t)stream, a, theta_out);
  HIP_TRY(hipGetLastError());
  return BBO_OK;
}

int64_t bbo_mlp_param_count(int32_t d, int32_t n_classes, const bbo_mlp_hparams* hp) {
  g_err.clear();
  if (check_problem(0, d, n_classes, 1, BBO_F32) || check_hparams(hp, 1)) return -1;
  return param_count(d, n_classes, *hp);
}

int bbo_mlp_kernel_class(int64_t n, int32_t d, int32_t n_classes, const bbo_mlp_hparams* hp, int32_t dtype) {
  g_err.clear();
  if (check_problem(n, d, n_classes, 1, dtype) || check_hparams(hp, 1)) return -1;
  int32_t dims[MAXL + 1];
  int L;
  fill_dims(*hp, d, n_classes, dims, &L);
  return kernel_class(dims, L, n, dtype);
}

const char* bbo_mlp_last_error(void) { return g_err.c_str(); }

}  // extern "C"
