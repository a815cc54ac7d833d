// LDS-resident training / scoring kernel for fp32 models with one hidden layer whose input or output side
// is too wide for train_small_f32.h (the digits shape: up to 127 inputs, hidden width up to 256, up to 16
// outputs, as far as the weights fit into one CU's LDS).
//
// One workgroup of 8 waves trains one model, one model per CU.  Both weight matrices stay in LDS for the
// whole run; the optimizer moments of both layers live in a per-workgroup global slot that stays in L2 and
// is read and written once per step.  A minibatch is processed in chunks of 64 rows.  Wave w owns the
// hidden-unit tiles w and w + 8 in every phase, so hidden activations and deltas never leave its registers:
//
//   forward   D[row][unit] = xs[row][k] . w1[unit][k] on MFMA (16x16x4 fp32; the bias rides in column d of
//             xs / w1), ReLU in the accumulators.  The output layer contracts over the hidden units, which
//             the accumulators hold along the lanes: each 16 x 16 tile goes through a 1 KB LDS patch of the
//             wave's own (no workgroup barrier) to become an MFMA operand, and the wave's partial outputs
//             z[row][out] over its 32 units go to LDS, where the 8 partials are summed.
//   outputs   wave w takes rows 8w..8w+7 (lane = output x row): softmax / loss / output delta with
//             reductions over the 16 lanes of a row; the delta goes to LDS.
//   backward  hidden delta = delta . w2^T on MFMA, in the accumulator layout of the activations, masked by
//             them; it is the B operand of the hidden layer's weight gradient D[k][unit] += xs[row][k] .
//             dh[row][unit], accumulated over the step's chunks in registers, and the activations are the A
//             operand of the output layer's weight gradient D[unit][out] += a[row][unit] . delta[row][out].
//   update    Adam / SGD on the gradients in registers, weights in LDS, moments in the slot.
//
// Four workgroup barriers per chunk.  The inputs of the next chunk are fetched into registers while the
// current one is processed.
#pragma once
#include "common.h"
#include "train_tiled_bf16.h"  // OptC, opt_update

namespace {

constexpr int MD_THREADS = 512;
constexpr int MD_WAVES = 8;
constexpr int MD_RC = 64;                            // rows per chunk
constexpr int MD_CP = 16;                            // padded outputs
constexpr int MD_PS = 17;                            // row stride of a wave's transposing patch
constexpr uint32_t MD_LDS_LIMIT = 160 * 1024 - 1536;  // dynamic LDS available to the kernel

struct MLay {
  int32_t d, h, c, K0, HP, ldw;
  int32_t cw[2], cb[2], P;
  uint32_t o_w1, o_w2, o_xs, o_zp, o_d3, o_patch, o_rows, o_ys, o_epoch, lds_total;
  int32_t epoch_cap;  // entries of the per-epoch row table in LDS (0: rows are permuted on the fly)
  uint32_t g_m1, g_v1, g_m2, g_v2, g_zero, g_best, g_total;  // byte offsets in the global slot
};

struct MItem {
  ItemDesc d;
  MLay y;
};

// k tiles (16 columns each) of the input layer the kernel is compiled for
__host__ __device__ inline int md_kt(int d) {
  const int kt = (d + 1 + 15) / 16;
  return kt <= 2 ? 2 : (kt <= 4 ? 4 : (kt <= 5 ? 5 : (kt <= 6 ? 6 : 8)));
}

__host__ __device__ inline bool mid_eligible(const int32_t* dims, int L) {
  return L == 2 && dims[0] <= 127 && dims[1] <= 256 && dims[2] <= MD_CP;
}

__host__ __device__ inline void make_mlay(MLay& y, const int32_t* dims, int64_t n) {
  y.d = dims[0];
  y.h = dims[1];
  y.c = dims[2];
  y.K0 = 16 * md_kt(dims[0]);
  y.HP = rup(dims[1], 16);
  y.ldw = y.K0 + 4;
  y.cw[0] = 0;
  y.cb[0] = y.d * y.h;
  y.cw[1] = y.cb[0] + y.h;
  y.cb[1] = y.cw[1] + y.h * y.c;
  y.P = y.cb[1] + y.c;
  uint32_t o = 0;
  auto take = [&](uint32_t floats) {
    uint32_t r = o;
    o += ((floats * 4) + 15) & ~15u;
    return r;
  };
  y.o_w1 = take(y.HP * y.ldw);
  y.o_w2 = take((y.HP + 1) * MD_CP);
  y.o_xs = take(MD_RC * y.ldw);
  y.o_zp = take(MD_WAVES * MD_RC * MD_CP);
  y.o_d3 = take(MD_RC * MD_CP);
  y.o_patch = take(MD_WAVES * 16 * MD_PS);
  y.o_rows = take(2 * MD_RC);
  y.o_ys = take(2 * MD_RC);
  y.o_epoch = o;
  y.epoch_cap = 0;
  if (n <= 4096 && o + 4 * (uint32_t)n + 16 <= MD_LDS_LIMIT) {
    y.epoch_cap = (int32_t)n;
    o += (4 * (uint32_t)n + 15) & ~15u;
  }
  y.lds_total = o;
  uint32_t g = 0;
  auto gtake = [&](uint32_t floats) {
    uint32_t r = g;
    g += ((floats * 4) + 255) & ~255u;
    return r;
  };
  y.g_m1 = gtake(y.HP * y.ldw);
  y.g_v1 = gtake(y.HP * y.ldw);
  y.g_m2 = gtake((y.HP + 1) * MD_CP);
  y.g_v2 = gtake((y.HP + 1) * MD_CP);
  y.g_zero = g;  // what a new model must find zeroed: the moments
  y.g_best = gtake(y.HP * y.ldw + (y.HP + 1) * MD_CP);  // weights of the best epoch so far (early stopping)
  y.g_total = g;
}

// Reductions over the 16 lanes of a DPP row (the lanes that share lane / 16); every lane gets the result.
// Rotations by 8 and 4 within the row, then the two quad permutations: four cross-lane moves, no LDS traffic.
template <int CTRL>
__device__ __forceinline__ int dpp_mov(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, false);
}
template <class Op>
__device__ __forceinline__ float r16_reduce(float v, Op op) {
  v = op(v, __builtin_bit_cast(float, dpp_mov<0x128>(__builtin_bit_cast(int, v))));
  v = op(v, __builtin_bit_cast(float, dpp_mov<0x124>(__builtin_bit_cast(int, v))));
  v = op(v, __builtin_bit_cast(float, dpp_mov<0x4E>(__builtin_bit_cast(int, v))));
  v = op(v, __builtin_bit_cast(float, dpp_mov<0xB1>(__builtin_bit_cast(int, v))));
  return v;
}
__device__ __forceinline__ float r16_sum(float v) {
  return r16_reduce(v, [](float a, float b) { return a + b; });
}
__device__ __forceinline__ float r16_max(float v) {
  return r16_reduce(v, [](float a, float b) { return fmaxf(a, b); });
}
__device__ __forceinline__ int r16_min(int v) {
  v = min(v, dpp_mov<0x128>(v));
  v = min(v, dpp_mov<0x124>(v));
  v = min(v, dpp_mov<0x4E>(v));
  v = min(v, dpp_mov<0xB1>(v));
  return v;
}

// KT: 16-wide k tiles of the input layer (inputs + bias column).
template <int KT>
struct Mid {
  static constexpr int K0 = 16 * KT, NX = K0 / 8;  // NX: input values a thread fetches per chunk
  const TrainParams& P;
  const ItemDesc& it;
  const MLay& y;
  char* lds;
  char* slot;
  double* red;

  __device__ __forceinline__ float* f(uint32_t off) const { return (float*)(lds + off); }
  __device__ __forceinline__ float* g(uint32_t off) const { return (float*)(slot + off); }
  __device__ __forceinline__ int32_t* rowlist(int par) const { return (int32_t*)(lds + y.o_rows) + par * MD_RC; }
  __device__ __forceinline__ float* ys(int par) const { return f(y.o_ys) + par * MD_RC; }
  // The thread index as a value the compiler cannot see through (see train_tiled_bf16.h): lane coordinates
  // are recomputed in each phase instead of being kept for the whole run.
  __device__ __forceinline__ static int tid() {
    int t = threadIdx.x;
    asm volatile("" : "+v"(t));
    return t;
  }
  // packed index (W1[in][out], b1, W2[in][out], b2) of hidden-layer element (unit j, column k); -1 for pads
  __device__ __forceinline__ int ci_hidden(int j, int k) const {
    if (j >= y.h || k > y.d) return -1;
    return k < y.d ? y.cw[0] + k * y.h + j : y.cb[0] + j;
  }
  __device__ __forceinline__ float init_value(int l, int e, bool isb) const {
    const uint64_t kt = key_fold(key_model(it.seed, it.fold), 16 + 2 * l + (isb ? 1 : 0));
    const uint32_t k24 = (uint32_t)(key_fold(kt, (uint64_t)e) >> 40);
    return it.bound[l] * ((float)((int32_t)k24 - 8388608) * 0x1p-23f);
  }

  // Keep the current weights (both layers, as they lie in LDS) aside / put the kept ones back.  Block-wide; the
  // caller orders it against updates.
  __device__ __forceinline__ void copy_best(bool keep) const {
    float* w1 = f(y.o_w1);
    float* w2 = f(y.o_w2);
    float* b = g(y.g_best);
    const int n1 = y.HP * y.ldw, n2 = (y.HP + 1) * MD_CP;
    for (int i = threadIdx.x; i < n1 + n2; i += blockDim.x) {
      float* l = i < n1 ? w1 + i : w2 + (i - n1);
      if (keep)
        b[i] = *l;
      else
        *l = b[i];
    }
  }

  // Weights into LDS (and, from a packed state, the moments into the slot).
  __device__ __forceinline__ void put_weights(const float* st) const {
    const int d = y.d, h = y.h, c = y.c;
    float* w1 = f(y.o_w1);
    float* w2 = f(y.o_w2);
    for (int ci = threadIdx.x; ci < y.P; ci += blockDim.x) {
      if (ci < y.cw[1]) {
        const bool isb = ci >= y.cb[0];
        const int o = isb ? (ci - y.cb[0]) * y.ldw + d : (ci % h) * y.ldw + ci / h;
        w1[o] = st ? st[ci] : init_value(0, isb ? ci - y.cb[0] : ci, isb);
        if (st) {
          g(y.g_m1)[o] = st[y.P + ci];
          g(y.g_v1)[o] = st[2 * y.P + ci];
        }
      } else {
        const bool isb = ci >= y.cb[1];
        const int e = isb ? ci - y.cb[1] : ci - y.cw[1];
        const int o = isb ? y.HP * MD_CP + e : (e / c) * MD_CP + e % c;
        w2[o] = st ? st[ci] : init_value(1, e, isb);
        if (st) {
          g(y.g_m2)[o] = st[y.P + ci];
          g(y.g_v2)[o] = st[2 * y.P + ci];
        }
      }
    }
  }

  // ---- input staging, one chunk ahead ---------------------------------------
  __device__ __forceinline__ int fetch_row_id(const int32_t* list, const RowSplit& sp, int mode, uint64_t key, int lo,
                                              int rows) const {
    const int p = threadIdx.x;
    if (p >= MD_RC || p >= rows) return -1;
    if (mode == ROWS_EPOCH && y.epoch_cap) return ((const int32_t*)(lds + y.o_epoch))[lo + p];
    return list[row_index(sp, mode, key, (uint32_t)(lo + p))];
  }
  __device__ __forceinline__ void build_epoch_table(const int32_t* list, const RowSplit& sp, uint64_t key) const {
    int32_t* tab = (int32_t*)(lds + y.o_epoch);
    for (int p = threadIdx.x; p < sp.n_fit; p += blockDim.x) tab[p] = list[fit_index(sp, key, (uint32_t)p)];
  }
  __device__ __forceinline__ void park_row_id(int par, int row) const {
    if ((int)threadIdx.x < MD_RC) rowlist(par)[threadIdx.x] = row;
  }
  // the chunk's input values (element t + 512 j of the 64 x K0 block) and labels into registers
  __device__ __forceinline__ void fetch_inputs(int par, float (&xr)[NX], float& yv) const {
    const int32_t* rl = rowlist(par);
    const float* X = (const float*)P.X;
    const int t_ = tid(), d = y.d;
#pragma unroll
    for (int j = 0; j < NX; j++) {
      const int idx = t_ + MD_THREADS * j, r = idx / K0, k = idx - r * K0;
      const int row = rl[r];
      xr[j] = 0.f;
      if (row >= 0) xr[j] = k < d ? X[row * d + k] : (k == d ? 1.f : 0.f);  // n*d < 2^31 (checked by the host)
    }
    yv = 0.f;
    if ((int)threadIdx.x < MD_RC) {
      const int row = rl[threadIdx.x];
      if (row >= 0) yv = P.n_classes >= 1 ? __int_as_float(((const int32_t*)P.y)[row]) : ((const float*)P.y)[row];
    }
  }
  __device__ __forceinline__ void commit_inputs(int par, const float (&xr)[NX], float yv) const {
    float* s = f(y.o_xs);
    const int t_ = tid();
#pragma unroll
    for (int j = 0; j < NX; j++) {
      const int idx = t_ + MD_THREADS * j, r = idx / K0, k = idx - r * K0;
      s[r * y.ldw + k] = xr[j];
    }
    if ((int)threadIdx.x < MD_RC) ys(par)[threadIdx.x] = yv;
  }

  // ---- forward: hidden activations into acc, the wave's partial outputs into zp ----
  __device__ __forceinline__ void forward(int nrt, f32x4 (&acc)[2][4]) const {
    const int t_ = tid(), lane = t_ & 63, w = t_ >> 6, li = lane & 15, q = lane >> 4;
    const int nut = y.HP / 16, ldw = y.ldw;
    const float* s = f(y.o_xs);
    const float* w1 = f(y.o_w1);
    const float* w2 = f(y.o_w2);
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
      for (int r = 0; r < 4; r++) acc[i][r] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < KT; kk++) {
      f32x4 a[4], b[2];
#pragma unroll
      for (int r = 0; r < 4; r++)
        if (r < nrt) a[r] = *(const f32x4*)(s + (r * 16 + li) * ldw + kk * 16 + 4 * q);
#pragma unroll
      for (int i = 0; i < 2; i++)
        if (w + 8 * i < nut) b[i] = *(const f32x4*)(w1 + ((w + 8 * i) * 16 + li) * ldw + kk * 16 + 4 * q);
#pragma unroll
      for (int i = 0; i < 2; i++)
        if (w + 8 * i < nut) {
#pragma unroll
          for (int r = 0; r < 4; r++)
            if (r < nrt) {
#pragma unroll
              for (int e = 0; e < 4; e++)
                acc[i][r] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[r][e], b[i][e], acc[i][r], 0, 0, 0);
            }
        }
    }
    // ReLU; then z[row][out] += a[row][unit] . w2[unit][out] over the wave's units: the tile (lane = unit, registers
    // = rows 4q..4q+3) is written to the wave's patch as p[row][unit] and read back with lane = row
    float* p = f(y.o_patch) + w * 16 * MD_PS;
    f32x4 zacc[4];
#pragma unroll
    for (int r = 0; r < 4; r++) zacc[r] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < 2; i++)
      if (w + 8 * i < nut) {
        float wb[4];  // B[k = unit 4s+q][n = out li]
#pragma unroll
        for (int sN = 0; sN < 4; sN++) wb[sN] = w2[((w + 8 * i) * 16 + 4 * sN + q) * MD_CP + li];
#pragma unroll
        for (int r = 0; r < 4; r++)
          if (r < nrt) {
#pragma unroll
            for (int e = 0; e < 4; e++) {
              const float av = fmaxf(acc[i][r][e], 0.f);
              acc[i][r][e] = av;
              p[(4 * q + e) * MD_PS + li] = av;
            }
            float ar[4];  // A[m = row li][k = unit 4s+q]; a wave's LDS accesses execute in order
#pragma unroll
            for (int sN = 0; sN < 4; sN++) ar[sN] = p[li * MD_PS + 4 * sN + q];
#pragma unroll
            for (int sN = 0; sN < 4; sN++) zacc[r] = __builtin_amdgcn_mfma_f32_16x16x4f32(ar[sN], wb[sN], zacc[r], 0, 0, 0);
          }
      }
    // the lane holds z[row 16r+4q+e][out li]
    float* zp = f(y.o_zp) + w * MD_RC * MD_CP;
#pragma unroll
    for (int r = 0; r < 4; r++)
      if (r < nrt) {
#pragma unroll
        for (int e = 0; e < 4; e++) zp[(r * 16 + 4 * q + e) * MD_CP + li] = zacc[r][e];
      }
  }

  // ---- outputs: wave w takes rows 8w..8w+7, lane (out li, row 8w + q and 8w + 4 + q) ----
  template <bool TRAIN>
  __device__ __forceinline__ void outputs(int par, int rows, int nrt, float inv_mb, double& lsum, double& hits) const {
    const int t_ = tid(), lane = t_ & 63, w = t_ >> 6, li = lane & 15, q = lane >> 4;
    const int c = y.c;
    const float* zp = f(y.o_zp);
    const float b2 = f(y.o_w2)[y.HP * MD_CP + li];
    float* d3 = f(y.o_d3);
#pragma unroll
    for (int half = 0; half < 2; half++) {
      const int row = 8 * w + 4 * half + q;
      if (row >= 16 * nrt) continue;  // a row tile nobody computed (uniform per wave: 8 rows lie in one tile)
      float z = b2;
#pragma unroll
      for (int ww = 0; ww < MD_WAVES; ww++) z += zp[(ww * MD_RC + row) * MD_CP + li];
      const bool valid = row < rows;
      const float yv = ys(par)[row];
      float dl = 0.f;
      if (P.n_classes >= 2) {
        const int yr = __float_as_int(yv);
        const float zz = li < c ? z : -INFINITY;
        const float mx = r16_max(zz);
        const int best = r16_min(zz == mx ? li : 99);
        const float se = r16_sum(li < c ? expf(zz - mx) : 0.f);
        const float lse = mx + logf(se);
        const float zy = r16_sum(li == yr && li < c ? zz : 0.f);
        if (valid && li == 0) {
          lsum += (double)(lse - zy);
          hits += best == yr ? 1.0 : 0.0;
        }
        if (TRAIN && valid && li < c) dl = (expf(zz - lse) - (li == yr ? 1.f : 0.f)) * inv_mb;
      } else if (P.n_classes == 1) {
        // one logit, labels 0/1: log(1 + e^z) - y z, delta (sigmoid(z) - y)/m
        const int yr = __float_as_int(yv);
        if (valid && li == 0) {
          lsum += (double)(fmaxf(z, 0.f) + log1pf(expf(-fabsf(z))) - (yr ? z : 0.f));
          hits += (z > 0.f) == (yr != 0) ? 1.0 : 0.0;
          if (TRAIN) dl = (1.f / (1.f + expf(-z)) - (float)yr) * inv_mb;
        }
      } else {
        const float e0 = z - yv;
        if (valid && li == 0) {
          lsum += TRAIN ? 0.5 * (double)e0 * (double)e0 : (double)e0 * (double)e0;
          hits += (double)fabsf(e0);  // the absolute error
          if (TRAIN) dl = e0 * inv_mb;
        }
      }
      if (TRAIN) d3[row * MD_CP + li] = dl;
    }
  }

  // ---- backward: hidden deltas, both weight gradients ----
  __device__ __forceinline__ void backward(int nrt, f32x4 (&acc)[2][4], f32x4 (&accg)[2][KT], f32x4 (&g2)[2], float& gb2) const {
    const int t_ = tid(), lane = t_ & 63, w = t_ >> 6, li = lane & 15, q = lane >> 4;
    const int nut = y.HP / 16, ldw = y.ldw;
    const float* s = f(y.o_xs);
    const float* w2 = f(y.o_w2);
    const float* d3 = f(y.o_d3);
    float wt[2][4];  // B[k = out 4s+q][n = unit li] = w2[unit][out]
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
      for (int sN = 0; sN < 4; sN++) wt[i][sN] = w + 8 * i < nut ? w2[((w + 8 * i) * 16 + li) * MD_CP + 4 * sN + q] : 0.f;
#pragma unroll
    for (int r = 0; r < 4; r++)
      if (r < nrt) {
        float da[4], db[4];
#pragma unroll
        for (int sN = 0; sN < 4; sN++) da[sN] = d3[(r * 16 + li) * MD_CP + 4 * sN + q];  // A[m = row li][k = out 4s+q]
#pragma unroll
        for (int e = 0; e < 4; e++) db[e] = d3[(r * 16 + 4 * q + e) * MD_CP + li];        // B[k = row 4q+e][n = out li]
        if (w == 0) {  // output bias gradient: column sums of the delta
#pragma unroll
          for (int e = 0; e < 4; e++) gb2 += db[e];
        }
        f32x4 dh[2];
#pragma unroll
        for (int i = 0; i < 2; i++) {
          dh[i] = f32x4{0.f, 0.f, 0.f, 0.f};
          if (w + 8 * i < nut) {
#pragma unroll
            for (int sN = 0; sN < 4; sN++) dh[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(da[sN], wt[i][sN], dh[i], 0, 0, 0);
#pragma unroll
            for (int e = 0; e < 4; e++) {
              const float av = acc[i][r][e];
              // output layer: D[unit][out] += a[row][unit] . delta[row][out]
              g2[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, db[e], g2[i], 0, 0, 0);
              dh[i][e] = av > 0.f ? dh[i][e] : 0.f;
            }
          }
        }
        // hidden layer: D[k][unit] += xs[row][k] . dh[row][unit]
#pragma unroll
        for (int m = 0; m < KT; m++) {
          float xa[4];
#pragma unroll
          for (int e = 0; e < 4; e++) xa[e] = s[(r * 16 + 4 * q + e) * ldw + m * 16 + li];
#pragma unroll
          for (int i = 0; i < 2; i++)
            if (w + 8 * i < nut) {
#pragma unroll
              for (int e = 0; e < 4; e++)
                accg[i][m] = __builtin_amdgcn_mfma_f32_16x16x4f32(xa[e], dh[i][e], accg[i][m], 0, 0, 0);
            }
        }
      }
  }

  // ---- optimizer step ----
  template <bool ADAM>
  __device__ __forceinline__ void update(const OptC& oc, const f32x4 (&accg)[2][KT], const f32x4 (&g2)[2], float gb2, float* rec) const {
    const int t_ = tid(), lane = t_ & 63, w = t_ >> 6, li = lane & 15, q = lane >> 4;
    const int nut = y.HP / 16, ldw = y.ldw, d = y.d, h = y.h, c = y.c;
    float* w1 = f(y.o_w1);
    float* m1 = g(y.g_m1);
    float* v1 = g(y.g_v1);
    OptC cc = oc;
    cc.adam = ADAM;
    // every load of a moment is issued before the first is used: one exposed L2 latency per step, not three
    float* w2 = f(y.o_w2);
    float* m2 = g(y.g_m2);
    float* v2 = g(y.g_v2);
    float m2r[2][4], v2r[2][4], mb = 0.f, vb = 0.f;
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
      for (int e = 0; e < 4; e++) {
        const int u = (w + 8 * i) * 16 + 4 * q + e;
        m2r[i][e] = v2r[i][e] = 0.f;
        if (w + 8 * i < nut && li < c && u < h) {
          m2r[i][e] = m2[u * MD_CP + li];
          if (ADAM) v2r[i][e] = v2[u * MD_CP + li];
        }
      }
    if (w == 0 && q == 0 && li < c) {
      mb = m2[y.HP * MD_CP + li];
      if (ADAM) vb = v2[y.HP * MD_CP + li];
    }
    // hidden layer: the lane holds gradient elements (unit j = tile*16 + li, columns k0..k0+3)
    f32x4 m1r[2][KT], v1r[2][KT];
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
      for (int m = 0; m < KT; m++) {
        const int j = (w + 8 * i) * 16 + li, k0 = m * 16 + 4 * q;
        m1r[i][m] = v1r[i][m] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (w + 8 * i < nut && j < h && k0 <= d) {
          m1r[i][m] = *(const f32x4*)(m1 + j * ldw + k0);
          if (ADAM) v1r[i][m] = *(const f32x4*)(v1 + j * ldw + k0);
        }
      }
#pragma unroll
    for (int i = 0; i < 2; i++)
      if (w + 8 * i < nut) {
        const int j = (w + 8 * i) * 16 + li;
#pragma unroll
        for (int m = 0; m < KT; m++) {
          const int k0 = m * 16 + 4 * q;
          if (j < h && k0 <= d) {
            const int o = j * ldw + k0;
            f32x4 wv = *(const f32x4*)(w1 + o);
            f32x4 mv = m1r[i][m], vv = v1r[i][m], gv;
#pragma unroll
            for (int e = 0; e < 4; e++) {
              const int k = k0 + e;
              float wr = wv[e], mr = mv[e], vr = vv[e];
              gv[e] = accg[i][m][e] + (k < d ? cc.am * wr : 0.f);  // column d is the bias: no penalty
              opt_update(cc, gv[e], wr, mr, vr);
              const bool real = k <= d;
              wv[e] = real ? wr : wv[e];
              mv[e] = real ? mr : mv[e];
              vv[e] = real ? vr : vv[e];
            }
            *(f32x4*)(w1 + o) = wv;
            *(f32x4*)(m1 + o) = mv;
            if (ADAM) *(f32x4*)(v1 + o) = vv;
            if (rec) {
#pragma unroll
              for (int e = 0; e < 4; e++)
                if (k0 + e <= d) {
                  const int ci = ci_hidden(j, k0 + e);
                  rec[1 + ci] = gv[e];
                  rec[1 + y.P + ci] = wv[e];
                }
            }
          }
        }
      }
    // output layer: the lane holds gradient elements (units tile*16 + 4q + e, out li)
#pragma unroll
    for (int i = 0; i < 2; i++)
      if (w + 8 * i < nut && li < c) {
#pragma unroll
        for (int e = 0; e < 4; e++) {
          const int u = (w + 8 * i) * 16 + 4 * q + e;
          if (u < h) {
            const int o = u * MD_CP + li;
            float wr = w2[o], mr = m2r[i][e], vr = v2r[i][e];
            const float gg = g2[i][e] + cc.am * wr;
            opt_update(cc, gg, wr, mr, vr);
            w2[o] = wr;
            m2[o] = mr;
            if (ADAM) v2[o] = vr;
            if (rec) {
              const int ci = y.cw[1] + u * c + li;
              rec[1 + ci] = gg;
              rec[1 + y.P + ci] = wr;
            }
          }
        }
      }
    if (w == 0) {  // output bias: the lane's partial covers the rows of its lane group
      float gb = gb2;
      gb += __shfl_xor(gb, 16);
      gb += __shfl_xor(gb, 32);
      if (q == 0 && li < c) {
        const int o = y.HP * MD_CP + li;
        float wr = w2[o], mr = mb, vr = vb;
        opt_update(cc, gb, wr, mr, vr);
        w2[o] = wr;
        m2[o] = mr;
        if (ADAM) v2[o] = vr;
        if (rec) {
          rec[1 + y.cb[1] + li] = gb;
          rec[1 + y.P + y.cb[1] + li] = wr;
        }
      }
    }
  }

  __device__ __forceinline__ double penalty_sum() const {
    double s = 0.0;
    const float* w1 = f(y.o_w1);
    const float* w2 = f(y.o_w2);
    for (int i = threadIdx.x; i < y.d * y.h; i += blockDim.x) {
      const float w = w1[(i / y.d) * y.ldw + i % y.d];
      s += (double)w * (double)w;
    }
    for (int i = threadIdx.x; i < y.h * y.c; i += blockDim.x) {
      const float w = w2[(i / y.c) * MD_CP + i % y.c];
      s += (double)w * (double)w;
    }
    return block_sum(s, red);
  }

  __device__ __forceinline__ void run() const {
    const int f_ = it.fold, fl = it.fold - P.fold_base;  // fl: which row list
    const int n_tr = P.counts[2 * fl], n_va = P.counts[2 * fl + 1];
    const int32_t* tr = P.train_idx + (int64_t)fl * P.n;
    const int32_t* va = P.val_idx + (int64_t)fl * P.n;
    const uint64_t km = key_model(it.seed, f_);
    const RowSplit sp = row_split(km, it.patience, it.val_frac, n_tr);
    const int n_fit = sp.n_fit;
    const int bs = eff_batch(it.batch_size, n_fit);
    const int steps = n_fit > 0 ? (n_fit + bs - 1) / bs : 0;
    const bool traced = P.trace_item == it.b * P.n_folds + fl;

    // zero the weights, input tile and exchange buffers (pads must be zero), and the moments
    {
      uint4* z = (uint4*)lds;
      const uint32_t n16 = y.o_rows / 16;
      for (uint32_t i = threadIdx.x; i < n16; i += blockDim.x) z[i] = uint4{0, 0, 0, 0};
      uint4* zg = (uint4*)slot;
      const uint32_t g16 = y.g_zero / 16;
      for (uint32_t i = threadIdx.x; i < g16; i += blockDim.x) zg[i] = uint4{0, 0, 0, 0};
    }
    double b1t = 1.0, b2t = 1.0;
    int64_t gstep = 0;
    ChunkPos pos = {0, 0, 0};
    const bool resume = traced && P.state_in && steps > 0;
    if (resume) {
      gstep = P.step_begin;
      pos.e = (int)(gstep / steps);
      pos.st = (int)(gstep % steps);
      for (int64_t i = 0; i < gstep; i++) {  // beta^gstep by repeated products, as the free run builds it
        b1t *= (double)it.beta1;
        b2t *= (double)it.beta2;
      }
    }
    __syncthreads();  // zeroed moments before a resumed state overwrites them
    put_weights(resume ? P.state_in : nullptr);
    __syncthreads();

    OptC oc;
    oc.adam = it.solver == BBO_ADAM;
    oc.nest = it.nesterov != 0;
    oc.b1 = it.beta1;
    oc.b2 = it.beta2;
    oc.omb1 = 1.f - it.beta1;
    oc.omb2 = 1.f - it.beta2;
    oc.eps = it.eps;
    oc.mu = it.momentum;
    oc.lr = it.lr;
    oc.lr_t = it.lr;

    // ---- training: the chunks of all steps of all epochs, inputs fetched one chunk ahead ----
    int epochs_lim = it.epochs;  // lowered when a stopping rule ends training
    auto chunk_valid = [&](const ChunkPos& p) { return steps > 0 && p.e < epochs_lim; };
    auto chunk_rows = [&](const ChunkPos& p) { return min(MD_RC, min(bs, n_fit - p.st * bs) - p.c0); };
    auto chunk_next = [&](ChunkPos p) {
      const int mb = min(bs, n_fit - p.st * bs);
      p.c0 += MD_RC;
      if (p.c0 >= mb) {
        p.c0 = 0;
        if (++p.st >= steps) {
          p.st = 0;
          p.e++;
        }
      }
      return p;
    };
    auto chunk_row_id = [&](const ChunkPos& p) {
      return fetch_row_id(tr, sp, ROWS_EPOCH, key_epoch(km, p.e), p.st * bs + p.c0, chunk_rows(p));
    };
    float xr[NX], yv = 0.f;
    int par = 0;
    if (chunk_valid(pos)) {
      if (y.epoch_cap) {
        build_epoch_table(tr, sp, key_epoch(km, pos.e));
        __syncthreads();
      }
      park_row_id(0, chunk_row_id(pos));
      __syncthreads();
      fetch_inputs(0, xr, yv);
    }
    f32x4 acc[2][4], accg[2][KT], g2[2];
    float gb2 = 0.f;
    double lsum = 0.0, hits = 0.0, pen = 0.0, esum = 0.0;  // esum: the lane's share of the epoch's summed data loss
    float* rec = nullptr;
    Plateau plateau;
    bool have_best = false;
    const bool watch = it.patience > 0 && !resume;
    // Loss and second score (the thread's share) of `count` rows of a list under the current weights.
    auto score_rows = [&](const int32_t* list, int mode, int count, double& ls, double& hs) {
      for (int off = 0; off < count; off += MD_RC) {
        const int rows = min(MD_RC, count - off), nrt = (rows + 15) / 16;
        park_row_id(0, fetch_row_id(list, sp, mode, 0, off, rows));
        __syncthreads();
        fetch_inputs(0, xr, yv);
        commit_inputs(0, xr, yv);
        __syncthreads();
        forward(nrt, acc);
        __syncthreads();
        outputs<false>(0, rows, nrt, 0.f, ls, hs);
        __syncthreads();
      }
    };
    while (chunk_valid(pos)) {
      const int mb = min(bs, n_fit - pos.st * bs);
      const int rows = chunk_rows(pos), nrt = (rows + 15) / 16;
      if (pos.c0 == 0) {  // first chunk of a step
        oc.am = it.alpha / (float)mb;
        if (!oc.adam) oc.lr = epoch_lr(it.lr, it.power_t, pos.e, n_fit);
        if (oc.adam) {
          b1t *= (double)it.beta1;
          b2t *= (double)it.beta2;
          oc.lr_t = (float)((double)it.lr * sqrt(1.0 - b2t) / (1.0 - b1t));
        }
        rec = nullptr;
        if (traced && gstep >= P.step_begin && gstep < P.step_end)
          rec = P.trace_out + (gstep - P.step_begin) * (1 + 2 * (int64_t)y.P);
        if (rec) {
          __syncthreads();  // the previous step's update, by every wave
          pen = penalty_sum();
        }
        lsum = 0.0;
#pragma unroll
        for (int i = 0; i < 2; i++) {
          g2[i] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int m = 0; m < KT; m++) accg[i][m] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        gb2 = 0.f;
      }
      commit_inputs(par, xr, yv);
      const ChunkPos nxt = chunk_next(pos);
      const bool more = chunk_valid(nxt);
      if (more && nxt.e != pos.e && y.epoch_cap) {
        // the next chunk opens an epoch: its row order replaces the table (this epoch's last rows are already read)
        build_epoch_table(tr, sp, key_epoch(km, nxt.e));
        __syncthreads();
      }
      int nrow = -1;
      if (more) nrow = chunk_row_id(nxt);  // load in flight across the forward phase
      __syncthreads();                     // inputs of this chunk (and last step's weights) visible
      forward(nrt, acc);
      if (more) park_row_id(par ^ 1, nrow);
      __syncthreads();  // all partial outputs, and the next chunk's row ids, visible
      if (more) fetch_inputs(par ^ 1, xr, yv);  // in flight across the rest of the chunk
      outputs<true>(par, rows, nrt, 1.f / (float)mb, lsum, hits);
      __syncthreads();  // output deltas visible
      backward(nrt, acc, accg, g2, gb2);
      __syncthreads();  // every wave is done with the input tile, the deltas and the output bias
      if (nxt.c0 == 0) {  // that was the last chunk of the step
        if (oc.adam)
          update<true>(oc, accg, g2, gb2, rec);
        else
          update<false>(oc, accg, g2, gb2, rec);
        if (rec) {
          const double data = block_sum(lsum, red) / (double)mb;
          if (threadIdx.x == 0) rec[0] = (float)(data + 0.5 * (double)it.alpha * pen / (double)mb);
        }
        gstep++;
        esum += lsum;
        if (watch && nxt.e != pos.e) {  // that was the last step of the epoch
          float watched;
          if (sp.n_hold) {
            // the loss of the rows set aside for early stopping, under the weights the epoch ends with; the
            // pass takes over the input tile, so the next chunk's rows and inputs are fetched again after it
            __syncthreads();  // the update, by every wave
            double hl = 0.0, hh = 0.0;
            score_rows(tr, ROWS_HELD, sp.n_hold, hl, hh);
            watched = (float)(block_sum(hl, red) / (double)sp.n_hold);
            if (more) {
              park_row_id(par ^ 1, chunk_row_id(nxt));
              __syncthreads();
              fetch_inputs(par ^ 1, xr, yv);
            }
          } else {
            watched = (float)(block_sum(esum, red) / (double)n_fit);
          }
          if (plateau.stop_after(watched, it.tol, it.patience)) epochs_lim = pos.e + 1;
          if (sp.n_hold && plateau.improved) {  // (the scoring pass ended with a barrier: the weights are at rest)
            copy_best(true);
            have_best = true;
          }
          esum = 0.0;
        }
      }
      pos = nxt;
      par ^= 1;
    }
    __syncthreads();
    if (have_best) {  // early stopping on held-out rows scores the best epoch's model
      copy_best(false);
      __syncthreads();
    }

    // ---- validation score on the held rows ----
    lsum = 0.0;
    hits = 0.0;
    score_rows(va, ROWS_PLAIN, n_va, lsum, hits);
    lsum = block_sum(lsum, red);
    hits = block_sum(hits, red);
    if (threadIdx.x == 0) {
      float* out = P.item_out + 2 * ((int64_t)it.b * P.n_folds + fl);
      out[0] = n_va > 0 ? (float)(lsum / (double)n_va) : __builtin_nanf("");
      out[1] = n_va > 0 ? (float)(hits / (double)n_va) : __builtin_nanf("");  // accuracy | mean absolute error
    }
  }
};

template <int KT>
__global__ __launch_bounds__(MD_THREADS) void k_train_mid(const TrainParams P) {
  extern __shared__ __align__(16) char smem[];
  __shared__ int s_item;
  __shared__ double red[MD_THREADS / 64];
  for (;;) {
    __syncthreads();
    if (threadIdx.x == 0) s_item = atomicAdd(P.queue, 1);
    __syncthreads();
    const int item = __builtin_amdgcn_readfirstlane(s_item);
    if (item >= P.n_items) break;
    const MItem* __restrict__ mi = (const MItem*)P.items + item;
    Mid<KT> T{P, mi->d, mi->y, smem, P.slots + (uint64_t)blockIdx.x * P.slot_bytes, red};
    T.run();
  }
}

}  // namespace
