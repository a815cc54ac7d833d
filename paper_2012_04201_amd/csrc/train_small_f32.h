// LDS-resident training / scoring kernel for small fp32 models with one hidden
// layer (the "many concurrent studies" shape: up to 63 inputs, hidden width up
// to 224, up to 4 outputs).
//
// One workgroup (4 waves) trains one model, and the model never leaves the
// chip: the weights of both layers stay in LDS for all epochs and the
// minibatch is processed in chunks of 64 rows.  The hidden layer's optimizer
// moments are the one thing kept in global memory (a per-workgroup slot that
// stays L2-resident, read and written once per step in the update); HBM is
// otherwise touched only for the gathered input rows, fetched one chunk ahead
// into registers.  The LDS footprint stays under half a CU's LDS so that two
// workgroups share a CU and cover each other's barriers.
//
// Each wave owns the same hidden-unit tiles in every phase, so the hidden
// activations never leave its registers:
//   phase 1  forward MFMA (16x16x4 fp32): D[row][unit] = xs[row][k] . w1[unit][k]
//            (bias rides in column d of xs/w1), ReLU in the accumulators; the
//            wave's share of the output layer is reduced over its 16 unit lanes
//            with DPP adds and parked in LDS (4 KB);
//   phase 2  every wave sums the four shares for all 64 rows (lane = row),
//            takes softmax / loss / output delta, then turns its accumulators
//            into hidden deltas in place and feeds them straight back to the
//            MFMA as the B operand of the weight gradient, D[k][unit] += xt[k][row]
//            . delta[unit][row], accumulated over the chunks of the step in
//            registers; the optimizer update reads the gradient from those
//            registers and the weights from LDS.
// Two block-wide barriers per chunk (the input-major tile is double-buffered).
//
// LDS (floats; rows padded by 4 against bank conflicts):
//   xs[row][k], xt[2][k][row]     gathered inputs, both orders; column d = 1 on real rows
//   w1[unit][k]                   hidden layer, bias in column d
//   w2, m2, v2 [unit][4]          output layer and its moments, bias in row HP
//   zp[wave][row][4], d2[wave][row][4], ys[2][row], row ids, the epoch's row order
#pragma once
#include "common.h"
#include "train_tiled_bf16.h"  // OptC, opt_update

namespace {

constexpr int SM_THREADS = 256;
constexpr int SM_RC = 64;                          // rows per chunk
constexpr uint32_t SM_LDS_LIMIT = 80 * 1024 - 64;  // per workgroup: two workgroups per CU

struct SLay {
  int32_t d, h, c, K0, HP, ldw, lda;
  int32_t cw[2], cb[2], P;
  uint32_t o_w1, o_w2, o_m2, o_v2, o_xs, o_xt, o_zp, o_d2, o_rows, o_ys, o_epoch, lds_total;
  int32_t epoch_cap;  // entries of the per-epoch row table in LDS (0: rows are permuted on the fly)
};

struct SItem {
  ItemDesc d;
  SLay y;
};

__host__ __device__ inline bool small_eligible(const int32_t* dims, int L) {
  return L == 2 && dims[0] <= 63 && dims[1] <= 224 && dims[2] <= 4;
}

__host__ __device__ inline void make_slay(SLay& y, const int32_t* dims, int64_t n) {
  y.d = dims[0];
  y.h = dims[1];
  y.c = dims[2];
  y.K0 = dims[0] + 1 <= 16 ? 16 : (dims[0] + 1 <= 32 ? 32 : 64);
  y.HP = rup(dims[1], 16);
  y.ldw = y.K0 + 4;
  y.lda = SM_RC + 4;
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
  y.o_w2 = take((y.HP + 1) * 4);
  y.o_m2 = take((y.HP + 1) * 4);
  y.o_v2 = take((y.HP + 1) * 4);
  y.o_xs = take(SM_RC * y.ldw);
  y.o_xt = take(2 * y.K0 * y.lda);
  y.o_zp = take(4 * SM_RC * 4);
  y.o_d2 = take(4 * SM_RC * 4);
  y.o_rows = take(2 * SM_RC);
  y.o_ys = take(2 * SM_RC);
  y.o_epoch = o;
  y.epoch_cap = 0;
  if (n <= 4096 && o + 4 * (uint32_t)n + 16 <= SM_LDS_LIMIT) {
    y.epoch_cap = (int32_t)n;
    o += (4 * (uint32_t)n + 15) & ~15u;
  }
  y.lds_total = o;
}

// Sum over the 16 lanes of a DPP row; every lane gets the total.
__device__ inline float row16_sum(float v) {
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x128, 0xf, 0xf, false));
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x124, 0xf, 0xf, false));
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xf, 0xf, false));
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xf, 0xf, false));
  return v;
}

// Position in the training schedule: epoch, step of the epoch, first row of
// the chunk within the step's minibatch.
struct ChunkPos {
  int e, st, c0;
};

// KT: 16-wide k tiles of the input layer (inputs + bias).  CO: output slots in use (1, 2 or 4); 1 and 2 are
// exact output counts, 4 serves 3 or 4 outputs.
template <int KT, int CO>
struct Small {
  static constexpr int K0 = 16 * KT, RSTEP = SM_THREADS / K0, NX = SM_RC / RSTEP;
  const TrainParams& P;
  const ItemDesc& it;
  const SLay& y;
  char* lds;
  char* slot;  // global: m1[unit][k], v1[unit][k]
  double* red;

  __device__ float* f(uint32_t off) const { return (float*)(lds + off); }
  __device__ float* m1g() const { return (float*)slot; }
  __device__ float* v1g() const { return (float*)slot + y.HP * y.ldw; }
  // weights of the best epoch so far (early stopping on held-out rows): both layers, as they lie in LDS
  __device__ float* bestg() const { return (float*)slot + 2 * y.HP * y.ldw; }
  // Keep the current weights aside / put the kept ones back.  Block-wide; the caller orders it against updates.
  __device__ __forceinline__ void copy_best(bool keep) const {
    float* w1 = f(y.o_w1);
    float* w2 = f(y.o_w2);
    float* b = bestg();
    const int n1 = y.HP * y.ldw, n2 = (y.HP + 1) * 4;
    for (int i = threadIdx.x; i < n1 + n2; i += blockDim.x) {
      float* l = i < n1 ? w1 + i : w2 + (i - n1);
      if (keep)
        b[i] = *l;
      else
        *l = b[i];
    }
  }
  __device__ int32_t* rowlist(int par) const { return (int32_t*)(lds + y.o_rows) + par * SM_RC; }
  __device__ float* xt(int par) const { return f(y.o_xt) + par * K0 * y.lda; }
  __device__ float* ys(int par) const { return f(y.o_ys) + par * SM_RC; }

  // packed index (W1[in][out], b1, W2[in][out], b2) of hidden-layer element (unit j, column k); -1 for pads
  __device__ __forceinline__ int ci_hidden(int j, int k) const {
    if (j >= y.h || k > y.d) return -1;
    return k < y.d ? y.cw[0] + k * y.h + j : y.cb[0] + j;
  }
  // The thread index as a value the compiler cannot see through: lane coordinates and the addresses derived
  // from them are recomputed in each phase instead of being kept in registers for the whole run.
  __device__ __forceinline__ static int tid() {
    int t = threadIdx.x;
    asm volatile("" : "+v"(t));
    return t;
  }
  __device__ __forceinline__ float init_value(int l, int e, bool isb) const {
    const uint64_t kt = key_fold(key_model(it.seed, it.fold), 16 + 2 * l + (isb ? 1 : 0));
    const uint32_t k24 = (uint32_t)(key_fold(kt, (uint64_t)e) >> 40);
    return it.bound[l] * ((float)((int32_t)k24 - 8388608) * 0x1p-23f);
  }

  // Weights (and the output layer's moments) into LDS, from the initial draw or from a packed state.
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
          m1g()[o] = st[y.P + ci];
          v1g()[o] = st[2 * y.P + ci];
        }
      } else {
        const bool isb = ci >= y.cb[1];
        const int e = isb ? ci - y.cb[1] : ci - y.cw[1];
        const int o = isb ? y.HP * 4 + e : (e / c) * 4 + e % c;
        w2[o] = st ? st[ci] : init_value(1, e, isb);
        if (st) {
          f(y.o_m2)[o] = st[y.P + ci];
          f(y.o_v2)[o] = st[2 * y.P + ci];
        }
      }
    }
  }

  // ---- input staging, one chunk ahead ---------------------------------------
  // (1) row ids of a chunk: the load is issued here, the value parked in LDS later
  __device__ __forceinline__ int fetch_row_id(const int32_t* list, const RowSplit& sp, int mode, uint64_t key, int lo,
                                              int rows) const {
    const int p = threadIdx.x;
    if (p >= SM_RC || p >= rows) return -1;
    if (mode == ROWS_EPOCH && y.epoch_cap) return ((const int32_t*)(lds + y.o_epoch))[lo + p];
    return list[row_index(sp, mode, key, (uint32_t)(lo + p))];
  }
  // Row ids of a whole epoch, in minibatch order, into the LDS table.
  __device__ __forceinline__ void build_epoch_table(const int32_t* list, const RowSplit& sp, uint64_t key) const {
    int32_t* tab = (int32_t*)(lds + y.o_epoch);
    for (int p = threadIdx.x; p < sp.n_fit; p += blockDim.x) tab[p] = list[fit_index(sp, key, (uint32_t)p)];
  }
  __device__ __forceinline__ void park_row_id(int par, int row) const {
    if ((int)threadIdx.x < SM_RC) rowlist(par)[threadIdx.x] = row;
  }
  // (2) the chunk's input values (and label) into registers
  __device__ __forceinline__ void fetch_inputs(int par, float (&xr)[NX], float& yv) const {
    const int32_t* rl = rowlist(par);
    const float* X = (const float*)P.X;
    const int t_ = tid(), k = t_ % K0, r0 = t_ / K0, d = y.d;
#pragma unroll
    for (int i = 0; i < NX; i++) {
      const int row = rl[r0 + i * RSTEP];
      xr[i] = 0.f;
      if (row >= 0) xr[i] = k < d ? X[row * d + k] : (k == d ? 1.f : 0.f);  // n*d < 2^31 (checked by the host)
    }
    yv = 0.f;
    if ((int)threadIdx.x < SM_RC) {
      const int row = rl[threadIdx.x];
      if (row >= 0) yv = P.n_classes >= 1 ? __int_as_float(((const int32_t*)P.y)[row]) : ((const float*)P.y)[row];
    }
  }
  // (3) registers -> the LDS tiles (the input-major tile and the labels of parity par)
  __device__ __forceinline__ void commit_inputs(int par, const float (&xr)[NX], float yv) const {
    float* s = f(y.o_xs);
    float* t = xt(par);
    const int t_ = tid(), k = t_ % K0, r0 = t_ / K0;
#pragma unroll
    for (int i = 0; i < NX; i++) {
      const int r = r0 + i * RSTEP;
      s[r * y.ldw + k] = xr[i];
      t[k * y.lda + r] = xr[i];
    }
    if ((int)threadIdx.x < SM_RC) ys(par)[threadIdx.x] = yv;
  }

  // ---- phase 1: hidden layer forward; the wave's share of the outputs -> zp ----
  // A full chunk (all four row tiles): one straight-line block per unit tile of the wave, with the input
  // operands of all row tiles in registers, so that the ReLU and output-layer arithmetic of one row tile can
  // be issued while the MFMAs of the next are in flight.  Same order of every accumulation as forward().
  __device__ __forceinline__ void forward_full(f32x4 (&acc)[4][4]) const {
    const int t_ = tid(), lane = t_ & 63, w = t_ >> 6, li = lane & 15, q = lane >> 4;
    const int nut = y.HP / 16, ldw = y.ldw;
    const float* s = f(y.o_xs);
    const float* w1 = f(y.o_w1);
    constexpr bool c2 = CO >= 2, c4 = CO >= 4;
    f32x4 a[4][KT];
#pragma unroll
    for (int r = 0; r < 4; r++)
#pragma unroll
      for (int kk = 0; kk < KT; kk++) a[r][kk] = *(const f32x4*)(s + (r * 16 + li) * ldw + kk * 16 + 4 * q);
    float pz[4][4][CO];  // [row tile][row 4q+e][output]
#pragma unroll
    for (int r = 0; r < 4; r++)
#pragma unroll
      for (int e = 0; e < 4; e++)
#pragma unroll
        for (int cc = 0; cc < CO; cc++) pz[r][e][cc] = 0.f;
#pragma unroll
    for (int i = 0; i < 4; i++) {
#pragma unroll
      for (int r = 0; r < 4; r++) acc[i][r] = f32x4{0.f, 0.f, 0.f, 0.f};
      if (w + 4 * i < nut) {
        f32x4 b[KT];
#pragma unroll
        for (int kk = 0; kk < KT; kk++) b[kk] = *(const f32x4*)(w1 + ((w + 4 * i) * 16 + li) * ldw + kk * 16 + 4 * q);
        const f32x4 w2 = *(const f32x4*)(f(y.o_w2) + ((w + 4 * i) * 16 + li) * 4);
#pragma unroll
        for (int r = 0; r < 4; r++) {
#pragma unroll
          for (int kk = 0; kk < KT; kk++)
#pragma unroll
            for (int e = 0; e < 4; e++)
              acc[i][r] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[r][kk][e], b[kk][e], acc[i][r], 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < 4; r++)
#pragma unroll
          for (int e = 0; e < 4; e++) {
            const float av = fmaxf(acc[i][r][e], 0.f);
            acc[i][r][e] = av;
            pz[r][e][0] += av * w2[0];
            if (c2) pz[r][e][1] += av * w2[1];
            if (c4) {
              pz[r][e][2] += av * w2[2];
              pz[r][e][3] += av * w2[3];
            }
          }
      }
    }
    float* zp = f(y.o_zp) + w * SM_RC * 4;
#pragma unroll
    for (int r = 0; r < 4; r++) {
      f32x4 o[4];
#pragma unroll
      for (int e = 0; e < 4; e++) {
        o[e] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int cc = 0; cc < CO; cc++) o[e][cc] = row16_sum(pz[r][e][cc]);
      }
      if (li == 0) {
#pragma unroll
        for (int e = 0; e < 4; e++) *(f32x4*)(zp + (r * 16 + 4 * q + e) * 4) = o[e];
      }
    }
  }

  __device__ __forceinline__ void forward(int nrt, f32x4 (&acc)[4][4]) const {
    if (KT <= 2 && CO <= 2 && nrt == 4) {
      forward_full(acc);
      return;
    }
    const int t_ = tid(), lane = t_ & 63, w = t_ >> 6, li = lane & 15, q = lane >> 4;
    const int nut = y.HP / 16, ldw = y.ldw;
    const float* s = f(y.o_xs);
    const float* w1 = f(y.o_w1);
    constexpr bool c2 = CO >= 2, c4 = CO >= 4;
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
      for (int r = 0; r < 4; r++) acc[i][r] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < KT; kk++) {
      f32x4 a[4], b[4];
#pragma unroll
      for (int r = 0; r < 4; r++)
        if (r < nrt) a[r] = *(const f32x4*)(s + (r * 16 + li) * ldw + kk * 16 + 4 * q);
#pragma unroll
      for (int i = 0; i < 4; i++)
        if (w + 4 * i < nut) b[i] = *(const f32x4*)(w1 + ((w + 4 * i) * 16 + li) * ldw + kk * 16 + 4 * q);
#pragma unroll
      for (int i = 0; i < 4; i++)
        if (w + 4 * i < nut) {
#pragma unroll
          for (int r = 0; r < 4; r++)
            if (r < nrt) {
#pragma unroll
              for (int e = 0; e < 4; e++)
                acc[i][r] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[r][e], b[i][e], acc[i][r], 0, 0, 0);
            }
        }
    }
    // ReLU, and the output layer restricted to this wave's units: lane (unit li, rows 4q..4q+3)
    f32x4 w2r[4];
#pragma unroll
    for (int i = 0; i < 4; i++)
      w2r[i] = w + 4 * i < nut ? *(const f32x4*)(f(y.o_w2) + ((w + 4 * i) * 16 + li) * 4) : f32x4{0.f, 0.f, 0.f, 0.f};
    float* zp = f(y.o_zp) + w * SM_RC * 4;
#pragma unroll
    for (int r = 0; r < 4; r++)
      if (r < nrt) {
        f32x4 pz[4];  // [row 4q+e][output]
#pragma unroll
        for (int e = 0; e < 4; e++) pz[e] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < 4; i++)
          if (w + 4 * i < nut) {
#pragma unroll
            for (int e = 0; e < 4; e++) {
              const float av = fmaxf(acc[i][r][e], 0.f);
              acc[i][r][e] = av;
              pz[e][0] += av * w2r[i][0];
              if (c2) pz[e][1] += av * w2r[i][1];
              if (c4) {
                pz[e][2] += av * w2r[i][2];
                pz[e][3] += av * w2r[i][3];
              }
            }
          }
#pragma unroll
        for (int e = 0; e < 4; e++) {
          pz[e][0] = row16_sum(pz[e][0]);
          if (c2) pz[e][1] = row16_sum(pz[e][1]);
          if (c4) {
            pz[e][2] = row16_sum(pz[e][2]);
            pz[e][3] = row16_sum(pz[e][3]);
          }
        }
        if (li == 0) {
#pragma unroll
          for (int e = 0; e < 4; e++) *(f32x4*)(zp + (r * 16 + 4 * q + e) * 4) = pz[e];
        }
      }
  }

  // ---- phase 2a: outputs, loss and output delta of all 64 rows (lane = row), per wave ----
  template <bool TRAIN>
  __device__ __forceinline__ void outputs(int par, int rows, float inv_mb, double& lsum, double& hits, f32x4& gb2) const {
    const int t_ = tid(), lane = t_ & 63, w = t_ >> 6, c = CO <= 2 ? CO : y.c;
    const float* zp = f(y.o_zp);
    const f32x4 b2 = *(const f32x4*)(f(y.o_w2) + y.HP * 4);
    float z0 = b2[0], z1 = b2[1], z2 = b2[2], z3 = b2[3];
#pragma unroll
    for (int ww = 0; ww < 4; ww++) {
      const f32x4 pv = *(const f32x4*)(zp + (ww * SM_RC + lane) * 4);
      z0 += pv[0];
      z1 += pv[1];
      z2 += pv[2];
      z3 += pv[3];
    }
    const float z[4] = {z0, z1, z2, z3};
    const float yv = ys(par)[lane];
    f32x4 dl = f32x4{0.f, 0.f, 0.f, 0.f};
    if (lane < rows) {
      double l = 0.0;
      double hit = 0.0;  // a correct prediction, or the absolute error
      if (P.n_classes >= 2) {
        const int yr = __float_as_int(yv);
        float mx = z[0], zy = z[0];
        int best = 0;
#pragma unroll
        for (int cc = 1; cc < CO; cc++)
          if (cc < c) {
            if (z[cc] > mx) {
              mx = z[cc];
              best = cc;
            }
            zy = cc == yr ? z[cc] : zy;
          }
        float se = 0.f;
#pragma unroll
        for (int cc = 0; cc < CO; cc++)
          if (cc < c) se += expf(z[cc] - mx);
        const float lse = mx + logf(se);
        l = (double)(lse - zy);
        hit = best == yr ? 1.0 : 0.0;
        if (TRAIN) {
#pragma unroll
          for (int cc = 0; cc < CO; cc++)
            if (cc < c) dl[cc] = (expf(z[cc] - lse) - (cc == yr ? 1.f : 0.f)) * inv_mb;
        }
      } else if (P.n_classes == 1) {
        // one logit, labels 0/1: log(1 + e^z) - y z, delta (sigmoid(z) - y)/m
        const int yr = __float_as_int(yv);
        const float zz = z[0];
        l = (double)(fmaxf(zz, 0.f) + log1pf(expf(-fabsf(zz))) - (yr ? zz : 0.f));
        hit = (zz > 0.f) == (yr != 0) ? 1.0 : 0.0;
        if (TRAIN) dl[0] = (1.f / (1.f + expf(-zz)) - (float)yr) * inv_mb;
      } else {
        const float e0 = z[0] - yv;
        l = TRAIN ? 0.5 * (double)e0 * (double)e0 : (double)e0 * (double)e0;
        hit = (double)fabsf(e0);
        if (TRAIN) dl[0] = e0 * inv_mb;
      }
      if (w == 0) {  // every wave computes the same values; one of them keeps the statistics
        lsum += l;
        hits += hit;
      }
    }
    if (TRAIN) {
      *(f32x4*)(f(y.o_d2) + (w * SM_RC + lane) * 4) = dl;
      if (w == 0) {
#pragma unroll
        for (int cc = 0; cc < CO; cc++) gb2[cc] += dl[cc];
      }
      // the wave reads back what its other lanes wrote: LDS executes a wave's accesses in order
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }
  }

  // ---- phase 2b: hidden deltas in the accumulators, output-layer gradient, hidden weight gradient ----
  __device__ __forceinline__ void backward(int par, int nrt, f32x4 (&acc)[4][4], f32x4 (&accg)[4][KT], f32x4 (&g2p)[4]) const {
    const int t_ = tid(), lane = t_ & 63, w = t_ >> 6, li = lane & 15, q = lane >> 4;
    const int nut = y.HP / 16, lda = y.lda;
    const float* t = xt(par);
    const float* d2 = f(y.o_d2) + w * SM_RC * 4;
    constexpr bool c2 = CO >= 2, c4 = CO >= 4;
    f32x4 w2r[4];
#pragma unroll
    for (int i = 0; i < 4; i++)
      w2r[i] = w + 4 * i < nut ? *(const f32x4*)(f(y.o_w2) + ((w + 4 * i) * 16 + li) * 4) : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int r = 0; r < 4; r++)
      if (r < nrt) {
        f32x4 dv[4], a[KT];
#pragma unroll
        for (int e = 0; e < 4; e++) dv[e] = *(const f32x4*)(d2 + (r * 16 + 4 * q + e) * 4);
#pragma unroll
        for (int m = 0; m < KT; m++) a[m] = *(const f32x4*)(t + (m * 16 + li) * lda + r * 16 + 4 * q);
#pragma unroll
        for (int i = 0; i < 4; i++)
          if (w + 4 * i < nut) {
            f32x4 dh;
#pragma unroll
            for (int e = 0; e < 4; e++) {
              const float av = acc[i][r][e];
              float s = dv[e][0] * w2r[i][0];
              g2p[i][0] += av * dv[e][0];
              if (c2) {
                s += dv[e][1] * w2r[i][1];
                g2p[i][1] += av * dv[e][1];
              }
              if (c4) {
                s += dv[e][2] * w2r[i][2] + dv[e][3] * w2r[i][3];
                g2p[i][2] += av * dv[e][2];
                g2p[i][3] += av * dv[e][3];
              }
              dh[e] = av > 0.f ? s : 0.f;
            }
#pragma unroll
            for (int m = 0; m < KT; m++) {
#pragma unroll
              for (int e = 0; e < 4; e++)
                accg[i][m] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[m][e], dh[e], accg[i][m], 0, 0, 0);
            }
          }
      }
  }

  // ---- optimizer step: gradients (and hidden moments) in registers, weights in LDS ----
  // Hidden-layer update of the wave's tiles.  ADAM and TRACED are compile-time so that the element loop is
  // straight-line code: the L2 term and the pad columns are handled by selects, not branches.
  template <bool ADAM, bool TRACED>
  __device__ __forceinline__ void update_hidden(const OptC& oc, const f32x4 (&accg)[4][KT], float* rec) const {
    const int t_ = tid(), lane = t_ & 63, w = t_ >> 6, li = lane & 15, q = lane >> 4;
    const int nut = y.HP / 16, ldw = y.ldw, d = y.d, h = y.h;
    float* w1 = f(y.o_w1);
    float* m1 = m1g();
    float* v1 = v1g();
    OptC c = oc;
    c.adam = ADAM;
    // all moment loads of the wave first, so that their latency overlaps
    f32x4 m1r[4][KT], v1r[4][KT];
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
      for (int m = 0; m < KT; m++) {
        const int j = (w + 4 * i) * 16 + li, k0 = m * 16 + 4 * q;
        m1r[i][m] = v1r[i][m] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (w + 4 * i < nut && j < h && k0 <= d) {
          m1r[i][m] = *(const f32x4*)(m1 + j * ldw + k0);
          if (ADAM) v1r[i][m] = *(const f32x4*)(v1 + j * ldw + k0);
        }
      }
#pragma unroll
    for (int i = 0; i < 4; i++)
      if (w + 4 * i < nut) {
        const int j = (w + 4 * i) * 16 + li;
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
              gv[e] = accg[i][m][e] + (k < d ? c.am * wr : 0.f);  // column d is the bias: no penalty
              opt_update(c, gv[e], wr, mr, vr);
              const bool real = k <= d;
              wv[e] = real ? wr : wv[e];
              mv[e] = real ? mr : mv[e];
              vv[e] = real ? vr : vv[e];
            }
            *(f32x4*)(w1 + o) = wv;
            *(f32x4*)(m1 + o) = mv;
            if (ADAM) *(f32x4*)(v1 + o) = vv;
            if (TRACED) {
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
  }

  __device__ __forceinline__ void update(const OptC& oc, const f32x4 (&accg)[4][KT], f32x4 (&g2p)[4], f32x4 gb2, float* rec) const {
    const int t_ = tid(), lane = t_ & 63, w = t_ >> 6, li = lane & 15, q = lane >> 4;
    const int h = y.h, c = CO <= 2 ? CO : y.c;
    if (rec) {
      if (oc.adam)
        update_hidden<true, true>(oc, accg, rec);
      else
        update_hidden<false, true>(oc, accg, rec);
    } else {
      if (oc.adam)
        update_hidden<true, false>(oc, accg, rec);
      else
        update_hidden<false, false>(oc, accg, rec);
    }
    // output layer: finish the sums over the rows held by the four lane groups, lane group 0 updates
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
      for (int cc = 0; cc < CO; cc++) {
        float v = g2p[i][cc];
        v += __shfl_xor(v, 16);
        v += __shfl_xor(v, 32);
        g2p[i][cc] = v;
      }
    if (w == 0) {
#pragma unroll
      for (int cc = 0; cc < CO; cc++) {
        float v = gb2[cc];
#pragma unroll
        for (int s = 1; s < 64; s <<= 1) v += __shfl_xor(v, s);
        gb2[cc] = v;
      }
    }
#pragma unroll
    for (int i = 0; i < 5; i++) {
      // i < 4: unit (w+4i)*16+li by lane group 0; i == 4: the bias row by lane 0 of wave 0
      const bool isb = i == 4;
      const int u = isb ? y.HP : (w + 4 * (i & 3)) * 16 + li;
      const bool mine = isb ? (w == 0 && lane == 0) : (q == 0 && u < h);
      if (mine) {
        const f32x4 g = isb ? gb2 : g2p[i & 3];
        float* w2 = f(y.o_w2) + u * 4;
        float* m2 = f(y.o_m2) + u * 4;
        float* v2 = f(y.o_v2) + u * 4;
        f32x4 wv = *(const f32x4*)w2, mv = *(const f32x4*)m2, vv = *(const f32x4*)v2;
#pragma unroll
        for (int cc = 0; cc < CO; cc++)
          if (cc < c) {
            float wr = wv[cc], mr = mv[cc], vr = vv[cc];
            const float gg = isb ? g[cc] : g[cc] + oc.am * wr;
            opt_update(oc, gg, wr, mr, vr);
            if (rec) {
              const int ci = isb ? y.cb[1] + cc : y.cw[1] + u * c + cc;
              rec[1 + ci] = gg;
              rec[1 + y.P + ci] = wr;
            }
            wv[cc] = wr;
            mv[cc] = mr;
            vv[cc] = vr;
          }
        *(f32x4*)w2 = wv;
        *(f32x4*)m2 = mv;
        *(f32x4*)v2 = vv;
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
      const float w = w2[(i / y.c) * 4 + i % y.c];
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

    // zero the weights and output-layer moments (pads must be zero), then the initial or given parameters
    {
      uint4* z = (uint4*)lds;
      const uint32_t n16 = y.o_xs / 16;
      for (uint32_t i = threadIdx.x; i < n16; i += blockDim.x) z[i] = uint4{0, 0, 0, 0};
    }
    __syncthreads();
    {
      uint4* z = (uint4*)slot;
      const uint32_t n16 = 2 * y.HP * y.ldw * 4 / 16;
      for (uint32_t i = threadIdx.x; i < n16; i += blockDim.x) z[i] = uint4{0, 0, 0, 0};
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
    int epochs_lim = it.epochs;  // lowered when the plateau rule ends training
    auto chunk_valid = [&](const ChunkPos& p) { return steps > 0 && p.e < epochs_lim; };
    auto chunk_rows = [&](const ChunkPos& p) { return min(SM_RC, min(bs, n_fit - p.st * bs) - p.c0); };
    auto chunk_next = [&](ChunkPos p) {
      const int mb = min(bs, n_fit - p.st * bs);
      p.c0 += SM_RC;
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
    f32x4 acc[4][4], accg[4][KT], g2p[4];
    f32x4 gb2 = f32x4{0.f, 0.f, 0.f, 0.f};
    double lsum = 0.0, hits = 0.0, pen = 0.0, esum = 0.0;  // esum: the lane's share of the epoch's summed data loss
    float* rec = nullptr;
    Plateau plateau;
    bool have_best = false;
    const bool watch = it.patience > 0 && !resume;
    // Loss and second score (the thread's share) of `count` rows of a list under the current weights; uses
    // the input tiles of parity 0 and the forward accumulators.
    auto score_rows = [&](const int32_t* list, int mode, int count, double& ls, double& hs) {
      for (int off = 0; off < count; off += SM_RC) {
        const int rows = min(SM_RC, count - off);
        park_row_id(0, fetch_row_id(list, sp, mode, 0, off, rows));
        __syncthreads();
        fetch_inputs(0, xr, yv);
        commit_inputs(0, xr, yv);
        __syncthreads();
        forward((rows + 15) / 16, acc);
        __syncthreads();
        outputs<false>(0, rows, 0.f, ls, hs, gb2);
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
        for (int i = 0; i < 4; i++) {
          g2p[i] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int m = 0; m < KT; m++) accg[i][m] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        gb2 = f32x4{0.f, 0.f, 0.f, 0.f};
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
      __syncthreads();  // all four shares of the outputs, and the next chunk's row ids, visible
      if (more) fetch_inputs(par ^ 1, xr, yv);  // in flight across the backward phase
      outputs<true>(par, rows, 1.f / (float)mb, lsum, hits, gb2);
      backward(par, nrt, acc, accg, g2p);
      if (nxt.c0 == 0) {  // that was the last chunk of the step
        __syncthreads();  // every wave is past its reads of the output bias
        update(oc, accg, g2p, gb2, rec);
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
            // pass takes over the input tiles, so the next chunk's rows and inputs are fetched again after it
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

template <int KT, int CO>
__global__ __launch_bounds__(SM_THREADS, 2) void k_train_small(const TrainParams P) {
  extern __shared__ __align__(16) char smem[];
  __shared__ int s_item;
  __shared__ double red[SM_THREADS / 64];
  for (;;) {
    __syncthreads();
    if (threadIdx.x == 0) s_item = atomicAdd(P.queue, 1);
    __syncthreads();
    const int item = __builtin_amdgcn_readfirstlane(s_item);
    if (item >= P.n_items) break;
    const SItem* __restrict__ si = (const SItem*)P.items + item;
    Small<KT, CO> T{P, si->d, si->y, smem, P.slots + (uint64_t)blockIdx.x * P.slot_bytes, red};
    T.run();
  }
}

}  // namespace
