// LDS-resident training / scoring kernel for small fp32 models with one hidden
// layer (the "many concurrent studies" shape: up to 63 inputs, hidden width up
// to 240, up to 4 outputs).
//
// One workgroup (4 waves) trains one model, and the model never leaves the
// chip: the weights of both layers stay in LDS for all epochs, the optimizer
// moments stay in registers (each lane always updates the same elements), the
// minibatch is processed in chunks of 64 (or 32) rows whose inputs and hidden
// activations are LDS tiles, and the hidden-layer weight gradient is
// accumulated across the chunks of a step in MFMA accumulator registers.  HBM
// is touched only for the gathered input rows, and those are fetched one
// chunk ahead into registers.  The LDS footprint is kept under half a CU's
// LDS so that two workgroups share a CU and cover each other's barriers.
//
// Layouts (floats; every row padded by 4 against bank conflicts):
//   xs  [row][k]      gathered inputs, column d = 1 on real rows (bias)
//   xt  [k][row]      the same tile, input-major (operand of the weight gradient)
//   a1t [unit][row]   hidden activations, later overwritten by their deltas
//   w1  [unit][k]     hidden layer (bias in column d)
//   w2  [unit][4]     output layer (bias in row HP)
// The hidden layer runs on fp32 MFMA (16x16x4): forward contracts over k with
// xs and w1 as operands and stores the tile unit-major, the weight gradient
// contracts over the rows with xt and a1t as operands and lands in w1's own
// layout.  The output layer (at most 4 units) is plain VALU work.
#pragma once
#include "common.h"
#include "train_tiled_bf16.h"  // OptC, opt_update

namespace {

constexpr int SM_THREADS = 256;
constexpr uint32_t SM_LDS_LIMIT = 79 * 1024;  // per workgroup: two workgroups per CU

struct SLay {
  int32_t d, h, c, K0, HP, RC, ldw, lda;
  int32_t cw[2], cb[2], P;
  uint32_t o_w1, o_w2, o_xs, o_xt, o_a1, o_red, o_d2, o_rows, o_ys, o_epoch, lds_total;
  int32_t epoch_cap;  // entries of the per-epoch row table in LDS (0: rows are permuted on the fly)
};

struct SItem {
  ItemDesc d;
  SLay y;
};

__host__ __device__ inline bool small_eligible(const int32_t* dims, int L) {
  return L == 2 && dims[0] <= 63 && dims[1] <= 240 && dims[2] <= 4;  // thread HP (<= 240) owns the output bias
}

__host__ __device__ inline void make_slay(SLay& y, const int32_t* dims, int64_t n) {
  y.d = dims[0];
  y.h = dims[1];
  y.c = dims[2];
  y.K0 = dims[0] + 1 <= 16 ? 16 : (dims[0] + 1 <= 32 ? 32 : 64);
  y.HP = rup(dims[1], 16);
  y.ldw = y.K0 + 4;
  y.cw[0] = 0;
  y.cb[0] = y.d * y.h;
  y.cw[1] = y.cb[0] + y.h;
  y.cb[1] = y.cw[1] + y.h * y.c;
  y.P = y.cb[1] + y.c;
  for (int rc = 64; rc >= 32; rc -= 32) {
    y.RC = rc;
    y.lda = rc + 4;
    uint32_t o = 0;
    auto take = [&](uint32_t floats) {
      uint32_t r = o;
      o += ((floats * 4) + 15) & ~15u;
      return r;
    };
    y.o_w1 = take(y.HP * y.ldw);
    y.o_w2 = take((y.HP + 1) * 4);
    y.o_xs = take(rc * y.ldw);
    y.o_xt = take(y.K0 * y.lda);
    y.o_a1 = take(y.HP * y.lda);
    y.o_red = take(SM_THREADS * 4);
    y.o_d2 = take(rc * 4);
    y.o_rows = take(2 * rc);
    y.o_ys = take(rc);
    y.o_epoch = o;
    y.epoch_cap = 0;
    y.lds_total = o;
    if (o <= SM_LDS_LIMIT) {
      // room left for the epoch's row order (all training rows of a fold)?
      if (n <= 4096 && o + 4 * (uint32_t)n <= SM_LDS_LIMIT) {
        y.epoch_cap = (int32_t)n;
        y.lds_total = o + ((4 * (uint32_t)n + 15) & ~15u);
      }
      break;
    }
  }
}

// Position in the training schedule: epoch, step of the epoch, first row of
// the chunk within the step's minibatch.
struct ChunkPos {
  int e, st, c0;
};

template <int KT>
struct Small {
  static constexpr int K0 = 16 * KT, RSTEP = SM_THREADS / K0, NX = 64 / RSTEP;
  const TrainParams& P;
  const ItemDesc& it;
  const SLay& y;
  char* lds;
  double* red;

  __device__ float* f(uint32_t off) const { return (float*)(lds + off); }
  __device__ int32_t* rowlist(int par) const { return (int32_t*)(lds + y.o_rows) + par * y.RC; }

  // packed index (W1[in][out], b1, W2[in][out], b2) of hidden-layer element (unit j, column k); -1 for pads
  __device__ int ci_hidden(int j, int k) const {
    if (j >= y.h || k > y.d) return -1;
    return k < y.d ? y.cw[0] + k * y.h + j : y.cb[0] + j;
  }
  __device__ float init_value(int l, int e, bool isb) const {
    const uint64_t kt = key_fold(key_model(it.seed, it.fold), 16 + 2 * l + (isb ? 1 : 0));
    const uint32_t k24 = (uint32_t)(key_fold(kt, (uint64_t)e) >> 40);
    return it.bound[l] * ((float)((int32_t)k24 - 8388608) * 0x1p-23f);
  }

  // Weights into LDS, from the initial draw or from a packed state.
  __device__ void put_weights(const float* st) const {
    const int d = y.d, h = y.h, c = y.c;
    float* w1 = f(y.o_w1);
    float* w2 = f(y.o_w2);
    for (int ci = threadIdx.x; ci < y.P; ci += blockDim.x) {
      if (ci < y.cb[0]) {
        w1[(ci % h) * y.ldw + ci / h] = st ? st[ci] : init_value(0, ci, false);
      } else if (ci < y.cw[1]) {
        w1[(ci - y.cb[0]) * y.ldw + d] = st ? st[ci] : init_value(0, ci - y.cb[0], true);
      } else if (ci < y.cb[1]) {
        const int e = ci - y.cw[1];
        w2[(e / c) * 4 + e % c] = st ? st[ci] : init_value(1, e, false);
      } else {
        w2[y.HP * 4 + (ci - y.cb[1])] = st ? st[ci] : init_value(1, ci - y.cb[1], true);
      }
    }
  }

  // ---- input staging, one chunk ahead ---------------------------------------
  // (1) row ids of a chunk: the load is issued here, the value parked in LDS later
  __device__ int fetch_row_id(const int32_t* list, uint64_t key, int n_list, int lo, int rows, bool permute) const {
    const int p = threadIdx.x;
    if (p >= y.RC || p >= rows) return -1;
    if (permute && y.epoch_cap) return ((const int32_t*)(lds + y.o_epoch))[lo + p];
    return list[permute ? perm_index(key, (uint32_t)n_list, (uint32_t)(lo + p)) : lo + p];
  }
  // Row ids of a whole epoch, in minibatch order, into the LDS table.
  __device__ void build_epoch_table(const int32_t* list, uint64_t key, int n_list) const {
    int32_t* tab = (int32_t*)(lds + y.o_epoch);
    for (int p = threadIdx.x; p < n_list; p += blockDim.x) tab[p] = list[perm_index(key, (uint32_t)n_list, (uint32_t)p)];
  }
  __device__ void park_row_id(int par, int row) const {
    if ((int)threadIdx.x < y.RC) rowlist(par)[threadIdx.x] = row;
  }
  // (2) the chunk's input values (and label) into registers
  __device__ void fetch_inputs(int par, float (&xr)[NX], float& yv) const {
    const int32_t* rl = rowlist(par);
    const float* X = (const float*)P.X;
    const int k = threadIdx.x % K0, r0 = threadIdx.x / K0, d = y.d;
#pragma unroll
    for (int i = 0; i < NX; i++) {
      const int r = r0 + i * RSTEP;
      xr[i] = 0.f;
      if (r < y.RC) {
        const int row = rl[r];
        if (row >= 0) xr[i] = k < d ? X[row * d + k] : (k == d ? 1.f : 0.f);  // n*d < 2^31 (checked by the host)
      }
    }
    yv = 0.f;
    if ((int)threadIdx.x < y.RC) {
      const int row = rl[threadIdx.x];
      if (row >= 0) yv = P.n_classes >= 2 ? __int_as_float(((const int32_t*)P.y)[row]) : ((const float*)P.y)[row];
    }
  }
  // (3) registers -> the LDS tiles
  __device__ void commit_inputs(const float (&xr)[NX], float yv) const {
    float* xs = f(y.o_xs);
    float* xt = f(y.o_xt);
    const int k = threadIdx.x % K0, r0 = threadIdx.x / K0;
#pragma unroll
    for (int i = 0; i < NX; i++) {
      const int r = r0 + i * RSTEP;
      if (r < y.RC) {
        xs[r * y.ldw + k] = xr[i];
        xt[k * y.lda + r] = xr[i];
      }
    }
    if ((int)threadIdx.x < y.RC) f(y.o_ys)[threadIdx.x] = yv;
  }

  // a1t[unit][row] = relu(sum_k xs[row][k] * w1[unit][k])   (bias rides in column d)
  // Two row tiles at a time, to keep the accumulator footprint small.
  __device__ void forward_hidden(int nrt) const {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, li = lane & 15, q = lane >> 4;
    const int nut = y.HP / 16, ldw = y.ldw, lda = y.lda;
    const float* xs = f(y.o_xs);
    const float* w1 = f(y.o_w1);
    float* a1 = f(y.o_a1);
    for (int r0 = 0; r0 < nrt; r0 += 2) {
      f32x4 acc[4][2];
#pragma unroll
      for (int i = 0; i < 4; i++)
#pragma unroll
        for (int r = 0; r < 2; r++) acc[i][r] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kk = 0; kk < KT; kk++) {
        f32x4 a[2], b[4];
#pragma unroll
        for (int r = 0; r < 2; r++) a[r] = *(const f32x4*)(xs + ((r0 + r) * 16 + li) * ldw + kk * 16 + 4 * q);
#pragma unroll
        for (int i = 0; i < 4; i++)
          if (w + 4 * i < nut) b[i] = *(const f32x4*)(w1 + ((w + 4 * i) * 16 + li) * ldw + kk * 16 + 4 * q);
#pragma unroll
        for (int i = 0; i < 4; i++)
          if (w + 4 * i < nut) {
#pragma unroll
            for (int r = 0; r < 2; r++) {
#pragma unroll
              for (int e = 0; e < 4; e++)
                acc[i][r] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[r][e], b[i][e], acc[i][r], 0, 0, 0);
            }
          }
      }
#pragma unroll
      for (int i = 0; i < 4; i++)
        if (w + 4 * i < nut) {
#pragma unroll
          for (int r = 0; r < 2; r++) {
            f32x4 v = acc[i][r];
#pragma unroll
            for (int e = 0; e < 4; e++) v[e] = fmaxf(v[e], 0.f);
            *(f32x4*)(a1 + ((w + 4 * i) * 16 + li) * lda + (r0 + r) * 16 + 4 * q) = v;
          }
        }
    }
    __syncthreads();
  }

  // Output layer: partial dot products of thread (row r, group g) over the units
  // g, g+G, ...; the caller synchronises before finish_out.
  __device__ void forward_out_partial() const {
    const int RC = y.RC, G = SM_THREADS / RC, lda = y.lda;
    const int r = threadIdx.x % RC, g = threadIdx.x / RC;
    const float* a1 = f(y.o_a1) + r;
    const float* w2 = f(y.o_w2);
    const bool c2 = y.c >= 2, c4 = y.c >= 3;
    f32x4 p = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
    for (int u = g; u < y.HP; u += G) {
      const float av = a1[u * lda];
      const f32x4 wv = *(const f32x4*)(w2 + u * 4);
      p[0] += av * wv[0];
      if (c2) p[1] += av * wv[1];
      if (c4) {
        p[2] += av * wv[2];
        p[3] += av * wv[3];
      }
    }
    *(f32x4*)(f(y.o_red) + threadIdx.x * 4) = p;
  }

  // Loss and output delta (TRAIN) or validation statistics of the chunk's rows.
  template <bool TRAIN>
  __device__ void finish_out(int rows, float inv_mb, double& lsum, double& hits) const {
    const int RC = y.RC, G = SM_THREADS / RC, c = y.c;
    const int r = threadIdx.x;
    if (r < RC) {
      const float* redf = f(y.o_red);
      const f32x4 b2 = *(const f32x4*)(f(y.o_w2) + y.HP * 4);
      float z[4] = {b2[0], b2[1], b2[2], b2[3]};
#pragma unroll 4
      for (int gg = 0; gg < G; gg++) {
        const f32x4 pv = *(const f32x4*)(redf + (gg * RC + r) * 4);
#pragma unroll
        for (int cc = 0; cc < 4; cc++) z[cc] += pv[cc];
      }
      const float yv = f(y.o_ys)[r];
      float dl[4] = {0.f, 0.f, 0.f, 0.f};
      if (r < rows) {
        if (P.n_classes >= 2) {
          const int yr = __float_as_int(yv);
          float mx = z[0], zy = z[0];
          int best = 0;
#pragma unroll
          for (int cc = 1; cc < 4; cc++)
            if (cc < c) {
              if (z[cc] > mx) {
                mx = z[cc];
                best = cc;
              }
              zy = cc == yr ? z[cc] : zy;
            }
          float se = 0.f;
#pragma unroll
          for (int cc = 0; cc < 4; cc++)
            if (cc < c) se += expf(z[cc] - mx);
          const float lse = mx + logf(se);
          lsum += (double)(lse - zy);
          hits += best == yr;
          if (TRAIN) {
#pragma unroll
            for (int cc = 0; cc < 4; cc++)
              if (cc < c) dl[cc] = (expf(z[cc] - lse) - (cc == yr ? 1.f : 0.f)) * inv_mb;
          }
        } else {
          const float e0 = z[0] - yv;
          lsum += TRAIN ? 0.5 * (double)e0 * (double)e0 : (double)e0 * (double)e0;
          if (TRAIN) dl[0] = e0 * inv_mb;
        }
      }
      if (TRAIN) *(f32x4*)(f(y.o_d2) + r * 4) = f32x4{dl[0], dl[1], dl[2], dl[3]};
    }
  }

  // Output-layer gradient (accumulated in g2 over the chunks of the step) and
  // the hidden delta written over the activations.  Thread u owns hidden unit u;
  // thread HP owns the output bias.
  __device__ void backward_out(int nrows4, f32x4& g2) const {
    const int u = threadIdx.x, lda = y.lda;
    const float* d2 = f(y.o_d2);
    const bool c2 = y.c >= 2, c4 = y.c >= 3;
    if (u < y.HP) {
      float* a1 = f(y.o_a1) + u * lda;
      const f32x4 wv = *(const f32x4*)(f(y.o_w2) + u * 4);
#pragma unroll 2
      for (int r4 = 0; r4 < nrows4; r4++) {
        const f32x4 av = *(const f32x4*)(a1 + 4 * r4);
        f32x4 out;
#pragma unroll
        for (int e = 0; e < 4; e++) {
          const f32x4 dv = *(const f32x4*)(d2 + (4 * r4 + e) * 4);
          float s = dv[0] * wv[0];
          g2[0] += av[e] * dv[0];
          if (c2) {
            g2[1] += av[e] * dv[1];
            s += dv[1] * wv[1];
          }
          if (c4) {
            g2[2] += av[e] * dv[2];
            g2[3] += av[e] * dv[3];
            s += dv[2] * wv[2] + dv[3] * wv[3];
          }
          out[e] = av[e] > 0.f ? s : 0.f;
        }
        *(f32x4*)(a1 + 4 * r4) = out;
      }
    } else if (u == y.HP) {
      for (int r = 0; r < 4 * nrows4; r++) {
        const f32x4 dv = *(const f32x4*)(d2 + r * 4);
#pragma unroll
        for (int cc = 0; cc < 4; cc++) g2[cc] += dv[cc];
      }
    }
    __syncthreads();
  }

  // accg[unit tile][k tile] += sum_rows xt[k][row] * a1t[unit][row]
  __device__ void wgrad_hidden(int nrt, f32x4 (&accg)[4][KT]) const {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, li = lane & 15, q = lane >> 4;
    const int nut = y.HP / 16, lda = y.lda;
    const float* xt = f(y.o_xt);
    const float* a1 = f(y.o_a1);
    for (int rt = 0; rt < nrt; rt++) {
      f32x4 a[KT], b[4];
#pragma unroll
      for (int m = 0; m < KT; m++) a[m] = *(const f32x4*)(xt + (m * 16 + li) * lda + rt * 16 + 4 * q);
#pragma unroll
      for (int i = 0; i < 4; i++)
        if (w + 4 * i < nut) b[i] = *(const f32x4*)(a1 + ((w + 4 * i) * 16 + li) * lda + rt * 16 + 4 * q);
#pragma unroll
      for (int i = 0; i < 4; i++)
        if (w + 4 * i < nut) {
#pragma unroll
          for (int m = 0; m < KT; m++) {
#pragma unroll
            for (int e = 0; e < 4; e++)
              accg[i][m] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[m][e], b[i][e], accg[i][m], 0, 0, 0);
          }
        }
    }
    __syncthreads();
  }

  // Optimizer step on both layers: gradients and moments in registers, weights in LDS.
  __device__ void update(const OptC& oc, const f32x4 (&accg)[4][KT], f32x4 (&m1r)[4][KT], f32x4 (&v1r)[4][KT],
                         const f32x4& g2, f32x4& m2r, f32x4& v2r, float* rec) const {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, li = lane & 15, q = lane >> 4;
    const int nut = y.HP / 16, ldw = y.ldw, d = y.d, h = y.h, c = y.c;
    float* w1 = f(y.o_w1);
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
#pragma unroll
            for (int e = 0; e < 4; e++) {
              const int k = k0 + e;
              if (k <= d) {
                float wr = wv[e], mr = m1r[i][m][e], vr = v1r[i][m][e];
                const float gg = k < d ? accg[i][m][e] + oc.am * wr : accg[i][m][e];
                opt_update(oc, gg, wr, mr, vr);
                if (rec) {
                  const int ci = ci_hidden(j, k);
                  rec[1 + ci] = gg;
                  rec[1 + y.P + ci] = wr;
                }
                wv[e] = wr;
                m1r[i][m][e] = mr;
                v1r[i][m][e] = vr;
              }
            }
            *(f32x4*)(w1 + o) = wv;
          }
        }
      }
    const int u = threadIdx.x;
    if (u < h || u == y.HP) {
      const bool isb = u == y.HP;
      float* w2 = f(y.o_w2) + u * 4;
      f32x4 wv = *(const f32x4*)w2;
#pragma unroll
      for (int cc = 0; cc < 4; cc++)
        if (cc < c) {
          float wr = wv[cc], mr = m2r[cc], vr = v2r[cc];
          const float gg = isb ? g2[cc] : g2[cc] + oc.am * wr;
          opt_update(oc, gg, wr, mr, vr);
          if (rec) {
            const int ci = isb ? y.cb[1] + cc : y.cw[1] + u * c + cc;
            rec[1 + ci] = gg;
            rec[1 + y.P + ci] = wr;
          }
          wv[cc] = wr;
          m2r[cc] = mr;
          v2r[cc] = vr;
        }
      *(f32x4*)w2 = wv;
    }
    __syncthreads();
  }

  __device__ double penalty_sum() const {
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
    const int f_ = it.fold;
    const int n_tr = P.counts[2 * f_], n_va = P.counts[2 * f_ + 1];
    const int32_t* tr = P.train_idx + (int64_t)f_ * P.n;
    const int32_t* va = P.val_idx + (int64_t)f_ * P.n;
    const int bs = eff_batch(it.batch_size, n_tr);
    const int steps = n_tr > 0 ? (n_tr + bs - 1) / bs : 0;
    const uint64_t km = key_model(it.seed, f_);
    const bool traced = P.trace_item == it.b * P.n_folds + f_;
    const int RC = y.RC;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, li = lane & 15, q = lane >> 4;

    // zero the weights (pads must be zero), then the initial or given parameters
    {
      uint4* z = (uint4*)lds;
      const uint32_t n16 = y.o_xs / 16;
      for (uint32_t i = threadIdx.x; i < n16; i += blockDim.x) z[i] = uint4{0, 0, 0, 0};
    }
    __syncthreads();
    f32x4 m1r[4][KT], v1r[4][KT], m2r = f32x4{0.f, 0.f, 0.f, 0.f}, v2r = m2r;
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
      for (int m = 0; m < KT; m++) m1r[i][m] = v1r[i][m] = f32x4{0.f, 0.f, 0.f, 0.f};
    double b1t = 1.0, b2t = 1.0;
    int64_t gstep = 0;
    ChunkPos pos = {0, 0, 0};
    const bool resume = traced && P.state_in && steps > 0;
    if (resume) {
      const float* st = P.state_in;
      gstep = P.step_begin;
      pos.e = (int)(gstep / steps);
      pos.st = (int)(gstep % steps);
      b1t = pow((double)it.beta1, (double)gstep);
      b2t = pow((double)it.beta2, (double)gstep);
#pragma unroll
      for (int i = 0; i < 4; i++)
#pragma unroll
        for (int m = 0; m < KT; m++)
#pragma unroll
          for (int e = 0; e < 4; e++) {
            const int ci = ci_hidden((w + 4 * i) * 16 + li, m * 16 + 4 * q + e);
            if (ci >= 0) {
              m1r[i][m][e] = st[y.P + ci];
              v1r[i][m][e] = st[2 * y.P + ci];
            }
          }
      const int u = threadIdx.x;
      if (u < y.h || u == y.HP) {
#pragma unroll
        for (int cc = 0; cc < 4; cc++)
          if (cc < y.c) {
            const int ci = u == y.HP ? y.cb[1] + cc : y.cw[1] + u * y.c + cc;
            m2r[cc] = st[y.P + ci];
            v2r[cc] = st[2 * y.P + ci];
          }
      }
    }
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
    auto chunk_valid = [&](const ChunkPos& p) { return steps > 0 && p.e < it.epochs; };
    auto chunk_rows = [&](const ChunkPos& p) { return min(RC, min(bs, n_tr - p.st * bs) - p.c0); };
    auto chunk_next = [&](ChunkPos p) {
      const int mb = min(bs, n_tr - p.st * bs);
      p.c0 += RC;
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
      return fetch_row_id(tr, key_epoch(km, p.e), n_tr, p.st * bs + p.c0, chunk_rows(p), true);
    };
    float xr[NX], yv = 0.f;
    int par = 0;
    if (chunk_valid(pos) && y.epoch_cap) {
      build_epoch_table(tr, key_epoch(km, pos.e), n_tr);
      __syncthreads();
    }
    if (chunk_valid(pos)) {
      park_row_id(0, chunk_row_id(pos));
      __syncthreads();
      fetch_inputs(0, xr, yv);
    }
    f32x4 accg[4][KT];
    f32x4 g2 = f32x4{0.f, 0.f, 0.f, 0.f};
    double lsum = 0.0, hits = 0.0, pen = 0.0;
    float* rec = nullptr;
    while (chunk_valid(pos)) {
      const int mb = min(bs, n_tr - pos.st * bs);
      const int rows = chunk_rows(pos), nrt = (rows + 15) / 16;
      if (pos.c0 == 0) {  // first chunk of a step
        oc.am = it.alpha / (float)mb;
        if (oc.adam) {
          b1t *= (double)it.beta1;
          b2t *= (double)it.beta2;
          oc.lr_t = (float)((double)it.lr * sqrt(1.0 - b2t) / (1.0 - b1t));
        }
        rec = nullptr;
        if (traced && gstep >= P.step_begin && gstep < P.step_end)
          rec = P.trace_out + (gstep - P.step_begin) * (1 + 2 * (int64_t)y.P);
        if (rec) pen = penalty_sum();
        lsum = 0.0;
#pragma unroll
        for (int i = 0; i < 4; i++)
#pragma unroll
          for (int m = 0; m < KT; m++) accg[i][m] = f32x4{0.f, 0.f, 0.f, 0.f};
        g2 = f32x4{0.f, 0.f, 0.f, 0.f};
      }
      commit_inputs(xr, yv);
      const ChunkPos nxt = chunk_next(pos);
      const bool more = chunk_valid(nxt);
      if (more && nxt.e != pos.e && y.epoch_cap) {
        // the next chunk opens an epoch: its row order replaces the table (this epoch's last rows are already read)
        build_epoch_table(tr, key_epoch(km, nxt.e), n_tr);
        __syncthreads();
      }
      int nrow = -1;
      if (more) nrow = chunk_row_id(nxt);  // load in flight across the hidden layer
      __syncthreads();
      forward_hidden(nrt);
      if (more) park_row_id(par ^ 1, nrow);
      forward_out_partial();
      __syncthreads();
      if (more) fetch_inputs(par ^ 1, xr, yv);  // in flight across the backward phases
      finish_out<true>(rows, 1.f / (float)mb, lsum, hits);
      __syncthreads();
      backward_out(4 * nrt, g2);
      wgrad_hidden(nrt, accg);
      if (nxt.c0 == 0) {  // that was the last chunk of the step
        update(oc, accg, m1r, v1r, g2, m2r, v2r, rec);
        if (rec) {
          const double data = block_sum(lsum, red) / (double)mb;
          if (threadIdx.x == 0) rec[0] = (float)(data + 0.5 * (double)it.alpha * pen / (double)mb);
        }
        gstep++;
      }
      pos = nxt;
      par ^= 1;
    }

    // ---- validation score on the held rows ----
    lsum = 0.0;
    hits = 0.0;
    for (int off = 0; off < n_va; off += RC) {
      const int rows = min(RC, n_va - off);
      park_row_id(0, fetch_row_id(va, 0, n_va, off, rows, false));
      __syncthreads();
      fetch_inputs(0, xr, yv);
      commit_inputs(xr, yv);
      __syncthreads();
      forward_hidden((rows + 15) / 16);
      forward_out_partial();
      __syncthreads();
      finish_out<false>(rows, 0.f, lsum, hits);
      __syncthreads();
    }
    lsum = block_sum(lsum, red);
    hits = block_sum(hits, red);
    if (threadIdx.x == 0) {
      float* out = P.item_out + 2 * ((int64_t)it.b * P.n_folds + f_);
      out[0] = n_va > 0 ? (float)(lsum / (double)n_va) : __builtin_nanf("");
      out[1] = P.n_classes >= 2 ? (n_va > 0 ? (float)(hits / (double)n_va) : __builtin_nanf("")) : 0.f;
    }
  }
};

template <int KT>
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
    Small<KT> T{P, si->d, si->y, smem, red};
    T.run();
  }
}

}  // namespace
