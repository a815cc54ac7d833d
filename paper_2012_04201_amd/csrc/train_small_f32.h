// LDS-resident training / scoring kernel for small fp32 models with one hidden
// layer (the "many concurrent studies" shape: up to 63 inputs, hidden width up
// to 240, up to 4 outputs).
//
// One workgroup (4 waves) trains one model, and the model never leaves the
// chip: weights and both optimizer moments of the two layers stay in LDS for
// all epochs, the minibatch is processed in chunks of 64 (or 32) rows whose
// inputs and hidden activations are LDS tiles, and the hidden-layer weight
// gradient is accumulated across the chunks of a step in MFMA accumulator
// registers, so the optimizer update reads the gradient from registers and
// the state from LDS.  HBM is touched only for the gathered input rows.
//
// Layouts (floats; every row padded by 4 against bank conflicts):
//   xs  [row][k]      gathered inputs, column d = 1 on real rows (bias)
//   xt  [k][row]      the same tile, input-major (operand of the weight gradient)
//   a1t [unit][row]   hidden activations, later overwritten by their deltas
//   w1, m1, v1 [unit][k]   hidden layer (bias in column d)
//   w2, m2, v2 [unit][4]   output layer (bias in row HP)
// The hidden layer runs on fp32 MFMA (16x16x4): forward contracts over k with
// xs and w1 as operands and stores the tile unit-major, the weight gradient
// contracts over the rows with xt and a1t as operands and lands in w1's own
// layout.  The output layer (at most 4 units) is plain VALU work.
#pragma once
#include "common.h"
#include "train_tiled_bf16.h"  // OptC, opt_update

namespace {

constexpr int SM_THREADS = 256;
constexpr uint32_t SM_LDS_LIMIT = 160 * 1024 - 1024;

struct SLay {
  int32_t d, h, c, K0, HP, RC, ldw, lda;
  int32_t cw[2], cb[2], P;
  uint32_t o_w1, o_m1, o_v1, o_w2, o_m2, o_v2, o_xs, o_xt, o_a1, o_red, o_d2, o_rows, lds_total;
};

struct SItem {
  ItemDesc d;
  SLay y;
};

__host__ __device__ inline bool small_eligible(const int32_t* dims, int L) {
  return L == 2 && dims[0] <= 63 && dims[1] <= 240 && dims[2] <= 4;  // thread HP (<= 240) owns the output bias
}

__host__ __device__ inline void make_slay(SLay& y, const int32_t* dims) {
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
    y.o_m1 = take(y.HP * y.ldw);
    y.o_v1 = take(y.HP * y.ldw);
    y.o_w2 = take((y.HP + 1) * 4);
    y.o_m2 = take((y.HP + 1) * 4);
    y.o_v2 = take((y.HP + 1) * 4);
    y.o_xs = take(rc * y.ldw);
    y.o_xt = take(y.K0 * y.lda);
    y.o_a1 = take(y.HP * y.lda);
    y.o_red = take(SM_THREADS * 4);
    y.o_d2 = take(rc * 4);
    y.o_rows = take(rc);
    y.lds_total = o;
    if (o <= SM_LDS_LIMIT) break;
  }
}

struct Small {
  const TrainParams& P;
  const ItemDesc& it;
  const SLay& y;
  char* lds;
  double* red;

  __device__ float* f(uint32_t off) const { return (float*)(lds + off); }
  __device__ int32_t* rowlist() const { return (int32_t*)(lds + y.o_rows); }

  // ---- parameters (packed order: W1[in][out], b1, W2[in][out], b2) --------
  __device__ void put_param(int ci, float val, float mv, float vv) const {
    const int d = y.d, h = y.h, c = y.c;
    uint32_t o;
    bool l1;
    if (ci < y.cb[0]) {  // W1[k][j]
      o = (ci % h) * y.ldw + ci / h;
      l1 = true;
    } else if (ci < y.cw[1]) {  // b1[j]
      o = (ci - y.cb[0]) * y.ldw + d;
      l1 = true;
    } else if (ci < y.cb[1]) {  // W2[u][cc]
      const int e = ci - y.cw[1];
      o = (e / c) * 4 + e % c;
      l1 = false;
    } else {  // b2[cc]
      o = y.HP * 4 + (ci - y.cb[1]);
      l1 = false;
    }
    f(l1 ? y.o_w1 : y.o_w2)[o] = val;
    f(l1 ? y.o_m1 : y.o_m2)[o] = mv;
    f(l1 ? y.o_v1 : y.o_v2)[o] = vv;
  }

  __device__ void init_params() const {
    const uint64_t km = key_model(it.seed, it.fold);
    for (int l = 0; l < 2; l++) {
      const int fi = l == 0 ? y.d : y.h, fo = l == 0 ? y.h : y.c;
      const uint64_t kw = key_fold(km, 16 + 2 * l), kb = key_fold(km, 16 + 2 * l + 1);
      const float bound = it.bound[l];
      for (int i = threadIdx.x; i < fi * fo + fo; i += blockDim.x) {
        const bool isb = i >= fi * fo;
        const int e = isb ? i - fi * fo : i;
        const uint32_t k24 = (uint32_t)(key_fold(isb ? kb : kw, (uint64_t)e) >> 40);
        const float val = bound * ((float)((int32_t)k24 - 8388608) * 0x1p-23f);
        put_param((isb ? y.cb[l] : y.cw[l]) + e, val, 0.f, 0.f);
      }
    }
  }

  __device__ void load_state(const float* st) const {
    for (int ci = threadIdx.x; ci < y.P; ci += blockDim.x) put_param(ci, st[ci], st[y.P + ci], st[2 * y.P + ci]);
  }

  // ---- chunk phases ---------------------------------------------------------
  __device__ void gather(const int32_t* list, uint64_t key, int n_list, int lo, int rows, bool permute) const {
    int32_t* rl = rowlist();
    const int RC = y.RC, K0 = y.K0, d = y.d;
    for (int p = threadIdx.x; p < RC; p += blockDim.x)
      rl[p] = p < rows ? list[permute ? perm_index(key, (uint32_t)n_list, (uint32_t)(lo + p)) : lo + p] : -1;
    __syncthreads();
    float* xs = f(y.o_xs);
    float* xt = f(y.o_xt);
    const float* X = (const float*)P.X;
    const int k = threadIdx.x % K0, rstep = SM_THREADS / K0;
    for (int r = threadIdx.x / K0; r < RC; r += rstep) {
      const int row = rl[r];
      float val = 0.f;
      if (row >= 0) val = k < d ? X[(size_t)row * d + k] : (k == d ? 1.f : 0.f);
      xs[r * y.ldw + k] = val;
      xt[k * y.lda + r] = val;
    }
    __syncthreads();
  }

  // a1t[unit][row] = relu(sum_k xs[row][k] * w1[unit][k])   (bias rides in column d)
  __device__ void forward_hidden(int nrt) const {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, li = lane & 15, q = lane >> 4;
    const int nut = y.HP / 16, ldw = y.ldw, lda = y.lda;
    const float* xs = f(y.o_xs);
    const float* w1 = f(y.o_w1);
    float* a1 = f(y.o_a1);
    f32x4 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
      for (int r = 0; r < 4; r++) acc[i][r] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int k0 = 0; k0 < y.K0; k0 += 16) {
      f32x4 a[4], b[4];
#pragma unroll
      for (int r = 0; r < 4; r++)
        if (r < nrt) a[r] = *(const f32x4*)(xs + (r * 16 + li) * ldw + k0 + 4 * q);
#pragma unroll
      for (int i = 0; i < 4; i++)
        if (w + 4 * i < nut) b[i] = *(const f32x4*)(w1 + ((w + 4 * i) * 16 + li) * ldw + k0 + 4 * q);
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
#pragma unroll
    for (int i = 0; i < 4; i++)
      if (w + 4 * i < nut) {
#pragma unroll
        for (int r = 0; r < 4; r++)
          if (r < nrt) {
            f32x4 v = acc[i][r];
#pragma unroll
            for (int e = 0; e < 4; e++) v[e] = fmaxf(v[e], 0.f);
            *(f32x4*)(a1 + ((w + 4 * i) * 16 + li) * lda + r * 16 + 4 * q) = v;
          }
      }
    __syncthreads();
  }

  // Output layer, loss and output delta (TRAIN) or validation statistics.
  template <bool TRAIN>
  __device__ void forward_out(int rows, float inv_mb, double& lsum, double& hits) const {
    const int RC = y.RC, G = SM_THREADS / RC, h = y.h, c = y.c, lda = y.lda;
    const int r = threadIdx.x % RC, g = threadIdx.x / RC;
    const float* a1 = f(y.o_a1);
    const float* w2 = f(y.o_w2);
    float* redf = f(y.o_red);
    float p[4] = {0.f, 0.f, 0.f, 0.f};
    for (int u = g; u < h; u += G) {
      const float av = a1[u * lda + r];
      const f32x4 wv = *(const f32x4*)(w2 + u * 4);
#pragma unroll
      for (int cc = 0; cc < 4; cc++) p[cc] += av * wv[cc];
    }
    *(f32x4*)(redf + threadIdx.x * 4) = f32x4{p[0], p[1], p[2], p[3]};
    __syncthreads();
    if (g == 0) {
      const f32x4 b2 = *(const f32x4*)(w2 + y.HP * 4);
      float z[4] = {b2[0], b2[1], b2[2], b2[3]};
      for (int gg = 0; gg < G; gg++) {
        const f32x4 pv = *(const f32x4*)(redf + (gg * RC + r) * 4);
#pragma unroll
        for (int cc = 0; cc < 4; cc++) z[cc] += pv[cc];
      }
      const int row = rowlist()[r];
      const bool valid = r < rows && row >= 0;
      float dl[4] = {0.f, 0.f, 0.f, 0.f};
      if (valid) {
        if (P.n_classes >= 2) {
          const int yr = ((const int32_t*)P.y)[row];
          float mx = z[0];
          int best = 0;
          for (int cc = 1; cc < c; cc++)
            if (z[cc] > mx) {
              mx = z[cc];
              best = cc;
            }
          float se = 0.f;
          for (int cc = 0; cc < c; cc++) se += expf(z[cc] - mx);
          const float lse = mx + logf(se);
          float zy = z[0];
          for (int cc = 1; cc < c; cc++) zy = cc == yr ? z[cc] : zy;
          lsum += (double)(lse - zy);
          hits += best == yr;
          if (TRAIN)
            for (int cc = 0; cc < c; cc++) dl[cc] = (expf(z[cc] - lse) - (cc == yr ? 1.f : 0.f)) * inv_mb;
        } else {
          const float e0 = z[0] - ((const float*)P.y)[row];
          lsum += TRAIN ? 0.5 * (double)e0 * (double)e0 : (double)e0 * (double)e0;
          if (TRAIN) dl[0] = e0 * inv_mb;
        }
      }
      if (TRAIN) *(f32x4*)(f(y.o_d2) + r * 4) = f32x4{dl[0], dl[1], dl[2], dl[3]};
    }
    __syncthreads();
  }

  // Output-layer gradient (accumulated in g2 over the chunks of the step) and
  // the hidden delta written over the activations.  Thread u owns hidden unit u;
  // thread HP owns the output bias.
  __device__ void backward_out(int nrows4, f32x4& g2) const {
    const int u = threadIdx.x, lda = y.lda;
    const float* d2 = f(y.o_d2);
    if (u < y.HP) {
      float* a1 = f(y.o_a1) + u * lda;
      const f32x4 wv = *(const f32x4*)(f(y.o_w2) + u * 4);
      for (int r4 = 0; r4 < nrows4; r4++) {
        f32x4 av = *(const f32x4*)(a1 + 4 * r4);
        f32x4 out;
#pragma unroll
        for (int e = 0; e < 4; e++) {
          const f32x4 dv = *(const f32x4*)(d2 + (4 * r4 + e) * 4);
          float s = 0.f;
#pragma unroll
          for (int cc = 0; cc < 4; cc++) {
            g2[cc] += av[e] * dv[cc];
            s += dv[cc] * wv[cc];
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
  __device__ void wgrad_hidden(int nrt, f32x4 (&accg)[4][4]) const {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, li = lane & 15, q = lane >> 4;
    const int nut = y.HP / 16, nkt = y.K0 / 16, lda = y.lda;
    const float* xt = f(y.o_xt);
    const float* a1 = f(y.o_a1);
    for (int rt = 0; rt < nrt; rt++) {
      f32x4 a[4], b[4];
#pragma unroll
      for (int m = 0; m < 4; m++)
        if (m < nkt) a[m] = *(const f32x4*)(xt + (m * 16 + li) * lda + rt * 16 + 4 * q);
#pragma unroll
      for (int i = 0; i < 4; i++)
        if (w + 4 * i < nut) b[i] = *(const f32x4*)(a1 + ((w + 4 * i) * 16 + li) * lda + rt * 16 + 4 * q);
#pragma unroll
      for (int i = 0; i < 4; i++)
        if (w + 4 * i < nut) {
#pragma unroll
          for (int m = 0; m < 4; m++)
            if (m < nkt) {
#pragma unroll
              for (int e = 0; e < 4; e++)
                accg[i][m] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[m][e], b[i][e], accg[i][m], 0, 0, 0);
            }
        }
    }
    __syncthreads();
  }

  // Optimizer step on both layers: gradients from registers, state in LDS.
  __device__ void update(const OptC& oc, f32x4 (&accg)[4][4], const f32x4& g2, float* rec) const {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, li = lane & 15, q = lane >> 4;
    const int nut = y.HP / 16, nkt = y.K0 / 16, ldw = y.ldw, d = y.d, h = y.h, c = y.c;
    float* w1 = f(y.o_w1);
    float* m1 = f(y.o_m1);
    float* v1 = f(y.o_v1);
#pragma unroll
    for (int i = 0; i < 4; i++)
      if (w + 4 * i < nut) {
        const int j = (w + 4 * i) * 16 + li;
#pragma unroll
        for (int m = 0; m < 4; m++)
          if (m < nkt) {
            const int k0 = m * 16 + 4 * q;
            if (j < h && k0 <= d) {
              const int o = j * ldw + k0;
              f32x4 wv = *(const f32x4*)(w1 + o), mv = *(const f32x4*)(m1 + o), vv = *(const f32x4*)(v1 + o);
#pragma unroll
              for (int e = 0; e < 4; e++) {
                const int k = k0 + e;
                if (k <= d) {
                  float wr = wv[e], mr = mv[e], vr = vv[e];
                  const float gg = k < d ? accg[i][m][e] + oc.am * wr : accg[i][m][e];
                  opt_update(oc, gg, wr, mr, vr);
                  if (rec) {
                    const int ci = k < d ? y.cw[0] + k * h + j : y.cb[0] + j;
                    rec[1 + ci] = gg;
                    rec[1 + y.P + ci] = wr;
                  }
                  wv[e] = wr;
                  mv[e] = mr;
                  vv[e] = vr;
                }
              }
              *(f32x4*)(w1 + o) = wv;
              *(f32x4*)(m1 + o) = mv;
              *(f32x4*)(v1 + o) = vv;
            }
          }
      }
    const int u = threadIdx.x;
    if (u < h || u == y.HP) {
      const bool isb = u == y.HP;
      float* w2 = f(y.o_w2) + u * 4;
      float* m2 = f(y.o_m2) + u * 4;
      float* v2 = f(y.o_v2) + u * 4;
      f32x4 wv = *(const f32x4*)w2, mv = *(const f32x4*)m2, vv = *(const f32x4*)v2;
#pragma unroll
      for (int cc = 0; cc < 4; cc++)
        if (cc < c) {
          float wr = wv[cc], mr = mv[cc], vr = vv[cc];
          const float gg = isb ? g2[cc] : g2[cc] + oc.am * wr;
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

  __device__ void run() const {
    const int f_ = it.fold;
    const int n_tr = P.counts[2 * f_], n_va = P.counts[2 * f_ + 1];
    const int32_t* tr = P.train_idx + (int64_t)f_ * P.n;
    const int32_t* va = P.val_idx + (int64_t)f_ * P.n;
    const int bs = eff_batch(it.batch_size, n_tr);
    const int steps = n_tr > 0 ? (n_tr + bs - 1) / bs : 0;
    const uint64_t km = key_model(it.seed, f_);
    const bool traced = P.trace_item == it.b * P.n_folds + f_;
    const int RC = y.RC;

    // zero the state region (pads must be zero), then the initial parameters
    {
      uint4* z = (uint4*)lds;
      const uint32_t n16 = y.o_xs / 16;
      for (uint32_t i = threadIdx.x; i < n16; i += blockDim.x) z[i] = uint4{0, 0, 0, 0};
    }
    __syncthreads();
    double b1t = 1.0, b2t = 1.0;
    int64_t gstep = 0;
    int e0 = 0, st0 = 0;
    if (traced && P.state_in && steps > 0) {
      gstep = P.step_begin;
      load_state(P.state_in);
      e0 = (int)(gstep / steps);
      st0 = (int)(gstep % steps);
      b1t = pow((double)it.beta1, (double)gstep);
      b2t = pow((double)it.beta2, (double)gstep);
    } else {
      init_params();
    }
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

    for (int e = e0; e < it.epochs; e++) {
      const uint64_t ke = key_epoch(km, e);
      for (int st = e == e0 ? st0 : 0; st < steps; st++, gstep++) {
        const int lo = st * bs, mb = min(bs, n_tr - lo);
        const float inv_mb = 1.f / (float)mb;
        oc.am = it.alpha / (float)mb;
        if (oc.adam) {
          b1t *= (double)it.beta1;
          b2t *= (double)it.beta2;
          oc.lr_t = (float)((double)it.lr * sqrt(1.0 - b2t) / (1.0 - b1t));
        }
        float* rec = nullptr;
        if (traced && gstep >= P.step_begin && gstep < P.step_end)
          rec = P.trace_out + (gstep - P.step_begin) * (1 + 2 * (int64_t)y.P);
        double pen = 0.0;
        if (rec) pen = penalty_sum();
        double lsum = 0.0, hits = 0.0;
        f32x4 accg[4][4];
#pragma unroll
        for (int i = 0; i < 4; i++)
#pragma unroll
          for (int m = 0; m < 4; m++) accg[i][m] = f32x4{0.f, 0.f, 0.f, 0.f};
        f32x4 g2 = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int c0 = 0; c0 < mb; c0 += RC) {
          const int rows = min(RC, mb - c0), nrt = (rows + 15) / 16;
          gather(tr, ke, n_tr, lo + c0, rows, true);
          forward_hidden(nrt);
          forward_out<true>(rows, inv_mb, lsum, hits);
          backward_out(4 * nrt, g2);
          wgrad_hidden(nrt, accg);
        }
        update(oc, accg, g2, rec);
        if (rec) {
          const double data = block_sum(lsum, red) / (double)mb;
          if (threadIdx.x == 0) rec[0] = (float)(data + 0.5 * (double)it.alpha * pen / (double)mb);
        }
      }
    }

    double lsum = 0.0, hits = 0.0;
    for (int off = 0; off < n_va; off += RC) {
      const int rows = min(RC, n_va - off);
      gather(va, 0, n_va, off, rows, false);
      forward_hidden((rows + 15) / 16);
      forward_out<false>(rows, 0.f, lsum, hits);
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
    Small T{P, si->d, si->y, smem, red};
    T.run();
  }
}

}  // namespace
