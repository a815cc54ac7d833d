// Training / scoring kernel for models WITHOUT a hidden layer (linear and
// logistic regression trained like the MLPs: same minibatch order, losses,
// penalty and optimizers; Section 2, Table 1's linear models).  fp32, or the
// bfloat16 mode of the other kernels: inputs stored as bfloat16, the weights
// and the deltas rounded to bfloat16 where they enter a product, everything
// else (master weights, moments, sums, the bias) in fp32.
//
// Such a model has (d + 1) * c parameters, a few dozen to a thousand: far too
// little work for a workgroup.  ONE WAVEFRONT trains one model, several
// independent wavefronts per workgroup, each taking models from the shared
// work queue, and the model never leaves the wavefront:
//   * lane t owns the rows k = t + 64 i of W[in][out], and lane j < c the bias
//     of output j, with their optimizer moments and the step's gradient, all in
//     registers for the whole run;
//   * a minibatch is taken in chunks of 64 rows.  The chunk's input rows are
//     gathered into LDS (row stride odd, so that both access patterns below are
//     conflict-free);
//   * forward: lane = row; the outputs are d + 1 multiply-adds per output from
//     the lane's LDS row and an LDS copy of the weights (broadcast reads), then
//     softmax / logistic / squared loss and the output deltas, written to LDS;
//   * gradient: lane = input k: sum over the chunk's rows of x[row][k] *
//     delta[row][:] (one conflict-free read of x and one broadcast vector read
//     of the deltas per row; the bias lanes sum their delta column),
//     accumulated over the chunks of the step;
//   * the optimizer update runs in the owning lane, which refreshes the LDS copy.
// No workgroup barrier anywhere: a wavefront's LDS accesses execute in order.
//
// LDS per wavefront (floats): xs[64][S] (S = d + 1 made odd), ws[d + 1][CO]
// (CO = outputs padded to 1, 2, 4, 8 or 16), ds[64][CO], wbest[d + 1][CO] (the best
// epoch's parameters when early stopping watches held-out rows), and, for data sets of
// up to LN_EPOCH_CAP rows, the epoch's row order ep[n]: the seeded permutation
// is walked for all positions of the epoch at once (a lane that finishes a
// position's walk starts its next one, so the lanes stay busy), instead of per
// chunk, where every chunk would wait for its slowest lane.  The network's
// round function depends on the round and on one half of the position only
// (at most 6 bits here), so its 4 x 2^hb values are tabled first (ft[256]) and a
// network evaluation costs four LDS reads instead of twelve 64-bit multiplies.
#pragma once
#include "common.h"
#include "train_tiled_bf16.h"  // OptC, opt_update

namespace {

constexpr int LN_MAX_D = 256;         // inputs: at most 4 rows of W per lane
constexpr int LN_MAX_OUT = 16;        // outputs
constexpr int LN_MAX_PER_LANE = 32;   // (rows of W per lane) x (padded outputs)
constexpr uint32_t LN_LDS_PER_WG = 64 * 1024;
constexpr int LN_EPOCH_CAP = 4096;    // rows whose epoch order is tabled in LDS

__host__ __device__ inline int ln_stride(int d) { return (d + 1) | 1; }
__host__ __device__ inline int ln_co(int c) { return c <= 1 ? 1 : (c <= 2 ? 2 : (c <= 4 ? 4 : (c <= 8 ? 8 : 16))); }
__host__ __device__ inline int ln_ki(int d) { return d <= 64 ? 1 : (d <= 128 ? 2 : 4); }  // rows of W per lane
__host__ __device__ inline int ln_epoch_rows(int64_t n) { return n <= LN_EPOCH_CAP ? (int)n : 0; }
__host__ __device__ inline uint32_t ln_wave_bytes(int d, int c, int64_t n) {
  const int co = ln_co(c);
  const int epoch_words = ln_epoch_rows(n) ? ln_epoch_rows(n) + 256 : 0;  // the row order and the round-function table
  // (ws twice: the operand copy, and the parameters of the best epoch under early stopping on held-out rows)
  return (uint32_t)(((64 * ln_stride(d) + 2 * (d + 1) * co + 64 * co + epoch_words) * 4 + 15) & ~15);
}
__host__ __device__ inline bool linear_eligible(const int32_t* dims, int L) {
  return L == 1 && dims[0] <= LN_MAX_D && dims[1] <= LN_MAX_OUT && ln_ki(dims[0]) * ln_co(dims[1]) <= LN_MAX_PER_LANE;
}
// wavefronts per workgroup for a problem shape
__host__ __device__ inline int ln_waves(int d, int c, int64_t n) {
  const int w = (int)(LN_LDS_PER_WG / ln_wave_bytes(d, c, n));
  return w < 1 ? 1 : (w > 4 ? 4 : w);
}

__device__ __forceinline__ void ln_lds_fence() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// CO consecutive floats of LDS (16-byte aligned for CO >= 4, 8-byte for CO = 2) as vector accesses
template <int CO>
__device__ __forceinline__ void lds_get(const float* p, float (&o)[CO]) {
  if constexpr (CO >= 4) {
#pragma unroll
    for (int q = 0; q < CO / 4; q++) {
      const f32x4 t = *(const f32x4*)(p + 4 * q);
#pragma unroll
      for (int e = 0; e < 4; e++) o[4 * q + e] = t[e];
    }
  } else if constexpr (CO == 2) {
    const float2 t = *(const float2*)p;
    o[0] = t.x;
    o[1] = t.y;
  } else {
    o[0] = p[0];
  }
}
template <int CO>
__device__ __forceinline__ void lds_put(float* p, const float (&o)[CO]) {
  if constexpr (CO >= 4) {
#pragma unroll
    for (int q = 0; q < CO / 4; q++) *(f32x4*)(p + 4 * q) = f32x4{o[4 * q], o[4 * q + 1], o[4 * q + 2], o[4 * q + 3]};
  } else if constexpr (CO == 2) {
    *(float2*)p = float2{o[0], o[1]};
  } else {
    p[0] = o[0];
  }
}

__device__ inline double wave_sum(double v) {
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  return v;
}

template <int CO, int KI>
struct Linear {
  const TrainParams& P;
  float* xs;
  float* ws;
  float* ds;
  float* wbest; // parameters of the best epoch so far (early stopping on held-out rows), unrounded
  int32_t* ep;  // the epoch's rows in visiting order, or null: permuted on the fly
  int lane, d, c, S, Pn;
  int r0, k0, q64, r64;  // element `lane` of a chunk's row-major block, and the step of 64 elements

  // a product's operand: rounded to bfloat16 in that mode
  __device__ __forceinline__ float opnd(float x) const { return P.x_bf16 ? (float)(__bf16)x : x; }
  __device__ __forceinline__ void put_weights(int k, const float (&wr)[CO]) const {
    float o[CO];
#pragma unroll
    for (int j = 0; j < CO; j++) o[j] = opnd(wr[j]);
    lds_put<CO>(ws + k * CO, o);
  }

  // rows of the chunk -> xs; `row` is the lane's row or -1
  __device__ __forceinline__ void stage(int row, int mbc) const {
    if (P.x_bf16)
      stage_as<__bf16>(row, mbc);
    else
      stage_as<float>(row, mbc);
  }
  template <typename XT>
  __device__ __forceinline__ void stage_as(int row, int mbc) const {
    const XT* X = (const XT*)P.X;
    const int total = mbc * d;
    int r = r0, k = k0;
    // eight loads in flight, then their eight LDS stores
    for (int e0 = 0; e0 < total; e0 += 64 * 8) {
      float v[8];
      int at[8];
#pragma unroll
      for (int u = 0; u < 8; u++) {
        const int rr = __shfl(row, r & 63);
        const bool in = e0 + 64 * u + lane < total;
        v[u] = (float)X[in ? rr * d + k : 0];  // n * d < 2^31 (checked by the host)
        at[u] = in ? r * S + k : -1;
        k += r64;
        r += q64;
        if (k >= d) {
          k -= d;
          r++;
        }
      }
#pragma unroll
      for (int u = 0; u < 8; u++)
        if (at[u] >= 0) xs[at[u]] = v[u];
    }
    ln_lds_fence();
  }

  // ep[p] = row visited at position p of the epoch with key ke
  // (n_tr = rows the model is fitted on; with an early-stopping cut their positions in the training list go
  // through the cut's own bijection)
  __device__ __forceinline__ void epoch_order(uint64_t ke, const int32_t* tr, const RowSplit& sp) const {
    const int n_tr = sp.n_fit;
    if (n_tr <= 1) {
      if (lane < n_tr) ep[lane] = 0;
    } else {
      const PermDomain dm = perm_domain((uint32_t)n_tr);  // n_tr <= 4096: halves of at most 6 bits
      uint32_t* ft = (uint32_t*)(ep + ln_epoch_rows(P.n));
      for (int i = lane; i < (4 << dm.hb); i += 64)
        ft[i] = (uint32_t)key_fold(ke, ((uint64_t)(i >> dm.hb) << 32) | ((uint32_t)i & dm.mask)) & dm.mask;
      ln_lds_fence();
      int p = lane;
      uint32_t x = (uint32_t)p;
      while (p < n_tr) {
        {  // one application of the network (the loop body of perm_index) from the table
          uint32_t Lh = x >> dm.hb, Rh = x & dm.mask;
#pragma unroll
          for (int r = 0; r < 4; r++) {
            const uint32_t t = Lh ^ ft[(r << dm.hb) + Rh];
            Lh = Rh;
            Rh = t;
          }
          x = (Lh << dm.hb) | Rh;
        }
        if (x < (uint32_t)n_tr) {
          ep[p] = (int32_t)x;
          p += 64;
          x = (uint32_t)p;
        }
      }
    }
    ln_lds_fence();
    // positions in the training list -> rows, eight loads in flight
    for (int p0 = 0; p0 < n_tr; p0 += 64 * 8) {
      int32_t v[8];
#pragma unroll
      for (int u = 0; u < 8; u++) {
        const int q = p0 + 64 * u + lane;
        const int at = q < n_tr ? ep[q] : 0;
        v[u] = tr[sp.n_hold ? (int)perm_index(sp.ksplit, (uint32_t)sp.n_tr, (uint32_t)at) : at];
      }
#pragma unroll
      for (int u = 0; u < 8; u++) {
        const int q = p0 + 64 * u + lane;
        if (q < n_tr) ep[q] = v[u];
      }
    }
    ln_lds_fence();
  }
  // the lane's row of the chunk of `left` rows that starts at position `pos` of the epoch
  __device__ __forceinline__ int chunk_row(uint64_t ke, const int32_t* tr, const RowSplit& sp, int pos, int left) const {
    if (lane >= min(64, left)) return -1;
    return ep ? ep[pos + lane] : tr[fit_index(sp, ke, (uint32_t)(pos + lane))];
  }

  // the label (class id or target, as stored) of a row, 0 for no row
  __device__ __forceinline__ uint32_t label(int row) const { return row >= 0 ? ((const uint32_t*)P.y)[row] : 0u; }

  // outputs of the lane's row
  __device__ __forceinline__ void forward(float (&z)[CO]) const {
    const float* xr = xs + lane * S;
    lds_get<CO>(ws + d * CO, z);
#pragma unroll 4
    for (int k = 0; k < d; k++) {
      const float x = xr[k];
      float wk[CO];
      lds_get<CO>(ws + k * CO, wk);
#pragma unroll
      for (int j = 0; j < CO; j++) z[j] += x * wk[j];
    }
  }

  // loss, prediction statistic and (TRAIN) output delta of the lane's row
  template <bool TRAIN>
  __device__ __forceinline__ void outputs(const float (&z)[CO], int row, uint32_t yraw, float inv_mb, double& lsum,
                                          double& hits) const {
    float dl[CO];
#pragma unroll
    for (int j = 0; j < CO; j++) dl[j] = 0.f;
    if (row >= 0) {
      if (P.n_classes >= 2) {
        const int yr = (int)yraw;
        float mx = z[0], zy = z[0];
        int best = 0;
#pragma unroll
        for (int j = 1; j < CO; j++)
          if (j < c) {
            if (z[j] > mx) {
              mx = z[j];
              best = j;
            }
            zy = j == yr ? z[j] : zy;
          }
        float se = 0.f;
#pragma unroll
        for (int j = 0; j < CO; j++)
          if (j < c) se += expf(z[j] - mx);
        const float lse = mx + logf(se);
        lsum += (double)(lse - zy);
        hits += best == yr ? 1.0 : 0.0;
        if (TRAIN) {
#pragma unroll
          for (int j = 0; j < CO; j++)
            if (j < c) dl[j] = (expf(z[j] - lse) - (j == yr ? 1.f : 0.f)) * inv_mb;
        }
      } else if (P.n_classes == 1) {
        const int yr = (int)yraw;
        const float zz = z[0];
        lsum += (double)(fmaxf(zz, 0.f) + log1pf(expf(-fabsf(zz))) - (yr ? zz : 0.f));
        hits += (zz > 0.f) == (yr != 0) ? 1.0 : 0.0;
        if (TRAIN) dl[0] = (1.f / (1.f + expf(-zz)) - (float)yr) * inv_mb;
      } else {
        const float e0 = z[0] - __uint_as_float(yraw);
        lsum += TRAIN ? 0.5 * (double)e0 * (double)e0 : (double)e0 * (double)e0;
        hits += (double)fabsf(e0);  // the absolute error
        if (TRAIN) dl[0] = e0 * inv_mb;
      }
    }
    if (TRAIN) {
#pragma unroll
      for (int j = 0; j < CO; j++) dl[j] = opnd(dl[j]);
      lds_put<CO>(ds + lane * CO, dl);
      ln_lds_fence();
    }
  }

  // Loss and second score, summed per lane, of `count` rows of a list (taken as it stands, or the rows of the
  // training list that the early-stopping cut sets aside) under the current weights.
  __device__ __forceinline__ void score_rows(const int32_t* list, const RowSplit& sp, int mode, int count, double& lsum,
                                             double& hits) const {
    auto row_at = [&](int p) { return p < count ? list[row_index(sp, mode, 0, (uint32_t)p)] : -1; };
    int vrow = row_at(lane);
    uint32_t vlab = label(vrow);
    for (int off = 0; off < count; off += 64) {
      const int mbc = min(64, count - off);
      const int row = vrow;
      const uint32_t lab = vlab;
      vrow = row_at(off + 64 + lane);
      stage(row, mbc);
      float z[CO];
      forward(z);
      outputs<false>(z, row, lab, 0.f, lsum, hits);
      ln_lds_fence();
      vlab = label(vrow);
    }
  }

  __device__ void run(const ItemDesc& it) const {
    const int f = it.fold, fl = f - P.fold_base;
    const int n_tr = P.counts[2 * fl], n_va = P.counts[2 * fl + 1];
    const int32_t* tr = P.train_idx + (int64_t)fl * P.n;
    const int32_t* va = P.val_idx + (int64_t)fl * P.n;
    const uint64_t km = key_model(it.seed, f);
    const RowSplit sp = row_split(km, it.patience, it.val_frac, n_tr);
    const int n_fit = sp.n_fit;
    const int bs = eff_batch(it.batch_size, n_fit);
    const int steps = n_fit > 0 ? (n_fit + bs - 1) / bs : 0;
    const int epochs = it.epochs, patience = it.patience;
    const float lr0 = it.lr, alpha = it.alpha, power_t = it.power_t, tol = it.tol, beta1 = it.beta1, beta2 = it.beta2;
    const bool traced = P.trace_item == it.b * P.n_folds + fl;

    OptC oc;
    oc.adam = it.solver == BBO_ADAM;
    oc.nest = it.nesterov != 0;
    oc.b1 = beta1;
    oc.b2 = beta2;
    oc.omb1 = 1.f - beta1;
    oc.omb2 = 1.f - beta2;
    oc.eps = it.eps;
    oc.mu = it.momentum;
    oc.lr = lr0;
    oc.lr_t = lr0;
    oc.am = 0.f;

    // the lane's parameters and moments
    float w[KI][CO], m[KI][CO], v[KI][CO];
    float bw = 0.f, bm = 0.f, bv = 0.f;  // lane j < c: the bias of output j
    double b1t = 1.0, b2t = 1.0;
    int64_t gstep = 0;
    int e0 = 0, st0 = 0;
    const bool resume = traced && P.state_in && steps > 0;
    if (resume) {
      gstep = P.step_begin;
      e0 = (int)(gstep / steps);
      st0 = (int)(gstep % steps);
      for (int64_t i = 0; i < gstep; i++) {  // beta^gstep by repeated products, as the free run builds it
        b1t *= (double)beta1;
        b2t *= (double)beta2;
      }
    }
    {
      const uint64_t kw = key_fold(km, 16), kb = key_fold(km, 17);
      const float bound = it.bound[0];
#pragma unroll
      for (int i = 0; i < KI; i++) {
        const int k = lane + 64 * i;
#pragma unroll
        for (int j = 0; j < CO; j++) {
          w[i][j] = m[i][j] = v[i][j] = 0.f;
          if (k < d && j < c) {
            const int p = k * c + j;  // the packed W[in][out], b[out] order
            if (resume) {
              w[i][j] = P.state_in[p];
              m[i][j] = P.state_in[Pn + p];
              v[i][j] = P.state_in[2 * Pn + p];
            } else {
              const uint32_t k24 = (uint32_t)(key_fold(kw, (uint64_t)p) >> 40);
              w[i][j] = bound * ((float)((int32_t)k24 - 8388608) * 0x1p-23f);
            }
          }
        }
        if (k < d) put_weights(k, w[i]);
      }
      if (lane < c) {
        if (resume) {
          bw = P.state_in[d * c + lane];
          bm = P.state_in[Pn + d * c + lane];
          bv = P.state_in[2 * Pn + d * c + lane];
        } else {
          const uint32_t k24 = (uint32_t)(key_fold(kb, (uint64_t)lane) >> 40);
          bw = bound * ((float)((int32_t)k24 - 8388608) * 0x1p-23f);
        }
      }
      if (lane < CO) ws[d * CO + lane] = bw;
      ln_lds_fence();
    }

    Plateau plateau;
    bool have_best = false;
    const bool watch = patience > 0 && steps > 0 && !resume;
    for (int e = e0; e < epochs; e++) {
      const uint64_t ke = key_epoch(km, e);
      if (!oc.adam) oc.lr = epoch_lr(lr0, power_t, e, n_fit);
      double esum = 0.0;  // the lane's share of the epoch's summed data loss
      // The lane's row of a chunk and its label are fetched one chunk ahead within the epoch.
      const int st_first = e == e0 ? st0 : 0;
      int nrow = -1;
      if (st_first < steps) {
        if (ep) epoch_order(ke, tr, sp);
        const int lo = st_first * bs;
        nrow = chunk_row(ke, tr, sp, lo, min(bs, n_fit - lo));
      }
      uint32_t nlab = label(nrow);
      for (int st = st_first; st < steps; st++, gstep++) {
        const int lo = st * bs, mb = min(bs, n_fit - lo);
        const float inv_mb = 1.f / (float)mb;
        float g[KI][CO];
#pragma unroll
        for (int i = 0; i < KI; i++)
#pragma unroll
          for (int j = 0; j < CO; j++) g[i][j] = 0.f;
        float bg = 0.f;
        double lstep = 0.0, unused = 0.0;
        for (int c0 = 0; c0 < mb; c0 += 64) {
          const int mbc = min(64, mb - c0);
          const int row = nrow;
          const uint32_t lab = nlab;
          {  // the next chunk of the epoch: the rest of this step, else the start of the next one
            const bool same = c0 + 64 < mb;
            const int nlo = same ? lo + c0 + 64 : lo + mb;
            const int nleft = same ? mb - c0 - 64 : (st + 1 < steps ? min(bs, n_fit - nlo) : 0);
            nrow = chunk_row(ke, tr, sp, nlo, nleft);
          }
          stage(row, mbc);
          float z[CO];
          forward(z);
          outputs<true>(z, row, lab, inv_mb, lstep, unused);
          // gradient: the lane's rows of W over the chunk's rows
#pragma unroll 4
          for (int r = 0; r < mbc; r++) {
            float dr[CO];
            lds_get<CO>(ds + r * CO, dr);
#pragma unroll
            for (int i = 0; i < KI; i++) {
              const float x = xs[r * S + min(lane + 64 * i, d - 1)];
#pragma unroll
              for (int j = 0; j < CO; j++) g[i][j] += x * dr[j];
            }
            bg += ds[r * CO + min(lane, CO - 1)];
          }
          ln_lds_fence();  // the next chunk overwrites xs and ds
          nlab = label(nrow);
        }
        esum += lstep;
        float* rec = nullptr;
        if (traced && gstep >= P.step_begin && gstep < P.step_end) {
          rec = P.trace_out + (gstep - P.step_begin) * (1 + 2 * (int64_t)Pn);
          double pen = 0.0;
#pragma unroll
          for (int i = 0; i < KI; i++)
#pragma unroll
            for (int j = 0; j < CO; j++)
              if (lane + 64 * i < d && j < c) pen += (double)w[i][j] * (double)w[i][j];
          const double data = wave_sum(lstep) / (double)mb;
          pen = wave_sum(pen);
          if (lane == 0) rec[0] = (float)(data + 0.5 * (double)alpha * pen / (double)mb);
        }
        oc.am = alpha / (float)mb;
        if (oc.adam) {
          b1t *= (double)beta1;
          b2t *= (double)beta2;
          oc.lr_t = (float)((double)lr0 * sqrt(1.0 - b2t) / (1.0 - b1t));
        }
#pragma unroll
        for (int i = 0; i < KI; i++) {
          const int k = lane + 64 * i;
          if (k < d) {
#pragma unroll
            for (int j = 0; j < CO; j++)
              if (j < c) {
                const float gg = g[i][j] + oc.am * w[i][j];
                opt_update(oc, gg, w[i][j], m[i][j], v[i][j]);
                if (rec) {
                  rec[1 + k * c + j] = gg;
                  rec[1 + Pn + k * c + j] = w[i][j];
                }
              }
            put_weights(k, w[i]);
          }
        }
        if (lane < c) {
          opt_update(oc, bg, bw, bm, bv);
          if (rec) {
            rec[1 + d * c + lane] = bg;
            rec[1 + Pn + d * c + lane] = bw;
          }
          ws[d * CO + lane] = bw;
        }
        ln_lds_fence();
      }
      if (watch) {
        float watched = (float)(wave_sum(esum) / (double)n_fit);
        if (sp.n_hold) {  // the loss of the rows set aside for early stopping, under the weights the epoch ends with
          double hl = 0.0, hh = 0.0;
          score_rows(tr, sp, ROWS_HELD, sp.n_hold, hl, hh);
          watched = (float)(wave_sum(hl) / (double)sp.n_hold);
        }
        const bool stop = plateau.stop_after(watched, tol, patience);
        if (sp.n_hold && plateau.improved) {  // keep the best epoch's parameters: every lane parks its own
#pragma unroll
          for (int i = 0; i < KI; i++)
            if (lane + 64 * i < d) lds_put<CO>(wbest + (lane + 64 * i) * CO, w[i]);
          if (lane < CO) wbest[d * CO + lane] = bw;
          have_best = true;
        }
        if (stop) break;
      }
    }
    if (have_best) {  // early stopping on held-out rows scores the best epoch's model
      ln_lds_fence();
#pragma unroll
      for (int i = 0; i < KI; i++)
        if (lane + 64 * i < d) {
          lds_get<CO>(wbest + (lane + 64 * i) * CO, w[i]);
          put_weights(lane + 64 * i, w[i]);
        }
      if (lane < CO) {
        bw = wbest[d * CO + lane];
        ws[d * CO + lane] = bw;
      }
      ln_lds_fence();
    }

    // validation score on the held rows
    double lsum = 0.0, hits = 0.0;
    score_rows(va, sp, ROWS_PLAIN, n_va, lsum, hits);
    lsum = wave_sum(lsum);
    hits = wave_sum(hits);
    if (lane == 0) {
      float* out = P.item_out + 2 * ((int64_t)it.b * P.n_folds + fl);
      out[0] = n_va > 0 ? (float)(lsum / (double)n_va) : __builtin_nanf("");
      out[1] = n_va > 0 ? (float)(hits / (double)n_va) : __builtin_nanf("");  // accuracy | mean absolute error
    }
  }
};

// CO: outputs padded to 1, 2, 4, 8 or 16; KI: rows of W per lane (1, 2 or 4).  The launch gives
// blockDim.x / 64 wavefronts ln_wave_bytes() of dynamic LDS each.
template <int CO, int KI>
__global__ __launch_bounds__(256) void k_train_linear(const TrainParams P) {
  extern __shared__ __align__(16) char ln_lds[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int d = P.d, c = P.n_classes >= 2 ? P.n_classes : 1, S = ln_stride(d), Pn = (d + 1) * c;
  float* xs = (float*)(ln_lds + (size_t)wave * ln_wave_bytes(d, c, P.n));
  float* ws = xs + 64 * S;
  float* ds = ws + (d + 1) * CO;
  float* wbest = ds + 64 * CO;
  int32_t* ep = ln_epoch_rows(P.n) ? (int32_t*)(wbest + (d + 1) * CO) : nullptr;
  Linear<CO, KI> T{P, xs, ws, ds, wbest, ep, lane, d, c, S, Pn, lane / d, lane % d, 64 / d, 64 % d};
  for (;;) {
    // Every lane takes part in the pop (lane 0 adds one, the others nothing) and lane 0's result is the
    // wavefront's item.  A pop under `if (lane == 0)` must not be used here: the loop body ends with
    // another branch on the same condition, and the compiler joins the two across the back edge, which
    // sends lanes 1..63 round the loop on their own, past the pop.
    __builtin_amdgcn_wave_barrier();
    const int item = __builtin_amdgcn_readfirstlane(atomicAdd(P.queue, lane == 0 ? 1 : 0));
    if (item >= P.n_items) break;
    T.run(((const ItemDesc*)P.items)[item]);
  }
}

}  // namespace
