// LDS-tiled training / scoring kernel for bf16 models with one or two hidden
// layers (the "scale-up" shape: up to 256 inputs, hidden widths up to 256, up
// to 16 outputs).
//
// One workgroup (8 waves) trains one model.  A minibatch is processed in
// chunks of 128 rows whose activations live entirely in LDS:
//   buf[0]: level 0 (gathered inputs), later level 2 and its delta
//   buf[1]: level 1 and its delta
//   dbuf  : output-layer delta
// each row-major [row][unit] with 16 pad columns, the first of which is 1 on
// real rows (it turns the weight-gradient GEMM into weight + bias gradient).
//
// Forward / data-gradient GEMMs are output-stationary with the weight matrix
// as the MFMA A operand (16-byte rows straight from global/L2, each wave owns
// a slice of the output units and so streams only that slice of the weights) and the
// LDS activations as the B operand; results go back to LDS as 8-byte stores,
// deltas overwrite the activations they are masked by.  Weight-gradient GEMMs
// contract over the rows: both operands come from the row-major LDS buffers
// through the transposing LDS read (ds_read_b64_tr_b16), which hands each
// lane the four row-consecutive values of its own unit.  The optimizer update
// runs in the weight-gradient epilogue on the accumulator registers: it reads
// and writes the fp32 master weights and moments once per step and emits the
// two bf16 operand copies ([out][in] for forward, [in][out] for backward, the
// latter double-buffered because the backward GEMM of the same step still
// needs the old weights).  With more than one chunk per step the partial
// gradients of the earlier chunks pass through an fp32 scratch in global
// memory.
#pragma once
#include <type_traits>

#include "common.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

constexpr int TB_ROWS = 128;  // rows per chunk
constexpr int TB_PAD = 16;    // pad columns per LDS row
constexpr int TB_MAXL = 3;    // weight layers
constexpr int TB_MAXU = 256;  // padded units per level
constexpr int TB_WAVES = 8;                   // waves per workgroup (2 per SIMD)
constexpr int TB_THREADS = 64 * TB_WAVES;
constexpr int TB_TPN = 16 / TB_WAVES > 1 ? 2 : 1;  // out tiles per wave in the rows-contracting GEMM
constexpr int TB_TPW = (16 + TB_WAVES - 1) / TB_WAVES;  // unit tiles per wave in the unit-split GEMMs
constexpr uint32_t TB_LDS_LIMIT = 160 * 1024 - 2048;  // dynamic LDS available to the kernel

struct TLay {
  int32_t L;
  int32_t U[TB_MAXL + 1];   // units per level: inputs, hidden..., outputs
  int32_t UP[TB_MAXL + 1];  // padded to 32 (levels < L) or 16 (outputs)
  int32_t S[2];             // LDS row strides in elements
  int32_t cw[TB_MAXL], cb[TB_MAXL], P;
  uint32_t lds_buf[2], lds_delta, lds_rows, lds_total;
  uint64_t w[TB_MAXL], m[TB_MAXL], v[TB_MAXL], gp[TB_MAXL], oi[TB_MAXL], io[TB_MAXL][2], bias[TB_MAXL], total;
};

__host__ __device__ inline bool tiled_eligible(const int32_t* dims, int L) {
  if (L < 2 || L > TB_MAXL) return false;
  if (dims[0] % 8 != 0 || dims[0] > TB_MAXU || dims[L] > 16) return false;
  for (int u = 1; u < L; u++)
    if (dims[u] > TB_MAXU) return false;
  return true;
}

__host__ __device__ inline void make_tlay(TLay& y, const int32_t* dims, int L) {
  y.L = L;
  y.S[0] = y.S[1] = 0;
  for (int u = 0; u <= L; u++) {
    y.U[u] = dims[u];
    y.UP[u] = u < L ? rup(dims[u], 32) : 16;
    if (u < L && y.UP[u] + TB_PAD > y.S[u & 1]) y.S[u & 1] = y.UP[u] + TB_PAD;
  }
  int c = 0;
  for (int l = 0; l < L; l++) {
    y.cw[l] = c;
    c += dims[l] * dims[l + 1];
    y.cb[l] = c;
    c += dims[l + 1];
  }
  y.P = c;
  uint32_t lo = 0;
  y.lds_buf[0] = lo;
  lo += TB_ROWS * y.S[0] * 2;
  y.lds_buf[1] = lo;
  lo += TB_ROWS * y.S[1] * 2;
  y.lds_delta = lo;
  lo += TB_ROWS * 16 * 2;
  y.lds_rows = lo;
  lo += TB_ROWS * 4;
  y.lds_total = lo;
  uint64_t off = 0;
  auto take = [&](uint64_t bytes) {
    uint64_t o = off;
    off += (bytes + 255) & ~(uint64_t)255;
    return o;
  };
  for (int l = 0; l < L; l++) {
    const uint64_t wn = (uint64_t)y.UP[l + 1] * (y.UP[l] + TB_PAD);
    y.w[l] = take(wn * 4);
    y.m[l] = take(wn * 4);
    y.v[l] = take(wn * 4);
    y.gp[l] = take(wn * 4);
    y.oi[l] = take((uint64_t)y.UP[l + 1] * y.UP[l] * 2);
    y.io[l][0] = y.io[l][1] = 0;
    if (l >= 1) {
      y.io[l][0] = take((uint64_t)y.UP[l] * y.UP[l + 1] * 2);
      y.io[l][1] = take((uint64_t)y.UP[l] * y.UP[l + 1] * 2);
    }
    y.bias[l] = take((uint64_t)y.UP[l + 1] * 4);
  }
  y.total = off;
}

// What the host stages per item for this kernel: the description and its
// layout, read by the kernel through scalar loads (the address is uniform).
struct TItem {
  ItemDesc d;
  TLay y;
};

struct OptC {
  bool adam, nest;
  float b1, b2, omb1, omb2, eps, lr_t, mu, lr, am;
};

__device__ inline void opt_update(const OptC& c, float g, float& w, float& m, float& v) {
  if (c.adam) {
    m = c.b1 * m + c.omb1 * g;
    v = c.b2 * v + c.omb2 * (g * g);
    // hardware reciprocal and square root (1 ulp each): far inside the per-step tolerance
    w = w - (c.lr_t * m) * __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(v) + c.eps);
  } else {
    const float u = c.mu * m - c.lr * g;
    m = u;
    w = w + (c.nest ? c.mu * u - c.lr * g : u);
  }
}

// Transposing LDS read: within each group of 16 lanes the 16 x 4 values that
// the lanes address (lane t: 4 consecutive units of row t/4, unit offset
// 4*(t%4)) come back transposed, lane t holding unit t of the 4 rows.
__device__ inline s16x4 lds_read_tr(const char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)p);
}

// Operand of a rows-contracting MFMA for the 16 units starting at u0 and the
// 32 rows starting at r0 of a row-major LDS buffer with row stride ld.
__device__ inline bf16x8 lds_operand_tr(const char* base, int ld, int r0, int u0, int li, int q) {
  const char* p = base + ((size_t)(r0 + 8 * q + (li >> 2)) * ld + u0 + 4 * (li & 3)) * 2;
  union {
    struct {
      s16x4 lo, hi;
    } s;
    bf16x8 v;
  } u;
  u.s.lo = lds_read_tr(p);
  u.s.hi = lds_read_tr(p + (size_t)4 * ld * 2);
  return u.v;
}

struct Tiled {
  const TrainParams& P;
  const ItemDesc& it;
  const TLay& y;
  char* slot;
  char* lds;
  double* red;

  __device__ float* fp(uint64_t off) const { return (float*)(slot + off); }
  __device__ __bf16* bp(uint64_t off) const { return (__bf16*)(slot + off); }
  __device__ char* buf(int level) const { return lds + y.lds_buf[level & 1]; }
  __device__ __forceinline__ int stride(int level) const { return y.S[level & 1]; }
  __device__ int32_t* rowlist() const { return (int32_t*)(lds + y.lds_rows); }

  // ---- parameters -------------------------------------------------------
  __device__ __forceinline__ void store_param(int l, int k, int j, bool isb, float val, int par) const {
    const int ldw = y.UP[l] + TB_PAD;
    if (isb) {
      fp(y.w[l])[(size_t)j * ldw + y.UP[l]] = val;
      fp(y.bias[l])[j] = val;
    } else {
      fp(y.w[l])[(size_t)j * ldw + k] = val;
      bp(y.oi[l])[(size_t)j * y.UP[l] + k] = (__bf16)val;
      if (l >= 1) bp(y.io[l][par])[(size_t)k * y.UP[l + 1] + j] = (__bf16)val;
    }
  }

  __device__ __forceinline__ void init_params() const {
    const uint64_t km = key_model(it.seed, it.fold);
    for (int l = 0; l < y.L; l++) {
      const int fi = y.U[l], fo = y.U[l + 1];
      const uint64_t kw = key_fold(km, 16 + 2 * l), kb = key_fold(km, 16 + 2 * l + 1);
      const float bound = it.bound[l];
      for (int i = threadIdx.x; i < fi * fo + fo; i += blockDim.x) {
        const bool isb = i >= fi * fo;
        const int e = isb ? i - fi * fo : i;
        const uint32_t k24 = (uint32_t)(key_fold(isb ? kb : kw, (uint64_t)e) >> 40);
        const float val = bound * ((float)((int32_t)k24 - 8388608) * 0x1p-23f);
        store_param(l, isb ? 0 : e / fo, isb ? e : e % fo, isb, val, 0);
      }
    }
  }

  __device__ __forceinline__ void load_state(const float* st, int par) const {
    for (int l = 0; l < y.L; l++) {
      const int fi = y.U[l], fo = y.U[l + 1], ldw = y.UP[l] + TB_PAD;
      for (int i = threadIdx.x; i < fi * fo + fo; i += blockDim.x) {
        const bool isb = i >= fi * fo;
        const int e = isb ? i - fi * fo : i;
        const int k = isb ? y.UP[l] : e / fo, j = isb ? e : e % fo;
        const int ci = (isb ? y.cb[l] : y.cw[l]) + e;
        store_param(l, k, j, isb, st[ci], par);
        fp(y.m[l])[(size_t)j * ldw + k] = st[y.P + ci];
        fp(y.v[l])[(size_t)j * ldw + k] = st[2 * y.P + ci];
      }
    }
  }

  // ---- chunk staging -----------------------------------------------------
  // Row list of the chunk, the gathered input rows into the level-0 buffer,
  // and that buffer's pad columns.
  __device__ __forceinline__ void stage_rows(const int32_t* list, uint64_t key, int n_list, int lo, int rows, bool permute,
                             bool want_list) const {
    int32_t* rl = rowlist();
    if (want_list) {
      for (int p = threadIdx.x; p < TB_ROWS; p += blockDim.x)
        rl[p] = p < rows ? list[permute ? perm_index(key, (uint32_t)n_list, (uint32_t)(lo + p)) : lo + p] : -1;
      __syncthreads();
    }
    const int d = y.U[0], up0 = y.UP[0], S0 = stride(0), vpr = up0 / 8;
    char* b0 = buf(0);
    const __bf16* X = (const __bf16*)P.X;
    for (int idx = threadIdx.x; idx < TB_ROWS * vpr; idx += blockDim.x) {
      const int r = idx / vpr, vv = idx - r * vpr;
      const int row = rl[r];
      uint4 val = uint4{0, 0, 0, 0};
      if (row >= 0 && vv * 8 < d) val = *(const uint4*)(X + (size_t)row * d + vv * 8);
      *(uint4*)(b0 + ((size_t)r * S0 + vv * 8) * 2) = val;
    }
    write_pad(0);
  }

  // Pad columns of a level's buffer: column UP is 1 on real rows, the rest 0.
  __device__ __forceinline__ void write_pad(int level) const {
    const int32_t* rl = rowlist();
    char* b = buf(level);
    const int S = stride(level), up = y.UP[level];
    for (int r = threadIdx.x; r < TB_ROWS; r += blockDim.x) {
      uint4 one = uint4{rl[r] >= 0 ? 0x3F80u : 0u, 0, 0, 0};  // bf16 1.0 in the low half
      *(uint4*)(b + ((size_t)r * S + up) * 2) = one;
      *(uint4*)(b + ((size_t)r * S + up + 8) * 2) = uint4{0, 0, 0, 0};
    }
  }

  // ---- GEMMs --------------------------------------------------------------
  // D[unit][row] = sum_k A[unit][k] * B[row][k]; A: global bf16 [units][lda],
  // B: LDS rows.  Wave w owns unit tiles w, w+NW, ... and all row blocks.
  template <int KS, bool FULL, typename Epi>
  __device__ __forceinline__ void gemm_units_t(const __bf16* __restrict__ A, int lda, const char* Bl, int ldb, int nt, int njb_,
                               int K, Epi epi) const {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, li = lane & 15, q = lane >> 4;
    const int njb = FULL ? 8 : njb_;  // a full chunk has all eight row blocks: no guards in the inner loops
    if (w >= nt) return;
    f32x4 acc[TB_TPW][8];
#pragma unroll
    for (int i = 0; i < TB_TPW; i++)
#pragma unroll
      for (int j = 0; j < 8; j++) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (KS == 32) {
      for (int k0 = 0; k0 < K; k0 += 32) {
        bf16x8 a[TB_TPW], b[8];
#pragma unroll
        for (int i = 0; i < TB_TPW; i++)
          if (w + TB_WAVES * i < nt)
            a[i] = *(const bf16x8*)(A + (size_t)((w + TB_WAVES * i) * 16 + li) * lda + k0 + q * 8);
#pragma unroll
        for (int j = 0; j < 8; j++)
          if (j < njb) b[j] = *(const bf16x8*)(Bl + ((size_t)(j * 16 + li) * ldb + k0 + q * 8) * 2);
#pragma unroll
        for (int i = 0; i < TB_TPW; i++)
          if (w + TB_WAVES * i < nt) {
#pragma unroll
            for (int j = 0; j < 8; j++)
              if (j < njb) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
          }
      }
    } else {  // K == 16: one MFMA of depth 16
      bf16x4 a[TB_TPW], b[8];
#pragma unroll
      for (int i = 0; i < TB_TPW; i++)
        if (w + TB_WAVES * i < nt) a[i] = *(const bf16x4*)(A + (size_t)((w + TB_WAVES * i) * 16 + li) * lda + q * 4);
#pragma unroll
      for (int j = 0; j < 8; j++)
        if (j < njb) b[j] = *(const bf16x4*)(Bl + ((size_t)(j * 16 + li) * ldb + q * 4) * 2);
#pragma unroll
      for (int i = 0; i < TB_TPW; i++)
        if (w + TB_WAVES * i < nt) {
#pragma unroll
          for (int j = 0; j < 8; j++)
            if (j < njb) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a[i], b[j], acc[i][j], 0, 0, 0);
        }
    }
#pragma unroll
    for (int i = 0; i < TB_TPW; i++)
      if (w + TB_WAVES * i < nt) {
#pragma unroll
        for (int j = 0; j < 8; j++)
          if (j < njb) epi(acc[i][j], (w + TB_WAVES * i) * 16 + 4 * q, j * 16 + li);
      }
  }

  template <int KS, typename Epi>
  __device__ __forceinline__ void gemm_units(const __bf16* A, int lda, const char* Bl, int ldb, int nt, int njb, int K,
                             Epi epi) const {
    if (njb == 8)
      gemm_units_t<KS, true>(A, lda, Bl, ldb, nt, njb, K, epi);
    else
      gemm_units_t<KS, false>(A, lda, Bl, ldb, nt, njb, K, epi);
  }

  // Output layer: one tile of (up to 16) output units; wave w owns row block w
  // (and w+NW).  epi(acc, jb): lane holds outputs 4q..4q+3 of row jb*16+li.
  template <typename Epi>
  __device__ __forceinline__ void gemm_out(const __bf16* __restrict__ A, int lda, const char* Bl, int ldb, int njb, int K,
                           Epi epi) const {
    constexpr int JPW = (8 + TB_WAVES - 1) / TB_WAVES;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, li = lane & 15, q = lane >> 4;
    if (w >= njb) return;
    f32x4 acc[JPW];
#pragma unroll
    for (int j = 0; j < JPW; j++) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int k0 = 0; k0 < K; k0 += 32) {
      const bf16x8 a = *(const bf16x8*)(A + (size_t)li * lda + k0 + q * 8);
#pragma unroll
      for (int j = 0; j < JPW; j++)
        if (w + TB_WAVES * j < njb) {
          const bf16x8 b = *(const bf16x8*)(Bl + ((size_t)((w + TB_WAVES * j) * 16 + li) * ldb + k0 + q * 8) * 2);
          acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[j], 0, 0, 0);
        }
    }
#pragma unroll
    for (int j = 0; j < JPW; j++)
      if (w + TB_WAVES * j < njb) epi(acc[j], w + TB_WAVES * j);
  }

  // D[in][out] = sum_rows A[row][in] * B[row][out], both operands from LDS
  // through the transposing read.  The waves form a WM x WN grid: a wave keeps
  // the B operands of its (at most two) out tiles in registers and walks the
  // in tiles wm, wm+WM, ...   pre(i0, j, slot) starts the loads the epilogue of a
  // tile will need before the tile's operand reads and MFMAs; epi(acc, i0, j,
  // slot) consumes them afterwards.
  template <typename Pre, typename Epi>
  __device__ __forceinline__ void gemm_rows(const char* Al, int lda, int Mt, const char* Bl, int ldb, int Nt, int KB, Pre pre,
                            Epi epi) const {
    if (KB == 4)
      gemm_rows_t<true>(Al, lda, Mt, Bl, ldb, Nt, KB, pre, epi);
    else
      gemm_rows_t<false>(Al, lda, Mt, Bl, ldb, Nt, KB, pre, epi);
  }

  template <bool FULL, typename Pre, typename Epi>
  __device__ __forceinline__ void gemm_rows_t(const char* Al, int lda, int Mt, const char* Bl, int ldb, int Nt, int KB_, Pre pre,
                              Epi epi) const {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, li = lane & 15, q = lane >> 4;
    const int KB = FULL ? 4 : KB_;
    const int WN = (Nt + TB_TPN - 1) / TB_TPN, WM = TB_WAVES / WN;
    const int wn = w % WN, wm = w / WN;
    if (wm >= WM) return;
    bf16x8 bop[TB_TPN][4];
    int ntile[TB_TPN];
#pragma unroll
    for (int i = 0; i < TB_TPN; i++) {
      ntile[i] = wn + WN * i;
      if (ntile[i] < Nt) {
#pragma unroll
        for (int kb = 0; kb < 4; kb++)
          if (kb < KB) bop[i][kb] = lds_operand_tr(Bl, ldb, kb * 32, ntile[i] * 16, li, q);
      }
    }
    for (int mt = wm; mt < Mt; mt += WM) {
#pragma unroll
      for (int i = 0; i < TB_TPN; i++)
        if (ntile[i] < Nt) pre(mt * 16 + 4 * q, ntile[i] * 16 + li, i);
      bf16x8 a[4];
#pragma unroll
      for (int kb = 0; kb < 4; kb++)
        if (kb < KB) a[kb] = lds_operand_tr(Al, lda, kb * 32, mt * 16, li, q);
      f32x4 acc[TB_TPN];
#pragma unroll
      for (int i = 0; i < TB_TPN; i++) {
        acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (ntile[i] < Nt) {
#pragma unroll
          for (int kb = 0; kb < 4; kb++)
            if (kb < KB) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[kb], bop[i][kb], acc[i], 0, 0, 0);
        }
      }
#pragma unroll
      for (int i = 0; i < TB_TPN; i++)
        if (ntile[i] < Nt) epi(acc[i], mt * 16 + 4 * q, ntile[i] * 16 + li, i);
    }
  }

  // ---- phases ---------------------------------------------------------------
  // Hidden layer l: level l -> level l+1 (ReLU), all in LDS.
  __device__ __forceinline__ void forward_hidden(int l, int njb) const {
    const float* bias = fp(y.bias[l]);
    char* out = buf(l + 1);
    const int So = stride(l + 1);
    write_pad(l + 1);
    gemm_units<32>(bp(y.oi[l]), y.UP[l], buf(l), stride(l), y.UP[l + 1] / 16, njb, y.UP[l],
                   [&](const f32x4& acc, int u0, int row) {
                     const f32x4 b = *(const f32x4*)(bias + u0);
                     bf16x4 pk;
#pragma unroll
                     for (int r = 0; r < 4; r++) pk[r] = (__bf16)fmaxf(acc[r] + b[r], 0.f);
                     *(bf16x4*)(out + ((size_t)row * So + u0) * 2) = pk;
                   });
    __syncthreads();
  }

  // Output layer + loss.  TRAIN: writes the output delta to dbuf and returns the
  // lane's share of the summed data loss.  Otherwise accumulates the validation
  // loss and hit count of the chunk's real rows.
  template <bool TRAIN>
  __device__ __forceinline__ void forward_out(int njb, int rows, float inv_mb, double& lsum, double& hits) const {
    const int l = y.L - 1, c = y.U[y.L];
    const float* bias = fp(y.bias[l]);
    const int32_t* rl = rowlist();
    char* db = lds + y.lds_delta;
    const int lane = threadIdx.x & 63, li = lane & 15, q = lane >> 4;
    const bool cls = P.n_classes >= 2;
    gemm_out(bp(y.oi[l]), y.UP[l], buf(l), stride(l), njb, y.UP[l], [&](const f32x4& acc, int jb) {
      const int r = jb * 16 + li;
      const int row = rl[r];
      const bool valid = r < rows && row >= 0;
      const f32x4 b = *(const f32x4*)(bias + 4 * q);
      float z[4];
#pragma unroll
      for (int e = 0; e < 4; e++) z[e] = acc[e] + b[e];
      float delta[4] = {0.f, 0.f, 0.f, 0.f};
      if (cls) {
        const int yr = valid ? ((const int32_t*)P.y)[row] : 0;
        float mx = -INFINITY;
        int best = 0;
#pragma unroll
        for (int e = 0; e < 4; e++) {
          if (4 * q + e >= c) z[e] = -INFINITY;
          if (z[e] > mx) {
            mx = z[e];
            best = 4 * q + e;
          }
        }
#pragma unroll
        for (int s = 16; s <= 32; s <<= 1) {
          const float omx = __shfl_xor(mx, s);
          const int ob = __shfl_xor(best, s);
          if (omx > mx || (omx == mx && ob < best)) {
            mx = omx;
            best = ob;
          }
        }
        float se = 0.f;
#pragma unroll
        for (int e = 0; e < 4; e++) se += expf(z[e] - mx);
        se += __shfl_xor(se, 16);
        se += __shfl_xor(se, 32);
        const float lse = mx + logf(se);
        float zy = (yr >> 2) == q ? z[yr & 3] : 0.f;
        zy += __shfl_xor(zy, 16);
        zy += __shfl_xor(zy, 32);
        if (valid && q == 0) {
          lsum += (double)(lse - zy);
          hits += best == yr;
        }
        if (TRAIN && valid) {
#pragma unroll
          for (int e = 0; e < 4; e++)
            if (4 * q + e < c) delta[e] = (expf(z[e] - lse) - (4 * q + e == yr ? 1.f : 0.f)) * inv_mb;
        }
      } else {
        const float e0 = valid ? z[0] - ((const float*)P.y)[row] : 0.f;
        if (valid && q == 0) lsum += TRAIN ? 0.5 * (double)e0 * (double)e0 : (double)e0 * (double)e0;
        if (TRAIN && q == 0) delta[0] = e0 * inv_mb;
      }
      if (TRAIN) {
        bf16x4 pk;
#pragma unroll
        for (int e = 0; e < 4; e++) pk[e] = (__bf16)delta[e];
        *(bf16x4*)(db + ((size_t)r * 16 + 4 * q) * 2) = pk;
      }
    });
    __syncthreads();
  }

  // Delta of level l (1 <= l < L) from the delta of level l+1, masked by and
  // written over the level-l activations.
  __device__ __forceinline__ void backward_data(int l, int njb, int par) const {
    char* a = buf(l);
    const int Sa = stride(l);
    auto epi = [&](const f32x4& acc, int u0, int row) {
      bf16x4* p = (bf16x4*)(a + ((size_t)row * Sa + u0) * 2);
      const bf16x4 act = *p;
      bf16x4 pk;
#pragma unroll
      for (int r = 0; r < 4; r++) pk[r] = (__bf16)((float)act[r] > 0.f ? acc[r] : 0.f);
      *p = pk;
    };
    if (l + 1 == y.L)
      gemm_units<16>(bp(y.io[l][par]), 16, lds + y.lds_delta, 16, y.UP[l] / 16, njb, 16, epi);
    else
      gemm_units<32>(bp(y.io[l][par]), y.UP[l + 1], buf(l + 1), stride(l + 1), y.UP[l] / 16, njb, y.UP[l + 1], epi);
    __syncthreads();
  }

  // Weight + bias gradient of layer l over the chunk's rows.  Every chunk but
  // the last of a step adds into the fp32 gradient scratch in global memory;
  // the last one finishes the sum and applies the optimizer in the epilogue:
  // master weights and moments are read and written once per step, and the
  // bf16 [out][in] copy, the [in][out] copy of the next step's parity and the
  // compact bias are refreshed.  The state loads are issued before the MFMAs
  // of the tile they belong to.
  __device__ __forceinline__ void wgrad(int l, int KB, bool first, bool last, const OptC& oc, int par_next, float* rec) const {
    float* W = fp(y.w[l]);
    float* Mo = fp(y.m[l]);
    float* Vo = fp(y.v[l]);
    float* Gp = fp(y.gp[l]);
    float* bias = fp(y.bias[l]);
    __bf16* oi = bp(y.oi[l]);
    __bf16* io = bp(y.io[l][par_next]);
    const int fi = y.U[l], fo = y.U[l + 1], up = y.UP[l], ldw = up + TB_PAD, ldo = y.UP[l + 1];
    const int cw = y.cw[l], cb = y.cb[l], Pn = y.P;
    const bool lastlayer = l + 1 == y.L;
    const char* Bl = lastlayer ? lds + y.lds_delta : buf(l + 1);
    const int ldb = lastlayer ? 16 : stride(l + 1);
    const bool adam = oc.adam;
    f32x4 pg[TB_TPN], pw[TB_TPN], pm[TB_TPN], pv[TB_TPN];
    auto live = [&](int i0, int j) { return j < fo && (i0 < fi || i0 == up); };
    gemm_rows(
        buf(l), stride(l), up / 16 + 1, Bl, ldb, y.UP[l + 1] / 16, KB,
        [&](int i0, int j, int s) {
          if (!live(i0, j)) return;
          const size_t o = (size_t)j * ldw + i0;
          if (!first) pg[s] = *(const f32x4*)(Gp + o);
          if (last) {
            pw[s] = *(const f32x4*)(W + o);
            pm[s] = *(const f32x4*)(Mo + o);
            if (adam) pv[s] = *(const f32x4*)(Vo + o);
          }
        },
        [&](const f32x4& acc, int i0, int j, int s) {
          if (!live(i0, j)) return;
          const bool isb = i0 == up;
          const size_t o = (size_t)j * ldw + i0;
          f32x4 g = acc;
          if (!first) {
#pragma unroll
            for (int r = 0; r < 4; r++) g[r] += pg[s][r];
          }
          if (!last) {
            *(f32x4*)(Gp + o) = g;
            return;
          }
          f32x4 w = pw[s], m = pm[s], v = adam ? pv[s] : f32x4{0.f, 0.f, 0.f, 0.f};
          bf16x4 pk;
#pragma unroll
          for (int r = 0; r < 4; r++) {
            const int i = i0 + r;
            const bool on = isb ? r == 0 : i < fi;
            float wr = w[r], mr = m[r], vr = v[r];
            if (on) {
              const float gg = isb ? g[r] : g[r] + oc.am * wr;
              opt_update(oc, gg, wr, mr, vr);
              if (rec) {
                const int ci = isb ? cb + j : cw + i * fo + j;
                rec[1 + ci] = gg;
                rec[1 + Pn + ci] = wr;
              }
              if (!isb && l >= 1) io[(size_t)i * ldo + j] = (__bf16)wr;
            }
            w[r] = wr;
            m[r] = mr;
            v[r] = vr;
            pk[r] = (__bf16)wr;
          }
          *(f32x4*)(W + o) = w;
          *(f32x4*)(Mo + o) = m;
          if (adam) *(f32x4*)(Vo + o) = v;
          if (isb)
            bias[j] = w[0];
          else
            *(bf16x4*)(oi + (size_t)j * up + i0) = pk;
        });
    __syncthreads();
  }

  __device__ __forceinline__ double penalty_sum() const {
    double s = 0.0;
    for (int l = 0; l < y.L; l++) {
      const float* W = fp(y.w[l]);
      const int fi = y.U[l], fo = y.U[l + 1], ldw = y.UP[l] + TB_PAD;
      for (int i = threadIdx.x; i < fi * fo; i += blockDim.x) {
        const float w = W[(size_t)(i / fi) * ldw + (i % fi)];
        s += (double)w * (double)w;
      }
    }
    return block_sum(s, red);
  }

  __device__ __forceinline__ void run() const {
    const int f = it.fold, L = y.L;
    const int n_tr = P.counts[2 * f], n_va = P.counts[2 * f + 1];
    const int32_t* tr = P.train_idx + (int64_t)f * P.n;
    const int32_t* va = P.val_idx + (int64_t)f * P.n;
    const int bs = eff_batch(it.batch_size, n_tr);
    const int steps = n_tr > 0 ? (n_tr + bs - 1) / bs : 0;
    const uint64_t km = key_model(it.seed, f);
    const bool traced = P.trace_item == it.b * P.n_folds + f;

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
      gstep = P.step_begin;
      load_state(P.state_in, (int)(gstep & 1));
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
        const int nch = (mb + TB_ROWS - 1) / TB_ROWS, par = (int)(gstep & 1);
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
        for (int ch = 0; ch < nch; ch++) {
          const int rows = min(TB_ROWS, mb - ch * TB_ROWS);
          const int KB = (rows + 31) / 32, njb = 2 * KB;
          stage_rows(tr, ke, n_tr, lo + ch * TB_ROWS, rows, true, true);
          __syncthreads();
          for (int l = 0; l + 1 < L; l++) forward_hidden(l, njb);
          forward_out<true>(njb, rows, inv_mb, lsum, hits);
          for (int l = L - 1; l >= 0; l--) {
            if (l == 0 && L == 3) {  // level 0 shared its buffer with level 2: gather the inputs again
              stage_rows(tr, ke, n_tr, lo + ch * TB_ROWS, rows, true, false);
              __syncthreads();
            }
            wgrad(l, KB, ch == 0, ch == nch - 1, oc, par ^ 1, rec);
            if (l >= 1) backward_data(l, njb, par);
          }
        }
        if (rec) {
          const double data = block_sum(lsum, red) / (double)mb;
          if (threadIdx.x == 0) rec[0] = (float)(data + 0.5 * (double)it.alpha * pen / (double)mb);
        }
      }
    }

    // validation score on the held rows
    double lsum = 0.0, hits = 0.0;
    for (int off = 0; off < n_va; off += TB_ROWS) {
      const int rows = min(TB_ROWS, n_va - off);
      const int njb = 2 * ((rows + 31) / 32);
      stage_rows(va, 0, n_va, off, rows, false, true);
      __syncthreads();
      for (int l = 0; l + 1 < L; l++) forward_hidden(l, njb);
      forward_out<false>(njb, rows, 0.f, lsum, hits);
    }
    lsum = block_sum(lsum, red);
    hits = block_sum(hits, red);
    if (threadIdx.x == 0) {
      float* out = P.item_out + 2 * ((int64_t)it.b * P.n_folds + f);
      out[0] = n_va > 0 ? (float)(lsum / (double)n_va) : __builtin_nanf("");
      out[1] = P.n_classes >= 2 ? (n_va > 0 ? (float)(hits / (double)n_va) : __builtin_nanf("")) : 0.f;
    }
  }
};

__global__ __launch_bounds__(TB_THREADS) void k_train_tiled(const TrainParams P) {
  extern __shared__ __align__(16) char smem[];
  __shared__ int s_item;
  __shared__ double red[TB_THREADS / 64];
  char* slot = P.slots + (uint64_t)blockIdx.x * P.slot_bytes;
  for (;;) {
    __syncthreads();
    if (threadIdx.x == 0) s_item = atomicAdd(P.queue, 1);
    __syncthreads();
    const int item = __builtin_amdgcn_readfirstlane(s_item);
    if (item >= P.n_items) break;
    const TItem* __restrict__ ti = (const TItem*)P.items + item;
    Tiled T{P, ti->d, ti->y, slot, smem, red};
    T.run();
  }
}

}  // namespace
