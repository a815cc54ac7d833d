// LDS-tiled training / scoring kernel for bf16 models with one or two hidden
// layers (the "scale-up" shape: up to 256 inputs, hidden widths up to 256, up
// to 16 outputs).
//
// One workgroup (8 waves) trains one model, one model per CU.  A minibatch of
// up to 256 rows is processed at once; its activations live in ONE row-major
// LDS buffer buf[row][unit], which every layer overwrites in place:
//
//   hidden layers, forward and data gradient: wave w owns units 32w..32w+31 of
//     the level it produces.  It fetches its tiles of the bf16 weight copy from
//     global memory as MFMA A operands (D[unit][row] = W[unit][k] . act[row][k]),
//     takes the level from the buffer as B operands, 128 rows at a time, keeps
//     the results in registers until every wave has read those rows (barrier),
//     then writes the next level over them.  ReLU masks are kept as bits in
//     registers, so a delta can overwrite the activation it is masked by.
//   output layer: one wave per 32 rows; softmax, loss and output delta in the
//     MFMA result layout; the 16-wide delta has a buffer of its own.
//   weight gradient: contraction over the rows.  The delta operand comes from
//     the LDS buffer through the transposing LDS read (ds_read_b64_tr_b16).  The
//     activation operand comes the same way for the last hidden level; lower
//     levels were overwritten by then, so each wave spills the transpose of its
//     rows to global memory before that happens (tile-blocked, read back as
//     16-byte operand vectors).  The bias gradient uses a row of ones as operand.
//   The optimizer runs in the weight-gradient epilogue on the accumulator
//   registers: fp32 master weights and moments are read (two tiles ahead) and
//   written once per step, and the bf16 [out][in] operand copy (double-buffered
//   by step parity, because the backward pass of the same step still needs the
//   old weights; the output layer keeps an [in][out] copy as well) is refreshed.
//
// The weight gradient exists three times.  wgrad_t handles every case (several
// chunks per minibatch, ragged chunks).  wgrad_stream (layers below the last)
// and wgrad_last (the output layer) handle a whole minibatch in one chunk (rows
// past a ragged chunk carry zero deltas), which is nearly every step of a run:
// straight-line tile bodies, all memory
// operations through buffer descriptors, so that the compiler's waits are exact
// and the state really is in flight two tiles ahead; for the input layer the
// activation operand is gathered from the input matrix itself, so the inputs
// are never spilled.
//
// Every global array is stored in the order its wave-level accesses touch it:
// fp32 state as 16 x 16 tiles [in tile][out tile][lane][4] (1 KB per access),
// operand copies as 16 x 16 bf16 tiles (512 B per store, 1 KB per load), spills
// as [unit tile][32-row block][unit][row].  Batches above 256 rows are processed
// in chunks whose partial gradients pass through an fp32 scratch.
#pragma once
#include <type_traits>

#include "common.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
// MFMA operands that live across loop iterations are kept as four dwords: the compiler carries vectors of
// 16-bit elements through loops half by half
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ bf16x8 as_bf16x8(i32x4 v) { return __builtin_bit_cast(bf16x8, v); }
__device__ __forceinline__ i32x4 as_i32x4(bf16x8 v) { return __builtin_bit_cast(i32x4, v); }

constexpr int TB_ROWS = 256;  // rows per chunk
constexpr int TB_PAD = 8;     // pad elements per LDS row: consecutive rows start 4 banks apart
constexpr int TB_MAXL = 3;    // weight layers
constexpr int TB_MAXU = 256;  // padded units per level
constexpr int TB_WAVES = 8;   // waves per workgroup (2 per SIMD); wave w owns rows 32w..32w+31 in the output layer and the spills
constexpr int TB_THREADS = 64 * TB_WAVES;
constexpr int TB_STATE_AHEAD = 2;  // tiles of optimizer state in flight per wave
constexpr uint32_t TB_LDS_LIMIT = 160 * 1024 - 1024;  // dynamic LDS available to the kernel
// The LDS layout is the same for every model (sized for the widest): the row stride and every offset are
// compile-time constants, so LDS addresses need no arithmetic beyond the lane's base.
constexpr int TB_S = TB_MAXU + TB_PAD;                        // LDS row stride in elements
constexpr uint32_t TB_LDS_BUF = 0;                            // buf[row][unit]
constexpr uint32_t TB_LDS_ROWS = TB_LDS_BUF + TB_ROWS * TB_S * 2;  // row list of the chunk
constexpr uint32_t TB_LDS_TARGETS = TB_LDS_ROWS + TB_ROWS * 4;     // the rows' targets (class index or value, 32 bits)
// 16 KB that serve as: output delta (8 KB) + a 16 x 16 bf16 patch per wave (4 KB) from the output layer to
// the last weight gradient, and in between as 2 KB per wave of weight staging for the hidden data gradient
constexpr uint32_t TB_LDS_STAGE = TB_LDS_TARGETS + TB_ROWS * 4;
constexpr uint32_t TB_LDS_DELTA = TB_LDS_STAGE;
constexpr uint32_t TB_LDS_TR = TB_LDS_STAGE + TB_ROWS * 16 * 2;
constexpr uint32_t TB_LDS_TOTAL = TB_LDS_STAGE + TB_WAVES * 2048;
static_assert(TB_LDS_TOTAL <= TB_LDS_LIMIT, "LDS layout does not fit");

struct TLay {
  int32_t L;
  int32_t U[TB_MAXL + 1];   // units per level: inputs, hidden..., outputs
  int32_t UP[TB_MAXL + 1];  // padded to 32 (levels < L) or 16 (outputs)
  int32_t cw[TB_MAXL], cb[TB_MAXL], P;
  uint32_t lds_total;
  uint64_t w[TB_MAXL], m[TB_MAXL], v[TB_MAXL], gp[TB_MAXL], oi[TB_MAXL][2], io[2], T[TB_MAXL];
  uint64_t bias[TB_MAXL], bm[TB_MAXL], bv[TB_MAXL], bg[TB_MAXL], total;  // bias: value, moments, partial gradient
  uint64_t wb[TB_MAXL], bb[TB_MAXL];  // weights and bias of the best epoch so far (early stopping on held-out rows)
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
  for (int u = 0; u <= L; u++) {
    y.U[u] = dims[u];
    y.UP[u] = u < L ? rup(dims[u], 32) : 16;
  }
  int c = 0;
  for (int l = 0; l < L; l++) {
    y.cw[l] = c;
    c += dims[l] * dims[l + 1];
    y.cb[l] = c;
    c += dims[l + 1];
  }
  y.P = c;
  y.lds_total = TB_LDS_TOTAL;
  uint64_t off = 0;
  auto take = [&](uint64_t bytes) {
    uint64_t o = off;
    off += (bytes + 255) & ~(uint64_t)255;
    return o;
  };
  for (int l = 0; l < L; l++) {
    const uint64_t wn = (uint64_t)y.UP[l + 1] * y.UP[l];
    y.w[l] = take(wn * 4);
    y.m[l] = take(wn * 4);
    y.v[l] = take(wn * 4);
    y.gp[l] = take(wn * 4);
    y.oi[l][0] = take((uint64_t)y.UP[l + 1] * y.UP[l] * 2);
    y.oi[l][1] = take((uint64_t)y.UP[l + 1] * y.UP[l] * 2);
    if (l == L - 1) {  // the output layer alone keeps an [in][out] copy
      y.io[0] = take((uint64_t)y.UP[l] * y.UP[l + 1] * 2);
      y.io[1] = take((uint64_t)y.UP[l] * y.UP[l + 1] * 2);
    }
    y.bias[l] = take((uint64_t)y.UP[l + 1] * 4);
    y.bm[l] = take((uint64_t)y.UP[l + 1] * 4);
    y.bv[l] = take((uint64_t)y.UP[l + 1] * 4);
    y.bg[l] = take((uint64_t)y.UP[l + 1] * 4);
    y.wb[l] = take(wn * 4);
    y.bb[l] = take((uint64_t)y.UP[l + 1] * 4);
    // transposed spill of level l: needed by the weight gradient of every layer but the last
    y.T[l] = l <= L - 2 ? take((uint64_t)y.UP[l] * TB_ROWS * 2) : 0;
  }
  y.total = off;
}

// What the host stages per item for this kernel: the description and its
// layout, read by the kernel through scalar loads (the address is uniform).
struct TItem {
  ItemDesc d;
  TLay y;
};

// The staged items are written by the host before the launch and never by a kernel: reading them through the
// constant address space lets the compiler use scalar loads and keep the layout in scalar registers.
typedef const __attribute__((address_space(4))) ItemDesc ConstItemDesc;
typedef const __attribute__((address_space(4))) TLay ConstTLay;

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
// 32 rows starting at r0 of a row-major LDS buffer with row stride ld: lane
// (li, q) gets rows r0+8q..r0+8q+7 of unit u0+li.
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

// A wave-uniform value that the compiler holds in vector registers (anything read from memory the kernel also
// writes), moved to scalar registers.
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
template <class T>
__device__ __forceinline__ T* uniform(T* p) {
  const uint64_t v = (uint64_t)p;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return (T*)(((uint64_t)hi << 32) | lo);
}

struct Tiled {
  const TrainParams& P;
  const ConstItemDesc& it;
  const ConstTLay& y;
  char* slot;
  char* lds;
  double* red;

  // The thread index as a value the compiler cannot see through: what a phase derives from it (lane
  // coordinates, LDS and global addresses) is then recomputed where it is used, in a few instructions, instead
  // of being computed once ahead of every loop and kept, mostly spilled, for the whole run.
  __device__ __forceinline__ static int tid() {
    int t = threadIdx.x;
    asm volatile("" : "+v"(t));
    return t;
  }
  __device__ __forceinline__ float* fp(uint64_t off) const { return (float*)(slot + off); }
  __device__ __forceinline__ __bf16* bp(uint64_t off) const { return (__bf16*)(slot + off); }
  __device__ __forceinline__ char* buf() const { return lds + TB_LDS_BUF; }
  __device__ __forceinline__ char* dbuf() const { return lds + TB_LDS_DELTA; }
  __device__ __forceinline__ int32_t* rowlist() const { return (int32_t*)(lds + TB_LDS_ROWS); }
  __device__ __forceinline__ int32_t* targets() const { return (int32_t*)(lds + TB_LDS_TARGETS); }

  // ---- blocked indices ------------------------------------------------------
  // state element (in unit k, out unit j) of layer l
  __device__ __forceinline__ size_t sidx(int l, int k, int j) const {
    const int nta = y.UP[l + 1] / 16;  // [in tile][out tile]: a wave walks the out tiles of one in tile
    return ((size_t)(k >> 4) * nta + (j >> 4)) * 256 + ((((k & 15) >> 2) << 4) + (j & 15)) * 4 + (k & 3);
  }
  // forward operand copy: 16 x 16 tiles [out tile][in tile][out unit][in unit]
  __device__ __forceinline__ size_t oidx(int l, int j, int k) const {
    return (((size_t)(j >> 4) * (y.UP[l] / 16) + (k >> 4)) * 16 + (j & 15)) * 16 + (k & 15);
  }
  // backward operand copy: 16 x 16 tiles [in tile][out tile][in unit][out unit]
  __device__ __forceinline__ size_t iidx(int l, int i, int j) const {
    return (((size_t)(i >> 4) * (y.UP[l + 1] / 16) + (j >> 4)) * 16 + (i & 15)) * 16 + (j & 15);
  }
  // Lane's share of a weight operand (unit li of a tile row, 8 contraction units from 8q) inside the 1 KB
  // that two neighbouring 16 x 16 tiles of an operand copy take.
  __device__ __forceinline__ static int opnd_lane(int li, int q) { return (q >> 1) * 256 + li * 16 + 8 * (q & 1); }

  // ---- parameters -------------------------------------------------------
  __device__ __forceinline__ void store_param(int l, int k, int j, bool isb, float val, int par) const {
    if (isb) {
      fp(y.bias[l])[j] = val;
    } else {
      fp(y.w[l])[sidx(l, k, j)] = val;
      bp(y.oi[l][par])[oidx(l, j, k)] = (__bf16)val;
      if (l + 1 == y.L) bp(y.io[par])[iidx(l, k, j)] = (__bf16)val;
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
      const int fi = y.U[l], fo = y.U[l + 1];
      for (int i = threadIdx.x; i < fi * fo + fo; i += blockDim.x) {
        const bool isb = i >= fi * fo;
        const int e = isb ? i - fi * fo : i;
        const int k = isb ? 0 : e / fo, j = isb ? e : e % fo;
        const int ci = (isb ? y.cb[l] : y.cw[l]) + e;
        store_param(l, k, j, isb, st[ci], par);
        if (isb) {
          fp(y.bm[l])[j] = st[y.P + ci];
          fp(y.bv[l])[j] = st[2 * y.P + ci];
        } else {
          fp(y.m[l])[sidx(l, k, j)] = st[y.P + ci];
          fp(y.v[l])[sidx(l, k, j)] = st[2 * y.P + ci];
        }
      }
    }
  }

  // Early stopping on held-out rows hands back the parameters of the best epoch: keep them aside ...
  __device__ __forceinline__ void keep_best() const {
    for (int l = 0; l < y.L; l++) {
      const uint4* W = (const uint4*)fp(y.w[l]);
      uint4* B = (uint4*)fp(y.wb[l]);
      const int n16 = y.UP[l + 1] * y.UP[l] / 4;
      for (int i = threadIdx.x; i < n16; i += blockDim.x) B[i] = W[i];
      for (int j = threadIdx.x; j < y.UP[l + 1]; j += blockDim.x) fp(y.bb[l])[j] = fp(y.bias[l])[j];
    }
    __syncthreads();
  }
  // ... and put them back, with the operand copies of parity `par`, before the held fold is scored.
  __device__ __forceinline__ void restore_best(int par) const {
    for (int l = 0; l < y.L; l++) {
      const int fi = y.U[l], fo = y.U[l + 1];
      for (int i = threadIdx.x; i < fi * fo + fo; i += blockDim.x) {
        const bool isb = i >= fi * fo;
        const int e = isb ? i - fi * fo : i;
        const int k = isb ? 0 : e / fo, j = isb ? e : e % fo;
        store_param(l, k, j, isb, isb ? fp(y.bb[l])[j] : fp(y.wb[l])[sidx(l, k, j)], par);
      }
    }
    __syncthreads();
  }

  // ---- staging --------------------------------------------------------------
  // Row list of the chunk and the gathered input rows (with their pad columns) into the buffer.
  __device__ __forceinline__ void stage_rows(const int32_t* list, const RowSplit& sp, int mode, uint64_t key, int lo,
                                             int rows) const {
    int32_t* rl = rowlist();
    int32_t* tg = targets();
    const int32_t* Y = (const int32_t*)P.y;  // class indices or float values: 32 bits either way
    for (int p = threadIdx.x; p < TB_ROWS; p += blockDim.x) {
      const int row = p < rows ? list[row_index(sp, mode, key, (uint32_t)(lo + p))] : -1;
      rl[p] = row;
      tg[p] = row >= 0 ? Y[row] : 0;  // in flight while the rows are gathered
    }
    __syncthreads();
    const int d = y.U[0], up0 = y.UP[0], vpr = up0 / 8;  // 16-byte vectors per row
    char* b0 = buf();
    const __bf16* X = (const __bf16*)P.X;
    // four vectors per thread in flight: the gather is all latency
    const int nvec = TB_ROWS * vpr;
    for (int base = threadIdx.x; base < nvec; base += 4 * TB_THREADS) {
      uint4 val[4];
      int r[4], vv[4];
#pragma unroll
      for (int u = 0; u < 4; u++) {
        const int idx = base + u * TB_THREADS;
        r[u] = idx / vpr;
        vv[u] = idx - r[u] * vpr;
        const int row = idx < nvec ? rl[r[u]] : -1;
        // always a valid address, so the four loads are unconditional; pad rows and columns become zeros
        const uint4 v = *(const uint4*)(X + (size_t)max(row, 0) * d + min(vv[u] * 8, d - 8));
        val[u] = row >= 0 && vv[u] * 8 < d ? v : uint4{0, 0, 0, 0};
      }
#pragma unroll
      for (int u = 0; u < 4; u++)
        if (base + u * TB_THREADS < nvec) *(uint4*)(b0 + ((size_t)r[u] * TB_S + vv[u] * 8) * 2) = val[u];
    }
    __syncthreads();
  }

  // Transpose of the wave's rows of level l to global, tile-blocked [unit tile][row block][unit][32 rows].
  __device__ __forceinline__ void spill_transposed(int l) const {
    const int t_ = tid(), lane = t_ & 63, w = t_ >> 6, li = lane & 15, q = lane >> 4;
    __bf16* T = bp(y.T[l]);
    const int mta = (y.U[l] + 15) / 16;  // unit tiles that hold real units: the others are never read back
    for (int mt = 0; mt < mta; mt++) {
      const bf16x8 v = lds_operand_tr(buf(), TB_S, 32 * w, mt * 16, li, q);
      *(bf16x8*)(T + (((size_t)mt * 8 + w) * 16 + li) * 32 + q * 8) = v;
    }
  }

  // ---- hidden layers, forward and data gradient: wave w owns units 32w..32w+31 of the level it produces ----
  // The wave's weight operands for a hidden-layer product: two unit tiles x up to 8 k blocks of the [out][in]
  // copy A, all fetched at once (one exposed latency per layer, exact waits afterwards).  TR = false: the wave
  // produces out units (forward).  TR = true: it produces in units (data gradient) and needs the transpose of
  // the same tiles: lanes 0..31 fetch the tile of out tile 2kb, lanes 32..63 that of out tile 2kb + 1, and each
  // pair passes through the wave's LDS staging patch and comes back through the transposing read; mt_a = in
  // tiles of A.
  template <bool TR>
  __device__ __forceinline__ void gemm_operands(const __bf16* __restrict__ A, int kbn, int mt_a, i32x4 (&ar)[8][2]) const {
    const int t_ = tid(), lane = t_ & 63, w = t_ >> 6, li = lane & 15, q = lane >> 4;
    const __bf16* A0 = TR ? A + ((size_t)(lane >> 5) * mt_a + 2 * w) * 256 + (lane & 31) * 8
                          : A + (size_t)(2 * w) * kbn * 512 + opnd_lane(li, q);
    const __bf16* A1 = A0 + (TR ? (size_t)256 : (size_t)kbn * 512);
    const size_t kstep = TR ? (size_t)mt_a * 512 : (size_t)512;
#pragma unroll
    for (int kb = 0; kb < 8; kb++)
      if (kb < kbn) {
        ar[kb][0] = *(const i32x4*)(A0 + (size_t)kb * kstep);
        ar[kb][1] = *(const i32x4*)(A1 + (size_t)kb * kstep);
      }
    if (TR) {
      char* patch = lds + TB_LDS_STAGE + w * 2048;
#pragma unroll
      for (int kb = 0; kb < 8; kb++)
        if (kb < kbn) {
#pragma unroll
          for (int ub = 0; ub < 2; ub++) {
            *(i32x4*)(patch + ub * 1024 + lane * 16) = ar[kb][ub];
            ar[kb][ub] = as_i32x4(lds_operand_tr(patch + ub * 1024, 16, 0, 0, li, q));
          }
        }
    }
  }

  // acc[ub][j] = sum_k A[(2w+ub)*16 + .][k] * level[128 half + 16j + .][k] for the 8 row tiles of one half of
  // the chunk.  The lane ends up with units (2w+ub)*16+4q..+3 of row 128 half + 16j + li.  All 8 tiles are
  // multiplied whatever the chunk holds: tiles past the rows in use only cost arithmetic on stale buffer
  // contents, and the callers never store their results.
  __device__ __forceinline__ void gemm_half(const i32x4 (&ar)[8][2], int kbn, int half, f32x4 (&acc)[2][8]) const {
    const int lane = tid() & 63, li = lane & 15, q = lane >> 4;
    const size_t tile_bytes = (size_t)16 * TB_S * 2;
    const char* bp = buf() + ((size_t)li * TB_S + q * 8) * 2 + half * 8 * tile_bytes;
#pragma unroll
    for (int j = 0; j < 8; j++) {
      acc[0][j] = f32x4{0.f, 0.f, 0.f, 0.f};
      acc[1][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int kb = 0; kb < 8; kb++)
      if (kb < kbn) {
        const bf16x8 o0 = as_bf16x8(ar[kb][0]), o1 = as_bf16x8(ar[kb][1]);
        // all 8 level operands of the k block are requested before the first product waits for one
        bf16x8 b[8];
#pragma unroll
        for (int j = 0; j < 8; j++) b[j] = *(const bf16x8*)(bp + j * tile_bytes + kb * 64);
#pragma unroll
        for (int j = 0; j < 8; j++) {
          acc[0][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(o0, b[j], acc[0][j], 0, 0, 0);
          acc[1][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(o1, b[j], acc[1][j], 0, 0, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);  // 8 LDS reads
        __builtin_amdgcn_sched_group_barrier(0x008, 16, 0);  // 16 MFMA
      }
  }

  // Hidden layer l: level l -> level l+1 in place, the chunk's two halves of 128 rows one after the other: a
  // half's results stay in registers until every wave has read that half, and are written while the other
  // half is read.  The ReLU pattern of the wave's units goes to `bits` (bit 4*(16*ub + jb) + r).  Called by
  // all waves.
  // The wave's weight operands and biases of hidden layer l (forward), requested, not waited for.
  __device__ __forceinline__ void fetch_hidden(int l, int par, i32x4 (&ar)[8][2], f32x4 (&bv)[2]) const {
    const int t_ = tid(), lane = t_ & 63, w = t_ >> 6, q = lane >> 4;
    if (32 * w < y.UP[l + 1]) {
      gemm_operands<false>(bp(y.oi[l][par]), y.UP[l] / 32, 0, ar);
      const float* bias = fp(y.bias[l]);
#pragma unroll
      for (int ub = 0; ub < 2; ub++) bv[ub] = *(const f32x4*)(bias + 32 * w + 16 * ub + 4 * q);
    }
  }

  // The operands (ar, bv) come from fetch_hidden.  `next` is called once, after the wave's last products, when
  // ar is dead: it requests the operands of the phase that follows into ar, so that their latency passes
  // behind this layer's last epilogue and barrier.
  template <class Next>
  __device__ __forceinline__ void forward_hidden(int l, int njb, uint32_t (&bits)[4], i32x4 (&ar)[8][2], const f32x4 (&bv_in)[2],
                                                 Next next) const {
    const int t_ = tid(), lane = t_ & 63, w = t_ >> 6, li = lane & 15, q = lane >> 4;
    const bool active = 32 * w < y.UP[l + 1];
    const int kbn = y.UP[l] / 32;
    const size_t tile_bytes = (size_t)16 * TB_S * 2;
    const f32x4 bv[2] = {bv_in[0], bv_in[1]};
#pragma unroll
    for (int i = 0; i < 4; i++) bits[i] = 0;
#pragma unroll
    for (int half = 0; half < 2; half++)
      if (half * 8 < njb) {
        f32x4 acc[2][8];
        if (active) gemm_half(ar, kbn, half, acc);
        if (half == 1 || njb <= 8) next();
        __syncthreads();
        if (active) {
          char* b = buf() + ((size_t)li * TB_S + 32 * w + 4 * q) * 2 + half * 8 * tile_bytes;
#pragma unroll
          for (int ub = 0; ub < 2; ub++)
#pragma unroll
            for (int j = 0; j < 8; j++)
              if (half * 8 + j < njb) {
                bf16x4 pk;
                uint32_t nib = 0;
#pragma unroll
                for (int r = 0; r < 4; r++) {
                  pk[r] = (__bf16)fmaxf(acc[ub][j][r] + bv[ub][r], 0.f);
                  nib |= ((float)pk[r] > 0.f ? 1u : 0u) << r;
                }
                *(bf16x4*)(b + j * tile_bytes + ub * 32) = pk;
                bits[ub * 2 + half] |= nib << (j * 4);
              }
        }
      }
    __syncthreads();
  }

  // Delta of level l (1 <= l < L) from the delta of level l+1 (in dbuf for the output level, else in
  // the buffer), masked by the ReLU pattern of level l, written over the buffer.  Called by all waves.
  __device__ __forceinline__ void backward_data(int l, int par, int njb, const uint32_t (&bits)[4]) const {
    const int t_ = tid(), lane = t_ & 63, w = t_ >> 6, li = lane & 15, q = lane >> 4;
    const bool active = 32 * w < y.UP[l];
    char* b = buf() + ((size_t)li * TB_S + 32 * w + 4 * q) * 2;
    const size_t tile_bytes = (size_t)16 * TB_S * 2;
    auto put = [&](const f32x4& acc, int ub, int jb) {
      const uint32_t nib = bits[ub * 2 + (jb >> 3)] >> ((jb & 7) * 4);
      bf16x4 pk;
#pragma unroll
      for (int r = 0; r < 4; r++) pk[r] = (__bf16)(((nib >> r) & 1u) ? acc[r] : 0.f);
      *(bf16x4*)(b + jb * tile_bytes + ub * 32) = pk;
    };
    // Row tiles past the chunk's rows get zeros: the single-chunk weight gradients contract over all 256 rows
    // whatever the minibatch holds, and a zero delta silences whatever the other operand has there.
    auto put_zero = [&](int ub, int jb) {
      *(bf16x4*)(b + jb * tile_bytes + ub * 32) = bf16x4{(__bf16)0.f, (__bf16)0.f, (__bf16)0.f, (__bf16)0.f};
    };
    if (l + 1 == y.L) {
      // the 16-wide output delta sits in its own buffer: nothing is overwritten while it is read
      if (active) {
        const __bf16* A = bp(y.io[par]);
        const char* db = dbuf() + ((size_t)li * 16 + 4 * q) * 2;
#pragma unroll
        for (int ub = 0; ub < 2; ub++) {
          const bf16x4 a = *(const bf16x4*)(A + ((size_t)(2 * w + ub) * 16 + li) * 16 + 4 * q);
#pragma unroll
          for (int jb = 0; jb < 16; jb++)
            if (jb < njb) {
              const bf16x4 d = *(const bf16x4*)(db + jb * 16 * 16 * 2);
              put(__builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, d, f32x4{0.f, 0.f, 0.f, 0.f}, 0, 0, 0), ub, jb);
            } else {
              put_zero(ub, jb);
            }
        }
      }
    } else {
      const int kbn = y.UP[l + 1] / 32;
      i32x4 ar[8][2];
      if (active) gemm_operands<true>(bp(y.oi[l][par]), kbn, y.UP[l] / 16, ar);
#pragma unroll
      for (int half = 0; half < 2; half++)
        if (half * 8 < njb) {
          f32x4 acc[2][8];
          if (active) gemm_half(ar, kbn, half, acc);
          __syncthreads();
          if (active) {
#pragma unroll
            for (int ub = 0; ub < 2; ub++)
#pragma unroll
              for (int j = 0; j < 8; j++) {
                if (half * 8 + j < njb)
                  put(acc[ub][j], ub, half * 8 + j);
                else
                  put_zero(ub, half * 8 + j);
              }
          }
        } else if (active) {  // nobody reads these rows in this pass
#pragma unroll
          for (int ub = 0; ub < 2; ub++)
#pragma unroll
            for (int j = 0; j < 8; j++) put_zero(ub, half * 8 + j);
        }
    }
    __syncthreads();
  }

  // Output layer + loss over the wave's rows (wave w: rows 32w..32w+31).  TRAIN: output delta -> dbuf.
  // The output layer's weight operand (the same 8 KB for every wave), requested, not waited for.
  __device__ __forceinline__ void fetch_out(int par, i32x4 (&ar)[8][2]) const {
    const int l = y.L - 1, lane = tid() & 63, li = lane & 15, q = lane >> 4;
    const int kbn = y.UP[l] / 32;
    const __bf16* Ap = bp(y.oi[l][par]) + opnd_lane(li, q);
#pragma unroll
    for (int kb = 0; kb < 8; kb++)
      if (kb < kbn) ar[kb][0] = *(const i32x4*)(Ap + kb * 512);
  }

  template <bool TRAIN>
  __device__ __forceinline__ void forward_out(const i32x4 (&ar)[8][2], int rows, float inv_mb, double& lsum, double& hits) const {
    const int l = y.L - 1, c = y.U[y.L];
    const int t_ = tid(), lane = t_ & 63, w = t_ >> 6, li = lane & 15, q = lane >> 4;
    const float* bias = fp(y.bias[l]);
    const int32_t* rl = rowlist();
    const int32_t* tg = targets();
    char* db = dbuf();
    const bool cls = P.n_classes >= 2;
    {
      const int kbn = y.UP[l] / 32;
      f32x4 accs[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
      const char* bq = buf() + ((size_t)(32 * w + li) * TB_S + q * 8) * 2;
      const size_t tile_bytes = (size_t)16 * TB_S * 2;
#pragma unroll
      for (int kb = 0; kb < 8; kb++)
        if (kb < kbn) {
          const bf16x8 a = as_bf16x8(ar[kb][0]);
          accs[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, *(const bf16x8*)(bq + kb * 64), accs[0], 0, 0, 0);
          accs[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, *(const bf16x8*)(bq + tile_bytes + kb * 64), accs[1], 0, 0, 0);
        }
#pragma unroll
      for (int jb = 0; jb < 2; jb++) {
        const f32x4 acc = accs[jb];
        const int r = 32 * w + jb * 16 + li;
        const int row = rl[r];
        const bool valid = r < rows && row >= 0;
        const f32x4 b = *(const f32x4*)(bias + 4 * q);
        float z[4];
#pragma unroll
        for (int e = 0; e < 4; e++) z[e] = acc[e] + b[e];
        float delta[4] = {0.f, 0.f, 0.f, 0.f};
        if (cls) {
          const int yr = valid ? tg[r] : 0;
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
          float zy = 0.f;
#pragma unroll
          for (int e = 0; e < 4; e++) zy = (4 * q + e == yr) ? z[e] : zy;
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
          // one output: a logit with labels 0/1 (log(1 + e^z) - y z, delta (sigmoid(z) - y)/m), or a
          // regression value (half squared error, delta (z - y)/m)
          const bool logit = P.n_classes == 1;
          const int tv = valid ? tg[r] : 0;
          const float zz = valid ? z[0] : 0.f;
          const float e0 = logit ? 1.f / (1.f + expf(-zz)) - (float)tv : zz - __builtin_bit_cast(float, tv);
          if (valid && q == 0) {
            if (logit) {
              lsum += (double)(fmaxf(zz, 0.f) + log1pf(expf(-fabsf(zz))) - (tv ? zz : 0.f));
              hits += (zz > 0.f) == (tv != 0);
            } else {
              lsum += TRAIN ? 0.5 * (double)e0 * (double)e0 : (double)e0 * (double)e0;
              hits += (double)fabsf(e0);  // the absolute error
            }
          }
          if (TRAIN && valid && q == 0) delta[0] = e0 * inv_mb;
        }
        if (TRAIN) {
          bf16x4 pk;
#pragma unroll
          for (int e = 0; e < 4; e++) pk[e] = (__bf16)delta[e];
          *(bf16x4*)(db + ((size_t)r * 16 + 4 * q) * 2) = pk;
        }
      }
    }
  }

  // ---- weight + bias gradient of layer l with the optimizer in the epilogue ------------------------
  // D[in][out] = sum_rows act[row][in] * delta[row][out].  The work is cut into units of one in tile x a
  // run of out tiles, dealt round-robin to the waves.  A wave holds the activation operand of its in tile
  // in registers (read once from the spilled transpose, the next unit's already in flight), takes the delta
  // operand of each out tile from the buffer, and has the optimizer state of the next tile in flight while
  // it multiplies and updates the current one.  One more "in tile" whose operand is a row of ones gives
  // the bias gradient (the deltas of unused rows are zero); the bias and its moments are plain arrays.
  __device__ __forceinline__ void wgrad_t(int l, int KB, bool first, bool last, const OptC& oc, int par_next,
                                          float* rec) const {
    const int t_ = tid(), lane = t_ & 63, w = t_ >> 6, li = lane & 15, q = lane >> 4;
    float* W = fp(y.w[l]);
    float* Mo = fp(y.m[l]);
    float* Vo = fp(y.v[l]);
    float* Gp = fp(y.gp[l]);
    float* bias = fp(y.bias[l]);
    float* bm = fp(y.bm[l]);
    float* bv = fp(y.bv[l]);
    float* bg = fp(y.bg[l]);
    __bf16* oi = bp(y.oi[l][par_next]);
    __bf16* io = bp(y.io[par_next]);
    const __bf16* T = bp(y.T[l]);
    const int fi = y.U[l], fo = y.U[l + 1];
    const int Mt = y.UP[l] / 16, Nt = y.UP[l + 1] / 16, Me = (fi + 15) / 16 + 1, Ne = (fo + 15) / 16;
    char* trp = lds + TB_LDS_TR + w * 512;
    const int cw = y.cw[l], cb = y.cb[l], Pn = y.P;
    const bool lastlayer = l + 1 == y.L;  // its activation operand is still in the buffer, its delta in dbuf
    const char* Bl = lastlayer ? dbuf() : buf();
    const int ldb = lastlayer ? 16 : TB_S;
    const bool adam = oc.adam;
    // number of runs the out tiles are cut into: the one that spreads Me * NS units most evenly
    int NS = 1, best = 1 << 30;
    for (int ns = 1; ns <= 4 && ns <= Ne; ns++) {
      const int c = ((Me * ns + TB_WAVES - 1) / TB_WAVES) * ((Ne + ns - 1) / ns);
      if (c < best) {
        best = c;
        NS = ns;
      }
    }
    const int NU = Me * NS;
    // unit u: in tile mt (mt == Me - 1: the bias) and out tiles nt0..nt1-1; the runs of one in tile go to
    // neighbouring waves, which fetch its operand at the same time
    auto unit_tiles = [&](int u, int& mt, int& nt0, int& nt1) {
      mt = u / NS;
      const int sg = u % NS;
      nt0 = sg * Ne / NS;
      nt1 = (sg + 1) * Ne / NS;
    };
    auto load_a = [&](int mt, i32x4(&a)[8]) {
      if (mt == Me - 1) {
        const int o = li == 0 ? 0x3F803F80 : 0;  // two bf16 ones
#pragma unroll
        for (int kb = 0; kb < 8; kb++) a[kb] = i32x4{o, o, o, o};
      } else {
#pragma unroll
        for (int kb = 0; kb < 8; kb++)
          if (kb < KB)
            a[kb] = lastlayer ? as_i32x4(lds_operand_tr(buf(), TB_S, kb * 32, mt * 16, li, q))
                              : *(const i32x4*)(T + (((size_t)mt * 8 + kb) * 16 + li) * 32 + q * 8);
      }
    };
    auto load_st = [&](int mt, int nt, f32x4& sw, f32x4& sm, f32x4& sv) {
      if (mt == Me - 1) {
        const int j = nt * 16 + li;
        sw[0] = bias[j];
        sm[0] = bm[j];
        if (adam) sv[0] = bv[j];
      } else {
        const size_t o = ((size_t)mt * Nt + nt) * 256 + lane * 4;
        sw = __builtin_nontemporal_load((const f32x4*)(W + o));
        sm = __builtin_nontemporal_load((const f32x4*)(Mo + o));
        if (adam) sv = __builtin_nontemporal_load((const f32x4*)(Vo + o));
      }
    };
    if (w >= NU) return;
    // The wave's tiles in order: position c is being worked on, pn[0..D-1] follow it.  The optimizer
    // state is fetched D tiles ahead into D + 1 rotating register sets.
    constexpr int D = TB_STATE_AHEAD;
    struct TPos {
      int u, mt, nt, nt1;
    };
    struct St {
      f32x4 w, m, v;
    };
    auto unit_first = [&](int u) {
      TPos p;
      int nt0;
      p.u = u;
      unit_tiles(u, p.mt, nt0, p.nt1);
      p.nt = nt0;
      return p;
    };
    auto next_pos = [&](const TPos& p, bool& ok) {
      TPos r = p;
      if (ok) {
        if (p.nt + 1 < p.nt1)
          r.nt++;
        else if (p.u + TB_WAVES < NU)
          r = unit_first(p.u + TB_WAVES);
        else
          ok = false;
      }
      return r;
    };
    TPos c = unit_first(w);
    TPos pn[D];
    bool okn[D];
    const f32x4 zero4 = f32x4{0.f, 0.f, 0.f, 0.f};
    St S[D + 1];
#pragma unroll
    for (int k = 0; k <= D; k++) S[k] = St{zero4, zero4, zero4};
    if (last) load_st(c.mt, c.nt, S[0].w, S[0].m, S[0].v);
#pragma unroll
    for (int k = 0; k < D; k++) {
      okn[k] = k ? okn[k - 1] : true;
      pn[k] = next_pos(k ? pn[k - 1] : c, okn[k]);
      if (last && k + 1 < D && okn[k]) load_st(pn[k].mt, pn[k].nt, S[k + 1].w, S[k + 1].m, S[k + 1].v);
    }
    i32x4 a[8], an[8];
    load_a(c.mt, a);
    if (c.u + TB_WAVES < NU) load_a(unit_first(c.u + TB_WAVES).mt, an);
    bool alive = true;
    auto tile = [&](St& cur, St& pre) __attribute__((always_inline)) {
      if (last && okn[D - 1]) load_st(pn[D - 1].mt, pn[D - 1].nt, pre.w, pre.m, pre.v);
      const int mt = c.mt, nt = c.nt;
      const bool isb = mt == Me - 1;
      const int j = nt * 16 + li;  // the lane's out unit
      const size_t o = ((size_t)mt * Nt + nt) * 256 + lane * 4;
      f32x4 g = zero4;
      if (!first) {
        if (isb)
          g[0] = bg[j];
        else
          g = *(const f32x4*)(Gp + o);
      }
#pragma unroll
      for (int kb = 0; kb < 8; kb++)
        if (kb < KB) g = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(a[kb]), lds_operand_tr(Bl, ldb, kb * 32, nt * 16, li, q), g, 0, 0, 0);
      if (!last) {
        if (isb) {
          if (q == 0) bg[j] = g[0];
        } else {
          *(f32x4*)(Gp + o) = g;
        }
      } else if (isb) {  // r = 0 of lane group 0 holds the bias gradient of out unit j
        if (q == 0 && j < fo) {
          float wr = cur.w[0], mr = cur.m[0], vr = cur.v[0];
          opt_update(oc, g[0], wr, mr, vr);
          if (rec) {
            rec[1 + cb + j] = g[0];
            rec[1 + Pn + cb + j] = wr;
          }
          bias[j] = wr;
          bm[j] = mr;
          if (adam) bv[j] = vr;
        }
      } else {
        // the lane holds in units i0..i0+3 of out unit j
        const int i0 = mt * 16 + 4 * q;
        f32x4 wv = cur.w, mv = cur.m, vv = cur.v;
        bf16x4 pk;
        if (!rec && mt * 16 + 16 <= fi && nt * 16 + 16 <= fo) {  // no pad unit in the tile
#pragma unroll
          for (int r = 0; r < 4; r++) {
            float wr = wv[r], mr = mv[r], vr = vv[r];
            opt_update(oc, g[r] + oc.am * wr, wr, mr, vr);
            wv[r] = wr;
            mv[r] = mr;
            vv[r] = vr;
            pk[r] = (__bf16)wr;
          }
        } else {
#pragma unroll
          for (int r = 0; r < 4; r++) {
            const int ii = i0 + r;
            float wr = wv[r], mr = mv[r], vr = vv[r];
            if (j < fo && ii < fi) {
              const float gg = g[r] + oc.am * wr;
              opt_update(oc, gg, wr, mr, vr);
              if (rec) {
                const int ci = cw + ii * fo + j;
                rec[1 + ci] = gg;
                rec[1 + Pn + ci] = wr;
              }
            }
            wv[r] = wr;
            mv[r] = mr;
            vv[r] = vr;
            pk[r] = (__bf16)wr;
          }
        }
        __builtin_nontemporal_store(wv, (f32x4*)(W + o));
        __builtin_nontemporal_store(mv, (f32x4*)(Mo + o));
        if (adam) __builtin_nontemporal_store(vv, (f32x4*)(Vo + o));
        // both bf16 operand copies are made of 16 x 16 tiles, so the wave writes 512 contiguous bytes each
        *(bf16x4*)(oi + ((size_t)nt * Mt + mt) * 256 + li * 16 + 4 * q) = pk;
        if (lastlayer) {
          // [out][in] -> [in][out] through the wave's LDS patch and the transposing read
          *(bf16x4*)(trp + (li * 16 + 4 * q) * 2) = pk;
          const s16x4 tv = lds_read_tr(trp + ((4 * q + (li >> 2)) * 16 + 4 * (li & 3)) * 2);
          *(s16x4*)(io + ((size_t)mt * Nt + nt) * 256 + li * 16 + 4 * q) = tv;
        }
      }
      // on to the next tile; a new unit brings its activation operand, fetched during the previous unit
      if (!okn[0]) {
        alive = false;
        return;
      }
      const int old_u = c.u;
      c = pn[0];
#pragma unroll
      for (int k = 0; k + 1 < D; k++) {
        pn[k] = pn[k + 1];
        okn[k] = okn[k + 1];
      }
      pn[D - 1] = next_pos(pn[D - 1], okn[D - 1]);
      if (c.u != old_u) {
#pragma unroll
        for (int kb = 0; kb < 8; kb++) a[kb] = an[kb];
        if (c.u + TB_WAVES < NU) load_a(unit_first(c.u + TB_WAVES).mt, an);
      }
    };
    while (alive) {
#pragma unroll
      for (int k = 0; k <= D; k++)
        if (alive) tile(S[k], S[(k + D) % (D + 1)]);
    }
  }

  // The same for the common case: a layer below the last one, the whole minibatch in one chunk.  All 8 row
  // blocks are contracted: rows past a ragged chunk carry zero deltas (backward_data) and finite activations.
  // Straight-line code per tile, so that the waits on memory are exact and the optimizer state really is in
  // flight TB_STATE_AHEAD tiles ahead: the in x out tiles of the layer are numbered in-tile-major and each
  // wave takes one contiguous eighth of them (its state is one contiguous stream per array, its activation
  // operand changes at most every Ne tiles and the next one is fetched a whole in tile early); the bias
  // tiles (ones operand) are dealt round-robin and their state is fetched before anything else.  Pad
  // elements of edge tiles keep their zeros through selects, not branches.
  // LD: cache policy of the state LOADS (see state_load_hint()); the stores are always non-temporal.
  template <bool ADAM, bool FROM_X, int LD>
  __device__ __forceinline__ void wgrad_stream(int l, const OptC& oc, int par_next, float* rec) const {
    const int t_ = tid(), lane = t_ & 63, li = lane & 15, q = lane >> 4;
    const int w = uniform(t_ >> 6);
    float* W = uniform(fp(y.w[l]));
    float* Mo = uniform(fp(y.m[l]));
    float* Vo = uniform(fp(y.v[l]));
    float* bias = uniform(fp(y.bias[l]));
    float* bm = uniform(fp(y.bm[l]));
    float* bv = uniform(fp(y.bv[l]));
    __bf16* oi = uniform(bp(y.oi[l][par_next]));
    const __bf16* T = uniform(bp(y.T[l]));
    const int fi = uniform(y.U[l]), fo = uniform(y.U[l + 1]);
    constexpr int S = TB_S;
    const int Mt = uniform(y.UP[l]) / 16, Nt = uniform(y.UP[l + 1]) / 16, Mr = (fi + 15) / 16, Ne = (fo + 15) / 16;
    const int cw = y.cw[l], cb = y.cb[l], Pn = y.P;
    const int TT = Mr * Ne, t0 = w * TT / TB_WAVES, t1 = (w + 1) * TT / TB_WAVES;
    constexpr int D = TB_STATE_AHEAD;
    struct St {
      f32x4 w, m, v;
    };
    const f32x4 zero4 = f32x4{0.f, 0.f, 0.f, 0.f};
    // the lane's delta operand of out tile 0, row block 0: rows 8q + li/4 (+4), units 4 (li%4)..
    const char* bl = buf() + ((size_t)(8 * q + (li >> 2)) * S + 4 * (li & 3)) * 2;
    const size_t kbs = (size_t)32 * S * 2, hs = (size_t)4 * S * 2;
    auto delta_operands = [&](int nt, bf16x8(&b)[8]) {
#pragma unroll
      for (int kb = 0; kb < 8; kb++) {
        union {
          struct {
            s16x4 lo, hi;
          } s;
          bf16x8 v;
        } u;
        u.s.lo = lds_read_tr(bl + nt * 32 + kb * kbs);
        u.s.hi = lds_read_tr(bl + nt * 32 + kb * kbs + hs);
        b[kb] = u.v;
      }
    };
    // bias state of the wave's bias tiles (out tiles w and w + 8)
    float bw_[2], bm_[2], bv_[2];
#pragma unroll
    for (int i = 0; i < 2; i++) {
      const int j = min(w + 8 * i, Ne - 1) * 16 + li;
      bw_[i] = bias[j];
      bm_[i] = bm[j];
      bv_[i] = ADAM ? bv[j] : 0.f;
    }
    if (t1 > t0) {
      // Every global address is a wave-uniform base plus a 32-bit lane offset that never changes.  The
      // fetches go through buffer descriptors: the look-ahead runs past the wave's last tile (and last in
      // tile), and there the lane offset is pushed out of the descriptor's range, which makes the fetch
      // return zeros without touching memory; the instruction stream stays the same for every tile.
      const uint32_t lane16 = (uint32_t)lane * 16, lane_t = (uint32_t)(li * 64 + q * 16), lane_oi = (uint32_t)(li * 32 + q * 8);
      constexpr uint32_t OUT_OF_RANGE = 0x40000000u;
      constexpr int NT_HINT = 2;  // cache policy bit 1: non-temporal
      const uint32_t state_bytes = (uint32_t)Mt * Nt * 1024;
      const __amdgpu_buffer_rsrc_t rW = __builtin_amdgcn_make_buffer_rsrc(W, 0, state_bytes, 0x00020000);
      const __amdgpu_buffer_rsrc_t rM = __builtin_amdgcn_make_buffer_rsrc(Mo, 0, state_bytes, 0x00020000);
      const __amdgpu_buffer_rsrc_t rV = __builtin_amdgcn_make_buffer_rsrc(Vo, 0, state_bytes, 0x00020000);
      const __amdgpu_buffer_rsrc_t rO = __builtin_amdgcn_make_buffer_rsrc(oi, 0, (uint32_t)Mt * Nt * 512, 0x00020000);
      const __amdgpu_buffer_rsrc_t rT = __builtin_amdgcn_make_buffer_rsrc(const_cast<__bf16*>(T), 0, (uint32_t)Mt * 8192, 0x00020000);
      const int mt_last = (t1 - 1) / Ne;
      // Activation operand of in tile mt.  Hidden levels: the spilled transpose, 16 bytes per lane and row
      // block.  Input level (FROM_X): no spill exists; the lane fetches 8 units of one row of the minibatch from
      // the input matrix itself (row block kb, row lane / 2, half lane % 2: 32 rows x 16 units per fetch), and
      // operand() passes each fetched block through the wave's LDS patch and the transposing read.  Rows past
      // the minibatch, units past the input width and in tiles past the wave's range are out of range: zeros.
      const __amdgpu_buffer_rsrc_t rX = __builtin_amdgcn_make_buffer_rsrc(
          const_cast<void*>(P.X), 0, FROM_X ? (uint32_t)((uint64_t)P.n * (uint64_t)fi * 2) : 0u, 0x00020000);
      const int32_t* rl = rowlist();
      char* patch = lds + TB_LDS_STAGE + w * 2048;
      auto load_a = [&](int mt, i32x4(&a)[8]) {
        if (FROM_X) {
          const int u0 = mt * 16 + (lane & 1) * 8;
#pragma unroll
          for (int kb = 0; kb < 8; kb++) {
            const int row = rl[kb * 32 + (lane >> 1)];
            const bool ok = row >= 0 && u0 < fi && mt <= mt_last;
            const uint32_t vo = ok ? (uint32_t)(row * fi + u0) * 2 : OUT_OF_RANGE;
            a[kb] = __builtin_bit_cast(i32x4, __builtin_amdgcn_raw_buffer_load_b128(rX, vo, 0, 0));
          }
        } else {
          const uint32_t vo = lane_t + (mt > mt_last ? OUT_OF_RANGE : 0u);
#pragma unroll
          for (int kb = 0; kb < 8; kb++)
            a[kb] = __builtin_bit_cast(i32x4, __builtin_amdgcn_raw_buffer_load_b128(rT, vo, mt * 8192 + kb * 1024, 0));
        }
      };
      // fetched form -> MFMA operand form
      auto operand = [&](const i32x4(&raw)[8], i32x4(&a)[8]) {
        if (FROM_X) {
#pragma unroll
          for (int kb = 0; kb < 8; kb++) {
            char* pk = patch + (kb & 1) * 1024;
            *(i32x4*)(pk + lane * 16) = raw[kb];
            a[kb] = as_i32x4(lds_operand_tr(pk, 16, 0, 0, li, q));
          }
        } else {
          // register moves written out: the prefetched operand's registers are free before the next fetch
          // is issued, so the fetch lands in them directly instead of in temporaries that must be waited for
#pragma unroll
          for (int kb = 0; kb < 8; kb++)
#pragma unroll
            for (int e = 0; e < 4; e++) asm volatile("v_mov_b32 %0, %1" : "=v"(a[kb][e]) : "v"(raw[kb][e]));
        }
      };
      int mt = t0 / Ne, nt = t0 - mt * Ne;  // the tile being worked on
      int pm = mt, pn = nt, pt = t0;        // the tile whose state is fetched next
      auto load_st = [&](St& s) {
        // also out of range: the lanes whose elements are all pad (their in units or their out unit)
        const uint32_t vo = lane16 + (pt >= t1 || pm * 16 + 4 * q >= fi || pn * 16 + li >= fo ? OUT_OF_RANGE : 0u);
        const int so = (pm * Nt + pn) * 1024;
        s.w = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rW, vo, so, LD));
        s.m = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rM, vo, so, LD));
        if (ADAM) s.v = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rV, vo, so, LD));
        pt++;
        pn++;
        const int wrap = pn == Ne ? 1 : 0;
        pn = wrap ? 0 : pn;
        pm += wrap;
      };
      St st[D + 1];
#pragma unroll
      for (int k = 0; k <= D; k++) st[k] = St{zero4, zero4, zero4};
      i32x4 a[8], an[8];
      load_a(mt, an);
#pragma unroll
      for (int k = 0; k < D; k++) load_st(st[k]);
      operand(an, a);
      load_a(mt + 1, an);
      auto tile = [&](St& cur, St& pre) __attribute__((always_inline)) {
        load_st(pre);
        bf16x8 b[8];
        delta_operands(nt, b);
        f32x4 g = zero4;
#pragma unroll
        for (int kb = 0; kb < 8; kb++) g = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(a[kb]), b[kb], g, 0, 0, 0);
        // the lane holds in units i0..i0+3 of out unit j
        const int j = nt * 16 + li, i0 = mt * 16 + 4 * q;
        const int tb = (mt * Nt + nt) * 1024;
        f32x4 wv = cur.w, mv = cur.m, vv = cur.v, gv;
        bf16x4 pk;
        auto update = [&](auto masked) __attribute__((always_inline)) {
#pragma unroll
          for (int r = 0; r < 4; r++) {
            float wr = wv[r], mr = mv[r], vr = vv[r];
            gv[r] = g[r] + oc.am * wr;
            opt_update(oc, gv[r], wr, mr, vr);
            if (decltype(masked)::value) {
              const bool real = j < fo && i0 + r < fi;
              wr = real ? wr : wv[r];
              mr = real ? mr : mv[r];
              vr = real ? vr : vv[r];
            }
            wv[r] = wr;
            mv[r] = mr;
            vv[r] = vr;
            pk[r] = (__bf16)wr;
          }
        };
        if ((mt + 1) * 16 > fi || (nt + 1) * 16 > fo)  // a tile with pad units
          update(std::true_type{});
        else
          update(std::false_type{});
        const uint32_t vs = lane16 + (i0 >= fi || j >= fo ? OUT_OF_RANGE : 0u);  // all-pad lanes: nothing to write back
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, wv), rW, vs, tb, NT_HINT);
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, mv), rM, vs, tb, NT_HINT);
        if (ADAM) __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, vv), rV, vs, tb, NT_HINT);
        __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, pk), rO, lane_oi, (nt * Mt + mt) * 512, 0);
        if (rec) {
#pragma unroll
          for (int r = 0; r < 4; r++)
            if (j < fo && i0 + r < fi) {
              const int ci = cw + (i0 + r) * fo + j;
              rec[1 + ci] = gv[r];
              rec[1 + Pn + ci] = wv[r];
            }
        }
        nt++;
        if (nt == Ne) {  // on to the next in tile: its operand has been in flight since the last change
          nt = 0;
          mt++;
          operand(an, a);
          load_a(mt + 1, an);
        }
      };
      // Whole groups of D + 1 tiles in a loop with one exit, the remaining tiles (at most D) after it: the
      // only way from one tile body to the next is the one the tiles take, so a wait placed in one body
      // can count on the memory operations of all the others.
      const int groups = (t1 - t0) / (D + 1), rest = (t1 - t0) - (D + 1) * groups;
      for (int i = 0; i < groups; i++) {
#pragma unroll
        for (int k = 0; k <= D; k++) tile(st[k], st[(k + D) % (D + 1)]);
      }
#pragma unroll
      for (int k = 0; k < D; k++)
        if (rest > k) tile(st[k], st[(k + D) % (D + 1)]);
    }
    // bias gradient: the column sums of the delta, through a row of ones
    const int ones = li == 0 ? 0x3F803F80 : 0;  // two bf16 ones
    const bf16x8 a1 = as_bf16x8(i32x4{ones, ones, ones, ones});
#pragma unroll
    for (int i = 0; i < 2; i++) {
      const int nt = w + 8 * i;
      if (nt < Ne) {
        bf16x8 b[8];
        delta_operands(nt, b);
        f32x4 g = zero4;
#pragma unroll
        for (int kb = 0; kb < 8; kb++) g = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b[kb], g, 0, 0, 0);
        const int j = nt * 16 + li;
        if (q == 0 && j < fo) {  // r = 0 of lane group 0 holds the bias gradient of out unit j
          float wr = bw_[i], mr = bm_[i], vr = bv_[i];
          opt_update(oc, g[0], wr, mr, vr);
          if (rec) {
            rec[1 + cb + j] = g[0];
            rec[1 + Pn + cb + j] = wr;
          }
          bias[j] = wr;
          bm[j] = mr;
          if (ADAM) bv[j] = vr;
        }
      }
    }
  }

  // The same for the last layer (one out tile, so at most 16 in tiles + the bias tile; whole minibatch in one
  // chunk, rows past it carry zero deltas): wave w takes in tiles w and w + 8, their state is requested before anything else, and the
  // two tile bodies are straight-line code.  The activation operand comes from the buffer, the delta from its
  // own buffer, both through the transposing read.  The bias tile goes to the wave with the fewest tiles.
  template <bool ADAM, int LD>
  __device__ __forceinline__ void wgrad_last(const OptC& oc, int par_next, float* rec) const {
    const int l = y.L - 1;
    const int t_ = tid(), lane = t_ & 63, li = lane & 15, q = lane >> 4;
    const int w = uniform(t_ >> 6);
    float* W = uniform(fp(y.w[l]));
    float* Mo = uniform(fp(y.m[l]));
    float* Vo = uniform(fp(y.v[l]));
    float* bias = uniform(fp(y.bias[l]));
    float* bm = uniform(fp(y.bm[l]));
    float* bv = uniform(fp(y.bv[l]));
    __bf16* oi = uniform(bp(y.oi[l][par_next]));
    __bf16* io = uniform(bp(y.io[par_next]));
    const int fi = uniform(y.U[l]), fo = uniform(y.U[l + 1]);
    const int Mt = uniform(y.UP[l]) / 16, Mr = (fi + 15) / 16;
    const int cw = y.cw[l], cb = y.cb[l], Pn = y.P;
    char* trp = lds + TB_LDS_TR + w * 512;
    const uint32_t lane16 = (uint32_t)lane * 16, lane_oi = (uint32_t)(li * 32 + q * 8);
    constexpr uint32_t OUT_OF_RANGE = 0x40000000u;
    constexpr int NT_HINT = 2;
    const uint32_t state_bytes = (uint32_t)Mt * 1024;
    const __amdgpu_buffer_rsrc_t rW = __builtin_amdgcn_make_buffer_rsrc(W, 0, state_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rM = __builtin_amdgcn_make_buffer_rsrc(Mo, 0, state_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rV = __builtin_amdgcn_make_buffer_rsrc(Vo, 0, state_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rO = __builtin_amdgcn_make_buffer_rsrc(oi, 0, (uint32_t)Mt * 512, 0x00020000);
    const __amdgpu_buffer_rsrc_t rI = __builtin_amdgcn_make_buffer_rsrc(io, 0, (uint32_t)Mt * 512, 0x00020000);
    const __amdgpu_buffer_rsrc_t rB = __builtin_amdgcn_make_buffer_rsrc(bias, 0, 64, 0x00020000);
    const __amdgpu_buffer_rsrc_t rBm = __builtin_amdgcn_make_buffer_rsrc(bm, 0, 64, 0x00020000);
    const __amdgpu_buffer_rsrc_t rBv = __builtin_amdgcn_make_buffer_rsrc(bv, 0, 64, 0x00020000);
    struct St {
      f32x4 w, m, v;
    };
    const f32x4 zero4 = f32x4{0.f, 0.f, 0.f, 0.f};
    St st[2];
#pragma unroll
    for (int k = 0; k < 2; k++) {
      const int mt = w + 8 * k;
      // out of range: tiles past the layer, and the lanes whose elements are all pad (out unit or in units)
      const uint32_t vo = lane16 + (mt < Mr && li < fo && mt * 16 + 4 * q < fi ? 0u : OUT_OF_RANGE);
      st[k].w = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rW, vo, mt * 1024, LD));
      st[k].m = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rM, vo, mt * 1024, LD));
      st[k].v = ADAM ? __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rV, vo, mt * 1024, LD)) : zero4;
    }
    // bias state: out unit li (lanes of group 0 use it)
    float bw_ = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rB, (uint32_t)li * 4, 0, 0));
    float bm_ = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rBm, (uint32_t)li * 4, 0, 0));
    float bv_ = ADAM ? __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rBv, (uint32_t)li * 4, 0, 0)) : 0.f;
    // the delta operand is the same for every tile
    bf16x8 b[8];
#pragma unroll
    for (int kb = 0; kb < 8; kb++) b[kb] = lds_operand_tr(dbuf(), 16, kb * 32, 0, li, q);
#pragma unroll
    for (int k = 0; k < 2; k++) {
      const int mt = w + 8 * k;
      if (mt < Mr) {
        f32x4 g = zero4;
#pragma unroll
        for (int kb = 0; kb < 8; kb++)
          g = __builtin_amdgcn_mfma_f32_16x16x32_bf16(lds_operand_tr(buf(), TB_S, kb * 32, mt * 16, li, q), b[kb], g, 0, 0, 0);
        // the lane holds in units i0..i0+3 of out unit li
        const int i0 = mt * 16 + 4 * q;
        f32x4 wv = st[k].w, mv = st[k].m, vv = st[k].v, gv;
        bf16x4 pk;
#pragma unroll
        for (int r = 0; r < 4; r++) {
          float wr = wv[r], mr = mv[r], vr = vv[r];
          gv[r] = g[r] + oc.am * wr;
          opt_update(oc, gv[r], wr, mr, vr);
          const bool real = li < fo && i0 + r < fi;
          wv[r] = real ? wr : wv[r];
          mv[r] = real ? mr : mv[r];
          vv[r] = real ? vr : vv[r];
          pk[r] = (__bf16)wv[r];
        }
        const uint32_t vs = lane16 + (li < fo && i0 < fi ? 0u : OUT_OF_RANGE);  // all-pad lanes: nothing to write back
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, wv), rW, vs, mt * 1024, NT_HINT);
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, mv), rM, vs, mt * 1024, NT_HINT);
        if (ADAM) __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, vv), rV, vs, mt * 1024, NT_HINT);
        __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, pk), rO, lane_oi, mt * 512, 0);
        // [out][in] -> [in][out] through the wave's LDS patch and the transposing read
        *(bf16x4*)(trp + (li * 16 + 4 * q) * 2) = pk;
        const s16x4 tv = lds_read_tr(trp + ((4 * q + (li >> 2)) * 16 + 4 * (li & 3)) * 2);
        __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, tv), rI, lane_oi, mt * 512, 0);
        if (rec) {
#pragma unroll
          for (int r = 0; r < 4; r++)
            if (li < fo && i0 + r < fi) {
              const int ci = cw + (i0 + r) * fo + li;
              rec[1 + ci] = gv[r];
              rec[1 + Pn + ci] = wv[r];
            }
        }
      }
    }
    if (w == (Mr & 7)) {  // bias gradient: the column sums of the delta, through a row of ones
      const int ones = li == 0 ? 0x3F803F80 : 0;  // two bf16 ones
      const bf16x8 a1 = as_bf16x8(i32x4{ones, ones, ones, ones});
      f32x4 g = zero4;
#pragma unroll
      for (int kb = 0; kb < 8; kb++) g = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b[kb], g, 0, 0, 0);
      if (q == 0 && li < fo) {  // r = 0 of lane group 0 holds the bias gradient of out unit li
        float wr = bw_, mr = bm_, vr = bv_;
        opt_update(oc, g[0], wr, mr, vr);
        if (rec) {
          rec[1 + cb + li] = g[0];
          rec[1 + Pn + cb + li] = wr;
        }
        bias[li] = wr;
        bm[li] = mr;
        if (ADAM) bv[li] = vr;
      }
    }
  }

  // Cache policy of the optimizer-state loads.  The state of all models in flight (about 200 MB) is far more
  // than the caches hold, so it streams with the non-temporal hint, which keeps it from evicting the operand
  // copies, spills and input rows that are re-read within a step.  But a share of the workgroups does better
  // with ordinary loads (measured on the scale-up workload: every fourth workgroup of an XCD, 64 of 256, is the
  // optimum, 5 % off the pass; all of them is 13 % slower than none).  The stores are non-temporal for everyone.
  __device__ __forceinline__ static bool state_loads_cached() { return ((blockIdx.x >> 3) & 3) == 0; }

  __device__ __forceinline__ void wgrad(int l, int KB, bool first, bool last, const OptC& oc, int par_next,
                                        float* rec) const {
    const bool cached = state_loads_cached();
    if (first && last && l + 1 < y.L) {
      if (l == 0) {
        if (oc.adam) {
          if (cached)
            wgrad_stream<true, true, 0>(l, oc, par_next, rec);
          else
            wgrad_stream<true, true, 2>(l, oc, par_next, rec);
        } else {
          wgrad_stream<false, true, 2>(l, oc, par_next, rec);
        }
      } else {
        if (oc.adam) {
          if (cached)
            wgrad_stream<true, false, 0>(l, oc, par_next, rec);
          else
            wgrad_stream<true, false, 2>(l, oc, par_next, rec);
        } else {
          wgrad_stream<false, false, 2>(l, oc, par_next, rec);
        }
      }
    } else if (first && last) {
      if (oc.adam) {
        if (cached)
          wgrad_last<true, 0>(oc, par_next, rec);
        else
          wgrad_last<true, 2>(oc, par_next, rec);
      } else {
        wgrad_last<false, 2>(oc, par_next, rec);
      }
    } else {
      wgrad_t(l, KB, first, last, oc, par_next, rec);
    }
    __syncthreads();
  }

  __device__ __forceinline__ double penalty_sum() const {
    double s = 0.0;
    for (int l = 0; l < y.L; l++) {
      const float* W = fp(y.w[l]);
      const int fi = y.U[l], fo = y.U[l + 1];
      for (int i = threadIdx.x; i < fi * fo; i += blockDim.x) {
        const float w = W[sidx(l, i % fi, i / fi)];
        s += (double)w * (double)w;
      }
    }
    return block_sum(s, red);
  }

  // Forward pass of the chunk through all layers.  TRAIN: spills the transposes the weight gradients
  // will need, keeps the ReLU patterns, writes the output delta.  Called by all waves.
  template <bool TRAIN>
  __device__ __forceinline__ void forward_all(int par, int rows, float inv_mb, uint32_t (&bits)[2][4], double& lsum,
                                              double& hits, bool spill_inputs = true) const {
    const int w = threadIdx.x >> 6;
    const int KB = (rows + 31) / 32;  // row blocks in use; whole blocks are computed
    // One operand set for the whole pass: each layer requests the next one's (or the output layer's) weights
    // into it after its own last products.
    i32x4 ar[8][2];
    f32x4 bv[2], bvn[2];
    fetch_hidden(0, par, ar, bv);
    for (int l = 0; l + 1 < y.L; l++) {
      if (TRAIN && w < KB && (l > 0 || spill_inputs)) spill_transposed(l);
      uint32_t bl[4];
      forward_hidden(l, 2 * KB, bl, ar, bv, [&]() {
        if (l + 2 < y.L)
          fetch_hidden(l + 1, par, ar, bvn);
        else
          fetch_out(par, ar);
      });
      bv[0] = bvn[0];
      bv[1] = bvn[1];
#pragma unroll
      for (int i = 0; i < 4; i++) {
        if (l & 1)
          bits[1][i] = bl[i];
        else
          bits[0][i] = bl[i];
      }
    }
    if (w < KB)
      forward_out<TRAIN>(ar, rows, inv_mb, lsum, hits);
    else if (TRAIN)  // no output delta for the rows of this wave: zeros (see backward_data)
      *(uint4*)(dbuf() + (32 * w) * 32 + (threadIdx.x & 63) * 16) = uint4{0, 0, 0, 0};
  }

  __device__ __forceinline__ void run() const {
    const int f = it.fold, fl = it.fold - P.fold_base, L = y.L;  // fl: which row list
    const int n_tr = P.counts[2 * fl], n_va = P.counts[2 * fl + 1];
    const int32_t* tr = P.train_idx + (int64_t)fl * P.n;
    const int32_t* va = P.val_idx + (int64_t)fl * P.n;
    const uint64_t km = key_model(it.seed, f);
    const RowSplit sp = row_split(km, it.patience, it.val_frac, n_tr);
    const int n_fit = sp.n_fit;
    const int bs = eff_batch(it.batch_size, n_fit);
    const int steps = n_fit > 0 ? (n_fit + bs - 1) / bs : 0;
    const bool traced = P.trace_item == it.b * P.n_folds + fl;

    {
      uint4* z = (uint4*)slot;
      const uint64_t n16 = y.total / 16;
      for (uint64_t i = threadIdx.x; i < n16; i += blockDim.x) z[i] = uint4{0, 0, 0, 0};
      // The activation buffer too: rows past a ragged chunk are never written, but the weight gradients read
      // them (against zero deltas), so they must hold finite numbers whatever ran on this CU before.
      uint4* zb = (uint4*)buf();
      for (uint32_t i = threadIdx.x; i < TB_ROWS * TB_S * 2 / 16; i += blockDim.x) zb[i] = uint4{0, 0, 0, 0};
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

    uint32_t bits[2][4];
    Plateau plateau;
    const bool watch = it.patience > 0 && steps > 0 && !(traced && P.state_in);
    // One loop over the epochs and, after the last one, the scoring of the held fold: the scoring pass (rows
    // set aside for early stopping after an epoch, the fold's held rows at the end) exists once in the code.
    bool stop = false, have_best = false;
    for (int e = e0;; e++) {
      const bool final = stop || e >= it.epochs;
      double esum = 0.0;  // the lane's share of the epoch's summed data loss
      if (!final) {
      const uint64_t ke = key_epoch(km, e);
      if (!oc.adam) oc.lr = epoch_lr(it.lr, it.power_t, e, n_fit);
      for (int st = e == e0 ? st0 : 0; st < steps; st++, gstep++) {
        const int lo = st * bs, mb = min(bs, n_fit - lo);
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
          const int KB = (rows + 31) / 32;
          const bool first = ch == 0, last = ch == nch - 1;
          stage_rows(tr, sp, ROWS_EPOCH, ke, lo + ch * TB_ROWS, rows);
          // a minibatch of one chunk takes the streaming weight gradient, which reads the inputs themselves
          forward_all<true>(par, rows, inv_mb, bits, lsum, hits, !(first && last));
          __syncthreads();
          for (int l = L - 1; l >= 0; l--) {
            wgrad(l, KB, first, last, oc, par ^ 1, last ? rec : nullptr);
            if (l >= 1) {
              uint32_t bl[4];
#pragma unroll
              for (int i = 0; i < 4; i++) bl[i] = ((l - 1) & 1) ? bits[1][i] : bits[0][i];
              backward_data(l, par, 2 * KB, bl);
            }
          }
        }
        esum += lsum;
        if (rec) {
          const double data = block_sum(lsum, red) / (double)mb;
          if (threadIdx.x == 0) rec[0] = (float)(data + 0.5 * (double)it.alpha * pen / (double)mb);
        }
      }
      }
      float watched = 0.f;
      if (watch && !final && !sp.n_hold) watched = (float)(block_sum(esum, red) / (double)n_fit);
      if (final && have_best) restore_best((int)(gstep & 1));
      if (final || (watch && sp.n_hold)) {
        // loss (and second score) of a list of rows under the current weights
        const int32_t* list = final ? va : tr;
        const int mode = final ? ROWS_PLAIN : ROWS_HELD, count = final ? n_va : sp.n_hold;
        double lsum = 0.0, hits = 0.0;
        for (int off = 0; off < count; off += TB_ROWS) {
          const int rows = min(TB_ROWS, count - off);
          stage_rows(list, sp, mode, 0, off, rows);
          forward_all<false>((int)(gstep & 1), rows, 0.f, bits, lsum, hits);
          __syncthreads();
        }
        lsum = block_sum(lsum, red);
        hits = block_sum(hits, red);
        if (final) {
          if (threadIdx.x == 0) {
            float* out = P.item_out + 2 * ((int64_t)it.b * P.n_folds + fl);
            out[0] = n_va > 0 ? (float)(lsum / (double)n_va) : __builtin_nanf("");
            out[1] = n_va > 0 ? (float)(hits / (double)n_va) : __builtin_nanf("");  // accuracy | mean absolute error
          }
          break;
        }
        watched = (float)(lsum / (double)count);  // the loss of the rows set aside, under the weights the epoch ends with
      }
      if (watch) {
        stop = plateau.stop_after(watched, it.tol, it.patience);
        if (sp.n_hold && plateau.improved) {
          keep_best();
          have_best = true;
        }
      }
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
    const __attribute__((address_space(4))) TItem* ti = (const __attribute__((address_space(4))) TItem*)P.items + item;
    Tiled T{P, ti->d, ti->y, slot, smem, red};
    T.run();
  }
}

}  // namespace
