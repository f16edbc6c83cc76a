// Block-sparse attention backward for gfx950, mask held constant (the paper restricts attention
// with the block mask "during both training and inference", Sec. 3.3 Step 2.1).
//
//   Delta = rowsum(dO * O)                        delta_kernel
//   dQ    = scale * dS K     per query block      dq_kernel   (walks the row list, CSR)
//   dK    = scale * dS^T Q,  dV = P^T dO  per key block   dkv_kernel  (walks the column list, CSC)
// with P = exp(scale*S - LSE), dS = P * (dO V^T - Delta) recomputed per tile in both kernels,
// so no atomics are needed and the result does not depend on scheduling.
//
// Operand orientation (32x32x16 bf16 MFMA, see asa_fwd.hip for kappa / rho):
//   dq_kernel : keys on the M axis, queries on lanes: S^T = K Q^T and dP^T = V dO^T share the
//               accumulator layout, LSE and Delta are per-lane scalars, and bf16(dS^T) is directly
//               the B operand of dQ^T = K^T dS^T (K^T tiles come from a per-block transposed copy of K).
//   dkv_kernel: queries on the M axis, keys on lanes: S = Q K^T, dP = dO V^T with K, V of the
//               wave's 32 keys resident in registers; bf16(P) and bf16(dS) are the B operands of
//               dV^T = dO^T P and dK^T = Q^T dS (dO^T, Q^T tiles from per-block transposed copies).
#include "asa_common.hpp"

namespace asa {

__device__ __forceinline__ int kappa_b(int r) {
  int g = r >> 3, h = (r >> 2) & 1, j = r & 3;
  return 16 * (g >> 1) + 8 * h + 4 * (g & 1) + j;
}
__device__ __forceinline__ int rho_b(int r) {
  int g = r >> 3, h = (r >> 2) & 1, j = r & 3;
  return 16 * h + 4 * g + j;
}

constexpr float kLog2e = 1.44269504088896340736f;

// ---------------------------------------------------------------------------------------
// Delta[slab][row] = sum_x dO[row][x] * (O[row][x] + O_lo[row][x])   (fp32).  16 lanes per row.
// ---------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void delta_kernel(const void *o, const void *o_lo,
                                                    const void *d_o, TensorView to, int H, int L,
                                                    float *delta) {
  const int slab = blockIdx.y;
  const int row = blockIdx.x * 16 + (threadIdx.x >> 4);
  const int sub = threadIdx.x & 15;
  float acc = 0.f;
  if (row < L) {
    const bf16 *po = slab_ptr(o, to, slab, H) + (int64_t)row * to.sL;
    const bf16 *pg = slab_ptr(d_o, to, slab, H) + (int64_t)row * to.sL;
    const bf16 *pl = o_lo ? slab_ptr(o_lo, to, slab, H) + (int64_t)row * to.sL : nullptr;
#pragma unroll
    for (int c = sub * 8; c < D; c += 128) {
      bf16x8 a = *reinterpret_cast<const bf16x8 *>(po + c);
      bf16x8 b = *reinterpret_cast<const bf16x8 *>(pg + c);
      if (pl) {
        bf16x8 lo = *reinterpret_cast<const bf16x8 *>(pl + c);
#pragma unroll
        for (int x = 0; x < 8; ++x) acc += ((float)a[x] + (float)lo[x]) * (float)b[x];
      } else {
#pragma unroll
        for (int x = 0; x < 8; ++x) acc += (float)a[x] * (float)b[x];
      }
    }
  }
  acc += __shfl_xor(acc, 8, 64);
  acc += __shfl_xor(acc, 4, 64);
  acc += __shfl_xor(acc, 2, 64);
  acc += __shfl_xor(acc, 1, 64);
  if (row < L && sub == 0) delta[(int64_t)slab * L + row] = acc;
}

struct BwdArgs {
  const void *q, *k, *v, *d_o;
  const bf16 *qt, *kt, *dot;  // [slab][Nb][d][block] transposed-tile copies of Q, K, dO
  const float *lse, *delta;
  const int32_t *row_ptr, *col_idx, *col_ptr, *row_idx;
  void *dq, *dk, *dv;
  TensorView tq, tk, tv, to;
  int H, L, Lpad, Nb, n_slabs;
  float scale, scale_log2e;
};

template <int BLK, int D>
struct BwdCfg {
  static constexpr int kThreads = BLK * 2;
  static constexpr int kRowStride = D + 8;   // row-major tile [BLK][D]
  static constexpr int kColStride = BLK + 8;  // transposed tile [D][BLK]
  static constexpr int kRowTile = BLK * kRowStride;
  static constexpr int kColTile = D * kColStride;
  static constexpr int kDqLds = (2 * kRowTile + kColTile) * 2;
  static constexpr int kDkvLds = (2 * kRowTile + 2 * kColTile) * 2 + 2 * BLK * 4;
};

// copy a [BLK][D] row-major tile (rows clamped to L-1) into LDS
template <int BLK, int D, int THREADS>
__device__ __forceinline__ void load_row_tile(bf16 *dst, const bf16 *src, int64_t sL, int row0,
                                              int L, int tid) {
  constexpr int CH = D / 8;
#pragma unroll
  for (int i = 0; i < BLK * CH / THREADS; ++i) {
    int c = tid + i * THREADS;
    int r = c / CH, cc = c % CH;
    int row = row0 + r;
    row = row < L ? row : L - 1;
    uint4 val = *reinterpret_cast<const uint4 *>(src + (int64_t)row * sL + cc * 8);
    *reinterpret_cast<uint4 *>(dst + r * (D + 8) + cc * 8) = val;
  }
}
// copy transposed tile `blk` ([D][BLK], contiguous) of a [Nb][d][block] array into LDS
template <int BLK, int D, int THREADS>
__device__ __forceinline__ void load_col_tile(bf16 *dst, const bf16 *src, int blk, int tid) {
  constexpr int CV = BLK / 8;
  const bf16 *tile = src + (int64_t)blk * D * BLK;
#pragma unroll
  for (int i = 0; i < D * CV / THREADS; ++i) {
    int c = tid + i * THREADS;
    int r = c / CV, cc = c % CV;
    uint4 val = *reinterpret_cast<const uint4 *>(tile + c * 8);
    *reinterpret_cast<uint4 *>(dst + r * (BLK + 8) + cc * 8) = val;
  }
}

// ---------------------------------------------------------------------------------------
// dQ: one workgroup per query block, one wavefront per 32 query rows.
// ---------------------------------------------------------------------------------------
template <int BLK, int D>
__global__ __launch_bounds__(BLK * 2, 1) void dq_kernel(BwdArgs a) {
  using C = BwdCfg<BLK, D>;
  extern __shared__ __align__(16) unsigned char smem[];
  bf16 *Ks = reinterpret_cast<bf16 *>(smem);
  bf16 *Vs = Ks + C::kRowTile;
  bf16 *Kt = Vs + C::kRowTile;

  const int work = xcd_contiguous_work(blockIdx.x, a.n_slabs * a.Nb);
  if (work < 0) return;
  const int slab = work / a.Nb;
  const int qb = work - slab * a.Nb;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, hl = lane >> 5, n = lane & 31;

  const bf16 *qs = slab_ptr(a.q, a.tq, slab, a.H);
  const bf16 *ks = slab_ptr(a.k, a.tk, slab, a.H);
  const bf16 *vs = slab_ptr(a.v, a.tv, slab, a.H);
  const bf16 *gs = slab_ptr(a.d_o, a.to, slab, a.H);
  const bf16 *kts = a.kt + (int64_t)slab * D * a.Lpad;
  const int32_t *cols = a.col_idx + (int64_t)slab * a.Nb * a.Nb;
  const int t_begin = a.row_ptr[slab * (a.Nb + 1) + qb];
  const int t_end = a.row_ptr[slab * (a.Nb + 1) + qb + 1];

  const int qrow = qb * BLK + wave * 32 + n;
  const bool qvalid = qrow < a.L;
  const int qrow_c = qvalid ? qrow : a.L - 1;
  bf16x8 qreg[D / 16], greg[D / 16];
#pragma unroll
  for (int s = 0; s < D / 16; ++s) {
    qreg[s] = *reinterpret_cast<const bf16x8 *>(qs + (int64_t)qrow_c * a.tq.sL + 16 * s + 8 * hl);
    greg[s] = *reinterpret_cast<const bf16x8 *>(gs + (int64_t)qrow_c * a.to.sL + 16 * s + 8 * hl);
  }
  // rows past L get LSE = +inf, so that every probability is exactly zero
  const float lse2 = qvalid ? a.lse[(int64_t)slab * a.L + qrow] * kLog2e : INFINITY;
  const float delta = qvalid ? a.delta[(int64_t)slab * a.L + qrow] : 0.f;

  f32x16 acc[D / 32];
#pragma unroll
  for (int dm = 0; dm < D / 32; ++dm)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[dm][i] = 0.f;

  const int row_off = kappa_b(n) * C::kRowStride + 8 * hl;
  const int col_off = rho_b(n) * C::kColStride + 8 * hl;
  const float c = a.scale_log2e;

  for (int t = t_begin; t < t_end; ++t) {
    const int j = cols[t];
    __syncthreads();
    load_row_tile<BLK, D, C::kThreads>(Ks, ks, a.tk.sL, j * BLK, a.L, tid);
    load_row_tile<BLK, D, C::kThreads>(Vs, vs, a.tv.sL, j * BLK, a.L, tid);
    load_col_tile<BLK, D, C::kThreads>(Kt, kts, j, tid);
    __syncthreads();
    const bool tail = j * BLK + BLK > a.L;
#pragma unroll
    for (int mt = 0; mt < BLK / 32; ++mt) {
      f32x16 sacc, pacc;
#pragma unroll
      for (int i = 0; i < 16; ++i) { sacc[i] = 0.f; pacc[i] = 0.f; }
#pragma unroll
      for (int s = 0; s < D / 16; ++s) {
        bf16x8 ka = *reinterpret_cast<const bf16x8 *>(Ks + mt * 32 * C::kRowStride + row_off + 16 * s);
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[s], sacc, 0, 0, 0);
        bf16x8 va = *reinterpret_cast<const bf16x8 *>(Vs + mt * 32 * C::kRowStride + row_off + 16 * s);
        pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, greg[s], pacc, 0, 0, 0);
      }
      uint32_t dsb[8];
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        float p0 = fast_exp2(fmaf(sacc[i], c, -lse2));
        float p1 = fast_exp2(fmaf(sacc[i + 1], c, -lse2));
        if (tail) {
          int key = j * BLK + mt * 32 + 16 * (i >> 3) + 8 * hl + (i & 7);
          if (key >= a.L) p0 = 0.f;
          if (key + 1 >= a.L) p1 = 0.f;
        }
        dsb[i >> 1] = pack_bf16x2(p0 * (pacc[i] - delta), p1 * (pacc[i + 1] - delta));
      }
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        uint4 raw = make_uint4(dsb[4 * tt], dsb[4 * tt + 1], dsb[4 * tt + 2], dsb[4 * tt + 3]);
        bf16x8 dsf = *reinterpret_cast<bf16x8 *>(&raw);
#pragma unroll
        for (int dm = 0; dm < D / 32; ++dm) {
          bf16x8 ta = *reinterpret_cast<const bf16x8 *>(Kt + dm * 32 * C::kColStride + col_off +
                                                        16 * (2 * mt + tt));
          acc[dm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ta, dsf, acc[dm], 0, 0, 0);
        }
      }
    }
  }

  if (qvalid) {
    bf16 *dst_row = slab_ptr(a.dq, a.tq, slab, a.H) + (int64_t)qrow * a.tq.sL;
#pragma unroll
    for (int dm = 0; dm < D / 32; ++dm) {
      uint32_t w[8];
#pragma unroll
      for (int i = 0; i < 16; i += 2)
        w[i >> 1] = pack_bf16x2(acc[dm][i] * a.scale, acc[dm][i + 1] * a.scale);
      uint4 *dst = reinterpret_cast<uint4 *>(dst_row + dm * 32 + 16 * hl);
      dst[0] = make_uint4(w[0], w[1], w[2], w[3]);
      dst[1] = make_uint4(w[4], w[5], w[6], w[7]);
    }
  }
}

// ---------------------------------------------------------------------------------------
// dK, dV: one workgroup per key block, one wavefront per 32 keys.
// ---------------------------------------------------------------------------------------
template <int BLK, int D>
__global__ __launch_bounds__(BLK * 2, 1) void dkv_kernel(BwdArgs a) {
  using C = BwdCfg<BLK, D>;
  extern __shared__ __align__(16) unsigned char smem[];
  bf16 *Qs = reinterpret_cast<bf16 *>(smem);
  bf16 *Gs = Qs + C::kRowTile;
  bf16 *Qt = Gs + C::kRowTile;
  bf16 *Gt = Qt + C::kColTile;
  float *sLse = reinterpret_cast<float *>(Gt + C::kColTile);
  float *sDelta = sLse + BLK;

  const int work = xcd_contiguous_work(blockIdx.x, a.n_slabs * a.Nb);
  if (work < 0) return;
  const int slab = work / a.Nb;
  const int kb = work - slab * a.Nb;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, hl = lane >> 5, n = lane & 31;

  const bf16 *qs = slab_ptr(a.q, a.tq, slab, a.H);
  const bf16 *ks = slab_ptr(a.k, a.tk, slab, a.H);
  const bf16 *vs = slab_ptr(a.v, a.tv, slab, a.H);
  const bf16 *gs = slab_ptr(a.d_o, a.to, slab, a.H);
  const bf16 *qts = a.qt + (int64_t)slab * D * a.Lpad;
  const bf16 *gts = a.dot + (int64_t)slab * D * a.Lpad;
  const int32_t *rows = a.row_idx + (int64_t)slab * a.Nb * a.Nb;
  const int t_begin = a.col_ptr[slab * (a.Nb + 1) + kb];
  const int t_end = a.col_ptr[slab * (a.Nb + 1) + kb + 1];

  const int krow = kb * BLK + wave * 32 + n;
  const bool kvalid = krow < a.L;
  const int krow_c = kvalid ? krow : a.L - 1;
  bf16x8 kreg[D / 16], vreg[D / 16];
#pragma unroll
  for (int s = 0; s < D / 16; ++s) {
    kreg[s] = *reinterpret_cast<const bf16x8 *>(ks + (int64_t)krow_c * a.tk.sL + 16 * s + 8 * hl);
    vreg[s] = *reinterpret_cast<const bf16x8 *>(vs + (int64_t)krow_c * a.tv.sL + 16 * s + 8 * hl);
  }
  f32x16 dkacc[D / 32], dvacc[D / 32];
#pragma unroll
  for (int dm = 0; dm < D / 32; ++dm)
#pragma unroll
    for (int i = 0; i < 16; ++i) { dkacc[dm][i] = 0.f; dvacc[dm][i] = 0.f; }

  const int row_off = kappa_b(n) * C::kRowStride + 8 * hl;
  const int col_off = rho_b(n) * C::kColStride + 8 * hl;
  const float c = a.scale_log2e;

  for (int t = t_begin; t < t_end; ++t) {
    const int i_blk = rows[t];
    __syncthreads();
    load_row_tile<BLK, D, C::kThreads>(Qs, qs, a.tq.sL, i_blk * BLK, a.L, tid);
    load_row_tile<BLK, D, C::kThreads>(Gs, gs, a.to.sL, i_blk * BLK, a.L, tid);
    load_col_tile<BLK, D, C::kThreads>(Qt, qts, i_blk, tid);
    load_col_tile<BLK, D, C::kThreads>(Gt, gts, i_blk, tid);
    if (tid < BLK) {
      int r = i_blk * BLK + tid;
      bool ok = r < a.L;
      sLse[tid] = ok ? a.lse[(int64_t)slab * a.L + r] * kLog2e : INFINITY;
      sDelta[tid] = ok ? a.delta[(int64_t)slab * a.L + r] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int mt = 0; mt < BLK / 32; ++mt) {
      f32x16 sacc, pacc;
#pragma unroll
      for (int i = 0; i < 16; ++i) { sacc[i] = 0.f; pacc[i] = 0.f; }
#pragma unroll
      for (int s = 0; s < D / 16; ++s) {
        bf16x8 qa = *reinterpret_cast<const bf16x8 *>(Qs + mt * 32 * C::kRowStride + row_off + 16 * s);
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa, kreg[s], sacc, 0, 0, 0);
        bf16x8 ga = *reinterpret_cast<const bf16x8 *>(Gs + mt * 32 * C::kRowStride + row_off + 16 * s);
        pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ga, vreg[s], pacc, 0, 0, 0);
      }
      // accumulator register i of lane half hl is query 32mt + 16(i/8) + 8hl + (i%8)
      uint32_t pb[8], dsb[8];
#pragma unroll
      for (int t8 = 0; t8 < 2; ++t8) {
        const int q0 = mt * 32 + 16 * t8 + 8 * hl;
        f32x4 l0 = *reinterpret_cast<const f32x4 *>(sLse + q0);
        f32x4 l1 = *reinterpret_cast<const f32x4 *>(sLse + q0 + 4);
        f32x4 d0 = *reinterpret_cast<const f32x4 *>(sDelta + q0);
        f32x4 d1 = *reinterpret_cast<const f32x4 *>(sDelta + q0 + 4);
        float lv[8] = {l0[0], l0[1], l0[2], l0[3], l1[0], l1[1], l1[2], l1[3]};
        float dv[8] = {d0[0], d0[1], d0[2], d0[3], d1[0], d1[1], d1[2], d1[3]};
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
          const int i = 8 * t8 + e;
          float p0 = kvalid ? fast_exp2(fmaf(sacc[i], c, -lv[e])) : 0.f;
          float p1 = kvalid ? fast_exp2(fmaf(sacc[i + 1], c, -lv[e + 1])) : 0.f;
          pb[i >> 1] = pack_bf16x2(p0, p1);
          dsb[i >> 1] = pack_bf16x2(p0 * (pacc[i] - dv[e]), p1 * (pacc[i + 1] - dv[e + 1]));
        }
      }
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        uint4 praw = make_uint4(pb[4 * tt], pb[4 * tt + 1], pb[4 * tt + 2], pb[4 * tt + 3]);
        uint4 draw = make_uint4(dsb[4 * tt], dsb[4 * tt + 1], dsb[4 * tt + 2], dsb[4 * tt + 3]);
        bf16x8 pf = *reinterpret_cast<bf16x8 *>(&praw);
        bf16x8 df = *reinterpret_cast<bf16x8 *>(&draw);
#pragma unroll
        for (int dm = 0; dm < D / 32; ++dm) {
          const int off = dm * 32 * C::kColStride + col_off + 16 * (2 * mt + tt);
          bf16x8 ga = *reinterpret_cast<const bf16x8 *>(Gt + off);
          dvacc[dm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ga, pf, dvacc[dm], 0, 0, 0);
          bf16x8 qa = *reinterpret_cast<const bf16x8 *>(Qt + off);
          dkacc[dm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa, df, dkacc[dm], 0, 0, 0);
        }
      }
    }
  }

  if (kvalid) {
    bf16 *dk_row = slab_ptr(a.dk, a.tk, slab, a.H) + (int64_t)krow * a.tk.sL;
    bf16 *dv_row = slab_ptr(a.dv, a.tv, slab, a.H) + (int64_t)krow * a.tv.sL;
#pragma unroll
    for (int dm = 0; dm < D / 32; ++dm) {
      uint32_t wk[8], wv[8];
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        wk[i >> 1] = pack_bf16x2(dkacc[dm][i] * a.scale, dkacc[dm][i + 1] * a.scale);
        wv[i >> 1] = pack_bf16x2(dvacc[dm][i], dvacc[dm][i + 1]);
      }
      uint4 *pk = reinterpret_cast<uint4 *>(dk_row + dm * 32 + 16 * hl);
      pk[0] = make_uint4(wk[0], wk[1], wk[2], wk[3]);
      pk[1] = make_uint4(wk[4], wk[5], wk[6], wk[7]);
      uint4 *pv = reinterpret_cast<uint4 *>(dv_row + dm * 32 + 16 * hl);
      pv[0] = make_uint4(wv[0], wv[1], wv[2], wv[3]);
      pv[1] = make_uint4(wv[4], wv[5], wv[6], wv[7]);
    }
  }
}

// ---------------------------------------------------------------------------------------
static size_t round256(size_t x) { return (x + 255) & ~(size_t)255; }
static size_t transposed_bytes(const Problem &pb) {
  return round256((size_t)pb.n_slabs * pb.d * pb.Lpad * sizeof(uint16_t));
}

size_t bwd_workspace_bytes(const Problem &pb) {
  // Q^T, K^T, dO^T as [slab][Nb][d][block] bf16, then Delta [slab][L] fp32
  return 3 * transposed_bytes(pb) + round256((size_t)pb.n_slabs * pb.L * sizeof(float));
}

template <int BLK, int D>
static hipError_t launch_bwd_t(const BwdArgs &a, hipStream_t st) {
  using C = BwdCfg<BLK, D>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&dq_kernel<BLK, D>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, C::kDqLds);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(&dkv_kernel<BLK, D>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, C::kDkvLds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int grid = xcd_grid(a.n_slabs * a.Nb);
  timing_begin(st);
  hipLaunchKernelGGL((dkv_kernel<BLK, D>), dim3(grid), dim3(C::kThreads), C::kDkvLds, st, a);
  hipError_t e = hipGetLastError();
  if (e == hipSuccess) {
    hipLaunchKernelGGL((dq_kernel<BLK, D>), dim3(grid), dim3(C::kThreads), C::kDqLds, st, a);
    e = hipGetLastError();
  }
  timing_end(st);
  return e;
}

hipError_t launch_bwd(const Problem &pb, const void *q, const void *k, const void *v,
                      const void *o, const void *o_lo, const void *d_o, const float *lse,
                      const int32_t *row_ptr, const int32_t *col_idx, const int32_t *col_ptr,
                      const int32_t *row_idx, void *dq, void *dk, void *dv, void *workspace,
                      hipStream_t st) {
  unsigned char *ws = reinterpret_cast<unsigned char *>(workspace);
  const size_t tb = transposed_bytes(pb);
  bf16 *qt = reinterpret_cast<bf16 *>(ws);
  bf16 *kt = reinterpret_cast<bf16 *>(ws + tb);
  bf16 *dot = reinterpret_cast<bf16 *>(ws + 2 * tb);
  float *delta = reinterpret_cast<float *>(ws + 3 * tb);

  hipError_t e = launch_transpose(pb, q, pb.q, qt, st);
  if (e != hipSuccess) return e;
  e = launch_transpose(pb, k, pb.k, kt, st);
  if (e != hipSuccess) return e;
  e = launch_transpose(pb, d_o, pb.o, dot, st);
  if (e != hipSuccess) return e;
  dim3 dgrid((pb.L + 15) / 16, pb.n_slabs);
  if (pb.d == 128)
    hipLaunchKernelGGL(delta_kernel<128>, dgrid, dim3(256), 0, st, o, o_lo, d_o, pb.o, pb.H, pb.L,
                       delta);
  else
    hipLaunchKernelGGL(delta_kernel<64>, dgrid, dim3(256), 0, st, o, o_lo, d_o, pb.o, pb.H, pb.L,
                       delta);
  e = hipGetLastError();
  if (e != hipSuccess) return e;

  BwdArgs a;
  a.q = q; a.k = k; a.v = v; a.d_o = d_o;
  a.qt = qt; a.kt = kt; a.dot = dot;
  a.lse = lse; a.delta = delta;
  a.row_ptr = row_ptr; a.col_idx = col_idx; a.col_ptr = col_ptr; a.row_idx = row_idx;
  a.dq = dq; a.dk = dk; a.dv = dv;
  a.tq = pb.q; a.tk = pb.k; a.tv = pb.v; a.to = pb.o;
  a.H = pb.H; a.L = pb.L; a.Lpad = pb.Lpad; a.Nb = pb.Nb; a.n_slabs = pb.n_slabs;
  a.scale = pb.scale;
  a.scale_log2e = pb.scale * kLog2e;
  if (pb.block == 128 && pb.d == 128) return launch_bwd_t<128, 128>(a, st);
  if (pb.block == 128 && pb.d == 64) return launch_bwd_t<128, 64>(a, st);
  if (pb.block == 64 && pb.d == 128) return launch_bwd_t<64, 128>(a, st);
  if (pb.block == 64 && pb.d == 64) return launch_bwd_t<64, 64>(a, st);
  return hipErrorInvalidValue;
}

}  // namespace asa
