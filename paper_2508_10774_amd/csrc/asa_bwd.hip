// Block-sparse attention backward for gfx950, mask held constant (the paper restricts attention
// with the block mask "during both training and inference", Sec. 3.3 Step 2.1).
//
//   Delta = rowsum(dO * O), LSE in log2 units     delta_kernel (both padded to whole blocks)
//   dQ    = scale * dS K     per query block      dq_kernel   (walks the row list, CSR)
//   dK    = scale * dS^T Q,  dV = P^T dO  per key block   dkv_kernel  (walks the column list, CSC)
// with P = exp(scale*S - LSE), dS = P * (dO V^T - Delta) recomputed per tile in both kernels,
// so no atomics are needed and the result does not depend on scheduling.
//
// Operand orientation (32x32x16 bf16 MFMA, see asa_fwd.hip for kappa / rho):
//   dq_kernel : keys on the M axis, queries on lanes: S^T = K Q^T and dP^T = V dO^T share the
//               accumulator layout, LSE and Delta are per-lane scalars, and bf16(dS^T) is directly
//               the B operand of dQ^T = K^T dS^T (K^T operand by transposing LDS reads of the K rows).
//   dkv_kernel: queries on the M axis, keys on lanes: S = Q K^T, dP = dO V^T with K, V of the
//               wave's 32 keys resident in registers; bf16(P) and bf16(dS) are the B operands of
//               dV^T = dO^T P and dK^T = Q^T dS (dO^T, Q^T operands by transposing LDS reads of
//               the row tiles).
#include <stdlib.h>

#include <type_traits>

#include "asa_common.hpp"
#include "asa_tiles.hpp"

namespace asa {

__device__ __forceinline__ int kappa_b(int r) { return kappa(r); }

constexpr float kLog2e = 1.44269504088896340736f;

// ---------------------------------------------------------------------------------------
// Row statistics of the backward, padded to whole blocks (pitch Lpad) so that the kernels can
// fetch 64 of them without a bounds test:
//   delta[slab][row] = sum_x dO[row][x] * (O[row][x] + O_lo[row][x])  (fp32), 0 past L
//   lse2[slab][row]  = LSE[row] * log2(e), +inf past L (every probability of such a row is 0)
//   lse2g            = lse2 - bias (for keys whose scores carry an additive bias), if asked for
// 16 lanes per row.
// ---------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void delta_kernel(const void *o, const void *o_lo,
                                                    const void *d_o, TensorView to, int H, int L,
                                                    int Lpad, const float *lse, float bias_log2,
                                                    float *delta, float *lse2, float *lse2g) {
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
  if (row < Lpad && sub == 0) {
    const int64_t at = (int64_t)slab * Lpad + row;
    const float l2 = row < L ? lse[(int64_t)slab * L + row] * kLog2e : INFINITY;
    delta[at] = acc;
    lse2[at] = l2;
    if (lse2g) lse2g[at] = l2 - bias_log2;
  }
}

struct BwdArgs {
  const void *q, *k, *v, *d_o;
  const float *lse2, *delta;  // [slab][Lpad]: LSE * log2(e) (minus this launch's key bias), Delta; padded with +inf, 0
  float *delta_out;           // where the Delta-only walk of dq_kernel writes (the same array as delta)
  const int32_t *row_ptr, *col_idx, *col_ptr, *row_idx;
  void *dq, *dk, *dv;
  TensorView tq, tk, tv, to;
  int H, L, Lpad, Nb, n_slabs;
  float scale, scale_log2e;
  const int32_t *order;   // dK/dV: work item of each workgroup slot, longest column first inside an XCD's share (null: natural order)
  const int32_t *order_q; // dQ: the same by rows
  // ---- global tokens of ASA_G (all zero / null when they are not used)
  // dK/dV kernels: the key side of a launch may be the pooled tokens instead of K, V
  int Lk, Nbk;            // valid key rows and key blocks of this launch (= L, Nb normally)
  float *gk32, *gv32;     // non-null: write fp32 gradients [chunk][slab][Nbk * block][d] here instead of dk / dv
  int q_chunks;           // with gk32 / gv32: the query blocks are split into this many ranges, one workgroup each
  const float *pool_gk, *pool_gv;   // non-null: add pool_g*[slab][row / pool_n] / count(window) to row's gradient
  int pool_n, pool_rows;  // pooling window; rows per slab of pool_gk / pool_gv
  // dQ kernel: pooled tiles appended to every query block's list
  const void *kg, *vg;    // [slab][Nbg * block][d] bf16
  int Lg, Nbg;
  float pooled_bias_log2;
};

template <int BLK, int D>
struct BwdCfg {
  static constexpr int kWaves = BLK / 32;
  static constexpr int kThreads = kWaves * 64;
  static constexpr int kST = 64;                 // rows (keys or queries) per step
  static constexpr int kSub = BLK / kST;         // steps per block
  static constexpr int kRowTile = kST * D;       // [64][D]  elements, swizzled, unpadded
  // LDS stages: two where the second does not cost a resident workgroup (block 128), else one
  static constexpr int kStages = BLK == 128 ? 2 : 1;
  static constexpr int kDqStage = 2 * kRowTile * 2;                  // K rows, V rows
  static constexpr int kDqLds = kStages * kDqStage;
  static constexpr int kDkvStage = 2 * kRowTile * 2 + 2 * kST * 4;   // Q rows, dO rows, LSE, Delta
  static constexpr int kDkvLds = kStages * kDkvStage;
};

// ---------------------------------------------------------------------------------------
// dQ: one workgroup per query block, one wavefront per 32 query rows (its Q and dO rows stay
// in registers as B operands).  Per step of 64 keys the workgroup copies K rows and V rows
// straight into one of two LDS stages while it works on the other; the "channels x keys"
// operand of dQ^T = K^T dS^T is gathered from the K row tile by the transposing LDS read.
// ---------------------------------------------------------------------------------------
// GT: with the pooled (global) tokens of ASA_G appended to every query block's list
// DELTA_ONLY: no gradient; the same walk forms Delta_q = sum_c P_qc dP_qc (= rowsum(dO * O) with
// the exact O, since the P of a row sum to 1) from the unrounded fp32 P and dP and writes it to
// a.delta_out.  Used when the caller has not kept the low half of O: Delta from the bf16 O alone
// is off by up to 0.05 in rows whose soft-max is spread over keys with similar values, and that
// error goes into dQ and dK times the size of the keys / queries.
template <int BLK, int D, bool GT, bool DELTA_ONLY = false>
__global__ __launch_bounds__(BLK * 2, 2) void dq_kernel(BwdArgs a) {
  using C = BwdCfg<BLK, D>;
  extern __shared__ __align__(1024) unsigned char smem[];
  __shared__ int cols[kMaxNb];
  constexpr int kStage = C::kDqStage;          // K rows [64][D], V rows [64][D] (t_swz images)
  constexpr int kVOff = C::kRowTile * 2;

  const int slot = xcd_contiguous_work(blockIdx.x, a.n_slabs * a.Nb);
  if (slot < 0) return;
  const int work = a.order_q ? a.order_q[slot] : slot;
  const int slab = work / a.Nb;
  const int qb = work - slab * a.Nb;
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63, hl = lane >> 5, n = lane & 31;

  const bf16 *qs = slab_ptr(a.q, a.tq, slab, a.H);
  const bf16 *ks = slab_ptr(a.k, a.tk, slab, a.H);
  const bf16 *vs = slab_ptr(a.v, a.tv, slab, a.H);
  const bf16 *gs = slab_ptr(a.d_o, a.to, slab, a.H);
  const bool dense = a.row_ptr == nullptr;   // no index lists: every key block
  const int t_begin = dense ? 0 : a.row_ptr[slab * (a.Nb + 1) + qb];
  const int n_own_tiles = dense ? a.Nb : a.row_ptr[slab * (a.Nb + 1) + qb + 1] - t_begin;
  const int n_tiles = n_own_tiles + (GT ? a.Nbg : 0);   // pooled blocks come after the row's own list
  {
    const int32_t *g = a.col_idx + (int64_t)slab * a.Nb * a.Nb + t_begin;
    for (int t = tid; t < n_tiles; t += C::kThreads)
      cols[t] = t >= n_own_tiles ? t - n_own_tiles : (dense ? t : g[t]);
  }
  // pooled keys / values of this slab: rows of D elements, padded to whole blocks
  const bf16 *kgs = reinterpret_cast<const bf16 *>(a.kg) + (int64_t)slab * a.Nbg * BLK * D;
  const bf16 *vgs = reinterpret_cast<const bf16 *>(a.vg) + (int64_t)slab * a.Nbg * BLK * D;

  const int qrow = qb * BLK + wave * 32 + n;
  const bool qvalid = qrow < a.L;
  const int qrow_c = qvalid ? qrow : a.L - 1;
  bf16x8 qreg[D / 16], greg[D / 16];
#pragma unroll
  for (int s = 0; s < D / 16; ++s) {
    qreg[s] = *reinterpret_cast<const bf16x8 *>(qs + (int64_t)qrow_c * a.tq.sL + 16 * s + 8 * hl);
    greg[s] = *reinterpret_cast<const bf16x8 *>(gs + (int64_t)qrow_c * a.to.sL + 16 * s + 8 * hl);
  }
  // rows past L have LSE = +inf there, so that every probability is exactly zero
  const float lse2 = a.lse2[(int64_t)slab * a.Lpad + qrow];
  const float delta = DELTA_ONLY ? 0.f : a.delta[(int64_t)slab * a.Lpad + qrow];
  float dsum = 0.f;   // DELTA_ONLY: sum of P * dP over my keys

  f32x16 acc[D / 32];
#pragma unroll
  for (int dm = 0; dm < D / 32; ++dm)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[dm][i] = 0.f;

  // row-wise A fragments (S^T = K Q^T, dP^T = V dO^T): row kappa(n) of a 32-key group
  const int kr = kappa_b(n);
  const int kx = (hl ^ t_swz<D>(kr)) * 8;
  // transposed A fragments "32 channels x 16 keys" of dQ^T += K^T dS^T (see dkv_kernel)
  const lds_char *smem_lds = (const lds_char *)smem;
  const uint32_t smem_addr = ASA_LDS_ADDR_OF(smem);
  const int tr_i = lane & 15, tr_w = tr_i & 3, tr_j = tr_i >> 2, tr_b = (lane >> 4) & 1;
  const uint32_t tr_lane = tr_piece<D>(8 * hl + tr_j, 16 * (tr_w & 1) + 8 * tr_b + 4 * (tr_w >> 1));
  const float c = a.scale_log2e;
  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f,
                         0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  const int n_steps = n_tiles * C::kSub;
  auto issue = [&](int step, int stage) {
    const int key0 = cols[step / C::kSub] * BLK + (step % C::kSub) * C::kST;
    int lane_o = lane;
    asm volatile("" : "+v"(lane_o));   // offsets are rebuilt here, not hoisted into registers
    using RowCopy = LeanRowTileCopy<C::kST, D, C::kWaves>;
    const uint32_t st = smem_addr + stage * kStage;
    if (GT && step >= n_own_tiles * C::kSub) {
      RowCopy::issue(st, kgs, key0, a.Nbg * BLK, D, wave, lane_o);   // never ragged
      RowCopy::issue(st + kVOff, vgs, key0, a.Nbg * BLK, D, wave, lane_o);
    } else {
      RowCopy::issue(st, ks, key0, a.L, a.tk.sL, wave, lane_o);
      RowCopy::issue(st + kVOff, vs, key0, a.L, a.tv.sL, wave, lane_o);
    }
  };
  if (C::kStages == 2) {
    __syncthreads();   // cols[] is written
    if (n_steps > 0) issue(0, 0);
  }
  for (int step = 0; step < n_steps; ++step) {
    __builtin_amdgcn_s_setprio(3);
    if (C::kStages == 1) {
      __syncthreads();                    // cols[] is written; everyone is done with the stage
      issue(step, 0);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): my copies of this step have landed
    __syncthreads();                      // everyone's have; everyone is done with the other stage
    const int stage = C::kStages == 2 ? (step & 1) : 0;
    if (C::kStages == 2 && step + 1 < n_steps) issue(step + 1, stage ^ 1);
    const bf16 *Ks = reinterpret_cast<const bf16 *>(smem + stage * kStage);
    const bf16 *Vs = Ks + C::kRowTile;
    const uint32_t tr_base = tr_lane + (uint32_t)(stage * kStage);   // kStage % 512 == 0
    const int key0 = cols[step / C::kSub] * BLK + (step % C::kSub) * C::kST;
    const bool pooled = GT && step >= n_own_tiles * C::kSub;
    const int key_end = pooled ? a.Lg : a.L;   // keys at or past it do not exist
    const bool tail = key0 + C::kST > key_end;
    const float lse_b = pooled ? lse2 - a.pooled_bias_log2 : lse2;
#pragma unroll
    for (int mt = 0; mt < C::kST / 32; ++mt) {
      __builtin_amdgcn_s_setprio(0);
      const bf16 *krow = Ks + (mt * 32 + kr) * D;
      const bf16 *vrow = Vs + (mt * 32 + kr) * D;
      f32x16 sacc = zero16, pacc = zero16;
#pragma unroll
      for (int s = 0; s < D / 16; ++s) {
        bf16x8 ka = *reinterpret_cast<const bf16x8 *>(krow + ((16 * s) ^ kx));
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[s], sacc, 0, 0, 0);
        bf16x8 va = *reinterpret_cast<const bf16x8 *>(vrow + ((16 * s) ^ kx));
        pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, greg[s], pacc, 0, 0, 0);
      }
      // accumulator register i of lane half hl is key 32mt + 16(i/8) + 8hl + (i%8)
      uint32_t dsb[8];
      __builtin_amdgcn_s_setprio(3);   // vector work goes ahead of the other workgroup's MFMA stream
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        float p0 = fast_exp2(fmaf(sacc[i], c, -lse_b));
        float p1 = fast_exp2(fmaf(sacc[i + 1], c, -lse_b));
        if (tail) {
          int key = key0 + mt * 32 + 16 * (i >> 3) + 8 * hl + (i & 7);
          if (key >= key_end) p0 = 0.f;
          if (key + 1 >= key_end) p1 = 0.f;
        }
        if (DELTA_ONLY) dsum += fmaf(p0, pacc[i], p1 * pacc[i + 1]);
        else dsb[i >> 1] = pack_bf16x2(p0 * (pacc[i] - delta), p1 * (pacc[i + 1] - delta));
      }
      __builtin_amdgcn_s_setprio(0);
      if (DELTA_ONLY) continue;
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        uint4 raw = make_uint4(dsb[4 * tt], dsb[4 * tt + 1], dsb[4 * tt + 2], dsb[4 * tt + 3]);
        bf16x8 dsf = *reinterpret_cast<bf16x8 *>(&raw);
#pragma unroll
        for (int dm = 0; dm < D / 32; ++dm) {
          // keys 32 mt + 16 tt + 8 hl + (0..7) of channels 32 dm + rho(lane % 32)
          const uint32_t x0 = (uint32_t)(((4 * dm) ^ t_swz<D>(0)) * 16), x1 = (uint32_t)(((4 * dm) ^ t_swz<D>(4)) * 16);
          const bf16x4 lo = lds_read_tr16(smem_lds + ((tr_base ^ x0) + (uint32_t)((32 * mt + 16 * tt) * D * 2)));
          const bf16x4 hi = lds_read_tr16(smem_lds + ((tr_base ^ x1) + (uint32_t)((32 * mt + 16 * tt + 4) * D * 2)));
          const bf16x8 ta = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          acc[dm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ta, dsf, acc[dm], 0, 0, 0);
        }
      }
    }
  }

  if (DELTA_ONLY) {
    // the two lane halves hold different keys of the same query; rows past L get 0 (their P is 0)
    const float total = dsum + swap_halves(dsum);
    if (hl == 0) a.delta_out[(int64_t)slab * a.Lpad + qrow] = total;
    return;
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
// dK, dV: one workgroup per key block, one wavefront per 32 keys; its K and V rows stay in
// registers as B operands and both 32 x d fp32 accumulators live in registers, so S and P are
// computed once per tile for both gradients.  Per step of 64 queries the workgroup copies Q rows
// and dO rows (and the 64 LSE and Delta values) into one of two LDS stages while it works on
// the other.  The products with P^T and dS^T need "channels x queries" operands: they are
// gathered from the same row tiles by the transposing LDS read, so no transposed copy of Q or
// dO exists, in LDS or in memory.  The register file is full (2 wavefronts per SIMD at 256
// registers): per-lane copy offsets are rebuilt at each use instead of kept.
// ---------------------------------------------------------------------------------------
template <int BLK, int D>
__global__ __launch_bounds__(BLK * 2, 2) void dkv_kernel(BwdArgs a) {
  using C = BwdCfg<BLK, D>;
  extern __shared__ __align__(1024) unsigned char smem[];
  __shared__ int rows[kMaxNb];
  // a stage: Q rows [64][D], dO rows [64][D] (t_swz images), LSE [64], Delta [64]
  constexpr int kStage = C::kDkvStage;
  constexpr int kGOff = C::kRowTile * 2, kLseOff = 2 * C::kRowTile * 2, kDeltaOff = kLseOff + C::kST * 4;

  const int work_c = xcd_contiguous_work(blockIdx.x, a.n_slabs * a.Nbk * a.q_chunks);
  if (work_c < 0) return;
  const int chunk = work_c % a.q_chunks;      // range of query blocks (1 range unless pooled keys)
  const int work = a.order ? a.order[work_c] : work_c / a.q_chunks;
  const int slab = work / a.Nbk;
  const int kb = work - slab * a.Nbk;
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63, hl = lane >> 5, n = lane & 31;

  const bf16 *qs = slab_ptr(a.q, a.tq, slab, a.H);
  const bf16 *ks = slab_ptr(a.k, a.tk, slab, a.H);
  const bf16 *vs = slab_ptr(a.v, a.tv, slab, a.H);
  const bf16 *gs = slab_ptr(a.d_o, a.to, slab, a.H);
  const float *lse_s = a.lse2 + (int64_t)slab * a.Lpad;      // padded: every copy is 64 whole values
  const float *delta_s = a.delta + (int64_t)slab * a.Lpad;
  const bool dense = a.col_ptr == nullptr;   // no index lists: every query block
  const int t_begin = dense ? 0 : a.col_ptr[slab * (a.Nb + 1) + kb];
  const int per_chunk = (a.Nb + a.q_chunks - 1) / a.q_chunks;
  const int first = chunk * per_chunk;          // dense: my range of query blocks
  const int n_tiles = dense ? max(0, min(per_chunk, a.Nb - first))
                            : a.col_ptr[slab * (a.Nb + 1) + kb + 1] - t_begin;
  {
    const int32_t *g = a.row_idx + (int64_t)slab * a.Nb * a.Nb + t_begin;
    for (int t = tid; t < n_tiles; t += C::kThreads) rows[t] = dense ? first + t : g[t];
  }

  const int krow = kb * BLK + wave * 32 + n;
  const bool kvalid = krow < a.Lk;
  const int krow_c = kvalid ? krow : a.Lk - 1;
  bf16x8 kreg[D / 16], vreg[D / 16];
#pragma unroll
  for (int s = 0; s < D / 16; ++s) {
    kreg[s] = *reinterpret_cast<const bf16x8 *>(ks + (int64_t)krow_c * a.tk.sL + 16 * s + 8 * hl);
    vreg[s] = *reinterpret_cast<const bf16x8 *>(vs + (int64_t)krow_c * a.tv.sL + 16 * s + 8 * hl);
  }
  f32x16 kacc[D / 32], vacc[D / 32];   // dK^T and dV^T of my 32 keys
#pragma unroll
  for (int dm = 0; dm < D / 32; ++dm)
#pragma unroll
    for (int i = 0; i < 16; ++i) kacc[dm][i] = vacc[dm][i] = 0.f;

  // row-wise A fragments (S = Q K^T, dP = dO V^T): row kappa(n) of a 32-query group
  const int kr = kappa_b(n);
  const int kx = (hl ^ t_swz<D>(kr)) * 8;
  // transposed A fragments "32 channels x 16 queries" (dV^T += dO^T P, dK^T += Q^T dS): lane i of
  // a 16-lane group addresses query i / 4 of 4 consecutive ones and 4 of the channels that
  // the MFMA rows of its group stand for (row order rho); two reads make the 8 queries of a lane
  const lds_char *smem_lds = (const lds_char *)smem;
  const uint32_t smem_addr = ASA_LDS_ADDR_OF(smem);
  const int tr_i = lane & 15, tr_w = tr_i & 3, tr_j = tr_i >> 2, tr_b = (lane >> 4) & 1;
  const uint32_t tr_lane = tr_piece<D>(8 * hl + tr_j, 16 * (tr_w & 1) + 8 * tr_b + 4 * (tr_w >> 1));
  const float c = a.scale_log2e;
  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f,
                         0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  const int n_steps = n_tiles * C::kSub;
  auto issue = [&](int step, int stage) {
    const int q0 = rows[step / C::kSub] * BLK + (step % C::kSub) * C::kST;
    int lane_o = lane;
    asm volatile("" : "+v"(lane_o));   // offsets are rebuilt here, not hoisted into registers
    using RowCopy = LeanRowTileCopy<C::kST, D, C::kWaves>;
    const uint32_t st = smem_addr + stage * kStage;
    RowCopy::issue(st, qs, q0, a.L, a.tq.sL, wave, lane_o);
    RowCopy::issue(st + kGOff, gs, q0, a.L, a.to.sL, wave, lane_o);
    if (wave == 0) lds_dma4_v(lse_s + q0 + lane_o, st + kLseOff);
    if (wave == 1) lds_dma4_v(delta_s + q0 + lane_o, st + kDeltaOff);
  };
  if (C::kStages == 2) {
    __syncthreads();   // rows[] is written
    if (n_steps > 0) issue(0, 0);
  }
  for (int step = 0; step < n_steps; ++step) {
    __builtin_amdgcn_s_setprio(3);
    if (C::kStages == 1) {
      __syncthreads();                    // rows[] is written; everyone is done with the stage
      issue(step, 0);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): my copies of this step have landed
    __syncthreads();                      // everyone's have; everyone is done with the other stage
    const int stage = C::kStages == 2 ? (step & 1) : 0;
    if (C::kStages == 2 && step + 1 < n_steps) issue(step + 1, stage ^ 1);
    const bf16 *Qs = reinterpret_cast<const bf16 *>(smem + stage * kStage);
    const bf16 *Gs = Qs + C::kRowTile;
    const float *sLse = reinterpret_cast<const float *>(smem + stage * kStage + kLseOff);
    const float *sDelta = sLse + C::kST;
    const uint32_t tr_base = tr_lane + (uint32_t)(stage * kStage);   // kStage % 512 == 0
    auto tr_operand = [&](int tile_bytes, int mt, int tt, int dm) -> bf16x8 {
      // queries 32 mt + 16 tt + 8 hl + (0..7) of channels 32 dm + rho(lane % 32)
      const uint32_t x0 = (uint32_t)(((4 * dm) ^ t_swz<D>(0)) * 16), x1 = (uint32_t)(((4 * dm) ^ t_swz<D>(4)) * 16);
      const bf16x4 lo = lds_read_tr16(smem_lds + ((tr_base ^ x0) + (uint32_t)(tile_bytes + (32 * mt + 16 * tt) * D * 2)));
      const bf16x4 hi = lds_read_tr16(smem_lds + ((tr_base ^ x1) + (uint32_t)(tile_bytes + (32 * mt + 16 * tt + 4) * D * 2)));
      return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    };
    // S -> P -> dV first, then dP -> dS -> dK, so that fewer registers are live at once
#pragma unroll
    for (int mt = 0; mt < C::kST / 32; ++mt) {
      __builtin_amdgcn_s_setprio(0);
      const bf16 *qrow = Qs + (mt * 32 + kr) * D;
      const bf16 *grow = Gs + (mt * 32 + kr) * D;
      f32x16 sacc = zero16;
#pragma unroll
      for (int s = 0; s < D / 16; ++s) {
        bf16x8 qa = *reinterpret_cast<const bf16x8 *>(qrow + ((16 * s) ^ kx));
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa, kreg[s], sacc, 0, 0, 0);
      }
      // accumulator register i of lane half hl is query 32mt + 16(i/8) + 8hl + (i%8)
      __builtin_amdgcn_s_setprio(3);   // vector work goes ahead of the other workgroup's MFMA stream
      uint32_t pb[8];
#pragma unroll
      for (int t8 = 0; t8 < 2; ++t8) {
        const int qq = mt * 32 + 16 * t8 + 8 * hl;
        f32x4 l0 = *reinterpret_cast<const f32x4 *>(sLse + qq);
        f32x4 l1 = *reinterpret_cast<const f32x4 *>(sLse + qq + 4);
        float lv[8] = {l0[0], l0[1], l0[2], l0[3], l1[0], l1[1], l1[2], l1[3]};
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
          const int i = 8 * t8 + e;
          sacc[i] = kvalid ? fast_exp2(fmaf(sacc[i], c, -lv[e])) : 0.f;
          sacc[i + 1] = kvalid ? fast_exp2(fmaf(sacc[i + 1], c, -lv[e + 1])) : 0.f;
          pb[i >> 1] = pack_bf16x2(sacc[i], sacc[i + 1]);
        }
      }
      __builtin_amdgcn_s_setprio(0);
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        uint4 raw = make_uint4(pb[4 * tt], pb[4 * tt + 1], pb[4 * tt + 2], pb[4 * tt + 3]);
        bf16x8 bp = *reinterpret_cast<bf16x8 *>(&raw);
#pragma unroll
        for (int dm = 0; dm < D / 32; ++dm)
          vacc[dm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tr_operand(kGOff, mt, tt, dm), bp, vacc[dm], 0, 0, 0);
      }
      f32x16 pacc = zero16;
#pragma unroll
      for (int s = 0; s < D / 16; ++s) {
        bf16x8 ga = *reinterpret_cast<const bf16x8 *>(grow + ((16 * s) ^ kx));
        pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ga, vreg[s], pacc, 0, 0, 0);
      }
      __builtin_amdgcn_s_setprio(3);
      uint32_t dsb[8];
#pragma unroll
      for (int t8 = 0; t8 < 2; ++t8) {
        const int qq = mt * 32 + 16 * t8 + 8 * hl;
        f32x4 d0 = *reinterpret_cast<const f32x4 *>(sDelta + qq);
        f32x4 d1 = *reinterpret_cast<const f32x4 *>(sDelta + qq + 4);
        float dv[8] = {d0[0], d0[1], d0[2], d0[3], d1[0], d1[1], d1[2], d1[3]};
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
          const int i = 8 * t8 + e;
          dsb[i >> 1] = pack_bf16x2(sacc[i] * (pacc[i] - dv[e]), sacc[i + 1] * (pacc[i + 1] - dv[e + 1]));
        }
      }
      __builtin_amdgcn_s_setprio(0);
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        uint4 raw = make_uint4(dsb[4 * tt], dsb[4 * tt + 1], dsb[4 * tt + 2], dsb[4 * tt + 3]);
        bf16x8 bd = *reinterpret_cast<bf16x8 *>(&raw);
#pragma unroll
        for (int dm = 0; dm < D / 32; ++dm)
          kacc[dm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tr_operand(0, mt, tt, dm), bd, kacc[dm], 0, 0, 0);
      }
    }
  }

  // epilogue of one gradient: acc holds its transpose for my 32 keys
  auto emit = [&](f32x16 *acc, const bool is_dv) {
    const float mul = is_dv ? 1.f : a.scale;
    float *out32 = is_dv ? a.gv32 : a.gk32;
    if (out32) {
      // gradients of pooled tokens: kept in fp32 for the launch that spreads them over the windows
      if (kvalid) {
        float *row = out32 + (((int64_t)chunk * a.n_slabs + slab) * a.Nbk * BLK + krow) * D;
#pragma unroll
        for (int dm = 0; dm < D / 32; ++dm)
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            f32x4 v = {acc[dm][4 * q4] * mul, acc[dm][4 * q4 + 1] * mul, acc[dm][4 * q4 + 2] * mul,
                       acc[dm][4 * q4 + 3] * mul};
            *reinterpret_cast<f32x4 *>(row + dm * 32 + 16 * hl + 4 * q4) = v;
          }
      }
      return;
    }
    if (!kvalid) return;
    bf16 *out_row = is_dv ? slab_ptr(a.dv, a.tv, slab, a.H) + (int64_t)krow * a.tv.sL
                          : slab_ptr(a.dk, a.tk, slab, a.H) + (int64_t)krow * a.tk.sL;
    const float *pool = is_dv ? a.pool_gv : a.pool_gk;
#pragma unroll
    for (int dm = 0; dm < D / 32; ++dm)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[dm][i] *= mul;
    if (pool) {
      // the mean over a window passes 1 / count of the pooled token's gradient to each token
      const int w = krow / a.pool_n;
      const int cnt = min(a.pool_n, a.Lk - w * a.pool_n);
      const float inv = 1.f / (float)cnt;
      const float *prow = pool + ((int64_t)slab * a.pool_rows + w) * D;
#pragma unroll
      for (int dm = 0; dm < D / 32; ++dm)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const f32x4 v = *reinterpret_cast<const f32x4 *>(prow + dm * 32 + 16 * hl + 4 * q4);
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[dm][4 * q4 + e] += v[e] * inv;
        }
    }
#pragma unroll
    for (int dm = 0; dm < D / 32; ++dm) {
      uint32_t w[8];
#pragma unroll
      for (int i = 0; i < 16; i += 2)
        w[i >> 1] = pack_bf16x2(acc[dm][i], acc[dm][i + 1]);
      uint4 *po = reinterpret_cast<uint4 *>(out_row + dm * 32 + 16 * hl);
      po[0] = make_uint4(w[0], w[1], w[2], w[3]);
      po[1] = make_uint4(w[4], w[5], w[6], w[7]);
    }
  };
  emit(kacc, false);
  emit(vacc, true);
}

static size_t round256(size_t x) { return (x + 255) & ~(size_t)255; }
static size_t order_bytes(const Problem &pb) {
  return round256((size_t)pb.n_slabs * pb.Nb * sizeof(int32_t));
}
static size_t rowstat_bytes(const Problem &pb) {
  return round256((size_t)pb.n_slabs * pb.Lpad * sizeof(float));
}
size_t bwd_workspace_bytes(const Problem &pb) {
  // three [slab][Lpad] fp32 arrays (Delta, LSE in log2 units, the same minus the pooled keys'
  // bias), then the orders of the dK / dV and of the dQ workgroups
  return 3 * rowstat_bytes(pb) + 2 * order_bytes(pb);
}
// sum of the per-range partial gradients of the pooled tokens into range 0's buffer
__global__ void pooled_reduce_kernel(float *buf, int chunks, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  f32x4 acc = reinterpret_cast<const f32x4 *>(buf)[i];
  for (int c = 1; c < chunks; ++c) {
    const f32x4 v = reinterpret_cast<const f32x4 *>(buf + c * n * 4)[i];
    acc += v;
  }
  reinterpret_cast<f32x4 *>(buf)[i] = acc;
}
static int pooled_chunks(const Problem &pb, int Nbg) {
  // enough workgroups to fill the chip, at most 16 ranges (each costs a partial buffer)
  int c = (1024 + pb.n_slabs * Nbg - 1) / (pb.n_slabs * Nbg);
  c = c > 16 ? 16 : c;
  return c > pb.Nb ? pb.Nb : (c < 1 ? 1 : c);
}
static size_t pooled_rows_bytes(const Problem &pb, int Nbg, size_t elem) {
  return round256((size_t)pb.n_slabs * Nbg * pb.block * pb.d * elem);
}
size_t bwd_g_workspace_bytes(const Problem &pb, int Nbg) {
  // ... then the pooled tokens' dK, dV (fp32, one buffer per range of query blocks)
  return bwd_workspace_bytes(pb) + 2 * pooled_chunks(pb, Nbg) * pooled_rows_bytes(pb, Nbg, 4);
}

template <int BLK, int D>
static hipError_t launch_bwd_t(const BwdArgs &a, const BwdArgs *pooled_launch, hipStream_t st) {
  using C = BwdCfg<BLK, D>;
  {
    const void *dq_fns[4] = {reinterpret_cast<const void *>(&dq_kernel<BLK, D, false>),
                             reinterpret_cast<const void *>(&dq_kernel<BLK, D, true>),
                             reinterpret_cast<const void *>(&dq_kernel<BLK, D, false, true>),
                             reinterpret_cast<const void *>(&dq_kernel<BLK, D, true, true>)};
    for (const void *fn : dq_fns) {
      hipError_t e0 = set_dynamic_lds_once(fn, C::kDqLds);
      if (e0 != hipSuccess) return e0;
    }
    hipError_t e0 = set_dynamic_lds_once(reinterpret_cast<const void *>(&dkv_kernel<BLK, D>), C::kDkvLds);
    if (e0 != hipSuccess) return e0;
  }
  const int grid = xcd_grid(a.n_slabs * a.Nb);
  hipError_t e = hipSuccess;
  if (a.delta_out) {
    // no low half of O from the caller: Delta from the tiles themselves, before anything uses it
    if (pooled_launch)
      hipLaunchKernelGGL((dq_kernel<BLK, D, true, true>), dim3(grid), dim3(C::kThreads), C::kDqLds, st, a);
    else
      hipLaunchKernelGGL((dq_kernel<BLK, D, false, true>), dim3(grid), dim3(C::kThreads), C::kDqLds, st, a);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  timing_begin(st);
  if (pooled_launch) {
    // gradients of the pooled tokens first (fp32, every query block attends them) ...
    const BwdArgs &g = *pooled_launch;
    const int ggrid = xcd_grid(g.n_slabs * g.Nbk * g.q_chunks);
    hipLaunchKernelGGL((dkv_kernel<BLK, D>), dim3(ggrid), dim3(C::kThreads), C::kDkvLds, st, g);
    e = hipGetLastError();
    if (e == hipSuccess && g.q_chunks > 1) {
      const int64_t n4 = (int64_t)g.n_slabs * g.Nbk * BLK * D / 4;
      const int rgrid = (int)((n4 + 255) / 256);
      hipLaunchKernelGGL(pooled_reduce_kernel, dim3(rgrid), dim3(256), 0, st, g.gv32, g.q_chunks, n4);
      hipLaunchKernelGGL(pooled_reduce_kernel, dim3(rgrid), dim3(256), 0, st, g.gk32, g.q_chunks, n4);
      e = hipGetLastError();
    }
  }
  // ... then the tokens' own gradients, which add their share of the pooled ones
  if (e == hipSuccess) {
    hipLaunchKernelGGL((dkv_kernel<BLK, D>), dim3(grid), dim3(C::kThreads), C::kDkvLds, st, a);
    e = hipGetLastError();
  }
  if (e == hipSuccess) {
    if (pooled_launch)
      hipLaunchKernelGGL((dq_kernel<BLK, D, true>), dim3(grid), dim3(C::kThreads), C::kDqLds, st, a);
    else
      hipLaunchKernelGGL((dq_kernel<BLK, D, false>), dim3(grid), dim3(C::kThreads), C::kDqLds, st, a);
    e = hipGetLastError();
  }
  timing_end(st);
  return e;
}

hipError_t launch_bwd(const Problem &pb, const void *q, const void *k, const void *v,
                      const void *o, const void *o_lo, const void *d_o, const float *lse,
                      const int32_t *row_ptr, const int32_t *col_idx, const int32_t *col_ptr,
                      const int32_t *row_idx, void *dq, void *dk, void *dv, void *workspace,
                      hipStream_t st, const GlobalTokens *gt) {
  unsigned char *ws = reinterpret_cast<unsigned char *>(workspace);
  const size_t rb = rowstat_bytes(pb);
  float *delta = reinterpret_cast<float *>(ws);
  float *lse2 = reinterpret_cast<float *>(ws + rb);
  float *lse2g = reinterpret_cast<float *>(ws + 2 * rb);
  int32_t *order = reinterpret_cast<int32_t *>(ws + 3 * rb);

  hipError_t e = hipSuccess;
  const float pooled_bias = gt ? log2f((float)gt->n) : 0.f;
  dim3 dgrid((pb.Lpad + 15) / 16, pb.n_slabs);
  if (pb.d == 128)
    hipLaunchKernelGGL(delta_kernel<128>, dgrid, dim3(256), 0, st, o, o_lo, d_o, pb.o, pb.H, pb.L,
                       pb.Lpad, lse, pooled_bias, delta, lse2, gt ? lse2g : nullptr);
  else
    hipLaunchKernelGGL(delta_kernel<64>, dgrid, dim3(256), 0, st, o, o_lo, d_o, pb.o, pb.H, pb.L,
                       pb.Lpad, lse, pooled_bias, delta, lse2, gt ? lse2g : nullptr);
  e = hipGetLastError();
  if (e != hipSuccess) return e;

  BwdArgs a;
  a.q = q; a.k = k; a.v = v; a.d_o = d_o;
  a.lse2 = lse2; a.delta = delta;
  a.delta_out = o_lo ? nullptr : delta;
  a.row_ptr = row_ptr; a.col_idx = col_idx; a.col_ptr = col_ptr; a.row_idx = row_idx;
  a.dq = dq; a.dk = dk; a.dv = dv;
  a.tq = pb.q; a.tk = pb.k; a.tv = pb.v; a.to = pb.o;
  a.H = pb.H; a.L = pb.L; a.Lpad = pb.Lpad; a.Nb = pb.Nb; a.n_slabs = pb.n_slabs;
  a.scale = pb.scale;
  a.scale_log2e = pb.scale * kLog2e;
  a.order = nullptr;
  a.order_q = nullptr;
  {
    const int total = pb.n_slabs * pb.Nb;
    if (col_ptr && length_order_fits(total)) {
      e = launch_length_order(col_ptr, pb.Nb, total, order, st);
      if (e != hipSuccess) return e;
      a.order = order;
      int32_t *order_q = reinterpret_cast<int32_t *>(ws + 3 * rb + order_bytes(pb));
      e = launch_length_order(row_ptr, pb.Nb, total, order_q, st);
      if (e != hipSuccess) return e;
      a.order_q = order_q;
    }
  }
  a.Lk = pb.L; a.Nbk = pb.Nb;
  a.gk32 = a.gv32 = nullptr; a.q_chunks = 1; a.pool_gk = a.pool_gv = nullptr; a.pool_n = 1; a.pool_rows = 0;
  a.kg = a.vg = nullptr; a.Lg = a.Nbg = 0; a.pooled_bias_log2 = 0.f;
  BwdArgs g;                       // the launch whose key side is the pooled tokens
  const BwdArgs *pooled = nullptr;
  if (gt) {
    unsigned char *wg = ws + bwd_workspace_bytes(pb);
    float *gk32 = reinterpret_cast<float *>(wg);
    const int chunks = pooled_chunks(pb, gt->Nbg);
    float *gv32 = reinterpret_cast<float *>(wg + chunks * pooled_rows_bytes(pb, gt->Nbg, 4));
    TensorView tvg;                // the pooled tensors: [slab][Nbg * block][d], rows of d elements
    tvg.sL = pb.d; tvg.sH = (int64_t)gt->Nbg * pb.block * pb.d; tvg.sB = tvg.sH * pb.H;
    const float bias = pooled_bias;
    g = a;
    g.order = nullptr;
    g.order_q = nullptr;
    g.k = gt->kg; g.v = gt->vg; g.tk = tvg; g.tv = tvg;
    g.col_ptr = nullptr; g.row_idx = nullptr;          // every query block attends the pooled tokens
    g.Lk = gt->Lg; g.Nbk = gt->Nbg; g.lse2 = lse2g;
    g.gk32 = gk32; g.gv32 = gv32; g.q_chunks = chunks;
    pooled = &g;
    a.pool_gk = gk32; a.pool_gv = gv32; a.pool_n = gt->n; a.pool_rows = gt->Nbg * pb.block;
    a.kg = gt->kg; a.vg = gt->vg; a.Lg = gt->Lg; a.Nbg = gt->Nbg;
    a.pooled_bias_log2 = bias;
  }
  if (pb.block == 128 && pb.d == 128) return launch_bwd_t<128, 128>(a, pooled, st);
  if (pb.block == 128 && pb.d == 64) return launch_bwd_t<128, 64>(a, pooled, st);
  if (pb.block == 64 && pb.d == 128) return launch_bwd_t<64, 128>(a, pooled, st);
  if (pb.block == 64 && pb.d == 64) return launch_bwd_t<64, 64>(a, pooled, st);
  return hipErrorInvalidValue;
}

}  // namespace asa
