// Block-sparse flash-attention forward for gfx950 (Sec. 3.3 Step 2.2 of the paper: the
// binary block mask "directly integrated with a block-sparse attention kernel").
//
// One workgroup owns one query block of one slab and walks that row's list of kept key
// blocks.  A wavefront owns 32 query rows.  Per key tile:
//   S^T = K Q^T      MFMA 32x32x16 bf16, keys on the M axis, queries on the N axis, so a
//                    lane holds 16 keys of ONE query and the row maximum / row sum of the
//                    online soft-max need a single cross-lane exchange;
//   O^T += V^T P^T   the accumulator of S^T, rounded to bf16, already IS the B operand of
//                    this product, provided the rows of K are read in the permuted order
//                    kappa; V is consumed from a per-block transposed copy so that both
//                    LDS operand reads are 16-byte loads.
// A key block is walked in steps of 64 keys.  The K rows and the V^T slice of a step are copied
// straight from global memory into LDS (no register staging) with an XOR swizzle of 16-byte
// chunks instead of row padding, which keeps the 16-byte fragment reads conflict-free.
#include <stdlib.h>

#include <type_traits>

#include "asa_common.hpp"
#include "asa_tiles.hpp"

namespace asa {

// ---------------------------------------------------------------------------------------
// [slab][L][d] -> [slab][Nb][d][block] bf16: every block of `block` positions becomes one
// contiguous transposed tile (channels major), zero-filled for positions >= L.  A tile is then
// a single contiguous run in memory for the attention kernels, instead of d rows that are
// Lpad * 2 bytes apart (a power-of-two pitch that lands every row on the same memory channel).
// ---------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void transpose_kernel(const void *src, TensorView tv, int H,
                                                        int L, int Lpad, int block, bf16 *dst) {
  constexpr int TL = 64;  // positions per workgroup
  __shared__ uint16_t tile[TL][D + 2];
  const int slab = blockIdx.y;
  const int l0 = blockIdx.x * TL;
  const uint16_t *s = reinterpret_cast<const uint16_t *>(slab_ptr(src, tv, slab, H));
  const int tid = threadIdx.x;
  constexpr int CH = D / 8;  // 16-byte chunks per row
  for (int c = tid; c < TL * CH; c += 256) {
    int r = c / CH, cc = c % CH;
    uint4 val = make_uint4(0, 0, 0, 0);
    if (l0 + r < L) val = *reinterpret_cast<const uint4 *>(s + (int64_t)(l0 + r) * tv.sL + cc * 8);
    const uint16_t *e = reinterpret_cast<const uint16_t *>(&val);
#pragma unroll
    for (int x = 0; x < 8; ++x) tile[r][cc * 8 + x] = e[x];
  }
  __syncthreads();
  // the 64 positions of this workgroup lie inside one block (block is a multiple of 64)
  uint16_t *out = reinterpret_cast<uint16_t *>(dst) + (int64_t)slab * D * Lpad +
                  (int64_t)(l0 / block) * D * block + (l0 % block);
  for (int c = tid; c < D * (TL / 8); c += 256) {
    int dd = c / (TL / 8), lc = c % (TL / 8);
    uint4 val;
    uint16_t *e = reinterpret_cast<uint16_t *>(&val);
#pragma unroll
    for (int x = 0; x < 8; ++x) e[x] = tile[lc * 8 + x][dd];
    *reinterpret_cast<uint4 *>(out + (int64_t)dd * block + lc * 8) = val;
  }
}

hipError_t launch_transpose(const Problem &pb, const void *src, const TensorView &tv, void *dst,
                            hipStream_t st) {
  dim3 grid(pb.Lpad / 64, pb.n_slabs);
  if (pb.d == 128)
    hipLaunchKernelGGL(transpose_kernel<128>, grid, dim3(256), 0, st, src, tv, pb.H, pb.L, pb.Lpad,
                       pb.block, reinterpret_cast<bf16 *>(dst));
  else
    hipLaunchKernelGGL(transpose_kernel<64>, grid, dim3(256), 0, st, src, tv, pb.H, pb.L, pb.Lpad,
                       pb.block, reinterpret_cast<bf16 *>(dst));
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Global tokens of ASA_G (Sec. 3.3): MeanPool_n over the token axis.  One workgroup per pooled
// row, one thread per channel; the mean of the window's valid tokens is formed in fp32 and
// rounded to bf16 (the tensor type of K_aug / V_aug); rows past Lg are zero.
// ---------------------------------------------------------------------------------------
__global__ void pool_kernel(const void *src, TensorView tv, int H, int L, int d, int n, int Lg,
                            int Lg_pad, bf16 *dst) {
  const int w = blockIdx.x, slab = blockIdx.y, c = threadIdx.x;
  bf16 *out = dst + ((int64_t)slab * Lg_pad + w) * d;
  if (w >= Lg) {
    out[c] = (bf16)0.f;
    return;
  }
  const bf16 *x = slab_ptr(src, tv, slab, H);
  const int r0 = w * n, r1 = min(L, r0 + n);
  float acc = 0.f;
  for (int r = r0; r < r1; ++r) acc += (float)x[(int64_t)r * tv.sL + c];
  out[c] = (bf16)(acc / (float)(r1 - r0));
}

hipError_t launch_pool(const Problem &pb, int n, const void *src, const TensorView &tv, void *dst,
                       hipStream_t st) {
  const int Lg = (pb.L + n - 1) / n;
  const int Lg_pad = ((Lg + pb.block - 1) / pb.block) * pb.block;
  hipLaunchKernelGGL(pool_kernel, dim3(Lg_pad, pb.n_slabs), dim3(pb.d), 0, st, src, tv, pb.H, pb.L,
                     pb.d, n, Lg, Lg_pad, reinterpret_cast<bf16 *>(dst));
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// forward kernel
// ---------------------------------------------------------------------------------------
struct FwdArgs {
  const void *q, *k;
  const bf16 *vt;  // [slab][Nb][d][block]: V, one transposed tile per key block
  const int32_t *row_ptr, *col_idx;
  void *o, *o_lo;
  float *lse;
  TensorView tq, tk, to;
  int H, L, Lpad, Nb, n_slabs;
  float scale_log2e;  // scale * log2(e)
  // global tokens (ASA_G); Nbg = 0 switches them off
  const void *kg;     // [slab][Nbg * block][d] bf16 pooled keys, zero rows past Lg
  const bf16 *vgt;    // [slab][Nbg][d][block]: pooled values, transposed tiles
  int Lg, Nbg;        // pooled tokens per slab, key blocks they fill
  float bias_log2;    // log2(n): the additive ln(n) of the pooled scores, in the exp2 domain
  // Choice between the two kernels per (batch, head) slab, made on the device from the slab's
  // tile count: 0 = this launch takes every slab; +1 = only slabs whose rows hold at least
  // `select_min_tiles` tiles on average; -1 = only the others.
  int select, select_min_tiles;
  const int32_t *order;   // work item of each workgroup slot (longest row first inside an XCD's share), or null
};

// does this launch leave the slab to the other kernel?  (wave-uniform; before any barrier)
__device__ __forceinline__ bool slab_not_mine(const FwdArgs &a, int slab) {
  if (a.select == 0) return false;
  const int tiles = a.row_ptr[slab * (a.Nb + 1) + a.Nb];
  const bool long_rows = tiles >= a.select_min_tiles * a.Nb;
  return (a.select > 0) != long_rows;
}

template <int BLK, int D>
struct FwdCfg {
  static constexpr int kWaves = BLK / 32;
  static constexpr int kThreads = kWaves * 64;
  static constexpr int kKT = 64;                   // keys per pipeline step
  static constexpr int kSub = BLK / kKT;           // steps per key block
  static constexpr int kKElems = kKT * D;          // one K stage:   [64 keys][D]  (unpadded)
  static constexpr int kVElems = D * kKT;          // one V^T stage: [D][64 keys]  (unpadded)
  // LDS stages of the lock-step kernel: two where the second does not cost a resident workgroup
  // (block 128: registers allow 2-3 workgroups per CU anyway), one at block 64 (measured at
  // block 64 / d 64: two stages 1.43 ms, one 1.29 ms; at block 128 / d 128: 1.695 vs 1.73 ms)
  static constexpr int kStages = BLK == 128 ? 2 : 1;
};

// The running maximum (and with it O and the row sum) is rescaled only on steps where some row
// of the wavefront actually found a larger logit; on all other steps the factor would be 1.
// The maximum is never allowed to lag behind: a row dominated by one key then has that key's
// probability equal to exactly 1, free of bf16 rounding, which the backward's Delta relies on.
//
// Lock-step kernel: one workgroup per query block, all wavefronts in lock step.  With two LDS
// stages (2 x 32 KB at d = 128) the copies of step s + 1 are requested right after the barrier
// that opens step s; with one, the copies of a step are waited for right away and the other
// workgroups on the CU compute meanwhile.  It serves the tile shapes other than block 128 / d 128 and tensors that the
// ping-pong kernel below does not take (slabs of 4 GiB and more).
template <int BLK, int D>
// (block 64 / d 64 fits 128 registers: four wavefronts per SIMD, 2 % faster than three)
__global__ __launch_bounds__(BLK * 2, (BLK == 64 && D == 64) ? 4 : 2) void fwd_kernel(FwdArgs a) {
  using C = FwdCfg<BLK, D>;
  extern __shared__ __align__(1024) unsigned char smem[];
  bf16 *lds = reinterpret_cast<bf16 *>(smem);
  __shared__ int cols[kMaxNb];

  const int slot = xcd_contiguous_work(blockIdx.x, a.n_slabs * a.Nb);
  if (slot < 0) return;
  const int work = a.order ? a.order[slot] : slot;
  const int slab = work / a.Nb;
  if (slab_not_mine(a, slab)) return;
  const int qb = work - slab * a.Nb;
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63, hl = lane >> 5, n = lane & 31;

  const bf16 *qs = slab_ptr(a.q, a.tq, slab, a.H);
  const bf16 *ks = slab_ptr(a.k, a.tk, slab, a.H);
  const bf16 *vts = a.vt + (int64_t)slab * D * a.Lpad;
  // no index lists: dense attention, every key block in order
  const bool dense = a.row_ptr == nullptr;
  const int t_begin = dense ? 0 : a.row_ptr[slab * (a.Nb + 1) + qb];
  const int n_tiles = dense ? a.Nb : a.row_ptr[slab * (a.Nb + 1) + qb + 1] - t_begin;
  {
    const int32_t *g = a.col_idx + (int64_t)slab * a.Nb * a.Nb + t_begin;
    for (int t = tid; t < n_tiles; t += C::kThreads) cols[t] = dense ? t : g[t];
  }
  const int qrow = qb * BLK + wave * 32 + n;
  const bool qvalid = qrow < a.L;
  const int qrow_c = qvalid ? qrow : a.L - 1;
  bf16x8 qreg[D / 16];
#pragma unroll
  for (int s = 0; s < D / 16; ++s)
    qreg[s] = *reinterpret_cast<const bf16x8 *>(qs + (int64_t)qrow_c * a.tq.sL + 16 * s + 8 * hl);
  f32x16 oacc[D / 32];
#pragma unroll
  for (int dm = 0; dm < D / 32; ++dm)
#pragma unroll
    for (int i = 0; i < 16; ++i) oacc[dm][i] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float c = a.scale_log2e;

  RowTileCopy<C::kKT, D, C::kWaves> copy_k;
  ColTileCopy<BLK, D, C::kWaves> copy_v;
  copy_k.init(wave, lane, a.tk.sL);
  copy_v.init(wave, lane);
  const int kr = kappa(n), cr = rho(n);
  const int kx = (hl ^ k_swz<D>(kr)) * 8, cx = (hl ^ v_swz(cr)) * 8;
  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f,
                         0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  const int n_steps = n_tiles * C::kSub;
  constexpr int kStageElems = C::kKElems + C::kVElems;
  const uint32_t lds_addr = ASA_LDS_ADDR_OF(smem);
  // copies of one step into one of the two stages, issued in the form the compiler does not
  // track (it would otherwise wait for them before the next LDS read of the other stage)
  auto fetch = [&](int step, int stage) __attribute__((always_inline)) {
    const int j = cols[step / C::kSub];
    const int sub = step % C::kSub;
    const int row0 = j * BLK + sub * C::kKT;
    const uint32_t st = lds_addr + stage * kStageElems * 2;
    const char *kbase = reinterpret_cast<const char *>(ks) + (int64_t)row0 * a.tk.sL * 2;
    const int lim = a.L - 1 - row0;
    if (lim >= C::kKT - 1) copy_k.issue_at(st, kbase);
    else copy_k.issue_at_ragged(st, kbase, lim);
    copy_v.issue_at(st + C::kKElems * 2,
                    reinterpret_cast<const char *>(vts + (int64_t)j * D * BLK + sub * C::kKT));
  };
  if (C::kStages == 2) {
    __syncthreads();                      // cols[] is complete
    if (n_steps > 0) fetch(0, 0);
  }
  for (int step = 0; step < n_steps; ++step) {
    if (C::kStages == 1) {
      __syncthreads();                    // cols[] is complete; the stage is free again
      fetch(step, 0);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);   // my copies of this step have landed
    __syncthreads();                      // everyone's have; everyone is done with the other stage
    if (C::kStages == 2 && step + 1 < n_steps) fetch(step + 1, (step + 1) & 1);
    const bf16 *Ks = lds + (C::kStages == 2 ? (step & 1) : 0) * kStageElems;
    const bf16 *Vs = Ks + C::kKElems;
    const int key0 = cols[step / C::kSub] * BLK + (step % C::kSub) * C::kKT;
    f32x16 sacc[C::kKT / 32];
#pragma unroll
    for (int mt = 0; mt < C::kKT / 32; ++mt) {
      const bf16 *krow = Ks + (mt * 32 + kr) * D;
      sacc[mt] = zero16;
#pragma unroll
      for (int s = 0; s < D / 16; ++s) {
        bf16x8 ka = *reinterpret_cast<const bf16x8 *>(krow + ((16 * s) ^ kx));
        sacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[s], sacc[mt], 0, 0, 0);
      }
    }
    if (key0 + C::kKT > a.L) {
#pragma unroll
      for (int mt = 0; mt < C::kKT / 32; ++mt)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          int key = key0 + mt * 32 + 16 * (i >> 3) + 8 * hl + (i & 7);
          if (key >= a.L) sacc[mt][i] = -INFINITY;
        }
    }
    float mx = -INFINITY;
#pragma unroll
    for (int mt = 0; mt < C::kKT / 32; ++mt)
#pragma unroll
      for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sacc[mt][i]);
    mx = fmaxf(mx, swap_halves(mx)) * c;
    if (__any(mx > m_run)) {
      const float m_new = fmaxf(m_run, mx);
      const float alpha = fast_exp2(m_run - ((m_new == -INFINITY) ? 0.f : m_new));
      m_run = m_new;
      l_run *= alpha;
#pragma unroll
      for (int dm = 0; dm < D / 32; ++dm)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[dm][i] *= alpha;
    }
    const float m_use = (m_run == -INFINITY) ? 0.f : m_run;
    float lsum = 0.f;
#pragma unroll
    for (int mt = 0; mt < C::kKT / 32; ++mt) {
      uint32_t pb[8];
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        const float p0 = fast_exp2(fmaf(sacc[mt][i], c, -m_use));
        const float p1 = fast_exp2(fmaf(sacc[mt][i + 1], c, -m_use));
        lsum += p0 + p1;
        pb[i >> 1] = pack_bf16x2(p0, p1);
      }
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        uint4 praw = make_uint4(pb[4 * tt], pb[4 * tt + 1], pb[4 * tt + 2], pb[4 * tt + 3]);
        bf16x8 pf = *reinterpret_cast<bf16x8 *>(&praw);
#pragma unroll
        for (int dm = 0; dm < D / 32; ++dm) {
          bf16x8 va = *reinterpret_cast<const bf16x8 *>(Vs + (dm * 32 + cr) * C::kKT +
                                                        ((16 * (2 * mt + tt)) ^ cx));
          oacc[dm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pf, oacc[dm], 0, 0, 0);
        }
      }
    }
    l_run += lsum;
  }

  const float l_tot = l_run + swap_halves(l_run);
  const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
  if (qvalid) {
    bf16 *os = slab_ptr(a.o, a.to, slab, a.H) + (int64_t)qrow * a.to.sL;
    bf16 *ls = a.o_lo ? slab_ptr(a.o_lo, a.to, slab, a.H) + (int64_t)qrow * a.to.sL : nullptr;
#pragma unroll
    for (int dm = 0; dm < D / 32; ++dm) {
      uint32_t w[8], r[8];
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        const float v0 = oacc[dm][i] * inv, v1 = oacc[dm][i + 1] * inv;
        const uint32_t pk = pack_bf16x2(v0, v1);
        w[i >> 1] = pk;
        r[i >> 1] = pack_bf16x2(v0 - bf16_bits_to_float(pk & 0xffffu),
                                v1 - bf16_bits_to_float(pk >> 16));
      }
      uint4 *dst = reinterpret_cast<uint4 *>(os + dm * 32 + 16 * hl);
      dst[0] = make_uint4(w[0], w[1], w[2], w[3]);
      dst[1] = make_uint4(w[4], w[5], w[6], w[7]);
      if (ls) {
        uint4 *dl = reinterpret_cast<uint4 *>(ls + dm * 32 + 16 * hl);
        dl[0] = make_uint4(r[0], r[1], r[2], r[3]);
        dl[1] = make_uint4(r[4], r[5], r[6], r[7]);
      }
    }
    if (hl == 0)
      a.lse[(int64_t)slab * a.L + qrow] =
          l_tot > 0.f ? m_run * 0.69314718055994530942f + __logf(l_tot) : -INFINITY;
  }
}

// ---------------------------------------------------------------------------------------
// Ping-pong forward.  The workgroup has two groups of BLK/32 wavefronts that own the SAME
// query rows; group g processes the 64-key steps s with s mod 2 = g and keeps its own
// (maximum, row sum, O) partial, merged once at the end.  Time is cut into phases separated by
// workgroup barriers.  In phase p group (p mod 2) is in its MATRIX phase -- P V of step p-2, then
// S^T of step p -- while the other group is in its VECTOR phase -- soft-max of step p-1.  The
// two groups share every SIMD pairwise (wavefronts w and w + BLK/32), so at any time one
// wavefront per SIMD feeds the matrix pipe and the other the vector ALU.
//
// What was measured on MI355X and shaped this kernel:
//  * A wavefront whose next instruction is an MFMA that waits for the matrix pipe keeps the
//    SIMD's issue slot: with equal priorities the older wavefront starves the other one's vector
//    instructions completely.  With the VECTOR wavefront at the higher priority both run: the
//    MFMA stream loses nothing and the vector stream runs at ~80 % of its stand-alone rate.
//  * One 64 x 16 B direct-to-LDS load occupies the issuing wavefront for 65..90 cycles (much
//    more on a low-priority wavefront that competes with a busy one).  The copies of a phase
//    are requested by its vector group (it has the priority and no MFMA stream to hold up), one
//    at a time between blocks of soft-max arithmetic.  Never as a burst behind the barrier.
//  * Scalar bookkeeping shows up directly as idle matrix time (the scalar unit is shared):
//    the phase loop is unrolled so that p mod 4 is a compile-time constant, every LDS address
//    is an immediate, and the column list is turned once into byte offsets of the K and V^T
//    tiles (LDS tables padded by repeats of the last entry, so copies past the last step need
//    no clamping).
// Tiles: four LDS buffers each for K and V^T steps, buffer = step mod 4.  Phase p requests K
// of step p+3 and V of step p+1; both buffers were last read in phase p-1.
// ---------------------------------------------------------------------------------------
template <int BLK, int D>
struct PpCfg {
  static constexpr int kGroupWaves = BLK / 32;
  static constexpr int kWaves = 2 * kGroupWaves;
  static constexpr int kThreads = kWaves * 64;
  static constexpr int kKT = 64;
  static constexpr int kSub = BLK / kKT;
  static constexpr int kKElems = kKT * D;
  static constexpr int kVElems = D * kKT;
  static constexpr int kStages = 4;
  static constexpr int kTabPad = 8;
  static constexpr int kLdsBytes = kStages * (kKElems + kVElems) * 2;
};

template <int N>
using Int = std::integral_constant<int, N>;

// GT: with the pooled (global) tokens of ASA_G appended to every query block's list
template <int BLK, int D, bool GT>
__global__ __launch_bounds__(BLK * 4, (BLK == 64 && D == 64) ? 2 : 1) void fwd_pp_kernel(FwdArgs a) {   // (2: its LDS allows it)
  using C = PpCfg<BLK, D>;
  extern __shared__ __align__(1024) unsigned char smem[];
  bf16 *ldsK = reinterpret_cast<bf16 *>(smem);
  bf16 *ldsV = ldsK + C::kStages * C::kKElems;
  const uint32_t ldsK_addr = ASA_LDS_ADDR_OF(smem);                       // for the copies
  const uint32_t ldsV_addr = ldsK_addr + C::kStages * C::kKElems * 2;
  __shared__ uint32_t tabK[kMaxNb + C::kTabPad], tabV[kMaxNb + C::kTabPad];

  const int slot = xcd_contiguous_work(blockIdx.x, a.n_slabs * a.Nb);
  if (slot < 0) return;
  const int work = a.order ? a.order[slot] : slot;
  const int slab = work / a.Nb;
  if (slab_not_mine(a, slab)) return;
  const int qb = work - slab * a.Nb;
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = wave / C::kGroupWaves;       // 0 or 1
  const int wq = wave % C::kGroupWaves;        // which 32 query rows
  const int lane = tid & 63, hl = lane >> 5, n = lane & 31;

  const bf16 *qs = slab_ptr(a.q, a.tq, slab, a.H);
  const bf16 *ks = slab_ptr(a.k, a.tk, slab, a.H);
  const bf16 *vts = a.vt + (int64_t)slab * D * a.Lpad;
  // no index lists: dense attention, every key block in order
  const bool dense = a.row_ptr == nullptr;
  const int t_begin = dense ? 0 : a.row_ptr[slab * (a.Nb + 1) + qb];
  const int n_own_tiles = dense ? a.Nb : a.row_ptr[slab * (a.Nb + 1) + qb + 1] - t_begin;
  // global tokens: Nbg more key blocks that every query block visits, after its own list
  const int n_tiles = n_own_tiles + (GT ? a.Nbg : 0);
  const int n_steps = n_tiles * C::kSub;
  const int n_own_steps = n_own_tiles * C::kSub;
  const uint32_t pitch_bytes = (uint32_t)a.tk.sL * 2u;
  const uint32_t k_tile_bytes = BLK * pitch_bytes;     // host checked: Nb * this < 2^32
  constexpr uint32_t v_tile_bytes = D * BLK * 2;
  {
    const int32_t *g = a.col_idx + (int64_t)slab * a.Nb * a.Nb + t_begin;
    for (int t = tid; t < n_tiles + C::kTabPad; t += C::kThreads) {
      const int tc = t < n_tiles ? t : n_tiles - 1;
      if (tc < n_own_tiles) {
        const uint32_t j = dense ? (uint32_t)tc : (uint32_t)g[tc];
        tabK[t] = j * k_tile_bytes;
        tabV[t] = j * v_tile_bytes;
      } else if (n_tiles > 0) {   // pooled tile tc - n_own_tiles, rows of D elements
        tabK[t] = (uint32_t)(tc - n_own_tiles) * (BLK * D * 2);
        tabV[t] = (uint32_t)(tc - n_own_tiles) * v_tile_bytes;
      } else {
        tabK[t] = 0;
        tabV[t] = 0;
      }
    }
  }
  const int qrow = qb * BLK + wq * 32 + n;
  const bool qvalid = qrow < a.L;
  const int qrow_c = qvalid ? qrow : a.L - 1;
  bf16x8 qreg[D / 16];
#pragma unroll
  for (int s = 0; s < D / 16; ++s)
    qreg[s] = *reinterpret_cast<const bf16x8 *>(qs + (int64_t)qrow_c * a.tq.sL + 16 * s + 8 * hl);
  f32x16 oacc[D / 32];
#pragma unroll
  for (int dm = 0; dm < D / 32; ++dm)
#pragma unroll
    for (int i = 0; i < 16; ++i) oacc[dm][i] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float c = a.scale_log2e;

  // Copies: wavefront wq of the requesting group copies a quarter (BLK = 64: half) of a tile.
  RowTileCopy<C::kKT, D, C::kGroupWaves> copy_k;
  ColTileCopy<BLK, D, C::kGroupWaves> copy_v;
  copy_k.init(wq, lane, a.tk.sL);
  copy_v.init(wq, lane);
  // The first kMatrixCopies of a phase's copy requests are made by its matrix group behind its
  // last MFMA (it finishes before the vector group and would wait at the barrier), the rest by
  // the vector group between blocks of its arithmetic.
#ifndef ASA_FWD_MATRIX_COPIES
#define ASA_FWD_MATRIX_COPIES 4   // the K rows (measured 0..4: within 3 % of each other, 4 ahead by 1 %)
#endif
  constexpr int kInstrK = RowTileCopy<C::kKT, D, C::kGroupWaves>::kInstr;
  constexpr int kBatchInstr = kInstrK + ColTileCopy<BLK, D, C::kGroupWaves>::kInstr;
  constexpr int kMatrixCopies = (BLK == 128 && D == 128) ? ASA_FWD_MATRIX_COPIES : 0;
  static_assert(kBatchInstr == 4 || kBatchInstr == 8 || kBatchInstr == 16, "unexpected copy size");
  const int kr = kappa(n), cr = rho(n);
  const int kx = (hl ^ k_swz<D>(kr)) * 8, cx = (hl ^ v_swz(cr)) * 8;
  const int k_frag0 = kr * D + kx;          // element offset of my K fragment 0 in a 32-key group
  const int v_frag0 = cr * C::kKT + cx;     // of my V^T fragment 0 in a 32-channel group
  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f,
                         0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  // Only the last key block can be ragged.  Per 64-key half of a block: the table entry that
  // means "this step reaches past L" (or an impossible value if that half of the last block is
  // complete).
  const int last_row0 = (a.Nb - 1) * BLK;
  uint32_t k_tail[C::kSub], v_tail[C::kSub];
  const char *k_base[C::kSub], *v_base[C::kSub];
#pragma unroll
  for (int sb = 0; sb < C::kSub; ++sb) {
    const bool ragged = last_row0 + sb * C::kKT + C::kKT > a.L;
    k_tail[sb] = ragged ? (uint32_t)(a.Nb - 1) * k_tile_bytes : 0xFFFFFFFFu;
    v_tail[sb] = ragged ? (uint32_t)(a.Nb - 1) * v_tile_bytes : 0xFFFFFFFFu;
    k_base[sb] = reinterpret_cast<const char *>(ks) + (int64_t)sb * C::kKT * pitch_bytes;
    v_base[sb] = reinterpret_cast<const char *>(vts) + sb * C::kKT * 2;
  }
  // pooled keys / values of this slab (rows of D elements; tiles like V's)
  const char *kg_slab = reinterpret_cast<const char *>(a.kg) + (int64_t)slab * a.Nbg * BLK * D * 2;
  const char *vg_slab = reinterpret_cast<const char *>(a.vgt) + (int64_t)slab * a.Nbg * D * BLK * 2;
  // is step s one over pooled tokens?  (steps past the end repeat the last step)
  auto pooled_step = [&](int step) __attribute__((always_inline)) {
    return GT && (step < n_steps ? step : n_steps - 1) >= n_own_steps;
  };

  __syncthreads();   // tables complete
  // Before phase 0: K of steps 0, 1, 2 and V of step 0 (group 0: K(0), K(2); group 1: K(1),
  // V(0)).  Any of the K tiles may be the ragged one.
  {
    const char *kb = reinterpret_cast<const char *>(ks);
    auto k_step = [&](int step) __attribute__((always_inline)) {
      const int j = (int)(__builtin_amdgcn_readfirstlane(tabV[step / C::kSub]) / v_tile_bytes);
      const int r = j * BLK + (step % C::kSub) * C::kKT;
      if (pooled_step(step)) {
#pragma unroll
        for (int i = 0; i < kInstrK; ++i)   // (with pooled tokens the rows of K are D elements apart, like theirs)
          lds_dma16_sv(kg_slab + (int64_t)r * (D * 2), copy_k.off[i],
                       ldsK_addr + step * C::kKElems * 2 + copy_k.lds_chunk(i));
      } else {
        copy_k.issue_at_ragged(ldsK_addr + step * C::kKElems * 2, kb + (int64_t)r * pitch_bytes, a.L - 1 - r);
      }
    };
    if (grp == 0) {
      k_step(0);
      k_step(2);
    } else {
      k_step(1);
      copy_v.issue_at(ldsV_addr, (pooled_step(0) ? vg_slab : v_base[0]) + __builtin_amdgcn_readfirstlane(tabV[0]));
    }
  }
  // Table entries of the copies of phase 0 (K of step 3, V of step 1) and the V entries of the
  // three phases before, which tell the soft-max whether its step is the ragged one.
  uint32_t ek_next = tabK[3 / C::kSub], ev_next = tabV[1 / C::kSub];
  uint32_t ek_cur = 0, ev_cur = tabV[0], ev_last = 0xFFFFFFFFu, ev_older = 0xFFFFFFFFu;
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)

  f32x16 sacc[C::kKT / 32];
  uint32_t pb[(C::kKT / 32) * 8];
#pragma unroll
  for (int mt = 0; mt < C::kKT / 32; ++mt) sacc[mt] = zero16;
#pragma unroll
  for (int e = 0; e < (C::kKT / 32) * 8; ++e) pb[e] = 0;

  // Start of phase p (R = p mod 4).  During phase p, K of step p+3 and V of step p+1 are
  // requested (their buffers were last read in phase p-1); every wavefront requests the same
  // number of loads per two phases.  Data needed in phase p -- K(p), V(p-2) -- was requested
  // during phase p-3: "all of my copies but the newest kBatchInstr have landed" on every
  // wavefront, followed by the barrier, makes it visible to all.
  int phase_now = 0;   // the phase in progress, set by phase_sync
  auto phase_sync = [&](int p) __attribute__((always_inline)) {
    __builtin_amdgcn_sched_barrier(0);
    if (kBatchInstr == 4) __builtin_amdgcn_s_waitcnt(0x0F74);
    else if (kBatchInstr == 8) __builtin_amdgcn_s_waitcnt(0x0F78);
    else __builtin_amdgcn_s_waitcnt(0x4F70);   // vmcnt(16): low bits 0, high bits (15:14) 1
    asm volatile("s_barrier" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    phase_now = p;
    ek_cur = __builtin_amdgcn_readfirstlane(ek_next);
    ev_older = ev_last;
    ev_last = ev_cur;
    ev_cur = __builtin_amdgcn_readfirstlane(ev_next);
    ek_next = tabK[(p + 4) / C::kSub];
    ev_next = tabV[(p + 2) / C::kSub];
    __builtin_amdgcn_sched_barrier(0);
  };

  // The K copy of this phase: wave-uniform base and per-lane offsets.  Normally the offsets are
  // the tile's own; for the one ragged step they are bent back to the last row (rare branch).
  const char *kdma_base = nullptr, *vdma_base = nullptr;
  uint32_t kdma_off[kInstrK];
  auto dma_prepare = [&](auto r_tag) __attribute__((always_inline)) {
    constexpr int sb = (decltype(r_tag)::value + 1) % C::kSub;
    kdma_base = k_base[sb] + ek_cur;
    vdma_base = v_base[sb] + ev_cur;
#pragma unroll
    for (int i = 0; i < kInstrK; ++i) kdma_off[i] = copy_k.off[i];
    if (GT) {   // K of step p+3, V of step p+1 may be pooled tiles (rows of D elements)
      if (pooled_step(phase_now + 1)) vdma_base = vg_slab + sb * C::kKT * 2 + ev_cur;
      if (pooled_step(phase_now + 3)) {
        // the host admits pooled tokens only where K's rows are D elements apart, like theirs:
        // the per-lane offsets are the same
        kdma_base = kg_slab + sb * C::kKT * (D * 2) + ek_cur;
        return;   // pooled rows are padded to whole blocks: never ragged
      }
    }
    if (ek_cur == k_tail[sb]) {
      int lim = a.L - 1 - (last_row0 + sb * C::kKT);
      if (lim < 0) {
        kdma_base += (int64_t)lim * pitch_bytes;
        lim = 0;
      }
#pragma unroll
      for (int i = 0; i < kInstrK; ++i) {
        const int row = copy_k.row_of(i);
        if (row > lim) kdma_off[i] -= (uint32_t)(row - lim) * pitch_bytes;
      }
    }
  };
  // i-th load of this wavefront's share of the batch of phase R: K of step R+3, V of step R+1
  auto dma_one = [&](auto r_tag, int i) __attribute__((always_inline)) {
    constexpr int R = decltype(r_tag)::value;
    if (i < kInstrK)
      lds_dma16_sv<GT>(kdma_base, kdma_off[i], ldsK_addr + ((R + 3) & 3) * C::kKElems * 2 + copy_k.lds_chunk(i));
    else
      copy_v.template issue_one_at<GT>(i - kInstrK, ldsV_addr + ((R + 1) & 3) * C::kVElems * 2, vdma_base);
  };
  // (idle phases) matrix_slot: this group is the phase's matrix group
  auto dma_idle = [&](auto r_tag, bool matrix_slot) __attribute__((always_inline)) {
    const int first = matrix_slot ? 0 : kMatrixCopies, last = matrix_slot ? kMatrixCopies : kBatchInstr;
    if (first < last) {
      dma_prepare(r_tag);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < kBatchInstr; ++i)
        if (i >= first && i < last) dma_one(r_tag, i);
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  // MATRIX phase p (R = p mod 4): P V of step p-2 followed by S^T of step p.  One wavefront
  // per SIMD runs it at a time, so the LDS fragment reads are software-pipelined kDepth tile
  // products ahead of the MFMA that consumes them.  Runs at the low priority.
  constexpr int kNPv = (C::kKT / 16) * (D / 32);
  constexpr int kNS = (D / 16) * (C::kKT / 32);
  constexpr int kDepth = 6, kRing = kDepth + 1;
  auto do_matrix = [&](auto r_tag, auto with_pv, auto with_s) __attribute__((always_inline)) {
    constexpr int R = decltype(r_tag)::value;
    constexpr bool kPv = decltype(with_pv)::value, kS = decltype(with_s)::value;
    constexpr int n0 = kPv ? 0 : kNPv, n1 = kS ? kNPv + kNS : kNPv;
    const bf16 *Vs = ldsV + ((R + 2) & 3) * C::kVElems;
    const bf16 *Ks = ldsK + R * C::kKElems;
    bf16x8 ring[kRing];
    int zero = 0;
    if (GT) asm volatile("s_mov_b32 %0, 0" : "=s"(zero));
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_setprio(0);
#pragma unroll
    for (int i = n0; i < n1 + kDepth; ++i) {
      if (i < n1) {
        // fragment addresses are formed here from two per-lane bases (the swizzle is an XOR of
        // the low address bits, so (base + x) ^ (16 s) = base + (x ^ 16 s)); `zero` keeps the
        // compiler from hoisting twelve loop-invariant address registers out of the loop
        // (only the pooled-token variant, which is short of registers; the other one keeps the
        // twelve addresses in registers and saves the XORs)
        if (i < kNPv) {
          const int t = i / (D / 32), dm = i % (D / 32);
          if (GT)
            ring[i % kRing] = *reinterpret_cast<const bf16x8 *>(Vs + dm * 32 * C::kKT + ((v_frag0 ^ (16 * t)) ^ zero));
          else
            ring[i % kRing] = *reinterpret_cast<const bf16x8 *>(Vs + (dm * 32 + cr) * C::kKT + ((16 * t) ^ cx));
        } else {
          const int e = i - kNPv, sk = e / (C::kKT / 32), mt = e % (C::kKT / 32);
          if (GT)
            ring[i % kRing] = *reinterpret_cast<const bf16x8 *>(Ks + mt * 32 * D + ((k_frag0 ^ (16 * sk)) ^ zero));
          else
            ring[i % kRing] = *reinterpret_cast<const bf16x8 *>(Ks + (mt * 32 + kr) * D + ((16 * sk) ^ kx));
        }
      }
      const int c_i = i - kDepth;
      if (c_i >= n0) {
        if (c_i < kNPv) {
          const int t = c_i / (D / 32), dm = c_i % (D / 32);
          const u32x4 praw = {pb[4 * t], pb[4 * t + 1], pb[4 * t + 2], pb[4 * t + 3]};
          oacc[dm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[c_i % kRing], __builtin_bit_cast(bf16x8, praw),
                                                            oacc[dm], 0, 0, 0);
        } else {
          const int e = c_i - kNPv, sk = e / (C::kKT / 32), mt = e % (C::kKT / 32);
          sacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[c_i % kRing], qreg[sk],
                                                            sk == 0 ? zero16 : sacc[mt], 0, 0, 0);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    __builtin_amdgcn_s_setprio(3);
    if (kMatrixCopies > 0) {
      // all MFMAs of the phase are issued: this wavefront's share of the copy requests
      dma_prepare(r_tag);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < kMatrixCopies; ++i) dma_one(r_tag, i);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // VECTOR phase p: online soft-max of step p-1 (RX = that step mod 4), whose S^T is in sacc;
  // leaves bf16 P in pb.  Runs at the high priority and requests the phase's copies, an eighth
  // of them at a time between blocks of arithmetic.
  auto do_x = [&](auto rx_tag) __attribute__((always_inline)) {
    constexpr int sb = decltype(rx_tag)::value % C::kSub;
    const Int<(decltype(rx_tag)::value + 1) & 3> r_tag{};   // the phase this runs in
    constexpr int kPortion = kBatchInstr / 8 > 0 ? kBatchInstr / 8 : 1;
    int next_copy = kMatrixCopies;
    auto request = [&](int n_instr) __attribute__((always_inline)) {
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int e = 0; e < n_instr; ++e)
        if (next_copy < kBatchInstr) dma_one(r_tag, next_copy++);
      __builtin_amdgcn_sched_barrier(0);
    };
    __builtin_amdgcn_s_setprio(3);
    if (kMatrixCopies < kBatchInstr) dma_prepare(r_tag);
    float bias = 0.f;   // added to the scaled scores of pooled keys (log2 domain)
    if (GT && pooled_step(phase_now - 1)) {
      bias = a.bias_log2;
      const int key0 = (int)(ev_older / v_tile_bytes) * BLK + sb * C::kKT;
      if (key0 + C::kKT > a.Lg) {
#pragma unroll
        for (int mt = 0; mt < C::kKT / 32; ++mt)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            int key = key0 + mt * 32 + 16 * (i >> 3) + 8 * hl + (i & 7);
            if (key >= a.Lg) sacc[mt][i] = -INFINITY;
          }
      }
    } else if (ev_older == v_tail[sb]) {
      const int key0 = last_row0 + sb * C::kKT;
#pragma unroll
      for (int mt = 0; mt < C::kKT / 32; ++mt)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          int key = key0 + mt * 32 + 16 * (i >> 3) + 8 * hl + (i & 7);
          if (key >= a.L) sacc[mt][i] = -INFINITY;
        }
    }
    float mx = -INFINITY;
#pragma unroll
    for (int mt = 0; mt < C::kKT / 32; ++mt)
#pragma unroll
      for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sacc[mt][i]);
    request(kPortion);
    mx = max_of_halves(mx) * c + bias;
    if (__any(mx > m_run)) {
      const float m_new = fmaxf(m_run, mx);
      const float alpha = fast_exp2(m_run - ((m_new == -INFINITY) ? 0.f : m_new));
      m_run = m_new;
      l_run *= alpha;
#pragma unroll
      for (int dm = 0; dm < D / 32; ++dm)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[dm][i] *= alpha;
    }
    request(kPortion);
    const float m_use = ((m_run == -INFINITY) ? 0.f : m_run) - bias;
    float lsum = 0.f;
#pragma unroll
    for (int mt = 0; mt < C::kKT / 32; ++mt) {
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        if (i == 4 || i == 8 || i == 12) request(kPortion);
        const float p0 = fast_exp2(fmaf(sacc[mt][i], c, -m_use));
        const float p1 = fast_exp2(fmaf(sacc[mt][i + 1], c, -m_use));
        lsum += p0 + p1;
        pb[mt * 8 + (i >> 1)] = pack_bf16x2(p0, p1);
      }
    }
    l_run += lsum;
    request(kBatchInstr);   // whatever is left
  };

  const std::true_type yes{};
  const std::false_type no{};
  // Group g owns steps g, g+2, ...; its k-th own step is step (= phase) 2k + g.
  auto run_group = [&](auto g_tag) __attribute__((always_inline)) {
    constexpr int G = decltype(g_tag)::value;
    using R0 = Int<G>;
    using R2 = Int<(G + 2) & 3>;
    int p = 0;
    if (G == 1) { phase_sync(p); dma_idle(Int<0>{}, false); ++p; }   // group 0's matrix slot
    const int n_own = n_steps > G ? (n_steps - G + 1) / 2 : 0;
    if (n_own > 0) {
      phase_sync(p); do_matrix(R0{}, no, yes); ++p;
      phase_sync(p); do_x(R0{}); ++p;
      int k = 1;
      for (; k + 1 < n_own; k += 2) {
        phase_sync(p); do_matrix(R2{}, yes, yes); ++p;
        phase_sync(p); do_x(R2{}); ++p;
        phase_sync(p); do_matrix(R0{}, yes, yes); ++p;
        phase_sync(p); do_x(R0{}); ++p;
      }
      if (k < n_own) {
        phase_sync(p); do_matrix(R2{}, yes, yes); ++p;
        phase_sync(p); do_x(R2{}); ++p;
        phase_sync(p); do_matrix(R0{}, yes, no); ++p;
      } else {
        phase_sync(p); do_matrix(R2{}, yes, no); ++p;
      }
    }
    // the other group may still have phases to run: keep the barriers and copies in step
    for (; p < n_steps + 2; ++p) {
      switch (p & 3) {
        case 0: phase_sync(p); dma_idle(Int<0>{}, G == 0); break;
        case 1: phase_sync(p); dma_idle(Int<1>{}, G == 1); break;
        case 2: phase_sync(p); dma_idle(Int<2>{}, G == 0); break;
        default: phase_sync(p); dma_idle(Int<3>{}, G == 1); break;
      }
    }
  };
  if (grp == 0) run_group(Int<0>{});
  else run_group(Int<1>{});

  // ---- merge the two groups' partials (group 1 -> LDS -> group 0), then write out
  __builtin_amdgcn_s_waitcnt(0x0F70);   // stray copies must land before the buffers are reused
  __syncthreads();
  f32x4 *xbuf = reinterpret_cast<f32x4 *>(smem);          // [4 * D/32][BLK * 2] f32x4
  float *xm = reinterpret_cast<float *>(xbuf + 4 * (D / 32) * (BLK * 2));
  float *xl = xm + BLK * 2;
  const int xslot = wq * 64 + lane;
  float l_half = l_run + swap_halves(l_run);
  if (grp == 1) {
#pragma unroll
    for (int dm = 0; dm < D / 32; ++dm)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        f32x4 v = {oacc[dm][4 * q4], oacc[dm][4 * q4 + 1], oacc[dm][4 * q4 + 2], oacc[dm][4 * q4 + 3]};
        xbuf[(dm * 4 + q4) * (BLK * 2) + xslot] = v;
      }
    xm[xslot] = m_run;
    xl[xslot] = l_half;
  }
  __syncthreads();
  if (grp == 1) return;
  {
    const float m_o = xm[xslot], l_o = xl[xslot];
    const float m_all = fmaxf(m_run, m_o);
    const float ms = (m_all == -INFINITY) ? 0.f : m_all;
    const float fa = fast_exp2(m_run - ms), fb = fast_exp2(m_o - ms);
    l_half = l_half * fa + l_o * fb;
#pragma unroll
    for (int dm = 0; dm < D / 32; ++dm)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const f32x4 v = xbuf[(dm * 4 + q4) * (BLK * 2) + xslot];
#pragma unroll
        for (int e = 0; e < 4; ++e) oacc[dm][4 * q4 + e] = oacc[dm][4 * q4 + e] * fa + v[e] * fb;
      }
    m_run = m_all;
  }
  const float l_tot = l_half;
  const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
  if (qvalid) {
    bf16 *os = slab_ptr(a.o, a.to, slab, a.H) + (int64_t)qrow * a.to.sL;
    bf16 *ls = a.o_lo ? slab_ptr(a.o_lo, a.to, slab, a.H) + (int64_t)qrow * a.to.sL : nullptr;
#pragma unroll
    for (int dm = 0; dm < D / 32; ++dm) {
      uint32_t w[8], r[8];
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        const float v0 = oacc[dm][i] * inv, v1 = oacc[dm][i + 1] * inv;
        const uint32_t pk = pack_bf16x2(v0, v1);
        w[i >> 1] = pk;
        r[i >> 1] = pack_bf16x2(v0 - bf16_bits_to_float(pk & 0xffffu),
                                v1 - bf16_bits_to_float(pk >> 16));
      }
      uint4 *dst = reinterpret_cast<uint4 *>(os + dm * 32 + 16 * hl);
      dst[0] = make_uint4(w[0], w[1], w[2], w[3]);
      dst[1] = make_uint4(w[4], w[5], w[6], w[7]);
      if (ls) {
        uint4 *dl = reinterpret_cast<uint4 *>(ls + dm * 32 + 16 * hl);
        dl[0] = make_uint4(r[0], r[1], r[2], r[3]);
        dl[1] = make_uint4(r[4], r[5], r[6], r[7]);
      }
    }
    if (hl == 0)
      a.lse[(int64_t)slab * a.L + qrow] =
          l_tot > 0.f ? m_run * 0.69314718055994530942f + __logf(l_tot) : -INFINITY;
  }
}

template <int BLK, int D>
static hipError_t launch_fwd_t(const FwdArgs &a, hipStream_t st) {
  using C = FwdCfg<BLK, D>;
  using P = PpCfg<BLK, D>;
  constexpr int lds = C::kStages * (C::kKElems + C::kVElems) * 2;
  const int grid = xcd_grid(a.n_slabs * a.Nb);
  // The ping-pong kernel is the faster one at block = 128, d = 128 (998 vs 914 TFLOP/s at the Wan
  // shape); with smaller blocks or heads its workgroup has too few wavefronts per SIMD or too
  // little work per phase and the lock-step kernel wins (e.g. 761 vs 511 TFLOP/s at block 64,
  // d 128).  It addresses K tiles by 32-bit byte offsets inside a slab, so slabs of 4 GiB and
  // more also take the lock-step kernel.  Global tokens exist in the ping-pong kernel only.
  // The tests can force one or the other (asa_test_force_fwd_kernel).
  const bool fits32 = (uint64_t)a.Nb * BLK * (uint64_t)a.tk.sL * 2u < 0xFFFFFFFFull;
  if (a.Nbg > 0 && (!fits32 || a.Nb + a.Nbg > kMaxNb || a.tk.sL != D)) return hipErrorNotSupported;
  const int forced = forced_fwd_kernel();
  const bool prefer_pp = forced == 2 || (forced == 0 && BLK == 128 && D == 128);
  FwdArgs b = a;
  b.select = 0;
  hipError_t e = hipSuccess;
  // Short lists: the ping-pong kernel costs ~8 us per workgroup around its steady state, the
  // lock-step kernel ~3 us; they cross at 16-20 tiles per row.  The host cannot see the lists, so
  // with lists BOTH kernels are launched and each workgroup leaves at once if its (batch, head)
  // slab's tile count belongs to the other kernel (the launch that finds nothing to do costs
  // 4-10 us).  Without lists (dense) every row holds Nb tiles and the choice is made here.
  constexpr int kPingPongMinTiles = 18;
  b.select_min_tiles = kPingPongMinTiles;
  const bool dense_short = !a.row_ptr && a.Nbg == 0 && a.Nb < kPingPongMinTiles && forced == 0;
  if (fits32 && (a.Nbg > 0 || prefer_pp) && !dense_short) {
    const bool both = a.Nbg == 0 && a.row_ptr && forced == 0;
    if (both) b.select = 1;
    const void *fn = a.Nbg > 0 ? reinterpret_cast<const void *>(&fwd_pp_kernel<BLK, D, true>)
                               : reinterpret_cast<const void *>(&fwd_pp_kernel<BLK, D, false>);
    e = set_dynamic_lds_once(fn, P::kLdsBytes);
    if (e != hipSuccess) return e;
    if (a.Nbg > 0)
      hipLaunchKernelGGL((fwd_pp_kernel<BLK, D, true>), dim3(grid), dim3(P::kThreads), P::kLdsBytes, st, b);
    else
      hipLaunchKernelGGL((fwd_pp_kernel<BLK, D, false>), dim3(grid), dim3(P::kThreads), P::kLdsBytes, st, b);
    e = hipGetLastError();
    if (e != hipSuccess || !both) return e;
    b.select = -1;
  }
  e = set_dynamic_lds_once(reinterpret_cast<const void *>(&fwd_kernel<BLK, D>), lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((fwd_kernel<BLK, D>), dim3(grid), dim3(C::kThreads), lds, st, b);
  return hipGetLastError();
}

hipError_t launch_fwd(const Problem &pb, const void *q, const void *k, const void *vt,
                      const int32_t *row_ptr, const int32_t *col_idx, void *o, void *o_lo,
                      float *lse, const int32_t *order, hipStream_t st, const GlobalTokens *gt) {
  FwdArgs a;
  a.order = order;
  a.kg = gt ? gt->kg : nullptr;
  a.vgt = gt ? reinterpret_cast<const bf16 *>(gt->vgt) : nullptr;
  a.Lg = gt ? gt->Lg : 0;
  a.Nbg = gt ? gt->Nbg : 0;
  a.bias_log2 = gt ? log2f((float)gt->n) : 0.f;
  a.q = q; a.k = k; a.vt = reinterpret_cast<const bf16 *>(vt);
  a.row_ptr = row_ptr; a.col_idx = col_idx; a.o = o; a.o_lo = o_lo; a.lse = lse;
  a.tq = pb.q; a.tk = pb.k; a.to = pb.o;
  a.H = pb.H; a.L = pb.L; a.Lpad = pb.Lpad; a.Nb = pb.Nb; a.n_slabs = pb.n_slabs;
  a.scale_log2e = pb.scale * 1.44269504088896340736f;
  a.select = 0;
  a.select_min_tiles = 0;
  if (pb.block == 128 && pb.d == 128) return launch_fwd_t<128, 128>(a, st);
  if (pb.block == 128 && pb.d == 64) return launch_fwd_t<128, 64>(a, st);
  if (pb.block == 64 && pb.d == 128) return launch_fwd_t<64, 128>(a, st);
  if (pb.block == 64 && pb.d == 64) return launch_fwd_t<64, 64>(a, st);
  return hipErrorInvalidValue;
}

}  // namespace asa
