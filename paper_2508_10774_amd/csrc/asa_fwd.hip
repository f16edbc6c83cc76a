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
};

template <int BLK, int D>
struct FwdCfg {
  static constexpr int kWaves = BLK / 32;
  static constexpr int kThreads = kWaves * 64;
  static constexpr int kKT = 64;                   // keys per pipeline step
  static constexpr int kSub = BLK / kKT;           // steps per key block
  static constexpr int kKElems = kKT * D;          // one K stage:   [64 keys][D]  (unpadded)
  static constexpr int kVElems = D * kKT;          // one V^T stage: [D][64 keys]  (unpadded)
};

// The running maximum (and with it O and the row sum) is rescaled only on steps where some row
// of the wavefront actually found a larger logit; on all other steps the factor would be 1.
// The maximum is never allowed to lag behind: a row dominated by one key then has that key's
// probability equal to exactly 1, free of bf16 rounding, which the backward's Delta relies on.
//
// PREFETCH = false: one LDS stage (32 KB at d = 128); the copies of a step are waited for right
// away and the second workgroup on the CU computes meanwhile.  PREFETCH = true: two stages, the
// next step's tiles are requested before the current step is computed.  Both were measured;
// the single-stage form is the faster one on MI355X and is the one that is launched.
template <int BLK, int D, bool PREFETCH>
__global__ __launch_bounds__(BLK * 2, 2) void fwd_kernel(FwdArgs a) {
  using C = FwdCfg<BLK, D>;
  extern __shared__ __align__(1024) unsigned char smem[];
  bf16 *lds = reinterpret_cast<bf16 *>(smem);
  constexpr int kStage = C::kKElems + C::kVElems;
  __shared__ int cols[kMaxNb];

  const int work = xcd_contiguous_work(blockIdx.x, a.n_slabs * a.Nb);
  if (work < 0) return;
  const int slab = work / a.Nb;
  const int qb = work - slab * a.Nb;
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63, hl = lane >> 5, n = lane & 31;

  const bf16 *qs = slab_ptr(a.q, a.tq, slab, a.H);
  const bf16 *ks = slab_ptr(a.k, a.tk, slab, a.H);
  const bf16 *vts = a.vt + (int64_t)slab * D * a.Lpad;
  const int t_begin = a.row_ptr[slab * (a.Nb + 1) + qb];
  const int n_tiles = a.row_ptr[slab * (a.Nb + 1) + qb + 1] - t_begin;
  {
    const int32_t *g = a.col_idx + (int64_t)slab * a.Nb * a.Nb + t_begin;
    for (int t = tid; t < n_tiles; t += C::kThreads) cols[t] = g[t];
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
  auto fetch = [&](int step, int stage) __attribute__((always_inline)) {
    const int j = cols[step / C::kSub];
    const int sub = step % C::kSub;
    bf16 *Kd = lds + stage * kStage;
    copy_k.issue(Kd, ks, j * BLK + sub * C::kKT, a.L);
    copy_v.issue(Kd + C::kKElems, vts + (int64_t)j * D * BLK, sub * C::kKT);
  };
  __syncthreads();   // cols[] is complete
  if (PREFETCH && n_steps > 0) fetch(0, 0);
  for (int step = 0; step < n_steps; ++step) {
    const int stage = PREFETCH ? (step & 1) : 0;
    if (PREFETCH) {
      __builtin_amdgcn_s_waitcnt(0x0F70);   // my copies of this step have landed
      __syncthreads();                      // everyone's have; the other stage is free
      if (step + 1 < n_steps) fetch(step + 1, stage ^ 1);
    } else {
      __syncthreads();
      fetch(step, 0);
      __builtin_amdgcn_s_waitcnt(0x0F70);
      __syncthreads();
    }
    const bf16 *Ks = lds + stage * kStage;
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

template <int BLK, int D>
static hipError_t launch_fwd_t(const FwdArgs &a, hipStream_t st) {
  using C = FwdCfg<BLK, D>;
  constexpr int lds = (C::kKElems + C::kVElems) * 2;   // one stage
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&fwd_kernel<BLK, D, false>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  int grid = xcd_grid(a.n_slabs * a.Nb);
  hipLaunchKernelGGL((fwd_kernel<BLK, D, false>), dim3(grid), dim3(C::kThreads), lds, st, a);
  return hipGetLastError();
}

hipError_t launch_fwd(const Problem &pb, const void *q, const void *k, const void *vt,
                      const int32_t *row_ptr, const int32_t *col_idx, void *o, void *o_lo,
                      float *lse, hipStream_t st) {
  FwdArgs a;
  a.q = q; a.k = k; a.vt = reinterpret_cast<const bf16 *>(vt);
  a.row_ptr = row_ptr; a.col_idx = col_idx; a.o = o; a.o_lo = o_lo; a.lse = lse;
  a.tq = pb.q; a.tk = pb.k; a.to = pb.o;
  a.H = pb.H; a.L = pb.L; a.Lpad = pb.Lpad; a.Nb = pb.Nb; a.n_slabs = pb.n_slabs;
  a.scale_log2e = pb.scale * 1.44269504088896340736f;
  if (pb.block == 128 && pb.d == 128) return launch_fwd_t<128, 128>(a, st);
  if (pb.block == 128 && pb.d == 64) return launch_fwd_t<128, 64>(a, st);
  if (pb.block == 64 && pb.d == 128) return launch_fwd_t<64, 128>(a, st);
  if (pb.block == 64 && pb.d == 64) return launch_fwd_t<64, 64>(a, st);
  return hipErrorInvalidValue;
}

}  // namespace asa
