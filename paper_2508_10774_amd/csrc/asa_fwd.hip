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
//                    kappa below; V is consumed from a [d][L] copy so that both LDS
//                    operand reads are 16-byte loads.
// K and V^T tiles go through LDS with 16 bytes of row padding (conflict-free b128 reads).
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
  static constexpr int kLdsBytes = 2 * (kKElems + kVElems) * 2;
  // direct-to-LDS copies move 1 KB (64 lanes x 16 B) per wavefront instruction
  static constexpr int kKInstr = kKElems * 2 / 1024 / kWaves;
  static constexpr int kVInstr = kVElems * 2 / 1024 / kWaves;
  static constexpr int kKChunkBits = (D == 128) ? 4 : 3;   // log2(16-byte chunks per K row)
};

// The running maximum (and with it O and the row sum) is rescaled only on steps where some row
// of the wavefront actually found a larger logit; on all other steps the factor would be 1.
// The maximum is never allowed to lag behind: a row dominated by one key then has that key's
// probability equal to exactly 1, free of bf16 rounding, which the backward's Delta relies on.

template <int BLK, int D>
__global__ __launch_bounds__(BLK * 2, 2) void fwd_kernel(FwdArgs a) {
  using C = FwdCfg<BLK, D>;
  extern __shared__ __align__(1024) unsigned char smem[];
  bf16 *ldsK = reinterpret_cast<bf16 *>(smem);          // 2 stages
  bf16 *ldsV = ldsK + 2 * C::kKElems;                   // 2 stages

  const int work = xcd_contiguous_work(blockIdx.x, a.n_slabs * a.Nb);
  if (work < 0) return;
  const int slab = work / a.Nb;
  const int qb = work - slab * a.Nb;

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, kept in an SGPR
  const int lane = tid & 63;
  const int hl = lane >> 5;  // which 32-lane half
  const int n = lane & 31;   // query within the wave / A row within an M tile

  const bf16 *qs = slab_ptr(a.q, a.tq, slab, a.H);
  const bf16 *ks = slab_ptr(a.k, a.tk, slab, a.H);
  const bf16 *vts = a.vt + (int64_t)slab * D * a.Lpad;
  const int t_begin = a.row_ptr[slab * (a.Nb + 1) + qb];
  const int n_tiles = a.row_ptr[slab * (a.Nb + 1) + qb + 1] - t_begin;
  const int n_steps = n_tiles * C::kSub;

  // The row's list of kept key blocks goes to LDS once: reading it from global memory inside
  // the loop would put a vector-memory wait in front of every step, and such a wait also waits
  // for all direct-to-LDS tile loads issued before it.
  __shared__ int cols[kMaxNb];
  {
    const int32_t *gcols = a.col_idx + (int64_t)slab * a.Nb * a.Nb + t_begin;
    for (int t = tid; t < n_tiles; t += C::kThreads) cols[t] = gcols[t];
  }
  __syncthreads();

  const int qrow = qb * BLK + wave * 32 + n;
  const bool qvalid = qrow < a.L;
  const int qrow_c = qvalid ? qrow : a.L - 1;

  // Q^T as the B operand of S^T: lane (hl, n) holds Q[qrow][16s + 8hl .. +8]
  bf16x8 qreg[D / 16];
#pragma unroll
  for (int s = 0; s < D / 16; ++s)
    qreg[s] = *reinterpret_cast<const bf16x8 *>(qs + (int64_t)qrow_c * a.tq.sL + 16 * s + 8 * hl);

  f32x16 oacc[D / 32];
#pragma unroll
  for (int dm = 0; dm < D / 32; ++dm)
#pragma unroll
    for (int i = 0; i < 16; ++i) oacc[dm][i] = 0.f;
  float m_run = -INFINITY;  // running maximum, log2 domain
  float l_run = 0.f;        // running sum of this lane half, relative to m_run
  const float c = a.scale_log2e;

  // ---- producers: this lane's share of a K stage / V^T stage, fetched straight into LDS.
  // Per-lane byte offsets are fixed for the whole kernel; per step only a wave-uniform base
  // pointer changes, so a load costs no vector ALU work.
  constexpr int KCH = D / 8;   // chunks per K row
  uint32_t k_off[C::kKInstr];  // byte offset of my chunk inside a K step, per instruction
  uint32_t v_off[C::kVInstr];
#pragma unroll
  for (int i = 0; i < C::kKInstr; ++i) {
    const int seg = wave * C::kKInstr + i;            // 1 KB LDS segment = 64 chunks
    const int row = seg * (64 / KCH) + lane / KCH;    // key row inside the stage
    const int pos = lane % KCH;                       // chunk position inside the row
    k_off[i] = (uint32_t)(((int64_t)row * a.tk.sL + ((pos ^ k_swz<D>(row)) * 8)) * 2);
  }
#pragma unroll
  for (int i = 0; i < C::kVInstr; ++i) {
    const int seg = wave * C::kVInstr + i;
    const int row = seg * 8 + lane / 8;               // channel row inside the stage
    v_off[i] = (uint32_t)((row * BLK + (((lane % 8) ^ v_swz(row)) * 8)) * 2);
  }
  auto fetch_k = [&](int step, int stage_idx) __attribute__((always_inline)) {
    const int key0 = cols[step / C::kSub] * BLK + (step % C::kSub) * C::kKT;
    bf16 *stage = ldsK + stage_idx * C::kKElems;
    const char *base = reinterpret_cast<const char *>(ks + (int64_t)key0 * a.tk.sL);
    const int lim = a.L - 1 - key0;                    // last valid row of this step
    if (lim >= C::kKT - 1) {
#pragma unroll
      for (int i = 0; i < C::kKInstr; ++i)
        lds_dma16(base + k_off[i], stage + (wave * C::kKInstr + i) * 512);
    } else {                                           // tail block: re-read the last real row
#pragma unroll
      for (int i = 0; i < C::kKInstr; ++i) {
        const char *src = base + k_off[i];
        const int row = (wave * C::kKInstr + i) * (64 / KCH) + lane / KCH;
        if (row > lim) src -= (int64_t)(row - lim) * a.tk.sL * 2;
        lds_dma16(src, stage + (wave * C::kKInstr + i) * 512);
      }
    }
  };
  auto fetch_v = [&](int step, int stage_idx) __attribute__((always_inline)) {
    const char *vtile = reinterpret_cast<const char *>(
        vts + (int64_t)cols[step / C::kSub] * D * BLK + (step % C::kSub) * C::kKT);
    bf16 *stage = ldsV + stage_idx * C::kVElems;
#pragma unroll
    for (int i = 0; i < C::kVInstr; ++i)
      lds_dma16(vtile + v_off[i], stage + (wave * C::kVInstr + i) * 512);
  };

  // ---- consumers: LDS addresses of this lane's MFMA A fragments (stage 0, M tile 0)
  // K fragment of k-step s: row kappa(n), chunk (2s + hl) ^ swizzle = (2s) ^ (hl ^ swizzle)
  const int kx = (hl ^ k_swz<D>(kappa(n))) * 8;
  const bf16 *k_frag[D / 16];
#pragma unroll
  for (int s = 0; s < D / 16; ++s) k_frag[s] = ldsK + kappa(n) * D + ((16 * s) ^ kx);
  // V^T fragment of 16-key step t: row rho(n), chunk (2t + hl) ^ swizzle
  const int vx = (hl ^ v_swz(rho(n))) * 8;
  const bf16 *v_frag[C::kKT / 16];
#pragma unroll
  for (int t = 0; t < C::kKT / 16; ++t) v_frag[t] = ldsV + rho(n) * C::kKT + ((16 * t) ^ vx);

  constexpr int NS = (C::kKT / 32) * (D / 16);   // MFMAs of one S^T step   (16 at D = 128)
  constexpr int NP = (C::kKT / 16) * (D / 32);   // MFMAs of one P V step   (16 at D = 128)
  constexpr int NE = (C::kKT / 32) * 8;          // probability pairs per lane and step (16)
  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f,
                         0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  // row maximum (log2 domain, both lane halves merged) of a finished S^T step
  auto row_max = [&](const f32x16 (&sv)[C::kKT / 32]) __attribute__((always_inline)) {
    float mx = -INFINITY;
#pragma unroll
    for (int mt = 0; mt < C::kKT / 32; ++mt)
#pragma unroll
      for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sv[mt][i]);
    return fmaxf(mx, swap_halves(mx)) * c;
  };
  // keys >= L do not exist (partial last key block)
  auto mask_tail = [&](int step, f32x16 (&sv)[C::kKT / 32]) __attribute__((always_inline)) {
    const int key0 = cols[step / C::kSub] * BLK + (step % C::kSub) * C::kKT;
    if (key0 + C::kKT > a.L) {
#pragma unroll
      for (int mt = 0; mt < C::kKT / 32; ++mt)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          int key = key0 + mt * 32 + 16 * (i >> 3) + 8 * hl + (i & 7);
          if (key >= a.L) sv[mt][i] = -INFINITY;
        }
    }
  };

  if (n_steps > 0) {
    fetch_k(0, 0);
    fetch_v(0, 0);
    if (n_steps > 1) fetch_k(1, 1);
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): my direct loads have landed
  __syncthreads();

  // S^T of step 0 (not overlapped with anything) and its row maximum
  f32x16 s_a[C::kKT / 32], s_b[C::kKT / 32];
  float mx_cur = -INFINITY;
  if (n_steps > 0) {
#pragma unroll
    for (int mt = 0; mt < C::kKT / 32; ++mt) {
      s_a[mt] = zero16;
#pragma unroll
      for (int s = 0; s < D / 16; ++s) {
        bf16x8 ka = *reinterpret_cast<const bf16x8 *>(k_frag[s] + mt * 32 * D);
        s_a[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[s], s_a[mt], 0, 0, 0);
      }
    }
    mask_tail(0, s_a);
    mx_cur = row_max(s_a);
  }

  // One pipeline step, software-pipelined across steps and scheduled by hand in "slices" of
  // one MFMA each, so that the matrix pipe and the VALU run side by side within a wavefront:
  //   phase 1: S^T of step+1 (MFMA)  ||  exp2 / sum / bf16 packing of step (VALU)
  //   phase 2: P V of step   (MFMA)  ||  nothing much; then the row maximum of step+1
  // LDS fragments are requested two slices ahead of the MFMA that consumes them.  PAR is the
  // parity of `step` (the loop is unrolled by two so that LDS stage offsets are immediates
  // and the two S^T register sets swap roles without copies).
  auto body = [&](auto par_tag, int step, f32x16 (&s_cur)[C::kKT / 32],
                  f32x16 (&s_nxt)[C::kKT / 32]) __attribute__((always_inline)) {
    constexpr int PAR = decltype(par_tag)::value;
    // everyone is past S(step) (reads K stage PAR) and past PV(step-1) (V stage 1-PAR), and
    // every wave's loads of K(step+1), V(step) have landed
    __syncthreads();
    if (step + 2 < n_steps) fetch_k(step + 2, PAR);
    if (step + 1 < n_steps) fetch_v(step + 1, 1 - PAR);

    // ---- raise the running maximum only if some row of the wavefront found a larger logit
    if (__any(mx_cur > m_run)) {
      const float m_new = fmaxf(m_run, mx_cur);
      const float alpha = fast_exp2(m_run - ((m_new == -INFINITY) ? 0.f : m_new));
      m_run = m_new;
      l_run *= alpha;
#pragma unroll
      for (int dm = 0; dm < D / 32; ++dm)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[dm][i] *= alpha;
    }
    const float m_use = (m_run == -INFINITY) ? 0.f : m_run;

    constexpr int k_stage = (1 - PAR) * C::kKElems;   // K(step+1)
    constexpr int v_stage = PAR * C::kVElems;         // V(step)
    uint32_t pb[NE];
    float lsum = 0.f;

    // ---- phase 1
    __builtin_amdgcn_sched_barrier(0);
    {
      bf16x8 kf[3];
      auto kread = [&](int sl) __attribute__((always_inline)) {
        return *reinterpret_cast<const bf16x8 *>(k_frag[sl / (C::kKT / 32)] + k_stage +
                                                 (sl % (C::kKT / 32)) * 32 * D);
      };
      kf[0] = kread(0);
      kf[1] = kread(1);
#pragma unroll
      for (int sl = 0; sl < NS; ++sl) {
        if (sl + 2 < NS) kf[(sl + 2) % 3] = kread(sl + 2);
        const int mt = sl % (C::kKT / 32), ks = sl / (C::kKT / 32);
        s_nxt[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[sl % 3], qreg[ks],
                                                            ks == 0 ? zero16 : s_nxt[mt], 0, 0, 0);
        // VALU share of this slice: NE pairs spread over NS slices
#pragma unroll
        for (int e = sl * NE / NS; e < (sl + 1) * NE / NS; ++e) {
          const int emt = e / 8, ei = (e % 8) * 2;
          const float p0 = fast_exp2(fmaf(s_cur[emt][ei], c, -m_use));
          const float p1 = fast_exp2(fmaf(s_cur[emt][ei + 1], c, -m_use));
          lsum += p0 + p1;   // unrounded: LSE must not inherit a dominant key's bf16 rounding
          pb[e] = pack_bf16x2(p0, p1);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    l_run += lsum;

    // ---- phase 2
    {
      bf16x8 vf[3];
      auto vread = [&](int sl) __attribute__((always_inline)) {
        return *reinterpret_cast<const bf16x8 *>(v_frag[sl / (D / 32)] + v_stage +
                                                 (sl % (D / 32)) * 32 * C::kKT);
      };
      vf[0] = vread(0);
      vf[1] = vread(1);
#pragma unroll
      for (int sl = 0; sl < NP; ++sl) {
        if (sl + 2 < NP) vf[(sl + 2) % 3] = vread(sl + 2);
        const int dm = sl % (D / 32), t = sl / (D / 32);
        uint4 praw = make_uint4(pb[4 * t], pb[4 * t + 1], pb[4 * t + 2], pb[4 * t + 3]);
        oacc[dm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
            vf[sl % 3], *reinterpret_cast<bf16x8 *>(&praw), oacc[dm], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    // row maximum of the next step (its S^T finished during phase 1; past the last step the
    // values come from a stale stage and are dropped)
    if (step + 1 < n_steps) {
      mask_tail(step + 1, s_nxt);
      mx_cur = row_max(s_nxt);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0) before the barrier that publishes my loads
  };

  for (int step = 0; step < n_steps; step += 2) {
    body(std::integral_constant<int, 0>{}, step, s_a, s_b);
    if (step + 1 < n_steps) body(std::integral_constant<int, 1>{}, step + 1, s_b, s_a);
  }

  // ---- epilogue
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
        // what the rounding to bf16 dropped, itself rounded to bf16
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
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&fwd_kernel<BLK, D>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, C::kLdsBytes);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  int grid = xcd_grid(a.n_slabs * a.Nb);
  hipLaunchKernelGGL((fwd_kernel<BLK, D>), dim3(grid), dim3(C::kThreads), C::kLdsBytes, st, a);
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
