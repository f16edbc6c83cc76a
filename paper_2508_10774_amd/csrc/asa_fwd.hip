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
#include "asa_common.hpp"

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
  static constexpr int kKStride = D + 8;    // bf16 per K row in LDS
  static constexpr int kVStride = BLK + 8;  // bf16 per V^T row in LDS
  static constexpr int kLdsBytes = (BLK * kKStride + D * kVStride) * 2;
};

// Row r of an MFMA A operand / accumulator splits as r = 8g + 4h + j (g<4, h<2, j<4); lane
// half h holds accumulator register 4g + j.
//
// kappa: which key of a 32-key group is loaded as A row r of S^T = K Q^T.  Chosen so that
// lane half h, registers 8t..8t+7 hold keys 16t + 8h + 0..7: exactly the 8 consecutive k
// slots that the B operand of the following 16-deep P^T step wants from that lane.
__device__ __forceinline__ int kappa(int r) {
  int g = r >> 3, h = (r >> 2) & 1, j = r & 3;
  return 16 * (g >> 1) + 8 * h + 4 * (g & 1) + j;
}
// rho: which channel of a 32-channel group is loaded as A row r of O^T = V^T P^T, chosen so
// that lane half h ends up with 16 consecutive channels 16h + (4g + j) of its query.
__device__ __forceinline__ int rho(int r) {
  int g = r >> 3, h = (r >> 2) & 1, j = r & 3;
  return 16 * h + 4 * g + j;
}

template <int BLK, int D>
__global__ __launch_bounds__(BLK * 2, 2) void fwd_kernel(FwdArgs a) {
  using C = FwdCfg<BLK, D>;
  extern __shared__ __align__(16) unsigned char smem[];
  bf16 *Ks = reinterpret_cast<bf16 *>(smem);
  bf16 *Vs = Ks + BLK * C::kKStride;

  const int work = xcd_contiguous_work(blockIdx.x, a.n_slabs * a.Nb);
  if (work < 0) return;
  const int slab = work / a.Nb;
  const int qb = work - slab * a.Nb;

  const int tid = threadIdx.x;
  const int wave = tid >> 6;
  const int lane = tid & 63;
  const int hl = lane >> 5;  // which 32-lane half
  const int n = lane & 31;   // query within the wave / A row within an M tile

  const bf16 *qs = slab_ptr(a.q, a.tq, slab, a.H);
  const bf16 *ks = slab_ptr(a.k, a.tk, slab, a.H);
  const bf16 *vts = a.vt + (int64_t)slab * D * a.Lpad;
  const int32_t *cols = a.col_idx + (int64_t)slab * a.Nb * a.Nb;
  const int t_begin = a.row_ptr[slab * (a.Nb + 1) + qb];
  const int t_end = a.row_ptr[slab * (a.Nb + 1) + qb + 1];

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
  float l_run = 0.f;        // running sum of this lane half

  const int k_row_off = kappa(n) * C::kKStride + 8 * hl;
  const int v_row_off = rho(n) * C::kVStride + 8 * hl;
  const float c = a.scale_log2e;

  for (int t = t_begin; t < t_end; ++t) {
    const int j = cols[t];
    __syncthreads();  // everyone is done with the previous tile
    {
      constexpr int CH = D / 8;
#pragma unroll
      for (int i = 0; i < BLK * CH / C::kThreads; ++i) {
        int cidx = tid + i * C::kThreads;
        int r = cidx / CH, cc = cidx % CH;
        int krow = j * BLK + r;
        krow = krow < a.L ? krow : a.L - 1;
        uint4 val = *reinterpret_cast<const uint4 *>(ks + (int64_t)krow * a.tk.sL + cc * 8);
        *reinterpret_cast<uint4 *>(Ks + r * C::kKStride + cc * 8) = val;
      }
      constexpr int CV = BLK / 8;
#pragma unroll
      for (int i = 0; i < D * CV / C::kThreads; ++i) {
        int cidx = tid + i * C::kThreads;
        int r = cidx / CV, cc = cidx % CV;
        uint4 val =
            *reinterpret_cast<const uint4 *>(vts + ((int64_t)j * D + r) * BLK + cc * 8);
        *reinterpret_cast<uint4 *>(Vs + r * C::kVStride + cc * 8) = val;
      }
    }
    __syncthreads();

    // ---- S^T = K Q^T
    f32x16 sacc[BLK / 32];
#pragma unroll
    for (int mt = 0; mt < BLK / 32; ++mt) {
#pragma unroll
      for (int i = 0; i < 16; ++i) sacc[mt][i] = 0.f;
#pragma unroll
      for (int s = 0; s < D / 16; ++s) {
        bf16x8 ka = *reinterpret_cast<const bf16x8 *>(Ks + mt * 32 * C::kKStride + k_row_off + 16 * s);
        sacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[s], sacc[mt], 0, 0, 0);
      }
    }

    // ---- online soft-max over this tile (one query per lane, 16*BLK/32 keys per lane half)
    if (j * BLK + BLK > a.L) {  // partial last key block: keys >= L do not exist
#pragma unroll
      for (int mt = 0; mt < BLK / 32; ++mt)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          int key = j * BLK + mt * 32 + 16 * (i >> 3) + 8 * hl + (i & 7);
          if (key >= a.L) sacc[mt][i] = -INFINITY;
        }
    }
    float mx = -INFINITY;
#pragma unroll
    for (int mt = 0; mt < BLK / 32; ++mt)
#pragma unroll
      for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sacc[mt][i]);
    mx = fmaxf(mx, swap_halves(mx));
    const float m_new = fmaxf(m_run, mx * c);
    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = fast_exp2(m_run - m_use);
    m_run = m_new;

    uint32_t pb[BLK / 32][8];
    float lsum = 0.f;
#pragma unroll
    for (int mt = 0; mt < BLK / 32; ++mt)
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        float p0 = fast_exp2(fmaf(sacc[mt][i], c, -m_use));
        float p1 = fast_exp2(fmaf(sacc[mt][i + 1], c, -m_use));
        lsum += p0 + p1;
        pb[mt][i >> 1] = pack_bf16x2(p0, p1);
      }
    l_run = l_run * alpha + lsum;
#pragma unroll
    for (int dm = 0; dm < D / 32; ++dm)
#pragma unroll
      for (int i = 0; i < 16; ++i) oacc[dm][i] *= alpha;

    // ---- O^T += V^T P^T
#pragma unroll
    for (int mt = 0; mt < BLK / 32; ++mt)
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        uint4 praw = make_uint4(pb[mt][4 * tt], pb[mt][4 * tt + 1], pb[mt][4 * tt + 2],
                                pb[mt][4 * tt + 3]);
        bf16x8 pfrag = *reinterpret_cast<bf16x8 *>(&praw);
#pragma unroll
        for (int dm = 0; dm < D / 32; ++dm) {
          bf16x8 va = *reinterpret_cast<const bf16x8 *>(Vs + dm * 32 * C::kVStride + v_row_off +
                                                        16 * (2 * mt + tt));
          oacc[dm] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pfrag, oacc[dm], 0, 0, 0);
        }
      }
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
