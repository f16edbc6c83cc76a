// Mask generation for gfx950: block importance map (Alg. 2 -> Alg. 1 of the paper's appendix),
// the threshold rule (Alg. 3 steps 6-11) and the CSR / CSC index lists that drive the
// block-sparse attention kernels.
#include "asa_common.hpp"

namespace asa {

// ---------------------------------------------------------------------------------------
// Probe: P_imp[i][j] = max over sampled rows of block i and sampled keys of block j of the
// soft-max (over ALL sampled keys of the slab) of scale * Qs Ks^T.
//
// One wavefront per query block, following Alg. 1: a first sweep over the key blocks keeps
// per sampled query the running maximum Mt, the running denominator lt and the per-block row
// maximum Rt[j] (LDS); a second sweep turns Rt into probabilities and max-pools over rows.
// The sampled rows are gathered straight from Q and K (Alg. 2 steps 1-3): a 16 x 16 logit
// tile is one chain of 16x16x32 bf16 MFMAs with the keys on the M axis, so a lane holds
// 4 keys of one sampled query.
// ---------------------------------------------------------------------------------------
struct ProbeArgs {
  const void *q, *k;
  float *p_imp;
  TensorView tq, tk;
  int H, L, Nb, n_slabs, block, ks;
  float scale;
  int offs[kMaxSamples];
};

template <int D>
__global__ __launch_bounds__(64) void probe_kernel(ProbeArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  float *Rt = reinterpret_cast<float *>(smem);  // [Nb][16]
  __shared__ float sM[16];
  __shared__ double sL[16];

  const int work = xcd_contiguous_work(blockIdx.x, a.n_slabs * a.Nb);
  if (work < 0) return;
  const int slab = work / a.Nb;
  const int i = work - slab * a.Nb;
  const int lane = threadIdx.x;
  const int g = lane >> 4;   // key group: keys 4g .. 4g+3 of a tile live in this lane
  const int n = lane & 15;   // sampled query (B column) / sampled key (A row)

  const bf16 *qs = slab_ptr(a.q, a.tq, slab, a.H);
  const bf16 *ks = slab_ptr(a.k, a.tk, slab, a.H);

  // offset of sample slot n inside a block; slots >= ks do not exist
  int my_off = 0;
#pragma unroll
  for (int u = 0; u < kMaxSamples; ++u)
    if (u == n) my_off = a.offs[u];
  const bool slot_ok = n < a.ks;

  // B operand: sampled query n of block i, channels 32s + 8g .. +8
  const int qpos = i * a.block + my_off;
  const bool q_ok = slot_ok && qpos < a.L;
  bf16x8 qreg[D / 32];
  {
    const int qp = q_ok ? qpos : 0;
#pragma unroll
    for (int s = 0; s < D / 32; ++s)
      qreg[s] = *reinterpret_cast<const bf16x8 *>(qs + (int64_t)qp * a.tq.sL + 32 * s + 8 * g);
  }
  // offsets of the 4 keys whose logits land in this lane (rows 4g .. 4g+3 of the tile)
  int koff[4];
  bool kslot[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    int u = 4 * g + r;
    kslot[r] = u < a.ks;
    int o = 0;
#pragma unroll
    for (int uu = 0; uu < kMaxSamples; ++uu)
      if (uu == u) o = a.offs[uu];
    koff[r] = o;
  }

  float Mt = -INFINITY;  // running maximum of my query (replicated over the 4 key groups)
  double lt = 0.0;       // running denominator

  for (int j = 0; j < a.Nb; ++j) {
    // A operand: sampled key n of block j
    const int kpos = j * a.block + my_off;
    const int kp = (slot_ok && kpos < a.L) ? kpos : 0;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < D / 32; ++s) {
      bf16x8 ka = *reinterpret_cast<const bf16x8 *>(ks + (int64_t)kp * a.tk.sL + 32 * s + 8 * g);
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, qreg[s], acc, 0, 0, 0);
    }
    float sv[4];
    float mij = -INFINITY;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      bool ok = kslot[r] && (j * a.block + koff[r] < a.L);
      sv[r] = ok ? acc[r] * a.scale : -INFINITY;
      mij = fmaxf(mij, sv[r]);
    }
    mij = fmaxf(mij, __shfl_xor(mij, 16, 64));
    mij = fmaxf(mij, __shfl_xor(mij, 32, 64));
    if (g == 0) Rt[j * 16 + n] = mij;
    // a tile without a valid key (mij = -inf) must leave the running pair untouched
    const float mij_s = (mij == -INFINITY) ? 0.f : mij;
    float lij = 0.f;
#pragma unroll
    for (int r = 0; r < 4; ++r) lij += __expf(sv[r] - mij_s);
    lij += __shfl_xor(lij, 16, 64);
    lij += __shfl_xor(lij, 32, 64);
    const float mnew = fmaxf(Mt, mij);
    const float mnew_s = (mnew == -INFINITY) ? 0.f : mnew;
    lt = (double)__expf(Mt - mnew_s) * lt + (double)__expf(mij - mnew_s) * (double)lij;
    Mt = mnew;
  }
  if (g == 0) {
    sM[n] = Mt;
    sL[n] = lt;
  }
  __syncthreads();

  float *out = a.p_imp + ((int64_t)slab * a.Nb + i) * a.Nb;
  for (int j = lane; j < a.Nb; j += 64) {
    float best = 0.f;
    for (int u = 0; u < a.ks; ++u) {
      const bool row_ok = i * a.block + a.offs[u] < a.L;
      const float rt = Rt[j * 16 + u];
      if (row_ok && rt != -INFINITY) {
        float pr = (float)((double)__expf(rt - sM[u]) / sL[u]);
        best = fmaxf(best, pr);
      }
    }
    out[j] = best;
  }
}

hipError_t launch_probe(const Problem &pb, const void *q, const void *k, float *p_imp,
                        hipStream_t st) {
  ProbeArgs a;
  a.q = q; a.k = k; a.p_imp = p_imp; a.tq = pb.q; a.tk = pb.k;
  a.H = pb.H; a.L = pb.L; a.Nb = pb.Nb; a.n_slabs = pb.n_slabs; a.block = pb.block; a.ks = pb.ks;
  a.scale = pb.scale;
  for (int u = 0; u < kMaxSamples; ++u) a.offs[u] = pb.offs[u];
  const int grid = xcd_grid(pb.n_slabs * pb.Nb);
  const size_t lds = (size_t)pb.Nb * 16 * sizeof(float);
  if (pb.d == 128)
    hipLaunchKernelGGL(probe_kernel<128>, dim3(grid), dim3(64), lds, st, a);
  else
    hipLaunchKernelGGL(probe_kernel<64>, dim3(grid), dim3(64), lds, st, a);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Threshold rule (Alg. 3 steps 6-11), one workgroup per row of the importance map.
// rank_j = number of blocks that come before j in (score descending, index ascending) order;
// scores are scattered to rank order, their fp64 running sums c_r are formed in that order
// (one lane, so the additions happen in exactly the sequence the algorithm states), then
// m* = #{r : c_r < tau * T}, m = clamp(m*, m_min, m_max), keep rank < m.
// ---------------------------------------------------------------------------------------
struct RuleArgs {
  const float *scores;
  uint8_t *mask;
  int Nb, m_min, m_max, n_prefix_blocks;
  float tau;
};

__global__ __launch_bounds__(256) void rule_kernel(RuleArgs a) {
  __shared__ float p[kMaxNb];
  __shared__ float sorted[kMaxNb];
  __shared__ double cum[kMaxNb + 1];
  __shared__ int mstar;
  const int row = blockIdx.x;          // slab * Nb + i
  const int i = row % a.Nb;
  const int tid = threadIdx.x;
  const float *src = a.scores + (int64_t)row * a.Nb;
  for (int j = tid; j < a.Nb; j += 256) {
    float v = src[j];
    p[j] = (v == v) ? v : 0.f;
  }
  if (tid == 0) mstar = 0;
  __syncthreads();
  int rank[kMaxNb / 256];
#pragma unroll
  for (int t = 0; t < kMaxNb / 256; ++t) {
    const int j = tid + t * 256;
    rank[t] = 0;
    if (j < a.Nb) {
      const float pj = p[j];
      int r = 0;
      for (int l = 0; l < a.Nb; ++l) {
        const float pl = p[l];
        r += (pl > pj) || (pl == pj && l < j);
      }
      rank[t] = r;
      sorted[r] = pj;
    }
  }
  __syncthreads();
  if (tid == 0) {
    double c = 0.0;
    cum[0] = 0.0;
    for (int r = 0; r < a.Nb; ++r) {
      c = c + (double)sorted[r];
      cum[r + 1] = c;
    }
  }
  __syncthreads();
  const double thr = (double)a.tau * cum[a.Nb];
  int inside = 0;
  for (int r = tid; r < a.Nb; r += 256) inside += (cum[r] < thr);
  if (inside) atomicAdd(&mstar, inside);
  __syncthreads();
  int m = mstar;
  m = m < a.m_min ? a.m_min : m;
  m = m > a.m_max ? a.m_max : m;
  uint8_t *dst = a.mask + (int64_t)row * a.Nb;
#pragma unroll
  for (int t = 0; t < kMaxNb / 256; ++t) {
    const int j = tid + t * 256;
    if (j < a.Nb)
      dst[j] = (rank[t] < m) || (i < a.n_prefix_blocks) || (j < a.n_prefix_blocks);
  }
}

hipError_t launch_rule(const Problem &pb, const float *scores, uint8_t *mask, hipStream_t st) {
  RuleArgs a;
  a.scores = scores; a.mask = mask; a.Nb = pb.Nb; a.m_min = pb.m_min; a.m_max = pb.m_max;
  a.n_prefix_blocks = pb.n_prefix_blocks; a.tau = pb.tau;
  hipLaunchKernelGGL(rule_kernel, dim3(pb.n_slabs * pb.Nb), dim3(256), 0, st, a);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Index lists.  blockIdx.x = slab, blockIdx.y = 0: by rows (CSR), 1: by columns (CSC).
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void csr_kernel(const uint8_t *mask, int Nb, int32_t *row_ptr,
                                                  int32_t *col_idx, int32_t *col_ptr,
                                                  int32_t *row_idx) {
  __shared__ int cnt[kMaxNb + 1];
  const bool by_col = blockIdx.y == 1;
  int32_t *ptr = by_col ? col_ptr : row_ptr;
  int32_t *idx = by_col ? row_idx : col_idx;
  if (ptr == nullptr) return;
  const int slab = blockIdx.x;
  const uint8_t *m = mask + (int64_t)slab * Nb * Nb;
  const int64_t s_major = by_col ? 1 : Nb;  // step between lists
  const int64_t s_minor = by_col ? Nb : 1;  // step inside a list
  const int tid = threadIdx.x;
  for (int r = tid; r < Nb; r += 256) {
    int c = 0;
    for (int x = 0; x < Nb; ++x) c += m[r * s_major + x * s_minor] != 0;
    cnt[r] = c;
  }
  __syncthreads();
  if (tid == 0) {
    int run = 0;
    for (int r = 0; r < Nb; ++r) {
      int c = cnt[r];
      cnt[r] = run;
      run += c;
    }
    cnt[Nb] = run;
  }
  __syncthreads();
  ptr += (int64_t)slab * (Nb + 1);
  idx += (int64_t)slab * Nb * Nb;
  for (int r = tid; r <= Nb; r += 256) ptr[r] = cnt[r];
  for (int r = tid; r < Nb; r += 256) {
    int o = cnt[r];
    for (int x = 0; x < Nb; ++x)
      if (m[r * s_major + x * s_minor] != 0) idx[o++] = x;
  }
}

hipError_t launch_csr(const Problem &pb, const uint8_t *mask, int32_t *row_ptr, int32_t *col_idx,
                      int32_t *col_ptr, int32_t *row_idx, hipStream_t st) {
  hipLaunchKernelGGL(csr_kernel, dim3(pb.n_slabs, 2), dim3(256), 0, st, mask, pb.Nb, row_ptr,
                     col_idx, col_ptr, row_idx);
  return hipGetLastError();
}

}  // namespace asa
