// Mask generation for gfx950: block importance map (Alg. 2 -> Alg. 1 of the paper's appendix),
// the threshold rule (Alg. 3 steps 6-11) and the CSR / CSC index lists that drive the
// block-sparse attention kernels.
#include "asa_common.hpp"

namespace asa {

// ---------------------------------------------------------------------------------------
// Probe: P_imp[i][j] = max over sampled rows of block i and sampled keys of block j of the
// soft-max (over ALL sampled keys of the slab) of scale * Qs Ks^T.
//
// Alg. 1 of the paper, reorganised for 64-wide wavefronts.  One wavefront owns TWO query
// blocks and sweeps the key blocks two at a time: one chain of 32x32x16 bf16 MFMAs gives the
// 32 x 32 logit tile (2 key blocks x 16 samples on the M axis, 2 query blocks x 16 samples
// on the N axis).  The rows of the A operand are ordered so that lane half h holds, for ONE
// sampled query, all 16 samples of key block j0 + h: the block-row maximum Rt[query][j] of
// Alg. 1 is then a lane-local maximum, and the running maximum / denominator of the row is
// kept lane-locally over the key blocks of that parity and merged across the two halves once,
// at the end.  No cross-lane traffic inside the sweep.  The sampled rows are gathered straight
// from Q and K (Alg. 2 steps 1-3); the next pair of key blocks is fetched while the current
// one is being reduced.  A second sweep turns Rt into probabilities and max-pools over rows.
// ---------------------------------------------------------------------------------------
struct ProbeArgs {
  const void *q, *k;
  float *p_imp;
  TensorView tq, tk;
  int H, L, Nb, n_slabs, block, ks;
  int n_valid_last;  // sampled tokens of the last block that lie below L
  float scale;
  int offs[kMaxSamples];
};

template <int D>
__global__ __launch_bounds__(64) void probe_kernel(ProbeArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  float *Rt = reinterpret_cast<float *>(smem);  // [2 * ceil(Nb / 2)][32]
  __shared__ float sM[32];
  __shared__ double sL[32];

  const int n_pairs = (a.Nb + 1) / 2;
  const int work = xcd_contiguous_work(blockIdx.x, a.n_slabs * n_pairs);
  if (work < 0) return;
  const int slab = work / n_pairs;
  const int i0 = (work - slab * n_pairs) * 2;
  const int lane = threadIdx.x;
  const int hl = lane >> 5;  // operand k-half on loads, key-block parity on results
  const int n = lane & 31;   // A row on loads; query column on results

  const bf16 *qs = slab_ptr(a.q, a.tq, slab, a.H);
  const bf16 *ks = slab_ptr(a.k, a.tk, slab, a.H);

  auto offset_of = [&](int u) {
    int o = 0;
#pragma unroll
    for (int x = 0; x < kMaxSamples; ++x)
      if (x == u) o = a.offs[x];
    return o;
  };
  auto valid_in_block = [&](int blk) {
    return blk >= a.Nb ? 0 : (blk == a.Nb - 1 ? a.n_valid_last : a.ks);
  };

  // B operand: column n = sampled query (n & 15) of query block i0 + (n >> 4)
  const int q_blk = i0 + (n >> 4);
  const int q_slot = n & 15;
  const bool q_ok = q_slot < valid_in_block(q_blk);
  bf16x8 qreg[D / 16];
  {
    const int64_t qpos = q_ok ? (int64_t)q_blk * a.block + offset_of(q_slot) : 0;
#pragma unroll
    for (int s = 0; s < D / 16; ++s)
      qreg[s] = *reinterpret_cast<const bf16x8 *>(qs + qpos * a.tq.sL + 16 * s + 8 * hl);
  }
  // A operand: row r = 8g + 4h + j is sample 4g + j of key block j0 + h
  const int k_par = (n >> 2) & 1;
  const int k_slot = 4 * (n >> 3) + (n & 3);
  const int k_off = offset_of(k_slot);
  auto load_keys = [&](int j0, bf16x8 *dst) {
    const int blk = j0 + k_par;
    const int64_t kpos = k_slot < valid_in_block(blk) ? (int64_t)blk * a.block + k_off : 0;
#pragma unroll
    for (int s = 0; s < D / 16; ++s)
      dst[s] = *reinterpret_cast<const bf16x8 *>(ks + kpos * a.tk.sL + 16 * s + 8 * hl);
  };

  float Mt = -INFINITY;  // running maximum of my query over the key blocks of parity hl
  double lt = 0.0;       // running denominator over the same keys

  bf16x8 kcur[D / 16], knext[D / 16];
  load_keys(0, kcur);
  for (int j0 = 0; j0 < a.Nb; j0 += 2) {
    if (j0 + 2 < a.Nb) load_keys(j0 + 2, knext);
    f32x16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
    for (int s = 0; s < D / 16; ++s)
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kcur[s], qreg[s], acc, 0, 0, 0);
    // register i of lane half hl is sample i of key block j0 + hl
    const int nv = valid_in_block(j0 + hl);
    float sv[16];
    float mij = -INFINITY;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      sv[i] = i < nv ? acc[i] * a.scale : -INFINITY;
      mij = fmaxf(mij, sv[i]);
    }
    Rt[(j0 + hl) * 32 + n] = mij;
    const float mnew = fmaxf(Mt, mij);
    const float mnew_s = (mnew == -INFINITY) ? 0.f : mnew;
    float lij = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) lij += __expf(sv[i] - mnew_s);
    lt = (double)__expf(Mt - mnew_s) * lt + (double)lij;
    Mt = mnew;
#pragma unroll
    for (int s = 0; s < D / 16; ++s) kcur[s] = knext[s];
  }
  // merge the two parities of each query
  {
    const float Mo = __shfl_xor(Mt, 32, 64);
    const double lo = __shfl_xor(lt, 32, 64);
    const float Mall = fmaxf(Mt, Mo);
    const float Ms = (Mall == -INFINITY) ? 0.f : Mall;
    const double lall = (double)__expf(Mt - Ms) * lt + (double)__expf(Mo - Ms) * lo;
    if (hl == 0) {
      sM[n] = Mall;
      sL[n] = lall;
    }
  }
  __syncthreads();

#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    const int i = i0 + qb;
    if (i >= a.Nb) break;
    const int rows_ok = valid_in_block(i);
    float *out = a.p_imp + ((int64_t)slab * a.Nb + i) * a.Nb;
    for (int j = lane; j < a.Nb; j += 64) {
      float best = 0.f;
      for (int u = 0; u < rows_ok; ++u) {
        const float rt = Rt[j * 32 + qb * 16 + u];
        if (rt != -INFINITY) {
          float pr = (float)((double)__expf(rt - sM[qb * 16 + u]) / sL[qb * 16 + u]);
          best = fmaxf(best, pr);
        }
      }
      out[j] = best;
    }
  }
}

hipError_t launch_probe(const Problem &pb, const void *q, const void *k, float *p_imp,
                        hipStream_t st) {
  ProbeArgs a;
  a.q = q; a.k = k; a.p_imp = p_imp; a.tq = pb.q; a.tk = pb.k;
  a.H = pb.H; a.L = pb.L; a.Nb = pb.Nb; a.n_slabs = pb.n_slabs; a.block = pb.block; a.ks = pb.ks;
  a.scale = pb.scale;
  for (int u = 0; u < kMaxSamples; ++u) a.offs[u] = pb.offs[u];
  a.n_valid_last = 0;
  for (int u = 0; u < pb.ks; ++u)
    if ((int64_t)(pb.Nb - 1) * pb.block + pb.offs[u] < pb.L) ++a.n_valid_last;
  const int n_pairs = (pb.Nb + 1) / 2;
  const int grid = xcd_grid(pb.n_slabs * n_pairs);
  const size_t lds = (size_t)n_pairs * 2 * 32 * sizeof(float);
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
// Both walk the mask row by row so that every load is coalesced: the CSR side gives a
// wavefront one row at a time (64 columns per step, positions from a ballot), the CSC side
// gives every thread one column.
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
  ptr += (int64_t)slab * (Nb + 1);
  idx += (int64_t)slab * Nb * Nb;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;

  if (by_col) {
    for (int c = tid; c < Nb; c += 256) {
      int n = 0;
      for (int r = 0; r < Nb; ++r) n += m[(int64_t)r * Nb + c] != 0;
      cnt[c] = n;
    }
  } else {
    for (int r = wave; r < Nb; r += 4) {
      int n = 0;
      for (int c0 = 0; c0 < Nb; c0 += 64) {
        const bool f = (c0 + lane < Nb) && m[(int64_t)r * Nb + c0 + lane] != 0;
        n += __popcll(__ballot(f));
      }
      if (lane == 0) cnt[r] = n;
    }
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
  for (int r = tid; r <= Nb; r += 256) ptr[r] = cnt[r];
  if (by_col) {
    for (int c = tid; c < Nb; c += 256) {
      int o = cnt[c];
      for (int r = 0; r < Nb; ++r)
        if (m[(int64_t)r * Nb + c] != 0) idx[o++] = r;
    }
  } else {
    for (int r = wave; r < Nb; r += 4) {
      int o = cnt[r];
      for (int c0 = 0; c0 < Nb; c0 += 64) {
        const bool f = (c0 + lane < Nb) && m[(int64_t)r * Nb + c0 + lane] != 0;
        const unsigned long long b = __ballot(f);
        if (f) idx[o + __popcll(b & ((1ull << lane) - 1ull))] = c0 + lane;
        o += __popcll(b);
      }
    }
  }
}

hipError_t launch_csr(const Problem &pb, const uint8_t *mask, int32_t *row_ptr, int32_t *col_idx,
                      int32_t *col_ptr, int32_t *row_idx, hipStream_t st) {
  hipLaunchKernelGGL(csr_kernel, dim3(pb.n_slabs, 2), dim3(256), 0, st, mask, pb.Nb, row_ptr,
                     col_idx, col_ptr, row_idx);
  return hipGetLastError();
}

}  // namespace asa
