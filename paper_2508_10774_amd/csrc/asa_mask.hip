// Mask generation for gfx950: block importance map (Alg. 2 -> Alg. 1 of the paper's appendix),
// the threshold rule (Alg. 3 steps 6-11) and the CSR / CSC index lists that drive the
// block-sparse attention kernels.
#include <type_traits>

#include "asa_common.hpp"

namespace asa {

// ---------------------------------------------------------------------------------------
// Probe: P_imp[i][j] = max over sampled rows of block i and sampled keys of block j of the
// soft-max (over ALL sampled keys of the slab) of scale * Qs Ks^T.
//
// Alg. 1 of the paper, reorganised for 64-wide wavefronts.  A workgroup of 8 wavefronts owns 8
// query blocks and sweeps one of kProbeKeySplits ranges of the key blocks of its slab:
// wavefronts w and w + 4 share two query blocks and split every chunk of key blocks between them.  The sampled key rows (Alg. 2
// steps 1-3) are gathered from K by direct global->LDS loads, 8 key blocks (128 rows) per
// chunk, double-buffered and shared by all wavefronts.  One chain of 32x32x16
// bf16 MFMAs gives a 32 x 32 logit tile: 2 key blocks x 16 samples on the M axis, 2 query
// blocks x 16 samples on the N axis.  The rows of the A operand are ordered so that lane half h
// holds, for ONE sampled query, all 16 samples of key block j0 + h: the block-row maximum
// Rt[query][j] of Alg. 1 is then a lane-local maximum, and the running maximum / denominator of
// the row is kept lane-locally over the key blocks of that parity and merged across the two
// halves (and the two wavefronts of a pair) once, at the end.  No cross-lane traffic inside the
// sweep; the exponentials of a tile depend only on that tile's own maximum (Alg. 1 steps 12-14),
// so consecutive tiles overlap.  Rt and each wavefront's (maximum, denominator) pair go to a
// workspace in global memory; finish_rule_kernel merges the pairs of a sampled row, turns Rt
// into probabilities, max-pools over the sampled rows and applies the rule to the row.
// ---------------------------------------------------------------------------------------
struct ProbeArgs {
  const void *q, *k;
  float *p_imp;
  float *rt;         // workspace [query group][pair][Nb rounded up to 8][32]: block-row maxima
  float *stat_m;     // workspace [work item][wave][32]: running maximum of the wavefront's keys
  double *stat_l;    //           and the matching denominator
  TensorView tq, tk;
  int H, L, Nb, n_slabs, block, ks;
  int n_valid_last;  // sampled tokens of the last block that lie below L
  float scale;
  int offs[kMaxSamples];
  const uint8_t *table;   // per-block sample positions [slab][Nb][ks] (TAB kernels), else null
};

constexpr int kProbeQBlocks = 8;   // query blocks per workgroup
constexpr int kProbeKBlocks = 8;   // key blocks per LDS chunk
// The key blocks of a slab are cut into this many ranges, one workgroup each: at the Wan2.1 shape
// 12 heads x 32 query groups x 2 = 768 workgroups, three per compute unit (one range per group
// gave 384 workgroups for 512 resident slots: half of the compute units carried twice the load).
constexpr int kProbeKeySplits = 2;

typedef __attribute__((address_space(3))) void lds_void_m;
__device__ __forceinline__ void probe_dma16(const void *src, void *lds_dst) {
#if defined(__HIP_DEVICE_COMPILE__)
  __builtin_amdgcn_global_load_lds(src, (lds_void_m *)lds_dst, 16, 0, 0);
#endif
}

// chunk-position swizzle of the sampled-key rows in LDS (16 rows read together differ in row
// bits 0..2 and 4; at D = 64 a row is half the banks and parity picks the half)
template <int D>
__device__ __forceinline__ int probe_swz(int row) {
  return D == 128 ? ((row & 7) | (((row >> 4) & 1) << 3)) : (((row >> 1) & 3) | (((row >> 4) & 1) << 2));
}

// TAB: the sample positions differ from block to block and come from a table (seeded random
// sampling) instead of one offset vector for all blocks.
template <int D, bool TAB>
__global__ __launch_bounds__(512, 4) void probe_kernel(ProbeArgs a) {   // (4 wavefronts per SIMD: two workgroups per CU)
  constexpr int ROWS = kProbeKBlocks * 16;          // sampled rows per chunk
  constexpr int CH = D / 8;                         // 16-byte chunks per row
  constexpr int DMA_PER_WAVE = ROWS * CH / 64 / 8;  // 1 KB per wave instruction, 8 wavefronts
  extern __shared__ __align__(1024) unsigned char probe_smem[];
  bf16 (*Kc)[ROWS * D] = reinterpret_cast<bf16 (*)[ROWS * D]>(probe_smem);   // two buffers

  const int n_groups = (a.Nb + kProbeQBlocks - 1) / kProbeQBlocks;
  const int item = xcd_contiguous_work(blockIdx.x, a.n_slabs * n_groups * kProbeKeySplits);
  if (item < 0) return;
  const int work = item / kProbeKeySplits;          // (slab, query group)
  const int split = item - work * kProbeKeySplits;  // which range of key blocks
  const int slab = work / n_groups;
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int pair = wave & 3;      // which two query blocks
  const int half = wave >> 2;     // which half of every chunk of key blocks
  const int i_base = (work - slab * n_groups) * kProbeQBlocks;
  const int i0 = i_base + 2 * pair;
  const int hl = lane >> 5;  // operand k-half on loads, key-block parity on results
  const int n = lane & 31;   // A row on loads; query column on results
  const int nb_pad = (a.Nb + kProbeKBlocks - 1) / kProbeKBlocks * kProbeKBlocks;
  float *rt = a.rt + ((int64_t)work * 4 + pair) * nb_pad * 32;

  const bf16 *qs = slab_ptr(a.q, a.tq, slab, a.H);
  const bf16 *ks = slab_ptr(a.k, a.tk, slab, a.H);

  // TAB: this slab's table in LDS; positions ascend inside a block, so the samples of the last
  // block that lie below L are a prefix
  __shared__ uint8_t tab[TAB ? kMaxNb * kMaxSamples : 16];
  int n_valid_last = a.n_valid_last;
  if (TAB) {
    const uint8_t *g = a.table + (int64_t)slab * a.Nb * a.ks;
    for (int t = tid; t < a.Nb * a.ks; t += 512) tab[t] = g[t];
    __syncthreads();
    n_valid_last = 0;
    for (int u = 0; u < a.ks; ++u)
      if ((a.Nb - 1) * a.block + tab[(a.Nb - 1) * a.ks + u] < a.L) ++n_valid_last;
  }
  auto offset_of = [&](int blk, int u) {
    if (TAB) return (blk < a.Nb && u < a.ks) ? (int)tab[blk * a.ks + u] : 0;
    int o = 0;
#pragma unroll
    for (int x = 0; x < kMaxSamples; ++x)
      if (x == u) o = a.offs[x];
    return o;
  };
  auto valid_in_block = [&](int blk) {
    return blk >= a.Nb ? 0 : (blk == a.Nb - 1 ? n_valid_last : a.ks);
  };

  // B operand: column n = sampled query (n & 15) of query block i0 + (n >> 4)
  const int q_blk = i0 + (n >> 4);
  const bool q_ok = (n & 15) < valid_in_block(q_blk);
  bf16x8 qreg[D / 16];
  {
    const int64_t qpos = q_ok ? (int64_t)q_blk * a.block + offset_of(q_blk, n & 15) : 0;
#pragma unroll
    for (int s = 0; s < D / 16; ++s)
      qreg[s] = *reinterpret_cast<const bf16x8 *>(qs + qpos * a.tq.sL + 16 * s + 8 * hl);
  }

  // producer: my share of a chunk of sampled key rows (row r of a chunk = key block r / 16,
  // sample r % 16)
  int dma_tok[DMA_PER_WAVE];   // token offset inside the chunk, or -1 for a sample slot >= ks
  int dma_pos[DMA_PER_WAVE];   // swizzled 16-byte position to fetch
#pragma unroll
  for (int i = 0; i < DMA_PER_WAVE; ++i) {
    const int seg = wave * DMA_PER_WAVE + i;
    const int row = seg * (64 / CH) + lane / CH;
    dma_tok[i] = (row / 16) * a.block + (TAB ? 0 : offset_of(0, row % 16));
    dma_pos[i] = ((lane % CH) ^ probe_swz<D>(row)) * 8;
  }
  auto fetch = [&](int chunk, int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < DMA_PER_WAVE; ++i) {
      const int seg = wave * DMA_PER_WAVE + i;
      int64_t tok = (int64_t)chunk * kProbeKBlocks * a.block + dma_tok[i];
      if (TAB) {
        const int row = seg * (64 / CH) + lane / CH;
        tok += offset_of(chunk * kProbeKBlocks + row / 16, row % 16);
      }
      tok = tok < a.L ? tok : 0;   // padded samples: any valid row, masked out below
      probe_dma16(ks + tok * a.tk.sL + dma_pos[i], &Kc[buf][seg * 512]);
    }
  };

  // The common case of that, with all address arithmetic taken out of the sweep: one offset
  // vector for all blocks and a chunk that lies wholly below L.  Per lane a byte offset inside
  // the chunk, per chunk one wave-uniform base.
  uint32_t dma_off0[DMA_PER_WAVE];   // bytes from the first token of the chunk
#pragma unroll
  for (int i = 0; i < DMA_PER_WAVE; ++i)
    dma_off0[i] = (uint32_t)(((int64_t)dma_tok[i] * a.tk.sL + dma_pos[i]) * 2);
  const int64_t chunk_stride = (int64_t)kProbeKBlocks * a.block * a.tk.sL * 2;   // bytes
  // chunks with no token >= L (none if a chunk's rows span 4 GiB or more: 32-bit offsets)
  const int n_full_chunks = (TAB || chunk_stride >= ((int64_t)1 << 32)) ? 0 : a.L / (kProbeKBlocks * a.block);
  auto fetch_any = [&](int chunk, int buf) __attribute__((always_inline)) {
    if (chunk < n_full_chunks) {
      const char *base = reinterpret_cast<const char *>(ks) + chunk * chunk_stride;   // wave-uniform
#pragma unroll
      for (int i = 0; i < DMA_PER_WAVE; ++i)
        probe_dma16(base + dma_off0[i], &Kc[buf][(wave * DMA_PER_WAVE + i) * 512]);
    } else {
      fetch(chunk, buf);
    }
  };

  // consumer: A row r = 8g + 4h + j is sample 4g + j of key block j0 + h
  const int a_row = ((n >> 2) & 1) * 16 + 4 * (n >> 3) + (n & 3);   // row inside a pair of key blocks
  const int a_swz = probe_swz<D>(a_row);
  // my fragment s of the first pair of key blocks of my half of a chunk (elements from the
  // start of the buffer); the second pair and the other buffer are constant distances away
  int a_off[D / 16];
#pragma unroll
  for (int s = 0; s < D / 16; ++s)
    a_off[s] = (half * (kProbeKBlocks / 4) * 32 + a_row) * D + (((2 * s + hl) ^ a_swz) * 8);
  // where my block-row maxima of chunk 0 go (floats from the start of rt)
  const int rt_off = (2 * half * (kProbeKBlocks / 4) + hl) * 32 + n;

  float rt_pend[kProbeKBlocks / 4];   // block-row maxima of the chunk just swept
  float Mt = -INFINITY;  // running maximum of my query over the key blocks of parity hl
  double lt = 0.0;       // running denominator over the same keys
  const float c2 = a.scale * 1.44269504088896340736f;

  // one chunk out of LDS buffer BUF (a compile-time constant: every LDS address of the sweep is
  // a per-lane register plus an immediate)
  auto sweep_chunk = [&](int chunk, auto buf_tag) __attribute__((always_inline)) {
    constexpr int BUF = decltype(buf_tag)::value;
    const bf16 *Kb = Kc[BUF];
#pragma unroll
    for (int sb = 0; sb < kProbeKBlocks / 4; ++sb) {
      const int j0 = chunk * kProbeKBlocks + 2 * (half * (kProbeKBlocks / 4) + sb);
      f32x16 acc;
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
      for (int s = 0; s < D / 16; ++s) {
        bf16x8 ka = *reinterpret_cast<const bf16x8 *>(Kb + sb * 32 * D + a_off[s]);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[s], acc, 0, 0, 0);
      }
      // register i of lane half hl is sample i of key block j0 + hl; samples past L (only in
      // the last block), past the last block, or in sample slots >= k are masked out
      if (a.ks < kMaxSamples || j0 + 2 >= a.Nb) {
        const int nv = valid_in_block(j0 + hl);
#pragma unroll
        for (int i = 0; i < 16; ++i)
          if (i >= nv) acc[i] = -INFINITY;
      }
      float mraw = -INFINITY;
#pragma unroll
      for (int i = 0; i < 16; ++i) mraw = fmaxf(mraw, acc[i]);
      const float mij = mraw * a.scale;                  // block-row maximum, Alg. 1 step 12
      rt_pend[sb] = mij;
      // Alg. 1 steps 12-15: tile-local exponentials exp(scale * (s - max)) as one fused
      // multiply-add and one exp2 each, then fold into the running pair
      const float bias = (mraw == -INFINITY) ? 0.f : -mraw * c2;
      float lij = 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i) lij += fast_exp2(fmaf(acc[i], c2, bias));
      if (__any(mij > Mt)) {
        const float mnew = fmaxf(Mt, mij);
        const float mnew_s = (mnew == -INFINITY) ? 0.f : mnew;
        lt = (double)__expf(Mt - mnew_s) * lt + (double)__expf(mij - mnew_s) * (double)lij;
        Mt = mnew;
      } else {
        // no row's maximum grew (the usual case once the sweep has passed the query's own
        // neighbourhood): the general update with a factor of exactly 1 on the old sum
        lt += (double)__expf(mij - ((Mt == -INFINITY) ? 0.f : Mt)) * (double)lij;
      }
    }
  };

  // The block-row maxima of a chunk are stored at the start of the NEXT chunk's turn, just before
  // its loads are requested: the wait for those loads at the top of the turn after that also
  // waits for the stores (one counter), and a store issued in the middle of a turn was not yet
  // acknowledged at its end.
  auto store_rt = [&](int chunk) __attribute__((always_inline)) {
    float *rt_c = rt + (int64_t)chunk * kProbeKBlocks * 32;
#pragma unroll
    for (int sb = 0; sb < kProbeKBlocks / 4; ++sb) rt_c[rt_off + sb * 64] = rt_pend[sb];
  };
  const int n_chunks = nb_pad / kProbeKBlocks;
  const int per_split = (n_chunks + kProbeKeySplits - 1) / kProbeKeySplits;
  const int c0 = min(n_chunks, split * per_split), c1 = min(n_chunks, c0 + per_split);   // my chunks
  if (c0 < c1) fetch_any(c0, 0);
  for (int chunk = c0; chunk < c1; chunk += 2) {
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): my loads of this chunk have landed
    __syncthreads();                     // everyone's have, and the other buffer is free
    if (chunk > c0) store_rt(chunk - 1);
    if (chunk + 1 < c1) fetch_any(chunk + 1, 1);
    sweep_chunk(chunk, std::integral_constant<int, 0>{});
    if (chunk + 1 >= c1) break;
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    store_rt(chunk);
    if (chunk + 2 < c1) fetch_any(chunk + 2, 0);
    sweep_chunk(chunk + 1, std::integral_constant<int, 1>{});
  }
  if (c0 < c1) store_rt(c1 - 1);
  // merge the two parities of each query; the pair (maximum, denominator) of this wavefront's
  // share of the keys goes to the workspace (the kernel that follows merges the shares)
  {
    const float Mo = __shfl_xor(Mt, 32, 64);
    const double lo = __shfl_xor(lt, 32, 64);
    const float Mall = fmaxf(Mt, Mo);
    const float Ms = (Mall == -INFINITY) ? 0.f : Mall;
    const double lall = (double)__expf(Mt - Ms) * lt + (double)__expf(Mo - Ms) * lo;
    if (hl == 0) {
      a.stat_m[((int64_t)item * 8 + wave) * 32 + n] = Mall;
      a.stat_l[((int64_t)item * 8 + wave) * 32 + n] = lall;
    }
  }
}

static size_t probe_rt_bytes(const Problem &pb) {
  const size_t n_groups = (pb.Nb + kProbeQBlocks - 1) / kProbeQBlocks;
  const size_t nb_pad = (pb.Nb + kProbeKBlocks - 1) / kProbeKBlocks * kProbeKBlocks;
  return ((size_t)pb.n_slabs * n_groups * 4 * nb_pad * 32 * sizeof(float) + 255) & ~(size_t)255;
}
static size_t probe_items(const Problem &pb) {
  return (size_t)pb.n_slabs * ((pb.Nb + kProbeQBlocks - 1) / kProbeQBlocks) * kProbeKeySplits;
}
size_t probe_workspace_bytes(const Problem &pb) {
  // block-row maxima, then the per-wavefront soft-max statistics (fp64 denominators first)
  return probe_rt_bytes(pb) + probe_items(pb) * 8 * 32 * (sizeof(double) + sizeof(float));
}

static void fill_probe_args(const Problem &pb, const void *q, const void *k, float *p_imp,
                            void *workspace, const uint8_t *table, ProbeArgs *a) {
  a->table = table;
  a->q = q; a->k = k; a->p_imp = p_imp;
  unsigned char *ws = reinterpret_cast<unsigned char *>(workspace);
  a->rt = reinterpret_cast<float *>(ws);
  a->stat_l = reinterpret_cast<double *>(ws + probe_rt_bytes(pb));
  a->stat_m = reinterpret_cast<float *>(ws + probe_rt_bytes(pb) + probe_items(pb) * 8 * 32 * sizeof(double));
  a->tq = pb.q; a->tk = pb.k;
  a->H = pb.H; a->L = pb.L; a->Nb = pb.Nb; a->n_slabs = pb.n_slabs; a->block = pb.block; a->ks = pb.ks;
  a->scale = pb.scale;
  for (int u = 0; u < kMaxSamples; ++u) a->offs[u] = pb.offs[u];
  a->n_valid_last = 0;
  for (int u = 0; u < pb.ks; ++u)
    if ((int64_t)(pb.Nb - 1) * pb.block + pb.offs[u] < pb.L) ++a->n_valid_last;
}

hipError_t launch_probe(const Problem &pb, const void *q, const void *k, void *workspace,
                        hipStream_t st, const uint8_t *table) {
  ProbeArgs a;
  fill_probe_args(pb, q, k, nullptr, workspace, table, &a);
  const int grid = xcd_grid((int)probe_items(pb));
  const int lds = 2 * kProbeKBlocks * 16 * pb.d * 2;   // two chunks of sampled key rows
  if (pb.d == 128) {
    const void *fn = table ? reinterpret_cast<const void *>(&probe_kernel<128, true>)
                           : reinterpret_cast<const void *>(&probe_kernel<128, false>);
    hipError_t e = set_dynamic_lds_once(fn, 2 * kProbeKBlocks * 16 * 128 * 2);
    if (e != hipSuccess) return e;
  }
  if (pb.d == 128 && table)
    hipLaunchKernelGGL((probe_kernel<128, true>), dim3(grid), dim3(512), lds, st, a);
  else if (pb.d == 128)
    hipLaunchKernelGGL((probe_kernel<128, false>), dim3(grid), dim3(512), lds, st, a);
  else if (table)
    hipLaunchKernelGGL((probe_kernel<64, true>), dim3(grid), dim3(512), lds, st, a);
  else
    hipLaunchKernelGGL((probe_kernel<64, false>), dim3(grid), dim3(512), lds, st, a);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Seeded random sampling (Alg. 3 step 2 made reproducible).  Philox-4x32 with 10 rounds
// (Salmon et al., SC'11) gives position j of block `blk` of slab `slab` the word
// Philox(counter = (j, blk, slab, 0), key = seed)[0]; the k positions with the smallest
// (word, j) are the block's sample, written in ascending position.  One wavefront per block.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t philox4x32_10_word0(uint32_t c0, uint32_t c1, uint32_t c2,
                                                        uint32_t c3, uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n1 = (uint32_t)p1;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1, n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return c0;
}

__global__ __launch_bounds__(64) void sample_offsets_kernel(uint32_t seed_lo, uint32_t seed_hi,
                                                            int Nb, int b, int ks, uint8_t *table) {
  __shared__ uint64_t word[128];   // (philox word, position): distinct, so ranks are too
  __shared__ uint8_t chosen[128];
  const int blk = blockIdx.x, slab = blockIdx.y, lane = threadIdx.x;
  for (int j = lane; j < b; j += 64)
    word[j] = ((uint64_t)philox4x32_10_word0((uint32_t)j, (uint32_t)blk, (uint32_t)slab, 0u, seed_lo, seed_hi) << 32) | (uint32_t)j;
  __syncthreads();
  for (int j = lane; j < b; j += 64) {
    int rank = 0;
    for (int x = 0; x < b; ++x) rank += word[x] < word[j];
    chosen[j] = rank < ks;
  }
  __syncthreads();
  if (lane == 0) {
    uint8_t *out = table + ((int64_t)slab * Nb + blk) * ks;
    int n = 0;
    for (int j = 0; j < b; ++j)
      if (chosen[j]) out[n++] = (uint8_t)j;
  }
}

hipError_t launch_sample_offsets(const Problem &pb, uint64_t seed, uint8_t *table, hipStream_t st) {
  hipLaunchKernelGGL(sample_offsets_kernel, dim3(pb.Nb, pb.n_slabs), dim3(64), 0, st,
                     (uint32_t)seed, (uint32_t)(seed >> 32), pb.Nb, pb.block, pb.ks, table);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Threshold rule (Alg. 3 steps 6-11), one wavefront per row of the importance map.
// The row is sorted by (score descending, block index ascending) with a bitonic network on
// 64-bit keys (inverted order-preserving image of the fp32 score in the high word, the block
// index in the low word).  The keys live in registers, NPAD / 64 consecutive ranks per lane:
// network stages whose partners sit in the same lane are register compare-exchanges, the others
// fetch the partner lane's key through the cross-lane network (no LDS memory traffic: with the
// keys in LDS the kernel was bound by LDS bandwidth).  One lane then forms the fp64 running sums
// c_r in rank order -- the additions happen in exactly the sequence the algorithm states, so the
// decision is bit-identical to a sequential implementation -- then m* = #{r : c_r < tau * T},
// m = clamp(m*, m_min, m_max), keep rank < m.  A NaN score counts as 0.
// ---------------------------------------------------------------------------------------
struct RuleArgs {
  const float *scores;
  uint8_t *mask;
  int Nb, n_rows, m_min, m_max, n_prefix_blocks;
  float tau;
};

__device__ __forceinline__ uint32_t desc_key(float v) {
  v = (v == v) ? v + 0.0f : 0.0f;                 // NaN -> 0, -0 -> +0
  uint32_t u = __float_as_uint(v);
  u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);  // ascending order-preserving image
  return ~u;                                       // larger score -> smaller key
}
__device__ __forceinline__ float key_score(uint32_t k) {
  uint32_t u = ~k;
  u = (u & 0x80000000u) ? (u & 0x7fffffffu) : ~u;
  return __uint_as_float(u);
}

// The rule on one row whose Nb scores sit in the wavefront's registers as sort keys, in any
// order (key = order image of the score in the high word, block index in the low word; slots
// beyond Nb hold ~0).  cum: NPAD doubles of LDS owned by this wavefront.  Every step is
// wave-synchronous: no workgroup barrier.  Writes the row's Nb mask bytes to dst.
template <int NPAD>
__device__ __forceinline__ void rule_on_keys(unsigned long long (&key)[NPAD / 64], double *cum, int lane,
                                             int i, int Nb, float tau, int m_min, int m_max,
                                             int n_prefix_blocks, uint8_t *dst) {
  constexpr int E = NPAD / 64;               // keys per lane; rank of key r of a lane = lane * E + r
  // ascending bitonic network over e = lane * E + r: stage (k, jj) orders the pair (e, e ^ jj)
  // upwards where (e & k) == 0 and downwards elsewhere
  for (int k = 2; k <= NPAD; k <<= 1) {
    // partners in other lanes: lane ^ (jj / E), same register
    for (int jj = k >> 1; jj >= E; jj >>= 1) {
      const int dl = jj / E;
      const bool up = ((lane * E) & k) == 0;           // (k > jj >= E: decided by the lane)
      const bool keep_min = ((lane & dl) == 0) == up;
#pragma unroll
      for (int r = 0; r < E; ++r) {
        const uint32_t lo = (uint32_t)key[r], hi = (uint32_t)(key[r] >> 32);
        const unsigned long long other =
            ((unsigned long long)(uint32_t)__shfl_xor((int)hi, dl, 64) << 32) | (uint32_t)__shfl_xor((int)lo, dl, 64);
        const bool other_smaller = other < key[r];
        key[r] = (other_smaller == keep_min) ? other : key[r];
      }
    }
    // partners in the same lane: registers r and r ^ jj
#pragma unroll
    for (int jj = E >> 1; jj > 0; jj >>= 1) {
      if (jj < k) {
#pragma unroll
        for (int r = 0; r < E; ++r) {
          if ((r & jj) == 0) {
            const bool up = ((lane * E + r) & k) == 0;
            const unsigned long long x = key[r], y = key[r ^ jj];
            const bool swap = (x > y) == up;
            key[r] = swap ? y : x;
            key[r ^ jj] = swap ? x : y;
          }
        }
      }
    }
  }
  // scores in rank order as fp64, zero-padded
#pragma unroll
  for (int r = 0; r < E; ++r) {
    const int e = lane * E + r;
    cum[e] = e < Nb ? (double)key_score((uint32_t)(key[r] >> 32)) : 0.0;
  }
  __builtin_amdgcn_wave_barrier();
  // Running sums in place: cum[r] becomes c_{r+1} = sum of the r+1 best scores.  Sequential on
  // purpose (see above): one lane, eight values fetched at a time so that only the additions
  // sit on the dependent chain.
  if (lane == 0) {
    double c = 0.0;
    for (int r0 = 0; r0 < Nb; r0 += 8) {
      double v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = cum[r0 + u];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        c = c + v[u];
        v[u] = c;
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) cum[r0 + u] = v[u];
    }
  }
  __builtin_amdgcn_wave_barrier();
  const double thr = (double)tau * cum[Nb - 1];   // tau * T
  int inside = 0;
#pragma unroll
  for (int r = 0; r < E; ++r) {
    const int e = lane * E + r;
    if (e < Nb) inside += ((e == 0 ? 0.0 : cum[e - 1]) < thr);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) inside += __shfl_xor(inside, off, 64);
  int m = inside;
  m = m < m_min ? m_min : m;
  m = m > m_max ? m_max : m;
#pragma unroll
  for (int r = 0; r < E; ++r) {
    const int e = lane * E + r;
    if (e < Nb) {
      const int j = (int)(key[r] & 0xffffffffu);
      dst[j] = (e < m) || (i < n_prefix_blocks) || (j < n_prefix_blocks);
    }
  }
}

// Four rows per workgroup, one per wavefront, so that the sequential running sums of different
// rows run on different SIMDs.
template <int NPAD>
__global__ __launch_bounds__(256) void rule_kernel(RuleArgs a) {
  constexpr int E = NPAD / 64;
  __shared__ double cum_all[4][NPAD];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + wave;          // slab * Nb + i
  if (row >= a.n_rows) return;                     // whole wavefront; no workgroup barriers below
  const float *src = a.scores + (int64_t)row * a.Nb;
  unsigned long long key[E];
#pragma unroll
  for (int r = 0; r < E; ++r) {
    const int j = lane * E + r;
    key[r] = j < a.Nb ? (((unsigned long long)desc_key(src[j]) << 32) | (unsigned)j)
                      : ~0ull;        // padding sorts last
  }
  rule_on_keys<NPAD>(key, cum_all[wave], lane, row % a.Nb, a.Nb, a.tau, a.m_min, a.m_max,
                     a.n_prefix_blocks, a.mask + (int64_t)row * a.Nb);
}

// ---------------------------------------------------------------------------------------
// Second half of the probe (Alg. 1, second loop) fused with the rule: one wavefront per query
// block.  It merges the soft-max statistics of the wavefronts that swept this block's sampled
// rows (two halves of every chunk x the ranges of key blocks), turns the block-row maxima into
// probabilities, max-pools them over the sampled rows -- the row P_imp[i][:], written out if the
// caller wants it -- and applies the rule to that row while it is still in registers.
// ---------------------------------------------------------------------------------------
template <int NPAD>
__global__ __launch_bounds__(256) void finish_rule_kernel(ProbeArgs a, RuleArgs ra) {
  constexpr int E = NPAD / 64;
  __shared__ double cum_all[4][NPAD];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + wave;          // slab * Nb + i
  if (row >= ra.n_rows) return;
  const int slab = row / a.Nb, i = row - slab * a.Nb;
  const int n_groups = (a.Nb + kProbeQBlocks - 1) / kProbeQBlocks;
  const int nb_pad = (a.Nb + kProbeKBlocks - 1) / kProbeKBlocks * kProbeKBlocks;
  const int work = slab * n_groups + i / kProbeQBlocks;      // the query group that swept this block
  const int w = i % kProbeQBlocks, pr_ = w >> 1, qb = w & 1;  // its pair and position in the pair
  const float *rtq = a.rt + ((int64_t)work * 4 + pr_) * nb_pad * 32 + qb * 16;
  // merge the shares: wavefronts pr_ and pr_ + 4 of every key range
  // (the denominator is summed in fp64; its reciprocal is rounded to fp32 once per sampled
  // row: the exponentials below are fp32 anyway)
  // Lane u < 16 merges the shares of sampled row u; the 16 results are then handed to every
  // lane through scalar registers (all lanes doing all 16 rows cost 16 fp64 divisions a lane).
  float my_m = -INFINITY, my_inv = 0.f;
  {
    const int u = lane & 15;
    float pm[2 * kProbeKeySplits];
    double pl[2 * kProbeKeySplits];
#pragma unroll
    for (int sp = 0; sp < kProbeKeySplits; ++sp)
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
        const int64_t at = (((int64_t)work * kProbeKeySplits + sp) * 8 + pr_ + 4 * hf) * 32 + qb * 16 + u;
        pm[2 * sp + hf] = a.stat_m[at];
        pl[2 * sp + hf] = a.stat_l[at];
        my_m = fmaxf(my_m, pm[2 * sp + hf]);
      }
    const float ms = (my_m == -INFINITY) ? 0.f : my_m;
    double l = 0.0;
#pragma unroll
    for (int x = 0; x < 2 * kProbeKeySplits; ++x) l += (double)__expf(pm[x] - ms) * pl[x];
    my_inv = (float)(1.0 / l);
  }
  float Mrow[16], Linv[16];
#pragma unroll
  for (int u = 0; u < 16; ++u) {
    Mrow[u] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, my_m), u));
    Linv[u] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, my_inv), u));
  }
  int rows_ok = a.ks;                       // sampled rows of this block that lie below L
  if (i == a.Nb - 1) {
    if (a.table) {
      rows_ok = 0;
      const uint8_t *t = a.table + ((int64_t)slab * a.Nb + i) * a.ks;
      for (int u = 0; u < a.ks; ++u) rows_ok += (int64_t)i * a.block + t[u] < a.L;
    } else {
      rows_ok = a.n_valid_last;
    }
  }
  float *out = a.p_imp ? a.p_imp + (int64_t)row * a.Nb : nullptr;
  unsigned long long key[E];
#pragma unroll
  for (int r = 0; r < E; ++r) {
    const int j = lane + 64 * r;
    key[r] = ~0ull;                         // padding sorts last
    if (j < a.Nb) {
      const f32x4 *src = reinterpret_cast<const f32x4 *>(rtq + (int64_t)j * 32);
      const f32x4 r0 = src[0], r1 = src[1], r2 = src[2], r3 = src[3];
      const float rv[16] = {r0[0], r0[1], r0[2], r0[3], r1[0], r1[1], r1[2], r1[3],
                            r2[0], r2[1], r2[2], r2[3], r3[0], r3[1], r3[2], r3[3]};
      float best = 0.f;
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        if (u < rows_ok && rv[u] != -INFINITY) best = fmaxf(best, __expf(rv[u] - Mrow[u]) * Linv[u]);
      }
      if (out) out[j] = best;
      key[r] = ((unsigned long long)desc_key(best) << 32) | (unsigned)j;
    }
  }
  if (ra.mask == nullptr) return;   // the caller only wanted the map (wave-uniform)
  rule_on_keys<NPAD>(key, cum_all[wave], lane, i, a.Nb, ra.tau, ra.m_min, ra.m_max, ra.n_prefix_blocks,
                     ra.mask + (int64_t)row * a.Nb);
}

// dst[s][i][j] = max of src[s][i g .. i g + g)[j g .. j g + g) (clipped at n_src): the importance
// map of blocks that are g times as large.  One thread per output element.
__global__ void pool_scores_kernel(const float *src, int n_src, float *dst, int n_dst, int g) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x, i = blockIdx.y, s = blockIdx.z;
  if (j >= n_dst) return;
  const float *in = src + (int64_t)s * n_src * n_src;
  float best = 0.f;
  for (int a = i * g; a < min(n_src, i * g + g); ++a)
    for (int b = j * g; b < min(n_src, j * g + g); ++b) best = fmaxf(best, in[(int64_t)a * n_src + b]);
  dst[((int64_t)s * n_dst + i) * n_dst + j] = best;
}
hipError_t launch_pool_scores(const float *src, int n_src, float *dst, int n_dst, int g, int n_slabs,
                              hipStream_t st) {
  hipLaunchKernelGGL(pool_scores_kernel, dim3((n_dst + 63) / 64, n_dst, n_slabs), dim3(64), 0, st, src,
                     n_src, dst, n_dst, g);
  return hipGetLastError();
}

hipError_t launch_finish_rule(const Problem &pb, void *workspace, float *p_imp, uint8_t *mask,
                              const uint8_t *table, hipStream_t st) {
  ProbeArgs a;
  fill_probe_args(pb, nullptr, nullptr, p_imp, workspace, table, &a);
  RuleArgs ra;
  ra.scores = nullptr; ra.mask = mask; ra.Nb = pb.Nb; ra.m_min = pb.m_min; ra.m_max = pb.m_max;
  ra.n_prefix_blocks = pb.n_prefix_blocks; ra.tau = pb.tau;
  ra.n_rows = pb.n_slabs * pb.Nb;
  const dim3 grid((ra.n_rows + 3) / 4), block(256);
  if (pb.Nb <= 128) hipLaunchKernelGGL(finish_rule_kernel<128>, grid, block, 0, st, a, ra);
  else if (pb.Nb <= 256) hipLaunchKernelGGL(finish_rule_kernel<256>, grid, block, 0, st, a, ra);
  else if (pb.Nb <= 512) hipLaunchKernelGGL(finish_rule_kernel<512>, grid, block, 0, st, a, ra);
  else hipLaunchKernelGGL(finish_rule_kernel<1024>, grid, block, 0, st, a, ra);
  return hipGetLastError();
}

hipError_t launch_rule(const Problem &pb, const float *scores, uint8_t *mask, hipStream_t st) {
  RuleArgs a;
  a.scores = scores; a.mask = mask; a.Nb = pb.Nb; a.m_min = pb.m_min; a.m_max = pb.m_max;
  a.n_prefix_blocks = pb.n_prefix_blocks; a.tau = pb.tau;
  a.n_rows = pb.n_slabs * pb.Nb;
  const dim3 grid((a.n_rows + 3) / 4), block(256);
  // network size: power of two >= Nb (and >= 128 so that every lane owns a pair)
  if (pb.Nb <= 128) hipLaunchKernelGGL(rule_kernel<128>, grid, block, 0, st, a);
  else if (pb.Nb <= 256) hipLaunchKernelGGL(rule_kernel<256>, grid, block, 0, st, a);
  else if (pb.Nb <= 512) hipLaunchKernelGGL(rule_kernel<512>, grid, block, 0, st, a);
  else hipLaunchKernelGGL(rule_kernel<1024>, grid, block, 0, st, a);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Index lists of a mask, by rows (CSR) and by columns (CSC), in three small fully parallel
// kernels: count (one workgroup per row i and column i), in-place scan of the counts, fill.
// ---------------------------------------------------------------------------------------
// blockIdx = (i, slab).  Wavefront 0 counts row i (coalesced), wavefront 1 counts column i.
__global__ __launch_bounds__(128) void csr_count_kernel(const uint8_t *mask, int Nb,
                                                        int32_t *row_ptr, int32_t *col_ptr) {
  const int i = blockIdx.x, slab = blockIdx.y;
  const uint8_t *m = mask + (int64_t)slab * Nb * Nb;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  int32_t *ptr = wave == 0 ? row_ptr : col_ptr;
  if (ptr == nullptr) return;
  int n = 0;
  for (int x0 = 0; x0 < Nb; x0 += 64) {
    const int x = x0 + lane;
    const bool f = x < Nb && (wave == 0 ? m[(int64_t)i * Nb + x] : m[(int64_t)x * Nb + i]) != 0;
    n += __popcll(__ballot(f));
  }
  if (lane == 0) {
    ptr[(int64_t)slab * (Nb + 1) + i + 1] = n;
    if (i == 0) ptr[(int64_t)slab * (Nb + 1)] = 0;
  }
}

// blockIdx = (slab, 0: rows / 1: columns).  Inclusive scan of ptr[1..Nb] in place.
__global__ __launch_bounds__(256) void csr_scan_kernel(int Nb, int32_t *row_ptr, int32_t *col_ptr) {
  __shared__ int part[256];
  int32_t *ptr = blockIdx.y == 0 ? row_ptr : col_ptr;
  if (ptr == nullptr) return;
  ptr += (int64_t)blockIdx.x * (Nb + 1) + 1;
  const int tid = threadIdx.x;
  const int per = (Nb + 255) / 256;
  const int lo = tid * per;
  int sum = 0;
  for (int x = lo; x < lo + per && x < Nb; ++x) sum += ptr[x];
  part[tid] = sum;
  __syncthreads();
  for (int off = 1; off < 256; off <<= 1) {
    int v = tid >= off ? part[tid - off] : 0;
    __syncthreads();
    part[tid] += v;
    __syncthreads();
  }
  int run = part[tid] - sum;   // exclusive prefix of my segment
  for (int x = lo; x < lo + per && x < Nb; ++x) {
    run += ptr[x];
    ptr[x] = run;
  }
}

// blockIdx = (i, slab).  Wavefront 0 writes the kept columns of row i, wavefront 1 the kept
// rows of column i, both ascending (ballot compaction, 64 entries per step).
__global__ __launch_bounds__(128) void csr_fill_kernel(const uint8_t *mask, int Nb,
                                                       const int32_t *row_ptr, int32_t *col_idx,
                                                       const int32_t *col_ptr, int32_t *row_idx) {
  const int i = blockIdx.x, slab = blockIdx.y;
  const uint8_t *m = mask + (int64_t)slab * Nb * Nb;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int32_t *ptr = wave == 0 ? row_ptr : col_ptr;
  int32_t *idx = wave == 0 ? col_idx : row_idx;
  if (ptr == nullptr) return;
  int o = ptr[(int64_t)slab * (Nb + 1) + i];
  idx += (int64_t)slab * Nb * Nb;
  for (int x0 = 0; x0 < Nb; x0 += 64) {
    const int x = x0 + lane;
    const bool f = x < Nb && (wave == 0 ? m[(int64_t)i * Nb + x] : m[(int64_t)x * Nb + i]) != 0;
    const unsigned long long b = __ballot(f);
    if (f) idx[o + __popcll(b & ((1ull << lane) - 1ull))] = x;
    o += __popcll(b);
  }
}

// The same in ONE kernel where a slab's mask fits in LDS (Nb <= 384).  kCsrParts workgroups per
// slab; each holds the whole mask (rows padded by 4 bytes, so that a walk down a column meets
// every bank once), counts every row and column (one thread each), scans the counts in a single
// wavefront and then fills its share of the lists (one wavefront per row or column, ballot
// compaction, so the lists come out ascending and the stores are coalesced).  The counting is
// repeated by every part of a slab: cheaper than a second launch and a trip through memory.
constexpr int kCsrLdsMaxNb = 384;
constexpr int kCsrParts = 16;
__global__ __launch_bounds__(1024) void csr_slab_kernel(const uint8_t *mask, int Nb, int32_t *row_ptr,
                                                        int32_t *col_idx, int32_t *col_ptr,
                                                        int32_t *row_idx) {
  extern __shared__ __align__(16) unsigned char csr_smem[];
  __shared__ int cnt[2][kCsrLdsMaxNb + 1];        // row counts, column counts -> exclusive offsets
  const int part = blockIdx.x, slab = blockIdx.y, tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int pitch = Nb + 4;
  const uint8_t *m = mask + (int64_t)slab * Nb * Nb;
  if ((Nb & 3) == 0 && (reinterpret_cast<uintptr_t>(mask) & 3) == 0) {   // four entries at a time
    const uint32_t *m4 = reinterpret_cast<const uint32_t *>(m);
    for (int t = tid; t < Nb * Nb / 4; t += 1024) {
      const int e = 4 * t;
      *reinterpret_cast<uint32_t *>(csr_smem + (e / Nb) * pitch + (e % Nb)) = m4[t];
    }
  } else {
    for (int t = tid; t < Nb * Nb; t += 1024) csr_smem[(t / Nb) * pitch + (t % Nb)] = m[t];
  }
  __syncthreads();
  const int n_dir = col_ptr ? 2 : 1;
  if (tid < n_dir * Nb) {                          // thread = one row (dir 0) or one column (dir 1)
    const int dir = tid / Nb, i = tid - dir * Nb;
    const unsigned char *src = csr_smem + (dir == 0 ? i * pitch : i);
    const int step = dir == 0 ? 1 : pitch;
    int n = 0;
    for (int x = 0; x < Nb; ++x) n += src[x * step] != 0;
    cnt[dir][i] = n;
  }
  __syncthreads();
  if (wave < n_dir) {                              // one wavefront per direction: exclusive scan
    int32_t *ptr = (wave == 0 ? row_ptr : col_ptr) + (int64_t)slab * (Nb + 1);
    int run = 0;
    for (int x0 = 0; x0 < Nb; x0 += 64) {
      const int x = x0 + lane;
      const int v = x < Nb ? cnt[wave][x] : 0;
      int inc = v;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_up(inc, off, 64);
        if (lane >= off) inc += o;
      }
      if (x < Nb) {
        cnt[wave][x] = run + inc - v;
        if (part == 0) ptr[x] = run + inc - v;
      }
      run += __shfl(inc, 63, 64);
    }
    if (part == 0 && lane == 0) ptr[Nb] = run;
  }
  __syncthreads();
  for (int item = part * 16 + wave; item < n_dir * Nb; item += 16 * kCsrParts) {
    const int dir = item / Nb, i = item - dir * Nb;
    int32_t *idx = (dir == 0 ? col_idx : row_idx) + (int64_t)slab * Nb * Nb;
    int o = cnt[dir][i];
    for (int x0 = 0; x0 < Nb; x0 += 64) {
      const int x = x0 + lane;
      const bool f = x < Nb && csr_smem[dir == 0 ? i * pitch + x : x * pitch + i] != 0;
      const unsigned long long b = __ballot(f);
      if (f) idx[o + __popcll(b & ((1ull << lane) - 1ull))] = x;
      o += __popcll(b);
    }
  }
}

hipError_t launch_csr(const Problem &pb, const uint8_t *mask, int32_t *row_ptr, int32_t *col_idx,
                      int32_t *col_ptr, int32_t *row_idx, hipStream_t st) {
  if (pb.Nb <= kCsrLdsMaxNb) {
    const int lds = pb.Nb * (pb.Nb + 4);
    hipError_t e0 = set_dynamic_lds_once(reinterpret_cast<const void *>(&csr_slab_kernel),
                                         kCsrLdsMaxNb * (kCsrLdsMaxNb + 4));
    if (e0 != hipSuccess) return e0;
    hipLaunchKernelGGL(csr_slab_kernel, dim3(kCsrParts, pb.n_slabs), dim3(1024), lds, st, mask, pb.Nb, row_ptr,
                       col_idx, col_ptr, row_idx);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(csr_count_kernel, dim3(pb.Nb, pb.n_slabs), dim3(128), 0, st, mask, pb.Nb,
                     row_ptr, col_ptr);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(csr_scan_kernel, dim3(pb.n_slabs, 2), dim3(256), 0, st, pb.Nb, row_ptr,
                     col_ptr);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(csr_fill_kernel, dim3(pb.Nb, pb.n_slabs), dim3(128), 0, st, mask, pb.Nb,
                     row_ptr, col_idx, col_ptr, row_idx);
  return hipGetLastError();
}

}  // namespace asa
