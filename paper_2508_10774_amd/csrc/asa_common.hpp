// Shared declarations of the libasa translation units (host side + device helpers).
// gfx950 only: 64-wide wavefronts, bf16 MFMA 32x32x16 / 16x16x32.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "asa.h"

namespace asa {

typedef __bf16 bf16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;  // one 16-byte load / store

constexpr int kMaxNb = 1024;
constexpr int kMaxSamples = 16;
constexpr int kNumXcd = 8;

// A [B, H, L, d] bf16 tensor seen from the device: element strides of B, H, L.
struct TensorView {
  int64_t sB, sH, sL;
};

// Parameters after validation and defaulting; passed by value to kernels.
struct Problem {
  int B, H, L, d, block;
  int Nb;        // ceil(L / block)
  int Lpad;      // Nb * block
  int n_slabs;   // B * H
  int ks;        // samples per block
  bool every_token;  // ks == block > kMaxSamples: every token is sampled (the exact map of Sec. 3.3 Step 1)
  int n_prefix_blocks;
  int m_min, m_max;
  float tau;
  float scale;
  TensorView q, k, v, o;
  int offs[kMaxSamples];
};

int resolve(const asa_params *p, Problem *out);  // asa_status
void set_hip_error(hipError_t e);

// One-shot profiling hook (asa_set_kernel_timing): record the armed events around the dominant
// kernel of a call.  timing_begin / timing_end are no-ops when nothing is armed.
void timing_begin(hipStream_t st);
void timing_end(hipStream_t st);

// hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes), issued once per
// (kernel, device) under a lock; later calls only look the pair up.
hipError_t set_dynamic_lds_once(const void *fn, int bytes);
// Which forward kernel the tests asked for (asa_test_force_fwd_kernel): 0 = the library's own
// choice, 1 = the lock-step kernel, 2 = the ping-pong kernel.
int forced_fwd_kernel();

// launchers (each returns a hipError_t from the launch)
hipError_t launch_transpose(const Problem &pb, const void *src, const TensorView &tv, void *dst,
                            hipStream_t st);
// Global tokens of ASA_G as the attention kernels see them (all device pointers).
struct GlobalTokens {
  int n;              // pooling window
  int Lg, Nbg;        // pooled tokens per slab; key blocks they fill (rows padded to Nbg * block)
  const void *kg;     // [slab][Nbg * block][d] bf16
  const void *vg;     // [slab][Nbg * block][d] bf16
  const void *vgt;    // [slab][Nbg][d][block] bf16, transposed tiles of vg (workspace)
};
hipError_t launch_pool(const Problem &pb, int n, const void *src, const TensorView &tv, void *dst,
                       hipStream_t st);
hipError_t launch_fwd(const Problem &pb, const void *q, const void *k, const void *vt,
                      const int32_t *row_ptr, const int32_t *col_idx, void *o, void *o_lo,
                      float *lse, const int32_t *order, hipStream_t st, const GlobalTokens *gt = nullptr);
hipError_t launch_csr(const Problem &pb, const uint8_t *mask, int32_t *row_ptr, int32_t *col_idx,
                      int32_t *col_ptr, int32_t *row_idx, hipStream_t st);
// first sweep of the probe (block-row maxima and soft-max statistics into the workspace) ...
hipError_t launch_probe(const Problem &pb, const void *q, const void *k, void *workspace,
                        hipStream_t st, const uint8_t *table = nullptr);
// ... and its second sweep fused with the rule: P_imp rows (written if p_imp is not null) -> mask
hipError_t launch_finish_rule(const Problem &pb, void *workspace, float *p_imp, uint8_t *mask,
                              const uint8_t *table, hipStream_t st);
int gilbert_order(int T, int Y, int X, int n_prefix, int32_t *order, int32_t *inverse);  // asa_status; host
hipError_t launch_reorder(const Problem &pb, int n_tensors, const void *const *src, void *const *dst,
                          const TensorView &ts, const TensorView &td, const int32_t *index,
                          hipStream_t st);
hipError_t launch_mfma_rate(int grid, int iters, int idle_sleep, bool vector_stream, float *sink, hipStream_t st);
hipError_t launch_add_rate(bool atomic, int grid, int tiles_per_wg, int n_qblocks, float *buf, hipStream_t st);
hipError_t launch_sample_offsets(const Problem &pb, uint64_t seed, uint8_t *table, hipStream_t st);
size_t probe_workspace_bytes(const Problem &pb);
hipError_t launch_rule(const Problem &pb, const float *scores, uint8_t *mask, hipStream_t st);
// dst[s][i][j] = max over the g x g block of src[s][i*g .. ][j*g .. ] (src rows/columns past n_src
// do not exist): the importance map of blocks of g * 16 tokens from the map of 16-token blocks
hipError_t launch_pool_scores(const float *src, int n_src, float *dst, int n_dst, int g, int n_slabs,
                              hipStream_t st);
hipError_t launch_bwd(const Problem &pb, const void *q, const void *k, const void *v,
                      const void *o, const void *o_lo, const void *d_o, const float *lse,
                      const int32_t *row_ptr,
                      const int32_t *col_idx, const int32_t *col_ptr, const int32_t *row_idx,
                      void *dq, void *dk, void *dv, void *workspace, hipStream_t st,
                      const GlobalTokens *gt = nullptr);
size_t bwd_workspace_bytes(const Problem &pb);
// order[w] = work item of workgroup slot w: inside each XCD's contiguous share of the
// total = n_slabs * Nb (slab, block) items, longest list first (ptr = row_ptr or col_ptr of all
// slabs).  Only where a share holds at most as many items as the sort takes (length_order_fits).
bool length_order_fits(int total);
hipError_t launch_length_order(const int32_t *ptr, int Nb, int total, int32_t *order, hipStream_t st);
size_t bwd_g_workspace_bytes(const Problem &pb, int Nbg);

#ifdef __HIPCC__
// ---------------------------------------------------------------- device helpers

__device__ __forceinline__ const bf16 *slab_ptr(const void *base, const TensorView &tv, int slab,
                                                int H) {
  int b = slab / H, h = slab - b * H;
  return reinterpret_cast<const bf16 *>(base) + (int64_t)b * tv.sB + (int64_t)h * tv.sH;
}
__device__ __forceinline__ bf16 *slab_ptr(void *base, const TensorView &tv, int slab, int H) {
  int b = slab / H, h = slab - b * H;
  return reinterpret_cast<bf16 *>(base) + (int64_t)b * tv.sB + (int64_t)h * tv.sH;
}

// Workgroups are handed to the 8 XCDs round-robin by their linear id.  Give each XCD one
// contiguous range of work items, so that the workgroups sharing an L2 work on the same slab.
__device__ __forceinline__ int xcd_contiguous_work(int wg, int total) {
  int chunk = (total + kNumXcd - 1) / kNumXcd;
  int w = (wg % kNumXcd) * chunk + wg / kNumXcd;
  return (wg / kNumXcd < chunk && w < total) ? w : -1;
}
inline int xcd_grid(int total) { return ((total + kNumXcd - 1) / kNumXcd) * kNumXcd; }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  f32x2 v = {lo, hi};
  bf16x2 r = __builtin_convertvector(v, bf16x2);
  return *reinterpret_cast<uint32_t *>(&r);
}

__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits16) {
  return __builtin_bit_cast(float, bits16 << 16);
}

// value of the other 32-lane half of the wavefront
__device__ __forceinline__ float swap_halves(float x) { return __shfl_xor(x, 32, 64); }
// max over the two 32-lane halves (lane i and lane i + 32), in every lane, by the register-file
// lane swap of gfx950: v_permlane32_swap(a, b) exchanges the upper half of a with the lower half
// of b; applied to two copies of x it leaves (x.lo, x.lo) and (x.hi, x.hi).  No trip through the
// LDS crossbar, whose queue the matrix wavefronts keep full.
__device__ __forceinline__ float max_of_halves(float x) {
#if defined(__HIP_DEVICE_COMPILE__)
  uint32_t a = __builtin_bit_cast(uint32_t, x), b = a;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
  return fmaxf(__builtin_bit_cast(float, a), __builtin_bit_cast(float, b));
#else
  return x;
#endif
}
#endif

}  // namespace asa
