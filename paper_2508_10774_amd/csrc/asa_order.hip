// Order in which the workgroups of the attention kernels take their work items.
//
// The selection rule gives every query block its own number of key blocks (Alg. 3 step 9 of the
// paper), and the columns of the mask differ even more (31..220 query blocks at 25 % density on
// video-like inputs).  A long item that starts late ends the kernel late.  Each XCD keeps its
// contiguous share of the (slab, block) items (its workgroups share an L2) but works through it
// longest list first.  One workgroup per XCD share: bitonic sort of (length descending, item
// ascending) keys in LDS.  A share whose lists all have one length (a fixed budget per row) keeps
// its natural order and skips the sort.
#include "asa_common.hpp"

namespace asa {

constexpr int kOrderMax = 2048;   // items per XCD share that the sort handles

__global__ __launch_bounds__(1024) void length_order_kernel(const int32_t *ptr, int Nb, int total,
                                                            int32_t *order) {
  __shared__ uint64_t key[kOrderMax];
  const int share = (total + kNumXcd - 1) / kNumXcd;
  const int first = blockIdx.x * share;
  const int count = max(0, min(share, total - first));
  int uneven = 0;
  uint32_t len0 = 0;
  if (count > 0) {
    const int slab = first / Nb, b = first - slab * Nb;
    len0 = (uint32_t)(ptr[slab * (Nb + 1) + b + 1] - ptr[slab * (Nb + 1) + b]);
  }
  for (int t = threadIdx.x; t < kOrderMax; t += 1024) {
    uint64_t kk = ~0ull;                       // padding sorts last
    if (t < count) {
      const int item = first + t, slab = item / Nb, b = item - slab * Nb;
      const uint32_t len = (uint32_t)(ptr[slab * (Nb + 1) + b + 1] - ptr[slab * (Nb + 1) + b]);
      kk = ((uint64_t)(0xFFFFFFFFu - len) << 32) | (uint32_t)item;
      uneven |= len != len0;
    }
    key[t] = kk;
  }
  if (!__syncthreads_or(uneven)) {             // (also the barrier behind the key writes)
    for (int t = threadIdx.x; t < count; t += 1024) order[first + t] = first + t;
    return;
  }
  int n2 = 2;                                   // network size: the share, rounded up to a power of two
  while (n2 < count) n2 <<= 1;
  for (int size = 2; size <= n2; size <<= 1)
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      for (int t = threadIdx.x; t < n2 / 2; t += 1024) {
        const int lo = 2 * t - (t & (stride - 1));       // index with bit `stride` clear
        const int hi = lo + stride;
        const bool up = (lo & size) == 0;
        const uint64_t x = key[lo], y = key[hi];
        if ((x > y) == up) { key[lo] = y; key[hi] = x; }
      }
      __syncthreads();
    }
  for (int t = threadIdx.x; t < count; t += 1024) order[first + t] = (int32_t)(uint32_t)key[t];
}

bool length_order_fits(int total) { return (total + kNumXcd - 1) / kNumXcd <= kOrderMax; }

hipError_t launch_length_order(const int32_t *ptr, int Nb, int total, int32_t *order, hipStream_t st) {
  hipLaunchKernelGGL(length_order_kernel, dim3(kNumXcd), dim3(1024), 0, st, ptr, Nb, total, order);
  return hipGetLastError();
}

}  // namespace asa
