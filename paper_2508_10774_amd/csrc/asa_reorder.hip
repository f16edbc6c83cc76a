// Token rearrangement along a Gilbert (generalised Hilbert) curve: Sec. 3.3 "Preprocessing and
// Importance Estimation" and Alg. 3 step 1.  The paper names the curve and cites it without a
// definition; the construction here is this library's own, built from three requirements: every
// cell once; unit steps wherever the chess-board parity of the grid allows them; the classical
// Hilbert curve on 2^k squares.  Host code makes the order, one gather kernel applies it.
#include <vector>

#include "asa_common.hpp"

namespace asa {

// ---------------------------------------------------------------------------------------
// host: the curve
// ---------------------------------------------------------------------------------------
namespace {

// A box edge: signed number of cells along one of the three grid axes.
struct Edge {
  int axis, len;
  int size() const { return len < 0 ? -len : len; }
  Edge part(int n) const { return Edge{axis, len < 0 ? -n : n}; }   // same direction, n cells
  Edge back(int n) const { return Edge{axis, len < 0 ? n : -n}; }   // opposite direction
};
struct Cell {
  int x[3];
  Cell along(Edge e, int k) const {  // k cells further in e's direction
    Cell c = *this;
    c.x[e.axis] += e.len < 0 ? -k : k;
    return c;
  }
};

// A walk in unit steps from a corner of an a x b x c box to the far end of its a-edge changes
// the chess-board colour a*b*c - 1 times and has to arrive on the colour of that corner.
bool clean(int a, int b, int c) {
  if (a == 1) return b == 1 && c == 1;
  return (a & 1) == 0 || ((b & 1) && (c & 1));
}

// cut positions of an axis of n cells, nearest the middle first, at most four
int cut_positions(int n, int out[4]) {
  int cnt = 0;
  const int lo = (n - 1) / 2, hi = n / 2 + 1;  // the middle pair of an odd n
  if (!(n & 1)) {
    if (n / 2 >= 1 && n / 2 <= n - 1) out[cnt++] = n / 2;
    for (int k = 1; cnt < 4; ++k) {
      const int l = n / 2 - k, r = n / 2 + k;
      if (l < 1) break;
      out[cnt++] = l;
      if (cnt < 4 && r <= n - 1) out[cnt++] = r;
    }
  } else {
    for (int k = 0; cnt < 4; ++k) {
      const int l = lo - k, r = hi + k;
      if (l < 1) break;
      out[cnt++] = l;
      if (cnt < 4 && r <= n - 1) out[cnt++] = r;
    }
  }
  return cnt;
}

enum Cut { kWide = 0, kUB = 1, kUC = 2, k3D = 3 };
struct Choice {
  Cut kind;
  int a1, m1, c1;  // m1: cut of B (kUB, k3D) or of C (kUC)
};

int unclean_pieces(Cut kind, int a, int b, int c, int a1, int m1, int c1) {
  switch (kind) {
    case kWide: return !clean(a1, b, c) + !clean(a - a1, b, c);
    case kUB: return !clean(m1, a1, c) + !clean(a, b - m1, c) + !clean(m1, a - a1, c);
    case kUC: return !clean(m1, a1, b) + !clean(a, c - m1, b) + !clean(m1, a - a1, b);
    default:
      return !clean(m1, c1, a1) + !clean(c, a1, b - m1) + !clean(a, m1, c - c1) +
             !clean(c, b - m1, a - a1) + !clean(m1, a - a1, c1);
  }
}

Choice choose_cut(int a, int b, int c) {
  const int longest = a > b ? (a > c ? a : c) : (b > c ? b : c);
  const bool b_long = b >= 2 && 3 * b >= 2 * longest;
  const bool c_long = c >= 2 && 3 * c >= 2 * longest;
  const Cut first = (b_long && c_long) ? k3D : b_long ? kUB : c_long ? kUC : kWide;
  Cut order[4] = {first, kWide, kUB, kUC};
  {
    int n = 1;
    for (int k = 0; k < 4; ++k)
      if ((Cut)k != first) order[n++] = (Cut)k;
  }
  int ca[4], cb[4], cc[4];
  const int na = cut_positions(a, ca), nb = cut_positions(b, cb), nc = cut_positions(c, cc);
  Choice best{kWide, 1, 0, 0};
  int best_unclean = 1 << 30;
  const int one[1] = {0};
  for (Cut kind : order) {
    // the second and third loop run over one dummy value where the kind has no such cut
    const int *l2 = kind == kUB || kind == k3D ? cb : kind == kUC ? cc : one;
    const int n2 = kind == kUB || kind == k3D ? nb : kind == kUC ? nc : 1;
    const int *l3 = kind == k3D ? cc : one;
    const int n3 = kind == k3D ? nc : 1;
    for (int i = 0; i < na; ++i)
      for (int j = 0; j < n2; ++j)
        for (int l = 0; l < n3; ++l) {
          const int u = unclean_pieces(kind, a, b, c, ca[i], l2[j], l3[l]);
          if (u < best_unclean) {
            best_unclean = u;
            best = Choice{kind, ca[i], l2[j], l3[l]};
            if (u == 0) return best;
          }
        }
  }
  return best;
}

struct Walker {
  int Y, X;
  int32_t base;
  int32_t *out;
  int64_t n = 0;

  void walk(Cell p, Edge A, Edge B, Edge C) {
    const int a = A.size(), b = B.size(), c = C.size();
    if (b == 1 && c == 1) {
      for (int i = 0; i < a; ++i) {
        const Cell q = p.along(A, i);
        out[n++] = base + (q.x[0] * Y + q.x[1]) * X + q.x[2];
      }
      return;
    }
    if (a == 1) {  // cannot end where it starts: take the longest side as the major axis
      if (b >= c) walk(p, B, C, A);
      else walk(p, C, B, A);
      return;
    }
    const Choice ch = choose_cut(a, b, c);
    const int a1 = ch.a1, a2 = a - a1;
    if (ch.kind == kWide) {
      walk(p, A.part(a1), B, C);
      walk(p.along(A, a1), A.part(a2), B, C);
    } else if (ch.kind == kUB || ch.kind == kUC) {
      const Edge M = ch.kind == kUB ? B : C, N = ch.kind == kUB ? C : B;
      const int m1 = ch.m1, m2 = M.size() - m1;
      walk(p, M.part(m1), A.part(a1), N);                               // up the near corner
      walk(p.along(M, m1), A, M.part(m2), N);                           // across the far strip
      walk(p.along(A, a - 1).along(M, m1 - 1), M.back(m1), A.back(a2), N);  // down the far corner
    } else {
      const int b1 = ch.m1, b2 = b - b1, c1 = ch.c1, c2 = c - c1;
      walk(p, B.part(b1), C.part(c1), A.part(a1));
      walk(p.along(B, b1), C, A.part(a1), B.part(b2));
      walk(p.along(B, b1 - 1).along(C, c - 1), A, B.back(b1), C.back(c2));
      walk(p.along(A, a - 1).along(B, b1).along(C, c - 1), C.back(c), B.part(b2), A.back(a2));
      walk(p.along(A, a - 1).along(B, b1 - 1), B.back(b1), A.back(a2), C.part(c1));
    }
  }
};

}  // namespace

int gilbert_order(int T, int Y, int X, int n_prefix, int32_t *order, int32_t *inverse) {
  const int dims[3] = {T, Y, X};
  // major axis: the longest of even length (the whole grid is then `clean`); all odd: the longest
  int major = -1;
  for (int pass = 0; pass < 2 && major < 0; ++pass)
    for (int i = 0; i < 3; ++i) {
      if (pass == 0 && (dims[i] & 1)) continue;
      if (major < 0 || dims[i] > dims[major]) major = i;
    }
  int second = -1, third = -1;
  for (int i = 0; i < 3; ++i) {
    if (i == major) continue;
    if (second < 0) second = i;
    else if (dims[i] > dims[second]) { third = second; second = i; }
    else third = i;
  }
  for (int i = 0; i < n_prefix; ++i) order[i] = i;
  Walker w{Y, X, n_prefix, order + n_prefix};
  w.walk(Cell{{0, 0, 0}}, Edge{major, dims[major]}, Edge{second, dims[second]}, Edge{third, dims[third]});
  const int64_t L = (int64_t)n_prefix + (int64_t)T * Y * X;
  if (w.n != L - n_prefix) return ASA_ERR_INVALID_ARG;  // (cannot happen: the pieces tile the box)
  if (inverse)
    for (int64_t i = 0; i < L; ++i) inverse[order[i]] = (int32_t)i;
  return ASA_OK;
}

// ---------------------------------------------------------------------------------------
// device: gather of token rows, dst[.., i, :] = src[.., index[i], :], up to three tensors per
// launch (Q, K, V).  HBM bound: 2 * d * 2 bytes per row and tensor.  A row of d bf16 is moved by
// d / 8 lanes as 16-byte pieces; a workgroup of 256 threads moves kRowsPerWg rows, all loads
// issued before the first store.
// ---------------------------------------------------------------------------------------
struct ReorderArgs {
  const void *src[3];
  void *dst[3];
  const int32_t *index;
  TensorView ts, td;
  int H, L;
};

template <int D>
__global__ __launch_bounds__(256) void reorder_kernel(ReorderArgs a) {
  constexpr int kLanesPerRow = D / 8;
  constexpr int kRowsPerPass = 256 / kLanesPerRow;
  constexpr int kPasses = 4;
  const int slab = blockIdx.y, t = blockIdx.z;
  const int bi = slab / a.H, h = slab % a.H;
  const char *src = reinterpret_cast<const char *>(a.src[t]) + (bi * a.ts.sB + h * a.ts.sH) * 2;
  char *dst = reinterpret_cast<char *>(a.dst[t]) + (bi * a.td.sB + h * a.td.sH) * 2;
  const int piece = threadIdx.x % kLanesPerRow;
  const int row0 = blockIdx.x * (kRowsPerPass * kPasses) + threadIdx.x / kLanesPerRow;
  uint4 val[kPasses];
#pragma unroll
  for (int i = 0; i < kPasses; ++i) {
    const int row = row0 + i * kRowsPerPass;
    val[i] = uint4{0, 0, 0, 0};
    if (row < a.L) {
      const int from = a.index[row];
      // (an entry outside [0, L) gives a zero row instead of a wild read)
      if ((unsigned)from < (unsigned)a.L)
        val[i] = *reinterpret_cast<const uint4 *>(src + (int64_t)from * a.ts.sL * 2 + piece * 16);
    }
  }
#pragma unroll
  for (int i = 0; i < kPasses; ++i) {
    const int row = row0 + i * kRowsPerPass;
    if (row < a.L) *reinterpret_cast<uint4 *>(dst + (int64_t)row * a.td.sL * 2 + piece * 16) = val[i];
  }
}

hipError_t launch_reorder(const Problem &pb, int n_tensors, const void *const *src, void *const *dst,
                          const TensorView &ts, const TensorView &td, const int32_t *index,
                          hipStream_t st) {
  ReorderArgs a{};
  for (int t = 0; t < n_tensors; ++t) {
    a.src[t] = src[t];
    a.dst[t] = dst[t];
  }
  a.index = index;
  a.ts = ts;
  a.td = td;
  a.H = pb.H;
  a.L = pb.L;
  const int rows_per_wg = (256 / (pb.d / 8)) * 4;
  const dim3 grid((pb.L + rows_per_wg - 1) / rows_per_wg, pb.n_slabs, n_tensors);
  timing_begin(st);
  if (pb.d == 128) hipLaunchKernelGGL(reorder_kernel<128>, grid, dim3(256), 0, st, a);
  else hipLaunchKernelGGL(reorder_kernel<64>, grid, dim3(256), 0, st, a);
  timing_end(st);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Calibration kernel for benchmarks: nothing but independent 32x32x16 bf16 MFMAs, so that a
// report can put the rate the matrix cores sustain on this device and at its clocks next to the
// published peak.  16 accumulators per wavefront are four independent chains; results are
// stored so that nothing is optimised away.
// SLEEP = 0, VEC = false: all 8 wavefronts of a workgroup run the MFMA loop (two per SIMD).
// SLEEP > 0: only wavefronts 0..3 do (one per SIMD) and pause for s_sleep SLEEP behind every 16
// MFMAs, which sets the duty cycle of the matrix pipes; the others leave at once.
// VEC: wavefronts 4..7 run a stream of exponentials and multiply-adds beside the MFMA loop of
// wavefronts 0..3 (at the higher priority, as in the attention kernels) until those have finished.
// What the shader clock does in each case shows how far the device's power limit takes back what
// a denser schedule of the matrix pipes gains.
// ---------------------------------------------------------------------------------------
template <int SLEEP, bool VEC>
__global__ __launch_bounds__(512) void mfma_rate_kernel(int iters, float *sink) {
  __shared__ volatile int finished;   // matrix wavefronts that have left their loop (VEC only)
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  if (VEC) {
    if (threadIdx.x == 0) finished = 0;
    __syncthreads();
  }
  if ((SLEEP > 0 || VEC) && wave >= 4) {
    float r = 0.f;
    if (VEC) {
      __builtin_amdgcn_s_setprio(3);
      float x[16];
      int blocks = 0;
#pragma unroll
      for (int i = 0; i < 16; ++i) x[i] = 0.5f + (float)(threadIdx.x & 63) * 0.001f + (float)i * 0.01f;
      // at most one block of arithmetic per 4 MFMAs of the matrix wavefronts: the loop ends with
      // theirs (looked up every eighth block), or by its own count if they are somehow slower
      for (int it = 0; it < iters; it += 8) {
        for (int u = 0; u < 8; ++u) {
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(x[i], 0.999f, -0.3f));
            r += e;
            x[i] = __builtin_fmaf(fmaxf(__builtin_fmaf(e, 0.5f, 0.1f), x[(i + 1) & 15] * 0.97f), 0.99f, 0.002f);
          }
        }
        blocks += 8;
        if (finished >= 4) break;
      }
      r += x[3];
      if (threadIdx.x == 256) r = (float)blocks;   // how far the stream got beside the MFMA loops
    }
    sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = r;
    return;
  }
  if (VEC) __builtin_amdgcn_s_setprio(0);
  // four different operand pairs of pseudo-random bf16 values in [-1, 1): consecutive MFMAs see
  // different data, as they do in a real kernel (identical operands switch far fewer gates and
  // let the clock run higher than any real kernel's)
  bf16x8 a[4], b[4];
  uint32_t h = 0x9E3779B9u * (threadIdx.x + 1u) + 0x85EBCA6Bu * (blockIdx.x + 1u);
#pragma unroll
  for (int c = 0; c < 4; ++c)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      h = h * 1664525u + 1013904223u;
      a[c][i] = (bf16)((float)(int)(h >> 16 & 0xFFFF) * (1.0f / 32768.0f) - 1.0f);
      h = h * 1664525u + 1013904223u;
      b[c][i] = (bf16)((float)(int)(h >> 16 & 0xFFFF) * (1.0f / 32768.0f) - 1.0f);
    }
  f32x16 acc[4];
#pragma unroll
  for (int c = 0; c < 4; ++c)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[c][i] = 0.f;
  const long long t0 = clock64(), w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int c = 0; c < 4; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[c], b[c], acc[c], 0, 0, 0);
    if (SLEEP > 0 && (it & 3) == 3) __builtin_amdgcn_s_sleep(SLEEP);
  }
  const long long t1 = clock64(), w1 = wall_clock64();
  if (VEC && (threadIdx.x & 63) == 0) atomicAdd(const_cast<int *>(&finished), 1);
  float r = 0.f;
#pragma unroll
  for (int c = 0; c < 4; ++c) r += acc[c][0] + acc[c][15];
  // lane 0 of wavefront 0 reports shader-clock cycles and 100 MHz wall ticks of its loop instead
  if (threadIdx.x == 0) r = (float)(t1 - t0);
  if (threadIdx.x == 1) r = (float)(w1 - w0);
  sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = r;
}

// launches grid x 512 threads; each wavefront that runs the MFMA loop issues 4 * iters MFMAs of
// 2 * 32 * 32 * 16 FLOP.  idle_sleep in 0..7 (the argument of s_sleep behind every 16 MFMAs).
hipError_t launch_mfma_rate(int grid, int iters, int idle_sleep, bool vector_stream, float *sink, hipStream_t st) {
  timing_begin(st);
#define ASA_RATE_CASE(S)                                                                                     \
  case S:                                                                                                    \
    if (vector_stream) hipLaunchKernelGGL((mfma_rate_kernel<S, true>), dim3(grid), dim3(512), 0, st, iters, sink); \
    else hipLaunchKernelGGL((mfma_rate_kernel<S, false>), dim3(grid), dim3(512), 0, st, iters, sink);        \
    break;
  switch (idle_sleep) {
    ASA_RATE_CASE(0) ASA_RATE_CASE(1) ASA_RATE_CASE(2) ASA_RATE_CASE(3)
    ASA_RATE_CASE(4) ASA_RATE_CASE(5) ASA_RATE_CASE(6) ASA_RATE_CASE(7)
    default: timing_end(st); return hipErrorInvalidValue;
  }
#undef ASA_RATE_CASE
  timing_end(st);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Calibration: fp32 atomic adds in the pattern that a backward with ONE pass over the tiles would
// need for dQ (every workgroup adds 128 x 128 fp32 tiles to pseudo-randomly chosen query blocks
// of a [n_qblocks][128][128] buffer, as the key blocks of a mask column do), or the same bytes
// as plain stores.  The eight XCDs of the device have separate L2 caches, so device-scope atomics
// are resolved beyond them; the rate this kernel reaches decides whether such a backward can pay.
// ---------------------------------------------------------------------------------------
template <bool ATOMIC>
__global__ __launch_bounds__(256) void add_rate_kernel(float *buf, int tiles_per_wg, int n_qblocks) {
  const int wg = blockIdx.x;
  for (int t = 0; t < tiles_per_wg; ++t) {
    unsigned h = (unsigned)(wg * 2654435761u) ^ (unsigned)(t * 40503u + 12345u);
    h ^= h >> 13; h *= 0x5bd1e995u; h ^= h >> 15;
    float *tile = buf + (size_t)(h % (unsigned)n_qblocks) * 128 * 128;
    for (int e = threadIdx.x; e < 128 * 128; e += 256) {
      const float v = 1.0f + (float)(e & 7);
      if (ATOMIC) unsafeAtomicAdd(tile + e, v);     // the hardware's fp32 add, no compare-and-swap loop
      else tile[e] = v;
    }
  }
}

hipError_t launch_add_rate(bool atomic, int grid, int tiles_per_wg, int n_qblocks, float *buf, hipStream_t st) {
  timing_begin(st);
  if (atomic) hipLaunchKernelGGL(add_rate_kernel<true>, dim3(grid), dim3(256), 0, st, buf, tiles_per_wg, n_qblocks);
  else hipLaunchKernelGGL(add_rate_kernel<false>, dim3(grid), dim3(256), 0, st, buf, tiles_per_wg, n_qblocks);
  hipError_t e = hipGetLastError();
  timing_end(st);
  return e;
}

}  // namespace asa
