// C-ABI entry points of libasa: argument checks, defaults, workspace carving, launches.
#include <math.h>
#include <string.h>

#include <atomic>
#include <mutex>
#include <utility>
#include <vector>

#include "asa_bench.h"

#include "asa_common.hpp"

namespace asa {

static thread_local char g_hip_error[256] = "";

void set_hip_error(hipError_t e) {
  const char *s = hipGetErrorString(e);
  strncpy(g_hip_error, s ? s : "unknown HIP error", sizeof(g_hip_error) - 1);
  g_hip_error[sizeof(g_hip_error) - 1] = 0;
}

static thread_local hipEvent_t g_ev_start = nullptr, g_ev_stop = nullptr;

void timing_begin(hipStream_t st) {
  if (g_ev_start) (void)hipEventRecord(g_ev_start, st);
}
void timing_end(hipStream_t st) {
  if (g_ev_stop) (void)hipEventRecord(g_ev_stop, st);
  g_ev_start = nullptr;
  g_ev_stop = nullptr;
}

hipError_t set_dynamic_lds_once(const void *fn, int bytes) {
  static std::mutex mu;
  static std::vector<std::pair<const void *, int>> done;   // (kernel, device) pairs already set
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  std::lock_guard<std::mutex> lock(mu);
  for (const auto &d : done)
    if (d.first == fn && d.second == dev) return hipSuccess;
  e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess) done.emplace_back(fn, dev);
  return e;
}

static std::atomic<int> g_forced_fwd_kernel{0};
int forced_fwd_kernel() { return g_forced_fwd_kernel.load(std::memory_order_relaxed); }

static bool view_from(const int64_t st[3], const Problem &pb, TensorView *tv) {
  if (st[0] == 0 && st[1] == 0 && st[2] == 0) {
    tv->sL = pb.d;
    tv->sH = (int64_t)pb.L * pb.d;
    tv->sB = (int64_t)pb.H * pb.L * pb.d;
    return true;
  }
  if (st[2] < pb.d || st[0] < 0 || st[1] < 0) return false;
  if ((st[0] % 8) || (st[1] % 8) || (st[2] % 8)) return false;  // rows are read 16 bytes at a time
  if (st[2] >= ((int64_t)1 << 24)) return false;  // 64 rows of a tile within 32-bit byte offsets
  tv->sB = st[0];
  tv->sH = st[1];
  tv->sL = st[2];
  return true;
}

int resolve(const asa_params *p, Problem *o) {
  if (!p || !o) return ASA_ERR_INVALID_ARG;
  if (p->B < 1 || p->H < 1 || p->L < 1) return ASA_ERR_INVALID_ARG;
  if ((int64_t)p->B * p->H > 65535) return ASA_ERR_UNSUPPORTED;
  if (p->d != 64 && p->d != 128) return ASA_ERR_UNSUPPORTED;
  if (p->block != 64 && p->block != 128) return ASA_ERR_UNSUPPORTED;
  memset(o, 0, sizeof(*o));
  o->B = p->B; o->H = p->H; o->L = p->L; o->d = p->d; o->block = p->block;
  o->Nb = (p->L + p->block - 1) / p->block;
  if (o->Nb > kMaxNb) return ASA_ERR_UNSUPPORTED;
  o->Lpad = o->Nb * p->block;
  o->n_slabs = p->B * p->H;
  // sampling (Alg. 2 steps 1-3): k offsets inside a block, shared by every block
  if (p->k_samples < 1 || p->k_samples > p->block) return ASA_ERR_INVALID_ARG;
  // up to 16 samples per block (the probe's MFMA tile is 2 blocks x 16 samples), or all of them
  o->every_token = p->k_samples == p->block && p->k_samples > kMaxSamples;
  if (p->k_samples > kMaxSamples && !o->every_token) return ASA_ERR_UNSUPPORTED;
  o->ks = p->k_samples;
  int prev = -1;
  for (int u = 0; u < o->ks; ++u) {
    int off = p->sample_offsets ? p->sample_offsets[u] : u * (p->block / p->k_samples);
    if (off < 0 || off >= p->block) return ASA_ERR_INVALID_ARG;
    if (off <= prev) return ASA_ERR_INVALID_ARG;
    prev = off;
    if (u < kMaxSamples) o->offs[u] = off;   // (k = block leaves no choice: the offsets are 0 .. block - 1)
  }
  // rule parameters (Alg. 3 step 9)
  if (p->tau != p->tau) return ASA_ERR_INVALID_ARG;
  if (!(p->r_min >= 0.f) || !(p->r_max <= 1.f) || !(p->r_min <= p->r_max)) return ASA_ERR_INVALID_ARG;
  o->tau = p->tau;
  int lo = (int)ceil((double)p->r_min * (double)o->Nb);
  if (lo < 1) lo = 1;
  if (lo > o->Nb) lo = o->Nb;
  int hi = (int)floor((double)p->r_max * (double)o->Nb);
  if (hi < lo) hi = lo;
  if (hi > o->Nb) hi = o->Nb;
  o->m_min = lo;
  o->m_max = hi;
  if (p->n_prefix_dense < 0 || p->n_prefix_dense > p->L) return ASA_ERR_INVALID_ARG;
  o->n_prefix_blocks = (p->n_prefix_dense + p->block - 1) / p->block;
  if (p->scale != p->scale || p->scale < 0.f || isinf(p->scale)) return ASA_ERR_INVALID_ARG;
  o->scale = p->scale == 0.f ? 1.0f / sqrtf((float)p->d) : p->scale;
  if (!view_from(p->q_stride, *o, &o->q) || !view_from(p->k_stride, *o, &o->k) ||
      !view_from(p->v_stride, *o, &o->v) || !view_from(p->o_stride, *o, &o->o))
    return ASA_ERR_INVALID_ARG;
  return ASA_OK;
}

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
static bool aligned4(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 3) == 0; }
static size_t round256(size_t x) { return (x + 255) & ~(size_t)255; }

static size_t transposed_bytes(const Problem &pb) {
  return round256((size_t)pb.n_slabs * pb.d * pb.Lpad * sizeof(uint16_t));
}

static int finish(hipError_t e) {
  if (e == hipSuccess) return ASA_OK;
  set_hip_error(e);
  return ASA_ERR_HIP;
}

}  // namespace asa

using namespace asa;

extern "C" {

int asa_version(void) { return ASA_VERSION; }

const char *asa_error_string(int status) {
  switch (status) {
    case ASA_OK: return "ok";
    case ASA_ERR_INVALID_ARG: return "invalid argument";
    case ASA_ERR_UNSUPPORTED: return "unsupported size or (block, d) combination";
    case ASA_ERR_WORKSPACE: return "workspace missing or too small";
    case ASA_ERR_HIP: return "HIP runtime error (see asa_last_hip_error)";
    case ASA_ERR_TOO_LARGE: return "problem needs more scratch memory than the library's fixed array holds";
    default: return "unknown status";
  }
}

const char *asa_last_hip_error(void) { return g_hip_error; }

int asa_test_force_fwd_kernel(int which) {
  if (which < 0 || which > 2) return ASA_ERR_INVALID_ARG;
  g_forced_fwd_kernel.store(which, std::memory_order_relaxed);
  return ASA_OK;
}

int asa_set_kernel_timing(void *start_event, void *stop_event) {
  if ((start_event == nullptr) != (stop_event == nullptr)) return ASA_ERR_INVALID_ARG;
  g_ev_start = reinterpret_cast<hipEvent_t>(start_event);
  g_ev_stop = reinterpret_cast<hipEvent_t>(stop_event);
  return ASA_OK;
}

// Every token sampled (k = block): the probe runs on blocks of 16 tokens (its own tile size,
// offsets 0..15) and the map of the real blocks is the (block / 16)^2 max-pool of that map.
static Problem fine_problem(const Problem &pb) {
  Problem f = pb;
  f.block = kMaxSamples;
  f.Nb = (pb.L + kMaxSamples - 1) / kMaxSamples;
  f.Lpad = f.Nb * kMaxSamples;
  f.ks = kMaxSamples;
  f.every_token = false;
  for (int u = 0; u < kMaxSamples; ++u) f.offs[u] = u;
  return f;
}
static size_t scores_bytes(const Problem &pb) {
  return round256((size_t)pb.n_slabs * pb.Nb * pb.Nb * sizeof(float));
}

size_t asa_mask_workspace_bytes(const asa_params *p) {
  Problem pb;
  if (resolve(p, &pb) != ASA_OK) return 0;
  if (pb.every_token) {
    const Problem f = fine_problem(pb);
    if (f.Nb > kMaxNb) return 0;
    // the probe's workspace on the fine blocks, the fine map, the pooled map
    return round256(probe_workspace_bytes(f)) + scores_bytes(f) + scores_bytes(pb);
  }
  // the probe's per-row block maxima and soft-max statistics
  return round256(probe_workspace_bytes(pb));
}

static size_t fwd_order_bytes(const Problem &pb) {
  return round256((size_t)pb.n_slabs * pb.Nb * sizeof(int32_t));
}

size_t asa_fwd_workspace_bytes(const asa_params *p) {
  Problem pb;
  if (resolve(p, &pb) != ASA_OK) return 0;
  // V as [slab][Nb][d][block], then the order of the workgroups
  return transposed_bytes(pb) + fwd_order_bytes(pb);
}

size_t asa_bwd_workspace_bytes(const asa_params *p) {
  Problem pb;
  if (resolve(p, &pb) != ASA_OK) return 0;
  return bwd_workspace_bytes(pb);
}

static size_t table_bytes(const Problem &pb) {
  return round256((size_t)pb.n_slabs * pb.Nb * pb.ks);
}

static int build_mask_impl(const asa_params *p, const uint64_t *seed, const void *q, const void *k,
                           uint8_t *mask, int32_t *row_ptr, int32_t *col_idx, int32_t *col_ptr,
                           int32_t *row_idx, float *p_imp, void *workspace, size_t workspace_bytes,
                           void *hip_stream) {
  Problem pb;
  int rc = resolve(p, &pb);
  if (rc != ASA_OK) return rc;
  if (!q || !k || !mask || !row_ptr || !col_idx) return ASA_ERR_INVALID_ARG;
  if ((col_ptr == nullptr) != (row_idx == nullptr)) return ASA_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k) || !aligned4(row_ptr) || !aligned4(col_idx) ||
      !aligned4(col_ptr) || !aligned4(row_idx) || !aligned4(p_imp))
    return ASA_ERR_INVALID_ARG;
  if (pb.every_token && fine_problem(pb).Nb > kMaxNb) return ASA_ERR_UNSUPPORTED;   // L <= 16 * 1024 there
  const size_t base = asa_mask_workspace_bytes(p);
  if (!workspace || workspace_bytes < base + (seed ? table_bytes(pb) : 0) || !aligned16(workspace))
    return ASA_ERR_WORKSPACE;
  unsigned char *ws = reinterpret_cast<unsigned char *>(workspace);
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  if (pb.every_token) {
    // (a seed changes nothing here: every position of every block is in the sample)
    const Problem f = fine_problem(pb);
    float *fine = reinterpret_cast<float *>(ws + round256(probe_workspace_bytes(f)));
    float *scores = p_imp ? p_imp : reinterpret_cast<float *>(ws + round256(probe_workspace_bytes(f)) + scores_bytes(f));
    timing_begin(st);
    hipError_t e = launch_probe(f, q, k, workspace, st, nullptr);
    timing_end(st);
    if (e != hipSuccess) return finish(e);
    e = launch_finish_rule(f, workspace, fine, nullptr, nullptr, st);   // the fine map only, no rule
    if (e != hipSuccess) return finish(e);
    e = launch_pool_scores(fine, f.Nb, scores, pb.Nb, pb.block / kMaxSamples, pb.n_slabs, st);
    if (e != hipSuccess) return finish(e);
    e = launch_rule(pb, scores, mask, st);
    if (e != hipSuccess) return finish(e);
    return finish(launch_csr(pb, mask, row_ptr, col_idx, col_ptr, row_idx, st));
  }
  uint8_t *table = nullptr;
  if (seed) {
    table = ws + base;
    hipError_t e0 = launch_sample_offsets(pb, *seed, table, st);
    if (e0 != hipSuccess) return finish(e0);
  }
  timing_begin(st);
  hipError_t e = launch_probe(pb, q, k, workspace, st, table);
  timing_end(st);
  if (e != hipSuccess) return finish(e);
  e = launch_finish_rule(pb, workspace, p_imp, mask, table, st);
  if (e != hipSuccess) return finish(e);
  return finish(launch_csr(pb, mask, row_ptr, col_idx, col_ptr, row_idx, st));
}

int asa_build_mask(const asa_params *p, const void *q, const void *k, uint8_t *mask,
                   int32_t *row_ptr, int32_t *col_idx, int32_t *col_ptr, int32_t *row_idx,
                   float *p_imp, void *workspace, size_t workspace_bytes, void *hip_stream) {
  return build_mask_impl(p, nullptr, q, k, mask, row_ptr, col_idx, col_ptr, row_idx, p_imp, workspace,
                         workspace_bytes, hip_stream);
}

size_t asa_mask_seeded_workspace_bytes(const asa_params *p) {
  Problem pb;
  if (resolve(p, &pb) != ASA_OK) return 0;
  return asa_mask_workspace_bytes(p) + table_bytes(pb);
}

int asa_build_mask_seeded(const asa_params *p, uint64_t seed, const void *q, const void *k,
                          uint8_t *mask, int32_t *row_ptr, int32_t *col_idx, int32_t *col_ptr,
                          int32_t *row_idx, float *p_imp, void *workspace, size_t workspace_bytes,
                          void *hip_stream) {
  return build_mask_impl(p, &seed, q, k, mask, row_ptr, col_idx, col_ptr, row_idx, p_imp, workspace,
                         workspace_bytes, hip_stream);
}

int asa_sample_offsets(const asa_params *p, uint64_t seed, uint8_t *table, void *hip_stream) {
  Problem pb;
  int rc = resolve(p, &pb);
  if (rc != ASA_OK) return rc;
  if (!table) return ASA_ERR_INVALID_ARG;
  return finish(launch_sample_offsets(pb, seed, table, reinterpret_cast<hipStream_t>(hip_stream)));
}

int asa_mask_from_scores(const asa_params *p, const float *scores, uint8_t *mask,
                         void *hip_stream) {
  Problem pb;
  int rc = resolve(p, &pb);
  if (rc != ASA_OK) return rc;
  if (!scores || !mask || !aligned4(scores)) return ASA_ERR_INVALID_ARG;
  return finish(launch_rule(pb, scores, mask, reinterpret_cast<hipStream_t>(hip_stream)));
}

int asa_csr_from_mask(const asa_params *p, const uint8_t *mask, int32_t *row_ptr,
                      int32_t *col_idx, int32_t *col_ptr, int32_t *row_idx, void *hip_stream) {
  Problem pb;
  int rc = resolve(p, &pb);
  if (rc != ASA_OK) return rc;
  if (!mask || !row_ptr || !col_idx) return ASA_ERR_INVALID_ARG;
  if ((col_ptr == nullptr) != (row_idx == nullptr)) return ASA_ERR_INVALID_ARG;
  if (!aligned4(row_ptr) || !aligned4(col_idx) || !aligned4(col_ptr) || !aligned4(row_idx))
    return ASA_ERR_INVALID_ARG;
  return finish(launch_csr(pb, mask, row_ptr, col_idx, col_ptr, row_idx,
                           reinterpret_cast<hipStream_t>(hip_stream)));
}

int asa_attn_fwd(const asa_params *p, const void *q, const void *k, const void *v,
                 const int32_t *row_ptr, const int32_t *col_idx, void *o, void *o_lo, float *lse,
                 void *workspace, size_t workspace_bytes, void *hip_stream) {
  Problem pb;
  int rc = resolve(p, &pb);
  if (rc != ASA_OK) return rc;
  if (!q || !k || !v || !o || !lse) return ASA_ERR_INVALID_ARG;
  if ((row_ptr == nullptr) != (col_idx == nullptr)) return ASA_ERR_INVALID_ARG;   // both or neither (dense)
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(o_lo) ||
      !aligned4(lse) || !aligned4(row_ptr) || !aligned4(col_idx))
    return ASA_ERR_INVALID_ARG;
  if (!workspace || workspace_bytes < transposed_bytes(pb) + fwd_order_bytes(pb) || !aligned16(workspace))
    return ASA_ERR_WORKSPACE;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  hipError_t e = launch_transpose(pb, v, pb.v, workspace, st);
  if (e != hipSuccess) return finish(e);
  // rows of uneven length (the rule's own m per row): longest first inside each XCD's share
  int32_t *order = nullptr;
  if (row_ptr && length_order_fits(pb.n_slabs * pb.Nb)) {
    order = reinterpret_cast<int32_t *>(reinterpret_cast<char *>(workspace) + transposed_bytes(pb));
    e = launch_length_order(row_ptr, pb.Nb, pb.n_slabs * pb.Nb, order, st);
    if (e != hipSuccess) return finish(e);
  }
  timing_begin(st);
  e = launch_fwd(pb, q, k, workspace, row_ptr, col_idx, o, o_lo, lse, order, st);
  timing_end(st);
  return finish(e);
}

// ------------------------------------------------------------------ ASA_G (global tokens)
static int global_dims(const Problem &pb, int n, int *Lg, int *Nbg) {
  if (n < 1 || n > pb.L) return ASA_ERR_INVALID_ARG;
  *Lg = (pb.L + n - 1) / n;
  *Nbg = (*Lg + pb.block - 1) / pb.block;
  if (pb.Nb + *Nbg > kMaxNb) return ASA_ERR_UNSUPPORTED;
  return ASA_OK;
}
static size_t pooled_tile_bytes(const Problem &pb, int Nbg) {
  return round256((size_t)pb.n_slabs * Nbg * pb.block * pb.d * sizeof(uint16_t));
}
// the pooled tensors seen as a problem of their own (contiguous [B, H, Nbg * block, d])
static Problem pooled_problem(const Problem &pb, int Lg, int Nbg) {
  Problem g = pb;
  g.L = Lg;
  g.Nb = Nbg;
  g.Lpad = Nbg * pb.block;
  TensorView tv;
  tv.sL = pb.d;
  tv.sH = (int64_t)g.Lpad * pb.d;
  tv.sB = tv.sH * pb.H;
  g.q = g.k = g.v = g.o = tv;
  return g;
}

size_t asa_global_token_count(const asa_params *p, int n) {
  Problem pb;
  int Lg, Nbg;
  if (resolve(p, &pb) != ASA_OK || global_dims(pb, n, &Lg, &Nbg) != ASA_OK) return 0;
  return (size_t)Nbg * pb.block;
}

int asa_global_tokens(const asa_params *p, int n, const void *k, const void *v, void *kg, void *vg,
                      void *hip_stream) {
  Problem pb;
  int rc = resolve(p, &pb);
  if (rc != ASA_OK) return rc;
  int Lg, Nbg;
  rc = global_dims(pb, n, &Lg, &Nbg);
  if (rc != ASA_OK) return rc;
  if (!k || !v || !kg || !vg) return ASA_ERR_INVALID_ARG;
  if (!aligned16(k) || !aligned16(v) || !aligned16(kg) || !aligned16(vg)) return ASA_ERR_INVALID_ARG;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  hipError_t e = launch_pool(pb, n, k, pb.k, kg, st);
  if (e != hipSuccess) return finish(e);
  return finish(launch_pool(pb, n, v, pb.v, vg, st));
}

size_t asa_fwd_g_workspace_bytes(const asa_params *p, int n) {
  Problem pb;
  int Lg, Nbg;
  if (resolve(p, &pb) != ASA_OK || global_dims(pb, n, &Lg, &Nbg) != ASA_OK) return 0;
  return transposed_bytes(pb) + pooled_tile_bytes(pb, Nbg) + fwd_order_bytes(pb);
}

int asa_attn_fwd_g(const asa_params *p, int n, const void *q, const void *k, const void *v,
                   const void *kg, const void *vg, const int32_t *row_ptr, const int32_t *col_idx,
                   void *o, void *o_lo, float *lse, void *workspace, size_t workspace_bytes,
                   void *hip_stream) {
  Problem pb;
  int rc = resolve(p, &pb);
  if (rc != ASA_OK) return rc;
  int Lg, Nbg;
  rc = global_dims(pb, n, &Lg, &Nbg);
  if (rc != ASA_OK) return rc;
  if (!q || !k || !v || !kg || !vg || !o || !lse) return ASA_ERR_INVALID_ARG;
  if ((row_ptr == nullptr) != (col_idx == nullptr)) return ASA_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(kg) || !aligned16(vg) ||
      !aligned16(o) || !aligned16(o_lo) || !aligned4(lse) || !aligned4(row_ptr) || !aligned4(col_idx))
    return ASA_ERR_INVALID_ARG;
  if ((uint64_t)pb.Nb * pb.block * (uint64_t)pb.k.sL * 2u >= 0xFFFFFFFFull) return ASA_ERR_UNSUPPORTED;
  if (pb.k.sL != pb.d) return ASA_ERR_UNSUPPORTED;   // rows of K must be contiguous here
  if (!workspace || workspace_bytes < transposed_bytes(pb) + pooled_tile_bytes(pb, Nbg) + fwd_order_bytes(pb) ||
      !aligned16(workspace))
    return ASA_ERR_WORKSPACE;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  char *ws = reinterpret_cast<char *>(workspace);
  void *vgt = ws + transposed_bytes(pb);
  hipError_t e = launch_transpose(pb, v, pb.v, ws, st);
  if (e != hipSuccess) return finish(e);
  const Problem g = pooled_problem(pb, Lg, Nbg);
  e = launch_transpose(g, vg, g.v, vgt, st);
  if (e != hipSuccess) return finish(e);
  GlobalTokens gt;
  gt.n = n; gt.Lg = Lg; gt.Nbg = Nbg; gt.kg = kg; gt.vg = vg; gt.vgt = vgt;
  int32_t *order = nullptr;
  if (row_ptr && length_order_fits(pb.n_slabs * pb.Nb)) {
    order = reinterpret_cast<int32_t *>(ws + transposed_bytes(pb) + pooled_tile_bytes(pb, Nbg));
    e = launch_length_order(row_ptr, pb.Nb, pb.n_slabs * pb.Nb, order, st);
    if (e != hipSuccess) return finish(e);
  }
  timing_begin(st);
  e = launch_fwd(pb, q, k, ws, row_ptr, col_idx, o, o_lo, lse, order, st, &gt);
  timing_end(st);
  return finish(e);
}

size_t asa_bwd_g_workspace_bytes(const asa_params *p, int n) {
  Problem pb;
  int Lg, Nbg;
  if (resolve(p, &pb) != ASA_OK || global_dims(pb, n, &Lg, &Nbg) != ASA_OK) return 0;
  return bwd_g_workspace_bytes(pb, Nbg);
}

int asa_attn_bwd_g(const asa_params *p, int n, const void *q, const void *k, const void *v,
                   const void *kg, const void *vg, const void *o, const void *o_lo, const void *d_o,
                   const float *lse, const int32_t *row_ptr, const int32_t *col_idx,
                   const int32_t *col_ptr, const int32_t *row_idx, void *dq, void *dk, void *dv,
                   void *workspace, size_t workspace_bytes, void *hip_stream) {
  Problem pb;
  int rc = resolve(p, &pb);
  if (rc != ASA_OK) return rc;
  int Lg, Nbg;
  rc = global_dims(pb, n, &Lg, &Nbg);
  if (rc != ASA_OK) return rc;
  {
    const int n_lists = (row_ptr != nullptr) + (col_idx != nullptr) + (col_ptr != nullptr) + (row_idx != nullptr);
    if (n_lists != 0 && n_lists != 4) return ASA_ERR_INVALID_ARG;
  }
  if (!q || !k || !v || !kg || !vg || !o || !d_o || !lse || !dq || !dk || !dv) return ASA_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(kg) || !aligned16(vg) ||
      !aligned16(o) || !aligned16(o_lo) || !aligned16(d_o) || !aligned16(dq) || !aligned16(dk) ||
      !aligned16(dv) || !aligned4(lse) || !aligned4(row_ptr) || !aligned4(col_idx) ||
      !aligned4(col_ptr) || !aligned4(row_idx))
    return ASA_ERR_INVALID_ARG;
  if (!workspace || workspace_bytes < bwd_g_workspace_bytes(pb, Nbg) || !aligned16(workspace))
    return ASA_ERR_WORKSPACE;
  GlobalTokens gt;
  gt.n = n; gt.Lg = Lg; gt.Nbg = Nbg; gt.kg = kg; gt.vg = vg; gt.vgt = nullptr;
  return finish(launch_bwd(pb, q, k, v, o, o_lo, d_o, lse, row_ptr, col_idx, col_ptr, row_idx, dq, dk,
                           dv, workspace, reinterpret_cast<hipStream_t>(hip_stream), &gt));
}

// Argument checks of the backward that do not depend on where the scratch memory comes from.
static int check_bwd_args(const asa_params *p, Problem *pb, const void *q, const void *k,
                          const void *v, const void *o, const void *o_lo, const void *d_o,
                          const float *lse, const int32_t *row_ptr, const int32_t *col_idx,
                          const int32_t *col_ptr, const int32_t *row_idx, void *dq, void *dk,
                          void *dv) {
  int rc = resolve(p, pb);
  if (rc != ASA_OK) return rc;
  {
    const int n_lists = (row_ptr != nullptr) + (col_idx != nullptr) + (col_ptr != nullptr) + (row_idx != nullptr);
    if (n_lists != 0 && n_lists != 4) return ASA_ERR_INVALID_ARG;   // all four or none (dense)
  }
  if (!q || !k || !v || !o || !d_o || !lse ||
      !dq || !dk || !dv)
    return ASA_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(o_lo) ||
      !aligned16(d_o) ||
      !aligned16(dq) || !aligned16(dk) || !aligned16(dv) || !aligned4(lse) ||
      !aligned4(row_ptr) || !aligned4(col_idx) || !aligned4(col_ptr) || !aligned4(row_idx))
    return ASA_ERR_INVALID_ARG;
  return ASA_OK;
}

int asa_attn_bwd(const asa_params *p, const void *q, const void *k, const void *v, const void *o,
                 const void *o_lo, const void *d_o, const float *lse, const int32_t *row_ptr,
                 const int32_t *col_idx, const int32_t *col_ptr, const int32_t *row_idx, void *dq,
                 void *dk, void *dv, void *workspace, size_t workspace_bytes, void *hip_stream) {
  Problem pb;
  int rc = check_bwd_args(p, &pb, q, k, v, o, o_lo, d_o, lse, row_ptr, col_idx, col_ptr, row_idx, dq,
                          dk, dv);
  if (rc != ASA_OK) return rc;
  if (!workspace || workspace_bytes < bwd_workspace_bytes(pb) || !aligned16(workspace))
    return ASA_ERR_WORKSPACE;
  return finish(launch_bwd(pb, q, k, v, o, o_lo, d_o, lse, row_ptr, col_idx, col_ptr, row_idx, dq, dk,
                           dv, workspace, reinterpret_cast<hipStream_t>(hip_stream)));
}

// ------------------------------------------------ backward for callers that cannot allocate
// The backward's scratch memory (row statistics, dK / dV workgroup order) in a device array of
// the library itself.  Every GPU the library runs on holds its own copy at its own address;
// the name `scratch` is only a handle for hipGetSymbolAddress on the host side.
static __device__ __align__(256) unsigned char scratch[ASA_NOALLOC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[kMaxDevices];   // device address of `scratch` per device, 0 = not asked yet

static int scratch_of_current_device(void **out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return finish(e);
  if (dev < 0 || dev >= kMaxDevices) return ASA_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return finish(e);
    if (!ptr) return finish(hipErrorInvalidSymbol);
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return ASA_OK;
}

int asa_attn_bwd_noalloc(const asa_params *p, const void *q, const void *k, const void *v,
                         const void *o, const void *o_lo, const void *d_o, const float *lse,
                         const int32_t *row_ptr, const int32_t *col_idx, const int32_t *col_ptr,
                         const int32_t *row_idx, void *dq, void *dk, void *dv, void *hip_stream) {
  Problem pb;
  int rc = check_bwd_args(p, &pb, q, k, v, o, o_lo, d_o, lse, row_ptr, col_idx, col_ptr, row_idx, dq,
                          dk, dv);
  if (rc != ASA_OK) return rc;
  if (bwd_workspace_bytes(pb) > (size_t)ASA_NOALLOC_SCRATCH_BYTES) return ASA_ERR_TOO_LARGE;
  void *ws = nullptr;
  rc = scratch_of_current_device(&ws);
  if (rc != ASA_OK) return rc;
  // nothing in the scratch has to start at zero: the row-statistics kernel and the order kernel
  // write every word that the gradient kernels read
  return finish(launch_bwd(pb, q, k, v, o, o_lo, d_o, lse, row_ptr, col_idx, col_ptr, row_idx, dq, dk,
                           dv, ws, reinterpret_cast<hipStream_t>(hip_stream)));
}

int asa_gilbert_order(int32_t T, int32_t Y, int32_t X, int32_t n_prefix, int32_t *order,
                      int32_t *inverse) {
  if (!order || T < 1 || Y < 1 || X < 1 || n_prefix < 0) return ASA_ERR_INVALID_ARG;
  if ((int64_t)T * Y * X + n_prefix > ((int64_t)1 << 30)) return ASA_ERR_UNSUPPORTED;
  return gilbert_order(T, Y, X, n_prefix, order, inverse);
}

int asa_reorder_tokens(const asa_params *p, int32_t n_tensors, const void *const *src,
                       void *const *dst, const int64_t *src_stride, const int64_t *dst_stride,
                       const int32_t *index, void *hip_stream) {
  // only B, H, L, d of `p` have a meaning here: the other fields are not looked at
  if (!p) return ASA_ERR_INVALID_ARG;
  asa_params shape;
  memset(&shape, 0, sizeof(shape));
  shape.B = p->B; shape.H = p->H; shape.L = p->L; shape.d = p->d;
  shape.block = 128; shape.k_samples = 1; shape.tau = 0.5f; shape.r_max = 1.f;
  if ((int64_t)p->L > (int64_t)kMaxNb * 128) return ASA_ERR_UNSUPPORTED;
  Problem pb;
  int rc = resolve(&shape, &pb);
  if (rc != ASA_OK) return rc;
  if (n_tensors < 1 || n_tensors > 3 || !src || !dst || !index || !aligned4(index)) return ASA_ERR_INVALID_ARG;
  for (int t = 0; t < n_tensors; ++t) {
    if (!src[t] || !dst[t] || !aligned16(src[t]) || !aligned16(dst[t])) return ASA_ERR_INVALID_ARG;
    if (src[t] == dst[t]) return ASA_ERR_INVALID_ARG;  // not an in-place operation
  }
  const int64_t packed[3] = {0, 0, 0};
  TensorView ts, td;
  if (!view_from(src_stride ? src_stride : packed, pb, &ts) ||
      !view_from(dst_stride ? dst_stride : packed, pb, &td))
    return ASA_ERR_INVALID_ARG;
  return finish(launch_reorder(pb, n_tensors, src, dst, ts, td, index,
                               reinterpret_cast<hipStream_t>(hip_stream)));
}

int asa_mfma_rate_probe(int32_t workgroups, int32_t iters, int32_t idle_sleep, int32_t vector_stream,
                        float *sink, double *flop, void *hip_stream) {
  if (workgroups < 1 || workgroups > 65535 || iters < 1 || iters > (1 << 24) || idle_sleep < 0 ||
      idle_sleep > 7 || !sink || !aligned4(sink))
    return ASA_ERR_INVALID_ARG;
  const double matrix_waves = (idle_sleep > 0 || vector_stream) ? 4.0 : 8.0;
  if (flop) *flop = (double)workgroups * matrix_waves * 4.0 * (double)iters * (2.0 * 32 * 32 * 16);
  return finish(launch_mfma_rate(workgroups, iters, idle_sleep, vector_stream != 0, sink,
                                 reinterpret_cast<hipStream_t>(hip_stream)));
}

int asa_add_rate_probe(int32_t atomic, int32_t workgroups, int32_t tiles_per_workgroup, int32_t n_qblocks,
                       float *buf, double *bytes, void *hip_stream) {
  if (workgroups < 1 || workgroups > 65535 || tiles_per_workgroup < 1 || tiles_per_workgroup > 4096 ||
      n_qblocks < 1 || !buf || !aligned4(buf))
    return ASA_ERR_INVALID_ARG;
  if (bytes) *bytes = (double)workgroups * tiles_per_workgroup * 128.0 * 128.0 * 4.0;
  return finish(launch_add_rate(atomic != 0, workgroups, tiles_per_workgroup, n_qblocks, buf,
                                reinterpret_cast<hipStream_t>(hip_stream)));
}

}  // extern "C"
