// Calls the host-only paths of libasa: every entry point with arguments that fail validation
// (so that nothing reaches the GPU), the size queries, the error strings and the Gilbert order
// (a host function).  Built by tests/test_sanitizers.py against a copy of the library whose HOST
// code is compiled with -fsanitize=address,undefined.  Prints "ok" at the end.
#include <cstdio>
#include <cstring>
#include <vector>

#include "asa.h"
#include "asa_bench.h"

#define EXPECT(cond) do { if (!(cond)) { std::printf("line %d: %s\n", __LINE__, #cond); return 1; } } while (0)

static asa_params base(int L, int d, int block) {
  asa_params p;
  std::memset(&p, 0, sizeof(p));
  p.B = 1; p.H = 2; p.L = L; p.d = d; p.block = block; p.k_samples = 16;
  p.tau = 0.9f; p.r_min = 0.f; p.r_max = 1.f;
  return p;
}

int main() {
  EXPECT(asa_version() == ASA_VERSION);
  for (int s = -6; s <= 0; ++s) EXPECT(asa_error_string(s) != nullptr && std::strlen(asa_error_string(s)) > 1);
  EXPECT(asa_last_hip_error() != nullptr);

  asa_params p = base(1000, 64, 64);
  EXPECT(asa_mask_workspace_bytes(&p) > 0 && asa_fwd_workspace_bytes(&p) > 0 && asa_bwd_workspace_bytes(&p) > 0);
  EXPECT(asa_mask_seeded_workspace_bytes(&p) > asa_mask_workspace_bytes(&p));
  EXPECT(asa_global_token_count(&p, 64) == 64 && asa_fwd_g_workspace_bytes(&p, 64) > 0 &&
         asa_bwd_g_workspace_bytes(&p, 64) > 0);
  EXPECT(asa_mask_workspace_bytes(nullptr) == 0);

  // parameters that validation must refuse, each alone
  {
    asa_params b = p; b.d = 96;               EXPECT(asa_fwd_workspace_bytes(&b) == 0);
    b = p; b.block = 32;                      EXPECT(asa_fwd_workspace_bytes(&b) == 0);
    b = p; b.L = 0;                           EXPECT(asa_fwd_workspace_bytes(&b) == 0);
    b = p; b.L = 64 * 1025;                   EXPECT(asa_fwd_workspace_bytes(&b) == 0);   // Nb > 1024
    b = p; b.k_samples = 0;                   EXPECT(asa_mask_workspace_bytes(&b) == 0);
    b = p; b.k_samples = 65;                  EXPECT(asa_mask_workspace_bytes(&b) == 0);
    b = p; b.r_min = 0.8f; b.r_max = 0.2f;    EXPECT(asa_mask_workspace_bytes(&b) == 0);
    b = p; b.tau = 0.f / 0.f;                 EXPECT(asa_mask_workspace_bytes(&b) == 0);
    b = p; b.n_prefix_dense = -1;             EXPECT(asa_mask_workspace_bytes(&b) == 0);
    b = p; b.scale = -1.f;                    EXPECT(asa_mask_workspace_bytes(&b) == 0);
    b = p; b.q_stride[0] = 64 * 2000; b.q_stride[1] = 64 * 1000; b.q_stride[2] = 60;   // row pitch < d
    EXPECT(asa_mask_workspace_bytes(&b) == 0);
    b = p; b.k_stride[0] = 3; b.k_stride[1] = 64 * 1000; b.k_stride[2] = 64;           // not a multiple of 8
    EXPECT(asa_mask_workspace_bytes(&b) == 0);
    const int32_t bad_offs[16] = {0, 4, 8, 12, 16, 20, 24, 28, 32, 36, 40, 44, 48, 52, 60, 56};
    b = p; b.sample_offsets = bad_offs;       EXPECT(asa_mask_workspace_bytes(&b) == 0);  // not ascending
    const int32_t good_offs[16] = {0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 63};
    b = p; b.sample_offsets = good_offs;      EXPECT(asa_mask_workspace_bytes(&b) > 0);
  }

  // null / misaligned pointers: refused before any HIP call (the fake addresses are never read)
  void *fake = reinterpret_cast<void *>(0x100000), *odd = reinterpret_cast<void *>(0x100002);
  uint8_t *fu = reinterpret_cast<uint8_t *>(fake);
  int32_t *fi = reinterpret_cast<int32_t *>(fake);
  float *ff = reinterpret_cast<float *>(fake);
  EXPECT(asa_build_mask(&p, nullptr, fake, fu, fi, fi, fi, fi, nullptr, fake, 1u << 30, nullptr) == ASA_ERR_INVALID_ARG);
  EXPECT(asa_build_mask(&p, fake, fake, fu, fi, fi, fi, nullptr, nullptr, fake, 1u << 30, nullptr) == ASA_ERR_INVALID_ARG);
  EXPECT(asa_build_mask(&p, odd, fake, fu, fi, fi, fi, fi, nullptr, fake, 1u << 30, nullptr) == ASA_ERR_INVALID_ARG);
  EXPECT(asa_build_mask(&p, fake, fake, fu, fi, fi, fi, fi, nullptr, fake, 16, nullptr) == ASA_ERR_WORKSPACE);
  EXPECT(asa_build_mask_seeded(&p, 7, fake, fake, fu, fi, fi, fi, fi, nullptr, nullptr, 0, nullptr) == ASA_ERR_WORKSPACE);
  EXPECT(asa_sample_offsets(&p, 7, nullptr, nullptr) == ASA_ERR_INVALID_ARG);
  EXPECT(asa_mask_from_scores(&p, nullptr, fu, nullptr) == ASA_ERR_INVALID_ARG);
  EXPECT(asa_csr_from_mask(&p, fu, fi, nullptr, nullptr, nullptr, nullptr) == ASA_ERR_INVALID_ARG);
  EXPECT(asa_attn_fwd(&p, fake, fake, fake, fi, nullptr, fake, nullptr, ff, fake, 1u << 30, nullptr) == ASA_ERR_INVALID_ARG);
  EXPECT(asa_attn_fwd(&p, fake, fake, fake, fi, fi, fake, nullptr, ff, fake, 16, nullptr) == ASA_ERR_WORKSPACE);
  EXPECT(asa_attn_bwd(&p, fake, fake, fake, fake, nullptr, fake, ff, fi, fi, fi, nullptr, fake, fake, fake, fake,
                      1u << 30, nullptr) == ASA_ERR_INVALID_ARG);
  EXPECT(asa_attn_bwd(&p, fake, fake, fake, fake, nullptr, fake, ff, fi, fi, fi, fi, fake, fake, fake, fake, 16,
                      nullptr) == ASA_ERR_WORKSPACE);
  EXPECT(asa_attn_bwd_noalloc(&p, fake, fake, fake, fake, nullptr, fake, ff, fi, fi, fi, fi, fake, fake, nullptr,
                              nullptr) == ASA_ERR_INVALID_ARG);
  {
    asa_params big = base(120000, 64, 128);
    big.H = 8;
    EXPECT(asa_attn_bwd_noalloc(&big, fake, fake, fake, fake, nullptr, fake, ff, nullptr, nullptr, nullptr, nullptr,
                                fake, fake, fake, nullptr) == ASA_ERR_TOO_LARGE);
  }
  EXPECT(asa_global_tokens(&p, 0, fake, fake, fake, fake, nullptr) == ASA_ERR_INVALID_ARG);
  EXPECT(asa_attn_fwd_g(&p, 64, fake, fake, fake, nullptr, fake, fi, fi, fake, nullptr, ff, fake, 1u << 30, nullptr) ==
         ASA_ERR_INVALID_ARG);
  EXPECT(asa_attn_bwd_g(&p, 64, fake, fake, fake, fake, fake, fake, nullptr, fake, ff, fi, fi, fi, fi, fake, fake,
                        fake, nullptr, 0, nullptr) == ASA_ERR_WORKSPACE);
  {
    const void *src[1] = {fake};
    void *dst[1] = {fake};
    EXPECT(asa_reorder_tokens(&p, 1, src, dst, nullptr, nullptr, fi, nullptr) == ASA_ERR_INVALID_ARG);  // in place
    EXPECT(asa_reorder_tokens(&p, 4, src, dst, nullptr, nullptr, fi, nullptr) == ASA_ERR_INVALID_ARG);
  }
  EXPECT(asa_mfma_rate_probe(0, 1, 0, 0, ff, nullptr, nullptr) == ASA_ERR_INVALID_ARG);
  EXPECT(asa_mfma_rate_probe(1, 1, 8, 0, ff, nullptr, nullptr) == ASA_ERR_INVALID_ARG);
  EXPECT(asa_add_rate_probe(1, 0, 1, 1, ff, nullptr, nullptr) == ASA_ERR_INVALID_ARG);
  EXPECT(asa_set_kernel_timing(fake, nullptr) == ASA_ERR_INVALID_ARG);
  EXPECT(asa_set_kernel_timing(nullptr, nullptr) == ASA_OK);
  EXPECT(asa_test_force_fwd_kernel(3) == ASA_ERR_INVALID_ARG && asa_test_force_fwd_kernel(0) == ASA_OK);

  // the Gilbert order is host code: a few grids, with and without leading tokens
  const int grids[][4] = {{1, 1, 1, 0}, {4, 16, 16, 0}, {3, 5, 7, 2}, {21, 30, 52, 0}, {13, 30, 45, 226}, {2, 2, 9, 0}};
  for (const auto &g : grids) {
    const int n = g[3] + g[0] * g[1] * g[2];
    std::vector<int32_t> order(n), inverse(n);
    EXPECT(asa_gilbert_order(g[0], g[1], g[2], g[3], order.data(), inverse.data()) == ASA_OK);
    for (int i = 0; i < n; ++i) EXPECT(order[i] >= 0 && order[i] < n && inverse[order[i]] == i);
    EXPECT(asa_gilbert_order(g[0], g[1], g[2], g[3], order.data(), nullptr) == ASA_OK);
  }
  EXPECT(asa_gilbert_order(0, 1, 1, 0, fi, nullptr) == ASA_ERR_INVALID_ARG);
  std::printf("ok\n");
  return 0;
}
