// Host-side checks of liblsq's C ABI that need no GPU, meant to be built with AddressSanitizer and
// UndefinedBehaviorSanitizer on the host code (tests/test_host_sanitizers.py does that): header parsing, the
// max-shape memory plan and every error path that must return before any device work, fed with valid,
// truncated, corrupted and randomly damaged model headers.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "../include/lsq.h"

static int failures = 0;
#define EXPECT(cond)                                                        \
  do {                                                                      \
    if (!(cond)) { std::printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond); ++failures; } \
  } while (0)

// a header as the blob format defines it (256 bytes, little endian), total = what the shapes add up to when asked
static std::vector<unsigned char> header(int arch, int n_enc, int n_dec, int d, int H, int F, int V, int dtype,
                                         uint64_t total) {
  std::vector<unsigned char> h(256, 0);
  std::memcpy(h.data(), "LSQBLOB1", 8);
  int32_t f[17] = {1, arch, n_enc, n_dec, d, H, F, V, 64, arch, arch, dtype, 0, 1, 2, 50, arch ? 8 : 0};
  std::memcpy(h.data() + 8, f, sizeof f);
  float alpha = 1.0f, eps = 1e-5f, topp = 0.f;
  std::memcpy(h.data() + 76, &alpha, 4);
  std::memcpy(h.data() + 80, &eps, 4);
  std::memcpy(h.data() + 84, &topp, 4);
  uint64_t seed = 1234;
  std::memcpy(h.data() + 88, &seed, 8);
  std::memcpy(h.data() + 96, &total, 8);
  return h;
}

int main() {
  size_t n = 0;
  // null / short / wrong magic
  EXPECT(lsq_workspace_bytes(nullptr, 0, 2, 4, 8, &n) == LSQ_E_ARG);
  auto h = header(0, 1, 1, 64, 4, 256, 1000, 0, 0);
  EXPECT(lsq_workspace_bytes(h.data(), 100, 2, 4, 8, &n) == LSQ_E_BLOB);
  EXPECT(lsq_workspace_bytes(h.data(), h.size(), 2, 4, 8, nullptr) == LSQ_E_ARG);
  // the size the shapes add up to: ask the library through a wrong total first (it reports the right one in its message)
  EXPECT(lsq_workspace_bytes(h.data(), h.size(), 2, 4, 8, &n) == LSQ_E_BLOB);
  unsigned long long want = 0;
  const char* msg = lsq_last_error();
  const char* at = std::strstr(msg, "add up to ");
  EXPECT(at != nullptr);
  if (at) std::sscanf(at, "add up to %llu", &want);
  EXPECT(want > 256);
  for (int arch = 0; arch < 2; ++arch)
    for (int dtype = 0; dtype < 2; ++dtype) {
      auto g = header(arch, arch ? 0 : 2, 3, 128, 2, 264, 1003, dtype, 0);
      int rc = lsq_workspace_bytes(g.data(), g.size(), 3, arch ? 1 : 4, 32, &n);
      EXPECT(rc == LSQ_E_BLOB);
      at = std::strstr(lsq_last_error(), "add up to ");
      EXPECT(at != nullptr);
      if (!at) continue;
      std::sscanf(at, "add up to %llu", &want);
      g = header(arch, arch ? 0 : 2, 3, 128, 2, 264, 1003, dtype, want);
      size_t a = 0, b = 0, c = 0;
      EXPECT(lsq_workspace_bytes(g.data(), g.size(), 3, arch ? 1 : 4, 32, &a) == LSQ_OK);
      EXPECT(lsq_workspace_bytes(g.data(), g.size(), 6, arch ? 1 : 4, 32, &b) == LSQ_OK);
      EXPECT(lsq_workspace_bytes(g.data(), g.size(), 3, arch ? 1 : 4, 64, &c) == LSQ_OK);
      EXPECT(a > want && b > a && c > a);          // the plan holds the weights and grows with every maximum
      // limits
      EXPECT(lsq_workspace_bytes(g.data(), g.size(), 0, 1, 32, &a) == LSQ_E_ARG);
      EXPECT(lsq_workspace_bytes(g.data(), g.size(), 3, LSQ_MAX_BEAM + 1, 32, &a) == LSQ_E_ARG);
      EXPECT(lsq_workspace_bytes(g.data(), g.size(), 3, 1, 0, &a) == LSQ_E_ARG);
      EXPECT(lsq_workspace_bytes(g.data(), g.size(), 3, 1, 1 << 20, &a) == LSQ_E_ARG);
      // every single header byte damaged in turn: an error or a plan, never a crash or an overflow
      for (size_t i = 0; i < 104; ++i)
        for (unsigned char v : {(unsigned char)0x00, (unsigned char)0x7f, (unsigned char)0x80, (unsigned char)0xff}) {
          auto bad = g;
          bad[i] = v;
          size_t out = 0;
          int r = lsq_workspace_bytes(bad.data(), bad.size(), 3, arch ? 1 : 4, 32, &out);
          EXPECT(r == LSQ_OK || r == LSQ_E_BLOB || r == LSQ_E_ARG);
        }
    }
  // a pseudo-random walk over whole headers
  uint32_t x = 12345;
  for (int it = 0; it < 20000; ++it) {
    auto g = header(0, 1, 1, 64, 4, 256, 1000, 0, 0);
    for (int k = 0; k < 6; ++k) {
      x = x * 1664525u + 1013904223u;
      g[8 + (x >> 8) % 96] = (unsigned char)(x >> 24);
    }
    size_t out = 0;
    int r = lsq_workspace_bytes(g.data(), g.size(), 1 + (int)(x % 7), 1 + (int)((x >> 3) % 8), 1 + (int)((x >> 6) % 200), &out);
    EXPECT(r == LSQ_OK || r == LSQ_E_BLOB || r == LSQ_E_ARG);
  }
  // calls out of order: state errors, no device work
  lsq_free();
  EXPECT(lsq_decode_step() == LSQ_E_STATE);
  EXPECT(lsq_decode_steps(3) == LSQ_E_STATE);
  int32_t ids[4] = {4, 5, 6, 7}, lens[1] = {4};
  EXPECT(lsq_encode(ids, lens, 1, 4) == LSQ_E_STATE);
  float sc[4];
  int32_t ol[4];
  EXPECT(lsq_get_beams(ids, ol, sc) == LSQ_E_STATE);
  EXPECT(lsq_init(h.data(), h.size(), 2, 4, 8) == LSQ_E_STATE);
  EXPECT(lsq_set_workspace(nullptr, 0, nullptr) == LSQ_E_ARG);
  EXPECT(lsq_set_workspace((void*)3, 1024, nullptr) == LSQ_E_ARG);
  EXPECT(lsq_set_diversity(0, 0.f) == LSQ_E_ARG);
  EXPECT(lsq_set_diversity(2, -1.f) == LSQ_E_ARG);
  EXPECT(lsq_set_diversity(1, 0.f) == LSQ_OK);
  EXPECT(lsq_set_cache_refresh(7) == LSQ_E_ARG);
  EXPECT(lsq_debug_read(LSQ_DBG_SCORE, sc, sizeof sc) == LSQ_E_STATE);
  EXPECT(lsq_k_packed_weight_bytes(64, 24) == 0);
  EXPECT(lsq_k_packed_weight_bytes(33, 32) == 64u * 32 * 2);
  EXPECT(lsq_k_gemm_add_layernorm_scratch(1, 512, 1024, 4096) >= 512u * 1024 * 4);
  EXPECT(lsq_k_gemm(1, nullptr, nullptr, nullptr, nullptr, 1, 1, 8, 0, nullptr) == LSQ_E_ARG);
  lsq_free();
  std::printf(failures ? "host checks: %d FAILED\n" : "host checks: all passed\n", failures);
  return failures ? 1 : 0;
}
