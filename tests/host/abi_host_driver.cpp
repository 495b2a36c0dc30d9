// Host-side driver for the sanitizer build of the C ABI: calls every entry point on the argument-error and
// no-op paths (which return before anything is enqueued, so no GPU is needed) and the pure size queries over
// a sweep of shapes.  Built with AddressSanitizer and UndefinedBehaviorSanitizer on the host code; exits 0
// when every status is the expected one (the sanitizers abort the process on a finding).
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <initializer_list>

#include "dirotq.h"

static int failures = 0;
#define EXPECT(call, want)                                                                 \
  do {                                                                                     \
    int got_ = (call);                                                                     \
    if (got_ != (want)) {                                                                  \
      std::printf("FAIL %s -> %d (%s), expected %d\n", #call, got_, dirotq_strerror(got_), (int)(want)); \
      failures++;                                                                          \
    }                                                                                      \
  } while (0)

int main() {
  alignas(256) static unsigned char fake[4096];      // aligned, never dereferenced by the library on these paths
  uint16_t* a16 = (uint16_t*)fake;
  uint8_t* a8 = fake;
  void* av = fake;
  size_t sz = 7;
  for (int s = -9; s <= 1; s++)
    if (!dirotq_strerror(s) || !dirotq_strerror(s)[0]) failures++;
  EXPECT(dirotq_last_hip_error(), 0);
  // size queries over a grid of shapes, valid and invalid
  long n_ok = 0;
  for (int N : {0, 1, 8, 129, 1 << 24, (1 << 24) + 1})
    for (int K : {0, 31, 32, 48, 64, 1152, 12288, 1 << 20, (1 << 20) + 32})
      for (int r : {-32, 0, 16, 32, 64, 1152, 12288})
        for (int g : {0, 16, 32, 48, 64, 128, 256}) {
          const bool ok = N >= 1 && N <= (1 << 24) && K >= 32 && K % 32 == 0 && K <= (1 << 20) && r >= 0 && r <= K &&
                          r % 32 == 0 && (g == 32 || g == 64 || g == 128) && (K - r) % g == 0;
          sz = 7;
          EXPECT(dirotq_weights_bytes(N, K, r, g, &sz), ok ? DIROTQ_OK : DIROTQ_ERR_SHAPE);
          if (!ok && sz != 7) failures++;
          if (ok && (sz % 256 != 0 || sz == 0)) failures++;
          n_ok += ok;
          for (int M : {-1, 0, 1, 300, 1 << 24}) {
            size_t ws = 7;
            const bool okm = ok && M >= 0;
            EXPECT(dirotq_workspace_bytes(M, K, r, g, &ws), (M >= 0 && K >= 32 && K % 32 == 0 && K <= (1 << 20) && r >= 0 &&
                                                             r <= K && r % 32 == 0 && (g == 32 || g == 64 || g == 128) &&
                                                             (K - r) % g == 0)
                                                                ? DIROTQ_OK
                                                                : DIROTQ_ERR_SHAPE);
            (void)okm;
          }
        }
  if (n_ok == 0) failures++;
  EXPECT(dirotq_weights_bytes(8, 64, 0, 32, nullptr), DIROTQ_ERR_NULL);
  EXPECT(dirotq_prepare_scratch_bytes(8, 64, nullptr), DIROTQ_ERR_NULL);
  EXPECT(dirotq_prepare_scratch_bytes(8, 64, &sz), DIROTQ_OK);
  EXPECT(dirotq_a8_scratch_bytes(4, 64, 0, &sz), DIROTQ_OK);
  EXPECT(dirotq_a8_workspace_bytes(4, 48, 0, &sz), DIROTQ_ERR_SHAPE);
  // argument errors: nothing is enqueued, nothing is dereferenced
  EXPECT(dirotq_prepare_rotation(nullptr, 64, a16, nullptr), DIROTQ_ERR_NULL);
  EXPECT(dirotq_prepare_rotation((const float*)av, 48, a16, nullptr), DIROTQ_ERR_SHAPE);
  EXPECT(dirotq_prepare_weights((const float*)av, (const float*)av, 8, 64, 0, 32, av, av, 8, nullptr), DIROTQ_ERR_WORKSPACE);
  EXPECT(dirotq_import_weights(nullptr, nullptr, nullptr, 8, 64, 0, 32, av, nullptr), DIROTQ_ERR_NULL);
  EXPECT(dirotq_export_weights(nullptr, 8, 64, 0, 32, a16, (int8_t*)av, a16, nullptr), DIROTQ_ERR_NULL);
  EXPECT(dirotq_rotate_quantize(nullptr, a16, 4, 64, 0, 32, nullptr, a8, a16, nullptr), DIROTQ_ERR_NULL);
  EXPECT(dirotq_rotate_quantize(a16, a16, -1, 64, 0, 32, nullptr, a8, a16, nullptr), DIROTQ_ERR_SHAPE);
  EXPECT(dirotq_rotate_quantize(a16 + 1, a16, 4, 64, 0, 32, nullptr, a8, a16, nullptr), DIROTQ_ERR_ALIGN);
  EXPECT(dirotq_rotate_quantize(a16, a16, 0, 64, 0, 32, nullptr, a8, a16, nullptr), DIROTQ_OK);
  EXPECT(dirotq_w4a4_gemm(nullptr, a8, a16, nullptr, nullptr, 4, 8, 64, 0, 32, av, 0, nullptr), DIROTQ_ERR_NULL);
  EXPECT(dirotq_w4a4_gemm(nullptr, a8, a16, av, nullptr, 4, 8, 64, 0, 32, av, 2, nullptr), DIROTQ_ERR_UNSUPPORTED);
  EXPECT(dirotq_w4a4_gemm(nullptr, a8, a16, av, nullptr, 1 << 24, 1 << 24, 64, 0, 32, av, 0, nullptr), DIROTQ_ERR_SHAPE);
  EXPECT(dirotq_w4a4_gemm(nullptr, a8, a16, av, nullptr, 0, 8, 64, 0, 32, av, 0, nullptr), DIROTQ_OK);
  EXPECT(dirotq_linear(a16, a16, av, nullptr, 4, 8, 64, 0, 32, a16, av, 16, nullptr), DIROTQ_ERR_WORKSPACE);
  EXPECT(dirotq_linear(a16, a16, av, nullptr, 4, 8, 64, 0, 32, a16, fake + 16, 1 << 20, nullptr), DIROTQ_ERR_ALIGN);
  EXPECT(dirotq_linear_static(a16, a16, nullptr, nullptr, 4, 8, 64, 0, 32, a16, nullptr), DIROTQ_ERR_NULL);
  EXPECT(dirotq_linear_static(a16, a16, av, nullptr, 16384, 8, 12288, 128, 64, a16, nullptr), DIROTQ_ERR_STATIC_LIMIT);
  EXPECT(dirotq_linear_static(a16, a16, av, nullptr, 0, 8, 64, 0, 32, a16, nullptr), DIROTQ_OK);
  {
    const void* blobs[2] = {av, av};
    const void* blobs_bad[2] = {av, nullptr};
    uint16_t* ys[2] = {a16, a16};
    int Ns[2] = {8, 16}, Ns_bad[2] = {8, 0};
    EXPECT(dirotq_linear_shared(a16, a16, 0, blobs, nullptr, Ns, ys, 4, 64, 0, 32, av, 1 << 20, nullptr), DIROTQ_ERR_SHAPE);
    EXPECT(dirotq_linear_shared(a16, a16, 17, blobs, nullptr, Ns, ys, 4, 64, 0, 32, av, 1 << 20, nullptr), DIROTQ_ERR_SHAPE);
    EXPECT(dirotq_linear_shared(a16, a16, 2, nullptr, nullptr, Ns, ys, 4, 64, 0, 32, av, 1 << 20, nullptr), DIROTQ_ERR_NULL);
    EXPECT(dirotq_linear_shared(a16, a16, 2, blobs, nullptr, Ns_bad, ys, 4, 64, 0, 32, av, 1 << 20, nullptr), DIROTQ_ERR_SHAPE);
    EXPECT(dirotq_linear_shared(a16, a16, 2, blobs_bad, nullptr, Ns, ys, 4, 64, 0, 32, av, 1 << 20, nullptr), DIROTQ_ERR_NULL);
    EXPECT(dirotq_linear_shared(a16, a16, 2, blobs, nullptr, Ns, ys, 4, 64, 0, 32, av, 16, nullptr), DIROTQ_ERR_WORKSPACE);
    EXPECT(dirotq_linear_shared(a16, a16, 2, blobs, nullptr, Ns, ys, 0, 64, 0, 32, av, 0, nullptr), DIROTQ_OK);
  }
  EXPECT(dirotq_rotate_quantize_asym(a16, a16, 4, 64, 0, 32, nullptr, a8, a16, nullptr, nullptr), DIROTQ_ERR_NULL);
  EXPECT(dirotq_w4a4_gemm_asym(nullptr, a8, a16, nullptr, av, nullptr, 4, 8, 64, 0, 32, av, 0, nullptr), DIROTQ_ERR_NULL);
  EXPECT(dirotq_linear_asym(a16, a16, av, nullptr, 4, 8, 64, 0, 32, a16, av, 16, nullptr), DIROTQ_ERR_WORKSPACE);
  EXPECT(dirotq_rotate_quantize_a8(a16, a16, 4, 64, 0, nullptr, nullptr, a16, av, 1 << 20, nullptr), DIROTQ_ERR_NULL);
  EXPECT(dirotq_rotate_quantize_a8(a16, a16, 4, 64, 0, nullptr, a8, a16, av, 16, nullptr), DIROTQ_ERR_WORKSPACE);
  EXPECT(dirotq_w4a8_gemm(nullptr, a8, nullptr, av, nullptr, 4, 8, 64, 0, 32, av, 0, nullptr), DIROTQ_ERR_NULL);
  EXPECT(dirotq_linear_a8(a16, a16, av, nullptr, 4, 8, 64, 0, 32, a16, av, 16, nullptr), DIROTQ_ERR_WORKSPACE);
  EXPECT(dirotq_w4a16_gemm(nullptr, av, nullptr, 4, 8, 64, 32, av, 0, nullptr), DIROTQ_ERR_NULL);
  EXPECT(dirotq_w4a16_gemm(a16, av, nullptr, 4, 8, 96, 64, av, 0, nullptr), DIROTQ_ERR_SHAPE);
  EXPECT(dirotq_w4a16_gemm(a16, av, nullptr, 0, 8, 64, 32, av, 0, nullptr), DIROTQ_OK);
  std::printf("abi host driver: %d failure(s)\n", failures);
  return failures ? 1 : 0;
}
