// Host-side error paths of the C ABI, for a build with AddressSanitizer and UndefinedBehaviorSanitizer on the
// host code of the launcher (no GPU is touched: every call below is rejected by the argument checks).
#include <stdio.h>
#include <string.h>

#include "../../include/lshmoe.h"

static int failures = 0;
#define EXPECT(call, want)                                                                 \
  do {                                                                                     \
    const int got_ = (int)(call);                                                          \
    if (got_ != (int)(want)) {                                                             \
      printf("FAIL %s: got %s (%s)\n", #call, lshmoe_status_string(got_), lshmoe_last_error()); \
      ++failures;                                                                          \
    }                                                                                      \
  } while (0)

int main() {
  void* p = (void*)0x1000;   // never dereferenced: the checks reject the calls before any device work
  int32_t* pi = (int32_t*)p;
  uint64_t* pu = (uint64_t*)p;
  float* pf = (float*)p;
  size_t bytes = 0;
  EXPECT(lshmoe_workspace_bytes(65536, 1024, 2, 64, 4, 64, LSHMOE_BF16, &bytes), LSHMOE_OK);
  if (bytes < (size_t)1 << 20 || bytes > LSHMOE_STATIC_SCRATCH_BYTES) { printf("FAIL workspace size %zu\n", bytes); ++failures; }
  EXPECT(lshmoe_workspace_bytes(65536, 1024, 2, 64, 4, 64, LSHMOE_BF16, nullptr), LSHMOE_ERR_NULL);
  EXPECT(lshmoe_workspace_bytes(0, 1024, 2, 64, 4, 64, LSHMOE_BF16, &bytes), LSHMOE_ERR_SHAPE);
  EXPECT(lshmoe_workspace_bytes(16, 1024, 3, 2, 4, 64, LSHMOE_BF16, &bytes), LSHMOE_ERR_SHAPE);
  EXPECT(lshmoe_workspace_bytes(16, 1024, 1, 2, 10, 64, LSHMOE_BF16, &bytes), LSHMOE_ERR_UNSUPPORTED);        // (2r)^L >= 2^63
  EXPECT(lshmoe_workspace_bytes((int64_t)1 << 30, 8, 1, 2, 2, 8, LSHMOE_BF16, &bytes), LSHMOE_ERR_UNSUPPORTED);
  EXPECT(lshmoe_workspace_bytes((int64_t)1 << 29, 8192, 1, 2, 2, 8, LSHMOE_F32, &bytes), LSHMOE_ERR_UNSUPPORTED);  // N*d too large
  EXPECT(lshmoe_workspace_bytes(16, 1024, 1, 1 << 20, 9, 64, LSHMOE_BF16, &bytes), LSHMOE_ERR_UNSUPPORTED);   // key wider than 64 bits
  EXPECT(lshmoe_hash(nullptr, p, 16, 64, 2, 8, LSHMOE_BF16, pu, nullptr), LSHMOE_ERR_NULL);
  EXPECT(lshmoe_hash(p, p, 16, 60, 2, 8, LSHMOE_BF16, pu, nullptr), LSHMOE_ERR_UNSUPPORTED);
  EXPECT(lshmoe_hash(p, p, 16, 64, 2, 512, LSHMOE_BF16, pu, nullptr), LSHMOE_ERR_UNSUPPORTED);
  EXPECT(lshmoe_hash(p, p, 16, 64, 2, 8, (lshmoe_dtype)7, pu, nullptr), LSHMOE_ERR_UNSUPPORTED);
  EXPECT(lshmoe_hash_sphere(p, p, nullptr, 16, 64, 8, LSHMOE_BF16, pu, nullptr), LSHMOE_ERR_NULL);
  EXPECT(lshmoe_hash_sphere(p, p, pf, 16, 64, 64, LSHMOE_BF16, pu, nullptr), LSHMOE_ERR_UNSUPPORTED);
  EXPECT(lshmoe_hash_gate(p, p, p, 16, 64, 2, 8, 0, LSHMOE_BF16, pu, pf, nullptr), LSHMOE_ERR_SHAPE);
  EXPECT(lshmoe_hash_gate(p, p, p, 16, 256, 2, 12, 4, LSHMOE_BF16, pu, pf, nullptr), LSHMOE_ERR_UNSUPPORTED);
  EXPECT(lshmoe_compress(p, pi, pu, 16, 64, 1, 4, 2, 8, LSHMOE_BF16, p, pi, pi, pi, pi, pi, pi, nullptr, 0, nullptr), LSHMOE_ERR_WORKSPACE);
  EXPECT(lshmoe_compress(p, pi, pu, 16, 64, 1, 4, 2, 8, LSHMOE_BF16, p, pi, pi, pi, pi, pi, pi, (void*)0x1010, (size_t)1 << 30, nullptr), LSHMOE_ERR_WORKSPACE);
  EXPECT(lshmoe_compress(p, pi, pu, 16, 64, 1, 4, 2, 8, LSHMOE_BF16, p, pi, pi, pi, pi, pi, pi, p, 64, nullptr), LSHMOE_ERR_WORKSPACE);
  EXPECT(lshmoe_compress(p, nullptr, pu, 16, 64, 1, 4, 2, 8, LSHMOE_BF16, p, pi, pi, pi, pi, pi, pi, p, (size_t)1 << 30, nullptr), LSHMOE_ERR_NULL);
  EXPECT(lshmoe_compress_static(p, pi, pu, 4 * 65536, 1024, 2, 64, 4, 64, LSHMOE_BF16, p, pi, pi, pi, pi, pi, pi, nullptr), LSHMOE_ERR_WORKSPACE);
  EXPECT(lshmoe_compress_static(p, pi, pu, 16, 64, 5, 4, 2, 8, LSHMOE_BF16, p, pi, pi, pi, pi, pi, pi, nullptr), LSHMOE_ERR_SHAPE);
  EXPECT(lshmoe_decompress(p, p, p, nullptr, nullptr, nullptr, nullptr, 16, 64, 1, LSHMOE_BF16, 0, p, nullptr), LSHMOE_ERR_NULL);
  EXPECT(lshmoe_decompress(p, p, p, pi, nullptr, pi, nullptr, 16, 64, 1, LSHMOE_BF16, 0, p, nullptr), LSHMOE_ERR_NULL);
  EXPECT(lshmoe_decompress(p, p, p, pi, nullptr, nullptr, nullptr, 16, 64, 1, LSHMOE_BF16, 8, p, nullptr), LSHMOE_ERR_UNSUPPORTED);
  EXPECT(lshmoe_decompress_combine(p, p, p, pi, nullptr, nullptr, 16, 64, 1, LSHMOE_BF16, 0, p, nullptr), LSHMOE_ERR_NULL);
  EXPECT(lshmoe_decompress_combine_backward(p, p, p, pi, nullptr, pf, p, 16, 64, 1, LSHMOE_BF16, 0, nullptr, p, nullptr), LSHMOE_ERR_NULL);
  EXPECT(lshmoe_decompress_combine_backward(p, p, p, pi, nullptr, pf, p, 16, 64, 1, LSHMOE_BF16, 2, pf, p, nullptr), LSHMOE_ERR_UNSUPPORTED);
  EXPECT(lshmoe_backward_workspace_bytes(16, 64, 1, LSHMOE_BF16, &bytes), LSHMOE_OK);
  EXPECT(lshmoe_decompress_backward(p, pi, pi, pi, pi, 16, 64, 1, LSHMOE_BF16, p, nullptr, 0, nullptr), LSHMOE_ERR_WORKSPACE);
  EXPECT(lshmoe_compress_backward(nullptr, p, nullptr, pi, pi, 16, 64, 1, LSHMOE_BF16, 0, p, nullptr), LSHMOE_ERR_NULL);
  if (strcmp(lshmoe_status_string(LSHMOE_ERR_HIP), "LSHMOE_ERR_HIP") != 0 || strcmp(lshmoe_status_string(99), "LSHMOE_ERR_UNKNOWN") != 0) {
    printf("FAIL status strings\n");
    ++failures;
  }
  if (lshmoe_abi_version() < 6) { printf("FAIL abi version\n"); ++failures; }
  printf(failures ? "%d failures\n" : "host error paths clean under the sanitizers (%d failures)\n", failures);
  return failures ? 1 : 0;
}
