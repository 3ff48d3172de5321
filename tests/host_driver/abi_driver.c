/* Host-only driver for the sanitizer build of the C ABI's validation layer: every call below must
 * be answered on the host (an error code, or a size), without touching a device: none of them is
 * a valid request, so none reaches a kernel launch even where a GPU is present.  The addresses
 * handed over as "device pointers" are never dereferenced by a correct library; the host arrays
 * (lengths, structs, outputs) are exactly as large as the interface says they must be, so an
 * out-of-bounds access of the validation code trips AddressSanitizer.  Prints "abi driver ok". */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include "../../include/energon.h"

static int failures = 0;
#define EXPECT(expr, want)                                                                   \
  do {                                                                                       \
    long long got_ = (long long)(expr);                                                      \
    if (got_ != (long long)(want)) { printf("FAIL %s: got %lld, want %lld\n", #expr, got_, (long long)(want)); ++failures; } \
  } while (0)

int main(void) {
  void* const dev = (void*)(uintptr_t)0x7f0000001000ull; /* 4 KiB aligned, never dereferenced */
  void* const dev2 = (void*)(uintptr_t)0x7f0000101000ull;
  EnergonLayerConfig cfg = {1024, 16, 64, 4096, 1e-5f, ENERGON_BF16};
  EnergonLayerWeights w;
  const void** wp = (const void**)&w;
  for (int i = 0; i < 12; ++i) wp[i] = dev;
  int32_t* lens = (int32_t*)malloc(2 * sizeof(int32_t)); /* exactly B entries */
  lens[0] = 3; lens[1] = 2;
  int64_t total = -1;
  size_t* off = (size_t*)malloc(ENERGON_WS_COUNT * sizeof(size_t));

  EXPECT(strcmp(energon_strerror(0), "ok"), 0);
  EXPECT(energon_workspace_bytes(NULL, 4) , 0);
  EXPECT(energon_workspace_bytes(&cfg, 577) >= (size_t)577 * (1024 * 4 + 3072 + 4096) * 2, 1);
  EXPECT(energon_workspace_layout(&cfg, 577, off), ENERGON_OK);
  EXPECT(energon_workspace_layout(&cfg, 577, NULL), ENERGON_ERR_NULL);
  EXPECT(off[ENERGON_WS_M] % 256, 0);

  EXPECT(energon_pack(NULL, lens, 2, 4, 64, ENERGON_BF16, dev, 8, (int32_t*)dev, (int32_t*)dev, &total, NULL), ENERGON_ERR_NULL);
  EXPECT(energon_pack(dev, lens, 2, 2, 64, ENERGON_BF16, dev, 8, (int32_t*)dev, (int32_t*)dev, &total, NULL), ENERGON_ERR_LENGTH);
  EXPECT(energon_pack(dev, lens, 2, 4, 64, ENERGON_BF16, dev, 4, (int32_t*)dev, (int32_t*)dev, &total, NULL), ENERGON_ERR_CAPACITY);
  EXPECT(energon_pack(dev, lens, 2, 4, 60, ENERGON_BF16, dev, 8, (int32_t*)dev, (int32_t*)dev, &total, NULL), ENERGON_ERR_SHAPE);
  EXPECT(energon_unpack(dev, (const int32_t*)dev, 9, 2, 4, 64, ENERGON_BF16, dev, NULL), ENERGON_ERR_SHAPE);

  EXPECT(energon_layer_forward(&cfg, &w, dev, dev, 6, (const int32_t*)dev, lens, 2, 4, dev, (size_t)1 << 30, NULL), ENERGON_ERR_LENGTH);
  EXPECT(energon_layer_forward(&cfg, &w, dev, dev, 5, (const int32_t*)dev, lens, 2, 4, dev, 1024, NULL), ENERGON_ERR_CAPACITY);
  EXPECT(energon_layer_forward(&cfg, &w, dev, (char*)dev + 2, 5, (const int32_t*)dev, lens, 2, 4, dev, (size_t)1 << 30, NULL), ENERGON_ERR_ALIGN);
  EXPECT(energon_layer_forward(&cfg, NULL, dev, dev, 5, (const int32_t*)dev, lens, 2, 4, dev, (size_t)1 << 30, NULL), ENERGON_ERR_NULL);
  {
    EnergonLayerConfig bad = cfg;
    bad.head_dim = 80;
    EXPECT(energon_layer_forward(&bad, &w, dev, dev, 5, (const int32_t*)dev, lens, 2, 4, dev, (size_t)1 << 30, NULL), ENERGON_ERR_UNSUPPORTED);
    bad = cfg; bad.hidden = 32768 + 64; bad.n_heads = 513;
    EXPECT(energon_workspace_bytes(&bad, 4), 0);
  }
  EXPECT(energon_layer_forward_profiled(&cfg, &w, dev, dev, 5, (const int32_t*)dev, lens, 2, 4, dev, (size_t)1 << 30, NULL, NULL), ENERGON_ERR_NULL);

  EXPECT(energon_layernorm(dev, dev, NULL, dev, 4, 64, 1e-5f, ENERGON_BF16, NULL), ENERGON_ERR_NULL);
  EXPECT(energon_linear(dev, dev, NULL, NULL, dev, 4, 64, 96, ENERGON_EPI_BIAS, ENERGON_BF16, NULL), ENERGON_ERR_SHAPE);
  EXPECT(energon_linear(dev, dev, NULL, NULL, dev, 4, 64, 1 << 24, ENERGON_EPI_BIAS, ENERGON_BF16, NULL), ENERGON_ERR_UNSUPPORTED);
  EXPECT(energon_linear_scratch_bytes(577, 1024, 1024, ENERGON_BF16), 0);
  {
    const size_t need = energon_linear_scratch_bytes(3184, 6144, 12288, ENERGON_BF16);
    EXPECT(need > 0, 1);
    EXPECT(energon_linear_with_scratch(dev, dev, NULL, NULL, dev, 3184, 6144, 12288, ENERGON_EPI_BIAS, ENERGON_BF16, dev2, need - 1, NULL), ENERGON_ERR_CAPACITY);
    EXPECT(energon_linear_with_scratch(dev, dev, NULL, NULL, dev, 3184, 6144, 12288, ENERGON_EPI_BIAS, ENERGON_BF16, NULL, need, NULL), ENERGON_ERR_NULL);
  }
  EXPECT(energon_attention(dev, dev, (const int32_t*)dev, 5, 2, 4, 2, 32, ENERGON_BF16, NULL), ENERGON_ERR_UNSUPPORTED);
  EXPECT(energon_attention(dev, dev, (const int32_t*)dev, 0, 2, 4, 2, 64, ENERGON_BF16, NULL), ENERGON_OK);

  EXPECT(energon_decode_layer_forward_static(&cfg, &w, dev, dev2, 2, (const int32_t*)dev, lens, dev, dev, 3, NULL), ENERGON_ERR_LENGTH);
  EXPECT(energon_decode_layer_forward_static(&cfg, &w, dev, dev2, 60000, (const int32_t*)dev, NULL, dev, dev, 8, NULL), ENERGON_ERR_CAPACITY);
  EXPECT(energon_decode_layer_forward(&cfg, &w, dev, dev2, 2, (const int32_t*)dev, lens, dev, dev, 8, dev, 16, NULL), ENERGON_ERR_CAPACITY);

  EXPECT(energon_layer_weights_bytes(&cfg) % 256, 0);
  EXPECT(energon_stack_forward_streamed(&cfg, &w, 1, dev, 5, (const int32_t*)dev, lens, 2, 4, dev, (size_t)1 << 30, dev, dev2,
                                        energon_layer_weights_bytes(&cfg) - 1, NULL, (void*)(uintptr_t)8), ENERGON_ERR_CAPACITY);
  EXPECT(energon_stack_forward_streamed(&cfg, &w, 1, dev, 5, (const int32_t*)dev, lens, 2, 4, dev, (size_t)1 << 30, dev, dev2,
                                        energon_layer_weights_bytes(&cfg), NULL, NULL), ENERGON_ERR_UNSUPPORTED);
  free(lens);
  free(off);
  if (failures) return 1;
  printf("abi driver ok\n");
  return 0;
}
