// Host validation paths of the C ABI under AddressSanitizer / UndefinedBehaviorSanitizer: every call below must be
// refused before anything is launched (no GPU needed; pointers are never dereferenced), and the host helpers are
// swept over wide argument ranges.  Built and run by tests/test_abi_sanitizers.py against a build of
// csrc/thrift_api.hip whose host code carries the sanitizers.
#include <stdio.h>
#include <stdint.h>
#include "thrift.h"
#define EXPECT(call, want) do { int got_ = (int)(call); if (got_ != (want)) { printf("line %d: got %d want %d\n", __LINE__, got_, (want)); bad++; } } while (0)
int main() {
  int bad = 0;
  void* fake = (void*)0x1000;
  float* ff = (float*)fake; uint8_t* fu = (uint8_t*)fake; int32_t* fi = (int32_t*)fake;
  EXPECT(thrift_block_means(nullptr, THRIFT_F16, 1, 1, 64, 128, 64, ff, nullptr), THRIFT_ERR_NULL);
  EXPECT(thrift_block_means(fake, THRIFT_F16, 1, 1, 64, 64, 64, ff, nullptr), THRIFT_ERR_SHAPE);
  EXPECT(thrift_block_means(fake, (thrift_dtype)7, 1, 1, 64, 128, 64, ff, nullptr), THRIFT_ERR_DTYPE);
  EXPECT(thrift_block_means(fake, THRIFT_F16, 1 << 30, 1 << 30, 1 << 30, 128, 1, ff, nullptr), THRIFT_ERR_SHAPE);
  EXPECT(thrift_quantize_mxfp4(fake, THRIFT_F16, 1, 1, 0, 128, 1, fu, fu, nullptr), THRIFT_ERR_SHAPE);
  EXPECT(thrift_quantize_mxfp4(fake, THRIFT_F16, 1 << 30, 1 << 30, 1 << 30, 128, 0, fu, fu, nullptr), THRIFT_ERR_SHAPE);
  EXPECT(thrift_select_topk(ff, ff, 1, 3, 2, 8, 8, 128, 64, 64, 1, 0.05, -1, 0, fi, fi, 8, nullptr), THRIFT_ERR_SHAPE);
  EXPECT(thrift_select_topk(ff, ff, 1, 4, 2, 8, 5000, 128, 64, 64, 1, 0.05, -1, 0, fi, fi, 8, nullptr), THRIFT_ERR_SHAPE);
  EXPECT(thrift_select_topk(ff, ff, 1, 4, 2, 8, 8, 128, 64, 64, 1, 1.5, -1, 0, fi, fi, 8, nullptr), THRIFT_ERR_BUDGET);
  EXPECT(thrift_select_topk(ff, ff, 1, 4, 2, 8, 8, 128, 64, 64, 1, 1.0, -1, 0, fi, fi, 4, nullptr), THRIFT_ERR_BUDGET);
  EXPECT(thrift_select_topk_shared(ff, ff, 1, 4, 2, 8, 8, 128, 64, 64, 1, -0.5, -1, 0, fi, fi, 8, nullptr), THRIFT_ERR_BUDGET);
  EXPECT(thrift_select_ablation(9, 1, 1, 4, 8, 8, 64, 64, 1, 0.05, -1, 0, fi, fi, 8, nullptr), THRIFT_ERR_SHAPE);
  EXPECT(thrift_attn_prefill(fake, fake, fake, THRIFT_F16, fu, fu, fu, fu, fu, fu, fi, fi, 4, 1, 4, 2, 256, 128, 32, 64, 1, 0.f, fake, THRIFT_F16, nullptr, nullptr, 0, nullptr), THRIFT_ERR_SHAPE);
  EXPECT(thrift_attn_prefill(fake, fake, fake, THRIFT_F16, fu, fu, fu, fu, fu, fu, fi, fi, 4, 1, 4, 2, 256, 128, 64, 64, 1, 0.f, nullptr, THRIFT_F16, nullptr, nullptr, 0, nullptr), THRIFT_ERR_NULL);
  EXPECT(thrift_attn_prefill_chunk(fake, fake, fake, THRIFT_F16, fu, fu, fu, fu, fu, fu, fi, fi, 4, 1, 4, 2, 256, 3, 256, 128, 64, 64, 1, 0.f, fake, THRIFT_F16, nullptr, nullptr, 0, nullptr), THRIFT_ERR_SHAPE);
  EXPECT(thrift_attn_prefill_ordered(fake, fake, fake, THRIFT_F16, fu, fu, fu, fu, fu, fu, fi, fi, 4, 1, 4, 2, 256, 0, 256, 128, 64, 64, 1, 9, 0.f, fake, THRIFT_F16, nullptr, nullptr, 0, nullptr), THRIFT_ERR_SHAPE);
  EXPECT(thrift_attn_decode(fake, THRIFT_F16, fake, fake, fu, fu, fu, fu, ff, nullptr, 1, 4, 2, 1024, 128, 64, 0.05, -1, 0, 0.f, fake, THRIFT_F16, nullptr, nullptr, 0, fake, 1 << 30, nullptr), THRIFT_ERR_SHAPE);
  EXPECT(thrift_attn_decode(fake, THRIFT_F16, fake, fake, fu, fu, fu, fu, ff, nullptr, 1, 4, 2, 1024, 128, 64, 0.05, -1, 8, 0.f, fake, THRIFT_F16, nullptr, nullptr, 0, fake, 16, nullptr), THRIFT_ERR_WORKSPACE);
  EXPECT(thrift_attn_decode_shared(fake, THRIFT_F16, fake, fake, fu, fu, fu, fu, ff, nullptr, 1, 4, 2, 1024, 128, 64, 2.0, -1, 8, 0.f, fake, THRIFT_F16, nullptr, nullptr, 0, fake, 1 << 30, nullptr), THRIFT_ERR_BUDGET);
  EXPECT(thrift_attn_decode_static(fake, THRIFT_F16, fake, fake, fu, fu, fu, fu, ff, nullptr, 4096, 4, 2, 131072, 128, 64, 0.05, -1, 256, 0.f, fake, THRIFT_F16, nullptr, nullptr, 0, nullptr), THRIFT_ERR_WORKSPACE);
  EXPECT(thrift_attn_decode_static(fake, THRIFT_F16, fake, fake, fu, fu, fu, fu, ff, nullptr, 1, 4, 2, 1000, 128, 64, 0.05, -1, 8, 0.f, fake, THRIFT_F16, nullptr, nullptr, 0, nullptr), THRIFT_ERR_SHAPE);
  EXPECT(thrift_kv_cache_append(nullptr, fake, THRIFT_F16, 1, fi, nullptr, fake, fake, fu, fu, fu, fu, ff, 1, 2, 1024, 128, 64, nullptr), THRIFT_ERR_NULL);
  EXPECT(thrift_kv_cache_append(fake, fake, THRIFT_F16, 2000, fi, nullptr, fake, fake, fu, fu, fu, fu, ff, 1, 2, 1024, 128, 64, nullptr), THRIFT_ERR_SHAPE);
  EXPECT(thrift_attention_forward(fake, fake, fake, THRIFT_BF16, 1, 4, 2, 300, 128, 128, 64, 1, 0.05, -1, 7, 0.f, fake, THRIFT_BF16, nullptr, fake, (size_t)1 << 30, nullptr), THRIFT_ERR_SHAPE);
  EXPECT(thrift_attention_forward(fake, fake, fake, THRIFT_BF16, 1, 4, 2, 300, 128, 128, 64, 1, 0.05, -1, 0, 0.f, fake, THRIFT_BF16, nullptr, fake, 16, nullptr), THRIFT_ERR_WORKSPACE);
  {
    double work = 0.0;
    EXPECT(thrift_peak_probe(THRIFT_PEAK_TILE_MIX, THRIFT_BF16, 10, nullptr, (size_t)1 << 30, &work, nullptr), THRIFT_ERR_NULL);
    EXPECT(thrift_peak_probe(9, THRIFT_BF16, 10, fake, (size_t)1 << 30, &work, nullptr), THRIFT_ERR_SHAPE);
    EXPECT(thrift_peak_probe(THRIFT_PEAK_TILE_MIX, THRIFT_BF16, 0, fake, (size_t)1 << 30, &work, nullptr), THRIFT_ERR_SHAPE);
    EXPECT(thrift_peak_probe(THRIFT_PEAK_HBM_READ, THRIFT_BF16, 1, fake, (size_t)1 << 20, &work, nullptr), THRIFT_ERR_SHAPE);
    EXPECT(thrift_peak_probe(THRIFT_PEAK_MFMA_16, THRIFT_F32, 10, fake, (size_t)1 << 30, &work, nullptr), THRIFT_ERR_DTYPE);
  }
  // host helpers over wide argument ranges (integer arithmetic, no overflow)
  long acc = 0;
  for (int vis = 0; vis <= 4096; vis += 7) for (double f = 0.0; f <= 1.0; f += 0.125) acc += thrift_row_budget(vis, f, -1) + thrift_row_budget(vis, f, 5);
  for (int i = 0; i < 2048; i += 13) acc += thrift_visible_blocks(i, 4096, 128, 64, 1, 1 << 20) + thrift_visible_blocks(i, 4096, 1, 64, 1, 0x7fffffff - 2048);
  for (int n = 1; n <= 4096; n *= 2) acc += thrift_budget_to_global_k(n, 0.05);
  acc += thrift_select_kmax(1024, 2048, 128, 64, 1, 0.05, -1, 0) + thrift_select_kmax(0, 0, 128, 64, 1, 0.05, -1, 0);
  acc += (long)(thrift_attn_decode_workspace(16, 32, 8, 131072, 128, 64, 256) >> 20) + (long)thrift_attention_forward_workspace(1, 32, 8, 131072, 128, 128, 64, 1, 0.05, -1);
  acc += (long)thrift_attn_decode_workspace(1 << 15, 1 << 15, 8, 262144, 128, 64, 4) & 1;
  for (int s = 0; s < 9; ++s) acc += thrift_status_string((thrift_status)s)[0];
  printf("abi sanitizer pass: %s (%d mismatches, checksum %ld)\n", bad ? "FAILED" : "ok", bad, acc);
  return bad != 0;
}
