// Host-side launch interface between the C ABI layer and the kernel translation units.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "thrift.h"

namespace thrift {

void launch_block_means(const void* x, thrift_dtype dt, long heads, int N, int block, float* means, hipStream_t st);
void launch_quantize(const void* x, thrift_dtype dt, long bh, int N, int axis, uint8_t* codes, uint8_t* scales, hipStream_t st);

struct SelectArgs {
  const float* qmean;
  const float* kmean;
  int32_t* idx;
  int32_t* cnt;
  int B, Hq, Hkv, Tq, Tk, Bq, Bk, causal, fixed_k, q_block_offset, kmax;
  long long ppm;                // budget in millionths
  int selector;                 // 0: TopK of the mean scores; 1: random keys; 2: largest block ids
  unsigned long long seed;      // random selector only
  int shared;                   // selector 0 only: one set per KV head from the query means summed over its group
};
void launch_select_topk(const SelectArgs& a, hipStream_t st);

struct PrefillArgs {
  const uint16_t* q;
  const uint16_t* k;
  const uint16_t* v;
  const uint8_t* q4;
  const uint8_t* qs;
  const uint8_t* k4;
  const uint8_t* ks;
  const uint8_t* v4;
  const uint8_t* vs;
  const int32_t* idx;
  const int32_t* cnt;
  void* out;
  float* lse;
  int kmax, B, Hq, Hkv, N, Bq, causal;   // N: key tokens per head
  int tile_order;                         // 0: key blocks ascending (Alg. 1); 1: 4-bit blocks first, then promoted (Sec. 3.3)
  int Nq, q_off;                          // query tokens per head; block position of query block 0 in the sequence
  float scale;            // softmax scale (already defaulted)
  thrift_dtype dt, out_dt;
};
void launch_prefill(const PrefillArgs& a, hipStream_t st);

struct DecodeArgs {
  const uint16_t* q;
  const uint16_t* k16;
  const uint16_t* v16;
  const uint8_t* k4;
  const uint8_t* ks;
  const uint8_t* v4;
  const uint8_t* vs;
  const int32_t* seqlens;
  const unsigned long long* bitmap;   // [B,Hq,bitmap_words] selected key blocks per query head
  void* out;
  float* part_o;          // [B,Hq,nparts,D] unnormalised partial outputs
  float* part_ml;         // [B,Hq,nparts,2] running max (raw score units) and row sum of each partial
  int* order;             // nullable [B*Hkv*nsplit]: scratch for the launch order of the split-K workgroups (heaviest first)
  int bitmap_words, B, Hq, Hkv, Nkv, split_blocks, nsplit;
  int nparts;             // partial slots per (sequence, query head): 1 per partition + 1 for a partly filled last block
  int nmerge;             // slots the merge reads (the last one only when lengths were given)
  float scale;
  thrift_dtype dt, out_dt;
};
void launch_decode(const DecodeArgs& a, hipStream_t st);
// entries of DecodeArgs::order that launch_decode wants; 0 = so many workgroups that their order does not matter (pass nullptr)
int decode_order_items(int B, int Hkv, int nsplit);
// decode-time selection: scores of the cached key-block means against the query heads, then per-row TopK
// as a bitmap ([B*Hq][words], bit j%64 of word j/64) and optionally as ascending id lists
void launch_decode_select(const uint16_t* q16, int q_is_bf16, const float* kmean, const int32_t* seqlens, uint64_t* keys,
                          unsigned long long* bitmap, int words, int32_t* idx_out, int32_t* cnt_out, int kmax_out,
                          int B, int Hq, int Hkv, int Tk, int fixed_k, long long ppm, int shared, hipStream_t st);

// Append to the dual cache: tokens seqlens[b] .. seqlens[b] + n - 1 of every (sequence, KV head)
struct CacheAppendArgs {
  const uint16_t* k_new;      // [B,Hkv,n_new,D]
  const uint16_t* v_new;
  const int32_t* seqlens;     // [B] tokens cached before the call
  const int32_t* new_lens;    // nullable [B]: tokens to take from k_new / v_new (<= n_new)
  uint16_t* k16;              // [B,Hkv,Nkv,D]
  uint16_t* v16;
  uint8_t* k4;
  uint8_t* ks;
  uint8_t* v4;
  uint8_t* vs;
  float* kmean;
  int B, Hkv, Nkv, n_new, blocks_per_unit;
};
void launch_cache_append(const CacheAppendArgs& a, thrift_dtype dt, hipStream_t st);

// measurement microbenchmarks (thrift_peak_probe): returns the work of the launch, 0 for an unknown kind
double launch_peak_probe(int kind, thrift_dtype dt, int iters, void* buffer, size_t bytes, hipStream_t st);

}  // namespace thrift
