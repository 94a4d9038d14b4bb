// Split-K decode over the dual MXFP4 / 16-bit KV cache (Sec. 4.1 and Sec. 5 of the paper describe the
// dual cache; the algorithm is Algorithm 1 with a one-token query block).
//
// One workgroup = one (sequence, KV head, partition of split_blocks key blocks).  Its four wavefronts
// each take a contiguous quarter of the partition and run Alg. 1 over it from a fresh (m, l, O) for all
// query heads of the GQA group at once: the group's G <= 32 heads are the "query rows" of the same
// transposed 32x32 MFMA tiles the prefill kernel uses (columns >= G carry zeros and are never stored).
// The kernel is bandwidth bound: each wavefront streams its key blocks straight from HBM into MFMA
// operand registers — 4-bit codes and scales for every block that some head of the group has not
// promoted, the 16-bit K/V rows for blocks that some head has promoted — so every cache byte is read
// once per KV head, not once per query head.  A head for which the block is promoted takes its scores
// and P.V from the 16-bit path, the others from the 4-bit path; both feed the same online softmax.
// Each wavefront writes one unnormalised partial (m, l, O); a second kernel merges the partials of a
// (sequence, head) by their log-sum-exp.
#include "thrift_launch.h"
#include "thrift_tile.h"

namespace thrift {

constexpr int kDecodeLdsPerWave = kBk * kRow16;   // one 16-bit V tile per wavefront (transposing reads)

// TAIL_ONLY = false: the full key blocks of every sequence, the instantiation that carries the traffic.
// TAIL_ONLY = true: one wavefront per (sequence, KV head) for the one key block a length that is not a multiple of
// the block size leaves partly filled: its keys past the length are masked, the staging of its 16-bit V rows stops
// at the last valid row, and the result is one more partial (the last slot) for the merge.  Kept out of the main
// instantiation so that its hot loop carries none of the masking.
template <typename T, bool TAIL_ONLY>
__global__ void __launch_bounds__(256, 2) decode_partial_kernel(DecodeArgs a) {
  __shared__ __align__(16) unsigned char lds_all[4 * kDecodeLdsPerWave];
  const int tid = threadIdx.x, lane = tid & 63, half = lane >> 5, r = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wavefront-uniform: loop bounds stay scalar
  unsigned char* lds = lds_all + wave * kDecodeLdsPerWave;
  const int G = a.Hq / a.Hkv;
  const int part = TAIL_ONLY ? 0 : blockIdx.x % a.nsplit;
  const int unit = TAIL_ONLY ? blockIdx.x : blockIdx.x / a.nsplit;
  const int b = unit / a.Hkv, kvh = unit % a.Hkv;
  // cached tokens of this sequence; the last key block may still be filling up
  const int len = a.seqlens ? min(a.Nkv, max(0, a.seqlens[b])) : a.Nkv;
  const int Tk = TAIL_ONLY ? (len + kBk - 1) / kBk : len / kBk;
  const bool real = r < G;                                   // this lane's column is a real query head
  const int hq = kvh * G + (real ? r : 0);
  const size_t qh = (size_t)b * a.Hq + hq, kh = (size_t)b * a.Hkv + kvh;

  // contiguous quarter of the partition for this wavefront
  const int quarter = a.split_blocks / 4;
  const int j_begin = TAIL_ONLY ? len / kBk : part * a.split_blocks + wave * quarter;
  const int j_end = TAIL_ONLY ? Tk : min(Tk, j_begin + quarter);

  // ---- Q fragments (zeros for padding columns): the lane quantises its own two MXFP4 groups of the query,
  // d-group 2*half + kk (channels 64*half + 32*kk .. +31) for fragment kk (Alg. 1 step 2 for the one-token
  // query block) ----
  v4i qf4[2] = {(v4i){0, 0, 0, 0}, (v4i){0, 0, 0, 0}};
  uint32_t qsc = 0x7f7f7f7fu;
  if (real) {
    uint32_t sb[2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
      const uint4* src = reinterpret_cast<const uint4*>(a.q + qh * kD + 64 * half + 32 * kk);
      uint32_t pair[16], codes[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const uint4 w = src[t];
        pair[4 * t] = w.x; pair[4 * t + 1] = w.y; pair[4 * t + 2] = w.z; pair[4 * t + 3] = w.w;
      }
      sb[kk] = quantize_group32<T>(pair, codes);
      qf4[kk] = (v4i){(int)codes[0], (int)codes[1], (int)codes[2], (int)codes[3]};
    }
    qsc = sb[0] | (sb[1] << 8);                              // byte kk: the scale of fragment kk
  }

  const uint8_t* k4base = a.k4 + kh * a.Nkv * 64;
  const uint8_t* v4base = a.v4 + kh * (size_t)(a.Nkv / 64) * 4096;
  const uint8_t* ksbase = a.ks + kh * a.Nkv * 4;
  const uint8_t* vsbase = a.vs + kh * (size_t)(a.Nkv / 32) * kD;
  const uint16_t* k16base = a.k16 + kh * a.Nkv * kD;
  const uint16_t* v16base = a.v16 + kh * a.Nkv * kD;
  const unsigned long long* bm = a.bitmap + qh * a.bitmap_words;

  RowState st = {kEmptyMax, 0.f};
  v16f o[4];
#pragma unroll
  for (int n = 0; n < 4; ++n) o[n] = (v16f){0.f};
  const float c = a.scale * 1.4426950408889634f;
  const unsigned long long group_mask = G >= 32 ? 0xffffffffULL : ((1ULL << G) - 1ULL);

  unsigned long long word = 0;
  int word_id = -1;
  for (int j = j_begin; j < j_end; ++j) {
    constexpr bool TAIL = TAIL_ONLY;
    if ((j >> 6) != word_id) { word_id = j >> 6; word = real ? bm[word_id] : 0ULL; }
    const bool mine16 = (word >> (j & 63)) & 1ULL;           // promoted for this lane's head
    const unsigned long long votes = __builtin_amdgcn_ballot_w64(mine16) & group_mask;
    const bool any16 = votes != 0ULL;
    const bool all16 = votes == group_mask;
    const int n_valid = TAIL ? len - j * kBk : kBk;

    v16f s[2];
    v4i vf4[4];
    uint32_t vsw = 0;
    if (!all16) {
      // the block's 4-bit V fragments and scales are requested together with its K rows: one memory round trip
      // per block instead of two (they are used after the softmax)
      const uint8_t* vt = v4base + (size_t)j * 4096 + r * 32 + half * 16;
      const uint8_t* vsr = vsbase + ((size_t)j * 2 + half) * kD + r;
#pragma unroll
      for (int n = 0; n < 4; ++n) vf4[n] = *reinterpret_cast<const v4i*>(vt + 1024 * n);
      vsw = (uint32_t)vsr[0] | ((uint32_t)vsr[32] << 8) | ((uint32_t)vsr[64] << 16) | ((uint32_t)vsr[96] << 24);
      // ---- 4-bit scores straight from global memory ----
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const int key = key_of_row(r, t);
        const uint8_t* krow = k4base + ((size_t)j * kBk + key) * 64 + 32 * half;
        const v4i a0 = *reinterpret_cast<const v4i*>(krow);
        const v4i a1 = *reinterpret_cast<const v4i*>(krow + 16);
        const uint32_t ksw = *reinterpret_cast<const uint16_t*>(ksbase + ((size_t)j * kBk + key) * 4 + 2 * half);
        v16f acc = {0.f};
        acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen(a0), widen(qf4[0]), acc, 4, 4, 0, ksw, 0, qsc);
        acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen(a1), widen(qf4[1]), acc, 4, 4, 1, ksw, 1, qsc);
        s[t] = acc;
      }
    }
    if (any16) {
      // ---- 16-bit scores; the V tile goes through this wavefront's LDS slice for the transposing reads ----
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        // rows past the cached tokens are never written by anyone: stage the last valid row in their place
        // (their probabilities are zero, but zero times an arbitrary bit pattern need not be)
        const int chunk = lane + 64 * u, row = chunk >> 4, col = chunk & 15;
        *reinterpret_cast<uint4*>(lds + row * kRow16 + col * 16) =
            *reinterpret_cast<const uint4*>(v16base + ((size_t)j * kBk + (TAIL ? min(row, n_valid - 1) : row)) * kD + col * 8);
      }
      v8s qf16[8];
#pragma unroll
      for (int s8 = 0; s8 < 8; ++s8)
        qf16[s8] = real ? *reinterpret_cast<const v8s*>(a.q + qh * kD + 16 * s8 + 8 * half) : (v8s){0, 0, 0, 0, 0, 0, 0, 0};
      v16f s16[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const uint16_t* krow = k16base + ((size_t)j * kBk + key_of_row(r, t)) * kD + 8 * half;
        v16f acc = {0.f};
#pragma unroll
        for (int s8 = 0; s8 < 8; ++s8) acc = T::mfma(*reinterpret_cast<const v8s*>(krow + 16 * s8), qf16[s8], acc);
        s16[t] = acc;
      }
      if (all16) { s[0] = s16[0]; s[1] = s16[1]; }
      else if (mine16) { s[0] = s16[0]; s[1] = s16[1]; }
    }
    float alpha;
    uint32_t pb;
    const bool grew = softmax_update(s, lane, TAIL, n_valid, c, st, alpha, pb);
    rescale(o, grew, alpha);
    if (!all16) {
      // heads that took the 16-bit scores contribute nothing on the 4-bit path (zero codes, whatever the scale)
      v16f p4[2] = {s[0], s[1]};
      if (mine16) { p4[0] = (v16f){0.f}; p4[1] = (v16f){0.f}; }
      pv_fp4_regs<true>(p4, pb, vsw, 0u, 0u, 0u, vf4[0], vf4[1], vf4[2], vf4[3], o);
    }
    if (any16) {
      v16f p16[2] = {s[0], s[1]};
      if (!mine16) { p16[0] = (v16f){0.f}; p16[1] = (v16f){0.f}; }
      __builtin_amdgcn_wave_barrier();
      pv_16<T, false>(lds, lane, p16, o);
      __builtin_amdgcn_wave_barrier();
    }
  }

  // ---- partial (m, l, O) of this wavefront: accumulator i of tile n is channel 32n + 8(i/4) + 4*half + i%4 ----
  const float l = st.l + other_half(st.l);
  if (real) {
    const int pid = TAIL_ONLY ? a.nparts - 1 : part * 4 + wave;
    float* po = a.part_o + (qh * a.nparts + pid) * kD;
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4)
        *reinterpret_cast<float4*>(po + 32 * n + 8 * g4 + 4 * half) =
            make_float4(o[n][4 * g4], o[n][4 * g4 + 1], o[n][4 * g4 + 2], o[n][4 * g4 + 3]);
    if (half == 0) {
      a.part_ml[(qh * a.nparts + pid) * 2] = st.m;
      a.part_ml[(qh * a.nparts + pid) * 2 + 1] = l;
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Decode-time block selection (Alg. 1 step 5 for one-token query blocks).  Two kernels, so that the
// whole chip works on the B*Hq short rows:
//   decode_scores_kernel  one workgroup per (sequence, KV head, 256 key blocks): stages the cached
//                         key-block means 64 at a time and scores them against the G query heads of the group
//                         (fp64, channels in ascending order), storing order-preserving 64-bit keys;
//   decode_select_kernel  one wavefront per (sequence, query head): finds the k-th largest key by a
//                         bitwise search with ballot counting and writes the selection as a bitmap
//                         (and, on request, as an ascending id list).
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ uint64_t order_key64(double s) {
  uint64_t u = (uint64_t)__double_as_longlong(s);
  return (u >> 63) ? ~u : (u | 0x8000000000000000ULL);   // larger double <=> larger key
}

constexpr int kScoreChunksPerWg = 8;     // 64-block chunks one workgroup of decode_scores_kernel walks

__global__ void __launch_bounds__(256) decode_scores_kernel(const uint16_t* __restrict__ q16, int q_is_bf16, const float* __restrict__ kmean,
                                                            const int32_t* __restrict__ seqlens, uint64_t* __restrict__ keys,
                                                            int Hq, int Hkv, int Tk, int shared) {
  constexpr int kStride = kD + 4;
  __shared__ __align__(16) float kst[64 * kStride];
  __shared__ __align__(16) float qst[32 * kD];
  __shared__ __align__(16) double qsum[kD];            // shared mode: the group's query vectors added up (fp64, head order)
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int G = Hq / Hkv, chunks = (Tk + 63) / 64;
  const int groups = (chunks + kScoreChunksPerWg - 1) / kScoreChunksPerWg;
  const int chunk0 = (blockIdx.x % groups) * kScoreChunksPerWg, unit = blockIdx.x / groups;
  const int b = unit / Hkv, kvh = unit % Hkv;
  const int cap = seqlens ? min(Tk, (max(0, seqlens[b]) + kBk - 1) / kBk) : Tk;
  if (chunk0 * 64 >= cap) return;                           // uniform: nothing of these chunks is valid
  const int chunk_end = min(chunk0 + kScoreChunksPerWg, (cap + 63) / 64);
  const float* kunit = kmean + (size_t)unit * Tk * kD;
  // the chunk after the one being scored travels through registers, so its latency hides behind the arithmetic
  float4 pre[8];
#define THRIFT_LOAD_CHUNK(C)                                                                                     \
  _Pragma("unroll") for (int u = 0; u < 8; ++u) {                                                                \
    const int c4 = tid + 256 * u, row = c4 >> 5, col = (c4 & 31) * 4;                                            \
    pre[u] = (C) * 64 + row < Tk ? *reinterpret_cast<const float4*>(kunit + ((size_t)(C) * 64 + row) * kD + col) \
                                 : make_float4(0.f, 0.f, 0.f, 0.f);                                              \
  }
  THRIFT_LOAD_CHUNK(chunk0)
  // the query token is its own block mean (one-token block): the 16-bit value widened exactly
  const uint16_t* qbase = q16 + ((size_t)b * Hq + (size_t)kvh * G) * kD;
  for (int e = tid; e < G * kD; e += 256) qst[e] = q_is_bf16 ? BF16::to_float(qbase[e]) : F16::to_float(qbase[e]);
  if (shared && tid < kD) {
    double t = 0.0;
    for (int g = 0; g < G; ++g) t += (double)(q_is_bf16 ? BF16::to_float(qbase[g * kD + tid]) : F16::to_float(qbase[g * kD + tid]));
    qsum[tid] = t;
  }
  for (int chunk = chunk0; chunk < chunk_end; ++chunk) {
    __syncthreads();                                        // everyone has finished the previous chunk
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int c4 = tid + 256 * u, row = c4 >> 5, col = (c4 & 31) * 4;
      *reinterpret_cast<float4*>(&kst[row * kStride + col]) = pre[u];
    }
    if (chunk + 1 < chunk_end) { THRIFT_LOAD_CHUNK(chunk + 1) }
    __syncthreads();
    const int j = chunk * 64 + lane;
    if (j >= cap) continue;
    if (shared) {
      // one score per block for the whole group; every head's key row receives it
      if (wave == 0) {
        double s = 0.0;
#pragma unroll 8
        for (int d = 0; d < kD; d += 4) {
          const float4 kv = *reinterpret_cast<const float4*>(&kst[lane * kStride + d]);
          s = fma(qsum[d], (double)kv.x, s);
          s = fma(qsum[d + 1], (double)kv.y, s);
          s = fma(qsum[d + 2], (double)kv.z, s);
          s = fma(qsum[d + 3], (double)kv.w, s);
        }
        const uint64_t key = order_key64(s);
        for (int g = 0; g < G; ++g) keys[((size_t)b * Hq + kvh * G + g) * Tk + j] = key;
      }
      continue;
    }
    for (int g = wave; g < G; g += 4) {
      double s = 0.0;
#pragma unroll 8
      for (int d = 0; d < kD; d += 4) {
        const float4 kv = *reinterpret_cast<const float4*>(&kst[lane * kStride + d]);
        const float4 qv = *reinterpret_cast<const float4*>(&qst[g * kD + d]);
        s = fma((double)qv.x, (double)kv.x, s);
        s = fma((double)qv.y, (double)kv.y, s);
        s = fma((double)qv.z, (double)kv.z, s);
        s = fma((double)qv.w, (double)kv.w, s);
      }
      keys[((size_t)b * Hq + kvh * G + g) * Tk + j] = order_key64(s);
    }
  }
#undef THRIFT_LOAD_CHUNK
}

struct DecodeSelectArgs {
  const uint64_t* keys;       // [B*Hq][Tk]
  const int32_t* seqlens;
  unsigned long long* bitmap; // [B*Hq][words]
  int32_t* idx_out;           // nullable [B*Hq][kmax_out]
  int32_t* cnt_out;           // nullable [B*Hq]
  int Hq, Tk, words, kmax_out, fixed_k;
  long long ppm;
};

// One wavefront per row, no barriers: lane l keeps key blocks l, l+64, ... in registers; the k-th largest
// key is found by a 64-step bitwise search whose counts are ballots + scalar popcounts.
template <int MAXC>
__global__ void __launch_bounds__(256) decode_select_kernel(DecodeSelectArgs p, long n_rows) {
  const int lane = threadIdx.x & 63;
  const long row = (long)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  if (row >= n_rows) return;
  const int b = (int)(row / p.Hq);
  const int vis = p.seqlens ? min(p.Tk, (max(0, p.seqlens[b]) + kBk - 1) / kBk) : p.Tk;
  int k;
  if (p.fixed_k >= 0) k = min(p.fixed_k, vis);
  else if (p.ppm <= 0 || vis == 0) k = 0;
  else {
    long long kk = (p.ppm * (long long)vis + 999999LL) / 1000000LL;
    k = (int)max(1LL, min(kk, (long long)vis));
  }
  uint64_t key[MAXC];
#pragma unroll
  for (int c = 0; c < MAXC; ++c) {
    const int j = c * 64 + lane;
    key[c] = j < vis ? p.keys[row * p.Tk + j] : 0ULL;
  }
  unsigned long long* bm = p.bitmap + row * p.words;
  int32_t* out = p.idx_out ? p.idx_out + row * p.kmax_out : nullptr;
  if (p.cnt_out && lane == 0) p.cnt_out[row] = k;
  if (k <= 0) {
    for (int w = lane; w < p.words; w += 64) bm[w] = 0ULL;
    if (out) for (int t = lane; t < p.kmax_out; t += 64) out[t] = -1;
    return;
  }
  // Invalid slots hold key 0, and every candidate below is >= 1, so they never count.  Each lane counts
  // its own keys (at most MAXC <= 64, seven bits); the wavefront total is the weighted popcount of the
  // ballots of those seven bits.
  auto wave_total = [&](int n_lane) -> int {
    int tot = 0;
#pragma unroll
    for (int b7 = 0; b7 < 7; ++b7) tot += __popcll(__ballot((n_lane >> b7) & 1)) << b7;
    return tot;
  };
  uint64_t T = 0;
  for (int bit = 63; bit >= 0; --bit) {
    const uint64_t cand = T | (1ULL << bit);
    int n_lane = 0;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) n_lane += key[c] >= cand ? 1 : 0;
    const int n = wave_total(n_lane);
    if (n >= k) T = cand;
    if (n == k) break;                                       // exactly the k largest lie at or above cand: done
  }
  int n_gt;
  {
    int n_lane = 0;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) n_lane += key[c] > T ? 1 : 0;
    n_gt = wave_total(n_lane);
  }
  const int need_ties = k - n_gt;                            // keys equal to T, taken from the smallest id up (0 after an early exit above a gap)
  const uint64_t lt_mask = (1ULL << lane) - 1ULL;
  int written = 0, ties_seen = 0;
#pragma unroll
  for (int c = 0; c < MAXC; ++c) {
    if (c * 64 < vis) {
      const bool valid = c * 64 + lane < vis;
      const bool tie = valid && key[c] == T;
      const uint64_t tie_b = __ballot(tie);
      const bool sel = valid && (key[c] > T || (tie && ties_seen + __popcll(tie_b & lt_mask) < need_ties));
      const uint64_t sel_b = __ballot(sel);
      if (sel && out) out[written + __popcll(sel_b & lt_mask)] = c * 64 + lane;
      written += __popcll(sel_b);
      ties_seen += __popcll(tie_b);
      if (lane == 0) bm[c] = sel_b;
    } else if (lane == 0 && c < p.words) {
      bm[c] = 0ULL;
    }
  }
  if (out) for (int t = k + lane; t < p.kmax_out; t += 64) out[t] = -1;
}

void launch_decode_select(const uint16_t* q16, int q_is_bf16, const float* kmean, const int32_t* seqlens, uint64_t* keys,
                          unsigned long long* bitmap, int words, int32_t* idx_out, int32_t* cnt_out, int kmax_out,
                          int B, int Hq, int Hkv, int Tk, int fixed_k, long long ppm, int shared, hipStream_t st) {
  const int chunks = (Tk + 63) / 64;
  const int score_groups = (chunks + kScoreChunksPerWg - 1) / kScoreChunksPerWg;
  decode_scores_kernel<<<dim3((unsigned)((long)B * Hkv * score_groups)), dim3(256), 0, st>>>(q16, q_is_bf16, kmean, seqlens, keys, Hq, Hkv, Tk, shared);
  DecodeSelectArgs p;
  p.keys = keys; p.seqlens = seqlens; p.bitmap = bitmap; p.idx_out = idx_out; p.cnt_out = cnt_out;
  p.Hq = Hq; p.Tk = Tk; p.words = words; p.kmax_out = kmax_out; p.fixed_k = fixed_k; p.ppm = ppm;
  const long n_rows = (long)B * Hq;
  const dim3 grid((unsigned)((n_rows + 3) / 4)), block(256);
  if (chunks <= 8) decode_select_kernel<8><<<grid, block, 0, st>>>(p, n_rows);
  else if (chunks <= 16) decode_select_kernel<16><<<grid, block, 0, st>>>(p, n_rows);
  else if (chunks <= 32) decode_select_kernel<32><<<grid, block, 0, st>>>(p, n_rows);
  else decode_select_kernel<64><<<grid, block, 0, st>>>(p, n_rows);
}

// Log-sum-exp merge of the partials of one (sequence, query head): 128 threads, one per channel.
__global__ void __launch_bounds__(128) decode_merge_kernel(DecodeArgs a) {
  const size_t qh = blockIdx.x;
  const int ch = threadIdx.x;
  const float c = a.scale * 1.4426950408889634f;
  const float* ml = a.part_ml + qh * a.nparts * 2;
  float M = -INFINITY;
  for (int p = 0; p < a.nmerge; ++p) M = fmaxf(M, ml[2 * p]);
  float L = 0.f, O = 0.f;
  if (M > -INFINITY) {
    // an empty partial has m = -inf, l = 0, O = 0: its weight exp2(-inf) is 0, no branch needed, and the
    // loads of all partials can be in flight together
#pragma unroll 8
    for (int p = 0; p < a.nmerge; ++p) {
      const float w = fast_exp2((ml[2 * p] - M) * c);
      L += w * ml[2 * p + 1];
      O += w * a.part_o[(qh * a.nparts + p) * kD + ch];
    }
  }
  const float x = L > 0.f ? O / L : 0.f;
  if (a.out_dt == THRIFT_F32) ((float*)a.out)[qh * kD + ch] = x;
  else if (a.out_dt == THRIFT_F16) ((uint16_t*)a.out)[qh * kD + ch] = F16::from_float(x);
  else ((uint16_t*)a.out)[qh * kD + ch] = BF16::from_float(x);
}

void launch_decode(const DecodeArgs& a, hipStream_t st) {
  const unsigned grid = (unsigned)((long)a.B * a.Hkv * a.nsplit);
  if (a.dt == THRIFT_F16) decode_partial_kernel<F16, false><<<dim3(grid), dim3(256), 0, st>>>(a);
  else decode_partial_kernel<BF16, false><<<dim3(grid), dim3(256), 0, st>>>(a);
  if (a.seqlens != nullptr) {                          // without lengths every sequence fills the cache: no partly filled block
    const unsigned tail_grid = (unsigned)((long)a.B * a.Hkv);
    if (a.dt == THRIFT_F16) decode_partial_kernel<F16, true><<<dim3(tail_grid), dim3(64), 0, st>>>(a);
    else decode_partial_kernel<BF16, true><<<dim3(tail_grid), dim3(64), 0, st>>>(a);
  }
  decode_merge_kernel<<<dim3((unsigned)((long)a.B * a.Hq)), dim3(128), 0, st>>>(a);
}

}  // namespace thrift
