// Pre-pass kernels of Algorithm 1: block token means (step 3), MXFP4 quantisation (step 2) and
// block-pair scoring + per-row TopK (step 5).  All three are streaming / latency kernels: coalesced
// 16-byte loads, wavefront shuffles and ballots for the reductions, no matrix units.
#include "thrift_device.h"
#include "thrift_launch.h"

namespace thrift {

// ------------------------------------------------------------------------------------------------
// Block means (Sec. 3.2): one workgroup per (b, h, block).  256 threads = 16 row slices x 16 column
// groups of 8 channels; each thread streams rows slice, slice+16, ... with 16-byte loads and adds
// in fp64 (the sum of a block of 16-bit values is then exact, so the result does not depend on the
// order of the additions and matches a serial fp64 mean bit for bit).
// ------------------------------------------------------------------------------------------------
// N need not be a multiple of the block: a head has ceil(N/block) blocks and the last one is the mean
// of the tokens it has.
template <typename T>
__global__ void __launch_bounds__(256) block_means_kernel(const uint16_t* __restrict__ x, float* __restrict__ means,
                                                          int block, int N, int blocks_per_head) {
  const int tid = threadIdx.x;
  const int cg = tid & 15, rs = tid >> 4;
  const int head = blockIdx.x / blocks_per_head, t = blockIdx.x % blocks_per_head;
  const int count = min(block, N - t * block);            // tokens of this block
  const uint16_t* base = x + ((size_t)head * N + (size_t)t * block) * kD + cg * 8;
  double acc[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) acc[c] = 0.0;
  for (int r = rs; r < count; r += 16) {
    uint4 w = *reinterpret_cast<const uint4*>(base + (size_t)r * kD);
    uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      acc[2 * c] += (double)T::to_float((uint16_t)(ww[c] & 0xffffu));
      acc[2 * c + 1] += (double)T::to_float((uint16_t)(ww[c] >> 16));
    }
  }
  // row slices rs and rs^1, rs^2 sit 16 and 32 lanes apart inside a wavefront
#pragma unroll
  for (int c = 0; c < 8; ++c) {
    acc[c] += __shfl_xor(acc[c], 16);
    acc[c] += __shfl_xor(acc[c], 32);
  }
  __shared__ double part[4][16][8];
  const int wave = tid >> 6;
  if ((tid & 63) < 16) {
#pragma unroll
    for (int c = 0; c < 8; ++c) part[wave][cg][c] = acc[c];
  }
  __syncthreads();
  if (tid < kD) {
    const int g = tid >> 3, c = tid & 7;
    double s = part[0][g][c] + part[1][g][c] + part[2][g][c] + part[3][g][c];
    means[(size_t)blockIdx.x * kD + tid] = (float)(s / (double)count);
  }
}

void launch_block_means(const void* x, thrift_dtype dt, long heads, int N, int block, float* means, hipStream_t st) {
  const int per_head = (N + block - 1) / block;
  const unsigned grid = (unsigned)(heads * per_head);
  if (dt == THRIFT_F16)
    block_means_kernel<F16><<<dim3(grid), dim3(256), 0, st>>>((const uint16_t*)x, means, block, N, per_head);
  else
    block_means_kernel<BF16><<<dim3(grid), dim3(256), 0, st>>>((const uint16_t*)x, means, block, N, per_head);
}

// axis 0: one thread per group of 32 consecutive channels (64 bytes in, 16 code bytes + 1 scale out).
template <typename T>
__global__ void __launch_bounds__(256) quantize_axis0_kernel(const uint16_t* __restrict__ x, uint8_t* __restrict__ codes,
                                                             uint8_t* __restrict__ scales, size_t n_groups) {
  const size_t g = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (g >= n_groups) return;
  const uint4* src = reinterpret_cast<const uint4*>(x + g * 32);
  uint32_t pair[16];
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    uint4 w = src[t];
    pair[4 * t] = w.x; pair[4 * t + 1] = w.y; pair[4 * t + 2] = w.z; pair[4 * t + 3] = w.w;
  }
  uint32_t out[4];
  const uint32_t sb = quantize_group32<T>(pair, out);
  *reinterpret_cast<uint4*>(codes + g * 16) = make_uint4(out[0], out[1], out[2], out[3]);
  scales[g] = (uint8_t)sb;
}

// axis 1: one workgroup per (b, h, 64-token block).  The 64 x 128 tile is staged through LDS with
// coalesced 16-byte loads; thread (token group g, channel c) then walks its 32 tokens down a column.
// Output tile: [channel][32 bytes] (tokens 2t, 2t+1 in byte t), scales [2 groups][128 channels].
// N need not be a multiple of 64: a head has ceil(N/64) blocks; tokens past the end count as +0 (they
// do not change a group's largest magnitude and encode as code 0), so a short last group is quantised
// from the tokens it has and the padded codes are zeros.
template <typename T>
__global__ void __launch_bounds__(256) quantize_axis1_kernel(const uint16_t* __restrict__ x, uint8_t* __restrict__ codes,
                                                             uint8_t* __restrict__ scales, int N, int blocks_per_head) {
  constexpr int kRow = kD + 8;  // padded row (in 16-bit elements): keeps 16-byte alignment, spreads banks
  __shared__ __align__(16) uint16_t tile[64 * kRow];
  const int tid = threadIdx.x;
  const int head = blockIdx.x / blocks_per_head, t = blockIdx.x % blocks_per_head;
  const int count = min(64, N - t * 64);
  const uint16_t* src = x + ((size_t)head * N + (size_t)t * 64) * kD;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int chunk = tid + 256 * u;           // 1024 chunks of 8 elements
    const int row = chunk >> 4, col = (chunk & 15) * 8;
    *reinterpret_cast<uint4*>(&tile[row * kRow + col]) =
        row < count ? *reinterpret_cast<const uint4*>(src + row * kD + col) : make_uint4(0, 0, 0, 0);
  }
  __syncthreads();
  const int g = tid >> 7, c = tid & 127;
  uint32_t pair[16];
#pragma unroll
  for (int u = 0; u < 16; ++u) {
    uint32_t lo = tile[(32 * g + 2 * u) * kRow + c], hi = tile[(32 * g + 2 * u + 1) * kRow + c];
    pair[u] = lo | (hi << 16);
  }
  uint32_t out[4];
  const uint32_t sb = quantize_group32<T>(pair, out);
  *reinterpret_cast<uint4*>(codes + ((size_t)blockIdx.x * kD + c) * 32 + g * 16) = make_uint4(out[0], out[1], out[2], out[3]);
  scales[((size_t)blockIdx.x * 2 + g) * kD + c] = (uint8_t)sb;
}

void launch_quantize(const void* x, thrift_dtype dt, long bh, int N, int axis, uint8_t* codes, uint8_t* scales, hipStream_t st) {
  const uint16_t* xs = (const uint16_t*)x;
  if (axis == 0) {
    size_t n_groups = (size_t)bh * N * (kD / 32);
    unsigned grid = (unsigned)((n_groups + 255) / 256);
    if (dt == THRIFT_F16) quantize_axis0_kernel<F16><<<dim3(grid), dim3(256), 0, st>>>(xs, codes, scales, n_groups);
    else quantize_axis0_kernel<BF16><<<dim3(grid), dim3(256), 0, st>>>(xs, codes, scales, n_groups);
  } else {
    const int per_head = (N + 63) / 64;
    unsigned grid = (unsigned)(bh * per_head);
    if (dt == THRIFT_F16) quantize_axis1_kernel<F16><<<dim3(grid), dim3(256), 0, st>>>(xs, codes, scales, N, per_head);
    else quantize_axis1_kernel<BF16><<<dim3(grid), dim3(256), 0, st>>>(xs, codes, scales, N, per_head);
  }
}

// ------------------------------------------------------------------------------------------------
// Scores + TopK (Sec. 3.2; Alg. 1 step 5).  A workgroup of 4 wavefronts serves 4 consecutive rows of
// one (b, kv head) in the order (query block, head of the group): they share the staged key-block
// means.  Each wavefront owns one row: lane l scores key blocks l, l+64, ... in fp64, keeps them in
// registers as order-preserving 64-bit keys, finds the k-th largest key by a bitwise search with
// ballot/popcount counting, and emits the selected ids in ascending order.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ int visible_blocks_dev(int i, int Tk, int Bq, int Bk, int causal, int off) {
  if (!causal) return Tk;
  long long last_q = ((long long)i + off + 1) * Bq - 1;
  long long v = last_q / Bk + 1;
  return (int)(v > Tk ? Tk : (v < 0 ? 0 : v));
}

__device__ __forceinline__ int row_budget_dev(int visible, long long ppm, int fixed_k) {
  if (fixed_k >= 0) return fixed_k < visible ? fixed_k : visible;
  if (ppm <= 0) return 0;
  long long k = (ppm * (long long)visible + 999999LL) / 1000000LL;
  if (k < 1) k = 1;
  if (k > visible) k = visible;
  return (int)k;
}

__device__ __forceinline__ uint64_t order_key(double s) {
  uint64_t u = (uint64_t)__double_as_longlong(s);
  return (u >> 63) ? ~u : (u | 0x8000000000000000ULL);   // larger double <=> larger key
}

// Output number n of the SplitMix64 generator seeded with `seed` (Steele, Lea, Flood 2014).
__device__ __forceinline__ uint64_t splitmix64_output(uint64_t seed, uint64_t n) {
  uint64_t z = seed + n * 0x9e3779b97f4a7c15ULL;
  z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ULL;
  z = (z ^ (z >> 27)) * 0x94d049bb133111ebULL;
  return z ^ (z >> 31);
}

template <int MAXC, int NW>
__global__ void __launch_bounds__(NW * 64) select_topk_kernel(SelectArgs p) {
  constexpr int kQuarter = kD / 4;                      // channels staged at a time
  constexpr int kStride = kQuarter + 4;                 // padded fp32 quarter row of a staged key mean: conflict-free 16-byte reads
  constexpr int kPer = 2048 / (NW * 64);                // 16-byte pieces of a staged piece per thread
  __shared__ __align__(16) float kst[256 * kStride];
  __shared__ __align__(16) double qsd[NW][kD];          // the row's query mean (shared mode: summed over the group's heads)
  const int tid = threadIdx.x, lane = tid & 63;
  // wavefront-uniform, and known to the compiler as such: the row, its visible blocks and budget, the threshold and the
  // counts of the search below then live in scalar registers (left as a per-lane value, every count of the search went
  // through vector registers and a branch per chunk: 3600 vector instructions per row instead of 1500)
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int G = p.Hq / p.Hkv;
  const int GR = p.shared ? 1 : G;                      // selection rows per query block and KV head
  const int nheads = p.shared ? G : 1;                  // heads that receive a row's result
  const int rows_per_unit = p.Tq * GR;                  // rows of one (b, kv head), ordered (i, head in group)
  const int wgs_per_unit = (rows_per_unit + NW - 1) / NW;
  // Grid order: the last (under a causal mask: longest) rows of every (b, kv head) first, the units interleaved, so
  // that the launch does not end on its longest workgroups and a KV head's means stay in one XCD's L2 (8 units)
  const int units = p.B * p.Hkv;
  const int unit = blockIdx.x % units;
  const int row0 = (wgs_per_unit - 1 - (int)(blockIdx.x / units)) * NW;
  const int b = unit / p.Hkv, kvh = unit % p.Hkv;
  const int row = row0 + wave;
  const bool active = row < rows_per_unit;
  const int i = active ? row / GR : 0;
  const int hq = kvh * G + (active ? row % GR : 0);     // first (or only) head of the row
  const int cap = p.Tk;
  const int vis = active ? min(cap, visible_blocks_dev(i, p.Tk, p.Bq, p.Bk, p.causal, p.q_block_offset)) : 0;
  const int k = row_budget_dev(vis, p.ppm, p.fixed_k);
  const int last_row = min(row0 + NW - 1, rows_per_unit - 1);
  const int vis_max = min(cap, visible_blocks_dev(last_row / GR, p.Tk, p.Bq, p.Bk, p.causal, p.q_block_offset));
  const size_t rowid = ((size_t)b * p.Hq + hq) * p.Tq + i;

  if (active && p.selector == 0) {
    // fp64 sum over the heads in ascending order (one head: the value itself)
    double q0 = 0.0, q1 = 0.0;
    for (int hh = 0; hh < nheads; ++hh) {
      const float* qm = p.qmean + (rowid + (size_t)hh * p.Tq) * kD;
      q0 += (double)qm[lane];
      q1 += (double)qm[lane + 64];
    }
    qsd[wave][lane] = q0;
    qsd[wave][lane + 64] = q1;
  }
  const float* kbase = p.kmean + ((size_t)b * p.Hkv + kvh) * p.Tk * kD;

  // Every step of a key's chain reads the key mean (per lane) and the query mean (the same address in all lanes, but a
  // full read all the same); with one chain per lane those reads took most of the CU's one LDS pipe.  So a lane walks the
  // chains of four keys (one of each of four 64-key chunks) side by side and reads the query mean once for the four:
  // half the LDS reads per score, and four independent chains of fused multiply-adds.  256 key means are staged a quarter of their channels at a time (36 KiB), fetched into registers while
  // the quarter before is being scored and handed to LDS between two barriers; the workgroup's rows share every
  // staged piece (16 rows: a quarter of the L2 reads of 4).
  float4 nx[kPer];
  auto fetch = [&](int t) {                              // piece t: keys 256*(t/4) .. +255, channels 32*(t%4) .. +31
    const int key0 = (t >> 2) * 256, ch0 = (t & 3) * kQuarter;
#pragma unroll
    for (int u = 0; u < kPer; ++u) {
      const int chunk = tid + NW * 64 * u;               // 2048 pieces of 4 floats
      const int r = chunk >> 3, col = (chunk & 7) * 4;
      nx[u] = key0 + r < p.Tk ? *reinterpret_cast<const float4*>(kbase + (size_t)(key0 + r) * kD + ch0 + col) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  };

  uint64_t key[MAXC];
#pragma unroll
  for (int c = 0; c < MAXC; ++c) key[c] = 0;
  if (p.selector != 0) {
    // Ablation selectors (App. A): the same k-th-largest search over other keys.  Random: output
    // number n+1 of the SplitMix64 stream of `seed`, n = rowid * 2^32 + j; diagonal: the block id.
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
      const int j = c * 64 + lane;
      if (j < vis) key[c] = p.selector == 1 ? splitmix64_output(p.seed, (((uint64_t)rowid << 32) | (uint64_t)j) + 1ULL) : (uint64_t)j + 1ULL;
    }
  } else {
    if (vis_max > 0) fetch(0);
#pragma unroll
    for (int cg = 0; cg < MAXC / 4; ++cg) {
      if (cg * 256 < vis_max) {                          // uniform over the workgroup
        double sc[4] = {0.0, 0.0, 0.0, 0.0};             // the chains of keys 256*cg + 64*cc + lane
#pragma unroll 1
        for (int h = 0; h < 4; ++h) {
          __syncthreads();                               // the piece before has been scored by every row
#pragma unroll
          for (int u = 0; u < kPer; ++u) {
            const int chunk = tid + NW * 64 * u;
            const int r = chunk >> 3, col = (chunk & 7) * 4;
            *reinterpret_cast<float4*>(&kst[r * kStride + col]) = nx[u];      // rows beyond Tk: zeros, never used
          }
          const int t1 = cg * 4 + h + 1;
          if (t1 < MAXC && (t1 >> 2) * 256 < vis_max) fetch(t1);              // uniform over the workgroup
          __syncthreads();
          if (cg * 256 < vis) {                          // uniform over the wavefront; keys past `vis` are scored and dropped
#pragma unroll
            for (int d = 0; d < kQuarter; d += 4) {
              const double2 qa = *reinterpret_cast<const double2*>(&qsd[wave][h * kQuarter + d]);
              const double2 qb = *reinterpret_cast<const double2*>(&qsd[wave][h * kQuarter + d + 2]);
#pragma unroll
              for (int cc = 0; cc < 4; ++cc) {
                const float4 kv = *reinterpret_cast<const float4*>(&kst[(cc * 64 + lane) * kStride + d]);
                sc[cc] = fma(qa.x, (double)kv.x, sc[cc]);
                sc[cc] = fma(qa.y, (double)kv.y, sc[cc]);
                sc[cc] = fma(qb.x, (double)kv.z, sc[cc]);
                sc[cc] = fma(qb.y, (double)kv.w, sc[cc]);
              }
            }
          }
        }
#pragma unroll
        for (int cc = 0; cc < 4; ++cc)
          if ((cg * 4 + cc) * 64 + lane < vis) key[cg * 4 + cc] = order_key(sc[cc]);
      }
    }
  }
  if (!active) return;

  if (lane == 0)
    for (int hh = 0; hh < nheads; ++hh) p.cnt[rowid + (size_t)hh * p.Tq] = k;
  if (k <= 0) {
    for (int hh = 0; hh < nheads; ++hh)
      for (int t = lane; t < p.kmax; t += 64) p.idx[(rowid + (size_t)hh * p.Tq) * p.kmax + t] = -1;
    return;
  }
  // k-th largest key: greatest T with |{key >= T}| >= k, built bit by bit from the top
  uint64_t T = 0;
  for (int bit = 63; bit >= 0; --bit) {
    const uint64_t cand = T | (1ULL << bit);
    int n = 0;
#pragma unroll
    for (int c = 0; c < MAXC; ++c)
      if (c * 64 < vis) n += __popcll(__ballot(key[c] >= cand));        // cand > 0 = the key of a lane without a block
    if (n >= k) T = cand;
    if (n == k) break;                                   // exactly the k largest lie at or above cand: done
  }
  int n_gt = 0;
#pragma unroll
  for (int c = 0; c < MAXC; ++c)
    if (c * 64 < vis) n_gt += __popcll(__ballot((c * 64 + lane < vis) && key[c] > T));
  const int need_ties = k - n_gt;                        // ties at T, taken from the smallest id up (0 after an early exit above a gap)
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
      if (sel)
        for (int hh = 0; hh < nheads; ++hh)
          p.idx[(rowid + (size_t)hh * p.Tq) * p.kmax + written + __popcll(sel_b & lt_mask)] = c * 64 + lane;
      written += __popcll(sel_b);
      ties_seen += __popcll(tie_b);
    }
  }
  for (int hh = 0; hh < nheads; ++hh)
    for (int t = k + lane; t < p.kmax; t += 64) p.idx[(rowid + (size_t)hh * p.Tq) * p.kmax + t] = -1;
}

void launch_select_topk(const SelectArgs& p, hipStream_t st) {
  const int G = p.shared ? 1 : p.Hq / p.Hkv;
  const int chunks = (p.Tk + 63) / 64;
  // 16 rows per workgroup where a (b, kv head) has that many and the keys of a row fit 128 registers per lane
  const int nw = (p.Tq * G >= 16 && chunks <= 32) ? 16 : 4;
  const int wgs_per_unit = (p.Tq * G + nw - 1) / nw;
  const dim3 grid((unsigned)((long)p.B * p.Hkv * wgs_per_unit));
  if (nw == 16) {
    if (chunks <= 8) select_topk_kernel<8, 16><<<grid, dim3(1024), 0, st>>>(p);
    else if (chunks <= 16) select_topk_kernel<16, 16><<<grid, dim3(1024), 0, st>>>(p);
    else select_topk_kernel<32, 16><<<grid, dim3(1024), 0, st>>>(p);
  } else {
    if (chunks <= 8) select_topk_kernel<8, 4><<<grid, dim3(256), 0, st>>>(p);
    else if (chunks <= 16) select_topk_kernel<16, 4><<<grid, dim3(256), 0, st>>>(p);
    else if (chunks <= 32) select_topk_kernel<32, 4><<<grid, dim3(256), 0, st>>>(p);
    else select_topk_kernel<64, 4><<<grid, dim3(256), 0, st>>>(p);
  }
}

}  // namespace thrift
