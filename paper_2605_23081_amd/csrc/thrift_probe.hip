// Measurement helpers: microbenchmarks of the hardware rates the roofline figures are priced against, built from
// the same tile routines the attention kernels use.  Not part of the method; the benchmark calls them through
// thrift_peak_probe and times each launch with events.
//   MFMA issue peaks (scaled-FP4 32x32x64, 16-bit 32x32x16): independent accumulators, nothing else in the loop.
//   HBM read stream: one pass over a buffer, 16-byte loads, a few in flight per lane.
//   Vector-ALU part of one 4-bit wave-tile (32 queries x 64 keys): the online-softmax update and the P quantiser
//   exactly as the fused kernel executes them, without matrix instructions, staging or barriers, at the fused
//   kernel's occupancy (three workgroups of four wavefronts per CU); and the same with the tile's eight MFMAs.
#include "thrift_launch.h"
#include "thrift_tile.h"

namespace thrift {

constexpr int kProbeLds = 50176;     // the fused kernel's LDS footprint: pins three workgroups per CU

template <int KIND, typename T>
__global__ void __launch_bounds__(256, 3) peak_mfma_kernel(float* out, int iters) {
  __shared__ unsigned char pad[kProbeLds];
  const int lane = threadIdx.x & 63;
  v4i a = {lane * 3, lane * 5, lane * 7, lane * 11}, b = {lane, lane ^ 21, lane * 13, lane + 5};
  v16f acc[4];
#pragma unroll
  for (int n = 0; n < 4; ++n) acc[n] = (v16f){0.f};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int n = 0; n < 4; ++n) {
        if (KIND == THRIFT_PEAK_MFMA_MXFP4)
          acc[n] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen(a), widen(b), acc[n], 4, 4, 0, 0x7f7f7f7f, 0, 0x7f7f7f7f);
        else
          acc[n] = T::mfma(__builtin_bit_cast(v8s, a), __builtin_bit_cast(v8s, b), acc[n]);
      }
  }
  float r = 0.f;
#pragma unroll
  for (int n = 0; n < 4; ++n) r += acc[n][0] + acc[n][9];
  pad[threadIdx.x] = (unsigned char)lane;
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = r + (float)pad[(threadIdx.x * 7) & 255];
}

__global__ void __launch_bounds__(256) peak_hbm_read_kernel(const uint4* __restrict__ src, size_t n16, float* out) {
  // Each workgroup streams one contiguous 16 KiB segment, four independent 16-byte loads per lane, marked as not to be
  // kept in the caches: the shape that read the fastest of those tried (grid-stride sweeps and fewer, longer segments
  // were 2 to 12 % slower).
  typedef unsigned int u4 __attribute__((ext_vector_type(4)));
  const u4* p = reinterpret_cast<const u4*>(src) + (size_t)blockIdx.x * 1024 + threadIdx.x;
  uint32_t acc = 0;
  if (((size_t)blockIdx.x + 1) * 1024 <= n16) {
    const u4 x0 = __builtin_nontemporal_load(p), x1 = __builtin_nontemporal_load(p + 256), x2 = __builtin_nontemporal_load(p + 512),
             x3 = __builtin_nontemporal_load(p + 768);
    acc = x0.x ^ x0.y ^ x0.z ^ x0.w ^ x1.x ^ x1.y ^ x1.z ^ x1.w ^ x2.x ^ x2.y ^ x2.z ^ x2.w ^ x3.x ^ x3.y ^ x3.z ^ x3.w;
  }
  if (acc == 0x9e3779b9u) out[blockIdx.x & 255] = 1.f;      // practically never: keeps the loads alive without a store per thread
}

template <bool WITH_MFMA>
__global__ void __launch_bounds__(256, 3) peak_tile_mix_kernel(float* out, int iters, float c) {
  __shared__ unsigned char pad[kProbeLds];
  const int lane = threadIdx.x & 63;
  v4i kf[2] = {(v4i){lane * 3, lane * 5, lane * 7, lane * 11}, (v4i){lane, lane ^ 21, lane * 13, lane + 5}};
  v4i qf[2] = {(v4i){lane * 17, lane * 19, lane, 3}, (v4i){lane + 9, lane * 23, 1, lane}};
  v4i vf[4];
#pragma unroll
  for (int n = 0; n < 4; ++n) vf[n] = (v4i){lane + n, lane * (n + 2), n, lane ^ n};
  v16f o[4];
#pragma unroll
  for (int n = 0; n < 4; ++n) o[n] = (v16f){0.f};
  RowState st = {kEmptyMax, 0.f};
  v16f s[2];
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int i = 0; i < 16; ++i) s[t][i] = 0.01f * (float)((lane * 7 + t * 16 + i) & 63) - 0.3f;
  uint32_t keep = 0;
  for (int it = 0; it < iters; ++it) {
    if (WITH_MFMA) {
      // S^T of the tile: four scaled-FP4 MFMAs on register operands (scores far below the running maximum)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        asm volatile("" : "+v"(kf[t]));               // a new K fragment as far as the compiler knows: the MFMAs stay in the loop
        v16f acc = {0.f};
        acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen(kf[t]), widen(qf[0]), acc, 4, 4, 0, 0x70707070, 0, 0x70707070);
        acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen(kf[t ^ 1]), widen(qf[1]), acc, 4, 4, 1, 0x70707070, 1, 0x70707070);
        s[t] = acc;
      }
    } else {
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) { float x = s[t][i]; asm volatile("" : "+v"(x)); s[t][i] = x; }   // last trip's probabilities serve as scores: no instruction spent
    }
    float alpha;
    uint32_t pb;
    const bool grew = softmax_update(s, lane, false, kBk, c, st, alpha, pb);
    rescale(o, grew, alpha);
    if (WITH_MFMA) {
      pv_fp4_regs<true>(s, pb, 0x7f7f7f7fu, 0u, 0u, 0u, vf[0], vf[1], vf[2], vf[3], o);
    } else {
      const v4i pq = quantize_p_group(s, pb);
      keep ^= (uint32_t)(pq[0] ^ pq[1] ^ pq[2] ^ pq[3]);
    }
  }
  float r = st.m + st.l + (float)(keep & 1u);
#pragma unroll
  for (int n = 0; n < 4; ++n) r += o[n][0] + o[n][9];
  pad[threadIdx.x] = (unsigned char)lane;
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = r + (float)pad[(threadIdx.x * 7) & 255];
}

// Returns the work of one launch: flops (MFMA kinds), bytes (HBM), wave-tiles (tile mixes); 0 for an unknown kind.
double launch_peak_probe(int kind, thrift_dtype dt, int iters, void* buffer, size_t bytes, hipStream_t st) {
  // 48 workgroups per CU in all: the CUs are refilled as workgroups retire and hold three at a time on average, like
  // under the fused kernel's long grid (a grid of exactly three per CU was placed unevenly and ran at two per SIMD)
  constexpr int kGrid = 256 * 3 * 16;
  float* out = (float*)buffer;                          // every probe but the HBM one writes kGrid * 256 floats
  switch (kind) {
    case THRIFT_PEAK_MFMA_MXFP4:
      peak_mfma_kernel<THRIFT_PEAK_MFMA_MXFP4, BF16><<<dim3(kGrid), dim3(256), 0, st>>>(out, iters);
      return (double)kGrid * 4 * iters * 16 * (2.0 * 32 * 32 * 64);
    case THRIFT_PEAK_MFMA_16:
      if (dt == THRIFT_F16) peak_mfma_kernel<THRIFT_PEAK_MFMA_16, F16><<<dim3(kGrid), dim3(256), 0, st>>>(out, iters);
      else peak_mfma_kernel<THRIFT_PEAK_MFMA_16, BF16><<<dim3(kGrid), dim3(256), 0, st>>>(out, iters);
      return (double)kGrid * 4 * iters * 16 * (2.0 * 32 * 32 * 16);
    case THRIFT_PEAK_HBM_READ: {
      const size_t tail = 65536;                        // the last 64 KiB are the (never read) output region
      const size_t segments = (bytes - tail) / 16384;   // whole 16 KiB segments only
      if (segments == 0 || segments > 0x7fffffffu) return -1.0;
      peak_hbm_read_kernel<<<dim3((unsigned)segments), dim3(256), 0, st>>>((const uint4*)buffer, segments * 1024,
                                                                           (float*)((char*)buffer + (bytes - tail)));
      return (double)segments * 16384.0;
    }
    case THRIFT_PEAK_VALU_SOFTMAX:
      peak_tile_mix_kernel<false><<<dim3(kGrid), dim3(256), 0, st>>>(out, iters, 0.1275f);
      return (double)kGrid * 4 * iters;
    case THRIFT_PEAK_TILE_MIX:
      peak_tile_mix_kernel<true><<<dim3(kGrid), dim3(256), 0, st>>>(out, iters, 0.1275f);
      return (double)kGrid * 4 * iters;
  }
  return 0.0;
}

}  // namespace thrift
