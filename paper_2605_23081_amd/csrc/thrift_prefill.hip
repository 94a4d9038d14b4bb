// Fused mixed-precision flash attention for prefill (Algorithm 1 steps 4-23; Sec. 3.3).
//
// One workgroup = one (batch, query head, query block); wavefront w owns query rows 32w .. 32w+31 of
// the block and keeps Q (4-bit and 16-bit fragments), the online-softmax state and the O^T accumulators
// in registers.  Key blocks are visited in ascending order (the order of Alg. 1); each block is staged
// once into LDS for all wavefronts — MXFP4 codes + scales for ordinary blocks, the 16-bit K/V tile for
// blocks listed in the row's TopK set — and dispatched per tile to the scaled-FP4 or the 16-bit MFMA
// path.  4-bit tiles are prefetched into registers two blocks ahead and written to the other of two LDS
// buffers one block ahead, so their global latency hides behind arithmetic and one barrier per block
// suffices.
//
// Differences from the kernel the paper sketches for Blackwell (Sec. 3.3): no two-phase split (4-bit
// tiles first, 16-bit helper afterwards) — on gfx950 both Q fragment sets fit in the 512-entry register
// file at two wavefronts per SIMD, and ascending order keeps the result independent of the schedule;
// LDS aliasing of the two tile formats is kept.
#include "thrift_launch.h"
#include "thrift_tile.h"

namespace thrift {

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also drains every outstanding global
// load (a full fence), which would wait for the 4-bit tile prefetched two blocks ahead at every key
// block; here only this wavefront's LDS reads and writes must have completed before the rendezvous.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <typename T, int NW>
__global__ void __launch_bounds__(NW * 64, 2) prefill_kernel(PrefillArgs a) {
  constexpr int NT = NW * 64;
  constexpr int CH = 256 / NT;                         // 16-byte chunks of a 4 KiB tile per thread
  __shared__ __align__(16) unsigned char lds[2 * kLdsBytes16];

  const int tid = threadIdx.x, lane = tid & 63, half = lane >> 5, r = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wavefront-uniform: loop bounds stay scalar
  const int N = a.N, Bq = NW * 32, Tq = N / Bq, Tk = N / kBk, G = a.Hq / a.Hkv;

  // ---- work item: heavy (late) query blocks first; KV heads spread over the 8 XCDs so that the query
  // heads and neighbouring query blocks that share a KV head also share an L2 ----
  const int units = a.B * a.Hkv, per_unit = G * Tq;
  int unit, within;
  if ((units & 7) == 0) {
    const int xcd = blockIdx.x & 7, t = blockIdx.x >> 3;
    unit = xcd + 8 * (t / per_unit);
    within = t % per_unit;
  } else {
    unit = blockIdx.x / per_unit;
    within = blockIdx.x % per_unit;
  }
  const int b = unit / a.Hkv, kvh = unit % a.Hkv;
  const int i = Tq - 1 - within / G;
  const int hq = kvh * G + within % G;
  const size_t qh = (size_t)b * a.Hq + hq, kh = (size_t)b * a.Hkv + kvh;
  const int q0 = i * Bq + wave * 32;                    // first query row of this wavefront
  const size_t qrow = qh * N + q0 + r;

  // ---- Q fragments ----
  v4i qf4[2];
  qf4[0] = *reinterpret_cast<const v4i*>(a.q4 + qrow * 64 + half * 16);
  qf4[1] = *reinterpret_cast<const v4i*>(a.q4 + qrow * 64 + 32 + half * 16);
  const uint32_t qsc = *reinterpret_cast<const uint32_t*>(a.qs + qrow * 4) >> (8 * half);
  const uint16_t* q16row = a.q + qrow * kD;

  const int vis = a.causal ? min(Tk, ((i + 1) * Bq - 1) / kBk + 1) : Tk;
  const int32_t* sel = a.idx + (qh * Tq + i) * a.kmax;
  const int nsel = a.cnt[qh * Tq + i];
  // the next three promoted block ids at or after the current block (ascending list)
  int ps = 0;
  int n0 = nsel > 0 ? sel[0] : 0x7fffffff, n1 = nsel > 1 ? sel[1] : 0x7fffffff, n2 = nsel > 2 ? sel[2] : 0x7fffffff;

  const uint8_t* k4base = a.k4 + kh * N * 64;
  const uint8_t* v4base = a.v4 + kh * (size_t)(N / 64) * 4096;
  const uint8_t* ksbase = a.ks + kh * N * 4;
  const uint8_t* vsbase = a.vs + kh * (size_t)(N / 32) * kD;
  const uint16_t* k16base = a.k + kh * N * kD;
  const uint16_t* v16base = a.v + kh * N * kD;

  // ---- staging.  A 4-bit tile travels global -> registers (one block ahead) -> LDS; each thread carries
  // CH 16-byte chunks of K and of V and (threads 0-127) one dword of scale bytes.  A 16-bit tile is copied
  // global -> LDS in place.  Two LDS buffers alternate, so one barrier per key block is enough. ----
  uint4 pk0 = make_uint4(0, 0, 0, 0), pk1 = pk0, pv0 = pk0, pv1 = pk0;
  uint32_t psc = 0;
#define THRIFT_PREFETCH4(J)                                                                                    \
  do {                                                                                                         \
    const uint8_t* kt_ = k4base + (size_t)(J) * 4096 + tid * 16;                                               \
    const uint8_t* vt_ = v4base + (size_t)(J) * 4096 + tid * 16;                                               \
    pk0 = *reinterpret_cast<const uint4*>(kt_);                                                                \
    pv0 = *reinterpret_cast<const uint4*>(vt_);                                                                \
    if (CH == 2) {                                                                                             \
      pk1 = *reinterpret_cast<const uint4*>(kt_ + NT * 16);                                                    \
      pv1 = *reinterpret_cast<const uint4*>(vt_ + NT * 16);                                                    \
    }                                                                                                          \
    if (tid < 64) psc = *reinterpret_cast<const uint32_t*>(ksbase + (size_t)(J) * 256 + tid * 4);              \
    else if (tid < 128) psc = *reinterpret_cast<const uint32_t*>(vsbase + (size_t)(J) * 256 + (tid - 64) * 4); \
  } while (0)
#define THRIFT_COMMIT4(BUF)                                                                                    \
  do {                                                                                                         \
    unsigned char* b_ = (BUF);                                                                                 \
    *reinterpret_cast<uint4*>(b_ + kLdsK4 + k4_fragment_offset(tid >> 2, tid & 3)) = pk0;                      \
    *reinterpret_cast<uint4*>(b_ + kLdsV4 + tid * 16) = pv0;                                                   \
    if (CH == 2) {                                                                                             \
      *reinterpret_cast<uint4*>(b_ + kLdsK4 + k4_fragment_offset((tid + NT) >> 2, (tid + NT) & 3)) = pk1;      \
      *reinterpret_cast<uint4*>(b_ + kLdsV4 + (tid + NT) * 16) = pv1;                                          \
    }                                                                                                          \
    if (tid < 64) {                                                                                            \
      *reinterpret_cast<uint32_t*>(b_ + kLdsKS + tid * 4) = psc;                                               \
    } else if (tid < 128) {                                                                                    \
      /* bytes 4w..4w+3 of the [2 groups][128 channels] scale rows -> [group][r][n], channel = 32n + r */      \
      const int w_ = tid - 64, grp_ = w_ >> 5, ch_ = (4 * w_) & 127, n_ = ch_ >> 5, rr_ = ch_ & 31;            \
      for (int bb = 0; bb < 4; ++bb) b_[kLdsVS + (grp_ * 32 + rr_ + bb) * 4 + n_] = (unsigned char)(psc >> (8 * bb)); \
    }                                                                                                          \
  } while (0)
#define THRIFT_STAGE16(J, BUF)                                                                                 \
  do {                                                                                                         \
    unsigned char* b_ = (BUF);                                                                                 \
    _Pragma("unroll") for (int u = 0; u < 1024 / NT; ++u) {                                                    \
      const int chunk = tid + NT * u, row = chunk >> 4, col = chunk & 15;                                      \
      const uint4 kk = *reinterpret_cast<const uint4*>(k16base + ((size_t)(J) * kBk + row) * kD + col * 8);    \
      const uint4 vv = *reinterpret_cast<const uint4*>(v16base + ((size_t)(J) * kBk + row) * kD + col * 8);    \
      *reinterpret_cast<uint4*>(b_ + kLdsK16 + row * kRow16 + col * 16) = kk;                                  \
      *reinterpret_cast<uint4*>(b_ + kLdsV16 + row * kRow16 + col * 16) = vv;                                  \
    }                                                                                                          \
  } while (0)

  RowState st = {-INFINITY, 0.f};
  v16f o[4];
#pragma unroll
  for (int n = 0; n < 4; ++n) o[n] = (v16f){0.f};
  const float c = a.scale * 1.4426950408889634f;

  // prologue: block 0 into buffer 0, block 1 (if 4-bit) into the prefetch registers
  if (vis > 0) {
    if (n0 == 0) {
      THRIFT_STAGE16(0, lds);
    } else {
      THRIFT_PREFETCH4(0);
      THRIFT_COMMIT4(lds);
    }
    const int t1 = n0 == 0 ? n1 : n0;
    if (vis > 1 && t1 != 1) THRIFT_PREFETCH4(1);
  }
  // Blocks this wavefront computes: those with at least one key at or before its last query row.  The
  // later blocks of the workgroup (visible only to wavefronts with later rows) are still staged and
  // synchronised on, in a final loop without arithmetic.
  const int vis_wave = a.causal ? min(vis, (q0 + 31) / kBk + 1) : vis;

  // One step of the staging pipeline at block J: wait until block J is complete in `cur`, then move block
  // J+1 into the other buffer and start the global loads of block J+2.  T1 / T2: the first promoted ids at
  // or after J+1 / J+2.
#define THRIFT_STEP(J, T1, T2)                                                                                 \
  unsigned char* cur = lds + ((J) & 1) * kLdsBytes16;                                                          \
  {                                                                                                            \
    unsigned char* nxt = lds + (((J) + 1) & 1) * kLdsBytes16;                                                  \
    lds_barrier();   /* everyone has finished block J-1, which used `nxt` */                                   \
    if ((J) + 1 < vis) {                                                                                       \
      if ((J) + 1 == (T1)) THRIFT_STAGE16((J) + 1, nxt);                                                       \
      else THRIFT_COMMIT4(nxt);                                                                                \
      if ((J) + 2 < vis && (J) + 2 != (T2)) THRIFT_PREFETCH4((J) + 2);                                         \
    }                                                                                                          \
  }
#define THRIFT_MASK(J)                                                                                         \
  const bool mask = a.causal && (J) * kBk + kBk - 1 > q0;                                                      \
  const int n_valid = q0 + r - (J) * kBk + 1; /* keys of the block at positions <= the query's */

  // The walk alternates between runs of 4-bit blocks (tight loop: only the scaled-FP4 path, accumulators
  // updated in place) and single promoted blocks.
  int j = 0;
  while (j < vis_wave) {
    const int run_end = min(vis_wave, n0);
    for (; j < run_end; ++j) {
      THRIFT_STEP(j, n0, (j + 1 == n0 ? n1 : n0))
      THRIFT_MASK(j)
      v16f s[2];
      float gmax;
      scores_fp4(cur, lane, qf4, qsc, s);
      const float alpha = softmax_update(s, lane, mask, n_valid, c, st, gmax);
      rescale(o, alpha);
      pv_fp4(cur, lane, s, gmax, o);
    }
    if (j < vis_wave) {                                 // j == n0: a promoted block
      THRIFT_STEP(j, n1, (j + 1 == n1 ? n2 : n1))
      THRIFT_MASK(j)
      v16f s[2];
      float gmax;
      scores_16<T>(cur, lane, q16row, s);
      const float alpha = softmax_update(s, lane, mask, n_valid, c, st, gmax);
      rescale(o, alpha);
      pv_16<T>(cur + kLdsV16, lane, s, o);
      ++ps;
      n0 = n1; n1 = n2; n2 = ps + 2 < nsel ? sel[ps + 2] : 0x7fffffff;
      ++j;
    }
  }
  for (; j < vis; ++j) {                                // staging only
    const bool is16 = j == n0;
    const int t1 = is16 ? n1 : n0;
    THRIFT_STEP(j, t1, (j + 1 == t1 ? (is16 ? n2 : n1) : t1))
    (void)cur;
    if (is16) {
      ++ps;
      n0 = n1; n1 = n2; n2 = ps + 2 < nsel ? sel[ps + 2] : 0x7fffffff;
    }
  }
#undef THRIFT_STEP
#undef THRIFT_MASK

  // ---- epilogue (Alg. 1 step 21): O / l; accumulator i of tile n is channel 32n + 8(i/4) + 4*half + i%4 ----
  const float l = st.l + other_half(st.l);
  const float inv = l > 0.f ? 1.0f / l : 0.f;
  const size_t orow = qrow * kD;
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int q4i = 0; q4i < 4; ++q4i) {
      const int ch = 32 * n + 8 * q4i + 4 * half;
      const float x0 = o[n][4 * q4i] * inv, x1 = o[n][4 * q4i + 1] * inv, x2 = o[n][4 * q4i + 2] * inv, x3 = o[n][4 * q4i + 3] * inv;
      if (a.out_dt == THRIFT_F32) {
        *reinterpret_cast<float4*>((float*)a.out + orow + ch) = make_float4(x0, x1, x2, x3);
      } else if (a.out_dt == THRIFT_F16) {
        uint2 w;
        w.x = (uint32_t)F16::from_float(x0) | ((uint32_t)F16::from_float(x1) << 16);
        w.y = (uint32_t)F16::from_float(x2) | ((uint32_t)F16::from_float(x3) << 16);
        *reinterpret_cast<uint2*>((uint16_t*)a.out + orow + ch) = w;
      } else {
        uint2 w;
        w.x = (uint32_t)BF16::from_float(x0) | ((uint32_t)BF16::from_float(x1) << 16);
        w.y = (uint32_t)BF16::from_float(x2) | ((uint32_t)BF16::from_float(x3) << 16);
        *reinterpret_cast<uint2*>((uint16_t*)a.out + orow + ch) = w;
      }
    }
  if (a.lse != nullptr && half == 0) a.lse[qrow] = st.m * a.scale + __logf(l);
}

#undef THRIFT_PREFETCH4
#undef THRIFT_COMMIT4
#undef THRIFT_STAGE16

void launch_prefill(const PrefillArgs& a, hipStream_t st) {
  const unsigned grid = (unsigned)((long)a.B * a.Hq * (a.N / a.Bq));
  if (a.Bq == 128) {
    if (a.dt == THRIFT_F16) prefill_kernel<F16, 4><<<dim3(grid), dim3(256), 0, st>>>(a);
    else prefill_kernel<BF16, 4><<<dim3(grid), dim3(256), 0, st>>>(a);
  } else {
    if (a.dt == THRIFT_F16) prefill_kernel<F16, 2><<<dim3(grid), dim3(128), 0, st>>>(a);
    else prefill_kernel<BF16, 2><<<dim3(grid), dim3(128), 0, st>>>(a);
  }
}

}  // namespace thrift
