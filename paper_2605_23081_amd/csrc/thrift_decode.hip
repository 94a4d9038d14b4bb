// Split-K decode over the dual MXFP4 / 16-bit KV cache (Sec. 4.1 and Sec. 5 of the paper describe the
// dual cache; the algorithm is Algorithm 1 with a one-token query block).
//
// One workgroup = one (sequence, KV head, partition of split_blocks key blocks) and ONE recurrence of Alg. 1
// per query head over the whole partition.  The group's heads are dealt to the four wavefronts (head g goes to
// wavefront g mod 4), so every wavefront walks every key block of the partition for its own heads.
// The kernel is bandwidth bound.  Each key block is brought from HBM once per workgroup by LDS DMA (with the
// streaming hint: nothing of the cache is read twice) and read from LDS by all four wavefronts: the 4-bit codes and
// scales of every block into a ring of five slots, up to three blocks ahead of the arithmetic; the 16-bit K and V
// tiles of a block that some head of the group has promoted into one tile buffer each, one step ahead when the
// buffer is idle then.  A head for which the block is promoted takes its scores and P.V from the 16-bit tiles, the
// others from the 4-bit slot; both feed the same online softmax.  The walk is software-pipelined: the scores of
// block t+1 are formed between the softmax and the P.V of block t.
// With one or two heads per wavefront (head groups of up to 8) the score tiles are formed as Q.K^T with each query
// in two rows, which leaves one register with a head's 64 scores of the block across the lanes (the row layout
// below); larger groups use the transposed tiles of the prefill kernel, head wave + 4r in column r.
// Each (head, partition) writes one unnormalised partial (m, l, O); a second kernel merges the partials of a
// (sequence, head) by their log-sum-exp.  A partly filled last block (a cache that is still growing) is a partition
// of its own, computed by a small second kernel with masking, so that the main walk carries none.
#include <type_traits>

#include "thrift_launch.h"
#include "thrift_tile.h"

namespace thrift {

constexpr int kDecRing = 5;                                   // 4-bit slots: block t of the partition sits in slot t mod kDecRing
constexpr int kDecAhead = kDecRing - 1;                       // step t issues block t + kDecAhead into the slot block t-1 has left
constexpr int kDecFlight = kDecRing - 3;                      // blocks in flight and not yet needed at a step: t+2 .. t+kDecRing-2
constexpr int kDecLdsK16 = kDecRing * kLdsBytes4;             // one swizzled 16-bit K tile
constexpr int kDecLdsV16 = kDecLdsK16 + kTile16;              // one swizzled 16-bit V tile
constexpr int kDecLds = kDecLdsV16 + kTile16;                 // 76288 B: two workgroups per CU
constexpr int kDmaPer4 = 3;                                   // DMA instructions one wavefront issues per 4-bit block
constexpr int kBmWin = 8;                                     // 64-block words of each head's selection bitmap cached in LDS

// Wait until at most n (a multiple of kDmaPer4 = 3) of this wavefront's DMA instructions are in flight.
__device__ __forceinline__ void vm_wait_dyn(int n) {
  static_assert(kDecFlight <= 5, "one case per possible count");
  if (n >= 15) vm_wait<15>();
  else if (n >= 12) vm_wait<12>();
  else if (n >= 9) vm_wait<9>();
  else if (n >= 6) vm_wait<6>();
  else if (n >= 3) vm_wait<3>();
  else vm_wait<0>();
}

// ---- one query row per wavefront: the row layout ----
// With a single head per wavefront the transposed tiles of the prefill kernel would spend a whole wavefront
// instruction on each of the row's 64 scores.  Here the score tiles are formed the other way round, S = Q . K^T
// with the query in rows 0 and 4 of the A operand (all other rows zero): accumulator register 0 of lane (half, r)
// is row 4*half, column r, i.e. the query against key r of the 32-key sub-tile.  Taking sub-tile 0 from the lower 32
// lanes and sub-tile 1 from the upper ones leaves ONE register with the score of key `lane` of the block in every
// lane: the online softmax of Alg. 1 then costs one exponential per block, its maxima come from lane permutes, and
// the probabilities are gathered into lanes 0 and 32 (the B-operand column of the query in O^T += V^T . P^T, 32 keys
// = one MXFP4 group per lane) by a few more permutes.

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u(uint32_t x) { return __builtin_amdgcn_update_dpp(0u, x, CTRL, 0xf, 0xf, true); }
template <int CTRL>
__device__ __forceinline__ float dpp_f(float x) { return __uint_as_float(dpp_u<CTRL>(__float_as_uint(x))); }
constexpr int kDppSwap1 = 0xb1;        // quad_perm [1,0,3,2]: lane ^ 1
constexpr int kDppSwap2 = 0x4e;        // quad_perm [2,3,0,1]: lane ^ 2
constexpr int kDppQuadHi = 0xee;       // quad_perm [2,3,2,3]: lanes 0,1 of a quad read lanes 2,3
constexpr int kDppHalfMirror = 0x141;  // lane i of each 8 reads lane 7 - i
constexpr int kDppMirror = 0x140;      // lane i of each 16 reads lane 15 - i
constexpr int kDppShl4 = 0x104;        // lane i reads lane i + 4 of its 16-lane row

// natural key order for the row layout: fragment (t, kk) of lane (half, r) = key 32t + r, d-group 2*half + kk
__device__ __forceinline__ K4Tile load_k4_rows(const unsigned char* slot, int lane) {
  const int half = lane >> 5, r = lane & 31;
  const unsigned char* ksrow = slot + kLdsKS + 4 * r + 2 * half;        // sub-tile 1: 32 keys = 128 bytes further
  K4Tile k;
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    k.ks[t] = *reinterpret_cast<const uint16_t*>(ksrow + 128 * t);
    k.a[2 * t] = *reinterpret_cast<const v4i*>(slot + kLdsK4 + ((t * 2 + 0) * 64 + lane) * 16);
    k.a[2 * t + 1] = *reinterpret_cast<const v4i*>(slot + kLdsK4 + ((t * 2 + 1) * 64 + lane) * 16);
  }
  return k;
}
// Scores of key `lane` of the block for the wavefront's NH heads (Alg. 1 step 15 for the one-token query block).
// qf / qsc: the fragments and scale bytes of head u in lanes r = u and r = u + 4 (u < 4), zeros elsewhere: accumulator
// register u is then row u + 4*half, head u against key r.
template <int NH>
__device__ __forceinline__ void scores4_row(const K4Tile& k, int lane, const v4i (&qf)[2], uint32_t qsc, float (&sv)[NH]) {
  v16f acc[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    acc[t] = (v16f){0.f};
    acc[t] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen(qf[0]), widen(k.a[2 * t]), acc[t], 4, 4, 0, qsc, 0, k.ks[t]);
    acc[t] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen(qf[1]), widen(k.a[2 * t + 1]), acc[t], 4, 4, 1, qsc, 1, k.ks[t]);
  }
#pragma unroll
  for (int u = 0; u < NH; ++u) sv[u] = (lane >> 5) ? acc[1][u] : acc[0][u];
}
// The same from the 16-bit K tile (Alg. 1 step 9).  Tile rows are keys in natural order, 256 B each, the 16-byte chunk c
// of row `row` stored at chunk position c ^ (row & 7) (eight neighbouring lanes read eight different positions).
// qf[s8]: head u's elements d = 16*s8 + 8*half + [0,8) in lanes r = u and r = u + 4, zeros elsewhere.
template <typename T, int NH>
__device__ __forceinline__ void scores16_row(const unsigned char* ktile, int lane, const v8s (&qf)[8], float (&sv)[NH]) {
  const int half = lane >> 5, r = lane & 31;
  v16f acc[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const unsigned char* row = ktile + (32 * t + r) * 256;
    acc[t] = (v16f){0.f};
#pragma unroll
    for (int s8 = 0; s8 < 8; ++s8) {
      const v8s kf = *reinterpret_cast<const v8s*>(row + 16 * ((2 * s8 + half) ^ (r & 7)));
      acc[t] = T::mfma(qf[s8], kf, acc[t]);
    }
  }
#pragma unroll
  for (int u = 0; u < NH; ++u) sv[u] = half ? acc[1][u] : acc[0][u];
}
// Online softmax of Alg. 1 (steps 10-12 / 16-17) on the row layout: sv = this lane's raw score.  st.m is the running
// maximum (the same in every lane), st.l this lane's share of the row sum.  Returns (for the whole wavefront) whether
// the maximum rose; only then does alpha hold exp(scale * (m_old - m_new)) and must the accumulators be rescaled.
// p: this lane's unnormalised probability; pbyte: the E8M0 byte of the lane's 32-key group of P (as in softmax_update).
__device__ __forceinline__ bool softmax_row(float sv, float c, RowState& st, float& alpha, uint32_t& pbyte, float& p) {
  float v = sv;
  v = fmaxf(v, dpp_f<kDppSwap1>(v));
  v = fmaxf(v, dpp_f<kDppSwap2>(v));
  v = fmaxf(v, dpp_f<kDppHalfMirror>(v));
  v = fmaxf(v, dpp_f<kDppMirror>(v));                               // maximum of the lane's 16
  const uint32_t vb = __float_as_uint(v);
  const auto s16 = __builtin_amdgcn_permlane16_swap(vb, vb, false, false);   // [0]: the even 16's value on both 16s of a 32, [1]: the odd's
  const float gmax = fmaxf(__uint_as_float(s16[0]), __uint_as_float(s16[1]));  // maximum of the lane's 32-key group
  const uint32_t gb = __float_as_uint(gmax);
  const auto s32 = __builtin_amdgcn_permlane32_swap(gb, gb, false, false);
  const float m_old = st.m;
  const float m_new = max3(m_old, __uint_as_float(s32[0]), __uint_as_float(s32[1]));
  const bool grew = __builtin_amdgcn_ballot_w64(m_new != m_old) != 0ULL;
  if (grew) {
    float d = m_old - m_new;
    asm volatile("" : "+v"(d));                                    // keeps the exponential inside the branch
    alpha = fast_exp2(d * c);
    float l = st.l;
    asm volatile("s_nop 1\n\tv_mul_f32 %0, %1, %0" : "+v"(l) : "v"(alpha));   // wait states: a transcendental result read by hand-written code
    st.l = l;
  }
  st.m = m_new;
  int e;
  {
    const float x = (gmax - m_new) * c;                            // the group maximum maps to exactly 2^floor(x) or above
    asm("v_cvt_flr_i32_f32 %0, %1" : "=v"(e) : "v"(x));
  }
  pbyte = (uint32_t)max(e + 125, 1);
  p = fast_exp2(__builtin_fmaf(sv, c, -(m_new * c)));
  st.l += p;
  return grew;
}
// Alg. 1 step 19 on the row layout: every lane turns its probability into an E2M1 code under its group's scale and the
// 32 codes of a group are collected, in key order, into the four registers of lane U (keys 0-31) / lane 32 + U (keys
// 32-63), the B-operand column of head U; what the other lanes receive belongs to no query.
template <int U>
__device__ __forceinline__ v4i gather_p4(float p, uint32_t pb) {
  static_assert(U >= 0 && U < 4, "the head's column must lie in the first four lanes");
  const float pscale = __uint_as_float(pb << 23);
  const float nb = dpp_f<kDppSwap1>(p);
  // even lanes: one byte = the codes of keys (lane, lane + 1)
  const uint32_t b8 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(0u, p, nb, pscale, 0);
  const uint32_t b16 = b8 | (dpp_u<kDppQuadHi>(b8) << 8);          // lanes 4q: keys 4q .. 4q+3
  const uint32_t b32 = b16 | (dpp_u<kDppShl4>(b16) << 16);         // lanes 8q: keys 8q .. 8q+7
  const auto sw = __builtin_amdgcn_permlane16_swap(b32, b32, false, false);
  // lane 0 of a 32: sw[0] = its own word (keys 0-7), sw[1] = lane 16's (keys 16-23); lane 8: keys 8-15 and 24-31.
  // Lane U reads lane 0 (a shift right by U) and lane 8 (a shift left by 8 - U) of its 16.
  constexpr int kFrom0 = 0x110 | U, kFrom8 = 0x100 | (8 - U);
  if constexpr (U == 0) return (v4i){(int)sw[0], (int)dpp_u<kFrom8>(sw[0]), (int)sw[1], (int)dpp_u<kFrom8>(sw[1])};
  else return (v4i){(int)dpp_u<kFrom0>(sw[0]), (int)dpp_u<kFrom8>(sw[0]), (int)dpp_u<kFrom0>(sw[1]), (int)dpp_u<kFrom8>(sw[1])};
}
// Alg. 1 step 13 on the row layout: the probabilities rounded to the input dtype and collected through a 128-byte LDS
// row of the wavefront's own: pf[s] of lane (half, *) = keys 32*half + 8s .. + 7 (the order pv_16_rounded contracts in).
template <typename T>
__device__ __forceinline__ void gather_p16(uint16_t* prow, int lane, float p, v8s (&pf)[4]) {
  prow[lane] = T::from_float(p);
#pragma unroll
  for (int s = 0; s < 4; ++s) pf[s] = *reinterpret_cast<const v8s*>(prow + 32 * (lane >> 5) + 8 * s);
}
// sum over the 64 lanes, in every lane
__device__ __forceinline__ float wave_sum(float x) {
  x += dpp_f<kDppSwap1>(x);
  x += dpp_f<kDppSwap2>(x);
  x += dpp_f<kDppHalfMirror>(x);
  x += dpp_f<kDppMirror>(x);
  const uint32_t xb = __float_as_uint(x);
  const auto s16 = __builtin_amdgcn_permlane16_swap(xb, xb, false, false);
  x = __uint_as_float(s16[0]) + __uint_as_float(s16[1]);
  return x + other_half(x);
}

// HPW = 1 or 2: at most HPW heads per wavefront (groups of up to 4 / 8 heads, the usual GQA ratios), in the row layout;
// the path of a block is a scalar choice per head.  HPW = 0: up to eight heads per wavefront in the transposed tiles of
// the prefill kernel (head wave + 4r in column r), which cost a wavefront instruction per score and key but no more for
// eight heads than for one; the heads may split over the two paths of a block, both tiles are then computed and each
// lane keeps its own head's.  That form finishes a block within its step (scores, softmax, P.V) instead of forming the
// next block's scores ahead: it has no registers to carry them.
template <typename T, int HPW>
__global__ void __launch_bounds__(256, 2) decode_partial_kernel(DecodeArgs a) {
  constexpr bool MULTI = HPW == 0;
  constexpr int NH = MULTI ? 1 : HPW;
  __shared__ __align__(1024) unsigned char lds[kDecLds];
  __shared__ unsigned long long bmw[32 * kBmWin];              // [head of the group][word of the window]
  __shared__ __align__(16) uint16_t qrow[MULTI ? 8 : 4 * NH * kD];   // row layout: the 16-bit query rows of each wavefront's heads
  __shared__ __align__(16) uint16_t prow[MULTI ? 8 : 4 * 64];        // row layout: a row of rounded probabilities per wavefront
  const int tid = threadIdx.x, lane = tid & 63, half = lane >> 5, r = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wavefront-uniform
  const int G = a.Hq / a.Hkv;
  const int item = a.order ? a.order[blockIdx.x] : (int)blockIdx.x;    // heaviest items first when an order was made
  const int part = item % a.nsplit, unit = item / a.nsplit;
  const int b = unit / a.Hkv, kvh = unit % a.Hkv;
  const int len = a.seqlens ? min(a.Nkv, max(0, a.seqlens[b])) : a.Nkv;
  const int Tk = len / kBk;                                    // full key blocks; a partly filled one is the other kernel's
  const int j_begin = min(Tk, part * a.split_blocks), j_end = min(Tk, j_begin + a.split_blocks);
  const int n = j_end - j_begin;                               // key blocks of this partition (workgroup-uniform)

  // this wavefront's heads: column r carries head wave + 4r of the group
  const int my_heads = G > wave ? (G - wave + 3) / 4 : 0;
  const bool real = r < my_heads;
  const size_t group0 = (size_t)b * a.Hq + (size_t)kvh * G;    // first query head of the group
  const size_t qh = group0 + (real ? wave + 4 * r : 0);       // the head whose result this lane stores (column r)
  const size_t kh = (size_t)b * a.Hkv + kvh;
  const unsigned long long my_mask = my_heads >= 32 ? 0xffffffffULL : ((1ULL << my_heads) - 1ULL);

  // ---- Q fragments (zeros for padding columns): the lane quantises its own two MXFP4 groups of the query,
  // d-group 2*half + kk (channels 64*half + 32*kk .. +31) for fragment kk (Alg. 1 step 2 for the one-token
  // query block); the 16-bit fragments of the same row stay in registers for the promoted blocks ----
  v4i qf4[2] = {(v4i){0, 0, 0, 0}, (v4i){0, 0, 0, 0}};
  uint32_t qsc = 0x7f7f7f7fu;
  const uint16_t* q16row = a.q + qh * kD + 8 * half;
  // lanes that carry a query as an MFMA operand: its column in the transposed tiles; rows u and u + 4 for head u of
  // the row layout
  const bool qlane = MULTI ? real : (r < 8 && (r & 3) < min(my_heads, NH));
  const size_t qhq = MULTI ? qh : group0 + (qlane ? wave + 4 * (r & 3) : 0);
  if (qlane) {
    uint32_t sb[2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
      const uint4* src = reinterpret_cast<const uint4*>(a.q + qhq * kD + 64 * half + 32 * kk);
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
  // Row layout: the 16-bit rows of the wavefront's heads are parked in LDS (each wavefront writes and reads only its own
  // rows) and read back at each promoted block: a global read inside the walk would wait for every tile DMA in flight.
  if constexpr (!MULTI) {
    if (lane < 16 * NH) {
      const int u = lane >> 4;
      uint4 w = make_uint4(0u, 0u, 0u, 0u);
      if (u < my_heads) w = *reinterpret_cast<const uint4*>(a.q + (group0 + wave + 4 * u) * kD + 8 * (lane & 15));
      *reinterpret_cast<uint4*>(qrow + (wave * NH + u) * kD + 8 * (lane & 15)) = w;
    }
  }

  const uint8_t* k4base = a.k4 + kh * a.Nkv * 64;
  const uint8_t* v4base = a.v4 + kh * (size_t)(a.Nkv / 64) * 4096;
  const uint8_t* k16base = reinterpret_cast<const uint8_t*>(a.k16 + kh * a.Nkv * kD);
  const uint8_t* v16base = reinterpret_cast<const uint8_t*>(a.v16 + kh * a.Nkv * kD);
  // the 256 scale bytes of K ride with the even wavefronts, V's with the odd ones
  const bool v_scales = (wave & 1) != 0;
  const uint8_t* scbase = v_scales ? a.vs + kh * (size_t)(a.Nkv / 32) * kD : a.ks + kh * a.Nkv * 4;
  const uint32_t sclds = v_scales ? (uint32_t)kLdsVS : (uint32_t)kLdsKS;

  // ---- staging: per-lane source offsets of this wavefront's DMA instructions (the LDS side of a DMA is linear
  // in the lane index, so the MFMA fragment order of the 4-bit tiles and the chunk swizzle of the 16-bit tiles are
  // expressed in the global offsets) ----
  const uint32_t lds0 = lds_address(lds);
  // K fragment (t, kk) = (wave>>1, wave&1): keys in the row permutation of the transposed tiles, or in natural order
  const uint32_t k4off = (uint32_t)((MULTI ? key_of_row(r, wave >> 1) : 32 * (wave >> 1) + r) * 64 + (2 * half + (wave & 1)) * 16);
  const uint32_t v4off = (uint32_t)((32 * wave + r) * 32 + half * 16);                               // V channels 32*wave .. +31
  const uint32_t scoff = (uint32_t)lane * 4;
  const uint32_t v16off = (uint32_t)((lane >> 4) * 256 + ((lane & 15) ^ v16_swizzle(lane >> 4)) * 16);
  // instruction q = 4u + wave covers rows 4q .. 4q+3.  Transposed tiles: k16_swizzle (rows 32..63: chunk ^ 4 more);
  // row layout: chunk ^ (row & 7), and row & 7 = 4*(wave & 1) + (lane >> 4) for every u
  const uint32_t k16off = MULTI ? (uint32_t)((lane >> 4) * 256 + ((lane & 15) ^ (lane >> 4)) * 16)
                                : (uint32_t)((lane >> 4) * 256 + ((lane & 15) ^ (4 * (wave & 1) + (lane >> 4))) * 16);
  auto issue4 = [&](int j, int slot_index) {            // block j (absolute id) into ring slot slot_index
    const int j_ = __builtin_amdgcn_readfirstlane(j);
    const uint32_t slot = lds0 + (uint32_t)(__builtin_amdgcn_readfirstlane(slot_index) * kLdsBytes4);
    dma_b128<true>(k4base + (size_t)j_ * 4096, k4off, slot + kLdsK4 + wave * 1024);
    dma_b32<true>(scbase + (size_t)j_ * 256, scoff, slot + sclds);
    dma_b128<true>(v4base + (size_t)j_ * 4096, v4off, slot + kLdsV4 + wave * 1024);
  };
  auto issue16k = [&](int j) {                          // the 16-bit K tile of block j: instruction q covers rows 4q .. 4q+3
    const int j_ = __builtin_amdgcn_readfirstlane(j);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int q_ = u * 4 + wave;
      dma_b128<true>(k16base + (size_t)j_ * kTile16 + q_ * 1024, (MULTI && u >= 2) ? k16off ^ 64u : k16off, lds0 + kDecLdsK16 + q_ * 1024);
    }
  };
  auto issue16v = [&](int j) {                          // the 16-bit V tile of block j
    const int j_ = __builtin_amdgcn_readfirstlane(j);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int q_ = u * 4 + wave;
      dma_b128<true>(v16base + (size_t)j_ * kTile16 + q_ * 1024, v16off, lds0 + kDecLdsV16 + q_ * 1024);
    }
  };

  // ---- selection bitmaps.  Staging decisions need the whole group's votes on a block (identical in all four
  // wavefronts); the arithmetic needs this lane's own head.  The walk reads them from a window of kBmWin 64-block
  // words per head kept in LDS: a global read inside the walk would make the compiler wait for every load in
  // flight, the tile DMAs included, at each key block. ----
  int win0 = 0;                                         // first word of the window (workgroup-uniform)
  int wcur = -1;                                        // word index the cached words (below) belong to
  auto refill = [&](int word0) {                        // called by all threads at the same point of the walk
    lds_barrier();                                      // nobody still reads the old window
    for (int e = tid; e < G * kBmWin; e += 256) {
      const int h = e / kBmWin, wi = word0 + e % kBmWin;
      bmw[e] = wi < a.bitmap_words ? a.bitmap[(group0 + h) * a.bitmap_words + wi] : 0ULL;
    }
    lds_barrier();
    win0 = word0;
  };
  // Per 64-block word: the OR of the group's words (some head has promoted the block) in scalar registers and this
  // wavefront's own word(s).  Formed once per 64 key blocks, so that a step of the walk only tests bits.
  auto scalar_word = [&](int index) -> unsigned long long {      // bmw[index], index wavefront-uniform
    const unsigned long long w = bmw[index];
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)w), hi = __builtin_amdgcn_readfirstlane((uint32_t)(w >> 32));
    return ((unsigned long long)hi << 32) | lo;
  };
  unsigned long long gor = 0;                           // group OR of word wcur
  unsigned long long own_s[NH];                         // row layout: the words of this wavefront's heads (scalar)
#pragma unroll
  for (int u = 0; u < NH; ++u) own_s[u] = 0ULL;
  unsigned long long own_v = 0;                         // transposed tiles: the word of this lane's head
  // Flags of block x of the partition (x may run past the end: all clear): bit 0 of the result = some head of the
  // group has promoted it (wavefront-uniform); mine = this lane's head has (transposed tiles) / bit u = head u of this
  // wavefront has (row layout, scalar).  Blocks are asked for in ascending order.
  using Mine = std::conditional_t<MULTI, bool, int>;
  auto flags = [&](int x, Mine& mine) -> int {
    mine = Mine(0);
    if (x >= n) return 0;
    const int j = j_begin + x, w = j >> 6;
    if (w != wcur) {
      if (w >= win0 + kBmWin || wcur < 0) refill(w);
      gor = 0;
      for (int g = 0; g < G; ++g) gor |= scalar_word(g * kBmWin + (w - win0));
      if constexpr (MULTI) {
        own_v = real ? bmw[(wave + 4 * r) * kBmWin + (w - win0)] : 0ULL;
      } else {
#pragma unroll
        for (int u = 0; u < NH; ++u) own_s[u] = u < my_heads ? scalar_word((wave + 4 * u) * kBmWin + (w - win0)) : 0ULL;
      }
      wcur = w;
    }
    if constexpr (MULTI) {
      mine = ((own_v >> (j & 63)) & 1ULL) != 0ULL;
    } else {
#pragma unroll
      for (int u = 0; u < NH; ++u) mine |= (int)((own_s[u] >> (j & 63)) & 1ULL) << u;
    }
    return (int)((gor >> (j & 63)) & 1ULL);
  };

  RowState st[NH];                                      // row layout: one per head; transposed tiles: this lane's column
#pragma unroll
  for (int u = 0; u < NH; ++u) st[u] = {kEmptyMax, 0.f};
  v16f o[4];
#pragma unroll
  for (int nn = 0; nn < 4; ++nn) o[nn] = (v16f){0.f};
  const float c = a.scale * 1.4426950408889634f;

  // ---- the walk, software-pipelined over the key blocks: step t (t = -1 .. n-1) finishes block t (softmax, P.V) and
  // forms the scores of block t+1 in between, so that the matrix unit works on one block while the vector unit works
  // on its neighbour and no LDS read is waited for where it is issued.
  // Residency at step t (kDecRing = 5): 4-bit slots of blocks t (V) and t+1 (K) in use, t+2 and t+3 in flight, t+4 issued into the
  // slot block t-1 has left; the K tile buffer holds block t+1's 16-bit keys, the V tile buffer block t's values.
  // A 16-bit tile is fetched one step before its use when its buffer is idle then (the neighbouring block is not
  // promoted), otherwise at the step of its use, which then waits for it.
  // P?/M?: promoted-by-the-group / promoted-for-this-head flags of blocks t-1 (a), t (b), t+1 (c), t+2 (d). ----
  int Pa = 0, Pb = 0, Pc, Pd;
  Mine Mb = Mine(0), Mc, Md;
  Pc = flags(0, Mc);
  Pd = flags(1, Md);
  // The K tile buffer holds block t + kKShift's keys at step t: the row layout forms the scores of block t+1 at step t,
  // the transposed tiles (which have no registers to carry scores from one step to the next) those of block t itself.
  constexpr int kKShift = MULTI ? 0 : 1;
  if (kKShift == 1 && Pc) issue16k(j_begin);
  for (int x = 0; x < kDecRing - 2 && x < n; ++x) issue4(j_begin + x, x);
  int slot_a = kDecRing - 2, slot_b = kDecRing - 1, slot_c = 0;   // ring slots of blocks t-1, t, t+1 at t = -1
  int early_prev = 0;                                   // the step before fetched 16-bit tiles ahead of its 4-bit block

  // Staging part of step t: waits for what the step reads, then issues what later steps will read.
  // `plain` (workgroup-uniform): the caller has seen that none of the decisions below can come out true (row layout:
  // the group has promoted none of the blocks t .. t+2, no 16-bit tile was fetched ahead, block t+kDecAhead exists).
  auto stage = [&](int t, bool plain) {
    const int j = j_begin + t;
    // in flight and not yet needed: the 4-bit blocks t+2 .. t+kDecRing-2 (where they exist); after 16-bit tiles fetched
    // ahead in the step before, only that step's 4-bit block t+kDecRing-2
    if (plain || (!early_prev && t + kDecRing - 2 < n)) {
      vm_wait<kDmaPer4 * kDecFlight>();                 // the steady state of the walk: one scalar test
    } else {
      const int newer = early_prev ? (t + kDecRing - 2 < n ? kDmaPer4 : 0) : kDmaPer4 * max(0, min(n - 2 - t, kDecFlight));
      vm_wait_dyn(newer);
    }
    lds_barrier();                                      // block t+1 (and block t's V tile) complete in LDS; step t-1 is behind everyone
    if (!plain) {
      const int Kprev = kKShift ? Pb : Pa, Kcur = kKShift ? Pc : Pb, Knext = kKShift ? Pd : Pc;   // promoted flags of blocks t + kKShift - 1, +0, +1
      const int lateK = Kcur & Kprev, lateV = Pb & Pa;  // the buffer was busy during the step before
      if (lateK) issue16k(j + kKShift);
      if (lateV) issue16v(j);
      if (lateK | lateV) {
        vm_wait<0>();
        lds_barrier();
      }
      const int earlyK = Knext & (Kcur ^ 1), earlyV = Pc & (Pb ^ 1);
      if (earlyK) issue16k(j + kKShift + 1);
      if (earlyV) issue16v(j + 1);
      early_prev = earlyK | earlyV;                     // a plain step leaves it at 0
    }
    if (plain || t + kDecAhead < n) issue4(j + kDecAhead, slot_a);
  };
  if constexpr (!MULTI) {
    // ---- up to NH heads per wavefront in the row layout; the (scalar) selection bit of a head decides its path ----
    const int all_heads = (1 << min(my_heads, NH)) - 1;          // mask of this wavefront's heads
    // scores of key `lane` of the block in the K tile buffer, for every head
    auto score16 = [&](float (&sv)[NH]) {
      // the lane-dependent LDS addresses of the 16-bit tiles are formed at the promoted block, from a copy of the lane
      // index the compiler cannot see through: formed once ahead of the walk they would occupy registers at every step
      int lane_ = lane;
      asm volatile("" : "+v"(lane_));
      const int half_ = lane_ >> 5, r_ = lane_ & 31;
      v8s q16[8];
#pragma unroll
      for (int s8 = 0; s8 < 8; ++s8)
        q16[s8] = qlane ? *reinterpret_cast<const v8s*>(qrow + (wave * NH + (r_ & 3)) * kD + 16 * s8 + 8 * half_) : (v8s){0, 0, 0, 0, 0, 0, 0, 0};
      scores16_row<T, NH>(lds + kDecLdsK16, lane_, q16, sv);
    };
    // scores of block x (flags Mx) from its slot and / or the K tile buffer: each head keeps its own path's
    auto scores = [&](int slot, int Mx, float (&sv)[NH]) {
      float s4[NH], s16[NH];
      if (Mx != all_heads) scores4_row<NH>(load_k4_rows(lds + slot * kLdsBytes4, lane), lane, qf4, qsc, s4);
      if (Mx != 0) score16(s16);
#pragma unroll
      for (int u = 0; u < NH; ++u) sv[u] = ((Mx >> u) & 1) ? s16[u] : s4[u];
    };
    float sv[NH];                                       // raw score of key `lane` of block t on entry to step t, per head
#pragma unroll
    for (int u = 0; u < NH; ++u) sv[u] = 0.f;
    stage(-1, false);                                   // step -1: only the scores of block 0
    if (my_heads > 0 && n > 0) scores(slot_c, Mc, sv);
    slot_a = slot_b; slot_b = slot_c; slot_c = 1;
    // One step; WITH_NEXT (a compile-time flag): block t+1 exists.
    auto step = [&](int t, auto with_next) {
      Pa = Pb; Pb = Pc; Pc = Pd; Mb = Mc; Mc = Md;      // shift the flags; block t+2's are new
      Pd = flags(t + 2, Md);
      // most steps have no promoted block in sight: they skip the buffer decisions (3.6 % of an all-4-bit pass)
      stage(t, (Pb | Pc | Pd | early_prev) == 0 && t + kDecAhead < n);
      if (my_heads > 0) {
        const unsigned char* slot_v = lds + slot_b * kLdsBytes4;     // block t
        constexpr bool kNext = decltype(with_next)::value;
        // the K fragments of a 4-bit block t+1 are asked for first and arrive while the softmax of block t runs; its
        // score MFMAs go between the quantisation and the P.V MFMAs of block t
        const bool next4 = kNext && Mc != all_heads, next16 = kNext && Mc != 0;
        K4Tile kt;
        if (next4) kt = load_k4_rows(lds + slot_c * kLdsBytes4, lane);
        // softmax of every head; the accumulators of head u are column u: its rescale factor goes to lanes r = u
        float p[NH], alpha_lane = 1.f;
        uint32_t pb[NH];
        bool grew = false;
#pragma unroll
        for (int u = 0; u < NH; ++u) {
          float alpha;
          const bool g = softmax_row(sv[u], c, st[u], alpha, pb[u], p[u]);
          if (g) alpha_lane = (NH == 1 || r == u) ? alpha : alpha_lane;
          grew |= g;
        }
        rescale(o, grew, alpha_lane);
        // P operands: head u's codes / rounded probabilities in lanes r = u, zeros for the path it does not take
        v4i pq = {0, 0, 0, 0};
        uint32_t pb_lane = 127u;
        v8s pf[4];
#pragma unroll
        for (int s4i = 0; s4i < 4; ++s4i) pf[s4i] = (v8s){0, 0, 0, 0, 0, 0, 0, 0};
        auto place = [&](auto uc) {
          constexpr int u = decltype(uc)::value;
          if (((Mb >> u) & 1) == 0) {
            const v4i mine4 = gather_p4<u>(p[u], pb[u]);
            if constexpr (NH == 1) { pq = mine4; pb_lane = pb[u]; }
            else if (r == u) { pq = mine4; pb_lane = pb[u]; }
          } else {
            v8s mine16[4];
            gather_p16<T>(prow + wave * 64, lane, p[u], mine16);
            if (NH == 1 || r == u) {
#pragma unroll
              for (int s4i = 0; s4i < 4; ++s4i) pf[s4i] = mine16[s4i];
            }
          }
        };
        place(std::integral_constant<int, 0>{});
        if constexpr (NH > 1) place(std::integral_constant<int, 1>{});
        static_assert(NH <= 2, "one place() call per head");
        float s4[NH], s16[NH];
        if (next4) scores4_row<NH>(kt, lane, qf4, qsc, s4);
        if (Mb != all_heads) pv_fp4_codes(slot_v, lane, pq, pb_lane, o);
        if (Mb != 0) {
          int lane_ = lane;
          asm volatile("" : "+v"(lane_));
          pv_16_rounded<T, true>(lds + kDecLdsV16, lane_, pf, o);
        }
        if (next16) score16(s16);
        if constexpr (kNext) {
#pragma unroll
          for (int u = 0; u < NH; ++u) sv[u] = ((Mc >> u) & 1) ? s16[u] : s4[u];
        }
      }
      slot_a = slot_b; slot_b = slot_c; slot_c = slot_c + 1 == kDecRing ? 0 : slot_c + 1;
    };
    for (int t = 0; t + 1 < n; ++t) step(t, std::true_type{});
    if (n > 0) step(n - 1, std::false_type{});
  } else {
    // ---- several heads per wavefront: the transposed tiles of the prefill kernel, head wave + 4r in column r.  The heads
    // may split over the two paths of a block: both tiles are computed and each lane keeps its own head's. ----
    auto scores = [&](int slot, bool mine, bool any, bool all, v16f (&s)[2]) {
      if (!all) scores_fp4(lds + slot * kLdsBytes4, lane, qf4, qsc, s);
      if (any) {
        int lane_ = lane;
        asm volatile("" : "+v"(lane_));                 // no address of the 16-bit tile kept in registers across steps
        v8s q16[8];
#pragma unroll
        for (int s8 = 0; s8 < 8; ++s8)
          q16[s8] = real ? *reinterpret_cast<const v8s*>(q16row + 16 * s8) : (v8s){0, 0, 0, 0, 0, 0, 0, 0};
        if (all) {
          scores_16<T>(lds + kDecLdsK16, lane_, q16, s);
        } else {
          v16f s16[2];
          scores_16<T>(lds + kDecLdsK16, lane_, q16, s16);
          if (mine) { s[0] = s16[0]; s[1] = s16[1]; }
        }
      }
    };
    // this wavefront's votes on a block the group has promoted: bit 0 = some head of the wavefront, bit 1 = all of them
    auto votes = [&](int P, bool mine) -> int {
      const unsigned long long v = P ? (__builtin_amdgcn_ballot_w64(mine) & my_mask) : 0ULL;
      return (v != 0ULL ? 1 : 0) | (v == my_mask ? 2 : 0);
    };
    stage(-1, false);                                   // step -1: staging only
    slot_a = slot_b; slot_b = slot_c; slot_c = 1;
    for (int t = 0; t < n; ++t) {
      Pa = Pb; Pb = Pc; Pc = Pd; Mb = Mc; Mc = Md;
      Pd = flags(t + 2, Md);
      stage(t, false);
      if (my_heads > 0) {
        // the whole of block t in this step: scores, softmax, P.V (nothing is carried over to the next step)
        const unsigned char* slot_v = lds + slot_b * kLdsBytes4;
        const int vb = votes(Pb, Mb);
        const bool any_b = (vb & 1) != 0, all_b = (vb & 2) != 0;
        v16f s[2];
        scores(slot_b, Mb, any_b, all_b, s);
        float alpha;
        uint32_t pb;
        const bool grew = softmax_update(s, lane, false, kBk, c, st[0], alpha, pb);
        rescale(o, grew, alpha);
        // each lane contributes nothing on the path its head did not take (zero codes / zero probabilities)
        if (!all_b) {
          v4i pq = quantize_p_group(s, pb);
          if (Mb) pq = (v4i){0, 0, 0, 0};
          pv_fp4_codes(slot_v, lane, pq, pb, o);
        }
        if (any_b) {
          if (!Mb) { s[0] = (v16f){0.f}; s[1] = (v16f){0.f}; }
          int lane_ = lane;
          asm volatile("" : "+v"(lane_));
          pv_16<T, true>(lds + kDecLdsV16, lane_, s, o);
        }
      }
      slot_a = slot_b; slot_b = slot_c; slot_c = slot_c + 1 == kDecRing ? 0 : slot_c + 1;
    }
  }
  vm_wait<0>();

  // ---- partial (m, l, O) of this (head, partition): accumulator i of tile n is channel 32n + 8(i/4) + 4*half + i%4 ----
  // the row sum and maximum of this lane's column: the two halves of a column of the transposed tiles; all 64 lanes of
  // head r's register in the row layout
  float l, m;
  if constexpr (MULTI) {
    l = st[0].l + other_half(st[0].l);
    m = st[0].m;
  } else {
    l = 0.f; m = kEmptyMax;
#pragma unroll
    for (int u = 0; u < NH; ++u) {
      const float lu = wave_sum(st[u].l);
      if (r == u) { l = lu; m = st[u].m; }
    }
  }
  if (real) {
    float* po = a.part_o + (qh * a.nparts + part) * kD;
#pragma unroll
    for (int nn = 0; nn < 4; ++nn)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4)
        *reinterpret_cast<float4*>(po + 32 * nn + 8 * g4 + 4 * half) =
            make_float4(o[nn][4 * g4], o[nn][4 * g4 + 1], o[nn][4 * g4 + 2], o[nn][4 * g4 + 3]);
    if (half == 0) {
      a.part_ml[(qh * a.nparts + part) * 2] = m;
      a.part_ml[(qh * a.nparts + part) * 2 + 1] = l;
    }
  }
}

// The one key block that a length which is not a multiple of the block size leaves partly filled: one wavefront per
// (sequence, KV head) for all heads of the group (columns of the same tiles), operands straight from global memory,
// the keys past the length masked, the staging of the 16-bit V rows stopping at the last valid row.  Its result is
// one more partial (the last slot) for the merge.
constexpr int kDecodeTailLds = kBk * kRow16;      // one 16-bit V tile (padded rows, transposing reads)

template <typename T>
__global__ void __launch_bounds__(64) decode_tail_kernel(DecodeArgs a) {
  __shared__ __align__(16) unsigned char lds[kDecodeTailLds];
  const int lane = threadIdx.x & 63, half = lane >> 5, r = lane & 31;
  const int G = a.Hq / a.Hkv;
  const int unit = blockIdx.x;
  const int b = unit / a.Hkv, kvh = unit % a.Hkv;
  const int len = a.seqlens ? min(a.Nkv, max(0, a.seqlens[b])) : a.Nkv;
  const bool real = r < G;                                   // this lane's column is a real query head
  const int hq = kvh * G + (real ? r : 0);
  const size_t qh = (size_t)b * a.Hq + hq, kh = (size_t)b * a.Hkv + kvh;
  const int j_begin = len / kBk, j_end = (len + kBk - 1) / kBk;   // zero or one block

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
    qsc = sb[0] | (sb[1] << 8);
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

  for (int j = j_begin; j < j_end; ++j) {
    const unsigned long long word = real ? bm[j >> 6] : 0ULL;
    const bool mine16 = (word >> (j & 63)) & 1ULL;           // promoted for this lane's head
    const unsigned long long votes = __builtin_amdgcn_ballot_w64(mine16) & group_mask;
    const bool any16 = votes != 0ULL;
    const bool all16 = votes == group_mask;
    const int n_valid = len - j * kBk;

    v16f s[2];
    v4i vf4[4];
    uint32_t vsw = 0;
    if (!all16) {
      const uint8_t* vt = v4base + (size_t)j * 4096 + r * 32 + half * 16;
      const uint8_t* vsr = vsbase + ((size_t)j * 2 + half) * kD + r;
#pragma unroll
      for (int n = 0; n < 4; ++n) vf4[n] = *reinterpret_cast<const v4i*>(vt + 1024 * n);
      vsw = (uint32_t)vsr[0] | ((uint32_t)vsr[32] << 8) | ((uint32_t)vsr[64] << 16) | ((uint32_t)vsr[96] << 24);
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
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        // rows past the cached tokens are never written by anyone: stage the last valid row in their place
        // (their probabilities are zero, but zero times an arbitrary bit pattern need not be)
        const int chunk = lane + 64 * u, row = chunk >> 4, col = chunk & 15;
        *reinterpret_cast<uint4*>(lds + row * kRow16 + col * 16) =
            *reinterpret_cast<const uint4*>(v16base + ((size_t)j * kBk + min(row, n_valid - 1)) * kD + col * 8);
      }
      v8s qf16[8];
#pragma unroll
      for (int s8 = 0; s8 < 8; ++s8)
        qf16[s8] = real ? *reinterpret_cast<const v8s*>(a.q + qh * kD + 16 * s8 + 8 * half) : (v8s){0, 0, 0, 0, 0, 0, 0, 0};
      v16f s16[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        // key rows past the length are not read either: the last valid row stands in, its scores are masked below
        const uint16_t* krow = k16base + ((size_t)j * kBk + min(key_of_row(r, t), n_valid - 1)) * kD + 8 * half;
        v16f acc = {0.f};
#pragma unroll
        for (int s8 = 0; s8 < 8; ++s8) acc = T::mfma(*reinterpret_cast<const v8s*>(krow + 16 * s8), qf16[s8], acc);
        s16[t] = acc;
      }
      if (all16 || mine16) { s[0] = s16[0]; s[1] = s16[1]; }
    }
    float alpha;
    uint32_t pb;
    const bool grew = softmax_update(s, lane, true, n_valid, c, st, alpha, pb);
    rescale(o, grew, alpha);
    if (!all16) {
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

  const float l = st.l + other_half(st.l);
  if (real) {
    const int pid = a.nparts - 1;
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
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wavefront-uniform: the loop over the heads stays scalar
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
  typedef float f4v __attribute__((ext_vector_type(4)));
#define THRIFT_LOAD_CHUNK(C)                                                                                     \
  _Pragma("unroll") for (int u = 0; u < 8; ++u) {                                                                \
    const int c4 = tid + 256 * u, row = c4 >> 5, col = (c4 & 31) * 4;                                            \
    pre[u] = make_float4(0.f, 0.f, 0.f, 0.f);                                                                    \
    if ((C) * 64 + row < Tk) {   /* read once by the whole grid: streaming hint */                               \
      const f4v t = __builtin_nontemporal_load(reinterpret_cast<const f4v*>(kunit + ((size_t)(C) * 64 + row) * kD + col)); \
      pre[u] = make_float4(t.x, t.y, t.z, t.w);                                                                  \
    }                                                                                                            \
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

// One workgroup per row: thread t keeps key blocks t, t+256, ... in registers; the k-th largest key is found by a
// bitwise search from the top bit (64 steps at most, typically 25-30: it stops once a candidate has exactly k keys at or
// above it; two bits per step were slower, the steps are bound by the ballots, not by the barrier).  A step counts per lane, sums a wavefront by the ballots of the count's bits and the four wavefronts
// through LDS (one barrier per step; the slots alternate so that a step's values outlive the next step's writes).
// With one wavefront per row the 512 rows of the benchmark occupied a quarter of the chip and took 21 us.
template <int MAXC>
__global__ void __launch_bounds__(256) decode_select_kernel(DecodeSelectArgs p, long n_rows) {
  __shared__ int cross[2][4];
  __shared__ int tcnt[MAXC][4], scnt[MAXC][4];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const long row = blockIdx.x;
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
    const int j = c * 256 + tid;
    key[c] = j < vis ? p.keys[row * p.Tk + j] : 0ULL;
  }
  unsigned long long* bm = p.bitmap + row * p.words;
  int32_t* out = p.idx_out ? p.idx_out + row * p.kmax_out : nullptr;
  if (p.cnt_out && tid == 0) p.cnt_out[row] = k;
  if (k <= 0) {                                              // uniform over the workgroup
    for (int w = tid; w < p.words; w += 256) bm[w] = 0ULL;
    if (out) for (int t = tid; t < p.kmax_out; t += 256) out[t] = -1;
    return;
  }
  // Invalid slots hold key 0, and every candidate below is >= 1, so they never count.  Each lane counts its own keys
  // (at most MAXC <= 16, five bits); the wavefront total is the weighted popcount of the ballots of those bits.
  int parity = 0;
  auto row_total = [&](int n_lane) -> int {                  // called by all threads at the same point
    int tot = 0;
#pragma unroll
    for (int b5 = 0; b5 < 5; ++b5) tot += __popcll(__ballot((n_lane >> b5) & 1)) << b5;
    if (lane == 0) cross[parity][wave] = tot;
    __syncthreads();
    const int n = cross[parity][0] + cross[parity][1] + cross[parity][2] + cross[parity][3];
    parity ^= 1;
    return n;
  };
  uint64_t T = 0;
  for (int bit = 63; bit >= 0; --bit) {
    const uint64_t cand = T | (1ULL << bit);
    int n_lane = 0;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) n_lane += key[c] >= cand ? 1 : 0;
    const int n = row_total(n_lane);
    if (n >= k) T = cand;
    if (n == k) break;                                       // exactly the k largest lie at or above cand: done
  }
  int n_gt;
  {
    int n_lane = 0;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) n_lane += key[c] > T ? 1 : 0;
    n_gt = row_total(n_lane);
  }
  const int need_ties = k - n_gt;                            // keys equal to T, taken from the smallest id up (0 after an early exit above a gap)
  // Ids ascend with (c, wavefront, lane).  First the tie counts of every (c, wavefront), then the selection, then the
  // output positions: two barriers in all.
  const uint64_t lt_mask = (1ULL << lane) - 1ULL;
  uint64_t tie_b[MAXC];
#pragma unroll
  for (int c = 0; c < MAXC; ++c) {
    tie_b[c] = __ballot(c * 256 + tid < vis && key[c] == T);
    if (lane == 0) tcnt[c][wave] = __popcll(tie_b[c]);
  }
  __syncthreads();
  uint64_t sel_b[MAXC];
  int ties_before = 0;                                       // ties in earlier chunks and earlier wavefronts of this chunk
#pragma unroll
  for (int c = 0; c < MAXC; ++c) {
    int before = ties_before;
    for (int w = 0; w < wave; ++w) before += tcnt[c][w];
    const bool valid = c * 256 + tid < vis;
    const bool tie = valid && key[c] == T;
    const bool sel = valid && (key[c] > T || (tie && before + __popcll(tie_b[c] & lt_mask) < need_ties));
    sel_b[c] = __ballot(sel);
    if (lane == 0) scnt[c][wave] = __popcll(sel_b[c]);
    ties_before += tcnt[c][0] + tcnt[c][1] + tcnt[c][2] + tcnt[c][3];
  }
  __syncthreads();
  int written = 0;
#pragma unroll
  for (int c = 0; c < MAXC; ++c) {
    int before = written;
    for (int w = 0; w < wave; ++w) before += scnt[c][w];
    if (out && ((sel_b[c] >> lane) & 1ULL)) out[before + __popcll(sel_b[c] & lt_mask)] = c * 256 + tid;
    const int word = c * 4 + wave;
    if (lane == 0 && word < p.words) bm[word] = sel_b[c];
    written += scnt[c][0] + scnt[c][1] + scnt[c][2] + scnt[c][3];
  }
  for (int w = MAXC * 4 + tid; w < p.words; w += 256) bm[w] = 0ULL;
  if (out) for (int t = k + tid; t < p.kmax_out; t += 256) out[t] = -1;
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
  const dim3 grid((unsigned)n_rows), block(256);
  if (chunks <= 8) decode_select_kernel<2><<<grid, block, 0, st>>>(p, n_rows);            // 256 key blocks per register slot
  else if (chunks <= 16) decode_select_kernel<4><<<grid, block, 0, st>>>(p, n_rows);
  else if (chunks <= 32) decode_select_kernel<8><<<grid, block, 0, st>>>(p, n_rows);
  else decode_select_kernel<16><<<grid, block, 0, st>>>(p, n_rows);
}

// Launch order of the split-K workgroups: heaviest first.  A workgroup's duration follows the bytes it stages (8.5 KiB
// per key block, 32 KiB more for a block that some head of the group has promoted), the selections differ between
// partitions and sequences differ in length, and a grid of a few workgroups per CU slot has no later rounds to even
// that out: in natural order the pass ends when the unluckiest slot does.  Handing the heaviest items out first pairs
// them with the lightest (measured on two rounds of workgroups whose bytes scatter by +-17 %: 1 to 3 % of the pass).
// One workgroup: weight of every item from the selection bitmaps, counting sort into kOrderBins bins, descending; items
// of one bin come out in no particular order (the results do not depend on the order at all).
constexpr int kOrderMaxItems = 8192;     // beyond this many items the grid has rounds enough: natural order
constexpr int kOrderBins = 1024;       // = the threads of the ordering workgroup

__global__ void __launch_bounds__(1024) decode_order_kernel(DecodeArgs a, int n_items, int* __restrict__ order) {
  __shared__ unsigned short bin_of[kOrderMaxItems];
  __shared__ int hist[kOrderBins];
  __shared__ int wave_total[16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int G = a.Hq / a.Hkv;
  hist[tid] = 0;
  __syncthreads();
  for (int item = tid; item < n_items; item += 1024) {
    const int part = item % a.nsplit, unit = item / a.nsplit;
    const int b = unit / a.Hkv, kvh = unit % a.Hkv;
    const int len = a.seqlens ? min(a.Nkv, max(0, a.seqlens[b])) : a.Nkv;
    const int Tk = len / kBk;
    const int j_begin = min(Tk, part * a.split_blocks), j_end = min(Tk, j_begin + a.split_blocks);
    int promoted = 0;                                          // key blocks of the partition that some head of the group has promoted
    if (j_end > j_begin) {
      const unsigned long long* bm = a.bitmap + ((size_t)b * a.Hq + (size_t)kvh * G) * a.bitmap_words;
      for (int w = j_begin >> 6; w <= (j_end - 1) >> 6; ++w) {
        unsigned long long any = 0ULL;
#pragma unroll 4
        for (int h = 0; h < G; ++h) any |= bm[(size_t)h * a.bitmap_words + w];
        const int lo = max(j_begin - 64 * w, 0), hi = min(j_end - 64 * w, 64);          // bits lo .. hi-1 of this word
        any >>= lo;
        if (hi - lo < 64) any &= (1ULL << (hi - lo)) - 1ULL;
        promoted += __popcll(any);
      }
    }
    // bytes in units of a 4-bit block: 1 per block + 4 per promoted block (32 KiB against 8.5 KiB), at most 5 per block
    const long weight = (long)(j_end - j_begin) + 4L * promoted;
    const int bin = (int)(weight * (kOrderBins - 1) / (5L * a.split_blocks));
    bin_of[item] = (unsigned short)bin;
    atomicAdd(&hist[bin], 1);
  }
  __syncthreads();
  // first position of every bin in descending order of weight: thread t owns bin kOrderBins-1-t; exclusive prefix sum
  const int mine = hist[kOrderBins - 1 - tid];
  int incl = mine;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int up = __shfl_up(incl, d);
    if (lane >= d) incl += up;
  }
  if (lane == 63) wave_total[wave] = incl;
  __syncthreads();
  int before = 0;
  for (int w = 0; w < wave; ++w) before += wave_total[w];
  __syncthreads();
  hist[kOrderBins - 1 - tid] = before + incl - mine;           // from here on: the bin's next free position
  __syncthreads();
  for (int item = tid; item < n_items; item += 1024) order[atomicAdd(&hist[bin_of[item]], 1)] = item;
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

int decode_order_items(int B, int Hkv, int nsplit) {
  const long items = (long)B * Hkv * nsplit;
  return items <= kOrderMaxItems ? (int)items : 0;
}

void launch_decode(const DecodeArgs& a, hipStream_t st) {
  const unsigned grid = (unsigned)((long)a.B * a.Hkv * a.nsplit);
  if (a.order != nullptr) decode_order_kernel<<<dim3(1), dim3(1024), 0, st>>>(a, (int)grid, a.order);
  // heads per wavefront: one or two in the row layout (groups of up to 4 / 8 heads), else the transposed tiles
  const int G = a.Hq / a.Hkv;
#define THRIFT_LAUNCH_PARTIAL(T)                                                             \
  do {                                                                                       \
    if (G <= 4) decode_partial_kernel<T, 1><<<dim3(grid), dim3(256), 0, st>>>(a);            \
    else if (G <= 8) decode_partial_kernel<T, 2><<<dim3(grid), dim3(256), 0, st>>>(a);       \
    else decode_partial_kernel<T, 0><<<dim3(grid), dim3(256), 0, st>>>(a);                   \
  } while (0)
  if (a.dt == THRIFT_F16) THRIFT_LAUNCH_PARTIAL(F16);
  else THRIFT_LAUNCH_PARTIAL(BF16);
#undef THRIFT_LAUNCH_PARTIAL
  if (a.seqlens != nullptr) {                          // without lengths every sequence fills the cache: no partly filled block
    const unsigned tail_grid = (unsigned)((long)a.B * a.Hkv);
    if (a.dt == THRIFT_F16) decode_tail_kernel<F16><<<dim3(tail_grid), dim3(64), 0, st>>>(a);
    else decode_tail_kernel<BF16><<<dim3(tail_grid), dim3(64), 0, st>>>(a);
  }
  decode_merge_kernel<<<dim3((unsigned)((long)a.B * a.Hq)), dim3(128), 0, st>>>(a);
}

}  // namespace thrift
