// Per-wavefront tile arithmetic of Algorithm 1 on gfx950 matrix units, shared by the prefill and the
// decode kernels.
//
// One wavefront owns 32 query rows and walks 64-key blocks.  Everything is computed transposed, so
// that each query lives in one lane column and no cross-lane traffic is needed inside a row:
//
//   S^T (keys x queries) = K_j . Q^T        two 32x32 MFMA tiles (keys 0-31 / 32-63 after the row
//                                           permutation below), accumulated over D = 128
//   O^T (channels x queries) += V_j^T . P^T  four 32x32 MFMA tiles (32 channels each)
//
// 32x32 MFMA register layouts (64 lanes; lane = 32*half + r):
//   A operand: row r, contraction slots [G*half, G*half + G)     (G = 32 for MXFP4 K=64, 8 for 16-bit K=16)
//   B operand: column r, same contraction slots
//   C/D: column r, rows 8*(i/4) + 4*half + i%4 for accumulator register i = 0..15
// Row permutation of the S^T tiles: MFMA row rho of sub-tile t is fed key
//   pi_t(rho) = 32*((rho>>2)&1) + 16*t + 4*(rho>>3) + (rho&3),
// so lane (half, r) ends up holding, for query r, the 32 consecutive keys 32*half + (16*t + i): exactly
// the 32-slot group it must supply as the B operand of the P.V MFMA, and exactly one MXFP4 scale group
// of P and of V.  Row max / row sum combine the two halves with one lane swap.
#pragma once

#include "thrift_device.h"

namespace thrift {

// LDS layout of one staged 4-bit key block (bytes): a slot of the prefill kernel's ring.
constexpr int kLdsK4 = 0;                    // 4096 B, stored in MFMA fragment order
constexpr int kLdsV4 = 4096;                 // 4096 B, MFMA fragment order: chunk (n*64 + lane) = channel 32n + r, token half
constexpr int kLdsKS = 8192;                 // 64 x 4 scale bytes of K, [key][d-group]
constexpr int kLdsVS = 8448;                 // 2 x 128 scale bytes of V, [token group][channel]
constexpr int kLdsBytes4 = 8704;
// 16-bit tiles.  Padded rows (272 B) where a wavefront stages its own tile through registers (decode);
// unpadded 256-byte rows with an XOR swizzle of the 16-byte chunks where the tile arrives by LDS DMA
// (prefill), which can only write 1 KiB of consecutive LDS per instruction.
constexpr int kRow16 = 2 * kD + 16;
constexpr int kTile16 = kBk * 2 * kD;        // 16384
// chunk c of row `row` lives at chunk position c ^ swz: K is read by rows (8 consecutive lanes take
// rows {R..R+3, R+32..R+35} at one chunk index), V by 4-row x 64-byte patches (transposing reads).
__device__ __forceinline__ int k16_swizzle(int row) { return (row & 3) | (((row >> 5) & 1) << 2); }
__device__ __forceinline__ int v16_swizzle(int row) { return 4 * (row & 3); }

__device__ __forceinline__ int key_of_row(int rho, int t) {
  return 32 * ((rho >> 2) & 1) + 16 * t + 4 * (rho >> 3) + (rho & 3);
}

__device__ __forceinline__ v8i widen(v4i x) { return __builtin_shufflevector(x, x, 0, 1, 2, 3, -1, -1, -1, -1); }

// ---- staging primitives shared by the prefill and the decode kernels ----

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also drains every outstanding global
// load (a full fence), which would wait for the tiles in flight at every key block; here only this
// wavefront's LDS reads must have completed before the rendezvous.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Wait until at most N of this wavefront's global loads (LDS DMA included) are still in flight.
template <int N>
__device__ __forceinline__ void vm_wait() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

typedef __attribute__((address_space(3))) void* lds_void_ptr;
__device__ __forceinline__ uint32_t lds_address(const void* p) { return (uint32_t)(uintptr_t)(lds_void_ptr)(p); }

// LDS DMA: the 64 lanes fetch 16 (4) bytes each from base + off and the hardware writes them to the
// 1 KiB (256 B) of consecutive LDS that starts at lds_base, lane l at lds_base + 16 l (4 l).  base and
// lds_base are wavefront-uniform.  The instruction takes its LDS base from M0, which each statement sets
// itself.  M0 is a reserved register for the compiler (it cannot be named as a clobber): it never keeps a
// value there across statements and loads it right before the few instructions of its own that read it; the
// build additionally checks that the kernel's listing mentions M0 only inside these statements.
// Completion is counted by vmcnt like any global load.
// STREAM: the bytes are read once by the whole grid (the decode kernel's cache tiles): the load carries the non-temporal
// hint, so that it does not displace what other kernels' data the caches hold and streams at the higher rate measured for
// such loads.
template <bool STREAM = false>
__device__ __forceinline__ void dma_b128(const void* base, uint32_t off, uint32_t lds_base) {
  if constexpr (STREAM)
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt" ::"v"(off), "s"(base), "s"(lds_base) : "memory");
  else
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off), "s"(base), "s"(lds_base) : "memory");
}
template <bool STREAM = false>
__device__ __forceinline__ void dma_b32(const void* base, uint32_t off, uint32_t lds_base) {
  if constexpr (STREAM)
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1 nt" ::"v"(off), "s"(base), "s"(lds_base) : "memory");
  else
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1" ::"v"(off), "s"(base), "s"(lds_base) : "memory");
}

struct RowState {
  float m;      // running maximum of the raw (unscaled) scores of this lane's query
  float l;      // this lane's partial row sum (the two halves of a query add up at the end)
};

// S^T for a 4-bit tile.  The two MFMAs of a sub-tile split D = 128 so that lane half h contracts d-group
// 2h + kk in MFMA kk (any split works as long as K and Q agree): the lane's two K scale bytes are then
// neighbours in the [key][d-group] scale row and arrive with one 16-bit LDS read, byte kk for MFMA kk.
// qf: the lane's two Q fragments (d-groups 2*half + kk), qsc: its Q scale bytes, byte kk for fragment kk.
struct K4Tile {
  v4i a[4];            // fragment (t, kk) at index 2t + kk
  uint32_t ks[2];      // the lane's two K scale bytes of sub-tile t
};
__device__ __forceinline__ K4Tile load_k4(const unsigned char* lds, int lane) {
  const int half = lane >> 5, r = lane & 31;
  const unsigned char* ksrow = lds + kLdsKS + 4 * key_of_row(r, 0) + 2 * half;   // sub-tile 1: 16 keys = 64 bytes further
  K4Tile k;
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    k.ks[t] = *reinterpret_cast<const uint16_t*>(ksrow + 64 * t);
    k.a[2 * t] = *reinterpret_cast<const v4i*>(lds + kLdsK4 + ((t * 2 + 0) * 64 + lane) * 16);
    k.a[2 * t + 1] = *reinterpret_cast<const v4i*>(lds + kLdsK4 + ((t * 2 + 1) * 64 + lane) * 16);
  }
  return k;
}
__device__ __forceinline__ void scores_fp4_regs(const K4Tile& k, const v4i (&qf)[2], uint32_t qsc, v16f (&s)[2]) {
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    v16f acc = {0.f};
    acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen(k.a[2 * t]), widen(qf[0]), acc, 4, 4, 0, k.ks[t], 0, qsc);
    acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen(k.a[2 * t + 1]), widen(qf[1]), acc, 4, 4, 1, k.ks[t], 1, qsc);
    s[t] = acc;
  }
}
__device__ __forceinline__ void scores_fp4(const unsigned char* lds, int lane, const v4i (&qf)[2], uint32_t qsc, v16f (&s)[2]) {
  scores_fp4_regs(load_k4(lds, lane), qf, qsc, s);
}

// S^T for a 16-bit tile.  ktile: the swizzled [64 keys][256 B] LDS tile; qf[s8]: the lane's query
// elements d = 16*s8 + 8*half + [0,8).
template <typename T>
__device__ __forceinline__ void scores_16(const unsigned char* ktile, int lane, const v8s (&qf)[8], v16f (&s)[2]) {
  const int half = lane >> 5, r = lane & 31;
  const int row0 = key_of_row(r, 0);                    // the row of sub-tile 1 is 16 further: same swizzle
  const uint32_t base = (uint32_t)(row0 * 256 + 16 * (half ^ k16_swizzle(row0)));
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    v16f acc = {0.f};
#pragma unroll
    for (int s8 = 0; s8 < 8; ++s8) {
      const v8s a = *reinterpret_cast<const v8s*>(ktile + ((base ^ (32u * s8)) + 4096u * t));
      acc = T::mfma(a, qf[s8], acc);
    }
    s[t] = acc;
  }
}

// Running maximum of a row that has seen no key yet: a large negative finite number instead of -inf, so that
// neither m - m nor m * c needs a guard (an exponent argument of -inf still gives probability 0).
constexpr float kEmptyMax = -1.0e30f;

__device__ __forceinline__ float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }   // one v_max3_f32

// Online-softmax update for the lane's 32 scores (Alg. 1 steps 10-12 / 16-17): masks, raises the
// running maximum, turns s into the unnormalised probabilities exp(scale*(s - m_new)) in place and adds
// them to the partial row sum.  Returns true, for the whole wavefront, when some row raised its maximum:
// only then does alpha hold exp(scale*(m_old - m_new)) (Alg. 1 steps 11 / 16), the row sum is already
// scaled by it and the caller must rescale its accumulators; otherwise alpha is 1 everywhere and no
// arithmetic was spent on it (the common case once the first blocks are behind).
// pbyte receives the E8M0 byte of the lane's 32-key group of P (Alg. 1 step 19 with a power-of-two scale):
// floor(log2(largest probability of the group)) - 2 + 127, at least 1 so that the scale is a normal float.
//   c = softmax_scale * log2(e);  n_valid = number of leading keys of the block this query may see.
__device__ __forceinline__ bool softmax_update(v16f (&s)[2], int lane, bool mask, int n_valid, float c, RowState& st,
                                               float& alpha, uint32_t& pbyte) {
  const int half = lane >> 5;
  if (mask) {
    int lim = n_valid - 32 * half;                      // the lane's keys 16t + i at or past lim are masked
    asm volatile("" : "+v"(lim));                       // keep one register: no per-element thresholds hoisted out of the key loop
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int i = 0; i < 16; ++i)
        if (16 * t + i >= lim) s[t][i] = -INFINITY;
  }
  float mloc = max3(s[0][0], s[0][1], s[0][2]);
#pragma unroll
  for (int i = 3; i < 15; i += 2) mloc = max3(mloc, s[0][i], s[0][i + 1]);
  mloc = max3(mloc, s[0][15], s[1][0]);
#pragma unroll
  for (int i = 1; i < 15; i += 2) mloc = max3(mloc, s[1][i], s[1][i + 1]);
  mloc = fmaxf(mloc, s[1][15]);
  // the other half of the row lives 32 lanes away: after the swap of two copies one register holds the lower
  // half's maximum in every lane and the other the upper half's
  uint32_t lo = __float_as_uint(mloc), hi = lo;
  {
    auto sw = __builtin_amdgcn_permlane32_swap(lo, hi, false, false);
    lo = sw[0]; hi = sw[1];
  }
  const float m_old = st.m;
  const float m_new = max3(m_old, __uint_as_float(lo), __uint_as_float(hi));
  const bool grew = __builtin_amdgcn_ballot_w64(m_new != m_old) != 0ULL;
  if (grew) {
    float d = m_old - m_new;
    asm volatile("" : "+v"(d));                                    // keeps the exponential inside the branch
    alpha = fast_exp2(d * c);
    float l = st.l;
    // stays inside the branch (no select on the common path).  The wait states are for the hand-written consumer of
    // a transcendental result: the compiler spaces its own instructions, not the inside of an asm statement.
    asm volatile("s_nop 1\n\tv_mul_f32 %0, %1, %0" : "+v"(l) : "v"(alpha));
    st.l = l;
  }
  st.m = m_new;
  // Elements use one fused multiply-add, s*c - m*c; its rounding residue (a few 1e-7 relative on p) is
  // harmless for the codes and the row sum.  The exponent of the group maximum, which fixes the power-of-two
  // scale of the P quantiser, is formed from (s - m)*c instead: the row maximum then maps to exactly 2^0 and
  // can never slip under the binade boundary (where the floor rule would scale it to 8 and saturate it to 6).
  int e;
  {
    const float x = (mloc - m_new) * c;
    asm("v_cvt_flr_i32_f32 %0, %1" : "=v"(e) : "v"(x));        // floor; -inf (nothing visible) saturates to INT_MIN
  }
  pbyte = (uint32_t)max(e + 125, 1);
  const float mc = m_new * c;
  float sum;
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float p = fast_exp2(__builtin_fmaf(s[t][i], c, -mc));
      s[t][i] = p;
      sum = (t == 0 && i == 0) ? p : sum + p;
    }
  st.l += sum;
  return grew;
}

__device__ __forceinline__ void rescale(v16f (&o)[4], bool grew, float alpha) {
  // Skipping is exact: alpha == 1 leaves every accumulator unchanged.  The multiplies are written as
  // in-place instructions so that the accumulators keep their registers on both sides of the branch
  // (otherwise the skip path pays 64 register copies per key block).
  if (grew) {
#pragma unroll
    for (int n = 0; n < 4; ++n)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        float x = o[n][i];
        asm volatile("v_mul_f32 %0, %1, %0" : "+v"(x) : "v"(alpha));
        o[n][i] = x;
      }
    asm volatile("s_nop 4");     // keep the matrix unit's read of the accumulators clear of the writes above
  }
}

// 4-bit P.V (Alg. 1 steps 19-20 with the first-level scale equal to 1): quantise the lane's 32
// probabilities as one MXFP4 group and accumulate O^T += V^T . P^T on the scaled MFMA.  v0..v3: the
// lane's V^T fragments (channel 32n + r, tokens 32*half .. +31).  pb: the E8M0 byte of the lane's P group
// (softmax_update).  The V scale bytes come either packed
// in one register (PACKED: byte n of vs0) or one per register (byte 0 of vs0..vs3).
// Alg. 1 step 19: the lane's 32 probabilities as one MXFP4 group, 16 code bytes in MFMA operand order.
__device__ __forceinline__ v4i quantize_p_group(const v16f (&p)[2], uint32_t pb) {
  const float pscale = __uint_as_float(pb << 23);              // pb: E8M0 byte of the group, >= 1 (a normal float)
  v4i pq;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    uint32_t o32;
    asm volatile("" : "=v"(o32));                              // all four bytes are written below: no initial value needed
    const int t = w >> 1, i0 = 8 * (w & 1);                    // slots 8w .. 8w+7 = p[t][i0 .. i0+7]
    o32 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(o32, p[t][i0 + 0], p[t][i0 + 1], pscale, 0);
    o32 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(o32, p[t][i0 + 2], p[t][i0 + 3], pscale, 1);
    o32 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(o32, p[t][i0 + 4], p[t][i0 + 5], pscale, 2);
    o32 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(o32, p[t][i0 + 6], p[t][i0 + 7], pscale, 3);
    pq[w] = (int)o32;
  }
  return pq;
}

// O^T += V^T . P^T for a group of P already quantised (pq: quantize_p_group's codes).
template <bool PACKED>
__device__ __forceinline__ void pv_fp4_codes_regs(v4i pq, uint32_t pb, uint32_t vs0, uint32_t vs1, uint32_t vs2, uint32_t vs3,
                                                  v4i v0, v4i v1, v4i v2, v4i v3, v16f (&o)[4]) {
  const v8i pb8 = widen(pq);
  if (PACKED) {
    o[0] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen(v0), pb8, o[0], 4, 4, 0, vs0, 0, pb);
    o[1] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen(v1), pb8, o[1], 4, 4, 1, vs0, 0, pb);
    o[2] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen(v2), pb8, o[2], 4, 4, 2, vs0, 0, pb);
    o[3] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen(v3), pb8, o[3], 4, 4, 3, vs0, 0, pb);
  } else {
    o[0] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen(v0), pb8, o[0], 4, 4, 0, vs0, 0, pb);
    o[1] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen(v1), pb8, o[1], 4, 4, 0, vs1, 0, pb);
    o[2] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen(v2), pb8, o[2], 4, 4, 0, vs2, 0, pb);
    o[3] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen(v3), pb8, o[3], 4, 4, 0, vs3, 0, pb);
  }
}

template <bool PACKED>
__device__ __forceinline__ void pv_fp4_regs(const v16f (&p)[2], uint32_t pb, uint32_t vs0, uint32_t vs1, uint32_t vs2,
                                            uint32_t vs3, v4i v0, v4i v1, v4i v2, v4i v3, v16f (&o)[4]) {
  pv_fp4_codes_regs<PACKED>(quantize_p_group(p, pb), pb, vs0, vs1, vs2, vs3, v0, v1, v2, v3, o);
}

// The same with V^T fragments and scales taken from a staged LDS slot: from the codes, or from the probabilities.
__device__ __forceinline__ void pv_fp4_codes(const unsigned char* slot, int lane, v4i pq, uint32_t pb, v16f (&o)[4]) {
  const int half = lane >> 5, r = lane & 31;
  const unsigned char* vs = slot + kLdsVS + half * kD + r;
  const unsigned char* vbase = slot + kLdsV4 + lane * 16;
  pv_fp4_codes_regs<false>(pq, pb, vs[0], vs[32], vs[64], vs[96], *reinterpret_cast<const v4i*>(vbase),
                           *reinterpret_cast<const v4i*>(vbase + 1024), *reinterpret_cast<const v4i*>(vbase + 2048),
                           *reinterpret_cast<const v4i*>(vbase + 3072), o);
}
__device__ __forceinline__ void pv_fp4(const unsigned char* slot, int lane, const v16f (&p)[2], uint32_t pb, v16f (&o)[4]) {
  pv_fp4_codes(slot, lane, quantize_p_group(p, pb), pb, o);
}

// 16-bit P.V (Alg. 1 step 13): P rounded to the input dtype; V^T fragments come straight out of the
// row-major LDS tile `vtile` through the transposing 64-bit LDS read (each 16-lane group turns a
// 4-key x 16-channel patch into 4 consecutive keys of one channel per lane).  SWZ: the tile has unpadded
// 256-byte rows with swizzled chunks (v16_swizzle), otherwise rows of kRow16 bytes.
// P rounded to the input dtype, in the B-operand order of the 16-bit P.V MFMAs (slot group s = keys 8s .. 8s+7 of the lane's 32).
template <typename T>
__device__ __forceinline__ void round_p16(const v16f (&p)[2], v8s (&pf)[4]) {
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const int t = s >> 1, i0 = 8 * (s & 1);
#pragma unroll
    for (int e = 0; e < 8; ++e) pf[s][e] = (short)T::from_float(p[t][i0 + e]);
  }
}

template <typename T, bool SWZ>
__device__ __forceinline__ void pv_16_rounded(const unsigned char* vtile, int lane, const v8s (&pf)[4], v16f (&o)[4]) {
  const int half = lane >> 5, r = lane & 31, g = r >> 4, i16 = r & 15;
  constexpr int kRow = SWZ ? 2 * kD : kRow16;
  typedef v4s __attribute__((address_space(3))) * lds_v4s_ptr;
  // keys 32*half + 8*s + 4*u + (i16>>2), channels 32*n + 16*g + 4*(i16&3); the swizzle term of all these
  // rows is 4*((i16>>2)&3), which turns the 64-byte step of n into an XOR
  const uint32_t lane_off = (uint32_t)((32 * half + (i16 >> 2)) * kRow + (16 * g + 4 * (i16 & 3)) * 2);
  const uint32_t sw = SWZ ? 64u * ((i16 >> 2) & 3) : 0u;
#pragma unroll
  for (int s = 0; s < 4; ++s) {
#pragma unroll
    for (int n = 0; n < 4; ++n) {
      const unsigned char* base = vtile + ((SWZ ? ((lane_off + sw) ^ (64u * n)) : lane_off + 64u * n) + 8u * s * kRow);
      const v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)(base));
      const v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)(base + 4 * kRow));
      const v8s a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      o[n] = T::mfma(a, pf[s], o[n]);
    }
  }
}

template <typename T, bool SWZ>
__device__ __forceinline__ void pv_16(const unsigned char* vtile, int lane, const v16f (&p)[2], v16f (&o)[4]) {
  v8s pf[4];
  round_p16<T>(p, pf);
  pv_16_rounded<T, SWZ>(vtile, lane, pf, o);
}

}  // namespace thrift
