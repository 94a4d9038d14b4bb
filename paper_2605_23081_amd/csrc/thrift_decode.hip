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

template <typename T>
__global__ void __launch_bounds__(256, 2) decode_partial_kernel(DecodeArgs a) {
  __shared__ __align__(16) unsigned char lds_all[4 * kDecodeLdsPerWave];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, half = lane >> 5, r = lane & 31;
  unsigned char* lds = lds_all + wave * kDecodeLdsPerWave;
  const int G = a.Hq / a.Hkv, Tk_all = a.Nkv / kBk;
  const int part = blockIdx.x % a.nsplit;
  const int unit = blockIdx.x / a.nsplit;
  const int b = unit / a.Hkv, kvh = unit % a.Hkv;
  const int Tk = a.seqlens ? min(Tk_all, max(0, a.seqlens[b]) / kBk) : Tk_all;
  const bool real = r < G;                                   // this lane's column is a real query head
  const int hq = kvh * G + (real ? r : 0);
  const size_t qh = (size_t)b * a.Hq + hq, kh = (size_t)b * a.Hkv + kvh;

  // contiguous quarter of the partition for this wavefront
  const int quarter = a.split_blocks / 4;
  const int j_begin = part * a.split_blocks + wave * quarter;
  const int j_end = min(Tk, j_begin + quarter);

  // ---- Q fragments (zeros for padding columns) ----
  v4i qf4[2] = {(v4i){0, 0, 0, 0}, (v4i){0, 0, 0, 0}};
  uint32_t qsc = 0x7f7f7f7fu;
  if (real) {
    qf4[0] = *reinterpret_cast<const v4i*>(a.q4 + qh * 64 + half * 16);
    qf4[1] = *reinterpret_cast<const v4i*>(a.q4 + qh * 64 + 32 + half * 16);
    qsc = *reinterpret_cast<const uint32_t*>(a.qs + qh * 4) >> (8 * half);
  }

  const uint8_t* k4base = a.k4 + kh * a.Nkv * 64;
  const uint8_t* v4base = a.v4 + kh * (size_t)(a.Nkv / 64) * 4096;
  const uint8_t* ksbase = a.ks + kh * a.Nkv * 4;
  const uint8_t* vsbase = a.vs + kh * (size_t)(a.Nkv / 32) * kD;
  const uint16_t* k16base = a.k16 + kh * a.Nkv * kD;
  const uint16_t* v16base = a.v16 + kh * a.Nkv * kD;
  const unsigned long long* bm = a.bitmap + qh * a.bitmap_words;

  RowState st = {-INFINITY, 0.f};
  v16f o[4];
#pragma unroll
  for (int n = 0; n < 4; ++n) o[n] = (v16f){0.f};
  const float c = a.scale * 1.4426950408889634f;
  const unsigned long long group_mask = G >= 32 ? 0xffffffffULL : ((1ULL << G) - 1ULL);

  unsigned long long word = 0;
  int word_id = -1;
  for (int j = j_begin; j < j_end; ++j) {
    if ((j >> 6) != word_id) { word_id = j >> 6; word = real ? bm[word_id] : 0ULL; }
    const bool mine16 = (word >> (j & 63)) & 1ULL;           // promoted for this lane's head
    const unsigned long long votes = __builtin_amdgcn_ballot_w64(mine16) & group_mask;
    const bool any16 = votes != 0ULL;
    const bool all16 = votes == group_mask;

    v16f s[2];
    if (!all16) {
      // ---- 4-bit scores straight from global memory ----
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const int key = key_of_row(r, t);
        const uint8_t* krow = k4base + ((size_t)j * kBk + key) * 64 + 16 * half;
        const v4i a0 = *reinterpret_cast<const v4i*>(krow);
        const v4i a1 = *reinterpret_cast<const v4i*>(krow + 32);
        const uint32_t ksw = *reinterpret_cast<const uint32_t*>(ksbase + ((size_t)j * kBk + key) * 4) >> (8 * half);
        v16f acc = {0.f};
        acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen(a0), widen(qf4[0]), acc, 4, 4, 0, ksw, 0, qsc);
        acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen(a1), widen(qf4[1]), acc, 4, 4, 2, ksw, 2, qsc);
        s[t] = acc;
      }
    }
    if (any16) {
      // ---- 16-bit scores; the V tile goes through this wavefront's LDS slice for the transposing reads ----
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const int chunk = lane + 64 * u, row = chunk >> 4, col = chunk & 15;
        *reinterpret_cast<uint4*>(lds + row * kRow16 + col * 16) =
            *reinterpret_cast<const uint4*>(v16base + ((size_t)j * kBk + row) * kD + col * 8);
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
    float gmax;
    const float alpha = softmax_update(s, lane, false, kBk, c, st, gmax);
    rescale(o, alpha);
    if (!all16) {
      // heads that took the 16-bit scores contribute nothing on the 4-bit path
      v16f p4[2] = {s[0], s[1]};
      float g4 = gmax;
      if (mine16) { p4[0] = (v16f){0.f}; p4[1] = (v16f){0.f}; g4 = 0.f; }
      // V fragments and scales straight from global memory
      const int vr = r * 32 + half * 16;
      const uint8_t* vt = v4base + (size_t)j * 4096 + vr;
      const uint8_t* vsr = vsbase + ((size_t)j * 2 + half) * kD + r;
      const uint32_t vsw = (uint32_t)vsr[0] | ((uint32_t)vsr[32] << 8) | ((uint32_t)vsr[64] << 16) | ((uint32_t)vsr[96] << 24);
      pv_fp4_regs(p4, g4, vsw, *reinterpret_cast<const v4i*>(vt), *reinterpret_cast<const v4i*>(vt + 1024),
                  *reinterpret_cast<const v4i*>(vt + 2048), *reinterpret_cast<const v4i*>(vt + 3072), o);
    }
    if (any16) {
      v16f p16[2] = {s[0], s[1]};
      if (!mine16) { p16[0] = (v16f){0.f}; p16[1] = (v16f){0.f}; }
      __builtin_amdgcn_wave_barrier();
      pv_16<T>(lds, lane, p16, o);
      __builtin_amdgcn_wave_barrier();
    }
  }

  // ---- partial (m, l, O) of this wavefront: accumulator i of tile n is channel 32n + 8(i/4) + 4*half + i%4 ----
  const float l = st.l + other_half(st.l);
  if (real) {
    const int pid = part * 4 + wave;
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

// Log-sum-exp merge of the partials of one (sequence, query head): 128 threads, one per channel.
__global__ void __launch_bounds__(128) decode_merge_kernel(DecodeArgs a) {
  const size_t qh = blockIdx.x;
  const int ch = threadIdx.x;
  const float c = a.scale * 1.4426950408889634f;
  const float* ml = a.part_ml + qh * a.nparts * 2;
  float M = -INFINITY;
  for (int p = 0; p < a.nparts; ++p) M = fmaxf(M, ml[2 * p]);
  float L = 0.f, O = 0.f;
  if (M > -INFINITY) {
    for (int p = 0; p < a.nparts; ++p) {
      const float m = ml[2 * p];
      if (m == -INFINITY) continue;
      const float w = fast_exp2((m - M) * c);
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
  if (a.dt == THRIFT_F16) decode_partial_kernel<F16><<<dim3(grid), dim3(256), 0, st>>>(a);
  else decode_partial_kernel<BF16><<<dim3(grid), dim3(256), 0, st>>>(a);
  decode_merge_kernel<<<dim3((unsigned)((long)a.B * a.Hq)), dim3(128), 0, st>>>(a);
}

}  // namespace thrift
