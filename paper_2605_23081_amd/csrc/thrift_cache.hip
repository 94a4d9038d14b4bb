// Maintenance of the dual MXFP4 / 16-bit KV cache the decode path reads (Sec. 4.1 and Sec. 5 of the paper
// describe the cache; how it is kept up to date is not spelled out there).
//
// Appending tokens must leave the cache exactly as the pre-pass (block means, MXFP4 quantisation) would
// build it from the longer sequence.  K is quantised along channels, so a new token's 4-bit row depends on
// nothing else.  V is quantised in groups of 32 consecutive tokens, and the group scale follows the
// largest magnitude of the tokens the group holds so far: a new token can change the scale and with it
// the codes of its group's earlier tokens, so the group is quantised again from the 16-bit rows.  The
// mean of a key block that is still filling up is the mean of the tokens it has.
//
// One workgroup per (sequence, KV head, key block that receives tokens): it stages the block's 64 x 128
// K and V tiles in LDS — rows already cached from the 16-bit cache, new rows from the caller's tensors,
// the rest zeros — writes the new 16-bit rows, the 4-bit K rows of the new tokens, the block's K mean,
// and both V groups of the block (a group without tokens becomes codes 0 with scale 2^0, so the whole
// block is always defined).
#include "thrift_device.h"
#include "thrift_launch.h"

namespace thrift {

template <typename T>
__global__ void __launch_bounds__(256) cache_append_kernel(CacheAppendArgs a) {
  constexpr int kRow = kD + 8;   // padded LDS row in 16-bit elements
  __shared__ __align__(16) uint16_t ktile[kBk * kRow];
  __shared__ __align__(16) uint16_t vtile[kBk * kRow];
  const int tid = threadIdx.x;
  const int slot = blockIdx.x % a.blocks_per_unit;            // which of the blocks this append can touch
  const int unit = blockIdx.x / a.blocks_per_unit;            // (sequence, KV head)
  const int b = unit / a.Hkv;
  const int len_old = min(a.Nkv, max(0, a.seqlens[b]));
  int n = a.new_lens ? min(a.n_new, max(0, a.new_lens[b])) : a.n_new;
  n = min(n, a.Nkv - len_old);                                // tokens past the capacity are dropped
  const int len_new = len_old + n;
  const int j = len_old / kBk + slot;                         // key block of this workgroup
  if (n <= 0 || j * kBk >= len_new) return;                   // uniform over the workgroup
  const int tok0 = j * kBk;
  const int count = min(kBk, len_new - tok0);                 // tokens the block holds after the append

  uint16_t* k16 = a.k16 + (size_t)unit * a.Nkv * kD;
  uint16_t* v16 = a.v16 + (size_t)unit * a.Nkv * kD;
  const uint16_t* knew = a.k_new + (size_t)unit * a.n_new * kD;
  const uint16_t* vnew = a.v_new + (size_t)unit * a.n_new * kD;

  // ---- stage both tiles; new rows also go to the 16-bit cache ----
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int chunk = tid + 256 * u;                          // 1024 chunks of 8 elements per tile
    const int row = chunk >> 4, col = (chunk & 15) * 8;
    const int tok = tok0 + row;
    uint4 kw = make_uint4(0, 0, 0, 0), vw = make_uint4(0, 0, 0, 0);
    if (tok < len_old) {
      kw = *reinterpret_cast<const uint4*>(k16 + (size_t)tok * kD + col);
      vw = *reinterpret_cast<const uint4*>(v16 + (size_t)tok * kD + col);
    } else if (tok < len_new) {
      kw = *reinterpret_cast<const uint4*>(knew + (size_t)(tok - len_old) * kD + col);
      vw = *reinterpret_cast<const uint4*>(vnew + (size_t)(tok - len_old) * kD + col);
      *reinterpret_cast<uint4*>(k16 + (size_t)tok * kD + col) = kw;
      *reinterpret_cast<uint4*>(v16 + (size_t)tok * kD + col) = vw;
    }
    *reinterpret_cast<uint4*>(&ktile[row * kRow + col]) = kw;
    *reinterpret_cast<uint4*>(&vtile[row * kRow + col]) = vw;
  }
  __syncthreads();

  // ---- K: 4-bit rows of the new tokens; thread = (row, group of 32 channels) ----
  {
    const int row = tid >> 2, g = tid & 3, tok = tok0 + row;
    if (tok >= len_old && tok < len_new) {
      uint32_t pair[16], out[4];
#pragma unroll
      for (int u = 0; u < 16; ++u) pair[u] = *reinterpret_cast<const uint32_t*>(&ktile[row * kRow + 32 * g + 2 * u]);
      const uint32_t sb = quantize_group32<T>(pair, out);
      *reinterpret_cast<uint4*>(a.k4 + ((size_t)unit * a.Nkv + tok) * (kD / 2) + 16 * g) = make_uint4(out[0], out[1], out[2], out[3]);
      a.ks[((size_t)unit * a.Nkv + tok) * (kD / 32) + g] = (uint8_t)sb;
    }
  }

  // ---- K mean of the block: fp64 sum of 16-bit values is exact, so the order of additions does not matter ----
  const size_t blk = (size_t)unit * (a.Nkv / kBk) + j;
  if (tid < kD) {
    double s = 0.0;
    for (int r = 0; r < count; ++r) s += (double)T::to_float(ktile[r * kRow + tid]);
    a.kmean[blk * kD + tid] = (float)(s / (double)count);
  }

  // ---- V: both 32-token groups of the block; thread = (group, channel) walks down a column ----
  {
    const int g = tid >> 7, c = tid & 127;
    uint32_t pair[16], out[4];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const uint32_t lo = vtile[(32 * g + 2 * u) * kRow + c], hi = vtile[(32 * g + 2 * u + 1) * kRow + c];
      pair[u] = lo | (hi << 16);
    }
    const uint32_t sb = quantize_group32<T>(pair, out);
    *reinterpret_cast<uint4*>(a.v4 + (blk * kD + c) * 32 + g * 16) = make_uint4(out[0], out[1], out[2], out[3]);
    a.vs[(blk * 2 + g) * kD + c] = (uint8_t)sb;
  }
}

void launch_cache_append(const CacheAppendArgs& a, thrift_dtype dt, hipStream_t st) {
  const unsigned grid = (unsigned)((long)a.B * a.Hkv * a.blocks_per_unit);
  if (dt == THRIFT_F16) cache_append_kernel<F16><<<dim3(grid), dim3(256), 0, st>>>(a);
  else cache_append_kernel<BF16><<<dim3(grid), dim3(256), 0, st>>>(a);
}

}  // namespace thrift
