// C ABI of the library: host-side validation, budget arithmetic and kernel dispatch.
// Nothing here allocates, frees or synchronises; on any error nothing is launched.
#include <math.h>
#include <string.h>

#include <mutex>

#include "thrift_launch.h"

using namespace thrift;

// Scratch of thrift_attn_decode_static: the decode workspace (score keys, selection bitmap, split-K partials) for
// callers that may not allocate.  One copy per GPU, held until the process ends.  In host code the array's name
// is only a handle; its device address on the current GPU comes from hipGetSymbolAddress, once per device.
constexpr size_t kStaticScratchBytes = (size_t)THRIFT_DECODE_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kHeadDim = 128;
constexpr int kKeyBlock = 64;
constexpr int kMaxKeyBlocks = 4096;

long long budget_ppm(double budget) { return llround(budget * 1e6); }

bool is16(thrift_dtype dt) { return dt == THRIFT_F16 || dt == THRIFT_BF16; }
bool is_out(thrift_dtype dt) { return dt == THRIFT_F16 || dt == THRIFT_BF16 || dt == THRIFT_F32; }

// gfx950 check, cached per device ordinal (read-mostly; a benign race writes the same value).
thrift_status check_arch() {
  static int cache[64] = {0};   // 0 unknown, 1 ok, 2 wrong
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return THRIFT_ERR_ARCH;
  if (dev >= 0 && dev < 64 && cache[dev] != 0) return cache[dev] == 1 ? THRIFT_OK : THRIFT_ERR_ARCH;
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return THRIFT_ERR_ARCH;
  const bool ok = strncmp(prop.gcnArchName, "gfx950", 6) == 0;
  if (dev >= 0 && dev < 64) cache[dev] = ok ? 1 : 2;
  return ok ? THRIFT_OK : THRIFT_ERR_ARCH;
}

thrift_status after_launch() { return hipGetLastError() == hipSuccess ? THRIFT_OK : THRIFT_ERR_LAUNCH; }

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// True when a, b, c are positive and a * b * c fits a 32-bit signed integer (grid sizes and row counts); the
// product is never formed when it could overflow.
bool fits_int(long a, long b, long c = 1) {
  const long lim = 0x7fffffffL;
  if (a <= 0 || b <= 0 || c <= 0 || a > lim || b > lim || c > lim) return false;
  if (a > lim / b) return false;
  return a * b <= lim / c;
}

constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void* scratch_address[kMaxDevices] = {nullptr};

// Device address of `scratch` on the current device (looked up on the first call per device, then cached).
thrift_status static_scratch(void** ptr) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return THRIFT_ERR_ARCH;
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (scratch_address[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
      (void)hipGetLastError();
      return THRIFT_ERR_LAUNCH;
    }
    scratch_address[dev] = p;
  }
  *ptr = scratch_address[dev];
  return THRIFT_OK;
}

struct DecodeLayout {
  size_t keys, bitmap, part_o, part_ml, order, total;
  int nsplit, nparts, words, order_items;
};

DecodeLayout decode_layout(int B, int Hq, int Hkv, int Nkv, int Bk, int split_blocks) {
  DecodeLayout L;
  const int Tk = Nkv / Bk;
  L.nsplit = (Tk + split_blocks - 1) / split_blocks;
  L.nparts = L.nsplit + 1;                       // one partial per partition + one for a partly filled last block
  L.words = (Tk + 63) / 64;
  size_t off = 0;
  L.keys = off; off += align256((size_t)B * Hq * Tk * sizeof(uint64_t));
  L.bitmap = off; off += align256((size_t)B * Hq * L.words * sizeof(unsigned long long));
  L.part_o = off; off += align256((size_t)B * Hq * L.nparts * kHeadDim * sizeof(float));
  L.part_ml = off; off += align256((size_t)B * Hq * L.nparts * 2 * sizeof(float));
  L.order_items = decode_order_items(B, Hkv, L.nsplit);
  L.order = off; off += align256((size_t)L.order_items * sizeof(int));
  L.total = off;
  return L;
}

// Workspace of the one-call form of Alg. 1: block means, selection, codes and scales of one problem.
struct FusedLayout {
  size_t qmean, kmean, idx, cnt, q4, qs, k4, ks, v4, vs, total;
  int Tq, Tk, kmax;
};

FusedLayout fused_layout(int B, int Hq, int Hkv, int N, int Bq, int Bk, int causal, double budget, int fixed_k) {
  FusedLayout L;
  L.Tq = (N + Bq - 1) / Bq;
  L.Tk = (N + Bk - 1) / Bk;
  const int need = thrift_select_kmax(L.Tq, L.Tk, Bq, Bk, causal, budget, fixed_k, 0);
  L.kmax = need > 0 ? need : 1;
  const size_t bq = (size_t)B * Hq, bk = (size_t)B * Hkv, n = (size_t)N, tv = (size_t)((N + 63) / 64);
  size_t off = 0;
  L.qmean = off; off += align256(bq * L.Tq * kHeadDim * sizeof(float));
  L.kmean = off; off += align256(bk * L.Tk * kHeadDim * sizeof(float));
  L.idx = off; off += align256(bq * L.Tq * L.kmax * sizeof(int32_t));
  L.cnt = off; off += align256(bq * L.Tq * sizeof(int32_t));
  L.q4 = off; off += align256(bq * n * (kHeadDim / 2));
  L.qs = off; off += align256(bq * n * (kHeadDim / 32));
  L.k4 = off; off += align256(bk * n * (kHeadDim / 2));
  L.ks = off; off += align256(bk * n * (kHeadDim / 32));
  L.v4 = off; off += align256(bk * tv * kHeadDim * 32);
  L.vs = off; off += align256(bk * tv * 2 * kHeadDim);
  L.total = off;
  return L;
}

}  // namespace

extern "C" {

const char* thrift_status_string(thrift_status s) {
  switch (s) {
    case THRIFT_OK: return "ok";
    case THRIFT_ERR_NULL: return "null pointer";
    case THRIFT_ERR_SHAPE: return "unsupported or inconsistent shape";
    case THRIFT_ERR_DTYPE: return "unknown dtype";
    case THRIFT_ERR_BUDGET: return "budget out of range or kmax too small";
    case THRIFT_ERR_WORKSPACE: return "workspace missing or too small";
    case THRIFT_ERR_ARCH: return "device is not gfx950";
    case THRIFT_ERR_LAUNCH: return "kernel launch failed";
  }
  return "unknown status";
}

int thrift_row_budget(int visible, double budget, int fixed_k) {
  if (visible < 0) visible = 0;
  if (fixed_k >= 0) return fixed_k < visible ? fixed_k : visible;
  const long long ppm = budget_ppm(budget);
  if (ppm <= 0) return 0;
  long long k = (ppm * (long long)visible + 999999LL) / 1000000LL;
  if (k < 1) k = 1;
  if (k > visible) k = visible;
  return (int)k;
}

int thrift_visible_blocks(int i, int Tk, int Bq, int Bk, int causal, int q_block_offset) {
  if (!causal) return Tk;
  const long long last_q = ((long long)i + q_block_offset + 1) * Bq - 1;
  long long v = last_q / Bk + 1;
  if (v > Tk) v = Tk;
  if (v < 0) v = 0;
  return (int)v;
}

int thrift_budget_to_global_k(int n, double fraction) {
  int best = 1;
  double bestd = INFINITY;
  for (int k = 1; k <= n; ++k) {
    const double frac = ((double)k * n - (double)k * (k - 1) / 2.0) / ((double)n * (n + 1) / 2.0);
    const double d = fabs(frac - fraction);
    if (d < bestd) { bestd = d; best = k; }
  }
  return best;
}

int thrift_select_kmax(int Tq, int Tk, int Bq, int Bk, int causal, double budget, int fixed_k, int q_block_offset) {
  // the row budget grows with the number of visible blocks, which grows with i
  int kmax = 0;
  if (Tq <= 0) return 0;
  const int v_last = thrift_visible_blocks(Tq - 1, Tk, Bq, Bk, causal, q_block_offset);
  const int v_first = thrift_visible_blocks(0, Tk, Bq, Bk, causal, q_block_offset);
  kmax = thrift_row_budget(v_last, budget, fixed_k);
  const int k0 = thrift_row_budget(v_first, budget, fixed_k);
  return kmax > k0 ? kmax : k0;
}

thrift_status thrift_block_means(const void* x, thrift_dtype dt, int B, int H, int N, int D, int block,
                                 float* means, void* stream) {
  if (!x || !means) return THRIFT_ERR_NULL;
  if (!is16(dt)) return THRIFT_ERR_DTYPE;
  if (B <= 0 || H <= 0 || N <= 0 || D != kHeadDim || block <= 0) return THRIFT_ERR_SHAPE;
  if (!fits_int(B, H, ((long)N + block - 1) / block)) return THRIFT_ERR_SHAPE;
  if (thrift_status s = check_arch()) return s;
  launch_block_means(x, dt, (long)B * H, N, block, means, (hipStream_t)stream);
  return after_launch();
}

static thrift_status select_topk_impl(const float* qmean, const float* kmean, int B, int Hq, int Hkv, int Tq, int Tk, int D,
                                      int Bq, int Bk, int causal, double budget, int fixed_k, int q_block_offset,
                                      int32_t* idx, int32_t* cnt, int kmax, int shared, void* stream) {
  if (!qmean || !kmean || !idx || !cnt) return THRIFT_ERR_NULL;
  if (B <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0 || Tq <= 0 || Tk <= 0 || Tk > kMaxKeyBlocks || D != kHeadDim ||
      Bq <= 0 || Bk <= 0 || q_block_offset < 0 || kmax <= 0)
    return THRIFT_ERR_SHAPE;
  if (fixed_k < 0 && !(budget >= 0.0 && budget <= 1.0)) return THRIFT_ERR_BUDGET;
  if (kmax < thrift_select_kmax(Tq, Tk, Bq, Bk, causal, budget, fixed_k, q_block_offset)) return THRIFT_ERR_BUDGET;
  if (!fits_int(B, Hq, Tq)) return THRIFT_ERR_SHAPE;                 // rows; the grid, one workgroup per 4 rows of a KV head, is smaller
  if (thrift_status s = check_arch()) return s;
  SelectArgs a;
  a.shared = shared;
  a.qmean = qmean; a.kmean = kmean; a.idx = idx; a.cnt = cnt;
  a.B = B; a.Hq = Hq; a.Hkv = Hkv; a.Tq = Tq; a.Tk = Tk; a.Bq = Bq; a.Bk = Bk; a.causal = causal ? 1 : 0;
  a.fixed_k = fixed_k; a.q_block_offset = q_block_offset; a.kmax = kmax; a.ppm = fixed_k >= 0 ? 0 : budget_ppm(budget);
  a.selector = 0; a.seed = 0;
  launch_select_topk(a, (hipStream_t)stream);
  return after_launch();
}

thrift_status thrift_select_topk(const float* qmean, const float* kmean, int B, int Hq, int Hkv, int Tq, int Tk, int D,
                                 int Bq, int Bk, int causal, double budget, int fixed_k, int q_block_offset,
                                 int32_t* idx, int32_t* cnt, int kmax, void* stream) {
  return select_topk_impl(qmean, kmean, B, Hq, Hkv, Tq, Tk, D, Bq, Bk, causal, budget, fixed_k, q_block_offset, idx, cnt, kmax, 0, stream);
}

thrift_status thrift_select_topk_shared(const float* qmean, const float* kmean, int B, int Hq, int Hkv, int Tq, int Tk, int D,
                                        int Bq, int Bk, int causal, double budget, int fixed_k, int q_block_offset,
                                        int32_t* idx, int32_t* cnt, int kmax, void* stream) {
  return select_topk_impl(qmean, kmean, B, Hq, Hkv, Tq, Tk, D, Bq, Bk, causal, budget, fixed_k, q_block_offset, idx, cnt, kmax, 1, stream);
}

thrift_status thrift_select_ablation(int selector, uint64_t seed, int B, int Hq, int Tq, int Tk, int Bq, int Bk,
                                     int causal, double budget, int fixed_k, int q_block_offset,
                                     int32_t* idx, int32_t* cnt, int kmax, void* stream) {
  if (!idx || !cnt) return THRIFT_ERR_NULL;
  if (selector != THRIFT_SELECT_RANDOM && selector != THRIFT_SELECT_DIAGONAL) return THRIFT_ERR_SHAPE;
  if (B <= 0 || Hq <= 0 || Tq <= 0 || Tk <= 0 || Tk > kMaxKeyBlocks || Bq <= 0 || Bk <= 0 || q_block_offset < 0 || kmax <= 0)
    return THRIFT_ERR_SHAPE;
  if (!fits_int(B, Hq, Tq)) return THRIFT_ERR_SHAPE;               // the row index is the high word of the random counter
  if (fixed_k < 0 && !(budget >= 0.0 && budget <= 1.0)) return THRIFT_ERR_BUDGET;
  if (kmax < thrift_select_kmax(Tq, Tk, Bq, Bk, causal, budget, fixed_k, q_block_offset)) return THRIFT_ERR_BUDGET;
  if (thrift_status s = check_arch()) return s;
  SelectArgs a;
  a.qmean = nullptr; a.kmean = nullptr; a.idx = idx; a.cnt = cnt;
  a.B = B; a.Hq = Hq; a.Hkv = Hq; a.Tq = Tq; a.Tk = Tk; a.Bq = Bq; a.Bk = Bk; a.causal = causal ? 1 : 0;   // no KV heads involved: one row group per head
  a.fixed_k = fixed_k; a.q_block_offset = q_block_offset; a.kmax = kmax; a.ppm = fixed_k >= 0 ? 0 : budget_ppm(budget);
  a.selector = selector; a.seed = seed; a.shared = 0;
  launch_select_topk(a, (hipStream_t)stream);
  return after_launch();
}

thrift_status thrift_quantize_mxfp4(const void* x, thrift_dtype dt, int B, int H, int N, int D, int axis,
                                    uint8_t* codes, uint8_t* scales, void* stream) {
  if (!x || !codes || !scales) return THRIFT_ERR_NULL;
  if (!is16(dt)) return THRIFT_ERR_DTYPE;
  if (B <= 0 || H <= 0 || N <= 0 || D != kHeadDim || (axis != 0 && axis != 1)) return THRIFT_ERR_SHAPE;
  // axis 1: one workgroup per 64-token block; axis 0: one thread per 32-group, 256 threads per workgroup
  if (!fits_int(B, H, ((long)N + 63) / 64)) return THRIFT_ERR_SHAPE;
  const long bh = (long)B * H;
  if (thrift_status s = check_arch()) return s;
  launch_quantize(x, dt, bh, N, axis, codes, scales, (hipStream_t)stream);
  return after_launch();
}

size_t thrift_attn_prefill_workspace(int, int, int, int, int, int, int, int) { return 0; }

thrift_status thrift_attn_prefill_ordered(const void* q, const void* k, const void* v, thrift_dtype dt,
                                          const uint8_t* q4, const uint8_t* qs, const uint8_t* k4, const uint8_t* ks,
                                          const uint8_t* v4, const uint8_t* vs,
                                          const int32_t* idx, const int32_t* cnt, int kmax,
                                          int B, int Hq, int Hkv, int Nq, int q_block_offset, int Nkv, int D, int Bq, int Bk,
                                          int causal, int tile_order, float softmax_scale,
                                          void* out, thrift_dtype out_dt, float* lse,
                                          void* workspace, size_t workspace_bytes, void* stream) {
  (void)workspace; (void)workspace_bytes;
  if (tile_order < 0 || tile_order > 4) return THRIFT_ERR_SHAPE;
  if (!q || !k || !v || !q4 || !qs || !k4 || !ks || !v4 || !vs || !idx || !cnt || !out) return THRIFT_ERR_NULL;
  if (!is16(dt) || !is_out(out_dt)) return THRIFT_ERR_DTYPE;
  if (B <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0 || Nq <= 0 || Nkv <= 0 || D != kHeadDim || Bk != kKeyBlock ||
      (Bq != 64 && Bq != 128) || kmax <= 0 || (Nkv + Bk - 1) / Bk > kMaxKeyBlocks || q_block_offset < 0)
    return THRIFT_ERR_SHAPE;
  // causal: the chunk must lie inside the sequence (its last query at or before the last key)
  if (causal && ((long)q_block_offset * Bq + Nq > (long)Nkv)) return THRIFT_ERR_SHAPE;
  if (!fits_int(B, Hq, (Nq + Bq - 1) / Bq)) return THRIFT_ERR_SHAPE;
  if (thrift_status s = check_arch()) return s;
  PrefillArgs a;
  a.q = (const uint16_t*)q; a.k = (const uint16_t*)k; a.v = (const uint16_t*)v;
  a.q4 = q4; a.qs = qs; a.k4 = k4; a.ks = ks; a.v4 = v4; a.vs = vs; a.idx = idx; a.cnt = cnt;
  a.out = out; a.lse = lse; a.kmax = kmax; a.B = B; a.Hq = Hq; a.Hkv = Hkv; a.N = Nkv; a.Bq = Bq; a.causal = causal ? 1 : 0;
  a.Nq = Nq; a.q_off = causal ? q_block_offset : 0; a.tile_order = tile_order;
  a.scale = softmax_scale > 0.f ? softmax_scale : 1.0f / sqrtf((float)D);
  a.dt = dt; a.out_dt = out_dt;
  launch_prefill(a, (hipStream_t)stream);
  return after_launch();
}

thrift_status thrift_attn_prefill_chunk(const void* q, const void* k, const void* v, thrift_dtype dt,
                                        const uint8_t* q4, const uint8_t* qs, const uint8_t* k4, const uint8_t* ks,
                                        const uint8_t* v4, const uint8_t* vs,
                                        const int32_t* idx, const int32_t* cnt, int kmax,
                                        int B, int Hq, int Hkv, int Nq, int q_block_offset, int Nkv, int D, int Bq, int Bk,
                                        int causal, float softmax_scale,
                                        void* out, thrift_dtype out_dt, float* lse,
                                        void* workspace, size_t workspace_bytes, void* stream) {
  return thrift_attn_prefill_ordered(q, k, v, dt, q4, qs, k4, ks, v4, vs, idx, cnt, kmax, B, Hq, Hkv, Nq, q_block_offset, Nkv, D,
                                     Bq, Bk, causal, 0, softmax_scale, out, out_dt, lse, workspace, workspace_bytes, stream);
}

thrift_status thrift_attn_prefill(const void* q, const void* k, const void* v, thrift_dtype dt,
                                  const uint8_t* q4, const uint8_t* qs, const uint8_t* k4, const uint8_t* ks,
                                  const uint8_t* v4, const uint8_t* vs,
                                  const int32_t* idx, const int32_t* cnt, int kmax,
                                  int B, int Hq, int Hkv, int N, int D, int Bq, int Bk, int causal, float softmax_scale,
                                  void* out, thrift_dtype out_dt, float* lse,
                                  void* workspace, size_t workspace_bytes, void* stream) {
  return thrift_attn_prefill_chunk(q, k, v, dt, q4, qs, k4, ks, v4, vs, idx, cnt, kmax, B, Hq, Hkv, N, 0, N, D, Bq, Bk, causal,
                                   softmax_scale, out, out_dt, lse, workspace, workspace_bytes, stream);
}

size_t thrift_attn_decode_workspace(int B, int Hq, int Hkv, int Nkv, int D, int Bk, int split_blocks) {
  if (B <= 0 || Hq <= 0 || Hkv <= 0 || Nkv <= 0 || D != kHeadDim || Bk != kKeyBlock || split_blocks <= 0 || Nkv % Bk != 0 ||
      Nkv / Bk > kMaxKeyBlocks || !fits_int(B, Hq, 64))
    return 0;
  return decode_layout(B, Hq, Hkv, Nkv, Bk, split_blocks).total;
}

static thrift_status attn_decode_impl(const void* q, thrift_dtype dt, const void* k16, const void* v16,
                                      const uint8_t* k4, const uint8_t* ks, const uint8_t* v4, const uint8_t* vs,
                                      const float* kmean, const int32_t* seqlens,
                                      int B, int Hq, int Hkv, int Nkv, int D, int Bk,
                                      double budget, int fixed_k, int split_blocks, float softmax_scale,
                                      void* out, thrift_dtype out_dt, int32_t* idx_out, int32_t* cnt_out, int kmax_out,
                                      void* workspace, size_t workspace_bytes, int shared, void* stream) {
  if (!q || !k16 || !v16 || !k4 || !ks || !v4 || !vs || !kmean || !out) return THRIFT_ERR_NULL;
  if (!is16(dt) || !is_out(out_dt)) return THRIFT_ERR_DTYPE;
  if (B <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0 || Hq / Hkv > 32 || Nkv <= 0 || D != kHeadDim || Bk != kKeyBlock ||
      Nkv % Bk != 0 || Nkv / Bk > kMaxKeyBlocks || split_blocks <= 0 || !fits_int(B, Hq, 64))
    return THRIFT_ERR_SHAPE;
  if (fixed_k < 0 && !(budget >= 0.0 && budget <= 1.0)) return THRIFT_ERR_BUDGET;
  const int Tk = Nkv / Bk;
  const int kneed = thrift_row_budget(Tk, budget, fixed_k);
  if (idx_out && (kmax_out < kneed || kmax_out <= 0)) return THRIFT_ERR_BUDGET;
  if (idx_out && !cnt_out) return THRIFT_ERR_NULL;
  const DecodeLayout L = decode_layout(B, Hq, Hkv, Nkv, Bk, split_blocks);
  if (!workspace) return THRIFT_ERR_WORKSPACE;
  if (workspace_bytes < L.total) return THRIFT_ERR_WORKSPACE;
  if (((uintptr_t)workspace & 15) != 0) return THRIFT_ERR_WORKSPACE;
  if (thrift_status s = check_arch()) return s;
  hipStream_t st = (hipStream_t)stream;
  char* ws = (char*)workspace;
  unsigned long long* bitmap = (unsigned long long*)(ws + L.bitmap);

  // (i) the query token is its own block mean; score it against the cached key-block means and select
  launch_decode_select((const uint16_t*)q, dt == THRIFT_BF16 ? 1 : 0, kmean, seqlens, (uint64_t*)(ws + L.keys), bitmap, L.words, idx_out, cnt_out, kmax_out,
                       B, Hq, Hkv, Tk, fixed_k, fixed_k >= 0 ? 0 : budget_ppm(budget), shared, st);

  // (ii) split-K partial attention, (iii) log-sum-exp merge
  DecodeArgs a;
  a.q = (const uint16_t*)q; a.k16 = (const uint16_t*)k16; a.v16 = (const uint16_t*)v16;
  a.k4 = k4; a.ks = ks; a.v4 = v4; a.vs = vs; a.seqlens = seqlens;
  a.bitmap = bitmap; a.bitmap_words = L.words;
  a.out = out; a.part_o = (float*)(ws + L.part_o); a.part_ml = (float*)(ws + L.part_ml);
  // heaviest-first launch order of the split-K workgroups; without promoted blocks and without lengths all items weigh the same
  a.order = (L.order_items > 0 && (kneed > 0 || seqlens != nullptr)) ? (int*)(ws + L.order) : nullptr;
  a.B = B; a.Hq = Hq; a.Hkv = Hkv; a.Nkv = Nkv; a.split_blocks = split_blocks; a.nsplit = L.nsplit; a.nparts = L.nparts; a.nmerge = seqlens ? L.nparts : L.nparts - 1;
  a.scale = softmax_scale > 0.f ? softmax_scale : 1.0f / sqrtf((float)D);
  a.dt = dt; a.out_dt = out_dt;
  launch_decode(a, st);
  return after_launch();
}

thrift_status thrift_attn_decode(const void* q, thrift_dtype dt, const void* k16, const void* v16,
                                 const uint8_t* k4, const uint8_t* ks, const uint8_t* v4, const uint8_t* vs,
                                 const float* kmean, const int32_t* seqlens,
                                 int B, int Hq, int Hkv, int Nkv, int D, int Bk,
                                 double budget, int fixed_k, int split_blocks, float softmax_scale,
                                 void* out, thrift_dtype out_dt, int32_t* idx_out, int32_t* cnt_out, int kmax_out,
                                 void* workspace, size_t workspace_bytes, void* stream) {
  return attn_decode_impl(q, dt, k16, v16, k4, ks, v4, vs, kmean, seqlens, B, Hq, Hkv, Nkv, D, Bk, budget, fixed_k, split_blocks,
                          softmax_scale, out, out_dt, idx_out, cnt_out, kmax_out, workspace, workspace_bytes, 0, stream);
}

thrift_status thrift_attn_decode_shared(const void* q, thrift_dtype dt, const void* k16, const void* v16,
                                        const uint8_t* k4, const uint8_t* ks, const uint8_t* v4, const uint8_t* vs,
                                        const float* kmean, const int32_t* seqlens,
                                        int B, int Hq, int Hkv, int Nkv, int D, int Bk,
                                        double budget, int fixed_k, int split_blocks, float softmax_scale,
                                        void* out, thrift_dtype out_dt, int32_t* idx_out, int32_t* cnt_out, int kmax_out,
                                        void* workspace, size_t workspace_bytes, void* stream) {
  return attn_decode_impl(q, dt, k16, v16, k4, ks, v4, vs, kmean, seqlens, B, Hq, Hkv, Nkv, D, Bk, budget, fixed_k, split_blocks,
                          softmax_scale, out, out_dt, idx_out, cnt_out, kmax_out, workspace, workspace_bytes, 1, stream);
}

thrift_status thrift_attn_decode_static(const void* q, thrift_dtype dt, const void* k16, const void* v16,
                                        const uint8_t* k4, const uint8_t* ks, const uint8_t* v4, const uint8_t* vs,
                                        const float* kmean, const int32_t* seqlens,
                                        int B, int Hq, int Hkv, int Nkv, int D, int Bk,
                                        double budget, int fixed_k, int split_blocks, float softmax_scale,
                                        void* out, thrift_dtype out_dt, int32_t* idx_out, int32_t* cnt_out, int kmax_out,
                                        void* stream) {
  // sizes first: a problem whose workspace does not fit the static array is refused before anything else happens
  const size_t need = thrift_attn_decode_workspace(B, Hq, Hkv, Nkv, D, Bk, split_blocks);
  if (need == 0) return THRIFT_ERR_SHAPE;
  if (need > kStaticScratchBytes) return THRIFT_ERR_WORKSPACE;
  void* ws = nullptr;
  if (thrift_status s = static_scratch(&ws)) return s;
  // Every byte of the workspace that the kernels read is written earlier in the same call (score keys and bitmap
  // words of the visible blocks, one partial per partition slot), so nothing has to be cleared between calls.
  return attn_decode_impl(q, dt, k16, v16, k4, ks, v4, vs, kmean, seqlens, B, Hq, Hkv, Nkv, D, Bk, budget, fixed_k, split_blocks,
                          softmax_scale, out, out_dt, idx_out, cnt_out, kmax_out, ws, kStaticScratchBytes, 0, stream);
}

static bool fused_shape_ok(int B, int Hq, int Hkv, int N, int D, int Bq, int Bk) {
  return B > 0 && Hq > 0 && Hkv > 0 && Hq % Hkv == 0 && N > 0 && D == kHeadDim && Bk == kKeyBlock && (Bq == 64 || Bq == 128) &&
         (N + Bk - 1) / Bk <= kMaxKeyBlocks && fits_int(B, Hq, (long)N / 64 + 1);
}

size_t thrift_attention_forward_workspace(int B, int Hq, int Hkv, int N, int D, int Bq, int Bk, int causal, double budget, int fixed_k) {
  if (!fused_shape_ok(B, Hq, Hkv, N, D, Bq, Bk)) return 0;
  if (fixed_k < 0 && !(budget >= 0.0 && budget <= 1.0)) return 0;
  return fused_layout(B, Hq, Hkv, N, Bq, Bk, causal, budget, fixed_k).total;
}

thrift_status thrift_attention_forward(const void* q, const void* k, const void* v, thrift_dtype dt,
                                       int B, int Hq, int Hkv, int N, int D, int Bq, int Bk, int causal,
                                       double budget, int fixed_k, int tile_order, float softmax_scale,
                                       void* out, thrift_dtype out_dt, float* lse,
                                       void* workspace, size_t workspace_bytes, void* stream) {
  if (!q || !k || !v || !out) return THRIFT_ERR_NULL;
  if (!is16(dt) || !is_out(out_dt)) return THRIFT_ERR_DTYPE;
  if (!fused_shape_ok(B, Hq, Hkv, N, D, Bq, Bk)) return THRIFT_ERR_SHAPE;
  if (tile_order < 0 || tile_order > 4) return THRIFT_ERR_SHAPE;          // before the first stage is enqueued
  if (fixed_k < 0 && !(budget >= 0.0 && budget <= 1.0)) return THRIFT_ERR_BUDGET;
  const FusedLayout L = fused_layout(B, Hq, Hkv, N, Bq, Bk, causal, budget, fixed_k);
  if (!workspace || workspace_bytes < L.total || ((uintptr_t)workspace & 255) != 0) return THRIFT_ERR_WORKSPACE;
  // the grid-size limits of the stages, so that none of them can refuse after an earlier one has been enqueued
  if (!fits_int(B, Hq, (long)N / 64 + 1) || !fits_int(B, Hkv, L.Tk)) return THRIFT_ERR_SHAPE;
  if (thrift_status s0 = check_arch()) return s0;
  char* ws = (char*)workspace;
  float* qmean = (float*)(ws + L.qmean);
  float* kmean = (float*)(ws + L.kmean);
  int32_t* idx = (int32_t*)(ws + L.idx);
  int32_t* cnt = (int32_t*)(ws + L.cnt);
  uint8_t *q4 = (uint8_t*)(ws + L.q4), *qs = (uint8_t*)(ws + L.qs), *k4 = (uint8_t*)(ws + L.k4), *ks = (uint8_t*)(ws + L.ks),
          *v4 = (uint8_t*)(ws + L.v4), *vs = (uint8_t*)(ws + L.vs);
  // every stage validates its own arguments again before it launches (the checks above cover all of them)
  thrift_status s;
  if ((s = thrift_block_means(q, dt, B, Hq, N, D, Bq, qmean, stream)) != THRIFT_OK) return s;                 // Alg. 1 step 3
  if ((s = thrift_block_means(k, dt, B, Hkv, N, D, Bk, kmean, stream)) != THRIFT_OK) return s;
  if ((s = thrift_select_topk(qmean, kmean, B, Hq, Hkv, L.Tq, L.Tk, D, Bq, Bk, causal, budget, fixed_k, 0, idx, cnt, L.kmax,
                              stream)) != THRIFT_OK) return s;                                                // step 5
  if ((s = thrift_quantize_mxfp4(q, dt, B, Hq, N, D, 0, q4, qs, stream)) != THRIFT_OK) return s;              // step 2
  if ((s = thrift_quantize_mxfp4(k, dt, B, Hkv, N, D, 0, k4, ks, stream)) != THRIFT_OK) return s;
  if ((s = thrift_quantize_mxfp4(v, dt, B, Hkv, N, D, 1, v4, vs, stream)) != THRIFT_OK) return s;
  return thrift_attn_prefill_ordered(q, k, v, dt, q4, qs, k4, ks, v4, vs, idx, cnt, L.kmax, B, Hq, Hkv, N, 0, N, D, Bq, Bk,   // steps 4-23
                                     causal, tile_order, softmax_scale, out, out_dt, lse, nullptr, 0, stream);
}

thrift_status thrift_kv_cache_append(const void* k_new, const void* v_new, thrift_dtype dt, int n_new,
                                     const int32_t* seqlens, const int32_t* new_lens,
                                     void* k16, void* v16, uint8_t* k4, uint8_t* ks, uint8_t* v4, uint8_t* vs, float* kmean,
                                     int B, int Hkv, int Nkv, int D, int Bk, void* stream) {
  if (!k_new || !v_new || !seqlens || !k16 || !v16 || !k4 || !ks || !v4 || !vs || !kmean) return THRIFT_ERR_NULL;
  if (!is16(dt)) return THRIFT_ERR_DTYPE;
  if (B <= 0 || Hkv <= 0 || Nkv <= 0 || n_new <= 0 || n_new > Nkv || D != kHeadDim || Bk != kKeyBlock || Nkv % Bk != 0 ||
      Nkv / Bk > kMaxKeyBlocks)
    return THRIFT_ERR_SHAPE;
  if (thrift_status s = check_arch()) return s;
  CacheAppendArgs a;
  a.k_new = (const uint16_t*)k_new; a.v_new = (const uint16_t*)v_new; a.seqlens = seqlens; a.new_lens = new_lens;
  a.k16 = (uint16_t*)k16; a.v16 = (uint16_t*)v16; a.k4 = k4; a.ks = ks; a.v4 = v4; a.vs = vs; a.kmean = kmean;
  a.B = B; a.Hkv = Hkv; a.Nkv = Nkv; a.n_new = n_new;
  // n tokens starting anywhere inside a block touch at most floor((63 + n - 1) / 64) + 1 blocks
  a.blocks_per_unit = (n_new + Bk - 2) / Bk + 1;
  launch_cache_append(a, dt, (hipStream_t)stream);
  return after_launch();
}

thrift_status thrift_peak_probe(int kind, thrift_dtype dt, int iters, void* buffer, size_t bytes, double* work, void* stream) {
  if (!buffer || !work) return THRIFT_ERR_NULL;
  if (kind < THRIFT_PEAK_MFMA_MXFP4 || kind > THRIFT_PEAK_TILE_MIX || iters < 1 || bytes < ((size_t)16 << 20)) return THRIFT_ERR_SHAPE;
  if (kind == THRIFT_PEAK_MFMA_16 && !is16(dt)) return THRIFT_ERR_DTYPE;
  if (((uintptr_t)buffer & 15) != 0) return THRIFT_ERR_SHAPE;
  if (thrift_status s = check_arch()) return s;
  *work = launch_peak_probe(kind, dt, iters, buffer, bytes, (hipStream_t)stream);
  if (*work < 0.0) return THRIFT_ERR_SHAPE;               // a buffer the probe cannot cover in one launch: nothing was launched
  return after_launch();
}

}  // extern "C"
