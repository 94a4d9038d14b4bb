// Fused mixed-precision flash attention for prefill (Algorithm 1 steps 4-23; Sec. 3.3).
//
// One workgroup = one (batch, query head, query block); wavefront w owns query rows 32w .. 32w+31 of
// the block and keeps Q, the online-softmax state and the O^T accumulators in registers.  Two walks over
// the key blocks are built, both dispatching per tile to the scaled-FP4 or the 16-bit MFMA path:
//   ORDER 0  ascending block order, Alg. 1 as written (a second staging schedule, WIDE, serves high budgets);
//   ORDER 1  the order of the kernel in Sec. 3.3: every 4-bit block first, then the promoted blocks with the
//            16-bit query fragments in registers only for that phase.  This is the benchmarked walk.
//
// The kernel is bound by the vector ALU work of the softmax and the P quantiser (exp and the FP4
// converter run at a quarter of the plain rate), and one wavefront can issue vector instructions at only
// about half the rate its SIMD can execute them.  Everything is therefore sized for THREE workgroups per
// CU (three wavefronts per SIMD): at most 168 vector registers and a third of the LDS per workgroup.
//   * Every block is staged once into LDS for all wavefronts by LDS DMA (global loads that write LDS
//     directly: no staging registers, no LDS write instructions), one block ahead of the arithmetic:
//     MXFP4 codes + scales into one of two 8.5 KiB slots, the 16-bit K and V tiles of a block listed in
//     the row's TopK set into 16 KiB tile buffers.
//   * One workgroup barrier per 4-bit key block orders the traffic, two per promoted block.
//
// Differences from the kernel the paper sketches for Blackwell (Sec. 3.3): MXFP4 instead of NVFP4, 32x32
// MFMA tiles in transposed form (one query per lane column) instead of warp-level MMA tiles, LDS regions
// per precision instead of one aliased region (three workgroups per CU are worth more than the aliasing).
#include <type_traits>

#include "thrift_launch.h"
#include "thrift_tile.h"

namespace thrift {

// LDS map of the prefill kernel (bytes)
constexpr int kLdsRing = 0;                                  // two slots of kLdsBytes4 (block j -> slot j & 1)
constexpr int kLdsV16 = 2 * kLdsBytes4;                      // one swizzled 16-bit V tile
constexpr int kLdsK16 = kLdsV16 + kTile16;                   // one swizzled 16-bit K tile
constexpr int kLdsPrefill = kLdsK16 + kTile16;               // 50176: three workgroups per CU
// LDS map of the wide schedule: two slots that hold one key block each, whatever its path
// (a 4-bit block in the first kLdsBytes4 bytes; a promoted block as its K tile followed by its V tile)
constexpr int kWideSlot = 2 * kTile16;                       // 32768
constexpr int kLdsPrefillWide = 2 * kWideSlot;               // 65536: two workgroups per CU
constexpr int kWidePercent = 15;                             // list length / key blocks (in %) from which the wide schedule is used

// One work item: a (sequence, query head, query block) and all its key blocks.  `work` is the item's position in the
// launch order (what blockIdx.x is in the one-item-per-workgroup launch).
template <typename T, int NW, int ORDER, int WIDE>
__device__ __forceinline__ void prefill_item(const PrefillArgs& a, unsigned char* lds, unsigned work) {
  constexpr int KF = 4 / NW;                 // 1 KiB fragments of a 4-bit K (and of a V) tile per wavefront
  constexpr int C16 = 16 / NW;               // ... for one 16-bit K or V tile
  constexpr int kSlotStride = WIDE ? kWideSlot : kLdsBytes4;

  const int tid = threadIdx.x, lane = tid & 63, half = lane >> 5, r = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wavefront-uniform: loop bounds stay scalar
  const int N = a.N, Nq = a.Nq, Bq = NW * 32, G = a.Hq / a.Hkv;
  const int Tq = (Nq + Bq - 1) / Bq, Tk = (N + kBk - 1) / kBk;   // the last query / key block may be short

  // ---- work item: heavy (late) query blocks first; KV heads spread over the 8 XCDs so that the query
  // heads and neighbouring query blocks that share a KV head also share an L2 ----
  const int units = a.B * a.Hkv, per_unit = G * Tq;
  int unit, within;
  if ((units & 7) == 0) {
    const int xcd = work & 7, t = work >> 3;
    unit = xcd + 8 * (t / per_unit);
    within = t % per_unit;
  } else {
    unit = work / per_unit;
    within = work % per_unit;
  }
  const int b = unit / a.Hkv, kvh = unit % a.Hkv;
  const int i = Tq - 1 - within / G;
  const int hq = kvh * G + within % G;
  const size_t qh = (size_t)b * a.Hq + hq, kh = (size_t)b * a.Hkv + kvh;
  const int q0 = (i + a.q_off) * Bq + wave * 32;        // sequence position of this wavefront's first query row
  // The lane's query row inside the head.  Rows past the last query repeat it and are never stored.  Only this
  // 32-bit index is kept; addresses are rebuilt from it and scalar bases where they are needed (registers are
  // what limits this kernel to three wavefronts per SIMD).
  const int lrow = min(i * Bq + wave * 32 + r, Nq - 1);
  const size_t qrow = qh * Nq + lrow;

  // ---- Q fragments ----
  v4i qf4[2];
  // fragment kk: d-group 2*half + kk (scores_fp4); its scale is byte kk of qsc
  qf4[0] = *reinterpret_cast<const v4i*>(a.q4 + qrow * 64 + half * 32);
  qf4[1] = *reinterpret_cast<const v4i*>(a.q4 + qrow * 64 + half * 32 + 16);
  const uint32_t qsc = *reinterpret_cast<const uint32_t*>(a.qs + qrow * 4) >> (16 * half);
  const uint8_t* q16head = reinterpret_cast<const uint8_t*>(a.q + qh * Nq * kD);   // wavefront-uniform

  const int vis = a.causal ? min(Tk, ((i + a.q_off + 1) * Bq - 1) / kBk + 1) : Tk;
  const int32_t* sel = a.idx + (qh * Tq + i) * a.kmax;
  const int nsel = min(a.cnt[qh * Tq + i], a.kmax);      // a count beyond the list length is cut, never followed
  // Entry t of the row's list, through the scalar data path.  The list index is wavefront-uniform, but the compiler
  // cannot prove that (it depends on list entries read earlier) nor that the list is not written here, and turns a
  // plain read into a vector load plus a wait for EVERY vector load in flight, the tile DMAs included.
  auto sel_at = [&](int t) -> int {
    const int32_t* p = sel + __builtin_amdgcn_readfirstlane(t);
    int v;
    asm volatile("s_load_dword %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(p) : "memory");
    return min(max(v, 0), Tk - 1);                      // whatever the list holds, only ids of existing key blocks become addresses
  };
  // the next two promoted block ids at or after the current block (ascending list)
  int ps = 0;
  int n0 = nsel > 0 ? sel_at(0) : 0x7fffffff, n1 = nsel > 1 ? sel_at(1) : 0x7fffffff;

  const uint8_t* k4base = a.k4 + kh * N * 64;
  const uint8_t* v4base = a.v4 + kh * (size_t)Tk * 4096;
  const uint8_t* ksbase = a.ks + kh * N * 4;
  const uint8_t* vsbase = a.vs + kh * (size_t)Tk * 2 * kD;
  const uint8_t* k16base = reinterpret_cast<const uint8_t*>(a.k + kh * N * kD);
  const uint8_t* v16base = reinterpret_cast<const uint8_t*>(a.v + kh * N * kD);

  // ---- staging: per-lane source offsets of the DMA instructions this wavefront issues.  The LDS side of
  // a DMA is linear in the lane index, so every layout change (MFMA fragment order of the 4-bit tiles,
  // chunk swizzle of the 16-bit tiles) is expressed in the global offsets. ----
  const uint32_t lds0 = lds_address(lds);
  uint32_t k4off[KF], v4off[KF];
#pragma unroll
  for (int u = 0; u < KF; ++u) {
    const int f = wave * KF + u;                         // K: fragment (t, kk) = (f>>1, f&1); V: channels 32f .. 32f+31
    k4off[u] = (uint32_t)(key_of_row(r, f >> 1) * 64 + (2 * half + (f & 1)) * 16);    // d-group 2*half + kk of the key
    v4off[u] = (uint32_t)((32 * f + r) * 32 + half * 16);
  }
  const uint32_t scoff = (uint32_t)lane * 4;
  // the 256 scale bytes of K ride with the even wavefronts, V's with the odd ones: picked once, in scalar registers
  const bool v_scales = (wave & 1) != 0;
  const uint8_t* scbase = v_scales ? vsbase : ksbase;
  const uint32_t sclds = v_scales ? (uint32_t)kLdsVS : (uint32_t)kLdsKS;
  // 16-bit tiles: one instruction covers 4 rows; lane l writes chunk position l&15 of row l>>4
  // (formed from the lane index where a 16-bit tile is issued, one block in twenty on the headline budget,
  // rather than held in registers through every 4-bit block)
#define THRIFT_V16OFF() ((uint32_t)((lane16 >> 4) * 256 + ((lane16 & 15) ^ v16_swizzle(lane16 >> 4)) * 16))
#define THRIFT_K16OFF() ((uint32_t)((lane16 >> 4) * 256 + ((lane16 & 15) ^ (lane16 >> 4)) * 16))   /* rows 32..63: chunk ^ 4 more */

  // A short last key block: the rows past the last key do not exist in the row-major arrays (K codes and
  // scales, 16-bit K and V); their lanes re-read the last key's row instead, and the mask below keeps
  // whatever lands there out of the arithmetic.  (V codes and scales are stored in whole, zero-padded blocks.)
  // The clamped offsets are formed inside the branch that handles the short block (the empty asm keeps the
  // compiler from hoisting a second set of per-lane offsets out of the key loop, which would cost registers
  // on the path every other block takes).
  const int last_key_row = (N - 1) & (kBk - 1);
#define THRIFT_CLAMP_ROWS(OFF, SHIFT, LAST) ((min((uint32_t)(OFF) >> (SHIFT), (LAST)) << (SHIFT)) | ((OFF) & ((1u << (SHIFT)) - 1u)))
#define THRIFT_ISSUE4(J) THRIFT_ISSUE4_SLOT(J, (J) & 1)
#define THRIFT_ISSUE4_SLOT(J, S)                                                                               \
  do {                                                                                                         \
    const int j_ = __builtin_amdgcn_readfirstlane(J), s_ = __builtin_amdgcn_readfirstlane(S); /* scalar operands */ \
    const uint8_t* kt_ = k4base + (size_t)j_ * 4096;                                                           \
    const uint8_t* vt_ = v4base + (size_t)j_ * 4096;                                                           \
    int wave_ = wave;                                                                                          \
    asm volatile("" : "+s"(wave_));   /* LDS destinations are formed here from one scalar, not kept per slot and fragment */ \
    const uint32_t sl_ = lds0 + kLdsRing + s_ * kSlotStride + (uint32_t)(wave_ * (KF * 1024));                 \
    if ((j_ + 1) * kBk <= N) {                                                                                 \
      _Pragma("unroll") for (int u = 0; u < KF; ++u) dma_b128(kt_, k4off[u], sl_ + kLdsK4 + u * 1024); \
      dma_b32(scbase + (size_t)j_ * 256, scoff, sl_ - (uint32_t)(wave_ * (KF * 1024)) + sclds);                                                  \
    } else {                                                                                                   \
      uint32_t last_ = (uint32_t)last_key_row;                                                                 \
      asm volatile("" : "+s"(last_));                                                                          \
      _Pragma("unroll") for (int u = 0; u < KF; ++u)                                                           \
        dma_b128(kt_, THRIFT_CLAMP_ROWS(k4off[u], 6, last_), sl_ + kLdsK4 + u * 1024);                         \
      /* V scales are stored in whole, zero-padded blocks; K's rows past the last key do not exist */          \
      dma_b32(scbase + (size_t)j_ * 256, v_scales ? scoff : THRIFT_CLAMP_ROWS(scoff, 2, last_),                \
              sl_ - (uint32_t)(wave_ * (KF * 1024)) + sclds);                                                  \
    }                                                                                                          \
    /* V codes: whole blocks */                                                                                \
    _Pragma("unroll") for (int u = 0; u < KF; ++u) dma_b128(vt_, v4off[u], sl_ + kLdsV4 + u * 1024); \
  } while (0)
  // 16-bit tiles: instruction q_ covers rows 4 q_ .. 4 q_ + 3
#define THRIFT_ISSUE_TILE16(BASE, J, OFFEXPR, LDSBASE)                                                         \
  do {                                                                                                         \
    const int j_ = __builtin_amdgcn_readfirstlane(J);                                                          \
    const uint8_t* t_ = (BASE) + (size_t)j_ * kTile16;                                                         \
    int lane16 = lane, wave_ = wave;                                                                           \
    asm volatile("" : "+v"(lane16), "+s"(wave_));   /* offsets and destinations are computed here, not carried through the key loop */ \
    if ((j_ + 1) * kBk <= N) {                                                                                 \
      _Pragma("unroll") for (int u = 0; u < C16; ++u) {                                                        \
        const int q_ = u * NW + wave_;                                                                         \
        dma_b128(t_ + q_ * 1024, (OFFEXPR), (LDSBASE) + q_ * 1024);                                            \
      }                                                                                                        \
    } else {                                                                                                   \
      uint32_t last_ = (uint32_t)last_key_row;                                                                 \
      asm volatile("" : "+s"(last_));                                                                          \
      _Pragma("unroll") for (int u = 0; u < C16; ++u) {                                                        \
        const int q_ = u * NW + wave_;                                                                         \
        const uint32_t o_ = (uint32_t)(q_ * 1024) + (OFFEXPR);   /* offset from the tile start */              \
        dma_b128(t_, THRIFT_CLAMP_ROWS(o_, 8, last_), (LDSBASE) + q_ * 1024);                                  \
      }                                                                                                        \
    }                                                                                                          \
  } while (0)
#define THRIFT_ISSUE_V16(J) THRIFT_ISSUE_TILE16(v16base, J, THRIFT_V16OFF(), lds0 + kLdsV16)
#define THRIFT_ISSUE_K16(J) THRIFT_ISSUE_TILE16(k16base, J, (u * NW >= 8 ? THRIFT_K16OFF() ^ 64u : THRIFT_K16OFF()), lds0 + kLdsK16)

  RowState st = {kEmptyMax, 0.f};
  v16f o[4];
#pragma unroll
  for (int n = 0; n < 4; ++n) o[n] = (v16f){0.f};
  const float c = a.scale * 1.4426950408889634f;

  // Blocks this wavefront computes: those with at least one key at or before its last query row.  The
  // later blocks of the workgroup (visible only to wavefronts with later rows) are still staged and
  // synchronised on, in a final loop without arithmetic.
  const int vis_wave = a.causal ? min(vis, (q0 + 31) / kBk + 1) : vis;
  // keys at positions below key_limit are visible to the lane's query: those at or before its own position
  // (causal) and only keys that exist
  const int key_limit = a.causal ? min(q0 + r + 1, N) : N;

  // One step of the staging pipeline at block J, with P0 / P1 = "block J / J+1 is promoted".
  //  SYNC:  wait for this wavefront's share of block J, then meet the others: block J is complete in LDS
  //         and everyone has finished block J-1 (whose buffers are free again).
  //  ISSUE: block J+1 — a 4-bit block into the other slot; a promoted block into the 16-bit buffers,
  //         unless block J is using them (then its K tile follows the score phase of block J and its V
  //         tile the start of step J+1: late_v).
  bool late_v = false;                                  // block J is promoted and its V tile is not issued yet
#define THRIFT_SYNC()                                                                                          \
  vm_wait<0>();                                                                                                \
  lds_barrier();
#define THRIFT_ISSUE(J, P0, P1)                                                                                \
  if ((J) + 1 < vis) {                                                                                         \
    if (!(P1)) {                                                                                               \
      THRIFT_ISSUE4((J) + 1);                                                                                  \
    } else if (!(P0)) {                                                                                        \
      THRIFT_ISSUE_K16((J) + 1);                                                                               \
      THRIFT_ISSUE_V16((J) + 1);                                                                               \
    }                                                                                                          \
  }
#define THRIFT_MASK(J)                                                                                         \
  const bool mask = (a.causal && (J) * kBk + kBk - 1 > q0) || ((J) + 1) * kBk > N;                             \
  const int n_valid = key_limit - (J) * kBk;   /* leading keys of the block this query may see */
#define THRIFT_NEXT_PROMOTED()                                                                                 \
  ++ps;                                                                                                        \
  n0 = n1;                                                                                                     \
  n1 = ps + 1 < nsel ? sel_at(ps + 1) : 0x7fffffff;
  // List entries behind the walk's position (a list that is not strictly ascending breaks the contract) are
  // dropped, at the same point of every wavefront's walk: the wavefronts of a workgroup must take identical
  // staging and barrier decisions whatever the list holds.
#define THRIFT_DROP_STALE(J)                                                                                   \
  while (n0 < (J)) { THRIFT_NEXT_PROMOTED() }

  // 16-bit query fragments of the lane's row (the wide schedule keeps them in registers for the whole walk; the
  // three-workgroup schedule has no registers to spare and fetches them again at every promoted block)
#define THRIFT_LOAD_Q16_ROW(QF, LROW)                                                                          \
  _Pragma("unroll") for (int s8 = 0; s8 < 8; ++s8)                                                             \
    QF[s8] = *reinterpret_cast<const v8s*>(q16head + (uint32_t)((LROW) * (2 * kD) + 32 * s8 + 16 * half));     \
  _Pragma("unroll") for (int s8 = 0; s8 < 8; ++s8) asm volatile("" : "+v"(QF[s8]));
#define THRIFT_LOAD_Q16(QF) THRIFT_LOAD_Q16_ROW(QF, lrow)
  // The lane's row index formed again from the thread id (the empty asm hides it from common-subexpression
  // elimination): used where keeping the first copy alive through a long loop would cost a register there.
#define THRIFT_ROW_AGAIN(UNCLAMPED)                                                                            \
  int UNCLAMPED = (int)(threadIdx.x & 31);                                                                     \
  asm volatile("" : "+v"(UNCLAMPED));                                                                          \
  UNCLAMPED += i * Bq + wave * 32;

  if constexpr (WIDE) {
    // ---- wide schedule: every block, 4-bit or promoted, is fetched one whole step ahead into the slot the
    // block before last has left; one barrier per key block, no second rendezvous for promoted blocks ----
#define THRIFT_ISSUE_WIDE(J1, P1)                                                                              \
  if ((J1) < vis) {                                                                                            \
    if (P1) {                                                                                                  \
      THRIFT_ISSUE_TILE16(k16base, J1, (u * NW >= 8 ? THRIFT_K16OFF() ^ 64u : THRIFT_K16OFF()),                \
                          lds0 + (uint32_t)(((J1) & 1) * kWideSlot));                                          \
      THRIFT_ISSUE_TILE16(v16base, J1, THRIFT_V16OFF(), lds0 + (uint32_t)(((J1) & 1) * kWideSlot + kTile16));  \
    } else {                                                                                                   \
      THRIFT_ISSUE4(J1);                                                                                       \
    }                                                                                                          \
  }
    // the 16-bit query fragments stay in registers (this schedule has 256 of them)
    v8s qf[8];
    THRIFT_LOAD_Q16(qf)
    if (vis > 0) { THRIFT_ISSUE_WIDE(0, n0 == 0) }
    int j = 0;
    while (j < vis_wave) {
      THRIFT_DROP_STALE(j)
      const int run_end = min(vis_wave, n0);
      for (; j < run_end; ++j) {                          // a run of 4-bit blocks
        THRIFT_SYNC()
        THRIFT_ISSUE_WIDE(j + 1, j + 1 == n0)
        THRIFT_MASK(j)
        const unsigned char* slot = lds + (j & 1) * kWideSlot;
        v16f s[2];
        float alpha;
        uint32_t pb;
        scores_fp4(slot, lane, qf4, qsc, s);
        const bool grew = softmax_update(s, lane, mask, n_valid, c, st, alpha, pb);
        rescale(o, grew, alpha);
        pv_fp4(slot, lane, s, pb, o);
      }
      if (j < vis_wave) {                                 // j == n0: a promoted block
        THRIFT_SYNC()
        THRIFT_ISSUE_WIDE(j + 1, j + 1 == n1)
        THRIFT_MASK(j)
        const unsigned char* slot = lds + (j & 1) * kWideSlot;
        v16f s[2];
        scores_16<T>(slot, lane, qf, s);
        float alpha;
        uint32_t pb;
        const bool grew = softmax_update(s, lane, mask, n_valid, c, st, alpha, pb);
        rescale(o, grew, alpha);
        pv_16<T, true>(slot + kTile16, lane, s, o);
        THRIFT_NEXT_PROMOTED()
        ++j;
      }
    }
    for (; j < vis; ++j) {                                // staging only: blocks that later wavefronts still need
      THRIFT_DROP_STALE(j)
      const bool p0 = j == n0;
      THRIFT_SYNC()
      THRIFT_ISSUE_WIDE(j + 1, j + 1 == (p0 ? n1 : n0))
      if (p0) { THRIFT_NEXT_PROMOTED() }
    }
#undef THRIFT_ISSUE_WIDE
  } else if constexpr (ORDER == 1) {
    // ---- the order of Sec. 3.3: every 4-bit block in ascending order, then the promoted blocks in ascending
    // order.  Same staging rules; the ring slot follows the step number because block ids now skip. ----
    int nselv = nsel;                                   // promoted ids inside the visible range (the list is ascending)
    if (nsel > 0 && sel_at(nsel - 1) >= vis) {
      nselv = 0;
      while (nselv < nsel && sel_at(nselv) < vis) ++nselv;
    }
    int pa = 0;                                         // promoted ids the 4-bit walk has passed
    const int first_promoted = nselv > 0 ? sel_at(0) : 0x7fffffff;
    int nx = first_promoted;                            // the next promoted id at or after the 4-bit walk's position
    int j = 0;
    while (j == nx) { ++j; ++pa; nx = pa < nselv ? sel_at(pa) : 0x7fffffff; }
    if (j < vis) {
      THRIFT_ISSUE4_SLOT(j, 0);
    } else if (nselv > 0) {
      THRIFT_ISSUE_K16(first_promoted);
      THRIFT_ISSUE_V16(first_promoted);
    }
    // Phase A, two steps per trip so that the ring slot of each step is a compile-time constant: every LDS
    // read of the step is then a lane-constant address register plus an immediate offset, no address arithmetic.
    auto step_a = [&](auto slot_c) __attribute__((always_inline)) {
      constexpr int SLOT = decltype(slot_c)::value;
      int jn = j + 1;
      while (jn == nx) { ++jn; ++pa; nx = pa < nselv ? sel_at(pa) : 0x7fffffff; }
      THRIFT_SYNC()
      if (jn < vis) {
        THRIFT_ISSUE4_SLOT(jn, SLOT ^ 1);
      } else if (nselv > 0) {
        THRIFT_ISSUE_K16(first_promoted);
        THRIFT_ISSUE_V16(first_promoted);
      }
      if (j < vis_wave) {
        THRIFT_MASK(j)
        const unsigned char* slot = lds + kLdsRing + SLOT * kLdsBytes4;
        v16f s[2];
        float alpha;
        uint32_t pb;
        scores_fp4(slot, lane, qf4, qsc, s);
        const bool grew = softmax_update(s, lane, mask, n_valid, c, st, alpha, pb);
        rescale(o, grew, alpha);
        pv_fp4(slot, lane, s, pb, o);
      }
      j = jn;
    };
    while (j < vis) {                                   // phase A
      step_a(std::integral_constant<int, 0>{});
      if (j >= vis) break;
      step_a(std::integral_constant<int, 1>{});
    }
    // phase B: the promoted blocks follow each other.  The lane's 16-bit query fragments are fetched once and stay
    // in registers for the whole phase (the 4-bit phase, which has no registers to spare, is over: Sec. 3.3 scopes
    // them the same way).  The 4-bit slots are idle now, so the 16-bit tiles rotate through THREE 16 KiB buffers in
    // the order they are consumed, K(b), V(b), K(b+1), ...: tile t sits in buffer t mod 3 and may be fetched as
    // soon as everyone has finished with tile t-3.  That puts K(b+1) in flight at the start of block b and V(b+1)
    // right after the scores of block b, half a block earlier each than two fixed buffers allow.
    v8s qf[8];
    if (nselv > 0 && first_promoted < vis_wave) {
      THRIFT_ROW_AGAIN(row_b)
      THRIFT_LOAD_Q16_ROW(qf, min(row_b, Nq - 1))
    }
    // buffer 0: the K region (holds K of the first promoted block), 1: the V region (its V), 2: the 4-bit slots' region
#define THRIFT_TILE_BUFFER(X) ((X) == 0 ? kLdsK16 : (X) == 1 ? kLdsV16 : kLdsRing)
    int kbuf = 0;
    int jb_next = first_promoted;
    for (int sidx = 0; sidx < nselv; ++sidx) {
      const int jb = jb_next;
      const bool p1 = sidx + 1 < nselv;
      if (p1) jb_next = sel_at(sidx + 1);
      const bool mine = jb < vis_wave;
      const int vbuf = kbuf == 2 ? 0 : kbuf + 1;
      const int kbuf_next = vbuf == 2 ? 0 : vbuf + 1;
      vm_wait<C16>();                                   // this wavefront's share of K(b); V(b) may still be on its way
      lds_barrier();                                    // K(b) complete; everyone has finished the block before
      if (p1) {
        THRIFT_ISSUE_TILE16(k16base, jb_next, (u * NW >= 8 ? THRIFT_K16OFF() ^ 64u : THRIFT_K16OFF()),
                            lds0 + (uint32_t)THRIFT_TILE_BUFFER(kbuf_next));
      }
      THRIFT_MASK(jb)
      v16f s[2];
      if (mine) scores_16<T>(lds + THRIFT_TILE_BUFFER(kbuf), lane, qf, s);
      if (p1) vm_wait<C16>();                           // V(b); K(b+1) may still be on its way
      else vm_wait<0>();
      lds_barrier();                                    // V(b) complete; everyone has its scores, K(b)'s buffer is free
      if (p1) { THRIFT_ISSUE_TILE16(v16base, jb_next, THRIFT_V16OFF(), lds0 + (uint32_t)THRIFT_TILE_BUFFER(kbuf)); }
      if (mine) {
        float alpha;
        uint32_t pb;
        const bool grew = softmax_update(s, lane, mask, n_valid, c, st, alpha, pb);
        rescale(o, grew, alpha);
        pv_16<T, true>(lds + THRIFT_TILE_BUFFER(vbuf), lane, s, o);
      }
      kbuf = kbuf_next;
    }
#undef THRIFT_TILE_BUFFER
  } else {
  // prologue: block 0 on its way
  if (vis > 0) {
    if (n0 == 0) {
      THRIFT_ISSUE_K16(0);
      THRIFT_ISSUE_V16(0);
    } else {
      THRIFT_ISSUE4(0);
    }
  }
  // The walk alternates between runs of 4-bit blocks (tight loop: only the scaled-FP4 path, accumulators
  // updated in place) and single promoted blocks.
  int j = 0;
  while (j < vis_wave) {
    THRIFT_DROP_STALE(j)
    const int run_end = min(vis_wave, n0);
    for (; j < run_end; ++j) {
      THRIFT_SYNC()
      THRIFT_ISSUE(j, false, j + 1 == n0)
      THRIFT_MASK(j)
      const unsigned char* slot = lds + kLdsRing + (j & 1) * kLdsBytes4;
      v16f s[2];
      float alpha;
      uint32_t pb;
      scores_fp4(slot, lane, qf4, qsc, s);
      const bool grew = softmax_update(s, lane, mask, n_valid, c, st, alpha, pb);
      rescale(o, grew, alpha);
      pv_fp4(slot, lane, s, pb, o);
      late_v = false;
    }
    if (j < vis_wave) {                                 // j == n0: a promoted block
      const bool p1 = j + 1 == n1 && j + 1 < vis;
      v16f s[2];
      float alpha;
      uint32_t pb;
      THRIFT_SYNC()
      THRIFT_ISSUE(j, true, j + 1 == n1)
      if (late_v) THRIFT_ISSUE_V16(j);
      THRIFT_MASK(j)
      {
        v8s qf[8];
        THRIFT_LOAD_Q16(qf)
        scores_16<T>(lds + kLdsK16, lane, qf, s);
      }
      if (p1) {                                         // the K buffer is free once every wavefront has its scores
        lds_barrier();
        THRIFT_ISSUE_K16(j + 1);
      }
      const bool grew = softmax_update(s, lane, mask, n_valid, c, st, alpha, pb);
      rescale(o, grew, alpha);
      if (late_v) {                                     // this block's V tile was issued in this step
        if (p1) vm_wait<C16>();
        else vm_wait<0>();
        lds_barrier();
      }
      pv_16<T, true>(lds + kLdsV16, lane, s, o);
      THRIFT_NEXT_PROMOTED()
      late_v = p1;
      ++j;
    }
  }
  for (; j < vis; ++j) {                                // staging only
    THRIFT_DROP_STALE(j)
    const bool p0 = j == n0;
    const bool p1 = (p0 ? j + 1 == n1 : j + 1 == n0);
    THRIFT_SYNC()
    THRIFT_ISSUE(j, p0, p1)
    if (p0) {
      const bool p1v = p1 && j + 1 < vis;
      if (late_v) THRIFT_ISSUE_V16(j);
      if (p1v) {
        lds_barrier();
        THRIFT_ISSUE_K16(j + 1);
      }
      if (late_v) {
        if (p1v) vm_wait<C16>();
        else vm_wait<0>();
        lds_barrier();
      }
      THRIFT_NEXT_PROMOTED()
      late_v = p1v;
    } else {
      late_v = false;
    }
  }
  }
  vm_wait<0>();
#undef THRIFT_SYNC
#undef THRIFT_LOAD_Q16
#undef THRIFT_LOAD_Q16_ROW
#undef THRIFT_ISSUE
#undef THRIFT_MASK
#undef THRIFT_NEXT_PROMOTED
#undef THRIFT_DROP_STALE
#undef THRIFT_ISSUE4
#undef THRIFT_ISSUE4_SLOT
#undef THRIFT_ISSUE_V16
#undef THRIFT_ISSUE_K16
#undef THRIFT_ISSUE_TILE16
#undef THRIFT_V16OFF
#undef THRIFT_K16OFF
#undef THRIFT_CLAMP_ROWS

  // ---- epilogue (Alg. 1 step 21): O / l; accumulator i of tile n is channel 32n + 8(i/4) + 4*half + i%4 ----
  const float l = st.l + other_half(st.l);
  const float inv = l > 0.f ? 1.0f / l : 0.f;
  THRIFT_ROW_AGAIN(row_e)
  const bool row_ok = row_e < Nq;
  const int lrow_again = min(row_e, Nq - 1);
  const size_t orow = (qh * Nq + lrow_again) * kD;
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int q4i = 0; q4i < 4; ++q4i) {
      const int ch = 32 * n + 8 * q4i + 4 * half;
      if (!row_ok) continue;
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
  if (a.lse != nullptr && half == 0 && row_ok) a.lse[qh * Nq + lrow_again] = st.m * a.scale + __logf(l);
#undef THRIFT_ROW_AGAIN
}

template <typename T, int NW, int ORDER, int WIDE>
__global__ void __launch_bounds__(NW * 64, WIDE ? 2 : 3) prefill_kernel(PrefillArgs a) {
  __shared__ __align__(1024) unsigned char lds[WIDE ? kLdsPrefillWide : kLdsPrefill];
  prefill_item<T, NW, ORDER, WIDE>(a, lds, blockIdx.x);
}

// The same items from a persistent launch: as many workgroups as the chip holds at once, each taking the next item
// (heaviest first, like the launch order above) from a device counter until none is left.  An item of this kernel
// leaves no DMA in flight and the barriers below keep the LDS of one item apart from the next.
static __device__ unsigned int prefill_next_item[64];       // one counter per launch in flight would be needed: see launch_prefill

__global__ void prefill_reset_counter_kernel() { prefill_next_item[0] = 0u; }

template <typename T, int NW, int ORDER>
__global__ void __launch_bounds__(NW * 64, 3) prefill_persistent_kernel(PrefillArgs a, unsigned items) {
  __shared__ __align__(1024) unsigned char lds[kLdsPrefill];
  __shared__ unsigned next;
  // the workgroup's position on its XCD decides nothing here: items keep the XCD of their KV head only while the
  // counter hands consecutive items to consecutive workgroups, which it does at the start and loses later
  for (;;) {
    if (threadIdx.x == 0) next = atomicAdd(&prefill_next_item[0], 1u);
    __syncthreads();
    const unsigned work = next;
    __syncthreads();
    if (work >= items) break;
    prefill_item<T, NW, ORDER, 0>(a, lds, work);
  }
}

// The wide schedule pays for itself once promoted blocks are frequent: their 32 KiB of 16-bit tiles then
// arrive a whole step ahead instead of half a step, at the price of two instead of three workgroups per CU
// for the 4-bit blocks.  The per-row list length bounds the promoted share from above.
static bool wide_schedule(const PrefillArgs& a) {
  if (a.Bq != 128 || a.tile_order == 1 || a.tile_order == 2) return false;
  if (a.tile_order == 3) return true;
  const long Tk = (a.N + kBk - 1) / kBk;
  return (long)a.kmax * 100L >= Tk * (long)kWidePercent;
}

void launch_prefill(const PrefillArgs& a, hipStream_t st) {
  const unsigned grid = (unsigned)((long)a.B * a.Hq * ((a.Nq + a.Bq - 1) / a.Bq));
  if (a.tile_order == 4 && a.Bq == 128) {
    // persistent launch of the Sec. 3.3 order: three workgroups per CU.  One counter per device: two such launches
    // must not overlap on a device.  The counter is cleared by a kernel (a memset node misbehaves under graph capture).
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    const unsigned resident = (unsigned)min((long)grid, 3L * cus);
    prefill_reset_counter_kernel<<<dim3(1), dim3(1), 0, st>>>();
    if (a.dt == THRIFT_F16) prefill_persistent_kernel<F16, 4, 1><<<dim3(resident), dim3(256), 0, st>>>(a, grid);
    else prefill_persistent_kernel<BF16, 4, 1><<<dim3(resident), dim3(256), 0, st>>>(a, grid);
    return;
  }
#define THRIFT_LAUNCH(T, NW)                                                                                   \
  do {                                                                                                         \
    if (a.tile_order == 1 || a.tile_order == 4) prefill_kernel<T, NW, 1, 0><<<dim3(grid), dim3(NW * 64), 0, st>>>(a);               \
    else prefill_kernel<T, NW, 0, 0><<<dim3(grid), dim3(NW * 64), 0, st>>>(a);                                 \
  } while (0)
  if (wide_schedule(a)) {
    if (a.dt == THRIFT_F16) prefill_kernel<F16, 4, 0, 1><<<dim3(grid), dim3(256), 0, st>>>(a);
    else prefill_kernel<BF16, 4, 0, 1><<<dim3(grid), dim3(256), 0, st>>>(a);
  } else if (a.Bq == 128) {
    if (a.dt == THRIFT_F16) THRIFT_LAUNCH(F16, 4);
    else THRIFT_LAUNCH(BF16, 4);
  } else {
    if (a.dt == THRIFT_F16) THRIFT_LAUNCH(F16, 2);
    else THRIFT_LAUNCH(BF16, 2);
  }
#undef THRIFT_LAUNCH
}

}  // namespace thrift
