/*
 * thrift.h — C ABI of the MI355X (gfx950) library for block-selective mixed-precision attention
 * (ThriftAttention, arXiv 2605.23081).
 *
 * The compute entry points are the steps of the paper's Algorithm 1:
 *   thrift_block_means      Alg. 1 step 3   (Sec. 3.2 "Block-importance scoring")
 *   thrift_select_topk      Alg. 1 step 5   (Sec. 3.2, TopK of  Qbar_i . Kbar_j ; causal restriction
 *                                            of the last paragraph of Sec. 3.2)
 *   thrift_select_ablation  App. A: random / diagonal selectors in place of the heuristic
 *   thrift_quantize_mxfp4   Alg. 1 step 2   (Sec. 3.2 "FP4 quantisation", in MXFP4: E2M1 elements with
 *                                            one E8M0 scale per 32 elements instead of NVFP4)
 *   thrift_attn_prefill     Alg. 1 steps 4-23 (Sec. 3.2 "Mixed-precision attention computation", Sec. 3.3)
 *   thrift_attn_prefill_chunk  the same kernel for a chunk of queries against a longer key range
 *   thrift_attn_decode      the same algorithm for one query token over a dual 4-bit / 16-bit KV
 *                           cache (Sec. 4.1, last sentences; Sec. 5), evaluated split-K
 *
 * Conventions shared by every call
 *   - Every pointer is a DEVICE pointer unless the comment says "host".  The caller owns every
 *     buffer; the library never allocates, frees or synchronises.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the default stream).
 *   - Arguments are validated on the host before anything is launched.  On a status other than
 *     THRIFT_OK nothing has been launched and no output has been touched.
 *   - No global state: calls on different streams are independent.
 *   - Tensors are contiguous, last index fastest.  16-bit tensors are IEEE fp16 (THRIFT_F16) or
 *     bfloat16 (THRIFT_BF16).
 *   - Shape limits of this version: D == 128, Bk == 64, Bq in {64, 128} (prefill), Hq a multiple of Hkv,
 *     at most 4096 key blocks per row (N <= 262144), a GQA group of at most 32 heads in decode, a decode
 *     cache capacity Nkv that is a multiple of Bk.  Sequence lengths need NOT be multiples of Bq or Bk (a
 *     short last block is handled as the entry points below describe).  Anything else returns
 *     THRIFT_ERR_SHAPE.
 *
 * MXFP4 as used here (OCP Microscaling v1.0 conversion)
 *   A group of 32 values with a = max|x| gets the scale byte e+127, e = floor(log2 a) - 2 clamped to
 *   [-127,127] (an all-zero group gets 127); each element is x * 2^-e rounded to the E2M1 grid
 *   {0, .5, 1, 1.5, 2, 3, 4, 6} to nearest, ties to the even code, magnitudes above 6 saturating to 6;
 *   code bit 3 is the sign (kept when the magnitude rounds to zero), bits 2-1 the exponent, bit 0 the
 *   mantissa.  Two codes share a byte: the element with the even index along the group axis sits in
 *   the low nibble.  Inf / NaN inputs are not supported.
 */
#ifndef THRIFT_H_
#define THRIFT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Callers in any language pass these as plain ints.  In C++ an enumeration without a fixed underlying type may only
 * hold values in the range of its enumerators (loading anything else is undefined behaviour), and the library, which
 * is C++, must be able to receive an invalid code in order to refuse it: hence the fixed underlying type there. */
#ifdef __cplusplus
#define THRIFT_ENUM_INT : int
#else
#define THRIFT_ENUM_INT
#endif

typedef enum THRIFT_ENUM_INT {
  THRIFT_OK = 0,
  THRIFT_ERR_NULL = 1,      /* a required pointer is NULL */
  THRIFT_ERR_SHAPE = 2,     /* unsupported or inconsistent sizes */
  THRIFT_ERR_DTYPE = 3,     /* unknown dtype code */
  THRIFT_ERR_BUDGET = 4,    /* budget outside [0,1] (and no fixed_k), or kmax too small for it */
  THRIFT_ERR_WORKSPACE = 5, /* workspace missing or smaller than thrift_*_workspace() */
  THRIFT_ERR_ARCH = 6,      /* the current device is not gfx950 */
  THRIFT_ERR_LAUNCH = 7     /* the HIP runtime refused a launch */
} thrift_status;

typedef enum THRIFT_ENUM_INT { THRIFT_F16 = 0, THRIFT_BF16 = 1, THRIFT_F32 = 2 /* outputs only */ } thrift_dtype;

/* Host: static string for a status code. */
const char* thrift_status_string(thrift_status s);

/* Host: FP16 budget of one query-block row (benchmark rule: ceil(budget * visible), at least 1 when
 * budget > 0, at most visible; budget is rounded to millionths and the ceiling is taken in integers).
 * fixed_k >= 0 overrides it: min(fixed_k, visible) — the paper's single global k. */
int thrift_row_budget(int visible, double budget, int fixed_k);

/* Host: key blocks visible to query block i (+ q_block_offset) under the causal restriction of
 * Sec. 3.2: block j is visible iff j*Bk <= (i + q_block_offset + 1)*Bq - 1.  Non-causal: Tk. */
int thrift_visible_blocks(int i, int Tk, int Bq, int Bk, int causal, int q_block_offset);

/* Host: the global k of App. B "ThriftAttention settings": the k in [1,n] whose causal tile fraction
 * (k n - k(k-1)/2) / (n(n+1)/2) is closest to `fraction` (ties: smaller k). */
int thrift_budget_to_global_k(int n_blocks, double fraction);

/* Host: the largest per-row count thrift_select_topk will write for these arguments (size of the
 * last axis the caller must give idx). */
int thrift_select_kmax(int Tq, int Tk, int Bq, int Bk, int causal, double budget, int fixed_k, int q_block_offset);

/*
 * Block token means (Sec. 3.2; Alg. 1 step 3).
 *   x      [B,H,N,D] 16-bit (dt)
 *   means  [B,H,ceil(N/block),D] fp32: arithmetic mean over the block's tokens, accumulated in fp64 and
 *          rounded once (any block >= 1).  N need not be a multiple of the block — the paper leaves the
 *          tail open (App. B counts n = floor(L/64) blocks); here a short last block is the mean of the
 *          tokens it has.
 */
thrift_status thrift_block_means(const void* x, thrift_dtype dt, int B, int H, int N, int D, int block,
                                 float* means, void* stream);

/*
 * Block-pair scores S_ij = Qbar_i . Kbar_j (no 1/sqrt(d); fp64 accumulation) and per-row TopK
 * (Sec. 3.2; Alg. 1 step 5), restricted to causally visible key blocks when causal != 0.
 *   qmean [B,Hq,Tq,D], kmean [B,Hkv,Tk,D] fp32; query head h uses KV head h / (Hq/Hkv).
 *   budget in [0,1] with fixed_k < 0, or fixed_k >= 0 (then budget is ignored); see thrift_row_budget.
 *   q_block_offset shifts the causal frontier (decode: Bq = 1, offset = position of the token).
 *   idx [B,Hq,Tq,kmax] int32: the selected block ids of each row in ascending order, padded with -1.
 *   cnt [B,Hq,Tq] int32: how many were selected.
 * Equal scores are ordered by the smaller block id.  kmax < thrift_select_kmax(...) is THRIFT_ERR_BUDGET.
 */
thrift_status thrift_select_topk(const float* qmean, const float* kmean, int B, int Hq, int Hkv, int Tq, int Tk, int D,
                                 int Bq, int Bk, int causal, double budget, int fixed_k, int q_block_offset,
                                 int32_t* idx, int32_t* cnt, int kmax, void* stream);

/*
 * Group-shared selection for grouped-query attention — an extension; the paper selects per head and
 * does not discuss GQA.  One set per (batch, KV head, query block), shared by the G = Hq/Hkv query
 * heads of the group: the heuristic of Sec. 3.2 applied to the group's summed query mean,
 * score_j = (sum_h Qbar_{h,i}) . Kbar_j  (per channel the fp64 sum over the heads in ascending order,
 * then an fp64 fused-multiply-add chain over the channels in ascending order).  Arguments, budget
 * rule, visibility and tie rule as thrift_select_topk; the set is written to the idx / cnt rows of
 * every head of the group, so the attention entry points take it unchanged.  In decode it cuts the
 * 16-bit cache traffic of a KV head from the union of G per-head sets to one set.
 */
thrift_status thrift_select_topk_shared(const float* qmean, const float* kmean, int B, int Hq, int Hkv, int Tq, int Tk, int D,
                                        int Bq, int Bk, int causal, double budget, int fixed_k, int q_block_offset,
                                        int32_t* idx, int32_t* cnt, int kmax, void* stream);

/*
 * Ablation selectors (App. A "Heuristic Ablation": randomly promoted blocks, diagonal-only selection).
 * Same outputs, budget rule and visibility as thrift_select_topk, but the k_i blocks of a row are
 *   THRIFT_SELECT_RANDOM    a uniformly random k_i-subset of the visible blocks: the blocks with the k_i
 *                           largest 64-bit keys, key(row, j) = output number (row * 2^32 + j) + 1 of the
 *                           SplitMix64 generator seeded with `seed`, row = (b*Hq + h)*Tq + i; equal keys
 *                           go to the smaller block id;
 *   THRIFT_SELECT_DIAGONAL  the k_i visible blocks closest to the causal diagonal (the largest ids).
 * The result feeds thrift_attn_prefill like any other selection.  Unknown selector: THRIFT_ERR_SHAPE.
 */
typedef enum THRIFT_ENUM_INT { THRIFT_SELECT_RANDOM = 1, THRIFT_SELECT_DIAGONAL = 2 } thrift_selector;
thrift_status thrift_select_ablation(int selector, uint64_t seed, int B, int Hq, int Tq, int Tk, int Bq, int Bk,
                                     int causal, double budget, int fixed_k, int q_block_offset,
                                     int32_t* idx, int32_t* cnt, int kmax, void* stream);

/*
 * MXFP4 quantisation (Sec. 3.2 "FP4 quantisation"; Alg. 1 step 2).
 *   x [B,H,N,D] 16-bit (dt).
 *   axis 0 (Q and K: groups of 32 along D):
 *       codes  [B,H,N,D/2]   byte t of a row holds elements 2t (low nibble) and 2t+1
 *       scales [B,H,N,D/32]
 *   axis 1 (V: groups of 32 along the token axis, the contraction axis of P.V):
 *       codes  [B,H,ceil(N/64),D,32]  per 64-token block and channel, byte t holds tokens 2t (low) and 2t+1
 *       scales [B,H,2*ceil(N/64),D]   (= [B,H,N/32,D] when 64 divides N)
 *     Tokens past N in the last block count as +0: a short last group is quantised from the tokens it
 *     has, padded positions hold code 0, a group with no token at all gets scale byte 127.
 */
thrift_status thrift_quantize_mxfp4(const void* x, thrift_dtype dt, int B, int H, int N, int D, int axis,
                                    uint8_t* codes, uint8_t* scales, void* stream);

/* Host: bytes of workspace thrift_attn_prefill needs (may be 0; then workspace may be NULL). */
size_t thrift_attn_prefill_workspace(int B, int Hq, int Hkv, int N, int D, int Bq, int Bk, int kmax);

/*
 * Fused mixed-precision flash attention (Alg. 1 steps 4-23).  For each query block i the key blocks
 * are visited in ascending order; block j runs on the 16-bit matrix path when j is in idx[b,h,i,:cnt]
 * and on the MXFP4 matrix path otherwise; both update one (m, l, O) online-softmax state per row; l
 * accumulates the unquantised probabilities on both paths; on the 4-bit path P is quantised per row in
 * groups of 32 keys (E8M0 scale: the first-level scale of Alg. 1 step 19 is identically 1), on the
 * 16-bit path P is rounded to dt.
 *   q [B,Hq,N,D], k,v [B,Hkv,N,D]                 16-bit (dt), read only for the selected tiles
 *   q4,qs / k4,ks : thrift_quantize_mxfp4(axis 0) of q / k;   v4,vs : axis 1 of v
 *   idx [B,Hq,ceil(N/Bq),kmax], cnt [B,Hq,ceil(N/Bq)]   from thrift_select_topk (ascending, padded -1)
 *     A list that breaks this contract (entries out of order, negative, past the last block, a count beyond kmax)
 *     gives unspecified numbers but is never followed outside the tensors: entries are clamped to existing
 *     blocks, the count to kmax, and entries behind the walk's position are dropped.
 *   N need not be a multiple of Bq or Bk: the last query block then has fewer rows and the keys past N
 *   in the last key block are masked out (block means, V codes: see thrift_block_means, thrift_quantize_mxfp4)
 *   softmax_scale <= 0 selects 1/sqrt(D)
 *   out [B,Hq,N,D] in out_dt (THRIFT_F16, THRIFT_BF16 or THRIFT_F32)
 *   lse (nullable) [B,Hq,N] fp32: log-sum-exp of the scaled scores of each row
 */
thrift_status thrift_attn_prefill(const void* q, const void* k, const void* v, thrift_dtype dt,
                                  const uint8_t* q4, const uint8_t* qs, const uint8_t* k4, const uint8_t* ks,
                                  const uint8_t* v4, const uint8_t* vs,
                                  const int32_t* idx, const int32_t* cnt, int kmax,
                                  int B, int Hq, int Hkv, int N, int D, int Bq, int Bk, int causal, float softmax_scale,
                                  void* out, thrift_dtype out_dt, float* lse,
                                  void* workspace, size_t workspace_bytes, void* stream);

/*
 * Chunked prefill: the same kernel for Nq query tokens per head against Nkv >= Nq key tokens, as needed
 * when a prompt is processed in pieces or extends a cached prefix (Alg. 1 is stated for Q and K, V of any
 * lengths; the causal restriction is the last paragraph of Sec. 3.2).  Query block i of the chunk stands
 * at block position i + q_block_offset of the sequence: its first token is token (i + q_block_offset)*Bq,
 * which fixes its causal mask and visible key range; with causal == 0 the offset is ignored.
 *   q, q4, qs, out, lse   hold Nq tokens per head ([B,Hq,Nq,...]);  k, v, k4, ks, v4, vs hold Nkv
 *   idx [B,Hq,Nq/Bq,kmax], cnt [B,Hq,Nq/Bq]: from thrift_select_topk with the same q_block_offset
 *   causal: (q_block_offset*Bq + Nq) <= Nkv, else THRIFT_ERR_SHAPE; Nq and Nkv need not be multiples of the blocks
 * thrift_attn_prefill is this call with Nq = Nkv = N and q_block_offset = 0.
 */
thrift_status thrift_attn_prefill_chunk(const void* q, const void* k, const void* v, thrift_dtype dt,
                                        const uint8_t* q4, const uint8_t* qs, const uint8_t* k4, const uint8_t* ks,
                                        const uint8_t* v4, const uint8_t* vs,
                                        const int32_t* idx, const int32_t* cnt, int kmax,
                                        int B, int Hq, int Hkv, int Nq, int q_block_offset, int Nkv, int D, int Bq, int Bk,
                                        int causal, float softmax_scale,
                                        void* out, thrift_dtype out_dt, float* lse,
                                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * thrift_attn_prefill_chunk with a choice of tile order.
 *   tile_order 0: key blocks in ascending order, as Alg. 1 is written (what the other entry points use);
 *   tile_order 1: the order of the kernel in Sec. 3.3 — every 4-bit block in ascending order first, then
 *                 the promoted blocks in ascending order.  The faster one at every budget: the 16-bit query
 *                 fragments are held in registers only during the promoted phase, as in the paper's kernel.
 * In exact arithmetic the two agree; the 4-bit rounding of P depends on the running maximum, so the
 * results differ at the level of the quantisation noise.
 *   tile_order 2, 3: ascending order like 0, with the staging schedule fixed instead of chosen by the library
 *                 (2: three workgroups per CU, 16-bit tiles of a promoted block half a step ahead; 3: two
 *                 workgroups per CU, every block a whole step ahead and the 16-bit query rows in registers,
 *                 Bq = 128 only, else it falls back to 2).  0 picks 3 when kmax is at least 15 % of the key
 *                 blocks, where the promoted blocks dominate the time.  The results of 0, 2 and 3 are bit-identical.
 *   tile_order 4: the order of 1 from a persistent launch: as many workgroups as the device holds at once (three
 *                 per CU) take the (head, query block) items, heaviest first, from a counter in device memory
 *                 instead of one workgroup being launched per item.  Bit-identical to 1; Bq = 128 only, else it
 *                 is 1.  The counter is one per device: two launches with tile_order 4 must not overlap on a device.
 *                 (Measured slower than 1 on the 131k layer: the hardware dispatcher already hands out the
 *                 heaviest-first launch order dynamically.  Kept for measurement.)
 * Other values: THRIFT_ERR_SHAPE.
 */
thrift_status thrift_attn_prefill_ordered(const void* q, const void* k, const void* v, thrift_dtype dt,
                                          const uint8_t* q4, const uint8_t* qs, const uint8_t* k4, const uint8_t* ks,
                                          const uint8_t* v4, const uint8_t* vs,
                                          const int32_t* idx, const int32_t* cnt, int kmax,
                                          int B, int Hq, int Hkv, int Nq, int q_block_offset, int Nkv, int D, int Bq, int Bk,
                                          int causal, int tile_order, float softmax_scale,
                                          void* out, thrift_dtype out_dt, float* lse,
                                          void* workspace, size_t workspace_bytes, void* stream);

/*
 * Alg. 1 in one call, the user-level form of the paper's signature (Q, K, V, block sizes, FP16 budget in; attention
 * output out): block means of Q and K, scores and per-row TopK, MXFP4 quantisation of Q, K, V, fused attention,
 * seven launches on `stream` in that order.  The intermediate tensors live in `workspace`
 * (thrift_attention_forward_workspace(...) bytes, 256-byte aligned, device), which may be reused by the next call
 * on the same stream.  q [B,Hq,N,D], k, v [B,Hkv,N,D] 16-bit (dt); out [B,Hq,N,D] in out_dt; lse nullable [B,Hq,N].
 * budget / fixed_k as in thrift_select_topk; tile_order as in thrift_attn_prefill_ordered (0: Alg. 1's order, 1: the
 * order of the kernel in Sec. 3.3, the faster one); softmax_scale <= 0 means 1/sqrt(D).  All arguments are
 * validated before the first stage is enqueued: on a status other than THRIFT_OK nothing has run (THRIFT_ERR_LAUNCH
 * excepted, which reports a launch the HIP runtime refused).
 */
size_t thrift_attention_forward_workspace(int B, int Hq, int Hkv, int N, int D, int Bq, int Bk, int causal, double budget, int fixed_k);
thrift_status thrift_attention_forward(const void* q, const void* k, const void* v, thrift_dtype dt,
                                       int B, int Hq, int Hkv, int N, int D, int Bq, int Bk, int causal,
                                       double budget, int fixed_k, int tile_order, float softmax_scale,
                                       void* out, thrift_dtype out_dt, float* lse,
                                       void* workspace, size_t workspace_bytes, void* stream);

/* Host: bytes of workspace thrift_attn_decode needs. */
size_t thrift_attn_decode_workspace(int B, int Hq, int Hkv, int Nkv, int D, int Bk, int split_blocks);

/*
 * Decode over a dual KV cache: one query token per (sequence, query head) at position seqlen-1, so
 * every cached key is visible.  The call (i) scores the cached key-block means against the query
 * (the block mean of a one-token block is the token) and selects ceil(budget * blocks) blocks per
 * query head (or fixed_k), (ii) runs Alg. 1 per (sequence, KV head, partition of split_blocks key
 * blocks) for the Hq/Hkv query heads of the group — MXFP4 codes for non-selected blocks, the 16-bit
 * copy for selected ones — and (iii) merges the partitions by their log-sum-exp.
 *   q [B,Hq,D] 16-bit (dt)
 *   k16,v16 [B,Hkv,Nkv,D] 16-bit (dt)             read only for selected blocks
 *   k4,ks (axis 0) and v4,vs (axis 1) of the same cache; kmean [B,Hkv,Nkv/Bk,D] fp32
 *   seqlens (nullable, device) [B] int32: cached tokens per sequence, 0 .. Nkv (values outside are clamped);
 *     NULL = Nkv.  A length that is not a multiple of Bk leaves the last key block partly filled: its keys past
 *     the length are masked, its kmean entry must be the mean of the tokens it has and its V groups must have
 *     been quantised from those tokens alone (what thrift_kv_cache_append, or the pre-pass on a tensor of that
 *     length, produces).  Cache contents past that block are never read.  A sequence of length 0 yields zeros.
 *     Split-K: the full key blocks are cut into the partitions; a partly filled last block is a partition of its own.
 *   split_blocks: key blocks per partition (> 0): each (query head, partition) is one recurrence of Alg. 1 over the
 *     partition's key blocks in ascending order; the rounding of P on the 4-bit path follows the running maximum, so
 *     the result depends on the partition size at the level of the quantisation noise (in exact arithmetic it does not)
 *   out [B,Hq,D] in out_dt
 *   idx_out (nullable) [B,Hq,kmax_out], cnt_out (nullable) [B,Hq]: the selection that was used
 *     (kmax_out >= thrift_select_kmax(1, Nkv/Bk, 1, Bk, 0, budget, fixed_k, 0))
 *   workspace: thrift_attn_decode_workspace(...) bytes
 */
thrift_status thrift_attn_decode(const void* q, thrift_dtype dt, const void* k16, const void* v16,
                                 const uint8_t* k4, const uint8_t* ks, const uint8_t* v4, const uint8_t* vs,
                                 const float* kmean, const int32_t* seqlens,
                                 int B, int Hq, int Hkv, int Nkv, int D, int Bk,
                                 double budget, int fixed_k, int split_blocks, float softmax_scale,
                                 void* out, thrift_dtype out_dt, int32_t* idx_out, int32_t* cnt_out, int kmax_out,
                                 void* workspace, size_t workspace_bytes, void* stream);

/* thrift_attn_decode with the group-shared selection of thrift_select_topk_shared in step (i). */
thrift_status thrift_attn_decode_shared(const void* q, thrift_dtype dt, const void* k16, const void* v16,
                                        const uint8_t* k4, const uint8_t* ks, const uint8_t* v4, const uint8_t* vs,
                                        const float* kmean, const int32_t* seqlens,
                                        int B, int Hq, int Hkv, int Nkv, int D, int Bk,
                                        double budget, int fixed_k, int split_blocks, float softmax_scale,
                                        void* out, thrift_dtype out_dt, int32_t* idx_out, int32_t* cnt_out, int kmax_out,
                                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * thrift_attn_decode for callers that cannot allocate device memory or hand over a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and results as
 * thrift_attn_decode, without the workspace: the score keys, the selection bitmap and the split-K partials live
 * in a static device array of THRIFT_DECODE_STATIC_SCRATCH_BYTES that every GPU the library runs on holds until
 * the process ends.  The call allocates and frees nothing.  A problem whose thrift_attn_decode_workspace(...)
 * exceeds that size returns THRIFT_ERR_WORKSPACE (nothing launched).  All calls on one GPU share the array:
 * calls that overlap on one GPU (different streams, different host threads) race on it; calls on one stream
 * are ordered and safe.  Nothing in the array has to be cleared between calls: every byte a call reads it has
 * written itself.
 */
#define THRIFT_DECODE_STATIC_SCRATCH_BYTES (32u << 20)
thrift_status thrift_attn_decode_static(const void* q, thrift_dtype dt, const void* k16, const void* v16,
                                        const uint8_t* k4, const uint8_t* ks, const uint8_t* v4, const uint8_t* vs,
                                        const float* kmean, const int32_t* seqlens,
                                        int B, int Hq, int Hkv, int Nkv, int D, int Bk,
                                        double budget, int fixed_k, int split_blocks, float softmax_scale,
                                        void* out, thrift_dtype out_dt, int32_t* idx_out, int32_t* cnt_out, int kmax_out,
                                        void* stream);

/*
 * Append tokens to the dual cache that thrift_attn_decode reads (Sec. 4.1 and Sec. 5 describe the cache: 4-bit
 * K and V for every block, the 16-bit copy for promoted blocks, and the key-block means).  After the call the
 * cache holds, for every sequence, exactly what the pre-pass (thrift_block_means with block Bk on K,
 * thrift_quantize_mxfp4 axis 0 on K and axis 1 on V) would produce from the sequence's first
 * seqlens[b] + n tokens: new 4-bit K rows; the V groups of 32 tokens that received tokens quantised again from
 * the tokens they now hold (a group's scale follows its largest magnitude so far); the mean of a block that is
 * still filling up taken over the tokens it has.  Every key block that receives a token is written whole (V codes
 * of absent tokens are 0), so a partly filled last block is always defined.
 *   k_new, v_new [B,Hkv,n_new,D] 16-bit (dt), device; must not overlap the cache
 *   seqlens (device) [B] int32: tokens cached before the call (clamped to 0 .. Nkv); NOT modified - the caller
 *     adds the appended count afterwards
 *   new_lens (nullable, device) [B] int32: tokens to take per sequence, clamped to 0 .. n_new; NULL = n_new for all.
 *     Tokens that would pass the capacity Nkv are dropped.
 *   k16,v16 [B,Hkv,Nkv,D]; k4 [B,Hkv,Nkv,D/2]; ks [B,Hkv,Nkv,D/32]; v4 [B,Hkv,Nkv/64,D,32]; vs [B,Hkv,Nkv/32,D];
 *   kmean [B,Hkv,Nkv/Bk,D] fp32: the cache, device, updated in place.  Nkv % Bk == 0, D == 128, Bk == 64.
 * Calls that touch the same sequence must be ordered (same stream); nothing is allocated.
 */
thrift_status thrift_kv_cache_append(const void* k_new, const void* v_new, thrift_dtype dt, int n_new,
                                     const int32_t* seqlens, const int32_t* new_lens,
                                     void* k16, void* v16, uint8_t* k4, uint8_t* ks, uint8_t* v4, uint8_t* vs, float* kmean,
                                     int B, int Hkv, int Nkv, int D, int Bk, void* stream);

/*
 * Measurement helper (not a step of the method): one launch of a microbenchmark of a hardware rate that the
 * roofline figures of the attention kernels are priced against.  The caller times the launch (events on `stream`)
 * and divides *work by the duration.
 *   THRIFT_PEAK_MFMA_MXFP4    scaled-FP4 32x32x64 matrix instructions back to back        *work = flops
 *   THRIFT_PEAK_MFMA_16       16-bit 32x32x16 matrix instructions (dt: fp16 or bf16)      *work = flops
 *   THRIFT_PEAK_HBM_READ      one streaming read of `buffer` (use >= 1 GiB)                *work = bytes read
 *   THRIFT_PEAK_VALU_SOFTMAX  the vector-ALU part of one 4-bit 32-query x 64-key wave-tile of the fused kernel
 *                             (online-softmax update + P quantiser, no matrix instructions, no staging), at the
 *                             fused kernel's occupancy                                    *work = wave-tiles
 *   THRIFT_PEAK_TILE_MIX      the same plus the tile's eight matrix instructions           *work = wave-tiles
 * buffer (device): at least 16 MiB (scratch for results; for THRIFT_PEAK_HBM_READ the data that is read, whatever it
 * holds; its last 64 KiB are not read).  iters >= 1: loop trips per wavefront (ignored by the HBM probe).
 * Unknown kind, iters < 1 or a buffer below 16 MiB: THRIFT_ERR_SHAPE.
 */
typedef enum THRIFT_ENUM_INT { THRIFT_PEAK_MFMA_MXFP4 = 0, THRIFT_PEAK_MFMA_16 = 1, THRIFT_PEAK_HBM_READ = 2,
                               THRIFT_PEAK_VALU_SOFTMAX = 3, THRIFT_PEAK_TILE_MIX = 4 } thrift_peak_kind;
thrift_status thrift_peak_probe(int kind, thrift_dtype dt, int iters, void* buffer, size_t bytes, double* work, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* THRIFT_H_ */
