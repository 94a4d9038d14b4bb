/*
 * Sanitizer pass over the CPU oracle (test infrastructure, like the oracle itself).
 *
 * Includes oracle/thrift_oracle.c and runs every exported routine once on small seeded inputs that span the
 * shapes the tests use: several heads in GQA groups, a sequence length that is not a block multiple, causal and
 * non-causal, both tile orders, the three number-format variants, a chunk with an offset, decode with a partly
 * filled last block.  Results are not checked here (the pins in tests/test_oracle_*.py do that); the point is
 * that AddressSanitizer and UndefinedBehaviorSanitizer see every path.  Built and run by
 * tests/test_oracle_sanitizers.py:
 *   gcc -O1 -g -std=c99 -fopenmp -fsanitize=address,undefined -fno-sanitize-recover=all oracle/sanitize_check.c -lm
 */
#include <stdio.h>

#include "thrift_oracle.c"

static uint64_t rng_state = 0x9E3779B97F4A7C15ULL;
static double uniform(void) {   /* xorshift64*, in [-1, 1) */
  rng_state ^= rng_state >> 12; rng_state ^= rng_state << 25; rng_state ^= rng_state >> 27;
  return (double)((rng_state * 0x2545F4914F6CDD1DULL) >> 11) / 4503599627370496.0 - 1.0;
}
/* 16-bit patterns of moderate values (fp16 or bf16), a few of them large so that scales spread */
static void fill16(uint16_t* x, long n, int dtype) {
  for (long i = 0; i < n; ++i) {
    double v = uniform() * ((i % 37) == 0 ? 8.0 : 1.0);
    float f = (float)v;
    uint32_t u; memcpy(&u, &f, 4);
    if (dtype == ORACLE_BF16) x[i] = (uint16_t)(u >> 16);
    else {
      /* crude fp32 -> fp16 by rounding through the oracle's own routine */
      double r = oracle_round_to_dtype(v, ORACLE_F16);
      int e; double mant = frexp(fabs(r), &e);   /* r = mant * 2^e, mant in [0.5, 1) */
      if (r == 0.0) x[i] = 0;
      else {
        int ex = e - 1 + 15; int man = (int)ldexp(mant * 2.0 - 1.0, 10);
        if (ex <= 0) x[i] = 0; else x[i] = (uint16_t)(((r < 0) << 15) | (ex << 10) | (man & 1023));
      }
    }
  }
}

int main(void) {
  enum { B = 1, Hq = 4, Hkv = 2, D = 128, Bk = 64 };
  const int lengths[2] = {256, 333};
  for (int dtype = 0; dtype < 2; ++dtype)
    for (int li = 0; li < 2; ++li)
      for (int Bq = 64; Bq <= 128; Bq += 64) {
        const int N = lengths[li], Tq = (N + Bq - 1) / Bq, Tk = (N + Bk - 1) / Bk;
        uint16_t* q = malloc(sizeof(uint16_t) * B * Hq * N * D);
        uint16_t* k = malloc(sizeof(uint16_t) * B * Hkv * N * D);
        uint16_t* v = malloc(sizeof(uint16_t) * B * Hkv * N * D);
        fill16(q, (long)B * Hq * N * D, dtype); fill16(k, (long)B * Hkv * N * D, dtype); fill16(v, (long)B * Hkv * N * D, dtype);
        float* qm = malloc(sizeof(float) * B * Hq * Tq * D);
        float* km = malloc(sizeof(float) * B * Hkv * Tk * D);
        oracle_block_means(q, dtype, B, Hq, N, D, Bq, qm);
        oracle_block_means(k, dtype, B, Hkv, N, D, Bk, km);
        double* sc = malloc(sizeof(double) * B * Hq * Tq * Tk);
        oracle_block_scores(qm, km, B, Hq, Hkv, Tq, Tk, D, sc);
        const int kmax = Tk;
        int32_t* idx = malloc(sizeof(int32_t) * B * Hq * Tq * kmax);
        int32_t* cnt = malloc(sizeof(int32_t) * B * Hq * Tq);
        const int n_units = Hq * Tq;
        int32_t* units = malloc(sizeof(int32_t) * 3 * n_units);
        for (int h = 0; h < Hq; ++h) for (int i = 0; i < Tq; ++i) { int32_t* u = units + 3 * (h * Tq + i); u[0] = 0; u[1] = h; u[2] = i; }
        double* out = malloc(sizeof(double) * n_units * Bq * D);
        double* lse = malloc(sizeof(double) * n_units * Bq);
        const double scale = 1.0 / sqrt((double)D);
        for (int causal = 0; causal < 2; ++causal) {
          const double budgets[4] = {0.0, 0.05, 0.3, 1.0};
          for (int bi = 0; bi < 4; ++bi) {
            if (oracle_select_topk(qm, km, B, Hq, Hkv, Tq, Tk, D, Bq, Bk, causal, budgets[bi], -1, 0, idx, cnt, kmax)) return 2;
            for (int order = 0; order < 2; ++order)
              if (oracle_attn_thrift_prefill(q, k, v, dtype, idx, cnt, kmax, B, Hq, Hkv, N, D, Bq, Bk, causal, scale, order, 1, -1,
                                             units, n_units, out, lse)) return 3;
          }
          if (oracle_select_topk(qm, km, B, Hq, Hkv, Tq, Tk, D, Bq, Bk, causal, 0.0, 2, 0, idx, cnt, kmax)) return 4;      /* fixed k */
          if (oracle_select_topk_shared(qm, km, B, Hq, Hkv, Tq, Tk, D, Bq, Bk, causal, 0.25, -1, 0, idx, cnt, kmax)) return 5;
          for (int sel = 1; sel <= 2; ++sel)
            if (oracle_select_ablation(sel, 1234567ULL, B, Hq, Tq, Tk, Bq, Bk, causal, 0.25, -1, 0, idx, cnt, kmax)) return 6;
          /* forced paths, P quantisation off, the study formats (fmt 2 needs N % 32 == 0) */
          for (int fmt = 0; fmt < 3; ++fmt) {
            if (fmt == 2 && N % 32) continue;
            for (int qp = 0; qp < 2; ++qp)
              if (oracle_attn_thrift_prefill_chunk(q, k, v, dtype, idx, cnt, kmax, B, Hq, Hkv, N, 0, N, D, Bq, Bk, causal, scale, 0, qp, 0,
                                                   fmt, units, n_units, out, NULL)) return 7;
          }
          if (oracle_attn_thrift_prefill(q, k, v, dtype, NULL, NULL, 0, B, Hq, Hkv, N, D, Bq, Bk, causal, scale, 0, 1, 1, units, n_units, out, lse))
            return 8;
        }
        /* a chunk: the last query block against the whole key range */
        {
          const int off = Tq - 1, Nq = N - off * Bq;
          int32_t u1[3 * Hq];
          for (int h = 0; h < Hq; ++h) { u1[3 * h] = 0; u1[3 * h + 1] = h; u1[3 * h + 2] = 0; }
          uint16_t* qc = malloc(sizeof(uint16_t) * Hq * Nq * D);
          for (int h = 0; h < Hq; ++h) memcpy(qc + (long)h * Nq * D, q + ((long)h * N + (long)off * Bq) * D, sizeof(uint16_t) * Nq * D);
          float* qmc = malloc(sizeof(float) * Hq * D);
          oracle_block_means(qc, dtype, B, Hq, Nq, D, Bq, qmc);
          if (oracle_select_topk(qmc, km, B, Hq, Hkv, 1, Tk, D, Bq, Bk, 1, 0.25, -1, off, idx, cnt, kmax)) return 9;
          if (oracle_attn_thrift_prefill_chunk(qc, k, v, dtype, idx, cnt, kmax, B, Hq, Hkv, Nq, off, N, D, Bq, Bk, 1, scale, 1, 1, -1, 0,
                                               u1, Hq, out, lse)) return 10;
          free(qc); free(qmc);
        }
        /* exact attention on a few rows */
        {
          int32_t rows[3 * 4] = {0, 0, 0, 0, 1, N / 2, 0, 2, N - 1, 0, 3, 7};
          oracle_attn_exact(q, k, v, dtype, B, Hq, Hkv, N, N, D, 1, 0, scale, rows, 4, out, lse);
          oracle_attn_exact(q, k, v, dtype, B, Hq, Hkv, N, N, D, 0, 0, scale, rows, 4, out, NULL);
        }
        /* quantiser round trip on both axes */
        {
          uint8_t* codes = malloc((size_t)B * Hkv * N * D);
          uint8_t* scales = malloc((size_t)B * Hkv * ((N + 31) / 32) * D + (size_t)B * Hkv * N * (D / 32));
          double* dq = malloc(sizeof(double) * B * Hkv * N * D);
          for (int axis = 0; axis < 2; ++axis) {
            oracle_quantize_mxfp4(k, dtype, B, Hkv, N, D, axis, codes, scales);
            oracle_dequantize_mxfp4(codes, scales, B, Hkv, N, D, axis, dq);
          }
          oracle_nvfp4_qdq(dq, (long)(B * Hkv * N * D / 16) * 16, dq);
          oracle_mx_nosat_qdq(dq, (long)(B * Hkv * N * D / 32) * 32, dq);
          free(codes); free(scales); free(dq);
        }
        /* decode: the query at the last position; full cache and a partly filled last block; split-K on and off */
        {
          uint16_t* q1 = malloc(sizeof(uint16_t) * Hq * D);
          for (int h = 0; h < Hq; ++h) memcpy(q1 + h * D, q + ((long)h * N + N - 1) * D, sizeof(uint16_t) * D);
          float* q1m = malloc(sizeof(float) * Hq * D);
          oracle_block_means(q1, dtype, B, Hq, 1, D, 1, q1m);
          const int Ncap = Tk * Bk;                       /* cache capacity: whole blocks */
          uint16_t* kc = calloc((size_t)Hkv * Ncap * D, sizeof(uint16_t));
          uint16_t* vc = calloc((size_t)Hkv * Ncap * D, sizeof(uint16_t));
          for (int g = 0; g < Hkv; ++g) {
            memcpy(kc + (long)g * Ncap * D, k + (long)g * N * D, sizeof(uint16_t) * N * D);
            memcpy(vc + (long)g * Ncap * D, v + (long)g * N * D, sizeof(uint16_t) * N * D);
          }
          int32_t sl[1] = {N};
          int32_t di[Hq * 8], dc[Hq];
          if (oracle_select_topk(q1m, km, B, Hq, Hkv, 1, Tk, D, 1, Bk, 0, 0.25, -1, 0, di, dc, 8)) return 11;
          for (int split = 0; split <= 2; ++split)
            for (int qp = 0; qp < 2; ++qp)
              if (oracle_attn_thrift_decode(q1, kc, vc, dtype, di, dc, 8, sl, B, Hq, Hkv, Ncap, D, Bk, scale, split, qp, -1, out)) return 12;
          if (oracle_attn_thrift_decode(q1, kc, vc, dtype, NULL, NULL, 0, NULL, B, Hq, Hkv, Ncap, D, Bk, scale, 1, 1, 0, out)) return 13;
          double per[16];
          (void)oracle_error_bound_rhs(q1, kc, vc, dtype, Ncap, D, Bk, N, scale, per);
          free(q1); free(q1m); free(kc); free(vc);
        }
        free(q); free(k); free(v); free(qm); free(km); free(sc); free(idx); free(cnt); free(units); free(out); free(lse);
      }
  /* scalar helpers over their whole domains */
  for (int vis = 0; vis <= 70; ++vis) { (void)oracle_row_k(vis, 0.05, -1); (void)oracle_row_k(vis, 1.0, 3); }
  for (int n = 1; n <= 40; ++n) (void)oracle_paper_global_k(n, 0.05);
  for (int i = 0; i < 8; ++i) (void)oracle_visible_blocks(i, 16, 128, 64, 1, 2);
  for (int c = 0; c < 16; ++c) (void)oracle_e2m1_decode(c);
  for (double x = -500.0; x < 500.0; x += 0.37) { (void)oracle_e4m3_round(x); (void)oracle_round_to_dtype(x, 0); (void)oracle_round_to_dtype(x * 1e-3, 1); }
  (void)oracle_splitmix64_output(1234567ULL, 5);
  {
    double g[32]; uint8_t codes[32];
    for (int t = 0; t < 32; ++t) g[t] = uniform() * 100.0;
    (void)oracle_mx_quantize_group(g, 32, codes);
    (void)oracle_mx_quantize_group(g, 7, codes);
  }
  printf("oracle sanitizer pass: ok (%d threads)\n", oracle_num_threads());
  return 0;
}
