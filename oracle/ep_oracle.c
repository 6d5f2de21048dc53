/*
 * CPU oracle for the expert-parallel layout / dispatch / combine path.
 *
 * TEST INFRASTRUCTURE, NOT PRODUCT: a plain, slow, scalar C implementation of
 * what the path computes, written from the paper's statement of the problem
 * (Section 2.1: tokens are dispatched to the GPUs hosting their selected
 * experts and expert outputs are merged back into the order of the tokens;
 * Section 2.2: the combine reduce is a weighted sum; Section 2.1 "Fine-grained
 * token-level transfers": a token is an FP8, hidden-7168, ~7 KB message).
 * It shares no code, header, table or constant with the HIP library and is
 * only called by tests, the smoke check and the benchmark's cpu_baseline leg.
 *
 * There is no blocking, fusion or reordering here beyond the definitions:
 * every function is the definition written out as loops.  The optional OpenMP
 * pragma splits the *token* loop of dispatch/combine over host threads; each
 * token is still computed by the same scalar statements.
 *
 * bf16 values travel as uint16_t bit patterns.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int g_threads = 1;

/* Number of host threads the token loops of dispatch/combine may use. */
void oracle_set_threads(int n) { g_threads = n < 1 ? 1 : n; }
int oracle_get_threads(void) { return g_threads; }
int oracle_max_threads(void) {
#ifdef _OPENMP
  return omp_get_num_procs();
#else
  return 1;
#endif
}

static float bf16_to_f32(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

/* float -> bf16, round to nearest, ties to even mantissa.  Finite inputs. */
static uint16_t f32_to_bf16_rne(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  uint32_t keep = u >> 16;
  uint32_t rest = u & 0xFFFFu;
  if (rest > 0x8000u || (rest == 0x8000u && (keep & 1u))) keep += 1;
  return (uint16_t)keep;
}
uint16_t oracle_f32_to_bf16(float f) { return f32_to_bf16_rne(f); }
float oracle_bf16_to_f32(uint16_t b) { return bf16_to_f32(b); }

/* ------------------------------------------------------------------ layout
 * Step (1) of the path: per-(source rank, expert) token counts, exclusive
 * prefix scans, and stable slot indices.  The paper only says that message
 * sizes and destinations must be worked out every step (Section 2.1,
 * "Irregular communication"); the definition used is the counting walk:
 * visit (s, t, k) in ascending order; the slot of an entry is the number of
 * earlier entries of the same source that chose the same expert.
 * Receive rows are expert-major, source-rank-minor:
 *   base[s][e] = sum_{e'<e} expert_total[e'] + sum_{s'<s} count[s'][e].
 * Entries with idx == -1 are masked: slot = dst_row = -1.
 * Returns 0, or -1 if an index is outside [-1, E) or E % R != 0.
 */
int oracle_layout(const int32_t *idx, int S, int T, int K, int E, int R,
                  int32_t *count, int32_t *expert_total, int32_t *rank_total,
                  int32_t *base, int32_t *expert_offset, int32_t *rank_offset,
                  int32_t *slot, int32_t *dst_row) {
  if (R <= 0 || E <= 0 || E % R != 0) return -1;
  int E_loc = E / R;
  for (int i = 0; i < S * E; ++i) count[i] = 0;
  for (int s = 0; s < S; ++s)
    for (int t = 0; t < T; ++t)
      for (int k = 0; k < K; ++k) {
        long i = ((long)s * T + t) * K + k;
        int e = idx[i];
        if (e == -1) { slot[i] = -1; continue; }
        if (e < 0 || e >= E) return -1;
        slot[i] = count[s * E + e];
        count[s * E + e] += 1;
      }
  for (int e = 0; e < E; ++e) {
    int tot = 0;
    for (int s = 0; s < S; ++s) tot += count[s * E + e];
    expert_total[e] = tot;
  }
  for (int r = 0; r < R; ++r) {
    int tot = 0;
    for (int j = 0; j < E_loc; ++j) tot += expert_total[r * E_loc + j];
    rank_total[r] = tot;
  }
  int run = 0;
  for (int e = 0; e < E; ++e) { expert_offset[e] = run; run += expert_total[e]; }
  expert_offset[E] = run;
  for (int r = 0; r < R; ++r) rank_offset[r] = expert_offset[r * E_loc];
  rank_offset[R] = run;
  for (int e = 0; e < E; ++e) {
    int b = expert_offset[e];
    for (int s = 0; s < S; ++s) { base[s * E + e] = b; b += count[s * E + e]; }
  }
  for (int s = 0; s < S; ++s)
    for (int t = 0; t < T; ++t)
      for (int k = 0; k < K; ++k) {
        long i = ((long)s * T + t) * K + k;
        int e = idx[i];
        dst_row[i] = (e == -1) ? -1 : base[s * E + e] + slot[i];
      }
  return 0;
}

/* ----------------------------------------------------------- dispatch bf16
 * Step (2): every valid (t, k) copies the token's hidden vector into its
 * receive row: recv[dst_row[t,k], :] = x[t, :]  (Section 2.1, the dispatch
 * phase: a token's activation goes to every rank that hosts one of its experts).
 * rank_filter >= 0 keeps only entries whose expert lives on that rank
 * (expert e lives on rank e / E_loc).  write_count (optional, [recv_rows])
 * is bumped once per row written so a test can see double writes.
 * Returns 0, or -2 if a destination row is outside [0, recv_rows).
 */
int oracle_dispatch_bf16(const uint16_t *x, const int32_t *idx, const int32_t *dst_row,
                         int T, int K, int H, int E_loc, int rank_filter,
                         uint16_t *recv, long recv_rows, uint8_t *write_count) {
  int bad = 0;
#pragma omp parallel for num_threads(g_threads) schedule(static) reduction(|:bad)
  for (int t = 0; t < T; ++t)
    for (int k = 0; k < K; ++k) {
      int e = idx[(long)t * K + k];
      if (e == -1) continue;
      if (rank_filter >= 0 && e / E_loc != rank_filter) continue;
      long row = dst_row[(long)t * K + k];
      if (row < 0 || row >= recv_rows) { bad = 1; continue; }
      memcpy(recv + row * H, x + (long)t * H, (size_t)H * 2);
      if (write_count) write_count[row] += 1;
    }
  return bad ? -2 : 0;
}

/* ------------------------------------------------------------ FP8 e4m3
 * OCP 8-bit float E4M3 ("fn": no infinities): 1 sign, 4 exponent (bias 7),
 * 3 mantissa bits; subnormals k * 2^-9 (k = 1..7); largest finite 448
 * (code 0x7E); 0x7F / 0xFF are NaN and never produced here.
 */
float oracle_e4m3_decode(uint8_t c) {
  int s = c >> 7, ex = (c >> 3) & 0xF, m = c & 7;
  float v;
  if (ex == 0) v = ldexpf((float)m, -9);
  else if (ex == 15 && m == 7) v = NAN;
  else v = ldexpf((float)(8 + m), ex - 7 - 3);
  return s ? -v : v;
}

/* Round a finite float to the nearest E4M3 value, ties to even mantissa,
 * results beyond the largest finite value saturate to +-448; the sign of
 * zero is kept. */
uint8_t oracle_e4m3_encode(float y) {
  uint32_t u;
  memcpy(&u, &y, 4);
  uint8_t sign = (uint8_t)((u >> 31) << 7);
  float a = fabsf(y);
  if (a == 0.0f) return sign;
  int e;
  (void)frexpf(a, &e); /* a = f * 2^e, f in [0.5,1)  =>  floor(log2 a) = e-1 */
  e -= 1;
  if (e < -6) { /* below the smallest normal 2^-6: multiples of 2^-9 */
    float q = rintf(ldexpf(a, 9)); /* exact scaling, then round-to-nearest-even */
    return (uint8_t)(sign | (uint8_t)q); /* q == 8 is exactly the code of 2^-6 */
  }
  float m = rintf(ldexpf(a, 3 - e)); /* in [8, 16] */
  if (m == 16.0f) { m = 8.0f; e += 1; }
  if (e > 8) return (uint8_t)(sign | 0x7E); /* >= 512 after rounding */
  uint8_t code = (uint8_t)(((e + 7) << 3) | ((int)m - 8));
  if (code > 0x7E) code = 0x7E; /* 480 (would be the NaN code) saturates to 448 */
  return (uint8_t)(sign | code);
}

/* Quantise one 128-channel block (payload format of the FP8 dispatch: one
 * fp32 scale per 128 channels, scale = amax / 448).
 *   amax  = max |v_i|                       (v_i = bf16 widened exactly)
 *   amax < 2^-100 (zero block, or so small that 448/amax could overflow):
 *           scale = inv = 1
 *   else    scale = amax / 448 ; inv = 448 / amax   (fp32 divisions, RN)
 *   q_i   = e4m3( v_i * inv )               (one fp32 multiply, RN)
 */
void oracle_quant_block(const uint16_t *v, int n, uint8_t *q, float *scale) {
  float amax = 0.0f;
  for (int i = 0; i < n; ++i) {
    float a = fabsf(bf16_to_f32(v[i]));
    if (a > amax) amax = a;
  }
  volatile float sc, inv; /* volatile: each operation rounds to fp32 on its own */
  if (amax < 0x1p-100f) { sc = 1.0f; inv = 1.0f; }
  else { sc = amax / 448.0f; inv = 448.0f / amax; }
  for (int i = 0; i < n; ++i) {
    volatile float y = bf16_to_f32(v[i]) * inv;
    q[i] = oracle_e4m3_encode(y);
  }
  *scale = sc;
}

/* Quantise whole rows: q [T,H] codes, scale [T,H/128].  H % 128 == 0. */
void oracle_quant_rows(const uint16_t *x, int T, int H, uint8_t *q, float *scale) {
  int nb = H / 128;
#pragma omp parallel for num_threads(g_threads) schedule(static)
  for (int t = 0; t < T; ++t)
    for (int b = 0; b < nb; ++b)
      oracle_quant_block(x + (long)t * H + b * 128, 128, q + (long)t * H + b * 128,
                         scale + (long)t * nb + b);
}

/* Step (2) with the FP8 payload: the token's codes and block scales go to
 * all of its destination rows. */
int oracle_dispatch_fp8(const uint16_t *x, const int32_t *idx, const int32_t *dst_row,
                        int T, int K, int H, int E_loc, int rank_filter,
                        uint8_t *recv_q, float *recv_scale, long recv_rows,
                        uint8_t *write_count) {
  int nb = H / 128;
  int bad = 0;
#pragma omp parallel for num_threads(g_threads) schedule(static) reduction(|:bad)
  for (int t = 0; t < T; ++t) {
    uint8_t qrow[H];
    float srow[nb];
    int done = 0;
    for (int k = 0; k < K; ++k) {
      int e = idx[(long)t * K + k];
      if (e == -1) continue;
      if (rank_filter >= 0 && e / E_loc != rank_filter) continue;
      long row = dst_row[(long)t * K + k];
      if (row < 0 || row >= recv_rows) { bad = 1; continue; }
      if (!done) {
        for (int b = 0; b < nb; ++b)
          oracle_quant_block(x + (long)t * H + b * 128, 128, qrow + b * 128, srow + b);
        done = 1;
      }
      memcpy(recv_q + row * H, qrow, (size_t)H);
      memcpy(recv_scale + row * nb, srow, (size_t)nb * 4);
      if (write_count) write_count[row] += 1;
    }
  }
  return bad ? -2 : 0;
}

/* Inverse of the payload format, for an identity-expert round trip:
 * y = bf16( decode(code) * scale ), one fp32 multiply then RNE to bf16. */
void oracle_dequant_rows(const uint8_t *q, const float *scale, long rows, int H, uint16_t *y) {
  int nb = H / 128;
  for (long r = 0; r < rows; ++r)
    for (int h = 0; h < H; ++h) {
      volatile float v = oracle_e4m3_decode(q[r * H + h]) * scale[r * nb + h / 128];
      y[r * H + h] = f32_to_bf16_rne(v);
    }
}

/* ---------------------------------------------------------------- combine
 * Step (4): expert outputs are gathered back to the original token order and
 * reduced by a weighted sum (Section 2.2):
 *   out[t,h] = bf16( sum_k w[t,k] * y[dst_row[t,k], h] )
 * with an fp32 accumulator that starts at +0 and takes the k terms in
 * ascending k as fused multiply-adds; masked k (dst_row == -1) are skipped;
 * one final round-to-nearest-even to bf16.
 */
int oracle_combine(const uint16_t *y, const float *w, const int32_t *dst_row,
                   int T, int K, int H, long rows, uint16_t *out) {
  int bad = 0;
#pragma omp parallel for num_threads(g_threads) schedule(static) reduction(|:bad)
  for (int t = 0; t < T; ++t)
    for (int h = 0; h < H; ++h) {
      float acc = 0.0f;
      for (int k = 0; k < K; ++k) {
        long row = dst_row[(long)t * K + k];
        if (row == -1) continue;
        if (row < 0 || row >= rows) { bad = 1; continue; }
        acc = fmaf(w[(long)t * K + k], bf16_to_f32(y[row * H + h]), acc);
      }
      out[(long)t * H + h] = f32_to_bf16_rne(acc);
    }
  return bad ? -2 : 0;
}

/* The same weighted sum as its plain definition in double precision, not
 * rounded to bf16: the yardstick the fp32 chain above is pinned against. */
int oracle_combine_f64(const uint16_t *y, const float *w, const int32_t *dst_row,
                       int T, int K, int H, long rows, double *out, double *abs_sum) {
  int bad = 0;
#pragma omp parallel for num_threads(g_threads) schedule(static) reduction(|:bad)
  for (int t = 0; t < T; ++t)
    for (int h = 0; h < H; ++h) {
      double acc = 0.0, mag = 0.0;
      for (int k = 0; k < K; ++k) {
        long row = dst_row[(long)t * K + k];
        if (row == -1) continue;
        if (row < 0 || row >= rows) { bad = 1; continue; }
        double term = (double)w[(long)t * K + k] * (double)bf16_to_f32(y[row * H + h]);
        acc += term;
        mag += fabs(term);
      }
      out[(long)t * H + h] = acc;
      if (abs_sum) abs_sum[(long)t * H + h] = mag;
    }
  return bad ? -2 : 0;
}

/* ------------------------------------------ high-throughput mode additions
 * Section 2.2 describes two optimisations of the high-throughput mode: a token
 * routed to several experts of one node is sent once and forwarded inside the
 * node ("message deduplication"), and expert outputs are first reduced inside
 * the node (weighted sum) and then once more at the sender ("hierarchical
 * reduce").  A "group" below is ranks_per_group consecutive ranks (1 = one GPU,
 * 8 = a node of eight).
 *
 * Dedup: group(e) = (e / E_loc) / ranks_per_group.  For every token, walking k
 * ascending: the first entry that names a group keeps it (group_idx = group),
 * later entries of the same group are duplicates (group_idx = -1); first_k is
 * the k of that first entry (-1 for masked entries).  group_idx is then a
 * routing table over groups that the ordinary layout/dispatch steps consume:
 * one copy per (token, group).
 */
int oracle_dedup(const int32_t *idx, long n_tokens, int K, int E_loc, int ranks_per_group,
                 int32_t *group_idx, int32_t *first_k) {
  for (long t = 0; t < n_tokens; ++t)
    for (int k = 0; k < K; ++k) {
      int e = idx[t * K + k];
      if (e < 0) { group_idx[t * K + k] = -1; first_k[t * K + k] = -1; continue; }
      int g = (e / E_loc) / ranks_per_group;
      int first = k;
      for (int j = 0; j < k; ++j) {
        int ej = idx[t * K + j];
        if (ej >= 0 && (ej / E_loc) / ranks_per_group == g) { first = j; break; }
      }
      group_idx[t * K + k] = (first == k) ? g : -1;
      first_k[t * K + k] = first;
    }
  return 0;
}

/* Per-expert index list: expert-major row i of the ordinary layout reads its
 * input from row index[i] of the deduplicated receive buffer. */
int oracle_gather_index(const int32_t *dst_row, const int32_t *dst_row_g, const int32_t *first_k,
                        long T, int K, long rows, int32_t *index) {
  for (long i = 0; i < rows; ++i) index[i] = -1;
  for (long t = 0; t < T; ++t)
    for (int k = 0; k < K; ++k) {
      long r = dst_row[t * K + k];
      if (r < 0) continue;
      if (r >= rows) return -2;
      index[r] = dst_row_g[t * K + first_k[t * K + k]];
    }
  return 0;
}

/* Hierarchical reduce, first level (done where the experts live): one partial
 * row per (token, group),
 *   partial[dst_row_g[t,j], h] = bf16( sum_{k : first_k[t,k] == j} w[t,k] * y[dst_row[t,k], h] )
 * fp32 accumulator from +0, k ascending, fused multiply-add, one rounding to
 * bf16 (the partial travels as bf16).  The second level is the ordinary
 * combine over the group rows with unit weights. */
int oracle_combine_partial(const uint16_t *y, const float *w, const int32_t *dst_row, const int32_t *first_k,
                           const int32_t *dst_row_g, int T, int K, int H, long rows, long rows_g,
                           uint16_t *partial) {
  int bad = 0;
#pragma omp parallel for num_threads(g_threads) schedule(static) reduction(|:bad)
  for (int t = 0; t < T; ++t)
    for (int j = 0; j < K; ++j) {
      if (first_k[(long)t * K + j] != j) continue; /* not the first entry of its group */
      long prow = dst_row_g[(long)t * K + j];
      if (prow < 0 || prow >= rows_g) { bad = 1; continue; }
      for (int h = 0; h < H; ++h) {
        float acc = 0.0f;
        for (int k = 0; k < K; ++k) {
          if (first_k[(long)t * K + k] != j) continue;
          long row = dst_row[(long)t * K + k];
          if (row < 0 || row >= rows) { bad = 1; continue; }
          acc = fmaf(w[(long)t * K + k], bf16_to_f32(y[row * H + h]), acc);
        }
        partial[prow * H + h] = f32_to_bf16_rne(acc);
      }
    }
  return bad ? -2 : 0;
}
