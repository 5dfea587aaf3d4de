/*
 * CPU oracle for relay-buffer-free MoE dispatch and combine.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, single-threaded
 * definition that the HIP library is checked against.  It shares no code with
 * the HIP path, is never linked into or called from the product library, and
 * may only be used by the tests, the smoke check and the benchmark's
 * cpu_baseline leg.
 *
 * Every function follows the paper's own order and notation (Section 5.1 for
 * the symbols; Algorithm 1 / Section 5.2 for the prefill chain; Algorithm 2 /
 * Section 5.3 for decode, which computes the same values in one procedure).
 * No blocking, fusion or reordering beyond those definitions.
 *
 * Readings taken where the paper is silent (all listed in the design notes):
 *   - "before" in the definition of s means smaller flat index i = t*k + j;
 *   - one source rank, so the large offset o_{e,r} has a single column and is
 *     an exclusive prefix sum of the expert counts inside each rank region;
 *   - combine reads the same row that dispatch wrote (q = p);
 *   - id -1 marks an unused slot (skipped, not counted); any other id outside
 *     [0,E) is skipped and counted in status[0];
 *   - windows are tight (region r holds exactly c_rank[r] rows) unless a fixed
 *     region stride is given, in which case region r starts at r*stride and
 *     branches that do not fit are dropped and counted in status[1];
 *   - combine accumulates in fp32 starting from +0, ascending j, one fused
 *     multiply-add per branch, then rounds once (nearest-even) to the storage
 *     type.  An fp64 variant is provided as an independent check.
 *
 * Parity pins: counts/offsets/s/row_map/dispatch are pinned by brute force,
 * numpy bincount/cumsum/stable-argsort and hand-worked fixtures; combine by
 * identity-expert closed forms, an fp64 numpy reference and torch's bf16
 * rounding.  Absolute values against the authors' Ascend implementation:
 * parity unpinned (the paper prints no tensors).
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

/* The token loops of dispatch and combine are independent per token (distinct rows, distinct outputs).
 * The tests use the serial build; the benchmark's all-cores baseline compiles this same file with
 * -fopenmp, which only hands the tokens of those two loops to several threads. */
#ifdef _OPENMP
#include <omp.h>
#define TOKENS_IN_PARALLEL _Pragma("omp parallel for schedule(static)")
int moe_ref_threads(void) { return omp_get_max_threads(); }
#else
#define TOKENS_IN_PARALLEL
int moe_ref_threads(void) { return 1; }
#endif

enum { MOE_REF_BF16 = 0, MOE_REF_F32 = 1 };

/* ---- storage conversions -------------------------------------------------- */

static float bf16_to_f32(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

/* fp32 -> bf16, round to nearest, ties to even; NaN stays a quiet NaN. */
static uint16_t f32_to_bf16_rne(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u);
  uint32_t lsb = (u >> 16) & 1u;
  u += 0x7FFFu + lsb;
  return (uint16_t)(u >> 16);
}

/* fp64 -> bf16 with a single nearest-even rounding, done on the double itself:
 * normal range: keep 7 explicit mantissa bits of the double; below 2^-126 the bf16
 * grid is the fixed subnormal spacing 2^-133. */
static uint16_t f64_to_bf16_rne(double d) {
  if (d != d) return 0x7FC0u;
  const double a = fabs(d);
  double r;
  if (a < 0x1p-126) {
    r = nearbyint(a * 0x1p133) * 0x1p-133;
  } else if (isinf(a)) {
    r = a;
  } else {
    uint64_t u;
    memcpy(&u, &a, 8);
    const uint64_t lsb = (u >> 45) & 1ull;
    u += ((1ull << 44) - 1ull) + lsb;
    u &= ~((1ull << 45) - 1ull);
    memcpy(&r, &u, 8);
  }
  const float f = (float)r; /* exact, or +inf when r reached 2^128 */
  uint32_t v;
  memcpy(&v, &f, 4);
  uint16_t h = (uint16_t)(v >> 16);
  if (signbit(d)) h |= 0x8000u;
  return h;
}

/* ---- Layout + Notify (Section 5.2; eq. for c^rank, c^exp, s; Section 5.1 rule row = o + s) */

int moe_ref_plan(int32_t T, int32_t k, int32_t E, int32_t R, int64_t region_stride_rows,
                 const int32_t *K,          /* [T*k]  routing ids */
                 int32_t *c_exp,            /* [E]    out */
                 int32_t *c_rank,           /* [R]    out */
                 int32_t *expert_offset,    /* [E+1]  out: o */
                 int32_t *region_base,      /* [R+1]  out */
                 int32_t *s,                /* [T*k]  out: small offset, -1 if skipped */
                 int32_t *row_map,          /* [T*k]  out: o[K] + s, -1 if skipped/dropped */
                 int32_t *status)           /* [2]    out: {#invalid ids, #dropped for capacity} */
{
  if (T < 0 || k < 1 || E < 1 || R < 1 || E % R != 0) return -2;
  const int32_t Er = E / R;
  status[0] = 0;
  status[1] = 0;
  status[2] = 0;   /* only several sources can outgrow int32 rows: T*k itself is int32 */
  for (int32_t e = 0; e < E; ++e) c_exp[e] = 0;

  /* Layout: running per-expert counter == number of earlier branches with the same expert */
  for (int32_t t = 0; t < T; ++t) {
    for (int32_t j = 0; j < k; ++j) {
      const int64_t i = (int64_t)t * k + j;
      const int32_t e = K[i];
      if (e == -1) { s[i] = -1; continue; }
      if (e < 0 || e >= E) { status[0] += 1; s[i] = -1; continue; }
      s[i] = c_exp[e];
      c_exp[e] += 1;
    }
  }
  /* destination rank of expert e is floor(e / E_r) */
  for (int32_t r = 0; r < R; ++r) {
    int32_t acc = 0;
    for (int32_t e = r * Er; e < (r + 1) * Er; ++e) acc += c_exp[e];
    c_rank[r] = acc;
  }
  /* Notify, single source rank: region bases, then expert blocks inside each region */
  region_base[0] = 0;
  for (int32_t r = 0; r < R; ++r) {
    if (region_stride_rows > 0) region_base[r + 1] = (int32_t)((int64_t)(r + 1) * region_stride_rows);
    else region_base[r + 1] = region_base[r] + c_rank[r];
  }
  for (int32_t r = 0; r < R; ++r) {
    int32_t run = region_base[r];
    for (int32_t e = r * Er; e < (r + 1) * Er; ++e) {
      expert_offset[e] = run;
      run += c_exp[e];
    }
  }
  expert_offset[E] = expert_offset[E - 1] + c_exp[E - 1];
  /* two-level rule */
  for (int64_t i = 0; i < (int64_t)T * k; ++i) {
    if (s[i] < 0) { row_map[i] = -1; continue; }
    const int32_t e = K[i];
    const int32_t row = expert_offset[e] + s[i];
    if (region_stride_rows > 0 && row >= region_base[e / Er + 1]) {
      status[1] += 1;
      row_map[i] = -1;
    } else {
      row_map[i] = row;
    }
  }
  return 0;
}

/* ---- Notify with several source ranks (Section 5.2 "Prefill Notify"; Section 5.1 definition of o_{e,r}) ----
 *
 * M[r][e] = routed branches that source rank r sends to expert e (the gathered count matrix, recvData).
 * This rank is source rank `me`; its row of M is replaced by the counts computed from its own K.
 * The window of destination rank d holds the blocks of its experts in expert order, and inside an
 * expert's block the sub-blocks of the source ranks in rank order; o_{e,r} is where sub-block (e,r)
 * starts.  Walking (d, e, r) in that order with one running row counter IS the definition.
 * Outputs beyond moe_ref_plan's:
 *   o_all[e*R + r] = o_{e,r} for every source (tests check that the sub-blocks tile the window);
 *   recv_count[e]  = sum_r M[r][e]   (n^exp: rows of expert e's whole block);
 *   recv_offset[e] = first row of expert e's whole block; [E] = end of the last block.
 * expert_offset[e] = o_{e,me}; row_map = o_{e,me} + s.  With a fixed region stride, region d starts at
 * d*stride and a branch whose row falls at or past (d+1)*stride is dropped and counted in status[1].
 * Rows are int32.  If the blocks of all sources together hold 2^31 rows or more, the layout cannot be
 * expressed: status = {invalid ids, 0, 1}, no branch is placed (row_map = -1 everywhere) and the offset
 * tables are zeroed (their content is unspecified for callers); counts and s are still those of Layout.
 */
int moe_ref_plan_multi(int32_t T, int32_t k, int32_t E, int32_t R, int64_t region_stride_rows, int32_t me,
                       const int32_t *K, const int32_t *M /* [R*E], row `me` ignored */,
                       int32_t *c_exp, int32_t *c_rank, int32_t *expert_offset, int32_t *region_base,
                       int32_t *s, int32_t *row_map, int32_t *status,
                       int32_t *o_all /* [E*R] */, int32_t *recv_count /* [E] */, int32_t *recv_offset /* [E+1] */)
{
  if (T < 0 || k < 1 || E < 1 || R < 1 || E % R != 0 || me < 0 || me >= R) return -2;
  const int32_t Er = E / R;
  status[0] = 0;
  status[1] = 0;
  for (int32_t e = 0; e < E; ++e) c_exp[e] = 0;
  /* Layout: identical to the single-source case */
  for (int64_t i = 0; i < (int64_t)T * k; ++i) {
    const int32_t e = K[i];
    if (e == -1) { s[i] = -1; continue; }
    if (e < 0 || e >= E) { status[0] += 1; s[i] = -1; continue; }
    s[i] = c_exp[e];
    c_exp[e] += 1;
  }
  for (int32_t r = 0; r < R; ++r) {
    int32_t acc = 0;
    for (int32_t e = r * Er; e < (r + 1) * Er; ++e) acc += c_exp[e];
    c_rank[r] = acc;
  }
  status[2] = 0;
  int64_t all_rows = 0;
  for (int32_t e = 0; e < E; ++e)
    for (int32_t r = 0; r < R; ++r) all_rows += r == me ? c_exp[e] : M[(int64_t)r * E + e];
  if (all_rows >= 2147483648LL) {
    status[2] = 1;
    for (int64_t i = 0; i < (int64_t)T * k; ++i) row_map[i] = -1;
    for (int32_t e = 0; e <= E; ++e) expert_offset[e] = recv_offset[e] = 0;
    for (int32_t e = 0; e < E; ++e) recv_count[e] = 0;
    for (int64_t x = 0; x < (int64_t)E * R; ++x) o_all[x] = 0;
    for (int32_t d = 0; d <= R; ++d) region_base[d] = 0;
    return 0;
  }
  /* Notify: one running row counter over (destination rank, expert, source rank) */
  int32_t run = 0;
  for (int32_t d = 0; d < R; ++d) {
    if (region_stride_rows > 0) run = (int32_t)((int64_t)d * region_stride_rows);
    region_base[d] = run;
    for (int32_t e = d * Er; e < (d + 1) * Er; ++e) {
      recv_offset[e] = run;
      int32_t n = 0;
      for (int32_t r = 0; r < R; ++r) {
        const int32_t m = r == me ? c_exp[e] : M[(int64_t)r * E + e];
        o_all[(int64_t)e * R + r] = run;
        run += m;
        n += m;
      }
      recv_count[e] = n;
      expert_offset[e] = o_all[(int64_t)e * R + me];
    }
  }
  recv_offset[E] = run;
  expert_offset[E] = run;
  region_base[R] = region_stride_rows > 0 ? (int32_t)((int64_t)R * region_stride_rows) : run;
  for (int64_t i = 0; i < (int64_t)T * k; ++i) {
    if (s[i] < 0) { row_map[i] = -1; continue; }
    const int32_t e = K[i];
    const int32_t row = expert_offset[e] + s[i];
    if (region_stride_rows > 0 && row >= (int32_t)((int64_t)(e / Er + 1) * region_stride_rows)) {
      status[1] += 1;
      row_map[i] = -1;
    } else {
      row_map[i] = row;
    }
  }
  return 0;
}

/* ---- Dispatch (Algorithm 1, first loop; Section 5.2 "Prefill Dispatch") ---- */

int moe_ref_dispatch(int32_t T, int32_t H, int32_t k, int32_t elem_bytes,
                     const void *X,             /* [T, H] */
                     const int32_t *row_map,    /* [T*k]  */
                     void *window)              /* [rows, H]; only mapped rows are written */
{
  const size_t row_bytes = (size_t)H * (size_t)elem_bytes;
  TOKENS_IN_PARALLEL
  for (int32_t t = 0; t < T; ++t) {
    for (int32_t j = 0; j < k; ++j) {
      const int32_t p = row_map[(int64_t)t * k + j];
      if (p < 0) continue;
      memcpy((char *)window + (size_t)p * row_bytes, (const char *)X + (size_t)t * row_bytes, row_bytes);
    }
  }
  return 0;
}

/* ---- Combine (Algorithm 1, second loop; Section 5.2 "Prefill Combine") ----- */

int moe_ref_combine(int32_t T, int32_t H, int32_t k, int32_t dtype,
                    const void *Yexp,          /* [rows, H] expert outputs, window layout */
                    const float *W,            /* [T*k] gate weights */
                    const int32_t *row_map,    /* [T*k] */
                    void *Y)                   /* [T, H] out */
{
  if (dtype != MOE_REF_BF16 && dtype != MOE_REF_F32) return -2;
  TOKENS_IN_PARALLEL
  for (int32_t t = 0; t < T; ++t) {
    for (int32_t h = 0; h < H; ++h) {
      float acc = 0.0f;
      for (int32_t j = 0; j < k; ++j) {
        const int32_t q = row_map[(int64_t)t * k + j];
        if (q < 0) continue;
        const size_t idx = (size_t)q * (size_t)H + (size_t)h;
        const float y = dtype == MOE_REF_BF16 ? bf16_to_f32(((const uint16_t *)Yexp)[idx])
                                              : ((const float *)Yexp)[idx];
        acc = fmaf(W[(int64_t)t * k + j], y, acc);
      }
      const size_t o = (size_t)t * (size_t)H + (size_t)h;
      if (dtype == MOE_REF_BF16) ((uint16_t *)Y)[o] = f32_to_bf16_rne(acc);
      else ((float *)Y)[o] = acc;
    }
  }
  return 0;
}

/* Same sum carried in fp64 (each product of an fp32 weight and a bf16/fp32 value is
 * exact in fp64), rounded once to the storage type: the mathematical value of the
 * combine equation, used to bound the fp32 path. */
int moe_ref_combine_f64(int32_t T, int32_t H, int32_t k, int32_t dtype, const void *Yexp,
                        const float *W, const int32_t *row_map, void *Y)
{
  if (dtype != MOE_REF_BF16 && dtype != MOE_REF_F32) return -2;
  for (int32_t t = 0; t < T; ++t) {
    for (int32_t h = 0; h < H; ++h) {
      double acc = 0.0;
      for (int32_t j = 0; j < k; ++j) {
        const int32_t q = row_map[(int64_t)t * k + j];
        if (q < 0) continue;
        const size_t idx = (size_t)q * (size_t)H + (size_t)h;
        const double y = dtype == MOE_REF_BF16 ? (double)bf16_to_f32(((const uint16_t *)Yexp)[idx])
                                               : (double)((const float *)Yexp)[idx];
        acc += (double)W[(int64_t)t * k + j] * y;
      }
      const size_t o = (size_t)t * (size_t)H + (size_t)h;
      if (dtype == MOE_REF_BF16) ((uint16_t *)Y)[o] = f64_to_bf16_rne(acc);
      else ((float *)Y)[o] = (float)acc;
    }
  }
  return 0;
}

/* ---- Stand-in for the expert FFNs (not part of the method) -----------------
 * Yexp[row] = round(f32(window[row]) * scale[e]) for the row of every placed branch
 * routed to expert e.  The real FFNs need trained weights; a per-expert scalar keeps
 * rows attributable to their expert. */
int moe_ref_expert_standin(int32_t T, int32_t H, int32_t k, int32_t dtype, const int32_t *K,
                           const int32_t *row_map, const float *scale, const void *window, void *Yexp)
{
  if (dtype != MOE_REF_BF16 && dtype != MOE_REF_F32) return -2;
  for (int64_t i = 0; i < (int64_t)T * k; ++i) {
    const int32_t row = row_map[i];
    if (row < 0) continue;
    const float sc = scale[K[i]];
    for (int32_t h = 0; h < H; ++h) {
      const size_t idx = (size_t)row * (size_t)H + (size_t)h;
      if (dtype == MOE_REF_BF16) {
        const float v = bf16_to_f32(((const uint16_t *)window)[idx]) * sc;
        ((uint16_t *)Yexp)[idx] = f32_to_bf16_rne(v);
      } else {
        ((float *)Yexp)[idx] = ((const float *)window)[idx] * sc;
      }
    }
  }
  return 0;
}

/* ---- Row-wise quantised dispatch (Section 5.2, last sentences of "Prefill Dispatch") -------------------
 *
 * The paper fixes only where the scales live: one per quantised row, in an array of their own that is
 * indexed like the window rows.  It gives no format.  Format chosen here (parity with the authors: unpinned):
 *   payload  OCP FP8 E4M3 (1-4-3 bits, bias 7, largest finite 448, no infinities, NaN = S.1111.111);
 *   amax   = max_h |x_h| over the row (as fp32);   scale = amax / 448   (stored, fp32, one rounding);
 *   inv    = 448 / amax (fp32, one rounding);      q_h = e4m3(x_h * inv), nearest-even, saturating at 448;
 *   amax == 0  ->  scale = 1, inv = 1.
 * The token row is quantised once and the same bytes and scale go to each of its k destination rows.
 */
static uint8_t f32_to_e4m3_rne_sat(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  const uint8_t sign = (uint8_t)((u >> 24) & 0x80u);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint8_t)(sign | 0x7Fu);
  const float a = fabsf(f);
  if (a >= 448.0f) return (uint8_t)(sign | 0x7Eu);              /* saturate (also covers +-inf) */
  if (a < 0x1p-6f) return (uint8_t)(sign | (uint8_t)nearbyintf(a * 0x1p9f)); /* subnormal grid 2^-9; 8 -> 2^-6 */
  uint32_t v;
  memcpy(&v, &a, 4);
  const uint32_t lsb = (v >> 20) & 1u;                          /* keep 3 mantissa bits */
  v += 0x7FFFFu + lsb;
  v >>= 20;                                                     /* [exponent(8) | mantissa(3)], carry included */
  const uint32_t code = v - ((127u - 7u) << 3);                 /* rebias 127 -> 7 */
  return (uint8_t)(sign | (code > 0x7Eu ? 0x7Eu : code));
}

int moe_ref_dispatch_quant(int32_t T, int32_t H, int32_t k,
                           const uint16_t *X,          /* [T, H] bf16 */
                           const int32_t *row_map,     /* [T*k] */
                           uint8_t *window_q,          /* [rows, H] e4m3; only mapped rows are written */
                           float *window_scale)        /* [rows] */
{
  for (int32_t t = 0; t < T; ++t) {
    const uint16_t *x = X + (size_t)t * (size_t)H;
    float amax = 0.0f;
    for (int32_t h = 0; h < H; ++h) amax = fmaxf(amax, fabsf(bf16_to_f32(x[h])));
    const float scale = amax == 0.0f ? 1.0f : amax / 448.0f;
    const float inv = amax == 0.0f ? 1.0f : 448.0f / amax;
    for (int32_t j = 0; j < k; ++j) {
      const int32_t p = row_map[(int64_t)t * k + j];
      if (p < 0) continue;
      uint8_t *q = window_q + (size_t)p * (size_t)H;
      for (int32_t h = 0; h < H; ++h) q[h] = f32_to_e4m3_rne_sat(bf16_to_f32(x[h]) * inv);
      window_scale[p] = scale;
    }
  }
  return 0;
}

void moe_ref_f32_to_e4m3(const float *in, uint8_t *out, int64_t n) {
  for (int64_t i = 0; i < n; ++i) out[i] = f32_to_e4m3_rne_sat(in[i]);
}

/* storage conversions, exported so tests can pin them against an independent library */
void moe_ref_f32_to_bf16(const float *in, uint16_t *out, int64_t n) {
  for (int64_t i = 0; i < n; ++i) out[i] = f32_to_bf16_rne(in[i]);
}
void moe_ref_f64_to_bf16(const double *in, uint16_t *out, int64_t n) {
  for (int64_t i = 0; i < n; ++i) out[i] = f64_to_bf16_rne(in[i]);
}
