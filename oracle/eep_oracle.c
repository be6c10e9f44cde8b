/*
 * eep_oracle.c -- plain, slow, serial CPU statement of what one dispatch/combine
 * step with explicit membership computes.
 *
 * THIS IS TEST INFRASTRUCTURE.  It exists to check the GPU library; nothing in
 * the product path may call it.  It shares no code, header, table or helper
 * with the HIP sources: every format rule (bf16, e4m3) is restated here.
 *
 * Each function is one step of the path, written as the definition itself:
 * running sums instead of scans, one loop per pair, no tiling, no threads.
 * Floating point: the combine accumulates in double (the paper fixes no
 * precision; Sec. 4.1 only says the combine "reduces expert outputs"); a
 * second variant, eeo_combine_chain32, follows the fp32 reading documented
 * for the GPU kernel (one fused multiply-add per term, ascending j).
 *
 * Paper anchors
 *   tables      Sec. 5.1: metadata maps every physical slot to a logical expert
 *               and records all physical locations of each logical expert.
 *   map         Fig. 7 (dispatch path): a peer whose `active` is 0 is skipped;
 *               Sec. 3.2 validity contract (1)-(3); Fig. 5 worked example.
 *   layout      Sec. 4.1: payload placement follows prior work (contiguous
 *               per-expert receive buffers); ordering inside a slot is by
 *               ascending token (the order a receiver of per-source-rank
 *               batches would see).
 *   combine     Sec. 4.1: reduce the expert outputs per token, weighted by the
 *               router weights (Sec. 2.1).
 *   detection   Sec. 3.4 and Sec. 4.1: a peer whose signal does not arrive
 *               within the time-out is dropped by the waiting kernel.
 *
 * Readings where the paper is silent:
 *   - canonical replica order: primary slots first, then ascending slot id;
 *   - selection: FIRST_LIVE (sel = 0) or SPREAD (sel = t mod n_live);
 *   - an index outside [0,E), or one that repeats an earlier index of the
 *     same token, is "masked"; an expert with no live replica is "uncovered";
 *     both are dropped from dispatch and contribute nothing to combine.
 *
 * Parity pins: see tests/test_oracle_*.py (Fig. 5 golden, invariants,
 * numpy stable-argsort/bincount/cumsum, closed forms, torch dtype casts).
 * Unpinned by the paper itself: the SPREAD rule (the paper gives none).
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

/* ---------- number formats ------------------------------------------------ */

/* bfloat16 = the upper 16 bits of an IEEE binary32. */
float eeo_bf16_to_f32(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

/* binary32 -> bfloat16, round to nearest, ties to even; NaN stays NaN. */
uint16_t eeo_f32_to_bf16(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
  uint32_t lower = u & 0xffffu;
  uint32_t upper = u >> 16;
  if (lower > 0x8000u || (lower == 0x8000u && (upper & 1u))) upper += 1u;
  return (uint16_t)upper;
}

/* OCP FP8 E4M3 ("e4m3fn"): 1 sign, 4 exponent (bias 7), 3 mantissa bits;
 * no infinities; S.1111.111 is NaN; largest finite value 448. */
float eeo_e4m3_to_f32(uint8_t q) {
  int sign = q >> 7;
  int ex = (q >> 3) & 0xf;
  int man = q & 0x7;
  double v;
  if (ex == 0xf && man == 0x7) return NAN;
  if (ex == 0) v = ldexp((double)man / 8.0, -6);
  else v = ldexp(1.0 + (double)man / 8.0, ex - 7);
  return (float)(sign ? -v : v);
}

/* binary32 -> e4m3fn code: nearest representable value, ties to the even code,
 * magnitudes of 448 and above saturate to 448 (0x7e); NaN -> 0x7f.
 * Written from the format's definition: find the binade with frexp, count
 * eighths of the binade (or 2^-9 steps below 2^-6), round with nearbyint. */
uint8_t eeo_f32_to_e4m3(float f) {
  uint8_t sign = signbit(f) ? 0x80 : 0x00;
  if (isnan(f)) return sign | 0x7f;
  double mag = fabs((double)f);
  if (mag >= 448.0) return sign | 0x7e;
  if (mag < ldexp(1.0, -6)) {
    int n = (int)nearbyint(mag * 512.0); /* steps of 2^-9; 8 steps = 2^-6, code 0x08 */
    return sign | (uint8_t)n;
  }
  int ex;
  (void)frexp(mag, &ex); /* mag = m * 2^ex, m in [0.5, 1) */
  int E = ex - 1;        /* mag = (1 + frac) * 2^E */
  int n = (int)nearbyint((mag / ldexp(1.0, E) - 1.0) * 8.0);
  if (n == 8) { n = 0; E += 1; }
  int code = ((E + 7) << 3) | n;
  if (code > 0x7e) code = 0x7e;
  return sign | (uint8_t)code;
}

/* Quantise-on-dispatch variant: per token and per `group` channels,
 * scale = max|x| / 448 in binary32 (1 if all zero), code = e4m3(x / scale) with
 * the division in binary32.  x: bf16 [T,H] -> q: codes [T,H], scale [T,H/group]. */
void eeo_quantize_e4m3(int T, int H, int group, const uint16_t* x, uint8_t* q, float* scale) {
  int G = H / group;
  for (int t = 0; t < T; ++t)
    for (int g = 0; g < G; ++g) {
      float amax = 0.0f;
      for (int c = 0; c < group; ++c) {
        float v = fabsf(eeo_bf16_to_f32(x[(int64_t)t * H + g * group + c]));
        if (v > amax) amax = v;
      }
      float sc = amax / 448.0f;
      if (sc == 0.0f) sc = 1.0f;
      scale[(int64_t)t * G + g] = sc;
      for (int c = 0; c < group; ++c) {
        int64_t i = (int64_t)t * H + g * group + c;
        q[i] = eeo_f32_to_e4m3(eeo_bf16_to_f32(x[i]) / sc);
      }
    }
}

/* ---------- O1: expert-location metadata ------------------------------------
 * p2l[P]: logical expert of each physical slot p = r*S + s (-1 = empty).
 * Output: for each logical expert e the list of its replicas in canonical
 * order, as CSR (l2p_off[E+1], l2p_list[P]); unused tail of l2p_list = -1.
 * Returns 0, or -1 if an entry is outside [-1, E). */
int eeo_tables(int P, int E, int S, int S_prim, const int32_t* p2l, int32_t* l2p_off,
               int32_t* l2p_list) {
  for (int p = 0; p < P; ++p)
    if (p2l[p] < -1 || p2l[p] >= E) return -1;
  int n = 0;
  for (int e = 0; e < E; ++e) {
    l2p_off[e] = n;
    for (int redundant = 0; redundant <= 1; ++redundant)
      for (int p = 0; p < P; ++p)
        if (p2l[p] == e && ((p % S) >= S_prim) == redundant) l2p_list[n++] = p;
  }
  l2p_off[E] = n;
  for (int i = n; i < P; ++i) l2p_list[i] = -1;
  return 0;
}

/* Validity condition 2 (Sec. 3.2): number of logical experts that have no
 * replica on an active rank. */
int eeo_uncovered_experts(int P, int E, int S, const int32_t* p2l, const int32_t* active) {
  int missing = 0;
  for (int e = 0; e < E; ++e) {
    int live = 0;
    for (int p = 0; p < P; ++p)
      if (p2l[p] == e && active[p / S] != 0) live = 1;
    if (!live) ++missing;
  }
  return missing;
}

/* ---------- O2: map every (token, j) to a live replica slot -----------------
 * policy: 0 = SPREAD, 1 = FIRST_LIVE.  counters[0] = uncovered pairs,
 * counters[1] = masked pairs. */
void eeo_map(int T, int k, int E, int S, int policy, const int32_t* topk_idx,
             const int32_t* l2p_off, const int32_t* l2p_list, const int32_t* active,
             int32_t* slot_of, int64_t* counters) {
  int64_t n_uncovered = 0, n_masked = 0;
  for (int t = 0; t < T; ++t) {
    for (int j = 0; j < k; ++j) {
      int e = topk_idx[t * k + j];
      int32_t* dst = &slot_of[t * k + j];
      *dst = -1;
      if (e < 0 || e >= E) { ++n_masked; continue; }
      int repeated = 0;
      for (int jj = 0; jj < j; ++jj)
        if (topk_idx[t * k + jj] == e) repeated = 1;
      if (repeated) { ++n_masked; continue; }
      int n_live = 0;
      for (int q = l2p_off[e]; q < l2p_off[e + 1]; ++q)
        if (active[l2p_list[q] / S] != 0) ++n_live;
      if (n_live == 0) { ++n_uncovered; continue; }
      int sel = (policy == 1) ? 0 : (t % n_live);
      int seen = 0;
      for (int q = l2p_off[e]; q < l2p_off[e + 1]; ++q) {
        int p = l2p_list[q];
        if (active[p / S] == 0) continue; /* skip failed peer (Fig. 7) */
        if (seen == sel) { *dst = p; break; }
        ++seen;
      }
    }
  }
  counters[0] = n_uncovered;
  counters[1] = n_masked;
}

/* ---------- O3-O5: counts, offsets, stable positions ------------------------
 * count[P], rank_count[R], cnt_src[R*P] (source rank b = t / (T/R)),
 * offset[P+1], rank_offset[R+1], row_of[T*k] (-1 if not routed),
 * src_of[T*k] (-1 for rows >= N).  T must be a multiple of R (or 0). */
void eeo_layout(int T, int k, int R, int S, const int32_t* slot_of, int32_t* count,
                int32_t* rank_count, int32_t* cnt_src, int32_t* offset, int32_t* rank_offset,
                int32_t* row_of, int32_t* src_of, int32_t* cursor /* scratch [P] */) {
  int P = R * S;
  int per_rank = (R > 0 && T > 0) ? T / R : 1;
  for (int p = 0; p < P; ++p) count[p] = 0;
  for (int i = 0; i < R * P; ++i) cnt_src[i] = 0;
  for (int t = 0; t < T; ++t)
    for (int j = 0; j < k; ++j) {
      int p = slot_of[t * k + j];
      if (p < 0) continue;
      count[p] += 1;
      cnt_src[(t / per_rank) * P + p] += 1;
    }
  for (int r = 0; r < R; ++r) {
    rank_count[r] = 0;
    for (int s = 0; s < S; ++s) rank_count[r] += count[r * S + s];
  }
  offset[0] = 0;
  for (int p = 0; p < P; ++p) offset[p + 1] = offset[p] + count[p];
  for (int r = 0; r < R; ++r) rank_offset[r] = offset[r * S];
  rank_offset[R] = offset[P];
  for (int p = 0; p < P; ++p) cursor[p] = offset[p];
  for (int i = 0; i < T * k; ++i) src_of[i] = -1;
  for (int t = 0; t < T; ++t)
    for (int j = 0; j < k; ++j) {
      int p = slot_of[t * k + j];
      if (p < 0) { row_of[t * k + j] = -1; continue; }
      int row = cursor[p]++;
      row_of[t * k + j] = row;
      src_of[row] = t * k + j;
    }
}

/* ---------- O6: pack -------------------------------------------------------
 * recv[row_of[t,j]] = x[t] as raw bytes (any dtype; also used for the scale
 * rows of fp8 payloads).  Rows that receive nothing are left as they were. */
void eeo_pack(int T, int k, int64_t row_bytes, const uint8_t* x, const int32_t* row_of,
              uint8_t* recv) {
  for (int t = 0; t < T; ++t)
    for (int j = 0; j < k; ++j) {
      int row = row_of[t * k + j];
      if (row < 0) continue;
      memcpy(recv + (int64_t)row * row_bytes, x + (int64_t)t * row_bytes, (size_t)row_bytes);
    }
}

/* ---------- de-duplicated dispatch (a data-path variant; the paper leaves
 * payload placement to prior work, Sec. 4.1) ---------------------------------
 * One row per (token, destination RANK) instead of one per (token, expert):
 * when several of a token's experts live on one rank the row travels once and
 * is expanded on the destination.
 *   dedup_count[r]  tokens with at least one routed pair on rank r
 *   dedup_offset    exclusive running sum over ranks; dedup_offset[R] = N_d
 *   dedup_row[t,j]  row of token t in rank r's part of the de-duplicated buffer,
 *                   r = slot_of[t,j] / S; token-ascending inside a rank; -1 for
 *                   pairs that are not routed
 *   lead[t,j]       1 for the first routed pair (lowest j) of token t on that
 *                   rank -- the pair that carries the row -- else 0
 *   expand_of[row]  for every row of the expert-major layout (row_of), the row of
 *                   the de-duplicated buffer that holds its token; -1 for rows >= N
 * seen: scratch [R]. */
void eeo_dedup_layout(int T, int k, int R, int S, const int32_t* slot_of, const int32_t* row_of,
                      int32_t* dedup_count, int32_t* dedup_offset, int32_t* dedup_row,
                      int32_t* lead, int32_t* expand_of, int32_t* seen) {
  for (int r = 0; r < R; ++r) dedup_count[r] = 0;
  for (int t = 0; t < T; ++t) {
    for (int r = 0; r < R; ++r) seen[r] = 0;
    for (int j = 0; j < k; ++j) {
      int p = slot_of[t * k + j];
      if (p < 0) continue;
      if (!seen[p / S]) { seen[p / S] = 1; dedup_count[p / S] += 1; }
    }
  }
  dedup_offset[0] = 0;
  for (int r = 0; r < R; ++r) dedup_offset[r + 1] = dedup_offset[r] + dedup_count[r];
  for (int i = 0; i < T * k; ++i) expand_of[i] = -1;
  /* cursor per rank, tokens ascending */
  for (int r = 0; r < R; ++r) seen[r] = dedup_offset[r];
  for (int t = 0; t < T; ++t) {
    for (int j = 0; j < k; ++j) {
      int p = slot_of[t * k + j];
      dedup_row[t * k + j] = -1;
      lead[t * k + j] = 0;
      if (p < 0) continue;
      int r = p / S, first = 1, at = -1;
      for (int jj = 0; jj < j; ++jj) {
        int q = slot_of[t * k + jj];
        if (q >= 0 && q / S == r) { first = 0; at = dedup_row[t * k + jj]; break; }
      }
      if (first) at = seen[r]++;
      dedup_row[t * k + j] = at;
      lead[t * k + j] = first;
      expand_of[row_of[t * k + j]] = at;
    }
  }
}

/* stage 1: recv_d[dedup_row[t,j]] = x[t] for the leading pair of every (token, rank) */
void eeo_pack_dedup(int T, int k, int64_t row_bytes, const uint8_t* x, const int32_t* dedup_row,
                    const int32_t* lead, uint8_t* recv_d) {
  for (int t = 0; t < T; ++t)
    for (int j = 0; j < k; ++j)
      if (lead[t * k + j])
        memcpy(recv_d + (int64_t)dedup_row[t * k + j] * row_bytes, x + (int64_t)t * row_bytes,
               (size_t)row_bytes);
}

/* stage 2, on the destination: recv[row] = recv_d[expand_of[row]] for rows < N */
void eeo_expand(int N, int64_t row_bytes, const uint8_t* recv_d, const int32_t* expand_of,
                uint8_t* recv) {
  for (int row = 0; row < N; ++row)
    memcpy(recv + (int64_t)row * row_bytes, recv_d + (int64_t)expand_of[row] * row_bytes,
           (size_t)row_bytes);
}

/* ---------- O7: expert stand-ins -------------------------------------------- */

/* Logical expert that owns receive row `row`: the slot whose [offset[p],
 * offset[p+1]) contains it. */
static int logical_of_row(int row, int P, const int32_t* offset, const int32_t* p2l) {
  for (int p = 0; p < P; ++p)
    if (row >= offset[p] && row < offset[p + 1]) return p2l[p];
  return -1;
}

/* y[row] = fl32(s[e(row)] * recv[row]) for rows < N; dtype 0 = f32, 1 = bf16
 * (then rounded to bf16).  The product of two binary32 values is exact in
 * double, so the cast to float rounds once. */
void eeo_stub_scale(int N, int H, int P, int dtype, const void* recv, const int32_t* offset,
                    const int32_t* p2l, const float* expert_scale, void* y) {
  for (int row = 0; row < N; ++row) {
    int e = logical_of_row(row, P, offset, p2l);
    float s = expert_scale[e];
    for (int h = 0; h < H; ++h) {
      int64_t i = (int64_t)row * H + h;
      if (dtype == 0) {
        ((float*)y)[i] = (float)((double)s * (double)((const float*)recv)[i]);
      } else {
        float v = eeo_bf16_to_f32(((const uint16_t*)recv)[i]);
        ((uint16_t*)y)[i] = eeo_f32_to_bf16((float)((double)s * (double)v));
      }
    }
  }
}

/* y[row,h] = bf16(fl32(e4m3(q[row,h]) * scale[row, h / group])) for rows < N. */
void eeo_stub_dequant(int N, int H, int group, const uint8_t* q, const float* scale,
                      uint16_t* y) {
  int G = H / group;
  for (int row = 0; row < N; ++row)
    for (int h = 0; h < H; ++h) {
      float v = eeo_e4m3_to_f32(q[(int64_t)row * H + h]);
      float sc = scale[(int64_t)row * G + h / group];
      y[(int64_t)row * H + h] = eeo_f32_to_bf16((float)((double)v * (double)sc));
    }
}

/* ---------- failure detection from the GPU side (Sec. 3.4; Sec. 4.1, the
 * paragraph on per-rank signal counters; the time-out remark in Fig. 7) --------
 * One round of waiting, seen from the combine side of a step whose routing
 * (slot_of, row_of) was made under the mask active[R]:
 *   arrived[r] != 0  rank r's signal for this round came within the time-out.
 * A side waits for the arrivals it EXPECTS from the active peer set (Sec. 3.4):
 * the ranks that hold rows of this step.  A rank that is not active, or from
 * which nothing is expected in this round, is not awaited.  An awaited rank
 * whose signal did not arrive is deemed failed: its active entry is cleared
 * (later steps route around it), it is put on the failure report that the host
 * reads after the step, and the pairs routed to it in this step contribute
 * nothing (their requests are failed, Sec. 3.1): their row_of entry becomes -1
 * so that the combine skips them.  Arrays are updated in place; report[R] is
 * written (1 = dropped now).  Returns the number of pairs withdrawn. */
int64_t eeo_detect_round(int T, int k, int R, int S, const int32_t* slot_of,
                         const int32_t* arrived, int32_t* active, int32_t* report,
                         int32_t* row_of) {
  for (int r = 0; r < R; ++r) {
    report[r] = 0;
    if (active[r] == 0) continue; /* not awaited */
    int expected = 0;             /* rows of this step that rank r holds */
    for (int i = 0; i < T * k; ++i)
      if (slot_of[i] >= 0 && row_of[i] >= 0 && slot_of[i] / S == r) ++expected;
    if (expected == 0) continue;  /* nothing to wait for in this round */
    if (arrived[r] != 0) continue;
    active[r] = 0;
    report[r] = 1;
  }
  int64_t withdrawn = 0;
  for (int i = 0; i < T * k; ++i) {
    int p = slot_of[i];
    if (p < 0 || row_of[i] < 0) continue;
    if (report[p / S]) {
      row_of[i] = -1;
      ++withdrawn;
    }
  }
  return withdrawn;
}

/* ---------- O8: combine ------------------------------------------------------
 * out[t,h] = sum_j w[t,j] * y[row_of[t,j], h] over routed pairs, in double.
 * y_dtype: 0 = f32, 1 = bf16. */
void eeo_combine(int T, int k, int H, int y_dtype, const void* y, const float* w,
                 const int32_t* row_of, double* out) {
  for (int t = 0; t < T; ++t)
    for (int h = 0; h < H; ++h) {
      double acc = 0.0;
      for (int j = 0; j < k; ++j) {
        int row = row_of[t * k + j];
        if (row < 0) continue;
        int64_t i = (int64_t)row * H + h;
        double v = (y_dtype == 0) ? (double)((const float*)y)[i]
                                  : (double)eeo_bf16_to_f32(((const uint16_t*)y)[i]);
        acc += (double)w[t * k + j] * v;
      }
      out[(int64_t)t * H + h] = acc;
    }
}

/* The fp32 reading of the same sum: acc = fmaf(w_j, y_j, acc), j ascending,
 * from 0.0f.  Lets a test ask for bit equality with an fp32 kernel that keeps
 * this order. */
void eeo_combine_chain32(int T, int k, int H, int y_dtype, const void* y, const float* w,
                         const int32_t* row_of, float* out) {
  for (int t = 0; t < T; ++t)
    for (int h = 0; h < H; ++h) {
      float acc = 0.0f;
      for (int j = 0; j < k; ++j) {
        int row = row_of[t * k + j];
        if (row < 0) continue;
        int64_t i = (int64_t)row * H + h;
        float v = (y_dtype == 0) ? ((const float*)y)[i]
                                 : eeo_bf16_to_f32(((const uint16_t*)y)[i]);
        acc = fmaf(w[t * k + j], v, acc);
      }
      out[(int64_t)t * H + h] = acc;
    }
}

/* Array forms of the scalar conversions, for the pinning tests. */
void eeo_bf16_to_f32_array(int64_t n, const uint16_t* in, float* out) {
  for (int64_t i = 0; i < n; ++i) out[i] = eeo_bf16_to_f32(in[i]);
}
void eeo_f32_to_bf16_array(int64_t n, const float* in, uint16_t* out) {
  for (int64_t i = 0; i < n; ++i) out[i] = eeo_f32_to_bf16(in[i]);
}
void eeo_f32_to_e4m3_array(int64_t n, const float* in, uint8_t* out) {
  for (int64_t i = 0; i < n; ++i) out[i] = eeo_f32_to_e4m3(in[i]);
}
void eeo_e4m3_to_f32_array(int64_t n, const uint8_t* in, float* out) {
  for (int64_t i = 0; i < n; ++i) out[i] = eeo_e4m3_to_f32(in[i]);
}
