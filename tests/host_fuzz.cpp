// Fuzz driver for a CPU-only AddressSanitizer + UBSan build (tests/test_host_sanitizers.py):
// the library's host logic (planners, replica lists, coverage check, tiling) and the C oracle
// run on thousands of small random instances; every index they produce is checked, and the
// two implementations of the replica lists and of the coverage count are compared.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

#include "eep.h"

extern "C" {  // oracle/eep_oracle.c
int eeo_tables(int P, int E, int S, int S_prim, const int32_t* p2l, int32_t* l2p_off, int32_t* l2p_list);
int eeo_uncovered_experts(int P, int E, int S, const int32_t* p2l, const int32_t* active);
void eeo_map(int T, int k, int E, int S, int policy, const int32_t* topk_idx, const int32_t* l2p_off,
             const int32_t* l2p_list, const int32_t* active, int32_t* slot_of, int64_t* counters);
void eeo_layout(int T, int k, int R, int S, const int32_t* slot_of, int32_t* count, int32_t* rank_count,
                int32_t* cnt_src, int32_t* offset, int32_t* rank_offset, int32_t* row_of, int32_t* src_of,
                int32_t* cursor);
void eeo_pack(int T, int k, int64_t row_bytes, const uint8_t* x, const int32_t* row_of, uint8_t* recv);
void eeo_combine_chain32(int T, int k, int H, int y_dtype, const void* y, const float* w,
                         const int32_t* row_of, float* out);
int64_t eeo_detect_round(int T, int k, int R, int S, const int32_t* slot_of, const int32_t* arrived,
                         int32_t* active, int32_t* report, int32_t* row_of);
void eeo_combine(int T, int k, int H, int y_dtype, const void* y, const float* w, const int32_t* row_of,
                 double* out);
void eeo_dedup_layout(int T, int k, int R, int S, const int32_t* slot_of, const int32_t* row_of,
                      int32_t* dedup_count, int32_t* dedup_offset, int32_t* dedup_row, int32_t* lead,
                      int32_t* expand_of, int32_t* seen);
void eeo_pack_dedup(int T, int k, int64_t row_bytes, const uint8_t* x, const int32_t* dedup_row,
                    const int32_t* lead, uint8_t* recv_d);
void eeo_expand(int N, int64_t row_bytes, const uint8_t* recv_d, const int32_t* expand_of, uint8_t* recv);
void eeo_stub_scale(int N, int H, int P, int dtype, const void* recv, const int32_t* offset,
                    const int32_t* p2l, const float* expert_scale, void* y);
void eeo_stub_dequant(int N, int H, int group, const uint8_t* q, const float* scale, uint16_t* y);
void eeo_quantize_e4m3(int T, int H, int group, const uint16_t* x, uint8_t* q, float* scale);
void eeo_bf16_to_f32_array(int64_t n, const uint16_t* in, float* out);
void eeo_f32_to_bf16_array(int64_t n, const float* in, uint16_t* out);
void eeo_f32_to_e4m3_array(int64_t n, const float* in, uint8_t* out);
void eeo_e4m3_to_f32_array(int64_t n, const uint8_t* in, float* out);
}

#define REQUIRE(cond)                                                   \
  do {                                                                  \
    if (!(cond)) {                                                      \
      std::printf("FAILED line %d iteration %d: %s\n", __LINE__, it, #cond); \
      return 1;                                                         \
    }                                                                   \
  } while (0)

int main(int argc, char** argv) {
  const int iterations = argc > 1 ? std::atoi(argv[1]) : 5000;
  std::mt19937 rng(7);
  for (int it = 0; it < iterations; ++it) {
    const int R = 1 + rng() % 9, S = 1 + rng() % 5, Sp = rng() % (S + 1), P = R * S;
    const int E = 1 + rng() % (P + 4);
    std::vector<int32_t> cur(P), act(R), nw(P), kind(P), src(P), off(E + 1), lst(P), off2(E + 1), lst2(P);
    std::vector<float> load(E);
    for (auto& v : cur) v = (int)(rng() % (E + 1)) - 1;
    for (auto& v : act) v = rng() % 4 != 0;
    for (auto& v : load) v = (float)(rng() % 5);
    int32_t sum[4];

    // planner: every output index in range, sources are what they claim to be
    int rc = eep_plan_repair(R, S, Sp, E, cur.data(), act.data(), it % 2 ? load.data() : nullptr,
                             nw.data(), kind.data(), src.data(), sum);
    REQUIRE(rc == EEP_OK || rc == EEP_ERR_COVERAGE);
    REQUIRE((rc == EEP_ERR_COVERAGE) == (sum[3] > 0));
    for (int p = 0; p < P; ++p) {
      REQUIRE(nw[p] >= -1 && nw[p] < E);
      REQUIRE(kind[p] >= EEP_SRC_NONE && kind[p] <= EEP_SRC_DRAM);
      if (kind[p] == EEP_SRC_PEER) REQUIRE(src[p] >= 0 && src[p] < P && act[src[p] / S] && cur[src[p]] == nw[p]);
      if (!act[p / S]) REQUIRE(nw[p] == cur[p] && kind[p] == EEP_SRC_NONE);
    }
    REQUIRE(eep_host_uncovered_experts(P, E, S, nw.data(), act.data()) == sum[3]);
    REQUIRE(eeo_uncovered_experts(P, E, S, nw.data(), act.data()) == sum[3]);

    // replica lists: library and oracle agree entry by entry
    REQUIRE(eep_host_replica_lists(P, E, S, Sp, nw.data(), off.data(), lst.data()) == EEP_OK);
    REQUIRE(eeo_tables(P, E, S, Sp, nw.data(), off2.data(), lst2.data()) == 0);
    REQUIRE(off == off2 && lst == lst2);

    // transition planner
    {
      std::vector<int32_t> tgt(P), wr(R), n2(P), k2(P), s2(P);
      int32_t sm[4];
      for (auto& v : tgt) v = (int)(rng() % (E + 1)) - 1;
      for (int r = 0; r < R; ++r) wr[r] = act[r] || rng() % 3 == 0;
      REQUIRE(eep_plan_transition(R, S, Sp, E, cur.data(), tgt.data(), act.data(), wr.data(), n2.data(),
                                  k2.data(), s2.data(), sm) == EEP_OK);
      for (int p = 0; p < P; ++p)
        if (k2[p] == EEP_SRC_PEER) REQUIRE(s2[p] >= 0 && s2[p] < P && act[s2[p] / S] && cur[s2[p]] == n2[p]);
      REQUIRE(sm[0] + sm[1] + sm[2] <= P);
    }

    // tiling: tiles cover T tokens, none larger than 128, none across two source ranks
    {
      int32_t tl[4];
      const int T = R * (int)(rng() % 700);
      REQUIRE(eep_host_tiling(T, R, tl) == EEP_OK);
      REQUIRE(tl[0] == T / R && tl[2] <= 128 && tl[1] * tl[2] >= tl[0] && (T == 0 || tl[3] == R * tl[1]));
    }

    // the oracle's step on a small batch: rows form a permutation of [0, N), packed bytes
    // come from the right token, a detection round withdraws exactly the dropped ranks' rows
    {
      const int k = 1 + rng() % 4, T = R * (int)(rng() % 5), H = 4;
      std::vector<int32_t> idx((size_t)T * k), slot((size_t)T * k), row((size_t)T * k), srcof((size_t)T * k);
      for (auto& v : idx) v = (int)(rng() % (E + 2)) - 1;   // includes -1 and E: masked
      int64_t counters[2];
      eeo_map(T, k, E, S, it % 2, idx.data(), off.data(), lst.data(), act.data(), slot.data(), counters);
      std::vector<int32_t> count(P), rcount(R), cnt_src((size_t)R * P), offset(P + 1), roff(R + 1), cursor(P);
      eeo_layout(T, k, R, S, slot.data(), count.data(), rcount.data(), cnt_src.data(), offset.data(),
                 roff.data(), row.data(), srcof.data(), cursor.data());
      const int N = offset[P];
      REQUIRE(N + counters[0] + counters[1] == (int64_t)T * k);
      std::vector<char> seen(N + 1, 0);
      for (int i = 0; i < T * k; ++i) {
        if (slot[i] < 0) { REQUIRE(row[i] == -1); continue; }
        REQUIRE(slot[i] < P && act[slot[i] / S] && nw[slot[i]] == idx[i]);
        REQUIRE(row[i] >= 0 && row[i] < N && !seen[row[i]] && srcof[row[i]] == i);
        seen[row[i]] = 1;
      }
      std::vector<float> x((size_t)T * H), recv((size_t)T * k * H, -1.0f), w((size_t)T * k, 0.5f), out((size_t)T * H);
      for (auto& v : x) v = (float)(rng() % 17) - 8.0f;
      eeo_pack(T, k, H * 4, (const uint8_t*)x.data(), row.data(), (uint8_t*)recv.data());
      for (int r = 0; r < N; ++r)
        REQUIRE(std::memcmp(&recv[(size_t)r * H], &x[(size_t)(srcof[r] / k) * H], H * 4) == 0);
      std::vector<int32_t> arrived(R), act2(act), report(R), row2(row);
      for (auto& v : arrived) v = rng() % 3 != 0;
      const int64_t gone = eeo_detect_round(T, k, R, S, slot.data(), arrived.data(), act2.data(),
                                            report.data(), row2.data());
      int64_t expect = 0;
      for (int r = 0; r < R; ++r) {
        REQUIRE(report[r] == (act[r] && !arrived[r] && rcount[r] > 0));  // awaited = holds rows
        if (report[r]) expect += rcount[r];
      }
      REQUIRE(gone == expect);
      eeo_combine_chain32(T, k, H, 0, recv.data(), w.data(), row2.data(), out.data());
      std::vector<double> out64((size_t)T * H);
      eeo_combine(T, k, H, 0, recv.data(), w.data(), row2.data(), out64.data());
      for (size_t i = 0; i < out.size(); ++i) REQUIRE((double)out[i] == out64[i]);  // small integers: exact

      // the remaining oracle functions, every buffer allocated at exactly the size the
      // function's contract names (so that the sanitizer sees any step past an end)
      std::vector<int32_t> dcount(R), doff(R + 1), drow((size_t)T * k), lead((size_t)T * k),
          expand((size_t)T * k), seen_r(R);
      eeo_dedup_layout(T, k, R, S, slot.data(), row.data(), dcount.data(), doff.data(), drow.data(),
                       lead.data(), expand.data(), seen_r.data());
      const int Nd = doff[R];
      REQUIRE(Nd <= N);
      std::vector<float> recv_d((size_t)Nd * H), recv_x((size_t)N * H);
      eeo_pack_dedup(T, k, H * 4, (const uint8_t*)x.data(), drow.data(), lead.data(), (uint8_t*)recv_d.data());
      eeo_expand(N, H * 4, (const uint8_t*)recv_d.data(), expand.data(), (uint8_t*)recv_x.data());
      REQUIRE(N == 0 || std::memcmp(recv_x.data(), recv.data(), (size_t)N * H * 4) == 0);  // two stages = pack
      std::vector<float> es(E), y32((size_t)N * H);
      for (int e = 0; e < E; ++e) es[e] = 1.0f + e;
      eeo_stub_scale(N, H, P, 0, recv_x.data(), offset.data(), nw.data(), es.data(), y32.data());
      for (int r = 0; r < N; ++r) REQUIRE(y32[(size_t)r * H] == es[idx[srcof[r]]] * recv_x[(size_t)r * H]);
      const int group = 2, G = H / group;
      std::vector<uint16_t> xb((size_t)T * H), yb((size_t)T * H);
      eeo_f32_to_bf16_array((int64_t)T * H, x.data(), xb.data());
      std::vector<uint8_t> q((size_t)T * H);
      std::vector<float> sc((size_t)T * G), back((size_t)T * H);
      eeo_quantize_e4m3(T, H, group, xb.data(), q.data(), sc.data());
      eeo_stub_dequant(T, H, group, q.data(), sc.data(), yb.data());
      eeo_bf16_to_f32_array((int64_t)T * H, yb.data(), back.data());
      for (size_t i = 0; i < back.size(); ++i) REQUIRE(back[i] - x[i] <= 0.5f && x[i] - back[i] <= 0.5f);
      eeo_f32_to_e4m3_array((int64_t)T * H, x.data(), q.data());
      eeo_e4m3_to_f32_array((int64_t)T * H, q.data(), back.data());
      for (size_t i = 0; i < back.size(); ++i) REQUIRE(back[i] == x[i]);  // |x| <= 8 integers are e4m3 values
    }
  }
  std::printf("ok %d\n", iterations);
  return 0;
}
