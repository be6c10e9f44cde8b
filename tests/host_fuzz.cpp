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
    }
  }
  std::printf("ok %d\n", iterations);
  return 0;
}
