// Host-side logic of libeep that needs no GPU: replica lists, coverage check,
// tiling plan.  Exported through the C ABI as eep_host_* so that it can be
// tested on a machine without a GPU; the GPU entry points call the same code.
#include <vector>

#include "eep_internal.hpp"

namespace eep {

// Number of logical experts without a replica on an active rank (validity
// condition 2 of Sec. 3.2).
int host_uncovered_experts(int P, int E, int S, const int32_t* p2l, const int32_t* active) {
  std::vector<char> live(E, 0);
  for (int p = 0; p < P; ++p)
    if (p2l[p] >= 0 && p2l[p] < E && active[p / S] != 0) live[p2l[p]] = 1;
  int missing = 0;
  for (int e = 0; e < E; ++e) missing += !live[e];
  return missing;
}

// All physical locations of each logical expert (Sec. 5.1) as CSR, replicas in
// canonical order: primary slots first, then redundant ones, each by ascending
// slot id.  Unused tail of l2p_list is -1.
void host_replica_lists(int P, int E, int S, int S_prim, const int32_t* p2l, int32_t* l2p_off,
                        int32_t* l2p_list) {
  for (int e = 0; e <= E; ++e) l2p_off[e] = 0;
  for (int p = 0; p < P; ++p) l2p_list[p] = -1;
  for (int p = 0; p < P; ++p)
    if (p2l[p] >= 0) l2p_off[p2l[p] + 1]++;
  for (int e = 0; e < E; ++e) l2p_off[e + 1] += l2p_off[e];
  std::vector<int32_t> cur(l2p_off, l2p_off + E);
  for (int pass = 0; pass < 2; ++pass)
    for (int p = 0; p < P; ++p) {
      bool redundant = (p % S) >= S_prim;
      if (p2l[p] >= 0 && redundant == (pass == 1)) l2p_list[cur[p2l[p]]++] = p;
    }
}

// ---------------------------------------------------------------------------
// Placement repair (Sec. 3.5 "Repairing Expert Coverage After Failure",
// Sec. 5.1): given what every slot holds now and which ranks are live, produce
// a placement that covers every logical expert on live ranks, and say where
// each slot's weights come from (the three-case source hierarchy).  The paper
// names an elasticity-aware load balancer but not its algorithm; this is a
// small deterministic greedy stand-in:
//   A. coverage: every expert with no live copy gets a slot (hottest first):
//      a free live slot on the least-loaded rank, else the cheapest evictable
//      replica (an expert that keeps another live copy; redundant slots first).
//      Its weights can only come from the DRAM backup.
//   B. replication: free slots left over re-create replicas that were lost
//      (largest load per live copy first) on the least-loaded rank that does
//      not hold the expert yet; the weights come from a surviving peer copy.
// Slots that keep their expert are local reuse.  Slots of failed ranks are
// left untouched.
// ---------------------------------------------------------------------------
namespace {

struct Planner {
  int R, S, S_prim, E, P;
  const int32_t* cur;
  const int32_t* active;
  std::vector<double> load;
  std::vector<int32_t> now;   // placement being built
  std::vector<int> live_cnt;  // live copies of each expert in `now`

  bool live(int p) const { return active[p / S] != 0; }
  double rank_load(int r) const {
    double sum = 0.0;
    for (int s = 0; s < S; ++s) {
      int e = now[r * S + s];
      if (e >= 0) sum += load[e] / (double)live_cnt[e];
    }
    return sum;
  }
  bool rank_holds(int r, int e) const {
    for (int s = 0; s < S; ++s)
      if (now[r * S + s] == e) return true;
    return false;
  }
  // free live slot for expert e on the least-loaded rank not holding e; -1 if none
  int pick_free(int e) const {
    int best = -1;
    double best_load = 0.0;
    for (int p = 0; p < P; ++p) {
      if (!live(p) || now[p] != -1 || rank_holds(p / S, e)) continue;
      double l = rank_load(p / S);
      if (best < 0 || l < best_load) {
        best = p;
        best_load = l;
      }
    }
    return best;
  }
  // live slot whose expert keeps another live copy: redundant slots first, then
  // the smallest load per copy, then the lowest slot id; -1 if none
  int pick_victim() const {
    int best = -1;
    bool best_primary = false;
    double best_cost = 0.0;
    for (int p = 0; p < P; ++p) {
      int e = now[p];
      if (!live(p) || e < 0 || live_cnt[e] < 2) continue;
      bool primary = (p % S) < S_prim;
      double cost = load[e] / (double)live_cnt[e];
      if (best < 0 || (primary != best_primary ? !primary : cost < best_cost)) {
        best = p;
        best_primary = primary;
        best_cost = cost;
      }
    }
    return best;
  }
};

}  // namespace

int host_plan_repair(int R, int S, int S_prim, int E, const int32_t* cur, const int32_t* active,
                     const float* load, int32_t* new_p2l, int32_t* kind, int32_t* src_slot,
                     int32_t summary[4]) {
  Planner pl;
  pl.R = R; pl.S = S; pl.S_prim = S_prim; pl.E = E; pl.P = R * S;
  pl.cur = cur; pl.active = active;
  pl.load.assign(E, 1.0);
  if (load)
    for (int e = 0; e < E; ++e) pl.load[e] = (double)load[e];
  pl.now.assign(cur, cur + pl.P);
  pl.live_cnt.assign(E, 0);
  std::vector<int> had(E, 0), live_before(E, 0);
  for (int p = 0; p < pl.P; ++p)
    if (cur[p] >= 0) {
      had[cur[p]]++;
      if (pl.live(p)) { pl.live_cnt[cur[p]]++; live_before[cur[p]]++; }
    }
  for (int p = 0; p < pl.P; ++p) {
    src_slot[p] = -1;
    kind[p] = (pl.live(p) && cur[p] >= 0) ? EEP_SRC_LOCAL : EEP_SRC_NONE;
  }
  // first live copy of e in canonical order, as things stand before the repair
  auto peer_source = [&](int e) {
    for (int pass = 0; pass < 2; ++pass)
      for (int p = 0; p < pl.P; ++p)
        if (cur[p] == e && pl.live(p) && ((p % S) >= S_prim) == (pass == 1)) return p;
    return -1;
  };
  int unplaced = 0;
  // A. coverage, hottest missing expert first (ties: lower id)
  std::vector<char> done(E, 0);
  for (;;) {
    int e = -1;
    for (int c = 0; c < E; ++c)
      if (pl.live_cnt[c] == 0 && !done[c] && (e < 0 || pl.load[c] > pl.load[e])) e = c;
    if (e < 0) break;
    done[e] = 1;
    int p = pl.pick_free(e);
    if (p < 0) {
      p = pl.pick_victim();
      if (p >= 0) pl.live_cnt[pl.now[p]]--;
    }
    if (p < 0) { ++unplaced; continue; }
    pl.now[p] = e;
    pl.live_cnt[e] = 1;
    kind[p] = EEP_SRC_DRAM;  // every GPU-resident copy was on a failed rank
  }
  // B. re-create lost replicas from surviving peers while free slots remain
  for (;;) {
    int e = -1, slot = -1;
    double e_cost = 0.0;
    for (int c = 0; c < E; ++c) {
      if (live_before[c] == 0 || pl.live_cnt[c] == 0 || pl.live_cnt[c] >= had[c]) continue;
      double cost = pl.load[c] / (double)pl.live_cnt[c];
      if (e >= 0 && !(cost > e_cost)) continue;
      int p = pl.pick_free(c);
      if (p < 0) continue;
      e = c; slot = p; e_cost = cost;
    }
    if (e < 0) break;
    pl.now[slot] = e;
    pl.live_cnt[e]++;
    kind[slot] = EEP_SRC_PEER;
    src_slot[slot] = peer_source(e);
  }
  int n_local = 0, n_peer = 0, n_dram = 0;
  for (int p = 0; p < pl.P; ++p) {
    new_p2l[p] = pl.now[p];
    n_local += kind[p] == EEP_SRC_LOCAL;
    n_peer += kind[p] == EEP_SRC_PEER;
    n_dram += kind[p] == EEP_SRC_DRAM;
  }
  summary[0] = n_local; summary[1] = n_peer; summary[2] = n_dram; summary[3] = unplaced;
  return unplaced;
}

void host_plan_transition(int R, int S, int S_prim, const int32_t* cur, const int32_t* target,
                          const int32_t* active, const int32_t* writable, int32_t* new_p2l,
                          int32_t* kind, int32_t* src_slot, int32_t summary[4]) {
  const int P = R * S;
  std::vector<char> gets_weights(P, 0);
  for (int p = 0; p < P; ++p) {
    new_p2l[p] = writable[p / S] ? target[p] : cur[p];
    gets_weights[p] = writable[p / S] && new_p2l[p] >= 0 && new_p2l[p] != cur[p];
    kind[p] = EEP_SRC_NONE;
    src_slot[p] = -1;
  }
  int n_local = 0, n_peer = 0, n_dram = 0;
  for (int p = 0; p < P; ++p) {
    if (!writable[p / S] || new_p2l[p] < 0) continue;
    if (!gets_weights[p]) { kind[p] = EEP_SRC_LOCAL; ++n_local; continue; }
    // canonical order: primary slots of all ranks first, then redundant ones
    int found = -1;
    for (int pass = 0; pass < 2 && found < 0; ++pass)
      for (int q = 0; q < P && found < 0; ++q)
        if (((q % S) >= S_prim) == (pass == 1) && active[q / S] && cur[q] == new_p2l[p] &&
            !gets_weights[q])
          found = q;
    if (found >= 0) { kind[p] = EEP_SRC_PEER; src_slot[p] = found; ++n_peer; }
    else { kind[p] = EEP_SRC_DRAM; ++n_dram; }
  }
  summary[0] = n_local; summary[1] = n_peer; summary[2] = n_dram; summary[3] = 0;
}

}  // namespace eep

extern "C" {

int eep_plan_transition(int32_t R, int32_t S, int32_t S_prim, int32_t E, const int32_t* cur_p2l,
                        const int32_t* target_p2l, const int32_t* active, const int32_t* writable,
                        int32_t* new_p2l, int32_t* source_kind, int32_t* source_slot,
                        int32_t summary[4]) {
  if (R < 1 || S < 1 || S_prim < 0 || S_prim > S || E < 1 || !cur_p2l || !target_p2l || !active ||
      !writable || !new_p2l || !source_kind || !source_slot || !summary)
    return EEP_ERR_INVALID_ARG;
  for (int p = 0; p < R * S; ++p)
    if (cur_p2l[p] < -1 || cur_p2l[p] >= E || target_p2l[p] < -1 || target_p2l[p] >= E)
      return EEP_ERR_INVALID_ARG;
  eep::host_plan_transition(R, S, S_prim, cur_p2l, target_p2l, active, writable, new_p2l,
                            source_kind, source_slot, summary);
  return EEP_OK;
}

int eep_plan_repair(int32_t R, int32_t S, int32_t S_prim, int32_t E, const int32_t* cur_p2l,
                    const int32_t* active, const float* load, int32_t* new_p2l,
                    int32_t* source_kind, int32_t* source_slot, int32_t summary[4]) {
  if (R < 1 || S < 1 || S_prim < 0 || S_prim > S || E < 1 || !cur_p2l || !active || !new_p2l ||
      !source_kind || !source_slot || !summary)
    return EEP_ERR_INVALID_ARG;
  for (int p = 0; p < R * S; ++p)
    if (cur_p2l[p] < -1 || cur_p2l[p] >= E) return EEP_ERR_INVALID_ARG;
  if (load)
    for (int e = 0; e < E; ++e)
      if (!(load[e] >= 0.0f)) return EEP_ERR_INVALID_ARG;
  int unplaced = eep::host_plan_repair(R, S, S_prim, E, cur_p2l, active, load, new_p2l,
                                       source_kind, source_slot, summary);
  return unplaced == 0 ? EEP_OK : EEP_ERR_COVERAGE;
}

int eep_host_replica_lists(int32_t P, int32_t E, int32_t S, int32_t S_prim, const int32_t* p2l,
                           int32_t* l2p_off, int32_t* l2p_list) {
  if (P < 1 || E < 1 || S < 1 || S_prim < 0 || S_prim > S || P % S != 0 || !p2l || !l2p_off ||
      !l2p_list)
    return EEP_ERR_INVALID_ARG;
  for (int p = 0; p < P; ++p)
    if (p2l[p] < -1 || p2l[p] >= E) return EEP_ERR_INVALID_ARG;
  eep::host_replica_lists(P, E, S, S_prim, p2l, l2p_off, l2p_list);
  return EEP_OK;
}

int eep_host_uncovered_experts(int32_t P, int32_t E, int32_t S, const int32_t* p2l,
                               const int32_t* active) {
  if (P < 1 || E < 1 || S < 1 || P % S != 0 || !p2l || !active) return EEP_ERR_INVALID_ARG;
  for (int p = 0; p < P; ++p)
    if (p2l[p] < -1 || p2l[p] >= E) return EEP_ERR_INVALID_ARG;
  return eep::host_uncovered_experts(P, E, S, p2l, active);
}

int eep_host_tiling(int32_t T, int32_t R, int32_t out[4]) {
  if (T < 0 || R < 1 || T % R != 0 || !out) return EEP_ERR_INVALID_ARG;
  eep::Tiling g = eep::make_tiling(T, R);
  out[0] = g.tokens_per_rank;
  out[1] = g.tiles_per_rank;
  out[2] = g.tile_tokens;
  out[3] = g.num_tiles;
  return EEP_OK;
}

}  // extern "C"
