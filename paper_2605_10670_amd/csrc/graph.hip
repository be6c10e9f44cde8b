// hipGraph helper: capture the per-step calls once, replay them many times.
// Paper Sec. 2.3 and Fig. 4: a captured graph fixes launch order and pointer
// identities; only the contents of memory behind those pointers may change.
// The library never re-instantiates or updates a graph; the counters let a
// test assert that a membership change needed neither.
#include <new>

#include "eep_internal.hpp"

struct eep_graph {
  hipGraph_t graph;
  hipGraphExec_t exec;
  int64_t instantiations, exec_updates, launches;
  // the instance whose contexts were captured with failure detection on (else null):
  // every replay then holds a waiting kernel that may drop a rank
  eep_membership* awaits;
};

extern "C" {

int eep_graph_begin(eep_ctx* c, void* stream) {
  if (!c || !stream) return EEP_ERR_INVALID_ARG;  // the default stream cannot be captured
  hipError_t e = hipStreamBeginCapture((hipStream_t)stream, hipStreamCaptureModeThreadLocal);
  if (e != hipSuccess) { c->last_hip_error = (int)e; return EEP_ERR_HIP; }
  return EEP_OK;
}

int eep_graph_end(eep_ctx* c, void* stream, eep_graph** out) {
  if (!c || !stream || !out) return EEP_ERR_INVALID_ARG;
  *out = nullptr;
  hipGraph_t graph = nullptr;
  hipError_t e = hipStreamEndCapture((hipStream_t)stream, &graph);
  if (e != hipSuccess || graph == nullptr) { c->last_hip_error = (int)e; return EEP_ERR_HIP; }
  eep_graph* g = new (std::nothrow) eep_graph();
  if (!g) { (void)hipGraphDestroy(graph); return EEP_ERR_INVALID_ARG; }
  g->graph = graph;
  g->exec = nullptr;
  g->instantiations = g->exec_updates = g->launches = 0;
  e = hipGraphInstantiate(&g->exec, graph, nullptr, nullptr, 0);
  if (e != hipSuccess) {
    c->last_hip_error = (int)e;
    (void)hipGraphDestroy(graph);
    delete g;
    return EEP_ERR_HIP;
  }
  g->instantiations = 1;
  g->awaits = nullptr;
  for (eep_ctx* o : c->mem->members)
    if (o->detect_timeout_ticks > 0) g->awaits = c->mem;
  *out = g;
  return EEP_OK;
}

int eep_graph_launch(eep_graph* g, void* stream) {
  if (!g || !g->exec) return EEP_ERR_INVALID_ARG;
  hipError_t e = hipGraphLaunch(g->exec, (hipStream_t)stream);
  if (e != hipSuccess) return EEP_ERR_HIP;
  if (g->awaits) g->awaits->unread_round = true;
  g->launches += 1;
  return EEP_OK;
}

int eep_graph_destroy(eep_graph* g) {
  if (!g) return EEP_OK;
  hipError_t e1 = g->exec ? hipGraphExecDestroy(g->exec) : hipSuccess;
  hipError_t e2 = g->graph ? hipGraphDestroy(g->graph) : hipSuccess;
  delete g;
  return (e1 == hipSuccess && e2 == hipSuccess) ? EEP_OK : EEP_ERR_HIP;
}

int eep_graph_counters(const eep_graph* g, int64_t counters[3]) {
  if (!g || !counters) return EEP_ERR_INVALID_ARG;
  counters[0] = g->instantiations;
  counters[1] = g->exec_updates;
  counters[2] = g->launches;
  return EEP_OK;
}

}  // extern "C"
