/*
 * eep.h -- C ABI of the membership-elastic MoE dispatch/combine library for
 * AMD MI355X (gfx950).
 *
 * The library implements, on ONE GPU, the per-step token dispatch and combine
 * of a wide expert-parallel (EP) MoE layer whose membership is explicit,
 * mutable device state (paper: Sec. 3.2 "Live EP Validity", Sec. 3.4 and
 * Sec. 4.1 "GPU-Resident Peer Table", Fig. 4, Fig. 5, Fig. 7, Sec. 5.1
 * "Expert-Location Metadata").  The R "virtual" EP ranks are partitions of one
 * GPU's HBM: rank r owns the physical expert slots p = r*S .. r*S+S-1 and the
 * rows of the receive buffer that those slots receive.
 *
 * Conventions
 *   - Every entry point returns an int: 0 (EEP_OK) or a negative eep_status.
 *     No C++ exception crosses this boundary.
 *   - "host" pointers are ordinary process memory, read before the call
 *     returns.  "device" pointers are HIP device memory of the GPU that was
 *     current when eep_create ran; the caller owns them and keeps them alive
 *     until the work queued on the stream has finished.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     All work is queued on it and no entry point synchronises, except where
 *     stated (eep_create, eep_destroy, eep_read_view, eep_read_failures,
 *     eep_graph_end).
 *   - The context owns the membership/placement tables and the layout arrays.
 *     Their device addresses never change during the context's lifetime:
 *     table updates rewrite contents only (Fig. 4, Fig. 8), which is what lets
 *     a captured hipGraph keep replaying across failure and rejoin.
 *   - Layouts are dense row-major; indices are int32.
 *   - Threads: calls on DIFFERENT contexts that share no membership instance
 *     may run concurrently.  Calls that name one context, or contexts of one
 *     instance (eep_create_attached, eep_create_staging), keep host-side state
 *     (shadow copies of the tables, the last laid-out T) without locks: the
 *     caller serialises them.  On the device, work of one context is ordered
 *     by the streams the caller passes; two steps of one context queued on two
 *     streams without an event between them race on its layout arrays.
 *
 * Notation: T tokens, k = top-k, H hidden elements, E logical experts,
 * R ranks, S slots per rank (S_prim primary + S_red redundant), P = R*S
 * physical slots, N = number of routed (token, k) pairs of the current step.
 */
#ifndef EEP_H_
#define EEP_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  EEP_OK = 0,
  EEP_ERR_INVALID_ARG = -1, /* null pointer, size out of range, T % R != 0, bad enum */
  EEP_ERR_ALIGN = -2,       /* a row size or a base pointer is not 16-byte aligned   */
  EEP_ERR_COVERAGE = -3,    /* update would leave a logical expert with no live replica */
  EEP_ERR_HIP = -4,         /* a HIP runtime call failed; see eep_last_hip_error     */
  EEP_ERR_STATE = -5,       /* call order violated (e.g. dispatch before dispatch_layout) */
  EEP_ERR_SCRATCH = -6      /* the batch needs more scratch than the fixed static array holds */
} eep_status;

typedef enum { EEP_F32 = 0, EEP_BF16 = 1, EEP_FP8_E4M3 = 2 } eep_dtype;

/* Which live replica serves a (token, expert) pair when several are live.
 * The paper shows a single route per expert (Fig. 4, Fig. 5) and says the
 * metadata records every location (Sec. 5.1) but gives no selection rule:
 *   EEP_FIRST_LIVE  first live replica in canonical order (reproduces Fig. 5);
 *   EEP_SPREAD      replica number (t mod n_live) for token t (balances load).
 * Canonical order of the replicas of one expert: primary slots before
 * redundant slots, then ascending slot id. */
typedef enum { EEP_SPREAD = 0, EEP_FIRST_LIVE = 1 } eep_policy;

typedef enum {
  EEP_STUB_IDENTITY = 0, /* y[row] = recv_x[row]                       (same dtype) */
  EEP_STUB_SCALE = 1,    /* y[row] = round(s[logical expert of row] * recv_x[row])  */
  EEP_STUB_DEQUANT = 2   /* y[row] = bf16(e4m3(recv_x[row]) * recv_scale[row, h/G]) */
} eep_stub_kind;

typedef struct {
  int32_t num_ranks;       /* R  >= 1                                              */
  int32_t slots_per_rank;  /* S  >= 1                                              */
  int32_t primary_slots;   /* S_prim in [0, S]; slots s >= S_prim are redundant    */
  int32_t num_logical;     /* E  >= 1                                              */
  int32_t max_tokens;      /* T_max >= 0, the largest T any per-step call may pass */
  int32_t topk;            /* k in [1, 32]                                         */
  int32_t hidden;          /* H  >= 1 elements per token row                       */
  int32_t x_dtype;         /* eep_dtype of dispatch payload rows                   */
  int32_t y_dtype;         /* eep_dtype of expert output rows (F32 or BF16)        */
  int32_t out_dtype;       /* eep_dtype of combined rows      (F32 or BF16)        */
  int32_t scale_group;     /* channels per fp32 scale (H % group == 0) when x_dtype
                              is FP8_E4M3, else 0                                  */
  int32_t policy;          /* eep_policy                                           */
  int32_t strict_coverage; /* 1: a table update that would leave a logical expert
                              without a live replica (validity condition 2,
                              Sec. 3.2) returns EEP_ERR_COVERAGE and changes
                              nothing; 0: it is applied and such pairs are dropped
                              and counted in status[1]                             */
} eep_config;

typedef struct eep_ctx eep_ctx;

/* Creates one EP instance's routing state: the GPU-resident table of the
 * instance's ranks (Sec. 4.1; here its `active` column), the expert-location
 * metadata (Sec. 5.1) and the per-step layout arrays, all at device addresses
 * that stay fixed until eep_destroy -- the stable pointers a captured graph
 * holds (Sec. 2.3; Fig. 4, Fig. 8).
 * Allocates them on the current device (hipMalloc; sizes depend only on the
 * config) and initialises them to "all ranks live, all slots empty".
 * Synchronises the device once.
 * Row sizes (H * sizeof(dtype)) must be multiples of 16 bytes (EEP_ERR_ALIGN).
 * On error *out is NULL. */
int eep_create(const eep_config* cfg, eep_ctx** out);

/* The same context in memory the CALLER owns (say a torch tensor), for callers
 * that keep all device memory under one allocator: the "stable pointers" of
 * Fig. 4 / Fig. 8 then lie inside a buffer whose lifetime the caller controls.
 * eep_workspace_bytes: host only, no GPU needed; *bytes = size the config needs
 * (same argument checks as eep_create).
 * eep_create_with_workspace: `workspace` is device memory of the current GPU,
 * 256-byte aligned, at least that large (checked: EEP_ERR_INVALID_ARG); the
 * library allocates no device memory, eep_destroy does not free it, and the
 * caller must keep it alive and untouched until eep_destroy returns. */
int eep_workspace_bytes(const eep_config* cfg, int64_t* bytes);
int eep_create_with_workspace(const eep_config* cfg, void* workspace, int64_t workspace_bytes,
                              eep_ctx** out);

/* A further context of the SAME EP instance as `parent`: it shares parent's
 * membership (the `active` mask -- one peer table per instance, Sec. 4.1) and has
 * its own placement tables, layout arrays and shapes.  This is how the MoE
 * layers of one model are set up: every layer has its own expert-location
 * metadata (Sec. 5.1) while a rank failure concerns all of them at once.
 * cfg->num_ranks must equal the parent's.  eep_set_membership through any
 * context of the instance updates the one shared mask (and checks the coverage
 * of every context that asked for strict_coverage); a rank dropped by one
 * context's failure detection is dropped for all.  Attached contexts must be
 * destroyed before the context that eep_create made. */
int eep_create_attached(const eep_config* cfg, eep_ctx* parent, eep_ctx** out);

/* Ends the lifetime of the stable pointers (Fig. 4, Fig. 8): graphs captured
 * with this context must not be replayed afterwards.  Waits for the device,
 * frees everything the context owns.  NULL is OK.
 * EEP_ERR_STATE if attached contexts of this instance, or staging contexts of
 * this context, still exist. */
int eep_destroy(eep_ctx* ctx);

/* ---- table updates: between steps, stream-ordered (Sec. 3.1: repair and
 * reintegration happen between forward passes; Sec. 4.1 "In-place peer-table
 * updates"; Fig. 4) -------------------------------------------------------
 * Both calls only queue small kernels that overwrite table CONTENTS at their
 * fixed addresses; they do not allocate, synchronise or move any buffer, and
 * they copy the host array before returning.  A step queued later on the same
 * stream sees the new tables, one queued earlier sees the old ones.  Both may
 * be called while a captured graph of the per-step calls exists; the graph
 * needs no update afterwards.
 *
 * To stay valid at every step boundary follow the paper's order (Fig. 6):
 *   failure: eep_update_placement(repaired), then eep_set_membership(dead);
 *   rejoin:  eep_set_membership(live), then eep_update_placement(preferred).
 *
 * With GPU-side failure detection on (eep_set_detection), a waiting kernel may
 * have dropped a rank that the host has not heard of yet (Sec. 4.1: the report
 * reaches the host only after the kernel has exited).  From the moment an
 * eep_combine with detection on is queued (or a graph holding one is launched)
 * until eep_read_failures has been called, the host's copy of the mask counts
 * as out of date: eep_set_membership returns EEP_ERR_STATE (it would rewrite the
 * whole mask and could bring a dropped rank back), and so do
 * eep_update_placement and eep_apply_repair of a context with strict_coverage
 * (their coverage check needs the current mask).  Nothing is changed then;
 * call eep_read_failures and repeat the call. */

/* active_host: host int32[R]; 0 = failed (receives nothing), non-zero = live.
 * This is the `active` column of the peer table (Fig. 7). */
int eep_set_membership(eep_ctx* ctx, const int32_t* active_host, void* stream);

/* phys_to_logical_host: host int32[P]; entry p is the logical expert held by
 * physical slot p = r*S + s, or -1 for an empty slot (Sec. 5.1).  Entries
 * outside [-1, E) give EEP_ERR_INVALID_ARG. */
int eep_update_placement(eep_ctx* ctx, const int32_t* phys_to_logical_host, void* stream);

/* ---- per-step calls: graph-capturable, grids depend only on T ----------- */

/* Routing + layout of one step: the table lookups of the dispatch path
 * (Fig. 7: every transfer consults the destination's entry and skips it when
 * `active` is 0; Sec. 5.1: slot -> logical expert and all locations of a
 * logical expert) and the placement of the payload rows into contiguous
 * per-expert receive buffers (Sec. 4.1 refers to prior work for it).  The
 * result satisfies the validity contract of Sec. 3.2: rows go to active ranks
 * only, and to a slot that holds the pair's logical expert.
 * topk_idx: device int32[T, k], the router's
 * logical expert per (token, j).  T must satisfy 0 <= T <= T_max, T % R == 0
 * (tokens [b*T/R, (b+1)*T/R) belong to source rank b).
 * For every pair it picks the live replica slot (slot_of, or -1 when the
 * index is outside [0, E), repeats an earlier index of the same token, or the
 * expert has no live replica), counts pairs per slot, prefix-sums the counts
 * into receive-buffer offsets, and gives every routed pair its row:
 * rows of one slot are contiguous and ordered by ascending token.
 * Results stay in the context (see eep_view). */
int eep_dispatch_layout(eep_ctx* ctx, const int32_t* topk_idx, int32_t T, void* stream);

/* eep_dispatch_layout for callers that cannot allocate device memory: code
 * under hipGraph capture, tight serving loops, harnesses that forbid hipMalloc
 * (and therefore eep_create).  Same kernels, same results, no context: the
 * caller passes the tables and every output array as device pointers, and the
 * pass's scratch (per-tile slot counts and prefixes, per-tile drop counters)
 * lives in a static device array of EEP_NOALLOC_SCRATCH_BYTES inside the
 * library; each GPU the library runs on holds that array until the process ends.
 * The call makes no hipMalloc / hipFree and no allocating library call.
 *   shape          R, S, E, k, eep_policy (host struct, read before returning)
 *   topk_idx       device int32[T, k]
 *   active         device int32[R]          (e.g. eep_view.active of a context)
 *   l2p_off        device int32[E+1]        replica lists in canonical order, as
 *   l2p_list       device int32[P]          eep_host_replica_lists writes them
 *   table_version  device int32[1] copied to status[3], or NULL for 0
 *   out            host struct of device pointers the caller owns:
 *                  slot_of[T*k], row_of[T*k], src_of[T*k], count[P], offset[P+1],
 *                  rank_count[R], rank_offset[R+1], cnt_src[R*P], status[4];
 *                  same contents as the eep_view arrays after eep_dispatch_layout
 * Limits: those of eep_create, and the batch's scratch must fit the array:
 * eep_noalloc_scratch_needed(R, S, T) <= EEP_NOALLOC_SCRATCH_BYTES, otherwise
 * EEP_ERR_SCRATCH and nothing is queued (512 + 8*tiles*(P+1) bytes rounded up,
 * tiles = R * ceil(T/R / 128): 75 KB at T=4096, R=32, P=288).
 * All calls on one GPU share the one array, which keeps the previous call's
 * contents (no word needs clearing: each pass overwrites what it reads): calls
 * whose kernels may overlap on one GPU -- different streams, or graphs launched
 * concurrently -- race; keep them on one stream or order them with events. */
#define EEP_NOALLOC_SCRATCH_BYTES (4 * 1024 * 1024)
typedef struct {
  int32_t num_ranks, slots_per_rank, num_logical, topk, policy;
} eep_layout_shape;
typedef struct {
  int32_t *slot_of, *row_of, *src_of, *count, *offset, *rank_count, *rank_offset, *cnt_src,
      *status;
} eep_layout_out;
int eep_dispatch_layout_noalloc(const eep_layout_shape* shape, const int32_t* topk_idx,
                                const int32_t* active, const int32_t* l2p_off,
                                const int32_t* l2p_list, const int32_t* table_version,
                                const eep_layout_out* out, int32_t T, void* stream);
/* Host only: scratch bytes a batch of T tokens needs (negative = eep_status). */
int64_t eep_noalloc_scratch_needed(int32_t num_ranks, int32_t slots_per_rank, int32_t T);

/* recv_x[row_of[t, j], :] = x[t, :] for every routed pair (Fig. 7, dispatch
 * path; inactive ranks are never written).  x: device [T, H] x_dtype;
 * recv_x: device [T*k, H] x_dtype; rows >= N are left untouched.  With fp8
 * payloads x_scale is device float[T, H/group] and recv_scale device
 * float[T*k, H/group], moved the same way; otherwise both are NULL.
 * Needs eep_dispatch_layout with the same T queued before it. */
int eep_dispatch(eep_ctx* ctx, const void* x, const float* x_scale, void* recv_x,
                 float* recv_scale, int32_t T, void* stream);

/* Variant of eep_dispatch with the fp8 quantisation fused in (a data-path variant
 * of the kind Sec. 4.1 leaves to prior work).  The context's x_dtype must be
 * FP8_E4M3 with scale_group a power-of-two multiple of 16 (16..1024); x_bf16 is
 * device bf16 [T, H].  Per token and per group of scale_group channels:
 * scale = max|x| / 448 in fp32 (1 if the group is all zero),
 * code = e4m3fn(x / scale), round to nearest even, saturating;
 * recv_x[row, :] gets the codes and recv_scale[row, :] the scales of the token,
 * for each of its routed rows.  Same call order and errors as eep_dispatch. */
int eep_dispatch_quant(eep_ctx* ctx, const void* x_bf16, void* recv_x, float* recv_scale,
                       int32_t T, void* stream);

/* out[t, :] = round( sum over routed j, ascending, of w[t, j] * y[row_of[t, j], :] ),
 * accumulated in fp32 with one fused multiply-add per term, starting from 0
 * (Sec. 4.1: combine reduces the expert outputs).  y: device [T*k, H] y_dtype;
 * topk_w: device float[T, k]; out: device [T, H] out_dtype (bf16: round to
 * nearest even).  A token with no routed pair gets zeros. */
int eep_combine(eep_ctx* ctx, const void* y, const float* topk_w, void* out, int32_t T,
                void* stream);

/* Stand-in for the expert kernels that sit between dispatch and combine in the
 * captured graph (Fig. 4).  Processes rows [0, N) only; the grid is sized for
 * T*k rows and reads N from device memory.
 *   IDENTITY: copies recv_x to y (callers may instead alias y = recv_x);
 *   SCALE:    expert_scale is device float[E]; x_dtype must equal y_dtype
 *             (F32 or BF16); product computed in fp32;
 *   DEQUANT:  x_dtype FP8_E4M3 (OCP e4m3fn), y_dtype BF16. */
int eep_expert_stub(eep_ctx* ctx, int32_t kind, const void* recv_x, const float* recv_scale,
                    const float* expert_scale, void* y, int32_t T, void* stream);

/* ---- GPU-side failure detection (Sec. 3.4; Sec. 4.1, the paragraph on
 * failure detection from the GPU side; the time-out remark in Fig. 7's listing)
 * One-GPU emulation of the paper's signal counters.  Every eep_dispatch_layout
 * advances a device-side step epoch.  The expert stage announces "the outputs of
 * rank r for this step are there" by storing the epoch into rank r's signal word
 * (release).  With detection on, the combine kernel itself polls those words:
 * before a wavefront reduces a token's rows it looks at the signal of every rank
 * the rows come from, and waits -- for at most the timeout -- for a word that
 * does not show the epoch yet.  Ranks from which the step expects nothing are
 * not awaited.  A rank that stays silent is dropped by the kernel: its active
 * entry is cleared in the device table, the membership version is bumped, its
 * failure is recorded, and the pairs routed to it contribute nothing to this
 * step's outputs and lose their row_of entry (the paper fails such in-flight
 * requests, Sec. 3.1).  Waiting wavefronts notice a drop made by another one, so
 * a step with a silent rank takes about one timeout longer, not more.  Later
 * steps, replayed graphs included, route around the rank with no host action;
 * the host finds out with eep_read_failures, then repairs the placement
 * (eep_plan_repair, eep_update_placement).
 * Switching detection on or off changes which kernels eep_combine and
 * eep_expert_stub launch, so choose before capturing a graph. */

/* timeout_ns = 0 switches detection off (the default); at most 2e9 (2 s; the
 * paper uses 1 s).  Host-side setting, no GPU work. */
int eep_set_detection(eep_ctx* ctx, int64_t timeout_ns);
/* Producer side: marks the current step's expert outputs of every active rank as
 * arrived.  eep_expert_stub does this itself when detection is on; callers that
 * run their own expert kernels (or alias y = recv_x) queue it after them. */
int eep_signal_experts_done(eep_ctx* ctx, void* stream);
/* Test knob: withhold_host[R], non-zero = that rank never signals (a silent
 * peer).  This is how a failure is injected on one GPU. */
int eep_debug_withhold_signal(eep_ctx* ctx, const int32_t* withhold_host, void* stream);
/* Waits for `stream` (for the whole device when the instance has attached
 * contexts, whose steps may run on other streams), copies the failure report of
 * every context of the instance to failed_host[R] (1 = dropped by a kernel since
 * the last call), folds it into the host's copy of the active mask and clears
 * the report.  Afterwards the table updates are accepted again (see above). */
int eep_read_failures(eep_ctx* ctx, int32_t* failed_host, void* stream);

/* ---- introspection ------------------------------------------------------ */

/* Device addresses of the context's arrays: the graph-visible state of
 * Sec. 3.2 (condition 3) and Fig. 4 / Fig. 8 -- fixed pointers, mutable
 * contents -- for callers whose own kernels read the routing results (expert
 * kernels need offset/count; Sec. 5.1's metadata is phys_to_logical + l2p_*).
 * All int32, stable for the context's lifetime; contents valid once the
 * producing call has finished on its stream.
 *   active[R], phys_to_logical[P], l2p_off[E+1], l2p_list[P]  tables
 *   slot_of[T,k], row_of[T,k]      per pair; -1 when not routed
 *   src_of[T*k]                    row -> t*k+j; -1 for rows >= N
 *   count[P], offset[P+1]          pairs per slot, exclusive prefix sum
 *   rank_count[R], rank_offset[R+1]
 *   cnt_src[R,P]                   pairs per (source rank, slot)
 *   status[4]                      {N, n_uncovered, n_masked, table version}
 *                                  (version = placement updates of this context
 *                                  + membership changes of the instance: host
 *                                  updates and drops made by waiting kernels) */
typedef struct {
  const int32_t *active, *phys_to_logical, *l2p_off, *l2p_list;
  const int32_t *slot_of, *row_of, *src_of;
  const int32_t *count, *offset, *rank_count, *rank_offset, *cnt_src, *status;
} eep_view;
int eep_get_view(eep_ctx* ctx, eep_view* out);

typedef enum {
  EEP_V_ACTIVE = 0, EEP_V_PHYS_TO_LOGICAL, EEP_V_L2P_OFF, EEP_V_L2P_LIST, EEP_V_SLOT_OF,
  EEP_V_ROW_OF, EEP_V_SRC_OF, EEP_V_COUNT, EEP_V_OFFSET, EEP_V_RANK_COUNT,
  EEP_V_RANK_OFFSET, EEP_V_CNT_SRC, EEP_V_STATUS, EEP_V_NUM_FIELDS
} eep_view_field;

/* Debug helper: waits for `stream`, then copies the first n int32 of one view
 * array into host memory.  n beyond the array's allocated size is an error. */
int eep_read_view(eep_ctx* ctx, int32_t field, int32_t* host_dst, int64_t n, void* stream);

/* Debug helper: the bounds assertion of the path as a call.  eep_dispatch and
 * eep_combine index the caller's buffers with row_of without further checks;
 * this checks, on the device, the layout that the last eep_dispatch_layout of
 * the same T left behind, waits for `stream` and returns four counts (all zero
 * for a sound layout):
 *   [0] pairs whose row lies outside its slot's rows [offset[p], offset[p+1]),
 *       or outside [0, N), or whose slot is outside [-1, P)
 *   [1] pairs whose row's src_of entry is not the pair
 *   [2] rows below N whose src_of is out of range or does not point at a pair
 *       holding the row; rows from N on whose src_of is not -1
 *   [3] routed pairs without a row: not a violation by itself, it is what
 *       failure detection leaves behind when it drops a rank within the step */
int eep_debug_check_layout(eep_ctx* ctx, int32_t T, int32_t violations_host[4], void* stream);

/* Measurement helper: a plain copy kernel (dst[i] = src[i], 16-byte vectors,
 * bytes a multiple of 16, both device pointers 16-byte aligned).  It moves
 * exactly `bytes` in and `bytes` out, which makes it the yardstick that
 * hardware HBM counters are scaled by when a profile is turned into bytes. */
int eep_calibration_copy(void* dst, const void* src, int64_t bytes, void* stream);

/* Measurement helper: a perfectly sequential streaming kernel with the read:write
 * mix of a stage of the step, as a yardstick for what the memory system gives
 * that mix when nothing is scattered (paper Sec. 6.2 names dispatch and combine
 * as the dominant cost; both are pure data movement).  Thread i reads 16-byte
 * vector i of `reads` source planes and writes vector i of `writes` destination
 * planes, with the loads and stores that pack and combine use (read-once
 * non-temporal loads, write-through stores).  (reads, writes) in {1, 8}^2:
 * (1, 8) is dispatch's mix, (8, 1) combine's, (1, 1) a copy.
 *   src, dst            device, 16-byte aligned; plane j starts j * plane_stride_bytes
 *                       in; src holds `reads` planes, dst `writes` planes; must not overlap
 *   plane_bytes         bytes per plane, a multiple of 16 (0: nothing is launched)
 *   plane_stride_bytes  >= plane_bytes, a multiple of 16 (a stride that is not a
 *                       power of two keeps the planes off one another's channels)
 * Moves exactly reads * plane_bytes in and writes * plane_bytes out.  Asynchronous
 * on `stream`; EEP_ERR_INVALID_ARG for anything else. */
int eep_calibration_stream(void* dst, const void* src, int64_t plane_bytes,
                           int64_t plane_stride_bytes, int32_t reads, int32_t writes,
                           void* stream);

const char* eep_strerror(int code);
/* hipError_t of the last failed HIP call made for this context (0 if none). */
int eep_last_hip_error(eep_ctx* ctx);

/* ---- host-only helpers: touch no GPU; the entry points above run the same
 * code.  Exposed so that the host logic can be checked on a CPU-only machine. */

/* All physical locations of each logical expert (Sec. 5.1) as CSR over host
 * arrays: l2p_off[E+1], l2p_list[P] (replicas in canonical order, unused tail
 * -1).  P must be a multiple of S. */
int eep_host_replica_lists(int32_t P, int32_t E, int32_t S, int32_t S_prim,
                           const int32_t* phys_to_logical, int32_t* l2p_off, int32_t* l2p_list);
/* Number (>= 0) of logical experts with no replica on an active rank: validity
 * condition 2 of Sec. 3.2 holds iff it is 0.  Negative = eep_status. */
int eep_host_uncovered_experts(int32_t P, int32_t E, int32_t S, const int32_t* phys_to_logical,
                               const int32_t* active);
/* How eep_dispatch_layout tiles T tokens of R source ranks:
 * out = {tokens per rank, tiles per rank, tokens per tile (<= 128), tiles}.
 * (Batches of at most 192 tokens and 1536 pairs are laid out by a single
 * workgroup without tiles; the results are the same.) */
int eep_host_tiling(int32_t T, int32_t R, int32_t out[4]);

/* Placement repair after a membership change (Sec. 3.5, Sec. 5.1; worked
 * example: Fig. 5, middle panel).  Host only.  Input: what every slot holds now
 * (cur_phys_to_logical[P], -1 = empty; slots of failed ranks included), the
 * active mask, and optionally a non-negative load per logical expert (NULL =
 * uniform).  Output: new_phys_to_logical[P] covering every logical expert on
 * live ranks (input for eep_update_placement), and for every slot where its
 * weights come from -- the paper's three-case source hierarchy:
 *   EEP_SRC_LOCAL  the slot keeps the expert it already holds (local reuse);
 *   EEP_SRC_PEER   copy from source_slot[p], a live slot holding the expert now
 *                  (GPU-to-GPU relocation);
 *   EEP_SRC_DRAM   no live copy existed: reload from the DRAM backup;
 *   EEP_SRC_NONE   empty slot or slot of a failed rank (left as it was).
 * The paper does not give its balancer's algorithm; this one is a deterministic
 * greedy rule: first cover experts with no live copy (hottest first; free slot
 * on the least-loaded live rank, else evict the cheapest replica that leaves
 * another live copy, redundant slots first), then use remaining free slots to
 * re-create lost replicas from surviving copies.
 * summary = {local, peer, dram, experts left uncovered}.  Returns EEP_OK, or
 * EEP_ERR_COVERAGE if some expert could not be placed (fewer live slots than
 * logical experts); outputs are filled in both cases. */
typedef enum { EEP_SRC_NONE = -1, EEP_SRC_LOCAL = 0, EEP_SRC_PEER = 1, EEP_SRC_DRAM = 2 }
    eep_repair_source;
int eep_plan_repair(int32_t R, int32_t S, int32_t S_prim, int32_t E,
                    const int32_t* cur_phys_to_logical, const int32_t* active, const float* load,
                    int32_t* new_phys_to_logical, int32_t* source_kind, int32_t* source_slot,
                    int32_t summary[4]);

/* Sources for moving from the current placement to a GIVEN target placement:
 * the step "resume preferred placement and full capacity" of the reintegration
 * sequence (Sec. 3.6; Fig. 5, right panel), classified with the same hierarchy
 * as eep_plan_repair.  Host only.
 *   active[R]    ranks whose copies can serve as sources;
 *   writable[R]  ranks whose slots may be filled: the active ranks plus, during
 *                reintegration, the relaunched rank, which loads its experts
 *                before it reports join-ready (mark the slots it lost as -1 in
 *                cur_phys_to_logical).
 * new_phys_to_logical[p] = target[p] on writable ranks, cur[p] elsewhere.  A slot
 * whose expert does not change is LOCAL; otherwise PEER from a slot on an active
 * rank that holds the expert now and gets no new weights in this batch (primary
 * slots first, then lowest slot id), else DRAM.  summary = {local, peer, dram, 0}.
 * Returns EEP_OK or EEP_ERR_INVALID_ARG. */
int eep_plan_transition(int32_t R, int32_t S, int32_t S_prim, int32_t E,
                        const int32_t* cur_phys_to_logical, const int32_t* target_phys_to_logical,
                        const int32_t* active, const int32_t* writable,
                        int32_t* new_phys_to_logical, int32_t* source_kind, int32_t* source_slot,
                        int32_t summary[4]);

/* Carry out a planned repair (Sec. 3.5: local reuse / batched GPU-to-GPU
 * relocation / reload from the DRAM backup; Sec. 5.1: the weights are moved to
 * where the new placement wants them, the active mask being looked up when
 * each transfer is issued), then publish the placement (as
 * eep_update_placement does), all in stream order.
 *   weights  device memory, [P][slot_bytes]: the expert weight store, slot-major
 *            (rank r owns slots [r*S, (r+1)*S)); updated in place.
 *   backup   [E][slot_bytes], readable by the GPU: device memory, or host memory
 *            pinned with hipHostMalloc (the paper's DRAM backup; read over the
 *            host link by the kernel).  May be NULL if the plan has no PEER and
 *            no DRAM slot.
 *   slot_bytes  > 0, multiple of 16; weights and backup 16-byte aligned.
 *   new_phys_to_logical, source_kind, source_slot  host int32[P], as written by
 *            eep_plan_repair for the placement this context holds now.
 *            (eep_plan_transition's output is accepted as well).
 * One kernel does the whole batch.  For each PEER slot p it reads the DEVICE
 * copy of the active mask: source rank active -> copy from source_slot[p];
 * source rank dropped out after planning -> copy backup[new_phys_to_logical[p]]
 * instead.  DRAM slots copy from the backup.  Only the source is looked up: the
 * destination may be a rank that is not active yet (Sec. 3.6: a relaunched rank
 * loads its experts before it joins).  What happened is recorded per slot
 * (eep_repair_outcome) and read back with eep_read_repair_outcome.
 * Checked on the host before anything is queued (EEP_ERR_INVALID_ARG):
 * a LOCAL slot keeps the expert the context's current placement gives it; a PEER
 * source is another slot that holds that expert now and is not itself rewritten
 * by this batch; both pointers are what they are said to be (weights: a device
 * allocation that contains all P slots; backup: GPU-accessible). */
typedef enum {
  EEP_REPAIR_UNTOUCHED = 0,
  EEP_REPAIR_FROM_PEER = 1,
  EEP_REPAIR_FROM_DRAM = 2,
  EEP_REPAIR_FROM_DRAM_FALLBACK = 3 /* planned peer source was no longer active */
} eep_repair_outcome;
int eep_apply_repair(eep_ctx* ctx, void* weights, const void* backup, int64_t slot_bytes,
                     const int32_t* new_phys_to_logical, const int32_t* source_kind,
                     const int32_t* source_slot, void* stream);
/* Outcome per slot of the last eep_apply_repair; synchronises the device. */
int eep_read_repair_outcome(eep_ctx* ctx, int32_t* outcome_host);

/* ---- De-duplicated dispatch (a data-path variant; Sec. 4.1 leaves payload
 * placement to prior work) --------------------------------------------------
 * One row per (token, destination RANK) instead of one per (token, expert): when
 * several of a token's experts live on one rank, the row crosses the fabric once
 * and is expanded on the destination.  Not for fp8 payloads (EEP_ERR_INVALID_ARG);
 * at most 1024 ranks.
 *   eep_dedup_layout    after eep_dispatch_layout of the same T: rank-major row of
 *                       every pair (token-ascending inside a rank), which pair
 *                       carries the row (the token's first on that rank), and for
 *                       every expert-major row the rank-major row behind it.
 *   eep_dispatch_dedup  recv_dedup[dedup_row] = x[t], once per (token, rank);
 *                       recv_dedup: device [T*k, H] x_dtype, the first N_d rows
 *                       are written (N_d <= N; rank r's rows are
 *                       [dedup_offset[r], dedup_offset[r+1])).
 *   eep_expand          on the destination: recv_x[row] = recv_dedup[expand_of[row]]
 *                       for the N routed rows; the result equals eep_dispatch's.
 *                       Expert kernels that can gather through expand_of skip it.
 * Call order violations return EEP_ERR_STATE. */
int eep_dedup_layout(eep_ctx* ctx, int32_t T, void* stream);
int eep_dispatch_dedup(eep_ctx* ctx, const void* x, void* recv_dedup, int32_t T, void* stream);
int eep_expand(eep_ctx* ctx, const void* recv_dedup, void* recv_x, int32_t T, void* stream);
/* Device arrays of the de-duplicated layout (fixed addresses, context-owned):
 * dedup_count[R], dedup_offset[R+1], dedup_row[T_max*k] (-1: pair not routed),
 * dedup_dst[T_max*k] (= dedup_row for the pair that carries the row, else -1),
 * expand_of[T_max*k] (-1 for rows >= N), status[1] = {N_d}. */
typedef struct {
  const int32_t *dedup_count, *dedup_offset, *dedup_row, *dedup_dst, *expand_of, *status;
} eep_dedup_view;
typedef enum {
  EEP_D_COUNT = 0, EEP_D_OFFSET, EEP_D_ROW, EEP_D_DST, EEP_D_EXPAND_OF, EEP_D_STATUS,
  EEP_D_NUM_FIELDS
} eep_dedup_field;
int eep_get_dedup_view(eep_ctx* ctx, eep_dedup_view* out);
/* Copies the first n ints of a field to the host after synchronising `stream`. */
int eep_read_dedup(eep_ctx* ctx, int32_t field, int32_t* host_dst, int64_t n, void* stream);

/* ---- hipGraph helper (Sec. 2.3, Fig. 4: capture once, replay, patch table
 * contents only) ------------------------------------------------------------
 * eep_graph_begin puts `stream` (not the default stream) into capture mode;
 * the per-step calls made on it until eep_graph_end are recorded, not run.
 * eep_graph_end instantiates the graph exactly once.  eep_graph_launch replays
 * it on `stream`.  The library never calls hipGraphExecUpdate and never
 * re-instantiates; eep_graph_counters reports how often each happened so that
 * a test can assert it. */
typedef struct eep_graph eep_graph;
int eep_graph_begin(eep_ctx* ctx, void* stream);
int eep_graph_end(eep_ctx* ctx, void* stream, eep_graph** out);
int eep_graph_launch(eep_graph* g, void* stream);
int eep_graph_destroy(eep_graph* g);
/* counters[0] = instantiations, [1] = exec updates, [2] = launches of this graph. */
int eep_graph_counters(const eep_graph* g, int64_t counters[3]);

#ifdef __cplusplus
}
#endif
#endif /* EEP_H_ */
