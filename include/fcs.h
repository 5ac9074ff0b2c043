/*
 * fcs.h - C ABI of the flow-controlled-scheduling sample-path engine (gfx950).
 *
 * The engine evaluates, as many independent sample paths, the slotted model of
 * one LLM-serving worker with a KV-cache budget M (Section 2.1 of the paper)
 * under the flow-control admission rule with unknown output length
 * (Algorithm 2, Section 3.3), under its greedy limit (remark after
 * Theorem 2; fit test "initial memory l+1" of Section 4.1) and under the
 * rule for known output lengths (Algorithm 1, Section 3.2), extended by a
 * per-slot token budget and chunked prefill (Section 1 describes both as
 * current practice; the paper's pure model is recovered with chunk >= l_max
 * and an unlimited budget).
 *
 * One slot of one path, in this order:
 *   1. n_t requests arrive and join the tail of the waiting queue Q.
 *   2. admission.  FLOW: the first min(B_t, |Q|) requests of Q join the active
 *      set P, B_t = b_floor + [u < b_frac_thr].  GREEDY: the head of Q joins
 *      while (sum_P (l+j)) + |P| + l_head + 1 <= M.
 *      CLASSES (Algorithm 1): every class k of the length mixture has its own
 *      arrival stream n_{t,k}, its own FIFO queue and an integer budget b_k; in
 *      class order the first min(b_k, |Q_k|) requests of class k join P.
 *      ALPHA (alpha-protection greedy baseline, Section 4.1): as GREEDY, against
 *      floor((1 - alpha) M) instead of M (fcs_protect_limit).
 *      MC (memory-check benchmark, Section 4.1): first come first served, the
 *      head joins P only if the memory stays within M in every future slot of the
 *      prediction in which each request produces assumed_o tokens, one per slot
 *      from the slot of its activation, holds l + (tokens so far) and leaves after
 *      its last one.  Needs the slot model without chunking or token budget:
 *      prefill_chunk >= largest l, token_budget = 2^30, largest l + assumed_o <= M.
 *   3. overflow.  While (sum_P (l+j)) + |P| > M the most recently activated
 *      request is evicted: it loses its progress and returns to the FRONT of Q.
 *      ALPHA: once that condition holds ALL active requests are evicted.
 *      CLASSES: Algorithm 1 has no such step (Theorem 1 keeps the usage below M
 *      when sum_k b_k w_k < M); the slots in which the condition holds are only
 *      counted in FCS_C_OVERFLOW_STEPS and the usage may exceed M.
 *   4. processing with token budget tau and chunk c.  Prefilling requests, in
 *      activation order, advance min(c, l-p, budget left); the slot in which
 *      the prompt ends also yields output token 1 at no extra budget.  Then the
 *      requests that were already decoding, in activation order, gain one token
 *      each while budget lasts; the others stall.
 *   5. U_t = sum_P (l+j), |P_t| and |Q_t| are measured.
 *   6. requests with j == o complete: completion slot t, latency t - t_arr + 1,
 *      footprint released at the end of the slot.
 *
 * Randomness.  Philox4x32-10 with key (seed & 0xffffffff, seed >> 32) and
 * counter (k, t, replica, purpose).  purpose 0, k 0: word 0 -> n_t, word 1 ->
 * B_t.  purpose 1, k = index of the arrival within slot t: word 0 -> class,
 * word 1 -> l, word 2 -> o.  A word u is inverted against a law's threshold
 * table: value = lo + #{ i : u >= thr[i] }.  CLASSES cells use purpose 2
 * instead, k = class: word 0 -> n_{t,k}; all requests of class k have l = lo of
 * its prompt law and o = lo of its decode law, which must be point laws, and
 * their ids are (index within the class) * n_classes + k.  All cells of one engine see the
 * same words (the policy and the cell are not part of the counter), so cells
 * are compared on identical arrival streams.
 *
 * Memory and ownership.  The library allocates no device memory.  The caller
 * owns one device workspace (size from fcs_workspace_bytes) and the device
 * output arrays of fcs_outputs, and passes raw device pointers; "stream" is a
 * hipStream_t passed as void*.  All fcs_law/fcs_cell/fcs_params pointers are
 * HOST pointers and are copied by fcs_create; they may be freed afterwards.
 *
 * Errors.  Every call returns FCS_OK (0) or a negative code; nothing throws or
 * aborts across this boundary.  The library needs a HIP device: there is no
 * CPU fallback, and calls that need the GPU return FCS_EDEVICE without one.
 */
#ifndef FCS_H_
#define FCS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fcs_engine* fcs_handle;

enum {
  FCS_OK = 0,
  FCS_EINVAL = -1,    /* bad argument or parameter combination                    */
  FCS_ENOMEM = -2,    /* workspace too small / host allocation failed             */
  FCS_ESTATE = -3,    /* call out of order (run before bind, stats before run)    */
  FCS_EOVERFLOW = -4, /* a path outgrew max_active or produced >= 2^31 arrivals   */
  FCS_EDEVICE = -5    /* HIP error or no device                                   */
};

enum { FCS_POLICY_FLOW = 0, FCS_POLICY_GREEDY = 1, FCS_POLICY_CLASSES = 2, FCS_POLICY_ALPHA = 3,
       FCS_POLICY_MC = 4 };
enum { FCS_BUDGET_SPLIT = 0, FCS_BUDGET_LAW = 1, FCS_BUDGET_CREDIT = 2 };

/* Integer law on {lo, ..., lo + n_thr}; thr non-decreasing (host pointer). */
typedef struct fcs_law {
  int32_t lo;
  int32_t n_thr;
  const uint32_t* thr;
} fcs_law;

/* One policy setting evaluated on the shared random streams. */
typedef struct fcs_cell {
  int32_t policy;      /* FCS_POLICY_*                                             */
  int32_t arrival;     /* index into fcs_params.arrival                            */
  int32_t b_floor;     /* FLOW: B_t = b_floor + [u < b_frac_thr]  (Theorem 2: any  */
  uint32_t b_frac_thr; /*   bounded i.i.d. integer budget with mean b)             */
  const int32_t* class_arrival; /* CLASSES: n_classes indices into fcs_params.arrival, */
                                /*   the law of n_{t,k} of each class (host pointer)   */
  const int32_t* class_budget;  /* CLASSES: n_classes budgets b_k, 0 .. 64, sum <= 64  */
  double alpha;                 /* ALPHA: protected share of the memory, 0 <= alpha <= 1;   */
                                /*   admission may fill fcs_protect_limit(alpha, M) tokens  */
  int32_t budget_mode;          /* FLOW: how B_t is formed.  FCS_BUDGET_SPLIT (0): b_floor  */
                                /*   + [u < b_frac_thr]; FCS_BUDGET_LAW: drawn from the     */
                                /*   count law fcs_params.arrival[budget_law] (any bounded  */
                                /*   integer law, Theorem 2; values <= 30000);              */
                                /*   FCS_BUDGET_CREDIT: floor(t b) - floor((t - 1) b), the  */
                                /*   deterministic budget of a credit accumulator, b =      */
                                /*   budget_b16 / 65536 <= 30000                            */
  int32_t budget_law;
  uint32_t budget_b16;
  int32_t assumed_o;            /* MC: the output length o_hat every request is taken to    */
                                /*   reach in the prediction, >= the largest o possible     */
} fcs_cell;

typedef struct fcs_params {
  int32_t capacity;       /* M, tokens, 1 .. 2^30                                  */
  int32_t token_budget;   /* tau per slot, 1 .. 2^30                               */
  int32_t prefill_chunk;  /* c, 1 .. 2^30                                          */
  int32_t n_classes;      /* classes of the length mixture nu, 1 .. 16             */
  const uint32_t* class_thr; /* n_classes - 1 cumulative class thresholds          */
  const fcs_law* prompt;  /* per class: law of l, lo >= 1                          */
  const fcs_law* decode;  /* per class: law of o, lo >= 1; max l + max o <= M      */
  int32_t n_arrival_laws;
  const fcs_law* arrival; /* count laws (at most 63 thresholds): of n_t and n_{t,k}, */
                          /* which need lo = 0, and of B_t under FCS_BUDGET_LAW      */
  int32_t n_cells;
  const fcs_cell* cells;
  int32_t trace_every;    /* > 0: record (|Q_t|, U_t) at t = k, 2k, ...            */
  int32_t hist_bins;      /* > 0: latency histogram, bucket = min(lat >> shift, bins-1) */
  int32_t hist_shift;
  int32_t max_requests;   /* > 0: per-path length of arrival_step/completion_step  */
  int32_t max_active;     /* per-path capacity of the active set, up to 2^24; 0 = default:
                           * M / (min l + 1) + 1, and with CLASSES cells at least
                           * sum_k b_k (ceil(l_k / min(c, tau)) + o_k + 1); the default
                           * is at most 8192 */
  int32_t lds_slots;      /* active-set slots kept in LDS per path; 0 = automatic, else 256, 320, 384,
                             448, 512 or a multiple of 256 up to 4096                               */
  /* Slots of variable duration (all three 0: every slot lasts one time unit).  Time runs
   * in the units of the arrival laws: n_u requests arrive in unit u; slot t starts at time
   * tau_t (tau_1 = 1), sees the arrivals of the units up to tau_t and lasts
   * d_t = time_c0 + time_cp * (prompt tokens it processed) + time_cd * (output tokens it
   * generated) units; a request completing in it does so in unit tau_t + d_t - 1.  Latencies,
   * arrival_step and completion_step are then in time units and FCS_C_ELAPSED is the time
   * the n_steps slots took.  time_c0 >= 1; not with CLASSES cells; n_steps times the
   * longest possible d_t must stay below 2^30 (checked by fcs_run). */
  int32_t time_c0, time_cp, time_cd;
  /* FCS_FLAG_* bits, 0 = none.
   * FCS_FLAG_SKIP_IDLE: event skipping.  A run of slots in which nothing happens but decode growth
   * (no arrival, no admission, no prefill, no completion, no overflow, no trace sample) is advanced in one
   * go inside the kernel's slot loop: with n decoding requests and usage U before the run, k such slots
   * add k U + n k (k + 1) / 2 to sum_t U_t (the growth term of the expression for U_t in the proof of
   * Theorem 2, summed), k |P| and k |Q| to the other sums, and leave U + k n.  Every output is the same as
   * without the flag; only the time differs.  Engines whose cells are all FLOW or GREEDY, no time model.
   * FCS_FLAG_GENERAL_CODE: a test switch; every slot runs in the kernel's general code and none in the
   * hand-scheduled loop (the two are separate renditions of the same slot and must agree). */
  int32_t flags;
} fcs_params;

enum { FCS_FLAG_SKIP_IDLE = 1, FCS_FLAG_GENERAL_CODE = 2 };

/* Per-path counters, uint64 each, FCS_N_COUNTERS per path. */
enum {
  FCS_C_ARRIVED = 0,     /* requests arrived in slots 1..T                          */
  FCS_C_ACTIVATIONS,     /* activations, re-activations after eviction included     */
  FCS_C_COMPLETED,
  FCS_C_EVICTIONS,
  FCS_C_OVERFLOW_STEPS,  /* slots in which U_t + |P_t| passed M after admission:
                          * with at least one eviction, or (CLASSES) only counted  */
  FCS_C_SUM_U,           /* sum_t U_t                                               */
  FCS_C_SUM_P,           /* sum_t |P_t| : the request-steps of the path             */
  FCS_C_SUM_Q,           /* sum_t |Q_t|                                             */
  FCS_C_DECODE_TOKENS,   /* output tokens generated, discarded ones included        */
  FCS_C_PREFILL_TOKENS,  /* prompt tokens processed, discarded ones included        */
  FCS_C_USEFUL_TOKENS,   /* sum of o over completed requests                        */
  FCS_C_STALLED,         /* request-slots in which a decoding request got no token  */
  FCS_C_SUM_LATENCY,     /* sum of (completion - arrival + 1) over completed        */
  FCS_C_MAX_LATENCY,
  FCS_C_MAX_U,
  FCS_C_MAX_P,
  FCS_C_MAX_Q,
  FCS_C_FINAL_U,
  FCS_C_FINAL_P,
  FCS_C_FINAL_Q,
  FCS_C_DIGEST,          /* FNV-1a (64-bit words) of the final state, see below     */
  FCS_C_ERROR,           /* 0, or -code of the error that stopped the path          */
  FCS_C_ERROR_STEP,      /* slot at which it stopped                                */
  FCS_C_ELAPSED,         /* time units the slots took (= n_steps while every slot   */
                         /* lasts one unit)                                         */
  FCS_C_CLOCK_START,     /* device wall clock (ticks of 10 ns, the GPU's constant   */
  FCS_C_CLOCK_END,       /* 100 MHz counter) when the path's workgroup started and  */
                         /* ended: for profiling; not reproducible from run to run  */
  FCS_N_COUNTERS
};
/* Digest: h = 14695981039346656037; for each word x: h = (h ^ x) * 1099511628211.
 * Words: |P|; for each active request in activation order: id, j, p; the number
 * of waiting requests that were active before; their ids in queue order; the
 * number of waiting requests never activated.  ids number a path's arrivals
 * 0,1,2,... in order of (slot, index within slot).  CLASSES: after the active
 * requests come n_classes words, the number of waiting requests of each class. */

/* Device output arrays (caller-owned).  counters is required; the others may be
 * NULL, and must be non-NULL only if the matching parameter is > 0 and wanted. */
typedef struct fcs_outputs {
  uint64_t* counters;        /* [n_paths][FCS_N_COUNTERS]                           */
  int32_t* trace_q;          /* [n_paths][n_steps / trace_every]                    */
  int32_t* trace_u;          /* same shape                                          */
  uint32_t* hist;            /* [n_paths][hist_bins]                                */
  int32_t* arrival_step;     /* [n_paths][max_requests], 0 = no such request        */
  int32_t* completion_step;  /* [n_paths][max_requests], 0 = not completed          */
  int64_t trace_entries;     /* int32 entries that trace_q and trace_u each hold    */
} fcs_outputs;
/* path = cell * n_replicas + replica, n_paths = n_cells * n_replicas, with the
 * n_replicas of the RUN for every array: a run of fewer replicas than were bound
 * packs its rows at the start of the arrays (cell c begins at row c * n_replicas
 * of that run), and fcs_stats / fcs_percentile index the same way.  The arrays
 * must hold the rows of the largest run; the trace rows also depend on n_steps,
 * and fcs_run refuses a run whose n_paths * (n_steps / trace_every) exceeds
 * trace_entries. */

typedef struct fcs_summary {
  int64_t n_paths;
  int64_t n_steps;
  uint64_t request_steps;   /* sum of FCS_C_SUM_P                                   */
  uint64_t arrived;
  uint64_t completed;
  uint64_t evictions;
  uint64_t overflow_steps;
  double mean_latency;      /* slots, over completed requests (Section 2.2)         */
  double kv_utilisation;    /* sum_t U_t / (T * M), averaged over paths             */
  double token_throughput;  /* useful output tokens per slot per path (Section 2.2) */
  double prompt_throughput; /* completed requests per slot per path                 */
  double mean_queue;        /* time-average |Q_t|                                   */
  double mean_active;       /* time-average |P_t|                                   */
  int64_t first_error_path; /* -1 if no path stopped with an error                  */
  int32_t error_code;
  int32_t reserved;
} fcs_summary;

/* Validates and copies the parameters.  FCS_EINVAL on any violated range above,
 * a decreasing threshold table, or max(l) + max(o) > M (Section 2.1 requires
 * U_t <= M; a request that cannot fit alone would be evicted forever). */
int fcs_create(const fcs_params* params, fcs_handle* out);

/* Bytes of device workspace needed to run n_replicas paths per cell. */
int fcs_workspace_bytes(fcs_handle h, int64_t n_replicas, size_t* bytes);

/* Uploads the tables into the workspace (asynchronously on stream) and records
 * the workspace and output pointers.  workspace must be 256-byte aligned.
 * FCS_ENOMEM if bytes is too small for n_replicas. */
int fcs_bind(fcs_handle h, void* dev_workspace, size_t bytes, int64_t n_replicas,
             const fcs_outputs* dev_out, void* stream);

/* Simulates n_replicas sample paths per cell for slots 1..n_steps (Algorithm 2's
 * loop over t), replica r of every cell using Philox replica index
 * replica_base + r.  Asynchronous on stream; one workgroup of one wavefront per
 * path.  n_replicas must not exceed the bound value; 1 <= n_steps < 2^30;
 * FCS_EINVAL also when the trace arrays are too short for the run. */
int fcs_run(fcs_handle h, int64_t n_replicas, int64_t n_steps, uint64_t seed, void* stream);

/* Same with an explicit first replica index (sharding a sweep over devices). */
int fcs_run_from(fcs_handle h, int64_t replica_base, int64_t n_replicas, int64_t n_steps,
                 uint64_t seed, void* stream);

/* For callers that cannot allocate device memory or pass a workspace around (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): fcs_bind and fcs_run in one call, on a
 * workspace that the library itself holds on every GPU it is loaded on, FCS_STATIC_WORKSPACE_BYTES of
 * device memory per GPU from load until the process ends.  The call allocates nothing.  dev_out are
 * caller-owned device arrays as for fcs_bind, sized for this call's n_replicas; replica indices start at 0.
 * FCS_ENOMEM when the tables plus the spill regions of n_replicas paths per cell (what
 * fcs_workspace_bytes reports) exceed the workspace: lower n_replicas or fcs_params.max_active.
 * The tables are uploaded when the workspace last held another engine's (that call waits for the
 * stream once); otherwise the call only launches.  All calls on one GPU share the workspace: calls that
 * overlap in time on one GPU race, whatever their streams; run them one after the other.  The current
 * device at the time of the call is the one that is used.  fcs_stats, fcs_percentile and fcs_geometry
 * afterwards refer to this run as they do after fcs_run. */
#define FCS_STATIC_WORKSPACE_BYTES (32u << 20)
int fcs_run_static(fcs_handle h, const fcs_outputs* dev_out, int64_t n_replicas, int64_t n_steps,
                   uint64_t seed, void* stream);

/* Waits for the last run, copies the per-path counters to host_counters
 * ([n_paths][FCS_N_COUNTERS], may be NULL) and fills the summary of one cell
 * (cell >= 0) or of all paths (cell = -1).  If a path stopped with an error
 * the call returns the first such path's code, FCS_EOVERFLOW (it outgrew
 * max_active or the evicted stack; raise max_active) or FCS_ESTATE (its state
 * became inconsistent: a defect, not an input error); the counters and the
 * summary still describe what was simulated, and summary->first_error_path
 * and error_code name the path and its code. */
int fcs_stats(fcs_handle h, int32_t cell, uint64_t* host_counters, fcs_summary* summary);

/* Nearest-rank percentile num/den of the request latency of every path, from
 * the device histogram of the last run (Section 4: average and tail latency):
 * value[p] = (bucket of the ceil(q*n)-th smallest latency) << hist_shift,
 * saturated[p] = 1 if that is the last bucket.  Host output arrays of n_paths. */
int fcs_percentile(fcs_handle h, int64_t num, int64_t den, int32_t* value, uint8_t* saturated);

/* lambda* = M / E[l o + (o + o^2)/2] for the parameter's mixture (Proposition 2,
 * eq. 3), l and o independent within a class.  Host only. */
int fcs_stability_bound(const fcs_params* params, double* lambda_star);

/* What admission may fill under the alpha-protection greedy baseline of Section 4.1:
 * *limit = floor((1 - alpha) * capacity), the product formed in IEEE double precision.
 * FCS_EINVAL unless 0 <= alpha <= 1 and 1 <= capacity <= 2^30.  Host only. */
int fcs_protect_limit(double alpha, int32_t capacity, int32_t* limit);

/* Launch geometry of the last run, or before any run the one chosen by fcs_bind: LDS slots per path,
 * LDS bytes per workgroup, spill slots per path. */
int fcs_geometry(fcs_handle h, int32_t* lds_slots, int32_t* lds_bytes, int32_t* spill_slots);

void fcs_destroy(fcs_handle h);
const char* fcs_strerror(int code);
int fcs_n_counters(void);
const char* fcs_counter_name(int index);

#ifdef __cplusplus
}
#endif
#endif /* FCS_H_ */
