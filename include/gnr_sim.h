/*
 * gnr_sim.h -- C ABI of the MI355X Monte-Carlo simulator of the multiclass many-server
 * LLM-inference queueing network under the gate-and-route policy.
 *
 * The network is the one of the paper's Sec. 2.3 ("The Stochastic Model"): class prefill
 * queues Q_p,i, prefill occupancy X_i, one decode buffer Q_d,i, mixed and solo decode
 * occupancy Y_m,i / Y_s,i, on n servers that each host at most one prefill and B decodes.
 * One batch iteration advances every decode of the batch by one token and the prefill by one
 * chunk of at most C tokens (Sec. 2.2); its duration is c0 + c_pre*prefill_tokens +
 * c_dec*n_decode, so a prefill in the batch slows the co-resident decodes.
 * Control is the policy of Sec. 4: static partition into M mixed and n-M solo servers,
 * occupancy-deviation prefill gate, solo-first work-conserving decode router.
 * Revenue is recognised as in Sec. 2.3 (bundled: at request completion; separate: prompt
 * tokens at prefill completion, output tokens at decode completion).
 * Other gates (static priority, FCFS) and routers (SLI-aware randomized and weighted routers, immediate
 * decode on the prefill's server) are selected by gate_mode and route_mode: see enum sim_gate, enum sim_route.
 *
 * Time advances in fixed steps of length dt. Every server keeps an exact clock (integer ns) for
 * the end of its running iteration; in step s (boundary time T_s = (s+1)*dt) the library
 *   0. removes from the class queues and from the decode buffer every request whose patience ends in this step,
 *   1. draws per-server Poisson arrivals for the window and appends them to the class queues,
 *   2. completes the iteration of every server whose clock is <= T_s,
 *   3. runs the prefill gate over idle prefill slots of the mixed group, ascending server index,
 *   4. routes the decode buffer (FIFO) to the least-loaded feasible server, solo group first,
 *   5. restarts servers back-to-back from their own clock (idle servers start at T_s),
 *   6. adds the end-of-step queue lengths and occupancies to their running sums.
 * Replications are independent copies of the system with their own random streams
 * (Philox4x32-10 keyed on the seed, counter = (step, stream, server, replication)).
 *
 * Abandonment (Sec. 2.3: a waiting class-i request has an exponential patience with rate theta_i, in the prefill
 * queue and again in the decode buffer). A request is asked at the start of every step after the one it joined
 * the queue in, so its patience in steps is geometric: Pr(patience >= m) = exp(-theta*dt*(m-1)), m = 1, 2, ...,
 * drawn by the same quantile-table lookup as the lengths (hence at most 32768 steps). The j-th accepted
 * class-k arrival of step s takes word 0 of block (s, stream 2+k, j, replication); a request whose prefill
 * completes on server g in step s takes word 0 of block (s, stream 10, g, replication) for the decode buffer.
 * A request that joined in step s with patience m can be admitted (routed) in steps s .. s+m-1 and leaves at
 * the start of step s+m.
 *
 * All functions return 0 on success or a negative sim_err; none throws, aborts or prints.
 * Pointers are host pointers unless a comment says "device".
 */
#ifndef GNR_SIM_H
#define GNR_SIM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SIM_MAXK 8      /* classes */
#define SIM_MAXB 128    /* decode slots per server */
#define SIM_MAXN 12288  /* servers per replication: no configuration may have more; how many fit depends on the
                           on-chip memory they need (see sim_onchip_bytes) */
#define SIM_NBIN 720    /* latency histogram bins: exact below 16 ns, then 16 bins per octave */
#define SIM_MAXR (1 << 20) /* replications of one handle: keeps every size of the workspace layout far below 2^64 */

enum sim_err { SIM_OK = 0, SIM_EINVAL = -1, SIM_ENOMEM = -2, SIM_EHIP = -3, SIM_EOVERFLOW = -4 };
enum sim_law { SIM_GEOMETRIC = 0, SIM_LOGNORMAL = 1, SIM_CONST = 2, SIM_TABLE = 3 };
enum sim_gate { SIM_GATE_OCCUPANCY = 0, SIM_GATE_PRIORITY = 1, SIM_GATE_FCFS = 2 };
/* Decode routers. SOLO_FIRST: the router of Sec. 4 (one buffer; solo group first, then the mixed group).
 * RANDOM_SPLIT: the SLI-aware randomized router of Sec. 5.2 (zero-buffer case): when the prefill of a class-i
 * request completes it is sent to the solo group with probability p_s,i, else to the mixed group; each group
 * has its own FIFO buffer (capacity dbuf_cap each) that feeds that group only; within the group the placement
 * rule is the same as for SOLO_FIRST (least-loaded feasible server, lowest index). The draw is word 1 of block
 * (step, stream 10, server of the prefill, replication): solo iff word < floor(p_s,i * 2^32) (clamped to
 * 2^32 - 1, so p_s,i = 1 sends one request in 2^32 to the mixed group).
 * IMMEDIATE: no decoupled router (the "I" decode rule of the paper's ablation study, policies GI-WSP and FI-WSP):
 * a request whose prefill completes goes on decoding on the same server, in the slot it already holds, and joins
 * the batch at the restart that follows; a server holds at most B requests, its prefill included, so the gate
 * admits only to servers with no prefill in service and fewer than B decodes; the decode buffer stays empty.
 * ("WSP", without static planning, is a configuration with M = N.)
 * WEIGHTED_SPLIT: the general SLI-aware router (EC, "General SLI-aware Extension"): requests are sent to the
 * solo or the mixed pool's buffer as under RANDOM_SPLIT; whenever a slot of a pool is filled, the class is drawn
 * with the pool's selection weights (w_solo = varpi_s, w_mixed = varpi_m) restricted to the classes that wait in
 * that pool's buffer, and the head-of-line request of that class is taken (FCFS within a class). Weights are
 * used in units of 2^-20, rounded to nearest and never below one unit (a class of weight zero is served when no
 * other class waits, so a pool stays work-conserving). The j-th placement of a step in a pool draws word 0 of
 * block (step, stream 11 for the solo / 12 for the mixed pool, j, replication): with W the sum of the units of
 * the waiting classes, x = (word * W) >> 32 falls into the interval of the chosen class, classes in ascending
 * order. The server is the least-loaded feasible one of the pool, as for the other routers. */
enum sim_route { SIM_ROUTE_SOLO_FIRST = 0, SIM_ROUTE_RANDOM_SPLIT = 1, SIM_ROUTE_IMMEDIATE = 2,
                 SIM_ROUTE_WEIGHTED_SPLIT = 3 };

/* Per-class cumulative tallies (uint64), in this order. Counting processes as in Sec. 2.3:
 * A arrivals, U_P admissions to prefill, S_P prefill completions, U_DM/U_DS admissions to a
 * decode slot of a server that does / does not hold a prefill, S_DM/S_DS decode completions by the
 * same distinction, M_SM/M_MS decodes switched solo->mixed / mixed->solo by a prefill admission /
 * completion on their server. DROP_* count requests lost to a full ring. TOKP_PRE: prompt tokens
 * recognised at prefill completion; TOKP_DEC/TOKD_DEC: prompt/output tokens recognised at decode
 * completion; TOK_EMIT output tokens emitted; TOK_PREF prompt tokens processed. SUM_*: end-of-step
 * values summed over steps. WAIT_STEPS: sum over admitted requests of (admission step - arrival
 * step). *_SUM: latency sums in ns (TTFT over S_P, E2E over S_DM+S_DS, TBT over TOK_EMIT).
 * AB_P / AB_D: abandonments from the class prefill queue / from the decode buffer (B_p,i and B_d,i). */
enum sim_tally {
  SIM_T_A = 0, SIM_T_DROP_P, SIM_T_U_P, SIM_T_S_P, SIM_T_U_DM, SIM_T_U_DS, SIM_T_S_DM, SIM_T_S_DS,
  SIM_T_M_SM, SIM_T_M_MS, SIM_T_DROP_D, SIM_T_TOKP_PRE, SIM_T_TOKP_DEC, SIM_T_TOKD_DEC, SIM_T_TOK_EMIT,
  SIM_T_TOK_PREF, SIM_T_SUM_QP, SIM_T_SUM_QD, SIM_T_SUM_X, SIM_T_SUM_YM, SIM_T_SUM_YS, SIM_T_WAIT_STEPS,
  SIM_T_TTFT_SUM, SIM_T_E2E_SUM, SIM_T_TBT_SUM, SIM_T_AB_P, SIM_T_AB_D, SIM_NTALLY
};
/* Per-replication tallies: executed iterations and busy ns by kind (a "mix" iteration holds a
 * prefill chunk), steps run, and 1 if any ring overflowed. */
enum sim_global { SIM_G_ITERS_MIX = 0, SIM_G_ITERS_SOLO, SIM_G_BUSY_MIX, SIM_G_BUSY_SOLO, SIM_G_STEPS,
                  SIM_G_OVERFLOW, SIM_NGLOBAL };

/* One request class (primitives of Sec. 2.3). Lengths are integers in [1, 32768] drawn by
 * inverse-cdf lookup in a 65536-entry quantile table: entry j is the smallest k whose cdf reaches
 * (j+0.5)/65536. GEOMETRIC: p0 = mean, Pr(X >= k) = (1-1/mean)^(k-1). LOGNORMAL: p0 = median,
 * p1 = sigma, rounded to the nearest integer and clamped. CONST: p0. TABLE: caller's table. */
typedef struct {
  double lambda;                 /* arrivals per server per unit time */
  int in_law, out_law;           /* enum sim_law */
  double in_p0, in_p1, out_p0, out_p1;
  const uint16_t *in_table, *out_table; /* 65536 entries each, copied; only for SIM_TABLE */
  double price_in, price_out;    /* c_p, c_d: price per prompt / output token */
  int bundled;                   /* 1: this class counts bundled revenue in rev_mixed, 0: separate */
  double priority;               /* static index of the priority gate (larger first), e.g. D_i/P_i */
  double theta;                  /* patience rate of a waiting request, >= 0; 0 = never abandons */
} sim_class;

typedef struct {
  int K, N, B, C;                /* classes <= 8, servers <= 12288, decode cap <= 128, chunk <= 8191 */
  double c0, c_pre, c_dec;       /* iteration time c0 + c_pre*ptok + c_dec*n_dec, rounded to ns */
  double dt;                     /* step length, 0 < dt <= c0; 0 selects dt = c0 */
  const sim_class *cls;          /* K entries, copied */
  int M;                         /* mixed servers 0..M-1 (ceil(n * sum x*)); servers M..N-1 are solo */
  const double *x_star;          /* K prefill-occupancy targets per server; 0 = never admit (occupancy gate) */
  const double *qp_star;         /* K prefill-queue targets per server (gate tie-break) */
  int gate_mode;                 /* enum sim_gate */
  int route_mode;                /* enum sim_route */
  double mod_amp;                /* arrival modulation lambda(s) = lambda*(1 + amp*sin(2*pi*(s mod period)/period)) */
  int64_t mod_period;            /* in steps; 0 = homogeneous */
  int64_t queue_cap, dbuf_cap;   /* ring capacities: per class prefill queue, decode buffer */
  const double *p_solo;          /* RANDOM_SPLIT, WEIGHTED_SPLIT: K probabilities p_s,i in [0,1], copied; else unused, may be NULL */
  const double *w_solo;          /* WEIGHTED_SPLIT: K class selection weights of the solo pool in [0,1] (varpi_s,i), copied */
  const double *w_mixed;         /* WEIGHTED_SPLIT: ... of the mixed pool (varpi_m,i); both unused otherwise, may be NULL */
} sim_config;

/* Totals over replications plus derived fp64 figures (rates per server per unit time). */
typedef struct {
  int32_t K, replications;
  int64_t steps;
  double sim_time;
  uint64_t tally[SIM_MAXK][SIM_NTALLY];
  uint64_t glob[SIM_NGLOBAL];
  double arrival_rate[SIM_MAXK], completion_rate[SIM_MAXK], served_fraction[SIM_MAXK];
  double tok_rate_prefill[SIM_MAXK], tok_rate_decode[SIM_MAXK];
  double rev_bundled[SIM_MAXK], rev_separate[SIM_MAXK], rev_mixed[SIM_MAXK];
  double rev_bundled_total, rev_separate_total, rev_mixed_total;
  double mean_qp[SIM_MAXK], mean_qd[SIM_MAXK], mean_x[SIM_MAXK], mean_ym[SIM_MAXK], mean_ys[SIM_MAXK];
  double ttft_mean[SIM_MAXK], ttft_p50[SIM_MAXK], ttft_p95[SIM_MAXK], ttft_p99[SIM_MAXK];
  double e2e_mean[SIM_MAXK], e2e_p50[SIM_MAXK], e2e_p95[SIM_MAXK], e2e_p99[SIM_MAXK];
  double tbt_mean[SIM_MAXK], tbt_p50[SIM_MAXK], tbt_p95[SIM_MAXK], tbt_p99[SIM_MAXK];
  double mean_wait[SIM_MAXK];
  double fair_gap_x, fair_gap_ys, fair_min_served;   /* fairness SLIs of Sec. 5.2, measured */
  double util_mix, util_solo, iter_rate;
  double abandon_rate_p[SIM_MAXK], abandon_rate_d[SIM_MAXK]; /* abandonments per server per unit time */
} sim_stats_t;

/* Integer state of one replication, copied into caller-allocated host arrays (NULL = skip).
 * A request is packed as stamp | cls<<29 | (P-1)<<32 | (D-1)<<48 (arrival step, class, prompt and
 * output length). Slot order within a server carries no meaning. */
typedef struct {
  int64_t *class_state;   /* [5][K]: Qp, X, Qd, Ym, Ys */
  int64_t *t_next;        /* [N] end of the running iteration in ns, INT64_MAX when idle */
  uint32_t *iter;         /* [N] completed iterations */
  int32_t *rem, *ptok;    /* [N] prompt tokens left of the prefill in service; tokens in the running chunk */
  uint64_t *pfjob;        /* [N] request in prefill service (0 when none) */
  uint8_t *n_cls, *n_join;/* [N][8] decodes per class; of those, joined after the running iteration started */
  uint32_t *fin;          /* [N][B] iteration index at which the slot's request emits its last token */
  uint64_t *job;          /* [N][B] request of the slot; slots 0..n_dec-1 are occupied */
  int32_t *n_dec;         /* [N] */
  uint64_t *queue[SIM_MAXK]; int64_t queue_len[SIM_MAXK]; /* arrival stamps, head first; capacity queue_cap */
  uint64_t *dbuf; int64_t dbuf_len;                        /* decode buffer requests, head first; capacity dbuf_cap */
  uint64_t *queue_dl[SIM_MAXK];  /* per queue entry: the step at whose start it abandons if still waiting (2^32-1: never) */
  uint64_t *dbuf_dl;             /* the same for the decode buffer entries */
  uint64_t *dbuf_m; int64_t dbuf_m_len; /* RANDOM_SPLIT: the mixed group's buffer (`dbuf` is then the solo group's) */
} sim_state_t;

typedef struct sim_t sim_t;  /* opaque; owned by the library */

/* Device bytes sim_create needs for `max_replications` replications of `cfg`. */
int sim_workspace_bytes(const sim_config *cfg, int max_replications, size_t *out_bytes);

/* Validates and deep-copies the config, builds the sampler tables on the host and uploads them
 * into `dev_workspace` (device pointer, 256-byte aligned, owned by the caller, must outlive the
 * handle). SIM_EINVAL: bad sizes (more than SIM_MAXR replications among them), negative target, M outside [0,N], dt > c0, negative theta, p_solo outside
 * [0,1] or missing under RANDOM_SPLIT, total
 * arrival mean per server-step above 0.05 (the per-step count is truncated at 3).
 * SIM_ENOMEM: workspace too small. The library never allocates device memory itself.
 * The handle belongs to the device that is current at this call: every later call on it must be made
 * with the same device current (SIM_EINVAL otherwise). The launch shape of the handle (see sim_launch_plan) is
 * fixed here for `max_replications` replications; runs with fewer use the same shape, results do not depend on it. */
int sim_create(const sim_config *cfg, int max_replications, void *dev_workspace, size_t bytes, sim_t **out);

/* sim_create for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): the workspace is a device array inside the library, SIM_STATIC_WORKSPACE_BYTES
 * large, that each GPU the library runs on holds until the process ends. Nothing is allocated: no hipMalloc,
 * no hipFree, on no path. Arguments, checks and results are those of sim_create; SIM_ENOMEM when
 * sim_workspace_bytes(cfg, max_replications) exceeds SIM_STATIC_WORKSPACE_BYTES. The handle is used and destroyed
 * like any other (sim_run, sim_stats, the read-outs, sim_destroy). Every handle made by this call on one GPU shares
 * that GPU's array, which keeps whatever the last one left: the call rewrites the tables and the first sim_run
 * clears the state, so handles used one after the other are independent, but two that are alive on one GPU at the
 * same time overwrite each other, and calls on them that overlap race. */
#define SIM_STATIC_WORKSPACE_BYTES (32u << 20)
int sim_create_static(const sim_config *cfg, int max_replications, sim_t **out);

/* Advances `replications` replications by `steps` steps, asynchronously on `hip_stream`
 * (a hipStream_t, NULL = default stream). Repeating the same (replications, seed) resumes; another
 * pair restarts from the empty system. Results depend only on (config, replications, seed, total
 * steps), not on how the steps were split over calls. Total steps must stay below 2^29. */
int sim_run(sim_t *h, int64_t steps, int replications, uint64_t seed, void *hip_stream);

/* Replaces the gate's targets x*_i (prefill occupancy per server) and q*_p,i (prefill backlog per server)
 * between two sim_run calls; the run goes on from its current state. This is the hook of the paper's online
 * adaptive algorithm (trace-driven online policy evaluation: the controller re-estimates the class arrival
 * rates from a rolling window, Eq. main-online-arrival-estimate, re-solves the fluid LP at every replanning
 * epoch, and the gate then ranks by the deviation from the current targets). Only the targets move: the
 * mixed/solo split M is moved by sim_set_split. x_star, qp_star: host arrays of K doubles. SIM_EINVAL: a negative or non-finite target.
 * The new values are copied to the device asynchronously on `hip_stream`, ordered after earlier runs. */
int sim_set_targets(sim_t *h, const double *x_star, const double *qp_star, void *hip_stream);

/* Moves the mixed/solo split between two sim_run calls: servers 0..M-1 are the mixed group from the next step
 * on (the online adaptive algorithm's M*(t_k) = ceil(n * sum_i x*_i(t_k)), Eq. main-online-mixed-target).
 * Existing service is not pre-empted: a prefill in service on a server that turns solo runs to its end (that
 * server admits no further prefill), decodes on a server that turns mixed stay (it takes new ones only while
 * it holds fewer than B-1); the new split governs later admissions and placements. SIM_EINVAL: M outside
 * [0, N], or the on-chip state of the enlarged mixed group no longer fits a compute unit's LDS. The new value
 * is copied to the device asynchronously on `hip_stream`, ordered after earlier runs. */
int sim_set_split(sim_t *h, int M, void *hip_stream);

/* Sums the tallies over replications on the device, copies them out and derives the fp64 figures.
 * Synchronises the stream. Returns SIM_EOVERFLOW (with `out` filled) if any ring overflowed. */
int sim_stats(sim_t *h, sim_stats_t *out, void *hip_stream);

/* Per-replication read-outs for parity checks; each synchronises the stream.
 * sim_tallies: out[K][SIM_NTALLY] then [SIM_NGLOBAL]. sim_hist: which = 0 TTFT, 1 E2E, 2 TBT,
 * out[K][SIM_NBIN]. sim_digest: 64-bit order-independent digest of the integer state. */
int sim_snapshot(sim_t *h, int replication, sim_state_t *out, void *hip_stream);
int sim_tallies(sim_t *h, int replication, uint64_t *out, void *hip_stream);
int sim_hist(sim_t *h, int replication, int which, uint64_t *out, void *hip_stream);
int sim_digest(sim_t *h, int replication, uint64_t *out, void *hip_stream);

/* Step-kernel launches and their accumulated device time (HIP events on the run's stream) since
 * the handle was created or this was last called with reset != 0. Synchronises the stream. */
int sim_kernel_time(sim_t *h, int64_t *launches, double *milliseconds, int reset, void *hip_stream);
/* Launch shape of the step kernel for this handle: threads per workgroup (one workgroup per replication) and
 * dynamic LDS bytes per workgroup; what occupancy follows from. Host only; either pointer may be NULL. */
int sim_launch_shape(sim_t *h, int *threads, size_t *lds_bytes);
/* The launch shape the library gives `replications` replications of `cfg` (what sim_create(cfg, replications, ...)
 * fixes for the handle): threads per workgroup, LDS bytes per workgroup, and the waves per SIMD the chosen form of
 * the kernel is compiled for (4: 128 registers a lane; 2: up to 256, for workgroups of up to 512 threads when all of
 * them find a place at once at that density). A replication is one workgroup that runs for the whole launch, so the
 * shape is the largest workgroup that keeps the rounds of workgroups lowest on the current device (256 compute units
 * are assumed when there is none). Host only; any out pointer may be NULL. SIM_EINVAL as for sim_create. */
int sim_launch_plan(const sim_config *cfg, int replications, int *threads, size_t *lds_bytes, int *waves_per_simd);

int sim_destroy(sim_t *h);
const char *sim_strerror(int err);

/* Host-only helpers (no device needed): the quantile table of a length law (65536 entries),
 * one Philox4x32-10 block, the sampler thresholds a config would use
 * (arr_thr[rows][3] for rows 0..rows-1, cls_thr[SIM_MAXK]). */
int sim_length_table(int law, double p0, double p1, uint16_t *out);
/* the patience table (65536 entries, in steps) of a class with patience rate theta > 0 at step length dt */
int sim_patience_table(double theta, double dt, uint16_t *out);
int sim_philox(uint64_t seed, uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t *out4);
int sim_thresholds(const sim_config *cfg, int64_t rows, uint32_t *arr_thr, uint32_t *cls_thr);
/* On-chip memory (LDS bytes of one compute unit) the step kernel needs for `cfg`, and the limit it must stay
 * within. The clocks, iteration counters and decode counts of all N servers of a replication stay on chip for
 * a whole launch (about 11.4 bytes per server, 2 more per mixed-group server, 6 KB more with abandonment, on top
 * of about 28 KB): sim_workspace_bytes and sim_create return SIM_EINVAL for a configuration above the limit, and
 * sim_set_split for a split that would exceed it. The figure is for the largest workgroup the library would launch
 * the configuration with (the one it takes for few replications; see sim_launch_plan for a given count). Host only;
 * reads K, N, M, B, C, c0, c_pre, c_dec, route_mode and the classes' theta. `out_limit` may be NULL. */
int sim_onchip_bytes(const sim_config *cfg, size_t *out_bytes, size_t *out_limit);
/* sizeof of the four ABI structs, in the order class, config, stats, state (for binding checks). */
int sim_abi_sizes(size_t *out4);

#ifdef __cplusplus
}
#endif
#endif
