/*
 * gnr_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * Plain, slow, single-threaded CPU oracle of the time-stepped Monte-Carlo
 * simulation of the multiclass many-server LLM-inference queueing network
 * (paper Sec. 2.3, "The Stochastic Model") under the occupancy-based
 * gate-and-route policy (paper Sec. 4, "Static Planning" / "Dynamic Control").
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 * It shares no code with the HIP library: its own Philox, its own table
 * builders, its own state layout (arrays of structs, growable FIFOs).
 *
 * What is a definition and what is a reading of the paper:
 *  - one iteration = every decode in the frozen batch emits one token and the
 *    prefill, if present, advances one chunk of at most C tokens (Sec. 2.2);
 *  - at most one prefill per server, B-1 decodes on a mixed-group server, B on a
 *    solo-group server (Sec. 2.3 capacity constraints, Sec. 4 static planning);
 *  - gate: admit the head-of-line job of the waiting class with the smallest
 *    occupancy deviation (X_i - n x_i*)/x_i*, ties by largest queue deviation
 *    (Sec. 4, prefill gate);
 *  - router: solo group first, then mixed group, else the decode buffer, FCFS
 *    (Sec. 4, decode routing);
 *  - revenue recognition events (Sec. 2.3, bundled and separate charging);
 *  - abandonment (Sec. 2.3): a job waiting in a prefill queue or in the decode
 *    buffer leaves when its exponential patience, rate theta of its class, ends;
 *  - balance equations and capacity constraints (Sec. 2.3) are checked by
 *    oracle_check(), recomputing every aggregate from the per-server state.
 *  Readings (time stepping, tie orders, samplers) are listed where they occur.
 *
 * Pins (tests/ -m "not gpu"): Philox against an independent implementation,
 * sampler tables against closed-form pmfs, a hand-traced worked example,
 * flow-balance / capacity / token-conservation invariants, Little's law as an
 * exact integer identity, the exact stationary law of the discrete M/Geo/c
 * chain and its Erlang-C limit, convergence of revenue to the fluid-LP optimum,
 * the gate and router rules replayed step by step from an independent statement;
 * abandonment: the patience table against the geometric law, queues that nobody
 * leaves by service rebuilt job by job from the patience blocks, the exact
 * stationary law of the discrete chain with abandonment (Erlang-A).
 *
 * Build: gcc -O2 -ffp-contract=off -fPIC -shared gnr_oracle.c -o libgnr_oracle.so -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define MAXK 8
#define MAXB 128
#define NBIN 720
#define T_IDLE INT64_MAX

enum { LAW_GEOMETRIC = 0, LAW_LOGNORMAL = 1, LAW_CONST = 2, LAW_TABLE = 3 };
enum { GATE_OCCUPANCY = 0, GATE_PRIORITY = 1, GATE_FCFS = 2 };
enum { ROUTE_SOLO_FIRST = 0, ROUTE_RANDOM_SPLIT = 1, ROUTE_IMMEDIATE = 2, ROUTE_WEIGHTED_SPLIT = 3 };

/* per-class tally indices */
enum {
  T_A = 0, T_DROP_P, T_U_P, T_S_P, T_U_DM, T_U_DS, T_S_DM, T_S_DS, T_M_SM, T_M_MS,
  T_DROP_D, T_TOKP_PRE, T_TOKP_DEC, T_TOKD_DEC, T_TOK_EMIT, T_TOK_PREF,
  T_SUM_QP, T_SUM_QD, T_SUM_X, T_SUM_YM, T_SUM_YS, T_WAIT_STEPS,
  T_TTFT_SUM, T_E2E_SUM, T_TBT_SUM, T_AB_P, T_AB_D, NTALLY
};
/* per-replication global tally indices */
enum { G_ITERS_MIX = 0, G_ITERS_SOLO, G_BUSY_MIX, G_BUSY_SOLO, G_STEPS, G_OVERFLOW, NGLOBAL };

typedef struct {
  double lambda;              /* arrivals per server per unit time (Sec. 2.3 primitives) */
  int in_law, out_law;
  double in_p0, in_p1, out_p0, out_p1;
  const uint16_t *in_table, *out_table;
  double price_in, price_out; /* c_p, c_d per token (Sec. 2.3 revenue models) */
  int bundled;                /* which recognition rule the "mixed" revenue uses */
  double priority;            /* static index of the Prioritize-and-Route gate (Sec. 5.1) */
  double theta;               /* patience rate of a waiting job (Sec. 2.3); 0 = never abandons */
} oracle_class;

typedef struct {
  int K, N, B, C;
  double c0, c_pre, c_dec, dt;
  const oracle_class *cls;
  int M;
  const double *x_star, *qp_star;
  int gate_mode, route_mode;
  double mod_amp;
  int64_t mod_period;
  int64_t queue_cap, dbuf_cap;
  const double *p_solo;       /* ROUTE_RANDOM_SPLIT, ROUTE_WEIGHTED_SPLIT: probability p_s,i that a class-i decode is
                                 sent to the solo group */
  const double *w_solo, *w_mixed; /* ROUTE_WEIGHTED_SPLIT: class selection weights of the two pools (the paper's
                                     varpi_s,i and varpi_m,i, EC "General SLI-aware Extension") */
} oracle_config;

typedef struct { int used; uint32_t fin; int cls, P, D; uint32_t stamp; } slot_t;

typedef struct {
  int64_t t_next;            /* end of the running iteration, T_IDLE when not busy */
  uint32_t iter;             /* completed iterations */
  int64_t d_frozen;          /* duration of the running iteration */
  int ptok_frozen;           /* prefill tokens in the running iteration */
  int pf_rem, pf_cls, pf_P, pf_D; /* prefill in service; pf_rem == 0 <=> slot idle */
  uint32_t pf_stamp;
  int n_dec, n_cls[MAXK], n_join[MAXK];
  int at_boundary;
  slot_t slot[MAXB];
} server_t;

#define DL_NEVER 0xFFFFFFFFu
/* dl: the step at whose start a job that is still waiting abandons (DL_NEVER: it never does) */
typedef struct { int cls, P, D; uint32_t stamp, dl; } job_t;
typedef struct { uint32_t stamp, dl; } qent_t;

typedef struct { qent_t *v; int64_t head, len, alloc; } fifoq;
typedef struct { job_t *v; int64_t head, len, alloc; } fifojob;

typedef struct {
  int inited;
  int64_t Qp[MAXK], X[MAXK], Qd[MAXK], Ym[MAXK], Ys[MAXK];
  fifoq q[MAXK];
  fifojob dbuf;              /* decode buffer; under ROUTE_RANDOM_SPLIT the solo component */
  fifojob dbuf_m;            /* ROUTE_RANDOM_SPLIT: the mixed component */
  server_t *sv;
  uint64_t tally[MAXK][NTALLY];
  uint64_t glob[NGLOBAL];
  uint64_t *hist; /* [3][MAXK][NBIN]: ttft, e2e, tbt */
} rep_t;

typedef struct oracle_t {
  oracle_config cfg;
  oracle_class cls[MAXK];
  double x_star[MAXK], qp_star[MAXK], p_solo[MAXK];
  uint32_t solo_thr[MAXK];   /* a decode goes to the solo group when its random word is below this */
  double w_pool[2][MAXK];    /* ROUTE_WEIGHTED_SPLIT: selection weights as given, [0] solo pool, [1] mixed pool */
  uint32_t wsel[2][MAXK];    /* ... and as integers in units of 2^-20, at least 1 */
  int64_t c0_ns, cpre_ns, cdec_ns, dt_ns;
  double nx[MAXK], invx[MAXK], nq[MAXK];
  uint32_t *arr_thr;      /* [rows][3] */
  int64_t rows;
  uint32_t cls_thr[MAXK];
  uint16_t *tab_in[MAXK], *tab_out[MAXK];
  uint16_t *tab_pat[MAXK]; /* patience in steps, NULL for a class that never abandons */
  int any_theta;
  int split_moved;        /* oracle_set_split changed M during the run: servers may hold work their new group would not take */
  int max_reps, reps;
  uint64_t seed;
  int64_t steps_done;
  rep_t *rep;
  int *sel; int nsel;
  int check_every;
  int64_t violations;
  int first_violation;
  int codes[64], ncodes;  /* the distinct violation codes seen so far */
} oracle_t;

/* ---------------------------------------------------------------- Philox ---- */
/* Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, SC'11): two 32x32->64
 * multiplies per round, Weyl key schedule. */
static void philox4x32_10(uint32_t k0, uint32_t k1, uint32_t c0, uint32_t c1,
                          uint32_t c2, uint32_t c3, uint32_t out[4])
{
  for (int r = 0; r < 10; r++) {
    uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    uint32_t n1 = (uint32_t)p1;
    uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

void oracle_philox(uint64_t seed, uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t *out)
{
  philox4x32_10((uint32_t)seed, (uint32_t)(seed >> 32), c0, c1, c2, c3, out);
}

/* block used by the simulation: counter = (step, stream, server, replication) */
static void draw(const oracle_t *o, int r, int g, uint32_t s, uint32_t stream, uint32_t w[4])
{
  philox4x32_10((uint32_t)o->seed, (uint32_t)(o->seed >> 32), s, stream, (uint32_t)g, (uint32_t)r, w);
}

/* ---------------------------------------------------------------- tables ---- */
static uint32_t thr32(double p)
{
  double v = floor(p * 4294967296.0);
  if (v < 0.0) v = 0.0;
  if (v > 4294967295.0) v = 4294967295.0;
  return (uint32_t)v;
}

/* A class selection weight in units of 2^-20, never below one unit: a class with weight zero is still served
 * when it is the only one waiting, so each pool stays work-conserving. */
static uint32_t weight_units(double w)
{
  double v = floor(w * 1048576.0 + 0.5);
  if (v < 1.0) v = 1.0;
  if (v > 1048576.0) v = 1048576.0;
  return (uint32_t)v;
}

/* cdf of the integer-valued length at k (k >= 1) */
static double len_cdf(int law, double p0, double p1, int k)
{
  if (law == LAW_GEOMETRIC) {            /* Pr(X >= k) = (1-p)^(k-1), p = 1/mean (EC, geometric check) */
    double p = 1.0 / p0;
    if (p >= 1.0) return 1.0;
    return -expm1((double)k * log1p(-p));
  } else {                               /* lognormal rounded to the nearest integer */
    double mu = log(p0);
    double z = (log((double)k + 0.5) - mu) / p1;
    return 0.5 * erfc(-z * M_SQRT1_2);
  }
}

/* quantile table: entry j is the smallest k in [1,32768] whose cdf reaches (j+0.5)/65536 */
int oracle_length_table(int law, double p0, double p1, uint16_t *out)
{
  if (law == LAW_CONST) {
    long long v = llround(p0);
    if (v < 1) v = 1;
    if (v > 32768) v = 32768;
    for (int j = 0; j < 65536; j++) out[j] = (uint16_t)v;
    return 0;
  }
  if (law != LAW_GEOMETRIC && law != LAW_LOGNORMAL) return -1;
  if (!(p0 > 0.0)) return -1;
  if (law == LAW_LOGNORMAL && !(p1 > 0.0)) return -1;
  int k = 1;
  for (int j = 0; j < 65536; j++) {
    double u = ((double)j + 0.5) / 65536.0;
    while (k < 32768 && len_cdf(law, p0, p1, k) < u) k++;
    out[j] = (uint16_t)k;
  }
  return 0;
}

/* Patience of a waiting job, in steps (Sec. 2.3: exponential patience with rate theta). A job is asked at the
 * start of every step after the one it joined the queue in; an exponential patience seen at those instants is
 * geometric on {1,2,...}: Pr(patience >= m) = exp(-theta*dt*(m-1)). Same quantile-table form as the lengths
 * (so clamped at 32768 steps). */
int oracle_patience_table(double theta, double dt, uint16_t *out)
{
  if (!(theta > 0.0) || !(dt > 0.0)) return -1;
  double p = -expm1(-theta * dt);
  return oracle_length_table(LAW_GEOMETRIC, 1.0 / p, 0.0, out);
}

static double total_rate(const oracle_t *o)
{
  double lam = 0.0;
  for (int k = 0; k < o->cfg.K; k++) lam += o->cls[k].lambda;
  return lam;
}

/* thresholds on the first random word for the per-server arrival count in one step:
 * Poisson with mean Lambda(s)*dt, truncated at 3 (Sec. 2.3: Poisson arrivals) */
static void arrival_row(const oracle_t *o, int64_t row, uint32_t thr[3])
{
  double lam = total_rate(o);
  double dts = (double)o->dt_ns * 1e-9;
  double mod = 1.0;
  if (o->cfg.mod_period > 0) {
    double ph = 2.0 * M_PI * (double)row / (double)o->cfg.mod_period;
    mod = 1.0 + o->cfg.mod_amp * sin(ph);
  }
  double m = lam * dts * mod;
  if (m < 0.0) m = 0.0;
  double p0 = exp(-m);
  double p1 = p0 * m;
  double p2 = p1 * m * 0.5;
  thr[0] = thr32(p0);
  thr[1] = thr32(p0 + p1);
  thr[2] = thr32((p0 + p1) + p2);
}

/* ---------------------------------------------------------------- fifos ---- */
static void fq_push(fifoq *f, qent_t v)
{
  if (f->head + f->len == f->alloc) {
    if (f->head > 0) { memmove(f->v, f->v + f->head, (size_t)f->len * sizeof *f->v); f->head = 0; }
    if (f->len == f->alloc) {
      f->alloc = f->alloc ? 2 * f->alloc : 64;
      f->v = realloc(f->v, (size_t)f->alloc * sizeof *f->v);
    }
  }
  f->v[f->head + f->len++] = v;
}
static qent_t fq_pop(fifoq *f) { qent_t v = f->v[f->head++]; f->len--; if (!f->len) f->head = 0; return v; }

static void fj_push(fifojob *f, job_t v)
{
  if (f->head + f->len == f->alloc) {
    if (f->head > 0) { memmove(f->v, f->v + f->head, (size_t)f->len * sizeof *f->v); f->head = 0; }
    if (f->len == f->alloc) {
      f->alloc = f->alloc ? 2 * f->alloc : 64;
      f->v = realloc(f->v, (size_t)f->alloc * sizeof *f->v);
    }
  }
  f->v[f->head + f->len++] = v;
}
static job_t fj_pop(fifojob *f) { job_t v = f->v[f->head++]; f->len--; if (!f->len) f->head = 0; return v; }

/* ------------------------------------------------------------- histogram ---- */
/* bin of a non-negative duration in ns: exact below 16, then 16 bins per octave */
static int hbin(int64_t v)
{
  if (v < 0) v = 0;
  if (v < 16) return (int)v;
  int e = 63 - __builtin_clzll((unsigned long long)v);
  int b = 16 * (e - 3) + (int)((v >> (e - 4)) & 15);
  return b < NBIN ? b : NBIN - 1;
}
int oracle_hbin(int64_t v) { return hbin(v); }

#define HIST(R, which, k) ((R)->hist + ((size_t)(which) * MAXK + (size_t)(k)) * NBIN)

/* ---------------------------------------------------------------- create ---- */
int oracle_destroy(oracle_t *o);

int oracle_create(const oracle_config *cfg, int max_reps, oracle_t **out)
{
  if (!cfg || !out || max_reps < 1) return -1;
  if (cfg->K < 1 || cfg->K > MAXK || cfg->N < 1 || cfg->B < 1 || cfg->B > MAXB) return -1;
  if (cfg->C < 1 || cfg->C > 32768 || cfg->M < 0 || cfg->M > cfg->N) return -1;
  if (cfg->queue_cap < 1 || cfg->dbuf_cap < 1) return -1;
  oracle_t *o = calloc(1, sizeof *o);
  o->cfg = *cfg;
  for (int k = 0; k < cfg->K; k++) {
    o->cls[k] = cfg->cls[k];
    o->x_star[k] = cfg->x_star[k];
    o->qp_star[k] = cfg->qp_star[k];
    if (!(cfg->cls[k].theta >= 0.0) || !isfinite(cfg->cls[k].theta) || !(cfg->cls[k].lambda >= 0.0) ||
        cfg->x_star[k] < 0.0) { free(o); return -1; }
  }
  if (cfg->route_mode < ROUTE_SOLO_FIRST || cfg->route_mode > ROUTE_WEIGHTED_SPLIT) { free(o); return -1; }
  if (cfg->route_mode == ROUTE_WEIGHTED_SPLIT) {
    if (!cfg->w_solo || !cfg->w_mixed) { free(o); return -1; }
    for (int k = 0; k < cfg->K; k++) {
      if (!(cfg->w_solo[k] >= 0.0) || !(cfg->w_solo[k] <= 1.0) || !(cfg->w_mixed[k] >= 0.0) || !(cfg->w_mixed[k] <= 1.0)) {
        free(o); return -1;
      }
      o->w_pool[0][k] = cfg->w_solo[k]; o->w_pool[1][k] = cfg->w_mixed[k];
      o->wsel[0][k] = weight_units(cfg->w_solo[k]); o->wsel[1][k] = weight_units(cfg->w_mixed[k]);
    }
  }
  if (cfg->route_mode == ROUTE_RANDOM_SPLIT || cfg->route_mode == ROUTE_WEIGHTED_SPLIT) {
    if (!cfg->p_solo) { free(o); return -1; }
    for (int k = 0; k < cfg->K; k++) {
      if (!(cfg->p_solo[k] >= 0.0) || !(cfg->p_solo[k] <= 1.0)) { free(o); return -1; }
      o->p_solo[k] = cfg->p_solo[k];
    }
  }
  o->cfg.cls = o->cls; o->cfg.x_star = o->x_star; o->cfg.qp_star = o->qp_star; o->cfg.p_solo = o->p_solo;
  o->cfg.w_solo = o->w_pool[0]; o->cfg.w_mixed = o->w_pool[1];
  o->c0_ns = llround(cfg->c0 * 1e9);
  o->cpre_ns = llround(cfg->c_pre * 1e9);
  o->cdec_ns = llround(cfg->c_dec * 1e9);
  o->dt_ns = cfg->dt > 0.0 ? llround(cfg->dt * 1e9) : o->c0_ns;
  if (o->c0_ns < 1 || o->cpre_ns < 0 || o->cdec_ns < 0 || o->dt_ns < 1 || o->dt_ns > o->c0_ns) { free(o); return -1; }
  double lam = total_rate(o);
  if (lam * ((double)o->dt_ns * 1e-9) * (1.0 + fabs(cfg->mod_amp)) > 0.05) { free(o); return -1; }
  for (int k = 0; k < cfg->K; k++) {
    o->nx[k] = (double)cfg->N * o->x_star[k];
    o->invx[k] = o->x_star[k] > 0.0 ? 1.0 / o->x_star[k] : 0.0;
    o->nq[k] = (double)cfg->N * o->qp_star[k];
  }
  for (int k = 0; k < cfg->K; k++) o->solo_thr[k] = thr32(o->p_solo[k]);
  o->rows = cfg->mod_period > 0 ? cfg->mod_period : 1;
  o->arr_thr = malloc((size_t)o->rows * 3 * sizeof(uint32_t));
  for (int64_t j = 0; j < o->rows; j++) arrival_row(o, j, o->arr_thr + 3 * j);
  double acc = 0.0;
  for (int k = 0; k + 1 < cfg->K; k++) {
    acc += o->cls[k].lambda;
    o->cls_thr[k] = lam > 0.0 ? thr32(acc / lam) : 0xFFFFFFFFu;
  }
  for (int k = 0; k < cfg->K; k++) {
    o->tab_in[k] = malloc(65536 * sizeof(uint16_t));
    o->tab_out[k] = malloc(65536 * sizeof(uint16_t));
    int e1, e2;
    if (o->cls[k].in_law == LAW_TABLE) { memcpy(o->tab_in[k], o->cls[k].in_table, 65536 * 2); e1 = 0; }
    else e1 = oracle_length_table(o->cls[k].in_law, o->cls[k].in_p0, o->cls[k].in_p1, o->tab_in[k]);
    if (o->cls[k].out_law == LAW_TABLE) { memcpy(o->tab_out[k], o->cls[k].out_table, 65536 * 2); e2 = 0; }
    else e2 = oracle_length_table(o->cls[k].out_law, o->cls[k].out_p0, o->cls[k].out_p1, o->tab_out[k]);
    o->cls[k].in_table = o->cls[k].out_table = NULL;
    if (o->cls[k].theta > 0.0) {
      o->tab_pat[k] = malloc(65536 * sizeof(uint16_t));
      if (oracle_patience_table(o->cls[k].theta, (double)o->dt_ns * 1e-9, o->tab_pat[k])) e1 = 1;
      o->any_theta = 1;
    }
    if (e1 || e2) { o->max_reps = 0; oracle_destroy(o); return -1; }
    for (int j = 0; j < 65536; j++)
      if (o->tab_in[k][j] < 1 || o->tab_in[k][j] > 32768 || o->tab_out[k][j] < 1 || o->tab_out[k][j] > 32768) {
        o->max_reps = 0; oracle_destroy(o); return -1;
      }
  }
  o->max_reps = max_reps;
  o->rep = calloc((size_t)max_reps, sizeof(rep_t));
  o->reps = 0;
  o->first_violation = 0;
  *out = o;
  return 0;
}

static void rep_free(rep_t *R)
{
  for (int k = 0; k < MAXK; k++) free(R->q[k].v);
  free(R->dbuf.v); free(R->dbuf_m.v); free(R->sv); free(R->hist);
  memset(R, 0, sizeof *R);
}

int oracle_destroy(oracle_t *o)
{
  if (!o) return -1;
  for (int r = 0; r < o->max_reps; r++) rep_free(&o->rep[r]);
  for (int k = 0; k < MAXK; k++) { free(o->tab_in[k]); free(o->tab_out[k]); free(o->tab_pat[k]); }
  free(o->arr_thr); free(o->rep); free(o->sel); free(o);
  return 0;
}

static void rep_init(const oracle_t *o, rep_t *R)
{
  rep_free(R);
  R->sv = calloc((size_t)o->cfg.N, sizeof(server_t));
  for (int g = 0; g < o->cfg.N; g++) R->sv[g].t_next = T_IDLE;
  R->hist = calloc((size_t)3 * MAXK * NBIN, sizeof(uint64_t));
  R->inited = 1;
}

/* restrict subsequent runs to a subset of replication indices (NULL/0: all) */
int oracle_select(oracle_t *o, const int *ids, int n)
{
  free(o->sel); o->sel = NULL; o->nsel = 0;
  if (ids && n > 0) {
    o->sel = malloc((size_t)n * sizeof(int));
    memcpy(o->sel, ids, (size_t)n * sizeof(int));
    o->nsel = n;
  }
  return 0;
}

int oracle_set_check(oracle_t *o, int every) { o->check_every = every; return 0; }
int64_t oracle_violations(const oracle_t *o) { return o->violations; }
int oracle_first_violation(const oracle_t *o) { return o->first_violation; }

/* ------------------------------------------------------------ invariants ---- */
static void viol(oracle_t *o, int code)
{
  if (!o->violations) o->first_violation = code;
  o->violations++;
  for (int i = 0; i < o->ncodes; i++) if (o->codes[i] == code) return;
  if (o->ncodes < 64) o->codes[o->ncodes++] = code;
}
/* The distinct codes seen so far (at most cap of them are written); returns how many there are. */
int oracle_violation_codes(const oracle_t *o, int *out, int cap)
{
  for (int i = 0; i < o->ncodes && i < cap; i++) out[i] = o->codes[i];
  return o->ncodes;
}

/* Recompute every aggregate from per-server state and compare with the running
 * counters: capacity constraints and balance equations of Sec. 2.3, token
 * conservation, FIFO lengths. Returns the number of violations found. */
static int64_t check_rep(oracle_t *o, int r)
{
  rep_t *R = &o->rep[r];
  const int K = o->cfg.K, N = o->cfg.N, B = o->cfg.B, M = o->cfg.M;
  int64_t before = o->violations;
  int64_t X[MAXK] = {0}, Ym[MAXK] = {0}, Ys[MAXK] = {0}, Qd[MAXK] = {0};
  int64_t prog_dec[MAXK] = {0}, prog_pre[MAXK] = {0};
  int64_t Xtot = 0, Ymtot = 0, Ystot = 0;
  for (int g = 0; g < N; g++) {
    server_t *s = &R->sv[g];
    int cnt[MAXK] = {0}, used = 0, joiners[MAXK] = {0};
    int busy = s->t_next != T_IDLE;
    for (int j = 0; j < B; j++) if (s->slot[j].used) {
      slot_t *e = &s->slot[j];
      used++; cnt[e->cls]++;
      int64_t left = (int64_t)e->fin - (int64_t)s->iter;
      if (left < 1 || left > (int64_t)e->D + 1) viol(o, 101);
      if (left == (int64_t)e->D + 1) joiners[e->cls]++;
      int64_t rem = left < e->D ? left : e->D;
      prog_dec[e->cls] += e->D - rem;
    }
    for (int j = B; j < MAXB; j++) if (s->slot[j].used) viol(o, 102);
    if (used != s->n_dec) viol(o, 103);
    for (int k = 0; k < MAXK; k++) {
      if (cnt[k] != s->n_cls[k]) viol(o, 104);
      if (joiners[k] != s->n_join[k]) viol(o, 105);
    }
    /* per-server capacity (Sec. 2.3). After the split has moved, work that was there before stays (no
     * pre-emption): a server that turned mixed may still hold B decodes, one that turned solo its prefill. */
    if (used > B) viol(o, 107);
    if (o->cfg.route_mode == ROUTE_IMMEDIATE) {
      if (used + (s->pf_rem ? 1 : 0) > B) viol(o, 106);   /* a request keeps its slot from prefill to its last token */
      if (g >= M && !o->split_moved && (used || s->pf_rem)) viol(o, 108);
    } else if (!o->split_moved) {
      if (g < M) { if (used > B - 1) viol(o, 106); } else { if (s->pf_rem) viol(o, 108); }
    }
    if (s->pf_rem) {
      if (s->pf_rem > s->pf_P || s->pf_rem < 0) viol(o, 109);
      X[s->pf_cls]++; Xtot++;
      prog_pre[s->pf_cls] += s->pf_P - s->pf_rem;
      for (int k = 0; k < K; k++) { Ym[k] += cnt[k]; Ymtot += cnt[k]; }
    } else {
      for (int k = 0; k < K; k++) { Ys[k] += cnt[k]; Ystot += cnt[k]; }
    }
    if (!busy && (used || s->pf_rem)) viol(o, 110);          /* work-conserving per server */
    if (busy && !used && !s->pf_rem) viol(o, 111);
    if (busy && s->t_next <= (int64_t)o->steps_done * o->dt_ns) viol(o, 112);
  }
  for (int64_t i = 0; i < R->dbuf.len; i++) Qd[R->dbuf.v[R->dbuf.head + i].cls]++;
  for (int64_t i = 0; i < R->dbuf_m.len; i++) Qd[R->dbuf_m.v[R->dbuf_m.head + i].cls]++;
  if (o->cfg.route_mode == ROUTE_SOLO_FIRST && R->dbuf_m.len) viol(o, 124);
  /* capacity constraints */
  if (Xtot > N) viol(o, 120);
  if (o->cfg.route_mode == ROUTE_IMMEDIATE) {
    if (Ymtot > (int64_t)(B - 1) * Xtot) viol(o, 121);
    if (R->dbuf.len || R->dbuf_m.len) viol(o, 125);      /* nobody ever waits for a decode slot */
  } else if (!o->split_moved) {
    if (Ymtot > (int64_t)(B - 1) * Xtot) viol(o, 121);
    if (Ystot > (int64_t)B * (N - Xtot)) viol(o, 122);
  } else {
    if (Ymtot > (int64_t)B * Xtot) viol(o, 121);
    if (Ystot > (int64_t)B * (N - Xtot)) viol(o, 122);
  }
  if (R->dbuf.len > o->cfg.dbuf_cap || R->dbuf_m.len > o->cfg.dbuf_cap) viol(o, 123);
  for (int k = 0; k < K; k++) {
    uint64_t *t = R->tally[k];
    if (X[k] != R->X[k]) viol(o, 130);
    if (Ym[k] != R->Ym[k]) viol(o, 131);
    if (Ys[k] != R->Ys[k]) viol(o, 132);
    if (Qd[k] != R->Qd[k]) viol(o, 133);
    if (R->q[k].len != R->Qp[k]) viol(o, 134);
    if (R->Qp[k] > o->cfg.queue_cap) viol(o, 135);
    /* balance equations of Sec. 2.3 from the empty initial state (B_p, B_d: abandonments) */
    if (R->Qp[k] != (int64_t)(t[T_A] - t[T_U_P] - t[T_AB_P])) viol(o, 140);
    if (R->X[k] != (int64_t)(t[T_U_P] - t[T_S_P])) viol(o, 141);
    if (R->Qd[k] != (int64_t)(t[T_S_P] - t[T_DROP_D] - t[T_U_DM] - t[T_U_DS] - t[T_AB_D])) viol(o, 142);
    if (R->Ym[k] != (int64_t)(t[T_U_DM] - t[T_S_DM] + t[T_M_SM] - t[T_M_MS])) viol(o, 143);
    if (R->Ys[k] != (int64_t)(t[T_U_DS] - t[T_S_DS] + t[T_M_MS] - t[T_M_SM])) viol(o, 144);
    /* token conservation */
    if ((int64_t)t[T_TOK_EMIT] != (int64_t)t[T_TOKD_DEC] + prog_dec[k]) viol(o, 150);
    if ((int64_t)t[T_TOK_PREF] != (int64_t)t[T_TOKP_PRE] + prog_pre[k]) viol(o, 151);
    /* FIFO stamps are non-decreasing and not in the future; nobody waits past the end of their patience */
    for (int64_t i = 0; i < R->q[k].len; i++) {
      uint32_t st = R->q[k].v[R->q[k].head + i].stamp;
      if (st >= (uint64_t)o->steps_done) viol(o, 152);
      if (i && st < R->q[k].v[R->q[k].head + i - 1].stamp) viol(o, 153);
      if ((uint64_t)R->q[k].v[R->q[k].head + i].dl < (uint64_t)o->steps_done) viol(o, 154);
      if ((R->q[k].v[R->q[k].head + i].dl != DL_NEVER) != (o->tab_pat[k] != NULL)) viol(o, 155);
    }
  }
  for (int64_t i = 0; i < R->dbuf.len; i++)
    if ((uint64_t)R->dbuf.v[R->dbuf.head + i].dl < (uint64_t)o->steps_done) viol(o, 156);
  for (int64_t i = 0; i < R->dbuf_m.len; i++)
    if ((uint64_t)R->dbuf_m.v[R->dbuf_m.head + i].dl < (uint64_t)o->steps_done) viol(o, 156);
  return o->violations - before;
}

int64_t oracle_check(oracle_t *o)
{
  int64_t n = 0;
  for (int r = 0; r < o->reps; r++) if (o->rep[r].inited) n += check_rep(o, r);
  return n;
}

/* TEST HOOKS (used by the tests of the checker itself, never by a simulation): oracle_poke adds `delta` to one
 * number of replication r's state so that a test can show which relation of check_rep() notices it.
 * what: 0 Q_p,i  1 X_i  2 Q_d,i  3 Y_m,i  4 Y_s,i (i = class); 5 tally word (i = class * NTALLY + word);
 * 6 decode count of server i; 7 prompt tokens left of server i's prefill; 8 end time of server i's iteration;
 * 9 finish index of server i's first occupied slot; 10 (delta ignored) server i's first free slot becomes a copy of
 * its first occupied one, counters untouched. oracle_clear_violations forgets what was found so far. */
int oracle_poke(oracle_t *o, int r, int what, int i, int64_t delta)
{
  if (!o || r < 0 || r >= o->reps || !o->rep[r].inited || i < 0) return -1;
  rep_t *R = &o->rep[r];
  const int K = o->cfg.K, N = o->cfg.N;
  if (what >= 0 && what <= 4 && i >= K) return -1;
  if (what == 5 && i >= K * NTALLY) return -1;
  if (what >= 6 && i >= N) return -1;
  switch (what) {
    case 0: R->Qp[i] += delta; break;
    case 1: R->X[i] += delta; break;
    case 2: R->Qd[i] += delta; break;
    case 3: R->Ym[i] += delta; break;
    case 4: R->Ys[i] += delta; break;
    case 5: R->tally[i / NTALLY][i % NTALLY] += (uint64_t)delta; break;
    case 6: R->sv[i].n_dec += (int)delta; break;
    case 7: R->sv[i].pf_rem += (int)delta; break;
    case 8: R->sv[i].t_next += delta; break;
    case 9:
      for (int j = 0; j < o->cfg.B; j++)
        if (R->sv[i].slot[j].used) { R->sv[i].slot[j].fin += (uint32_t)delta; return 0; }
      return -1;
    case 10: {
      slot_t *src = NULL, *dst = NULL;
      for (int j = 0; j < o->cfg.B; j++) {
        if (R->sv[i].slot[j].used && !src) src = &R->sv[i].slot[j];
        if (!R->sv[i].slot[j].used && !dst) dst = &R->sv[i].slot[j];
      }
      if (!src || !dst) return -1;
      *dst = *src;
      break;
    }
    default: return -1;
  }
  return 0;
}
int oracle_clear_violations(oracle_t *o) { o->violations = 0; o->first_violation = 0; o->ncodes = 0; return 0; }

/* ------------------------------------------------------------------ step ---- */
static int64_t iter_time(const oracle_t *o, int ptok, int n)
{
  /* t = c0 + c_pre * prefill_tokens + c_dec * n_decode, all in integer ns (Sec. 2.2) */
  return o->c0_ns + o->cpre_ns * (int64_t)ptok + o->cdec_ns * (int64_t)n;
}

static void step_rep(oracle_t *o, int r, uint32_t s)
{
  rep_t *R = &o->rep[r];
  const int K = o->cfg.K, N = o->cfg.N, B = o->cfg.B, M = o->cfg.M, C = o->cfg.C;
  const int64_t T = ((int64_t)s + 1) * o->dt_ns;       /* boundary time of this step */
  uint32_t w[4];

  /* 0. abandonment (Sec. 2.3): a job still waiting at the start of the step its patience ends in leaves,
   *    from the class prefill queues and from the decode buffer; the order of the others is kept */
  if (o->any_theta) {
    for (int k = 0; k < K; k++) {
      fifoq *f = &R->q[k];
      int64_t w = 0;
      for (int64_t i = 0; i < f->len; i++) {
        qent_t e = f->v[f->head + i];
        if (e.dl <= s) { R->Qp[k]--; R->tally[k][T_AB_P]++; }
        else f->v[f->head + w++] = e;
      }
      f->len = w;
    }
    for (int b = 0; b < 2; b++) {
      fifojob *d = b ? &R->dbuf_m : &R->dbuf;
      int64_t w = 0;
      for (int64_t i = 0; i < d->len; i++) {
        job_t e = d->v[d->head + i];
        if (e.dl <= s) { R->Qd[e.cls]--; R->tally[e.cls][T_AB_D]++; }
        else d->v[d->head + w++] = e;
      }
      d->len = w;
    }
  }

  /* 1. arrivals: one block per server, word 0 -> count, words 1.. -> classes */
  {
    const uint32_t *thr = o->arr_thr + 3 * (o->cfg.mod_period > 0 ? (int64_t)(s % (uint64_t)o->cfg.mod_period) : 0);
    int64_t acc[MAXK] = {0};
    for (int g = 0; g < N; g++) {
      draw(o, r, g, s, 0, w);
      int a = (w[0] >= thr[0]) + (w[0] >= thr[1]) + (w[0] >= thr[2]);
      for (int j = 0; j < a; j++) {
        int k = 0;
        for (int i = 0; i + 1 < K; i++) k += (w[1 + j] >= o->cls_thr[i]);
        acc[k]++;
      }
    }
    for (int k = 0; k < K; k++) {
      int64_t room = o->cfg.queue_cap - R->Qp[k];
      int64_t take = acc[k] < room ? acc[k] : room;
      /* the accepted arrivals of a class are exchangeable; the j-th of this step draws its patience from
       * block (step, stream 2+k, j, replication) */
      for (int64_t j = 0; j < take; j++) {
        qent_t e = { s, DL_NEVER };
        if (o->tab_pat[k]) { draw(o, r, (int)j, s, 2u + (uint32_t)k, w); e.dl = s + o->tab_pat[k][w[0] >> 16]; }
        fq_push(&R->q[k], e);
      }
      R->Qp[k] += take;
      R->tally[k][T_A] += (uint64_t)take;
      R->tally[k][T_DROP_P] += (uint64_t)(acc[k] - take);
      if (acc[k] > take) R->glob[G_OVERFLOW] = 1;
    }
  }

  /* 2. iteration completion on due servers, ascending server index */
  for (int g = 0; g < N; g++) {
    server_t *sv = &R->sv[g];
    sv->at_boundary = 0;
    if (sv->t_next == T_IDLE || sv->t_next > T) continue;
    const int64_t tc = sv->t_next;                     /* exact completion time */
    const int64_t d = sv->d_frozen;
    sv->iter++;
    if (sv->ptok_frozen > 0) { R->glob[G_ITERS_MIX]++; R->glob[G_BUSY_MIX] += (uint64_t)d; }
    else { R->glob[G_ITERS_SOLO]++; R->glob[G_BUSY_SOLO] += (uint64_t)d; }
    /* every decode of the frozen batch emits one token */
    for (int k = 0; k < K; k++) {
      int em = sv->n_cls[k] - sv->n_join[k];
      R->tally[k][T_TOK_EMIT] += (uint64_t)em;
      R->tally[k][T_TBT_SUM] += (uint64_t)em * (uint64_t)d;
      HIST(R, 2, k)[hbin(d)] += (uint64_t)em;
    }
    /* decodes that have emitted their last token leave */
    const int mixed_now = sv->pf_rem > 0;
    for (int j = 0; j < B; j++) {
      slot_t *e = &sv->slot[j];
      if (!e->used || e->fin != sv->iter) continue;
      const int k = e->cls;
      R->tally[k][mixed_now ? T_S_DM : T_S_DS]++;
      if (mixed_now) R->Ym[k]--; else R->Ys[k]--;
      R->tally[k][T_TOKP_DEC] += (uint64_t)e->P;
      R->tally[k][T_TOKD_DEC] += (uint64_t)e->D;
      int64_t e2e = tc - ((int64_t)e->stamp + 1) * o->dt_ns;
      R->tally[k][T_E2E_SUM] += (uint64_t)e2e;
      HIST(R, 1, k)[hbin(e2e)]++;
      e->used = 0; sv->n_cls[k]--; sv->n_dec--;
    }
    /* the prefill advances by the chunk frozen at the start of the iteration */
    if (sv->ptok_frozen > 0) {
      const int k = sv->pf_cls;
      R->tally[k][T_TOK_PREF] += (uint64_t)sv->ptok_frozen;
      sv->pf_rem -= sv->ptok_frozen;
      if (sv->pf_rem == 0) {
        R->tally[k][T_S_P]++; R->X[k]--;
        R->tally[k][T_TOKP_PRE] += (uint64_t)sv->pf_P;
        int64_t ttft = tc - ((int64_t)sv->pf_stamp + 1) * o->dt_ns;
        R->tally[k][T_TTFT_SUM] += (uint64_t)ttft;
        HIST(R, 0, k)[hbin(ttft)]++;
        for (int i = 0; i < K; i++) {                  /* co-resident decodes switch mixed -> solo */
          R->tally[i][T_M_MS] += (uint64_t)sv->n_cls[i];
          R->Ym[i] -= sv->n_cls[i]; R->Ys[i] += sv->n_cls[i];
        }
        /* block (step, stream 10, server, replication): word 0 -> patience for the wait in the decode
         * buffer; word 1 -> under the randomized router (Sec. 5.2), the group the decode is sent to:
         * solo with probability p_s,i, else mixed, each with its own FIFO buffer */
        if (o->cfg.route_mode == ROUTE_IMMEDIATE) {
          /* Immediate same-slot decode (the "I" rule of the paper's ablation study): the request goes on
           * decoding on the server that prefilled it, in the slot it already holds; the gate has seen to
           * it that the slot exists. It joins the batch at the restart that follows this completion. */
          int j = 0; while (j < B && sv->slot[j].used) j++;
          if (j < B) {
            slot_t *e = &sv->slot[j];
            e->used = 1; e->cls = k; e->P = sv->pf_P; e->D = sv->pf_D; e->stamp = sv->pf_stamp;
            e->fin = sv->iter + (uint32_t)sv->pf_D;
            sv->n_dec++; sv->n_cls[k]++;
            R->tally[k][T_U_DS]++; R->Ys[k]++;
          } else { R->tally[k][T_DROP_D]++; R->glob[G_OVERFLOW] = 1; }
          goto prefill_done;
        }
        fifojob *buf = &R->dbuf;
        if (o->cfg.route_mode == ROUTE_RANDOM_SPLIT || o->cfg.route_mode == ROUTE_WEIGHTED_SPLIT) {
          draw(o, r, g, s, 10u, w);
          if (!(w[1] < o->solo_thr[k])) buf = &R->dbuf_m;
        }
        if (buf->len < o->cfg.dbuf_cap) {
          job_t jb = { k, sv->pf_P, sv->pf_D, sv->pf_stamp, DL_NEVER };
          if (o->tab_pat[k]) { draw(o, r, g, s, 10u, w); jb.dl = s + o->tab_pat[k][w[0] >> 16]; }
          fj_push(buf, jb); R->Qd[k]++;
        } else { R->tally[k][T_DROP_D]++; R->glob[G_OVERFLOW] = 1; }
        prefill_done: ;
      }
    }
    for (int k = 0; k < K; k++) sv->n_join[k] = 0;
    sv->at_boundary = 1;
  }

  /* 3. prefill gate on mixed-group servers with an idle prefill slot, ascending index */
  for (int g = 0; g < M; g++) {
    server_t *sv = &R->sv[g];
    if (sv->pf_rem) continue;
    if (o->cfg.route_mode == ROUTE_IMMEDIATE && sv->n_dec >= B) continue;   /* no slot for one more request */
    int best = -1; double bxi = 0.0, bdl = 0.0;
    for (int i = 0; i < K; i++) {
      if (R->Qp[i] <= 0) continue;
      if (o->cfg.gate_mode == GATE_OCCUPANCY) {
        if (!(o->x_star[i] > 0.0)) continue;
        double xi = ((double)R->X[i] - o->nx[i]) * o->invx[i];
        double dl = (double)R->Qp[i] - o->nq[i];
        if (best < 0 || xi < bxi || (xi == bxi && dl > bdl)) { best = i; bxi = xi; bdl = dl; }
      } else if (o->cfg.gate_mode == GATE_PRIORITY) {  /* largest static index, ties lowest class */
        double pr = o->cls[i].priority;
        if (best < 0 || pr > bxi) { best = i; bxi = pr; }
      } else {                                         /* FCFS across classes: oldest head, ties lowest class */
        double st = (double)R->q[i].v[R->q[i].head].stamp;
        if (best < 0 || st < bxi) { best = i; bxi = st; }
      }
    }
    if (best < 0) break;
    const int k = best;
    uint32_t stamp = fq_pop(&R->q[k]).stamp;
    R->Qp[k]--; R->X[k]++; R->tally[k][T_U_P]++;
    R->tally[k][T_WAIT_STEPS] += (uint64_t)(s - stamp);
    draw(o, r, g, s, 1, w);
    sv->pf_cls = k; sv->pf_stamp = stamp;
    sv->pf_P = o->tab_in[k][w[0] >> 16];
    sv->pf_D = o->tab_out[k][w[1] >> 16];
    sv->pf_rem = sv->pf_P;
    for (int i = 0; i < K; i++) {                      /* co-resident decodes switch solo -> mixed */
      R->tally[i][T_M_SM] += (uint64_t)sv->n_cls[i];
      R->Ys[i] -= sv->n_cls[i]; R->Ym[i] += sv->n_cls[i];
    }
  }

  /* 4. decode routing: buffer in FIFO order; solo group first, then mixed group;
   *    least-loaded feasible server, ties to the lowest index */
  /*    Under the randomized router each component of the buffer feeds its own group only: first the
   *    solo component to the solo group, then the mixed component to the mixed group (the two do not
   *    interact); within the group the same least-loaded rule. */
  /*    General SLI-aware router (EC "General SLI-aware Extension"): the two pools as above, but whenever a slot of
   *    a pool is filled the class is drawn with the pool's selection weights restricted to the classes that wait
   *    in the pool's buffer, and the head-of-line job of that class is taken (FCFS within a class). The j-th
   *    placement of the step in a pool uses word 0 of block (step, stream 11 for solo / 12 for mixed, j,
   *    replication): with W the sum of the weights (in units of 2^-20) of the waiting classes, x = (word * W) >> 32
   *    falls into the weight interval of the chosen class, classes in ascending order. */
  for (int pass = 0; pass < 2; pass++) {
  const int weighted = o->cfg.route_mode == ROUTE_WEIGHTED_SPLIT;
  const int split = o->cfg.route_mode == ROUTE_RANDOM_SPLIT || weighted;
  fifojob *buf = (split && pass == 1) ? &R->dbuf_m : &R->dbuf;
  if (!split && pass == 1) break;
  uint32_t placed = 0;
  while (buf->len > 0) {
    int dst = -1, bl = 0;
    if (!split || pass == 0)
      for (int g = M; g < N; g++) { int l = R->sv[g].n_dec; if (l < B && (dst < 0 || l < bl)) { dst = g; bl = l; } }
    if (dst < 0 && (!split || pass == 1))
      for (int g = 0; g < M; g++) { int l = R->sv[g].n_dec; if (l < B - 1 && (dst < 0 || l < bl)) { dst = g; bl = l; } }
    if (dst < 0) break;
    job_t jb;
    if (weighted) {
      int64_t first[MAXK];
      uint64_t total = 0;
      for (int k = 0; k < K; k++) first[k] = -1;
      for (int64_t i = 0; i < buf->len; i++) {
        int c = buf->v[buf->head + i].cls;
        if (first[c] < 0) first[c] = i;
      }
      for (int k = 0; k < K; k++) if (first[k] >= 0) total += o->wsel[pass][k];
      draw(o, r, (int)placed, s, 11u + (uint32_t)pass, w);
      uint64_t x = ((uint64_t)w[0] * total) >> 32, cum = 0;
      int c = -1;
      for (int k = 0; k < K && c < 0; k++) {
        if (first[k] < 0) continue;
        cum += o->wsel[pass][k];
        if (x < cum) c = k;
      }
      jb = buf->v[buf->head + first[c]];
      for (int64_t i = first[c]; i + 1 < buf->len; i++) buf->v[buf->head + i] = buf->v[buf->head + i + 1];
      buf->len--;
    } else {
      jb = fj_pop(buf);
    }
    placed++;
    server_t *sv = &R->sv[dst];
    R->Qd[jb.cls]--;
    int j = 0; while (sv->slot[j].used) j++;
    const int mid = sv->t_next != T_IDLE && !sv->at_boundary;   /* joins at the next start */
    slot_t *e = &sv->slot[j];
    e->used = 1; e->cls = jb.cls; e->P = jb.P; e->D = jb.D; e->stamp = jb.stamp;
    e->fin = sv->iter + (uint32_t)jb.D + (mid ? 1u : 0u);
    sv->n_dec++; sv->n_cls[jb.cls]++;
    if (mid) sv->n_join[jb.cls]++;
    if (sv->pf_rem > 0) { R->tally[jb.cls][T_U_DM]++; R->Ym[jb.cls]++; }
    else { R->tally[jb.cls][T_U_DS]++; R->Ys[jb.cls]++; }
  }
  }

  /* 5. (re)start: servers at an iteration boundary, and idle servers that got work */
  for (int g = 0; g < N; g++) {
    server_t *sv = &R->sv[g];
    const int idle = sv->t_next == T_IDLE;
    if (!sv->at_boundary && !idle) continue;
    int ptok = sv->pf_rem > 0 ? (sv->pf_rem < C ? sv->pf_rem : C) : 0;
    int n = sv->n_dec;
    if (ptok == 0 && n == 0) { sv->t_next = T_IDLE; sv->ptok_frozen = 0; sv->d_frozen = 0; continue; }
    int64_t base = sv->at_boundary ? sv->t_next : T;   /* back-to-back after a completion */
    sv->d_frozen = iter_time(o, ptok, n);
    sv->ptok_frozen = ptok;
    sv->t_next = base + sv->d_frozen;
  }

  /* 6. end-of-step occupancy integrals */
  for (int k = 0; k < K; k++) {
    R->tally[k][T_SUM_QP] += (uint64_t)R->Qp[k];
    R->tally[k][T_SUM_QD] += (uint64_t)R->Qd[k];
    R->tally[k][T_SUM_X] += (uint64_t)R->X[k];
    R->tally[k][T_SUM_YM] += (uint64_t)R->Ym[k];
    R->tally[k][T_SUM_YS] += (uint64_t)R->Ys[k];
  }
  R->glob[G_STEPS]++;
}

/* Replaces the gate's targets between runs; the state is kept (the hook of the paper's online adaptive
 * algorithm, trace-driven online policy evaluation: only x* and q_p* move here, the split M stays). */
int oracle_set_targets(oracle_t *o, const double *x_star, const double *qp_star)
{
  if (!o || !x_star || !qp_star) return -1;
  for (int k = 0; k < o->cfg.K; k++)
    if (!(x_star[k] >= 0.0) || !isfinite(x_star[k]) || !isfinite(qp_star[k])) return -1;
  for (int k = 0; k < o->cfg.K; k++) {
    o->x_star[k] = x_star[k];
    o->qp_star[k] = qp_star[k];
    o->nx[k] = (double)o->cfg.N * x_star[k];
    o->invx[k] = x_star[k] > 0.0 ? 1.0 / x_star[k] : 0.0;
    o->nq[k] = (double)o->cfg.N * qp_star[k];
  }
  return 0;
}

/* Moves the mixed/solo split between runs: servers 0..M-1 are the mixed group from here on (the online
 * adaptive algorithm's M*(t_k), Eq. main-online-mixed-target). Existing service is not pre-empted: a prefill
 * in service on a server that turns solo runs to its end (no further admission there), decodes on a server
 * that turns mixed stay (it takes new ones only below B-1); the new split governs later admissions and
 * placements. */
int oracle_set_split(oracle_t *o, int M)
{
  if (!o || M < 0 || M > o->cfg.N) return -1;
  if (M != o->cfg.M) { o->cfg.M = M; o->split_moved = 1; }
  return 0;
}

/* run `steps` more steps; a different (replications, seed) pair restarts from the empty system */
int oracle_run(oracle_t *o, int64_t steps, int replications, uint64_t seed)
{
  if (!o || steps < 0 || replications < 1 || replications > o->max_reps) return -1;
  if (replications != o->reps || seed != o->seed || o->steps_done == 0) {
    for (int r = 0; r < o->max_reps; r++) rep_free(&o->rep[r]);
    o->reps = replications; o->seed = seed; o->steps_done = 0; o->split_moved = 0;
  }
  if (o->steps_done + steps >= ((int64_t)1 << 29)) return -1;
  int n = o->nsel ? o->nsel : replications;
  for (int i = 0; i < n; i++) {
    int r = o->nsel ? o->sel[i] : i;
    if (r < 0 || r >= replications) return -1;
    if (!o->rep[r].inited) rep_init(o, &o->rep[r]);
  }
  int64_t s0 = o->steps_done;
  for (int64_t s = s0; s < s0 + steps; s++) {
    for (int i = 0; i < n; i++) {
      int r = o->nsel ? o->sel[i] : i;
      step_rep(o, r, (uint32_t)s);
    }
    o->steps_done = s + 1;
    if (o->check_every > 0 && ((s + 1) % o->check_every == 0))
      for (int i = 0; i < n; i++) check_rep(o, o->nsel ? o->sel[i] : i);
  }
  return 0;
}

/* ------------------------------------------------------------- read-outs ---- */
static uint64_t jobword(int cls, int P, int D, uint32_t stamp)
{
  return (uint64_t)stamp | ((uint64_t)cls << 29) | ((uint64_t)(P - 1) << 32) | ((uint64_t)(D - 1) << 48);
}

static rep_t *getrep(oracle_t *o, int r) { return (o && r >= 0 && r < o->reps && o->rep[r].inited) ? &o->rep[r] : NULL; }

/* out[5][K]: Qp, X, Qd, Ym, Ys */
int oracle_get_class_state(oracle_t *o, int r, int64_t *out)
{
  rep_t *R = getrep(o, r); if (!R) return -1;
  int K = o->cfg.K;
  for (int k = 0; k < K; k++) {
    out[0 * K + k] = R->Qp[k]; out[1 * K + k] = R->X[k]; out[2 * K + k] = R->Qd[k];
    out[3 * K + k] = R->Ym[k]; out[4 * K + k] = R->Ys[k];
  }
  return 0;
}

int oracle_get_servers(oracle_t *o, int r, int64_t *t_next, uint32_t *iter, int32_t *rem, int32_t *ptok,
                       uint64_t *pfjob, uint8_t *n_cls, uint8_t *n_join)
{
  rep_t *R = getrep(o, r); if (!R) return -1;
  for (int g = 0; g < o->cfg.N; g++) {
    server_t *s = &R->sv[g];
    t_next[g] = s->t_next; iter[g] = s->iter; rem[g] = s->pf_rem; ptok[g] = s->ptok_frozen;
    pfjob[g] = s->pf_rem ? jobword(s->pf_cls, s->pf_P, s->pf_D, s->pf_stamp) : 0;
    for (int k = 0; k < MAXK; k++) { n_cls[g * MAXK + k] = (uint8_t)s->n_cls[k]; n_join[g * MAXK + k] = (uint8_t)s->n_join[k]; }
  }
  return 0;
}

/* occupied slots of every server, packed to the front in slot order: fin[N][B], job[N][B], n_dec[N] */
int oracle_get_slots(oracle_t *o, int r, uint32_t *fin, uint64_t *job, int32_t *n_dec)
{
  rep_t *R = getrep(o, r); if (!R) return -1;
  int B = o->cfg.B;
  for (int g = 0; g < o->cfg.N; g++) {
    server_t *s = &R->sv[g];
    int c = 0;
    for (int j = 0; j < B; j++) if (s->slot[j].used) {
      fin[(size_t)g * B + c] = s->slot[j].fin;
      job[(size_t)g * B + c] = jobword(s->slot[j].cls, s->slot[j].P, s->slot[j].D, s->slot[j].stamp);
      c++;
    }
    for (int j = c; j < B; j++) { fin[(size_t)g * B + j] = 0; job[(size_t)g * B + j] = 0; }
    n_dec[g] = c;
  }
  return 0;
}

/* k in [0,K): arrival stamps of the class prefill queue, head first (as u64); k = -1: decode buffer job words */
int oracle_get_queue(oracle_t *o, int r, int k, uint64_t *out, int64_t cap, int64_t *len)
{
  rep_t *R = getrep(o, r); if (!R) return -1;
  if (k < 0) {   /* -1: decode buffer (solo component), -2: mixed component */
    fifojob *b = k == -2 ? &R->dbuf_m : &R->dbuf;
    *len = b->len;
    for (int64_t i = 0; i < b->len && i < cap; i++) {
      job_t *j = &b->v[b->head + i];
      out[i] = jobword(j->cls, j->P, j->D, j->stamp);
    }
  } else {
    if (k >= o->cfg.K) return -1;
    *len = R->q[k].len;
    for (int64_t i = 0; i < R->q[k].len && i < cap; i++) out[i] = R->q[k].v[R->q[k].head + i].stamp;
  }
  return 0;
}

/* the steps at which the same entries abandon if still waiting (0xFFFFFFFF: never), same order */
int oracle_get_queue_deadlines(oracle_t *o, int r, int k, uint64_t *out, int64_t cap, int64_t *len)
{
  rep_t *R = getrep(o, r); if (!R) return -1;
  if (k < 0) {
    fifojob *b = k == -2 ? &R->dbuf_m : &R->dbuf;
    *len = b->len;
    for (int64_t i = 0; i < b->len && i < cap; i++) out[i] = b->v[b->head + i].dl;
  } else {
    if (k >= o->cfg.K) return -1;
    *len = R->q[k].len;
    for (int64_t i = 0; i < R->q[k].len && i < cap; i++) out[i] = R->q[k].v[R->q[k].head + i].dl;
  }
  return 0;
}

/* tallies of one replication: out[K][NTALLY] then glob[NGLOBAL] */
int oracle_get_tallies(oracle_t *o, int r, uint64_t *out)
{
  rep_t *R = getrep(o, r); if (!R) return -1;
  int K = o->cfg.K;
  for (int k = 0; k < K; k++) for (int t = 0; t < NTALLY; t++) out[k * NTALLY + t] = R->tally[k][t];
  for (int t = 0; t < NGLOBAL; t++) out[K * NTALLY + t] = R->glob[t];
  return 0;
}

/* which: 0 ttft, 1 e2e, 2 tbt; out[K][NBIN] */
int oracle_get_hist(oracle_t *o, int r, int which, uint64_t *out)
{
  rep_t *R = getrep(o, r); if (!R || which < 0 || which > 2) return -1;
  for (int k = 0; k < o->cfg.K; k++) memcpy(out + (size_t)k * NBIN, HIST(R, which, k), NBIN * sizeof(uint64_t));
  return 0;
}

int oracle_get_tables(oracle_t *o, int k, uint16_t *tin, uint16_t *tout, uint32_t *cls_thr, uint32_t *arr_thr, int64_t arr_rows)
{
  if (!o || k < 0 || k >= o->cfg.K) return -1;
  if (tin) memcpy(tin, o->tab_in[k], 65536 * 2);
  if (tout) memcpy(tout, o->tab_out[k], 65536 * 2);
  if (cls_thr) memcpy(cls_thr, o->cls_thr, MAXK * sizeof(uint32_t));
  if (arr_thr) memcpy(arr_thr, o->arr_thr, (size_t)(arr_rows < o->rows ? arr_rows : o->rows) * 3 * sizeof(uint32_t));
  return 0;
}

int64_t oracle_steps_done(const oracle_t *o) { return o->steps_done; }
int oracle_ntally(void) { return NTALLY; }
int oracle_nglobal(void) { return NGLOBAL; }
int oracle_nbin(void) { return NBIN; }

/* --------------------------------------------------------------- digest ---- */
/* 64-bit order-independent digest of the integer state of one replication:
 * sum mod 2^64 of a chained splitmix64 finaliser over tagged items; slot items
 * do not depend on the slot position, everything else carries its position. */
static uint64_t mix64(uint64_t z)
{
  z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
  z ^= z >> 27; z *= 0x94D049BB133111EBull;
  z ^= z >> 31;
  return z;
}
static uint64_t chain(uint64_t h, uint64_t w) { return mix64(h + w + 0x9E3779B97F4A7C15ull); }

int oracle_digest(oracle_t *o, int r, uint64_t *out)
{
  rep_t *R = getrep(o, r); if (!R) return -1;
  const int K = o->cfg.K, N = o->cfg.N, B = o->cfg.B;
  uint64_t d = 0;
  for (int k = 0; k < K; k++) {
    uint64_t h = chain(1, (uint64_t)k);
    h = chain(h, (uint64_t)R->Qp[k]); h = chain(h, (uint64_t)R->X[k]); h = chain(h, (uint64_t)R->Qd[k]);
    h = chain(h, (uint64_t)R->Ym[k]); h = chain(h, (uint64_t)R->Ys[k]);
    d += h;
    for (int64_t i = 0; i < R->q[k].len; i++) {
      uint64_t h2 = chain(chain(chain(2, (uint64_t)k), (uint64_t)i), R->q[k].v[R->q[k].head + i].stamp);
      if (o->any_theta) h2 = chain(h2, R->q[k].v[R->q[k].head + i].dl);
      d += h2;
    }
  }
  for (int64_t i = 0; i < R->dbuf.len; i++) {
    job_t *j = &R->dbuf.v[R->dbuf.head + i];
    uint64_t h2 = chain(chain(3, (uint64_t)i), jobword(j->cls, j->P, j->D, j->stamp));
    if (o->any_theta) h2 = chain(h2, j->dl);
    d += h2;
  }
  for (int64_t i = 0; i < R->dbuf_m.len; i++) {
    job_t *j = &R->dbuf_m.v[R->dbuf_m.head + i];
    uint64_t h2 = chain(chain(6, (uint64_t)i), jobword(j->cls, j->P, j->D, j->stamp));
    if (o->any_theta) h2 = chain(h2, j->dl);
    d += h2;
  }
  for (int g = 0; g < N; g++) {
    server_t *s = &R->sv[g];
    uint64_t nc = 0, nj = 0;
    for (int k = 0; k < MAXK; k++) { nc |= (uint64_t)s->n_cls[k] << (8 * k); nj |= (uint64_t)s->n_join[k] << (8 * k); }
    uint64_t h = chain(4, (uint64_t)g);
    h = chain(h, (uint64_t)s->t_next); h = chain(h, s->iter);
    h = chain(h, (uint64_t)s->pf_rem); h = chain(h, (uint64_t)s->ptok_frozen);
    h = chain(h, s->pf_rem ? jobword(s->pf_cls, s->pf_P, s->pf_D, s->pf_stamp) : 0);
    h = chain(h, nc); h = chain(h, nj);
    d += h;
    for (int j = 0; j < B; j++) if (s->slot[j].used) {
      slot_t *e = &s->slot[j];
      d += chain(chain(chain(5, (uint64_t)g), e->fin), jobword(e->cls, e->P, e->D, e->stamp));
    }
  }
  *out = d;
  return 0;
}

/* ---------------------------------------------------------------- stats ---- */
typedef struct {
  int32_t K, replications;
  int64_t steps;
  double sim_time;                        /* steps * dt, in time units */
  uint64_t tally[MAXK][NTALLY];           /* summed over replications */
  uint64_t glob[NGLOBAL];
  double arrival_rate[MAXK];              /* per server per unit time */
  double completion_rate[MAXK];
  double served_fraction[MAXK];           /* decode completions / arrivals */
  double tok_rate_prefill[MAXK], tok_rate_decode[MAXK];
  double rev_bundled[MAXK], rev_separate[MAXK], rev_mixed[MAXK];
  double rev_bundled_total, rev_separate_total, rev_mixed_total;
  double mean_qp[MAXK], mean_qd[MAXK], mean_x[MAXK], mean_ym[MAXK], mean_ys[MAXK]; /* per server */
  double ttft_mean[MAXK], ttft_p50[MAXK], ttft_p95[MAXK], ttft_p99[MAXK];
  double e2e_mean[MAXK], e2e_p50[MAXK], e2e_p95[MAXK], e2e_p99[MAXK];
  double tbt_mean[MAXK], tbt_p50[MAXK], tbt_p95[MAXK], tbt_p99[MAXK];
  double mean_wait[MAXK];                 /* prefill-queue wait of admitted jobs, time units */
  double fair_gap_x, fair_gap_ys, fair_min_served;
  double util_mix, util_solo;             /* busy time per server-time, by iteration kind */
  double iter_rate;                       /* executed iterations per server per unit time */
  double abandon_rate_p[MAXK], abandon_rate_d[MAXK]; /* abandonments per server per unit time: prefill queue, decode buffer */
} oracle_stats_t;

static int64_t hedge(int b)
{
  if (b < 16) return b;
  int e = b / 16 + 3, m = b % 16;
  return (int64_t)(16 + m) << (e - 4);
}
int64_t oracle_hedge(int b) { return hedge(b); }

static double pctl(const uint64_t *h, int pct)
{
  uint64_t n = 0;
  for (int b = 0; b < NBIN; b++) n += h[b];
  if (!n) return 0.0;
  uint64_t rank = (n * (uint64_t)pct + 99) / 100, cum = 0;
  for (int b = 0; b < NBIN; b++) { cum += h[b]; if (cum >= rank) return (double)hedge(b) * 1e-9; }
  return (double)hedge(NBIN - 1) * 1e-9;
}

static double ratio(double a, double b) { return b > 0.0 ? a / b : 0.0; }

int oracle_stats(oracle_t *o, oracle_stats_t *st)
{
  if (!o || !st) return -1;
  memset(st, 0, sizeof *st);
  const int K = o->cfg.K;
  uint64_t *hs = calloc((size_t)3 * MAXK * NBIN, sizeof(uint64_t));
  int nrep = 0;
  for (int r = 0; r < o->reps; r++) {
    rep_t *R = &o->rep[r];
    if (!R->inited) continue;
    nrep++;
    for (int k = 0; k < K; k++) for (int t = 0; t < NTALLY; t++) st->tally[k][t] += R->tally[k][t];
    for (int t = 0; t < NGLOBAL; t++) st->glob[t] += R->glob[t];
    for (size_t i = 0; i < (size_t)3 * MAXK * NBIN; i++) hs[i] += R->hist[i];
  }
  st->K = K; st->replications = nrep; st->steps = o->steps_done;
  st->sim_time = (double)o->steps_done * ((double)o->dt_ns * 1e-9);
  const double nt = (double)o->cfg.N * st->sim_time * (double)nrep;        /* server-time */
  const double ns = (double)o->cfg.N * (double)o->steps_done * (double)nrep; /* server-steps */
  double xmin = 0, xmax = 0, ymin = 0, ymax = 0, smin = 0;
  for (int k = 0; k < K; k++) {
    const uint64_t *t = st->tally[k];
    double sd = (double)(t[T_S_DM] + t[T_S_DS]);
    st->arrival_rate[k] = ratio((double)t[T_A], nt);
    st->completion_rate[k] = ratio(sd, nt);
    st->served_fraction[k] = ratio(sd, (double)t[T_A]);
    st->tok_rate_prefill[k] = ratio((double)t[T_TOK_PREF], nt);
    st->tok_rate_decode[k] = ratio((double)t[T_TOK_EMIT], nt);
    double rb = o->cls[k].price_in * (double)t[T_TOKP_DEC] + o->cls[k].price_out * (double)t[T_TOKD_DEC];
    double rs = o->cls[k].price_in * (double)t[T_TOKP_PRE] + o->cls[k].price_out * (double)t[T_TOKD_DEC];
    st->rev_bundled[k] = ratio(rb, nt);
    st->rev_separate[k] = ratio(rs, nt);
    st->rev_mixed[k] = o->cls[k].bundled ? st->rev_bundled[k] : st->rev_separate[k];
    st->rev_bundled_total += st->rev_bundled[k];
    st->rev_separate_total += st->rev_separate[k];
    st->rev_mixed_total += st->rev_mixed[k];
    st->mean_qp[k] = ratio((double)t[T_SUM_QP], ns);
    st->mean_qd[k] = ratio((double)t[T_SUM_QD], ns);
    st->mean_x[k] = ratio((double)t[T_SUM_X], ns);
    st->mean_ym[k] = ratio((double)t[T_SUM_YM], ns);
    st->mean_ys[k] = ratio((double)t[T_SUM_YS], ns);
    st->ttft_mean[k] = ratio((double)t[T_TTFT_SUM] * 1e-9, (double)t[T_S_P]);
    st->e2e_mean[k] = ratio((double)t[T_E2E_SUM] * 1e-9, sd);
    st->tbt_mean[k] = ratio((double)t[T_TBT_SUM] * 1e-9, (double)t[T_TOK_EMIT]);
    st->abandon_rate_p[k] = ratio((double)t[T_AB_P], nt);
    st->abandon_rate_d[k] = ratio((double)t[T_AB_D], nt);
    st->mean_wait[k] = ratio((double)t[T_WAIT_STEPS] * ((double)o->dt_ns * 1e-9), (double)t[T_U_P]);
    const uint64_t *h0 = hs + ((size_t)0 * MAXK + k) * NBIN, *h1 = hs + ((size_t)1 * MAXK + k) * NBIN,
                   *h2 = hs + ((size_t)2 * MAXK + k) * NBIN;
    st->ttft_p50[k] = pctl(h0, 50); st->ttft_p95[k] = pctl(h0, 95); st->ttft_p99[k] = pctl(h0, 99);
    st->e2e_p50[k] = pctl(h1, 50); st->e2e_p95[k] = pctl(h1, 95); st->e2e_p99[k] = pctl(h1, 99);
    st->tbt_p50[k] = pctl(h2, 50); st->tbt_p95[k] = pctl(h2, 95); st->tbt_p99[k] = pctl(h2, 99);
    if (k == 0 || st->mean_x[k] < xmin) xmin = st->mean_x[k];
    if (k == 0 || st->mean_x[k] > xmax) xmax = st->mean_x[k];
    if (k == 0 || st->mean_ys[k] < ymin) ymin = st->mean_ys[k];
    if (k == 0 || st->mean_ys[k] > ymax) ymax = st->mean_ys[k];
    if (k == 0 || st->served_fraction[k] < smin) smin = st->served_fraction[k];
  }
  st->fair_gap_x = xmax - xmin;        /* max_{i,j} (x_i - x_j), prefill fairness SLI (Sec. 5.2) */
  st->fair_gap_ys = ymax - ymin;       /* max_{i,j} (y_s,i - y_s,j), decode fairness SLI */
  st->fair_min_served = smin;
  st->util_mix = ratio((double)st->glob[G_BUSY_MIX] * 1e-9, nt);
  st->util_solo = ratio((double)st->glob[G_BUSY_SOLO] * 1e-9, nt);
  st->iter_rate = ratio((double)(st->glob[G_ITERS_MIX] + st->glob[G_ITERS_SOLO]), nt);
  free(hs);
  return 0;
}
int oracle_stats_size(void) { return (int)sizeof(oracle_stats_t); }
