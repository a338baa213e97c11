// C ABI of the simulator: configuration checks, workspace layout, launches, read-outs.
#include <hip/hip_runtime_api.h>

#include <cmath>
#include <cstring>
#include <memory>
#include <new>
#include <vector>

#include "gnr_internal.h"

using namespace gnr;

struct sim_t {
  sim_config cfg;
  sim_class cls[kMaxK];
  double x_star[kMaxK], qp_star[kMaxK], p_solo[kMaxK], w_solo[kMaxK], w_mixed[kMaxK];
  Params p;
  int max_reps;
  int reps;
  uint64_t seed;
  int64_t steps_done;
  bool started;
  int threads;
  size_t lds_bytes;
  int64_t rows;
  unsigned char *ws;
  size_t ws_bytes;
  int device;
  // kernel timing: one pair of events per launch, read out and destroyed by drain_events
  std::vector<std::pair<hipEvent_t, hipEvent_t>> pending;
  int64_t launches;
  double kernel_ms;
};

namespace {

constexpr uint32_t kStepsPerLaunch = 2048;

struct Layout {
  size_t arr_thr, len_tab, t_next, iter, remptok, pf_job, n_cls, n_join, fin, job, qring, dring, cstate, tally, hist,
      digest, reduced, params, pat_tab, qdl, ddl, cal, dcal, dring_m, ddl_m, dcal_m, total;
};

bool any_patience(const sim_config &c)
{
  for (int k = 0; k < c.K; ++k)
    if (c.cls[k].theta > 0.0) return true;
  return false;
}

size_t align_up(size_t v) { return (v + 255) & ~size_t(255); }

// `cal_entries`: size of one deadline calendar (0 when no class has a patience rate)
Layout make_layout(const sim_config &c, int R, int64_t rows, size_t cal_entries)
{
  Layout L{};
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
  const size_t RN = static_cast<size_t>(R) * c.N;
  L.arr_thr = take(static_cast<size_t>(rows) * 3 * sizeof(uint32_t));
  L.len_tab = take(static_cast<size_t>(c.K) * 2 * kTableSize * sizeof(uint16_t));
  L.t_next = take(RN * sizeof(int64_t));
  L.iter = take(RN * sizeof(uint32_t));
  L.remptok = take(RN * sizeof(uint32_t));
  L.pf_job = take(RN * sizeof(uint64_t));
  L.n_cls = take(RN * sizeof(uint64_t));
  L.n_join = take(RN * sizeof(uint64_t));
  const size_t BS = (static_cast<size_t>(c.B) + 3) & ~size_t(3);
  L.fin = take(RN * BS * sizeof(uint32_t));
  L.job = take(RN * BS * sizeof(uint64_t));
  L.qring = take(static_cast<size_t>(R) * c.K * c.queue_cap * sizeof(uint32_t));
  L.dring = take(static_cast<size_t>(R) * c.dbuf_cap * sizeof(uint64_t));
  L.cstate = take(static_cast<size_t>(R) * CS_WORDS * sizeof(int32_t));
  L.tally = take(static_cast<size_t>(R) * kTallyWords * sizeof(uint64_t));
  L.hist = take(static_cast<size_t>(R) * 3 * c.K * kNBin * sizeof(uint64_t));
  L.digest = take(static_cast<size_t>(R) * sizeof(uint64_t));
  L.reduced = take((kTallyWords + static_cast<size_t>(3) * c.K * kNBin) * sizeof(uint64_t));
  L.params = take(sizeof(Params));
  if (cal_entries) {
    L.pat_tab = take(static_cast<size_t>(c.K) * kTableSize * sizeof(uint16_t));
    L.qdl = take(static_cast<size_t>(R) * c.K * c.queue_cap * sizeof(uint32_t));
    L.ddl = take(static_cast<size_t>(R) * c.dbuf_cap * sizeof(uint32_t));
    L.cal = take(static_cast<size_t>(R) * c.K * cal_entries * sizeof(uint32_t));
    L.dcal = take(static_cast<size_t>(R) * c.K * cal_entries * sizeof(uint32_t));
  }
  if (c.route_mode == SIM_ROUTE_RANDOM_SPLIT || c.route_mode == SIM_ROUTE_WEIGHTED_SPLIT) {
    L.dring_m = take(static_cast<size_t>(R) * c.dbuf_cap * sizeof(uint64_t));
    if (cal_entries) {
      L.ddl_m = take(static_cast<size_t>(R) * c.dbuf_cap * sizeof(uint32_t));
      L.dcal_m = take(static_cast<size_t>(R) * c.K * cal_entries * sizeof(uint32_t));
    }
  }
  L.total = off;
  return L;
}

struct Ticks { int64_t c0, cpre, cdec, dt; };

int host_hbin(int64_t v)
{
  if (v < 16) return v < 0 ? 0 : static_cast<int>(v);
  const int e = 63 - __builtin_clzll(static_cast<unsigned long long>(v));
  const int b = 16 * (e - 3) + static_cast<int>((v >> (e - 4)) & 15);
  return b < kNBin ? b : kNBin - 1;
}

int64_t host_hedge(int b)
{
  if (b < 16) return b;
  return static_cast<int64_t>(16 + b % 16) << (b / 16 - 1);
}

constexpr size_t kOnChipLimit = 160 * 1024;   // LDS of a compute unit; a replication's workgroup runs there alone

// What decides the step kernel's launch shape, for a configuration with the mixed group at servers 0..M-1 and a
// launch of `reps` replications (few replications get the largest workgroups, which need most on-chip bytes).
Params shape_params(const sim_config &c, const Ticks &t, int M, int reps)
{
  Params q;
  std::memset(&q, 0, sizeof q);
  q.K = c.K; q.N = c.N; q.Mp = M;
  q.tbt_w = host_hbin(t.c0 + t.cpre * c.C + t.cdec * c.B) - host_hbin(t.c0) + 1;
  q.nwords = (c.N + 63) / 64;
  q.route_mode = c.route_mode;   // the weighted router keeps its class selections on chip
  for (int k = 0; k < c.K; ++k)
    if (c.cls[k].theta > 0.0) q.ab_classes |= 1u << k;
  q.dl_rings = q.ab_classes != 0 || c.route_mode == SIM_ROUTE_WEIGHTED_SPLIT;
  q.threads = step_threads(q, reps);
  return q;
}

size_t on_chip_bytes(const sim_config &c, const Ticks &t, int M, int reps)
{
  return step_lds_bytes(shape_params(c, t, M, reps));
}

int validate(const sim_config *c, int max_reps, Ticks *t)
{
  if (!c || max_reps < 1 || max_reps > SIM_MAXR || !c->cls || !c->x_star || !c->qp_star) return SIM_EINVAL;
  if (c->K < 1 || c->K > kMaxK || c->N < 1 || c->N > kMaxN || c->B < 1 || c->B > kMaxB) return SIM_EINVAL;
  if (c->C < 1 || c->C > kMaxChunk || c->M < 0 || c->M > c->N) return SIM_EINVAL;
  if (c->queue_cap < 1 || c->queue_cap > (int64_t(1) << 30) || c->dbuf_cap < 1 || c->dbuf_cap > (int64_t(1) << 30))
    return SIM_EINVAL;
  if (c->gate_mode < SIM_GATE_OCCUPANCY || c->gate_mode > SIM_GATE_FCFS) return SIM_EINVAL;
  if (c->route_mode < SIM_ROUTE_SOLO_FIRST || c->route_mode > SIM_ROUTE_WEIGHTED_SPLIT) return SIM_EINVAL;
  if (c->route_mode == SIM_ROUTE_WEIGHTED_SPLIT) {
    if (!c->w_solo || !c->w_mixed) return SIM_EINVAL;
    for (int k = 0; k < c->K; ++k)
      if (!(c->w_solo[k] >= 0.0) || !(c->w_solo[k] <= 1.0) || !(c->w_mixed[k] >= 0.0) || !(c->w_mixed[k] <= 1.0))
        return SIM_EINVAL;
  }
  if (c->route_mode == SIM_ROUTE_RANDOM_SPLIT || c->route_mode == SIM_ROUTE_WEIGHTED_SPLIT) {
    if (!c->p_solo) return SIM_EINVAL;
    for (int k = 0; k < c->K; ++k)
      if (!(c->p_solo[k] >= 0.0) || !(c->p_solo[k] <= 1.0)) return SIM_EINVAL;
  }
  // one threshold row per step of the period; a run stays below 2^29 steps, so a longer period is never needed
  if (c->mod_period < 0 || c->mod_period > (int64_t(1) << 29) || !(std::fabs(c->mod_amp) <= 1.0)) return SIM_EINVAL;
  if (!(c->c0 > 0.0) || !(c->c_pre >= 0.0) || !(c->c_dec >= 0.0) || !(c->dt >= 0.0)) return SIM_EINVAL;
  t->c0 = std::llround(c->c0 * 1e9);
  t->cpre = std::llround(c->c_pre * 1e9);
  t->cdec = std::llround(c->c_dec * 1e9);
  t->dt = c->dt > 0.0 ? std::llround(c->dt * 1e9) : t->c0;
  if (t->c0 < 1 || t->dt < 1 || t->dt > t->c0) return SIM_EINVAL;
  if (t->c0 > (int64_t(1) << 40) || t->cpre > (int64_t(1) << 32) || t->cdec > (int64_t(1) << 32)) return SIM_EINVAL;
  for (int k = 0; k < c->K; ++k) {
    const sim_class &q = c->cls[k];
    if (!(q.theta >= 0.0) || !std::isfinite(q.theta) || !(q.lambda >= 0.0) || !(c->x_star[k] >= 0.0) || !std::isfinite(c->qp_star[k])) return SIM_EINVAL;
    if (!std::isfinite(q.price_in) || !std::isfinite(q.price_out) || !std::isfinite(q.priority)) return SIM_EINVAL;
  }
  const double lam = total_rate(c->cls, c->K);
  if (lam * (static_cast<double>(t->dt) * 1e-9) * (1.0 + std::fabs(c->mod_amp)) > 0.05) return SIM_EINVAL;
  const int lo = host_hbin(t->c0), hi = host_hbin(t->c0 + t->cpre * c->C + t->cdec * c->B);
  if (hi - lo + 1 > kMaxTbtBins) return SIM_EINVAL;
  // clocks are compared modulo 2^32 ns on the device: the longest iteration must stay far below 2^31 ns
  if (t->c0 + t->cpre * c->C + t->cdec * c->B > 2000000000ll) return SIM_EINVAL;
  // the per-server records of a replication stay on chip for a whole launch
  if (on_chip_bytes(*c, *t, c->M, max_reps) > kOnChipLimit) return SIM_EINVAL;
  return SIM_OK;
}

// Patience tables of the classes that have a rate (others zero-filled) and the calendar size they need:
// the power of two above the longest patience. Returns 0 entries when no class abandons, unless the weighted
// router is on: it needs the deadline rings (it marks the entries it takes out of a buffer as expired), so it
// gets the smallest calendars even when nobody abandons.
int patience_tables(const sim_config &c, const Ticks &t, std::vector<uint16_t> *tab, size_t *cal_entries)
{
  *cal_entries = 0;
  if (!any_patience(c) && c.route_mode != SIM_ROUTE_WEIGHTED_SPLIT) return SIM_OK;
  tab->assign(static_cast<size_t>(c.K) * kTableSize, 0);
  uint32_t longest = 1;
  for (int k = 0; k < c.K; ++k) {
    if (!(c.cls[k].theta > 0.0)) continue;
    uint16_t *out = tab->data() + static_cast<size_t>(k) * kTableSize;
    const int rc = build_patience_table(c.cls[k].theta, static_cast<double>(t.dt) * 1e-9, out);
    if (rc != SIM_OK) return rc;
    if (out[kTableSize - 1] > longest) longest = out[kTableSize - 1];
  }
  size_t n = 2;
  while (n <= longest) n <<= 1;
  *cal_entries = n;
  return SIM_OK;
}

// The workspace lives on the device that was current at sim_create: later calls must be made with it current.
bool on_device(const sim_t *h)
{
  int d = -1;
  return hipGetDevice(&d) == hipSuccess && d == h->device;
}

int sync(sim_t *, void *stream)
{
  return hipStreamSynchronize(static_cast<hipStream_t>(stream)) == hipSuccess ? SIM_OK : SIM_EHIP;
}

int copy_out(void *dst, const void *src, size_t bytes)
{
  return hipMemcpy(dst, src, bytes, hipMemcpyDeviceToHost) == hipSuccess ? SIM_OK : SIM_EHIP;
}

void drain_events(sim_t *h)
{
  for (auto &pr : h->pending) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, pr.first, pr.second) == hipSuccess) h->kernel_ms += ms;
    (void)hipEventDestroy(pr.first);
    (void)hipEventDestroy(pr.second);
  }
  h->pending.clear();
}

double ratio(double a, double b) { return b > 0.0 ? a / b : 0.0; }

double percentile(const uint64_t *hist, int pct)
{
  uint64_t n = 0;
  for (int b = 0; b < kNBin; ++b) n += hist[b];
  if (n == 0) return 0.0;
  const uint64_t rank = (n * static_cast<uint64_t>(pct) + 99) / 100;
  uint64_t cum = 0;
  for (int b = 0; b < kNBin; ++b) {
    cum += hist[b];
    if (cum >= rank) return static_cast<double>(host_hedge(b)) * 1e-9;
  }
  return static_cast<double>(host_hedge(kNBin - 1)) * 1e-9;
}

}  // namespace

namespace {
int create_in(const sim_config *cfg, int max_replications, void *dev_workspace, size_t bytes, sim_t **out);
}

extern "C" {

int sim_workspace_bytes(const sim_config *cfg, int max_replications, size_t *out_bytes)
{
  try {
    Ticks t;
    const int rc = validate(cfg, max_replications, &t);
    if (rc != SIM_OK || !out_bytes) return rc != SIM_OK ? rc : SIM_EINVAL;
    const int64_t rows = cfg->mod_period > 0 ? cfg->mod_period : 1;
    std::vector<uint16_t> pat;
    size_t cal_entries = 0;
    const int rp = patience_tables(*cfg, t, &pat, &cal_entries);
    if (rp != SIM_OK) return rp;
    *out_bytes = make_layout(*cfg, max_replications, rows, cal_entries).total;
    return SIM_OK;
  } catch (...) {   // host allocation failed (std::bad_alloc, std::length_error): nothing crosses the C boundary
    return SIM_ENOMEM;
  }
}

int sim_create(const sim_config *cfg, int max_replications, void *dev_workspace, size_t bytes, sim_t **out)
{
  return create_in(cfg, max_replications, dev_workspace, bytes, out);
}

int sim_create_static(const sim_config *cfg, int max_replications, sim_t **out)
{
  void *ws = nullptr;
  size_t bytes = 0;
  const int rc = static_workspace(&ws, &bytes);   // no allocation: the address of the library's own device array
  if (rc != SIM_OK) return rc;
  return create_in(cfg, max_replications, ws, bytes, out);
}

}  // extern "C"

namespace {
int create_in(const sim_config *cfg, int max_replications, void *dev_workspace, size_t bytes, sim_t **out)
{
  try {
    Ticks t;
    int rc = validate(cfg, max_replications, &t);
    if (rc != SIM_OK) return rc;
    if (!dev_workspace || !out || (reinterpret_cast<uintptr_t>(dev_workspace) & 255u)) return SIM_EINVAL;
    const int64_t rows = cfg->mod_period > 0 ? cfg->mod_period : 1;
    std::vector<uint16_t> pat;
    size_t cal_entries = 0;
    rc = patience_tables(*cfg, t, &pat, &cal_entries);
    if (rc != SIM_OK) return rc;
    const Layout L = make_layout(*cfg, max_replications, rows, cal_entries);
    if (bytes < L.total) return SIM_ENOMEM;
  
    sim_t *h = new (std::nothrow) sim_t();
    if (!h) return SIM_ENOMEM;
    std::unique_ptr<sim_t> hold(h);   // freed on every early return below, and if a host allocation throws
    h->cfg = *cfg;
    for (int k = 0; k < cfg->K; ++k) {
      h->cls[k] = cfg->cls[k];
      h->x_star[k] = cfg->x_star[k];
      h->qp_star[k] = cfg->qp_star[k];
    }
    const bool split = cfg->route_mode == SIM_ROUTE_RANDOM_SPLIT || cfg->route_mode == SIM_ROUTE_WEIGHTED_SPLIT;
    for (int k = 0; k < cfg->K; ++k) {
      h->p_solo[k] = split ? cfg->p_solo[k] : 1.0;
      h->w_solo[k] = cfg->route_mode == SIM_ROUTE_WEIGHTED_SPLIT ? cfg->w_solo[k] : 0.0;
      h->w_mixed[k] = cfg->route_mode == SIM_ROUTE_WEIGHTED_SPLIT ? cfg->w_mixed[k] : 0.0;
    }
    h->cfg.w_solo = h->w_solo; h->cfg.w_mixed = h->w_mixed;
    h->cfg.cls = h->cls; h->cfg.x_star = h->x_star; h->cfg.qp_star = h->qp_star; h->cfg.p_solo = h->p_solo;
    h->max_reps = max_replications;
    h->reps = 0; h->seed = 0; h->steps_done = 0; h->started = false;
    h->rows = rows;
    h->ws = static_cast<unsigned char *>(dev_workspace);
    h->ws_bytes = bytes;
    h->launches = 0; h->kernel_ms = 0.0;
    if (hipGetDevice(&h->device) != hipSuccess) return SIM_EHIP;
  
    // sampler tables
    std::vector<uint16_t> tab(static_cast<size_t>(cfg->K) * 2 * kTableSize);
    for (int k = 0; k < cfg->K; ++k) {
      const sim_class &q = cfg->cls[k];
      rc = build_length_table(q.in_law, q.in_p0, q.in_p1, q.in_table, &tab[(static_cast<size_t>(k) * 2 + 0) * kTableSize]);
      if (rc == SIM_OK)
        rc = build_length_table(q.out_law, q.out_p0, q.out_p1, q.out_table, &tab[(static_cast<size_t>(k) * 2 + 1) * kTableSize]);
      if (rc != SIM_OK) return rc;
      h->cls[k].in_table = h->cls[k].out_table = nullptr;
    }
    std::vector<uint32_t> arr(static_cast<size_t>(rows) * 3);
    const double lam = total_rate(cfg->cls, cfg->K);
    for (int64_t j = 0; j < rows; ++j) build_arrival_row(lam, t.dt, cfg->mod_amp, cfg->mod_period, j, &arr[3 * j]);
  
    Params &p = h->p;
    std::memset(&p, 0, sizeof p);
    p.K = cfg->K; p.N = cfg->N; p.B = cfg->B; p.C = cfg->C; p.M = cfg->M; p.R = max_replications;
    p.Mp = cfg->M;
    p.BS = (cfg->B + 3) & ~3;
    p.gate_mode = cfg->gate_mode;
    p.route_mode = cfg->route_mode;
    for (int k = 0; k < cfg->K; ++k) {
      p.solo_thr[k] = probability_threshold(h->p_solo[k]);
      p.wsel[0][k] = selection_weight_units(h->w_solo[k]);
      p.wsel[1][k] = selection_weight_units(h->w_mixed[k]);
    }
    p.tbt_lo = host_hbin(t.c0);
    p.tbt_w = host_hbin(t.c0 + t.cpre * cfg->C + t.cdec * cfg->B) - p.tbt_lo + 1;
    p.nwords = (cfg->N + 63) / 64;
    p.queue_cap = static_cast<uint32_t>(cfg->queue_cap);
    p.dbuf_cap = static_cast<uint32_t>(cfg->dbuf_cap);
    p.c0 = t.c0; p.cpre = t.cpre; p.cdec = t.cdec; p.dt = t.dt;
    p.mod_period = cfg->mod_period;
    for (int k = 0; k < cfg->K; ++k) {
      p.nx[k] = static_cast<double>(cfg->N) * cfg->x_star[k];
      p.invx[k] = cfg->x_star[k] > 0.0 ? 1.0 / cfg->x_star[k] : 0.0;
      p.xstar[k] = cfg->x_star[k];
      p.nq[k] = static_cast<double>(cfg->N) * cfg->qp_star[k];
      p.prio[k] = cfg->cls[k].priority;
    }
    build_class_thresholds(cfg->cls, cfg->K, p.cls_thr);
    unsigned char *w = h->ws;
    p.arr_thr = reinterpret_cast<uint32_t *>(w + L.arr_thr);
    p.len_tab = reinterpret_cast<uint16_t *>(w + L.len_tab);
    p.t_next = reinterpret_cast<int64_t *>(w + L.t_next);
    p.iter = reinterpret_cast<uint32_t *>(w + L.iter);
    p.remptok = reinterpret_cast<uint32_t *>(w + L.remptok);
    p.pf_job = reinterpret_cast<uint64_t *>(w + L.pf_job);
    p.n_cls = reinterpret_cast<uint64_t *>(w + L.n_cls);
    p.n_join = reinterpret_cast<uint64_t *>(w + L.n_join);
    p.fin = reinterpret_cast<uint32_t *>(w + L.fin);
    p.job = reinterpret_cast<uint64_t *>(w + L.job);
    p.qring = reinterpret_cast<uint32_t *>(w + L.qring);
    p.dring = reinterpret_cast<uint64_t *>(w + L.dring);
    p.cstate = reinterpret_cast<int32_t *>(w + L.cstate);
    p.tally = reinterpret_cast<uint64_t *>(w + L.tally);
    p.hist = reinterpret_cast<uint64_t *>(w + L.hist);
    p.digest = reinterpret_cast<uint64_t *>(w + L.digest);
    p.reduced = reinterpret_cast<uint64_t *>(w + L.reduced);
    if (split) p.dring_m = reinterpret_cast<uint64_t *>(w + L.dring_m);
    if (cal_entries) {
      for (int k = 0; k < cfg->K; ++k)
        if (cfg->cls[k].theta > 0.0) p.ab_classes |= 1u << k;
      p.cal_mask = static_cast<uint32_t>(cal_entries - 1);
      p.pat_tab = reinterpret_cast<uint16_t *>(w + L.pat_tab);
      p.qdl = reinterpret_cast<uint32_t *>(w + L.qdl);
      p.ddl = reinterpret_cast<uint32_t *>(w + L.ddl);
      p.cal = reinterpret_cast<uint32_t *>(w + L.cal);
      p.dcal = reinterpret_cast<uint32_t *>(w + L.dcal);
      p.dl_rings = 1;
      if (split) {
        p.ddl_m = reinterpret_cast<uint32_t *>(w + L.ddl_m);
        p.dcal_m = reinterpret_cast<uint32_t *>(w + L.dcal_m);
      }
    }
  
    p.self = reinterpret_cast<const Params *>(w + L.params);
    h->threads = step_threads(p, max_replications);
    p.threads = h->threads;
    h->lds_bytes = step_lds_bytes(p);
    if (h->lds_bytes > kOnChipLimit) return SIM_EINVAL;
    if (hipMemcpy(w + L.arr_thr, arr.data(), arr.size() * sizeof(uint32_t), hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(w + L.len_tab, tab.data(), tab.size() * sizeof(uint16_t), hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(w + L.params, &p, sizeof(Params), hipMemcpyHostToDevice) != hipSuccess ||
        (cal_entries &&
         hipMemcpy(w + L.pat_tab, pat.data(), pat.size() * sizeof(uint16_t), hipMemcpyHostToDevice) != hipSuccess)) {
      return SIM_EHIP;
    }
    *out = hold.release();
    return SIM_OK;
  } catch (...) {   // host allocation failed (std::bad_alloc, std::length_error): nothing crosses the C boundary
    return SIM_ENOMEM;
  }
}

}  // namespace

extern "C" {

int sim_run(sim_t *h, int64_t steps, int replications, uint64_t seed, void *hip_stream)
{
  try {
    if (!h || steps < 0 || replications < 1 || replications > h->max_reps || !on_device(h)) return SIM_EINVAL;
    if (!h->started || replications != h->reps || seed != h->seed) {
      const int rc = launch_reset(h->p, h->max_reps, hip_stream);
      if (rc != SIM_OK) return rc;
      h->reps = replications; h->seed = seed; h->steps_done = 0; h->started = true;
      h->p.key0 = static_cast<uint32_t>(seed);
      h->p.key1 = static_cast<uint32_t>(seed >> 32);
    }
    if (steps >= (int64_t(1) << 29) - h->steps_done) return SIM_EINVAL;   // (written so that no sum can overflow)
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    int64_t left = steps;
    while (left > 0) {
      const uint32_t n = static_cast<uint32_t>(left < kStepsPerLaunch ? left : kStepsPerLaunch);
      hipEvent_t e0 = nullptr, e1 = nullptr;
      bool timed = hipEventCreate(&e0) == hipSuccess;
      if (timed && hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); timed = false; }
      if (timed) (void)hipEventRecord(e0, st);
      const int rc = launch_steps(h->p, replications, h->threads, h->lds_bytes, static_cast<uint32_t>(h->steps_done), n, hip_stream);
      if (timed) { (void)hipEventRecord(e1, st); h->pending.emplace_back(e0, e1); }
      if (rc != SIM_OK) return rc;
      h->launches += 1;
      h->steps_done += n;
      left -= n;
      if (h->pending.size() >= 64) {   // bound the number of live events
        if (hipStreamSynchronize(st) != hipSuccess) return SIM_EHIP;
        drain_events(h);
      }
    }
    return SIM_OK;
  } catch (...) {   // host allocation failed (std::bad_alloc, std::length_error): nothing crosses the C boundary
    return SIM_ENOMEM;
  }
}

int sim_set_targets(sim_t *h, const double *x_star, const double *qp_star, void *hip_stream)
{
  if (!h || !x_star || !qp_star || !on_device(h)) return SIM_EINVAL;
  for (int k = 0; k < h->p.K; ++k)
    if (!(x_star[k] >= 0.0) || !std::isfinite(x_star[k]) || !std::isfinite(qp_star[k])) return SIM_EINVAL;
  for (int k = 0; k < h->p.K; ++k) {
    h->p.nx[k] = static_cast<double>(h->p.N) * x_star[k];
    h->p.invx[k] = x_star[k] > 0.0 ? 1.0 / x_star[k] : 0.0;
    h->p.xstar[k] = x_star[k];
    h->p.nq[k] = static_cast<double>(h->p.N) * qp_star[k];
  }
  // the step kernel reads its parameters from the device copy; stream order puts the update after earlier runs
  // (the source is pageable host memory: the call returns once the bytes have been staged)
  if (hipMemcpyAsync(const_cast<Params *>(h->p.self), &h->p, sizeof(Params), hipMemcpyHostToDevice,
                     static_cast<hipStream_t>(hip_stream)) != hipSuccess)
    return SIM_EHIP;
  return SIM_OK;
}

int sim_set_split(sim_t *h, int M, void *hip_stream)
{
  if (!h || M < 0 || M > h->p.N || !on_device(h)) return SIM_EINVAL;
  Params q = h->p;
  q.M = M;
  if (M > q.Mp) q.Mp = M;   // never lowered: a server that turns solo may still hold a prefill
  const size_t lds = step_lds_bytes(q);
  if (lds > kOnChipLimit) return SIM_EINVAL;
  h->p = q;
  h->cfg.M = M;
  h->lds_bytes = lds;
  if (hipMemcpyAsync(const_cast<Params *>(h->p.self), &h->p, sizeof(Params), hipMemcpyHostToDevice,
                     static_cast<hipStream_t>(hip_stream)) != hipSuccess)
    return SIM_EHIP;
  return SIM_OK;
}

int sim_kernel_time(sim_t *h, int64_t *launches, double *milliseconds, int reset, void *hip_stream)
{
  try {
    if (!h || !on_device(h)) return SIM_EINVAL;
    const int rc = sync(h, hip_stream);
    if (rc != SIM_OK) return rc;
    drain_events(h);
    if (launches) *launches = h->launches;
    if (milliseconds) *milliseconds = h->kernel_ms;
    if (reset) { h->launches = 0; h->kernel_ms = 0.0; }
    return SIM_OK;
  } catch (...) {   // host allocation failed (std::bad_alloc, std::length_error): nothing crosses the C boundary
    return SIM_ENOMEM;
  }
}

int sim_launch_shape(sim_t *h, int *threads, size_t *lds_bytes)
{
  if (!h) return SIM_EINVAL;
  if (threads) *threads = h->threads;
  if (lds_bytes) *lds_bytes = h->lds_bytes;
  return SIM_OK;
}

int sim_stats(sim_t *h, sim_stats_t *st, void *hip_stream)
{
  try {
    if (!h || !st || !h->started || !on_device(h)) return SIM_EINVAL;
    int rc = launch_reduce(h->p, h->reps, hip_stream);
    if (rc != SIM_OK) return rc;
    rc = sync(h, hip_stream);
    if (rc != SIM_OK) return rc;
    const int K = h->cfg.K;
    const size_t nh = static_cast<size_t>(3) * K * kNBin;
    std::vector<uint64_t> red(kTallyWords + nh);
    rc = copy_out(red.data(), h->p.reduced, red.size() * sizeof(uint64_t));
    if (rc != SIM_OK) return rc;
  
    std::memset(st, 0, sizeof *st);
    st->K = K; st->replications = h->reps; st->steps = h->steps_done;
    const double dts = static_cast<double>(h->p.dt) * 1e-9;
    st->sim_time = static_cast<double>(h->steps_done) * dts;
    for (int k = 0; k < K; ++k)
      for (int t = 0; t < kNTally; ++t) st->tally[k][t] = red[static_cast<size_t>(k) * kNTally + t];
    for (int t = 0; t < kNGlobal; ++t) st->glob[t] = red[static_cast<size_t>(kMaxK) * kNTally + t];
    const uint64_t *hs = red.data() + kTallyWords;
    const double server_time = static_cast<double>(h->cfg.N) * st->sim_time * static_cast<double>(h->reps);
    const double server_steps = static_cast<double>(h->cfg.N) * static_cast<double>(h->steps_done) * static_cast<double>(h->reps);
    double xlo = 0, xhi = 0, ylo = 0, yhi = 0, slo = 0;
    for (int k = 0; k < K; ++k) {
      const uint64_t *t = st->tally[k];
      const sim_class &q = h->cls[k];
      const double done = static_cast<double>(t[SIM_T_S_DM] + t[SIM_T_S_DS]);
      st->arrival_rate[k] = ratio(static_cast<double>(t[SIM_T_A]), server_time);
      st->completion_rate[k] = ratio(done, server_time);
      st->served_fraction[k] = ratio(done, static_cast<double>(t[SIM_T_A]));
      st->tok_rate_prefill[k] = ratio(static_cast<double>(t[SIM_T_TOK_PREF]), server_time);
      st->tok_rate_decode[k] = ratio(static_cast<double>(t[SIM_T_TOK_EMIT]), server_time);
      // bundled: prompt and output tokens recognised when the request completes;
      // separate: prompt tokens at prefill completion, output tokens at decode completion
      const double bundled = q.price_in * static_cast<double>(t[SIM_T_TOKP_DEC]) + q.price_out * static_cast<double>(t[SIM_T_TOKD_DEC]);
      const double separate = q.price_in * static_cast<double>(t[SIM_T_TOKP_PRE]) + q.price_out * static_cast<double>(t[SIM_T_TOKD_DEC]);
      st->rev_bundled[k] = ratio(bundled, server_time);
      st->rev_separate[k] = ratio(separate, server_time);
      st->rev_mixed[k] = q.bundled ? st->rev_bundled[k] : st->rev_separate[k];
      st->rev_bundled_total += st->rev_bundled[k];
      st->rev_separate_total += st->rev_separate[k];
      st->rev_mixed_total += st->rev_mixed[k];
      st->mean_qp[k] = ratio(static_cast<double>(t[SIM_T_SUM_QP]), server_steps);
      st->mean_qd[k] = ratio(static_cast<double>(t[SIM_T_SUM_QD]), server_steps);
      st->mean_x[k] = ratio(static_cast<double>(t[SIM_T_SUM_X]), server_steps);
      st->mean_ym[k] = ratio(static_cast<double>(t[SIM_T_SUM_YM]), server_steps);
      st->mean_ys[k] = ratio(static_cast<double>(t[SIM_T_SUM_YS]), server_steps);
      st->ttft_mean[k] = ratio(static_cast<double>(t[SIM_T_TTFT_SUM]) * 1e-9, static_cast<double>(t[SIM_T_S_P]));
      st->e2e_mean[k] = ratio(static_cast<double>(t[SIM_T_E2E_SUM]) * 1e-9, done);
      st->tbt_mean[k] = ratio(static_cast<double>(t[SIM_T_TBT_SUM]) * 1e-9, static_cast<double>(t[SIM_T_TOK_EMIT]));
      st->abandon_rate_p[k] = ratio(static_cast<double>(t[SIM_T_AB_P]), server_time);
      st->abandon_rate_d[k] = ratio(static_cast<double>(t[SIM_T_AB_D]), server_time);
      st->mean_wait[k] = ratio(static_cast<double>(t[SIM_T_WAIT_STEPS]) * dts, static_cast<double>(t[SIM_T_U_P]));
      const uint64_t *h0 = hs + (static_cast<size_t>(0) * K + k) * kNBin;
      const uint64_t *h1 = hs + (static_cast<size_t>(1) * K + k) * kNBin;
      const uint64_t *h2 = hs + (static_cast<size_t>(2) * K + k) * kNBin;
      st->ttft_p50[k] = percentile(h0, 50); st->ttft_p95[k] = percentile(h0, 95); st->ttft_p99[k] = percentile(h0, 99);
      st->e2e_p50[k] = percentile(h1, 50); st->e2e_p95[k] = percentile(h1, 95); st->e2e_p99[k] = percentile(h1, 99);
      st->tbt_p50[k] = percentile(h2, 50); st->tbt_p95[k] = percentile(h2, 95); st->tbt_p99[k] = percentile(h2, 99);
      if (k == 0 || st->mean_x[k] < xlo) xlo = st->mean_x[k];
      if (k == 0 || st->mean_x[k] > xhi) xhi = st->mean_x[k];
      if (k == 0 || st->mean_ys[k] < ylo) ylo = st->mean_ys[k];
      if (k == 0 || st->mean_ys[k] > yhi) yhi = st->mean_ys[k];
      if (k == 0 || st->served_fraction[k] < slo) slo = st->served_fraction[k];
    }
    st->fair_gap_x = xhi - xlo;
    st->fair_gap_ys = yhi - ylo;
    st->fair_min_served = slo;
    st->util_mix = ratio(static_cast<double>(st->glob[SIM_G_BUSY_MIX]) * 1e-9, server_time);
    st->util_solo = ratio(static_cast<double>(st->glob[SIM_G_BUSY_SOLO]) * 1e-9, server_time);
    st->iter_rate = ratio(static_cast<double>(st->glob[SIM_G_ITERS_MIX] + st->glob[SIM_G_ITERS_SOLO]), server_time);
    return st->glob[SIM_G_OVERFLOW] ? SIM_EOVERFLOW : SIM_OK;
  } catch (...) {   // host allocation failed (std::bad_alloc, std::length_error): nothing crosses the C boundary
    return SIM_ENOMEM;
  }
}

int sim_tallies(sim_t *h, int r, uint64_t *out, void *hip_stream)
{
  try {
    if (!h || !out || !h->started || r < 0 || r >= h->reps || !on_device(h)) return SIM_EINVAL;
    int rc = sync(h, hip_stream);
    if (rc != SIM_OK) return rc;
    std::vector<uint64_t> buf(kTallyWords);
    rc = copy_out(buf.data(), h->p.tally + static_cast<size_t>(r) * kTallyWords, buf.size() * sizeof(uint64_t));
    if (rc != SIM_OK) return rc;
    const int K = h->cfg.K;
    for (int k = 0; k < K; ++k)
      for (int t = 0; t < kNTally; ++t) out[k * kNTally + t] = buf[static_cast<size_t>(k) * kNTally + t];
    for (int t = 0; t < kNGlobal; ++t) out[K * kNTally + t] = buf[static_cast<size_t>(kMaxK) * kNTally + t];
    return SIM_OK;
  } catch (...) {   // host allocation failed (std::bad_alloc, std::length_error): nothing crosses the C boundary
    return SIM_ENOMEM;
  }
}

int sim_hist(sim_t *h, int r, int which, uint64_t *out, void *hip_stream)
{
  if (!h || !out || !h->started || r < 0 || r >= h->reps || which < 0 || which > 2 || !on_device(h)) return SIM_EINVAL;
  const int rc = sync(h, hip_stream);
  if (rc != SIM_OK) return rc;
  const int K = h->cfg.K;
  return copy_out(out, h->p.hist + (static_cast<size_t>(r) * 3 + which) * K * kNBin, static_cast<size_t>(K) * kNBin * sizeof(uint64_t));
}

int sim_digest(sim_t *h, int r, uint64_t *out, void *hip_stream)
{
  if (!h || !out || !h->started || r < 0 || r >= h->reps || !on_device(h)) return SIM_EINVAL;
  int rc = launch_digest(h->p, h->reps, hip_stream);
  if (rc != SIM_OK) return rc;
  rc = sync(h, hip_stream);
  if (rc != SIM_OK) return rc;
  return copy_out(out, h->p.digest + r, sizeof(uint64_t));
}

int sim_snapshot(sim_t *h, int r, sim_state_t *out, void *hip_stream)
{
  try {
    if (!h || !out || !h->started || r < 0 || r >= h->reps || !on_device(h)) return SIM_EINVAL;
    int rc = sync(h, hip_stream);
    if (rc != SIM_OK) return rc;
    const int K = h->cfg.K, N = h->cfg.N, B = h->cfg.B;
    const size_t base = static_cast<size_t>(r) * N;
    const Params &p = h->p;
    int32_t cs[CS_WORDS];
    rc = copy_out(cs, p.cstate + static_cast<size_t>(r) * CS_WORDS, sizeof cs);
    if (rc != SIM_OK) return rc;
    if (out->class_state)
      for (int k = 0; k < K; ++k) {
        out->class_state[0 * K + k] = cs[CS_QP + k]; out->class_state[1 * K + k] = cs[CS_X + k];
        out->class_state[2 * K + k] = cs[CS_QD + k]; out->class_state[3 * K + k] = cs[CS_YM + k];
        out->class_state[4 * K + k] = cs[CS_YS + k];
      }
    if (out->t_next && (rc = copy_out(out->t_next, p.t_next + base, N * sizeof(int64_t))) != SIM_OK) return rc;
    if (out->iter && (rc = copy_out(out->iter, p.iter + base, N * sizeof(uint32_t))) != SIM_OK) return rc;
    std::vector<uint32_t> pk(N);
    std::vector<uint64_t> nc(N), nj(N), pj(N);
    if ((rc = copy_out(pk.data(), p.remptok + base, N * sizeof(uint32_t))) != SIM_OK) return rc;
    if ((rc = copy_out(nc.data(), p.n_cls + base, N * sizeof(uint64_t))) != SIM_OK) return rc;
    if ((rc = copy_out(nj.data(), p.n_join + base, N * sizeof(uint64_t))) != SIM_OK) return rc;
    if ((rc = copy_out(pj.data(), p.pf_job + base, N * sizeof(uint64_t))) != SIM_OK) return rc;
    for (int g = 0; g < N; ++g) {
      const int rem = static_cast<int>(pk[g] & 0xFFFFu);
      if (out->rem) out->rem[g] = rem;
      if (out->ptok) out->ptok[g] = static_cast<int>((pk[g] >> 16) & 0x1FFFu);
      if (out->pfjob) out->pfjob[g] = rem ? pj[g] : 0;
      int nd = 0;
      for (int k = 0; k < kMaxK; ++k) {
        const uint8_t c = static_cast<uint8_t>(nc[g] >> (8 * k));
        if (out->n_cls) out->n_cls[g * kMaxK + k] = c;
        if (out->n_join) out->n_join[g * kMaxK + k] = static_cast<uint8_t>(nj[g] >> (8 * k));
        nd += c;
      }
      if (out->n_dec) out->n_dec[g] = nd;
    }
    if (out->fin || out->job) {
      const size_t BS = static_cast<size_t>(p.BS);
      std::vector<uint32_t> f(static_cast<size_t>(N) * BS);
      std::vector<uint64_t> j(static_cast<size_t>(N) * BS);
      if ((rc = copy_out(f.data(), p.fin + base * BS, f.size() * sizeof(uint32_t))) != SIM_OK) return rc;
      if ((rc = copy_out(j.data(), p.job + base * BS, j.size() * sizeof(uint64_t))) != SIM_OK) return rc;
      for (int g = 0; g < N; ++g) {
        int nd = 0;
        for (int k = 0; k < kMaxK; ++k) nd += static_cast<uint8_t>(nc[g] >> (8 * k));
        for (int s = 0; s < B; ++s) {
          const size_t i = static_cast<size_t>(g) * B + s, d = static_cast<size_t>(g) * BS + s;
          if (out->fin) out->fin[i] = s < nd ? f[d] : 0;
          if (out->job) out->job[i] = s < nd ? j[d] : 0;
        }
      }
    }
    for (int k = 0; k < K; ++k) {
      const int64_t len = cs[CS_QP + k];
      out->queue_len[k] = len;
      if (!out->queue[k] || len == 0) continue;
      std::vector<uint32_t> ring(h->p.queue_cap);
      rc = copy_out(ring.data(), p.qring + (static_cast<size_t>(r) * K + k) * p.queue_cap, ring.size() * sizeof(uint32_t));
      if (rc != SIM_OK) return rc;
      for (int64_t i = 0; i < len; ++i) out->queue[k][i] = ring[(static_cast<uint32_t>(cs[CS_QHEAD + k]) + i) % p.queue_cap];
      if (!out->queue_dl[k]) continue;
      if (p.ab_classes) {
        rc = copy_out(ring.data(), p.qdl + (static_cast<size_t>(r) * K + k) * p.queue_cap, ring.size() * sizeof(uint32_t));
        if (rc != SIM_OK) return rc;
      }
      for (int64_t i = 0; i < len; ++i)
        out->queue_dl[k][i] = p.ab_classes ? ring[(static_cast<uint32_t>(cs[CS_QHEAD + k]) + i) % p.queue_cap] : kNever;
    }
    out->dbuf_len = cs[CS_DCOUNT];
    if (out->dbuf && cs[CS_DCOUNT] > 0) {
      std::vector<uint64_t> ring(p.dbuf_cap);
      rc = copy_out(ring.data(), p.dring + static_cast<size_t>(r) * p.dbuf_cap, ring.size() * sizeof(uint64_t));
      if (rc != SIM_OK) return rc;
      for (int64_t i = 0; i < cs[CS_DCOUNT]; ++i) out->dbuf[i] = ring[(static_cast<uint32_t>(cs[CS_DHEAD]) + i) % p.dbuf_cap];
    }
    out->dbuf_m_len = (p.route_mode == SIM_ROUTE_RANDOM_SPLIT || p.route_mode == SIM_ROUTE_WEIGHTED_SPLIT) ? cs[CS_DCOUNT_M] : 0;
    if (out->dbuf_m && out->dbuf_m_len > 0) {
      std::vector<uint64_t> ring(p.dbuf_cap);
      rc = copy_out(ring.data(), p.dring_m + static_cast<size_t>(r) * p.dbuf_cap, ring.size() * sizeof(uint64_t));
      if (rc != SIM_OK) return rc;
      for (int64_t i = 0; i < out->dbuf_m_len; ++i) out->dbuf_m[i] = ring[(static_cast<uint32_t>(cs[CS_DHEAD_M]) + i) % p.dbuf_cap];
    }
    if (out->dbuf_dl && cs[CS_DCOUNT] > 0) {
      std::vector<uint32_t> ring(p.dbuf_cap, kNever);
      if (p.ab_classes) {
        rc = copy_out(ring.data(), p.ddl + static_cast<size_t>(r) * p.dbuf_cap, ring.size() * sizeof(uint32_t));
        if (rc != SIM_OK) return rc;
      }
      for (int64_t i = 0; i < cs[CS_DCOUNT]; ++i) out->dbuf_dl[i] = ring[(static_cast<uint32_t>(cs[CS_DHEAD]) + i) % p.dbuf_cap];
    }
    return SIM_OK;
  } catch (...) {   // host allocation failed (std::bad_alloc, std::length_error): nothing crosses the C boundary
    return SIM_ENOMEM;
  }
}

int sim_destroy(sim_t *h)
{
  if (!h) return SIM_EINVAL;
  for (auto &pr : h->pending) { (void)hipEventDestroy(pr.first); (void)hipEventDestroy(pr.second); }
  delete h;
  return SIM_OK;
}

const char *sim_strerror(int err)
{
  switch (err) {
    case SIM_OK: return "ok";
    case SIM_EINVAL: return "invalid argument or configuration";
    case SIM_ENOMEM: return "workspace too small (the static workspace holds 32 MiB) or out of host memory";
    case SIM_EHIP: return "HIP runtime error";
    case SIM_EOVERFLOW: return "a prefill queue or the decode buffer overflowed; requests were dropped";
    default: return "unknown error";
  }
}

int sim_length_table(int law, double p0, double p1, uint16_t *out)
{
  if (!out || law == SIM_TABLE) return SIM_EINVAL;
  return build_length_table(law, p0, p1, nullptr, out);
}

int sim_patience_table(double theta, double dt, uint16_t *out)
{
  if (!out) return SIM_EINVAL;
  return build_patience_table(theta, dt, out);
}

int sim_philox(uint64_t seed, uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t *out4)
{
  if (!out4) return SIM_EINVAL;
  uint32_t k0 = static_cast<uint32_t>(seed), k1 = static_cast<uint32_t>(seed >> 32);
  for (int round = 0; round < 10; ++round) {
    const uint64_t a = static_cast<uint64_t>(0xD2511F53u) * c0;
    const uint64_t b = static_cast<uint64_t>(0xCD9E8D57u) * c2;
    const uint32_t n0 = static_cast<uint32_t>(b >> 32) ^ c1 ^ k0;
    const uint32_t n2 = static_cast<uint32_t>(a >> 32) ^ c3 ^ k1;
    c1 = static_cast<uint32_t>(b); c3 = static_cast<uint32_t>(a); c0 = n0; c2 = n2;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
  out4[0] = c0; out4[1] = c1; out4[2] = c2; out4[3] = c3;
  return SIM_OK;
}

int sim_thresholds(const sim_config *cfg, int64_t rows, uint32_t *arr_thr, uint32_t *cls_thr)
{
  try {
    Ticks t;
    const int rc = validate(cfg, 1, &t);
    if (rc != SIM_OK) return rc;
    const double lam = total_rate(cfg->cls, cfg->K);
    if (arr_thr)
      for (int64_t j = 0; j < rows; ++j) build_arrival_row(lam, t.dt, cfg->mod_amp, cfg->mod_period, j, arr_thr + 3 * j);
    if (cls_thr) build_class_thresholds(cfg->cls, cfg->K, cls_thr);
    return SIM_OK;
  } catch (...) {   // host allocation failed (std::bad_alloc, std::length_error): nothing crosses the C boundary
    return SIM_ENOMEM;
  }
}

int sim_onchip_bytes(const sim_config *cfg, size_t *out_bytes, size_t *out_limit)
{
  Ticks t;
  if (!cfg || !out_bytes || !cfg->cls || cfg->K < 1 || cfg->K > kMaxK || cfg->N < 1 || cfg->N > kMaxN || cfg->M < 0 ||
      cfg->M > cfg->N || cfg->B < 1 || cfg->B > kMaxB || cfg->C < 1 || cfg->C > kMaxChunk || !(cfg->c0 > 0.0) ||
      !(cfg->c_pre >= 0.0) || !(cfg->c_dec >= 0.0))
    return SIM_EINVAL;
  t.c0 = std::llround(cfg->c0 * 1e9); t.cpre = std::llround(cfg->c_pre * 1e9); t.cdec = std::llround(cfg->c_dec * 1e9);
  t.dt = t.c0;
  *out_bytes = on_chip_bytes(*cfg, t, cfg->M, 1);
  if (out_limit) *out_limit = kOnChipLimit;
  return SIM_OK;
}

int sim_launch_plan(const sim_config *cfg, int replications, int *threads, size_t *lds_bytes, int *waves_per_simd)
{
  try {
    Ticks t;
    const int rc = validate(cfg, replications, &t);
    if (rc != SIM_OK) return rc;
    const Params q = shape_params(*cfg, t, cfg->M, replications);
    const size_t lds = step_lds_bytes(q);
    if (threads) *threads = q.threads;
    if (lds_bytes) *lds_bytes = lds;
    if (waves_per_simd) *waves_per_simd = q.threads > 512 || step_dense(replications, q.threads, lds) ? 4 : 2;
    return SIM_OK;
  } catch (...) {
    return SIM_ENOMEM;
  }
}

int sim_abi_sizes(size_t *out4)
{
  if (!out4) return SIM_EINVAL;
  out4[0] = sizeof(sim_class); out4[1] = sizeof(sim_config); out4[2] = sizeof(sim_stats_t); out4[3] = sizeof(sim_state_t);
  return SIM_OK;
}

}  // extern "C"
