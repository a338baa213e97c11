// Test driver (CPU only): calls the host side of the simulator's C ABI - configuration checks, workspace layout,
// sampler and threshold tables, launch plans, error paths - in a build whose host code carries AddressSanitizer and
// the undefined-behaviour checks; any finding aborts the process. No kernel is launched and no device memory is
// touched: without a GPU the calls that need one return SIM_EHIP, which is checked as such.
#include <cmath>
#include <cstdio>
#include <cstring>
#include <vector>

#include "gnr_sim.h"

static int failures = 0;
#define EXPECT(cond)                                                      \
  do {                                                                    \
    if (!(cond)) { std::printf("line %d: %s\n", __LINE__, #cond); ++failures; } \
  } while (0)

struct Case {
  sim_class cls[SIM_MAXK];
  double x_star[SIM_MAXK], qp_star[SIM_MAXK], p_solo[SIM_MAXK], w_solo[SIM_MAXK], w_mixed[SIM_MAXK];
  sim_config cfg;
};

// K classes with alternating length laws, N servers, B slots; everything else as in the small reference instance.
static void make_case(Case *c, int K, int N, int B, int M)
{
  std::memset(c, 0, sizeof *c);
  for (int k = 0; k < K; ++k) {
    sim_class &q = c->cls[k];
    q.lambda = 0.4 / K;
    q.in_law = k % 3 == 0 ? SIM_GEOMETRIC : k % 3 == 1 ? SIM_LOGNORMAL : SIM_CONST;
    q.in_p0 = 100.0 + 300.0 * k; q.in_p1 = 0.8;
    q.out_law = k % 2 ? SIM_GEOMETRIC : SIM_LOGNORMAL;
    q.out_p0 = 40.0 + 100.0 * k; q.out_p1 = 1.0;
    q.price_in = 1.0; q.price_out = 2.0; q.bundled = k & 1; q.priority = 0.1 * k;
    c->x_star[k] = 0.02; c->qp_star[k] = 0.1 * k;
    c->p_solo[k] = 0.5; c->w_solo[k] = 1.0 / K; c->w_mixed[k] = 1.0 / K;
  }
  sim_config &g = c->cfg;
  g.K = K; g.N = N; g.B = B; g.C = 256;
  g.c0 = 0.010; g.c_pre = 0.00005; g.c_dec = 0.0002; g.dt = 0.0;
  g.cls = c->cls; g.M = M; g.x_star = c->x_star; g.qp_star = c->qp_star;
  g.gate_mode = SIM_GATE_OCCUPANCY; g.route_mode = SIM_ROUTE_SOLO_FIRST;
  g.queue_cap = 4096; g.dbuf_cap = 4096;
  g.p_solo = c->p_solo; g.w_solo = c->w_solo; g.w_mixed = c->w_mixed;
}

static void host_calls(const sim_config *g)
{
  size_t bytes = 0, lds = 0, limit = 0;
  size_t last = 0;
  for (int R : {1, 16, 1024, SIM_MAXR}) {
    EXPECT(sim_workspace_bytes(g, R, &bytes) == SIM_OK);
    EXPECT(bytes > last);
    last = bytes;
  }
  EXPECT(sim_workspace_bytes(g, SIM_MAXR + 1, &bytes) == SIM_EINVAL);
  EXPECT(sim_workspace_bytes(g, 0, &bytes) == SIM_EINVAL);
  EXPECT(sim_onchip_bytes(g, &lds, &limit) == SIM_OK && lds > 0 && lds <= limit);
  for (int R : {1, 200, 256, 1024, 2048, 100000}) {
    int threads = 0, per_simd = 0;
    EXPECT(sim_launch_plan(g, R, &threads, &lds, &per_simd) == SIM_OK);
    EXPECT(threads >= 64 && threads <= 1024 && (threads & (threads - 1)) == 0 && lds <= limit && (per_simd == 2 || per_simd == 4));
  }
  std::vector<uint32_t> arr(3 * 64), cth(SIM_MAXK);
  EXPECT(sim_thresholds(g, 64, arr.data(), cth.data()) == SIM_OK);
  EXPECT(arr[0] <= arr[1] && arr[1] <= arr[2]);
  // a handle cannot be made without a device workspace, nor in one that is too small (checked before any device call)
  sim_t *h = nullptr;
  EXPECT(sim_create(g, 4, nullptr, 1u << 30, &h) == SIM_EINVAL && h == nullptr);
  EXPECT(sim_create(g, 4, reinterpret_cast<void *>(uintptr_t(256)), 1, &h) == SIM_ENOMEM && h == nullptr);
  EXPECT(sim_create(g, 4, reinterpret_cast<void *>(uintptr_t(257)), 1u << 30, &h) == SIM_EINVAL && h == nullptr);
}

int main()
{
  size_t sizes[4];
  EXPECT(sim_abi_sizes(sizes) == SIM_OK && sizes[0] == sizeof(sim_class) && sizes[1] == sizeof(sim_config));
  for (int e = 0; e >= -5; --e) EXPECT(sim_strerror(e) != nullptr && std::strlen(sim_strerror(e)) > 0);

  uint32_t w[4];
  EXPECT(sim_philox(0x123456789abcdef0ull, 1, 2, 3, 4, w) == SIM_OK);
  EXPECT(sim_philox(1, 0, 0, 0, 0, nullptr) == SIM_EINVAL);

  std::vector<uint16_t> tab(65536);
  const double means[] = {1.0, 1.5, 64.0, 512.0, 8192.0, 32768.0, 1e6};
  for (double m : means) {
    EXPECT(sim_length_table(SIM_GEOMETRIC, m, 0.0, tab.data()) == SIM_OK);
    EXPECT(tab[0] >= 1 && tab[65535] <= 32768 && tab[0] <= tab[65535]);
    EXPECT(sim_length_table(SIM_LOGNORMAL, m, 0.8, tab.data()) == SIM_OK);
    EXPECT(sim_length_table(SIM_LOGNORMAL, m, 3.5, tab.data()) == SIM_OK);
    EXPECT(tab[0] >= 1 && tab[65535] <= 32768);
  }
  EXPECT(sim_length_table(SIM_CONST, 513.0, 0.0, tab.data()) == SIM_OK && tab[0] == 513 && tab[65535] == 513);
  EXPECT(sim_length_table(SIM_TABLE, 1.0, 0.0, tab.data()) == SIM_EINVAL);
  EXPECT(sim_length_table(SIM_GEOMETRIC, 0.5, 0.0, tab.data()) == SIM_OK && tab[65535] == 1);   // a mean of at most 1: always 1
  EXPECT(sim_length_table(SIM_GEOMETRIC, -3.0, 0.0, tab.data()) == SIM_EINVAL);
  EXPECT(sim_length_table(SIM_GEOMETRIC, std::nan(""), 0.0, tab.data()) == SIM_EINVAL);
  EXPECT(sim_length_table(SIM_LOGNORMAL, 100.0, 0.0, tab.data()) == SIM_EINVAL);
  EXPECT(sim_length_table(SIM_GEOMETRIC, 10.0, 0.0, nullptr) == SIM_EINVAL);
  const double thetas[] = {1e-3, 0.1, 4.0, 25.0, 1e4};
  for (double th : thetas) {
    const int rc = sim_patience_table(th, 0.010, tab.data());
    EXPECT(rc == SIM_OK || rc == SIM_EINVAL);
    if (rc == SIM_OK) EXPECT(tab[0] <= tab[65535]);
  }
  EXPECT(sim_patience_table(0.1, 0.010, nullptr) == SIM_EINVAL);

  Case c;
  make_case(&c, 2, 8, 32, 1);            host_calls(&c.cfg);
  make_case(&c, 4, 1024, 64, 300);       host_calls(&c.cfg);
  make_case(&c, 8, 2048, 64, 700);       host_calls(&c.cfg);
  make_case(&c, 6, 10000, 128, 2377);    c.cfg.mod_amp = 0.5; c.cfg.mod_period = 100000; host_calls(&c.cfg);
  make_case(&c, 1, 1, 1, 0);             host_calls(&c.cfg);
  make_case(&c, 3, 300, 7, 300);         c.cfg.route_mode = SIM_ROUTE_IMMEDIATE; host_calls(&c.cfg);
  make_case(&c, 6, 5000, 128, 1000);     c.cfg.route_mode = SIM_ROUTE_RANDOM_SPLIT; c.cls[2].theta = 0.1; host_calls(&c.cfg);
  make_case(&c, 6, 10000, 128, 2377);    c.cfg.route_mode = SIM_ROUTE_WEIGHTED_SPLIT; c.cls[0].theta = 4.0; host_calls(&c.cfg);

  // what the checks refuse
  size_t bytes = 0;
  make_case(&c, 2, 8, 32, 1);
  const sim_config good = c.cfg;
  auto refused = [&](sim_config g) { return sim_workspace_bytes(&g, 16, &bytes) == SIM_EINVAL; };
  { sim_config g = good; g.K = 0; EXPECT(refused(g)); }
  { sim_config g = good; g.K = SIM_MAXK + 1; EXPECT(refused(g)); }
  { sim_config g = good; g.N = SIM_MAXN + 1; EXPECT(refused(g)); }
  { sim_config g = good; g.B = SIM_MAXB + 1; EXPECT(refused(g)); }
  { sim_config g = good; g.M = 9; EXPECT(refused(g)); }
  { sim_config g = good; g.C = 0; EXPECT(refused(g)); }
  { sim_config g = good; g.dt = 0.02; EXPECT(refused(g)); }
  { sim_config g = good; g.c0 = 0.0; EXPECT(refused(g)); }
  { sim_config g = good; g.c_dec = 1e3; EXPECT(refused(g)); }
  { sim_config g = good; g.queue_cap = 0; EXPECT(refused(g)); }
  { sim_config g = good; g.dbuf_cap = (int64_t(1) << 30) + 1; EXPECT(refused(g)); }
  { sim_config g = good; g.gate_mode = 3; EXPECT(refused(g)); }
  { sim_config g = good; g.route_mode = 9; EXPECT(refused(g)); }
  { sim_config g = good; g.mod_period = -1; EXPECT(refused(g)); }
  { sim_config g = good; g.mod_period = int64_t(1) << 40; EXPECT(refused(g)); }
  { sim_config g = good; g.mod_amp = 1.5; EXPECT(refused(g)); }
  { sim_config g = good; g.cls = nullptr; EXPECT(refused(g)); }
  { sim_config g = good; g.x_star = nullptr; EXPECT(refused(g)); }
  { sim_config g = good; g.route_mode = SIM_ROUTE_RANDOM_SPLIT; g.p_solo = nullptr; EXPECT(refused(g)); }
  { sim_config g = good; g.route_mode = SIM_ROUTE_WEIGHTED_SPLIT; g.w_mixed = nullptr; EXPECT(refused(g)); }
  c.cls[1].theta = -1.0; EXPECT(refused(good)); c.cls[1].theta = 0.0;
  c.cls[0].lambda = 60.0; EXPECT(refused(good)); c.cls[0].lambda = 0.2;
  c.x_star[1] = -0.5; EXPECT(refused(good)); c.x_star[1] = 0.02;
  EXPECT(sim_workspace_bytes(nullptr, 1, &bytes) == SIM_EINVAL);
  EXPECT(sim_workspace_bytes(&good, 1, nullptr) == SIM_EINVAL);
  EXPECT(sim_onchip_bytes(nullptr, &bytes, nullptr) == SIM_EINVAL);
  EXPECT(sim_launch_plan(nullptr, 1, nullptr, nullptr, nullptr) == SIM_EINVAL);
  EXPECT(sim_launch_plan(&good, 4, nullptr, nullptr, nullptr) == SIM_OK);

  // entry points that take a handle refuse a null one
  EXPECT(sim_run(nullptr, 1, 1, 1, nullptr) == SIM_EINVAL);
  EXPECT(sim_stats(nullptr, nullptr, nullptr) == SIM_EINVAL);
  EXPECT(sim_set_targets(nullptr, nullptr, nullptr, nullptr) == SIM_EINVAL);
  EXPECT(sim_set_split(nullptr, 0, nullptr) == SIM_EINVAL);
  EXPECT(sim_snapshot(nullptr, 0, nullptr, nullptr) == SIM_EINVAL);
  EXPECT(sim_tallies(nullptr, 0, nullptr, nullptr) == SIM_EINVAL);
  EXPECT(sim_hist(nullptr, 0, 0, nullptr, nullptr) == SIM_EINVAL);
  EXPECT(sim_digest(nullptr, 0, nullptr, nullptr) == SIM_EINVAL);
  EXPECT(sim_kernel_time(nullptr, nullptr, nullptr, 0, nullptr) == SIM_EINVAL);
  EXPECT(sim_launch_shape(nullptr, nullptr, nullptr) == SIM_EINVAL);
  EXPECT(sim_destroy(nullptr) == SIM_EINVAL);

  // the static workspace: a handle where a GPU is present, SIM_EHIP where there is none
  sim_t *h = nullptr;
  const int rc = sim_create_static(&good, 4, &h);
  EXPECT(rc == SIM_OK || rc == SIM_EHIP);
  if (rc == SIM_OK) EXPECT(sim_destroy(h) == SIM_OK);

  if (failures == 0) std::printf("clean\n");
  return failures != 0;
}
