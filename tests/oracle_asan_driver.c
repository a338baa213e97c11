/* Test driver (CPU only): runs the oracle's policy variants on a small overloaded instance in a build with
 * AddressSanitizer and the undefined-behaviour checks; any finding aborts the process. The oracle source is
 * compiled into this program, so the sanitizer runtime is the program's own. */
#include <stdio.h>

#include "../oracle/gnr_oracle.c"

static oracle_class classes[3];
static double x_star[3] = {0.2, 0.15, 0.05}, qp_star[3] = {0.5, 0.0, 0.1};
static double p_solo[3] = {0.8, 0.3, 0.55}, w_solo[3] = {0.5, 0.0, 0.5}, w_mixed[3] = {0.1, 0.6, 0.3};

static oracle_config base_config(void)
{
  memset(classes, 0, sizeof classes);
  classes[0] = (oracle_class){.lambda = 1.6, .in_law = LAW_GEOMETRIC, .in_p0 = 300.0, .out_law = LAW_GEOMETRIC, .out_p0 = 40.0,
                              .price_in = 1.0, .price_out = 1.0, .bundled = 1, .priority = 0.2};
  classes[1] = (oracle_class){.lambda = 1.2, .in_law = LAW_LOGNORMAL, .in_p0 = 90.0, .in_p1 = 0.8, .out_law = LAW_LOGNORMAL,
                              .out_p0 = 150.0, .out_p1 = 1.0, .price_in = 0.5, .price_out = 2.0, .bundled = 0, .priority = 1.5};
  classes[2] = (oracle_class){.lambda = 0.8, .in_law = LAW_CONST, .in_p0 = 513.0, .out_law = LAW_GEOMETRIC, .out_p0 = 20.0,
                              .price_in = 1.0, .price_out = 1.0, .bundled = 1, .priority = 0.9};
  oracle_config c;
  memset(&c, 0, sizeof c);
  c.K = 3; c.N = 12; c.B = 4; c.C = 128;
  c.c0 = 0.010; c.c_pre = 0.00005; c.c_dec = 0.0002; c.dt = 0.0;
  c.cls = classes; c.M = 5; c.x_star = x_star; c.qp_star = qp_star;
  c.gate_mode = GATE_OCCUPANCY; c.route_mode = ROUTE_SOLO_FIRST;
  c.queue_cap = 40; c.dbuf_cap = 12;
  c.p_solo = p_solo; c.w_solo = w_solo; c.w_mixed = w_mixed;
  return c;
}

static int run_case(const char *name, oracle_config c, int impatient)
{
  classes[0].theta = impatient ? 4.0 : 0.0;
  classes[1].theta = 0.0;
  classes[2].theta = impatient ? 25.0 : 0.0;
  oracle_t *o = NULL;
  if (oracle_create(&c, 3, &o)) { printf("%s: create failed\n", name); return 1; }
  oracle_set_check(o, 1);
  if (oracle_run(o, 1500, 3, 11)) { printf("%s: run failed\n", name); return 1; }
  oracle_set_split(o, c.M / 2);
  if (oracle_run(o, 500, 3, 11)) { printf("%s: run failed\n", name); return 1; }
  oracle_stats_t st;
  uint64_t d = 0;
  oracle_stats(o, &st);
  for (int r = 0; r < 3; r++) oracle_digest(o, r, &d);
  const int64_t v = oracle_violations(o);
  oracle_destroy(o);
  if (v) { printf("%s: %lld invariant violations\n", name, (long long)v); return 1; }
  return 0;
}

int main(void)
{
  int bad = 0;
  oracle_config c = base_config();
  bad += run_case("base", c, 0);
  bad += run_case("abandonment", c, 1);
  c.gate_mode = GATE_FCFS; bad += run_case("fcfs gate", c, 0);
  c.gate_mode = GATE_PRIORITY; bad += run_case("priority gate", c, 1);
  c = base_config(); c.route_mode = ROUTE_RANDOM_SPLIT; bad += run_case("randomized router", c, 0);
  bad += run_case("randomized router, abandonment", c, 1);
  c.route_mode = ROUTE_WEIGHTED_SPLIT; bad += run_case("weighted router", c, 0);
  bad += run_case("weighted router, abandonment", c, 1);
  c = base_config(); c.route_mode = ROUTE_IMMEDIATE; c.M = c.N; bad += run_case("immediate decode", c, 1);
  c = base_config(); c.queue_cap = 1; c.dbuf_cap = 1; bad += run_case("tiny rings", c, 0);
  c = base_config(); c.mod_amp = 0.3; c.mod_period = 500; c.B = 1; bad += run_case("modulated arrivals, B = 1", c, 1);
  c = base_config(); c.M = 0; bad += run_case("no mixed group", c, 0);
  c = base_config(); c.N = 1; c.M = 1; c.B = 3; bad += run_case("one server", c, 1);
  if (!bad) printf("clean\n");
  return bad ? 1 : 0;
}
