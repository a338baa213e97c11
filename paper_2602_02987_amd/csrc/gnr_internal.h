// Internal declarations shared by the host glue and the HIP kernels of the simulator.
#ifndef GNR_INTERNAL_H
#define GNR_INTERNAL_H

#include <cstddef>
#include <cstdint>

#include "gnr_sim.h"

namespace gnr {

constexpr int kMaxK = SIM_MAXK;
constexpr int kMaxB = SIM_MAXB;
constexpr int kMaxN = SIM_MAXN;
constexpr int kNBin = SIM_NBIN;
constexpr int kTableSize = 65536;
constexpr int kMaxLen = 32768;
constexpr int kMaxChunk = 8191;   // the running chunk is kept in 13 bits of the prefill word
constexpr int kNTally = SIM_NTALLY;
constexpr int kNGlobal = SIM_NGLOBAL;
constexpr int kTallyWords = kMaxK * kNTally + kNGlobal;  // per replication, uint64
constexpr int64_t kIdle = INT64_MAX;
constexpr int kAdmChunk = 256;    // admissions decided per gate pass
constexpr int kMaxTbtBins = 256;  // width of the on-chip time-between-tokens histogram window

// Per-replication class-level state, int32 words (persisted between launches).
enum ClassStateWord {
  CS_QP = 0, CS_X = 8, CS_QD = 16, CS_YM = 24, CS_YS = 32, CS_QHEAD = 40, CS_DHEAD = 48, CS_DCOUNT = 49,
  CS_DHEAD_M = 50, CS_DCOUNT_M = 51,   // the mixed group's buffer under the randomized router
  CS_QDS = 52,                         // [8] weighted router: waiting requests per class in the solo group's buffer
  CS_WORDS = 64
};
constexpr uint32_t kNever = 0xFFFFFFFFu;   // deadline of a request that never abandons
constexpr int kStreamPatienceP = 2;        // random streams: 0 arrivals, 1 lengths, 2+k prefill-queue patience of class k,
constexpr int kStreamPatienceD = 10;       // 10 decode-buffer patience (word 0) and group of the randomized routers (word 1)
constexpr int kStreamSelect = 11;          // 11, 12: class selection of the weighted router in the solo / mixed pool

// Everything a kernel needs, passed by value.
struct Params {
  int K, N, B, C, M, R;
  int Mp;                     // servers below this may hold a prefill: the largest M the handle has had
  int BS;                     // slot-row stride in words: B rounded up to a multiple of 4
  int gate_mode;
  int tbt_lo, tbt_w;          // first bin and width of the TBT histogram window kept in LDS
  int nwords;                 // ceil(N/64) bitmap words
  int threads;                // workgroup size of the step kernel
  uint32_t key0, key1;
  uint32_t queue_cap, dbuf_cap;
  int64_t c0, cpre, cdec, dt;
  int64_t mod_period;
  double nx[kMaxK], invx[kMaxK], xstar[kMaxK], nq[kMaxK], prio[kMaxK];   // n x*, 1/x*, x*, n q*, priority index
  uint32_t cls_thr[kMaxK];
  // abandonment: classes with a patience rate (bit k), mask of the deadline calendars (entries - 1, a power of two
  // above the longest patience in steps)
  uint32_t ab_classes, cal_mask;
  // deadline rings and calendars are in use: some class has a patience rate, or the weighted router is on (it
  // takes requests out of the middle of a buffer and marks their entries with a deadline that has passed)
  uint32_t dl_rings;
  // randomized router: a decode of class k goes to the solo group when its random word is below solo_thr[k]
  int route_mode;
  uint32_t solo_thr[kMaxK];
  // weighted router: class selection weights of the solo [0] and the mixed [1] pool in units of 2^-20, at least 1
  uint32_t wsel[2][kMaxK];
  // tables (device)
  const uint32_t *arr_thr;    // [rows][3]
  const uint16_t *len_tab;    // [K][2][65536]: in, out
  const uint16_t *pat_tab;    // [K][65536] patience in steps (abandonment only)
  // per-server state, [R][N]
  int64_t *t_next;
  uint32_t *iter;
  uint32_t *remptok;          // prompt tokens left | tokens in the running chunk << 16 | class << 29
  uint64_t *pf_job;
  uint64_t *n_cls, *n_join;   // 8 x uint8 packed
  // decode slots, [R][N][BS]; slots 0..n_dec-1 of a server are occupied
  uint32_t *fin;
  uint64_t *job;
  // rings
  uint32_t *qring;            // [R][K][queue_cap] arrival stamps
  uint64_t *dring;            // [R][dbuf_cap] requests
  uint64_t *dring_m;          // [R][dbuf_cap] randomized router only: the mixed group's buffer
  // abandonment only: the step at whose start a waiting request leaves, beside each ring entry; per class and
  // step (modulo the calendar size), how many waiting requests leave at that step
  uint32_t *qdl;              // [R][K][queue_cap]
  uint32_t *ddl;              // [R][dbuf_cap]
  uint32_t *cal;              // [R][K][cal_mask+1] prefill queues
  uint32_t *dcal;             // [R][K][cal_mask+1] decode buffer
  uint32_t *ddl_m, *dcal_m;   // the same for the mixed group's buffer of the randomized router
  // class state, tallies, histograms
  int32_t *cstate;            // [R][CS_WORDS]
  uint64_t *tally;            // [R][kTallyWords]
  uint64_t *hist;             // [R][3][K][kNBin]
  uint64_t *digest;           // [R]
  uint64_t *reduced;          // [kTallyWords + 3*K*kNBin] totals over replications
  const Params *self;         // device copy of this struct (key0/key1 there are unused)
};

// host-side table builders (gnr_tables.cpp)
int build_length_table(int law, double p0, double p1, const uint16_t *user, uint16_t *out);
int build_patience_table(double theta, double dt_seconds, uint16_t *out);
double total_rate(const sim_class *cls, int K);
void build_arrival_row(double lam, int64_t dt_ns, double amp, int64_t period, int64_t row, uint32_t thr[3]);
void build_class_thresholds(const sim_class *cls, int K, uint32_t *thr);
uint32_t probability_threshold(double p);   // floor(p * 2^32) clamped to [0, 2^32 - 1]
uint32_t selection_weight_units(double w);  // round(w * 2^20) clamped to [1, 2^20]

// kernel launchers (gnr_kernels.hip); stream is a hipStream_t
int launch_reset(const Params &p, int reps, void *stream);
int launch_steps(const Params &p, int reps, int threads, size_t lds_bytes, uint32_t step_begin, uint32_t n_steps,
                 void *stream);
int launch_reduce(const Params &p, int reps, void *stream);
int launch_digest(const Params &p, int reps, void *stream);
// the library's static device workspace on the current device (address resolved once per device)
int static_workspace(void **dev_ptr, size_t *bytes);
size_t step_lds_bytes(const Params &p);
int step_threads(Params q, int reps);
bool step_dense(int reps, int threads, size_t lds_bytes);   // whether such a launch takes the four-waves-per-SIMD form of a small size class   // workgroup size for a launch of `reps` replications (q.threads is not read)

}  // namespace gnr
#endif
