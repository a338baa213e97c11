// HIP kernels of the gate-and-route network simulator (gfx950, wave64).
//
// One workgroup owns one replication for a whole launch and loops over the steps itself.
// Server g is owned by thread g % blockDim of its replication's workgroup: only the owner ever
// touches that server's record and slot row, so per-server updates need no synchronisation.
// Class-level counters (queue lengths, occupancies, tallies) live in LDS and are updated with
// integer atomics, which commute; everything that the policy defines sequentially (order of
// simultaneous prefill completions, of gate admissions, of routed requests) is reproduced with
// 64-server ballot words in LDS and prefix popcounts over them.
#include <hip/hip_runtime.h>

#include "gnr_internal.h"

namespace gnr {

// ------------------------------------------------------------------ primitives ----
// Philox4x32-10 (Salmon et al., SC'11).
__device__ __forceinline__ void philox4x32_10(uint32_t k0, uint32_t k1, uint32_t c0, uint32_t c1, uint32_t c2,
                                              uint32_t c3, uint32_t (&w)[4])
{
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    const uint64_t a = static_cast<uint64_t>(0xD2511F53u) * c0;
    const uint64_t b = static_cast<uint64_t>(0xCD9E8D57u) * c2;
    const uint32_t n0 = static_cast<uint32_t>(b >> 32) ^ c1 ^ k0;
    const uint32_t n2 = static_cast<uint32_t>(a >> 32) ^ c3 ^ k1;
    c1 = static_cast<uint32_t>(b);
    c3 = static_cast<uint32_t>(a);
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  w[0] = c0; w[1] = c1; w[2] = c2; w[3] = c3;
}

// Histogram bin of a duration in ns: exact below 16, then 16 bins per octave.
__device__ __forceinline__ int hbin(int64_t v)
{
  if (v < 16) return v < 0 ? 0 : static_cast<int>(v);
  const int e = 63 - __clzll(static_cast<unsigned long long>(v));
  const int b = 16 * (e - 3) + static_cast<int>((v >> (e - 4)) & 15);
  return b < kNBin ? b : kNBin - 1;
}

__device__ __forceinline__ uint32_t byte_sum(uint64_t packed)
{
  return static_cast<uint32_t>((packed * 0x0101010101010101ull) >> 56);
}
__device__ __forceinline__ uint32_t byte_at(uint64_t packed, int k) { return static_cast<uint32_t>(packed >> (8 * k)) & 255u; }

// Prefill word of a server: prompt tokens left | tokens in the running chunk << 16 | class << 29.
__device__ __forceinline__ int pk_rem(uint32_t pk) { return static_cast<int>(pk & 0xFFFFu); }
__device__ __forceinline__ int pk_ptok(uint32_t pk) { return static_cast<int>((pk >> 16) & 0x1FFFu); }
__device__ __forceinline__ int pk_cls(uint32_t pk) { return static_cast<int>(pk >> 29); }

// Position of the n-th set bit (n counted from 0) of a word that has more than n bits set.
__device__ __forceinline__ int nth_set_bit(uint64_t word, int n)
{
  int pos = 0;
#pragma unroll
  for (int sh = 32; sh > 0; sh >>= 1) {
    const int c = __popcll(word & ((1ull << sh) - 1ull));
    if (n >= c) { n -= c; word >>= sh; pos += sh; }
  }
  return pos;
}

// Index of the j-th set bit of a bitmap given the exclusive prefix popcounts of its words.
__device__ __forceinline__ int select_bit(const uint64_t *bm, const uint32_t *pre, int nwords, uint32_t j)
{
  int lo = 0, hi = nwords - 1;   // largest w with pre[w] <= j
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (pre[mid] <= j) lo = mid; else hi = mid - 1;
  }
  return lo * 64 + nth_set_bit(bm[lo], static_cast<int>(j - pre[lo]));
}

__device__ __forceinline__ uint64_t lanes_below() { return (1ull << (threadIdx.x & 63)) - 1ull; }

__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v)
{
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t o = __shfl_up(v, d, 64);
    if (lane >= d) v += o;
  }
  return v;
}

__device__ __forceinline__ void lds_add64(uint64_t *p, uint64_t v)
{
  atomicAdd(reinterpret_cast<unsigned long long *>(p), static_cast<unsigned long long>(v));
}

// Optional per-phase cycle counters (compiled out unless GNR_PROF is defined).
#ifdef GNR_PROF
__device__ unsigned long long g_prof[16];
#define PROF_DECL unsigned long long prof_acc[16] = {0}; unsigned long long prof_last = clock64();
#define PROF(i) { const unsigned long long t_ = clock64(); prof_acc[i] += t_ - prof_last; prof_last = t_; }
#define PROF_FLUSH if ((threadIdx.x & 63) == 0) { for (int i_ = 0; i_ < 16; ++i_) atomicAdd(&g_prof[i_], prof_acc[i_]); }
#else
#define PROF_DECL
#define PROF(i)
#define PROF_FLUSH
#endif

// ------------------------------------------------------------------ LDS layout ----
enum Scalar {
  SC_NIDLE = 0, SC_NCOMP,
  SC_TAKE = 16,   // [8] accepted arrivals this step
  SC_TAIL = 24,   // [8] ring position of the first accepted arrival
  SC_ADMK = 40,   // [8] admissions per class in this gate pass
  SC_WORDS = 48
};
constexpr int kLoadBins = kMaxB + 1;
constexpr int kEvPerWave = 128;   // completions a wave can queue per step; any beyond are finished inline
constexpr int kMaxWaves = 16;

struct Lds {
  int32_t *cs;        // [CS_WORDS]
  uint32_t *acc;      // [8]
  int32_t *sc;        // [SC_WORDS]
  uint64_t *tl;       // [kTallyWords]
  uint64_t *tbth;     // [K][tbt_w]
  uint64_t *bm_idle;  // [nwords] mixed-group servers whose prefill slot is idle
  uint64_t *bm_comp;  // [nwords] servers whose prefill completed this step
  uint64_t *bm_lvl;   // [nwords] servers at the routing level
  uint64_t *bm_busy;  // [nwords] servers running an iteration
  uint64_t *bm_join;  // [nwords] servers holding a decode that joined after the running iteration started
  uint64_t *bm_due;   // [nwords] servers that completed an iteration this step
  uint64_t *bm_touch; // [nwords] idle servers that were given work this step
  uint32_t *pre_c;    // [nwords] exclusive prefix popcounts of bm_comp
  uint32_t *pre;      // [nwords] exclusive prefix popcounts of bm_idle / bm_lvl
  uint32_t *adm;      // [kAdmChunk] class | sequence-in-class << 3 of each admission
  uint32_t *lh;       // [2][kLoadBins] servers per decode count: solo group, mixed group
  uint32_t *ev_g;     // [waves][kEvPerWave] servers with decodes leaving this step, queued per wave
  uint32_t *ev_q;     // [waves][kEvPerWave] their slot-quad masks
  uint32_t *t32;      // [N] low 32 bits of the end time of the running iteration
  uint32_t *iter;     // [N] completed iterations
  uint8_t *loads;     // [N] decodes per server
};

// Carves the dynamic LDS block; 8-byte granules, 64-bit arrays first.
__host__ __device__ __forceinline__ Lds lds_carve(const Params &p, unsigned char *base, size_t *total)
{
  Lds L;
  size_t off = 0;
#define GNR_TAKE(field, type, count)                       \
  L.field = reinterpret_cast<type *>(base + off);          \
  off += (sizeof(type) * static_cast<size_t>(count) + 7) & ~size_t(7);
  GNR_TAKE(tl, uint64_t, kTallyWords)
  GNR_TAKE(tbth, uint64_t, p.K * p.tbt_w)
  GNR_TAKE(bm_idle, uint64_t, p.nwords)
  GNR_TAKE(bm_comp, uint64_t, p.nwords)
  GNR_TAKE(bm_lvl, uint64_t, p.nwords)
  GNR_TAKE(bm_busy, uint64_t, p.nwords)
  GNR_TAKE(bm_join, uint64_t, p.nwords)
  GNR_TAKE(bm_due, uint64_t, p.nwords)
  GNR_TAKE(bm_touch, uint64_t, p.nwords)
  GNR_TAKE(cs, int32_t, CS_WORDS)
  GNR_TAKE(acc, uint32_t, 8)
  GNR_TAKE(sc, int32_t, SC_WORDS)
  GNR_TAKE(pre_c, uint32_t, p.nwords + 1)
  GNR_TAKE(pre, uint32_t, p.nwords + 1)
  GNR_TAKE(adm, uint32_t, kAdmChunk)
  GNR_TAKE(lh, uint32_t, 2 * kLoadBins)
  GNR_TAKE(ev_g, uint32_t, kMaxWaves * kEvPerWave)
  GNR_TAKE(ev_q, uint32_t, kMaxWaves * kEvPerWave)
  GNR_TAKE(t32, uint32_t, p.N)
  GNR_TAKE(iter, uint32_t, p.N)
  GNR_TAKE(loads, uint8_t, p.N)
#undef GNR_TAKE
  if (total) *total = off;
  return L;
}

size_t step_lds_bytes(const Params &p)
{
  size_t total = 0;
  lds_carve(p, nullptr, &total);
  return total;
}

int step_threads(int N)
{
  int t = (N + 63) / 64 * 64;
  // 512 threads leave each wave 256 registers; with 1024 the step kernel spills to scratch
#ifdef GNR_MAX_THREADS
  return t > GNR_MAX_THREADS ? GNR_MAX_THREADS : t;
#else
  return t > 512 ? 512 : t;
#endif
}

// Exclusive prefix popcounts of a bitmap, computed by one whole wave; returns the total in every lane.
__device__ __forceinline__ uint32_t rank_bitmap(const uint64_t *bm, uint32_t *pre, int nwords)
{
  const int lane = threadIdx.x & 63;
  uint32_t running = 0;
  for (int base = 0; base < nwords; base += 64) {
    const int w = base + lane;
    const uint32_t v = w < nwords ? static_cast<uint32_t>(__popcll(bm[w])) : 0u;
    const uint32_t inc = wave_incl_scan(v);
    if (w < nwords) pre[w] = running + inc - v;
    running += __shfl(inc, 63, 64);
  }
  return running;
}

__device__ __forceinline__ uint64_t wave_sum64(uint64_t v)
{
#pragma unroll
  for (int d = 32; d > 0; d >>= 1) {
    const uint32_t lo = __shfl_xor(static_cast<uint32_t>(v), d, 64);
    const uint32_t hi = __shfl_xor(static_cast<uint32_t>(v >> 32), d, 64);
    v += (static_cast<uint64_t>(hi) << 32) | lo;
  }
  return v;
}
__device__ __forceinline__ uint32_t wave_sum32(uint32_t v)
{
#pragma unroll
  for (int d = 32; d > 0; d >>= 1) v += __shfl_xor(v, d, 64);
  return v;
}

// Per-lane sums of the tallies every executed iteration touches. The step sums are folded into
// the workgroup's totals once per step; the time-between-tokens counts stay cached per lane for
// the bin they fall in and are written out when the bin changes or the launch ends. Three bins are
// cached because a lane's servers have three typical durations: solo group, mixed group without
// and with a prefill chunk.
struct LaneTallies {
  uint32_t iters[2];            // this step: [decode-only, with a prefill chunk]
  uint64_t busy[2];
  uint64_t tbt_sum[kMaxK];
  int hist_bin[3];              // across steps: [solo group, mixed group decode-only, with a chunk]
  uint32_t hist_cnt[3][kMaxK];
};

// One executed iteration of duration d whose batch held the decodes nc minus the late joiners nj.
template <int SLOT>
__device__ __forceinline__ void tally_iteration(LaneTallies &lt, uint64_t *tbth, int tbt_w, int K, int64_t d, int tb,
                                                uint64_t nc, uint64_t nj)
{
  constexpr int KIND = SLOT == 2 ? 1 : 0;
  lt.iters[KIND] += 1;
  lt.busy[KIND] += static_cast<uint64_t>(d);
  if (tb != lt.hist_bin[SLOT]) {   // the duration moved to another bin: flush the cached counts
#pragma unroll
    for (int k = 0; k < kMaxK; ++k)
      if (k < K && lt.hist_cnt[SLOT][k]) {
        lds_add64(&tbth[k * tbt_w + lt.hist_bin[SLOT]], lt.hist_cnt[SLOT][k]);
        lt.hist_cnt[SLOT][k] = 0;
      }
    lt.hist_bin[SLOT] = tb;
  }
#pragma unroll
  for (int k = 0; k < kMaxK; ++k) {
    const uint32_t em = byte_at(nc, k) - byte_at(nj, k);
    lt.tbt_sum[k] += static_cast<uint64_t>(em) * static_cast<uint64_t>(d);
    lt.hist_cnt[SLOT][k] += em;
  }
}

// ---- wave-level folding of per-event class updates: lanes of one class are combined first, so that a
// counter sees one LDS atomic per wave and class instead of one per event. All take uniform control flow.
__device__ __forceinline__ void wave_count_by_class(bool active, int k, int K, uint64_t *base, int stride)
{
  for (int c = 0; c < K; ++c) {
    const uint64_t m = __ballot(active && k == c);
    if (m && (threadIdx.x & 63) == 0) lds_add64(&base[c * stride], static_cast<uint64_t>(__popcll(m)));
  }
}
__device__ __forceinline__ void wave_count_by_class_i32(bool active, int k, int K, int32_t *base, int sign)
{
  for (int c = 0; c < K; ++c) {
    const uint64_t m = __ballot(active && k == c);
    if (m && (threadIdx.x & 63) == 0) atomicAdd(&base[c], sign * __popcll(m));
  }
}
__device__ __forceinline__ void wave_sum_by_class(bool active, int k, int K, uint64_t v, uint64_t *base, int stride)
{
  for (int c = 0; c < K; ++c) {
    const bool in = active && k == c;
    if (__ballot(in)) {
      const uint64_t t = wave_sum64(in ? v : 0ull);
      if ((threadIdx.x & 63) == 0) lds_add64(&base[c * stride], t);
    }
  }
}
// Sum over the wave of per-class byte vectors (8 x uint8, each <= 128): 16-bit fields, even and odd classes.
__device__ __forceinline__ void wave_sum_bytes(uint64_t v, uint64_t &even, uint64_t &odd)
{
  even = wave_sum64(v & 0x00FF00FF00FF00FFull);
  odd = wave_sum64((v >> 8) & 0x00FF00FF00FF00FFull);
}
__device__ __forceinline__ uint32_t class_field(uint64_t even, uint64_t odd, int c)
{
  return static_cast<uint32_t>(((c & 1) ? odd : even) >> (16 * (c >> 1))) & 0xFFFFu;
}

// What finishing an iteration reports back for folding: the first decode that left the server and
// the end of its prefill. Further decodes leaving in the same iteration are tallied directly.
struct Leaving { int k; uint32_t P, D; int64_t e2e; bool mixed; };
struct PrefillEnd { bool done; int k; uint32_t P; int64_t ttft; uint64_t nc; };

// Sort key of a gate candidate: the m-th waiting request of class k (m counted from the head).
// Occupancy gate: (X_k + m - n x_k*)/x_k*, ties by the larger queue deviation Q_k - m - n q_k*;
// priority gate: larger static index first; FCFS gate: older arrival stamp first.
// Ties that remain go to the lower class. Within a class the key does not decrease with m, so the
// gate's one-at-a-time argmin is the merge of the classes' sequences in this order.
struct GateKey { double a, b; };

__device__ __forceinline__ GateKey gate_key(const Params &p, const uint32_t *qring, const int (&xs)[kMaxK],
                                            const int (&qp)[kMaxK], const uint32_t (&head)[kMaxK], int k, int m)
{
  GateKey key;
  if (p.gate_mode == SIM_GATE_OCCUPANCY) {
    key.a = (static_cast<double>(xs[k] + m) - p.nx[k]) * p.invx[k];
    key.b = static_cast<double>(qp[k] - m) - p.nq[k];
  } else if (p.gate_mode == SIM_GATE_PRIORITY) {
    key.a = -p.prio[k];
    key.b = 0.0;
  } else {
    uint32_t pos = head[k] + static_cast<uint32_t>(m);
    if (pos >= p.queue_cap) pos -= p.queue_cap;
    key.a = static_cast<double>(qring[static_cast<size_t>(k) * p.queue_cap + pos]);
    key.b = 0.0;
  }
  return key;
}

// true if candidate (k1, key1) is admitted before candidate (k2, key2), k1 != k2
__device__ __forceinline__ bool gate_before(const GateKey &x, int k1, const GateKey &y, int k2)
{
  if (x.a != y.a) return x.a < y.a;
  if (x.b != y.b) return x.b > y.b;
  return k1 < k2;
}

// ------------------------------------------------------------------ step kernel ----
// What the completion pass knows about one server of the round being processed.
struct RoundState {
  bool due;        // the server's iteration ends within this step
  uint32_t t32;    // low 32 bits of its end time
  uint32_t it;     // index of the iteration that ends
  int nd;          // decodes on the server
  uint64_t nc, nj; // per-class decode counts; of those, late joiners
  uint32_t pk;     // prefill word (mixed group only)
  uint64_t due_mask, join_word;
};

template <int MAXT>
__global__ void __launch_bounds__(MAXT) gnr_step_kernel(const Params *__restrict__ params, const uint32_t key0,
                                                        const uint32_t key1, const uint32_t step_begin,
                                                        const uint32_t n_steps)
{
  const Params &p = *params;   // immutable after creation; read through the scalar cache on demand
  extern __shared__ __align__(16) unsigned char lds_raw[];
  const Lds L = lds_carve(p, lds_raw, nullptr);

  const int r = blockIdx.x;
  const int tid = threadIdx.x;
  const int NT = blockDim.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wave_base = tid & ~63;
  const int K = p.K, N = p.N, B = p.B, M = p.M, BS = p.BS;
  const int nper = (N + NT - 1) / NT;
  const int nwords_m = (M + 63) >> 6;   // bitmap words that hold mixed-group servers

  int64_t *t_next = p.t_next + static_cast<size_t>(r) * N;
  uint32_t *iter_g = p.iter + static_cast<size_t>(r) * N;
  uint32_t *remptok = p.remptok + static_cast<size_t>(r) * N;
  uint64_t *pf_job = p.pf_job + static_cast<size_t>(r) * N;
  uint64_t *n_cls = p.n_cls + static_cast<size_t>(r) * N;
  uint64_t *n_join = p.n_join + static_cast<size_t>(r) * N;
  uint32_t *fin = p.fin + static_cast<size_t>(r) * N * BS;
  uint64_t *job = p.job + static_cast<size_t>(r) * N * BS;
  uint32_t *qring = p.qring + static_cast<size_t>(r) * K * p.queue_cap;
  uint64_t *dring = p.dring + static_cast<size_t>(r) * p.dbuf_cap;
  uint64_t *hist = p.hist + static_cast<size_t>(r) * 3 * K * kNBin;
  uint32_t *ev_g = L.ev_g + wave * kEvPerWave;
  uint32_t *ev_q = L.ev_q + wave * kEvPerWave;

  // ---- load the replication's class state and rebuild the on-chip views of the server state
  for (int i = tid; i < CS_WORDS; i += NT) L.cs[i] = p.cstate[static_cast<size_t>(r) * CS_WORDS + i];
  for (int i = tid; i < kTallyWords; i += NT) L.tl[i] = 0;
  for (int i = tid; i < K * p.tbt_w; i += NT) L.tbth[i] = 0;
  for (int i = tid; i < SC_WORDS; i += NT) L.sc[i] = 0;
  for (int i = tid; i < 2 * kLoadBins; i += NT) L.lh[i] = 0;
  __syncthreads();
  for (int i = 0; i < nper; ++i) {
    const int g = i * NT + tid;
    const bool valid = g < N;
    bool busy = false, joined = false;
    if (valid) {
      const uint32_t nd = byte_sum(n_cls[g]);
      L.loads[g] = static_cast<uint8_t>(nd);
      atomicAdd(&L.lh[(g < M ? kLoadBins : 0) + nd], 1u);
      const int64_t tn = t_next[g];
      busy = tn != kIdle;
      L.t32[g] = static_cast<uint32_t>(tn);
      L.iter[g] = iter_g[g];
      joined = n_join[g] != 0;
    }
    const bool idle_slot = valid && g < M && pk_rem(remptok[g]) == 0;
    const uint64_t bi = __ballot(idle_slot), bb = __ballot(busy), bj = __ballot(joined);
    const int wi = (i * NT + wave_base) >> 6;
    if (lane == 0 && wi < p.nwords) { L.bm_idle[wi] = bi; L.bm_busy[wi] = bb; L.bm_join[wi] = bj; }
  }
  LaneTallies lt;
  lt.hist_bin[0] = lt.hist_bin[1] = lt.hist_bin[2] = 0;
#pragma unroll
  for (int k = 0; k < kMaxK; ++k) lt.hist_cnt[0][k] = lt.hist_cnt[1][k] = lt.hist_cnt[2][k] = 0;
  __syncthreads();

  int64_t T = 0;
  PROF_DECL
  for (uint32_t s = step_begin; s < step_begin + n_steps; ++s) {
    PROF(0)
    T = (static_cast<int64_t>(s) + 1) * p.dt;
    const uint32_t T32 = static_cast<uint32_t>(T);
    if (tid < 8) L.acc[tid] = 0;
    lt.iters[0] = lt.iters[1] = 0; lt.busy[0] = lt.busy[1] = 0;
#pragma unroll
    for (int k = 0; k < kMaxK; ++k) lt.tbt_sum[k] = 0;
    const uint32_t *thr = p.arr_thr + 3 * (p.mod_period > 0 ? static_cast<int64_t>(s % static_cast<uint64_t>(p.mod_period)) : 0);
    const uint32_t thr0 = thr[0], thr1 = thr[1], thr2 = thr[2];
    __syncthreads();

    // ---- 1. arrivals of one server: one random block, word 0 -> count, words 1.. -> classes
    auto arrivals = [&](int g) __attribute__((always_inline)) {
      uint32_t w[4];
      philox4x32_10(key0, key1, s, 0u, static_cast<uint32_t>(g), static_cast<uint32_t>(r), w);
      if (w[0] >= thr0) {
        const int a = 1 + (w[0] >= thr1) + (w[0] >= thr2);
#pragma unroll
        for (int j = 0; j < 3; ++j) {
          if (j >= a) break;
          int k = 0;
#pragma unroll
          for (int c = 0; c + 1 < kMaxK; ++c) k += (c + 1 < K && w[1 + j] >= p.cls_thr[c]);
          atomicAdd(&L.acc[k], 1u);
        }
      }
    };

    // ---- 2. finishing the iteration of server g: tallies, decodes that emitted their last token
    //      (slot quads flagged in `quads`), prefill progress. Class-level effects of the first decode
    //      that leaves and of a prefill that ends are reported in lv / pe for folding by the caller.
    auto leave_direct = [&](int k, uint32_t Pl, uint32_t Dl, int64_t e2e, bool mixed_now) __attribute__((always_inline)) {
      lds_add64(&L.tl[k * kNTally + (mixed_now ? SIM_T_S_DM : SIM_T_S_DS)], 1);
      atomicSub(&L.cs[(mixed_now ? CS_YM : CS_YS) + k], 1);
      lds_add64(&L.tl[k * kNTally + SIM_T_TOKP_DEC], Pl);
      lds_add64(&L.tl[k * kNTally + SIM_T_TOKD_DEC], Dl);
      lds_add64(&L.tl[k * kNTally + SIM_T_E2E_SUM], static_cast<uint64_t>(e2e));
    };
    auto finish_iteration = [&](int g, uint32_t it, int nd, uint64_t nc, uint64_t nj, uint32_t pk, uint32_t t32,
                                uint32_t quads, Leaving &lv, PrefillEnd &pe) __attribute__((always_inline)) {
      int rem = pk_rem(pk);
      const int ptok = pk_ptok(pk);
      const int64_t tn = T + static_cast<int64_t>(static_cast<int32_t>(t32 - T32));   // exact completion time
      const int64_t d = p.c0 + p.cpre * ptok + p.cdec * static_cast<int64_t>(nd - static_cast<int>(byte_sum(nj)));
      const int tb = hbin(d) - p.tbt_lo;
      if (g >= M) tally_iteration<0>(lt, L.tbth, p.tbt_w, K, d, tb, nc, nj);
      else if (ptok == 0) tally_iteration<1>(lt, L.tbth, p.tbt_w, K, d, tb, nc, nj);
      else tally_iteration<2>(lt, L.tbth, p.tbt_w, K, d, tb, nc, nj);
      lv.k = -1;
      pe.done = false;
      const bool mixed_now = rem > 0;
      const int nd_before = nd;
      if (quads) {
        // Highest slot first, so the slot moved into a hole has already been checked.
        uint32_t *frow = fin + static_cast<size_t>(g) * BS;
        uint64_t *jrow = job + static_cast<size_t>(g) * BS;
        while (quads) {
          const int q = 31 - __clz(quads);
          quads &= ~(1u << q);
          const uint4 v = *reinterpret_cast<const uint4 *>(frow + 4 * q);
          const uint32_t wv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
          for (int w = 3; w >= 0; --w) {
            const int j = 4 * q + w;
            if (j < nd && wv[w] == it) {
              const uint64_t jw = jrow[j];
              const int k = static_cast<int>(jw >> 29) & 7;
              const uint32_t stamp = static_cast<uint32_t>(jw) & 0x1FFFFFFFu;
              const uint32_t Pl = (static_cast<uint32_t>(jw >> 32) & 0xFFFFu) + 1, Dl = static_cast<uint32_t>(jw >> 48) + 1;
              const int64_t e2e = tn - (static_cast<int64_t>(stamp) + 1) * p.dt;
              if (lv.k < 0) { lv.k = k; lv.P = Pl; lv.D = Dl; lv.e2e = e2e; lv.mixed = mixed_now; }
              else leave_direct(k, Pl, Dl, e2e, mixed_now);
              atomicAdd(reinterpret_cast<unsigned long long *>(&hist[(1 * K + k) * kNBin + hbin(e2e)]), 1ull);
              nc -= 1ull << (8 * k);
              --nd;
              if (j < nd) { frow[j] = frow[nd]; jrow[j] = jrow[nd]; }
            }
          }
        }
        if (nd != nd_before) {
          n_cls[g] = nc;
          L.loads[g] = static_cast<uint8_t>(nd);
          const int hb = g < M ? kLoadBins : 0;
          atomicSub(&L.lh[hb + nd_before], 1u);
          atomicAdd(&L.lh[hb + nd], 1u);
        }
      }
      // the prefill advances by the chunk frozen at the start of the iteration
      if (ptok > 0) {
        const int k = pk_cls(pk);
        rem -= ptok;
        if (rem == 0) {
          const uint64_t jw = pf_job[g];
          const uint32_t stamp = static_cast<uint32_t>(jw) & 0x1FFFFFFFu;
          pe.done = true; pe.k = k; pe.nc = nc;
          pe.P = (static_cast<uint32_t>(jw >> 32) & 0xFFFFu) + 1;
          pe.ttft = tn - (static_cast<int64_t>(stamp) + 1) * p.dt;
          atomicAdd(reinterpret_cast<unsigned long long *>(&hist[(0 * K + k) * kNBin + hbin(pe.ttft)]), 1ull);
        }
        // running chunk cleared; it is set again at the restart
        remptok[g] = static_cast<uint32_t>(rem) | (static_cast<uint32_t>(k) << 29);
      }
      if (nj) n_join[g] = 0;
    };
    // class-level effects of the decodes that left (one per lane), folded over the wave
    auto fold_leaving = [&](const Leaving &lv) __attribute__((always_inline)) {
      const bool any = lv.k >= 0;
      if (__ballot(any) == 0) return;
      const bool am = any && lv.mixed, as = any && !lv.mixed;
      wave_count_by_class(am, lv.k, K, &L.tl[SIM_T_S_DM], kNTally);
      wave_count_by_class(as, lv.k, K, &L.tl[SIM_T_S_DS], kNTally);
      wave_count_by_class_i32(am, lv.k, K, &L.cs[CS_YM], -1);
      wave_count_by_class_i32(as, lv.k, K, &L.cs[CS_YS], -1);
      wave_sum_by_class(any, lv.k, K, lv.P, &L.tl[SIM_T_TOKP_DEC], kNTally);
      wave_sum_by_class(any, lv.k, K, lv.D, &L.tl[SIM_T_TOKD_DEC], kNTally);
      wave_sum_by_class(any, lv.k, K, static_cast<uint64_t>(lv.e2e), &L.tl[SIM_T_E2E_SUM], kNTally);
    };
    // class-level effects of the prefills that ended: completion counts, recognised prompt tokens,
    // time to first token; the co-resident decodes switch mixed -> solo
    auto fold_prefill_end = [&](const PrefillEnd &pe) __attribute__((always_inline)) {
      if (__ballot(pe.done) == 0) return;
      wave_count_by_class(pe.done, pe.k, K, &L.tl[SIM_T_S_P], kNTally);
      wave_count_by_class_i32(pe.done, pe.k, K, &L.cs[CS_X], -1);
      wave_sum_by_class(pe.done, pe.k, K, pe.P, &L.tl[SIM_T_TOKP_PRE], kNTally);
      wave_sum_by_class(pe.done, pe.k, K, static_cast<uint64_t>(pe.ttft), &L.tl[SIM_T_TTFT_SUM], kNTally);
      uint64_t even, odd;
      wave_sum_bytes(pe.done ? pe.nc : 0ull, even, odd);
      if (lane == 0)
        for (int c = 0; c < K; ++c) {
          const int v = static_cast<int>(class_field(even, odd, c));
          if (v) {
            lds_add64(&L.tl[c * kNTally + SIM_T_M_MS], static_cast<uint64_t>(v));
            atomicSub(&L.cs[CS_YM + c], v);
            atomicAdd(&L.cs[CS_YS + c], v);
          }
        }
    };
    // the same effects for a single server, without folding (divergent callers)
    auto commit_direct = [&](const Leaving &lv, const PrefillEnd &pe) __attribute__((always_inline)) {
      if (lv.k >= 0) leave_direct(lv.k, lv.P, lv.D, lv.e2e, lv.mixed);
      if (pe.done) {
        lds_add64(&L.tl[pe.k * kNTally + SIM_T_S_P], 1);
        atomicSub(&L.cs[CS_X + pe.k], 1);
        lds_add64(&L.tl[pe.k * kNTally + SIM_T_TOKP_PRE], pe.P);
        lds_add64(&L.tl[pe.k * kNTally + SIM_T_TTFT_SUM], static_cast<uint64_t>(pe.ttft));
        for (int c = 0; c < K; ++c) {
          const int v = static_cast<int>(byte_at(pe.nc, c));
          if (v) {
            lds_add64(&L.tl[c * kNTally + SIM_T_M_MS], static_cast<uint64_t>(v));
            atomicSub(&L.cs[CS_YM + c], v);
            atomicAdd(&L.cs[CS_YS + c], v);
          }
        }
      }
    };

    // a server whose finishing was put off because decodes leave it: reload its record and finish it
    auto finish_deferred = [&](int g, uint32_t quads, Leaving &lv, PrefillEnd &pe) __attribute__((always_inline)) {
      const uint64_t nc = n_cls[g];
      const bool joined = (L.bm_join[g >> 6] >> (g & 63)) & 1ull;
      const uint64_t nj = joined ? n_join[g] : 0ull;
      const uint32_t pk = g < M ? remptok[g] : 0u;
      finish_iteration(g, L.iter[g], L.loads[g], nc, nj, pk, L.t32[g], quads, lv, pe);
      if (pe.done) {
        atomicOr(reinterpret_cast<unsigned long long *>(&L.bm_comp[g >> 6]), 1ull << (g & 63));
        atomicOr(reinterpret_cast<unsigned long long *>(&L.bm_idle[g >> 6]), 1ull << (g & 63));
      }
      if (joined) atomicAnd(reinterpret_cast<unsigned long long *>(&L.bm_join[g >> 6]), ~(1ull << (g & 63)));
    };

    // which servers of round i are due, and their records (global loads are issued, not waited for)
    auto probe = [&](int i) __attribute__((always_inline)) -> RoundState {
      RoundState st;
      st.due = false; st.t32 = 0; st.it = 0; st.nd = 0; st.nc = 0; st.nj = 0; st.pk = 0; st.due_mask = 0; st.join_word = 0;
      const int gw = i * NT + wave_base;
      if (gw < N) {
        const int g = gw + lane;
        const bool valid = g < N;
        const uint64_t busy_word = L.bm_busy[gw >> 6];
        st.join_word = L.bm_join[gw >> 6];
        st.t32 = valid ? L.t32[g] : 0u;
        st.due = valid && ((busy_word >> lane) & 1ull) && static_cast<int32_t>(st.t32 - T32) <= 0;
        st.due_mask = __ballot(st.due);
        if (st.due) {
          st.it = L.iter[g] + 1;
          L.iter[g] = st.it;
          st.nd = L.loads[g];
          st.nc = n_cls[g];
          if ((st.join_word >> lane) & 1ull) st.nj = n_join[g];
          if (g < M) st.pk = remptok[g];
        }
      }
      return st;
    };

    int nev = 0;   // completions queued by this wave (wave-uniform)
    RoundState nx = probe(0);
    PROF(1)
    for (int i = 0; i < nper; ++i) {
      const int gw = i * NT + wave_base;          // first server of this wave's 64-server block
      if (gw >= N) break;                         // wave-uniform
      const int wi = gw >> 6;
      const int g = gw + lane;
      const RoundState cur = nx;
      if (i + 1 < nper) nx = probe(i + 1);        // next round's records travel while this round is scanned
      PROF(2)
      uint32_t quads = 0;   // owner lane: bit q set <=> one of slots 4q..4q+3 finishes now
      if (cur.due_mask) {
        // ---- cooperative scan of the slot rows: half a wave reads one server's row (4 words per lane)
        uint64_t todo = __ballot(cur.due && cur.nd > 0);
        const int q = lane & 31;
        const bool hi = lane >= 32;
        bool first_batch = true;
        do {
          int la[4], lb[4];
          bool va[4], vb[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            va[u] = todo != 0;
            la[u] = va[u] ? __ffsll(static_cast<long long>(todo)) - 1 : 0;
            if (va[u]) todo &= todo - 1;
            vb[u] = todo != 0;
            lb[u] = vb[u] ? __ffsll(static_cast<long long>(todo)) - 1 : 0;
            if (vb[u]) todo &= todo - 1;
          }
          uint4 v[4];
          uint32_t its[4];
          int nds[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const uint32_t ita = __builtin_amdgcn_readlane(cur.it, la[u]), itb = __builtin_amdgcn_readlane(cur.it, lb[u]);
            const int nda = __builtin_amdgcn_readlane(cur.nd, la[u]), ndb = __builtin_amdgcn_readlane(cur.nd, lb[u]);
            const bool on = hi ? vb[u] : va[u];
            its[u] = hi ? itb : ita;
            nds[u] = on ? (hi ? ndb : nda) : 0;
            const int gs = gw + (hi ? lb[u] : la[u]);
            v[u] = make_uint4(0u, 0u, 0u, 0u);
            if (4 * q < nds[u]) v[u] = *reinterpret_cast<const uint4 *>(fin + static_cast<size_t>(gs) * BS + 4 * q);
          }
          if (first_batch) {   // the arrival draws of this round run while the first rows travel
            if (g < N) arrivals(g);
            first_batch = false;
          }
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int left = nds[u] - 4 * q;   // occupied words of this lane's quad
            const bool m = (left > 0 && v[u].x == its[u]) || (left > 1 && v[u].y == its[u]) ||
                           (left > 2 && v[u].z == its[u]) || (left > 3 && v[u].w == its[u]);
            const uint64_t hit = __ballot(m);
            if (hit) {
              if (va[u] && lane == la[u]) quads = static_cast<uint32_t>(hit);
              if (vb[u] && lane == lb[u]) quads = static_cast<uint32_t>(hit >> 32);
            }
          }
        } while (todo);
      } else if (g < N) {
        arrivals(g);
      }
      PROF(3)
      const bool deferred = cur.due && quads != 0;
      Leaving lv; lv.k = -1;
      PrefillEnd pe; pe.done = false;
      if (cur.due && quads == 0) finish_iteration(g, cur.it, cur.nd, cur.nc, cur.nj, cur.pk, cur.t32, 0u, lv, pe);
      fold_prefill_end(pe);
      const uint64_t done = __ballot(pe.done), later = __ballot(deferred);
      if (later) {   // queue the servers that have decodes leaving; they are finished after the pass
        const int slot = nev + __popcll(later & lanes_below());
        if (deferred) {
          if (slot < kEvPerWave) { ev_g[slot] = static_cast<uint32_t>(g); ev_q[slot] = quads; }
          else { Leaving l2; PrefillEnd p2; finish_deferred(g, quads, l2, p2); commit_direct(l2, p2); }
        }
        nev += __popcll(later);
        if (nev > kEvPerWave) nev = kEvPerWave;
      }
      if (lane == 0) {
        L.bm_due[wi] = cur.due_mask;
        L.bm_touch[wi] = 0;
        L.bm_comp[wi] = done;
        if (done) L.bm_idle[wi] |= done;
        const uint64_t nj_word = cur.join_word & ~(cur.due_mask & ~later);
        if (nj_word != cur.join_word) L.bm_join[wi] = nj_word;
      }
      PROF(4)
    }
    for (int e0 = 0; e0 < nev; e0 += 64) {   // the queued servers, one per lane
      const int e = e0 + lane;
      Leaving lv; lv.k = -1;
      PrefillEnd pe; pe.done = false;
      if (e < nev) finish_deferred(static_cast<int>(ev_g[e]), ev_q[e], lv, pe);
      fold_leaving(lv);
      fold_prefill_end(pe);
    }
    // fold this step's per-lane sums into the workgroup tallies
    {
      const uint32_t i0 = wave_sum32(lt.iters[0]), i1 = wave_sum32(lt.iters[1]);
      const uint64_t b0 = wave_sum64(lt.busy[0]), b1 = wave_sum64(lt.busy[1]);
      if (lane == 0) {
        if (i0) { lds_add64(&L.tl[kMaxK * kNTally + SIM_G_ITERS_SOLO], i0); lds_add64(&L.tl[kMaxK * kNTally + SIM_G_BUSY_SOLO], b0); }
        if (i1) { lds_add64(&L.tl[kMaxK * kNTally + SIM_G_ITERS_MIX], i1); lds_add64(&L.tl[kMaxK * kNTally + SIM_G_BUSY_MIX], b1); }
      }
#pragma unroll
      for (int k = 0; k < kMaxK; ++k) {
        if (k >= K) continue;
        const uint64_t ts = wave_sum64(lt.tbt_sum[k]);
        if (lane == 0 && ts) lds_add64(&L.tl[k * kNTally + SIM_T_TBT_SUM], ts);
      }
    }
    PROF(5)
    __syncthreads();
    PROF(6)

    // ================= arrivals into the class queues; ranks of completions and idle slots =================
    if (tid < K) {
      const int k = tid;
      const uint32_t a = L.acc[k];
      const uint32_t room = p.queue_cap - static_cast<uint32_t>(L.cs[CS_QP + k]);
      const uint32_t take = a < room ? a : room;
      uint32_t tail = static_cast<uint32_t>(L.cs[CS_QHEAD + k]) + static_cast<uint32_t>(L.cs[CS_QP + k]);
      if (tail >= p.queue_cap) tail -= p.queue_cap;
      L.sc[SC_TAKE + k] = static_cast<int32_t>(take);
      L.sc[SC_TAIL + k] = static_cast<int32_t>(tail);
      L.cs[CS_QP + k] += static_cast<int32_t>(take);
      L.tl[k * kNTally + SIM_T_A] += take;
      L.tl[k * kNTally + SIM_T_DROP_P] += a - take;
      if (a > take) L.tl[kMaxK * kNTally + SIM_G_OVERFLOW] = 1;
    }
    if (tid < 64) {
      const uint32_t ncomp = rank_bitmap(L.bm_comp, L.pre_c, nwords_m);
      if (tid == 0) L.sc[SC_NCOMP] = static_cast<int32_t>(ncomp);
    }
    if (NT == 64 ? tid < 64 : (tid >= 64 && tid < 128)) {
      const uint32_t nidle = rank_bitmap(L.bm_idle, L.pre, nwords_m);
      if (lane == 0) L.sc[SC_NIDLE] = static_cast<int32_t>(nidle);
    }
    __syncthreads();
    for (int k = 0; k < K; ++k) {
      const uint32_t take = static_cast<uint32_t>(L.sc[SC_TAKE + k]), tail = static_cast<uint32_t>(L.sc[SC_TAIL + k]);
      for (uint32_t j = tid; j < take; j += NT) {
        uint32_t pos = tail + j;
        if (pos >= p.queue_cap) pos -= p.queue_cap;
        qring[static_cast<size_t>(k) * p.queue_cap + pos] = s;
      }
    }
    // completed prefills join the decode buffer in ascending server order
    {
      const uint32_t ncomp = static_cast<uint32_t>(L.sc[SC_NCOMP]);
      const uint32_t dcount = static_cast<uint32_t>(L.cs[CS_DCOUNT]), dhead = static_cast<uint32_t>(L.cs[CS_DHEAD]);
      for (uint32_t j0 = wave_base; j0 < ncomp; j0 += NT) {   // wave-uniform trip count
        const uint32_t j = j0 + lane;
        const bool active = j < ncomp;
        int k = 0;
        bool kept = false;
        if (active) {
          const int g = select_bit(L.bm_comp, L.pre_c, nwords_m, j);
          const uint64_t jw = pf_job[g];
          k = static_cast<int>(jw >> 29) & 7;
          kept = dcount + j < p.dbuf_cap;
          if (kept) {
            uint32_t pos = dhead + dcount + j;
            if (pos >= p.dbuf_cap) pos -= p.dbuf_cap;
            dring[pos] = jw;
          }
        }
        wave_count_by_class_i32(active && kept, k, K, &L.cs[CS_QD], 1);
        if (__ballot(active && !kept)) {
          wave_count_by_class(active && !kept, k, K, &L.tl[SIM_T_DROP_D], kNTally);
          if (lane == 0) L.tl[kMaxK * kNTally + SIM_G_OVERFLOW] = 1;
        }
      }
    }
    PROF(7)

    // ================= 3. prefill gate =================
    // The m-th waiting request of class k is a candidate; its position in the admission sequence is
    // the number of candidates that sort before it. Candidates are ranked in parallel; the idle
    // prefill slot of rank j (ascending server index) takes the candidate of rank j.
    for (bool first = true;; first = false) {
      if (!first) {
        if (tid < 64) {
          const uint32_t nidle = rank_bitmap(L.bm_idle, L.pre, nwords_m);
          if (tid == 0) L.sc[SC_NIDLE] = static_cast<int32_t>(nidle);
        }
        __syncthreads();
      }
      if (p.gate_mode == SIM_GATE_FCFS && first) __syncthreads();   // stamps written above are read below
      const int nidle = L.sc[SC_NIDLE];
      const int limit = nidle < kAdmChunk ? nidle : kAdmChunk;
      int cnt[kMaxK], xs[kMaxK], qp[kMaxK], ncand = 0;
      uint32_t head[kMaxK];
#pragma unroll
      for (int k = 0; k < kMaxK; ++k) {
        qp[k] = k < K ? L.cs[CS_QP + k] : 0;
        xs[k] = k < K ? L.cs[CS_X + k] : 0;
        head[k] = k < K ? static_cast<uint32_t>(L.cs[CS_QHEAD + k]) : 0u;
        const bool eligible = k < K && qp[k] > 0 && (p.gate_mode != SIM_GATE_OCCUPANCY || p.invx[k] > 0.0);
        cnt[k] = eligible ? (qp[k] < limit ? qp[k] : limit) : 0;
        ncand += cnt[k];
      }
      const int nadm = ncand < limit ? ncand : limit;
      for (int c = tid; c < ncand; c += NT) {
        int k = 0, m = c;
#pragma unroll
        for (int kk = 0; kk < kMaxK - 1; ++kk)
          if (k == kk && m >= cnt[kk]) { m -= cnt[kk]; k = kk + 1; }
        GateKey key = {0.0, 0.0};
#pragma unroll
        for (int kk = 0; kk < kMaxK; ++kk)
          if (k == kk) key = gate_key(p, qring, xs, qp, head, kk, m);
        int rank = m;
#pragma unroll
        for (int k2 = 0; k2 < kMaxK; ++k2) {
          if (k2 == k || cnt[k2] == 0 || rank >= nadm) continue;
          int lo = 0, hi = cnt[k2];
          while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (gate_before(gate_key(p, qring, xs, qp, head, k2, mid), k2, key, k)) lo = mid + 1; else hi = mid;
          }
          rank += lo;
        }
        if (rank < nadm) {
          L.adm[rank] = static_cast<uint32_t>(k) | (static_cast<uint32_t>(m) << 3);
          atomicAdd(&L.sc[SC_ADMK + k], 1);
        }
      }
      PROF(14)
      __syncthreads();
      PROF(15)
      if (first && tid == 0) {   // every thread has read the old count by now: completions are in the buffer
        const uint32_t room = p.dbuf_cap - static_cast<uint32_t>(L.cs[CS_DCOUNT]);
        const uint32_t ncp = static_cast<uint32_t>(L.sc[SC_NCOMP]);
        L.cs[CS_DCOUNT] += static_cast<int32_t>(ncp < room ? ncp : room);
      }
      // admission j goes to the idle prefill slot of rank j; one thread per admission
      for (int j0 = wave_base; j0 < nadm; j0 += NT) {   // wave-uniform trip count
        const int j = j0 + lane;
        const bool active = j < nadm;
        int k = 0;
        uint64_t wait = 0, nc = 0;
        if (active) {
          const int g = select_bit(L.bm_idle, L.pre, nwords_m, static_cast<uint32_t>(j));
          const uint32_t e = L.adm[j];
          k = static_cast<int>(e & 7u);
          uint32_t pos = head[0];
#pragma unroll
          for (int kk = 1; kk < kMaxK; ++kk) pos = k == kk ? head[kk] : pos;
          pos += e >> 3;
          if (pos >= p.queue_cap) pos -= p.queue_cap;
          const uint32_t stamp = qring[static_cast<size_t>(k) * p.queue_cap + pos];
          if (L.loads[g]) nc = n_cls[g];
          wait = static_cast<uint64_t>(s - stamp);
          uint32_t w[4];
          philox4x32_10(key0, key1, s, 1u, static_cast<uint32_t>(g), static_cast<uint32_t>(r), w);
          const uint32_t Pl = p.len_tab[(static_cast<size_t>(k) * 2 + 0) * kTableSize + (w[0] >> 16)];
          const uint32_t Dl = p.len_tab[(static_cast<size_t>(k) * 2 + 1) * kTableSize + (w[1] >> 16)];
          pf_job[g] = static_cast<uint64_t>(stamp) | (static_cast<uint64_t>(k) << 29) |
                      (static_cast<uint64_t>(Pl - 1) << 32) | (static_cast<uint64_t>(Dl - 1) << 48);
          // an idle prefill slot implies that the running iteration holds no chunk
          remptok[g] = Pl | (static_cast<uint32_t>(k) << 29);
          const uint64_t bit = 1ull << (g & 63);
          atomicAnd(reinterpret_cast<unsigned long long *>(&L.bm_idle[g >> 6]), ~bit);
          if (!(L.bm_busy[g >> 6] & bit)) atomicOr(reinterpret_cast<unsigned long long *>(&L.bm_touch[g >> 6]), bit);
        }
        wave_sum_by_class(active, k, K, wait, &L.tl[SIM_T_WAIT_STEPS], kNTally);
        uint64_t even, odd;   // co-resident decodes switch solo -> mixed
        wave_sum_bytes(nc, even, odd);
        if (lane == 0 && (even | odd))
          for (int c = 0; c < K; ++c) {
            const int v = static_cast<int>(class_field(even, odd, c));
            if (v) {
              lds_add64(&L.tl[c * kNTally + SIM_T_M_SM], static_cast<uint64_t>(v));
              atomicSub(&L.cs[CS_YS + c], v);
              atomicAdd(&L.cs[CS_YM + c], v);
            }
          }
      }
      bool more = false;
      if (nadm == kAdmChunk && nidle > kAdmChunk) {   // rare: more idle slots than one pass serves
#pragma unroll
        for (int k = 0; k < kMaxK; ++k)
          if (k < K && cnt[k] > 0 && qp[k] - L.sc[SC_ADMK + k] > 0) more = true;
      }
      __syncthreads();
      if (tid < K) {   // class counters follow the admissions of this pass
        const int k = tid, a = L.sc[SC_ADMK + k];
        if (a) {
          uint32_t h = static_cast<uint32_t>(L.cs[CS_QHEAD + k]) + static_cast<uint32_t>(a);
          if (h >= p.queue_cap) h -= p.queue_cap;
          L.cs[CS_QHEAD + k] = static_cast<int32_t>(h);
          L.cs[CS_QP + k] -= a;
          L.cs[CS_X + k] += a;
          L.tl[k * kNTally + SIM_T_U_P] += static_cast<uint64_t>(a);
          L.sc[SC_ADMK + k] = 0;
        }
      }
      if (!more) break;
      __syncthreads();
    }
    PROF(8)

    // ================= 4. decode routing =================
    // Each pass serves the servers at the lowest decode count of the group, in index order; the job
    // of rank j in the decode buffer goes to the j-th of them. Every wave derives the pass parameters
    // from the load histogram, so no thread has to broadcast them.
    {
      int jrem = L.cs[CS_DCOUNT], next = 0;
      const uint32_t dhead0 = static_cast<uint32_t>(L.cs[CS_DHEAD]);
      for (int grp = 0; grp < 2 && jrem > 0; ++grp) {
        const int lo = grp == 0 ? M : 0, hi = grp == 0 ? N : M;
        const int capg = grp == 0 ? B : B - 1;
        if (lo >= hi) continue;
        for (;;) {
          if (jrem <= 0) break;
          // lowest non-empty level below the cap, and the number of servers on it
          int level = -1, cnt = 0;
          for (int base = 0; base < capg && level < 0; base += 64) {
            const int l = base + lane;
            const uint32_t c = l < capg ? L.lh[grp * kLoadBins + l] : 0u;
            const uint64_t nz = __ballot(c != 0);
            if (nz) {
              const int first = __ffsll(static_cast<long long>(nz)) - 1;
              level = base + first;
              cnt = static_cast<int>(__builtin_amdgcn_readlane(c, first));
            }
          }
          if (level < 0) break;
          const int take = cnt < jrem ? cnt : jrem;
          for (int i = 0; i < nper; ++i) {
            const int gw = i * NT + wave_base;
            if (gw >= N) break;
            const int g = gw + lane;
            const bool at_level = g >= lo && g < hi && L.loads[g] == level;
            const uint64_t b = __ballot(at_level);
            if (lane == 0) L.bm_lvl[gw >> 6] = b;
          }
          __syncthreads();
          if (tid < 64) rank_bitmap(L.bm_lvl, L.pre, p.nwords);
          __syncthreads();
          for (int j0 = wave_base; j0 < take; j0 += NT) {   // wave-uniform trip count
            const int j = j0 + lane;
            const bool active = j < take;
            int k = 0;
            bool has_prefill = false;
            if (active) {
              const int g = select_bit(L.bm_lvl, L.pre, p.nwords, static_cast<uint32_t>(j));
              uint32_t pos = dhead0 + static_cast<uint32_t>(next + j);
              if (pos >= p.dbuf_cap) pos -= p.dbuf_cap;
              if (pos >= p.dbuf_cap) pos -= p.dbuf_cap;
              const uint64_t jw = dring[pos];
              k = static_cast<int>(jw >> 29) & 7;
              const uint32_t Dl = static_cast<uint32_t>(jw >> 48) + 1;
              const uint64_t bit = 1ull << (g & 63);
              const bool busy = L.bm_busy[g >> 6] & bit;
              const bool mid = busy && !(L.bm_due[g >> 6] & bit);   // joins at the next restart
              const int nd = level;
              fin[static_cast<size_t>(g) * BS + nd] = L.iter[g] + Dl + (mid ? 1u : 0u);
              job[static_cast<size_t>(g) * BS + nd] = jw;
              n_cls[g] += 1ull << (8 * k);
              if (mid) {
                n_join[g] += 1ull << (8 * k);
                atomicOr(reinterpret_cast<unsigned long long *>(&L.bm_join[g >> 6]), bit);
              }
              L.loads[g] = static_cast<uint8_t>(nd + 1);
              has_prefill = g < M && pk_rem(remptok[g]) != 0;
              if (!busy) atomicOr(reinterpret_cast<unsigned long long *>(&L.bm_touch[g >> 6]), bit);
            }
            const bool am = active && has_prefill, as = active && !has_prefill;
            wave_count_by_class(am, k, K, &L.tl[SIM_T_U_DM], kNTally);
            wave_count_by_class(as, k, K, &L.tl[SIM_T_U_DS], kNTally);
            wave_count_by_class_i32(am, k, K, &L.cs[CS_YM], 1);
            wave_count_by_class_i32(as, k, K, &L.cs[CS_YS], 1);
            wave_count_by_class_i32(active, k, K, &L.cs[CS_QD], -1);
          }
          __syncthreads();
          if (tid == 0) {   // `take` servers moved up one level
            L.lh[grp * kLoadBins + level] -= static_cast<uint32_t>(take);
            L.lh[grp * kLoadBins + level + 1] += static_cast<uint32_t>(take);
          }
          jrem -= take;
          next += take;
          __syncthreads();
        }
      }
      if (tid == 0 && next > 0) {
        uint32_t h = dhead0 + static_cast<uint32_t>(next);
        if (h >= p.dbuf_cap) h -= p.dbuf_cap;
        L.cs[CS_DHEAD] = static_cast<int32_t>(h);
        L.cs[CS_DCOUNT] -= next;
      }
    }
    PROF(9)

    // ================= 5. (re)start =================
    for (int i = 0; i < nper; ++i) {
      const int gw = i * NT + wave_base;
      if (gw >= N) break;
      const int wi = gw >> 6;
      const uint64_t due_word = L.bm_due[wi];
      const uint64_t todo = due_word | L.bm_touch[wi];
      if (todo == 0) continue;
      const int g = gw + lane;
      const uint64_t busy_word = L.bm_busy[wi];
      bool busy = (busy_word >> lane) & 1ull;
      if ((todo >> lane) & 1ull) {
        const uint32_t pk = g < M ? remptok[g] : 0u;
        const int rem = pk_rem(pk);
        const int ptok = rem > 0 ? (rem < p.C ? rem : p.C) : 0;
        const int n = L.loads[g];
        if (ptok == 0 && n == 0) {
          busy = false;
        } else {
          // back-to-back after a completion, otherwise from the step boundary
          const int64_t base = ((due_word >> lane) & 1ull) ? T + static_cast<int64_t>(static_cast<int32_t>(L.t32[g] - T32)) : T;
          const int64_t tn = base + p.c0 + p.cpre * ptok + p.cdec * static_cast<int64_t>(n);
          L.t32[g] = static_cast<uint32_t>(tn);
          busy = true;
          if (ptok > 0) remptok[g] = pk | (static_cast<uint32_t>(ptok) << 16);
        }
      }
      const uint64_t nb = __ballot(busy);
      if (lane == 0 && nb != busy_word) L.bm_busy[wi] = nb;
    }
    PROF(10)

    // ================= 6. end-of-step occupancy integrals =================
    if (tid < K) {
      const int k = tid;
      L.tl[k * kNTally + SIM_T_SUM_QP] += static_cast<uint64_t>(L.cs[CS_QP + k]);
      L.tl[k * kNTally + SIM_T_SUM_QD] += static_cast<uint64_t>(L.cs[CS_QD + k]);
      L.tl[k * kNTally + SIM_T_SUM_X] += static_cast<uint64_t>(L.cs[CS_X + k]);
      L.tl[k * kNTally + SIM_T_SUM_YM] += static_cast<uint64_t>(L.cs[CS_YM + k]);
      L.tl[k * kNTally + SIM_T_SUM_YS] += static_cast<uint64_t>(L.cs[CS_YS + k]);
    }
    if (tid == 0) L.tl[kMaxK * kNTally + SIM_G_STEPS] += 1;
  }
  PROF_FLUSH

  // ---- write out the cached time-between-tokens counts; the emitted-token tally is their total
#pragma unroll
  for (int k = 0; k < kMaxK; ++k) {
    if (k >= K) continue;
    if (lt.hist_cnt[0][k]) lds_add64(&L.tbth[k * p.tbt_w + lt.hist_bin[0]], lt.hist_cnt[0][k]);
    if (lt.hist_cnt[1][k]) lds_add64(&L.tbth[k * p.tbt_w + lt.hist_bin[1]], lt.hist_cnt[1][k]);
    if (lt.hist_cnt[2][k]) lds_add64(&L.tbth[k * p.tbt_w + lt.hist_bin[2]], lt.hist_cnt[2][k]);
  }
  __syncthreads();
  if (tid < K) {
    uint64_t tot = 0;
    for (int b = 0; b < p.tbt_w; ++b) tot += L.tbth[tid * p.tbt_w + b];
    L.tl[tid * kNTally + SIM_T_TOK_EMIT] += tot;
  }
  __syncthreads();

  // ---- write the server clocks and the class state back; add this launch's tallies to the totals
  if (tid < 8) L.acc[tid] = 0;
  __syncthreads();
  for (int i = 0; i < nper; ++i) {
    const int g = i * NT + tid;
    if (g >= N) break;
    const bool busy = (L.bm_busy[g >> 6] >> (g & 63)) & 1ull;
    t_next[g] = busy ? T + static_cast<int64_t>(static_cast<int32_t>(L.t32[g] - static_cast<uint32_t>(T))) : kIdle;
    iter_g[g] = L.iter[g];
    if (g < M) {   // prompt tokens already processed of the prefill in service
      const uint32_t pk = remptok[g];
      if (pk_rem(pk)) {
        const uint32_t Pl = (static_cast<uint32_t>(pf_job[g] >> 32) & 0xFFFFu) + 1;
        atomicAdd(&L.acc[pk_cls(pk)], Pl - static_cast<uint32_t>(pk_rem(pk)));
      }
    }
  }
  for (int i = tid; i < CS_WORDS; i += NT) p.cstate[static_cast<size_t>(r) * CS_WORDS + i] = L.cs[i];
  uint64_t *gt = p.tally + static_cast<size_t>(r) * kTallyWords;
  for (int i = tid; i < kTallyWords; i += NT) {
    if (i == kMaxK * kNTally + SIM_G_OVERFLOW) gt[i] |= L.tl[i]; else gt[i] += L.tl[i];
  }
  for (int i = tid; i < K * p.tbt_w; i += NT) {
    const int k = i / p.tbt_w, b = i % p.tbt_w;
    if (L.tbth[i]) hist[(2 * K + k) * kNBin + p.tbt_lo + b] += L.tbth[i];
  }
  __syncthreads();
  // prompt tokens processed so far = prompt tokens of completed prefills + progress of those in service
  if (tid < K) gt[tid * kNTally + SIM_T_TOK_PREF] = gt[tid * kNTally + SIM_T_TOKP_PRE] + L.acc[tid];
}

// ------------------------------------------------------------------ reset ----
__global__ void gnr_reset_kernel(const Params p, const int reps)
{
  const size_t n_srv = static_cast<size_t>(reps) * p.N;
  const size_t stride = static_cast<size_t>(gridDim.x) * blockDim.x;
  const size_t t0 = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  for (size_t i = t0; i < n_srv; i += stride) {
    p.t_next[i] = kIdle; p.iter[i] = 0; p.remptok[i] = 0; p.pf_job[i] = 0; p.n_cls[i] = 0; p.n_join[i] = 0;
  }
  for (size_t i = t0; i < static_cast<size_t>(reps) * CS_WORDS; i += stride) p.cstate[i] = 0;
  for (size_t i = t0; i < static_cast<size_t>(reps) * kTallyWords; i += stride) p.tally[i] = 0;
  for (size_t i = t0; i < static_cast<size_t>(reps) * 3 * p.K * kNBin; i += stride) p.hist[i] = 0;
}

// ------------------------------------------------------------------ reduce ----
// Totals over replications, each output element summed in replication order.
__global__ void gnr_reduce_kernel(const Params p, const int reps)
{
  const int nh = 3 * p.K * kNBin;
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < kTallyWords) {
    uint64_t acc = 0;
    for (int r = 0; r < reps; ++r) acc += p.tally[static_cast<size_t>(r) * kTallyWords + i];
    p.reduced[i] = acc;
  } else if (i < kTallyWords + nh) {
    const int h = i - kTallyWords;
    uint64_t acc = 0;
    for (int r = 0; r < reps; ++r) acc += p.hist[static_cast<size_t>(r) * nh + h];
    p.reduced[i] = acc;
  }
}

// ------------------------------------------------------------------ digest ----
// Sum mod 2^64 of a chained 64-bit finaliser (Steele-Lea-Flood / Vigna splitmix64 output
// function) over tagged items of the integer state; slot items ignore the slot position.
__device__ __forceinline__ uint64_t mix64(uint64_t z)
{
  z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
  z ^= z >> 27; z *= 0x94D049BB133111EBull;
  z ^= z >> 31;
  return z;
}
__device__ __forceinline__ uint64_t chain(uint64_t h, uint64_t w) { return mix64(h + w + 0x9E3779B97F4A7C15ull); }

__global__ void gnr_digest_kernel(const Params p)
{
  __shared__ unsigned long long total;
  const int r = blockIdx.x, tid = threadIdx.x, NT = blockDim.x;
  const int K = p.K, N = p.N;
  if (tid == 0) total = 0;
  __syncthreads();
  const int32_t *cs = p.cstate + static_cast<size_t>(r) * CS_WORDS;
  uint64_t d = 0;
  if (tid < K) {
    const int k = tid;
    uint64_t h = chain(1, static_cast<uint64_t>(k));
    h = chain(h, static_cast<uint64_t>(static_cast<int64_t>(cs[CS_QP + k])));
    h = chain(h, static_cast<uint64_t>(static_cast<int64_t>(cs[CS_X + k])));
    h = chain(h, static_cast<uint64_t>(static_cast<int64_t>(cs[CS_QD + k])));
    h = chain(h, static_cast<uint64_t>(static_cast<int64_t>(cs[CS_YM + k])));
    h = chain(h, static_cast<uint64_t>(static_cast<int64_t>(cs[CS_YS + k])));
    d += h;
  }
  for (int k = 0; k < K; ++k) {
    const uint32_t head = static_cast<uint32_t>(cs[CS_QHEAD + k]), len = static_cast<uint32_t>(cs[CS_QP + k]);
    const uint32_t *ring = p.qring + (static_cast<size_t>(r) * K + k) * p.queue_cap;
    for (uint32_t i = tid; i < len; i += NT) {
      uint32_t pos = head + i;
      if (pos >= p.queue_cap) pos -= p.queue_cap;
      d += chain(chain(chain(2, static_cast<uint64_t>(k)), i), ring[pos]);
    }
  }
  {
    const uint32_t head = static_cast<uint32_t>(cs[CS_DHEAD]), len = static_cast<uint32_t>(cs[CS_DCOUNT]);
    const uint64_t *ring = p.dring + static_cast<size_t>(r) * p.dbuf_cap;
    for (uint32_t i = tid; i < len; i += NT) {
      uint32_t pos = head + i;
      if (pos >= p.dbuf_cap) pos -= p.dbuf_cap;
      d += chain(chain(3, i), ring[pos]);
    }
  }
  for (int g = tid; g < N; g += NT) {
    const size_t sg = static_cast<size_t>(r) * N + g;
    const uint32_t pk = p.remptok[sg];
    const uint32_t rem = pk & 0xFFFFu;
    const uint32_t ptok = (pk >> 16) & 0x1FFFu;
    uint64_t h = chain(4, static_cast<uint64_t>(g));
    h = chain(h, static_cast<uint64_t>(p.t_next[sg]));
    h = chain(h, p.iter[sg]);
    h = chain(h, rem);
    h = chain(h, ptok);
    h = chain(h, rem ? p.pf_job[sg] : 0ull);
    h = chain(h, p.n_cls[sg]);
    h = chain(h, p.n_join[sg]);
    d += h;
    const int nd = static_cast<int>(byte_sum(p.n_cls[sg]));
    for (int j = 0; j < nd; ++j)
      d += chain(chain(chain(5, static_cast<uint64_t>(g)), p.fin[sg * p.BS + j]), p.job[sg * p.BS + j]);
  }
  atomicAdd(&total, static_cast<unsigned long long>(d));
  __syncthreads();
  if (tid == 0) p.digest[r] = total;
}

// ------------------------------------------------------------------ launchers ----
static int hip_ok(hipError_t e) { return e == hipSuccess ? SIM_OK : SIM_EHIP; }

int launch_reset(const Params &p, int reps, void *stream)
{
  hipLaunchKernelGGL(gnr_reset_kernel, dim3(1024), dim3(256), 0, static_cast<hipStream_t>(stream), p, reps);
  return hip_ok(hipGetLastError());
}

int launch_steps(const Params &p, int reps, int threads, size_t lds_bytes, uint32_t step_begin, uint32_t n_steps,
                 void *stream)
{
  auto kernel = threads > 512 ? gnr_step_kernel<1024> : gnr_step_kernel<512>;
  if (lds_bytes > 64 * 1024) {   // more than the default dynamic LDS limit has to be asked for
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds_bytes));
    if (e != hipSuccess) return SIM_EHIP;
  }
  hipLaunchKernelGGL(kernel, dim3(reps), dim3(threads), lds_bytes, static_cast<hipStream_t>(stream), p.self, p.key0,
                     p.key1, step_begin, n_steps);
  return hip_ok(hipGetLastError());
}

int launch_reduce(const Params &p, int reps, void *stream)
{
  const int n = kTallyWords + 3 * p.K * kNBin;
  hipLaunchKernelGGL(gnr_reduce_kernel, dim3((n + 255) / 256), dim3(256), 0, static_cast<hipStream_t>(stream), p, reps);
  return hip_ok(hipGetLastError());
}

#ifdef GNR_PROF
extern "C" int gnr_prof_read(unsigned long long *out16, int reset)
{
  if (hipMemcpyFromSymbol(out16, HIP_SYMBOL(g_prof), sizeof(unsigned long long) * 16) != hipSuccess) return SIM_EHIP;
  if (reset) {
    unsigned long long z[16] = {0};
    if (hipMemcpyToSymbol(HIP_SYMBOL(g_prof), z, sizeof z) != hipSuccess) return SIM_EHIP;
  }
  return SIM_OK;
}
#endif

int launch_digest(const Params &p, int reps, void *stream)
{
  hipLaunchKernelGGL(gnr_digest_kernel, dim3(reps), dim3(256), 0, static_cast<hipStream_t>(stream), p);
  return hip_ok(hipGetLastError());
}

}  // namespace gnr
