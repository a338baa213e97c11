// HIP kernels of the gate-and-route network simulator (gfx950, wave64).
//
// One workgroup owns one replication for a whole launch and loops over the steps itself. The servers are
// handled in blocks of 64 (one per lane); wave w takes the blocks w, w + nwaves, ... in every sweep, and the
// servers a wave queues for finishing are finished by that wave, so a server's record and slot row are
// touched by one wave at a time. Class-level counters (queue lengths, occupancies, tallies) live in LDS and
// are updated with integer atomics, which commute; the lanes of a wave are combined first, because atomics of
// several lanes on one LDS address serialise. Everything that the policy defines sequentially (order of
// simultaneous prefill completions, of gate admissions, of routed requests) is reproduced with 64-server
// ballot words in LDS and prefix popcounts over them.
#ifndef GNR_STEP_H
#define GNR_STEP_H
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

// A wave-uniform value pinned in a scalar register. Without this the compiler, short of registers, re-reads
// parameters from memory through the scalar cache wherever they are used (a round trip of hundreds of cycles in
// the middle of a hot loop) instead of keeping them.
__device__ __forceinline__ uint32_t pinned(uint32_t v)
{
  v = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(v)));
  asm volatile("" : "+s"(v));
  return v;
}

// Sixteen bytes of a slot row, read with the non-temporal hint: the rows stream through once per completed
// iteration and are not needed again before they would have left the caches anyway, so they should not push out
// the per-server records, ring entries and tables that the rest of the step reads (measured on 10000 servers x
// 256 replications: 2.9 % faster; the same hint on the few slot and request words that are read again when a
// decode leaves made it slower).
__device__ __forceinline__ uint4 stream_load(const uint32_t *p)
{
  typedef uint32_t word4 __attribute__((ext_vector_type(4)));
  const word4 x = __builtin_nontemporal_load(reinterpret_cast<const word4 *>(p));
  return make_uint4(x.x, x.y, x.z, x.w);
}

__device__ __forceinline__ uint64_t lanes_below() { return (1ull << (threadIdx.x & 63)) - 1ull; }

// Inclusive prefix sum over the wave with data-parallel-primitive adds: shifts by 1, 2, 4 and 8 inside each
// row of 16 lanes, then the row totals are passed on (row 0 -> 1, 2 -> 3, then 1 -> 2 and 3). All 64 lanes
// must be active.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_add(uint32_t v)
{
  return v + static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), CTRL, ROW_MASK, 0xF, false));
}
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v)
{
  v = dpp_add<0x111, 0xF>(v);   // row_shr 1
  v = dpp_add<0x112, 0xF>(v);   // row_shr 2
  v = dpp_add<0x114, 0xF>(v);   // row_shr 4
  v = dpp_add<0x118, 0xF>(v);   // row_shr 8
  v = dpp_add<0x142, 0xA>(v);   // row_bcast 15 into rows 1 and 3
  v = dpp_add<0x143, 0xC>(v);   // row_bcast 31 into rows 2 and 3
  return v;
}

__device__ __forceinline__ void lds_add64(uint64_t *p, uint64_t v)
{
  atomicAdd(reinterpret_cast<unsigned long long *>(p), static_cast<unsigned long long>(v));
}

// ------------------------------------------------------------------ LDS layout ----
enum Scalar {
  SC_NIDLE = 0, SC_NCOMP,
  // abandonment only:
  SC_LEAD = 2,    // [8] 1 if the gate's scan of the class queue found a waiting request in this pass
  SC_DLEN = 10,   // entries of the decode buffer ring between head and tail, abandoned ones included
  SC_DSCAN = 11,  // entries of that ring the routing passes of this step have gone past
  SC_COMPACT = 12,// bit k: class queue ring k (bit 8: the decode buffer ring) must be compacted before the appends
  // randomized router only:
  SC_NCS = 13,    // completed prefills of this step that joined the solo group's buffer
  SC_NCM = 14,    // ... the mixed group's buffer
  SC_DLEN_M = 15, // randomized router with abandonment: SC_DLEN / SC_DSCAN of the mixed group's buffer ring
  SC_DSCAN_M = 52,
  SC_QLEN = 32,   // [8] entries of each class queue ring between head and tail, abandoned ones included
  SC_TAKE = 16,   // [8] accepted arrivals this step
  SC_TAIL = 24,   // [8] ring position of the first accepted arrival
  SC_ADMK = 40,   // [8] admissions per class in this gate pass
  SC_TAKE_T = 48, // [kRouteLevels] jobs each level of the routing pass takes
  SC_W_T = 56,    // [kRouteLevels] jobs of the pass that come before each level
  SC_WORDS = 64
};
constexpr int kLoadBins = kMaxB + 1;
// Table sizes. Workgroups of one or two waves (N up to 2560) share a compute unit with others of their kind and are
// given smaller tables, so that eight of them fit its LDS: gate and routing passes then decide 64 admissions and stage
// 64 requests at a time (more passes when a step brings more), and a wave finishes its queued servers when more than
// 32 wait.
constexpr int kEvPerWave = 128;   // servers a wave can queue for finishing; when full the queue is drained early
constexpr int kEvPerWaveSmall = 96, kJobsLdsSmall = 64, kAdmChunkSmall = 64;
constexpr int kRouteLevels = 4;
constexpr int kJobsLds = 256;      // requests of a routing pass staged in LDS; later ones are read from the buffer
constexpr int kMaxPend = 254;     // untallied iterations a server may accumulate (kept in a byte)

struct Lds {
  int32_t *cs;        // [CS_WORDS]
  uint32_t *acc;      // [8]
  double *gtab;       // [5][kMaxK] gate targets of the launch: n x*, 1/x*, x*, n q*, priority index
  int32_t *sc;        // [SC_WORDS]
  uint64_t *tl;       // [kTallyWords]
  uint64_t *tbth;     // [K][tbt_w]
  uint64_t *bm_idle;  // [nwords] servers below Mp with no prefill in service (the gate looks at those below M)
  uint64_t *bm_comp;  // [nwords] servers whose prefill completed this step
  uint64_t *bm_busy;  // [nwords] servers running an iteration
  uint64_t *bm_join;  // [nwords] servers holding decodes that are not part of their untallied iterations
  uint64_t *bm_due;   // [nwords] servers that completed an iteration this step
  uint64_t *bm_touch; // [nwords] idle servers that were given work this step
  uint64_t *bm_flush; // [nwords] servers whose untallied iterations must be tallied at the restart
  uint64_t *bm_chunk; // [nwords] mixed-group servers whose running iteration carries a prefill chunk
  uint64_t *jobs;     // [kJobsLds] the first requests a routing pass places, copied from the decode buffer
  uint32_t *pre_lvl;  // [kRouteLevels][nwords] servers of the routed group with at most (level) decodes: per word, then ranks
  uint32_t *pre_c;    // [nwords] exclusive prefix popcounts of bm_comp
  uint32_t *pre;      // [nwords] exclusive prefix popcounts of bm_idle
  uint32_t *adm;      // [kAdmChunk] class | sequence-in-class << 3 of each admission
  uint16_t *adm_slot; // [kAdmChunk] prefill slot (server) that takes the admission of each rank
  uint32_t *lh;       // [2][kLoadBins] servers per decode count: solo group, mixed group
  uint32_t *ev_g;     // [waves][kEvPerWave] servers queued for finishing, per wave
  uint32_t *ev_q;     // [waves][kEvPerWave] their slot-quad masks
  uint16_t *stage;    // [waves][128] row halves to scan of the block a wave has open: lane | half << 6 | decodes << 8
  uint32_t *t32;      // [N] low 32 bits of the end time of the running iteration
  uint32_t *iter;     // [N] completed iterations
  uint8_t *loads;     // [N] decodes per server
  uint8_t *pend;      // [N] completed iterations not yet tallied (all with the server's current batch)
  uint16_t *rem;      // [Mp] prompt tokens left of the prefill a server has in service (0: none)
  uint32_t *live_off; // [K][kAdmChunk] abandonment only: ring offset from the head of the m-th waiting request of a class
  // weighted router only: the class selections of a routing pass
  uint32_t *sel_u;    // [kJobsLds] random word of each selection
  uint16_t *sel_co;   // [kJobsLds] class | (how many selections before it chose the same class) << 3
  uint16_t *sel_j;    // [kJobsLds] list position of each selection, ordered by class, then by order within the class
  int32_t *sel_n;     // [8] requests the pass takes from the solo group's buffer, per class
  // two-buffer routers only:
  uint64_t *solo_w;   // [4] per chunk of 64 completed prefills of a round: which of them go to the solo group
};

// Carves the dynamic LDS block; 8-byte granules. NWS > 0: the arrays indexed by 64-server word are sized for NWS
// words and the per-wave arrays for sixteen waves, whatever the configuration has; every array but the per-server
// ones and those behind them then sits at an offset the compiler knows (an immediate in the LDS instruction)
// instead of one it has to keep in a register, or to spill and fetch back, at every access. Used for the
// workgroups of sixteen waves (N up to 64 NWS servers). NWS = 0: everything sized by the configuration.
constexpr int kStaticWordsLarge = kMaxN / 64;   // any N the library accepts
constexpr int kStaticWordsMedium = 160;          // N up to 10240: three kilobytes less
template <int NWS, bool SMALL = false>
__host__ __device__ __forceinline__ Lds lds_carve(const Params &p, unsigned char *base, size_t *total)
{
  constexpr int kEvPerWave = SMALL ? kEvPerWaveSmall : gnr::kEvPerWave;       // (these shadow the large tables' sizes)
  constexpr int kJobsLds = SMALL ? kJobsLdsSmall : gnr::kJobsLds;
  constexpr int kAdmChunk = SMALL ? kAdmChunkSmall : gnr::kAdmChunk;
  Lds L;
  size_t off = 0;
  const size_t nw = NWS ? static_cast<size_t>(NWS) : static_cast<size_t>(p.nwords);
  const size_t waves = NWS ? 16u : static_cast<size_t>(p.threads / 64);
#define GNR_TAKE(field, type, count)                       \
  L.field = reinterpret_cast<type *>(base + off);          \
  off += (sizeof(type) * static_cast<size_t>(count) + 7) & ~size_t(7);
  GNR_TAKE(tl, uint64_t, kTallyWords)
  GNR_TAKE(jobs, uint64_t, kJobsLds)
  GNR_TAKE(cs, int32_t, CS_WORDS)
  GNR_TAKE(acc, uint32_t, 8)
  GNR_TAKE(gtab, double, 5 * kMaxK)
  GNR_TAKE(sc, int32_t, SC_WORDS)
  GNR_TAKE(adm, uint32_t, kAdmChunk)
  GNR_TAKE(adm_slot, uint16_t, kAdmChunk)
  GNR_TAKE(lh, uint32_t, 2 * kLoadBins)
  GNR_TAKE(ev_g, uint32_t, waves * kEvPerWave)
  GNR_TAKE(ev_q, uint32_t, waves * kEvPerWave)
  GNR_TAKE(stage, uint16_t, waves * 128)
  GNR_TAKE(bm_idle, uint64_t, nw)
  GNR_TAKE(bm_comp, uint64_t, nw)
  GNR_TAKE(bm_busy, uint64_t, nw)
  GNR_TAKE(bm_join, uint64_t, nw)
  GNR_TAKE(bm_due, uint64_t, nw)
  GNR_TAKE(bm_touch, uint64_t, nw)
  GNR_TAKE(bm_flush, uint64_t, nw)
  GNR_TAKE(bm_chunk, uint64_t, nw)
  GNR_TAKE(pre_lvl, uint32_t, kRouteLevels * nw)
  GNR_TAKE(pre_c, uint32_t, nw + 1)
  GNR_TAKE(pre, uint32_t, nw + 1)
  // from here on the offsets depend on the configuration
  GNR_TAKE(t32, uint32_t, p.N)
  GNR_TAKE(iter, uint32_t, p.N)
  GNR_TAKE(loads, uint8_t, p.N)
  GNR_TAKE(pend, uint8_t, p.N)
  GNR_TAKE(rem, uint16_t, p.Mp)
  GNR_TAKE(tbth, uint64_t, p.K * p.tbt_w)
  GNR_TAKE(live_off, uint32_t, p.dl_rings ? p.K * kAdmChunk : 0)
  GNR_TAKE(sel_u, uint32_t, p.route_mode == SIM_ROUTE_WEIGHTED_SPLIT ? kJobsLds : 0)
  GNR_TAKE(sel_co, uint16_t, p.route_mode == SIM_ROUTE_WEIGHTED_SPLIT ? kJobsLds : 0)
  GNR_TAKE(sel_j, uint16_t, p.route_mode == SIM_ROUTE_WEIGHTED_SPLIT ? kJobsLds : 0)
  GNR_TAKE(sel_n, int32_t, p.route_mode == SIM_ROUTE_WEIGHTED_SPLIT ? 8 : 0)
  GNR_TAKE(solo_w, uint64_t, p.route_mode == SIM_ROUTE_RANDOM_SPLIT || p.route_mode == SIM_ROUTE_WEIGHTED_SPLIT ? 4 : 0)
#undef GNR_TAKE
  if (total) *total = off;
  return L;
}
// Size classes of the step kernel: 0 workgroups of one or two waves (small tables, arrays sized by the
// configuration), 1 up to 512 threads (arrays sized by the configuration), 2 and 3 sixteen waves with the
// word-indexed arrays sized for 160 words and for the largest N.
__host__ __device__ constexpr int size_class(int threads, int nwords)
{
  return threads <= 128 ? 0 : threads <= 512 ? 1 : (nwords <= kStaticWordsMedium ? 2 : 3);
}
// Waves of an instantiation that are guaranteed to fit a SIMD together (the compiler keeps its registers within
// 512 / this many). A workgroup of 1024 threads needs four; the smaller classes are compiled twice: roomy, with up
// to 256 registers and two waves per SIMD, which is fastest while every workgroup of the launch finds a place at
// that density, and dense, with 128 registers and four waves per SIMD, for launches that would otherwise run their
// workgroups in more rounds.
__host__ __device__ constexpr int waves_per_simd(int max_threads, bool dense)
{
  return max_threads > 512 || dense ? 4 : 2;
}
__host__ __device__ constexpr int static_words(int size_class)
{
  return size_class <= 1 ? 0 : (size_class == 2 ? kStaticWordsMedium : kStaticWordsLarge);
}

// Bits of bitmap word w that belong to servers below `nbits`.
__device__ __forceinline__ uint64_t bits_below(int w, int nbits)
{
  const int left = nbits - (w << 6);
  return left >= 64 ? ~0ull : (left <= 0 ? 0ull : (1ull << left) - 1ull);
}

// Exclusive prefix popcounts of the first `nbits` bits of a bitmap, computed by one whole wave; returns the
// total in every lane.
__device__ __forceinline__ uint32_t rank_bitmap(const uint64_t *bm, uint32_t *pre, int nwords, int nbits)
{
  const int lane = threadIdx.x & 63;
  uint32_t running = 0;
  for (int base = 0; base < nwords; base += 64) {
    const int w = base + lane;
    const uint32_t v = w < nwords ? static_cast<uint32_t>(__popcll(bm[w] & bits_below(w, nbits))) : 0u;
    const uint32_t inc = wave_incl_scan(v);
    if (w < nwords) pre[w] = running + inc - v;
    running += static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(inc), 63));
  }
  return running;
}

// Wave totals with data-parallel-primitive adds: four steps inside each row of 16 lanes, then the row
// totals are passed on (row 0 -> 1, 2 -> 3, then 1 -> 2 and 3); lane 63 ends with the total, which is
// returned as a wave-uniform value. All 64 lanes must be active.
__device__ __forceinline__ uint32_t wave_sum32(uint32_t v)
{
  v = dpp_add<0xB1, 0xF>(v);    // quad_perm [1,0,3,2]
  v = dpp_add<0x4E, 0xF>(v);    // quad_perm [2,3,0,1]
  v = dpp_add<0x141, 0xF>(v);   // row_half_mirror
  v = dpp_add<0x140, 0xF>(v);   // row_mirror
  v = dpp_add<0x142, 0xA>(v);   // row_bcast 15 into rows 1 and 3
  v = dpp_add<0x143, 0xC>(v);   // row_bcast 31 into rows 2 and 3
  return static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(v), 63));
}
// 64-bit total of values below 2^58: three 32-bit totals of 16-, 16- and 26-bit pieces.
__device__ __forceinline__ uint64_t wave_sum64(uint64_t v)
{
  const uint64_t s0 = wave_sum32(static_cast<uint32_t>(v) & 0xFFFFu);
  const uint64_t s1 = wave_sum32(static_cast<uint32_t>(v >> 16) & 0xFFFFu);
  const uint64_t s2 = wave_sum32(static_cast<uint32_t>(v >> 32));
  return s0 + (s1 << 16) + (s2 << 32);
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

// Per-lane sums of this step's iteration tallies; folded into the workgroup's totals once per step.
// m executed iterations of duration d whose batch held the per-class decode counts `comp`; lanes with
// nothing to tally pass m = 0. Uniform control flow (all 64 lanes). The tallies every lane shares are summed
// over the wave first (same-address LDS atomics serialise); the time-between-tokens histogram, whose bins
// differ from lane to lane, gets m*comp_k tokens in the bin of d by LDS atomics directly.
__device__ __forceinline__ void tally_iterations(uint64_t *tl, uint64_t *tbth, int tbt_w, int tbt_lo, int K, uint32_t m,
                                                 int64_t d, bool chunk, uint64_t comp)
{
  if (__ballot(m != 0) == 0) return;
  const int lane = threadIdx.x & 63;
  const uint64_t md = static_cast<uint64_t>(m) * static_cast<uint64_t>(d);   // < 2^8 * 2^31
  const uint32_t its = wave_sum32(chunk ? m << 16 : m);                      // m <= 255: both totals fit 16 bits
  const uint64_t busy_solo = wave_sum64(chunk ? 0ull : md), busy_mix = wave_sum64(chunk ? md : 0ull);
  if (lane == 0) {
    if (its & 0xFFFFu) { lds_add64(&tl[kMaxK * kNTally + SIM_G_ITERS_SOLO], its & 0xFFFFu); lds_add64(&tl[kMaxK * kNTally + SIM_G_BUSY_SOLO], busy_solo); }
    if (its >> 16) { lds_add64(&tl[kMaxK * kNTally + SIM_G_ITERS_MIX], its >> 16); lds_add64(&tl[kMaxK * kNTally + SIM_G_BUSY_MIX], busy_mix); }
  }
  const int b = hbin(d) - tbt_lo;
#pragma unroll
  for (int k = 0; k < kMaxK; ++k) {
    if (k < K) {   // wave-uniform
      const uint32_t c = m ? byte_at(comp, k) : 0u;
      const uint64_t t = wave_sum64(static_cast<uint64_t>(c) * md);   // < 2^7 * 2^39
      if (lane == 0 && t) lds_add64(&tl[k * kNTally + SIM_T_TBT_SUM], t);
      if (c) lds_add64(&tbth[k * tbt_w + b], static_cast<uint64_t>(m) * c);
    }
  }
}


// Sort key of a gate candidate: the m-th waiting request of class k (m counted from the head).
// Occupancy gate: (X_k + m - n x_k*)/x_k*, ties by the larger queue deviation Q_k - m - n q_k*;
// priority gate: larger static index first; FCFS gate: older arrival stamp first.
// Ties that remain go to the lower class. Within a class the key does not decrease with m, so the
// gate's one-at-a-time argmin is the merge of the classes' sequences in this order.
struct GateKey { double a, b; };

// `live_off` (abandonment only, else null): ring offset of the m-th request of class k that still waits.
// The gate's targets live in an LDS table for the launch, [5][kMaxK]: n x*, 1/x*, x*, n q*, priority index (a copy
// of the parameter block's, which would be read through the scalar cache, a long round trip, at every comparison of
// the ranking loops). The values of one class are fetched together, once, before they are used.
enum GateTab { GT_NX = 0, GT_INVX = 1, GT_XSTAR = 2, GT_NQ = 3, GT_PRIO = 4 };
struct ClassTargets { double nx, invx, xstar, nq, prio; };
__device__ __forceinline__ ClassTargets load_targets(const double *tab, int k)
{
  ClassTargets t;
  t.nx = tab[GT_NX * kMaxK + k]; t.invx = tab[GT_INVX * kMaxK + k]; t.xstar = tab[GT_XSTAR * kMaxK + k];
  t.nq = tab[GT_NQ * kMaxK + k]; t.prio = tab[GT_PRIO * kMaxK + k];
  return t;
}
// Key of the m-th waiting request of class k, of which X_k = xs_k are in prefill and Q_p,k = qp_k wait; head_k: ring
// position of the class queue's head.
__device__ __forceinline__ GateKey gate_key(const int gate_mode, const uint32_t queue_cap, const ClassTargets &t,
                                            const uint32_t *qring, const uint32_t *live_off, int xs_k, int qp_k,
                                            uint32_t head_k, int k, int m, int adm_chunk)
{
  GateKey key;
  if (gate_mode == SIM_GATE_OCCUPANCY) {
    key.a = (static_cast<double>(xs_k + m) - t.nx) * t.invx;
    key.b = static_cast<double>(qp_k - m) - t.nq;
  } else if (gate_mode == SIM_GATE_PRIORITY) {
    key.a = -t.prio;
    key.b = 0.0;
  } else {
    uint32_t pos = head_k + (live_off ? live_off[k * adm_chunk + m] : static_cast<uint32_t>(m));
    if (pos >= queue_cap) pos -= queue_cap;
    key.a = static_cast<double>(qring[static_cast<size_t>(k) * queue_cap + pos]);
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

// The end of a server's prefill, kept until the lane has left the divergent part of the finishing code.
struct PrefillEnd { bool done; int k; uint32_t P; int64_t ttft; uint64_t nc; };

// ------------------------------------------------------------------ step kernel ----
// Iteration tallies are lazy. A server whose batch does not change runs identical iterations, so the
// completion pass only counts them (`pend`); they are tallied, with their multiplicity, when the batch is
// about to change: a decode leaves, a decode that joined mid-iteration becomes part of the batch, a prefill
// is present, work is placed on a server that is at an iteration boundary, or the launch ends.
// The arrays of the simulation state, handed to the step kernel by value: pointers that arrive as kernel
// arguments are known to point to global memory, so their loads and stores are plain global accesses
// (counted apart from LDS traffic) instead of generic ones that a wait on LDS would also wait for.
struct StepArrays {
  const uint32_t *arr_thr;
  const uint16_t *len_tab;
  int64_t *t_next;
  uint32_t *iter, *remptok;
  uint64_t *pf_job, *n_cls, *n_join;
  uint32_t *fin;
  uint64_t *job;
  uint32_t *qring;
  uint64_t *dring;
  int32_t *cstate;
  uint64_t *tally, *hist;
  // abandonment only
  const uint16_t *pat_tab;
  uint32_t *qdl, *ddl, *cal, *dcal;
  // randomized router only
  uint64_t *dring_m;
  uint32_t *ddl_m, *dcal_m;   // ... with abandonment
};

// AB: the variant with abandonment (some class has a patience rate). Ring entries then carry the step at whose
// start the request leaves if it still waits. Such entries stay in the rings as dead entries until the head
// passes them: the counters Q_p, Q_d follow the abandonments eagerly through per-step calendars, the gate and
// the router skip dead entries when they take requests, and a ring is compacted when it would not hold the
// step's appends and at the end of every launch (so the state between launches holds waiting requests only).
// RR: the variant with the randomized decode router: every completed prefill is sent to the solo or to the
// mixed group by a random word, each group has its own buffer ring and is fed from that ring only. A routing
// pass then takes jobs from both rings: the staged list holds the solo ring's jobs first.
// IM: the variant with immediate same-slot decode (no router): a request whose prefill ends goes on decoding on
// its own server, placed there by the lane that finishes the server; a server is offered to the gate while it
// holds no prefill and fewer than B decodes.
template <int MAXT, int NWS, bool AB, bool RR, bool IM, bool WS = false, bool DENSE = false>
__global__ void __launch_bounds__(MAXT) __attribute__((amdgpu_waves_per_eu(waves_per_simd(MAXT, DENSE)))) gnr_step_kernel(const Params *__restrict__ params, const StepArrays a,
                                                        const uint32_t key0, const uint32_t key1,
                                                        const uint32_t step_begin, const uint32_t n_steps)
{
  const Params &p = *params;   // immutable after creation; read through the scalar cache on demand
  extern __shared__ __align__(16) unsigned char lds_raw[];
  constexpr bool SMALL = MAXT <= 128;
  constexpr int kEvPerWave = SMALL ? kEvPerWaveSmall : gnr::kEvPerWave;       // (these shadow the large tables' sizes)
  constexpr int kJobsLds = SMALL ? kJobsLdsSmall : gnr::kJobsLds;
  constexpr int kAdmChunk = SMALL ? kAdmChunkSmall : gnr::kAdmChunk;
  const Lds L = lds_carve<NWS, SMALL>(p, lds_raw, nullptr);

  const int r = blockIdx.x;
  const int tid = threadIdx.x;
  const int NT = blockDim.x;
  const int lane = tid & 63;
  // wave-uniform values are made scalar explicitly, so that loops and branches on them are scalar too
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nwaves = NT >> 6;
  const int wave_base = wave << 6;
  // The instruction arbiter of a SIMD prefers its oldest wave: left alone, the first four waves of the workgroup
  // finish every sweep early and the last four late, and the barrier waits for those. Raising the priority of the
  // younger waves evens this out.
  if (nwaves > 4) {
    if (wave >= 12) __builtin_amdgcn_s_setprio(3);
    else if (wave >= 8) __builtin_amdgcn_s_setprio(2);
    else if (wave >= 4) __builtin_amdgcn_s_setprio(1);
  }
  const int K = p.K, N = p.N, B = p.B, M = p.M, BS = p.BS;
  const int nper = (N + NT - 1) / NT;
  const int nwords = p.nwords;
  // Servers 0..M-1 are the mixed group for the gate and the router. Servers below Mp >= M may hold a prefill:
  // Mp is the largest M the run has had (a prefill in service stays when its server turns solo).
  const int Mp = p.Mp;
  const int nwords_m = (Mp + 63) >> 6;   // bitmap words that hold servers with prefill state
  // Iteration-time coefficients, chunk size and step length in ns (each below 2^31: the longest iteration is),
  // window of the on-chip time-between-tokens histogram, class thresholds of the arrival draw: used in every block.
  const uint32_t c0_ns = pinned(static_cast<uint32_t>(p.c0)), cpre_ns = pinned(static_cast<uint32_t>(p.cpre));
  const uint32_t cdec_ns = pinned(static_cast<uint32_t>(p.cdec)), dt_ns = pinned(static_cast<uint32_t>(p.dt));
  const int chunk_max = static_cast<int>(pinned(static_cast<uint32_t>(p.C)));
  const int tbt_w = static_cast<int>(pinned(static_cast<uint32_t>(p.tbt_w))), tbt_lo = static_cast<int>(pinned(static_cast<uint32_t>(p.tbt_lo)));
  // an arrival's class is the number of thresholds its random word has reached; classes beyond K-1 do not exist:
  // their thresholds are the largest word, and the count is capped
  uint32_t cthr[kMaxK - 1];
#pragma unroll
  for (int c = 0; c + 1 < kMaxK; ++c) cthr[c] = pinned(c + 1 < K ? p.cls_thr[c] : 0xFFFFFFFFu);
  const int gate_mode = static_cast<int>(pinned(static_cast<uint32_t>(p.gate_mode)));
  const uint32_t queue_cap = pinned(p.queue_cap), dbuf_cap = pinned(p.dbuf_cap);

  int64_t *t_next = a.t_next + static_cast<size_t>(r) * N;
  uint32_t *iter_g = a.iter + static_cast<size_t>(r) * N;
  uint32_t *remptok = a.remptok + static_cast<size_t>(r) * N;
  uint64_t *pf_job = a.pf_job + static_cast<size_t>(r) * N;
  uint64_t *n_cls = a.n_cls + static_cast<size_t>(r) * N;
  uint64_t *n_join = a.n_join + static_cast<size_t>(r) * N;
  uint32_t *fin = a.fin + static_cast<size_t>(r) * N * BS;
  uint64_t *job = a.job + static_cast<size_t>(r) * N * BS;
  uint32_t *qring = a.qring + static_cast<size_t>(r) * K * queue_cap;
  uint64_t *dring = a.dring + static_cast<size_t>(r) * dbuf_cap;
  uint64_t *hist = a.hist + static_cast<size_t>(r) * 3 * K * kNBin;
  uint32_t *ev_g = L.ev_g + wave * kEvPerWave;
  uint32_t *ev_q = L.ev_q + wave * kEvPerWave;
  // abandonment only
  const uint32_t cal_n = p.cal_mask + 1u;
  uint32_t *qdl = AB ? a.qdl + static_cast<size_t>(r) * K * queue_cap : nullptr;
  uint32_t *ddl = AB ? a.ddl + static_cast<size_t>(r) * dbuf_cap : nullptr;
  uint32_t *cal = AB ? a.cal + static_cast<size_t>(r) * K * cal_n : nullptr;
  uint32_t *dcal = AB ? a.dcal + static_cast<size_t>(r) * K * cal_n : nullptr;
  const uint32_t *lo_tab = AB ? L.live_off : nullptr;
  uint64_t *dring_m = RR ? a.dring_m + static_cast<size_t>(r) * dbuf_cap : nullptr;
  uint32_t *ddl_m = AB && RR ? a.ddl_m + static_cast<size_t>(r) * dbuf_cap : nullptr;
  uint32_t *dcal_m = AB && RR ? a.dcal_m + static_cast<size_t>(r) * K * cal_n : nullptr;

  // ---- load the replication's class state and rebuild the on-chip views of the server state
  for (int i = tid; i < CS_WORDS; i += NT) L.cs[i] = a.cstate[static_cast<size_t>(r) * CS_WORDS + i];
  for (int i = tid; i < kTallyWords; i += NT) L.tl[i] = 0;
  for (int i = tid; i < K * p.tbt_w; i += NT) L.tbth[i] = 0;
  for (int i = tid; i < SC_WORDS; i += NT) L.sc[i] = 0;
  if (tid < kMaxK) {
    L.gtab[GT_NX * kMaxK + tid] = tid < K ? p.nx[tid] : 0.0;
    L.gtab[GT_INVX * kMaxK + tid] = tid < K ? p.invx[tid] : 0.0;
    L.gtab[GT_XSTAR * kMaxK + tid] = tid < K ? p.xstar[tid] : 0.0;
    L.gtab[GT_NQ * kMaxK + tid] = tid < K ? p.nq[tid] : 0.0;
    L.gtab[GT_PRIO * kMaxK + tid] = tid < K ? p.prio[tid] : 0.0;
  }
  for (int i = tid; i < 2 * kLoadBins; i += NT) L.lh[i] = 0;
  __syncthreads();
  if constexpr (AB) {   // between launches the rings hold waiting requests only
    if (tid < K) L.sc[SC_QLEN + tid] = L.cs[CS_QP + tid];
    if (tid == 0) {
      L.sc[SC_DLEN] = L.cs[CS_DCOUNT];
      if constexpr (RR) L.sc[SC_DLEN_M] = L.cs[CS_DCOUNT_M];
    }
  }
  for (int i = 0; i < nper; ++i) {
    const int g = i * NT + tid;
    const bool valid = g < N;
    bool busy = false, joined = false;
    if (valid) {
      const uint32_t nd = byte_sum(n_cls[g]);
      L.loads[g] = static_cast<uint8_t>(nd);
      L.pend[g] = 0;
      atomicAdd(&L.lh[(g < M ? kLoadBins : 0) + nd], 1u);
      const int64_t tn = t_next[g];
      busy = tn != kIdle;
      L.t32[g] = static_cast<uint32_t>(tn);
      L.iter[g] = iter_g[g];
      joined = n_join[g] != 0;
    }
    bool idle_slot = false, chunk = false;
    if (valid && g < Mp) {   // the prefill word stays in LDS during the launch: tokens left, and whether a chunk runs
      const uint32_t pk = remptok[g];
      L.rem[g] = static_cast<uint16_t>(pk_rem(pk));
      idle_slot = pk_rem(pk) == 0 && (!IM || static_cast<int>(byte_sum(n_cls[g])) < B);
      chunk = pk_ptok(pk) > 0;
    }
    const uint64_t bi = __ballot(idle_slot), bb = __ballot(busy), bj = __ballot(joined), bc = __ballot(chunk);
    const int wi = (i * NT + wave_base) >> 6;
    if (lane == 0 && wi < nwords) {
      L.bm_idle[wi] = bi; L.bm_busy[wi] = bb; L.bm_join[wi] = bj; L.bm_flush[wi] = 0; L.bm_chunk[wi] = bc;
      L.bm_due[wi] = 0; L.bm_touch[wi] = 0;   // nothing waits for a restart when a launch begins
    }
  }
  __syncthreads();

  // ---- abandonment only: ring compaction, one wave per ring. Entries whose deadline is not after `now` are
  //      dropped, the others keep their order and move towards the head (a lane never writes ahead of what
  //      the wave has read). `pending`: entries already counted in the ring length but not yet written.
  auto compact_queue = [&](int k, uint32_t now, uint32_t pending) __attribute__((always_inline)) {
    uint32_t *ring = qring + static_cast<size_t>(k) * queue_cap;
    uint32_t *dlr = qdl + static_cast<size_t>(k) * queue_cap;
    const uint32_t hd = static_cast<uint32_t>(L.cs[CS_QHEAD + k]);
    uint32_t n = static_cast<uint32_t>(L.sc[SC_QLEN + k]) - pending;
    if (n > queue_cap) n = queue_cap;   // (a ring never holds more; keeps every access inside it regardless)
    uint32_t w = 0;
    for (uint32_t off = 0; off < n; off += 64) {   // wave-uniform
      const uint32_t i = off + lane;
      uint32_t pos = hd + i;
      if (pos >= queue_cap) pos -= queue_cap;
      const uint32_t st = i < n ? ring[pos] : 0u, dl = i < n ? dlr[pos] : 0u;
      const bool live = i < n && dl > now;
      const uint64_t bal = __ballot(live);
      if (live) {
        uint32_t wp = hd + w + static_cast<uint32_t>(__popcll(bal & lanes_below()));
        if (wp >= queue_cap) wp -= queue_cap;
        ring[wp] = st; dlr[wp] = dl;
      }
      w += static_cast<uint32_t>(__popcll(bal));
    }
    if (lane == 0) {
      uint32_t tail = hd + w;
      if (tail >= queue_cap) tail -= queue_cap;
      L.sc[SC_QLEN + k] = static_cast<int32_t>(w + pending);
      L.sc[SC_TAIL + k] = static_cast<int32_t>(tail);
    }
  };
  // (`mixed`: the mixed group's buffer ring of the randomized router)
  auto compact_buffer = [&](uint32_t now, bool mixed) __attribute__((always_inline)) {
    uint64_t *dring = mixed ? dring_m : a.dring + static_cast<size_t>(r) * dbuf_cap;
    uint32_t *ddl = mixed ? ddl_m : a.ddl + static_cast<size_t>(r) * dbuf_cap;
    const uint32_t hd = static_cast<uint32_t>(L.cs[mixed ? CS_DHEAD_M : CS_DHEAD]);
    uint32_t n = static_cast<uint32_t>(L.sc[mixed ? SC_DLEN_M : SC_DLEN]);
    if (n > dbuf_cap) n = dbuf_cap;
    uint32_t w = 0;
    for (uint32_t off = 0; off < n; off += 64) {   // wave-uniform
      const uint32_t i = off + lane;
      uint32_t pos = hd + i;
      if (pos >= dbuf_cap) pos -= dbuf_cap;
      const uint64_t jw = i < n ? dring[pos] : 0ull;
      const uint32_t dl = i < n ? ddl[pos] : 0u;
      const bool live = i < n && dl > now;
      const uint64_t bal = __ballot(live);
      if (live) {
        uint32_t wp = hd + w + static_cast<uint32_t>(__popcll(bal & lanes_below()));
        if (wp >= dbuf_cap) wp -= dbuf_cap;
        dring[wp] = jw; ddl[wp] = dl;
      }
      w += static_cast<uint32_t>(__popcll(bal));
    }
    if (lane == 0) L.sc[mixed ? SC_DLEN_M : SC_DLEN] = static_cast<int32_t>(w);
  };

  int64_t T = 0;
  // A server that completed an iteration, or was given work while idle, is restarted lazily: when its block
  // is opened in the next step's completion pass (same lane, no extra sweep). After the last step of the launch
  // one more pass over the blocks does only that, and tallies every iteration still untallied.
  for (uint32_t s = step_begin; s <= step_begin + n_steps; ++s) {
    const bool final_pass = s == step_begin + n_steps;
    T = (static_cast<int64_t>(s) + 1) * dt_ns;
    const uint32_t T32 = static_cast<uint32_t>(T);
    const int64_t Tp = T - dt_ns;   // the boundary of the previous step: restarts refer to it
    const uint32_t Tp32 = static_cast<uint32_t>(Tp);
    if (tid < 8) L.acc[tid] = 0;
    // abandonment only: how many waiting requests of class `tid` leave at the start of this step (asked for
    // here, used after the completion pass)
    uint32_t n_leave_p = 0, n_leave_d = 0, n_leave_dm = 0;
    if constexpr (AB) {
      if (!final_pass && tid < K) {
        n_leave_p = atomicExch(&cal[static_cast<size_t>(tid) * cal_n + (s & p.cal_mask)], 0u);
        n_leave_d = atomicExch(&dcal[static_cast<size_t>(tid) * cal_n + (s & p.cal_mask)], 0u);
        if constexpr (RR) n_leave_dm = atomicExch(&dcal_m[static_cast<size_t>(tid) * cal_n + (s & p.cal_mask)], 0u);
      }
    }
    const uint32_t *thr = a.arr_thr + 3 * (p.mod_period > 0 ? static_cast<int64_t>(s % static_cast<uint64_t>(p.mod_period)) : 0);
    const uint32_t thr0 = pinned(thr[0]), thr1 = pinned(thr[1]), thr2 = pinned(thr[2]);
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
          for (int c = 0; c + 1 < kMaxK; ++c) k += w[1 + j] >= cthr[c];
          atomicAdd(&L.acc[k < K ? k : K - 1], 1u);
        }
      }
    };

    // ---- 2. finishing queued servers, one per lane (uniform control flow; lanes beyond the queue idle).
    //      Tallies the server's untallied iterations and the one that just ended, removes the decodes
    //      that emitted their last token (slot quads flagged in the queue entry), advances the prefill.
    auto drain_events = [&](int nev) __attribute__((always_inline)) {
      for (int e0 = 0; e0 < nev; e0 += 64) {
        const int e = e0 + lane;
        const bool active = e < nev;
        uint32_t m = 0;
        int64_t d = 0;
        bool chunk = false;
        uint64_t comp = 0;
        PrefillEnd pe; pe.done = false; pe.k = 0; pe.P = 0; pe.ttft = 0; pe.nc = 0;
        if (active) {
          const int g = static_cast<int>(ev_g[e]);
          uint32_t quads = ev_q[e];
          uint64_t nc = n_cls[g];
          const uint64_t bit = 1ull << (g & 63);
          const bool joined = L.bm_join[g >> 6] & bit;
          const uint64_t nj = joined ? n_join[g] : 0ull;
          const bool has_chunk = g < Mp && (L.bm_chunk[g >> 6] & bit);
          const uint32_t it = L.iter[g];
          int nd = L.loads[g];
          int rem = g < Mp ? static_cast<int>(L.rem[g]) : 0;
          const int ptok = has_chunk ? (rem < chunk_max ? rem : chunk_max) : 0;   // the chunk frozen at the start of the iteration
          const int64_t tn = T + static_cast<int64_t>(static_cast<int32_t>(L.t32[g] - T32));   // exact completion time
          comp = nc - nj;   // bytewise: no class joins more decodes than it holds
          d = static_cast<int64_t>(c0_ns + cpre_ns * static_cast<uint32_t>(ptok) + cdec_ns * byte_sum(comp));
          chunk = ptok > 0;
          m = static_cast<uint32_t>(L.pend[g]) + 1u;
          L.pend[g] = 0;
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
                  const int64_t e2e = tn - (static_cast<int64_t>(stamp) + 1) * dt_ns;
                  lds_add64(&L.tl[k * kNTally + (mixed_now ? SIM_T_S_DM : SIM_T_S_DS)], 1);
                  atomicSub(&L.cs[(mixed_now ? CS_YM : CS_YS) + k], 1);
                  lds_add64(&L.tl[k * kNTally + SIM_T_TOKP_DEC], Pl);
                  lds_add64(&L.tl[k * kNTally + SIM_T_TOKD_DEC], Dl);
                  lds_add64(&L.tl[k * kNTally + SIM_T_E2E_SUM], static_cast<uint64_t>(e2e));
                  atomicAdd(reinterpret_cast<unsigned long long *>(&hist[(1 * K + k) * kNBin + hbin(e2e)]), 1ull);
                  nc -= 1ull << (8 * k);
                  --nd;
                  if (j < nd) { frow[j] = frow[nd]; jrow[j] = jrow[nd]; }
                  frow[nd] = 0;   // a vacated slot must never match a later iteration index
                }
              }
            }
            if (nd != nd_before) {
              n_cls[g] = nc;
              L.loads[g] = static_cast<uint8_t>(nd);
              const int hb = g < M ? kLoadBins : 0;
              atomicSub(&L.lh[hb + nd_before], 1u);
              atomicAdd(&L.lh[hb + nd], 1u);
              if constexpr (IM) {   // a full server (it holds no prefill then) has a slot again
                if (nd_before == B && g < Mp) atomicOr(reinterpret_cast<unsigned long long *>(&L.bm_idle[g >> 6]), bit);
              }
            }
          }
          // the prefill advances by the chunk frozen at the start of the iteration
          if (ptok > 0) {
            rem -= ptok;
            L.rem[g] = static_cast<uint16_t>(rem);
            atomicAnd(reinterpret_cast<unsigned long long *>(&L.bm_chunk[g >> 6]), ~bit);   // set again at the restart
            if (rem == 0) {
              const uint64_t jw = pf_job[g];
              const int k = static_cast<int>(jw >> 29) & 7;
              const uint32_t stamp = static_cast<uint32_t>(jw) & 0x1FFFFFFFu;
              pe.done = true; pe.k = k; pe.nc = nc;
              pe.P = (static_cast<uint32_t>(jw >> 32) & 0xFFFFu) + 1;
              pe.ttft = tn - (static_cast<int64_t>(stamp) + 1) * dt_ns;
              atomicAdd(reinterpret_cast<unsigned long long *>(&hist[(0 * K + k) * kNBin + hbin(pe.ttft)]), 1ull);
              if constexpr (IM) {
                // the request keeps its slot: it joins the batch at the restart that follows this completion
                // (the gate admits only where a slot is left, so nd < B here; were it not, the request is dropped)
                if (nd >= B) {
                  lds_add64(&L.tl[k * kNTally + SIM_T_DROP_D], 1);
                  L.tl[kMaxK * kNTally + SIM_G_OVERFLOW] = 1;
                } else {
                const uint32_t Dl = static_cast<uint32_t>(jw >> 48) + 1;
                fin[static_cast<size_t>(g) * BS + nd] = it + Dl;
                job[static_cast<size_t>(g) * BS + nd] = jw;
                n_cls[g] = nc + (1ull << (8 * k));
                const int hb = g < M ? kLoadBins : 0;
                atomicSub(&L.lh[hb + nd], 1u);
                atomicAdd(&L.lh[hb + nd + 1], 1u);
                ++nd;
                L.loads[g] = static_cast<uint8_t>(nd);
                lds_add64(&L.tl[k * kNTally + SIM_T_U_DS], 1);
                atomicAdd(&L.cs[CS_YS + k], 1);
                if (nd < B) atomicOr(reinterpret_cast<unsigned long long *>(&L.bm_idle[g >> 6]), bit);
                }
              } else {
              atomicOr(reinterpret_cast<unsigned long long *>(&L.bm_comp[g >> 6]), bit);
              atomicOr(reinterpret_cast<unsigned long long *>(&L.bm_idle[g >> 6]), bit);
              }
            }
          }
          if (joined) {
            n_join[g] = 0;
            atomicAnd(reinterpret_cast<unsigned long long *>(&L.bm_join[g >> 6]), ~bit);
          }
        }
        tally_iterations(L.tl, L.tbth, tbt_w, tbt_lo, K, m, d, chunk, comp);
        // a prefill that ended: completion count, recognised prompt tokens, time to first token; the
        // co-resident decodes switch mixed -> solo
        if (pe.done) {
          lds_add64(&L.tl[pe.k * kNTally + SIM_T_S_P], 1);
          atomicSub(&L.cs[CS_X + pe.k], 1);
          lds_add64(&L.tl[pe.k * kNTally + SIM_T_TOKP_PRE], pe.P);
          lds_add64(&L.tl[pe.k * kNTally + SIM_T_TTFT_SUM], static_cast<uint64_t>(pe.ttft));
#pragma unroll
          for (int c = 0; c < kMaxK; ++c) {
            const int v = static_cast<int>(byte_at(pe.nc, c));
            if (v) {
              lds_add64(&L.tl[c * kNTally + SIM_T_M_MS], static_cast<uint64_t>(v));
              atomicSub(&L.cs[CS_YM + c], v);
              atomicAdd(&L.cs[CS_YS + c], v);
            }
          }
        }
      }
    };

    // ---- completion pass, one round of 64 servers (one per lane) at a time.
    //      open_round: due test; the slot rows of the due servers are listed in `stage`, 64 slots (half a row)
    //      per entry. issue_batch: eight lanes read one entry, 16 bytes per lane and load; a group is eight
    //      entries, a batch Q groups. process_group: the finish words are compared with the server's iteration
    //      index; the hit masks travel back to the owning lanes. The first batch of a block is issued when the
    //      block is opened, before the arrivals of the block are drawn. finalize: a server whose batch changes,
    //      or that carries a prefill, is queued for finishing; for any other the iteration is only counted.
    //      Slots beyond a server's decode count never hold a future iteration index (they are cleared when
    //      vacated), so the comparison needs no occupancy mask.
    {
      constexpr int Q = 5;   // groups of eight row halves in flight
      const int l8 = lane & 7, grp = lane >> 3;
      const uint64_t below = lanes_below();
      uint16_t *stage = L.stage + wave * 128;
      int nev = 0;          // servers queued by this wave (wave-uniform)
      int ne = 0;           // row halves listed for the open block (wave-uniform)
      bool o_due = false, o_must = false, o_scan = false, o_big = false;   // owner-lane state of the open round
      int o_rank = 0, o_nd = 0, o_pend = 0;
      uint32_t o_it = 0, o_q = 0;
      uint4 v[Q][2];
      uint32_t vit[Q];

      auto open_round = [&](int wi) __attribute__((always_inline)) {
        const int gw = wi << 6;
        const int g = gw + lane;
        const uint64_t lbit = 1ull << lane;
        const bool valid = g < N;
        // everything the block needs from LDS is read here in one go: a chain of dependent LDS round trips
        // costs far more than a few reads that turn out unused
        const uint64_t busy_word = L.bm_busy[wi], due_prev = L.bm_due[wi], touch_prev = L.bm_touch[wi];
        const uint64_t flush_prev = L.bm_flush[wi], idle_word = L.bm_idle[wi], chunk_word = L.bm_chunk[wi];
        uint64_t join_word = L.bm_join[wi];
        uint32_t t32v = valid ? L.t32[g] : 0u;
        const uint32_t iter_v = valid ? L.iter[g] : 0u;
        const int nd = valid ? static_cast<int>(L.loads[g]) : 0;
        int pend = valid ? static_cast<int>(L.pend[g]) : 0;
        const int rem_v = g < Mp ? static_cast<int>(L.rem[g]) : 0;
        bool busy = busy_word & lbit;
        // ---- (re)start of the servers that completed an iteration or were given work in the previous step.
        //      Untallied iterations are tallied before the batch changes, and all of them when the launch ends.
        const bool flush = valid && ((flush_prev & lbit) || (final_pass && pend != 0));
        if (__ballot(flush)) {
          uint32_t m = 0;
          int64_t d = 0;
          uint64_t comp = 0;
          bool unjoin = false;
          if (flush) {
            const uint64_t nc = n_cls[g];
            const bool joined = join_word & lbit;
            const uint64_t nj = joined ? n_join[g] : 0ull;
            comp = nc - nj;   // bytewise: no class joins more decodes than it holds
            d = static_cast<int64_t>(c0_ns + cdec_ns * byte_sum(comp));   // untallied iterations never hold a chunk
            m = static_cast<uint32_t>(pend);
            pend = 0;
            L.pend[g] = 0;
            unjoin = (flush_prev & lbit) && joined;   // the decodes placed at the boundary joined the batch there
            if (unjoin) n_join[g] = 0;
          }
          tally_iterations(L.tl, L.tbth, tbt_w, tbt_lo, K, m, d, false, comp);
          const uint64_t unjoin_m = __ballot(unjoin);
          if (unjoin_m) {   // this wave alone works on the block's words
            join_word &= ~unjoin_m;
            if (lane == 0) L.bm_join[wi] = join_word;
          }
          if (lane == 0 && flush_prev) L.bm_flush[wi] = 0;
        }
        const uint64_t todo = due_prev | touch_prev;
        if (todo) {
          bool chunk_now = false;
          if (todo & lbit) {
            const int ptok = rem_v > 0 ? (rem_v < chunk_max ? rem_v : chunk_max) : 0;
            chunk_now = ptok > 0;
            if (ptok == 0 && nd == 0) {
              busy = false;
            } else {
              // back-to-back after a completion, otherwise from the step boundary; only the low 32 bits of the
              // clock are kept and an iteration lasts less than 2^31 ns, so 32-bit arithmetic is exact here
              const uint32_t dur = c0_ns + cpre_ns * static_cast<uint32_t>(ptok) + cdec_ns * static_cast<uint32_t>(nd);
              t32v = ((due_prev & lbit) ? t32v : Tp32) + dur;
              L.t32[g] = t32v;
              busy = true;
            }
          }
          const uint64_t nb = __ballot(busy), nchunk = __ballot(chunk_now);
          if (lane == 0) {
            if (nb != busy_word) L.bm_busy[wi] = nb;
            if (gw < Mp) L.bm_chunk[wi] = (chunk_word & ~todo) | nchunk;
          }
        }
        o_due = false; o_it = 0; o_nd = 0; o_pend = 0; o_q = 0;
        if (final_pass) {   // only the restarts: the launch ends here
          if (lane == 0) { L.bm_due[wi] = 0; L.bm_touch[wi] = 0; }
          o_must = o_scan = o_big = false;
          ne = 0;
          return;
        }
        // ---- which servers complete an iteration in this step
        o_due = busy && static_cast<int32_t>(t32v - T32) <= 0;
        if (o_due) {
          o_it = iter_v + 1;
          L.iter[g] = o_it;
          o_nd = nd;
          o_pend = pend;
        }
        // (with immediate decode the bitmap marks the servers the gate may admit to: a full one is not in it)
        const bool prefill_here = IM ? rem_v != 0 : (g < Mp && !(idle_word & lbit));
        o_must = o_due && ((join_word & lbit) || prefill_here || o_pend >= kMaxPend);
        o_scan = o_due && o_nd > 0;
        o_big = o_scan && o_nd > 64;   // the row's second half holds decodes too
        const uint64_t dm = __ballot(o_due), sm = __ballot(o_scan), bg = __ballot(o_big);
        o_rank = __popcll(sm & below) + __popcll(bg & below);
        ne = __popcll(sm) + __popcll(bg);
        if (o_scan) {   // entry: lane | second half << 6 | decode count << 8
          const uint32_t e = static_cast<uint32_t>(lane) | (static_cast<uint32_t>(o_nd) << 8);
          stage[o_rank] = static_cast<uint16_t>(e);
          if (o_big) stage[o_rank + 1] = static_cast<uint16_t>(e | 64u);
        }
        if (lane == 0) {
          L.bm_due[wi] = dm;
          L.bm_touch[wi] = 0;
          L.bm_comp[wi] = 0;
        }
      };
      // Groups g0 .. g0+Q-1 of the open block go into the Q register sets. The LDS reads of all of them are
      // issued together, then the loads, then the shuffles that fetch the iteration indices (needed only when
      // the words are compared): two LDS round trips per batch instead of two per group.
      auto issue_batch = [&](int wi, int g0) __attribute__((always_inline)) {
        const uint32_t gw = static_cast<uint32_t>(wi) << 6;
        uint32_t e[Q];
#pragma unroll
        for (int t = 0; t < Q; ++t) {
          const int pidx = 8 * (g0 + t) + grp;
          e[t] = pidx < ne ? stage[pidx] : 0u;   // no entry: decode count 0, nothing is loaded
        }
#pragma unroll
        for (int t = 0; t < Q; ++t) {
          const uint32_t sid = e[t] & 63u, half = (e[t] >> 6) & 1u;
          const int nds = static_cast<int>(e[t] >> 8);
          const int q0 = 16 * static_cast<int>(half) + l8;   // this lane's quads of the row: q0 and q0 + 8
          const uint32_t off = (gw + sid) * static_cast<uint32_t>(BS) + 4u * q0;
          // a register that is not loaded holds zeros, which no iteration index equals (the first is 1)
          v[t][0] = v[t][1] = make_uint4(0u, 0u, 0u, 0u);
          if (4 * q0 < nds) v[t][0] = stream_load(fin + off);
          if (4 * q0 + 32 < nds) v[t][1] = stream_load(fin + off + 32u);
        }
#pragma unroll
        for (int t = 0; t < Q; ++t) {
          const uint32_t it_owner = __shfl(o_it, static_cast<int>(e[t] & 63u), 64);   // every lane takes part
          vit[t] = 8 * (g0 + t) + grp < ne ? it_owner : 0xFFFFFFFFu;                  // no entry: matches nothing
        }
      };
      auto process_group = [&](int t, int gi) __attribute__((always_inline)) {
        const uint32_t it = vit[t];
        const bool m0 = v[t][0].x == it || v[t][0].y == it || v[t][0].z == it || v[t][0].w == it;
        const bool m1 = v[t][1].x == it || v[t][1].y == it || v[t][1].z == it || v[t][1].w == it;
        if (__ballot(m0 || m1)) {   // a decode emits its last token: rare
          const uint64_t bal0 = __ballot(m0), bal1 = __ballot(m1);
          const int d0 = o_rank - 8 * gi, d1 = d0 + 1;   // this owner's entries, counted within the group
          if (o_scan && static_cast<unsigned>(d0) < 8u)
            o_q |= (static_cast<uint32_t>(bal0 >> (8 * d0)) & 0xFFu) | ((static_cast<uint32_t>(bal1 >> (8 * d0)) & 0xFFu) << 8);
          if (o_big && static_cast<unsigned>(d1) < 8u)
            o_q |= ((static_cast<uint32_t>(bal0 >> (8 * d1)) & 0xFFu) | ((static_cast<uint32_t>(bal1 >> (8 * d1)) & 0xFFu) << 8)) << 16;
        }
      };
      auto finalize = [&](int wi) __attribute__((always_inline)) {
        const int g = (wi << 6) + lane;
        const bool event = o_due && (o_must || o_q != 0);
        if (o_due && !event) L.pend[g] = static_cast<uint8_t>(o_pend + 1);
        const uint64_t evm = __ballot(event);
        if (evm) {
          if (event) {
            const int slot = nev + __popcll(evm & below);
            ev_g[slot] = static_cast<uint32_t>(g);
            ev_q[slot] = o_q;
          }
          nev += __popcll(evm);
        }
      };

      // wave w owns the 64-server blocks w, w + nwaves, w + 2 nwaves, ...
      int blk = wave;
      if (blk < nwords) { open_round(blk); issue_batch(blk, 0); }
      while (blk < nwords) {
        const int nblk = blk + nwaves;
        if (!final_pass) {
          const int g = (blk << 6) + lane;
          if (g < N) arrivals(g);
        }
        for (int g0 = 0; 8 * g0 < ne; g0 += Q) {
          if (g0 > 0) issue_batch(blk, g0);   // the first batch of a block was issued when the block was opened
#pragma unroll
          for (int t = 0; t < Q; ++t)
            if (8 * (g0 + t) < ne) process_group(t, g0 + t);   // wave-uniform
        }
        finalize(blk);
        if (nev > kEvPerWave - 64 || nblk >= nwords) {   // before the next block is opened: fewer live registers
          drain_events(nev);
          nev = 0;
        }
        if (nblk < nwords) { open_round(nblk); issue_batch(nblk, 0); }   // its loads travel while the arrivals are drawn
        blk = nblk;
      }
    }
    if (final_pass) break;   // wave-uniform; the barrier after the loop follows
    __syncthreads();

    // ================= arrivals into the class queues; ranks of completions and idle slots =================
    if (tid < K) {
      const int k = tid;
      if constexpr (AB) {   // abandonments come first: they free room in the queue
        if (n_leave_p) {
          L.cs[CS_QP + k] -= static_cast<int32_t>(n_leave_p);
          L.tl[k * kNTally + SIM_T_AB_P] += n_leave_p;
        }
        if (n_leave_d) {
          L.cs[CS_QD + k] -= static_cast<int32_t>(n_leave_d);
          L.tl[k * kNTally + SIM_T_AB_D] += n_leave_d;
          atomicSub(&L.cs[CS_DCOUNT], static_cast<int32_t>(n_leave_d));
          if constexpr (WS) L.cs[CS_QDS + k] -= static_cast<int32_t>(n_leave_d);
        }
        if constexpr (RR) {
          if (n_leave_dm) {
            L.cs[CS_QD + k] -= static_cast<int32_t>(n_leave_dm);
            L.tl[k * kNTally + SIM_T_AB_D] += n_leave_dm;
            atomicSub(&L.cs[CS_DCOUNT_M], static_cast<int32_t>(n_leave_dm));
          }
        }
      }
      const uint32_t a = L.acc[k];
      const uint32_t room = queue_cap - static_cast<uint32_t>(L.cs[CS_QP + k]);
      const uint32_t take = a < room ? a : room;
      // entries between head and tail: the waiting requests, with abandonment also the dead entries
      const uint32_t in_ring = static_cast<uint32_t>(AB ? L.sc[SC_QLEN + k] : L.cs[CS_QP + k]);
      uint32_t tail = static_cast<uint32_t>(L.cs[CS_QHEAD + k]) + in_ring;
      if (tail >= queue_cap) tail -= queue_cap;
      if constexpr (AB) {
        if (in_ring + take > queue_cap) atomicOr(&L.sc[SC_COMPACT], 1 << k);
        L.sc[SC_QLEN + k] = static_cast<int32_t>(in_ring + take);
      }
      L.sc[SC_TAKE + k] = static_cast<int32_t>(take);
      L.sc[SC_TAIL + k] = static_cast<int32_t>(tail);
      L.cs[CS_QP + k] += static_cast<int32_t>(take);
      L.tl[k * kNTally + SIM_T_A] += take;
      L.tl[k * kNTally + SIM_T_DROP_P] += a - take;
      if (a > take) L.tl[kMaxK * kNTally + SIM_G_OVERFLOW] = 1;
    }
    uint32_t ncomp_own = 0;   // (the first wave's count of completed prefills)
    if (tid < 64) {
      const uint32_t ncomp = rank_bitmap(L.bm_comp, L.pre_c, nwords_m, Mp);
      ncomp_own = ncomp;
      if (tid == 0) {
        L.sc[SC_NCOMP] = static_cast<int32_t>(ncomp);
        if constexpr (AB) {
          // a buffer ring that cannot hold this step's completions behind its dead entries is compacted first
          // (this wave has already taken the step's abandonments off the counters above)
          const uint32_t room = dbuf_cap - static_cast<uint32_t>(L.cs[CS_DCOUNT]);
          if (static_cast<uint32_t>(L.sc[SC_DLEN]) + (ncomp < room ? ncomp : room) > dbuf_cap) atomicOr(&L.sc[SC_COMPACT], 256);
          if constexpr (RR) {   // how the completions split between the two rings is not known yet: either may get all
            const uint32_t room_m = dbuf_cap - static_cast<uint32_t>(L.cs[CS_DCOUNT_M]);
            if (static_cast<uint32_t>(L.sc[SC_DLEN_M]) + (ncomp < room_m ? ncomp : room_m) > dbuf_cap) atomicOr(&L.sc[SC_COMPACT], 512);
          }
        }
      }
    }
    if (NT == 64 ? tid < 64 : (tid >= 64 && tid < 128)) {
      const uint32_t nidle = rank_bitmap(L.bm_idle, L.pre, nwords_m, M);   // idle prefill slots of the mixed group
      if (lane == 0) L.sc[SC_NIDLE] = static_cast<int32_t>(nidle);
    }
    // Two-buffer routers: word 1 of a completed prefill's block picks its group, and its rank within the group's
    // ring is the number of earlier completions (in server order) sent to the same group. Up to four waves take a
    // chunk of 64 completions each: before the barrier they fetch the request, draw its block and publish which of
    // their 64 go to the solo group; after it every chunk knows the counts before it and appends its requests.
    // What a wave fetched stays in its registers across the barrier.
    const int chunk_waves = nwaves < 4 ? nwaves : 4, chunk_first = nwaves >= 6 ? 2 : 0;
    const int my_chunk = wave - chunk_first;
    const bool chunk_wave = RR && my_chunk >= 0 && my_chunk < chunk_waves;
    bool c_active = false, c_solo = false;
    uint64_t c_jw = 0;
    uint32_t c_dl = kNever;
    int c_k = 0;
    auto draw_chunk = [&](uint32_t first, uint32_t ncomp_all) __attribute__((always_inline)) {
      const uint32_t j = first + 64u * static_cast<uint32_t>(my_chunk) + lane;
      c_active = j < ncomp_all;
      c_solo = false;
      c_dl = kNever;
      const int g = c_active ? select_bit(L.bm_comp, L.pre_c, nwords_m, j) : 0;
      c_jw = pf_job[g];   // (slot 0 for the lanes past the end: read, not used)
      uint32_t w[4];
      philox4x32_10(key0, key1, s, static_cast<uint32_t>(kStreamPatienceD), static_cast<uint32_t>(g), static_cast<uint32_t>(r), w);
      c_k = static_cast<int>(c_jw >> 29) & 7;
      c_solo = c_active && w[1] < p.solo_thr[c_k];
      if constexpr (AB) {
        if (c_active && ((p.ab_classes >> c_k) & 1u)) c_dl = s + a.pat_tab[static_cast<size_t>(c_k) * kTableSize + (w[0] >> 16)];
      }
      const uint64_t to_solo = __ballot(c_solo);
      if (lane == 0) L.solo_w[my_chunk] = to_solo;
    };
    if constexpr (RR) {
      if (chunk_wave) {
        // (each of these waves ranks the completion bitmap itself: the same values as the first wave writes)
        const uint32_t ncomp_all = wave == 0 ? ncomp_own : rank_bitmap(L.bm_comp, L.pre_c, nwords_m, Mp);
        draw_chunk(0u, ncomp_all);
      }
    }
    __syncthreads();
    if constexpr (AB) {
      // a ring that cannot hold this step's appends behind its dead entries is compacted first
      const int flags = L.sc[SC_COMPACT];   // cleared at the end of the step
      if (flags) {   // the same for every thread
        for (int k = wave; k < K; k += nwaves)
          if ((flags >> k) & 1) compact_queue(k, s, static_cast<uint32_t>(L.sc[SC_TAKE + k]));
        if ((flags & 256) && wave == nwaves - 1) compact_buffer(s, false);
        if constexpr (RR) {
          if ((flags & 512) && wave == (nwaves > 1 ? nwaves - 2 : 0)) compact_buffer(s, true);
        }
        __syncthreads();
      }
    }
    if constexpr (AB) {
      // One thread per accepted arrival of any class, so that the table reads of all classes are in flight together;
      // the last waves take them, while the first ones move the completions below. The accepted arrivals of a class
      // are exchangeable: the j-th of this step draws its patience.
      uint32_t upto[kMaxK];   // accepted arrivals of the classes up to and including k
      {
        uint32_t run = 0;
#pragma unroll
        for (int k = 0; k < kMaxK; ++k) {
          if (k < K) run += static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(L.sc[SC_TAKE + k]));
          upto[k] = run;
        }
      }
      for (uint32_t i = static_cast<uint32_t>((nwaves - 1 - wave) * 64 + lane); i < upto[kMaxK - 1]; i += NT) {
        int k = 0;
        uint32_t before = 0;
#pragma unroll
        for (int c = 0; c + 1 < kMaxK; ++c)
          if (i >= upto[c]) { k = c + 1; before = upto[c]; }
        const uint32_t j = i - before;
        uint32_t pos = static_cast<uint32_t>(L.sc[SC_TAIL + k]) + j;
        if (pos >= queue_cap) pos -= queue_cap;
        qring[static_cast<size_t>(k) * queue_cap + pos] = s;
        uint32_t dl = kNever;
        if ((p.ab_classes >> k) & 1u) {
          uint32_t w[4];
          philox4x32_10(key0, key1, s, static_cast<uint32_t>(kStreamPatienceP + k), j, static_cast<uint32_t>(r), w);
          dl = s + a.pat_tab[static_cast<size_t>(k) * kTableSize + (w[0] >> 16)];
          atomicAdd(&cal[static_cast<size_t>(k) * cal_n + (dl & p.cal_mask)], 1u);
        }
        qdl[static_cast<size_t>(k) * queue_cap + pos] = dl;
      }
    } else {
      for (int k = 0; k < K; ++k) {
        const uint32_t take = static_cast<uint32_t>(L.sc[SC_TAKE + k]), tail = static_cast<uint32_t>(L.sc[SC_TAIL + k]);
        for (uint32_t j = tid; j < take; j += NT) {
          uint32_t pos = tail + j;
          if (pos >= queue_cap) pos -= queue_cap;
          qring[static_cast<size_t>(k) * queue_cap + pos] = s;
        }
      }
    }
    // completed prefills join the decode buffer in ascending server order
    if constexpr (RR) {
      const uint32_t ncomp = static_cast<uint32_t>(L.sc[SC_NCOMP]);
      const uint32_t dc0 = static_cast<uint32_t>(L.cs[CS_DCOUNT]), dc1 = static_cast<uint32_t>(L.cs[CS_DCOUNT_M]);
      const uint32_t dh0 = static_cast<uint32_t>(L.cs[CS_DHEAD]), dh1 = static_cast<uint32_t>(L.cs[CS_DHEAD_M]);
      // ring entries before the tail (with abandonment the dead entries count)
      const uint32_t fill0 = AB ? static_cast<uint32_t>(L.sc[SC_DLEN]) : dc0, fill1 = AB ? static_cast<uint32_t>(L.sc[SC_DLEN_M]) : dc1;
      uint32_t seen0 = 0, seen1 = 0;   // completions sent to either group in the rounds before this one
      const uint32_t per_round = 64u * static_cast<uint32_t>(chunk_waves);
      for (uint32_t first = 0; first < ncomp; first += per_round) {   // wave-uniform; one round is the rule
        if (first > 0) {
          __syncthreads();   // every wave has read the words of the round before
          if (chunk_wave) draw_chunk(first, ncomp);
          __syncthreads();
        }
        uint32_t solo_before = 0, solo_round = 0;   // in the chunks before this wave's, in the whole round
        for (int c = 0; c < chunk_waves; ++c) {
          const uint32_t n = static_cast<uint32_t>(__popcll(L.solo_w[c]));
          if (c < my_chunk) solo_before += n;
          solo_round += n;
        }
        const uint32_t in_round = ncomp - first < per_round ? ncomp - first : per_round;
        if (chunk_wave && 64u * static_cast<uint32_t>(my_chunk) < in_round) {   // wave-uniform
          const bool active = c_active, solo = c_solo;
          const int k = c_k;
          const uint64_t bal0 = __ballot(active && solo), bal1 = __ballot(active && !solo);
          // (the chunks before this one are full)
          const uint32_t idx = solo ? seen0 + solo_before + static_cast<uint32_t>(__popcll(bal0 & lanes_below()))
                                    : seen1 + (64u * static_cast<uint32_t>(my_chunk) - solo_before) + static_cast<uint32_t>(__popcll(bal1 & lanes_below()));
          const bool kept = active && (solo ? dc0 : dc1) + idx < dbuf_cap;
          if (kept) {
            uint32_t pos = (solo ? dh0 + fill0 : dh1 + fill1) + idx;
            if (pos >= dbuf_cap) pos -= dbuf_cap;
            (solo ? dring : dring_m)[pos] = c_jw;
            if constexpr (AB) {
              (solo ? ddl : ddl_m)[pos] = c_dl;
              if (c_dl != kNever) atomicAdd(&(solo ? dcal : dcal_m)[static_cast<size_t>(k) * cal_n + (c_dl & p.cal_mask)], 1u);
            }
          }
          wave_count_by_class_i32(kept, k, K, &L.cs[CS_QD], 1);
          if constexpr (AB) {   // the weighted router also counts what waits in the solo group's buffer per class
            if constexpr (WS) wave_count_by_class_i32(kept && solo, k, K, &L.cs[CS_QDS], 1);
          }
          if (__ballot(active && !kept)) {
            wave_count_by_class(active && !kept, k, K, &L.tl[SIM_T_DROP_D], kNTally);
            if (lane == 0) L.tl[kMaxK * kNTally + SIM_G_OVERFLOW] = 1;
          }
        }
        seen0 += solo_round;
        seen1 += in_round - solo_round;
      }
      if (tid == 0) {   // what each ring accepted (a prefix of what it was sent)
        const uint32_t room0 = dbuf_cap - dc0, room1 = dbuf_cap - dc1;
        L.sc[SC_NCS] = static_cast<int32_t>(seen0 < room0 ? seen0 : room0);
        L.sc[SC_NCM] = static_cast<int32_t>(seen1 < room1 ? seen1 : room1);
      }
      __syncthreads();
    } else {
      const uint32_t ncomp = static_cast<uint32_t>(L.sc[SC_NCOMP]);
      const uint32_t dcount = static_cast<uint32_t>(L.cs[CS_DCOUNT]), dhead = static_cast<uint32_t>(L.cs[CS_DHEAD]);
      const uint32_t dfill = AB ? static_cast<uint32_t>(L.sc[SC_DLEN]) : dcount;   // ring entries before the tail
      // (64 to a wave; in a large workgroup not the first waves, which have ranked the bitmaps and go on to rank the
      // gate's candidates: the last waves, or with abandonment, whose arrivals the last two waves take, the ones before them)
      const int comp_turn = nwaves < 8 ? wave : (AB ? (2 * nwaves - 3 - wave) % nwaves : nwaves - 1 - wave);
      for (uint32_t j0 = static_cast<uint32_t>(comp_turn) * 64u; j0 < ncomp; j0 += NT) {   // wave-uniform trip count
        const uint32_t j = j0 + lane;
        const bool active = j < ncomp;
        int k = 0;
        bool kept = false;
        if (active) {
          const int g = select_bit(L.bm_comp, L.pre_c, nwords_m, j);
          const uint64_t jw = pf_job[g];
          k = static_cast<int>(jw >> 29) & 7;
          kept = dcount + j < dbuf_cap;
          if (kept) {
            uint32_t pos = dhead + dfill + j;
            if (pos >= dbuf_cap) pos -= dbuf_cap;
            dring[pos] = jw;
            if constexpr (AB) {   // patience for the wait in the decode buffer
              uint32_t dl = kNever;
              if ((p.ab_classes >> k) & 1u) {
                uint32_t w[4];
                philox4x32_10(key0, key1, s, static_cast<uint32_t>(kStreamPatienceD), static_cast<uint32_t>(g),
                              static_cast<uint32_t>(r), w);
                dl = s + a.pat_tab[static_cast<size_t>(k) * kTableSize + (w[0] >> 16)];
                atomicAdd(&dcal[static_cast<size_t>(k) * cal_n + (dl & p.cal_mask)], 1u);
              }
              ddl[pos] = dl;
            }
          }
        }
        wave_count_by_class_i32(active && kept, k, K, &L.cs[CS_QD], 1);
        if (__ballot(active && !kept)) {
          wave_count_by_class(active && !kept, k, K, &L.tl[SIM_T_DROP_D], kNTally);
          if (lane == 0) L.tl[kMaxK * kNTally + SIM_G_OVERFLOW] = 1;
        }
      }
    }

    // ================= 3.-5. prefill gate, decode routing and restart =================
    // Gate: the m-th waiting request of class k is a candidate; its position in the admission sequence is
    // the number of candidates that sort before it. Candidates are ranked in parallel; the idle prefill slot
    // of rank j (ascending server index) takes the candidate of rank j.
    // Routing: sequentially every job goes to the least-loaded feasible server, lowest index first: all
    // servers with the lowest decode count l get one job in index order, then all servers with at most l+1,
    // and so on. One pass fills up to kRouteLevels such levels at once. Level t takes take_t jobs, the first
    // of them job w_t of the pass; the server of rank q among those with at most lmin+t decodes takes job
    // w_t + q into slot lmin+t. Every lane places the jobs of its own server.
    // Both run side by side in passes of three segments with a barrier after each:
    //   A  gate: rank the candidates          routing: pass parameters from the load histogram, then the
    //                                          servers of each level are counted per 64-server word
    //   B  gate: admissions take their slots  routing: one wave per level turns the counts into ranks
    //   C  gate: class counters               routing: placement; in the last pass every lane then restarts
    //                                          its servers
    // One pass is the rule; more follow only when more than kAdmChunk slots are idle or the jobs reach past
    // kRouteLevels levels or into the mixed group.
    {
      const int dcount0 = L.cs[CS_DCOUNT];
      int jrem, next = 0;
      {
        const int ncp = L.sc[SC_NCOMP], room = static_cast<int>(dbuf_cap) - dcount0;
        jrem = dcount0 + (ncp < room ? ncp : room);
      }
      const uint32_t dhead0 = static_cast<uint32_t>(L.cs[CS_DHEAD]);
      // randomized router only: jobs left, jobs placed and ring head of the solo [0] and the mixed [1] group's buffer
      int jremL[2] = {0, 0}, nextL[2] = {0, 0}, takenL[2] = {0, 0};
      const uint32_t dheadL[2] = {dhead0, RR ? static_cast<uint32_t>(L.cs[CS_DHEAD_M]) : 0u};
      if constexpr (RR) {
        jremL[0] = dcount0 + L.sc[SC_NCS];
        jremL[1] = L.cs[CS_DCOUNT_M] + L.sc[SC_NCM];
        jrem = jremL[0] + jremL[1];
      }
      // abandonment only: ring entries of the decode buffer, this step's completions included
      uint32_t dlen_all = AB ? static_cast<uint32_t>(L.sc[SC_DLEN]) + static_cast<uint32_t>(RR ? L.sc[SC_NCS] : jrem - dcount0) : 0u;
      if (dlen_all > dbuf_cap) dlen_all = dbuf_cap;   // (never more: the ring was compacted if it had to be)
      uint32_t dlen_all_m = AB && RR ? static_cast<uint32_t>(L.sc[SC_DLEN_M]) + static_cast<uint32_t>(L.sc[SC_NCM]) : 0u;
      if (dlen_all_m > dbuf_cap) dlen_all_m = dbuf_cap;
      if constexpr (AB) {
        if (tid == 0) {
          L.sc[SC_DSCAN] = 0;
          if constexpr (RR) L.sc[SC_DSCAN_M] = 0;
        }
      }
      bool gate_on = true, route_on = jrem > 0;
      for (int pass = 0; gate_on || route_on; ++pass) {
        if (gate_on && pass > 0) {
          if (tid < 64) {
            const uint32_t nidle = rank_bitmap(L.bm_idle, L.pre, nwords_m, M);
            if (tid == 0) L.sc[SC_NIDLE] = static_cast<int32_t>(nidle);
          }
          __syncthreads();
        }
        if ((AB || gate_mode == SIM_GATE_FCFS) && pass == 0) __syncthreads();   // ring entries written above are read below
        // With abandonment the requests a routing pass places are first staged in LDS, by the waves that own the decode
        // buffers (each buffer has a wave of its own, on different SIMDs).
        const int ring_wave = nwaves >= 8 ? (WS ? 4 : nwaves / 2) : nwaves - 1;
        const int ring_wave_m = nwaves >= 8 ? ring_wave + 1 : nwaves - 1;
        // the weighted router's selection is long: it runs in segment A beside the gate's ranking, on waves that are
        // given nothing else to do there; the plain walk of a ring runs in segment B
        constexpr bool kStageEarly = AB && WS;
        // one wave walks a ring from where the last pass stopped and stages the next `need` waiting jobs
        auto stage_ring = [&](const uint64_t *ring, const uint32_t *dlr, uint32_t *calr, uint32_t hd, uint32_t len,
                              int scan_word, uint32_t need, int first_job) __attribute__((always_inline)) {
          uint32_t off = static_cast<uint32_t>(L.sc[scan_word]), found = 0, stop = off;
          // four chunks of 64 entries per round: deadlines and requests are loaded together
          for (; off < len && found < need; off += 256) {   // wave-uniform
            uint32_t dl4[4];
            uint64_t jw4[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
              const uint32_t i = off + 64u * u + lane;
              uint32_t pos = hd + i;
              if (pos >= dbuf_cap) pos -= dbuf_cap;
              dl4[u] = i < len ? dlr[pos] : 0u;   // (beyond the ring: counts as dead)
              jw4[u] = i < len ? ring[pos] : 0ull;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
              const uint32_t dl = dl4[u];
              const bool live = dl > s;
              const uint64_t bal = __ballot(live);
              const uint32_t rk = found + static_cast<uint32_t>(__popcll(bal & lanes_below()));
              const bool mine = live && rk < need;
              if (mine) {
                L.jobs[first_job + rk] = jw4[u];
                if (dl != kNever)
                  atomicSub(&calr[static_cast<size_t>((jw4[u] >> 29) & 7u) * cal_n + (dl & p.cal_mask)], 1u);
              }
              const uint64_t last = __ballot(mine && rk + 1 == need);
              if (last) stop = off + 64u * u + static_cast<uint32_t>(__ffsll(static_cast<long long>(last)));   // one past the last staged entry
              found += static_cast<uint32_t>(__popcll(bal));
            }
          }
          if (lane == 0) L.sc[scan_word] = static_cast<int32_t>(found >= need ? stop : len);   // (found < need: see the gate's scan)
        };
        // Weighted router: the pass's `need` placements in a pool each draw a class among those that still
        // wait in the pool's buffer (one after the other: a class that runs out drops from the later draws) and
        // take that class's requests in their order of arrival. The ring keeps the others where they are: an
        // entry that is taken gets a deadline that has passed, like an abandoned one.
        auto select_and_stage = [&](int pool, uint64_t *ring, uint32_t *dlr, uint32_t *calr, uint32_t hd, uint32_t len,
                                    int scan_word, int need, int first_job, int placed_before,
                                    int (&nsel)[kMaxK]) __attribute__((always_inline)) {
          for (int j = lane; j < need; j += 64) {
            uint32_t w[4];
            philox4x32_10(key0, key1, s, static_cast<uint32_t>(kStreamSelect + pool), static_cast<uint32_t>(placed_before + j),
                          static_cast<uint32_t>(r), w);
            L.sel_u[first_job + j] = w[0];
          }
          // Lane c knows class c's selection weight; what each class still has waiting (a pass takes at most
          // 256, larger counts are capped), which classes wait, and the running sums of their weights are
          // wave-uniform. The draws do not depend on one another until a class runs out, so they are evaluated
          // 64 at a time, one per lane: a draw's class is the number of running sums it has reached. If the
          // draws of a round would take more of a class than waits, the round ends with the draw that takes the
          // last one, the sums are recomputed without that class, and the next round starts behind it.
          int cntv = 0;
          uint32_t wtv = 0;
          if (lane < K) {
            const int solo_c = L.cs[CS_QDS + lane];
            cntv = pool == 0 ? solo_c : L.cs[CS_QD + lane] - solo_c;
            wtv = p.wsel[pool][lane];
          }
          cntv = cntv < 0 ? 0 : (cntv > 0xFFFF ? 0xFFFF : cntv);
          uint64_t waits = __ballot(cntv > 0);
          uint32_t cumv = wave_incl_scan(cntv > 0 ? wtv : 0u);
          int rem[kMaxK];
          uint32_t cum[kMaxK];
#pragma unroll
          for (int c = 0; c < kMaxK; ++c) {
            rem[c] = __builtin_amdgcn_readlane(cntv, c);
            cum[c] = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(cumv), c));
          }
          uint32_t total = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(cumv), 63));
          __builtin_amdgcn_wave_barrier();
          for (int done = 0; done < need;) {   // wave-uniform
            const int j = done + lane;
            const bool valid = j < need;
            const uint32_t u = valid ? L.sel_u[first_job + j] : 0u;
            const uint32_t x = __umulhi(u, total);
            int pick = 0;
#pragma unroll
            for (int c = 0; c < kMaxK; ++c)
              if (c < K) pick += x >= cum[c] ? 1 : 0;
            if (pick > K - 1) pick = K - 1;   // (no class waits: cannot happen, the pass takes no more than wait)
            int last = 64;   // lane of the first draw that takes the last waiting request of its class
#pragma unroll
            for (int c = 0; c < kMaxK; ++c) {
              if (c < K && rem[c] > 0) {   // wave-uniform
                const uint64_t bal = __ballot(valid && pick == c);
                if (__popcll(bal) >= rem[c]) {
                  const int pos = nth_set_bit(bal, rem[c] - 1);
                  last = pos < last ? pos : last;
                }
              }
            }
            const int n_valid = need - done < 64 ? need - done : 64;
            const int n_acc = last < 64 ? last + 1 : n_valid;
            const bool mine = lane < n_acc;
            if (mine) L.sel_co[first_job + j] = static_cast<uint16_t>(pick);
            bool ran_out = false;
#pragma unroll
            for (int c = 0; c < kMaxK; ++c) {
              if (c < K && rem[c] > 0) {   // wave-uniform
                const int took = __popcll(__ballot(mine && pick == c));
                rem[c] -= took;
                if (rem[c] == 0) { waits &= ~(1ull << c); ran_out = true; }
              }
            }
            if (ran_out) {   // wave-uniform
              cumv = wave_incl_scan(((waits >> lane) & 1ull) ? wtv : 0u);
#pragma unroll
              for (int c = 0; c < kMaxK; ++c) cum[c] = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(cumv), c));
              total = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(cumv), 63));
            }
            done += n_acc;
          }
          __builtin_amdgcn_wave_barrier();
          // how many earlier selections of the pass chose the same class: counted over the lanes, 64 at a time
#pragma unroll
          for (int c = 0; c < kMaxK; ++c) nsel[c] = 0;
          for (int j0 = 0; j0 < need; j0 += 64) {   // wave-uniform
            const int j = j0 + lane;
            const int c = j < need ? static_cast<int>(L.sel_co[first_job + j]) : -1;
            int ord = 0;
#pragma unroll
            for (int cc = 0; cc < kMaxK; ++cc) {
              if (cc < K) {   // wave-uniform
                const uint64_t bal = __ballot(c == cc);
                if (c == cc) ord = nsel[cc] + __popcll(bal & lanes_below());
                nsel[cc] += __popcll(bal);
              }
            }
            if (j < need) L.sel_co[first_job + j] = static_cast<uint16_t>(c | (ord << 3));
          }
          int base[kMaxK];
          {
            int run = 0;
#pragma unroll
            for (int c = 0; c < kMaxK; ++c) { base[c] = run; run += nsel[c]; }
          }
          __builtin_amdgcn_wave_barrier();
          for (int j = lane; j < need; j += 64) {
            const int co = L.sel_co[first_job + j], c = co & 7;
            int b = 0;
#pragma unroll
            for (int cc = 0; cc < kMaxK; ++cc)
              if (cc == c) b = base[cc];
            L.sel_j[first_job + b + (co >> 3)] = static_cast<uint16_t>(j);
          }
          __builtin_amdgcn_wave_barrier();
          // walk the ring from the first entry that may still wait; the o-th waiting request of class c met on
          // the way is taken if the pass selected that class more than o times
          uint32_t off = static_cast<uint32_t>(L.sc[scan_word]), stop = off, first_left = 0xFFFFFFFFu;
          int left = need;
          int seen[kMaxK];
#pragma unroll
          for (int c = 0; c < kMaxK; ++c) seen[c] = 0;
          for (; off < len && left > 0; off += 256) {   // wave-uniform
            uint32_t dl4[4], pos4[4];
            uint64_t jw4[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
              const uint32_t i = off + 64u * u + lane;
              uint32_t pos = hd + i;
              if (pos >= dbuf_cap) pos -= dbuf_cap;
              pos4[u] = pos;
              dl4[u] = i < len ? dlr[pos] : 0u;   // (beyond the ring: counts as gone)
              jw4[u] = i < len ? ring[pos] : 0ull;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
              if (left > 0) {   // wave-uniform
                const uint32_t dl = dl4[u];
                const bool live = dl > s;
                const int c = static_cast<int>(jw4[u] >> 29) & 7;
                int ord = 0, quota = 0, b = 0;
#pragma unroll
                for (int cc = 0; cc < kMaxK; ++cc) {
                  if (cc < K) {   // wave-uniform
                    const uint64_t bal = __ballot(live && c == cc);
                    if (c == cc) { ord = seen[cc] + __popcll(bal & lanes_below()); quota = nsel[cc]; b = base[cc]; }
                    seen[cc] += __popcll(bal);
                  }
                }
                const bool mine = live && ord < quota;
                if (mine) {
                  L.jobs[first_job + L.sel_j[first_job + b + ord]] = jw4[u];
                  dlr[pos4[u]] = 0u;   // gone from the buffer
                  if (dl != kNever) atomicSub(&calr[static_cast<size_t>(c) * cal_n + (dl & p.cal_mask)], 1u);
                }
                const uint64_t stay = __ballot(live && !mine), took = __ballot(mine);
                if (first_left == 0xFFFFFFFFu && stay)
                  first_left = off + 64u * u + static_cast<uint32_t>(__ffsll(static_cast<long long>(stay))) - 1u;
                if (took) {
                  left -= __popcll(took);
                  stop = off + 64u * u + 64u - static_cast<uint32_t>(__clzll(static_cast<long long>(took)));   // one past the last taken entry
                }
              }
            }
          }
          // the next pass (and the head, at the end of the step) starts at the first entry that still waits
          if (lane == 0)
            L.sc[scan_word] = static_cast<int32_t>(first_left != 0xFFFFFFFFu ? first_left : (left > 0 ? len : stop));
        };
        auto stage_pass = [&](int total_pass) __attribute__((always_inline)) {
          // (each buffer has a wave of its own, on different SIMDs; in a large workgroup these waves leave the
          // level counts below to the others)
          if constexpr (RR) {
            if (wave == ring_wave) {
              if constexpr (WS) {
                int nsel_s[kMaxK];
#pragma unroll
                for (int c = 0; c < kMaxK; ++c) nsel_s[c] = 0;
                if (takenL[0] > 0)
                  select_and_stage(0, dring, ddl, dcal, dheadL[0], dlen_all, SC_DSCAN, takenL[0], 0, nextL[0], nsel_s);
                // what the pass took from the solo group's buffer per class comes off that buffer's counts in
                // segment C: the other buffer's wave reads them meanwhile (what waits in the mixed group's buffer is
                // the class total less the solo buffer's share, and the total follows the placements later)
                if (lane < K) {
                  int mine = 0;
#pragma unroll
                  for (int c = 0; c < kMaxK; ++c)
                    if (c == lane) mine = nsel_s[c];
                  L.sel_n[lane] = mine;
                }
              } else {
                if (takenL[0] > 0)
                  stage_ring(dring, ddl, dcal, dheadL[0], dlen_all, SC_DSCAN, static_cast<uint32_t>(takenL[0]), 0);
              }
            }
            if (wave == ring_wave_m && takenL[1] > 0) {
              if constexpr (WS) {
                int nsel_m[kMaxK];
                select_and_stage(1, dring_m, ddl_m, dcal_m, dheadL[1], dlen_all_m, SC_DSCAN_M, takenL[1], takenL[0], nextL[1], nsel_m);
              } else {
                stage_ring(dring_m, ddl_m, dcal_m, dheadL[1], dlen_all_m, SC_DSCAN_M, static_cast<uint32_t>(takenL[1]), takenL[0]);
              }
            }
          } else {
            if (wave == ring_wave) stage_ring(dring, ddl, dcal, dhead0, dlen_all, SC_DSCAN, static_cast<uint32_t>(total_pass), 0);
          }
        };

        // ---------------- segment A ----------------
        int nadm = 0, nidle = 0, ncand_pass = 0;
        if (gate_on) {
          nidle = __builtin_amdgcn_readfirstlane(L.sc[SC_NIDLE]);
          const int limit = nidle < kAdmChunk ? nidle : kAdmChunk;
          int cnt[kMaxK], qp[kMaxK], xs[kMaxK], ncand = 0;
          uint32_t head[kMaxK];
          const int cs_lane = L.cs[lane];   // the class state, one word per lane: one trip to LDS
#pragma unroll
          for (int k = 0; k < kMaxK; ++k) {
            // wave-uniform values, kept in scalar registers
            qp[k] = k < K ? __builtin_amdgcn_readlane(cs_lane, CS_QP + k) : 0;
            xs[k] = k < K ? __builtin_amdgcn_readlane(cs_lane, CS_X + k) : 0;
            head[k] = k < K ? static_cast<uint32_t>(__builtin_amdgcn_readlane(cs_lane, CS_QHEAD + k)) : 0u;
            const bool eligible = k < K && qp[k] > 0 && (gate_mode != SIM_GATE_OCCUPANCY || L.gtab[GT_INVX * kMaxK + k] > 0.0);
            cnt[k] = eligible ? (qp[k] < limit ? qp[k] : limit) : 0;
            ncand += cnt[k];
          }
          nadm = ncand < limit ? ncand : limit;
          ncand_pass = ncand;
          if constexpr (AB) {
            // where the candidates sit in their rings: a wave per class walks from the head past the dead entries
            // (the last waves take this: the first ones rank the candidates below)
            for (int k = nwaves - 1 - wave; k < K; k += nwaves) {   // wave-uniform
              uint32_t need = 0;
#pragma unroll
              for (int kk = 0; kk < kMaxK; ++kk)
                if (kk == k) need = static_cast<uint32_t>(cnt[kk]);
              uint32_t qlen = static_cast<uint32_t>(L.sc[SC_QLEN + k]);
              if (qlen > queue_cap) qlen = queue_cap;
              const uint32_t hd = static_cast<uint32_t>(L.cs[CS_QHEAD + k]);
              const uint32_t *dlr = qdl + static_cast<size_t>(k) * queue_cap;
              uint32_t found = 0;
              // four chunks of 64 entries per round: their deadlines are loaded together, one trip to memory
              for (uint32_t off = 0; off < qlen && found < need; off += 256) {   // wave-uniform
                uint32_t dl4[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                  const uint32_t i = off + 64u * u + lane;
                  uint32_t pos = hd + i;
                  if (pos >= queue_cap) pos -= queue_cap;
                  dl4[u] = i < qlen ? dlr[pos] : 0u;   // (beyond the ring: counts as dead)
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                  const uint32_t i = off + 64u * u + lane;
                  const bool live = dl4[u] > s;
                  const uint64_t bal = __ballot(live);
                  const uint32_t rk = found + static_cast<uint32_t>(__popcll(bal & lanes_below()));
                  if (live && rk < need) L.live_off[k * kAdmChunk + rk] = i;
                  found += static_cast<uint32_t>(__popcll(bal));
                }
              }
              // (the ring holds as many live entries as the class counter says; if it ever did not, the
              // candidates beyond them would point at the head entry)
              for (uint32_t rk = found + lane; rk < need; rk += 64) L.live_off[k * kAdmChunk + rk] = 0;
              if (lane == 0) L.sc[SC_LEAD + k] = (need > 0 && found > 0) ? 1 : 0;
            }
            // only the FCFS gate reads the offsets while it ranks the candidates; the other gates first use them
            // after the barrier that ends this segment
            if (gate_mode == SIM_GATE_FCFS) __syncthreads();
          }
          // The admissions take the first nadm idle prefill slots, whatever their order: the slot bitmaps are
          // updated here a word at a time (no atomics).
          // A wave takes a word, a lane a slot; the slot of every admission rank goes into a table.
          for (int w = wave; w < nwords_m; w += nwaves) {   // wave-uniform
            const uint64_t idle_all = L.bm_idle[w], busy_w = L.bm_busy[w], touch_w = L.bm_touch[w];
            const uint64_t idle = idle_all & bits_below(w, M);   // the gate admits to the mixed group only
            const int before = static_cast<int>(L.pre[w]);   // idle slots in the words before this one
            uint64_t adm = 0;
            if (before < nadm)
              adm = before + __popcll(idle) <= nadm ? idle : idle & ((1ull << nth_set_bit(idle, nadm - before)) - 1ull);
            if (adm) {
              if ((adm >> lane) & 1ull)
                L.adm_slot[before + __popcll(adm & lanes_below())] = static_cast<uint16_t>((w << 6) + lane);
              if (lane == 0) {
                L.bm_idle[w] = idle_all & ~adm;
                L.bm_touch[w] = touch_w | (adm & ~busy_w);   // an idle server is given work
              }
            }
          }
          // (the waves that run the weighted router's selection in this segment rank no candidates)
          int rank_first = wave_base, rank_step = NT;
          if constexpr (kStageEarly) {
            if (nwaves >= 8) {
              rank_step = NT - 128;
              rank_first = wave < ring_wave ? wave_base : wave_base - 128;
            }
          }
          const bool ranks = !(kStageEarly && nwaves >= 8 && (wave == ring_wave || wave == ring_wave_m));   // wave-uniform
          for (int c0 = rank_first; ranks && c0 < ncand; c0 += rank_step) {   // wave-uniform trip count
            const int c = c0 + lane;
            bool admitted = false;
            int k = 0, m = c;
            if (c < ncand) {
#pragma unroll
            for (int kk = 0; kk < kMaxK - 1; ++kk)
              if (k == kk && m >= cnt[kk]) { m -= cnt[kk]; k = kk + 1; }
            // this candidate's own key: its class's targets and counters, fetched by class (one trip to LDS)
            const ClassTargets own = load_targets(L.gtab, k);
            const int xs_own = L.cs[CS_X + k], qp_own = L.cs[CS_QP + k];
            const uint32_t head_own = static_cast<uint32_t>(L.cs[CS_QHEAD + k]);
            const GateKey key = gate_key(gate_mode, queue_cap, own, qring, lo_tab, xs_own, qp_own, head_own, k, m, kAdmChunk);
            int rank = m;
#pragma unroll
            for (int k2 = 0; k2 < kMaxK; ++k2) {
              if (k2 == k || cnt[k2] == 0 || rank >= nadm) continue;
              // number of candidates of class k2 that sort before this one: they form a prefix of the class
              const ClassTargets t2 = load_targets(L.gtab, k2);
              int lo = 0, hi = cnt[k2];
              if (gate_mode == SIM_GATE_OCCUPANCY) {
                // the key is linear in the sequence number: bracket the crossing next to its estimate with two
                // exact comparisons, so the search below runs over a few candidates only (or, if the
                // estimate is off, over the side the comparisons point to)
                const double est = key.a * t2.xstar - (static_cast<double>(xs[k2]) - t2.nx);
                const int g0 = est > 0.0 ? (est < static_cast<double>(hi) ? static_cast<int>(est) : hi) : 0;
                const int l2 = g0 > 1 ? g0 - 1 : 0, h2 = g0 + 2 < hi ? g0 + 2 : hi;
                if (l2 > 0) {
                  if (gate_before(gate_key(gate_mode, queue_cap, t2, qring, lo_tab, xs[k2], qp[k2], head[k2], k2, l2 - 1, kAdmChunk), k2, key, k)) lo = l2; else hi = l2 - 1;
                }
                if (h2 < hi) {
                  if (gate_before(gate_key(gate_mode, queue_cap, t2, qring, lo_tab, xs[k2], qp[k2], head[k2], k2, h2, kAdmChunk), k2, key, k)) lo = h2 + 1; else hi = h2;
                }
              }
              while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (gate_before(gate_key(gate_mode, queue_cap, t2, qring, lo_tab, xs[k2], qp[k2], head[k2], k2, mid, kAdmChunk), k2, key, k)) lo = mid + 1; else hi = mid;
              }
              rank += lo;
            }
            admitted = rank < nadm;
            if (admitted) L.adm[rank] = static_cast<uint32_t>(k) | (static_cast<uint32_t>(m) << 3);
            }
            // admissions per class: counted over the wave first (candidates of a class sit in neighbouring lanes)
            for (int c = 0; c < K; ++c) {
              const uint64_t mk = __ballot(admitted && k == c);
              if (mk && lane == 0) atomicAdd(&L.sc[SC_ADMK + c], __popcll(mk));
            }
          }
        }
        // routing pass: up to kRouteLevels levels, first of the solo group (servers M..N-1), then, if that group
        // is full by then, of the mixed group (servers 0..M-1, one slot less). Level t of group G holds the
        // servers of G with at most lminG + (t - firstG) decodes.
        int nl = 0, total = 0;
        int lminG[2] = {0, 0}, nG[2] = {0, 0}, csumG[2] = {0, 0}, tlastG[2] = {0, 0};
        // Placements on a mixed-group server must see every admission of the step (it decides whether the job
        // counts as mixed or solo decode): while the gate may need another pass, only the solo group is routed.
        const bool gate_unfinished = gate_on && nadm == kAdmChunk && nidle > kAdmChunk;
        bool route_wait = false;   // nothing to route in this pass, but the mixed group is still to come
        if (route_on) {
          // (every wave computes the same values and stores them: no broadcast, no barrier)
          // (with abandonment a pass places no more jobs than are staged in LDS)
          const int jpass = AB && jrem > kJobsLds ? kJobsLds : jrem;
          int rem_jobs = jpass;
          // The load histograms of both groups (servers per decode count below the cap) are read once, one bin per
          // lane and register; the lowest non-empty level and the counts of the levels above it then come from
          // ballots and lane reads instead of a chain of LDS round trips.
          uint32_t hv[2][2];
#pragma unroll
          for (int gi = 0; gi < 2; ++gi) {
            hv[gi][0] = L.lh[gi * kLoadBins + lane];
            hv[gi][1] = L.lh[gi * kLoadBins + 64 + lane];
          }
          auto lowest_level = [&](int gi, int capg) __attribute__((always_inline)) -> int {
            const uint64_t nz0 = __ballot(lane < capg && hv[gi][0] != 0);
            if (nz0) return __ffsll(static_cast<long long>(nz0)) - 1;
            const uint64_t nz1 = __ballot(64 + lane < capg && hv[gi][1] != 0);
            return nz1 ? 63 + __ffsll(static_cast<long long>(nz1)) : -1;
          };
          auto level_count = [&](int gi, int level) __attribute__((always_inline)) -> uint32_t {   // level: wave-uniform, below 128
            const int lo = __builtin_amdgcn_readlane(static_cast<int>(hv[gi][0]), level & 63);
            const int hi = __builtin_amdgcn_readlane(static_cast<int>(hv[gi][1]), level & 63);
            return static_cast<uint32_t>(level < 64 ? lo : hi);
          };
          if constexpr (RR) {
            // each group takes jobs from its own ring; the pass's list holds the solo ring's jobs first and is
            // never longer than what is staged in LDS
            int listed = 0;
            takenL[0] = takenL[1] = 0;
#pragma unroll
            for (int gi = 0; gi < 2; ++gi) {
              const int glo = gi == 0 ? M : 0, ghi = gi == 0 ? N : M;
              const int capg = gi == 0 ? B : B - 1;
              int rem_g = jremL[gi] < kJobsLds - listed ? jremL[gi] : kJobsLds - listed;
              const int start_g = rem_g;
              if (glo >= ghi || nl >= kRouteLevels || rem_g <= 0 || (gi == 1 && gate_unfinished)) continue;   // wave-uniform
              const int lm = lowest_level(gi, capg);
              if (lm < 0) continue;   // no free slot in this group
              lminG[gi] = lm;
              for (int u = 0; nl < kRouteLevels && rem_g > 0 && lm + u < capg; ++u) {
                csumG[gi] += static_cast<int>(level_count(gi, lm + u));
                const int tk = csumG[gi] < rem_g ? csumG[gi] : rem_g;
                if (lane == 0) { L.sc[SC_TAKE_T + nl] = tk; L.sc[SC_W_T + nl] = listed + (start_g - rem_g); }
                rem_g -= tk;
                tlastG[gi] = tk;
                ++nG[gi];
                ++nl;
              }
              takenL[gi] = start_g - rem_g;
              listed += takenL[gi];
            }
            rem_jobs = jpass - listed;
          } else {
#pragma unroll
          for (int gi = 0; gi < 2; ++gi) {
            const int glo = gi == 0 ? M : 0, ghi = gi == 0 ? N : M;
            const int capg = gi == 0 ? B : B - 1;
            if (glo >= ghi || nl >= kRouteLevels || rem_jobs <= 0 || (gi == 1 && gate_unfinished)) continue;   // wave-uniform
            const int lm = lowest_level(gi, capg);
            if (lm < 0) continue;   // no free slot in this group
            lminG[gi] = lm;
            for (int u = 0; nl < kRouteLevels && rem_jobs > 0 && lm + u < capg; ++u) {
              csumG[gi] += static_cast<int>(level_count(gi, lm + u));
              const int tk = csumG[gi] < rem_jobs ? csumG[gi] : rem_jobs;
              if (lane == 0) { L.sc[SC_TAKE_T + nl] = tk; L.sc[SC_W_T + nl] = jpass - rem_jobs; }
              rem_jobs -= tk;
              tlastG[gi] = tk;
              ++nG[gi];
              ++nl;
            }
          }
          }
          total = jpass - rem_jobs;
          if (nl == 0) {
            if (gate_unfinished) route_wait = true;
            else route_on = false;   // every slot is taken: the jobs stay in the buffer
          } else {
            // Waves that count the servers of each level, and this wave's place among them. With abandonment the
            // requests the pass places are first staged in LDS by the waves that own the decode buffers: a large
            // workgroup gives them no counting to do, so that the staging runs beside the gate's ranking.
            int cw = wave, cn = nwaves;
            if constexpr (kStageEarly) {
              stage_pass(total);
              if (nwaves >= 8) {
                constexpr int n_ring = RR ? 2 : 1;
                cn = nwaves - n_ring;
                cw = wave < ring_wave ? wave : wave - n_ring;   // (negative for the buffers' waves)
                if (wave >= ring_wave && wave < ring_wave + n_ring) cw = nwords;   // nothing to count
              }
            }
            // In a sixteen-wave workgroup the first waves also rank the gate's candidates, the first four most of
            // them: when there are candidates for four waves or more, the words are dealt out in runs of unequal
            // length (2 : 7 : 11 : 19 per wave of each quarter).
            int w_lo = cw, w_hi = nwords, w_next = cn;
            if (nwaves == 16 && ncand_pass >= 256) {
              // (halves of a word: with the weighted router waves 4 and 5 run the selection and the others take runs of
              // 6, 6, 6, 6, 0, 0, then 11 a wave and 16.5 for the last four)
              const int q = wave >> 2, o = wave & 3;   // quarter of the workgroup, place in it
              int lo2, len2;   // start and length of the run, in halves of a word (312 in all)
              if (kStageEarly) {
                lo2 = q == 0 ? 12 * o : q == 1 ? (o < 2 ? 48 : 48 + 22 * (o - 2)) : q == 2 ? 92 + 22 * o : 180 + 33 * o;
                len2 = q == 0 ? 12 : q == 1 ? (o < 2 ? 0 : 22) : q == 2 ? 22 : 33;
              } else {
                lo2 = q == 0 ? 4 * o : q == 1 ? 16 + 14 * o : q == 2 ? 72 + 22 * o : 160 + 38 * o;
                len2 = q == 0 ? 4 : q == 1 ? 14 : q == 2 ? 22 : 38;
              }
              w_lo = nwords * lo2 / 312;
              w_hi = nwords * (lo2 + len2) / 312;
              w_next = 1;
            }
            // four blocks per round: their decode counts are read together, then compared level by level
            for (int w0 = w_lo; w0 < w_hi; w0 += 4 * w_next) {
              int tmin4[4], tend4[4];
#pragma unroll
              for (int u = 0; u < 4; ++u) {
                const int wi = w0 + u * w_next;
                const int g = (wi << 6) + lane;
                tmin4[u] = 0; tend4[u] = 0;
                if (wi < w_hi && g < N) {
                  const int gi = g >= M ? 0 : 1;
                  const int first = gi == 0 ? 0 : nG[0];
                  const int d = static_cast<int>(L.loads[g]) - (gi == 0 ? lminG[0] : lminG[1]);
                  tmin4[u] = first + (d > 0 ? d : 0);
                  tend4[u] = first + (gi == 0 ? nG[0] : nG[1]);
                }
              }
#pragma unroll
              for (int u = 0; u < 4; ++u) {
                const int wi = w0 + u * w_next;
                if (wi < w_hi) {   // wave-uniform
#pragma unroll
                  for (int t = 0; t < kRouteLevels; ++t) {
                    if (t < nl) {
                      const uint64_t bal = __ballot(t >= tmin4[u] && t < tend4[u]);
                      if (lane == 0) L.pre_lvl[t * nwords + wi] = static_cast<uint32_t>(__popcll(bal));
                    }
                  }
                }
              }
            }
          }
        }
        __syncthreads();

        // ---------------- segment B ----------------
        bool gate_more = false;
        bool a_active = false;   // this lane's admission of the pass: slot, class, arrival stamp, decodes beside it
        int a_g = 0, a_k = 0;
        uint32_t a_stamp = 0;
        uint64_t a_nc = 0;
        if (gate_on) {
          if (pass == 0 && tid == 0) {   // the completions of this step are in the buffer
            if constexpr (RR) { L.cs[CS_DCOUNT] = jremL[0]; L.cs[CS_DCOUNT_M] = jremL[1]; }
            else L.cs[CS_DCOUNT] = jrem;
          }
          // Admission j goes to the idle prefill slot of rank j; one thread per admission (a pass admits no more than
          // the workgroup has threads). Here the wave only reads what segment C changes (queue heads, decode
          // counts of the servers) and asks memory for the request's stamp; the rest follows in segment C.
          if (wave_base < nadm) {   // wave-uniform
            const int j = wave_base + lane;
            a_active = j < nadm;
            if (a_active) {
              a_g = L.adm_slot[j];
              const uint32_t e = L.adm[j];
              a_k = static_cast<int>(e & 7u);
              uint32_t pos = static_cast<uint32_t>(L.cs[CS_QHEAD + a_k]) + (AB ? L.live_off[a_k * kAdmChunk + (e >> 3)] : (e >> 3));
              if (pos >= queue_cap) pos -= queue_cap;
              a_stamp = qring[static_cast<size_t>(a_k) * queue_cap + pos];
              if constexpr (AB) {   // the request no longer waits: it leaves the calendar of its deadline
                const uint32_t dl = qdl[static_cast<size_t>(a_k) * queue_cap + pos];
                if (dl != kNever) atomicSub(&cal[static_cast<size_t>(a_k) * cal_n + (dl & p.cal_mask)], 1u);
              }
              if (L.loads[a_g]) a_nc = n_cls[a_g];   // (before this pass's placements on the server)
            }
          }
          if (nadm == kAdmChunk && nidle > kAdmChunk) {   // rare: more idle slots than one pass serves
            for (int k = 0; k < K; ++k) {
              const bool eligible = gate_mode != SIM_GATE_OCCUPANCY || L.gtab[GT_INVX * kMaxK + k] > 0.0;
              if (eligible && L.cs[CS_QP + k] - L.sc[SC_ADMK + k] > 0) gate_more = true;
            }
          }
        }
        if (route_on && !route_wait) {
          // the requests this pass places are staged in LDS
          const int nstage = total < kJobsLds ? total : kJobsLds;
          if constexpr (AB) {
            if constexpr (!kStageEarly) stage_pass(total);
          } else if constexpr (RR) {
            for (int j = tid; j < nstage; j += NT) {
              const int li = j < takenL[0] ? 0 : 1;
              uint32_t pos = dheadL[li] + static_cast<uint32_t>(nextL[li] + (li ? j - takenL[0] : j));
              if (pos >= dbuf_cap) pos -= dbuf_cap;
              if (pos >= dbuf_cap) pos -= dbuf_cap;
              L.jobs[j] = (li ? dring_m : dring)[pos];
            }
          } else {
          for (int j = tid; j < nstage; j += NT) {
            uint32_t pos = dhead0 + static_cast<uint32_t>(next + j);
            if (pos >= dbuf_cap) pos -= dbuf_cap;
            if (pos >= dbuf_cap) pos -= dbuf_cap;
            L.jobs[j] = dring[pos];
          }
          }
          // counts -> exclusive prefix over the words; the last waves take this
          for (int t = nwaves - 1 - wave; t < nl; t += nwaves) {
            uint32_t *pre = L.pre_lvl + t * nwords;
            uint32_t running = 0;
            for (int base = 0; base < nwords; base += 64) {
              const int w = base + lane;
              const uint32_t v = w < nwords ? pre[w] : 0u;
              const uint32_t inc = wave_incl_scan(v);
              if (w < nwords) pre[w] = running + inc - v;
              running += static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(inc), 63));
            }
          }
        }
        __syncthreads();

        // ---------------- segment C ----------------
        if (gate_on && wave_base < nadm) {   // wave-uniform: the admissions this wave began in segment B
          uint64_t wait = 0;
          if (a_active) {
            const int g = a_g, k = a_k;
            wait = static_cast<uint64_t>(s - a_stamp);
            uint32_t w[4];
            philox4x32_10(key0, key1, s, 1u, static_cast<uint32_t>(g), static_cast<uint32_t>(r), w);
            const uint32_t Pl = a.len_tab[(static_cast<size_t>(k) * 2 + 0) * kTableSize + (w[0] >> 16)];
            const uint32_t Dl = a.len_tab[(static_cast<size_t>(k) * 2 + 1) * kTableSize + (w[1] >> 16)];
            pf_job[g] = static_cast<uint64_t>(a_stamp) | (static_cast<uint64_t>(k) << 29) |
                        (static_cast<uint64_t>(Pl - 1) << 32) | (static_cast<uint64_t>(Dl - 1) << 48);
            // an idle prefill slot implies that the running iteration holds no chunk
            L.rem[g] = static_cast<uint16_t>(Pl);
            const uint64_t bit = 1ull << (g & 63);
            // at an iteration boundary the next iteration carries a chunk: tally the untallied ones first
            if ((L.bm_busy[g >> 6] & bit) && (L.bm_due[g >> 6] & bit) && L.pend[g])
              atomicOr(reinterpret_cast<unsigned long long *>(&L.bm_flush[g >> 6]), bit);
          }
          wave_sum_by_class(a_active, a_k, K, wait, &L.tl[SIM_T_WAIT_STEPS], kNTally);
          uint64_t even, odd;   // co-resident decodes switch solo -> mixed
          wave_sum_bytes(a_nc, even, odd);
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
        if (gate_on && tid < K) {   // class counters follow the admissions of this pass
          const int k = tid, adm_k = L.sc[SC_ADMK + k];
          // ring entries the head moves past: the admitted requests; with abandonment also the dead entries
          // before the last of them (before the first waiting request when none was admitted)
          uint32_t past = static_cast<uint32_t>(adm_k);
          if constexpr (AB) {
            past = adm_k ? L.live_off[k * kAdmChunk + adm_k - 1] + 1u : (L.sc[SC_LEAD + k] ? L.live_off[k * kAdmChunk] : 0u);
            if (past) {
              L.sc[SC_QLEN + k] -= static_cast<int32_t>(past);
              if (!adm_k) {
                uint32_t h = static_cast<uint32_t>(L.cs[CS_QHEAD + k]) + past;
                if (h >= queue_cap) h -= queue_cap;
                L.cs[CS_QHEAD + k] = static_cast<int32_t>(h);
              }
            }
          }
          if (adm_k) {
            uint32_t h = static_cast<uint32_t>(L.cs[CS_QHEAD + k]) + past;
            if (h >= queue_cap) h -= queue_cap;
            L.cs[CS_QHEAD + k] = static_cast<int32_t>(h);
            L.cs[CS_QP + k] -= adm_k;
            L.cs[CS_X + k] += adm_k;
            L.tl[k * kNTally + SIM_T_U_P] += static_cast<uint64_t>(adm_k);
            L.sc[SC_ADMK + k] = 0;
          }
        }
        if (route_on && !route_wait) {
          int take_r[kRouteLevels], w_r[kRouteLevels];
#pragma unroll
          for (int t = 0; t < kRouteLevels; ++t) {
            take_r[t] = __builtin_amdgcn_readfirstlane(L.sc[SC_TAKE_T + t]);
            w_r[t] = __builtin_amdgcn_readfirstlane(L.sc[SC_W_T + t]);
          }
          // (sixteen waves, a pass with admissions: the first waves have just finished those, so they take shorter runs of
          // words, and the later waves of a SIMD, which are served first, longer ones: 4, 4, 7, 9, then 9, 11 and 13 a wave)
          int c_lo = wave, c_hi = nwords, c_next = nwaves;
          if (nwaves == 16 && gate_on && nadm > 32) {
            // (with two buffers a word costs more, and the last waves gain less from being served first: 5, 5, 8, 10,
            // then 10, 11, 11)
            auto run_start = [](int i) {
              if (RR) return i < 2 ? 5 * i : i == 2 ? 10 : i == 3 ? 18 : i < 8 ? 28 + 10 * (i - 4) : 68 + 11 * (i - 8);
              return i < 2 ? 4 * i : i == 2 ? 8 : i == 3 ? 15 : i < 8 ? 24 + 9 * (i - 4) : i < 12 ? 60 + 11 * (i - 8) : 104 + 13 * (i - 12);
            };
            c_lo = nwords * run_start(wave) / 156;
            c_hi = nwords * run_start(wave + 1) / 156;
            c_next = 1;
          }
          for (int wi = c_lo; wi < c_hi; wi += c_next) {
            const int gw = wi << 6;
            const int g = gw + lane;
            const uint64_t bit = 1ull << lane;
            // what the block needs from LDS is read in one go
            const int n_own = g < N ? static_cast<int>(L.loads[g]) : 0;   // decodes of this lane's server
            const int pend_own = g < N ? static_cast<int>(L.pend[g]) : 0;
            const uint64_t busy_word = L.bm_busy[wi], due_word = L.bm_due[wi], idle_word = L.bm_idle[wi];
            int pre_r[kRouteLevels];
#pragma unroll
            for (int t = 0; t < kRouteLevels; ++t)
              pre_r[t] = __builtin_amdgcn_readfirstlane(static_cast<int>(L.pre_lvl[(t < nl ? t : 0) * nwords + wi]));
            // levels tmin..tend-1 of the pass hold this lane's server
            const int gi = g >= M ? 0 : 1;
            const int first = gi == 0 ? 0 : nG[0], my_n = gi == 0 ? nG[0] : nG[1], my_lmin = gi == 0 ? lminG[0] : lminG[1];
            const int tend = g < N ? first + my_n : 0;
            const int tmin = first + (n_own > my_lmin ? n_own - my_lmin : 0);
            if (__ballot(tmin < tend) == 0) continue;   // wave-uniform
            const bool busy0 = busy_word & bit, at_boundary = due_word & bit;
            const bool mid = busy0 && !at_boundary;   // a job placed now joins at the next restart
            const bool has_prefill = g < Mp && !(idle_word & bit);
            // the new decode is not part of the iterations still to be tallied for this server
            const bool joins = mid || (at_boundary && pend_own != 0);
            bool got = false, got_last = false;
#pragma unroll
            for (int t = 0; t < kRouteLevels; ++t) {
              if (t < nl) {   // wave-uniform
                const bool in = t >= tmin && t < tend;
                const uint64_t bal = __ballot(in);
                if (bal) {
                  const int q = pre_r[t] + __popcll(bal & lanes_below());
                  if (in && q < take_r[t]) {
                    got = true;
                    got_last = t == tend - 1;
                    const int j = w_r[t] + q;   // position in this pass
                    uint64_t jw;
                    if (j < kJobsLds) {
                      jw = L.jobs[j];
                    } else {
                      uint32_t pos = dhead0 + static_cast<uint32_t>(next + j);
                      if (pos >= dbuf_cap) pos -= dbuf_cap;
                      if (pos >= dbuf_cap) pos -= dbuf_cap;
                      jw = dring[pos];
                    }
                    const int k = static_cast<int>(jw >> 29) & 7;
                    const uint32_t Dl = static_cast<uint32_t>(jw >> 48) + 1;
                    const int nd = my_lmin + (t - first);   // the server holds exactly this many decodes by now
                    fin[static_cast<size_t>(g) * BS + nd] = L.iter[g] + Dl + (mid ? 1u : 0u);
                    job[static_cast<size_t>(g) * BS + nd] = jw;
                    atomicAdd(reinterpret_cast<unsigned long long *>(&n_cls[g]), 1ull << (8 * k));
                    if (joins) atomicAdd(reinterpret_cast<unsigned long long *>(&n_join[g]), 1ull << (8 * k));
                    lds_add64(&L.tl[k * kNTally + (has_prefill ? SIM_T_U_DM : SIM_T_U_DS)], 1);
                    atomicAdd(&L.cs[(has_prefill ? CS_YM : CS_YS) + k], 1);
                    atomicSub(&L.cs[CS_QD + k], 1);
                  }
                }
              }
            }
            // marks for the next completion pass: decodes that are not part of the untallied iterations;
            // untallied iterations to tally before the restart; idle servers that now hold work
            const uint64_t join_m = __ballot(got && joins), flush_m = __ballot(got && joins && !mid);
            const uint64_t touch_m = __ballot(got && !busy0);
            if (lane == 0) {   // fire and forget: nothing here waits for the old words
              if (join_m) atomicOr(reinterpret_cast<unsigned long long *>(&L.bm_join[wi]), join_m);
              if (flush_m) atomicOr(reinterpret_cast<unsigned long long *>(&L.bm_flush[wi]), flush_m);
              if (touch_m) atomicOr(reinterpret_cast<unsigned long long *>(&L.bm_touch[wi]), touch_m);
            }
            // every server below the last level of its group now holds that level, plus one if that level reached it
            if (tmin < tend) L.loads[g] = static_cast<uint8_t>(my_lmin + my_n - 1 + (got_last ? 1 : 0));
          }
          if constexpr (WS) {   // what the pass took from the solo group's buffer, per class
            if (tid >= NT - 64 && lane < K) L.cs[CS_QDS + lane] -= L.sel_n[lane];
          }
          if (tid == 0) {
#pragma unroll
            for (int gi = 0; gi < 2; ++gi) {
              if (nG[gi] > 0) {
                const int lmaxg = lminG[gi] + nG[gi] - 1;
                for (int t = 0; t + 1 < nG[gi]; ++t) L.lh[gi * kLoadBins + lminG[gi] + t] = 0;
                L.lh[gi * kLoadBins + lmaxg] = static_cast<uint32_t>(csumG[gi] - tlastG[gi]);
                L.lh[gi * kLoadBins + lmaxg + 1] += static_cast<uint32_t>(tlastG[gi]);
              }
            }
          }
          jrem -= total;
          next += total;
          if constexpr (RR) {
            jremL[0] -= takenL[0]; nextL[0] += takenL[0];
            jremL[1] -= takenL[1]; nextL[1] += takenL[1];
          }
          route_on = jrem > 0;
        }
        gate_on = gate_more;
        __syncthreads();
      }
      if constexpr (AB) {
        if (tid == 0) {   // the head moves past everything the routing passes walked over
          const uint32_t past = static_cast<uint32_t>(L.sc[SC_DSCAN]);
          uint32_t h = dhead0 + past;
          if (h >= dbuf_cap) h -= dbuf_cap;
          L.cs[CS_DHEAD] = static_cast<int32_t>(h);
          L.cs[CS_DCOUNT] -= RR ? nextL[0] : next;
          L.sc[SC_DLEN] = static_cast<int32_t>(dlen_all - past);
          if constexpr (RR) {
            const uint32_t past_m = static_cast<uint32_t>(L.sc[SC_DSCAN_M]);
            h = dheadL[1] + past_m;
            if (h >= dbuf_cap) h -= dbuf_cap;
            L.cs[CS_DHEAD_M] = static_cast<int32_t>(h);
            L.cs[CS_DCOUNT_M] -= nextL[1];
            L.sc[SC_DLEN_M] = static_cast<int32_t>(dlen_all_m - past_m);
          }
          L.sc[SC_COMPACT] = 0;
        }
      } else if constexpr (RR) {
        if (tid == 0 && next > 0) {
          uint32_t h = dheadL[0] + static_cast<uint32_t>(nextL[0]);
          if (h >= dbuf_cap) h -= dbuf_cap;
          L.cs[CS_DHEAD] = static_cast<int32_t>(h);
          L.cs[CS_DCOUNT] -= nextL[0];
          h = dheadL[1] + static_cast<uint32_t>(nextL[1]);
          if (h >= dbuf_cap) h -= dbuf_cap;
          L.cs[CS_DHEAD_M] = static_cast<int32_t>(h);
          L.cs[CS_DCOUNT_M] -= nextL[1];
        }
      } else {
      if (tid == 0 && next > 0) {
        uint32_t h = dhead0 + static_cast<uint32_t>(next);
        if (h >= dbuf_cap) h -= dbuf_cap;
        L.cs[CS_DHEAD] = static_cast<int32_t>(h);
        L.cs[CS_DCOUNT] -= next;
      }
      }
    }

    // ================= 6. end-of-step sums =================
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
  __syncthreads();
  if constexpr (AB) {   // the rings leave the launch without dead entries
    const uint32_t s_last = step_begin + n_steps - 1u;
    for (int k = wave; k < K; k += nwaves) compact_queue(k, s_last, 0u);
    if (wave == nwaves - 1) compact_buffer(s_last, false);
    if constexpr (RR) {
      if (wave == (nwaves > 1 ? nwaves - 2 : 0)) compact_buffer(s_last, true);
    }
    __syncthreads();
  }

  // ---- the emitted-token tally is the total of the time-between-tokens counts of this launch
  if (tid < K) {
    uint64_t tot = 0;
    for (int b = 0; b < p.tbt_w; ++b) tot += L.tbth[tid * p.tbt_w + b];
    L.tl[tid * kNTally + SIM_T_TOK_EMIT] += tot;
  }
  if (tid < 8) L.acc[tid] = 0;
  __syncthreads();

  // ---- write the server clocks and the class state back; add this launch's tallies to the totals
  for (int i = 0; i < nper; ++i) {
    const int g = i * NT + tid;
    if (g >= N) break;
    const bool busy = (L.bm_busy[g >> 6] >> (g & 63)) & 1ull;
    t_next[g] = busy ? T + static_cast<int64_t>(static_cast<int32_t>(L.t32[g] - static_cast<uint32_t>(T))) : kIdle;
    iter_g[g] = L.iter[g];
    if (g < Mp) {   // prompt tokens already processed of the prefill in service
      const uint32_t rem = L.rem[g];
      uint32_t pk = 0;
      if (rem) {
        const uint64_t jw = pf_job[g];
        const uint32_t Pl = (static_cast<uint32_t>(jw >> 32) & 0xFFFFu) + 1, k = static_cast<uint32_t>(jw >> 29) & 7u;
        atomicAdd(&L.acc[k], Pl - rem);
        const bool chunk = (L.bm_chunk[g >> 6] >> (g & 63)) & 1ull;
        const uint32_t cmax = static_cast<uint32_t>(p.C);
        pk = rem | ((chunk ? (rem < cmax ? rem : cmax) : 0u) << 16) | (k << 29);
      }
      remptok[g] = pk;
    }
  }
  for (int i = tid; i < CS_WORDS; i += NT) a.cstate[static_cast<size_t>(r) * CS_WORDS + i] = L.cs[i];
  uint64_t *gt = a.tally + static_cast<size_t>(r) * kTallyWords;
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

// The step kernel of one policy variant for a size class (see size_class), in its roomy or, for the two smaller
// classes, its dense form (see waves_per_simd). Each variant is compiled in a translation unit of its own.
using StepKernel = void (*)(const Params *, StepArrays, uint32_t, uint32_t, uint32_t, uint32_t);
#define GNR_STEP_VARIANT(name, AB, RR, IM, WS)                                                             \
  StepKernel name(int size_class, bool dense)                                                              \
  {                                                                                                        \
    static const StepKernel table[6] = {gnr_step_kernel<128, static_words(0), AB, RR, IM, WS>,             \
                                        gnr_step_kernel<512, static_words(1), AB, RR, IM, WS>,             \
                                        gnr_step_kernel<1024, static_words(2), AB, RR, IM, WS>,            \
                                        gnr_step_kernel<1024, static_words(3), AB, RR, IM, WS>,            \
                                        gnr_step_kernel<128, static_words(0), AB, RR, IM, WS, true>,       \
                                        gnr_step_kernel<512, static_words(1), AB, RR, IM, WS, true>};      \
    return table[dense && size_class <= 1 ? 4 + size_class : size_class];                                  \
  }

}  // namespace gnr
#endif

