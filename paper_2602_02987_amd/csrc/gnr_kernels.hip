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

// ------------------------------------------------------------------ LDS layout ----
enum Scalar {
  SC_NADM = 0, SC_NIDLE, SC_NCOMP, SC_MORE, SC_LMIN, SC_CNT, SC_JREM, SC_NEXT, SC_DHEAD0,
  SC_TAKE = 16,  // [8] accepted arrivals this step
  SC_TAIL = 24,  // [8] ring position of the first accepted arrival
  SC_QH0 = 32,   // [8] ring head at the start of the gate pass
  SC_WORDS = 40
};

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
  uint32_t *pre;      // [nwords] exclusive prefix popcounts of the bitmap being ranked
  uint32_t *adm;      // [kAdmChunk] class | sequence-in-class << 3 of each admission
  uint32_t *t32;      // [N] low 32 bits of the end time of the running iteration
  uint8_t *loads;     // [N] decodes per server
};

__host__ __device__ inline size_t lds_carve(const Params &p, unsigned char *base, Lds *out)
{
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += (bytes + 7) & ~size_t(7); return o; };
  const size_t o_tl = take(sizeof(uint64_t) * kTallyWords);
  const size_t o_tb = take(sizeof(uint64_t) * p.K * p.tbt_w);
  const size_t o_bi = take(sizeof(uint64_t) * p.nwords);
  const size_t o_bc = take(sizeof(uint64_t) * p.nwords);
  const size_t o_bl = take(sizeof(uint64_t) * p.nwords);
  const size_t o_bb = take(sizeof(uint64_t) * p.nwords);
  const size_t o_cs = take(sizeof(int32_t) * CS_WORDS);
  const size_t o_ac = take(sizeof(uint32_t) * 8);
  const size_t o_sc = take(sizeof(int32_t) * SC_WORDS);
  const size_t o_pr = take(sizeof(uint32_t) * (p.nwords + 1));
  const size_t o_ad = take(sizeof(uint32_t) * kAdmChunk);
  const size_t o_t3 = take(sizeof(uint32_t) * p.N);
  const size_t o_ld = take(static_cast<size_t>(p.N));
  if (out) {
    out->tl = reinterpret_cast<uint64_t *>(base + o_tl);
    out->tbth = reinterpret_cast<uint64_t *>(base + o_tb);
    out->bm_idle = reinterpret_cast<uint64_t *>(base + o_bi);
    out->bm_comp = reinterpret_cast<uint64_t *>(base + o_bc);
    out->bm_lvl = reinterpret_cast<uint64_t *>(base + o_bl);
    out->bm_busy = reinterpret_cast<uint64_t *>(base + o_bb);
    out->cs = reinterpret_cast<int32_t *>(base + o_cs);
    out->acc = reinterpret_cast<uint32_t *>(base + o_ac);
    out->sc = reinterpret_cast<int32_t *>(base + o_sc);
    out->pre = reinterpret_cast<uint32_t *>(base + o_pr);
    out->adm = reinterpret_cast<uint32_t *>(base + o_ad);
    out->t32 = reinterpret_cast<uint32_t *>(base + o_t3);
    out->loads = reinterpret_cast<uint8_t *>(base + o_ld);
  }
  return off;
}

size_t step_lds_bytes(const Params &p) { return lds_carve(p, nullptr, nullptr); }

int step_threads(int N)
{
  int t = (N + 63) / 64 * 64;
  return t > 1024 ? 1024 : t;
}

// Exclusive prefix popcounts of a bitmap (wave 0 only); returns the total in every lane of wave 0.
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
  for (int d = 32; d > 0; d >>= 1) v += __shfl_xor(v, d, 64);
  return v;
}

// Per-lane running sums of the tallies every executed iteration touches; they are added to the
// workgroup's totals once per launch instead of once per iteration.
struct LaneTallies {
  uint32_t iters[2];            // [decode-only, with a prefill chunk]
  uint64_t busy[2];
  uint32_t tok_emit[kMaxK];
  uint64_t tbt_sum[kMaxK];
  int hist_bin[2];              // time-between-tokens bin currently accumulated, by iteration kind
  uint32_t hist_cnt[2][kMaxK];
};

// One executed iteration of duration d whose batch held the decodes nc minus the late joiners nj.
template <int KIND>
__device__ __forceinline__ void tally_iteration(LaneTallies &lt, uint64_t *tbth, int tbt_w, int K, int64_t d, int tb,
                                                uint64_t nc, uint64_t nj)
{
  lt.iters[KIND] += 1;
  lt.busy[KIND] += static_cast<uint64_t>(d);
  if (tb != lt.hist_bin[KIND]) {   // the duration moved to another bin: flush the cached counts
#pragma unroll
    for (int k = 0; k < kMaxK; ++k)
      if (k < K && lt.hist_cnt[KIND][k]) {
        lds_add64(&tbth[k * tbt_w + lt.hist_bin[KIND]], lt.hist_cnt[KIND][k]);
        lt.hist_cnt[KIND][k] = 0;
      }
    lt.hist_bin[KIND] = tb;
  }
#pragma unroll
  for (int k = 0; k < kMaxK; ++k) {
    const uint32_t em = byte_at(nc, k) - byte_at(nj, k);
    lt.tok_emit[k] += em;
    lt.tbt_sum[k] += static_cast<uint64_t>(em) * static_cast<uint64_t>(d);
    lt.hist_cnt[KIND][k] += em;
  }
}

// ------------------------------------------------------------------ step kernel ----
__global__ void __launch_bounds__(1024) gnr_step_kernel(const Params p, const uint32_t step_begin, const uint32_t n_steps)
{
  extern __shared__ __align__(16) unsigned char lds_raw[];
  Lds L;
  lds_carve(p, lds_raw, &L);

  const int r = blockIdx.x;
  const int tid = threadIdx.x;
  const int NT = blockDim.x;
  const int lane = tid & 63;
  const int wave_base = tid & ~63;
  const int K = p.K, N = p.N, B = p.B, M = p.M, BS = p.BS;
  const int nper = (N + NT - 1) / NT;

  int64_t *t_next = p.t_next + static_cast<size_t>(r) * N;
  uint32_t *iter = p.iter + static_cast<size_t>(r) * N;
  uint32_t *remptok = p.remptok + static_cast<size_t>(r) * N;
  uint64_t *pf_job = p.pf_job + static_cast<size_t>(r) * N;
  uint64_t *n_cls = p.n_cls + static_cast<size_t>(r) * N;
  uint64_t *n_join = p.n_join + static_cast<size_t>(r) * N;
  uint32_t *fin = p.fin + static_cast<size_t>(r) * N * BS;
  uint64_t *job = p.job + static_cast<size_t>(r) * N * BS;
  uint32_t *qring = p.qring + static_cast<size_t>(r) * K * p.queue_cap;
  uint64_t *dring = p.dring + static_cast<size_t>(r) * p.dbuf_cap;
  uint64_t *hist = p.hist + static_cast<size_t>(r) * 3 * K * kNBin;

  // ---- load the replication's class state and rebuild the on-chip views of the server state
  for (int i = tid; i < CS_WORDS; i += NT) L.cs[i] = p.cstate[static_cast<size_t>(r) * CS_WORDS + i];
  for (int i = tid; i < kTallyWords; i += NT) L.tl[i] = 0;
  for (int i = tid; i < K * p.tbt_w; i += NT) L.tbth[i] = 0;
  for (int i = tid; i < SC_WORDS; i += NT) L.sc[i] = 0;
  for (int i = 0; i < nper; ++i) {
    const int g = i * NT + tid;
    const bool valid = g < N;
    bool busy = false;
    if (valid) {
      L.loads[g] = static_cast<uint8_t>(byte_sum(n_cls[g]));
      const int64_t tn = t_next[g];
      busy = tn != kIdle;
      L.t32[g] = static_cast<uint32_t>(tn);
    }
    const bool idle_slot = valid && g < M && (remptok[g] & 0xFFFFu) == 0;
    const uint64_t bi = __ballot(idle_slot), bb = __ballot(busy);
    const int wi = (i * NT + wave_base) >> 6;
    if (lane == 0 && wi < p.nwords) { L.bm_idle[wi] = bi; L.bm_busy[wi] = bb; }
  }
  LaneTallies lt;
  lt.iters[0] = lt.iters[1] = 0; lt.busy[0] = lt.busy[1] = 0;
  lt.hist_bin[0] = lt.hist_bin[1] = 0;
#pragma unroll
  for (int k = 0; k < kMaxK; ++k) { lt.tok_emit[k] = 0; lt.tbt_sum[k] = 0; lt.hist_cnt[0][k] = lt.hist_cnt[1][k] = 0; }
  __syncthreads();

  int64_t T = 0;
  for (uint32_t s = step_begin; s < step_begin + n_steps; ++s) {
    T = (static_cast<int64_t>(s) + 1) * p.dt;
    const uint32_t T32 = static_cast<uint32_t>(T);
    if (tid < 8) L.acc[tid] = 0;

    // ================= 1. arrivals =================
    const uint32_t *thr = p.arr_thr + 3 * (p.mod_period > 0 ? static_cast<int64_t>(s % static_cast<uint64_t>(p.mod_period)) : 0);
    const uint32_t thr0 = thr[0], thr1 = thr[1], thr2 = thr[2];
    uint64_t at_boundary = 0, touched = 0;
    __syncthreads();
    for (int i = 0; i < nper; ++i) {
      const int g = i * NT + tid;
      if (g < N) {
        uint32_t w[4];
        philox4x32_10(p.key0, p.key1, s, 0u, static_cast<uint32_t>(g), static_cast<uint32_t>(r), w);
        if (w[0] >= thr0) {
          const int a = 1 + (w[0] >= thr1) + (w[0] >= thr2);
          for (int j = 0; j < a; ++j) {
            int k = 0;
            for (int c = 0; c + 1 < K; ++c) k += (w[1 + j] >= p.cls_thr[c]);
            atomicAdd(&L.acc[k], 1u);
          }
        }
      }
    }

    // ================= 2. iteration completion on due servers =================
    for (int i = 0; i < nper; ++i) {
      const int gw = i * NT + wave_base;          // first server of this wave's 64-server block
      const int wi = gw >> 6;
      if (gw >= N) break;                         // wave-uniform
      const int g = gw + lane;
      const bool valid = g < N;
      const uint64_t busy_word = L.bm_busy[wi];
      const uint32_t t32 = valid ? L.t32[g] : 0u;
      const bool due = valid && ((busy_word >> lane) & 1ull) && static_cast<int32_t>(t32 - T32) <= 0;
      const uint64_t due_mask = __ballot(due);
      if (due_mask == 0) {
        if (lane == 0) L.bm_comp[wi] = 0;
        continue;
      }
      uint32_t it = 0, pk = 0;
      uint64_t nc = 0, nj = 0;
      int nd = 0;
      if (due) {
        at_boundary |= 1ull << i;
        it = iter[g] + 1;
        pk = g < M ? remptok[g] : 0u;
        nc = n_cls[g];
        nj = n_join[g];
        nd = static_cast<int>(byte_sum(nc));
      }
      // ---- cooperative scan of the slot rows: half a wave reads one server's row (4 words per lane)
      uint32_t quads = 0;   // owner lane: bit q set <=> one of slots 4q..4q+3 finishes now
      {
        uint64_t todo = __ballot(due && nd > 0);
        while (todo) {
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
          const int q = lane & 31;
          const bool hi = lane >= 32;
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const uint32_t ita = __builtin_amdgcn_readlane(it, la[u]), itb = __builtin_amdgcn_readlane(it, lb[u]);
            const int nda = __builtin_amdgcn_readlane(nd, la[u]), ndb = __builtin_amdgcn_readlane(nd, lb[u]);
            const bool on = hi ? vb[u] : va[u];
            its[u] = hi ? itb : ita;
            nds[u] = on ? (hi ? ndb : nda) : 0;
            const int gs = gw + (hi ? lb[u] : la[u]);
            v[u] = make_uint4(0u, 0u, 0u, 0u);
            if (4 * q < nds[u]) v[u] = *reinterpret_cast<const uint4 *>(fin + static_cast<size_t>(gs) * BS + 4 * q);
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
        }
      }
      bool pf_done = false;
      if (due) {
        int rem = static_cast<int>(pk & 0xFFFFu);
        const int ptok = static_cast<int>(pk >> 16);
        const int64_t tn = T + static_cast<int64_t>(static_cast<int32_t>(t32 - T32));   // exact completion time
        const int64_t d = p.c0 + p.cpre * ptok + p.cdec * static_cast<int64_t>(nd - static_cast<int>(byte_sum(nj)));
        const int tb = hbin(d) - p.tbt_lo;
        if (ptok > 0) tally_iteration<1>(lt, L.tbth, p.tbt_w, K, d, tb, nc, nj);
        else tally_iteration<0>(lt, L.tbth, p.tbt_w, K, d, tb, nc, nj);
        // decodes that emitted their last token leave; the last occupied slot fills the hole.
        // Highest slot first, so the slot moved into a hole has already been checked.
        const bool mixed_now = rem > 0;
        const uint64_t nc_before = nc;
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
              lds_add64(&L.tl[k * kNTally + (mixed_now ? SIM_T_S_DM : SIM_T_S_DS)], 1);
              atomicSub(&L.cs[(mixed_now ? CS_YM : CS_YS) + k], 1);
              lds_add64(&L.tl[k * kNTally + SIM_T_TOKP_DEC], Pl);
              lds_add64(&L.tl[k * kNTally + SIM_T_TOKD_DEC], Dl);
              const int64_t e2e = tn - (static_cast<int64_t>(stamp) + 1) * p.dt;
              lds_add64(&L.tl[k * kNTally + SIM_T_E2E_SUM], static_cast<uint64_t>(e2e));
              atomicAdd(reinterpret_cast<unsigned long long *>(&hist[(1 * K + k) * kNBin + hbin(e2e)]), 1ull);
              nc -= 1ull << (8 * k);
              --nd;
              if (j < nd) { frow[j] = frow[nd]; jrow[j] = jrow[nd]; }
            }
          }
        }
        // the prefill advances by the chunk frozen at the start of the iteration
        if (ptok > 0) {
          const uint64_t jw = pf_job[g];
          const int k = static_cast<int>(jw >> 29) & 7;
          lds_add64(&L.tl[k * kNTally + SIM_T_TOK_PREF], static_cast<uint64_t>(ptok));
          rem -= ptok;
          if (rem == 0) {
            pf_done = true;
            const uint32_t stamp = static_cast<uint32_t>(jw) & 0x1FFFFFFFu;
            const uint32_t Pl = (static_cast<uint32_t>(jw >> 32) & 0xFFFFu) + 1;
            lds_add64(&L.tl[k * kNTally + SIM_T_S_P], 1);
            atomicSub(&L.cs[CS_X + k], 1);
            lds_add64(&L.tl[k * kNTally + SIM_T_TOKP_PRE], Pl);
            const int64_t ttft = tn - (static_cast<int64_t>(stamp) + 1) * p.dt;
            lds_add64(&L.tl[k * kNTally + SIM_T_TTFT_SUM], static_cast<uint64_t>(ttft));
            atomicAdd(reinterpret_cast<unsigned long long *>(&hist[(0 * K + k) * kNBin + hbin(ttft)]), 1ull);
            for (int c = 0; c < K; ++c) {   // co-resident decodes switch mixed -> solo
              const int v = static_cast<int>(byte_at(nc, c));
              if (v) {
                lds_add64(&L.tl[c * kNTally + SIM_T_M_MS], static_cast<uint64_t>(v));
                atomicSub(&L.cs[CS_YM + c], v);
                atomicAdd(&L.cs[CS_YS + c], v);
              }
            }
          }
        }
        iter[g] = it;
        if (g < M) remptok[g] = static_cast<uint32_t>(rem);   // running chunk cleared; set again at the restart
        if (nc != nc_before) { n_cls[g] = nc; L.loads[g] = static_cast<uint8_t>(nd); }
        if (nj) n_join[g] = 0;
      }
      const uint64_t done = __ballot(pf_done);
      if (lane == 0) {
        L.bm_comp[wi] = done;
        if (done) L.bm_idle[wi] |= done;
      }
    }
    __syncthreads();

    // ================= arrivals into the class queues; order of prefill completions =================
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
      const uint32_t ncomp = rank_bitmap(L.bm_comp, L.pre, p.nwords);
      if (tid == 0) L.sc[SC_NCOMP] = static_cast<int32_t>(ncomp);
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
    if (L.sc[SC_NCOMP] > 0) {
      const uint32_t dcount = static_cast<uint32_t>(L.cs[CS_DCOUNT]), dhead = static_cast<uint32_t>(L.cs[CS_DHEAD]);
      for (int i = 0; i < nper; ++i) {
        const int g = i * NT + tid;
        if (g >= M || g >= N) break;
        const uint64_t word = L.bm_comp[g >> 6];
        if (!((word >> (g & 63)) & 1ull)) continue;
        const uint32_t rank = L.pre[g >> 6] + static_cast<uint32_t>(__popcll(word & lanes_below()));
        const uint64_t jw = pf_job[g];
        const int k = static_cast<int>(jw >> 29) & 7;
        if (dcount + rank < p.dbuf_cap) {
          uint32_t pos = dhead + dcount + rank;
          if (pos >= p.dbuf_cap) pos -= p.dbuf_cap;
          dring[pos] = jw;
          atomicAdd(&L.cs[CS_QD + k], 1);
        } else {
          lds_add64(&L.tl[k * kNTally + SIM_T_DROP_D], 1);
          L.tl[kMaxK * kNTally + SIM_G_OVERFLOW] = 1;
        }
      }
    }
    __syncthreads();
    if (tid == 0) {
      const uint32_t room = p.dbuf_cap - static_cast<uint32_t>(L.cs[CS_DCOUNT]);
      const uint32_t ncp = static_cast<uint32_t>(L.sc[SC_NCOMP]);
      L.cs[CS_DCOUNT] += static_cast<int32_t>(ncp < room ? ncp : room);
    }

    // ================= 3. prefill gate =================
    for (;;) {
      if (tid < 64) {
        const uint32_t nidle = rank_bitmap(L.bm_idle, L.pre, p.nwords);
        if (tid == 0) {
          // the admission sequence is decided serially on the class counters; servers pick it up by rank
          int nadm = 0;
          const int limit = static_cast<int>(nidle) < kAdmChunk ? static_cast<int>(nidle) : kAdmChunk;
          int qp[kMaxK], xs[kMaxK];
          uint32_t popped[kMaxK], head[kMaxK];
#pragma unroll
          for (int k = 0; k < kMaxK; ++k) {
            qp[k] = k < K ? L.cs[CS_QP + k] : 0;
            xs[k] = k < K ? L.cs[CS_X + k] : 0;
            head[k] = k < K ? static_cast<uint32_t>(L.cs[CS_QHEAD + k]) : 0u;
            popped[k] = 0;
            if (k < K) L.sc[SC_QH0 + k] = static_cast<int32_t>(head[k]);
          }
          while (nadm < limit) {
            int best = -1;
            double bkey = 0.0, bdl = 0.0;
#pragma unroll
            for (int k = 0; k < kMaxK; ++k) {
              if (k >= K || qp[k] <= 0) continue;
              if (p.gate_mode == SIM_GATE_OCCUPANCY) {
                if (!(p.invx[k] > 0.0)) continue;
                const double xi = (static_cast<double>(xs[k]) - p.nx[k]) * p.invx[k];
                const double dl = static_cast<double>(qp[k]) - p.nq[k];
                if (best < 0 || xi < bkey || (xi == bkey && dl > bdl)) { best = k; bkey = xi; bdl = dl; }
              } else if (p.gate_mode == SIM_GATE_PRIORITY) {
                if (best < 0 || p.prio[k] > bkey) { best = k; bkey = p.prio[k]; }
              } else {
                uint32_t pos = head[k] + popped[k];
                if (pos >= p.queue_cap) pos -= p.queue_cap;
                const double st = static_cast<double>(qring[static_cast<size_t>(k) * p.queue_cap + pos]);
                if (best < 0 || st < bkey) { best = k; bkey = st; }
              }
            }
            if (best < 0) break;
#pragma unroll
            for (int k = 0; k < kMaxK; ++k)
              if (k == best) {
                L.adm[nadm] = static_cast<uint32_t>(k) | (popped[k] << 3);
                ++popped[k]; --qp[k]; ++xs[k];
              }
            ++nadm;
          }
          bool waiting = false;
#pragma unroll
          for (int k = 0; k < kMaxK; ++k) {
            if (k >= K) continue;
            uint32_t h = head[k] + popped[k];
            if (h >= p.queue_cap) h -= p.queue_cap;
            L.cs[CS_QHEAD + k] = static_cast<int32_t>(h);
            L.cs[CS_QP + k] = qp[k];
            L.cs[CS_X + k] = xs[k];
            L.tl[k * kNTally + SIM_T_U_P] += popped[k];
            if (qp[k] > 0 && (p.gate_mode != SIM_GATE_OCCUPANCY || p.invx[k] > 0.0)) waiting = true;
          }
          L.sc[SC_NADM] = nadm;
          L.sc[SC_MORE] = (nadm == kAdmChunk && static_cast<int>(nidle) > kAdmChunk && waiting) ? 1 : 0;
        }
      }
      __syncthreads();
      const int nadm = L.sc[SC_NADM];
      if (nadm > 0) {
        for (int i = 0; i < nper; ++i) {
          const int gw = i * NT + wave_base;
          if (gw >= M || gw >= N) break;     // wave-uniform: no mixed-group server in this block
          const int g = gw + lane;
          bool admitted = false;
          const uint64_t word = L.bm_idle[gw >> 6];
          if (g < M && g < N && ((word >> lane) & 1ull)) {
            const uint32_t rank = L.pre[gw >> 6] + static_cast<uint32_t>(__popcll(word & lanes_below()));
            if (rank < static_cast<uint32_t>(nadm)) {
              admitted = true;
              const uint32_t e = L.adm[rank];
              const int k = static_cast<int>(e & 7u);
              uint32_t pos = static_cast<uint32_t>(L.sc[SC_QH0 + k]) + (e >> 3);
              if (pos >= p.queue_cap) pos -= p.queue_cap;
              const uint32_t stamp = qring[static_cast<size_t>(k) * p.queue_cap + pos];
              lds_add64(&L.tl[k * kNTally + SIM_T_WAIT_STEPS], static_cast<uint64_t>(s - stamp));
              uint32_t w[4];
              philox4x32_10(p.key0, p.key1, s, 1u, static_cast<uint32_t>(g), static_cast<uint32_t>(r), w);
              const uint32_t Pl = p.len_tab[(static_cast<size_t>(k) * 2 + 0) * kTableSize + (w[0] >> 16)];
              const uint32_t Dl = p.len_tab[(static_cast<size_t>(k) * 2 + 1) * kTableSize + (w[1] >> 16)];
              pf_job[g] = static_cast<uint64_t>(stamp) | (static_cast<uint64_t>(k) << 29) |
                          (static_cast<uint64_t>(Pl - 1) << 32) | (static_cast<uint64_t>(Dl - 1) << 48);
              remptok[g] = Pl;   // an idle prefill slot implies that the running iteration holds no chunk
              const uint64_t nc = n_cls[g];
              for (int c = 0; c < K; ++c) {   // co-resident decodes switch solo -> mixed
                const int v = static_cast<int>(byte_at(nc, c));
                if (v) {
                  lds_add64(&L.tl[c * kNTally + SIM_T_M_SM], static_cast<uint64_t>(v));
                  atomicSub(&L.cs[CS_YS + c], v);
                  atomicAdd(&L.cs[CS_YM + c], v);
                }
              }
              if (!((L.bm_busy[gw >> 6] >> lane) & 1ull)) touched |= 1ull << i;
            }
          }
          const uint64_t adm_mask = __ballot(admitted);
          if (lane == 0 && adm_mask) L.bm_idle[gw >> 6] = word & ~adm_mask;
        }
      }
      __syncthreads();
      if (!L.sc[SC_MORE]) break;
    }

    // ================= 4. decode routing =================
    if (tid == 0) { L.sc[SC_JREM] = L.cs[CS_DCOUNT]; L.sc[SC_NEXT] = 0; L.sc[SC_DHEAD0] = L.cs[CS_DHEAD]; }
    for (int grp = 0; grp < 2; ++grp) {
      const int lo = grp == 0 ? M : 0, hi = grp == 0 ? N : M;
      const int capg = grp == 0 ? B : B - 1;
      for (;;) {
        if (tid == 0) L.sc[SC_LMIN] = 255;
        __syncthreads();
        if (L.sc[SC_JREM] <= 0 || lo >= hi) break;
        int lmin = 255;
        for (int i = 0; i < nper; ++i) {
          const int g = i * NT + tid;
          if (g >= lo && g < hi) { const int l = L.loads[g]; if (l < capg && l < lmin) lmin = l; }
        }
        for (int d = 32; d > 0; d >>= 1) { const int o = __shfl_xor(lmin, d, 64); lmin = o < lmin ? o : lmin; }
        if (lane == 0 && lmin < 255) atomicMin(&L.sc[SC_LMIN], lmin);
        __syncthreads();
        const int level = L.sc[SC_LMIN];
        if (level == 255) break;
        for (int i = 0; i < nper; ++i) {
          const int gw = i * NT + wave_base;
          if (gw >= N) break;
          const int g = gw + lane;
          const bool at_level = g >= lo && g < hi && L.loads[g] == level;
          const uint64_t b = __ballot(at_level);
          if (lane == 0) L.bm_lvl[gw >> 6] = b;
        }
        __syncthreads();
        if (tid < 64) {
          const uint32_t cnt = rank_bitmap(L.bm_lvl, L.pre, p.nwords);
          if (tid == 0) L.sc[SC_CNT] = static_cast<int32_t>(cnt);
        }
        __syncthreads();
        const int jrem = L.sc[SC_JREM], next = L.sc[SC_NEXT];
        const int take = L.sc[SC_CNT] < jrem ? L.sc[SC_CNT] : jrem;
        const uint32_t dhead0 = static_cast<uint32_t>(L.sc[SC_DHEAD0]);
        for (int i = 0; i < nper; ++i) {
          const int g = i * NT + tid;
          if (g >= N) break;
          if (g < lo || g >= hi) continue;
          const uint64_t word = L.bm_lvl[g >> 6];
          if (!((word >> (g & 63)) & 1ull)) continue;
          const uint32_t rank = L.pre[g >> 6] + static_cast<uint32_t>(__popcll(word & lanes_below()));
          if (rank >= static_cast<uint32_t>(take)) continue;
          uint32_t pos = dhead0 + static_cast<uint32_t>(next) + rank;
          if (pos >= p.dbuf_cap) pos -= p.dbuf_cap;
          if (pos >= p.dbuf_cap) pos -= p.dbuf_cap;
          const uint64_t jw = dring[pos];
          const int k = static_cast<int>(jw >> 29) & 7;
          const uint32_t Dl = static_cast<uint32_t>(jw >> 48) + 1;
          const bool busy = (L.bm_busy[g >> 6] >> (g & 63)) & 1ull;
          const bool mid = busy && !((at_boundary >> i) & 1ull);   // joins at the next restart
          const int nd = L.loads[g];
          fin[static_cast<size_t>(g) * BS + nd] = iter[g] + Dl + (mid ? 1u : 0u);
          job[static_cast<size_t>(g) * BS + nd] = jw;
          n_cls[g] += 1ull << (8 * k);
          if (mid) n_join[g] += 1ull << (8 * k);
          L.loads[g] = static_cast<uint8_t>(nd + 1);
          const bool has_prefill = g < M && (remptok[g] & 0xFFFFu) != 0;
          lds_add64(&L.tl[k * kNTally + (has_prefill ? SIM_T_U_DM : SIM_T_U_DS)], 1);
          atomicAdd(&L.cs[(has_prefill ? CS_YM : CS_YS) + k], 1);
          atomicSub(&L.cs[CS_QD + k], 1);
          if (!busy) touched |= 1ull << i;
        }
        __syncthreads();
        if (tid == 0) { L.sc[SC_JREM] = jrem - take; L.sc[SC_NEXT] = next + take; }
      }
    }
    __syncthreads();
    if (tid == 0) {
      const uint32_t routed = static_cast<uint32_t>(L.sc[SC_NEXT]);
      uint32_t h = static_cast<uint32_t>(L.cs[CS_DHEAD]) + routed;
      if (h >= p.dbuf_cap) h -= p.dbuf_cap;
      L.cs[CS_DHEAD] = static_cast<int32_t>(h);
      L.cs[CS_DCOUNT] -= static_cast<int32_t>(routed);
    }

    // ================= 5. (re)start =================
    {
      const uint64_t todo = at_boundary | touched;
      for (int i = 0; i < nper; ++i) {
        const int gw = i * NT + wave_base;
        if (gw >= N) break;
        const bool mine = (todo >> i) & 1ull;
        if (__ballot(mine) == 0) continue;
        const int g = gw + lane;
        const uint64_t busy_word = L.bm_busy[gw >> 6];
        bool busy = (busy_word >> lane) & 1ull;
        if (mine) {
          const int rem = g < M ? static_cast<int>(remptok[g] & 0xFFFFu) : 0;
          const int ptok = rem > 0 ? (rem < p.C ? rem : p.C) : 0;
          const int n = L.loads[g];
          if (ptok == 0 && n == 0) {
            busy = false;
          } else {
            // back-to-back after a completion, otherwise from the step boundary
            const int64_t base = ((at_boundary >> i) & 1ull) ? T + static_cast<int64_t>(static_cast<int32_t>(L.t32[g] - T32)) : T;
            const int64_t tn = base + p.c0 + p.cpre * ptok + p.cdec * static_cast<int64_t>(n);
            L.t32[g] = static_cast<uint32_t>(tn);
            busy = true;
            if (ptok > 0) remptok[g] = static_cast<uint32_t>(rem) | (static_cast<uint32_t>(ptok) << 16);
          }
        }
        const uint64_t nb = __ballot(busy);
        if (lane == 0 && nb != busy_word) L.bm_busy[gw >> 6] = nb;
      }
    }

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
  __syncthreads();

  // ---- fold the per-lane sums into the workgroup's tallies
  {
#pragma unroll
    for (int kind = 0; kind < 2; ++kind) {
      const uint64_t it = wave_sum64(lt.iters[kind]), bz = wave_sum64(lt.busy[kind]);
      if (lane == 0) {
        lds_add64(&L.tl[kMaxK * kNTally + (kind ? SIM_G_ITERS_MIX : SIM_G_ITERS_SOLO)], it);
        lds_add64(&L.tl[kMaxK * kNTally + (kind ? SIM_G_BUSY_MIX : SIM_G_BUSY_SOLO)], bz);
      }
#pragma unroll
      for (int k = 0; k < kMaxK; ++k)
        if (k < K && lt.hist_cnt[kind][k]) lds_add64(&L.tbth[k * p.tbt_w + lt.hist_bin[kind]], lt.hist_cnt[kind][k]);
    }
#pragma unroll
    for (int k = 0; k < kMaxK; ++k) {
      if (k >= K) continue;
      const uint64_t te = wave_sum64(lt.tok_emit[k]), ts = wave_sum64(lt.tbt_sum[k]);
      if (lane == 0) {
        lds_add64(&L.tl[k * kNTally + SIM_T_TOK_EMIT], te);
        lds_add64(&L.tl[k * kNTally + SIM_T_TBT_SUM], ts);
      }
    }
  }
  __syncthreads();

  // ---- write the server clocks and the class state back; add this launch's tallies to the totals
  for (int i = 0; i < nper; ++i) {
    const int g = i * NT + tid;
    if (g >= N) break;
    const bool busy = (L.bm_busy[g >> 6] >> (g & 63)) & 1ull;
    t_next[g] = busy ? T + static_cast<int64_t>(static_cast<int32_t>(L.t32[g] - static_cast<uint32_t>(T))) : kIdle;
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
    uint64_t h = chain(4, static_cast<uint64_t>(g));
    h = chain(h, static_cast<uint64_t>(p.t_next[sg]));
    h = chain(h, p.iter[sg]);
    h = chain(h, rem);
    h = chain(h, pk >> 16);
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
  if (lds_bytes > 64 * 1024) {   // more than the default dynamic LDS limit has to be asked for
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(gnr_step_kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds_bytes));
    if (e != hipSuccess) return SIM_EHIP;
  }
  hipLaunchKernelGGL(gnr_step_kernel, dim3(reps), dim3(threads), lds_bytes, static_cast<hipStream_t>(stream), p,
                     step_begin, n_steps);
  return hip_ok(hipGetLastError());
}

int launch_reduce(const Params &p, int reps, void *stream)
{
  const int n = kTallyWords + 3 * p.K * kNBin;
  hipLaunchKernelGGL(gnr_reduce_kernel, dim3((n + 255) / 256), dim3(256), 0, static_cast<hipStream_t>(stream), p, reps);
  return hip_ok(hipGetLastError());
}

int launch_digest(const Params &p, int reps, void *stream)
{
  hipLaunchKernelGGL(gnr_digest_kernel, dim3(reps), dim3(256), 0, static_cast<hipStream_t>(stream), p);
  return hip_ok(hipGetLastError());
}

}  // namespace gnr
