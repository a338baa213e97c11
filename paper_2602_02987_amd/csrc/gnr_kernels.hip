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
  SC_NADM = 0, SC_NIDLE, SC_NCOMP, SC_MORE, SC_LMIN, SC_CNT, SC_JREM, SC_NEXT, SC_DHEAD0, SC_DROPPED,
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
  uint32_t *pre;      // [nwords] exclusive prefix popcounts of the bitmap being ranked
  uint32_t *adm;      // [kAdmChunk] class | sequence-in-class << 3 of each admission
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
  const size_t o_cs = take(sizeof(int32_t) * CS_WORDS);
  const size_t o_ac = take(sizeof(uint32_t) * 8);
  const size_t o_sc = take(sizeof(int32_t) * SC_WORDS);
  const size_t o_pr = take(sizeof(uint32_t) * (p.nwords + 1));
  const size_t o_ad = take(sizeof(uint32_t) * kAdmChunk);
  const size_t o_ld = take(static_cast<size_t>(p.N));
  if (out) {
    out->tl = reinterpret_cast<uint64_t *>(base + o_tl);
    out->tbth = reinterpret_cast<uint64_t *>(base + o_tb);
    out->bm_idle = reinterpret_cast<uint64_t *>(base + o_bi);
    out->bm_comp = reinterpret_cast<uint64_t *>(base + o_bc);
    out->bm_lvl = reinterpret_cast<uint64_t *>(base + o_bl);
    out->cs = reinterpret_cast<int32_t *>(base + o_cs);
    out->acc = reinterpret_cast<uint32_t *>(base + o_ac);
    out->sc = reinterpret_cast<int32_t *>(base + o_sc);
    out->pre = reinterpret_cast<uint32_t *>(base + o_pr);
    out->adm = reinterpret_cast<uint32_t *>(base + o_ad);
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
  const int K = p.K, N = p.N, B = p.B, M = p.M;
  const int nper = (N + NT - 1) / NT;

  int64_t *t_next = p.t_next + static_cast<size_t>(r) * N;
  uint32_t *iter = p.iter + static_cast<size_t>(r) * N;
  uint32_t *remptok = p.remptok + static_cast<size_t>(r) * N;
  uint64_t *pf_job = p.pf_job + static_cast<size_t>(r) * N;
  uint64_t *n_cls = p.n_cls + static_cast<size_t>(r) * N;
  uint64_t *n_join = p.n_join + static_cast<size_t>(r) * N;
  uint32_t *fin = p.fin + static_cast<size_t>(r) * N * B;
  uint64_t *job = p.job + static_cast<size_t>(r) * N * B;
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
    if (valid) L.loads[g] = static_cast<uint8_t>(byte_sum(n_cls[g]));
    const bool idle_slot = valid && g < M && (remptok[g] & 0xFFFFu) == 0;
    const uint64_t b = __ballot(idle_slot);
    const int wi = (i * NT + (tid & ~63)) >> 6;
    if (lane == 0 && wi < p.nwords) L.bm_idle[wi] = b;
  }
  __syncthreads();

  for (uint32_t s = step_begin; s < step_begin + n_steps; ++s) {
    const int64_t T = (static_cast<int64_t>(s) + 1) * p.dt;
    if (tid < 8) L.acc[tid] = 0;
    __syncthreads();

    // ================= 1. arrivals and 2. iteration completion =================
    const uint32_t *thr = p.arr_thr + 3 * (p.mod_period > 0 ? static_cast<int64_t>(s % static_cast<uint64_t>(p.mod_period)) : 0);
    const uint32_t thr0 = thr[0], thr1 = thr[1], thr2 = thr[2];
    uint64_t at_boundary = 0, touched = 0;
    for (int i = 0; i < nper; ++i) {
      const int g = i * NT + tid;
      const bool valid = g < N;
      bool pf_done = false;
      if (valid) {
        uint32_t w[4];
        philox4x32_10(p.key0, p.key1, s, 0u, static_cast<uint32_t>(g), static_cast<uint32_t>(r), w);
        const int a = (w[0] >= thr0) + (w[0] >= thr1) + (w[0] >= thr2);
        for (int j = 0; j < a; ++j) {
          int k = 0;
          for (int c = 0; c + 1 < K; ++c) k += (w[1 + j] >= p.cls_thr[c]);
          atomicAdd(&L.acc[k], 1u);
        }
        const int64_t tn = t_next[g];
        if (tn <= T) {
          at_boundary |= 1ull << i;
          const uint32_t it = iter[g] + 1;
          iter[g] = it;
          const uint32_t pk = remptok[g];
          int rem = static_cast<int>(pk & 0xFFFFu);
          const int ptok = static_cast<int>(pk >> 16);
          uint64_t nc = n_cls[g];
          const uint64_t nj = n_join[g];
          int nd = static_cast<int>(byte_sum(nc));
          const int64_t d = p.c0 + p.cpre * ptok + p.cdec * static_cast<int64_t>(nd - static_cast<int>(byte_sum(nj)));
          lds_add64(&L.tl[kMaxK * kNTally + (ptok > 0 ? SIM_G_ITERS_MIX : SIM_G_ITERS_SOLO)], 1);
          lds_add64(&L.tl[kMaxK * kNTally + (ptok > 0 ? SIM_G_BUSY_MIX : SIM_G_BUSY_SOLO)], static_cast<uint64_t>(d));
          const int tb = hbin(d) - p.tbt_lo;
          for (int k = 0; k < K; ++k) {
            const uint32_t em = byte_at(nc, k) - byte_at(nj, k);
            if (em) {
              lds_add64(&L.tl[k * kNTally + SIM_T_TOK_EMIT], em);
              lds_add64(&L.tl[k * kNTally + SIM_T_TBT_SUM], static_cast<uint64_t>(em) * static_cast<uint64_t>(d));
              lds_add64(&L.tbth[k * p.tbt_w + tb], em);
            }
          }
          // decodes that emitted their last token leave; the last occupied slot fills the hole
          const bool mixed_now = rem > 0;
          uint32_t *frow = fin + static_cast<size_t>(g) * B;
          uint64_t *jrow = job + static_cast<size_t>(g) * B;
          for (int j = 0; j < nd;) {
            if (frow[j] == it) {
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
            } else {
              ++j;
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
          remptok[g] = static_cast<uint32_t>(rem);   // running chunk cleared; set again at the restart
          n_cls[g] = nc;
          n_join[g] = 0;
          L.loads[g] = static_cast<uint8_t>(nd);
        }
      }
      const uint64_t done = __ballot(pf_done);
      const int wi = (i * NT + (tid & ~63)) >> 6;
      if (lane == 0 && wi < p.nwords) {
        L.bm_comp[wi] = done;
        L.bm_idle[wi] |= done;
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
      if (tid == 0) { L.sc[SC_NCOMP] = static_cast<int32_t>(ncomp); L.sc[SC_DHEAD0] = L.cs[CS_DHEAD]; }
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
      const uint32_t nc = static_cast<uint32_t>(L.sc[SC_NCOMP]);
      L.cs[CS_DCOUNT] += static_cast<int32_t>(nc < room ? nc : room);
    }

    // ================= 3. prefill gate =================
    for (;;) {
      if (tid < 64) {
        const uint32_t nidle = rank_bitmap(L.bm_idle, L.pre, p.nwords);
        if (tid == 0) L.sc[SC_NIDLE] = static_cast<int32_t>(nidle);
      }
      __syncthreads();
      if (tid == 0) {
        // the admission sequence is decided serially on the class counters; servers pick it up by rank
        int nadm = 0;
        const int limit = L.sc[SC_NIDLE] < kAdmChunk ? L.sc[SC_NIDLE] : kAdmChunk;
        uint32_t popped[kMaxK];
        for (int k = 0; k < K; ++k) { popped[k] = 0; L.sc[SC_QH0 + k] = L.cs[CS_QHEAD + k]; }
        while (nadm < limit) {
          int best = -1;
          double bkey = 0.0, bdl = 0.0;
          for (int k = 0; k < K; ++k) {
            const int qp = L.cs[CS_QP + k];
            if (qp <= 0) continue;
            if (p.gate_mode == SIM_GATE_OCCUPANCY) {
              if (!(p.invx[k] > 0.0)) continue;
              const double xi = (static_cast<double>(L.cs[CS_X + k]) - p.nx[k]) * p.invx[k];
              const double dl = static_cast<double>(qp) - p.nq[k];
              if (best < 0 || xi < bkey || (xi == bkey && dl > bdl)) { best = k; bkey = xi; bdl = dl; }
            } else if (p.gate_mode == SIM_GATE_PRIORITY) {
              if (best < 0 || p.prio[k] > bkey) { best = k; bkey = p.prio[k]; }
            } else {
              uint32_t pos = static_cast<uint32_t>(L.cs[CS_QHEAD + k]);
              const double st = static_cast<double>(qring[static_cast<size_t>(k) * p.queue_cap + pos]);
              if (best < 0 || st < bkey) { best = k; bkey = st; }
            }
          }
          if (best < 0) break;
          L.adm[nadm++] = static_cast<uint32_t>(best) | (popped[best] << 3);
          ++popped[best];
          L.cs[CS_QP + best] -= 1;
          L.cs[CS_X + best] += 1;
          uint32_t h = static_cast<uint32_t>(L.cs[CS_QHEAD + best]) + 1;
          if (h >= p.queue_cap) h -= p.queue_cap;
          L.cs[CS_QHEAD + best] = static_cast<int32_t>(h);
          L.tl[best * kNTally + SIM_T_U_P] += 1;
        }
        L.sc[SC_NADM] = nadm;
        bool waiting = false;
        for (int k = 0; k < K; ++k)
          if (L.cs[CS_QP + k] > 0 && (p.gate_mode != SIM_GATE_OCCUPANCY || p.invx[k] > 0.0)) waiting = true;
        L.sc[SC_MORE] = (nadm == kAdmChunk && L.sc[SC_NIDLE] > kAdmChunk && waiting) ? 1 : 0;
      }
      __syncthreads();
      const int nadm = L.sc[SC_NADM];
      for (int i = 0; i < nper; ++i) {
        const int g = i * NT + tid;
        bool admitted = false;
        if (g < M && g < N && nadm > 0) {
          const uint64_t word = L.bm_idle[g >> 6];
          if ((word >> (g & 63)) & 1ull) {
            const uint32_t rank = L.pre[g >> 6] + static_cast<uint32_t>(__popcll(word & lanes_below()));
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
              remptok[g] = (remptok[g] & 0xFFFF0000u) | Pl;
              const uint64_t nc = n_cls[g];
              for (int c = 0; c < K; ++c) {   // co-resident decodes switch solo -> mixed
                const int v = static_cast<int>(byte_at(nc, c));
                if (v) {
                  lds_add64(&L.tl[c * kNTally + SIM_T_M_SM], static_cast<uint64_t>(v));
                  atomicSub(&L.cs[CS_YS + c], v);
                  atomicAdd(&L.cs[CS_YM + c], v);
                }
              }
              if (t_next[g] == kIdle) touched |= 1ull << i;
            }
          }
        }
        const uint64_t adm_mask = __ballot(admitted);
        const int wi = (i * NT + (tid & ~63)) >> 6;
        if (lane == 0 && wi < p.nwords && adm_mask) L.bm_idle[wi] &= ~adm_mask;
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
          const int g = i * NT + tid;
          const bool at_level = g >= lo && g < hi && L.loads[g] == level;
          const uint64_t b = __ballot(at_level);
          const int wi = (i * NT + (tid & ~63)) >> 6;
          if (lane == 0 && wi < p.nwords) L.bm_lvl[wi] = b;
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
          const bool busy = t_next[g] != kIdle;
          const bool mid = busy && !((at_boundary >> i) & 1ull);   // joins at the next restart
          const int nd = L.loads[g];
          fin[static_cast<size_t>(g) * B + nd] = iter[g] + Dl + (mid ? 1u : 0u);
          job[static_cast<size_t>(g) * B + nd] = jw;
          n_cls[g] += 1ull << (8 * k);
          if (mid) n_join[g] += 1ull << (8 * k);
          L.loads[g] = static_cast<uint8_t>(nd + 1);
          const bool has_prefill = (remptok[g] & 0xFFFFu) != 0;
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
      uint64_t todo = at_boundary | touched;
      while (todo) {
        const int i = __ffsll(static_cast<long long>(todo)) - 1;
        todo &= todo - 1;
        const int g = i * NT + tid;
        const int rem = static_cast<int>(remptok[g] & 0xFFFFu);
        const int ptok = rem > 0 ? (rem < p.C ? rem : p.C) : 0;
        const int n = L.loads[g];
        if (ptok == 0 && n == 0) {
          t_next[g] = kIdle;
          remptok[g] = static_cast<uint32_t>(rem);
        } else {
          const int64_t base = ((at_boundary >> i) & 1ull) ? t_next[g] : T;   // back-to-back after a completion
          t_next[g] = base + p.c0 + p.cpre * ptok + p.cdec * static_cast<int64_t>(n);
          remptok[g] = static_cast<uint32_t>(rem) | (static_cast<uint32_t>(ptok) << 16);
        }
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
    __syncthreads();
  }

  // ---- write the class state back and add this launch's tallies to the running totals
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
  const int K = p.K, N = p.N, B = p.B;
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
      d += chain(chain(chain(5, static_cast<uint64_t>(g)), p.fin[sg * B + j]), p.job[sg * B + j]);
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
