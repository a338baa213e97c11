// Small kernels of the simulator (reset, totals over replications, state digest) and the launchers (gfx950).
#include <hip/hip_runtime.h>

#include <atomic>
#include <mutex>

#include "gnr_step.h"

namespace gnr {

size_t step_lds_bytes(const Params &p)
{
  // The layout is carved out of a host block that is never read or written: only the total is wanted, but the
  // same code as on the device forms the pointers, and those stay inside a real object this way (the largest
  // configuration the library accepts needs less than a fifth of it).
  alignas(16) static unsigned char block[1 << 20];
  size_t total = 0;
  switch (size_class(p.threads, p.nwords)) {
    case 0: lds_carve<static_words(0), true>(p, block, &total); break;
    case 1: lds_carve<static_words(1)>(p, block, &total); break;
    case 2: lds_carve<static_words(2)>(p, block, &total); break;
    default: lds_carve<static_words(3)>(p, block, &total); break;
  }
  return total;
}

constexpr size_t kLdsPerComputeUnit = 160 * 1024;

// Compute units of the current device (asked once per device; 256 if the runtime does not say).
static int compute_units()
{
  constexpr int kMaxDevices = 64;
  static std::atomic<int> known[kMaxDevices] = {};
  int d = 0;
  if (hipGetDevice(&d) != hipSuccess || d < 0 || d >= kMaxDevices) return 256;
  int n = known[d].load(std::memory_order_relaxed);
  if (n == 0) {
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, d) != hipSuccess || n < 1) n = 256;
    known[d].store(n, std::memory_order_relaxed);
  }
  return n;
}

// Rounds of workgroups a launch of `reps` workgroups needs when a SIMD holds `per_simd` waves of the kernel: every
// workgroup runs for the whole launch, so one that finds no place at first waits for another to end.
static int launch_rounds(int reps, int threads, size_t lds_bytes, int per_simd)
{
  const int by_waves = 4 * per_simd / (threads / 64);   // wave slots of the four SIMDs
  const int by_lds = static_cast<int>(kLdsPerComputeUnit / (lds_bytes ? lds_bytes : 1));
  int wgs = by_waves < by_lds ? by_waves : by_lds;
  wgs = wgs < 1 ? 1 : wgs;
  const int at_once = compute_units() * wgs;
  return (reps + at_once - 1) / at_once;
}

bool step_dense(int reps, int threads, size_t lds_bytes)
{
  return threads <= 512 && launch_rounds(reps, threads, lds_bytes, waves_per_simd(threads, true)) <
                               launch_rounds(reps, threads, lds_bytes, waves_per_simd(threads, false));
}

int step_threads(Params q, int reps)
{
  // A replication with many servers fills the LDS of a compute unit, runs alone there and wants all sixteen
  // waves to hide latency.
  if (q.N > 5120) return 1024;
  // Smaller replications share a compute unit. A workgroup steps faster the more waves it has, as long as its
  // waves have blocks of servers to work on and all workgroups of the launch find a place at once (at most four
  // waves per SIMD): measured on 256, 1024 and 2048 servers with 128 to 2048 replications, the largest workgroup
  // that keeps the number of rounds lowest was the fastest or within 3 % of it in every case; sixteen waves
  // measured 4 to 26 % faster than eight on 2048 to 5000 servers with up to 256 replications.
  // With fewer than two blocks to a wave the larger workgroup only pays where it can still run in the roomy form
  // (256 servers, 1024 replications: 128 threads roomy 19.0 ms per 1000 steps, 256 threads dense 19.6).
  const int blocks = (q.N + 63) / 64;
  int best = 64, best_rounds = 0;
  for (int t = 64; t <= 1024 && t / 64 < 2 * blocks; t *= 2) {   // (a wave more than there are blocks only waits)
    q.threads = t;
    const size_t lds = step_lds_bytes(q);
    if (lds > kLdsPerComputeUnit) break;
    const int rounds = launch_rounds(reps, t, lds, 4);
    // few blocks a wave, and dense (sixteen waves have no roomy form)
    const bool thin = blocks < 2 * (t / 64) && (t > 512 || launch_rounds(reps, t, lds, 2) > rounds);
    if (best_rounds == 0 || rounds < best_rounds || (rounds == best_rounds && !thin)) { best = t; best_rounds = rounds; }
  }
  return best;
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
  for (size_t i = t0; i < n_srv * p.BS; i += stride) p.fin[i] = 0;   // free slots never match an iteration index
  for (size_t i = t0; i < static_cast<size_t>(reps) * CS_WORDS; i += stride) p.cstate[i] = 0;
  for (size_t i = t0; i < static_cast<size_t>(reps) * kTallyWords; i += stride) p.tally[i] = 0;
  for (size_t i = t0; i < static_cast<size_t>(reps) * 3 * p.K * kNBin; i += stride) p.hist[i] = 0;
  if (p.dl_rings)
    for (size_t i = t0; i < static_cast<size_t>(reps) * p.K * (p.cal_mask + 1u); i += stride) {
      p.cal[i] = 0; p.dcal[i] = 0;
      if (p.dcal_m) p.dcal_m[i] = 0;
    }
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
    const uint32_t *dlr = p.ab_classes ? p.qdl + (static_cast<size_t>(r) * K + k) * p.queue_cap : nullptr;
    for (uint32_t i = tid; i < len; i += NT) {
      uint32_t pos = head + i;
      if (pos >= p.queue_cap) pos -= p.queue_cap;
      uint64_t h = chain(chain(chain(2, static_cast<uint64_t>(k)), i), ring[pos]);
      if (dlr) h = chain(h, dlr[pos]);   // with abandonment the deadline is part of the state
      d += h;
    }
  }
  {
    const uint32_t head = static_cast<uint32_t>(cs[CS_DHEAD]), len = static_cast<uint32_t>(cs[CS_DCOUNT]);
    const uint64_t *ring = p.dring + static_cast<size_t>(r) * p.dbuf_cap;
    const uint32_t *dlr = p.ab_classes ? p.ddl + static_cast<size_t>(r) * p.dbuf_cap : nullptr;
    for (uint32_t i = tid; i < len; i += NT) {
      uint32_t pos = head + i;
      if (pos >= p.dbuf_cap) pos -= p.dbuf_cap;
      uint64_t h = chain(chain(3, i), ring[pos]);
      if (dlr) h = chain(h, dlr[pos]);
      d += h;
    }
  }
  if (p.route_mode == SIM_ROUTE_RANDOM_SPLIT || p.route_mode == SIM_ROUTE_WEIGHTED_SPLIT) {   // the mixed group's buffer
    const uint32_t head = static_cast<uint32_t>(cs[CS_DHEAD_M]), len = static_cast<uint32_t>(cs[CS_DCOUNT_M]);
    const uint64_t *ring = p.dring_m + static_cast<size_t>(r) * p.dbuf_cap;
    const uint32_t *dlr = p.ab_classes ? p.ddl_m + static_cast<size_t>(r) * p.dbuf_cap : nullptr;
    for (uint32_t i = tid; i < len; i += NT) {
      uint32_t pos = head + i;
      if (pos >= p.dbuf_cap) pos -= p.dbuf_cap;
      uint64_t h = chain(chain(6, i), ring[pos]);
      if (dlr) h = chain(h, dlr[pos]);
      d += h;
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

// ------------------------------------------------------------------ static workspace ----
// Device memory for handles whose caller cannot allocate any (sim_create_static). In host code the array's name
// is only a stand-in for the symbol: its address on a device comes from hipGetSymbolAddress, asked once per device
// with that device current, and that pointer is what the kernels are given.
static __device__ __align__(256) unsigned char scratch[SIM_STATIC_WORKSPACE_BYTES];

int static_workspace(void **dev_ptr, size_t *bytes)
{
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void *resolved[kMaxDevices] = {};
  int d = -1;
  if (hipGetDevice(&d) != hipSuccess || d < 0 || d >= kMaxDevices) return SIM_EHIP;
  std::lock_guard<std::mutex> lock(mu);
  if (!resolved[d]) {
    void *ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return SIM_EHIP;
    resolved[d] = ptr;
  }
  *dev_ptr = resolved[d];
  *bytes = sizeof(scratch);
  return SIM_OK;
}

// ------------------------------------------------------------------ launchers ----
// The step kernel's policy variants, each compiled in a translation unit of its own (gnr_step_<variant>.hip).
StepKernel step_kernel_plain(int size_class, bool dense);
StepKernel step_kernel_rr(int size_class, bool dense);
StepKernel step_kernel_im(int size_class, bool dense);
StepKernel step_kernel_ab(int size_class, bool dense);
StepKernel step_kernel_ab_rr(int size_class, bool dense);
StepKernel step_kernel_ab_im(int size_class, bool dense);
StepKernel step_kernel_ws(int size_class, bool dense);

static int hip_ok(hipError_t e) { return e == hipSuccess ? SIM_OK : SIM_EHIP; }

int launch_reset(const Params &p, int reps, void *stream)
{
  hipLaunchKernelGGL(gnr_reset_kernel, dim3(1024), dim3(256), 0, static_cast<hipStream_t>(stream), p, reps);
  return hip_ok(hipGetLastError());
}

int launch_steps(const Params &p, int reps, int threads, size_t lds_bytes, uint32_t step_begin, uint32_t n_steps,
                 void *stream)
{
  const int size = size_class(threads, p.nwords);
  const bool ab = p.dl_rings != 0;
  // The roomy form of a small size class holds two waves per SIMD, the dense form four: the dense one is taken when
  // the launch then needs fewer rounds of workgroups (every workgroup runs for the whole launch, so a workgroup
  // that finds no place at first waits for another to end).
  const bool dense = step_dense(reps, threads, lds_bytes);
  StepKernel kernel = nullptr;
  switch (p.route_mode) {
    case SIM_ROUTE_SOLO_FIRST: kernel = ab ? step_kernel_ab(size, dense) : step_kernel_plain(size, dense); break;
    case SIM_ROUTE_RANDOM_SPLIT: kernel = ab ? step_kernel_ab_rr(size, dense) : step_kernel_rr(size, dense); break;
    case SIM_ROUTE_IMMEDIATE: kernel = ab ? step_kernel_ab_im(size, dense) : step_kernel_im(size, dense); break;
    // (the weighted router is the randomized router's variant with deadline rings plus the class draws)
    case SIM_ROUTE_WEIGHTED_SPLIT: kernel = ab ? step_kernel_ws(size, dense) : nullptr; break;
    default: break;
  }
  if (!kernel) return SIM_EINVAL;
  if (lds_bytes > 64 * 1024) {   // more than the default dynamic LDS limit has to be asked for
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds_bytes));
    if (e != hipSuccess) return SIM_EHIP;
  }
  const StepArrays a = {p.arr_thr, p.len_tab, p.t_next, p.iter, p.remptok, p.pf_job, p.n_cls, p.n_join,
                        p.fin,     p.job,     p.qring,  p.dring, p.cstate, p.tally,  p.hist,
                        p.pat_tab, p.qdl,     p.ddl,    p.cal,   p.dcal,   p.dring_m, p.ddl_m, p.dcal_m};
  hipLaunchKernelGGL(kernel, dim3(reps), dim3(threads), lds_bytes, static_cast<hipStream_t>(stream), p.self, a, p.key0,
                     p.key1, step_begin, n_steps);
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
