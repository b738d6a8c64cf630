// Measurement hook: what one synchronisation of the workgroups of a launch costs on this machine.
// The resident launches (forward chains, sweeps) replace a kernel boundary per time step by an
// arrival counter per XCD plus an exchange of the new operand through that XCD's L2; this file
// times exactly those primitives, alone, so that the per-step times of the real kernels can be
// set against their floor.  Nothing here takes part in a gradient computation.
//
// Variants (256 workgroups of 256 threads, one per compute unit, 96 KiB of LDS each so that no two
// share a compute unit):
//   0  all 256 workgroups meet at one agent-scope counter (release fence, add, poll, acquire fence)
//   1  the 32 workgroups of each XCD meet at their XCD's counter: arrive by a relaxed agent-scope
//      add, poll with agent-scope loads; no fences
//   2  as 1, and every workgroup first stores 512 bytes which, after the meeting, the 32 of its XCD
//      read (16 KiB per workgroup) with loads that bypass the compute unit's cache; every word read
//      is checked
// The XCD of a workgroup is the hardware's XCC id, its rank there a ticket drawn from a per-XCD
// counter.  Every wait is bounded; a workgroup that gives up raises a flag all others leave on.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "mebptt.h"

namespace {

constexpr unsigned SPIN_LIMIT = 400000u;
constexpr int WGS = 256, GROUPS = 8, MEMBERS = 32, SLAB_WORDS = 128, RING = 4;

__device__ inline unsigned hw_xcc_id() {
  unsigned v;
  asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(v));
  return v & 0xf;
}

struct SyncParams {
  unsigned* all;      // one counter
  unsigned* grp;      // GROUPS counters, 256 bytes apart
  unsigned* ticket;   // GROUPS ticket counters, 256 bytes apart
  unsigned* flag;     // [0] give-up flag, [1] wrong words, [2] placement errors
  unsigned* buf;      // RING x WGS x SLAB_WORDS exchange words
  int iters;
};

template <int V>
__global__ __launch_bounds__(256) void sync_kernel(SyncParams p) {
  extern __shared__ float lds[];
  __shared__ int ok, s_g, s_rank;
  if (threadIdx.x == 1) lds[0] = 1.0f;
  if (threadIdx.x == 0) {
    const unsigned xcc = hw_xcc_id();
    int good = xcc < (unsigned)GROUPS;
    unsigned t = 0;
    if (good) {
      t = __hip_atomic_fetch_add(p.ticket + xcc * 64, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      good = t < (unsigned)MEMBERS;
    }
    if (!good) {
      __hip_atomic_store(p.flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_fetch_add(p.flag + 2, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    ok = good;
    s_g = good ? (int)xcc : 0;
    s_rank = (int)(t % MEMBERS);
  }
  __syncthreads();
  if (!ok) return;
  const int g = s_g, rank = s_rank;
  const unsigned me = (unsigned)(g * MEMBERS + rank);
  unsigned bad = 0;
  for (int it = 1; it <= p.iters; ++it) {
    unsigned* slab = p.buf + (size_t)(it % RING) * WGS * SLAB_WORDS;
    if (V == 2) {
      if (threadIdx.x < SLAB_WORDS) slab[me * SLAB_WORDS + threadIdx.x] = (unsigned)it * 1000003u + me * 131u + threadIdx.x;
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the stores have reached the L2
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      int good = 1;
      unsigned spins = 0;
      if (V == 0) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        __hip_atomic_fetch_add(p.all, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        while (__hip_atomic_load(p.all, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < (unsigned)it * WGS) {
          if (++spins > SPIN_LIMIT || ((spins & 63) == 0 &&
                                       __hip_atomic_load(p.flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u)) {
            good = 0;
            break;
          }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
      } else {
        unsigned* ctr = p.grp + g * 64;
        __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        while (__hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < (unsigned)it * MEMBERS) {
          if (++spins > SPIN_LIMIT || ((spins & 63) == 0 &&
                                       __hip_atomic_load(p.flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u)) {
            good = 0;
            break;
          }
        }
      }
      if (!good) __hip_atomic_store(p.flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      ok = good;
    }
    __syncthreads();
    if (!ok) break;
    if (V == 2) {
      // the 32 x 512 bytes of this XCD: 4096 words, 256 threads x 4 loads of 16 bytes
      const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(slab, 0, 0x7fffffff, 0x00020000);
      typedef unsigned u4 __attribute__((ext_vector_type(4)));
      u4 v[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int idx = (q * 256 + (int)threadIdx.x) * 4;
        const int member = idx / SLAB_WORDS, off = idx % SLAB_WORDS;
        v[q] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)(((g * MEMBERS + member) * SLAB_WORDS + off) * 4), 0, 16);
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int idx = (q * 256 + (int)threadIdx.x) * 4;
        const int member = idx / SLAB_WORDS, off = idx % SLAB_WORDS;
        const unsigned want = (unsigned)it * 1000003u + (unsigned)(g * MEMBERS + member) * 131u + off;
        bad += (v[q].x != want) + (v[q].y != want + 1) + (v[q].z != want + 2) + (v[q].w != want + 3);
      }
    }
  }
  if (bad) atomicAdd(p.flag + 1, bad);
}

// A kernel of 256 workgroups that does nothing for `ticks` ticks of the 100 MHz wall clock.
__global__ __launch_bounds__(256) void wait_kernel(long long ticks) {
  const long long t0 = wall_clock64();
  while (wall_clock64() - t0 < ticks) {
  }
}

struct Buffers {
  unsigned* base = nullptr;
  ~Buffers() {
    if (base) (void)hipFree(base);
  }
};

}  // namespace

extern "C" int mebptt_measure_sync(int32_t variant, int32_t iters, void* stream, double* us_per_sync, int32_t* status) {
  if (variant < 0 || variant > 2 || iters < 1 || iters > 100000 || !us_per_sync || !status) return MEBPTT_EINVAL;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  // layout in words: all @0, grp @64.., ticket @1024.., flag @2048.., exchange ring after 4096
  const size_t words = 4096 + (size_t)RING * WGS * SLAB_WORDS;
  Buffers b;
  if (hipMalloc(&b.base, words * sizeof(unsigned)) != hipSuccess) return MEBPTT_EHIP;
  if (hipMemsetAsync(b.base, 0, words * sizeof(unsigned), st) != hipSuccess) return MEBPTT_EHIP;
  SyncParams p{b.base, b.base + 64, b.base + 1024, b.base + 2048, b.base + 4096, iters};
  const void* fn = variant == 0 ? reinterpret_cast<const void*>(sync_kernel<0>)
                   : variant == 1 ? reinterpret_cast<const void*>(sync_kernel<1>)
                                  : reinterpret_cast<const void*>(sync_kernel<2>);
  const int lds = 96 * 1024;
  if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess) return MEBPTT_EHIP;
  hipEvent_t a = nullptr, z = nullptr;
  if (hipEventCreate(&a) != hipSuccess) return MEBPTT_EHIP;
  hipError_t e = hipEventCreate(&z);
  if (e == hipSuccess) e = hipEventRecord(a, st);
  if (e == hipSuccess) {
    if (variant == 0)
      sync_kernel<0><<<dim3(WGS), dim3(256), lds, st>>>(p);
    else if (variant == 1)
      sync_kernel<1><<<dim3(WGS), dim3(256), lds, st>>>(p);
    else
      sync_kernel<2><<<dim3(WGS), dim3(256), lds, st>>>(p);
    e = hipGetLastError();
  }
  if (e == hipSuccess) e = hipEventRecord(z, st);
  if (e == hipSuccess) e = hipEventSynchronize(z);
  float ms = 0.0f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, a, z);
  unsigned flags[3] = {0, 0, 0};
  if (e == hipSuccess) e = hipMemcpy(flags, p.flag, sizeof flags, hipMemcpyDeviceToHost);
  (void)hipEventDestroy(a);
  if (z) (void)hipEventDestroy(z);
  if (e != hipSuccess) return MEBPTT_EHIP;
  *us_per_sync = (double)ms * 1e3 / iters;
  *status = flags[2] ? 2 : flags[0] ? 1 : flags[1] ? 3 : 0;   // 2 placement, 1 a wait gave up, 3 wrong words read
  return MEBPTT_OK;
}

// What a pair of events around a single launch adds to the launch's own time, for a kernel that
// lasts about `kernel_us`: `reps` such launches back to back inside one event pair give the time
// per launch, the same launches each inside its own event pair give the bracketed time; the
// difference is what event-sampled per-launch times carry on top (it depends on the kernel's
// length: part of the event processing hides behind a kernel that runs for a while).
extern "C" int mebptt_bracket_overhead_us(double kernel_us, int32_t reps, void* stream, double* per_launch_us,
                                          double* bracketed_us) {
  if (!(kernel_us >= 0.0) || kernel_us > 1000.0 || reps < 1 || reps > 2000 || !per_launch_us || !bracketed_us) return MEBPTT_EINVAL;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  const long long ticks = (long long)(kernel_us * 100.0);
  const int n = reps;
  hipEvent_t* ev = new hipEvent_t[2 * n + 2]();
  hipError_t e = hipSuccess;
  for (int i = 0; i < 2 * n + 2 && e == hipSuccess; ++i) e = hipEventCreate(&ev[i]);
  if (e == hipSuccess) {
    for (int i = 0; i < 8; ++i) wait_kernel<<<dim3(256), dim3(256), 0, st>>>(ticks);   // warm-up
    e = hipEventRecord(ev[2 * n], st);
  }
  if (e == hipSuccess) {
    for (int i = 0; i < n; ++i) wait_kernel<<<dim3(256), dim3(256), 0, st>>>(ticks);
    e = hipEventRecord(ev[2 * n + 1], st);
  }
  for (int i = 0; i < n && e == hipSuccess; ++i) {
    e = hipEventRecord(ev[2 * i], st);
    wait_kernel<<<dim3(256), dim3(256), 0, st>>>(ticks);
    if (e == hipSuccess) e = hipEventRecord(ev[2 * i + 1], st);
  }
  if (e == hipSuccess) e = hipGetLastError();
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  float ms = 0.0f;
  double sum = 0.0;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, ev[2 * n], ev[2 * n + 1]);
  const double plain = (double)ms * 1e3 / n;
  for (int i = 0; i < n && e == hipSuccess; ++i) {
    e = hipEventElapsedTime(&ms, ev[2 * i], ev[2 * i + 1]);
    sum += (double)ms * 1e3;
  }
  for (int i = 0; i < 2 * n + 2; ++i)
    if (ev[i]) (void)hipEventDestroy(ev[i]);
  delete[] ev;
  if (e != hipSuccess) return MEBPTT_EHIP;
  *per_launch_us = plain;
  *bracketed_us = sum / n;
  return MEBPTT_OK;
}
