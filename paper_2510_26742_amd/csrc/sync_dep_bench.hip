// Grid-synchronisation experiment with a REAL dependency between blocks (Section 5.2 of the paper:
// a software barrier inside one persistent kernel instead of kernel boundaries).  Table 3's update
// x <- x + b touches only a thread's own elements, so it prices the wait but says nothing about what
// it costs to make one block's results visible to the others - on this chip eight dies with an L2
// each, which ordinary loads and stores do not keep coherent inside a kernel.  Here update k is
//     x_{k+1}[r][c] = max_{j = 1 .. fan} x_k[(r + j) mod 256][c] + b[r][c]
// on a 256 x 1024 fp32 array, one 256-thread block per row r: every block reads `fan` rows that other
// blocks (on other dies) wrote in the update before.  max and + are exact in fp32, so the result is
// checked bit for bit against a host simulation: a stale read shows up as a wrong value, never as a
// hang (all waits are bounded).
//
// Barriers
//   COUNTER  one arrival counter, every block adds 1 and polls it
//   XCD      two levels: one counter per group of blocks (block index mod 8 = die under round-robin
//            dispatch), the last of a group adds to a root counter, the last of all publishes the
//            epoch in one word per group, which the group polls with s_sleep back-off
//   FLAGS    no read-modify-write at all: block i stores the epoch in word i of a 1 KiB array, one
//            wave per block polls the whole array with one 16-byte load per lane
//   FLAGS8   the same with 8 copies of the array 4 KiB apart: a block stores into all 8 and polls one
//   GROUPADD one add without return value per block on its group's counter, everyone polls the 8 counters
//   XCC      as XCD, but the groups are the real dies (hardware register XCC_ID): arrivals are counted in
//            the die's own L2, and only the last block of a die performs the device-scope release
// Data paths (how update k+1 is made to see update k's rows)
//   NONE     no dependency (own row, in place): the barrier alone, comparable with Table 3
//   BYPASS   write-through stores and loads that bypass the die's L2 (device-scope bits on the
//            instructions), no fence
//   INV      write-through stores; after the wait one wave per block invalidates the caches
//            (acquire fence), then ordinary cached loads
//   FENCE    ordinary stores and loads with the device-scope release / acquire fences of the
//            language memory model (cache write-back + invalidate)
//   FRESH    write-through stores, ordinary loads, and every update writes a plane that nobody has
//            read before (planes >= n_ops + 1), so no cache can hold a stale copy
//   WBACK    ordinary (write-back) stores, loads that bypass the L2; the release writes the lines back
// Every dependent data path performs a device-scope release (cache write-back, which also waits for
// write-through stores in flight) between a block's stores and its arrival: one per block, or - XCC - one
// per die.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/pi0_bench.h"

namespace {

constexpr int ROWS = 256, COLS = 1024, PLANE = ROWS * COLS;
constexpr int MAX_FAN = 32;

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

// cache-policy bits of gfx950 buffer instructions
constexpr int AUX_SC1 = 16;   // device scope: stores write through to memory, loads do not hit in a die's L2

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

// state layout (unsigned words): [0] error flag, [32] counter, [64 + 32 g] group counters, [320] root counter,
// [352 + 32 g] group epochs, [768 .. 1023] per-block flags,
// [1024 + 1024 g + i] copy g of block i's flag (FLAGS8)
enum { ST_ERR = 0, ST_CNT = 32, ST_GCNT = 64, ST_ROOT = 320, ST_GEPOCH = 352, ST_FLAGS = 768, ST_WORDS = 1024,
       ST_MEMBERS = 640 /* + 32 x: blocks on die x */, ST_REP = 1024, ST_REP_STRIDE = 1024 /* words: 8 copies of the 256 flags, 4 KiB apart */, ST_ALL_WORDS = 1024 + 8 * 1024 };

__device__ __forceinline__ unsigned ld_relaxed(const unsigned* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_relaxed(unsigned* p, unsigned v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Called by wave 0 of the block after the block's stores have completed (s_barrier behind vmcnt(0)).
// epoch = number of the barrier, 1-based.  Returns when every block has arrived or the bound ran out.
// die (XCC) the calling wave runs on: bits 3:0 of hardware register XCC_ID (id 20)
__device__ __forceinline__ unsigned xcc_id() { return (unsigned)__builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) & 15u; }

template <int BAR, int DATA>
__device__ __forceinline__ void grid_wait(unsigned* state, unsigned epoch, unsigned spin_limit, unsigned xcc, unsigned members,
                                          unsigned n_xcc) {
  const int lane = threadIdx.x & 63;
  const unsigned nblk = gridDim.x;
  if (BAR == PI0_BARRIER_COUNTER) {
    if (lane == 0) {
      __hip_atomic_fetch_add(&state[ST_CNT], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const unsigned target = epoch * nblk;
      unsigned spins = 0;
      while (ld_relaxed(&state[ST_CNT]) < target) {
        if (++spins > spin_limit || ld_relaxed(&state[ST_ERR]) != 0u) { st_relaxed(&state[ST_ERR], 1u); break; }
      }
    }
  } else if (BAR == PI0_BARRIER_XCD) {
    if (lane == 0) {
      const unsigned g = blockIdx.x & 7u;
      const unsigned gsize = (nblk + 7u - g) >> 3;
      const unsigned old = __hip_atomic_fetch_add(&state[ST_GCNT + 32 * g], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (old + 1u == epoch * gsize) {
        const unsigned ngroups = nblk < 8u ? nblk : 8u;
        const unsigned oldr = __hip_atomic_fetch_add(&state[ST_ROOT], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (oldr + 1u == epoch * ngroups) {
          for (unsigned k = 0; k < ngroups; k++) st_relaxed(&state[ST_GEPOCH + 32 * k], epoch);
        }
      }
      unsigned spins = 0;
      while (ld_relaxed(&state[ST_GEPOCH + 32 * g]) < epoch) {
        __builtin_amdgcn_s_sleep(1);
        if (++spins > spin_limit || ld_relaxed(&state[ST_ERR]) != 0u) { st_relaxed(&state[ST_ERR], 1u); break; }
      }
    }
  } else if (BAR == PI0_BARRIER_XCC) {
    // arrivals are counted inside the die (an atomic without device scope is performed in the die's own L2); the
    // last block of a die releases the die's writes to memory ONCE for all of them, adds to the root counter at
    // device scope, and the last die publishes the epoch per die
    if (lane == 0) {
      const unsigned old = __hip_atomic_fetch_add(&state[ST_GCNT + 32 * xcc], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      if (old + 1u == epoch * members) {
        if (DATA != PI0_SYNCDATA_NONE) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        const unsigned oldr = __hip_atomic_fetch_add(&state[ST_ROOT], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (oldr + 1u == epoch * n_xcc) {
          for (unsigned k = 0; k < 8u; k++) st_relaxed(&state[ST_GEPOCH + 32 * k], epoch);
        }
      }
      unsigned spins = 0;
      while (ld_relaxed(&state[ST_GEPOCH + 32 * xcc]) < epoch) {
        __builtin_amdgcn_s_sleep(1);
        if (++spins > spin_limit || ld_relaxed(&state[ST_ERR]) != 0u) { st_relaxed(&state[ST_ERR], 1u); break; }
      }
    }
  } else if (BAR == PI0_BARRIER_GROUPADD) {
    // arrivals: one fire-and-forget add per block on its group's counter; everybody polls the 8 counters
    const unsigned g = blockIdx.x & 7u;
    if (lane == 0) (void)__hip_atomic_fetch_add(&state[ST_GCNT + 32 * g], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    unsigned spins = 0;
    while (true) {
      bool ok = true;
      if (lane < 8 && (unsigned)lane < nblk) {
        const unsigned gsize = (nblk + 7u - (unsigned)lane) >> 3;
        ok = ld_relaxed(&state[ST_GCNT + 32 * lane]) >= epoch * gsize;
      }
      if (__builtin_amdgcn_ballot_w64(!ok) == 0ull) break;
      __builtin_amdgcn_s_sleep(1);
      if (++spins > spin_limit || ld_relaxed(&state[ST_ERR]) != 0u) {
        if (lane == 0) st_relaxed(&state[ST_ERR], 1u);
        break;
      }
    }
  } else if (BAR == PI0_BARRIER_FLAGS8) {
    // block i stores the epoch in word i of 8 copies of the flag array (lanes 0..7, one store instruction); the
    // blocks of group g = i mod 8 poll copy g only, so a copy has 32 pollers instead of 256
    if (lane < 8) st_relaxed(&state[ST_REP + ST_REP_STRIDE * lane + blockIdx.x], epoch);
    const __amdgpu_buffer_rsrc_t fr = make_rsrc(state + ST_REP + ST_REP_STRIDE * (blockIdx.x & 7u), 256 * 4);
    unsigned spins = 0;
    while (true) {
      const u32x4 f = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(fr, lane * 16, 0, AUX_SC1));
      bool ok = true;
#pragma unroll
      for (int j = 0; j < 4; j++) ok = ok && (f[j] >= epoch || (unsigned)(4 * lane + j) >= nblk);
      if (__builtin_amdgcn_ballot_w64(!ok) == 0ull) break;
      __builtin_amdgcn_s_sleep(1);
      if (++spins > spin_limit || ld_relaxed(&state[ST_ERR]) != 0u) {
        if (lane == 0) st_relaxed(&state[ST_ERR], 1u);
        break;
      }
    }
  } else {   // FLAGS
    if (lane == 0) st_relaxed(&state[ST_FLAGS + blockIdx.x], epoch);
    const __amdgpu_buffer_rsrc_t fr = make_rsrc(state + ST_FLAGS, 256 * 4);
    unsigned spins = 0;
    while (true) {
      // lane l reads flags 4 l .. 4 l + 3 past the L2; words of blocks that do not exist count as arrived
      const u32x4 f = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(fr, lane * 16, 0, AUX_SC1));
      bool ok = true;
#pragma unroll
      for (int j = 0; j < 4; j++) ok = ok && (f[j] >= epoch || (unsigned)(4 * lane + j) >= nblk);
      if (__builtin_amdgcn_ballot_w64(!ok) == 0ull) break;
      __builtin_amdgcn_s_sleep(1);
      if (++spins > spin_limit || ld_relaxed(&state[ST_ERR]) != 0u) {
        if (lane == 0) st_relaxed(&state[ST_ERR], 1u);
        break;
      }
    }
  }
}

template <int BAR, int DATA>
__global__ __launch_bounds__(256) void sync_dep_kernel(float* x, int planes, const float* b, int n_ops, int op0, int fan,
                                                       unsigned* state, unsigned spin_limit, unsigned epoch0) {
  const int r = blockIdx.x, t = threadIdx.x;
  const f32x4 bv = *reinterpret_cast<const f32x4*>(b + (size_t)r * COLS + 4 * t);
  unsigned xcc = 0, members = 0, n_xcc = 0;
  if (BAR == PI0_BARRIER_XCC) {
    // who shares a die with whom: every block registers on its die's member counter (cleared by the host before each
    // launch); one counter barrier later the counts are final
    xcc = xcc_id() & 7u;
    if (t == 0) {
      __hip_atomic_fetch_add(&state[ST_MEMBERS + 32 * xcc], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_fetch_add(&state[ST_CNT], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      unsigned spins = 0;
      while (ld_relaxed(&state[ST_CNT]) < gridDim.x) {
        if (++spins > spin_limit || ld_relaxed(&state[ST_ERR]) != 0u) { st_relaxed(&state[ST_ERR], 1u); break; }
      }
    }
    __syncthreads();
    members = ld_relaxed(&state[ST_MEMBERS + 32 * xcc]);
    for (unsigned k = 0; k < 8u; k++) n_xcc += ld_relaxed(&state[ST_MEMBERS + 32 * k]) != 0u ? 1u : 0u;
  }
  for (int op = 0; op < n_ops; op++) {
    const int ps = (op0 + op) % planes, pd = (op0 + op + 1) % planes;
    const float* src = x + (size_t)ps * PLANE;
    float* dst = x + (size_t)pd * PLANE;
    f32x4 v;
    if (DATA == PI0_SYNCDATA_NONE) {
      v = *reinterpret_cast<const f32x4*>(x + (size_t)r * COLS + 4 * t);
      v += bv;
      *reinterpret_cast<f32x4*>(x + (size_t)r * COLS + 4 * t) = v;
    } else {
      f32x4 in[MAX_FAN];
      const f32x4 ninf = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
      if (DATA == PI0_SYNCDATA_BYPASS || DATA == PI0_SYNCDATA_WBACK) {
        const __amdgpu_buffer_rsrc_t sr = make_rsrc(src, PLANE * 4);
#pragma unroll
        for (int j = 0; j < MAX_FAN; j++) {
          const int rr = (r + 1 + j) & (ROWS - 1);
          if (j < fan) in[j] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(sr, (rr * COLS + 4 * t) * 4, 0, AUX_SC1));
          else in[j] = ninf;
        }
      } else {
#pragma unroll
        for (int j = 0; j < MAX_FAN; j++) {
          const int rr = (r + 1 + j) & (ROWS - 1);
          if (j < fan) in[j] = *reinterpret_cast<const f32x4*>(src + (size_t)rr * COLS + 4 * t);
          else in[j] = ninf;
        }
      }
      v = in[0];
#pragma unroll
      for (int j = 1; j < MAX_FAN; j++) {
#pragma unroll
        for (int e = 0; e < 4; e++) v[e] = fmaxf(v[e], in[j][e]);
      }
      v += bv;
      if (DATA == PI0_SYNCDATA_FENCE || DATA == PI0_SYNCDATA_WBACK) {
        *reinterpret_cast<f32x4*>(dst + (size_t)r * COLS + 4 * t) = v;
      } else {
        const __amdgpu_buffer_rsrc_t dr = make_rsrc(dst, PLANE * 4);
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), dr, (r * COLS + 4 * t) * 4, 0, AUX_SC1);
      }
    }
    if (op + 1 < n_ops) {
      // every store of the block has been acknowledged before anyone announces the block's arrival
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // a workgroup-scope fence does not wait for global stores
      __syncthreads();
      if (t < 64) {
        // device-scope release: the die's dirty lines are written back (FENCE) and - for every dependent data path -
        // the write-through stores issued before are complete, not merely accepted, before the arrival is announced
        // (without it an arrival was seen to overtake the data it announces)
        if (DATA != PI0_SYNCDATA_NONE && BAR != PI0_BARRIER_XCC) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        grid_wait<BAR, DATA>(state, epoch0 + (unsigned)op + 1u, spin_limit, xcc, members, n_xcc);
        if (DATA == PI0_SYNCDATA_INV || DATA == PI0_SYNCDATA_FENCE) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
      }
      __syncthreads();
    }
  }
}

__global__ void sync_dep_clear_kernel(unsigned* state, int first) {   // first = 1 keeps the error flag
  for (int i = first + threadIdx.x; i < ST_ALL_WORDS; i += blockDim.x) state[i] = 0u;
}

template <int BAR>
void launch_dep(int data, hipStream_t s, float* x, int planes, const float* b, int n_ops, int op0, int fan, unsigned* state,
                unsigned spin_limit, unsigned epoch0) {
  const dim3 grid(ROWS), block(256);
  switch (data) {
    case PI0_SYNCDATA_NONE: sync_dep_kernel<BAR, PI0_SYNCDATA_NONE><<<grid, block, 0, s>>>(x, planes, b, n_ops, op0, fan, state, spin_limit, epoch0); break;
    case PI0_SYNCDATA_BYPASS: sync_dep_kernel<BAR, PI0_SYNCDATA_BYPASS><<<grid, block, 0, s>>>(x, planes, b, n_ops, op0, fan, state, spin_limit, epoch0); break;
    case PI0_SYNCDATA_INV: sync_dep_kernel<BAR, PI0_SYNCDATA_INV><<<grid, block, 0, s>>>(x, planes, b, n_ops, op0, fan, state, spin_limit, epoch0); break;
    case PI0_SYNCDATA_FENCE: sync_dep_kernel<BAR, PI0_SYNCDATA_FENCE><<<grid, block, 0, s>>>(x, planes, b, n_ops, op0, fan, state, spin_limit, epoch0); break;
    case PI0_SYNCDATA_WBACK: sync_dep_kernel<BAR, PI0_SYNCDATA_WBACK><<<grid, block, 0, s>>>(x, planes, b, n_ops, op0, fan, state, spin_limit, epoch0); break;
    default: sync_dep_kernel<BAR, PI0_SYNCDATA_FRESH><<<grid, block, 0, s>>>(x, planes, b, n_ops, op0, fan, state, spin_limit, epoch0); break;
  }
}

}  // namespace

extern "C" int pi0_sync_dep_bench(int barrier, int data, int fan, int n_ops, int reps, float* d_x, int planes, const float* d_b,
                                  unsigned* d_state, double* h_ms, void* hip_stream) {
  if (d_x == nullptr || d_b == nullptr || d_state == nullptr || h_ms == nullptr) return PI0_EINVAL;
  if (barrier < PI0_BARRIER_COUNTER || barrier > PI0_BARRIER_XCC || data < PI0_SYNCDATA_NONE || data > PI0_SYNCDATA_WBACK) return PI0_EINVAL;
  if (n_ops < 1 || n_ops > 100000 || reps < 1 || reps > 1000 || fan < 1 || fan > MAX_FAN) return PI0_EINVAL;
  if (planes < 1 || planes > 4096) return PI0_EINVAL;
  if (data != PI0_SYNCDATA_NONE && planes < 2) return PI0_EINVAL;
  if (data == PI0_SYNCDATA_FRESH && (reps != 1 || planes < n_ops + 1)) return PI0_EINVAL;
  if ((reinterpret_cast<uintptr_t>(d_x) & 15) != 0 || (reinterpret_cast<uintptr_t>(d_b) & 15) != 0 ||
      (reinterpret_cast<uintptr_t>(d_state) & 15) != 0)
    return PI0_EINVAL;
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  int dev = 0, cus = 0;   // the barrier needs every block resident at once
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
    return PI0_EHIP;
  if (cus < ROWS) return PI0_ESTATE;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  hipError_t e = hipEventCreate(&e0);
  if (e == hipSuccess) e = hipEventCreate(&e1);
  const unsigned spin_limit = 1u << 20;
  int rc = PI0_OK;
  if (e == hipSuccess) {
    sync_dep_clear_kernel<<<1, 256, 0, s>>>(d_state, 0);
    e = hipEventRecord(e0, s);
    for (int r = 0; r < reps && e == hipSuccess; r++) {
      // epochs keep counting across repetitions (n_ops - 1 barriers each), so the counters and flags need no clearing in between
      const unsigned epoch0 = (unsigned)r * (unsigned)(n_ops - 1);
      const int op0 = (int)(((long long)r * n_ops) % planes);
      if (barrier == PI0_BARRIER_COUNTER) launch_dep<PI0_BARRIER_COUNTER>(data, s, d_x, planes, d_b, n_ops, op0, fan, d_state, spin_limit, epoch0);
      else if (barrier == PI0_BARRIER_XCD) launch_dep<PI0_BARRIER_XCD>(data, s, d_x, planes, d_b, n_ops, op0, fan, d_state, spin_limit, epoch0);
      else if (barrier == PI0_BARRIER_FLAGS) launch_dep<PI0_BARRIER_FLAGS>(data, s, d_x, planes, d_b, n_ops, op0, fan, d_state, spin_limit, epoch0);
      else if (barrier == PI0_BARRIER_FLAGS8) launch_dep<PI0_BARRIER_FLAGS8>(data, s, d_x, planes, d_b, n_ops, op0, fan, d_state, spin_limit, epoch0);
      else if (barrier == PI0_BARRIER_GROUPADD) launch_dep<PI0_BARRIER_GROUPADD>(data, s, d_x, planes, d_b, n_ops, op0, fan, d_state, spin_limit, epoch0);
      else {
        // the member registration restarts with every launch: its counter and the die counters are cleared, epochs restart
        sync_dep_clear_kernel<<<1, 256, 0, s>>>(d_state, 1);
        launch_dep<PI0_BARRIER_XCC>(data, s, d_x, planes, d_b, n_ops, op0, fan, d_state, spin_limit, 0u);
      }
      e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipEventRecord(e1, s);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (e == hipSuccess) *h_ms = (double)ms / reps;
    unsigned flag = 0;
    if (e == hipSuccess) e = hipMemcpyAsync(&flag, d_state + ST_ERR, sizeof(flag), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e == hipSuccess && flag != 0u) rc = PI0_ESTATE;   // a bounded wait ran out
  }
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (rc != PI0_OK) return rc;
  return e == hipSuccess ? PI0_OK : PI0_EHIP;
}
