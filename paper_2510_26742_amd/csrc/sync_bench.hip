// Synchronisation-overhead micro-benchmark (Section 5.2, Table 3 of the paper): the same trivial
// element-wise update x <- x + b on a 256 x 1024 fp32 array, one 256-thread block per row, n_ops
// times in a row, with the dependency between consecutive updates enforced in different ways:
// eager kernel launches, one hipGraph of n_ops kernel nodes, one kernel with a software grid
// barrier between updates (with and without device-scope release/acquire), and one kernel with
// no synchronisation at all (the baseline).  Every thread only ever touches its own 4 elements,
// so all variants produce exactly x0 + n_ops * b; the barriers are timed, not needed.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/pi0_bench.h"

namespace {

constexpr int ROWS = 256, COLS = 1024;

__global__ __launch_bounds__(256) void sync_add_kernel(float4* x, const float4* b) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  float4 v = x[i];
  const float4 w = b[i];
  v.x += w.x; v.y += w.y; v.z += w.z; v.w += w.w;
  x[i] = v;
}

// state[0] = arrival counter, state[1] = error flag (a bounded wait ran out)
template <int MODE>   // 0 no synchronisation, 1 relaxed barrier, 2 release/acquire barrier
__global__ __launch_bounds__(256) void sync_loop_kernel(float4* x, const float4* b, int n_ops, unsigned* state,
                                                        unsigned spin_limit) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  for (int op = 0; op < n_ops; op++) {
    float4 v = x[i];
    const float4 w = b[i];
    v.x += w.x; v.y += w.y; v.z += w.z; v.w += w.w;
    x[i] = v;
    if (MODE != 0 && op + 1 < n_ops) {
      __syncthreads();
      if (threadIdx.x == 0) {
        const unsigned target = (unsigned)(op + 1) * gridDim.x;
        if (MODE == 2) __hip_atomic_fetch_add(&state[0], 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        else __hip_atomic_fetch_add(&state[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // bounded wait: every wave leaves this loop, a run that times out is reported, not hung
        unsigned spins = 0;
        while (true) {
          const unsigned seen = MODE == 2 ? __hip_atomic_load(&state[0], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT)
                                          : __hip_atomic_load(&state[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          if (seen >= target) break;
          if (++spins > spin_limit || __hip_atomic_load(&state[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) {
            __hip_atomic_store(&state[1], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            break;
          }
        }
      }
      __syncthreads();
    }
  }
}

__global__ void sync_clear_kernel(unsigned* state, int n) {
  if ((int)threadIdx.x < n) state[threadIdx.x] = 0u;
}

}  // namespace

extern "C" int pi0_sync_bench(int mode, int n_ops, int reps, float* d_x, const float* d_b, unsigned* d_state, double* h_ms,
                              void* hip_stream) {
  if (d_x == nullptr || d_b == nullptr || d_state == nullptr || h_ms == nullptr) return PI0_EINVAL;
  if (mode < PI0_SYNC_EAGER || mode > PI0_SYNC_FUSED || n_ops < 1 || n_ops > 100000 || reps < 1 || reps > 1000) return PI0_EINVAL;
  if ((reinterpret_cast<uintptr_t>(d_x) & 15) != 0 || (reinterpret_cast<uintptr_t>(d_b) & 15) != 0) return PI0_EINVAL;
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  float4* x = reinterpret_cast<float4*>(d_x);
  const float4* b = reinterpret_cast<const float4*>(d_b);
  const dim3 grid(ROWS * COLS / 4 / 256), block(256);     // 256 blocks
  if (mode == PI0_SYNC_BARRIER || mode == PI0_SYNC_BARRIER_FENCE) {
    // the barrier needs every block resident at once
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
      return PI0_EHIP;
    if (cus < (int)grid.x) return PI0_ESTATE;
  }
  hipEvent_t e0 = nullptr, e1 = nullptr;
  hipGraph_t graph = nullptr;
  hipGraphExec_t exec = nullptr;
  int rc = PI0_OK;
  hipError_t e = hipEventCreate(&e0);
  if (e == hipSuccess) e = hipEventCreate(&e1);
  if (e == hipSuccess && mode == PI0_SYNC_GRAPH) {
    if (s == nullptr) {
      rc = PI0_EINVAL;   // capture needs a real stream
    } else {
      e = hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal);
      if (e == hipSuccess) {
        for (int op = 0; op < n_ops; op++) sync_add_kernel<<<grid, block, 0, s>>>(x, b);
        hipError_t e2 = hipStreamEndCapture(s, &graph);
        e = hipGetLastError();
        if (e == hipSuccess) e = e2;
      }
      if (e == hipSuccess) e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
    }
  }
  const unsigned spin_limit = 1u << 22;
  if (e == hipSuccess && rc == PI0_OK) {
    sync_clear_kernel<<<1, 64, 0, s>>>(d_state, 2);
    e = hipEventRecord(e0, s);
    for (int r = 0; r < reps && e == hipSuccess; r++) {
      switch (mode) {
        case PI0_SYNC_EAGER:
          for (int op = 0; op < n_ops; op++) sync_add_kernel<<<grid, block, 0, s>>>(x, b);
          break;
        case PI0_SYNC_GRAPH:
          e = hipGraphLaunch(exec, s);
          break;
        case PI0_SYNC_BARRIER:
          sync_clear_kernel<<<1, 64, 0, s>>>(d_state, 1);   // the counter restarts, a raised error flag stays
          sync_loop_kernel<1><<<grid, block, 0, s>>>(x, b, n_ops, d_state, spin_limit);
          break;
        case PI0_SYNC_BARRIER_FENCE:
          sync_clear_kernel<<<1, 64, 0, s>>>(d_state, 1);
          sync_loop_kernel<2><<<grid, block, 0, s>>>(x, b, n_ops, d_state, spin_limit);
          break;
        default:
          sync_loop_kernel<0><<<grid, block, 0, s>>>(x, b, n_ops, d_state, spin_limit);
          break;
      }
      if (e == hipSuccess) e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipEventRecord(e1, s);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (e == hipSuccess) *h_ms = (double)ms / reps;
    unsigned flag = 0;
    if (e == hipSuccess) e = hipMemcpyAsync(&flag, d_state + 1, sizeof(flag), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e == hipSuccess && flag != 0u) rc = PI0_ESTATE;   // a bounded barrier wait ran out
  }
  if (exec) (void)hipGraphExecDestroy(exec);
  if (graph) (void)hipGraphDestroy(graph);
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (rc != PI0_OK) return rc;
  return e == hipSuccess ? PI0_OK : PI0_EHIP;
}
