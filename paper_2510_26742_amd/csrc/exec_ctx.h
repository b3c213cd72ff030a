// Execution contexts of the action expert's kernel bodies.
//
// Every operation of the expert (Table 2, rows of the action expert) is written once as a device
// function ("body") templated on a context that answers three questions:
//   - which work item am I?                       cx.bx / cx.by / cx.bz  (blockIdx of a per-operation launch)
//   - how do I read what OTHER blocks produced in the operation before, and how do I publish what I produce?
//                                                  cx.ld(ptr) / cx.st(ptr, v)
//   - when may I start reading it?                 cx.wait_inputs()
// LaunchCtx is the per-operation launch (one graph node per operation, Section 3.1 of the paper): the kernel
// boundary orders and publishes everything, loads and stores are ordinary, the wait is empty.
// PersistCtx is one persistent kernel for the whole denoise loop (Section 5.2: software barriers instead of
// kernel boundaries, weights requested before the wait).  The chip has eight dies with an L2 each that
// ordinary accesses do not keep coherent inside a kernel, so data that crosses blocks is stored write-through
// and loaded past the L2 (device-scope bits of the buffer instructions), and a barrier releases a die's
// writes once per die; see grid barrier below.  Weights, tables and the prefix key/value cache are constant
// during the kernel and are read with ordinary loads before the wait.
// Both contexts run the same arithmetic in the same order, so the two paths agree bit for bit.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned u32x2_t __attribute__((ext_vector_type(2)));

struct LaunchCtx {
  static constexpr bool kPersistent = false;
  int bx, by, bz;
  __device__ __forceinline__ static LaunchCtx from_block_idx() { return LaunchCtx{(int)blockIdx.x, (int)blockIdx.y, (int)blockIdx.z}; }
  template <class T>
  __device__ __forceinline__ T ld(const T* p) const { return *p; }
  template <class T>
  __device__ __forceinline__ T ld_bulk(const T* p) const { return *p; }
  template <class T>
  __device__ __forceinline__ void st(T* p, const T& v) const { *p = v; }
  __device__ __forceinline__ void wait_inputs() const {}
  __device__ __forceinline__ void mark(int) const {}
  __device__ __forceinline__ int tid() const { return (int)threadIdx.x; }
};

// ------------------------------------------------------------------------------------------------
// Grid barrier of the persistent kernel.  Arrivals are counted per die (hardware register XCC_ID names
// the die a wave runs on); the block that completes a die's count performs ONE device-scope release for
// the whole die (cache write-back, which also waits for the write-through stores in flight) and then tells
// every die, in a word of that die's own cache line, that this die has completed the epoch; a block polls
// its die's line (one 32-byte load) until all dies that hold blocks have.  One read-modify-write and one
// store-to-poll hop per barrier; a root counter between the two cost a second read-modify-write round trip.  Arrive and wait are separate calls, so a block requests the next operation's constant
// operands between them.  Every wait is bounded: when the bound runs out the error word is raised, every
// later wait returns at once, and the host reports the failure.
// Words (unsigned, 128 bytes apart so that no two are in one cache line):
enum {
  GB_ERR = 0,          // != 0: a bounded wait ran out
  GB_START = 32,       // start-up counter: blocks registered
  GB_MEMBERS = 64,     // + 32 x: blocks resident on die x
  GB_COUNT = 320,      // + 32 x: arrivals on die x (monotonic)
  GB_DONE = 576,       // + 32 y + x: last epoch that die x completed, as told to die y (one cache line per reading die)
  GB_SINK = 832,       // never read: where a read-ahead block would store its folded loads (keeps the loads alive)
  GB_WORDS = 864
};

struct GridBarrier {
  unsigned* w;          // GB_WORDS words, zeroed before the launch
  unsigned xcc;         // die of this block
  unsigned members;     // blocks on this die
  unsigned present;     // bit x set: die x holds at least one block
  unsigned spin_limit;
  unsigned epoch;       // barriers this block has arrived at
  unsigned waited;      // last barrier this block has seen completed
  long long* trace;     // optional: where thread 0 notes the wall clock (100 MHz) when a wait ends

  __device__ __forceinline__ static unsigned ld_dev(const unsigned* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
  __device__ __forceinline__ static void st_dev(unsigned* p, unsigned v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

  // all threads of the block; one counter barrier, after which every block knows who shares its die
  __device__ __forceinline__ void init(unsigned* words, unsigned limit) {
    w = words;
    spin_limit = limit;
    epoch = 0;
    waited = 0;
    trace = nullptr;
    xcc = (unsigned)__builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) & 7u;   // XCC_ID, bits 3:0
    if (threadIdx.x == 0) {
      __hip_atomic_fetch_add(&w[GB_MEMBERS + 32 * xcc], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_fetch_add(&w[GB_START], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      unsigned spins = 0;
      while (ld_dev(&w[GB_START]) < gridDim.x) {
        __builtin_amdgcn_s_sleep(2);
        if (++spins > spin_limit || ld_dev(&w[GB_ERR]) != 0u) { st_dev(&w[GB_ERR], 1u); break; }
      }
    }
    __syncthreads();
    members = ld_dev(&w[GB_MEMBERS + 32 * xcc]);
    present = 0;
    for (unsigned k = 0; k < 8u; k++) present |= ld_dev(&w[GB_MEMBERS + 32 * k]) != 0u ? 1u << k : 0u;
  }

  // all threads of the block, after the block's last store of the operation
  __device__ __forceinline__ void arrive() {
    // A block with no work item in an operation does not wait for that operation's inputs; it must still see the
    // barrier before completed, or its two arrivals in a row would be counted towards one barrier of its die.
    if (waited != epoch) wait();
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's stores have been acknowledged (a workgroup-scope
                                                        // fence does not wait for them)
    __syncthreads();
    epoch++;
    if (threadIdx.x == 0) {
      const unsigned old = __hip_atomic_fetch_add(&w[GB_COUNT + 32 * xcc], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (old + 1u == epoch * members) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");   // the die's writes are in memory
        for (unsigned k = 0; k < 8u; k++) st_dev(&w[GB_DONE + 32 * k + xcc], epoch);
      }
    }
  }

  // all threads of the block: returns once every block has arrived at the barrier this block arrived at last
  __device__ __forceinline__ void wait() {
    if (threadIdx.x < 8) {   // lane x reads what die x has told this die
      const unsigned lane = threadIdx.x;
      const bool counts = ((present >> lane) & 1u) != 0u;
      unsigned spins = 0;
      while (true) {
        const bool behind = counts && ld_dev(&w[GB_DONE + 32 * xcc + lane]) < epoch;
        if (__builtin_amdgcn_ballot_w64(behind) == 0ull) break;
        __builtin_amdgcn_s_sleep(1);
        if (++spins > spin_limit || ld_dev(&w[GB_ERR]) != 0u) {
          if (lane == 0) st_dev(&w[GB_ERR], 1u);
          break;
        }
      }
    }
    __syncthreads();
    waited = epoch;
    if (trace != nullptr && threadIdx.x == 0) *trace = (long long)wall_clock64();
  }
};

// cache-policy bit of gfx950 buffer instructions: device scope (stores write through to memory, loads do
// not hit in the die's L2 or the compute unit's L1)
#define PI0_AUX_DEVICE_SCOPE 16

// BULK_CACHED: the operation's large inputs (activation matrices, statistic partials, attention operands) are read
// with ordinary cached loads, so that the 32 blocks of a die fetch them from memory once instead of 32 times (read
// past the L2 by every block, an operation's inputs cross the fabric 256 times: measured 2 - 3.5 us per operation).
// That is only coherent if no cache of the reading die can hold an older copy of those addresses, which the caller
// guarantees by giving every operation instance of the loop its own never-read buffers whose cache lines are each
// written by one block only ("fresh" data path of the barrier experiment).
template <bool BULK_CACHED>
struct PersistCtxT {
  static constexpr bool kPersistent = true;
  int bx, by, bz;                  // work item of the current operation
  __amdgpu_buffer_rsrc_t arena;    // buffer resource over the activation arena
  const char* arena_base;
  GridBarrier* bar;
  int thread;                      // threadIdx.x, made opaque per operation: per-lane address arithmetic of one operation
                                   // is then not hoisted out of the layer loop, where it would hold registers throughout

  __device__ __forceinline__ int tid() const { return thread; }
  __device__ __forceinline__ unsigned off(const void* p) const { return (unsigned)(reinterpret_cast<const char*>(p) - arena_base); }

  template <class T>
  __device__ __forceinline__ T ld(const T* p) const {
    static_assert(sizeof(T) == 16 || sizeof(T) == 8 || sizeof(T) == 4 || sizeof(T) == 2, "access size");
    if constexpr (sizeof(T) == 16) return __builtin_bit_cast(T, __builtin_amdgcn_raw_buffer_load_b128(arena, off(p), 0, PI0_AUX_DEVICE_SCOPE));
    else if constexpr (sizeof(T) == 8) return __builtin_bit_cast(T, __builtin_amdgcn_raw_buffer_load_b64(arena, off(p), 0, PI0_AUX_DEVICE_SCOPE));
    else if constexpr (sizeof(T) == 4) return __builtin_bit_cast(T, __builtin_amdgcn_raw_buffer_load_b32(arena, off(p), 0, PI0_AUX_DEVICE_SCOPE));
    else return __builtin_bit_cast(T, __builtin_amdgcn_raw_buffer_load_b16(arena, off(p), 0, PI0_AUX_DEVICE_SCOPE));
  }
  template <class T>
  __device__ __forceinline__ void st(T* p, const T& v) const {
    static_assert(sizeof(T) == 16 || sizeof(T) == 8 || sizeof(T) == 4 || sizeof(T) == 2, "access size");
    if constexpr (sizeof(T) == 16) __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4_t, v), arena, off(p), 0, PI0_AUX_DEVICE_SCOPE);
    else if constexpr (sizeof(T) == 8) __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2_t, v), arena, off(p), 0, PI0_AUX_DEVICE_SCOPE);
    else if constexpr (sizeof(T) == 4) __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), arena, off(p), 0, PI0_AUX_DEVICE_SCOPE);
    else __builtin_amdgcn_raw_buffer_store_b16(__builtin_bit_cast(unsigned short, v), arena, off(p), 0, PI0_AUX_DEVICE_SCOPE);
  }
  template <class T>
  __device__ __forceinline__ T ld_bulk(const T* p) const {
    if constexpr (BULK_CACHED) return *p;
    else return ld(p);
  }
  __device__ __forceinline__ void wait_inputs() const { bar->wait(); }
  // timeline sample k (1 .. 4) of the current operation, by thread 0, when a timeline is being recorded
  __device__ __forceinline__ void mark(int k) const {
    if (bar->trace != nullptr && thread == 0) bar->trace[2 + k] = (long long)wall_clock64();
  }
  template <bool B>
  __device__ __forceinline__ PersistCtxT<B> as() const {
    PersistCtxT<B> c;
    c.bx = bx; c.by = by; c.bz = bz; c.arena = arena; c.arena_base = arena_base; c.bar = bar; c.thread = thread;
    return c;
  }
};
using PersistCtx = PersistCtxT<false>;
