/*
 * pi0_bench.h - measurement and tuning entry points of the pi0 library (same shared library as pi0.h).
 *
 * Nothing here is on the inference path: per-class timing of a pass, the synchronisation experiments of the
 * paper's Section 5.2 / Table 3, attainable-peak micro-benchmarks for the roofline of Section 5.1, a clock sample,
 * the read-ahead kernel alone, the launch count, and the per-shape kernel choices for tuning runs.
 * Conventions (pointers named d_* are device pointers, h_* host pointers; error codes) are those of pi0.h.
 */
#ifndef PI0_BENCH_H
#define PI0_BENCH_H

#include "pi0.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Operation classes of the pass, for per-class timing (the rows of Table 2 grouped by launch).
 */
enum pi0_op_class {
  PI0_OP_MISC = 0,        /* copies, patch extraction, embeddings, row statistics */
  PI0_OP_VIS_PATCH,       /* patch embedding GEMM */
  PI0_OP_VIS_QKV,         /* LayerNorm-folded QKV projection */
  PI0_OP_VIS_ATTN,
  PI0_OP_VIS_O,           /* split-K partial GEMM of the output projection */
  PI0_OP_VIS_UP,
  PI0_OP_VIS_DOWN,        /* split-K partial GEMM */
  PI0_OP_VIS_PROJ,        /* final LayerNorm + projector */
  PI0_OP_REDUCE,          /* split-K reductions (bias, residual, row statistics) of any stage */
  PI0_OP_LLM_QKV,         /* RMSNorm-folded QKV + RoPE, writes the key/value cache */
  PI0_OP_LLM_ATTN,
  PI0_OP_LLM_O,
  PI0_OP_LLM_GATEUP,
  PI0_OP_LLM_DOWN,
  PI0_OP_EXP_EMBED,       /* folded action/time embedding and its second linear layer */
  PI0_OP_EXP_QKV,
  PI0_OP_EXP_ATTN,
  PI0_OP_EXP_O,
  PI0_OP_EXP_GATEUP,
  PI0_OP_EXP_DOWN,
  PI0_OP_EXP_OUT,         /* final norm, output projection, Euler update */
  PI0_OP_CLASSES
};

/*
 * Timing run: `passes` complete passes (as pi0_infer) launched eagerly with a HIP event pair
 * around every kernel launch on hip_stream.  Synchronises the stream, then adds the elapsed
 * microseconds and the launch count of every class to the HOST arrays h_class_us[PI0_OP_CLASSES]
 * and h_class_launches[PI0_OP_CLASSES] (both are overwritten).  Eager launches: each elapsed time
 * is the kernel's duration as the stream's timestamps see it, without graph-launch effects.
 * Errors as pi0_infer; ENOMEM if events cannot be created.
 */
int pi0_debug_profile(pi0_ctx* ctx, const float* d_images, int n_views, const int32_t* d_prompt_ids,
                      int n_prompt, const float* d_state, const float* d_noise, float* d_actions,
                      int passes, double* h_class_us, int* h_class_launches, void* hip_stream);

/*
 * Synchronisation-overhead micro-benchmark (Section 5.2, Table 3 of the paper; no ctx needed).
 * Applies x <- x + b to a 256 x 1024 fp32 array n_ops times per repetition, `reps` repetitions,
 * one 256-thread block per row, with consecutive updates ordered by
 *   PI0_SYNC_EAGER          n_ops separate kernel launches
 *   PI0_SYNC_GRAPH          one hipGraph of n_ops kernel nodes (captured on hip_stream, which must not be NULL)
 *   PI0_SYNC_BARRIER        one kernel, software grid barrier with relaxed atomics between updates
 *   PI0_SYNC_BARRIER_FENCE  same with release / acquire at device scope (what dependent data would need)
 *   PI0_SYNC_FUSED          one kernel, no synchronisation (the baseline)
 * d_x, d_b: device, float32 [256][1024], 16-byte aligned; afterwards x = x0 + reps * n_ops * b exactly
 * (for values that are exact in fp32).  d_state: device, 2 x uint32 scratch (cleared by the call).
 * h_ms: HOST, receives the milliseconds of one repetition (HIP events on hip_stream, averaged over
 * reps).  The call synchronises the stream.  Barrier waits are bounded: if one runs out, or the
 * device has fewer compute units than blocks, the result is PI0_ESTATE.  Other errors: EINVAL, EHIP.
 */
enum pi0_sync_mode {
  PI0_SYNC_EAGER = 0,
  PI0_SYNC_GRAPH = 1,
  PI0_SYNC_BARRIER = 2,
  PI0_SYNC_BARRIER_FENCE = 3,
  PI0_SYNC_FUSED = 4
};
int pi0_sync_bench(int mode, int n_ops, int reps, float* d_x, const float* d_b, unsigned* d_state,
                   double* h_ms, void* hip_stream);

/*
 * Attainable-peak micro-benchmarks (no ctx needed): what this device sustains on the two resources
 * the roofline of Section 5.1 prices operations by.
 *   PI0_PEAK_HBM_READ   streams `bytes` bytes at d_buf (device, 16-byte aligned, bytes a multiple of
 *                       16; give far more than the 256 MB last-level cache) through all compute units
 *                       with 16-byte loads; *h_result = GB/s (1e9 bytes per second).  iters unused.
 *   PI0_PEAK_MFMA_BF16  runs `iters` (1 .. 2^22) rounds of 4 independent 32x32x16 bf16 MFMAs per wave,
 *                       2 waves per SIMD on 256 compute units' worth of blocks, operands and
 *                       accumulators in registers, non-zero operands; *h_result = TFLOP/s.
 *                       d_buf / bytes unused.
 *   PI0_PEAK_CACHE_READ 256 blocks of 512 threads (one per compute unit, the shape of the pass's own kernels); block b
 *                       reads the slice (b mod 8) of d_buf - `bytes` / 8 bytes each, so the blocks of one die share
 *                       a slice under round-robin dispatch - `iters` (1 .. 2^20) times with 16-byte loads, 8 in flight
 *                       per lane; *h_result = GB/s delivered to the compute units.  With slices that fit a die's L2
 *                       (4 MB) this is the rate of L2 hits, with larger ones that of the memory-side cache.
 *                       bytes: a multiple of 128, at least 65536.
 * One untimed launch, then `reps` (1 .. 1000) launches timed with HIP events on hip_stream; the call
 * synchronises the stream.  d_sink: device, one uint32 the kernels may write (never read back).
 * h_result: HOST.  Nothing is allocated on the device.  Errors: EINVAL, EHIP.
 */
enum pi0_peak_kind { PI0_PEAK_HBM_READ = 0, PI0_PEAK_MFMA_BF16 = 1, PI0_PEAK_CACHE_READ = 2 };
int pi0_peak_bench(int kind, const void* d_buf, size_t bytes, int iters, int reps, unsigned* d_sink,
                   double* h_result, void* hip_stream);

/*
 * Clock sample (no ctx needed): enqueues one single-lane kernel on hip_stream that writes d_out[0] = the shader
 * cycle counter and d_out[1] = the constant 100 MHz counter (d_out: device, 2 x int64, 8-byte aligned).  Two
 * samples around a piece of work on the same stream give the shader clock the device actually ran at:
 * (cycles_1 - cycles_0) / ((ticks_1 - ticks_0) * 10 ns) - the figure the published peaks (quoted at 2.4 GHz)
 * have to be scaled by.  The cycle counters of the chip's dies are not aligned with each other and the two sample
 * kernels may run on different dies, so the interval has to be long (>= 100 ms) for the offset not to matter.
 * Errors: EINVAL, EHIP.
 */
int pi0_clock_sample(long long* d_out, void* hip_stream);

/*
 * The read-ahead kernel that pi0_denoise runs beside the expert's compute launches (Section 5.2: prefetch across
 * synchronisation points), alone on hip_stream, over a caller's buffer (no ctx needed).  The buffer is cut into
 * `layers` equal slices; the kernel reads slice i % layers for i = 0 .. steps * layers - 1, each once the int32
 * counter *d_progress is >= i + 1 - lead (lead >= 1; nothing in this call ever writes the counter: whoever
 * sets it - the caller beforehand, or a kernel on another stream - sets the pace), and skips slice i when the
 * counter is already >= i + 2 (too late to be of use).  lead >= steps * layers reads everything without waiting;
 * a counter far ahead makes the kernel skip everything.  A block that waits longer than
 * wait_ticks (100 MHz wall-clock ticks) for the counter gives up and exits, which is what keeps the kernel from
 * hanging when its partner stream does not run: with a counter that never moves the call returns after about one
 * bound.  The loads change nothing anywhere.
 *   d_buf      device, 16-byte aligned, bytes a multiple of layers * 16, a slice below 2 GiB
 *   d_progress device int32      d_sink device, 1024 x uint32 (never written in practice)
 *   blocks     1 .. 1024 blocks of 256 threads      h_ms  HOST, elapsed milliseconds (the call synchronises)
 * Errors: EINVAL, EHIP.
 */
int pi0_read_ahead_probe(const void* d_buf, size_t bytes, int layers, int steps, int lead, const int* d_progress,
                         long long wait_ticks, int blocks, unsigned* d_sink, double* h_ms, void* hip_stream);

/* Number of kernel launches one pi0_infer issues on hip_stream for the given shape (0 on bad
 * arguments); the read-ahead kernel on the ctx's own stream is not counted. */
int pi0_kernel_count(const pi0_ctx* ctx, int n_views, int n_prompt);

/*
 * Grid synchronisation WITH a data dependency between blocks (Section 5.2 of the paper: software barriers inside
 * one persistent kernel; no ctx needed).  Table 3's update only touches a thread's own elements; here update k is
 *     x_{k+1}[r][c] = max_{j = 1 .. fan} x_k[(r + j) mod 256][c] + b[r][c]      (256 x 1024 fp32, block r owns row r)
 * so every block reads `fan` rows (4 KiB each) that other blocks wrote in the update before, and the result - exact
 * in fp32 - shows whether the chosen barrier and data path really made them visible across the chip's dies.
 *   barrier  PI0_BARRIER_COUNTER  one arrival counter (read-modify-write + poll of the same word)
 *            PI0_BARRIER_XCD      two levels: a counter per group of blocks (block index mod 8), a root counter, the
 *                                 epoch published in one word per group and polled with back-off
 *            PI0_BARRIER_FLAGS    block i stores the epoch in word i; one wave per block polls all 256 words with
 *                                 one 16-byte load per lane; no read-modify-write
 *            PI0_BARRIER_FLAGS8   the same with 8 copies of the flag array 4 KiB apart: a block stores into all of
 *                                 them and polls copy (block index mod 8) only
 *            PI0_BARRIER_GROUPADD one add without return value per block on its group's counter; everyone polls
 *                                 the 8 group counters
 *            PI0_BARRIER_XCC      as XCD with the real dies as groups (hardware die id): arrivals counted in the
 *                                 die's own L2, one device-scope release per die instead of one per block
 *   data     PI0_SYNCDATA_NONE    no dependency: x[r] += b[r] in place (fan, planes ignored beyond validation)
 *            PI0_SYNCDATA_BYPASS  write-through stores, loads that bypass the L2 (device-scope instruction bits)
 *            PI0_SYNCDATA_INV     write-through stores, one cache invalidate per block after the wait, cached loads
 *            PI0_SYNCDATA_FENCE   ordinary stores / loads with device-scope release / acquire fences
 *            PI0_SYNCDATA_FRESH   write-through stores, cached loads, a never-read plane per update
 *                                 (needs planes >= n_ops + 1 and reps == 1)
 *            PI0_SYNCDATA_WBACK   ordinary stores, loads that bypass the L2
 *            (every dependent path releases at device scope between a block's stores and its arrival: without it
 *            an arrival was observed to overtake the write-through data it announces)
 *   d_x      device, float32 [planes][256][1024], 16-byte aligned; update k reads plane k mod planes and writes
 *            plane (k + 1) mod planes, k counting on across repetitions (data NONE uses plane 0 only).  planes >= 2
 *            for the dependent data paths, at most 4096.
 *   d_b      device, float32 [256][1024].   d_state  device, 9216 x uint32 scratch, 16-byte aligned (cleared by the call).
 *   h_ms     HOST, milliseconds of one repetition of n_ops updates (HIP events on hip_stream; the call synchronises).
 * Every wait is bounded; PI0_ESTATE if one ran out or the device has fewer than 256 compute units.  Other
 * errors: EINVAL, EHIP.
 */
enum pi0_barrier_kind {
  PI0_BARRIER_COUNTER = 0,
  PI0_BARRIER_XCD = 1,
  PI0_BARRIER_FLAGS = 2,
  PI0_BARRIER_FLAGS8 = 3,
  PI0_BARRIER_GROUPADD = 4,
  PI0_BARRIER_XCC = 5
};
enum pi0_syncdata_kind {
  PI0_SYNCDATA_NONE = 0,
  PI0_SYNCDATA_BYPASS = 1,
  PI0_SYNCDATA_INV = 2,
  PI0_SYNCDATA_FENCE = 3,
  PI0_SYNCDATA_FRESH = 4,
  PI0_SYNCDATA_WBACK = 5
};
int pi0_sync_dep_bench(int barrier, int data, int fan, int n_ops, int reps, float* d_x, int planes, const float* d_b,
                       unsigned* d_state, double* h_ms, void* hip_stream);

/*
 * Timeline of the persistent denoise kernel (Section 5.2: where the time between two software barriers goes).
 * With a buffer set, thread 0 of every block notes the 100 MHz wall clock per operation of the loop: [0] operation
 * entered (its constant operands are requested next), [1] inputs complete (the wait for the barrier of the operation
 * before is over; 0 if the block has no work item in this operation), [2] body done, [3] arrival announced, [4..7]
 * points inside the body (0 where a body has none): GEMMs - products done, partial tiles in shared memory;
 * attention - Q in shared memory, scores done, probabilities in shared memory, P V done.
 *   d_trace  device, int64 [ops_cap][256 blocks][8], 8-byte aligned; NULL with ops_cap 0 switches the timeline off
 *   operations are numbered in execution order: 0 = state token; per Euler step: embed, second linear, per layer
 *   QKV, attention, O, gate||up, down; then out-projection + Euler.  pi0_loop_trace_ops gives their number.
 * Drops every captured graph.  Must not be called while work of this ctx is in flight.  Errors: EINVAL.
 */
int pi0_loop_trace_ops(const pi0_ctx* ctx);
int pi0_set_loop_trace(pi0_ctx* ctx, long long* d_trace, int ops_cap);

/*
 * Per-shape kernel choices for tuning runs (Section 4.1 of the paper tunes tiles per GEMM shape): `spec` is a
 * comma-separated list of key=value pairs, e.g. "lgu=7,zld=16,ras=0"; unknown keys and values outside a key's
 * range are ignored.  Keys: tile ids (vis, vqkv, vup, lqkv, lgu, vo, vd, lo, ld), split counts (zvo, zvd, zlo,
 * zld), the expert's read-ahead kernel (ras blocks, 0 = off; rat threads; rad loads in flight; ral layers ahead),
 * warm-up block counts (pfq, pfa, pfo, pfd), switches (ae16, qms, ksplit, kcps, avs, fko, fkl), pdn (1: the denoise loop as
 * one persistent kernel, 0: one launch per operation) and pra (what the persistent kernel's blocks without a work item read
 * ahead: 1 gate||up, 2 down, 4 next layer's QKV, 8 next layer's O weights during the attention; 16 this layer's O weights,
 * 32 this layer's prefix keys / values during QKV) and psb (blocks of the persistent kernel inside a two-stream frame;
 * 0: per-operation launches there, -1: chosen from the prefix size).
 * Drops every captured graph, so the next call of a shape captures again.  Must not be called while work of this
 * ctx is in flight.  The library itself never reads the environment.  Errors: EINVAL (null).
 */
int pi0_tune(pi0_ctx* ctx, const char* spec);

/* Attention kernels on operands in natural order (Table 2: the attention rows of the vision encoder, the prefix and
 * the action expert).  A test entry: it allocates and frees staging buffers and synchronises the stream.
 * All pointers are device memory, fp32; values are rounded to bf16 on entry.
 *   d_q  [heads][Tq][head_dim]        d_k0, d_v0 [kv_heads][n0][head_dim]      d_k1, d_v1 [1][n1][head_dim] or NULL
 *   d_out [shares][Tq][heads * head_dim]            d_ml [shares][heads][ceil32(Tq)][2] (only written if shares > 1)
 * kv_heads is heads or 1 (shared head); head_dim is 256 or 68 .. 80; n1 is 0 or 64 (needs kv_heads == 1, head_dim
 * 256).  view_tokens > 0: query row m sees the keys of its own view only (needs n0 == Tq).  suffix_mask = 1: row 0
 * sees all of segment 0 and key 0 of segment 1, the other rows see everything.  chunks_per_share > 0 and
 * ceil(n0 / 32) > chunks_per_share: the keys of segment 0 are shared out over shares = ceil(ceil(n0 / 32) /
 * chunks_per_share) blocks (segment 1 goes with the last); share z returns its own normalised output and, in d_ml,
 * (row maximum of the scaled logits, sum of exponentials relative to it), which the consumer merges as
 * sum_z c_z out_z, c_z = l_z exp(m_z - max m) / sum.  v_split: 0, or 2 / 4 / 8 blocks per (query tile, head) with a
 * part of the value slices each (head_dim 256).  Unsupported combinations return PI0_EINVAL. */
int pi0_attention_probe(int heads, int kv_heads, int head_dim, int Tq, int n0, int n1, int view_tokens,
                        int suffix_mask, int chunks_per_share, int v_split, float scale, const float* d_q,
                        const float* d_k0, const float* d_v0, const float* d_k1, const float* d_v1, float* d_out,
                        float* d_ml, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* PI0_BENCH_H */
