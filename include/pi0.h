/*
 * pi0.h - C ABI of the MI355X (gfx950) pi0 forward-pass library.
 *
 * One complete low-latency pi0 inference at batch 1 (paper Section 2): a SigLIP ViT over 1-3
 * camera views, a Gemma-style prefix transformer that fills a per-layer key/value cache, and an
 * action expert that integrates a flow with `steps` Euler steps against that cache and returns a
 * chunk of `chunk` actions.  The sequence of GEMMs and fused scalar ops is the one listed in the
 * paper's Table 2; the algebraic rewrites of Section 3.2 (norm gains folded out of the norm - here
 * into the bf16 cast of the activations that the next linear reads -, action/time encoder
 * folded, fused QKV with RoPE in the epilogue), Section 4.1 (last
 * prefix layer only produces keys/values), Section 4.2 (fused gated MLP) and Section 4.4 (norm
 * statistics applied after accumulation) are done inside the library at load time / in kernels.
 * Section 3.1's graph replay: pi0_prefill / pi0_denoise / pi0_infer record their kernel
 * sequence into a HIP graph on first use of a shape and replay it afterwards.
 *
 * Conventions
 *  - Every pointer named d_* is a DEVICE pointer (HIP global memory), row-major, contiguous.
 *    The caller owns all device memory: weight blob, workspace, inputs, outputs, and the stream.
 *    The library allocates no device memory; it owns only the host-side pi0_ctx.
 *  - Every call only enqueues work on `hip_stream` (a hipStream_t, may be NULL for the default
 *    stream); results are valid after the caller synchronises that stream.  One exception that the
 *    caller never sees: pi0_denoise / pi0_infer fork one read-ahead kernel (it only loads the
 *    expert's weights ahead of the compute launches, Section 5.2) onto a stream the ctx owns and
 *    join it back into `hip_stream` before the call's last launch, with events, also inside the
 *    captured graph; work enqueued on `hip_stream` after the call is ordered after both.
 *  - Return value: 0 on success, a negative PI0_E* code otherwise.  Argument checks happen before
 *    any GPU call, so error paths touch no GPU state.  Nothing throws or aborts across the ABI.
 *  - Calls on one ctx must not overlap in time (one workspace, one set of activations); the only
 *    concurrency is the one pi0_stream_frame arranges itself between its two streams.
 */
#ifndef PI0_H
#define PI0_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pi0_ctx pi0_ctx; /* opaque, host memory, owned by the library */

/* Model geometry.  Plain data, copied by pi0_create.  Values in comments are the full model. */
typedef struct pi0_config {
  int32_t vis_layers;  /* 27   SigLIP blocks                                              */
  int32_t vis_width;   /* 1152 must be a multiple of 64                                   */
  int32_t vis_heads;   /* 16   head dim = vis_width / vis_heads (72), multiple of 4, <= 80 */
  int32_t vis_mlp;     /* 4304                                                            */
  int32_t img_size;    /* 224                                                             */
  int32_t patch;       /* 14   tokens per view = (img_size/patch)^2 (256), multiple of 32 */
  int32_t llm_layers;  /* 18                                                              */
  int32_t llm_width;   /* 2048                                                            */
  int32_t llm_q_heads; /* 8    query heads sharing one key/value head                     */
  int32_t head_dim;    /* 256  (prefix and expert); must be 256                           */
  int32_t llm_mlp;     /* 16384                                                           */
  int32_t exp_layers;  /* 18   must equal llm_layers                                      */
  int32_t exp_width;   /* 1024                                                            */
  int32_t exp_mlp;     /* 4096                                                            */
  int32_t state_dim;   /* 32   must be <= 32                                              */
  int32_t action_dim;  /* 32   must be <= 32                                              */
  int32_t chunk;       /* 63   chunk + 1 suffix tokens (state + actions) must be 64       */
  int32_t steps;       /* 10   Euler steps, t = 1 - k/steps, dt = -1/steps                */
  int32_t vocab;       /* rows of the prompt embedding table in the blob; 0 = no table    */
  int32_t max_views;   /* 3                                                               */
  int32_t max_prompt;  /* 48   (0 allowed)                                                */
} pi0_config;

enum {
  PI0_OK = 0,
  PI0_EINVAL = -1,  /* null pointer, bad shape or count                                  */
  PI0_ESTATE = -2,  /* weights not loaded, or denoise without a valid prefill            */
  PI0_ENOMEM = -3,  /* workspace too small / host allocation failed                      */
  PI0_EFORMAT = -4, /* weight blob has the wrong size for this config                    */
  PI0_EHIP = -5     /* a HIP runtime call failed; see pi0_last_hip_error                 */
};

/* Validates the geometry and creates a context.  *out is set only on success. */
int pi0_create(const pi0_config* cfg, pi0_ctx** out);
/* Destroys graphs and the context.  NULL is a no-op.  Does not touch caller-owned memory. */
void pi0_destroy(pi0_ctx* ctx);

/*
 * Size in bytes of the canonical weight blob for `cfg` (0 if cfg is invalid).
 * Blob format: bfloat16, little endian; tensors stored "x @ W" style as [in][out] row-major, in
 * this order, each starting at a multiple of 128 elements (gaps are ignored):
 *   vis.patch.w [patch*patch*3][Dv] (patch vector order dy,dx,channel), vis.patch.b [Dv],
 *   vis.pos [T][Dv];
 *   per vision layer: ln1.g ln1.b, wq bq wk bk wv bv ([Dv][Dv] / [Dv]), wo bo, ln2.g ln2.b,
 *     w1 [Dv][Fv] b1, w2 [Fv][Dv] b2;
 *   vis.lnf.g vis.lnf.b, vis.proj.w [Dv][E], vis.proj.b [E];
 *   llm.embed [vocab][E] (only if vocab > 0);
 *   per prefix layer: g_attn [E], wq [E][H*256], wk [E][256], wv [E][256], wo [H*256][E],
 *     g_mlp [E], wg [E][F], wu [E][F], wd [F][E];
 *   per expert layer: the same with width X and MLP Fx;
 *   exp.state.w [state_dim][X] b, exp.action_in.w [action_dim][X] b, exp.time_in.w [2X][X] b
 *     (rows 0..X-1 act on the action embedding, rows X..2X-1 on the time encoding),
 *   exp.time_out.w [X][X] b, exp.g_final [X], exp.out.w [X][action_dim] b.
 * LayerNorm gains are stored directly; RMSNorm gains g are applied as (1 + g).
 */
size_t pi0_weights_bytes(const pi0_config* cfg);

/* Bytes of caller-provided device workspace needed: packed bf16 weights (and, if llm_width and llm_mlp are
 * multiples of 256, an MXFP8 copy of the prefix feed-forward weights, about 1.03 bytes per weight), tables, both
 * copies of the key/value cache, activations, split-K partial sums.  0 if cfg is invalid. */
size_t pi0_workspace_bytes(const pi0_config* cfg);

/*
 * Packs the canonical blob into the workspace (Section 3.2 folds, MFMA fragment order, zero
 * padding) and zero-fills the activation area.  d_blob may be freed once the stream has been
 * synchronised; d_workspace must stay alive and untouched by the caller until pi0_destroy.
 * d_workspace must be 256-byte aligned.  Errors: EINVAL (null / misaligned), EFORMAT
 * (blob_bytes != pi0_weights_bytes), ENOMEM (ws_bytes too small), EHIP.
 */
int pi0_load_weights(pi0_ctx* ctx, const void* d_blob, size_t blob_bytes, void* d_workspace,
                     size_t ws_bytes, void* hip_stream);

/*
 * Table 2 rows of the vision encoder and the LLM: encodes the views, appends the prompt
 * embeddings, runs the prefix transformer and leaves its keys/values in the workspace.
 *   d_images     float32 [n_views][img_size][img_size][3], values nominally in [-1, 1]
 *   n_views      1..max_views
 *   d_prompt_ids int32 [n_prompt], each in [0, vocab); may be NULL iff n_prompt == 0
 *   n_prompt     0..max_prompt; > 0 requires vocab > 0
 * Errors: EINVAL, ESTATE (weights not loaded), EHIP.
 */
int pi0_prefill(pi0_ctx* ctx, const float* d_images, int n_views, const int32_t* d_prompt_ids,
                int n_prompt, void* hip_stream);

/*
 * Table 2 rows of the action expert, `steps` times: Euler integration of the flow from the
 * given noise against the cached prefix.  May be called repeatedly after one pi0_prefill
 * (streaming use: fresh state/noise on the same cache).
 *   d_state   float32 [state_dim]
 *   d_noise   float32 [chunk][action_dim]
 *   d_actions float32 [chunk][action_dim] (output; may alias d_noise)
 * Errors: EINVAL, ESTATE (no valid prefill), EHIP.
 */
int pi0_denoise(pi0_ctx* ctx, const float* d_state, const float* d_noise, float* d_actions,
                void* hip_stream);

/* pi0_prefill followed by pi0_denoise as one graph launch. */
int pi0_infer(pi0_ctx* ctx, const float* d_images, int n_views, const int32_t* d_prompt_ids,
              int n_prompt, const float* d_state, const float* d_noise, float* d_actions,
              void* hip_stream);

/*
 * One frame of the two-stream mode of Section 6 (concurrent prefix and expert): enqueues, on
 * stream_prefill, the prefill of THIS frame's images into the second copy of the key/value cache
 * and, on stream_denoise, the denoise of d_state / d_noise against the cache that the PREVIOUS
 * prefill (pi0_prefill, pi0_infer or the previous pi0_stream_frame) filled; the two run
 * concurrently on the GPU.  d_actions therefore belongs to the previous frame's images, exactly as
 * pi0_denoise after that prefill would compute them (same kernels, bit-identical).  After the call
 * the cache filled by this frame is the current one.  Ordering between successive frames is kept
 * with events owned by ctx: use the same two (distinct, non-NULL) streams for every frame, and
 * enqueue the priming prefill on stream_prefill.  The results are valid once both streams are
 * synchronised.  Errors as pi0_infer; ESTATE if there is no valid prefill to denoise against.
 */
int pi0_stream_frame(pi0_ctx* ctx, const float* d_images, int n_views, const int32_t* d_prompt_ids,
                     int n_prompt, const float* d_state, const float* d_noise, float* d_actions,
                     void* stream_prefill, void* stream_denoise);

/*
 * Debug run for parity checks: the same kernels launched eagerly (no graph), copying
 * intermediate results into d_taps (float32) after each layer.  Tap layout, in order:
 *   vision residual stream after each vision layer      vis_layers x [I][Dv]
 *   projector output (prefix image embeddings)          [I][E]
 *   prefix residual stream after layers 0..L-2          (llm_layers-1) x [P][E]
 *   key cache, value cache (natural order)              2 x llm_layers x [P][256]
 *   expert residual stream after each layer, step 0     exp_layers x [64][X]
 *   expert residual stream after each layer, last step  exp_layers x [64][X]
 *   x after each Euler step                             steps x [chunk][action_dim]
 * with I = n_views * tokens per view and P = I + n_prompt.  pi0_debug_taps_elems gives the
 * total element count.  Also writes d_actions.  Errors as pi0_infer, plus ENOMEM if cap_elems is
 * too small.
 */
size_t pi0_debug_taps_elems(const pi0_config* cfg, int n_views, int n_prompt);
int pi0_debug_forward(pi0_ctx* ctx, const float* d_images, int n_views, const int32_t* d_prompt_ids,
                      int n_prompt, const float* d_state, const float* d_noise, float* d_actions,
                      float* d_taps, size_t cap_elems, void* hip_stream);

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
 * One untimed launch, then `reps` (1 .. 1000) launches timed with HIP events on hip_stream; the call
 * synchronises the stream.  d_sink: device, one uint32 the kernels may write (never read back).
 * h_result: HOST.  Nothing is allocated on the device.  Errors: EINVAL, EHIP.
 */
enum pi0_peak_kind { PI0_PEAK_HBM_READ = 0, PI0_PEAK_MFMA_BF16 = 1 };
int pi0_peak_bench(int kind, const void* d_buf, size_t bytes, int iters, int reps, unsigned* d_sink,
                   double* h_result, void* hip_stream);

/*
 * Arithmetic of the prefix transformer's feed-forward GEMMs (gate||up and down; everything else stays bf16).
 * The paper runs everything in bf16 and names 8-bit multiplication as a direction (Section 9.1); the
 * reduced-precision mode is this library's reading of it and changes the numerics contract:
 *   PI0_PRECISION_BF16 (default)        bf16 operands, fp32 accumulation
 *   PI0_PRECISION_MXFP8_PREFIX_MLP      OCP MXFP8 operands (FP8 E4M3 elements, one power-of-two E8M0 scale per 32
 *                                       consecutive elements of the contraction axis), fp32 accumulation, block
 *                                       scales applied by the MFMA.  Quantised: the weights (at load time, both
 *                                       copies are kept), the gain-scaled input x * (1 + g) of gate||up (1 / rms is
 *                                       applied to the products), and gelu(gate) * up before the down projection.
 * Takes effect from the next pi0_prefill / pi0_infer / pi0_stream_frame; may be changed at any time between calls
 * (graphs are kept per mode).  EINVAL for an unknown mode, or if llm_width / llm_mlp are not multiples of 256.
 */
enum pi0_precision { PI0_PRECISION_BF16 = 0, PI0_PRECISION_MXFP8_PREFIX_MLP = 1 };
int pi0_set_precision(pi0_ctx* ctx, int precision);

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

/* Graph replay on (1, default) or off (0: every call launches kernels eagerly). */
int pi0_set_graph_mode(pi0_ctx* ctx, int enabled);

/* Number of kernel launches one pi0_infer issues on hip_stream for the given shape (0 on bad
 * arguments); the read-ahead kernel on the ctx's own stream is not counted. */
int pi0_kernel_count(const pi0_ctx* ctx, int n_views, int n_prompt);

/* Static, never-NULL description of an error code. */
const char* pi0_strerror(int code);
/* hipError_t value of the last failed HIP call on this ctx (0 if none). */
int pi0_last_hip_error(const pi0_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* PI0_H */
