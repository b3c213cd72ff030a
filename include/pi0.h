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
 *    stream); results are valid after the caller synchronises that stream.  pi0_denoise / pi0_infer
 *    run the expert's loop as one persistent kernel of 256 blocks that must all be resident at once:
 *    on a device with fewer than 256 compute units, or when the shape is outside what that kernel
 *    covers, the loop is issued as one launch per operation instead, together with one read-ahead
 *    kernel (it only loads the expert's weights ahead of the compute launches, Section 5.2) forked onto
 *    a stream the ctx owns and joined back into `hip_stream` before the call's last launch, with events,
 *    also inside the captured graph; work enqueued on `hip_stream` after the call is ordered after both.
 *    Do not run other kernels that occupy whole compute units for long beside pi0_denoise / pi0_infer:
 *    the persistent kernel's blocks wait for each other (bounded, see pi0_device_status).
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
  int32_t vis_heads;   /* 16   head dim = vis_width / vis_heads (72), multiple of 4, 68 .. 80 */
  int32_t vis_mlp;     /* 4304                                                            */
  int32_t img_size;    /* 224                                                             */
  int32_t patch;       /* 14   tokens per view = (img_size/patch)^2 (256), multiple of 32, <= 256 */
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
  int32_t max_views;   /* 3    1 .. 8                                                     */
  int32_t max_prompt;  /* 48   (0 allowed); max_views * tokens per view + max_prompt <= 1024 */
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

/*
 * pi0_denoise for callers that cannot allocate or hand over device memory at call time beyond inputs and outputs
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same kernels, launched
 * one per operation directly on hip_stream - no graph is built or replayed, no stream or event is created, no
 * device or host memory is allocated - with the expert's scratch (staged state / noise, residual stream,
 * projections, attention shares, split-K partial sums, statistic partials: about 3.4 MB for the full model) in a
 * device array that is part of the library itself instead of the workspace.  That array holds
 * PI0_STATIC_SCRATCH_BYTES; a geometry whose expert scratch is larger gets PI0_ENOMEM (checked first, before any
 * GPU call).  Weights and the prefix key/value cache are read from the workspace as usual.  Every GPU the library
 * runs on holds one copy of the array until the process ends; all calls on a GPU share it, whichever ctx they
 * belong to, so calls that overlap in time on one GPU race (calls on one stream do not overlap).  Must be called
 * with the device of pi0_load_weights current.  Same results as pi0_denoise, bit for bit.
 * Errors: EINVAL, ENOMEM, ESTATE (no valid prefill, or another device is current), EHIP.
 */
#define PI0_STATIC_SCRATCH_BYTES (4u << 20)
int pi0_denoise_static(pi0_ctx* ctx, const float* d_state, const float* d_noise, float* d_actions,
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
 * The denoise runs as the persistent kernel on a part of the compute units (96 .. 160 blocks, by prefix size), the
 * prefill on the rest; the same bounded waits and pi0_device_status apply.
 * How far the two streams overlap depends on the hardware queues the runtime gives them: a process has few (4 by
 * default), handed out in order of first use, and not every pair of queues runs kernels side by side equally well
 * (measured: the same frames 9.1 or 10.3 ms apart).  Create and first use the two streams early in the process,
 * before streams that other code or this library (the read-ahead stream of the per-operation denoise) creates.
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

/* Graph replay on (1, default) or off (0: every call launches kernels eagerly). */
int pi0_set_graph_mode(pi0_ctx* ctx, int enabled);

/*
 * Synchronises hip_stream and reports whether a bounded wait inside a kernel of this ctx ever ran out
 * (the denoise loop runs as one persistent kernel whose blocks synchronise with software grid barriers,
 * Section 5.2 of the paper; a barrier that is not completed within its bound - about a second - gives up
 * instead of hanging, and every result after that is undefined).  PI0_OK if none did, PI0_ESTATE if one
 * did or no weights are loaded; the condition stays set until pi0_load_weights.  Errors: EINVAL, EHIP.
 */
int pi0_device_status(pi0_ctx* ctx, void* hip_stream);

/* Static, never-NULL description of an error code. */
const char* pi0_strerror(int code);
/* hipError_t value of the last failed HIP call on this ctx (0 if none). */
int pi0_last_hip_error(const pi0_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* PI0_H */
