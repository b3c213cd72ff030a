// Parameters of the persistent kernel that runs the action expert's whole denoise loop (expert_persistent.hip).
#pragma once
#include "embed_bodies.h"

struct ExpertLoopParams {
  // operations of layer 0 / step 0, filled exactly as for the per-operation launches; what changes per layer or
  // step is derived in the kernel from the strides below
  GemmParams qkv, o, gu, dn;      // per layer
  GemmParams tout, outp;          // per step: second linear of the action/time MLP; final norm + out-projection + Euler
  AttnParams att;
  StateTokenArgs stok;
  struct {
    ActionEmbedArgs a;            // a.bias_k = row of step 0 (rows a.X floats apart); a.x == x_rw
    float* x_rw;                  // x of the Euler integration [chunk][action_dim], inside the arena; holds the actions at the end
  } emb;
  const float* noise;             // [x_elems] initial x (staged input, constant during the kernel)
  int x_elems;
  int layers, steps;
  int read_ahead;                 // bit i set: blocks without an attention item read ahead range i of {gate||up, down, next QKV, next O}; 16: blocks without a QKV item read this layer's O
  size_t w_stride;                // elements between consecutive layers, the same for the four packed matrices
  size_t kcache_stride, vcache_stride;   // elements between consecutive layers of the prefix cache
  const float* g_attn0;           // gain vector of layer 0's attention norm; layer l at + l * gain_stride
  const float* g_mlp0;            // same for the feed-forward norm
  const float* g_final;
  size_t gain_stride;             // floats
  int parts_first, parts_rest;    // row-statistic partials the QKV projection of layer 0 / of the other layers reads
  int m16;                        // 16-token tiles of the O / down projections
  int dn_ns;                      // k steps per wave of the down projection: 16 (k = 4096) or 8 (k = 2048)
  int att_gx, att_items;          // attention work items: att_gx = 2 query tiles x value parts; x heads x key shares
  // Ring of per-layer-step buffers (slot ls = step * layers + layer at ring + ls * ring_stride).  Every activation
  // that one operation writes and the next reads with cached loads has its own place per layer-step, which nothing
  // has read before in this launch (exec_ctx.h, BULK_CACHED); byte offsets inside a slot:
  //   r_yb_o / r_st_o   gain-scaled bf16 copy of the residual stream and its statistic partials after the O projection
  //   r_yb_d / r_st_d   the same after the down projection (input of the next layer's QKV / of the out-projection)
  //   r_q, r_k, r_v     the QKV projection's outputs;  r_attn, r_ml  attention output shares and their (max, sum)
  //   r_mid             GeGLU product
  // The operation parameters above name the buffers of the per-operation launches; the kernel uses them for the first
  // QKV projection of a step (its input rows come from two operations and share cache lines: read past the L2) and
  // for the fp32 residual stream, which only ever crosses blocks as 1 KiB tiles read past the L2.
  char* ring;
  size_t ring_stride;
  unsigned r_yb_o, r_st_o, r_yb_d, r_st_d, r_q, r_k, r_v, r_attn, r_ml, r_mid;
  // synchronisation and the memory that blocks exchange
  unsigned* sync;                 // GB_WORDS words, words >= GB_START zeroed before the launch
  const char* arena;              // every buffer written by one block and read by another lies in [arena, arena + arena_bytes)
  unsigned arena_bytes;
  unsigned spin_limit;            // bound of one barrier wait, in polls
  // optional timeline for measurements: [operation][block][8] wall-clock samples (100 MHz) taken by thread 0:
  // operation entered, its inputs complete (wait over), body done, arrival announced, four points inside the body;
  // null = off
  long long* trace;
  int trace_ops;                  // capacity in operations
};

int expert_loop_smem_bytes();
hipError_t expert_loop_init_attributes();
hipError_t expert_loop_max_blocks_per_cu(int* out);
// d_params: device memory for one ExpertLoopParams (16-byte aligned), written by a small launch ahead of the loop kernel
hipError_t launch_expert_loop(hipStream_t s, const ExpertLoopParams& P, ExpertLoopParams* d_params, int blocks);
