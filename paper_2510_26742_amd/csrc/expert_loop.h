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
  // synchronisation and the memory that blocks exchange
  unsigned* sync;                 // GB_WORDS words, words >= GB_START zeroed before the launch
  const char* arena;              // every buffer written by one block and read by another lies in [arena, arena + arena_bytes)
  unsigned arena_bytes;
  unsigned spin_limit;            // bound of one barrier wait, in polls
};

int expert_loop_smem_bytes();
hipError_t expert_loop_init_attributes();
hipError_t expert_loop_max_blocks_per_cu(int* out);
// d_params: device memory for one ExpertLoopParams (16-byte aligned), written by a small launch ahead of the loop kernel
hipError_t launch_expert_loop(hipStream_t s, const ExpertLoopParams& P, ExpertLoopParams* d_params, int blocks);
