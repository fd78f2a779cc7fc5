// Internal launch interface between the host ABI (api.hip) and the kernel files.
// Not part of the public boundary; include/lawcat.h is.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace lawcat {

// Storage element of the bf16 path: raw 16-bit pattern.
typedef uint16_t bf16_t;

struct ConvParams {
  const void* x;     // [B,T,H,d]
  const void* w;     // [H,d,W]
  const void* halo;  // nullable [B,W-1,H,d]
  void* y;           // [B,T,H,d]
  void* tail_out;    // nullable [B,W-1,H,d]
  int B, T, H, d, W;
  int phi;           // 0 identity, 1 = 1+ELU
  int bf16;          // storage type
};
hipError_t launch_conv1d(const ConvParams& p, hipStream_t stream);
// Copies the last W-1 raw rows of [halo ; x] (the conv cache) into p.tail_out without running the conv.
hipError_t launch_conv_tail(const ConvParams& p, hipStream_t stream);
// Conv followed by the shared linear layer with nonlinearity (section 4.1): y = phi(conv(x) Wf), Wf [H / group, d, d]
// in the storage type; head h uses matrix h / group.  p.tail_out is not written (see launch_conv_tail).
// Adjoint of the normalized gated linear attention: gradients with respect to q-dot, k-dot, v, the gate logits and
// the start state, given dO and the forward's den.
struct GlaBackwardParams {
  const void *q, *k, *v, *g;   // as lawcat_gla_prefill took them
  const void* dO;              // [B,T,Hq,d] storage type
  const float* den;            // [B,T,Hq]
  const float *S0, *z0;        // nullable
  void *dq, *dk, *dv, *dg;     // storage type, shapes of q, k, v, g
  float *dS0, *dz0;            // nullable
  void* workspace;
  int B, T, Hq, Hkv, d;
  float gate_scale;             // den already holds eps: the adjoint does not need it
  int bf16;
};
bool gla_backward_supports(int d, int group);
size_t gla_backward_workspace_bytes(int B, int T, int Hq, int Hkv, int d);
hipError_t launch_gla_backward(const GlaBackwardParams& p, hipStream_t stream);

// Adjoint of launch_conv1d (conv + pointwise feature map): dx, dw (fp32, [H,d,W]) and dhalo from dy.
struct ConvBackwardParams {
  const void *x, *w, *halo, *dy;   // as the forward took them; halo nullable; dy [B,T,H,d]
  void *dx, *dhalo;                // storage type; dhalo nullable [B,W-1,H,d]
  float* dw;                       // [H,d,W]
  void* workspace;                 // conv_backward_workspace_bytes()
  int B, T, H, d, W;
  int phi, bf16;
};
size_t conv_backward_workspace_bytes(int B, int T, int H, int d, int W);
hipError_t launch_conv_backward(const ConvBackwardParams& p, hipStream_t stream);

// gate logits from the layer input: g = (x w1^T) w2^T + bias (two consecutive low-rank linear layers)
struct GateProjectParams {
  const void *x, *w1, *w2, *bias;  // [B,T,dm], [rank,dm], [N,rank], [N] or null; storage type
  void* g;                         // [B,T,N]
  int B, T, dm, rank, N;
  int bf16;
};
hipError_t launch_gate_project(const GateProjectParams& p, hipStream_t stream);

hipError_t launch_conv_feature(const ConvParams& p, const void* wf, int group, hipStream_t stream);

struct RecurrentParams {
  const void* q;  // [B,T,Hq,d]  (q-dot)
  const void* k;  // [B,T,Hkv,d] (k-dot)
  const void* v;  // [B,T,Hkv,d]
  const void* g;  // [B,T,Hkv,d] gate logits
  const float* S0;  // nullable [B,Hkv,d,d]
  const float* z0;  // nullable [B,Hkv,d]
  void* o;          // [B,T,Hq,d]
  float* den_out;   // nullable [B,T,Hq]
  float* S_out;     // [B,Hkv,d,d]
  float* z_out;     // [B,Hkv,d]
  int B, T, Hq, Hkv, d;
  float gate_scale, eps;
  int bf16;
};
hipError_t launch_gla_recurrent(const RecurrentParams& p, hipStream_t stream);
// One token per sequence, S_out/z_out updated in place (S0, z0, den_out, T are not read).
hipError_t launch_gla_step(const RecurrentParams& p, hipStream_t stream);
// T consecutive tokens per sequence in one launch, S_out/z_out updated in place (S0, z0, den_out are not read).
hipError_t launch_gla_steps(const RecurrentParams& p, hipStream_t stream);

// How the bf16 matrix-core prefill splits a sequence: `nseg` segments of `seg_len` tokens per
// (batch, kv head), each carried sequentially by one workgroup.  With nseg > 1 a first pass
// computes every segment's state contribution and a scan turns them into start states.
struct ChunkPlan {
  int seg_len;
  int nseg;
  size_t workspace_bytes;
};
ChunkPlan make_chunk_plan(int B, int T, int Hkv, int d, int carry_mode, int segment);
bool chunk_path_supports(int group);  // query heads per kv head the kernel is built for

struct ChunkParams {
  const void* q;  // raw Q (fuse_conv) or q-dot: [B,T,Hq,d] bf16
  const void* k;
  const void* v;
  const void* g;
  const void* wq;      // [Hq,d,W]  (fuse_conv only)
  const void* wk;      // [Hkv,d,W] (fuse_conv only)
  const void* q_halo;  // nullable [B,W-1,Hq,d]
  const void* k_halo;  // nullable [B,W-1,Hkv,d]
  const float* S0;
  const float* z0;
  void* o;
  float* den_out;
  float* S_out;
  float* z_out;
  void* q_tail;  // nullable [B,W-1,Hq,d]  (fuse_conv only)
  void* k_tail;  // nullable [B,W-1,Hkv,d]
  void* workspace;
  // nullable device array of B + 1 row offsets: sequences of different lengths packed along the token axis
  // (then T is the longest length, and the tensors above hold seq_start[B] rows)
  const int* seq_start;
  int B, T, Hq, Hkv, d, W;
  int phi;
  int fuse_conv;
  float gate_scale, eps;
  ChunkPlan plan;
  // measurement only: when both are set, the (first) output-pass kernel is launched with them as its start and
  // stop events
  hipEvent_t ev_start, ev_stop;
};
hipError_t launch_gla_chunk(const ChunkParams& p, hipStream_t stream);

}  // namespace lawcat
