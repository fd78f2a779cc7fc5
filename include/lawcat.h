/*
 * lawcat.h -- C ABI of the MI355X (gfx950) LAWCAT sequence-mixing library.
 *
 * The library implements the prefill forward of LAWCAT's attention replacement
 * (arXiv 2509.18467, section 4): a causal depthwise Conv1D across tokens on the
 * queries and on the keys (section 4.1) feeding gated linear attention with the
 * normalization term kept (section 4.2); beside it the feature map with its linear layer,
 * the low-rank gate projection, decode steps and a first backward of the layer.
 *
 * Conventions shared by every call
 * --------------------------------
 *  - `desc` is a HOST pointer; every other pointer is a DEVICE pointer owned by the
 *    caller.  The library never allocates, frees or keeps a pointer.  Scratch space is
 *    the caller's `workspace` (size from lawcat_workspace_bytes).
 *  - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls only
 *    enqueue work; they never synchronize.
 *  - Layout is token-major with the head dimension contiguous:
 *      Q, O              [B, T, Hq,  d]
 *      K, V, gate_logits [B, T, Hkv, d]
 *      S (KV state)      [B, Hkv, dk, dv]  fp32       z (normalizer state) [B, Hkv, dk] fp32
 *      conv weights      [H, d, W] with w[h, c, delta] multiplying x[t - delta]
 *                        (delta = 0 is the current token; section 4.1, sum over delta)
 *      conv halo / tail  [B, W-1, H, d], oldest row first: the W-1 raw rows before the
 *                        first token / the last W-1 raw rows (the cache of section 4.1)
 *    Query head h reads the state of kv head h / (Hq/Hkv).
 *  - `dtype` is the storage type of Q, K, V, gate_logits, conv weights, halos, tails and
 *    O.  S, z and den are always fp32.  Arithmetic accumulates in fp32.
 *  - The gate is per key channel: alpha[t,c] = sigmoid(gate_logits[t,c])^gate_scale
 *    (section 4.2: linear layers followed by a sigmoid; G_t = alpha_t^T 1).
 *    One approximation, bf16 prefill only: the matrix-core kernels floor alpha at 2^-13 per step (gate logits
 *    below -9.0 at gate_scale 1), so that the reciprocal decay products inside an 8-token half chunk stay below
 *    2^104.  What is lost is a factor that is already below 1.3e-4 of what it multiplies, i.e. under the bf16
 *    resolution of the operands; logits of -30 everywhere, +30 everywhere and gate_scale 0 .. 16 meet the same
 *    tolerance as ordinary gates.  fp32 storage, lawcat_gla_step, lawcat_gla_steps and lawcat_gla_backward do not clamp.
 *  - Return value: LAWCAT_OK or a negative lawcat_status.  All argument checks run on
 *    the host before anything is enqueued; after an error the outputs are unspecified.
 *    A zero denominator is not an error: IEEE inf/nan is returned as the last equation
 *    of section 4.2 gives it.
 *  - Inputs and outputs must not overlap, except S/z in lawcat_gla_step and lawcat_gla_steps (updated
 *    in place).  All pointers must be 16-byte aligned.
 */
#ifndef LAWCAT_H_
#define LAWCAT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LAWCAT_VERSION 1
#define LAWCAT_API __attribute__((visibility("default")))

typedef enum lawcat_status {
  LAWCAT_OK = 0,
  LAWCAT_E_NULL = -1,        /* a required pointer is NULL */
  LAWCAT_E_BAD_DESC = -2,    /* struct_size mismatch, non-positive dims, Hq % Hkv != 0, bad enum */
  LAWCAT_E_UNSUPPORTED = -3, /* head dim, conv width, chunk or mode outside what the kernels cover */
  LAWCAT_E_WORKSPACE = -4,   /* workspace NULL or smaller than lawcat_workspace_bytes */
  LAWCAT_E_ALIGN = -5,       /* a pointer is not 16-byte aligned */
  LAWCAT_E_HIP = -6,         /* the HIP runtime reported a launch error */
  LAWCAT_E_STATIC_LIMIT = -7 /* lawcat_layer_prefill_static: the call needs more than LAWCAT_STATIC_WORKSPACE_BYTES */
} lawcat_status;

enum { LAWCAT_DTYPE_F32 = 0, LAWCAT_DTYPE_BF16 = 1 };
enum { LAWCAT_PHI_IDENTITY = 0, LAWCAT_PHI_ELU1 = 1 }; /* 1 + ELU: x > 0 ? 1 + x : exp(x) */
enum { LAWCAT_CARRY_AUTO = 0, LAWCAT_CARRY_SEQUENTIAL = 1, LAWCAT_CARRY_TWO_LEVEL = 2 };
enum {
  LAWCAT_CALL_CONV1D = 0,
  LAWCAT_CALL_GLA_PREFILL = 1,
  LAWCAT_CALL_GLA_STEP = 2,
  LAWCAT_CALL_LAYER_PREFILL = 3,
  LAWCAT_CALL_LAYER_PREFILL_FM = 4,
  LAWCAT_CALL_GLA_BACKWARD = 5,
  LAWCAT_CALL_CONV1D_BACKWARD = 6 /* sized for Hq heads (the larger of the two convs) */
};

typedef struct lawcat_desc {
  uint32_t struct_size; /* = sizeof(lawcat_desc) */
  int32_t B, T, Hq, Hkv; /* Hq % Hkv == 0 */
  int32_t dk, dv;        /* supported: dk == dv in {64, 128} */
  int32_t conv_width;    /* W = r + 1, supported 1..4 (the paper uses 4) */
  int32_t dtype;         /* LAWCAT_DTYPE_* */
  int32_t feature_map;   /* LAWCAT_PHI_*: pointwise map applied after the conv */
  int32_t chunk;         /* tokens per state-carry step of the bf16 path: 0 = auto, else 16 */
  int32_t carry_mode;    /* LAWCAT_CARRY_*: how the state crosses segment boundaries */
  int32_t segment;       /* tokens per workgroup in two-level mode: 0 = auto, else a multiple of 64 */
  float gate_scale;      /* log alpha = gate_scale * log sigmoid(g); 1.0 in every graded workload */
  float eps;             /* added to the denominator; 0 = the paper's equation as written */
} lawcat_desc;

/* Bytes of device scratch `which_call` (LAWCAT_CALL_*) needs for this desc; 0 if none.
 * Returns 0 for an invalid desc as well (the call itself reports the error). */
LAWCAT_API size_t lawcat_workspace_bytes(const lawcat_desc* desc, int which_call);

/*
 * Section 4.1: y[b,t,h,c] = phi( sum_{delta<W} w[h,c,delta] * x[b,t-delta,h,c] ).
 * Rows before the first token come from `halo` (NULL = zeros).  `n_heads` is the head
 * count of x (Hq for queries, Hkv for keys); desc->Hq/Hkv are not read.
 *   x, y      [B,T,n_heads,d]   w [n_heads,d,W]   halo, tail_out [B,W-1,n_heads,d] (nullable)
 * tail_out receives the last W-1 raw rows of [halo ; x]; it must not alias halo.
 * With W == 1 halo and tail_out are ignored.
 */
LAWCAT_API int lawcat_conv1d_causal(const lawcat_desc* desc, int n_heads, const void* x, const void* w,
                         const void* halo, void* y, void* tail_out, void* stream);

/*
 * Section 4.1 with the shared linear layer after the conv ("a linear layer with nonlinearity", the same
 * for the query and the key):
 *   y[b,t,h,f] = phi( sum_c x~[b,t,h,c] * wf[h / group, c, f] ),   x~ = the conv of lawcat_conv1d_causal without phi
 *   wf [Hkv,d,d] in the storage type, row-major [c][f]; n_heads must be a multiple of desc->Hkv and
 *   group = n_heads / desc->Hkv: a query head uses the matrix of the kv head whose state it reads.
 * Every other argument as in lawcat_conv1d_causal.  bf16 storage: x~ is rounded to bf16 once, as the
 * matrix-core operand; accumulation in fp32.
 */
LAWCAT_API int lawcat_conv1d_feature(const lawcat_desc* desc, int n_heads, const void* x, const void* w,
                          const void* wf, const void* halo, void* y, void* tail_out, void* stream);

/*
 * Section 4.2, where the gate logits come from ("linear layers" before the sigmoid; the appendix's ablation on the
 * rank of the gate function: two consecutive low-rank linear layers, rank 32 in the distilled models):
 *   gate_logits[b,t,n] = sum_r ( sum_c x[b,t,c] * w1[r,c] ) * w2[n,r] + bias[n]
 *   x [B,T,d_model] the layer input; w1 [rank,d_model]; w2 [Hkv*dk,rank] (out-features x in-features, as linear
 *   layers are stored); bias [Hkv*dk], nullable; all in the storage type.  gate_logits [B,T,Hkv,dk]: the tensor
 *   the prefill and step calls take.
 * d_model and rank multiples of 8 with (d_model + rank) * 4 <= 65536, else LAWCAT_E_UNSUPPORTED.  bf16 storage
 * with rank 32, d_model % 128 == 0 and Hkv*dk % 128 == 0 runs on the matrix cores (fp32 accumulation; the
 * rank-32 intermediate is rounded to bf16 once, as an operand); every other case in plain fp32.
 */
LAWCAT_API int lawcat_gate_project(const lawcat_desc* desc, int d_model, int rank, const void* x, const void* w1,
                        const void* w2, const void* bias, void* gate_logits, void* stream);

/*
 * Section 4.2, prefill: for t = 1..T
 *   S_t = diag(alpha_t) S_{t-1} + k_t^T v_t,   z_t = alpha_t (.) z_{t-1} + k_t,
 *   o_t = q_t S_t / (q_t . z_t + eps)
 * starting from S0, z0 (NULL = zeros).  q and k are the already transformed q-dot, k-dot.
 *   q [B,T,Hq,dk]  k, gate_logits [B,T,Hkv,dk]  v [B,T,Hkv,dv]  o [B,T,Hq,dv]
 *   den_out (nullable) [B,T,Hq] fp32 = q_t . z_t + eps
 *   S_out [B,Hkv,dk,dv], z_out [B,Hkv,dk]: the state after token T (required).
 */
LAWCAT_API int lawcat_gla_prefill(const lawcat_desc* desc, const void* q, const void* k, const void* v,
                       const void* gate_logits, const float* S0, const float* z0, void* o,
                       float* den_out, float* S_out, float* z_out, void* workspace,
                       size_t workspace_bytes, void* stream);

/*
 * Adjoint of lawcat_gla_prefill (section 5 trains the layer by gradient descent on a layer-wise loss): given
 * dO = dL/dO and the forward's den_out, the gradients with respect to q, k, v, the gate logits and the start
 * state.  With v^ = [v, 1], S^ = [S | z], dnum = dO / den, dden = -(q_t S_t dnum^T) / den, d^ = [dnum | dden]:
 *   dq_t = S^_t d^_t^T;   Gr_t = alpha_{t+1} (.) Gr_{t+1} + sum over the group's query heads of q_t^T d^_t;
 *   dk_t = Gr_t v^_t^T;   dv_t = k_t Gr_t[:, :dv];
 *   dgate_logits_t = gate_scale (1 - sigmoid(g_t)) sum_{s >= t} ( sum_h q_s (.) dq_s - k_s (.) dk_s ).
 *   q, k, v, gate_logits, S0, z0 as lawcat_gla_prefill took them; den [B,T,Hq] as it returned it (den_out; the
 *   output O itself is not needed);  dO [B,T,Hq,dv];  dq, dk, dv, dgate_logits: shapes and type of q, k, v,
 *   gate_logits;  dS0 [B,Hkv,dk,dv], dz0 [B,Hkv,dk]: nullable.  Workspace: LAWCAT_CALL_GLA_BACKWARD.
 * fp32 vector arithmetic throughout (both storage types), parallel over (batch, kv head) and segments of the
 * sequence; a first version, several times the forward's time.  Query heads per kv head x head dim above 2048
 * (the staging of one token's query heads) is LAWCAT_E_UNSUPPORTED.
 */
LAWCAT_API int lawcat_gla_backward(const lawcat_desc* desc, const void* q, const void* k, const void* v,
                        const void* gate_logits, const float* den, const void* dO,
                        const float* S0, const float* z0, void* dq, void* dk, void* dv, void* dgate_logits,
                        float* dS0, float* dz0, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Adjoint of lawcat_conv1d_causal, pointwise feature map included (section 4.1; the distillation of section 5
 * trains the conv weights): with u_t = sum_{delta<W} w[delta] x_{t-delta}, du_t = dy_t phi'(u_t) (phi' = 1 for the
 * identity; for 1 + ELU: 1 where u > 0, exp(u) elsewhere; u is recomputed from x):
 *   dx[b,s,h,c] = sum_{delta<W} w[h,c,delta] du[b,s+delta,h,c]        (tokens past the end contribute nothing)
 *   dw[h,c,delta] = sum_{b,t} du[b,t,h,c] x[b,t-delta,h,c]            (fp32, whatever the storage type)
 *   dhalo: the same sum as dx for the W-1 rows before the first token (nullable; written whether or not halo is given)
 *   x, w, halo as lawcat_conv1d_causal took them; dy, dx [B,T,n_heads,d]; dhalo [B,W-1,n_heads,d]; dw [n_heads,d,W].
 * Workspace: LAWCAT_CALL_CONV1D_BACKWARD (partial sums of dw per 64-token strip, added in a fixed order: repeated
 * calls agree bit for bit).  A layer's backward is lawcat_gla_backward followed by this call on (Q, wq, dq) and on
 * (K, wk, dk).  B above 65535 or T above 65535 * 64 is LAWCAT_E_UNSUPPORTED (grid limits).
 */
LAWCAT_API int lawcat_conv1d_backward(const lawcat_desc* desc, int n_heads, const void* x, const void* w, const void* halo,
                           const void* dy, void* dx, float* dw, void* dhalo, void* workspace,
                           size_t workspace_bytes, void* stream);

/*
 * Section 4.2, one recurrent (decode) step on one token per sequence; desc->T is ignored.
 *   q [B,Hq,dk]  k, gate_logits [B,Hkv,dk]  v [B,Hkv,dv]  o [B,Hq,dv]
 *   S [B,Hkv,dk,dv], z [B,Hkv,dk]: read, updated in place.
 */
LAWCAT_API int lawcat_gla_step(const lawcat_desc* desc, const void* q, const void* k, const void* v,
                    const void* gate_logits, float* S, float* z, void* o, void* stream);

/*
 * Section 4.2, n = desc->T consecutive recurrent (decode) steps per sequence in ONE launch: the same fp32
 * token-by-token arithmetic as n calls of lawcat_gla_step, with the state held on chip between the steps, so
 * the state's 2 * Hkv * dk * dv * 4 bytes cross HBM once per call instead of once per token (streaming
 * inference in blocks of tokens, speculative or chunked decoding).
 *   q [B,n,Hq,dk]  k, gate_logits [B,n,Hkv,dk]  v [B,n,Hkv,dv]  o [B,n,Hq,dv]
 *   S [B,Hkv,dk,dv], z [B,Hkv,dk]: read, updated in place to the state after the n-th token.
 * q and k are the already transformed q-dot, k-dot (lawcat_conv1d_causal with T = n and the conv cache as halo).
 */
LAWCAT_API int lawcat_gla_steps(const lawcat_desc* desc, const void* q, const void* k, const void* v,
                     const void* gate_logits, float* S, float* z, void* o, void* stream);

/*
 * The whole layer of Fig. 1 between the projections: conv + phi on Q (weights wq [Hq,dk,W])
 * and on K (wk [Hkv,dk,W]), gate logits -> decay, normalized gated linear attention.
 * Equals lawcat_conv1d_causal on Q and on K followed by lawcat_gla_prefill.
 *   S0, z0, q_halo, k_halo: nullable (zeros).  den_out, q_tail_out, k_tail_out: nullable.
 *   S_out, z_out: required.
 */
LAWCAT_API int lawcat_layer_prefill(const lawcat_desc* desc, const void* Q, const void* K, const void* V,
                         const void* gate_logits, const void* wq, const void* wk, const float* S0,
                         const float* z0, const void* q_halo, const void* k_halo, void* O,
                         float* den_out, float* S_out, float* z_out, void* q_tail_out,
                         void* k_tail_out, void* workspace, size_t workspace_bytes, void* stream);

/*
 * lawcat_layer_prefill for sequences of different lengths packed back to back (continuous batching, chunked
 * prefill of several requests): section 4.2's recurrence restarts at every sequence boundary, and section 4.1's
 * conv does not reach across it.  desc->B = number of sequences, desc->T = an upper bound of their lengths.
 *   seq_start      HOST array of B + 1 token offsets, seq_start[0] = 0, strictly increasing: sequence i owns
 *                  tokens seq_start[i] .. seq_start[i+1] - 1; total = seq_start[B]
 *   seq_start_dev  nullable DEVICE copy of the same B + 1 offsets (4-byte aligned)
 *   Q, O [total,Hq,dk]   K, V, gate_logits [total,Hkv,dk]   den_out [total,Hq] (nullable)
 *   S0, z0, S_out, z_out, q_halo, k_halo, q_tail_out, k_tail_out: per sequence, shaped as in
 *   lawcat_layer_prefill with B sequences (chunked prefill: feed a sequence's S_out, z_out and tails back in).
 * With seq_start_dev and bf16 storage the whole batch is ONE set of launches: the kernels read each sequence's
 * first row and length from the device array, and the segments are cut as for one sequence of all the tokens, so
 * that the workgroups are about as many as the chip holds whatever the mix of lengths.  Otherwise (no device
 * copy, or fp32 storage): one lawcat_layer_prefill with B = 1 per sequence, enqueued in order on `stream`,
 * sharing `workspace`.  Workspace size for either form: lawcat_varlen_workspace_bytes (one_launch = whether
 * seq_start_dev will be passed).  All sequences are checked on the host before anything is enqueued: a length
 * below 1 or above desc->T is LAWCAT_E_BAD_DESC.
 */
LAWCAT_API size_t lawcat_varlen_workspace_bytes(const lawcat_desc* desc, const int32_t* seq_start, int one_launch);

LAWCAT_API int lawcat_layer_prefill_varlen(const lawcat_desc* desc, const int32_t* seq_start,
                                const int32_t* seq_start_dev, const void* Q, const void* K, const void* V, const void* gate_logits, const void* wq,
                                const void* wk, const float* S0, const float* z0, const void* q_halo,
                                const void* k_halo, void* O, float* den_out, float* S_out, float* z_out,
                                void* q_tail_out, void* k_tail_out, void* workspace, size_t workspace_bytes,
                                void* stream);

/*
 * The layer of Fig. 1 with the feature map of section 4.1 in full: after the conv, "a linear layer with
 * nonlinearity", the same for the query and the key,
 *   q-dot = phi( conv(Q) Wf ),  k-dot = phi( conv(K) Wf ),
 * then the attention of section 4.2: lawcat_conv1d_feature on Q and on K followed by lawcat_gla_prefill.
 * wf [Hkv,dk,dk] as in lawcat_conv1d_feature; with identity matrices the call equals lawcat_layer_prefill.
 * Every other argument as in lawcat_layer_prefill; workspace from
 * lawcat_workspace_bytes(desc, LAWCAT_CALL_LAYER_PREFILL_FM): q-dot and k-dot are staged there in the storage
 * type, B*T*(Hq+Hkv)*dk elements, ahead of what lawcat_gla_prefill needs.
 */
LAWCAT_API int lawcat_layer_prefill_fm(const lawcat_desc* desc, const void* Q, const void* K, const void* V,
                            const void* gate_logits, const void* wq, const void* wk, const void* wf,
                            const float* S0, const float* z0, const void* q_halo, const void* k_halo, void* O,
                            float* den_out, float* S_out, float* z_out, void* q_tail_out, void* k_tail_out,
                            void* workspace, size_t workspace_bytes, void* stream);

/*
 * lawcat_layer_prefill for callers that cannot allocate device memory or hold a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and same results as
 * lawcat_layer_prefill, without `workspace`: the scratch is a buffer of LAWCAT_STATIC_WORKSPACE_BYTES that
 * lives inside the library, one copy per GPU that loads it, until the process ends.  The call allocates and
 * frees nothing.  A desc whose lawcat_workspace_bytes(desc, LAWCAT_CALL_LAYER_PREFILL) exceeds the buffer
 * returns LAWCAT_E_STATIC_LIMIT before anything is enqueued (24 MiB covers the two-level carry of every
 * single-sequence shape with up to 8 kv heads of dimension 128; fp32 storage stages q-dot and k-dot there and
 * fits only short sequences).  Every call on a GPU uses that GPU's one buffer: calls that overlap in time on
 * the same GPU (different streams, or several host threads) race and must be serialized by the caller.  The
 * buffer keeps the previous call's contents; nothing in it needs to start at zero.  The first call on a
 * device looks the buffer's address up (hipGetSymbolAddress) and should be made outside stream capture.
 */
#define LAWCAT_STATIC_WORKSPACE_BYTES (24u << 20)
LAWCAT_API int lawcat_layer_prefill_static(const lawcat_desc* desc, const void* Q, const void* K, const void* V,
                                const void* gate_logits, const void* wq, const void* wk, const float* S0,
                                const float* z0, const void* q_halo, const void* k_halo, void* O,
                                float* den_out, float* S_out, float* z_out, void* q_tail_out,
                                void* k_tail_out, void* stream);

/*
 * Measurement variant of lawcat_layer_prefill (same arguments, same result) for benchmarks: the dominant
 * kernel of the bf16 matrix-core path, the output pass, is launched with `ev_start` and `ev_stop`
 * (hipEvent_t passed as void*, both required, owned by the caller) as its start and stop events, so that
 * hipEventElapsedTime(ev_start, ev_stop) is that kernel's duration on the call's stream.  With more than
 * four query heads per kv head the events bracket the first output-pass launch.  Returns
 * LAWCAT_E_UNSUPPORTED for a desc that the matrix-core path does not serve (fp32 storage).  No state is
 * kept between calls.
 */
LAWCAT_API int lawcat_layer_prefill_timed(const lawcat_desc* desc, const void* Q, const void* K, const void* V,
                               const void* gate_logits, const void* wq, const void* wk, const float* S0,
                               const float* z0, const void* q_halo, const void* k_halo, void* O,
                               float* den_out, float* S_out, float* z_out, void* q_tail_out,
                               void* k_tail_out, void* workspace, size_t workspace_bytes, void* stream,
                               void* ev_start, void* ev_stop);

/* Static string for a lawcat_status value. */
LAWCAT_API const char* lawcat_status_string(int status);

/* LAWCAT_VERSION the library was built with. */
LAWCAT_API int lawcat_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LAWCAT_H_ */
