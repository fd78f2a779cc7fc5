// Token-by-token form of the normalized gated linear attention (paper section 4.2):
//   S_t = diag(alpha_t) S_{t-1} + k_t^T v_t,  z_t = alpha_t (.) z_{t-1} + k_t,
//   o_t = q_t S_t / (q_t . z_t + eps)
// in plain fp32 vector arithmetic.  Two kernels: gla_recurrent_kernel walks a whole sequence (prefill with
// fp32 storage, where bf16 matrix-core operands would not meet the fp32 error bound), gla_step_kernel is
// the decode step (lawcat_gla_step, one token, state updated in place).
//
// gla_recurrent_kernel: one 256-thread block owns a (batch, kv head) and a slice of 16 value columns.
// Lane layout: tid = j*16 + cg; the thread keeps S[c][col] for the d/16 key channels c = cg + 16 r of
// column col = 16 slice + j in registers, plus a replica of z[c].  q_t S_t is reduced over the 16 cg-lanes
// with cross-lane shuffles.
#include "kernels.h"

namespace lawcat {
namespace {

__device__ inline float ldf(const float* p) { return *p; }
__device__ inline float ldf(const bf16_t* p) { return __uint_as_float((uint32_t)(*p) << 16); }
__device__ inline void stf(float* p, float v) { *p = v; }
__device__ inline void stf(bf16_t* p, float v) {
  __bf16 h = (__bf16)v;  // round to nearest even
  *p = __builtin_bit_cast(bf16_t, h);
}

// log(sigmoid(g)), accurate on both tails.
__device__ inline float log_sigmoid(float g) {
  return g < 0.f ? g - log1pf(expf(g)) : -log1pf(expf(-g));
}

template <typename T, int D, int NJ>
__global__ void __launch_bounds__(256) gla_recurrent_kernel(
    const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v, const T* __restrict__ g,
    const float* S0, const float* z0, T* __restrict__ o, float* __restrict__ den_out, float* S_out,
    float* z_out, int Tn, int Hq, int Hkv, float gate_scale, float eps) {
  constexpr int R = D / 16;
  const int tid = threadIdx.x;
  const int cg = tid & 15;
  const int j = tid >> 4;
  const int bh = blockIdx.x;  // b * Hkv + hk
  const int b = bh / Hkv, hk = bh % Hkv;
  const int group = Hq / Hkv;
  const int slice0 = blockIdx.y * NJ;

  float S[NJ][R], z[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int c = cg + 16 * r;
    z[r] = z0 ? z0[(size_t)bh * D + c] : 0.f;
#pragma unroll
    for (int s = 0; s < NJ; ++s) {
      const int col = (slice0 + s) * 16 + j;
      S[s][r] = S0 ? S0[((size_t)bh * D + c) * D + col] : 0.f;
    }
  }
  if (NJ * 16 == D) __syncthreads();  // in-place update: every read of S/z precedes every write

  // One token's operands of this thread: its key channels of k and g, its value columns of v, and its key channels
  // of the first HB query heads of the group.  They are requested one token ahead, so that a token costs one
  // memory round trip hidden behind the previous token's arithmetic instead of five exposed ones.
  constexpr int HB = 4;
  struct Tok { float k[R], g[R], v[NJ], q[HB][R]; };
  const int nhb = group < HB ? group : HB;
  auto load_tok = [&](int t, Tok& x) {
    const size_t tok = (size_t)b * Tn + t;
    const T* kt = k + (tok * Hkv + hk) * D;
    const T* gt = g + (tok * Hkv + hk) * D;
    const T* vt = v + (tok * Hkv + hk) * D;
#pragma unroll
    for (int r = 0; r < R; ++r) { x.k[r] = ldf(kt + cg + 16 * r); x.g[r] = ldf(gt + cg + 16 * r); }
#pragma unroll
    for (int s = 0; s < NJ; ++s) x.v[s] = ldf(vt + (slice0 + s) * 16 + j);
#pragma unroll
    for (int hh = 0; hh < HB; ++hh)
      if (hh < nhb) {
        const T* qt = q + (tok * Hq + hk * group + hh) * D;
#pragma unroll
        for (int r = 0; r < R; ++r) x.q[hh][r] = ldf(qt + cg + 16 * r);
      }
  };
  Tok cur, nxt;
  load_tok(0, cur);
  const bool gs1 = gate_scale == 1.0f;
  for (int t = 0; t < Tn; ++t) {
    const size_t tok = (size_t)b * Tn + t;
    if (t + 1 < Tn) load_tok(t + 1, nxt);
#pragma unroll
    for (int r = 0; r < R; ++r) {
      // alpha = sigmoid(g)^gate_scale; at gate_scale 1 directly 1 / (1 + e^-g)
      const float alpha = gs1 ? 1.f / (1.f + expf(-cur.g[r])) : expf(gate_scale * log_sigmoid(cur.g[r]));
      const float kk = cur.k[r];
      z[r] = fmaf(alpha, z[r], kk);
#pragma unroll
      for (int s = 0; s < NJ; ++s) S[s][r] = fmaf(alpha, S[s][r], kk * cur.v[s]);
    }
    for (int hh = 0; hh < group; ++hh) {
      const int hq = hk * group + hh;
      float qq[R];
      if (hh < HB) {
#pragma unroll
        for (int h2 = 0; h2 < HB; ++h2)
          if (h2 == hh) {
#pragma unroll
            for (int r = 0; r < R; ++r) qq[r] = cur.q[h2][r];
          }
      } else {
        const T* qt = q + (tok * Hq + hq) * D;
#pragma unroll
        for (int r = 0; r < R; ++r) qq[r] = ldf(qt + cg + 16 * r);
      }
      float pd = 0.f, pn[NJ];
#pragma unroll
      for (int s = 0; s < NJ; ++s) pn[s] = 0.f;
#pragma unroll
      for (int r = 0; r < R; ++r) {
        pd = fmaf(qq[r], z[r], pd);
#pragma unroll
        for (int s = 0; s < NJ; ++s) pn[s] = fmaf(qq[r], S[s][r], pn[s]);
      }
#pragma unroll
      for (int m = 8; m >= 1; m >>= 1) {
        pd += __shfl_xor(pd, m, 16);
#pragma unroll
        for (int s = 0; s < NJ; ++s) pn[s] += __shfl_xor(pn[s], m, 16);
      }
      if (cg == 0) {
        const float den = pd + eps;
        T* ot = o + (tok * Hq + hq) * D;
#pragma unroll
        for (int s = 0; s < NJ; ++s) stf(ot + (slice0 + s) * 16 + j, pn[s] / den);
        if (den_out != nullptr && j == 0 && slice0 == 0) den_out[tok * Hq + hq] = den;
      }
    }
    cur = nxt;
  }
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int c = cg + 16 * r;
    if (j == 0 && slice0 == 0) z_out[(size_t)bh * D + c] = z[r];
#pragma unroll
    for (int s = 0; s < NJ; ++s) S_out[((size_t)bh * D + c) * D + (slice0 + s) * 16 + j] = S[s][r];
  }
}

// Decode step (T = 1), state in place.  One block per (batch, kv head).  Thread t owns value column
// t % D and a contiguous band of D*D/256 key channels of it, so a wave reads and writes whole 256-byte
// rows of S; alpha, k, z and the query heads are staged in LDS and read as broadcasts; the partial
// q.S sums of the 256/D bands are combined through LDS.  Query heads go four at a time.
template <typename T, int D>
__global__ void __launch_bounds__(256) gla_step_kernel(const T* __restrict__ q, const T* __restrict__ k,
                                                       const T* __restrict__ v, const T* __restrict__ g,
                                                       float* S, float* z, T* __restrict__ o, int Hq, int Hkv,
                                                       float gate_scale, float eps) {
  constexpr int NPART = 256 / D;      // bands of key channels
  constexpr int RPT = D / NPART;      // key channels per thread
  constexpr int HT = 4;               // query heads per pass
  __shared__ float sh_a[D], sh_k[D], sh_z[D], sh_q[HT][D], sh_part[HT][NPART][D];
  const int tid = threadIdx.x;
  const int bh = blockIdx.x;  // b * Hkv + hk
  const int b = bh / Hkv, hk = bh % Hkv;
  const int group = Hq / Hkv;
  const T* kt = k + (size_t)bh * D;
  const T* gt = g + (size_t)bh * D;
  const T* vt = v + (size_t)bh * D;
  float* Sh = S + (size_t)bh * D * D;
  float* zh = z + (size_t)bh * D;
  if (tid < D) {
    const float alpha = expf(gate_scale * log_sigmoid(ldf(gt + tid)));
    const float kk = ldf(kt + tid);
    const float zn = fmaf(alpha, zh[tid], kk);
    sh_a[tid] = alpha;
    sh_k[tid] = kk;
    sh_z[tid] = zn;
    zh[tid] = zn;
  }
  __syncthreads();
  const int col = tid % D, part = tid / D;
  const float vv = ldf(vt + col);
  float sreg[RPT];
#pragma unroll
  for (int r = 0; r < RPT; ++r) sreg[r] = Sh[(size_t)(part * RPT + r) * D + col];
#pragma unroll
  for (int r = 0; r < RPT; ++r) {
    const int c = part * RPT + r;
    sreg[r] = fmaf(sh_a[c], sreg[r], sh_k[c] * vv);
    Sh[(size_t)c * D + col] = sreg[r];
  }
  for (int h0 = 0; h0 < group; h0 += HT) {
    const int nh = min(HT, group - h0);
    __syncthreads();  // previous pass is done with sh_q / sh_part
    for (int e = tid; e < nh * D; e += 256) {
      const int hh = e / D, c = e % D;
      sh_q[hh][c] = ldf(q + ((size_t)b * Hq + hk * group + h0 + hh) * D + c);
    }
    __syncthreads();
    float pn[HT] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int r = 0; r < RPT; ++r) {
      const int c = part * RPT + r;
#pragma unroll
      for (int hh = 0; hh < HT; ++hh) pn[hh] = fmaf(sh_q[hh][c], sreg[r], pn[hh]);
    }
#pragma unroll
    for (int hh = 0; hh < HT; ++hh) sh_part[hh][part][col] = pn[hh];
    __syncthreads();
    // thread (hh = part', col): one output element each for up to 256 / D heads at a time
    for (int hh = part; hh < nh; hh += NPART) {
      float num = 0.f, den = eps;
#pragma unroll
      for (int pp = 0; pp < NPART; ++pp) num += sh_part[hh][pp][col];
      for (int c = 0; c < D; ++c) den = fmaf(sh_q[hh][c], sh_z[c], den);
      stf(o + ((size_t)b * Hq + hk * group + h0 + hh) * D + col, num / den);
    }
  }
}

template <typename T, int D>
hipError_t launch_step_d(const RecurrentParams& p, hipStream_t stream) {
  hipLaunchKernelGGL((gla_step_kernel<T, D>), dim3(p.B * p.Hkv), dim3(256), 0, stream, (const T*)p.q, (const T*)p.k,
                     (const T*)p.v, (const T*)p.g, p.S_out, p.z_out, (T*)p.o, p.Hq, p.Hkv, p.gate_scale, p.eps);
  return hipGetLastError();
}

template <typename T, int D>
hipError_t launch_d(const RecurrentParams& p, hipStream_t stream) {
  const int heads = p.B * p.Hkv;
  {
    hipLaunchKernelGGL((gla_recurrent_kernel<T, D, 1>), dim3(heads, D / 16), dim3(256), 0, stream, (const T*)p.q,
                       (const T*)p.k, (const T*)p.v, (const T*)p.g, p.S0, p.z0, (T*)p.o, p.den_out, p.S_out,
                       p.z_out, p.T, p.Hq, p.Hkv, p.gate_scale, p.eps);
  }
  return hipGetLastError();
}

}  // namespace

// n consecutive decode steps in one launch: the token-by-token kernel with one block per (batch, kv head) that
// owns every value column (NJ = D / 16), so the state stays in registers for all n tokens and the in-place
// update is safe (every read of S and z precedes every write inside the one block that touches them).
template <typename T, int D>
hipError_t launch_steps_d(const RecurrentParams& p, hipStream_t stream) {
  hipLaunchKernelGGL((gla_recurrent_kernel<T, D, D / 16>), dim3(p.B * p.Hkv, 1), dim3(256), 0, stream, (const T*)p.q,
                     (const T*)p.k, (const T*)p.v, (const T*)p.g, p.S_out, p.z_out, (T*)p.o, (float*)nullptr, p.S_out,
                     p.z_out, p.T, p.Hq, p.Hkv, p.gate_scale, p.eps);
  return hipGetLastError();
}

hipError_t launch_gla_steps(const RecurrentParams& p, hipStream_t stream) {
  if (p.bf16) return p.d == 64 ? launch_steps_d<bf16_t, 64>(p, stream) : launch_steps_d<bf16_t, 128>(p, stream);
  return p.d == 64 ? launch_steps_d<float, 64>(p, stream) : launch_steps_d<float, 128>(p, stream);
}

hipError_t launch_gla_step(const RecurrentParams& p, hipStream_t stream) {
  if (p.bf16) return p.d == 64 ? launch_step_d<bf16_t, 64>(p, stream) : launch_step_d<bf16_t, 128>(p, stream);
  return p.d == 64 ? launch_step_d<float, 64>(p, stream) : launch_step_d<float, 128>(p, stream);
}

hipError_t launch_gla_recurrent(const RecurrentParams& p, hipStream_t stream) {
  if (p.bf16) return p.d == 64 ? launch_d<bf16_t, 64>(p, stream) : launch_d<bf16_t, 128>(p, stream);
  return p.d == 64 ? launch_d<float, 64>(p, stream) : launch_d<float, 128>(p, stream);
}

}  // namespace lawcat
