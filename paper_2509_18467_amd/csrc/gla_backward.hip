// Adjoint of the normalized gated linear attention of paper section 4.2 (what the layer-wise distillation of
// section 5 differentiates through): given dO = dL/do and the forward's den, the gradients with respect to
// q-dot, k-dot, v, the gate logits and the start state.  With v^ = [v, 1], S^ = [S | z]:
//   dnum = dO / den,  dden = -(dO . o) / den = -(q_t S_t dnum^T) / den,   d^ = [dnum | dden]
//   (o is never read: rounded to the storage type it would spoil dq, where S dnum^T and z dden nearly cancel)
//   dq_t = S^_t d^_t^T                                    (forward sweep: S^_t is at hand there)
//   Gr_t = alpha_{t+1} (.) Gr_{t+1} + sum_h q_{h,t}^T d^_{h,t}   (reverse sweep)
//   dk_t = Gr_t v^_t^T,   dv_t = k_t Gr_t[:, :dv]
//   dlog alpha_t = sum_{s >= t} ( sum_h q_{h,s} (.) dq_{h,s} - k_s (.) dk_s )     (every pair i < t <= s carries
//                  alpha_t once, in the query's gradient and not in the key's)
//   dg_t = dlog alpha_t * gate_scale * (1 - sigmoid(g_t))
// Plain fp32 vector arithmetic, token by token, parallel over (batch, kv head) and over segments of the
// sequence: like the forward's two-level carry, a first sweep per segment from a zero state gives the segment's
// contribution and total decay, a scan turns those into the states at the segment boundaries (forwards for S^,
// backwards for Gr), and a second sweep produces the outputs.  A workgroup of 256 threads holds one d x (d + 1)
// state in registers: thread = one key channel (row) x a run of value columns, so products that contract the
// value dimension (dq, dk) reduce inside a few adjacent lanes; dv contracts the key dimension and is reduced
// through shuffles and LDS in a fixed order (no atomics: repeated calls agree bit for bit).  Tokens are staged
// through LDS in blocks.  A first version: correct and segment-parallel, several times the forward's time.
#include <mutex>

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
__device__ inline float log_sigmoid(float g) { return g < 0.f ? g - log1pf(expf(g)) : -log1pf(expf(-g)); }

struct BwdArgs {
  const void *q, *k, *v, *g, *dO;
  const float* den;
  const float *S0, *z0;
  void *dq, *dk, *dv, *dg;
  float *dS0, *dz0;
  float* dnum;       // [B,T,Hq,D]
  float* dden;       // [B,T,Hq]
  float* slots_f;    // [heads][nseg][D*D + 2D]: forward contributions, then start states
  float* slots_r;    // the same for Gr, segments in reverse order
  float* gate_local; // [B,T,Hkv,D]: sum_h q (.) dq, then the suffix sum of the gate term within the segment
  float* gate_tot;   // [heads][nseg][D]: the segment's total, then the sum over all later segments
  int B, T, Hq, Hkv, group, seg_len, nseg, tb;
  float gate_scale, eps;
};

// ---- dnum = dO / den
template <typename T, int D>
__global__ void __launch_bounds__(256) bwd_prepare_kernel(const T* __restrict__ dO, const float* __restrict__ den,
                                                         float* __restrict__ dnum, long long total) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i < total) dnum[i] = ldf(dO + i) / den[i / D];
}

enum { kFwdContrib = 0, kFwdOut = 1, kRevContrib = 2, kRevOut = 3 };

// grid (nseg, B * Hkv), 256 threads, dynamic LDS.
template <typename T, int D, int MODE>
__global__ void __launch_bounds__(256) bwd_pass_kernel(const BwdArgs a) {
  constexpr int TPR = 256 / D;       // threads per state row
  constexpr int CPT = D / TPR;       // value columns per thread
  constexpr bool REV = MODE >= kRevContrib;
  constexpr bool OUT = MODE == kFwdOut || MODE == kRevOut;
  constexpr int kSlot = D * D + 2 * D;
  extern __shared__ float sm[];
  const int tid = threadIdx.x;
  const int c = tid / TPR, j0 = (tid % TPR) * CPT;
  const int seg = blockIdx.x, bh = blockIdx.y;
  const int b = bh / a.Hkv, hk = bh % a.Hkv;
  const int group = a.group, tb = a.tb;
  const int s0 = seg * a.seg_len, s1 = min(a.T, s0 + a.seg_len);
  // LDS: per staged token  alpha[D] k[D] v[D] | per head q[D] dn[D] dq[D] | dd[group] ; then the output staging
  float* s_al = sm;
  float* s_k = s_al + tb * D;
  float* s_v = s_k + tb * D;
  float* s_q = s_v + tb * D;                 // [tb][group][D]
  float* s_dn = s_q + tb * group * D;        // [tb][group][D]
  float* s_dq = s_dn + tb * group * D;       // [tb][group][D]: dq out (forward) / dq in (reverse)
  float* s_dd = s_dq + tb * group * D;       // [tb][group]
  float* s_dk = s_dd + tb * group;           // [tb][D]
  float* s_gl = s_dk + tb * D;               // [tb][D]
  float* s_dv = s_gl + tb * D;               // [tb][4 waves][D]

  const T* q = static_cast<const T*>(a.q);
  const T* k = static_cast<const T*>(a.k);
  const T* v = static_cast<const T*>(a.v);
  const T* g = static_cast<const T*>(a.g);

  // ---- state of this thread: row c, columns j0 .. j0 + CPT - 1, and the normalizer column
  float X[CPT], xz = 0.f, decay = 1.f, gsum = 0.f;
#pragma unroll
  for (int j = 0; j < CPT; ++j) X[j] = 0.f;
  if (OUT) {
    const float* src = nullptr;
    const float* zsrc = nullptr;
    if (a.nseg > 1) {
      src = (REV ? a.slots_r : a.slots_f) + ((size_t)bh * a.nseg + (REV ? a.nseg - 1 - seg : seg)) * kSlot;
      zsrc = src + D * D;
    } else if (!REV) {
      if (a.S0) src = a.S0 + (size_t)bh * D * D;
      if (a.z0) zsrc = a.z0 + (size_t)bh * D;
    }
    if (src) {
#pragma unroll
      for (int j = 0; j < CPT; ++j) X[j] = src[(size_t)c * D + j0 + j];
    }
    if (zsrc) xz = zsrc[c];
  }

  const int len = s1 - s0;
  const int nblk = (len + tb - 1) / tb;
  for (int bi = 0; bi < nblk; ++bi) {
    const int blk = REV ? nblk - 1 - bi : bi;
    const int t_lo = s0 + blk * tb;
    const int n = min(tb, s1 - t_lo);
    // ---- stage the block's tokens
    for (int idx = tid; idx < n * D; idx += 256) {
      const int tl = idx / D, cc = idx % D;
      const size_t row = ((size_t)b * a.T + t_lo + tl) * a.Hkv + hk;
      const float gl = ldf(g + row * D + cc);
      s_al[idx] = a.gate_scale == 1.0f ? 1.f / (1.f + expf(-gl)) : expf(a.gate_scale * log_sigmoid(gl));
      s_k[idx] = ldf(k + row * D + cc);
      s_v[idx] = ldf(v + row * D + cc);
    }
    if (MODE != kFwdContrib) {
      for (int idx = tid; idx < n * group * D; idx += 256) {
        const int tl = idx / (group * D), hh = (idx / D) % group, cc = idx % D;
        const size_t row = ((size_t)b * a.T + t_lo + tl) * a.Hq + hk * group + hh;
        s_dn[idx] = a.dnum[row * D + cc];
        s_q[idx] = ldf(q + row * D + cc);
      }
      if (MODE == kRevOut) {
        // sum_h q (.) dq as the forward sweep left it, in fp32: against k (.) dk it nearly cancels, and dq rounded
        // to the storage type would not do
        for (int idx = tid; idx < n * D; idx += 256) {
          const size_t row = ((size_t)b * a.T + t_lo + idx / D) * a.Hkv + hk;
          s_dq[idx] = a.gate_local[row * D + idx % D];
        }
      }
      for (int idx = tid; idx < n * group; idx += 256) {
        const size_t row = ((size_t)b * a.T + t_lo + idx / group) * a.Hq + hk * group + idx % group;
        s_dd[idx] = REV ? a.dden[row] : a.den[row];   // the forward sweep forms dden itself, from den
      }
    }
    __syncthreads();
    // ---- the block's tokens, one after the other
    for (int ti = 0; ti < n; ++ti) {
      const int tl = REV ? n - 1 - ti : ti;
      const float al = s_al[tl * D + c], kk = s_k[tl * D + c];
      if (!REV) {
        // S^_t = alpha_t (.) S^_{t-1} + k_t^T v^_t
        xz = fmaf(al, xz, kk);
#pragma unroll
        for (int j = 0; j < CPT; ++j) X[j] = fmaf(al, X[j], kk * s_v[tl * D + j0 + j]);
        decay *= al;
        if (MODE == kFwdOut) {
          // u[c] = S_t[c, :] . dnum;  dden = -(q . u) / den needs all rows: this wave's share goes to LDS, the
          // four are added and dq = u + z dden is formed after the block
          if (tid % TPR == 0) s_dk[tl * D + c] = xz;           // z_t of this row (s_dk is free in this sweep)
          for (int hh = 0; hh < group; ++hh) {
            const float* dn = s_dn + (tl * group + hh) * D + j0;
            float acc = 0.f;
#pragma unroll
            for (int j = 0; j < CPT; ++j) acc = fmaf(X[j], dn[j], acc);
#pragma unroll
            for (int m = TPR / 2; m >= 1; m >>= 1) acc += __shfl_xor(acc, m, TPR);
            float part = 0.f;
            if (tid % TPR == 0) {
              s_dq[(tl * group + hh) * D + c] = acc;
              part = s_q[(tl * group + hh) * D + c] * acc;
            }
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) part += __shfl_xor(part, m, 64);
            if ((tid & 63) == 0) s_gl[(tl * group + hh) * 4 + (tid >> 6)] = part;   // s_gl is free in this sweep
          }
        }
      } else {
        // Gr_t = (what flows in from token t + 1) + sum_h q_t^T d^_t
        for (int hh = 0; hh < group; ++hh) {
          const float qc = s_q[(tl * group + hh) * D + c];
          const float* dn = s_dn + (tl * group + hh) * D + j0;
          xz = fmaf(qc, s_dd[tl * group + hh], xz);
#pragma unroll
          for (int j = 0; j < CPT; ++j) X[j] = fmaf(qc, dn[j], X[j]);
        }
        if (MODE == kRevOut) {
          // dk_t[c] = Gr_t[c, :] . v^_t
          float acc = (tid % TPR == 0) ? xz : 0.f;
          float pv[CPT];
#pragma unroll
          for (int j = 0; j < CPT; ++j) {
            acc = fmaf(X[j], s_v[tl * D + j0 + j], acc);
            pv[j] = kk * X[j];               // this row's share of dv_t
          }
#pragma unroll
          for (int m = TPR / 2; m >= 1; m >>= 1) acc += __shfl_xor(acc, m, TPR);
          // dv_t[col] = sum over the rows: first the rows of this wave (lanes with the same column run) ...
#pragma unroll
          for (int m = TPR; m < 64; m <<= 1) {
#pragma unroll
            for (int j = 0; j < CPT; ++j) pv[j] += __shfl_xor(pv[j], m, 64);
          }
          if ((tid & 63) < TPR) {
#pragma unroll
            for (int j = 0; j < CPT; ++j) s_dv[(tl * 4 + (tid >> 6)) * D + j0 + j] = pv[j];   // ... then the four waves, below
          }
          if (tid % TPR == 0) {
            s_dk[tl * D + c] = acc;
            // the gate term of this token and everything after it in the segment
            gsum += fmaf(-kk, acc, s_dq[tl * D + c]);
            s_gl[tl * D + c] = gsum;
          }
        }
        // what flows on to token t - 1
        xz *= al;
#pragma unroll
        for (int j = 0; j < CPT; ++j) X[j] *= al;
        decay *= al;
      }
    }
    __syncthreads();
    // ---- the block's outputs, whole rows at a time
    if (MODE == kFwdOut) {
      T* dq = static_cast<T*>(a.dq);
      for (int idx = tid; idx < n * D; idx += 256) {
        const int tl = idx / D, cc = idx % D;
        const size_t tok = (size_t)b * a.T + t_lo + tl;
        float qdq = 0.f;
        for (int hh = 0; hh < group; ++hh) {
          const size_t row = tok * a.Hq + hk * group + hh;
          const float* p = s_gl + (tl * group + hh) * 4;
          const float dden = -((p[0] + p[1]) + (p[2] + p[3])) / s_dd[tl * group + hh];
          const float dqv = fmaf(s_dk[tl * D + cc], dden, s_dq[(tl * group + hh) * D + cc]);
          stf(dq + row * D + cc, dqv);
          qdq = fmaf(s_q[(tl * group + hh) * D + cc], dqv, qdq);
          if (cc == 0) a.dden[row] = dden;
        }
        a.gate_local[(tok * a.Hkv + hk) * D + cc] = qdq;   // the query's share of the gate term, for the reverse sweep
      }
    }
    if (MODE == kRevOut) {
      T* dk = static_cast<T*>(a.dk);
      T* dv = static_cast<T*>(a.dv);
      for (int idx = tid; idx < n * D; idx += 256) {
        const int tl = idx / D, cc = idx % D;
        const size_t row = ((size_t)b * a.T + t_lo + tl) * a.Hkv + hk;
        stf(dk + row * D + cc, s_dk[idx]);
        const float* p = s_dv + (tl * 4) * D + cc;
        stf(dv + row * D + cc, (p[0] + p[D]) + (p[2 * D] + p[3 * D]));
        a.gate_local[row * D + cc] = s_gl[idx];
      }
    }
    __syncthreads();
  }

  // ---- what the sweep leaves behind
  if (!OUT) {
    float* slot = (REV ? a.slots_r : a.slots_f) + ((size_t)bh * a.nseg + (REV ? a.nseg - 1 - seg : seg)) * kSlot;
#pragma unroll
    for (int j = 0; j < CPT; ++j) slot[(size_t)c * D + j0 + j] = X[j];
    if (tid % TPR == 0) {
      slot[D * D + c] = xz;
      slot[D * D + D + c] = decay;
    }
  }
  if (MODE == kRevOut) {
    if (tid % TPR == 0) a.gate_tot[((size_t)bh * a.nseg + seg) * D + c] = gsum;
    if (seg == 0) {
      if (a.dS0 != nullptr) {
#pragma unroll
        for (int j = 0; j < CPT; ++j) a.dS0[((size_t)bh * D + c) * D + j0 + j] = X[j];
      }
      if (a.dz0 != nullptr && tid % TPR == 0) a.dz0[(size_t)bh * D + c] = xz;
    }
  }
}

// Contributions -> states at the segment boundaries, in place: slot[i] <- state before segment i (in slot order);
// state <- decay[i] (.) state + contribution[i].  grid (ceil((D*D + D) / 256), heads).
template <int D>
__global__ void __launch_bounds__(256) bwd_scan_kernel(float* __restrict__ slots, const float* __restrict__ S0,
                                                      const float* __restrict__ z0, int nseg) {
  constexpr int kSlot = D * D + 2 * D;
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= D * D + D) return;
  const int bh = blockIdx.y;
  const int c = e < D * D ? e / D : e - D * D;
  float st = 0.f;
  if (e < D * D) { if (S0) st = S0[(size_t)bh * D * D + e]; }
  else if (z0) st = z0[(size_t)bh * D + c];
  float* slot = slots + (size_t)bh * nseg * kSlot;
  constexpr int U = 8;
  for (int s = 0; s < nseg; s += U) {
    float delta[U], dec[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int sg = min(s + u, nseg - 1);
      delta[u] = slot[(size_t)sg * kSlot + e];
      dec[u] = slot[(size_t)sg * kSlot + D * D + D + c];
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (s + u < nseg) {
        slot[(size_t)(s + u) * kSlot + e] = st;
        st = fmaf(dec[u], st, delta[u]);
      }
  }
}

// gate_tot[seg] <- sum of the totals of all later segments.  grid (heads), D threads.
template <int D>
__global__ void bwd_gate_suffix_kernel(float* __restrict__ tot, int nseg) {
  const int bh = blockIdx.x, c = threadIdx.x;
  float* p = tot + (size_t)bh * nseg * D + c;
  float acc = 0.f;
  for (int s = nseg - 1; s >= 0; --s) {
    const float t = p[(size_t)s * D];
    p[(size_t)s * D] = acc;
    acc += t;
  }
}

// dg = (suffix within the segment + all later segments) * gate_scale * (1 - sigmoid(g))
template <typename T, int D>
__global__ void __launch_bounds__(256) bwd_gate_finish_kernel(const T* __restrict__ g, const float* __restrict__ local,
                                                             const float* __restrict__ tot, T* __restrict__ dg, int Tn,
                                                             int Hkv, int seg_len, int nseg, float gate_scale,
                                                             long long total) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int c = (int)(i % D);
  const long long row = i / D;           // (b * T + t) * Hkv + hk
  const int hk = (int)(row % Hkv);
  const long long bt = row / Hkv;
  const int t = (int)(bt % Tn), b = (int)(bt / Tn);
  const int seg = t / seg_len;
  const float later = nseg > 1 ? tot[(((size_t)b * Hkv + hk) * nseg + seg) * D + c] : 0.f;
  const float gl = ldf(g + i);
  const float sg = 1.f / (1.f + expf(-gl));
  stf(dg + i, (local[i] + later) * gate_scale * (1.f - sg));
}

template <typename T, int D>
hipError_t launch_typed(const GlaBackwardParams& p, const BwdArgs& a, hipStream_t stream) {
  const int heads = p.B * p.Hkv;
  const long long nd = (long long)p.B * p.T * p.Hq * D;
  hipLaunchKernelGGL((bwd_prepare_kernel<T, D>), dim3((unsigned)((nd + 255) / 256)), dim3(256), 0, stream, (const T*)p.dO,
                     p.den, a.dnum, nd);
  const size_t lds = (size_t)a.tb * (3 * D + a.group * (3 * D + 1) + 2 * D + 4 * D) * sizeof(float);
  const dim3 grid(a.nseg, heads);
  if (a.nseg > 1) {
    hipLaunchKernelGGL((bwd_pass_kernel<T, D, kFwdContrib>), grid, dim3(256), lds, stream, a);
    hipLaunchKernelGGL((bwd_scan_kernel<D>), dim3((D * D + D + 255) / 256, heads), dim3(256), 0, stream, a.slots_f, p.S0,
                       p.z0, a.nseg);
  }
  hipLaunchKernelGGL((bwd_pass_kernel<T, D, kFwdOut>), grid, dim3(256), lds, stream, a);
  if (a.nseg > 1) {
    hipLaunchKernelGGL((bwd_pass_kernel<T, D, kRevContrib>), grid, dim3(256), lds, stream, a);
    hipLaunchKernelGGL((bwd_scan_kernel<D>), dim3((D * D + D + 255) / 256, heads), dim3(256), 0, stream, a.slots_r,
                       (const float*)nullptr, (const float*)nullptr, a.nseg);
  }
  hipLaunchKernelGGL((bwd_pass_kernel<T, D, kRevOut>), grid, dim3(256), lds, stream, a);
  if (a.nseg > 1) hipLaunchKernelGGL((bwd_gate_suffix_kernel<D>), dim3(heads), dim3(D), 0, stream, a.gate_tot, a.nseg);
  const long long total = (long long)p.B * p.T * p.Hkv * D;
  hipLaunchKernelGGL((bwd_gate_finish_kernel<T, D>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream,
                     (const T*)p.g, a.gate_local, a.gate_tot, (T*)p.dg, p.T, p.Hkv, a.seg_len, a.nseg, p.gate_scale, total);
  return hipGetLastError();
}

}  // namespace

// Tokens staged per block: as many as keep the staging under 48 KB of LDS.
static int backward_block_tokens(int d, int group) {
  const size_t per_token = (size_t)(3 * d + group * (3 * d + 1) + 2 * d + 4 * d) * sizeof(float);
  int tb = (int)(48 * 1024 / per_token);
  return tb > 16 ? 16 : tb;
}

// (the forward sweep parks four partial sums per query head in a row of d floats)
bool gla_backward_supports(int d, int group) { return backward_block_tokens(d, group) >= 1 && group * 4 <= d; }

size_t gla_backward_workspace_bytes(int B, int T, int Hq, int Hkv, int d, int seg_len, int nseg) {
  const size_t rows = (size_t)B * T;
  size_t n = rows * Hq * d + rows * Hq + rows * Hkv * d;           // dnum, dden, gate_local
  n += 2 * (size_t)B * Hkv * nseg * (d * d + 2 * d);               // slots, both directions
  n += (size_t)B * Hkv * nseg * d;                                 // gate totals
  return n * sizeof(float) + 256;
}

hipError_t launch_gla_backward(const GlaBackwardParams& p, hipStream_t stream) {
  BwdArgs a{};
  a.q = p.q; a.k = p.k; a.v = p.v; a.g = p.g; a.dO = p.dO; a.den = p.den; a.S0 = p.S0; a.z0 = p.z0;
  a.dq = p.dq; a.dk = p.dk; a.dv = p.dv; a.dg = p.dg; a.dS0 = p.dS0; a.dz0 = p.dz0;
  a.B = p.B; a.T = p.T; a.Hq = p.Hq; a.Hkv = p.Hkv; a.group = p.Hq / p.Hkv; a.seg_len = p.seg_len; a.nseg = p.nseg;
  a.gate_scale = p.gate_scale; a.eps = p.eps;
  a.tb = backward_block_tokens(p.d, a.group);
  if (a.tb < 1) return hipErrorInvalidValue;
  const size_t rows = (size_t)p.B * p.T;
  float* w = static_cast<float*>(p.workspace);
  a.dnum = w; w += rows * p.Hq * p.d;
  a.dden = w; w += rows * p.Hq;
  a.gate_local = w; w += rows * p.Hkv * p.d;
  a.slots_f = w; w += (size_t)p.B * p.Hkv * p.nseg * (p.d * p.d + 2 * p.d);
  a.slots_r = w; w += (size_t)p.B * p.Hkv * p.nseg * (p.d * p.d + 2 * p.d);
  a.gate_tot = w;
  if (p.bf16) return p.d == 64 ? launch_typed<bf16_t, 64>(p, a, stream) : launch_typed<bf16_t, 128>(p, a, stream);
  return p.d == 64 ? launch_typed<float, 64>(p, a, stream) : launch_typed<float, 128>(p, a, stream);
}

}  // namespace lawcat
