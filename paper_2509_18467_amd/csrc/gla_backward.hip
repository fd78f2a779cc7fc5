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
// through LDS in blocks of up to 8, the next block's loads in flight while the current one is worked on.
// A first version: correct and segment-parallel, several times the forward's time.

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
  float* dden;       // [B,T,Hq]
  float* slots_f;    // [heads][nseg][D*D + 2D]: forward contributions, then start states
  float* slots_r;    // the same for Gr, segments in reverse order
  float* gate_local; // [B,T,Hkv,D]: sum_h q (.) dq, then the suffix sum of the gate term within the segment
  float* gate_tot;   // [heads][nseg][D]: the segment's total, then the sum over all later segments
  int B, T, Hq, Hkv, group, seg_len, nseg;
  float gate_scale;
};

enum { kFwdContrib = 0, kFwdOut = 1, kRevContrib = 2, kRevOut = 3 };

constexpr int pad4(int n) { return (n + 3) & ~3; }

// LDS floats of a sweep that stages TB tokens: alpha | k, v | q, dnum per query head, den or dden per head |
// forward outputs: S dnum^T per head, z, dden | reverse outputs: sum_h q (.) dq, dk, gate suffix, dv of the 4 waves
template <int D, int MODE>
constexpr int lds_floats(int TB, int group) {
  int n = TB * D;
  if (MODE != kRevContrib) n += 2 * TB * D;
  if (MODE != kFwdContrib) n += 2 * TB * group * D + pad4(TB * group);
  if (MODE == kFwdOut) n += TB * group * D + 2 * TB * D;
  if (MODE == kRevOut) n += 3 * TB * D + 4 * TB * D;
  return n;
}

// value of the lane whose index differs in bit 0 / bit 1 (inside a group of four lanes: no LDS traffic)
__device__ inline float lane_xor1(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xF, 0xF, true));
}
__device__ inline float lane_xor2(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xF, 0xF, true));
}
// sum over the TPR adjacent lanes that share a state row
template <int TPR>
__device__ inline float row_sum(float x) {
  x += lane_xor1(x);
  if (TPR == 4) x += lane_xor2(x);
  return x;
}

// Sum over the rows of a wave by recursive halving: with lane stride M a lane hands the half of its columns that
// its partner keeps and adds the partner's half of its own; after the last step a lane holds CNT columns, summed
// over all the wave's rows, starting at column (row within the wave) * CNT of its run.  Fixed order.
template <int CNT, int M, int MSTOP>
__device__ inline void halve_rows(float* pv, int lane) {
  if constexpr (M >= MSTOP) {
    constexpr int H = CNT / 2;
    const bool upper = (lane & M) != 0;
#pragma unroll
    for (int j = 0; j < H; ++j) {
      const float send = upper ? pv[j] : pv[j + H];
      const float keep = upper ? pv[j + H] : pv[j];
      pv[j] = keep + __shfl_xor(send, M, 64);
    }
    halve_rows<H, M / 2, MSTOP>(pv, lane);
  }
}

// grid (nseg, B * Hkv), 256 threads, dynamic LDS.  GR = query heads per kv head (0: read from the arguments, and
// one token per block); EI = ceil(group * D / 256) elements of a token's query heads per thread; 8 / EI tokens
// are staged per block, fetched into registers while the block before is worked on.
template <typename T, int D, int MODE, int GR>
__global__ void __launch_bounds__(256) bwd_pass_kernel(const BwdArgs a) {
  constexpr int TPR = 256 / D;       // threads per state row
  constexpr int CPT = D / TPR;       // value columns per thread
  constexpr int EI = GR ? (GR * D + 255) / 256 : 8;
  constexpr int TB = 8 / EI;         // tokens per block
  constexpr int UH = GR ? GR : 1;    // unroll of the loops over the query heads
  constexpr int KV = (TB * D + 255) / 256;   // elements of k, v, gate per thread and block
  constexpr int FIN = CPT / (64 / TPR);      // columns of dv a lane ends up with
  constexpr bool REV = MODE >= kRevContrib;
  constexpr bool OUT = MODE == kFwdOut || MODE == kRevOut;
  constexpr int kSlot = D * D + 2 * D;
  extern __shared__ __align__(16) float sm[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = tid / TPR, j0 = (tid % TPR) * CPT;
  const int seg = blockIdx.x, bh = blockIdx.y;
  const int b = bh / a.Hkv, hk = bh % a.Hkv;
  const int group = GR ? GR : a.group, gD = group * D;
  const int s0 = seg * a.seg_len, s1 = min(a.T, s0 + a.seg_len);
  // LDS, in the order of lds_floats()
  float* w = sm;
  float* s_al = w; w += TB * D;
  float *s_k = nullptr, *s_v = nullptr, *s_q = nullptr, *s_dn = nullptr, *s_dd = nullptr, *s_dq = nullptr;
  float *s_dk = nullptr, *s_gl = nullptr, *s_dv = nullptr;
  if (MODE != kRevContrib) { s_k = w; w += TB * D; s_v = w; w += TB * D; }
  if (MODE != kFwdContrib) { s_q = w; w += TB * gD; s_dn = w; w += TB * gD; s_dd = w; w += pad4(TB * group); }
  if (MODE == kFwdOut) { s_dq = w; w += TB * gD; s_dk = w; w += TB * D; s_gl = w; }   // S dnum^T | z_t | dden
  if (MODE == kRevOut) { s_dq = w; w += TB * D; s_dk = w; w += TB * D; s_gl = w; w += TB * D; s_dv = w; }

  const T* q = static_cast<const T*>(a.q);
  const T* k = static_cast<const T*>(a.k);
  const T* v = static_cast<const T*>(a.v);
  const T* g = static_cast<const T*>(a.g);
  const T* dO = static_cast<const T*>(a.dO);

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

  // ---- a block's inputs, first into registers (fetch), a block later into LDS (stash)
  float pg[KV], pk[KV], pv_[KV], pqd[KV], pq[TB * EI], pdo[TB * EI], pden[TB * EI], pdd = 0.f;
  const int ddt = tid / group, ddh = tid - ddt * group;      // (token, head) of this thread's den / dden element
  auto fetch = [&](int blk) {
    const int t_lo = s0 + blk * TB;
    const int n = min(TB, s1 - t_lo);
#pragma unroll
    for (int i = 0; i < KV; ++i) {
      const int idx = i * 256 + tid;
      if (idx < n * D) {
        const size_t at = (((size_t)b * a.T + t_lo + idx / D) * a.Hkv + hk) * D + idx % D;
        pg[i] = ldf(g + at);
        if (MODE != kRevContrib) {
          pk[i] = ldf(k + at);
          pv_[i] = ldf(v + at);
        }
        if (MODE == kRevOut) pqd[i] = a.gate_local[at];
      }
    }
    if (MODE != kFwdContrib) {
#pragma unroll
      for (int tl = 0; tl < TB; ++tl) {
        if (tl < n) {
          const size_t row0 = ((size_t)b * a.T + t_lo + tl) * a.Hq + (size_t)hk * group;
#pragma unroll
          for (int e = 0; e < EI; ++e) {
            const int el = e * 256 + tid;
            if (el < gD) {
              pq[tl * EI + e] = ldf(q + row0 * D + el);
              pdo[tl * EI + e] = ldf(dO + row0 * D + el);
              pden[tl * EI + e] = a.den[row0 + el / D];
            }
          }
        }
      }
      if (tid < n * group) {
        const size_t row = ((size_t)b * a.T + t_lo + ddt) * a.Hq + hk * group + ddh;
        pdd = REV ? a.dden[row] : a.den[row];   // the forward sweep forms dden itself, from den
      }
    }
  };
  auto stash = [&](int n) {
#pragma unroll
    for (int i = 0; i < KV; ++i) {
      const int idx = i * 256 + tid;
      if (idx < n * D) {
        s_al[idx] = a.gate_scale == 1.0f ? __frcp_rn(1.f + __expf(-pg[i])) : expf(a.gate_scale * log_sigmoid(pg[i]));
        if (MODE != kRevContrib) {
          s_k[idx] = pk[i];
          s_v[idx] = pv_[i];
        }
        // sum_h q (.) dq as the forward sweep left it, in fp32: against k (.) dk it nearly cancels, and dq rounded
        // to the storage type would not do
        if (MODE == kRevOut) s_dq[idx] = pqd[i];
      }
    }
    if (MODE != kFwdContrib) {
#pragma unroll
      for (int tl = 0; tl < TB; ++tl) {
        if (tl < n) {
#pragma unroll
          for (int e = 0; e < EI; ++e) {
            const int el = e * 256 + tid;
            if (el < gD) {
              s_q[tl * gD + el] = pq[tl * EI + e];
              s_dn[tl * gD + el] = pdo[tl * EI + e] * __frcp_rn(pden[tl * EI + e]);     // dnum = dO / den
            }
          }
        }
      }
      if (tid < n * group) s_dd[tid] = pdd;
    }
  };

  const int len = s1 - s0;
  const int nblk = (len + TB - 1) / TB;
  if (nblk > 0) fetch(REV ? nblk - 1 : 0);
  for (int bi = 0; bi < nblk; ++bi) {
    const int blk = REV ? nblk - 1 - bi : bi;
    const int t_lo = s0 + blk * TB;
    const int n = min(TB, s1 - t_lo);
    stash(n);
    __syncthreads();
    if (bi + 1 < nblk) fetch(REV ? blk - 1 : blk + 1);
    // ---- the block's tokens, one after the other
    for (int ti = 0; ti < n; ++ti) {
      const int tl = REV ? n - 1 - ti : ti;
      const float al = s_al[tl * D + c];
      if (!REV) {
        // S^_t = alpha_t (.) S^_{t-1} + k_t^T v^_t
        const float kk = s_k[tl * D + c];
        const float4* v4 = reinterpret_cast<const float4*>(s_v + tl * D + j0);
        xz = fmaf(al, xz, kk);
#pragma unroll
        for (int j = 0; j < CPT / 4; ++j) {
          const float4 vv = v4[j];
          X[4 * j + 0] = fmaf(al, X[4 * j + 0], kk * vv.x);
          X[4 * j + 1] = fmaf(al, X[4 * j + 1], kk * vv.y);
          X[4 * j + 2] = fmaf(al, X[4 * j + 2], kk * vv.z);
          X[4 * j + 3] = fmaf(al, X[4 * j + 3], kk * vv.w);
        }
        decay *= al;
        if (MODE == kFwdOut) {
          // u[c] = S_t[c, :] . dnum;  dden = -(q . u) / den needs all rows: formed after the block, and then
          // dq = u + z dden
          if (tid % TPR == 0) s_dk[tl * D + c] = xz;           // z_t of this row
#pragma unroll UH
          for (int hh = 0; hh < group; ++hh) {
            const float4* dn = reinterpret_cast<const float4*>(s_dn + (tl * group + hh) * D + j0);
            float acc = 0.f;
#pragma unroll
            for (int j = 0; j < CPT / 4; ++j) {
              const float4 d4 = dn[j];
              acc = fmaf(X[4 * j + 0], d4.x, acc);
              acc = fmaf(X[4 * j + 1], d4.y, acc);
              acc = fmaf(X[4 * j + 2], d4.z, acc);
              acc = fmaf(X[4 * j + 3], d4.w, acc);
            }
            acc = row_sum<TPR>(acc);
            if (tid % TPR == 0) s_dq[(tl * group + hh) * D + c] = acc;
          }
        }
      } else {
        // Gr_t = (what flows in from token t + 1) + sum_h q_t^T d^_t
#pragma unroll UH
        for (int hh = 0; hh < group; ++hh) {
          const float qc = s_q[(tl * group + hh) * D + c];
          const float4* dn = reinterpret_cast<const float4*>(s_dn + (tl * group + hh) * D + j0);
          xz = fmaf(qc, s_dd[tl * group + hh], xz);
#pragma unroll
          for (int j = 0; j < CPT / 4; ++j) {
            const float4 d4 = dn[j];
            X[4 * j + 0] = fmaf(qc, d4.x, X[4 * j + 0]);
            X[4 * j + 1] = fmaf(qc, d4.y, X[4 * j + 1]);
            X[4 * j + 2] = fmaf(qc, d4.z, X[4 * j + 2]);
            X[4 * j + 3] = fmaf(qc, d4.w, X[4 * j + 3]);
          }
        }
        if (MODE == kRevOut) {
          // dk_t[c] = Gr_t[c, :] . v^_t
          const float kk = s_k[tl * D + c];
          const float4* v4 = reinterpret_cast<const float4*>(s_v + tl * D + j0);
          float acc = (tid % TPR == 0) ? xz : 0.f;
          float pv[CPT];
#pragma unroll
          for (int j = 0; j < CPT / 4; ++j) {
            const float4 vv = v4[j];
            acc = fmaf(X[4 * j + 0], vv.x, acc);
            acc = fmaf(X[4 * j + 1], vv.y, acc);
            acc = fmaf(X[4 * j + 2], vv.z, acc);
            acc = fmaf(X[4 * j + 3], vv.w, acc);
          }
#pragma unroll
          for (int j = 0; j < CPT; ++j) pv[j] = kk * X[j];               // this row's share of dv_t
          acc = row_sum<TPR>(acc);
          // dv_t[col] = sum over the rows: first the rows of this wave, then the four waves (below)
          halve_rows<CPT, 32, TPR>(pv, lane);
#pragma unroll
          for (int f = 0; f < FIN; ++f) s_dv[(tl * 4 + wave) * D + j0 + (lane / TPR) * FIN + f] = pv[f];
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
      // dden of every (token, head) of the block (at most 32 pairs): eight threads per pair, each over every
      // eighth key channel (rotated by the pair, so that the pairs of a wave read different banks)
      {
        const int p = tid >> 3, r = tid & 7;
        float part = 0.f;
        if (p < n * group) {
#pragma unroll
          for (int i = 0; i < D / 8; ++i) {
            const int ch = (r + 8 * i + 8 * p) & (D - 1);
            part = fmaf(s_q[p * D + ch], s_dq[p * D + ch], part);
          }
        }
        part += lane_xor1(part);
        part += lane_xor2(part);
        part += __shfl_xor(part, 4, 64);
        if (r == 0 && p < n * group) s_gl[p] = -part / s_dd[p];
      }
      __syncthreads();
      T* dq = static_cast<T*>(a.dq);
      for (int idx = tid; idx < n * D; idx += 256) {
        const int tl = idx / D, cc = idx % D;
        const size_t tok = (size_t)b * a.T + t_lo + tl;
        float qdq = 0.f;
#pragma unroll UH
        for (int hh = 0; hh < group; ++hh) {
          const size_t row = tok * a.Hq + hk * group + hh;
          const float dden = s_gl[tl * group + hh];
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

// gate_tot[seg] <- sum of the totals of all later segments.  grid (heads), D threads.  The loads do not depend
// on the running sum: eight are issued at a time.
template <int D>
__global__ void bwd_gate_suffix_kernel(float* __restrict__ tot, int nseg) {
  const int bh = blockIdx.x, c = threadIdx.x;
  float* p = tot + (size_t)bh * nseg * D + c;
  float acc = 0.f;
  constexpr int U = 8;
  for (int s1 = nseg; s1 > 0; s1 -= U) {
    float t[U];
#pragma unroll
    for (int u = 0; u < U; ++u) t[u] = s1 - 1 - u >= 0 ? p[(size_t)(s1 - 1 - u) * D] : 0.f;
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (s1 - 1 - u >= 0) {
        p[(size_t)(s1 - 1 - u) * D] = acc;
        acc += t[u];
      }
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

template <typename T, int D, int GR>
hipError_t launch_sized(const GlaBackwardParams& p, const BwdArgs& a, hipStream_t stream) {
  constexpr int TB = GR ? 8 / ((GR * D + 255) / 256) : 1;
  const int heads = p.B * p.Hkv;
  const dim3 grid(a.nseg, heads);
  const auto bytes = [&](int floats) { return (size_t)floats * sizeof(float); };
  if (a.nseg > 1) {
    hipLaunchKernelGGL((bwd_pass_kernel<T, D, kFwdContrib, GR>), grid, dim3(256), bytes(lds_floats<D, kFwdContrib>(TB, a.group)),
                       stream, a);
    hipLaunchKernelGGL((bwd_scan_kernel<D>), dim3((D * D + D + 255) / 256, heads), dim3(256), 0, stream, a.slots_f, p.S0,
                       p.z0, a.nseg);
  }
  hipLaunchKernelGGL((bwd_pass_kernel<T, D, kFwdOut, GR>), grid, dim3(256), bytes(lds_floats<D, kFwdOut>(TB, a.group)), stream, a);
  if (a.nseg > 1) {
    hipLaunchKernelGGL((bwd_pass_kernel<T, D, kRevContrib, GR>), grid, dim3(256), bytes(lds_floats<D, kRevContrib>(TB, a.group)),
                       stream, a);
    hipLaunchKernelGGL((bwd_scan_kernel<D>), dim3((D * D + D + 255) / 256, heads), dim3(256), 0, stream, a.slots_r,
                       (const float*)nullptr, (const float*)nullptr, a.nseg);
  }
  hipLaunchKernelGGL((bwd_pass_kernel<T, D, kRevOut, GR>), grid, dim3(256), bytes(lds_floats<D, kRevOut>(TB, a.group)), stream, a);
  if (a.nseg > 1) hipLaunchKernelGGL((bwd_gate_suffix_kernel<D>), dim3(heads), dim3(D), 0, stream, a.gate_tot, a.nseg);
  const long long total = (long long)p.B * p.T * p.Hkv * D;
  hipLaunchKernelGGL((bwd_gate_finish_kernel<T, D>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream,
                     (const T*)p.g, a.gate_local, a.gate_tot, (T*)p.dg, p.T, p.Hkv, a.seg_len, a.nseg, p.gate_scale, total);
  return hipGetLastError();
}

template <typename T, int D>
hipError_t launch_typed(const GlaBackwardParams& p, const BwdArgs& a, hipStream_t stream) {
  switch (a.group) {
    case 1: return launch_sized<T, D, 1>(p, a, stream);
    case 2: return launch_sized<T, D, 2>(p, a, stream);
    case 4: return launch_sized<T, D, 4>(p, a, stream);
    case 8: return launch_sized<T, D, 8>(p, a, stream);
    default: return launch_sized<T, D, 0>(p, a, stream);     // any other group: one token per block
  }
}

}  // namespace

// A token's query heads are staged by 256 threads in at most 8 rounds; dden of a block's (token, head) pairs must
// fit one LDS row of d floats per token.
bool gla_backward_supports(int d, int group) { return group * d <= 2048 && group <= d; }

// Segments of the sequence: about four workgroups per compute unit over all (batch, kv head) pairs (what the
// output sweeps' registers and LDS allow to be resident), segments a multiple of 64 tokens.
void gla_backward_plan(int B, int T, int Hkv, int* seg_len, int* nseg) {
  const long long heads = (long long)B * Hkv;
  long long want = 1024 / heads;                 // segments per head
  if (want < 1) want = 1;
  long long len = (T + want - 1) / want;
  len = (len + 63) / 64 * 64;
  *seg_len = (int)len;
  *nseg = (int)((T + len - 1) / len);
}

size_t gla_backward_workspace_bytes(int B, int T, int Hq, int Hkv, int d) {
  int seg_len, nseg;
  gla_backward_plan(B, T, Hkv, &seg_len, &nseg);
  const size_t rows = (size_t)B * T;
  size_t n = rows * Hq + rows * Hkv * d;                           // dden, gate term
  n += 2 * (size_t)B * Hkv * nseg * (d * d + 2 * d);               // segment states, both directions
  n += (size_t)B * Hkv * nseg * d;                                 // gate totals
  return n * sizeof(float) + 256;
}

hipError_t launch_gla_backward(const GlaBackwardParams& p, hipStream_t stream) {
  BwdArgs a{};
  a.q = p.q; a.k = p.k; a.v = p.v; a.g = p.g; a.dO = p.dO; a.den = p.den; a.S0 = p.S0; a.z0 = p.z0;
  a.dq = p.dq; a.dk = p.dk; a.dv = p.dv; a.dg = p.dg; a.dS0 = p.dS0; a.dz0 = p.dz0;
  a.B = p.B; a.T = p.T; a.Hq = p.Hq; a.Hkv = p.Hkv; a.group = p.Hq / p.Hkv;
  a.gate_scale = p.gate_scale;
  gla_backward_plan(p.B, p.T, p.Hkv, &a.seg_len, &a.nseg);
  if (!gla_backward_supports(p.d, a.group)) return hipErrorInvalidValue;
  const size_t rows = (size_t)p.B * p.T;
  float* w = static_cast<float*>(p.workspace);
  a.dden = w; w += rows * p.Hq;
  a.gate_local = w; w += rows * p.Hkv * p.d;
  a.slots_f = w; w += (size_t)p.B * p.Hkv * a.nseg * (p.d * p.d + 2 * p.d);
  a.slots_r = w; w += (size_t)p.B * p.Hkv * a.nseg * (p.d * p.d + 2 * p.d);
  a.gate_tot = w;
  if (p.bf16) return p.d == 64 ? launch_typed<bf16_t, 64>(p, a, stream) : launch_typed<bf16_t, 128>(p, a, stream);
  return p.d == 64 ? launch_typed<float, 64>(p, a, stream) : launch_typed<float, 128>(p, a, stream);
}

}  // namespace lawcat
