// bf16 matrix-core prefill of the normalized gated linear attention (paper section 4.2)
// with the causal depthwise Conv1D of section 4.1 and the pointwise feature map fused into
// the load stage.
//
// Algebra.  Split the sum over i in the state/output equations of section 4.2 at the start
// of a 16-token chunk.  With E_t = prod of alpha over the chunk's tokens up to t (per key
// channel) the output of token t in the chunk is
//   num_t = (q_t (.) E_t) S_start + sum_{i<=t} [(q_t (.) E_t) . (k_i / E_i)] v_i
//   den_t = (q_t (.) E_t) z_start + sum_{i<=t} [(q_t (.) E_t) . (k_i / E_i)]
// and the state after the chunk is S_end = diag(E_last) S_start + sum_i (k_i E_last/E_i)^T v_i.
// All four products are bf16 MFMAs with fp32 accumulation.  The normalizer rides along as 16
// extra value columns that are all ones, so num and den come out of the same MFMAs and the
// division needs no cross-lane traffic.
//
// Parallel decomposition.  One 256-thread workgroup owns one (batch, kv head) and one
// segment of the sequence, and walks it 16 tokens at a time with the [dk x (dv+16)] state in
// MFMA accumulators; the query heads of the group share k, v, the decay and the state.  With
// more than one segment a first pass computes each segment's state contribution and total
// decay, a small scan turns them into segment start states, and the output pass starts from
// those.
//
// Per-step decay is floored at 2^-7.5 so that a chunk's 1/E stays below 2^120.
#include "kernels.h"

namespace lawcat {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kAlphaMin = 0.005524271728019903f;  // 2^-7.5
constexpr float kInvAlphaMax = 181.01933598375618f;  // 2^7.5
constexpr int kChunk = 16;

hipEvent_t g_ev_before = nullptr, g_ev_after = nullptr;

struct ChunkArgs {
  const bf16_t *q, *k, *v, *g, *wq, *wk, *q_halo, *k_halo;
  const float *S0, *z0;
  bf16_t* o;
  float* den_out;
  float* S_out;
  float* z_out;
  float* ws;
  int B, T, Hq, Hkv, W, phi;
  int seg_len, nseg;
  float gate_scale, eps;
};

template <int D, int GR>
struct Geo {
  static constexpr int CH = D / 64;          // 64-channel slabs per row = waves per 16-token chunk in the load stage
  static constexpr int NTG = 4096 / D;       // tokens per granule (one load stage of the workgroup)
  static constexpr int MCG = NTG / kChunk;   // chunks per granule
  static constexpr int RT = D / 16;          // 16-row tiles of the state (key channels)
  static constexpr int CT = D / 64;          // value-column tiles owned by a wave
  static constexpr int NT = CT + 1;          // plus the normalizer tile
  static constexpr int KS = D / 32;          // k-steps of a 16x16x32 MFMA over the key channels
  static constexpr int QRS = D * 2 + 8;      // LDS row stride (bytes) of token-major bf16 rows
  static constexpr int TRS = NTG * 2 + 8;    // LDS row stride (bytes) of channel-major bf16 rows
  static constexpr int kQp = 0;
  static constexpr int kKp = kQp + GR * NTG * QRS;
  static constexpr int kKd = kKp + NTG * QRS;
  static constexpr int kVt = kKd + D * TRS;
  static constexpr int kEb = kVt + D * TRS;
  static constexpr int kWl = kEb + MCG * D * 4;
  static constexpr int kBytes = kWl + (GR + 1) * D * 16;
  static constexpr int kSlot = D * D + 2 * D;  // floats per workspace slot: S | z | decay
};

__device__ inline float bf_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ inline float bf_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }
__device__ inline uint32_t pack2(float a, float b) {
  bf16x2 v = {(__bf16)a, (__bf16)b};  // v_cvt_pk_bf16_f32, round to nearest even
  return __builtin_bit_cast(uint32_t, v);
}
__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ inline float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }
__device__ inline float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

__device__ inline float feature(float y, int phi) {
  if (phi == 1) return y > 0.f ? 1.f + y : fast_exp2(y * kLog2e);
  return y;
}

// Raw rows tok0-3 .. tok0+7 of two adjacent channels (one dword each) of one head.
// Rows before the sequence come from the halo (or are zero); rows at or past T are zero.
template <bool FUSE>
__device__ inline void load_rows(const bf16_t* __restrict__ x, const bf16_t* __restrict__ halo, int b, int T,
                                 int H, int head, int D, int c0, int tok0, int W, uint32_t (&raw)[11]) {
  const size_t rowlen = (size_t)H * D;
  const size_t col = (size_t)head * D + c0;
#pragma unroll
  for (int j = 0; j < 11; ++j) {
    if (!FUSE && j < 3) { raw[j] = 0u; continue; }
    const int tok = tok0 - 3 + j;
    uint32_t r = 0u;
    if (tok >= 0) {
      if (tok < T) r = *reinterpret_cast<const uint32_t*>(x + ((size_t)b * T + tok) * rowlen + col);
    } else if (FUSE && halo != nullptr && tok >= -(W - 1)) {
      r = *reinterpret_cast<const uint32_t*>(halo + ((size_t)b * (W - 1) + (W - 1 + tok)) * rowlen + col);
    }
    raw[j] = r;
  }
}

// conv (section 4.1 sum over delta) + feature map on the 8 tokens x 2 channels of a patch.
template <bool FUSE>
__device__ inline void conv_phi(const uint32_t (&raw)[11], const float* wts /*[2][4] in LDS*/, int phi,
                                float (&y)[8][2]) {
  if (FUSE) {
    const floatx4 w0 = *reinterpret_cast<const floatx4*>(wts);
    const floatx4 w1 = *reinterpret_cast<const floatx4*>(wts + 4);
    float x0[11], x1[11];
#pragma unroll
    for (int j = 0; j < 11; ++j) { x0[j] = bf_lo(raw[j]); x1[j] = bf_hi(raw[j]); }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float a0 = w0[0] * x0[i + 3];
      a0 = fmaf(w0[1], x0[i + 2], a0); a0 = fmaf(w0[2], x0[i + 1], a0); a0 = fmaf(w0[3], x0[i], a0);
      float a1 = w1[0] * x1[i + 3];
      a1 = fmaf(w1[1], x1[i + 2], a1); a1 = fmaf(w1[2], x1[i + 1], a1); a1 = fmaf(w1[3], x1[i], a1);
      y[i][0] = feature(a0, phi);
      y[i][1] = feature(a1, phi);
    }
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) { y[i][0] = bf_lo(raw[i + 3]); y[i][1] = bf_hi(raw[i + 3]); }
  }
}

template <int D, int GR, bool FUSE, bool OUTPUT>
__global__ void __launch_bounds__(256) gla_chunk_kernel(const ChunkArgs a) {
  using G = Geo<D, GR>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x;
  const int w = tid >> 6;   // wave
  const int l = tid & 63;   // lane
  const int g4 = l >> 4;    // MFMA lane group
  const int n = l & 15;     // MFMA row/column within a tile
  const int seg = blockIdx.x;
  const int bh = blockIdx.y;
  const int b = bh / a.Hkv, hk = bh % a.Hkv;
  const int T = a.T;
  const int s0 = seg * a.seg_len;
  const int s1 = min(T, s0 + a.seg_len);

  // load-stage patch of this thread: 8 tokens x 2 channels
  const int cp = l & 31, th = l >> 5;
  const int mcw = w / G::CH;                       // chunk of the granule this wave loads
  const int c0 = 64 * (w % G::CH) + 2 * cp;        // first of the two channels
  const int tl0 = kChunk * mcw + 8 * th;           // first token of the patch within the granule

  float* wl = reinterpret_cast<float*>(smem + G::kWl);
  if (FUSE) {
    // conv weights as fp32 [head][channel][4 taps], taps beyond W zero; row GR is the key head
    for (int e = tid; e < (GR + 1) * D * 4; e += 256) {
      const int dl = e & 3, c = (e >> 2) % D, hh = e / (4 * D);
      float val = 0.f;
      if (dl < a.W) {
        const bf16_t* src = hh < GR ? a.wq + ((size_t)(hk * GR + hh) * D + c) * a.W + dl
                                    : a.wk + ((size_t)hk * D + c) * a.W + dl;
        val = __uint_as_float((uint32_t)(*src) << 16);
      }
      wl[e] = (OUTPUT || hh == GR) ? val : 0.f;
    }
  }

  // ---- state in accumulators: Sacc[rt][ct][i] = S[16 rt + 4 g4 + i][16 tile(ct) + n]; ct == CT holds z replicated
  floatx4 Sacc[G::RT][G::NT];
  {
    const float* Sin = nullptr;
    const float* zin = nullptr;
    if (OUTPUT) {
      if (a.nseg > 1) {
        Sin = a.ws + ((size_t)bh * a.nseg + seg) * G::kSlot;
        zin = Sin + D * D;
      } else if (a.S0 != nullptr) {
        Sin = a.S0 + (size_t)bh * D * D;
      }
      if (a.nseg == 1 && a.z0 != nullptr) zin = a.z0 + (size_t)bh * D;
    }
#pragma unroll
    for (int rt = 0; rt < G::RT; ++rt) {
#pragma unroll
      for (int ct = 0; ct < G::NT; ++ct) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int c = 16 * rt + 4 * g4 + i;
          float val = 0.f;
          if (ct < G::CT) {
            if (Sin) val = Sin[(size_t)c * D + 16 * (w * G::CT + ct) + n];
          } else {
            if (zin) val = zin[c];
          }
          Sacc[rt][ct][i] = val;
        }
      }
    }
  }
  float dprod[G::RT][4];  // running product of the decay over the segment (first pass only)
#pragma unroll
  for (int rt = 0; rt < G::RT; ++rt)
#pragma unroll
    for (int i = 0; i < 4; ++i) dprod[rt][i] = 1.f;

  const bool gs1 = a.gate_scale == 1.0f;
  __syncthreads();

  for (int t0 = s0; t0 < s1; t0 += G::NTG) {
    // =========================== load stage: HBM -> registers -> LDS operands ===========================
    const int tok0 = t0 + tl0;
    float E[8][2];
    {
      // ---- gate logits -> alpha, 1/alpha; running products over the chunk
      uint32_t graw[11];
      load_rows<false>(a.g, nullptr, b, T, a.Hkv, hk, D, c0, tok0, 1, graw);
      float IE[8][2];
      float run[2] = {1.f, 1.f}, irun[2] = {1.f, 1.f};
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const bool valid = tok0 + i < s1;
#pragma unroll
        for (int ch = 0; ch < 2; ++ch) {
          const float gl = ch ? bf_hi(graw[i + 3]) : bf_lo(graw[i + 3]);
          const float u = fminf(fast_exp2(-kLog2e * gl), 1e30f);  // exp(-g)
          float al, ia;
          if (gs1) {
            ia = fminf(1.f + u, kInvAlphaMax);  // 1/sigmoid(g) = 1 + exp(-g)
            al = fmaxf(fast_rcp(1.f + u), kAlphaMin);
          } else {
            const float a2 = fmaxf(-a.gate_scale * fast_log2(1.f + u), -7.5f);
            al = fast_exp2(a2);
            ia = fast_exp2(-a2);
          }
          if (!valid) { al = 1.f; ia = 1.f; }
          run[ch] *= al;
          irun[ch] *= ia;
          E[i][ch] = run[ch];
          IE[i][ch] = irun[ch];
        }
      }
      // the other half of the chunk lives 32 lanes away
      float pre[2], ipre[2], btot[2];
#pragma unroll
      for (int ch = 0; ch < 2; ++ch) {
        const float ot = __shfl_xor(run[ch], 32);
        const float oit = __shfl_xor(irun[ch], 32);
        pre[ch] = th ? ot : 1.f;
        ipre[ch] = th ? oit : 1.f;
        btot[ch] = th ? ot * run[ch] : run[ch] * ot;  // first-half product times second-half product
      }
      // ---- keys: conv + phi, then K' = k/E (for the in-chunk scores) and Kdec = k E_last/E (state update)
      uint32_t kraw[11];
      load_rows<FUSE>(a.k, a.k_halo, b, T, a.Hkv, hk, D, c0, tok0, a.W, kraw);
      float kf[8][2];
      conv_phi<FUSE>(kraw, wl + ((size_t)GR * D + c0) * 4, a.phi, kf);
      uint32_t kd0[4], kd1[4];
      unsigned char* kp = smem + G::kKp + tl0 * G::QRS + c0 * 2;
      float kdv[8][2];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const bool valid = tok0 + i < s1;
#pragma unroll
        for (int ch = 0; ch < 2; ++ch) {
          E[i][ch] *= pre[ch];
          const float kk = valid ? kf[i][ch] : 0.f;
          const float kprime = kk * (IE[i][ch] * ipre[ch]);
          kf[i][ch] = kprime;
          kdv[i][ch] = kprime * btot[ch];
        }
        if (OUTPUT) *reinterpret_cast<uint32_t*>(kp + i * G::QRS) = pack2(kf[i][0], kf[i][1]);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        kd0[i] = pack2(kdv[2 * i][0], kdv[2 * i + 1][0]);
        kd1[i] = pack2(kdv[2 * i][1], kdv[2 * i + 1][1]);
      }
      unsigned char* kdp = smem + G::kKd + c0 * G::TRS + tl0 * 2;
      // rows are 8-byte, not 16-byte, aligned (odd multiples of the padded stride): 8-byte writes
      *reinterpret_cast<uint2*>(kdp) = make_uint2(kd0[0], kd0[1]);
      *reinterpret_cast<uint2*>(kdp + 8) = make_uint2(kd0[2], kd0[3]);
      *reinterpret_cast<uint2*>(kdp + G::TRS) = make_uint2(kd1[0], kd1[1]);
      *reinterpret_cast<uint2*>(kdp + G::TRS + 8) = make_uint2(kd1[2], kd1[3]);
      if (th == 0) {
        float* eb = reinterpret_cast<float*>(smem + G::kEb) + mcw * D + c0;
        *reinterpret_cast<float2*>(eb) = make_float2(btot[0], btot[1]);
      }
      // ---- values, transposed to channel-major
      uint32_t vraw[11];
      load_rows<false>(a.v, nullptr, b, T, a.Hkv, hk, D, c0, tok0, 1, vraw);
      uint32_t v0[4], v1[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint32_t ra = (tok0 + 2 * i < s1) ? vraw[3 + 2 * i] : 0u;
        const uint32_t rb = (tok0 + 2 * i + 1 < s1) ? vraw[4 + 2 * i] : 0u;
        v0[i] = (ra & 0xffffu) | (rb << 16);
        v1[i] = (ra >> 16) | (rb & 0xffff0000u);
      }
      unsigned char* vp = smem + G::kVt + c0 * G::TRS + tl0 * 2;
      *reinterpret_cast<uint2*>(vp) = make_uint2(v0[0], v0[1]);
      *reinterpret_cast<uint2*>(vp + 8) = make_uint2(v0[2], v0[3]);
      *reinterpret_cast<uint2*>(vp + G::TRS) = make_uint2(v1[0], v1[1]);
      *reinterpret_cast<uint2*>(vp + G::TRS + 8) = make_uint2(v1[2], v1[3]);
    }
    if (OUTPUT) {
      // ---- queries: conv + phi, times E
#pragma unroll 1
      for (int hh = 0; hh < GR; ++hh) {
        uint32_t qraw[11];
        load_rows<FUSE>(a.q, a.q_halo, b, T, a.Hq, hk * GR + hh, D, c0, tok0, a.W, qraw);
        float qf[8][2];
        conv_phi<FUSE>(qraw, wl + ((size_t)hh * D + c0) * 4, a.phi, qf);
        unsigned char* qp = smem + G::kQp + (hh * G::NTG + tl0) * G::QRS + c0 * 2;
#pragma unroll
        for (int i = 0; i < 8; ++i)
          *reinterpret_cast<uint32_t*>(qp + i * G::QRS) = pack2(qf[i][0] * E[i][0], qf[i][1] * E[i][1]);
      }
    }
    __syncthreads();

    // =========================== MFMA stage: 16 tokens at a time ===========================
#pragma unroll 1
    for (int mc = 0; mc < G::MCG; ++mc) {
      const int tq = t0 + kChunk * mc;  // first token of the chunk
      if (tq >= s1) break;
      // value fragments: lane (g4, n) holds V[tok 4 g4 .. +3][dv 16 tile + n]; serves as A (V^T) and as B (V)
      short4v vfrag[G::NT];
#pragma unroll
      for (int ct = 0; ct < G::CT; ++ct) {
        const uint2 r = *reinterpret_cast<const uint2*>(smem + G::kVt + (16 * (w * G::CT + ct) + n) * G::TRS +
                                                        (kChunk * mc + 4 * g4) * 2);
        vfrag[ct] = __builtin_bit_cast(short4v, r);
      }
      vfrag[G::CT] = short4v{0x3F80, 0x3F80, 0x3F80, 0x3F80};  // ones: the normalizer columns

      if (OUTPUT) {
        // key fragments of the score product
        bf16x8 ka[G::KS];
#pragma unroll
        for (int ks = 0; ks < G::KS; ++ks) {
          const unsigned char* p = smem + G::kKp + (kChunk * mc + n) * G::QRS + (32 * ks + 4 * g4) * 2;
          const uint2 lo = *reinterpret_cast<const uint2*>(p);
          const uint2 hi = *reinterpret_cast<const uint2*>(p + 32);
          ka[ks] = __builtin_bit_cast(bf16x8, make_uint4(lo.x, lo.y, hi.x, hi.y));
        }
        // state as bf16 A-fragments: rows = value columns, k = key channels {4 g4 + i, 16 + 4 g4 + i} of each 32
        bf16x8 sa[G::NT][G::KS];
#pragma unroll
        for (int ct = 0; ct < G::NT; ++ct)
#pragma unroll
          for (int ks = 0; ks < G::KS; ++ks) {
            const floatx4 lo = Sacc[2 * ks][ct], hi = Sacc[2 * ks + 1][ct];
            sa[ct][ks] = __builtin_bit_cast(
                bf16x8, make_uint4(pack2(lo[0], lo[1]), pack2(lo[2], lo[3]), pack2(hi[0], hi[1]), pack2(hi[2], hi[3])));
          }
#pragma unroll 1
        for (int hh = 0; hh < GR; ++hh) {
          bf16x8 qb[G::KS];
#pragma unroll
          for (int ks = 0; ks < G::KS; ++ks) {
            const unsigned char* p =
                smem + G::kQp + (hh * G::NTG + kChunk * mc + n) * G::QRS + (32 * ks + 4 * g4) * 2;
            const uint2 lo = *reinterpret_cast<const uint2*>(p);
            const uint2 hi = *reinterpret_cast<const uint2*>(p + 32);
            qb[ks] = __builtin_bit_cast(bf16x8, make_uint4(lo.x, lo.y, hi.x, hi.y));
          }
          // P^T[key 4 g4 + i][query n]
          floatx4 pt = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int ks = 0; ks < G::KS; ++ks) pt = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[ks], qb[ks], pt, 0, 0, 0);
#pragma unroll
          for (int i = 0; i < 4; ++i) pt[i] = (4 * g4 + i <= n) ? pt[i] : 0.f;  // causal: key <= query
          // The weights of the few nearest keys dominate the output, so their bf16 rounding would not
          // average out: carry P as a bf16 pair (high part + residual), two small MFMAs instead of one.
          const uint32_t ph0 = pack2(pt[0], pt[1]), ph1 = pack2(pt[2], pt[3]);
          const short4v pb = __builtin_bit_cast(short4v, make_uint2(ph0, ph1));
          const short4v pl = __builtin_bit_cast(
              short4v, make_uint2(pack2(pt[0] - bf_lo(ph0), pt[1] - bf_hi(ph0)), pack2(pt[2] - bf_lo(ph1), pt[3] - bf_hi(ph1))));
          floatx4 oacc[G::NT];
#pragma unroll
          for (int ct = 0; ct < G::NT; ++ct) {
            floatx4 acc = {0.f, 0.f, 0.f, 0.f};
            acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vfrag[ct], pl, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vfrag[ct], pb, acc, 0, 0, 0);
#pragma unroll
            for (int ks = 0; ks < G::KS; ++ks)
              acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(sa[ct][ks], qb[ks], acc, 0, 0, 0);
            oacc[ct] = acc;
          }
          // o^T[dv 16 tile + 4 g4 + i][query n]; the normalizer tile holds den for query n in every row
          const int tok = tq + n;
          const float den = oacc[G::CT][0] + a.eps;
          const float rden = 1.0f / den;
          if (tok < s1) {
            bf16_t* orow = a.o + (((size_t)b * T + tok) * a.Hq + hk * GR + hh) * D;
#pragma unroll
            for (int ct = 0; ct < G::CT; ++ct) {
              const uint2 pk = make_uint2(pack2(oacc[ct][0] * rden, oacc[ct][1] * rden),
                                          pack2(oacc[ct][2] * rden, oacc[ct][3] * rden));
              *reinterpret_cast<uint2*>(orow + 16 * (w * G::CT + ct) + 4 * g4) = pk;
            }
            if (a.den_out != nullptr && w == 0 && g4 == 0)
              a.den_out[((size_t)b * T + tok) * a.Hq + hk * GR + hh] = den;
          }
        }
      }
      // ---- state update: S <- diag(E_last) S + Kdec^T [V | 1]
#pragma unroll
      for (int rt = 0; rt < G::RT; ++rt) {
        const floatx4 eb = *reinterpret_cast<const floatx4*>(smem + G::kEb + (mc * D + 16 * rt + 4 * g4) * 4);
        const uint2 kr = *reinterpret_cast<const uint2*>(smem + G::kKd + (16 * rt + n) * G::TRS +
                                                         (kChunk * mc + 4 * g4) * 2);
        const short4v kdf = __builtin_bit_cast(short4v, kr);
        if (!OUTPUT) {
#pragma unroll
          for (int i = 0; i < 4; ++i) dprod[rt][i] *= eb[i];
        }
#pragma unroll
        for (int ct = 0; ct < G::NT; ++ct) {
          floatx4 acc = Sacc[rt][ct];
#pragma unroll
          for (int i = 0; i < 4; ++i) acc[i] *= eb[i];
          Sacc[rt][ct] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(kdf, vfrag[ct], acc, 0, 0, 0);
        }
      }
    }
    __syncthreads();
  }

  // ---- state out: first pass -> workspace slot (S | z | decay); last segment of the output pass -> S_out, z_out
  float* Sdst = nullptr;
  float* zdst = nullptr;
  float* ddst = nullptr;
  if (!OUTPUT) {
    Sdst = a.ws + ((size_t)bh * a.nseg + seg) * G::kSlot;
    zdst = Sdst + D * D;
    ddst = zdst + D;
  } else if (seg == a.nseg - 1) {
    Sdst = a.S_out + (size_t)bh * D * D;
    zdst = a.z_out + (size_t)bh * D;
  }
  if (Sdst != nullptr) {
#pragma unroll
    for (int rt = 0; rt < G::RT; ++rt)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int c = 16 * rt + 4 * g4 + i;
#pragma unroll
        for (int ct = 0; ct < G::CT; ++ct) Sdst[(size_t)c * D + 16 * (w * G::CT + ct) + n] = Sacc[rt][ct][i];
        if (w == 0 && n == 0) {
          zdst[c] = Sacc[rt][G::CT][i];
          if (ddst != nullptr) ddst[c] = dprod[rt][i];
        }
      }
  }
}

// Turns per-segment contributions into segment start states, in place:
//   slot[seg] <- state before segment seg;  state <- decay[seg] (.) state + contribution[seg].
template <int D>
__global__ void __launch_bounds__(256) segment_scan_kernel(float* __restrict__ ws, const float* __restrict__ S0,
                                                          const float* __restrict__ z0, int nseg) {
  constexpr int kSlot = D * D + 2 * D;
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= D * D + D) return;
  const int bh = blockIdx.y;
  const int c = e < D * D ? e / D : e - D * D;
  float s = 0.f;
  if (e < D * D) { if (S0) s = S0[(size_t)bh * D * D + e]; }
  else if (z0) s = z0[(size_t)bh * D + c];
  float* slot = ws + (size_t)bh * nseg * kSlot;
  for (int seg = 0; seg + 1 < nseg; ++seg, slot += kSlot) {
    const float delta = slot[e];
    const float dec = slot[D * D + D + c];
    slot[e] = s;
    s = fmaf(dec, s, delta);
  }
  slot[e] = s;
}

template <int D, int GR, bool FUSE>
hipError_t launch_all(const ChunkArgs& a, hipStream_t stream) {
  using G = Geo<D, GR>;
  const int heads = a.B * a.Hkv;
  hipError_t e;
  if (a.nseg > 1) {
    auto k1 = gla_chunk_kernel<D, 1, FUSE, false>;
    constexpr int lds1 = Geo<D, 1>::kBytes;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(k1), hipFuncAttributeMaxDynamicSharedMemorySize, lds1);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k1, dim3(a.nseg - 1, heads), dim3(256), lds1, stream, a);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(segment_scan_kernel<D>, dim3((D * D + D + 255) / 256, heads), dim3(256), 0, stream, a.ws, a.S0,
                       a.z0, a.nseg);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  auto k3 = gla_chunk_kernel<D, GR, FUSE, true>;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(k3), hipFuncAttributeMaxDynamicSharedMemorySize, G::kBytes);
  if (e != hipSuccess) return e;
  const bool trace = g_ev_before != nullptr && g_ev_after != nullptr;
  if (trace) {
    e = hipEventRecord(g_ev_before, stream);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(k3, dim3(a.nseg, heads), dim3(256), G::kBytes, stream, a);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (trace) e = hipEventRecord(g_ev_after, stream);
  return e;
}

template <int D, int GR>
hipError_t launch_fuse(const ChunkArgs& a, bool fuse, hipStream_t stream) {
  return fuse ? launch_all<D, GR, true>(a, stream) : launch_all<D, GR, false>(a, stream);
}

template <int D>
hipError_t launch_group(const ChunkArgs& a, int group, bool fuse, hipStream_t stream) {
  switch (group) {
    case 1: return launch_fuse<D, 1>(a, fuse, stream);
    case 2: return launch_fuse<D, 2>(a, fuse, stream);
    case 4: return launch_fuse<D, 4>(a, fuse, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

void set_output_pass_events(hipEvent_t before, hipEvent_t after) {
  g_ev_before = before;
  g_ev_after = after;
}

bool chunk_path_supports(int group) { return group == 1 || group == 2 || group == 4; }

ChunkPlan make_chunk_plan(int B, int T, int Hkv, int d, int carry_mode, int segment) {
  ChunkPlan p;
  const int heads = B * Hkv;
  int seg_len;
  if (carry_mode == 1) {
    seg_len = (T + 63) / 64 * 64;
  } else if (segment > 0) {
    seg_len = segment;
  } else {
    // enough workgroups for two per compute unit, segments no shorter than 128 tokens
    const int want = (512 + heads - 1) / heads;
    seg_len = (T + want - 1) / want;
    seg_len = (seg_len + 63) / 64 * 64;
    if (seg_len < 128) seg_len = 128;
  }
  p.seg_len = seg_len;
  p.nseg = (T + seg_len - 1) / seg_len;
  p.workspace_bytes = p.nseg > 1 ? (size_t)heads * p.nseg * (d * d + 2 * d) * sizeof(float) : 0;
  return p;
}

hipError_t launch_gla_chunk(const ChunkParams& p, hipStream_t stream) {
  ChunkArgs a;
  a.q = (const bf16_t*)p.q; a.k = (const bf16_t*)p.k; a.v = (const bf16_t*)p.v; a.g = (const bf16_t*)p.g;
  a.wq = (const bf16_t*)p.wq; a.wk = (const bf16_t*)p.wk;
  a.q_halo = (const bf16_t*)p.q_halo; a.k_halo = (const bf16_t*)p.k_halo;
  a.S0 = p.S0; a.z0 = p.z0; a.o = (bf16_t*)p.o; a.den_out = p.den_out; a.S_out = p.S_out; a.z_out = p.z_out;
  a.ws = (float*)p.workspace;
  a.B = p.B; a.T = p.T; a.Hq = p.Hq; a.Hkv = p.Hkv; a.W = p.W; a.phi = p.phi;
  a.seg_len = p.plan.seg_len; a.nseg = p.plan.nseg;
  a.gate_scale = p.gate_scale; a.eps = p.eps;
  const int group = p.Hq / p.Hkv;
  return p.d == 64 ? launch_group<64>(a, group, p.fuse_conv != 0, stream)
                   : launch_group<128>(a, group, p.fuse_conv != 0, stream);
}

}  // namespace lawcat
