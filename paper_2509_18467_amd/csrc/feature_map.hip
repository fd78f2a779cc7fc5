// The layer that follows the conv in paper section 4.1: a linear layer with nonlinearity, the same for the
// query and the key,
//   y[b,t,h,f] = phi( sum_c x~[b,t,h,c] * Wf[h / group, c, f] ),   x~ = causal depthwise conv of x (no phi)
// fused with that conv: one kernel reads the raw rows, slides the conv window in registers, keeps the conv
// output of a 64-token tile in LDS and multiplies it by the head's d x d matrix.
//   bf16 storage: the product runs on the matrix cores (v_mfma_f32_16x16x32_bf16, fp32 accumulate), computed
//     transposed (y^T = Wf^T x~^T) so that a lane ends up with four adjacent features of one token and stores
//     8 bytes; the conv output is rounded to bf16 once, as an MFMA operand.
//   fp32 storage: plain fp32 FMAs (the 1e-4 bar leaves no room for bf16 operands).
// Streaming and HBM-bound: 2 bytes read and 2 written per element; the matrix (8 or 32 KB) is re-read from L2
// once per 256 tokens.
#include "kernels.h"

namespace lawcat {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kTile = 64;        // tokens per tile
constexpr int kTilesPerBlock = 4;

__device__ inline float apply_phi(float x, int phi) { return phi == 1 ? (x > 0.f ? 1.f + x : __expf(x)) : x; }
__device__ inline float bf_to_f(bf16_t u) { return __uint_as_float((uint32_t)u << 16); }
__device__ inline uint32_t pack2(float a, float b) {
  bf16x2 v = {(__bf16)a, (__bf16)b};  // round to nearest even
  return __builtin_bit_cast(uint32_t, v);
}

// ---- conv of one 64-token tile into LDS (no phi).  Thread = one channel pair x a run of tokens.
// xs: [kTile][D] elements of XS (bf16_t packed pairs or float), row stride `rs` bytes.
template <typename T, int D>
__device__ inline void conv_tile(const T* __restrict__ x, const T* __restrict__ w, const T* __restrict__ halo, int b,
                                 int h, int H, int Tn, int W, int t0, unsigned char* xs, int rs) {
  constexpr int PAIRS = D / 2;
  constexpr int NTOK = kTile * PAIRS / 256;   // tokens per thread: 8 (d = 64) or 16 (d = 128)
  const int cp = threadIdx.x % PAIRS, tg = threadIdx.x / PAIRS;
  const int c0 = 2 * cp;
  float wt[2][4];
#pragma unroll
  for (int ch = 0; ch < 2; ++ch)
#pragma unroll
    for (int dl = 0; dl < 4; ++dl) {
      float v = 0.f;
      if (dl < W) {
        const T* p = w + ((size_t)h * D + c0 + ch) * W + dl;
        if constexpr (sizeof(T) == 2) v = bf_to_f(*p); else v = *p;
      }
      wt[ch][dl] = v;
    }
  auto row = [&](int t, float (&v)[2]) {   // raw row t of this thread's two channels; rows < 0 from the halo or zero
    v[0] = 0.f; v[1] = 0.f;
    const T* p = nullptr;
    if (t >= 0 && t < Tn) p = x + (((size_t)b * Tn + t) * H + h) * D + c0;
    else if (t < 0 && halo != nullptr && t >= -(W - 1)) p = halo + (((size_t)b * (W - 1) + (W - 1 + t)) * H + h) * D + c0;
    if (p != nullptr) {
      if constexpr (sizeof(T) == 2) {
        const uint32_t u = *reinterpret_cast<const uint32_t*>(p);
        v[0] = __uint_as_float(u << 16); v[1] = __uint_as_float(u & 0xffff0000u);
      } else {
        const float2 f = *reinterpret_cast<const float2*>(p);
        v[0] = f.x; v[1] = f.y;
      }
    }
  };
  const int ts = t0 + tg * NTOK;
  float win[3][2];
#pragma unroll
  for (int j = 0; j < 3; ++j) row(ts - 1 - j, win[j]);
#pragma unroll
  for (int i = 0; i < NTOK; ++i) {
    float cur[2];
    row(ts + i, cur);
    float out[2];
#pragma unroll
    for (int ch = 0; ch < 2; ++ch) {
      float acc = wt[ch][0] * cur[ch];
      acc = fmaf(wt[ch][1], win[0][ch], acc);
      acc = fmaf(wt[ch][2], win[1][ch], acc);
      acc = fmaf(wt[ch][3], win[2][ch], acc);
      out[ch] = acc;
      win[2][ch] = win[1][ch]; win[1][ch] = win[0][ch]; win[0][ch] = cur[ch];
    }
    unsigned char* dst = xs + (size_t)(tg * NTOK + i) * rs;
    if constexpr (sizeof(T) == 2) *reinterpret_cast<uint32_t*>(dst + c0 * 2) = pack2(out[0], out[1]);
    else *reinterpret_cast<float2*>(dst + c0 * 4) = make_float2(out[0], out[1]);
  }
}

// bf16 storage, matrix cores.  grid (ceil(T / 256), B * H), 256 threads.
template <int D>
__global__ void __launch_bounds__(256) conv_feature_mfma_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ w,
                                                                const bf16_t* __restrict__ halo,
                                                                const bf16_t* __restrict__ wf, bf16_t* __restrict__ y,
                                                                int B, int Tn, int H, int group, int W, int phi) {
  constexpr int RS = D * 2 + 16;              // LDS row stride in bytes (16-byte reads of 16 rows hit distinct banks)
  constexpr int KS = D / 32, FT = D / 16;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* wts = smem;                  // Wf^T: [f][c] bf16
  unsigned char* xs = smem + D * RS;          // conv output of the tile: [token][c] bf16
  const int bh = blockIdx.y, b = bh / H, h = bh % H;
  const int tid = threadIdx.x, l = tid & 63, wv = tid >> 6;
  const int n = l & 15, g = l >> 4;
  const bf16_t* wsrc = wf + (size_t)(h / group) * D * D;
  for (int e = tid; e < D * D; e += 256) {
    const int c = e / D, f = e % D;           // read with f fastest (coalesced), write transposed
    *reinterpret_cast<bf16_t*>(wts + f * RS + c * 2) = wsrc[e];
  }
  for (int tile = 0; tile < kTilesPerBlock; ++tile) {
    const int t0 = (blockIdx.x * kTilesPerBlock + tile) * kTile;
    if (t0 >= Tn) break;
    __syncthreads();                          // the previous tile's readers are done with xs (and wts is written)
    conv_tile<bf16_t, D>(x, w, halo, b, h, H, Tn, W, t0, xs, RS);
    __syncthreads();
    // y^T[f][token] = Wf^T x~^T: A = Wf^T rows (features), B = x~ rows (tokens); wave wv owns tokens 16 wv .. + 15
    bf16x8 bfrag[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      bfrag[ks] = *reinterpret_cast<const bf16x8*>(xs + (16 * wv + n) * RS + (32 * ks + 8 * g) * 2);
    const int tok = t0 + 16 * wv + n;
#pragma unroll
    for (int ft = 0; ft < FT; ++ft) {
      floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8 afrag = *reinterpret_cast<const bf16x8*>(wts + (16 * ft + n) * RS + (32 * ks + 8 * g) * 2);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(afrag, bfrag[ks], acc, 0, 0, 0);
      }
      // lane (n, g): features 16 ft + 4 g + i of token n
      if (tok < Tn) {
        const uint2 pk = make_uint2(pack2(apply_phi(acc[0], phi), apply_phi(acc[1], phi)),
                                    pack2(apply_phi(acc[2], phi), apply_phi(acc[3], phi)));
        *reinterpret_cast<uint2*>(y + (((size_t)b * Tn + tok) * H + h) * D + 16 * ft + 4 * g) = pk;
      }
    }
  }
}

// fp32 storage, plain FMAs.  Same grid.
template <int D>
__global__ void __launch_bounds__(256) conv_feature_f32_kernel(const float* __restrict__ x, const float* __restrict__ w,
                                                               const float* __restrict__ halo,
                                                               const float* __restrict__ wf, float* __restrict__ y,
                                                               int B, int Tn, int H, int group, int W, int phi) {
  constexpr int RS = (D + 2) * 4;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* xs = smem;
  const int bh = blockIdx.y, b = bh / H, h = bh % H;
  const int tid = threadIdx.x;
  const float* wsrc = wf + (size_t)(h / group) * D * D;
  for (int tile = 0; tile < kTilesPerBlock; ++tile) {
    const int t0 = (blockIdx.x * kTilesPerBlock + tile) * kTile;
    if (t0 >= Tn) break;
    __syncthreads();
    conv_tile<float, D>(x, w, halo, b, h, H, Tn, W, t0, xs, RS);
    __syncthreads();
    for (int e = tid; e < kTile * D; e += 256) {
      const int tl = e / D, f = e % D;
      const float* xr = reinterpret_cast<const float*>(xs + (size_t)tl * RS);
      float acc = 0.f;
      for (int c = 0; c < D; ++c) acc = fmaf(xr[c], wsrc[(size_t)c * D + f], acc);
      if (t0 + tl < Tn) y[(((size_t)b * Tn + t0 + tl) * H + h) * D + f] = apply_phi(acc, phi);
    }
  }
}

}  // namespace

hipError_t launch_conv_feature(const ConvParams& p, const void* wf, int group, hipStream_t stream) {
  const dim3 grid((p.T + kTile * kTilesPerBlock - 1) / (kTile * kTilesPerBlock), p.B * p.H);
  hipError_t e = hipSuccess;
  if (p.bf16) {
    if (p.d == 64) {
      constexpr int lds = (64 + kTile) * (64 * 2 + 16);
      hipLaunchKernelGGL(conv_feature_mfma_kernel<64>, grid, dim3(256), lds, stream, (const bf16_t*)p.x, (const bf16_t*)p.w,
                         (const bf16_t*)p.halo, (const bf16_t*)wf, (bf16_t*)p.y, p.B, p.T, p.H, group, p.W, p.phi);
    } else {
      constexpr int lds = (128 + kTile) * (128 * 2 + 16);
      hipLaunchKernelGGL(conv_feature_mfma_kernel<128>, grid, dim3(256), lds, stream, (const bf16_t*)p.x, (const bf16_t*)p.w,
                         (const bf16_t*)p.halo, (const bf16_t*)wf, (bf16_t*)p.y, p.B, p.T, p.H, group, p.W, p.phi);
    }
  } else {
    if (p.d == 64) {
      constexpr int lds = kTile * (64 + 2) * 4;
      hipLaunchKernelGGL(conv_feature_f32_kernel<64>, grid, dim3(256), lds, stream, (const float*)p.x, (const float*)p.w,
                         (const float*)p.halo, (const float*)wf, (float*)p.y, p.B, p.T, p.H, group, p.W, p.phi);
    } else {
      constexpr int lds = kTile * (128 + 2) * 4;
      hipLaunchKernelGGL(conv_feature_f32_kernel<128>, grid, dim3(256), lds, stream, (const float*)p.x, (const float*)p.w,
                         (const float*)p.halo, (const float*)wf, (float*)p.y, p.B, p.T, p.H, group, p.W, p.phi);
    }
  }
  e = hipGetLastError();
  return e;
}

}  // namespace lawcat
