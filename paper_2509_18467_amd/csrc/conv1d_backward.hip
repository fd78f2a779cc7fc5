// Adjoint of the causal depthwise conv with its pointwise feature map (paper section 4.1; the layer-wise
// distillation of section 5 trains the conv weights through it):
//   u_t = sum_{dl < W} w[dl] x_{t-dl},   y_t = phi(u_t),   du_t = dy_t phi'(u_t)   (phi' = 1, or for 1 + ELU: 1 if u > 0, else e^u)
//   dx_s = sum_{dl < W} w[dl] du_{s+dl},   dw[dl] = sum_{b,t} du_t x_{t-dl},   rows before the first token: dhalo like dx
// u is recomputed from x (one more pass of W multiply-adds beats reading a stored copy).  Streaming: a thread owns
// four adjacent channels and walks a strip of 64 tokens (plus the W - 1 tokens after it, whose du the strip's last
// dx need) with x and du of the last W tokens in registers; 6 bytes per element moved in bf16 storage.  dw: every
// (strip, batch) writes its partial sums to the workspace, a second kernel adds them in strip order (no atomics:
// repeated calls agree bit for bit).
#include "kernels.h"

namespace lawcat {
namespace {

constexpr int kStrip = 64;

struct f4 { float v[4]; };
__device__ inline f4 ld4(const float* p) {
  const float4 t = *reinterpret_cast<const float4*>(p);
  return {{t.x, t.y, t.z, t.w}};
}
__device__ inline f4 ld4(const bf16_t* p) {
  const uint2 t = *reinterpret_cast<const uint2*>(p);
  return {{__uint_as_float(t.x << 16), __uint_as_float(t.x & 0xffff0000u), __uint_as_float(t.y << 16),
           __uint_as_float(t.y & 0xffff0000u)}};
}
__device__ inline void st4(float* p, const f4& a) { *reinterpret_cast<float4*>(p) = make_float4(a.v[0], a.v[1], a.v[2], a.v[3]); }
__device__ inline uint32_t pack2(float a, float b) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 h = {(__bf16)a, (__bf16)b};  // round to nearest even
  return __builtin_bit_cast(uint32_t, h);
}
__device__ inline void st4(bf16_t* p, const f4& a) {
  *reinterpret_cast<uint2*>(p) = make_uint2(pack2(a.v[0], a.v[1]), pack2(a.v[2], a.v[3]));
}

// grid (ceil(row / 1024), strips, B), 256 threads; row = H * d channels of a token.
template <typename T, int W, int PHI>
__global__ void __launch_bounds__(256) conv_bwd_kernel(const T* __restrict__ x, const T* __restrict__ w,
                                                      const T* __restrict__ halo, const T* __restrict__ dy,
                                                      T* __restrict__ dx, T* __restrict__ dhalo,
                                                      float* __restrict__ partial, int Tn, int row) {
  const int e0 = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (e0 >= row) return;
  const int strip = blockIdx.y, b = blockIdx.z;
  const int t0 = strip * kStrip, t1 = min(Tn, t0 + kStrip);
  const size_t base = (size_t)b * Tn * row + e0;

  float wv[4][W], dw[4][W];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int dl = 0; dl < W; ++dl) {
      wv[i][dl] = sizeof(T) == 2 ? __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(w)[(size_t)(e0 + i) * W + dl] << 16)
                                 : reinterpret_cast<const float*>(w)[(size_t)(e0 + i) * W + dl];
      dw[i][dl] = 0.f;
    }
  // xw[j] = x_{t-j}, du[j] = du_{t-j} of the token t being worked on
  f4 xw[W], du[W];
#pragma unroll
  for (int j = 0; j < W; ++j) {
    xw[j] = {{0.f, 0.f, 0.f, 0.f}};
    du[j] = {{0.f, 0.f, 0.f, 0.f}};
  }
#pragma unroll
  for (int j = 1; j < W; ++j) {   // history of the strip's first token: x_{t0-j} goes to xw[j-1], shifted below
    const int s = t0 - j;
    if (s >= 0) xw[j - 1] = ld4(x + base + (size_t)s * row);
    else if (halo != nullptr) xw[j - 1] = ld4(halo + ((size_t)b * (W - 1) + (W - 1 + s)) * row + e0);
  }

  const int t_end = t1 + W - 1;
#pragma unroll 2
  for (int t = t0; t < t_end; ++t) {
#pragma unroll
    for (int j = W - 1; j >= 1; --j) {
      xw[j] = xw[j - 1];
      du[j] = du[j - 1];
    }
    f4 d0 = {{0.f, 0.f, 0.f, 0.f}};
    xw[0] = d0;
    if (t < Tn) {
      xw[0] = ld4(x + base + (size_t)t * row);
      const f4 g = ld4(dy + base + (size_t)t * row);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float u = 0.f;
#pragma unroll
        for (int dl = 0; dl < W; ++dl) u = fmaf(wv[i][dl], xw[dl].v[i], u);
        d0.v[i] = PHI == 1 ? (u > 0.f ? g.v[i] : g.v[i] * __expf(u)) : g.v[i];
      }
    }
    du[0] = d0;
    if (t < t1) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int dl = 0; dl < W; ++dl) dw[i][dl] = fmaf(d0.v[i], xw[dl].v[i], dw[i][dl]);
    }
    // dx of token s = t - (W - 1) is complete now
    const int s = t - (W - 1);
    f4 o;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float acc = 0.f;
#pragma unroll
      for (int dl = 0; dl < W; ++dl) acc = fmaf(wv[i][dl], du[W - 1 - dl].v[i], acc);
      o.v[i] = acc;
    }
    if (s >= t0) st4(dx + base + (size_t)s * row, o);
    else if (s < 0 && dhalo != nullptr) st4(dhalo + ((size_t)b * (W - 1) + (W - 1 + s)) * row + e0, o);
  }
  float* out = partial + ((size_t)b * gridDim.y + strip) * row * W + (size_t)e0 * W;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int dl = 0; dl < W; ++dl) out[i * W + dl] = dw[i][dl];
}

// dw[e] = sum of the partial sums in (batch, strip) order.  One thread per element of [H, d, W].
__global__ void __launch_bounds__(256) conv_bwd_reduce_kernel(const float* __restrict__ partial, float* __restrict__ dw,
                                                             int n_partial, int n) {
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= n) return;
  float acc = 0.f;
  int p = 0;
  for (; p + 8 <= n_partial; p += 8) {
    float t[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) t[u] = partial[(size_t)(p + u) * n + e];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc += t[u];
  }
  for (; p < n_partial; ++p) acc += partial[(size_t)p * n + e];
  dw[e] = acc;
}

template <typename T, int W>
hipError_t launch_w(const ConvBackwardParams& p, hipStream_t stream) {
  const int row = p.H * p.d;
  const int strips = (p.T + kStrip - 1) / kStrip;
  const dim3 grid((row / 4 + 255) / 256, strips, p.B);
  float* partial = static_cast<float*>(p.workspace);
  if (p.phi == 1)
    hipLaunchKernelGGL((conv_bwd_kernel<T, W, 1>), grid, dim3(256), 0, stream, (const T*)p.x, (const T*)p.w, (const T*)p.halo,
                       (const T*)p.dy, (T*)p.dx, (T*)p.dhalo, partial, p.T, row);
  else
    hipLaunchKernelGGL((conv_bwd_kernel<T, W, 0>), grid, dim3(256), 0, stream, (const T*)p.x, (const T*)p.w, (const T*)p.halo,
                       (const T*)p.dy, (T*)p.dx, (T*)p.dhalo, partial, p.T, row);
  const int n = row * W;
  hipLaunchKernelGGL(conv_bwd_reduce_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, partial, p.dw, p.B * strips, n);
  return hipGetLastError();
}

template <typename T>
hipError_t launch_t(const ConvBackwardParams& p, hipStream_t stream) {
  switch (p.W) {
    case 1: return launch_w<T, 1>(p, stream);
    case 2: return launch_w<T, 2>(p, stream);
    case 3: return launch_w<T, 3>(p, stream);
    case 4: return launch_w<T, 4>(p, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

size_t conv_backward_workspace_bytes(int B, int T, int H, int d, int W) {
  return (size_t)B * ((T + kStrip - 1) / kStrip) * H * d * W * sizeof(float);
}

hipError_t launch_conv_backward(const ConvBackwardParams& p, hipStream_t stream) {
  return p.bf16 ? launch_t<bf16_t>(p, stream) : launch_t<float>(p, stream);
}

}  // namespace lawcat
