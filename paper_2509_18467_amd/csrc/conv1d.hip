// Causal depthwise Conv1D across tokens (paper section 4.1, the sum over delta):
//   y[b,t,h,c] = phi( sum_{delta<W} w[h,c,delta] * x[b,t-delta,h,c] )
// Streaming kernel: each thread owns one 16-byte column group of a row and slides a
// register window down a strip of tokens, so every row is fetched from HBM once and
// the W-1 rows above a strip are the only re-reads (they hit L2).  Rows are contiguous
// H*d elements, so consecutive lanes read consecutive 16-byte pieces.
#include "kernels.h"

namespace lawcat {
namespace {

constexpr int kGroup = 4;   // rows fetched together, one group ahead of the arithmetic

template <typename T> struct Io;
template <> struct Io<float> {
  static constexpr int VEC = 4;
  typedef float4 Raw;
  __device__ static Raw load_raw(const float* p) { return *reinterpret_cast<const float4*>(p); }
  __device__ static Raw zero_raw() { return make_float4(0.f, 0.f, 0.f, 0.f); }
  __device__ static void unpack(const Raw& r, float (&f)[VEC]) { f[0] = r.x; f[1] = r.y; f[2] = r.z; f[3] = r.w; }
  __device__ static void load(const float* p, float (&f)[VEC]) {
    float4 r = *reinterpret_cast<const float4*>(p);
    f[0] = r.x; f[1] = r.y; f[2] = r.z; f[3] = r.w;
  }
  __device__ static void store(float* p, const float (&f)[VEC]) {
    *reinterpret_cast<float4*>(p) = make_float4(f[0], f[1], f[2], f[3]);
  }
  __device__ static float scalar(const float* p) { return *p; }
};
template <> struct Io<bf16_t> {
  static constexpr int VEC = 8;
  typedef uint4 Raw;
  __device__ static Raw load_raw(const bf16_t* p) { return *reinterpret_cast<const uint4*>(p); }
  __device__ static Raw zero_raw() { return make_uint4(0u, 0u, 0u, 0u); }
  __device__ static void unpack(const Raw& r, float (&f)[VEC]) {
    const uint32_t u[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __uint_as_float(u[i] << 16);
      f[2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u);
    }
  }
  __device__ static void load(const bf16_t* p, float (&f)[VEC]) {
    uint4 r = *reinterpret_cast<const uint4*>(p);
    uint32_t u[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __uint_as_float(u[i] << 16);
      f[2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u);
    }
  }
  __device__ static uint32_t pack(float a, float b) {
    typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
    bf2 v = {(__bf16)a, (__bf16)b};  // round to nearest even
    return __builtin_bit_cast(uint32_t, v);
  }
  __device__ static void store(bf16_t* p, const float (&f)[VEC]) {
    uint4 r;
    r.x = pack(f[0], f[1]); r.y = pack(f[2], f[3]); r.z = pack(f[4], f[5]); r.w = pack(f[6], f[7]);
    *reinterpret_cast<uint4*>(p) = r;
  }
  __device__ static float scalar(const bf16_t* p) { return __uint_as_float((uint32_t)(*p) << 16); }
};

__device__ inline float apply_phi(float x, int phi) {
  if (phi == 1) return x > 0.f ? 1.f + x : __expf(x);
  return x;
}

// kStrip: tokens per thread (64; 32 or 16 where longer strips would leave compute units without a workgroup)
template <typename T, int kStrip>
__global__ void __launch_bounds__(256) conv1d_causal_kernel(const T* __restrict__ x, const T* __restrict__ w,
                                                            const T* __restrict__ halo, T* __restrict__ y,
                                                            int B, int Tn, int rowlen, int W, int phi) {
  constexpr int VEC = Io<T>::VEC;
  const int vecs = rowlen / VEC;
  const int nstrips = (Tn + kStrip - 1) / kStrip;
  const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const int col = (int)(gid % vecs);
  const long long rest = gid / vecs;
  const int s = (int)(rest % nstrips);
  const int b = (int)(rest / nstrips);
  if (b >= B) return;
  const int e0 = col * VEC;  // first element (h*d + c) of this thread's column group

  float wt[4][VEC];  // wt[delta][i]
  if (W == 4) {
    // the VEC x 4 taps of this column group are contiguous: four whole-vector loads instead of 4 VEC scalar
    // ones (the scalar form made every thread start with a long chain of small dependent loads)
    float flat[4 * VEC];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float part[VEC];
      Io<T>::load(w + (size_t)e0 * 4 + j * VEC, part);
#pragma unroll
      for (int i = 0; i < VEC; ++i) flat[j * VEC + i] = part[i];
    }
#pragma unroll
    for (int i = 0; i < VEC; ++i)
#pragma unroll
      for (int dl = 0; dl < 4; ++dl) wt[dl][i] = flat[i * 4 + dl];
  } else {
#pragma unroll
    for (int i = 0; i < VEC; ++i)
#pragma unroll
      for (int dl = 0; dl < 4; ++dl) wt[dl][i] = dl < W ? Io<T>::scalar(w + (size_t)(e0 + i) * W + dl) : 0.f;
  }

  const int t0 = s * kStrip;
  float win[3][VEC];  // win[j] = row t-1-j
#pragma unroll
  for (int j = 0; j < 3; ++j) {
    const int src = t0 - 1 - j;
    if (j >= W - 1) {
#pragma unroll
      for (int i = 0; i < VEC; ++i) win[j][i] = 0.f;
    } else if (src >= 0) {
      Io<T>::load(x + ((size_t)b * Tn + src) * rowlen + e0, win[j]);
    } else if (halo != nullptr) {
      Io<T>::load(halo + ((size_t)b * (W - 1) + (W - 1 + src)) * rowlen + e0, win[j]);
    } else {
#pragma unroll
      for (int i = 0; i < VEC; ++i) win[j][i] = 0.f;
    }
  }
  // Rows travel in groups of kGroup, the next group's loads issued before this group's arithmetic, so that
  // every thread keeps kGroup 16-byte loads in flight.
  typedef typename Io<T>::Raw Raw;
  const T* xb = x + ((size_t)b * Tn) * rowlen + e0;
  T* yb = y + ((size_t)b * Tn) * rowlen + e0;
  Raw nxt[kGroup];
#pragma unroll
  for (int r = 0; r < kGroup; ++r) nxt[r] = (t0 + r < Tn) ? Io<T>::load_raw(xb + (size_t)(t0 + r) * rowlen) : Io<T>::zero_raw();
#pragma unroll 1
  for (int tg = t0; tg < t0 + kStrip && tg < Tn; tg += kGroup) {
    Raw cur[kGroup];
#pragma unroll
    for (int r = 0; r < kGroup; ++r) cur[r] = nxt[r];
    if (tg + kGroup < t0 + kStrip) {
#pragma unroll
      for (int r = 0; r < kGroup; ++r) {
        const int t = tg + kGroup + r;
        nxt[r] = (t < Tn) ? Io<T>::load_raw(xb + (size_t)t * rowlen) : Io<T>::zero_raw();
      }
    }
#pragma unroll
    for (int r = 0; r < kGroup; ++r) {
      float c[VEC], out[VEC];
      Io<T>::unpack(cur[r], c);
#pragma unroll
      for (int i = 0; i < VEC; ++i) {
        float acc = wt[0][i] * c[i];
        acc = fmaf(wt[1][i], win[0][i], acc);
        acc = fmaf(wt[2][i], win[1][i], acc);
        acc = fmaf(wt[3][i], win[2][i], acc);
        out[i] = apply_phi(acc, phi);
        win[2][i] = win[1][i];
        win[1][i] = win[0][i];
        win[0][i] = c[i];
      }
      if (tg + r < Tn) Io<T>::store(yb + (size_t)(tg + r) * rowlen, out);
    }
  }
}

// tail_out[b, r] = row (T - (W-1) + r) of [halo ; x]: the conv cache for a continuation.
template <typename T>
__global__ void conv_tail_kernel(const T* __restrict__ x, const T* __restrict__ halo, T* __restrict__ tail,
                                 int B, int Tn, int rowlen, int W) {
  const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const long long total = (long long)B * (W - 1) * rowlen;
  if (gid >= total) return;
  const int e = (int)(gid % rowlen);
  const int r = (int)((gid / rowlen) % (W - 1));
  const int b = (int)(gid / ((long long)rowlen * (W - 1)));
  const int src = Tn - (W - 1) + r;
  T val = T(0);
  if (src >= 0) val = x[((size_t)b * Tn + src) * rowlen + e];
  else if (halo != nullptr) val = halo[((size_t)b * (W - 1) + (W - 1 + src)) * rowlen + e];
  tail[gid] = val;
}

template <typename T>
hipError_t launch_typed(const ConvParams& p, hipStream_t stream) {
  const int rowlen = p.H * p.d;
  const int vecs = rowlen / Io<T>::VEC;
  const int block = 256;
  auto blocks = [&](int strip) { return ((long long)p.B * ((p.T + strip - 1) / strip) * vecs + block - 1) / block; };
  // 64-token strips unless that leaves fewer than two workgroups per compute unit (few heads, short sequences)
  constexpr long long kWant = 512;
  if (blocks(64) >= kWant)
    hipLaunchKernelGGL((conv1d_causal_kernel<T, 64>), dim3((unsigned)blocks(64)), dim3(block), 0, stream, (const T*)p.x,
                       (const T*)p.w, (const T*)p.halo, (T*)p.y, p.B, p.T, rowlen, p.W, p.phi);
  else if (blocks(32) >= kWant)
    hipLaunchKernelGGL((conv1d_causal_kernel<T, 32>), dim3((unsigned)blocks(32)), dim3(block), 0, stream, (const T*)p.x,
                       (const T*)p.w, (const T*)p.halo, (T*)p.y, p.B, p.T, rowlen, p.W, p.phi);
  else
    hipLaunchKernelGGL((conv1d_causal_kernel<T, 16>), dim3((unsigned)blocks(16)), dim3(block), 0, stream, (const T*)p.x,
                       (const T*)p.w, (const T*)p.halo, (T*)p.y, p.B, p.T, rowlen, p.W, p.phi);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (p.tail_out != nullptr && p.W > 1) {
    const long long total = (long long)p.B * (p.W - 1) * rowlen;
    hipLaunchKernelGGL(conv_tail_kernel<T>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream,
                       (const T*)p.x, (const T*)p.halo, (T*)p.tail_out, p.B, p.T, rowlen, p.W);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace

hipError_t launch_conv1d(const ConvParams& p, hipStream_t stream) {
  return p.bf16 ? launch_typed<bf16_t>(p, stream) : launch_typed<float>(p, stream);
}

hipError_t launch_conv_tail(const ConvParams& p, hipStream_t stream) {
  if (p.W <= 1 || p.tail_out == nullptr) return hipSuccess;
  const int rowlen = p.H * p.d;
  const long long total = (long long)p.B * (p.W - 1) * rowlen;
  const unsigned grid = (unsigned)((total + 255) / 256);
  if (p.bf16)
    hipLaunchKernelGGL(conv_tail_kernel<bf16_t>, dim3(grid), dim3(256), 0, stream, (const bf16_t*)p.x,
                       (const bf16_t*)p.halo, (bf16_t*)p.tail_out, p.B, p.T, rowlen, p.W);
  else
    hipLaunchKernelGGL(conv_tail_kernel<float>, dim3(grid), dim3(256), 0, stream, (const float*)p.x,
                       (const float*)p.halo, (float*)p.tail_out, p.B, p.T, rowlen, p.W);
  return hipGetLastError();
}

}  // namespace lawcat
