// The layer that follows the conv in paper section 4.1: a linear layer with nonlinearity, the same for the
// query and the key,
//   y[b,t,h,f] = phi( sum_c x~[b,t,h,c] * Wf[h / group, c, f] ),   x~ = causal depthwise conv of x (no phi)
// fused with that conv: one kernel reads the raw rows, slides the conv window in registers, keeps the conv
// output of a tile in LDS and multiplies it by the head's d x d matrix.
//   bf16 storage: the product runs on the matrix cores (v_mfma_f32_16x16x32_bf16, fp32 accumulate), computed
//     transposed (y^T = Wf^T x~^T) so that a lane ends up with four adjacent features of one token; the results
//     go back through LDS and leave as whole rows; the conv output is rounded to bf16 once, as an MFMA operand.
//   fp32 storage: plain fp32 FMAs (the 1e-4 bar leaves no room for bf16 operands).
// Streaming and HBM-bound: 2 bytes read and 2 written per element; the matrix (8 or 32 KB) is read from L2 once
// per workgroup, which walks a run of tiles.
#include <mutex>

#include "kernels.h"

namespace lawcat {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kTile = 64;        // fp32 kernel: tokens per tile
constexpr int kTilesPerBlock = 4;

typedef unsigned int u32x4 __attribute__((vector_size(16)));

__device__ inline float apply_phi(float x, int phi) { return phi == 1 ? (x > 0.f ? 1.f + x : __expf(x)) : x; }
template <bool ELU>
__device__ inline float apply_phi(float x) { return ELU ? (x > 0.f ? 1.f + x : __expf(x)) : x; }
__device__ inline float bf_to_f(bf16_t u) { return __uint_as_float((uint32_t)u << 16); }
__device__ inline uint32_t pack2(float a, float b) {
  bf16x2 v = {(__bf16)a, (__bf16)b};  // round to nearest even
  return __builtin_bit_cast(uint32_t, v);
}

// ---- fp32 kernel: conv of one 64-token tile into LDS (no phi).  Thread = one channel pair x a run of tokens.
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

// bf16 storage, matrix cores.  One workgroup (4 waves) walks `tiles_per_block` consecutive tiles of one
// (batch, head group): a tile is TT tokens x GH adjacent heads that share one matrix, ROWS = TT * GH rows of D
// channels (256 rows at D = 64, 128 at D = 128).
//   load  : thread = 8 adjacent channels (16 bytes) x a run of 8 tokens; 11 raw rows in registers (the run and
//           the three before it), read through a buffer descriptor over the workgroup's own token range, so
//           that rows before the first token and past the last read as zero without a branch; the next tile's
//           rows are requested before the current tile's products start
//   conv  : in registers, fp32; rounded to bf16 into LDS, row = token * GH + head (the order in memory)
//   matrix: wave w takes the 16-row groups w, w + 4, ...: B operand = the 16 rows, A operand = Wf^T from LDS,
//           so a lane ends up with 4 adjacent features of one row; phi; back into the same LDS rows
//   store : the wave reads its 16 finished rows back 16 bytes per lane and stores whole 128/256-byte rows
//           (buffer stores: rows past the last token are dropped)
// WT: the conv width when it is the paper's 4 (no per-tap branches), 0 = any width up to 4, read from W.
template <int D, int GH, int TT, bool ELU, int WT>
__global__ void __launch_bounds__(256) conv_feature_mfma_kernel(const bf16_t* __restrict__ x, const bf16_t* __restrict__ w,
                                                                const bf16_t* __restrict__ halo,
                                                                const bf16_t* __restrict__ wf, bf16_t* __restrict__ y,
                                                                int Tn, int H, int group, int Wrt, int tiles_per_block) {
  const int W = WT != 0 ? WT : Wrt;
  constexpr int RS = D * 2 + 16;              // LDS row stride in bytes (16-byte reads of 16 rows hit distinct banks)
  constexpr int KS = D / 32, FT = D / 16;
  constexpr int ROWS = TT * GH;
  constexpr int VPH = D / 8;                  // 16-byte vectors per head row
  constexpr int VECS = GH * VPH;              // per token
  constexpr int NTOK = ROWS * VPH / 256;      // tokens per thread
  constexpr int kRsrcFlags = 0x00020000;      // raw buffer, 32-bit data format of gfx9-family descriptors
  static_assert(ROWS * VPH == 256 * NTOK && 256 % VECS == 0, "tile must give every thread NTOK tokens of one vector");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* wts = smem;                  // Wf^T: [f][c] bf16
  unsigned char* xs = smem + D * RS;          // the tile: [row][c] bf16
  const int hgroups = H / GH;
  const int b = blockIdx.y / hgroups, h0 = (blockIdx.y % hgroups) * GH;
  const int tid = threadIdx.x, l = tid & 63, wv = tid >> 6;
  const int n = l & 15, g = l >> 4;
  const int v = tid % VECS, run = tid / VECS;
  const int hh = v / VPH, c0 = (v % VPH) * 8;
  const unsigned stride = (unsigned)H * D * 2;                 // bytes per token row
  const unsigned coff = (unsigned)((h0 + hh) * D + c0) * 2;    // this thread's columns, in bytes

  const int ntiles = (Tn + TT - 1) / TT;
  const int tile0 = blockIdx.x * tiles_per_block;
  const int tile_end = min(ntiles, tile0 + tiles_per_block);
  // this workgroup's tokens [first, last) and the three rows before them; the host has checked that the range
  // stays far below 2^32 bytes, so that the wrapped offsets of rows -3 .. -1 fall outside the descriptor
  const int first = tile0 * TT, last = min(tile_end * TT, Tn), lo = max(first - 3, 0);
  const __amdgpu_buffer_rsrc_t src = __builtin_amdgcn_make_buffer_rsrc(
      (void*)(reinterpret_cast<const char*>(x) + ((size_t)b * Tn + lo) * stride), 0, (int)((unsigned)(last - lo) * stride),
      kRsrcFlags);
  const __amdgpu_buffer_rsrc_t dst = __builtin_amdgcn_make_buffer_rsrc(
      (void*)(reinterpret_cast<char*>(y) + ((size_t)b * Tn + first) * stride), 0, (int)((unsigned)(last - first) * stride),
      kRsrcFlags);

  u32x4 raw[NTOK + 3];
  auto load_tile = [&](int t0) {
    const unsigned base = (unsigned)(t0 + run * NTOK - 3 - lo) * stride + coff;
#pragma unroll
    for (int j = 0; j < NTOK + 3; ++j) raw[j] = __builtin_amdgcn_raw_buffer_load_b128(src, (int)(base + j * stride), 0, 0);
  };
  load_tile(first);
  if (first == 0 && halo != nullptr && run == 0) {
    // the rows before the first token come from the caller's halo (oldest row first, W - 1 rows)
    const __amdgpu_buffer_rsrc_t hsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(reinterpret_cast<const char*>(halo) + (size_t)b * (W - 1) * stride), 0, (int)((unsigned)(W - 1) * stride),
        kRsrcFlags);
#pragma unroll
    for (int j = 0; j < 3; ++j)
      if (j - 3 >= -(W - 1)) raw[j] = __builtin_amdgcn_raw_buffer_load_b128(hsrc, (int)((unsigned)(W - 4 + j) * stride + coff), 0, 0);
  }
  // conv weights of this thread's 8 channels
  float wt[8][4];
#pragma unroll
  for (int c = 0; c < 8; ++c)
#pragma unroll
    for (int dl = 0; dl < 4; ++dl) wt[c][dl] = dl < W ? bf_to_f(w[((size_t)(h0 + hh) * D + c0 + c) * W + dl]) : 0.f;
  // the matrix, transposed into LDS
  {
    const bf16_t* wsrc = wf + (size_t)(h0 / group) * D * D;
    for (int e = tid; e < D * D / 8; e += 256) {
      const int c = e / VPH, f0 = (e % VPH) * 8;
      const uint4 u = *reinterpret_cast<const uint4*>(wsrc + (size_t)c * D + f0);
      const uint32_t uu[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
      for (int i = 0; i < 8; ++i)
        *reinterpret_cast<bf16_t*>(wts + (f0 + i) * RS + c * 2) = (bf16_t)(uu[i >> 1] >> (16 * (i & 1)));
    }
  }

  for (int tile = tile0; tile < tile_end; ++tile) {
    const int t0 = tile * TT;
    // conv of this thread's 8 tokens x 8 channels; taps beyond W are skipped, not multiplied by zero
#pragma unroll
    for (int i = 0; i < NTOK; ++i) {
      float acc[8];
#pragma unroll
      for (int c = 0; c < 8; ++c) acc[c] = 0.f;
#pragma unroll
      for (int dl = 0; dl < 4; ++dl) {
        if (dl < W) {
          const u32x4 r = raw[i + 3 - dl];
#pragma unroll
          for (int c = 0; c < 8; ++c) {
            const float xv = (c & 1) ? __uint_as_float(r[c >> 1] & 0xffff0000u) : __uint_as_float(r[c >> 1] << 16);
            acc[c] = fmaf(wt[c][dl], xv, acc[c]);
          }
        }
      }
      const uint4 pk = make_uint4(pack2(acc[0], acc[1]), pack2(acc[2], acc[3]), pack2(acc[4], acc[5]), pack2(acc[6], acc[7]));
      *reinterpret_cast<uint4*>(xs + (size_t)((run * NTOK + i) * GH + hh) * RS + c0 * 2) = pk;
    }
    __syncthreads();                          // the tile (and, the first time, the matrix) is in LDS
    if (tile + 1 < tile_end) load_tile(t0 + TT);
#pragma unroll 1
    for (int rg = wv; rg < ROWS / 16; rg += 4) {
      unsigned char* rows = xs + (size_t)(16 * rg) * RS;
      bf16x8 bfrag[KS];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) bfrag[ks] = *reinterpret_cast<const bf16x8*>(rows + n * RS + (32 * ks + 8 * g) * 2);
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int ft = 0; ft < FT; ++ft) {
        floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const bf16x8 afrag = *reinterpret_cast<const bf16x8*>(wts + (16 * ft + n) * RS + (32 * ks + 8 * g) * 2);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(afrag, bfrag[ks], acc, 0, 0, 0);
        }
        // lane (n, g): features 16 ft + 4 g + i of row n; every lane of the wave has read the rows already
        *reinterpret_cast<uint2*>(rows + n * RS + (16 * ft + 4 * g) * 2) =
            make_uint2(pack2(apply_phi<ELU>(acc[0]), apply_phi<ELU>(acc[1])),
                       pack2(apply_phi<ELU>(acc[2]), apply_phi<ELU>(acc[3])));
      }
      __builtin_amdgcn_wave_barrier();        // LDS serves one wave's requests in order: the rows are complete below
#pragma unroll
      for (int it = 0; it < 16 * VPH / 64; ++it) {
        const int idx = it * 64 + l;
        const int r = idx / VPH, vec = idx % VPH;
        const int grow = 16 * rg + r;          // row of the tile: token * GH + head
        const u32x4 u = *reinterpret_cast<const u32x4*>(rows + r * RS + vec * 16);
        const unsigned off = (unsigned)(t0 - first + grow / GH) * stride + (unsigned)((h0 + grow % GH) * D + vec * 8) * 2;
        __builtin_amdgcn_raw_buffer_store_b128(u, dst, (int)off, 0, 0);
      }
    }
    __syncthreads();                          // every wave is done with the tile before the next conv overwrites it
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

namespace {

constexpr int kComputeUnits = 256;   // MI355X

template <int D, int GH, int TT>
hipError_t launch_mfma(const ConvParams& p, const void* wf, int group, hipStream_t stream) {
  constexpr int RS = D * 2 + 16;
  constexpr int lds = (D + TT * GH) * RS;
  constexpr int kResident = (160 * 1024 / lds) < 3 ? (160 * 1024 / lds) : 3;   // workgroups per compute unit (LDS, registers)
  if (lds > 64 * 1024) {
    // above the default limit: raise it once per device, for both instances
    constexpr int kMaxDev = 64;
    static std::once_flag once[kMaxDev];
    static hipError_t status[kMaxDev];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    auto set = [&] {
      const void* instances[4] = {reinterpret_cast<const void*>(conv_feature_mfma_kernel<D, GH, TT, true, 4>),
                                  reinterpret_cast<const void*>(conv_feature_mfma_kernel<D, GH, TT, false, 4>),
                                  reinterpret_cast<const void*>(conv_feature_mfma_kernel<D, GH, TT, true, 0>),
                                  reinterpret_cast<const void*>(conv_feature_mfma_kernel<D, GH, TT, false, 0>)};
      for (const void* k : instances) {
        hipError_t r = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (r != hipSuccess) return r;
      }
      return hipSuccess;
    };
    if (dev < 0 || dev >= kMaxDev) {
      e = set();
    } else {
      std::call_once(once[dev], [&] { status[dev] = set(); });
      e = status[dev];
    }
    if (e != hipSuccess) return e;
  }
  const int ntiles = (p.T + TT - 1) / TT;
  const int nbh = p.B * (p.H / GH);
  // one round of workgroups: as many per (batch, head group) as the chip holds at once, each walking a
  // contiguous run of tiles (the matrix is transposed into LDS once per workgroup)
  const int per_bh = kComputeUnits * kResident / nbh > 0 ? kComputeUnits * kResident / nbh : 1;
  const int tpb = (ntiles + per_bh - 1) / per_bh;
  // a workgroup addresses its own token range with 32-bit byte offsets
  if (((unsigned long long)tpb * TT + 16) * p.H * D * 2 >= (1ull << 31) || nbh > 65535) return hipErrorInvalidValue;
  const dim3 grid((ntiles + tpb - 1) / tpb, nbh);
  auto kernel = p.W == 4 ? (p.phi == 1 ? conv_feature_mfma_kernel<D, GH, TT, true, 4> : conv_feature_mfma_kernel<D, GH, TT, false, 4>)
                         : (p.phi == 1 ? conv_feature_mfma_kernel<D, GH, TT, true, 0> : conv_feature_mfma_kernel<D, GH, TT, false, 0>);
  hipLaunchKernelGGL(kernel, grid, dim3(256), lds, stream, (const bf16_t*)p.x, (const bf16_t*)p.w, (const bf16_t*)p.halo,
                     (const bf16_t*)wf, (bf16_t*)p.y, p.T, p.H, group, p.W, tpb);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_conv_feature(const ConvParams& p, const void* wf, int group, hipStream_t stream) {
  if (p.bf16) {
    // four adjacent heads per workgroup where they share a matrix (wider contiguous rows), else one
    const bool four = group % 4 == 0;
    // rows per tile: 256 at d = 64; at d = 128 the matrix takes 34 KB of LDS, and 64-row tiles (three workgroups
    // per compute unit instead of two) measured 15 % faster for the four-head case, 128 rows for single heads
    if (p.d == 64) return four ? launch_mfma<64, 4, 64>(p, wf, group, stream) : launch_mfma<64, 1, 256>(p, wf, group, stream);
    return four ? launch_mfma<128, 4, 16>(p, wf, group, stream) : launch_mfma<128, 1, 128>(p, wf, group, stream);
  }
  const dim3 grid((p.T + kTile * kTilesPerBlock - 1) / (kTile * kTilesPerBlock), p.B * p.H);
  if (p.d == 64) {
    constexpr int lds = kTile * (64 + 2) * 4;
    hipLaunchKernelGGL(conv_feature_f32_kernel<64>, grid, dim3(256), lds, stream, (const float*)p.x, (const float*)p.w,
                       (const float*)p.halo, (const float*)wf, (float*)p.y, p.B, p.T, p.H, group, p.W, p.phi);
  } else {
    constexpr int lds = kTile * (128 + 2) * 4;
    hipLaunchKernelGGL(conv_feature_f32_kernel<128>, grid, dim3(256), lds, stream, (const float*)p.x, (const float*)p.w,
                       (const float*)p.halo, (const float*)wf, (float*)p.y, p.B, p.T, p.H, group, p.W, p.phi);
  }
  return hipGetLastError();
}

}  // namespace lawcat
