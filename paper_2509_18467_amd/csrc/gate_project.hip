// Where the gate logits of paper section 4.2 come from: two consecutive low-rank linear layers on the layer
// input (the appendix's ablation on the rank of the gate function; rank 32 in the distilled models),
//   g[b,t,n] = sum_r ( sum_c x[b,t,c] * w1[r,c] ) * w2[n,r] + bias[n],   n over the Hkv * dk key channels.
// Streaming and HBM-bound: dm * 2 bytes read and N * 2 written per token against 2 * rank * (dm + N) flops
// (26 flop/B at dm = 2048, N = 512), so the matrix cores are used for what they are, a dense contraction, and
// the kernel is laid out around the reads of x.
//   bf16 storage, rank 32: both products transposed so that no operand is ever shuffled,
//     H^T = W1 x^T   (A = 16 rows of w1, read from L2 in fragment layout; B = 16 tokens of x, read from HBM as whole
//                     row pieces and turned into fragment layout through the wave's own LDS rows),
//     G^T = W2 H^T   (the two accumulator tiles of H^T, rounded to bf16, ARE the B operand: k slot s < 4 is
//                     rank 4g + s, slot s >= 4 rank 16 + 4g + s - 4; w2 rows are read with the same permutation),
//     a lane then holds 4 adjacent channels of one token; they pass through the wave's own LDS rows and leave
//     as whole 256-byte row pieces.  The four waves of a workgroup share 16 or 32 tokens and split the channels
//     of both products.
//   anything else (fp32 storage, other ranks): one workgroup per token, plain fp32 FMAs.
#include "kernels.h"

namespace lawcat {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((vector_size(16)));

constexpr int kRsrcFlags = 0x00020000;  // raw buffer, 32-bit data format of gfx9-family descriptors
constexpr int kRank = 32;               // what the matrix-core kernel is built for
constexpr int kSlab = 128;              // channels of x per step of the first product
constexpr int kGroupCh = 128;           // output channels staged per store round

__device__ inline uint32_t pack2(float a, float b) {
  bf16x2 v = {(__bf16)a, (__bf16)b};  // round to nearest even
  return __builtin_bit_cast(uint32_t, v);
}
__device__ inline float bf_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ inline float bf_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// grid (ceil(rows / (16 TT))), 4 waves; rows = B * T tokens.  A workgroup owns 16 TT tokens (TT tiles of 16): its
// waves split the channels of x four ways for the first product (slab w, w + 4, ...), add their partial H^T
// through LDS, and split the output channels four ways for the second (group w, w + 4, ...): short dependent
// chains and many waves per compute unit, which is what a streaming kernel needs to keep HBM busy.  With TT = 2
// every fragment of w1 (which comes from L2, 8 KB per slab) serves two MFMAs: half the L2 traffic per token,
// which measured 20 % of the kernel's time; TT = 1 where there are too few tokens to fill the chip otherwise.
constexpr int kWaves = 4;
template <int TT>
__global__ void __launch_bounds__(64 * kWaves) gate_project_mfma_kernel(const bf16_t* __restrict__ x,
                                                                        const bf16_t* __restrict__ w1,
                                                                        const bf16_t* __restrict__ w2,
                                                                        const bf16_t* __restrict__ bias,
                                                                        bf16_t* __restrict__ g, long long rows, int dm, int N) {
  constexpr int RS = kGroupCh * 2 + 16;   // LDS row stride (a 256-byte row piece plus padding), bytes
  constexpr int NR = 16 * TT;             // tokens of the workgroup
  __shared__ __attribute__((aligned(16))) unsigned char stage[kWaves * NR * RS];
  __shared__ __attribute__((aligned(16))) float part[kWaves][TT][2][64][4];
  const int l = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int n = l & 15, gq = l >> 4;
  const long long row0 = (long long)blockIdx.x * NR;   // first token of this workgroup
  const int nrows = (int)((rows - row0) < NR ? (rows - row0) : NR);
  // the rows of x and of g, each through a descriptor of its own: rows past the last token read as zero and are
  // not written
  const __amdgpu_buffer_rsrc_t xsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void*)(reinterpret_cast<const char*>(x) + (size_t)row0 * dm * 2), 0, nrows * dm * 2, kRsrcFlags);
  const __amdgpu_buffer_rsrc_t gdst = __builtin_amdgcn_make_buffer_rsrc(
      (void*)(reinterpret_cast<char*>(g) + (size_t)row0 * N * 2), 0, nrows * N * 2, kRsrcFlags);

  // ---- H^T[rank][token] = sum_c w1[rank][c] x[token][c], this wave's slabs
  // x: the slab's NR rows x 256 bytes are read as whole row pieces (16 lanes per row, 4 rows per instruction --
  // the order in which HBM likes to be asked), pass through this wave's own LDS rows and come back in fragment
  // layout (lane (token n, group gq): 16 bytes at 64 j + 16 gq).  w1 comes from L2 and is read in fragment
  // layout directly.
  floatx4 acc[TT][2];
#pragma unroll
  for (int tt = 0; tt < TT; ++tt) { acc[tt][0] = floatx4{0.f, 0.f, 0.f, 0.f}; acc[tt][1] = floatx4{0.f, 0.f, 0.f, 0.f}; }
  unsigned char* mine = stage + (size_t)wv * NR * RS;
  const int lr = l >> 4, lp = l & 15;                                   // row within a group of 4, 16-byte piece
  const unsigned xoff = (unsigned)lr * dm * 2 + lp * 16;
  const bf16_t* wrow0 = w1 + (size_t)n * dm + gq * 8;                    // rank n, and rank 16 + n below
  const bf16_t* wrow1 = wrow0 + (size_t)16 * dm;
  u32x4 xb[4 * TT], wa[2][4];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int it = 0; it < 4 * TT; ++it)
      xb[it] = __builtin_amdgcn_raw_buffer_load_b128(xsrc, (int)(xoff + (unsigned)(4 * it) * dm * 2 + k0 * 2), 0, 0);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      wa[0][j] = *reinterpret_cast<const u32x4*>(wrow0 + k0 + 32 * j);
      wa[1][j] = *reinterpret_cast<const u32x4*>(wrow1 + k0 + 32 * j);
    }
  };
  constexpr int kStep = kSlab * kWaves;
  if (wv * kSlab < dm) fetch(wv * kSlab);
#pragma unroll 1
  for (int k0 = wv * kSlab; k0 < dm; k0 += kStep) {
    // this slab's rows into LDS (the previous slab's fragment reads were issued before these writes, and LDS
    // serves one wave's requests in order)
#pragma unroll
    for (int it = 0; it < 4 * TT; ++it) *reinterpret_cast<u32x4*>(mine + (4 * it + lr) * RS + lp * 16) = xb[it];
    u32x4 wc[2][4];
#pragma unroll
    for (int j = 0; j < 4; ++j) { wc[0][j] = wa[0][j]; wc[1][j] = wa[1][j]; }
    __builtin_amdgcn_wave_barrier();
    if (k0 + kStep < dm) fetch(k0 + kStep);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
#pragma unroll
      for (int tt = 0; tt < TT; ++tt) {
        const bf16x8 b = *reinterpret_cast<const bf16x8*>(mine + (16 * tt + n) * RS + 64 * j + 16 * gq);
        acc[tt][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wc[0][j]), b, acc[tt][0], 0, 0, 0);
        acc[tt][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wc[1][j]), b, acc[tt][1], 0, 0, 0);
      }
    }
  }
  // the four partial sums meet in LDS; every wave adds them up in the same order
#pragma unroll
  for (int tt = 0; tt < TT; ++tt) {
    *reinterpret_cast<floatx4*>(&part[wv][tt][0][l][0]) = acc[tt][0];
    *reinterpret_cast<floatx4*>(&part[wv][tt][1][l][0]) = acc[tt][1];
  }
  __syncthreads();
  bf16x8 hb[TT];
#pragma unroll
  for (int tt = 0; tt < TT; ++tt) {
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
      floatx4 sum = *reinterpret_cast<const floatx4*>(&part[0][tt][mt][l][0]);
#pragma unroll
      for (int w = 1; w < kWaves; ++w) {
        const floatx4 p = *reinterpret_cast<const floatx4*>(&part[w][tt][mt][l][0]);
#pragma unroll
        for (int i = 0; i < 4; ++i) sum[i] += p[i];
      }
      acc[tt][mt] = sum;
    }
    // lane (token n, group gq): acc[tt][mt][i] = H^T[16 mt + 4 gq + i][16 tt + n]; as the next product's B operand
    const u32x4 hbits = {pack2(acc[tt][0][0], acc[tt][0][1]), pack2(acc[tt][0][2], acc[tt][0][3]),
                         pack2(acc[tt][1][0], acc[tt][1][1]), pack2(acc[tt][1][2], acc[tt][1][3])};
    hb[tt] = __builtin_bit_cast(bf16x8, hbits);
  }

  // ---- G^T[channel][token] = sum_r w2[channel][r] H^T[r][token] + bias[channel], this wave's groups of 128 channels
  // (staged for the store in the same LDS rows: every wave is past its slabs, the barrier above says so)
  for (int c0 = wv * kGroupCh; c0 < N; c0 += kGroupCh * kWaves) {
#pragma unroll
    for (int ct = 0; ct < kGroupCh / 16; ++ct) {
      const bf16_t* wr = w2 + (size_t)(c0 + 16 * ct + n) * kRank;      // row of w2 = 32 ranks = 64 bytes
      const uint2 lo = *reinterpret_cast<const uint2*>(wr + 4 * gq);
      const uint2 hi = *reinterpret_cast<const uint2*>(wr + 16 + 4 * gq);
      const u32x4 abits = {lo.x, lo.y, hi.x, hi.y};
      float bv[4] = {0.f, 0.f, 0.f, 0.f};
      if (bias != nullptr) {
        const uint2 bb = *reinterpret_cast<const uint2*>(bias + c0 + 16 * ct + 4 * gq);
        bv[0] = bf_lo(bb.x); bv[1] = bf_hi(bb.x); bv[2] = bf_lo(bb.y); bv[3] = bf_hi(bb.y);
      }
#pragma unroll
      for (int tt = 0; tt < TT; ++tt) {
        floatx4 out = {bv[0], bv[1], bv[2], bv[3]};
        out = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, abits), hb[tt], out, 0, 0, 0);
        // lane (token 16 tt + n, gq): channels c0 + 16 ct + 4 gq + i
        *reinterpret_cast<uint2*>(mine + (16 * tt + n) * RS + (16 * ct + 4 * gq) * 2) =
            make_uint2(pack2(out[0], out[1]), pack2(out[2], out[3]));
      }
    }
    __builtin_amdgcn_wave_barrier();   // LDS serves one wave's requests in order: the rows are complete below
#pragma unroll
    for (int it = 0; it < NR * (kGroupCh / 8) / 64; ++it) {
      const int idx = it * 64 + l;
      const int r = idx / (kGroupCh / 8), vec = idx % (kGroupCh / 8);
      const u32x4 u = *reinterpret_cast<const u32x4*>(mine + r * RS + vec * 16);
      __builtin_amdgcn_raw_buffer_store_b128(u, gdst, (int)((unsigned)r * N * 2 + (c0 + vec * 8) * 2), 0, 0);
    }
    __builtin_amdgcn_wave_barrier();   // the rows are read before the next round overwrites them
  }
}

// Any storage type, any rank: one workgroup per token.
template <typename T>
__device__ inline float to_f(T v);
template <>
__device__ inline float to_f<float>(float v) { return v; }
template <>
__device__ inline float to_f<bf16_t>(bf16_t v) { return __uint_as_float((uint32_t)v << 16); }
__device__ inline void from_f(float v, float* p) { *p = v; }
__device__ inline void from_f(float v, bf16_t* p) { *p = (bf16_t)(pack2(v, 0.f) & 0xffffu); }

template <typename T>
__global__ void __launch_bounds__(256) gate_project_generic_kernel(const T* __restrict__ x, const T* __restrict__ w1,
                                                                   const T* __restrict__ w2, const T* __restrict__ bias,
                                                                   T* __restrict__ g, int dm, int rank, int N) {
  extern __shared__ float sm[];   // x row (dm floats), then h (rank floats)
  float* xs = sm;
  float* h = sm + dm;
  const size_t row = blockIdx.x;
  for (int c = threadIdx.x; c < dm; c += 256) xs[c] = to_f<T>(x[row * dm + c]);
  __syncthreads();
  for (int r = threadIdx.x; r < rank; r += 256) {
    float acc = 0.f;
    for (int c = 0; c < dm; ++c) acc = fmaf(xs[c], to_f<T>(w1[(size_t)r * dm + c]), acc);
    h[r] = acc;
  }
  __syncthreads();
  for (int nn = threadIdx.x; nn < N; nn += 256) {
    float acc = bias != nullptr ? to_f<T>(bias[nn]) : 0.f;
    for (int r = 0; r < rank; ++r) acc = fmaf(h[r], to_f<T>(w2[(size_t)nn * rank + r]), acc);
    from_f(acc, g + row * N + nn);
  }
}

}  // namespace

hipError_t launch_gate_project(const GateProjectParams& p, hipStream_t stream) {
  const long long rows = (long long)p.B * p.T;
  if (rows > 0x7fffffffLL) return hipErrorInvalidValue;
  if (p.bf16 && p.rank == kRank && p.dm % kSlab == 0 && p.N % kGroupCh == 0 && (long long)32 * p.dm * 2 < (1ll << 31) &&
      (long long)32 * p.N * 2 < (1ll << 31)) {
    // 32 tokens per workgroup where that still leaves two workgroups for every compute unit, else 16
    if ((rows + 31) / 32 >= 512)
      hipLaunchKernelGGL(gate_project_mfma_kernel<2>, dim3((unsigned)((rows + 31) / 32)), dim3(64 * kWaves), 0, stream,
                         (const bf16_t*)p.x, (const bf16_t*)p.w1, (const bf16_t*)p.w2, (const bf16_t*)p.bias, (bf16_t*)p.g, rows, p.dm, p.N);
    else
      hipLaunchKernelGGL(gate_project_mfma_kernel<1>, dim3((unsigned)((rows + 15) / 16)), dim3(64 * kWaves), 0, stream,
                         (const bf16_t*)p.x, (const bf16_t*)p.w1, (const bf16_t*)p.w2, (const bf16_t*)p.bias, (bf16_t*)p.g, rows, p.dm, p.N);
    return hipGetLastError();
  }
  const size_t lds = (size_t)(p.dm + p.rank) * sizeof(float);
  if (lds > 64 * 1024) return hipErrorInvalidValue;
  if (p.bf16)
    hipLaunchKernelGGL(gate_project_generic_kernel<bf16_t>, dim3((unsigned)rows), dim3(256), lds, stream, (const bf16_t*)p.x,
                       (const bf16_t*)p.w1, (const bf16_t*)p.w2, (const bf16_t*)p.bias, (bf16_t*)p.g, p.dm, p.rank, p.N);
  else
    hipLaunchKernelGGL(gate_project_generic_kernel<float>, dim3((unsigned)rows), dim3(256), lds, stream, (const float*)p.x,
                       (const float*)p.w1, (const float*)p.w2, (const float*)p.bias, (float*)p.g, p.dm, p.rank, p.N);
  return hipGetLastError();
}

}  // namespace lawcat
