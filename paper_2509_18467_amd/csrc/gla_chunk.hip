// Host side of the bf16 matrix-core prefill: segment plan, workspace size, dispatch to the
// per-head-dimension translation units.
#include "gla_chunk_impl.h"

namespace lawcat {
namespace chunk {
hipError_t launch_d64(const ChunkArgs& a, int group, int mode, hipStream_t stream, const TraceEvents& ev);
hipError_t launch_d128(const ChunkArgs& a, int group, int mode, hipStream_t stream, const TraceEvents& ev);
}  // namespace chunk

bool chunk_path_supports(int group) { return group >= 1 && group <= 64; }

ChunkPlan make_chunk_plan(int B, int T, int Hkv, int d, int carry_mode, int segment) {
  ChunkPlan p;
  const int heads = B * Hkv;
  int seg_len;
  if (carry_mode == 1) {
    seg_len = (T + 63) / 64 * 64;
  } else if (segment > 0) {
    seg_len = segment;
  } else {
    // enough workgroups to fill 256 compute units once (two 4-wave teams per unit at head dim 64, one
    // 8-wave team at 128).  Segments of two granules (128 tokens) at least, except where even those would leave
    // more than half of the chip without a workgroup: short sequences are bound by the serial work of one
    // workgroup, and one-granule segments halve it (T = 1K .. 2K: 31 -> 23 us at head dim 64, 51 -> 41 at 128)
    const int slots = d == 64 ? 512 : 256;
    const int want = (slots + heads - 1) / heads;
    seg_len = (T + want - 1) / want;
    seg_len = (seg_len + 63) / 64 * 64;
    if (seg_len < 128) seg_len = (long long)((T + 127) / 128) * heads * 2 <= slots ? 64 : 128;
  }
  p.seg_len = seg_len;
  p.nseg = (T + seg_len - 1) / seg_len;
  // per (head, segment): contribution or start state S | z | total decay, then one flag word each
  p.workspace_bytes = p.nseg > 1 ? (size_t)heads * p.nseg * ((d * d + 2 * d) * sizeof(float) + sizeof(int)) : 0;
  return p;
}

hipError_t launch_gla_chunk(const ChunkParams& p, hipStream_t stream) {
  chunk::ChunkArgs a;
  a.q = (const bf16_t*)p.q; a.k = (const bf16_t*)p.k; a.v = (const bf16_t*)p.v; a.g = (const bf16_t*)p.g;
  a.wq = (const bf16_t*)p.wq; a.wk = (const bf16_t*)p.wk;
  a.q_halo = (const bf16_t*)p.q_halo; a.k_halo = (const bf16_t*)p.k_halo;
  a.S0 = p.S0; a.z0 = p.z0; a.o = (bf16_t*)p.o; a.den_out = p.den_out; a.S_out = p.S_out; a.z_out = p.z_out;
  a.q_tail = (bf16_t*)p.q_tail; a.k_tail = (bf16_t*)p.k_tail;
  a.ws = (float*)p.workspace;
  a.seq_start = p.seq_start;
  a.seg_live = reinterpret_cast<int*>(a.ws + (size_t)p.B * p.Hkv * p.plan.nseg * (p.d * p.d + 2 * p.d));
  a.B = p.B; a.T = p.T; a.Hq = p.Hq; a.Hkv = p.Hkv; a.W = p.W;
  a.seg_len = p.plan.seg_len; a.nseg = p.plan.nseg;
  a.gate_scale = p.gate_scale; a.eps = p.eps;
  const int group = p.Hq / p.Hkv;
  const int mode = !p.fuse_conv ? chunk::kPlain : (p.phi == 1 ? chunk::kConvElu : chunk::kConvId);
  const chunk::TraceEvents ev{p.ev_start, p.ev_stop};
  return p.d == 64 ? chunk::launch_d64(a, group, mode, stream, ev) : chunk::launch_d128(a, group, mode, stream, ev);
}

}  // namespace lawcat
