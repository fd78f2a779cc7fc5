// Host side of the C ABI declared in include/lawcat.h: argument checks, workspace
// layout, kernel selection.  Every check runs before anything is enqueued, so the
// error paths can be exercised on a machine without a GPU.
#include "../../include/lawcat.h"

#include <algorithm>
#include <cmath>
#include <mutex>

#include "kernels.h"

using namespace lawcat;

namespace {

// Scratch of lawcat_layer_prefill_static: one copy per GPU that loads the library, kept until the process ends.
// In host code the array's name is only a handle for hipGetSymbolAddress; kernels receive the device address
// that static_scratch() looks up once per device.
__device__ __align__(256) unsigned char scratch[LAWCAT_STATIC_WORKSPACE_BYTES];

hipError_t static_scratch(void** out) {
  constexpr int kMaxDev = 64;
  static std::once_flag once[kMaxDev];
  static hipError_t err[kMaxDev];
  static void* ptr[kMaxDev];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDev) return hipErrorInvalidDevice;
  std::call_once(once[dev], [&] {
    void* p = nullptr;
    err[dev] = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));  // the current device's copy
    ptr[dev] = p;
  });
  if (err[dev] != hipSuccess) return err[dev];
  *out = ptr[dev];
  return hipSuccess;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t align_up(size_t n, size_t a) { return (n + a - 1) / a * a; }

// Checks common to every call.  `need_T` is false for the decode step.
int check_desc(const lawcat_desc* d, bool need_T) {
  if (d == nullptr) return LAWCAT_E_NULL;
  if (d->struct_size != sizeof(lawcat_desc)) return LAWCAT_E_BAD_DESC;
  if (d->B <= 0 || d->Hq <= 0 || d->Hkv <= 0 || d->dk <= 0 || d->dv <= 0) return LAWCAT_E_BAD_DESC;
  if (need_T && d->T <= 0) return LAWCAT_E_BAD_DESC;
  if (d->Hq % d->Hkv != 0) return LAWCAT_E_BAD_DESC;
  if (d->dtype != LAWCAT_DTYPE_F32 && d->dtype != LAWCAT_DTYPE_BF16) return LAWCAT_E_BAD_DESC;
  if (d->feature_map != LAWCAT_PHI_IDENTITY && d->feature_map != LAWCAT_PHI_ELU1) return LAWCAT_E_BAD_DESC;
  if (d->carry_mode < LAWCAT_CARRY_AUTO || d->carry_mode > LAWCAT_CARRY_TWO_LEVEL) return LAWCAT_E_BAD_DESC;
  if (!(d->gate_scale >= 0.f) || !std::isfinite(d->gate_scale) || !std::isfinite(d->eps)) return LAWCAT_E_BAD_DESC;
  if (d->conv_width <= 0 || d->segment < 0 || d->chunk < 0) return LAWCAT_E_BAD_DESC;
  if (d->dk != d->dv || (d->dk != 64 && d->dk != 128)) return LAWCAT_E_UNSUPPORTED;
  if (d->conv_width > 4) return LAWCAT_E_UNSUPPORTED;
  if (d->chunk != 0 && d->chunk != 16) return LAWCAT_E_UNSUPPORTED;
  if (d->segment % 64 != 0) return LAWCAT_E_UNSUPPORTED;
  return LAWCAT_OK;
}

inline size_t elem_bytes(const lawcat_desc* d) { return d->dtype == LAWCAT_DTYPE_BF16 ? 2 : 4; }

// Which prefill implementation a desc selects.
enum class Path { kRecurrentF32, kChunkBf16 };
inline Path prefill_path(const lawcat_desc* d) {
  // the chunk kernels address one batch element's rows with 32-bit byte offsets (buffer loads): offsets of the
  // three rows before the first token wrap around and must still land past the end of the buffer, and the rows
  // of the last granule past T (fewer than 64) must not wrap at all, so that they read as zero
  const bool rows_fit = ((uint64_t)d->T + 128) * d->Hq * d->dk * 2 < (1ull << 32);
  // one workgroup row per (batch, kv head) on the grid's y axis
  const bool heads_fit = (uint64_t)d->B * d->Hkv <= 65535;
  return (d->dtype == LAWCAT_DTYPE_BF16 && chunk_path_supports(d->Hq / d->Hkv) && rows_fit && heads_fit)
             ? Path::kChunkBf16
             : Path::kRecurrentF32;
}

ChunkPlan plan_for(const lawcat_desc* d) {
  return make_chunk_plan(d->B, d->T, d->Hkv, d->dk, d->carry_mode, d->segment);
}

size_t workspace_bytes_checked(const lawcat_desc* d, int which) {
  switch (which) {
    case LAWCAT_CALL_CONV1D:
    case LAWCAT_CALL_GLA_STEP:
      return 0;
    case LAWCAT_CALL_GLA_PREFILL:
      return prefill_path(d) == Path::kChunkBf16 ? plan_for(d).workspace_bytes : 0;
    case LAWCAT_CALL_LAYER_PREFILL: {
      if (prefill_path(d) == Path::kChunkBf16) return plan_for(d).workspace_bytes;
      // unfused: q-dot and k-dot staged in the storage type
      const size_t rows = (size_t)d->B * d->T;
      return align_up(rows * d->Hq * d->dk * elem_bytes(d), 256) + align_up(rows * d->Hkv * d->dk * elem_bytes(d), 256);
    }
    case LAWCAT_CALL_LAYER_PREFILL_FM: {
      // q-dot and k-dot staged in the storage type, then whatever lawcat_gla_prefill needs
      const size_t rows = (size_t)d->B * d->T;
      const size_t inner = prefill_path(d) == Path::kChunkBf16 ? plan_for(d).workspace_bytes : 0;
      return align_up(rows * d->Hq * d->dk * elem_bytes(d), 256) + align_up(rows * d->Hkv * d->dk * elem_bytes(d), 256) +
             align_up(inner, 256);
    }
    case LAWCAT_CALL_GLA_BACKWARD:
      return gla_backward_workspace_bytes(d->B, d->T, d->Hq, d->Hkv, d->dk);
    case LAWCAT_CALL_CONV1D_BACKWARD:
      return conv_backward_workspace_bytes(d->B, d->T, d->Hq, d->dk, d->conv_width);
    default:
      return 0;
  }
}

// Segments of a packed batch of sequences (one set of launches): cut as for ONE sequence of all the tokens, so that
// the workgroups are about as many as the chip holds and about equally long whatever the mix of lengths; slots are
// laid out for the longest sequence.
ChunkPlan varlen_plan(const lawcat_desc* d, const int32_t* seq_start) {
  const long long total = seq_start[d->B];
  int longest = 1;
  for (int i = 0; i < d->B; ++i) longest = std::max(longest, (int)(seq_start[i + 1] - seq_start[i]));
  ChunkPlan one = make_chunk_plan(1, (int)std::min<long long>(total, 0x7fffffc0LL), d->Hkv, d->dk, d->carry_mode, d->segment);
  ChunkPlan p;
  const int whole = (longest + 63) / 64 * 64;
  p.seg_len = std::min(one.seg_len, whole);
  if (d->carry_mode == LAWCAT_CARRY_SEQUENTIAL) p.seg_len = whole;
  if (d->segment == 0 && d->carry_mode != LAWCAT_CARRY_SEQUENTIAL) {
    // every sequence rounds its segment count up: lengthen the segments until the workgroups fit the chip in one
    // round (a few too many would double the time of the pass)
    const long long slots = d->dk == 64 ? 512 : 256;
    auto groups = [&](int seg_len) {
      long long n = 0;
      for (int i = 0; i < d->B; ++i) n += (seq_start[i + 1] - seq_start[i] + seg_len - 1) / seg_len;
      return n * d->Hkv;
    };
    while (p.seg_len < whole && groups(p.seg_len) > slots) p.seg_len += 64;
  }
  p.nseg = (longest + p.seg_len - 1) / p.seg_len;
  p.workspace_bytes = p.nseg > 1 ? (size_t)d->B * d->Hkv * p.nseg * ((d->dk * d->dk + 2 * d->dk) * sizeof(float) + sizeof(int)) : 0;
  return p;
}

int hip_status(hipError_t e) { return e == hipSuccess ? LAWCAT_OK : LAWCAT_E_HIP; }

}  // namespace

extern "C" {

size_t lawcat_workspace_bytes(const lawcat_desc* desc, int which_call) {
  const bool need_T = which_call != LAWCAT_CALL_GLA_STEP;
  if (check_desc(desc, need_T) != LAWCAT_OK) return 0;
  return workspace_bytes_checked(desc, which_call);
}

int lawcat_conv1d_causal(const lawcat_desc* desc, int n_heads, const void* x, const void* w, const void* halo,
                         void* y, void* tail_out, void* stream) {
  int st = check_desc(desc, true);
  if (st != LAWCAT_OK) return st;
  if (n_heads <= 0) return LAWCAT_E_BAD_DESC;
  if (x == nullptr || w == nullptr || y == nullptr) return LAWCAT_E_NULL;
  if (!aligned16(x) || !aligned16(w) || !aligned16(y) || !aligned16(halo) || !aligned16(tail_out))
    return LAWCAT_E_ALIGN;
  ConvParams p{};
  p.x = x; p.w = w; p.halo = desc->conv_width > 1 ? halo : nullptr; p.y = y;
  p.tail_out = desc->conv_width > 1 ? tail_out : nullptr;
  p.B = desc->B; p.T = desc->T; p.H = n_heads; p.d = desc->dk; p.W = desc->conv_width;
  p.phi = desc->feature_map; p.bf16 = desc->dtype == LAWCAT_DTYPE_BF16;
  return hip_status(launch_conv1d(p, static_cast<hipStream_t>(stream)));
}

int lawcat_conv1d_feature(const lawcat_desc* desc, int n_heads, const void* x, const void* w, const void* wf,
                          const void* halo, void* y, void* tail_out, void* stream) {
  int st = check_desc(desc, true);
  if (st != LAWCAT_OK) return st;
  if (n_heads <= 0 || n_heads % desc->Hkv != 0) return LAWCAT_E_BAD_DESC;
  if (x == nullptr || w == nullptr || wf == nullptr || y == nullptr) return LAWCAT_E_NULL;
  if (!aligned16(x) || !aligned16(w) || !aligned16(wf) || !aligned16(y) || !aligned16(halo) || !aligned16(tail_out))
    return LAWCAT_E_ALIGN;
  ConvParams p{};
  p.x = x; p.w = w; p.halo = desc->conv_width > 1 ? halo : nullptr; p.y = y;
  p.tail_out = desc->conv_width > 1 ? tail_out : nullptr;
  p.B = desc->B; p.T = desc->T; p.H = n_heads; p.d = desc->dk; p.W = desc->conv_width;
  p.phi = desc->feature_map; p.bf16 = desc->dtype == LAWCAT_DTYPE_BF16;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  if (launch_conv_feature(p, wf, n_heads / desc->Hkv, hs) != hipSuccess) return LAWCAT_E_HIP;
  return hip_status(launch_conv_tail(p, hs));
}

int lawcat_gla_backward(const lawcat_desc* desc, const void* q, const void* k, const void* v, const void* gate_logits,
                        const float* den, const void* dO, const float* S0, const float* z0, void* dq,
                        void* dk, void* dv, void* dgate_logits, float* dS0, float* dz0, void* workspace,
                        size_t workspace_bytes, void* stream) {
  int st = check_desc(desc, true);
  if (st != LAWCAT_OK) return st;
  if (!gla_backward_supports(desc->dk, desc->Hq / desc->Hkv) || (uint64_t)desc->B * desc->Hkv > 65535) return LAWCAT_E_UNSUPPORTED;
  if (!q || !k || !v || !gate_logits || !den || !dO || !dq || !dk || !dv || !dgate_logits) return LAWCAT_E_NULL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(gate_logits) || !aligned16(den) ||
      !aligned16(dO) || !aligned16(S0) || !aligned16(z0) || !aligned16(dq) || !aligned16(dk) || !aligned16(dv) ||
      !aligned16(dgate_logits) || !aligned16(dS0) || !aligned16(dz0) || !aligned16(workspace))
    return LAWCAT_E_ALIGN;
  const size_t need = workspace_bytes_checked(desc, LAWCAT_CALL_GLA_BACKWARD);
  if (workspace == nullptr || workspace_bytes < need) return LAWCAT_E_WORKSPACE;
  GlaBackwardParams p{};
  p.q = q; p.k = k; p.v = v; p.g = gate_logits; p.den = den; p.dO = dO; p.S0 = S0; p.z0 = z0;
  p.dq = dq; p.dk = dk; p.dv = dv; p.dg = dgate_logits; p.dS0 = dS0; p.dz0 = dz0; p.workspace = workspace;
  p.B = desc->B; p.T = desc->T; p.Hq = desc->Hq; p.Hkv = desc->Hkv; p.d = desc->dk;
  p.gate_scale = desc->gate_scale; p.bf16 = desc->dtype == LAWCAT_DTYPE_BF16;
  return hip_status(launch_gla_backward(p, static_cast<hipStream_t>(stream)));
}

int lawcat_conv1d_backward(const lawcat_desc* desc, int n_heads, const void* x, const void* w, const void* halo,
                           const void* dy, void* dx, float* dw, void* dhalo, void* workspace, size_t workspace_bytes,
                           void* stream) {
  int st = check_desc(desc, true);
  if (st != LAWCAT_OK) return st;
  if (n_heads <= 0) return LAWCAT_E_BAD_DESC;
  if (!x || !w || !dy || !dx || !dw) return LAWCAT_E_NULL;
  if (!aligned16(x) || !aligned16(w) || !aligned16(halo) || !aligned16(dy) || !aligned16(dx) || !aligned16(dw) ||
      !aligned16(dhalo) || !aligned16(workspace))
    return LAWCAT_E_ALIGN;
  if ((uint64_t)desc->B > 65535 || ((uint64_t)desc->T + 63) / 64 > 65535) return LAWCAT_E_UNSUPPORTED;   // grid limits
  const size_t need = conv_backward_workspace_bytes(desc->B, desc->T, n_heads, desc->dk, desc->conv_width);
  if (workspace == nullptr || workspace_bytes < need) return LAWCAT_E_WORKSPACE;
  ConvBackwardParams p{};
  p.x = x; p.w = w; p.halo = desc->conv_width > 1 ? halo : nullptr; p.dy = dy;
  p.dx = dx; p.dw = dw; p.dhalo = desc->conv_width > 1 ? dhalo : nullptr; p.workspace = workspace;
  p.B = desc->B; p.T = desc->T; p.H = n_heads; p.d = desc->dk; p.W = desc->conv_width;
  p.phi = desc->feature_map; p.bf16 = desc->dtype == LAWCAT_DTYPE_BF16;
  return hip_status(launch_conv_backward(p, static_cast<hipStream_t>(stream)));
}

int lawcat_gate_project(const lawcat_desc* desc, int d_model, int rank, const void* x, const void* w1, const void* w2,
                        const void* bias, void* gate_logits, void* stream) {
  int st = check_desc(desc, true);
  if (st != LAWCAT_OK) return st;
  if (d_model < 1 || rank < 1) return LAWCAT_E_BAD_DESC;
  // rows of x and of the weights are read 16 bytes at a time; the one-token-per-workgroup kernel keeps a row of x
  // and the intermediate in 64 KB of LDS
  if (d_model % 8 != 0 || rank % 8 != 0 || ((size_t)d_model + rank) * sizeof(float) > 64 * 1024) return LAWCAT_E_UNSUPPORTED;
  if (x == nullptr || w1 == nullptr || w2 == nullptr || gate_logits == nullptr) return LAWCAT_E_NULL;
  if (!aligned16(x) || !aligned16(w1) || !aligned16(w2) || !aligned16(bias) || !aligned16(gate_logits)) return LAWCAT_E_ALIGN;
  GateProjectParams p{};
  p.x = x; p.w1 = w1; p.w2 = w2; p.bias = bias; p.g = gate_logits;
  p.B = desc->B; p.T = desc->T; p.dm = d_model; p.rank = rank; p.N = desc->Hkv * desc->dk;
  p.bf16 = desc->dtype == LAWCAT_DTYPE_BF16;
  return hip_status(launch_gate_project(p, static_cast<hipStream_t>(stream)));
}

int lawcat_gla_prefill(const lawcat_desc* desc, const void* q, const void* k, const void* v,
                       const void* gate_logits, const float* S0, const float* z0, void* o, float* den_out,
                       float* S_out, float* z_out, void* workspace, size_t workspace_bytes, void* stream) {
  int st = check_desc(desc, true);
  if (st != LAWCAT_OK) return st;
  if (!q || !k || !v || !gate_logits || !o || !S_out || !z_out) return LAWCAT_E_NULL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(gate_logits) || !aligned16(S0) ||
      !aligned16(z0) || !aligned16(o) || !aligned16(den_out) || !aligned16(S_out) || !aligned16(z_out) ||
      !aligned16(workspace))
    return LAWCAT_E_ALIGN;
  const size_t need = workspace_bytes_checked(desc, LAWCAT_CALL_GLA_PREFILL);
  if (need > 0 && (workspace == nullptr || workspace_bytes < need)) return LAWCAT_E_WORKSPACE;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  if (prefill_path(desc) == Path::kChunkBf16) {
    ChunkParams c{};
    c.q = q; c.k = k; c.v = v; c.g = gate_logits; c.S0 = S0; c.z0 = z0; c.o = o; c.den_out = den_out;
    c.S_out = S_out; c.z_out = z_out; c.workspace = workspace;
    c.B = desc->B; c.T = desc->T; c.Hq = desc->Hq; c.Hkv = desc->Hkv; c.d = desc->dk;
    c.W = 1; c.phi = LAWCAT_PHI_IDENTITY; c.fuse_conv = 0;
    c.gate_scale = desc->gate_scale; c.eps = desc->eps; c.plan = plan_for(desc);
    return hip_status(launch_gla_chunk(c, hs));
  }
  RecurrentParams r{};
  r.q = q; r.k = k; r.v = v; r.g = gate_logits; r.S0 = S0; r.z0 = z0; r.o = o; r.den_out = den_out;
  r.S_out = S_out; r.z_out = z_out; r.B = desc->B; r.T = desc->T; r.Hq = desc->Hq; r.Hkv = desc->Hkv;
  r.d = desc->dk; r.gate_scale = desc->gate_scale; r.eps = desc->eps;
  r.bf16 = desc->dtype == LAWCAT_DTYPE_BF16;
  return hip_status(launch_gla_recurrent(r, hs));
}

int lawcat_gla_step(const lawcat_desc* desc, const void* q, const void* k, const void* v, const void* gate_logits,
                    float* S, float* z, void* o, void* stream) {
  int st = check_desc(desc, false);
  if (st != LAWCAT_OK) return st;
  if (!q || !k || !v || !gate_logits || !S || !z || !o) return LAWCAT_E_NULL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(gate_logits) || !aligned16(S) ||
      !aligned16(z) || !aligned16(o))
    return LAWCAT_E_ALIGN;
  RecurrentParams r{};
  r.q = q; r.k = k; r.v = v; r.g = gate_logits; r.S0 = S; r.z0 = z; r.o = o; r.den_out = nullptr;
  r.S_out = S; r.z_out = z; r.B = desc->B; r.T = 1; r.Hq = desc->Hq; r.Hkv = desc->Hkv; r.d = desc->dk;
  r.gate_scale = desc->gate_scale; r.eps = desc->eps; r.bf16 = desc->dtype == LAWCAT_DTYPE_BF16;
  return hip_status(launch_gla_step(r, static_cast<hipStream_t>(stream)));
}

int lawcat_gla_steps(const lawcat_desc* desc, const void* q, const void* k, const void* v, const void* gate_logits,
                     float* S, float* z, void* o, void* stream) {
  int st = check_desc(desc, true);
  if (st != LAWCAT_OK) return st;
  if (!q || !k || !v || !gate_logits || !S || !z || !o) return LAWCAT_E_NULL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(gate_logits) || !aligned16(S) ||
      !aligned16(z) || !aligned16(o))
    return LAWCAT_E_ALIGN;
  RecurrentParams r{};
  r.q = q; r.k = k; r.v = v; r.g = gate_logits; r.S0 = S; r.z0 = z; r.o = o; r.den_out = nullptr;
  r.S_out = S; r.z_out = z; r.B = desc->B; r.T = desc->T; r.Hq = desc->Hq; r.Hkv = desc->Hkv; r.d = desc->dk;
  r.gate_scale = desc->gate_scale; r.eps = desc->eps; r.bf16 = desc->dtype == LAWCAT_DTYPE_BF16;
  return hip_status(launch_gla_steps(r, static_cast<hipStream_t>(stream)));
}

}  // extern "C"

namespace {

int layer_prefill_impl(const lawcat_desc* desc, const void* Q, const void* K, const void* V,
                       const void* gate_logits, const void* wq, const void* wk, const float* S0,
                       const float* z0, const void* q_halo, const void* k_halo, void* O, float* den_out,
                       float* S_out, float* z_out, void* q_tail_out, void* k_tail_out, void* workspace,
                       size_t workspace_bytes, void* stream, hipEvent_t ev_start, hipEvent_t ev_stop,
                       bool den_rows_packed = false) {
  int st = check_desc(desc, true);
  if (st != LAWCAT_OK) return st;
  if (!Q || !K || !V || !gate_logits || !wq || !wk || !O || !S_out || !z_out) return LAWCAT_E_NULL;
  // den_out is written one float at a time; a sequence inside a packed batch may start at any row of it
  const bool den_ok = den_rows_packed ? (reinterpret_cast<uintptr_t>(den_out) % sizeof(float) == 0) : aligned16(den_out);
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(gate_logits) || !aligned16(wq) ||
      !aligned16(wk) || !aligned16(S0) || !aligned16(z0) || !aligned16(q_halo) || !aligned16(k_halo) ||
      !aligned16(O) || !den_ok || !aligned16(S_out) || !aligned16(z_out) ||
      !aligned16(q_tail_out) || !aligned16(k_tail_out) || !aligned16(workspace))
    return LAWCAT_E_ALIGN;
  const size_t need = workspace_bytes_checked(desc, LAWCAT_CALL_LAYER_PREFILL);
  if (need > 0 && (workspace == nullptr || workspace_bytes < need)) return LAWCAT_E_WORKSPACE;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  const int bf16 = desc->dtype == LAWCAT_DTYPE_BF16;

  if (prefill_path(desc) == Path::kChunkBf16) {
    ChunkParams c{};
    c.q = Q; c.k = K; c.v = V; c.g = gate_logits; c.wq = wq; c.wk = wk; c.q_halo = q_halo; c.k_halo = k_halo;
    c.S0 = S0; c.z0 = z0; c.o = O; c.den_out = den_out; c.S_out = S_out; c.z_out = z_out;
    c.workspace = workspace;
    c.B = desc->B; c.T = desc->T; c.Hq = desc->Hq; c.Hkv = desc->Hkv; c.d = desc->dk;
    c.W = desc->conv_width; c.phi = desc->feature_map; c.fuse_conv = 1;
    c.gate_scale = desc->gate_scale; c.eps = desc->eps; c.plan = plan_for(desc);
    c.q_tail = q_tail_out; c.k_tail = k_tail_out;
    c.ev_start = ev_start; c.ev_stop = ev_stop;
    return hip_status(launch_gla_chunk(c, hs));
  }
  if (ev_start != nullptr || ev_stop != nullptr) return LAWCAT_E_UNSUPPORTED;  // only the bf16 path has the hook

  // Unfused path (fp32 storage): conv + phi into the workspace, then the fp32 recurrence.
  const size_t rows = (size_t)desc->B * desc->T;
  char* ws = static_cast<char*>(workspace);
  void* qd = ws;
  void* kd = ws + align_up(rows * desc->Hq * desc->dk * elem_bytes(desc), 256);
  ConvParams p{};
  p.B = desc->B; p.T = desc->T; p.d = desc->dk; p.W = desc->conv_width; p.phi = desc->feature_map; p.bf16 = bf16;
  p.x = Q; p.w = wq; p.halo = desc->conv_width > 1 ? q_halo : nullptr; p.y = qd;
  p.tail_out = desc->conv_width > 1 ? q_tail_out : nullptr; p.H = desc->Hq;
  hipError_t e = launch_conv1d(p, hs);
  if (e != hipSuccess) return LAWCAT_E_HIP;
  p.x = K; p.w = wk; p.halo = desc->conv_width > 1 ? k_halo : nullptr; p.y = kd;
  p.tail_out = desc->conv_width > 1 ? k_tail_out : nullptr; p.H = desc->Hkv;
  e = launch_conv1d(p, hs);
  if (e != hipSuccess) return LAWCAT_E_HIP;
  RecurrentParams r{};
  r.q = qd; r.k = kd; r.v = V; r.g = gate_logits; r.S0 = S0; r.z0 = z0; r.o = O; r.den_out = den_out;
  r.S_out = S_out; r.z_out = z_out; r.B = desc->B; r.T = desc->T; r.Hq = desc->Hq; r.Hkv = desc->Hkv;
  r.d = desc->dk; r.gate_scale = desc->gate_scale; r.eps = desc->eps; r.bf16 = bf16;
  return hip_status(launch_gla_recurrent(r, hs));
}

}  // namespace

extern "C" {

int lawcat_layer_prefill(const lawcat_desc* desc, const void* Q, const void* K, const void* V,
                         const void* gate_logits, const void* wq, const void* wk, const float* S0,
                         const float* z0, const void* q_halo, const void* k_halo, void* O, float* den_out,
                         float* S_out, float* z_out, void* q_tail_out, void* k_tail_out, void* workspace,
                         size_t workspace_bytes, void* stream) {
  return layer_prefill_impl(desc, Q, K, V, gate_logits, wq, wk, S0, z0, q_halo, k_halo, O, den_out, S_out, z_out,
                            q_tail_out, k_tail_out, workspace, workspace_bytes, stream, nullptr, nullptr);
}

size_t lawcat_varlen_workspace_bytes(const lawcat_desc* desc, const int32_t* seq_start, int one_launch) {
  if (check_desc(desc, true) != LAWCAT_OK || seq_start == nullptr || seq_start[0] != 0) return 0;
  for (int i = 0; i < desc->B; ++i) {
    const long long len = (long long)seq_start[i + 1] - seq_start[i];
    if (len < 1 || len > desc->T) return 0;
  }
  if (one_launch && prefill_path(desc) == Path::kChunkBf16) return varlen_plan(desc, seq_start).workspace_bytes;
  size_t need = 0;
  for (int i = 0; i < desc->B; ++i) {
    lawcat_desc one = *desc;
    one.B = 1; one.T = seq_start[i + 1] - seq_start[i];
    need = std::max(need, workspace_bytes_checked(&one, LAWCAT_CALL_LAYER_PREFILL));
  }
  return need;
}

int lawcat_layer_prefill_varlen(const lawcat_desc* desc, const int32_t* seq_start, const int32_t* seq_start_dev,
                                const void* Q, const void* K,
                                const void* V, const void* gate_logits, const void* wq, const void* wk,
                                const float* S0, const float* z0, const void* q_halo, const void* k_halo, void* O,
                                float* den_out, float* S_out, float* z_out, void* q_tail_out, void* k_tail_out,
                                void* workspace, size_t workspace_bytes, void* stream) {
  int st = check_desc(desc, true);
  if (st != LAWCAT_OK) return st;
  if (seq_start == nullptr || !Q || !K || !V || !gate_logits || !wq || !wk || !O || !S_out || !z_out) return LAWCAT_E_NULL;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(gate_logits) || !aligned16(wq) ||
      !aligned16(wk) || !aligned16(S0) || !aligned16(z0) || !aligned16(q_halo) || !aligned16(k_halo) ||
      !aligned16(O) || !aligned16(den_out) || !aligned16(S_out) || !aligned16(z_out) ||
      !aligned16(q_tail_out) || !aligned16(k_tail_out) || !aligned16(workspace))
    return LAWCAT_E_ALIGN;
  if (seq_start[0] != 0 || (reinterpret_cast<uintptr_t>(seq_start_dev) & 3u) != 0) return seq_start[0] != 0 ? LAWCAT_E_BAD_DESC : LAWCAT_E_ALIGN;
  const size_t eb = elem_bytes(desc);
  // everything is checked for every sequence before anything is enqueued
  for (int i = 0; i < desc->B; ++i) {
    const long long len = (long long)seq_start[i + 1] - seq_start[i];
    if (len < 1 || len > desc->T) return LAWCAT_E_BAD_DESC;
  }
  if (seq_start_dev != nullptr && prefill_path(desc) == Path::kChunkBf16) {
    // one set of launches for the whole batch: the kernels take every sequence's first row and length from
    // the device copy of the offsets; segments are cut for the longest sequence
    const ChunkPlan plan = varlen_plan(desc, seq_start);
    if (plan.workspace_bytes > 0 && (workspace == nullptr || workspace_bytes < plan.workspace_bytes)) return LAWCAT_E_WORKSPACE;
    ChunkParams c{};
    c.q = Q; c.k = K; c.v = V; c.g = gate_logits; c.wq = wq; c.wk = wk; c.q_halo = q_halo; c.k_halo = k_halo;
    c.S0 = S0; c.z0 = z0; c.o = O; c.den_out = den_out; c.S_out = S_out; c.z_out = z_out;
    c.workspace = workspace; c.seq_start = seq_start_dev;
    c.B = desc->B; c.T = desc->T; c.Hq = desc->Hq; c.Hkv = desc->Hkv; c.d = desc->dk;
    c.W = desc->conv_width; c.phi = desc->feature_map; c.fuse_conv = 1;
    c.gate_scale = desc->gate_scale; c.eps = desc->eps; c.plan = plan;
    c.q_tail = q_tail_out; c.k_tail = k_tail_out;
    return hip_status(launch_gla_chunk(c, static_cast<hipStream_t>(stream)));
  }
  for (int i = 0; i < desc->B; ++i) {
    const long long len = (long long)seq_start[i + 1] - seq_start[i];
    lawcat_desc one = *desc;
    one.B = 1; one.T = (int32_t)len;
    const size_t need = workspace_bytes_checked(&one, LAWCAT_CALL_LAYER_PREFILL);
    if (need > 0 && (workspace == nullptr || workspace_bytes < need)) return LAWCAT_E_WORKSPACE;
  }
  const size_t qrow = (size_t)desc->Hq * desc->dk * eb, krow = (size_t)desc->Hkv * desc->dk * eb;
  const size_t Wm = (size_t)(desc->conv_width - 1);
  const size_t sz = (size_t)desc->Hkv * desc->dk * desc->dk, zz = (size_t)desc->Hkv * desc->dk;
  auto at = [](const void* p, size_t bytes) -> const void* { return p ? static_cast<const char*>(p) + bytes : nullptr; };
  auto atw = [](void* p, size_t bytes) -> void* { return p ? static_cast<char*>(p) + bytes : nullptr; };
  for (int i = 0; i < desc->B; ++i) {
    lawcat_desc one = *desc;
    one.B = 1; one.T = seq_start[i + 1] - seq_start[i];
    const size_t t0 = (size_t)seq_start[i];
    st = layer_prefill_impl(&one, at(Q, t0 * qrow), at(K, t0 * krow), at(V, t0 * krow), at(gate_logits, t0 * krow), wq, wk,
                            S0 ? S0 + i * sz : nullptr, z0 ? z0 + i * zz : nullptr, at(q_halo, i * Wm * qrow),
                            at(k_halo, i * Wm * krow), atw(O, t0 * qrow), den_out ? den_out + t0 * desc->Hq : nullptr,
                            S_out ? S_out + i * sz : nullptr, z_out ? z_out + i * zz : nullptr,
                            atw(q_tail_out, i * Wm * qrow), atw(k_tail_out, i * Wm * krow), workspace, workspace_bytes,
                            stream, nullptr, nullptr, /*den_rows_packed=*/true);
    if (st != LAWCAT_OK) return st;
  }
  return LAWCAT_OK;
}

int lawcat_layer_prefill_fm(const lawcat_desc* desc, const void* Q, const void* K, const void* V,
                            const void* gate_logits, const void* wq, const void* wk, const void* wf, const float* S0,
                            const float* z0, const void* q_halo, const void* k_halo, void* O, float* den_out,
                            float* S_out, float* z_out, void* q_tail_out, void* k_tail_out, void* workspace,
                            size_t workspace_bytes, void* stream) {
  int st = check_desc(desc, true);
  if (st != LAWCAT_OK) return st;
  if (!Q || !K || !V || !gate_logits || !wq || !wk || !wf || !O || !S_out || !z_out) return LAWCAT_E_NULL;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(gate_logits) || !aligned16(wq) ||
      !aligned16(wk) || !aligned16(wf) || !aligned16(S0) || !aligned16(z0) || !aligned16(q_halo) ||
      !aligned16(k_halo) || !aligned16(O) || !aligned16(den_out) || !aligned16(S_out) || !aligned16(z_out) ||
      !aligned16(q_tail_out) || !aligned16(k_tail_out) || !aligned16(workspace))
    return LAWCAT_E_ALIGN;
  const size_t need = workspace_bytes_checked(desc, LAWCAT_CALL_LAYER_PREFILL_FM);
  if (workspace == nullptr || workspace_bytes < need) return LAWCAT_E_WORKSPACE;
  const size_t rows = (size_t)desc->B * desc->T;
  char* ws = static_cast<char*>(workspace);
  void* qd = ws;
  void* kd = ws + align_up(rows * desc->Hq * desc->dk * elem_bytes(desc), 256);
  char* inner = static_cast<char*>(kd) + align_up(rows * desc->Hkv * desc->dk * elem_bytes(desc), 256);
  const size_t inner_bytes = workspace_bytes - (size_t)(inner - ws);
  // queries: each head with the matrix of the kv head whose state it reads
  st = lawcat_conv1d_feature(desc, desc->Hq, Q, wq, wf, q_halo, qd, q_tail_out, stream);
  if (st != LAWCAT_OK) return st;
  st = lawcat_conv1d_feature(desc, desc->Hkv, K, wk, wf, k_halo, kd, k_tail_out, stream);
  if (st != LAWCAT_OK) return st;
  // the attention on the transformed q-dot, k-dot
  return lawcat_gla_prefill(desc, qd, kd, V, gate_logits, S0, z0, O, den_out, S_out, z_out, inner, inner_bytes, stream);
}

int lawcat_layer_prefill_static(const lawcat_desc* desc, const void* Q, const void* K, const void* V,
                                const void* gate_logits, const void* wq, const void* wk, const float* S0,
                                const float* z0, const void* q_halo, const void* k_halo, void* O, float* den_out,
                                float* S_out, float* z_out, void* q_tail_out, void* k_tail_out, void* stream) {
  const int st = check_desc(desc, true);
  if (st != LAWCAT_OK) return st;
  if (workspace_bytes_checked(desc, LAWCAT_CALL_LAYER_PREFILL) > (size_t)LAWCAT_STATIC_WORKSPACE_BYTES)
    return LAWCAT_E_STATIC_LIMIT;
  if (!Q || !K || !V || !gate_logits || !wq || !wk || !O || !S_out || !z_out) return LAWCAT_E_NULL;
  void* ws = nullptr;
  if (static_scratch(&ws) != hipSuccess) return LAWCAT_E_HIP;
  return layer_prefill_impl(desc, Q, K, V, gate_logits, wq, wk, S0, z0, q_halo, k_halo, O, den_out, S_out, z_out,
                            q_tail_out, k_tail_out, ws, LAWCAT_STATIC_WORKSPACE_BYTES, stream, nullptr, nullptr);
}

int lawcat_layer_prefill_timed(const lawcat_desc* desc, const void* Q, const void* K, const void* V,
                               const void* gate_logits, const void* wq, const void* wk, const float* S0,
                               const float* z0, const void* q_halo, const void* k_halo, void* O, float* den_out,
                               float* S_out, float* z_out, void* q_tail_out, void* k_tail_out, void* workspace,
                               size_t workspace_bytes, void* stream, void* ev_start, void* ev_stop) {
  if (ev_start == nullptr || ev_stop == nullptr) return LAWCAT_E_NULL;
  return layer_prefill_impl(desc, Q, K, V, gate_logits, wq, wk, S0, z0, q_halo, k_halo, O, den_out, S_out, z_out,
                            q_tail_out, k_tail_out, workspace, workspace_bytes, stream,
                            static_cast<hipEvent_t>(ev_start), static_cast<hipEvent_t>(ev_stop));
}

const char* lawcat_status_string(int status) {
  switch (status) {
    case LAWCAT_OK: return "ok";
    case LAWCAT_E_NULL: return "a required pointer is NULL";
    case LAWCAT_E_BAD_DESC: return "invalid descriptor";
    case LAWCAT_E_UNSUPPORTED: return "configuration not supported by the kernels";
    case LAWCAT_E_WORKSPACE: return "workspace missing or too small";
    case LAWCAT_E_ALIGN: return "pointer not 16-byte aligned";
    case LAWCAT_E_HIP: return "HIP launch error";
    case LAWCAT_E_STATIC_LIMIT: return "call needs more scratch than the library's static buffer holds";
    default: return "unknown status";
  }
}

int lawcat_version(void) { return LAWCAT_VERSION; }

}  // extern "C"
