// Head dimension 128 instantiations of the matrix-core prefill kernels.
#include "gla_chunk_impl.h"
namespace lawcat {
namespace chunk {
hipError_t launch_d128(const ChunkArgs& a, int group, int mode, hipStream_t stream, const TraceEvents& ev) {
  return launch_d<128>(a, group, mode, stream, ev);
}
}  // namespace chunk
}  // namespace lawcat
