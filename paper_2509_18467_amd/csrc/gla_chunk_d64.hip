// Head dimension 64 instantiations of the matrix-core prefill kernels.
#include "gla_chunk_impl.h"
namespace lawcat {
namespace chunk {
hipError_t launch_d64(const ChunkArgs& a, int group, int mode, int teams, hipStream_t stream) {
  return teams == 2 ? launch_d<64, 2>(a, group, mode, stream) : launch_d<64, 1>(a, group, mode, stream);
}
}  // namespace chunk
}  // namespace lawcat
