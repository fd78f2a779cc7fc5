// placeholder until the matrix-core kernel lands: bf16 prefill uses the recurrent kernel
#include "kernels.h"
namespace lawcat {
bool chunk_path_supports(int) { return false; }
ChunkPlan make_chunk_plan(int, int T, int, int, int, int) { return ChunkPlan{T, 1, 0}; }
hipError_t launch_gla_chunk(const ChunkParams&, hipStream_t) { return hipErrorNotSupported; }
}  // namespace lawcat
