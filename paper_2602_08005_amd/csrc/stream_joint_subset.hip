// Streaming-kernel variants: one bf16 latent stream, selected pages (all ranks).
#include "stream_kernel.h"

namespace dkv {

hipError_t stream_joint_subset(const DecodeParams& P, dim3 grid, size_t lds, hipStream_t st) {
  return dispatch_stream<8, true, true>(P, grid, lds, st);
}

}  // namespace dkv
