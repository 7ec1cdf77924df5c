// Streaming-kernel variants: two bf16 latent streams, selected pages (all ranks).
#include "stream_kernel.h"

namespace dkv {

hipError_t stream_split_subset(const DecodeParams& P, dim3 grid, size_t lds, hipStream_t st) {
  return dispatch_stream<8, false, true>(P, grid, lds, st);
}

}  // namespace dkv
