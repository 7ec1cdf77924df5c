// Streaming-kernel variants: two bf16 latent streams, whole cache (all ranks).
#include "stream_kernel.h"

namespace dkv {

hipError_t stream_split_full(const DecodeParams& P, dim3 grid, size_t lds, hipStream_t st) {
  return dispatch_stream<8, false, false>(P, grid, lds, st);
}

}  // namespace dkv
