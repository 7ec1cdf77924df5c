// Streaming-kernel variants: two streams of 4-bit token-wise latents (all ranks).
#include "stream_kernel.h"

namespace dkv {

hipError_t stream_q4_split(const DecodeParams& P, dim3 grid, size_t lds, hipStream_t st) {
  // two streams of 4-bit codes: four 16-column blocks share a dword, so ranks 64 and 128 only
  if (P.R == 64)
    return P.sel_pages ? launch_stream<64, 8, false, true, true>(P, grid, lds, st)
                       : launch_stream<64, 8, false, false, true>(P, grid, lds, st);
  if (P.R == 128)
    return P.sel_pages ? launch_stream<128, 8, false, true, true>(P, grid, lds, st)
                       : launch_stream<128, 8, false, false, true>(P, grid, lds, st);
  return hipErrorInvalidValue;
}

}  // namespace dkv
